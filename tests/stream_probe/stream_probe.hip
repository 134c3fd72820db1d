// Streaming probe: what the memory system of one MI355X delivers to kernels that move the bytes of
// the benchmark's workload (four bf16 input streams and one bf16 output stream of [8][4096][32][64],
// 671 MB) with no arithmetic.  It is the yardstick the chunked prefill kernel's time is read against:
// one workgroup per compute unit, every workgroup streams one (batch, head) the way the kernel
// does (rows of 128 bytes that lie H*128 = 4096 bytes apart), or, for comparison, a contiguous slab.
//
//   stream_probe [launches]        prints one line per variant: microseconds per launch and TB/s
//
// Built by __graft_entry__.build(); run by tests/test_gpu_stream_probe.py.  Cache-policy codes of the
// raw buffer instructions: 0 plain, 2 non-temporal, 16 scope bit sc1 (write through the XCD's L2).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef unsigned u4v __attribute__((ext_vector_type(4)));

struct Params {
    const char* in[4];
    char* out;
    int row_bytes;        // contiguous bytes per row: 128 (one head) ... 4096 (all heads: a contiguous slab)
    int inputs, outputs;  // streams actually read / written
};

constexpr int kThreads = 512;
constexpr long long kTokenBytes = 4096;            // H * N * 2
constexpr long long kSeqBytes = 4096 * kTokenBytes;

#define CHECK_HIP(x)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            std::exit(2);                                                                \
        }                                                                                \
    } while (0)

// Workgroup w streams rows of `row_bytes` bytes, 4096 bytes apart: with 128-byte rows that is one
// (batch, head) of the [B][T][H][N] layout over all 4096 tokens; with longer rows a workgroup takes
// several neighbouring heads over a proportionally shorter token range (same bytes per workgroup);
// 4096-byte rows are a contiguous slab.  16 bytes per lane, DEPTH steps of 8 KB in flight.
template <int DEPTH, int LOAD_POLICY, int STORE_POLICY>
__global__ __launch_bounds__(kThreads) void stream_kernel(Params p) {
    const int tid = threadIdx.x;
    const int groups = static_cast<int>(kTokenBytes) / p.row_bytes;      // row groups per token row
    const int segs = p.row_bytes / 128;                                   // token segments per sequence
    const int b = blockIdx.x / (segs * groups), rem = blockIdx.x % (segs * groups);
    const int seg = rem / groups, grp = rem % groups;
    const int rows = 4096 / segs;
    const long long base = b * kSeqBytes + static_cast<long long>(seg) * rows * kTokenBytes +
                           static_cast<long long>(grp) * p.row_bytes;
    const int per_row = p.row_bytes / 16;
    const int steps = rows * per_row / kThreads;
    __amdgpu_buffer_rsrc_t rin[4];
    for (int i = 0; i < 4; ++i)
        rin[i] = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(p.in[i] + base), 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(p.out + base, 0, 0x7fffffff, 0x00020000);
    auto offset_of = [&](int s) {
        const int e = s * kThreads + tid;
        return static_cast<int>((e / per_row) * kTokenBytes + (e % per_row) * 16);
    };
    u4v buf[DEPTH][4];
    unsigned acc = 0;
    auto issue = [&](int s, u4v (&d)[4]) {
        const int o = offset_of(s);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < p.inputs) d[i] = __builtin_bit_cast(u4v, __builtin_amdgcn_raw_buffer_load_b128(rin[i], o, 0, LOAD_POLICY));
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        buf[d][0] = buf[d][1] = buf[d][2] = buf[d][3] = u4v{0, 0, 0, 0};
        if (d < steps) issue(d, buf[d]);
    }
    for (int s = 0; s < steps; s += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (s + d < steps) {
                u4v t = buf[d][0] ^ buf[d][1] ^ buf[d][2] ^ buf[d][3];
                acc += t.x;
                const int o = offset_of(s + d);
                if (s + d + DEPTH < steps) issue(s + d + DEPTH, buf[d]);
                t.y += acc;
                if (p.outputs) __builtin_amdgcn_raw_buffer_store_b128(t, rout, o, 0, STORE_POLICY);
            }
        }
    }
    if (!p.outputs && acc == 0x12345678u) p.out[0] = 1;      // keeps the loads alive
}

int main(int argc, char** argv) {
    const int launches = argc > 1 ? std::atoi(argv[1]) : 50;
    const size_t bytes = 8ull * kSeqBytes;                     // 128 MiB per stream
    Params p;
    char* raw[5];                                              // four inputs and the output, 4 KiB of slack each
    for (int i = 0; i < 5; ++i) {
        CHECK_HIP(hipMalloc(reinterpret_cast<void**>(&raw[i]), bytes + 4096));
        CHECK_HIP(hipMemset(raw[i], i + 1, bytes + 4096));
    }
    hipEvent_t e0, e1;
    CHECK_HIP(hipEventCreate(&e0));
    CHECK_HIP(hipEventCreate(&e1));
    // stagger: bytes by which the i-th buffer's base is shifted (0: all bases agree modulo 4 KiB, as
    // tensors from an allocator do)
    auto run = [&](const char* name, auto kernel, int row_bytes, int inputs, int outputs, int stagger = 0) {
        for (int i = 0; i < 4; ++i) p.in[i] = raw[i] + i * stagger;
        p.out = raw[4] + 4 * stagger;
        p.row_bytes = row_bytes;
        p.inputs = inputs;
        p.outputs = outputs;
        for (int i = 0; i < 3 * launches; ++i) hipLaunchKernelGGL(kernel, dim3(256), dim3(kThreads), 0, 0, p);   // clocks up
        CHECK_HIP(hipDeviceSynchronize());
        std::vector<float> us;
        for (int rep = 0; rep < 5; ++rep) {
            CHECK_HIP(hipEventRecord(e0));
            for (int i = 0; i < launches; ++i) hipLaunchKernelGGL(kernel, dim3(256), dim3(kThreads), 0, 0, p);
            CHECK_HIP(hipEventRecord(e1));
            CHECK_HIP(hipEventSynchronize(e1));
            float ms = 0;
            CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
            us.push_back(ms / launches * 1000.f);
        }
        std::sort(us.begin(), us.end());
        const double mb = (inputs + outputs) * (bytes / 1e6);
        std::printf("%-58s %7.1f us  %5.2f TB/s\n", name, us[2], mb / us[2]);
        std::fflush(stdout);
    };
    run("kernel layout (128 B rows), nt loads, write-through stores", stream_kernel<4, 2, 16>, 128, 4, 1);
    run("kernel layout (128 B rows), nt loads, nt stores", stream_kernel<4, 2, 2>, 128, 4, 1);
    run("kernel layout (128 B rows), plain loads and stores", stream_kernel<4, 0, 0>, 128, 4, 1);
    run("kernel layout, 8 steps in flight, nt loads, write-through", stream_kernel<8, 2, 16>, 128, 4, 1);
    run("256 B rows, nt loads, write-through stores", stream_kernel<4, 2, 16>, 256, 4, 1);
    run("contiguous slabs, nt loads, write-through stores", stream_kernel<4, 2, 16>, 4096, 4, 1);
    run("kernel layout, the four input streams only", stream_kernel<4, 2, 16>, 128, 4, 0);
    run("kernel layout, the output stream only", stream_kernel<4, 2, 16>, 128, 0, 1);
    run("kernel layout, buffer bases 128 B apart modulo 1 KiB", stream_kernel<4, 2, 16>, 128, 4, 1, 128);
    run("contiguous slabs, buffer bases 128 B apart modulo 1 KiB", stream_kernel<4, 2, 16>, 4096, 4, 1, 128);
    return 0;
}
