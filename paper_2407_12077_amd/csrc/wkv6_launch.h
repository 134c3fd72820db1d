// Internal launch interface between the C ABI (wkv6_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>

namespace wkv6 {

constexpr int kHeadSize = 64;   // N: the only head size the kernels are built for

struct Args {
    int B, T, H;
    const void* r;
    const void* k;
    const void* v;
    const void* x;
    const float* u;
    const float* state_in;    // may be nullptr (zero state)
    void* out;
    float* state_out;         // may be nullptr (not written)
    long long batch_stride;   // elements between consecutive batches of r,k,v,x,out
};

// Token-by-token fp32 kernel; inputs bf16 or fp32, out always fp32.
hipError_t launch_recurrent(const Args& a, bool in_bf16, hipStream_t stream);

// Chunked matrix-core kernel; inputs bf16, out bf16 or fp32.
hipError_t launch_chunked(const Args& a, bool out_f32, hipStream_t stream);

// T == 0: state_out = state_in (or zero).
hipError_t launch_state_passthrough(const Args& a, hipStream_t stream);

}  // namespace wkv6
