"""Thin ctypes binding of ``libwkv6.so``: argument marshalling only.

Every entry point has the name and argument order of ``include/wkv6.h``.  Tensors are
PyTorch-ROCm tensors used purely as device memory (``data_ptr``) and the current HIP
stream; nothing is computed here.  There is no fallback: if the library is missing,
loading raises.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libwkv6.so")

WKV6_OK = 0
WKV6_DTYPE_BF16 = 0
WKV6_DTYPE_F32 = 1

EXPORTS = ("wkv6_prefill_bf16", "wkv6_prefill_bf16_f32out", "wkv6_prefill_bf16_strided",
           "wkv6_prefill_f32", "wkv6_prefill_bf16_recurrent", "wkv6_prefill_bf16_split",
           "wkv6_prefill_bf16_split_noalloc",
           "wkv6_split_workspace_bytes", "wkv6_split_segments", "wkv6_finch_c2_prefill_bf16",
           "wkv6_finch_c2_prefill_bf16_f32out", "wkv6_finch_c2_prefill_bf16_strided",
           "wkv6_finch_c2_prefill_bf16_split", "wkv6_finch_c2_prefill_bf16_moments",
           "wkv6_layernorm_finalize", "wkv6_layernorm_apply_bf16", "wkv6_decay_lora_input_bf16", "wkv6_finch_c2_prefill_lora_bf16", "wkv6_prefill_lora_bf16",
           "wkv6_decode_bf16", "wkv6_finch_c2_decode_bf16", "wkv6_append_bf16",
           "wkv6_finch_c2_append_bf16", "wkv6_key_compress_bf16", "wkv6_arena_layout", "wkv6_status_string",
           "wkv6_version")

_lib = None


class Wkv6Error(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"wkv6 status {status}: {text}")
        self.status = status


def load():
    """Load the C-ABI library built by ``paper_2407_12077_amd.build`` (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -m paper_2407_12077_amd.build` first")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i, ll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
        common = [i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]
        for name in ("wkv6_prefill_bf16", "wkv6_prefill_bf16_f32out", "wkv6_prefill_f32",
                     "wkv6_prefill_bf16_recurrent", "wkv6_finch_c2_prefill_bf16",
                     "wkv6_finch_c2_prefill_bf16_f32out", "wkv6_append_bf16",
                     "wkv6_finch_c2_append_bf16"):
            fn = getattr(lib, name)
            fn.restype = i
            fn.argtypes = common + [vp]
        lib.wkv6_prefill_bf16_strided.restype = i
        lib.wkv6_prefill_bf16_strided.argtypes = common + [ll, i, vp]
        lib.wkv6_finch_c2_prefill_bf16_strided.restype = i
        lib.wkv6_finch_c2_prefill_bf16_strided.argtypes = common + [ll, i, vp]
        for name in ("wkv6_decode_bf16", "wkv6_finch_c2_decode_bf16"):
            fn = getattr(lib, name)
            fn.restype = i
            fn.argtypes = [i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.wkv6_finch_c2_prefill_bf16_moments.restype = i
        lib.wkv6_finch_c2_prefill_bf16_moments.argtypes = [i, i, i, i] + [vp] * 10
        lib.wkv6_finch_c2_prefill_lora_bf16.restype = i
        lib.wkv6_finch_c2_prefill_lora_bf16.argtypes = [i, i, i, i, i] + [vp] * 12
        lib.wkv6_prefill_lora_bf16.restype = i
        lib.wkv6_prefill_lora_bf16.argtypes = [i, i, i, i, i] + [vp] * 11
        lib.wkv6_decay_lora_input_bf16.restype = i
        lib.wkv6_decay_lora_input_bf16.argtypes = [i, i, i, i, i] + [vp] * 8 + [i, vp]
        lib.wkv6_layernorm_apply_bf16.restype = i
        lib.wkv6_layernorm_apply_bf16.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, i, vp]
        lib.wkv6_layernorm_finalize.restype = i
        lib.wkv6_layernorm_finalize.argtypes = [i, i, i, i, vp, ctypes.c_float, vp, vp]
        lib.wkv6_key_compress_bf16.restype = i
        lib.wkv6_key_compress_bf16.argtypes = [ll, i, vp, vp, vp, i, vp]
        lib.wkv6_prefill_bf16_split.restype = i
        lib.wkv6_prefill_bf16_split.argtypes = common + [i, i, vp, ll, vp]
        lib.wkv6_prefill_bf16_split_noalloc.restype = i
        lib.wkv6_prefill_bf16_split_noalloc.argtypes = common + [i, i, vp]
        lib.wkv6_finch_c2_prefill_bf16_split.restype = i
        lib.wkv6_finch_c2_prefill_bf16_split.argtypes = common + [i, i, vp, ll, vp]
        lib.wkv6_split_workspace_bytes.restype = ll
        lib.wkv6_split_workspace_bytes.argtypes = [i, i, i, i, i]
        lib.wkv6_split_segments.restype = i
        lib.wkv6_split_segments.argtypes = [i, i, i, i]
        lib.wkv6_arena_layout.restype = ctypes.c_longlong
        lib.wkv6_arena_layout.argtypes = [i, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(ctypes.c_longlong)]
        lib.wkv6_status_string.restype = ctypes.c_char_p
        lib.wkv6_status_string.argtypes = [i]
        lib.wkv6_version.restype = i
        lib.wkv6_version.argtypes = []
        _lib = lib
    return _lib


def status_string(status):
    return load().wkv6_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status):
    if status != WKV6_OK:
        raise Wkv6Error(status, status_string(status))


def _call(name, B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream, *extra):
    fn = getattr(load(), name)
    _check(fn(B, T, H, N, _ptr(r), _ptr(k), _ptr(v), _ptr(x), _ptr(u), _ptr(state_in),
              _ptr(out), _ptr(state_out), *extra, _stream(stream)))


def wkv6_prefill_bf16(B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream=None):
    _call("wkv6_prefill_bf16", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream)


def wkv6_prefill_bf16_f32out(B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream=None):
    _call("wkv6_prefill_bf16_f32out", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream)


def wkv6_prefill_bf16_strided(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
                              batch_stride, out_dtype, stream=None):
    _call("wkv6_prefill_bf16_strided", B, T, H, N, r, k, v, x, u, state_in, out, state_out,
          stream, ctypes.c_longlong(batch_stride), int(out_dtype))


def wkv6_prefill_bf16_split(B, T, H, N, r, k, v, x, u, state_in, out, state_out, out_dtype,
                            segments, workspace, workspace_bytes, stream=None):
    _call("wkv6_prefill_bf16_split", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream,
          int(out_dtype), int(segments), _ptr(workspace), ctypes.c_longlong(workspace_bytes))


def wkv6_prefill_bf16_split_noalloc(B, T, H, N, r, k, v, x, u, state_in, out, state_out, out_dtype,
                                    segments, stream=None):
    _call("wkv6_prefill_bf16_split_noalloc", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream,
          int(out_dtype), int(segments))


def wkv6_finch_c2_prefill_bf16_split(B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out,
                                     out_dtype, segments, workspace, workspace_bytes, stream=None):
    _call("wkv6_finch_c2_prefill_bf16_split", B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out,
          stream, int(out_dtype), int(segments), _ptr(workspace), ctypes.c_longlong(workspace_bytes))


def wkv6_split_workspace_bytes(B, T, H, N, segments):
    return load().wkv6_split_workspace_bytes(B, T, H, N, segments)


def wkv6_split_segments(B, T, H, N):
    return load().wkv6_split_segments(B, T, H, N)


def wkv6_arena_layout(sizes):
    """(arena bytes, [offset of each tensor]) for tensors of the given byte sizes; (-1, []) if rejected."""
    n = len(sizes)
    arr = (ctypes.c_longlong * max(n, 1))(*[int(b) for b in sizes])
    offs = (ctypes.c_longlong * max(n, 1))()
    total = load().wkv6_arena_layout(n, arr, offs)
    return total, ([int(offs[j]) for j in range(n)] if total >= 0 else [])


def wkv6_prefill_f32(B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream=None):
    _call("wkv6_prefill_f32", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream)


def wkv6_prefill_bf16_recurrent(B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream=None):
    _call("wkv6_prefill_bf16_recurrent", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream)


def wkv6_finch_c2_prefill_bf16(B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out, stream=None):
    _call("wkv6_finch_c2_prefill_bf16", B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out, stream)


def wkv6_finch_c2_prefill_bf16_f32out(B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out,
                                      stream=None):
    _call("wkv6_finch_c2_prefill_bf16_f32out", B, T, H, N, r, kbar, v, x, uprime, state_in, out,
          state_out, stream)


def wkv6_finch_c2_prefill_bf16_strided(B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out,
                                       batch_stride, out_dtype, stream=None):
    _call("wkv6_finch_c2_prefill_bf16_strided", B, T, H, N, r, kbar, v, x, uprime, state_in, out,
          state_out, stream, ctypes.c_longlong(batch_stride), int(out_dtype))


def wkv6_finch_c2_prefill_bf16_moments(B, T, H, N, r, kbar, v, x, uprime, state_in, out, moments, state_out,
                                       stream=None):
    _check(load().wkv6_finch_c2_prefill_bf16_moments(
        B, T, H, N, _ptr(r), _ptr(kbar), _ptr(v), _ptr(x), _ptr(uprime), _ptr(state_in), _ptr(out),
        _ptr(moments), _ptr(state_out), _stream(stream)))


def wkv6_finch_c2_prefill_lora_bf16(B, T, H, N, R, r, kbar, v, y, lam, b_omega, uprime, state_in, out, moments,
                                    state_out, stream=None):
    _check(load().wkv6_finch_c2_prefill_lora_bf16(
        B, T, H, N, R, _ptr(r), _ptr(kbar), _ptr(v), _ptr(y), _ptr(lam), _ptr(b_omega), _ptr(uprime),
        _ptr(state_in), _ptr(out), _ptr(moments), _ptr(state_out), _stream(stream)))


def wkv6_prefill_lora_bf16(B, T, H, N, R, r, k, v, y, lam, b_omega, u, state_in, out, state_out, stream=None):
    _check(load().wkv6_prefill_lora_bf16(
        B, T, H, N, R, _ptr(r), _ptr(k), _ptr(v), _ptr(y), _ptr(lam), _ptr(b_omega), _ptr(u), _ptr(state_in),
        _ptr(out), _ptr(state_out), _stream(stream)))


def wkv6_decay_lora_input_bf16(B, T, D, R_d, R, x, x_prev, mu_x, lambda_d, a_d, b_d, a_omega, y, out_dtype, stream=None):
    _check(load().wkv6_decay_lora_input_bf16(B, T, D, R_d, R, _ptr(x), _ptr(x_prev), _ptr(mu_x), _ptr(lambda_d),
                                             _ptr(a_d), _ptr(b_d), _ptr(a_omega), _ptr(y), int(out_dtype),
                                             _stream(stream)))


def wkv6_layernorm_apply_bf16(B, T, H, N, o, mean_rstd, gamma, beta, y, out_dtype, stream=None):
    _check(load().wkv6_layernorm_apply_bf16(B, T, H, N, _ptr(o), _ptr(mean_rstd), _ptr(gamma), _ptr(beta), _ptr(y),
                                            int(out_dtype), _stream(stream)))


def wkv6_layernorm_finalize(B, T, H, N, moments, eps, mean_rstd, stream=None):
    _check(load().wkv6_layernorm_finalize(B, T, H, N, _ptr(moments), ctypes.c_float(eps), _ptr(mean_rstd),
                                          _stream(stream)))


def wkv6_append_bf16(B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream=None):
    _call("wkv6_append_bf16", B, T, H, N, r, k, v, x, u, state_in, out, state_out, stream)


def wkv6_finch_c2_append_bf16(B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out, stream=None):
    _call("wkv6_finch_c2_append_bf16", B, T, H, N, r, kbar, v, x, uprime, state_in, out, state_out, stream)


def wkv6_decode_bf16(B, H, N, r, k, v, x, u, state, out, stream=None):
    _check(load().wkv6_decode_bf16(B, H, N, _ptr(r), _ptr(k), _ptr(v), _ptr(x), _ptr(u), _ptr(state),
                                   _ptr(out), _stream(stream)))


def wkv6_finch_c2_decode_bf16(B, H, N, r, kbar, v, x, uprime, state, out, stream=None):
    _check(load().wkv6_finch_c2_decode_bf16(B, H, N, _ptr(r), _ptr(kbar), _ptr(v), _ptr(x), _ptr(uprime),
                                            _ptr(state), _ptr(out), _stream(stream)))


def wkv6_key_compress_bf16(M, D, x, w_kd, c, out_dtype, stream=None):
    _check(load().wkv6_key_compress_bf16(M, D, _ptr(x), _ptr(w_kd), _ptr(c), int(out_dtype), _stream(stream)))


def wkv6_version():
    return load().wkv6_version()
