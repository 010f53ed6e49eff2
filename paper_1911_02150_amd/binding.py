"""ctypes binding of libmqa_decode.so: same names as the C ABI (include/mqa.h),
argument marshalling only.  torch is used for device memory and the current
stream; every step of the path runs in the library's HIP kernels.  There is no
fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libmqa_decode.so")

MQA_F32, MQA_BF16 = 0, 1
MQA_PROJ_Q, MQA_PROJ_KV, MQA_PROJ_KV_MH, MQA_PROJ_O, MQA_PROJ_LINEAR = 0, 1, 2, 3, 4
MQA_EPI_STORE, MQA_EPI_RELU, MQA_EPI_ADD = 0, 1, 2

EXPORTS = [
    "mqa_project_qkvo", "mqa_project_qkvo_ex", "mqa_project_append_qkv", "mqa_append_kv", "mqa_decode_step", "mha_decode_step",
    "mqa_decode_step_window", "mha_decode_step_window", "mqa_append_kv_rows", "mqa_prefill_attention", "mha_prefill_attention",
    "mqa_decode_step_beams", "mqa_decode_beams_workspace_bytes", "mqa_beam_reorder_kv", "mqa_decode_step_ex", "mha_decode_step_ex", "mqa_decode_partials", "mqa_decode_combine",
    "mqa_decode_workspace_bytes", "mha_decode_workspace_bytes", "mqa_decode_workspace_bytes_default", "mqa_decode_num_splits",
    "mqa_decode_plan", "mqa_decode_step_noalloc", "mqa_project_memory_kv", "mqa_memory_decode_step",
    "mqa_stream_read", "mqa_stream_copy", "mqa_status_string",
    "mqa_stack_layernorm", "mqa_stack_embed", "mqa_stack_add", "mqa_stack_relu", "mqa_stack_argmax",
]


class mqa_tuning(ctypes.Structure):
    _fields_ = [("splits", ctypes.c_int32), ("kernel", ctypes.c_int32), ("flags", ctypes.c_int32)]


class MqaError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn} failed: status {status} ({status_string(status)})")


_lib = None


def load_library(path: str = LIB_PATH):
    """Loads the shared library (once).  Raises OSError if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise OSError(f"{path} not found: build it with `python -m paper_1911_02150_amd.build` "
                      "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(path)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    tp = ctypes.POINTER(mqa_tuning)
    dec = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp]
    lib.mqa_project_qkvo.argtypes = [ci, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.mqa_project_qkvo_ex.argtypes = [ci, vp, vp, vp, ci, ci, ci, ci, ci, vp]
    lib.mqa_project_append_qkv.argtypes = [vp] * 9 + [ci] * 8 + [vp]
    lib.mqa_append_kv.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp]
    lib.mqa_project_memory_kv.argtypes = [vp] * 7 + [ci] * 8 + [vp]
    lib.mqa_memory_decode_step.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp]
    lib.mqa_decode_step.argtypes = dec
    lib.mha_decode_step.argtypes = dec
    win = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.mqa_decode_step_window.argtypes = win
    lib.mha_decode_step_window.argtypes = win
    lib.mqa_append_kv_rows.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.mqa_prefill_attention.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp]
    lib.mha_prefill_attention.argtypes = lib.mqa_prefill_attention.argtypes
    lib.mqa_decode_step_beams.argtypes = [vp] * 8 + [ci] * 8 + [cf, vp, sz, vp]
    lib.mqa_decode_beams_workspace_bytes.argtypes = [ci] * 8
    lib.mqa_decode_beams_workspace_bytes.restype = sz
    lib.mqa_beam_reorder_kv.argtypes = [vp] * 7 + [ci] * 6 + [vp]
    lib.mqa_decode_step_ex.argtypes = dec + [tp]
    lib.mha_decode_step_ex.argtypes = dec + [tp]
    lib.mqa_decode_partials.argtypes = dec + [tp]
    lib.mqa_decode_combine.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, sz, vp, tp]
    lib.mqa_decode_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.mqa_decode_workspace_bytes.restype = sz
    lib.mha_decode_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.mha_decode_workspace_bytes.restype = sz
    lib.mqa_decode_workspace_bytes_default.argtypes = [ci] * 7
    lib.mqa_decode_workspace_bytes_default.restype = sz
    lib.mqa_decode_num_splits.argtypes = [ci, ci, ci, ci, ci, ci, ci, tp]
    lib.mqa_decode_plan.argtypes = [ci] * 8 + [tp, vp, vp, vp]
    lib.mqa_decode_step_noalloc.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp]
    lib.mqa_stream_read.argtypes = [vp, sz, vp, vp]
    lib.mqa_stream_copy.argtypes = [vp, vp, sz, vp]
    lib.mqa_stack_layernorm.argtypes = [vp, vp, ci, ci, cf, vp]
    lib.mqa_stack_embed.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.mqa_stack_add.argtypes = [vp, vp, sz, vp]
    lib.mqa_stack_relu.argtypes = [vp, sz, vp]
    lib.mqa_stack_argmax.argtypes = [vp, vp, ci, ci, vp]
    lib.mqa_status_string.argtypes = [ci]
    lib.mqa_status_string.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("mqa_decode_workspace_bytes", "mha_decode_workspace_bytes", "mqa_status_string",
                        "mqa_decode_beams_workspace_bytes", "mqa_decode_workspace_bytes_default"):
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().mqa_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _tuning(tuning):
    if tuning is None:
        return None
    if isinstance(tuning, mqa_tuning):
        return ctypes.byref(tuning)
    t = mqa_tuning(int(tuning.get("splits", 0)), int(tuning.get("kernel", 0)), int(tuning.get("flags", 0)))
    return ctypes.byref(t)


def _cache_dtype(K):
    if K.dtype == torch.bfloat16:
        return MQA_BF16
    if K.dtype == torch.float32:
        return MQA_F32
    raise TypeError(f"cache dtype {K.dtype} not supported (float32 or bfloat16)")


def _check(t, name, dtype=None):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}")


def mqa_decode_workspace_bytes(b, h, cap, v) -> int:
    return int(load_library().mqa_decode_workspace_bytes(b, h, cap, v))


def mha_decode_workspace_bytes(b, h, cap, v) -> int:
    return int(load_library().mha_decode_workspace_bytes(b, h, cap, v))


def mqa_decode_workspace_bytes_default(b, h, cap, k, v, dt, multi_head=False) -> int:
    """Exactly what the default plan of mqa_decode_step / mha_decode_step uses for this shape."""
    return int(load_library().mqa_decode_workspace_bytes_default(b, h, cap, k, v, dt, int(multi_head)))


def mqa_decode_plan(b, h, cap, k, v, dt, multi_head=False, window=0, tuning=None):
    """(ranges per sequence, positions per range, head groups) the decode calls will use."""
    S, chunk, HG = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    rc = load_library().mqa_decode_plan(b, h, cap, k, v, dt, int(multi_head), int(window), _tuning(tuning),
                                        ctypes.byref(S), ctypes.byref(chunk), ctypes.byref(HG))
    if rc != 0:
        raise MqaError("mqa_decode_plan", rc)
    return S.value, chunk.value, HG.value


_ws_cache = {}


def _default_workspace(device, nbytes, stream=None):
    """Workspace owned by the binding for callers that pass none: one per (device, stream), grown on
    demand.  A replaced buffer goes back to torch's caching allocator, which keeps it out of other
    streams' hands until the work queued on the stream it was allocated on has finished -- so
    allocate it with that stream current."""
    if stream is None:
        stream = torch.cuda.current_stream(device)
    key = (device.type, device.index, int(stream.cuda_stream))
    ws = _ws_cache.get(key)
    if ws is None or ws.numel() < nbytes:
        with torch.cuda.stream(stream):
            ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _ws_cache[key] = ws
    return ws


def mqa_decode_num_splits(b, h, cap, k, v, dt, multi_head=False, tuning=None) -> int:
    return int(load_library().mqa_decode_num_splits(b, h, cap, k, v, dt, int(multi_head), _tuning(tuning)))


def _decode(fn_name, multi_head, q, K, V, lens, o, scale, workspace, stream, tuning, with_tuning=True, window=None):
    lib = load_library()
    _check(q, "q", torch.float32), _check(K, "K"), _check(V, "V"), _check(lens, "lens", torch.int32)
    b, h, k = q.shape
    cap, v = V.shape[-2], V.shape[-1]
    want_k = (b, h, cap, k) if multi_head else (b, cap, k)
    want_v = (b, h, cap, v) if multi_head else (b, cap, v)
    if tuple(K.shape) != want_k or tuple(V.shape) != want_v or K.dtype != V.dtype or lens.numel() != b:
        raise ValueError(f"shape mismatch: q {tuple(q.shape)} K {tuple(K.shape)} V {tuple(V.shape)} lens {tuple(lens.shape)}")
    if o is None:
        o = torch.empty((b, h, v), dtype=torch.float32, device=q.device)
    _check(o, "o", torch.float32)
    if tuple(o.shape) != (b, h, v):
        raise ValueError("o must be [b,h,v]")
    if workspace is None:
        nbytes = mha_decode_workspace_bytes(b, h, cap, v) if multi_head else mqa_decode_workspace_bytes(b, h, cap, v)
        workspace = _default_workspace(q.device, nbytes, stream)
    args = [_ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(o), b, h, cap, k, v, _cache_dtype(K), float(scale)]
    if window is not None:
        args.append(int(window))
    args += [_ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)]
    if with_tuning:
        args.append(_tuning(tuning))
    rc = getattr(lib, fn_name)(*args)
    if rc != 0:
        raise MqaError(fn_name, rc)
    return o


def mqa_decode_step(q, K, V, lens, o=None, scale=1.0, workspace=None, stream=None, tuning=None):
    """q [b,h,k] f32, K [b,cap,k], V [b,cap,v] (f32 or bf16), lens [b] int32 -> o [b,h,v] f32."""
    if tuning is None:
        return _decode("mqa_decode_step", False, q, K, V, lens, o, scale, workspace, stream, None, False)
    return _decode("mqa_decode_step_ex", False, q, K, V, lens, o, scale, workspace, stream, tuning)


def mha_decode_step(q, K, V, lens, o=None, scale=1.0, workspace=None, stream=None, tuning=None):
    """q [b,h,k] f32, K [b,h,cap,k], V [b,h,cap,v], lens [b] int32 -> o [b,h,v] f32."""
    if tuning is None:
        return _decode("mha_decode_step", True, q, K, V, lens, o, scale, workspace, stream, None, False)
    return _decode("mha_decode_step_ex", True, q, K, V, lens, o, scale, workspace, stream, tuning)


def mqa_decode_step_noalloc(q, K, V, lens, o, scale=1.0, stream=None):
    """mqa_decode_step without a workspace argument and without any allocation: `o` must be given; the
    partial states live in the library's static device buffer (calls on one GPU must not overlap)."""
    lib = load_library()
    _check(q, "q", torch.float32), _check(K, "K"), _check(V, "V"), _check(lens, "lens", torch.int32), _check(o, "o", torch.float32)
    b, h, k = q.shape
    cap, v = V.shape[-2], V.shape[-1]
    if (tuple(K.shape) != (b, cap, k) or tuple(V.shape) != (b, cap, v) or K.dtype != V.dtype or lens.numel() != b
            or tuple(o.shape) != (b, h, v)):
        raise ValueError("shape mismatch in mqa_decode_step_noalloc")
    rc = lib.mqa_decode_step_noalloc(_ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(o), b, h, cap, k, v, _cache_dtype(K),
                                     float(scale), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_decode_step_noalloc", rc)
    return o


def mqa_decode_step_window(q, K, V, lens, window, o=None, scale=1.0, workspace=None, stream=None):
    """Local attention: sequence i attends to its last `window` valid positions only."""
    return _decode("mqa_decode_step_window", False, q, K, V, lens, o, scale, workspace, stream, None, False, window)


def mha_decode_step_window(q, K, V, lens, window, o=None, scale=1.0, workspace=None, stream=None):
    return _decode("mha_decode_step_window", True, q, K, V, lens, o, scale, workspace, stream, None, False, window)


def mqa_decode_partials(q, K, V, lens, o, workspace, scale=1.0, stream=None, tuning=None):
    return _decode("mqa_decode_partials", False, q, K, V, lens, o, scale, workspace, stream, tuning)


def mqa_decode_combine(lens, o, cap, k, cache_dtype, workspace, stream=None, tuning=None):
    lib = load_library()
    b, h, v = o.shape
    rc = lib.mqa_decode_combine(_ptr(lens), _ptr(o), b, h, cap, k, v, cache_dtype, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream), _tuning(tuning))
    if rc != 0:
        raise MqaError("mqa_decode_combine", rc)
    return o


def mqa_append_kv(K, V, k_new, v_new, lens, stream=None):
    """Appends k_new/v_new ([b,k]/[b,v] multi-query, [b,h,k]/[b,h,v] multi-head) in place; lens += 1."""
    lib = load_library()
    for t, n in ((K, "K"), (V, "V"), (k_new, "k_new"), (v_new, "v_new"), (lens, "lens")):
        _check(t, n)
    if k_new.dtype != torch.float32 or v_new.dtype != torch.float32 or lens.dtype != torch.int32:
        raise TypeError("k_new/v_new must be float32 and lens int32")
    b = K.shape[0]
    h_kv = K.shape[1] if K.dim() == 4 else 1
    cap, k, v = K.shape[-2], K.shape[-1], V.shape[-1]
    if k_new.numel() != b * h_kv * k or v_new.numel() != b * h_kv * v or lens.numel() != b or V.shape[:-1] != K.shape[:-1]:
        raise ValueError("shape mismatch in mqa_append_kv")
    rc = lib.mqa_append_kv(_ptr(K), _ptr(V), _ptr(k_new), _ptr(v_new), _ptr(lens), b, h_kv, cap, k, v,
                           _cache_dtype(K), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_append_kv", rc)


def mqa_append_kv_rows(K, V, k_new, v_new, lens, stream=None):
    """Appends n rows per sequence: k_new [b,n,k] / v_new [b,n,v] (multi-query) or [b,n,h,k] / [b,n,h,v]."""
    lib = load_library()
    for t, nm in ((K, "K"), (V, "V"), (k_new, "k_new"), (v_new, "v_new"), (lens, "lens")):
        _check(t, nm)
    b, n = k_new.shape[0], k_new.shape[1]
    h_kv = K.shape[1] if K.dim() == 4 else 1
    cap, k, v = K.shape[-2], K.shape[-1], V.shape[-1]
    if k_new.numel() != b * n * h_kv * k or v_new.numel() != b * n * h_kv * v or K.shape[0] != b or lens.numel() != b:
        raise ValueError("shape mismatch in mqa_append_kv_rows")
    rc = lib.mqa_append_kv_rows(_ptr(K), _ptr(V), _ptr(k_new), _ptr(v_new), _ptr(lens), b, n, h_kv, cap, k, v,
                                _cache_dtype(K), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_append_kv_rows", rc)


def mqa_prefill_attention(q, K, V, lens, o=None, scale=1.0, workspace=None, stream=None):
    """q [b,n,h,k], K [b,cap,k], V [b,cap,v] bf16, lens [b] (after the append) -> o [b,n,h,v]."""
    lib = load_library()
    _check(q, "q", torch.float32), _check(K, "K"), _check(V, "V"), _check(lens, "lens", torch.int32)
    b, n, h, k = q.shape
    cap, v = V.shape[-2], V.shape[-1]
    if tuple(K.shape) != (b, cap, k) or tuple(V.shape) != (b, cap, v) or lens.numel() != b:
        raise ValueError("shape mismatch in mqa_prefill_attention")
    if o is None:
        o = torch.empty((b, n, h, v), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _default_workspace(q.device, mqa_decode_workspace_bytes(b, n * h, cap, v), stream)
    rc = lib.mqa_prefill_attention(_ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(o), b, n, h, cap, k, v,
                                   _cache_dtype(K), float(scale), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_prefill_attention", rc)
    return o


def mha_prefill_attention(q, K, V, lens, o=None, scale=1.0, workspace=None, stream=None):
    """q [b,h,n,k], K [b,h,cap,k], V [b,h,cap,v] bf16, lens [b] (after the append) -> o [b,h,n,v]."""
    lib = load_library()
    _check(q, "q", torch.float32), _check(K, "K"), _check(V, "V"), _check(lens, "lens", torch.int32)
    b, h, n, k = q.shape
    cap, v = V.shape[-2], V.shape[-1]
    if tuple(K.shape) != (b, h, cap, k) or tuple(V.shape) != (b, h, cap, v) or lens.numel() != b:
        raise ValueError("shape mismatch in mha_prefill_attention")
    if o is None:
        o = torch.empty((b, h, n, v), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _default_workspace(q.device, mha_decode_workspace_bytes(b, n * h, cap, v), stream)
    rc = lib.mha_prefill_attention(_ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(o), b, n, h, cap, k, v,
                                   _cache_dtype(K), float(scale), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != 0:
        raise MqaError("mha_prefill_attention", rc)
    return o


def mqa_project_append_qkv(x, P_q, P_k, P_v, K, V, lens_in, lens_out, q=None, stream=None):
    """x [b,d], P_q [h,d,k], P_k [d,k] or [h,d,k], P_v likewise, K/V caches, lens_in/lens_out [b] int32
    (different tensors) -> q [b,h,k]; the new rows are written into the caches."""
    lib = load_library()
    for name, t in (("x", x), ("P_q", P_q), ("P_k", P_k), ("P_v", P_v)):
        _check(t, name, torch.float32)
    _check(K, "K"), _check(V, "V"), _check(lens_in, "lens_in", torch.int32), _check(lens_out, "lens_out", torch.int32)
    b, d = x.shape
    h, _, k = P_q.shape
    v = P_v.shape[-1]
    h_kv = P_k.shape[0] if P_k.dim() == 3 else 1
    cap = K.shape[-2]
    kshape = (b, cap, k) if K.dim() == 3 else (b, h_kv, cap, k)
    if (tuple(P_q.shape) != (h, d, k) or tuple(P_k.shape)[-2:] != (d, k) or tuple(P_v.shape)[-2:] != (d, v)
            or P_v.dim() != P_k.dim() or (K.dim() == 3) != (P_k.dim() == 2) or tuple(K.shape) != kshape
            or tuple(V.shape) != kshape[:-1] + (v,) or K.dtype != V.dtype or lens_in.numel() != b or lens_out.numel() != b):
        raise ValueError("shape mismatch in mqa_project_append_qkv")
    if q is None:
        q = torch.empty((b, h, k), dtype=torch.float32, device=x.device)
    rc = lib.mqa_project_append_qkv(_ptr(x), _ptr(P_q), _ptr(P_k), _ptr(P_v), _ptr(q), _ptr(K), _ptr(V), _ptr(lens_in),
                                    _ptr(lens_out), b, d, h, h_kv, cap, k, v, _cache_dtype(K), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_project_append_qkv", rc)
    return q


def mqa_project_memory_kv(M, P_k, P_v, K, V, lens, mem_lens=None, stream=None):
    """M [b,m,d], P_k [d,k] or [h,d,k], P_v likewise, caches K/V ([b,cap,k] or [b,h,cap,k]), lens [b] int32
    (output), mem_lens [b] int32 or None: projects the whole memory into the caches in one launch."""
    lib = load_library()
    for name, t in (("M", M), ("P_k", P_k), ("P_v", P_v)):
        _check(t, name, torch.float32)
    _check(K, "K"), _check(V, "V"), _check(lens, "lens", torch.int32)
    if mem_lens is not None:
        _check(mem_lens, "mem_lens", torch.int32)
    b, m, d = M.shape
    k, v = P_k.shape[-1], P_v.shape[-1]
    h_kv = P_k.shape[0] if P_k.dim() == 3 else 1
    cap = K.shape[-2]
    kshape = (b, cap, k) if K.dim() == 3 else (b, h_kv, cap, k)
    if (tuple(P_k.shape)[-2:] != (d, k) or tuple(P_v.shape)[-2:] != (d, v) or P_v.dim() != P_k.dim()
            or (K.dim() == 3) != (P_k.dim() == 2) or tuple(K.shape) != kshape or tuple(V.shape) != kshape[:-1] + (v,)
            or K.dtype != V.dtype or lens.numel() != b or (mem_lens is not None and mem_lens.numel() != b)):
        raise ValueError("shape mismatch in mqa_project_memory_kv")
    rc = lib.mqa_project_memory_kv(_ptr(M), _ptr(P_k), _ptr(P_v), _ptr(K), _ptr(V), _ptr(mem_lens), _ptr(lens),
                                   b, m, d, h_kv, cap, k, v, _cache_dtype(K), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_project_memory_kv", rc)


def mqa_memory_decode_step(q, K, V, lens, o=None, scale=1.0, workspace=None, stream=None):
    """q [b,queries,h,k] (the queries of the decoder positions sharing memory i), K [b,cap,k], V [b,cap,v],
    lens [b] -> o [b,queries,h,v]."""
    lib = load_library()
    _check(q, "q", torch.float32), _check(K, "K"), _check(V, "V"), _check(lens, "lens", torch.int32)
    b, nq, h, k = q.shape
    cap, v = V.shape[-2], V.shape[-1]
    if tuple(K.shape) != (b, cap, k) or tuple(V.shape) != (b, cap, v) or K.dtype != V.dtype or lens.numel() != b:
        raise ValueError("shape mismatch in mqa_memory_decode_step")
    if o is None:
        o = torch.empty((b, nq, h, v), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _default_workspace(q.device, mqa_decode_workspace_bytes(b, nq * h, cap, v), stream)
    rc = lib.mqa_memory_decode_step(_ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(o), b, nq, h, cap, k, v, _cache_dtype(K),
                                    float(scale), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream))
    if rc != 0:
        raise MqaError("mqa_memory_decode_step", rc)
    return o


def mqa_decode_beams_workspace_bytes(b, beam, h, cap_src, cap_own, k, v, dt):
    return int(load_library().mqa_decode_beams_workspace_bytes(b, beam, h, cap_src, cap_own, k, v, dt))


def mqa_decode_step_beams(q, K_src, V_src, lens_src, K_own, V_own, lens_own, o=None, scale=1.0,
                          workspace=None, stream=None):
    """q [b,beam,h,k]; K_src [b,cap_src,k], V_src [b,cap_src,v], lens_src [b]; K_own [b,beam,cap_own,k],
    V_own [b,beam,cap_own,v], lens_own [b*beam] -> o [b,beam,h,v]."""
    lib = load_library()
    _check(q, "q", torch.float32), _check(lens_src, "lens_src", torch.int32), _check(lens_own, "lens_own", torch.int32)
    for name, t in (("K_src", K_src), ("V_src", V_src), ("K_own", K_own), ("V_own", V_own)):
        _check(t, name)
    b, beam, h, k = q.shape
    cap_src, v = V_src.shape[-2], V_src.shape[-1]
    cap_own = V_own.shape[-2]
    if (tuple(K_src.shape) != (b, cap_src, k) or tuple(V_src.shape) != (b, cap_src, v)
            or tuple(K_own.shape) != (b, beam, cap_own, k) or tuple(V_own.shape) != (b, beam, cap_own, v)
            or lens_src.numel() != b or lens_own.numel() != b * beam or K_own.dtype != K_src.dtype):
        raise ValueError("shape mismatch in mqa_decode_step_beams")
    dt = _cache_dtype(K_src)
    if o is None:
        o = torch.empty((b, beam, h, v), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _default_workspace(q.device, mqa_decode_beams_workspace_bytes(b, beam, h, cap_src, cap_own, k, v, dt), stream)
    rc = lib.mqa_decode_step_beams(_ptr(q), _ptr(K_src), _ptr(V_src), _ptr(lens_src), _ptr(K_own), _ptr(V_own),
                                   _ptr(lens_own), _ptr(o), b, beam, h, cap_src, cap_own, k, v, dt, float(scale),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_decode_step_beams", rc)
    return o


def mqa_beam_reorder_kv(K_src, V_src, lens_src, parent, K_dst, V_dst, lens_dst, stream=None):
    """K_* [n,cap,k] or [n,h_kv,cap,k], V_* likewise, lens_* [n], parent [n] int32: slot r of the
    destination takes the valid rows and the length of slot parent[r] of the source."""
    lib = load_library()
    for name, t in (("K_src", K_src), ("V_src", V_src), ("K_dst", K_dst), ("V_dst", V_dst)):
        _check(t, name)
    for name, t in (("lens_src", lens_src), ("parent", parent), ("lens_dst", lens_dst)):
        _check(t, name, torch.int32)
    n, cap, k = K_src.shape[0], K_src.shape[-2], K_src.shape[-1]
    v = V_src.shape[-1]
    h_kv = K_src.shape[1] if K_src.dim() == 4 else 1
    if (K_dst.shape != K_src.shape or V_dst.shape != V_src.shape or K_dst.dtype != K_src.dtype
            or V_src.shape[:-1] != K_src.shape[:-1] or lens_src.numel() != n or parent.numel() != n
            or lens_dst.numel() != n):
        raise ValueError("shape mismatch in mqa_beam_reorder_kv")
    rc = lib.mqa_beam_reorder_kv(_ptr(K_src), _ptr(V_src), _ptr(lens_src), _ptr(parent), _ptr(K_dst), _ptr(V_dst),
                                 _ptr(lens_dst), n, h_kv, cap, k, v, _cache_dtype(K_src), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_beam_reorder_kv", rc)


def _project(fn_name, mode, x, P, out, epilogue, stream):
    lib = load_library()
    _check(x, "in", torch.float32), _check(P, "P", torch.float32)
    rows = x.shape[0]
    if mode in (MQA_PROJ_KV, MQA_PROJ_LINEAR):
        d, kv = P.shape
        h, oshape = 1, (rows, kv)
        ok = x.shape == (rows, d)
    elif mode in (MQA_PROJ_Q, MQA_PROJ_KV_MH):
        h, d, kv = P.shape
        oshape = (rows, h, kv)
        ok = x.shape == (rows, d)
    elif mode == MQA_PROJ_O:
        h, d, kv = P.shape
        oshape = (rows, d)
        ok = x.shape == (rows, h, kv)
    else:
        raise ValueError("unknown projection mode")
    if not ok:
        raise ValueError(f"shape mismatch: in {tuple(x.shape)} P {tuple(P.shape)} mode {mode}")
    if out is None:
        if epilogue == MQA_EPI_ADD:
            raise ValueError("MQA_EPI_ADD accumulates into `out`: pass it")
        out = torch.empty(oshape, dtype=torch.float32, device=x.device)
    _check(out, "out", torch.float32)
    if out.numel() != rows * (oshape[1] if len(oshape) == 2 else oshape[1] * oshape[2]):
        raise ValueError("out has the wrong size")
    if epilogue is None:
        rc = lib.mqa_project_qkvo(mode, _ptr(x), _ptr(P), _ptr(out), rows, d, h, kv, _stream(stream))
    else:
        rc = lib.mqa_project_qkvo_ex(mode, _ptr(x), _ptr(P), _ptr(out), rows, d, h, kv, int(epilogue), _stream(stream))
    if rc != 0:
        raise MqaError(fn_name, rc)
    return out


def mqa_project_qkvo(mode, x, P, out=None, stream=None):
    """mode Q/KV_MH: x [rows,d], P [h,d,kv] -> [rows,h,kv];  KV / LINEAR: P [d,kv] -> [rows,kv];
    O: x [rows,h,kv], P [h,d,kv] -> [rows,d]."""
    return _project("mqa_project_qkvo", mode, x, P, out, None, stream)


def mqa_project_qkvo_ex(mode, x, P, out=None, epilogue=MQA_EPI_STORE, stream=None):
    """As mqa_project_qkvo with an epilogue: MQA_EPI_RELU stores max(x, 0), MQA_EPI_ADD adds to `out`."""
    return _project("mqa_project_qkvo_ex", mode, x, P, out, epilogue, stream)


def mqa_stream_read(src, sink, stream=None):
    lib = load_library()
    rc = lib.mqa_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_stream_read", rc)


def mqa_stream_copy(src, dst, stream=None):
    lib = load_library()
    rc = lib.mqa_stream_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream(stream))
    if rc != 0:
        raise MqaError("mqa_stream_copy", rc)


def _rc(name, rc):
    if rc != 0:
        raise MqaError(name, rc)


def mqa_stack_layernorm(x, out=None, eps=1e-6, stream=None):
    _check(x, "x", torch.float32)
    if out is None:
        out = torch.empty_like(x)
    rows, d = x.shape
    _rc("mqa_stack_layernorm", load_library().mqa_stack_layernorm(_ptr(x), _ptr(out), rows, d, float(eps), _stream(stream)))
    return out


def mqa_stack_embed(tokens, positions, E, P, out=None, stream=None):
    _check(tokens, "tokens", torch.int32), _check(positions, "positions", torch.int32)
    _check(E, "E", torch.float32), _check(P, "P", torch.float32)
    rows, d = tokens.numel(), E.shape[1]
    if out is None:
        out = torch.empty((rows, d), dtype=torch.float32, device=E.device)
    if P.shape[1] != d or positions.numel() != rows:
        raise ValueError("size mismatch in mqa_stack_embed")
    _rc("mqa_stack_embed", load_library().mqa_stack_embed(_ptr(tokens), _ptr(positions), _ptr(E), _ptr(P), _ptr(out),
                                                        rows, d, E.shape[0], P.shape[0], _stream(stream)))
    return out


def mqa_stack_add(a, b, stream=None):
    _check(a, "a", torch.float32), _check(b, "b", torch.float32)
    if a.numel() != b.numel():
        raise ValueError("size mismatch in mqa_stack_add")
    _rc("mqa_stack_add", load_library().mqa_stack_add(_ptr(a), _ptr(b), a.numel(), _stream(stream)))
    return a


def mqa_stack_relu(a, stream=None):
    _check(a, "a", torch.float32)
    _rc("mqa_stack_relu", load_library().mqa_stack_relu(_ptr(a), a.numel(), _stream(stream)))
    return a


def mqa_stack_argmax(x, out=None, stream=None):
    _check(x, "x", torch.float32)
    rows, n = x.shape
    if out is None:
        out = torch.empty((rows,), dtype=torch.int32, device=x.device)
    _rc("mqa_stack_argmax", load_library().mqa_stack_argmax(_ptr(x), _ptr(out), rows, n, _stream(stream)))
    return out
