"""Thin ctypes binding of libs2o.so (the C ABI declared in include/s2o.h).

Argument marshalling only: every step of the path runs in the HIP kernels behind the
library.  PyTorch appears only as the owner of device memory and streams.  There is no
CPU fallback: if the library has not been built, loading raises."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs2o.so")

S2O_OK, S2O_EINVAL, S2O_EUNSUPPORTED, S2O_ESCRATCH, S2O_EHIP = 0, -1, -2, -3, -4

STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ("s2o_version", "s2o_strerror", "s2o_last_hip_error", "s2o_plan_sizes", "s2o_plan", "s2o_plan_static",
           "s2o_attention_sizes", "s2o_attention", "s2o_attention_local", "s2o_attention_prefix")


class S2OParams(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("batch", C.c_int32), ("q_heads", C.c_int32),
                ("kv_heads", C.c_int32), ("seq_len", C.c_int32), ("head_dim", C.c_int32),
                ("seg_len", C.c_int32), ("block_m", C.c_int32), ("block_n", C.c_int32),
                ("use_q_perm", C.c_int32), ("stop_mode", C.c_int32), ("softmax_scale", C.c_float),
                ("max_prefix_tiles", C.c_int32), ("non_causal", C.c_int32),
                ("q_stride", C.c_int64 * 3), ("k_stride", C.c_int64 * 3),
                ("v_stride", C.c_int64 * 3), ("o_stride", C.c_int64 * 3)]


class S2OPlanOut(C.Structure):
    _fields_ = [("q_perm", C.c_void_p), ("kv_perm", C.c_void_p), ("s_q", C.c_void_p),
                ("s_k", C.c_void_p), ("q_mean", C.c_void_p), ("k_guide", C.c_void_p),
                ("status", C.c_void_p)]


class S2OError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"s2o error {code}: {msg}")
        self.code = code


_lib = None


def load_library():
    """Load libs2o.so (once).  Import torch first so that both share one HIP runtime."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2602_22575_amd.build` (there is no fallback path)")
    import torch  # noqa: F401  (loads libamdhip64 that libs2o.so resolves against)
    lib = C.CDLL(LIB_PATH)
    lib.s2o_version.restype = C.c_int
    lib.s2o_strerror.restype = C.c_char_p
    lib.s2o_strerror.argtypes = [C.c_int]
    lib.s2o_last_hip_error.restype = C.c_int
    szp = C.POINTER(C.c_size_t)
    lib.s2o_plan_sizes.restype = C.c_int
    lib.s2o_plan_sizes.argtypes = [C.POINTER(S2OParams)] + [szp] * 7
    lib.s2o_plan.restype = C.c_int
    lib.s2o_plan.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(S2OParams), C.POINTER(S2OPlanOut),
                             C.c_void_p, C.c_size_t, C.c_void_p]
    lib.s2o_plan_static.restype = C.c_int
    lib.s2o_plan_static.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(S2OParams), C.POINTER(S2OPlanOut), C.c_void_p]
    lib.s2o_attention_sizes.restype = C.c_int
    lib.s2o_attention_sizes.argtypes = [C.POINTER(S2OParams), szp, szp]
    lib.s2o_attention.restype = C.c_int
    lib.s2o_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(S2OParams),
                                  C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.s2o_attention_prefix.restype = C.c_int
    lib.s2o_attention_prefix.argtypes = lib.s2o_attention.argtypes
    lib.s2o_attention_local.restype = C.c_int
    lib.s2o_attention_local.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(S2OParams),
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    _lib = lib
    return lib


def _check(rc: int):
    if rc != S2O_OK:
        lib = load_library()
        msg = lib.s2o_strerror(rc).decode()
        if rc == S2O_EHIP:
            msg += f" (hipError {lib.s2o_last_hip_error()})"
        raise S2OError(rc, msg)


def make_params(Z, H, Hkv, L, D, S, BM=64, BN=64, use_q_perm=1, stop_mode=0, softmax_scale=0.0,
                q_stride=(0, 0, 0), k_stride=(0, 0, 0), v_stride=(0, 0, 0),
                o_stride=(0, 0, 0), max_prefix_tiles=0, non_causal=0) -> S2OParams:
    p = S2OParams()
    p.struct_size = C.sizeof(S2OParams)
    p.batch, p.q_heads, p.kv_heads, p.seq_len, p.head_dim = Z, H, Hkv, L, D
    p.seg_len, p.block_m, p.block_n = S, BM, BN
    p.use_q_perm, p.stop_mode, p.softmax_scale = use_q_perm, stop_mode, softmax_scale
    p.max_prefix_tiles, p.non_causal = max_prefix_tiles, non_causal
    for name, val in (("q_stride", q_stride), ("k_stride", k_stride), ("v_stride", v_stride),
                      ("o_stride", o_stride)):
        setattr(p, name, (C.c_int64 * 3)(*val))
    return p


def s2o_plan_sizes(params: S2OParams) -> dict:
    lib = load_library()
    v = [C.c_size_t(0) for _ in range(7)]
    _check(lib.s2o_plan_sizes(C.byref(params), *[C.byref(x) for x in v]))
    names = ("q_perm", "kv_perm", "s_q", "s_k", "q_mean", "k_guide", "scratch")
    return {n: int(x.value) for n, x in zip(names, v)}


def s2o_attention_sizes(params: S2OParams) -> dict:
    lib = load_library()
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib.s2o_attention_sizes(C.byref(params), C.byref(a), C.byref(b)))
    return {"counts": int(a.value), "scratch": int(b.value)}


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check_qkv(params: S2OParams, **tensors):
    """The library sees only pointers: refuse tensors it would silently misread (wrong dtype,
    another device, or a memory layout that params' strides do not describe)."""
    import torch
    dev = None
    for name, t in tensors.items():
        if t is None:
            continue
        if t.dtype != torch.bfloat16 or not t.is_cuda:
            raise ValueError(f"{name}: expected a CUDA bfloat16 tensor, got {t.dtype} on {t.device}")
        dev = t.device if dev is None else dev
        if t.device != dev:
            raise ValueError(f"{name}: on {t.device}, the other tensors on {dev}")
        stride = tuple(getattr(params, {"Q": "q_stride", "K": "k_stride", "V": "v_stride", "O": "o_stride"}[name]))
        if stride == (0, 0, 0):
            if not t.is_contiguous():
                raise ValueError(f"{name}: params describe a packed [Z,heads,L,D] tensor but this one is not "
                                 "contiguous (pass its strides in params or call .contiguous())")
        elif t.stride(-1) != 1:
            raise ValueError(f"{name}: the last dimension must be contiguous")


def _keep_alive_on(stream, *tensors):
    """Buffers allocated here and handed to kernels on a stream other than torch's current one
    must not be recycled by the caching allocator before that stream has passed them."""
    if stream is None:
        return
    for t in tensors:
        if t is not None:
            t.record_stream(stream)


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


@dataclass
class Plan:
    q_perm: "object"
    kv_perm: "object"
    s_q: "object" = None
    s_k: "object" = None
    q_mean: "object" = None
    k_guide: "object" = None
    status: "object" = None      # int32[1] on the device: 0, or S2O_PLAN_* bits (see s2o.h)


def s2o_plan(Q, K, params: S2OParams, want_scores: bool = True, scratch=None, stream=None,
             maps=None, static_scratch: bool = False) -> Plan:
    """Step 1.  Q, K: torch CUDA bf16 tensors [Z,H,L,D] / [Z,Hkv,L,D].  Returns device
    tensors; the call is asynchronous on the current (or given) torch stream.
    maps: optional (q_perm [Z,H,N,S], kv_perm [Z,H,max(P,4)]) int32 tensors to write into
    (P = entries of the key rows of one head: S*N(N-1)/2, or N*L when params.non_causal).
    static_scratch: call s2o_plan_static (the library's built-in scratch) instead of s2o_plan."""
    import torch
    lib = load_library()
    _check_qkv(params, Q=Q, K=K)
    sz = s2o_plan_sizes(params)
    dev = Q.device
    Z, H, Hkv, L, D, S = (params.batch, params.q_heads, params.kv_heads, params.seq_len,
                          params.head_dim, params.seg_len)
    N = L // S
    P = N * L if params.non_causal else S * N * (N - 1) // 2
    if maps is not None:
        out = Plan(q_perm=maps[0], kv_perm=maps[1])
        if (out.q_perm.numel() != Z * H * N * S or out.kv_perm.numel() != Z * H * max(P, 4)
                or out.q_perm.dtype != torch.int32 or out.kv_perm.dtype != torch.int32):
            raise ValueError("maps: wrong size or dtype")
    else:
        out = Plan(q_perm=torch.empty((Z, H, N, S), dtype=torch.int32, device=dev),
                   kv_perm=torch.empty((Z, H, max(P, 4)), dtype=torch.int32, device=dev))
    if want_scores:
        out.s_q = torch.empty((Z, H, N, S), dtype=torch.float32, device=dev)
        out.s_k = torch.empty((Z, H, max(P, 4)), dtype=torch.float32, device=dev)
        out.q_mean = torch.empty((Z, H, N, D), dtype=torch.float32, device=dev)
        out.k_guide = torch.empty((Z, Hkv, D), dtype=torch.float32, device=dev)
    own_scratch = scratch is None and not static_scratch
    if own_scratch:
        scratch = torch.empty(sz["scratch"], dtype=torch.uint8, device=dev)
    out.status = torch.empty(1, dtype=torch.int32, device=dev)
    _keep_alive_on(stream, scratch if own_scratch else None, out.status, out.s_q, out.s_k, out.q_mean, out.k_guide,
                   None if maps is not None else out.q_perm, None if maps is not None else out.kv_perm)
    po = S2OPlanOut(_ptr(out.q_perm), _ptr(out.kv_perm), _ptr(out.s_q), _ptr(out.s_k),
                    _ptr(out.q_mean), _ptr(out.k_guide), _ptr(out.status))
    if static_scratch:
        _check(lib.s2o_plan_static(Q.data_ptr(), K.data_ptr(), C.byref(params), C.byref(po), _stream_handle(stream)))
    else:
        _check(lib.s2o_plan(Q.data_ptr(), K.data_ptr(), C.byref(params), C.byref(po),
                            scratch.data_ptr(), scratch.numel(), _stream_handle(stream)))
    if P == 0:
        out.kv_perm = out.kv_perm[:, :, :0]
        if out.s_k is not None:
            out.s_k = out.s_k[:, :, :0]
    else:
        out.kv_perm = out.kv_perm[:, :, :P]
        if out.s_k is not None:
            out.s_k = out.s_k[:, :, :P]
    out._scratch = scratch  # keep alive until the caller synchronises
    return out


def s2o_attention(Q, K, V, params: S2OParams, q_perm, kv_perm, tau: float, O=None,
                  computed=None, skipped=None, stream=None, scratch=None, two_pass=True):
    """Step 2.  Returns (O [Z,H,L,D] bf16, computed, skipped int32 [Z,H,L/B_M]).
    two_pass: launch Alg. 2 and Alg. 3 separately (needs `scratch`, allocated here if not
    given); False: one fused launch."""
    import torch
    lib = load_library()
    _check_qkv(params, Q=Q, K=K, V=V, O=O)
    sz = s2o_attention_sizes(params)
    dev = Q.device
    Z, H, L, D = params.batch, params.q_heads, params.seq_len, params.head_dim
    fresh = []
    if O is None:
        O = torch.empty((Z, H, L, D), dtype=torch.bfloat16, device=dev)
        fresh.append(O)
    if computed is None:
        computed = torch.empty((Z, H, L // params.block_m), dtype=torch.int32, device=dev)
        fresh.append(computed)
    if skipped is None:
        skipped = torch.empty((Z, H, L // params.block_m), dtype=torch.int32, device=dev)
        fresh.append(skipped)
    if two_pass and scratch is None and sz["scratch"] > 0:
        scratch = torch.empty(sz["scratch"], dtype=torch.uint8, device=dev)
        fresh.append(scratch)
    if not two_pass:
        scratch = None
    _keep_alive_on(stream, *fresh)
    _check(lib.s2o_attention(Q.data_ptr(), K.data_ptr(), V.data_ptr(), C.byref(params),
                             _ptr(q_perm), _ptr(kv_perm), float(tau), O.data_ptr(),
                             computed.data_ptr(), skipped.data_ptr(), _ptr(scratch),
                             0 if scratch is None else scratch.numel(), _stream_handle(stream)))
    return O, computed, skipped


def s2o_attention_local(Q, K, V, params: S2OParams, scratch=None, stream=None):
    """Pass 1 (Alg. 2) alone.  Returns the state buffer (uint8 tensor) s2o_attention_prefix reads."""
    import torch
    lib = load_library()
    _check_qkv(params, Q=Q, K=K, V=V)
    if scratch is None:
        scratch = torch.empty(s2o_attention_sizes(params)["scratch"], dtype=torch.uint8, device=Q.device)
        _keep_alive_on(stream, scratch)
    _check(lib.s2o_attention_local(Q.data_ptr(), K.data_ptr(), V.data_ptr(), C.byref(params),
                                   scratch.data_ptr(), scratch.numel(), _stream_handle(stream)))
    return scratch


def s2o_attention_prefix(Q, K, V, params: S2OParams, q_perm, kv_perm, tau: float, scratch, O=None,
                         computed=None, skipped=None, stream=None):
    """Pass 2 (Alg. 3) alone, resuming from the state s2o_attention_local left in `scratch`
    (None when params.non_causal: there is no state)."""
    import torch
    lib = load_library()
    _check_qkv(params, Q=Q, K=K, V=V, O=O)
    dev = Q.device
    Z, H, L, D = params.batch, params.q_heads, params.seq_len, params.head_dim
    fresh = []
    if O is None:
        O = torch.empty((Z, H, L, D), dtype=torch.bfloat16, device=dev)
        fresh.append(O)
    if computed is None:
        computed = torch.empty((Z, H, L // params.block_m), dtype=torch.int32, device=dev)
        fresh.append(computed)
    if skipped is None:
        skipped = torch.empty((Z, H, L // params.block_m), dtype=torch.int32, device=dev)
        fresh.append(skipped)
    _keep_alive_on(stream, *fresh)
    _check(lib.s2o_attention_prefix(Q.data_ptr(), K.data_ptr(), V.data_ptr(), C.byref(params),
                                    _ptr(q_perm), _ptr(kv_perm), float(tau), O.data_ptr(),
                                    computed.data_ptr(), skipped.data_ptr(), _ptr(scratch),
                                    0 if scratch is None else scratch.numel(), _stream_handle(stream)))
    return O, computed, skipped
