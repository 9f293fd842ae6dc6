"""ctypes binding of libturboboa.so: argument marshalling only.

Tensors are torch CUDA tensors (device memory and the stream come from PyTorch-ROCm); every
computation happens inside the library's HIP kernels.  Importing this module without the built
library raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libturboboa.so")

F32, BF16, F64 = 0, 1, 2
GEMM_LOWER, GEMM_CAUSAL_K, GEMM_PERSISTENT, GEMM_A_TILED, GEMM_B_TILED, GEMM_C_TILED, GEMM_F16, GEMM_KLO = 1, 2, 4, 8, 16, 32, 64, 128

STATUS = {0: "OK", -1: "EINVAL", -2: "ENOTSPD", -3: "ENOMEM", -4: "EHIP", -5: "ENAN"}


class TurboBoAError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s: %s" % (STATUS.get(code, code), msg))
        self.code = code


class AttnDesc(C.Structure):
    _fields_ = [("d_model", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("n_seqs", C.c_int), ("seq_len", C.c_int), ("x_dtype", C.c_int), ("causal", C.c_int),
                ("alpha", C.c_double), ("seq_chunk", C.c_int)]


class LayerDesc(C.Structure):
    _fields_ = [("d_out", C.c_int), ("d_in", C.c_int), ("n_heads", C.c_int), ("hin_per_head", C.c_int),
                ("bits", C.c_int), ("block", C.c_int), ("group", C.c_int), ("w_dtype", C.c_int),
                ("cd_iters", C.c_int), ("adaptive_grid", C.c_int), ("grid_points", C.c_int),
                ("max_shrink", C.c_double), ("damp", C.c_double), ("grid_guard", C.c_double)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libturboboa.so is not built (run `python -c 'import __graft_entry__ as g; g.build()'`): "
                          + LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, f64 = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_double
    sigs = {
        "tboa_create": ([C.POINTER(vp), i32, vp], i32),
        "tboa_destroy": ([vp], None),
        "tboa_last_error": ([vp], C.c_char_p),
        "tboa_workspace_bytes": ([vp], C.c_size_t),
        "tboa_reserve_workspace": ([vp, C.c_size_t], i32),
        "tboa_quantize_workspace_bytes": ([C.POINTER(LayerDesc), C.c_int, C.c_int], C.c_size_t),
        "tboa_gemm_f64": ([vp, i32, i32, i32, f64, vp, i64, i64, vp, i64, i64, f64, vp, i64, i32, i64, i64, i64], i32),
        "tboa_gemm_bf16_nt": ([vp, i32, i32, i32, f32, vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i64, i64, i64], i32),
        "tboa_chol_inv_upper": ([vp, i32, i32, vp, f64, vp], i32),
        "tboa_chol_inv_upper_static": ([vp, i32, i32, vp, f64, vp], i32),
        "tboa_chol_inv_upper_static_max_elems": ([], C.c_size_t),
        "tboa_build_hessians": ([vp, C.POINTER(AttnDesc)] + [vp] * 14, i32),
        "tboa_build_hessian_out_proj": ([vp, C.POINTER(AttnDesc)] + [vp] * 11, i32),
        "tboa_fp_cache_bytes": ([C.POINTER(AttnDesc)], C.c_size_t),
        "tboa_hessian_workspace_bytes": ([C.POINTER(AttnDesc)], C.c_size_t),
        "tboa_act_fakequant": ([vp, i64, i32, i32, i32, vp, vp], i32),
        "tboa_hadamard_rotate": ([vp, i64, i32, i32, vp, vp, vp], i32),
        "tboa_build_hessian_linear": ([vp, i64, i32, i32, f64, vp, vp, vp, vp], i32),
        "tboa_swiglu_forward": ([vp, i64, i32, i32, i32, vp, i32, vp, vp, vp], i32),
        "tboa_build_hout": ([vp, i32, i32, i32, i32, vp, i32, vp, vp], i32),
        "tboa_build_hout_q_kv_cache": ([vp, C.POINTER(AttnDesc), vp, vp, i32, vp], i32),
        "tboa_attention_forward": ([vp, C.POINTER(AttnDesc), vp, i32, vp, vp, vp, vp], i32),
        "tboa_linear_forward": ([vp, i64, i32, i32, i32, vp, i32, vp, vp, vp], i32),
        "tboa_packed_words_per_row": ([i32, i32], i64),
        "tboa_pack_codes": ([vp, i32, i32, i32, vp, vp], i32),
        "tboa_dequant_gemv": ([vp, i32, i32, i32, i32, vp, vp, vp, vp, vp], i32),
        "tboa_quantize_layer": ([vp, C.POINTER(LayerDesc)] + [vp] * 8 + [C.POINTER(f64), C.POINTER(f64)], i32),
        "tboa_counter": ([vp, i32], i64),
        "tboa_profile_enable": ([vp, i32], i32),
        "tboa_profile_reset": ([vp], i32),
        "tboa_profile_read": ([vp, i32, C.POINTER(f64), C.POINTER(i64), C.POINTER(f64)], i32),
    }
    missing = [n for n in sigs if not hasattr(lib, n)]
    if missing:
        raise ImportError("libturboboa.so lacks %s: rebuild it" % ", ".join(missing))
    for name, (args, res) in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = res
    return lib


_lib = _load()



def _dtype_code(t):
    return {torch.float32: F32, torch.bfloat16: BF16, torch.float64: F64}[t.dtype]


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev(t, dtype=None):
    assert t.is_cuda and t.is_contiguous(), "expected a contiguous CUDA tensor"
    if dtype is not None:
        assert t.dtype == dtype, "expected %s, got %s" % (dtype, t.dtype)
    return t


class Context:
    """One library context on the current torch device and stream."""

    def __init__(self, device=None, stream=None):
        dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
        self.device = dev
        st = torch.cuda.current_stream(dev) if stream is None else stream
        self._stream = st
        h = C.c_void_p()
        rc = _lib.tboa_create(C.byref(h), dev.index or 0, C.c_void_p(st.cuda_stream))
        if rc != 0:
            raise TurboBoAError(rc, "tboa_create failed")
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.tboa_destroy(self._h)
        self._h = None
        self._fp_cache = None

    __del__ = close

    def _check(self, rc):
        if rc != 0:
            raise TurboBoAError(rc, _lib.tboa_last_error(self._h).decode())

    def counter(self, which):
        """tboa_counter_id: 0 two-phase grid-search passes, 1 quantize_layer calls run again with exact grid-search costs,
        2 unused, 3 near-minimal candidates evaluated exactly, 4 / 5 dequantized weight matrices taken in integer form / split."""
        return int(_lib.tboa_counter(self._h, which))

    def workspace_bytes(self):
        return int(_lib.tboa_workspace_bytes(self._h))

    def reserve_workspace(self, nbytes):
        self._check(_lib.tboa_reserve_workspace(self._h, int(nbytes)))

    @staticmethod
    def layer_desc(W, H_in, n_heads, bits, block, group=0, cd_iters=1, adaptive_grid=True, grid_points=100, max_shrink=0.8,
                   damp=0.01, grid_guard=0.0):
        d_out, d_in = W.shape
        return LayerDesc(d_out, d_in, n_heads, int(H_in.dim() == 3), bits, block, group, _dtype_code(W), cd_iters,
                         int(adaptive_grid), grid_points, max_shrink, damp, grid_guard)

    @staticmethod
    def hessian_workspace_bytes(d_model, n_q_heads, n_kv_heads, head_dim, n_seqs, seq_len, dtype, causal=True, seq_chunk=0):
        desc = AttnDesc(d_model, n_q_heads, n_kv_heads, head_dim, n_seqs, seq_len, {torch.float32: F32, torch.bfloat16: BF16}[dtype],
                        int(causal), 0.0, seq_chunk)
        return int(_lib.tboa_hessian_workspace_bytes(C.byref(desc)))

    @staticmethod
    def quantize_workspace_bytes(desc, with_H_out=True, with_R=True):
        return int(_lib.tboa_quantize_workspace_bytes(C.byref(desc), int(with_H_out), int(with_R)))

    # ---- live kernel timing
    PROF_TAGS = {"hv_syrk": 0, "ax": 1, "rv": 2, "gram": 3, "proj": 4, "grid": 5,
                 "f64_grid": 6, "f64_factor": 7, "f64_sweep": 8, "f64_comp": 9, "f64_cd": 10, "ata": 11, "scores": 12, "pv": 13}

    def profile(self, on=True):
        self._check(_lib.tboa_profile_enable(self._h, int(on)))
        self._check(_lib.tboa_profile_reset(self._h))

    def profile_read(self, tag):
        ms, n, fl = C.c_double(), C.c_int64(), C.c_double()
        self._check(_lib.tboa_profile_read(self._h, self.PROF_TAGS[tag], C.byref(ms), C.byref(n), C.byref(fl)))
        return dict(ms=ms.value, launches=n.value, flops=fl.value)

    # ---- building blocks
    def gemm_f64(self, A, B, C_out=None, alpha=1.0, beta=0.0, transA=False, transB=False):
        """C = alpha op(A) op(B) + beta C for 2-D or batched 3-D fp64 tensors."""
        batched = A.dim() == 3
        A3 = A if batched else A[None]; B3 = B if batched else B[None]
        _dev(A3, torch.float64); _dev(B3, torch.float64)
        bs = A3.shape[0]
        M, K = (A3.shape[2], A3.shape[1]) if transA else (A3.shape[1], A3.shape[2])
        N = B3.shape[1] if transB else B3.shape[2]
        if C_out is None:
            C_out = torch.empty((bs, M, N) if batched else (M, N), dtype=torch.float64, device=A.device)
        lda, ldb = A3.shape[2], B3.shape[2]
        sam, sak = (1, lda) if transA else (lda, 1)
        sbk, sbn = (1, ldb) if transB else (ldb, 1)
        self._check(_lib.tboa_gemm_f64(self._h, M, N, K, alpha, _ptr(A3), sam, sak, _ptr(B3), sbk, sbn, beta,
                                       _ptr(C_out), N, bs, A3.shape[1] * A3.shape[2], B3.shape[1] * B3.shape[2], M * N))
        return C_out

    def gemm_bf16_nt(self, A, B, out_dtype=torch.float32, alpha=1.0, C_out=None, accumulate=False, flags=0):
        """C = alpha A B^T (+ C) for bf16 (or, both, float16: TBOA_GEMM_F16 is then set) A [.., M, K], B [.., N, K]; rows may be
        pitched (views of a wider tensor).  A 16-bit C has the operands' type."""
        batched = A.dim() == 3
        A3 = A if batched else A[None]; B3 = B if batched else B[None]
        for t in (A3, B3):
            assert t.is_cuda and t.dtype == A.dtype and t.dtype in (torch.bfloat16, torch.float16) and t.stride(2) == 1, \
                "expected K-contiguous bf16 or float16 CUDA tensors"
        if A.dtype == torch.float16:
            flags |= GEMM_F16
        bs, M, K = A3.shape; N = B3.shape[1]
        if C_out is None:
            C_out = torch.zeros((bs, M, N) if batched else (M, N), dtype=out_dtype, device=A.device)
        assert C_out.dtype in (torch.float32, A.dtype)
        self._check(_lib.tboa_gemm_bf16_nt(self._h, M, N, K, alpha, _ptr(A3), A3.stride(1), _ptr(B3), B3.stride(1), _ptr(C_out), N,
                                           F32 if C_out.dtype == torch.float32 else BF16, int(accumulate), flags, bs, A3.stride(0), B3.stride(0), M * N))
        return C_out

    def chol_inv_upper(self, H, damp=0.0, out=None, static=False):
        """U = Chol(H^-1)^T for fp32 H [n, n] or [batch, n, n]; returns fp64 (written into `out` when given).
        static: the entry point that allocates nothing (temporaries in the library's static device array; small sizes only)."""
        H3 = _dev(H if H.dim() == 3 else H[None], torch.float32)
        U = torch.empty(H3.shape, dtype=torch.float64, device=H.device) if out is None else _dev(out, torch.float64)
        fn = _lib.tboa_chol_inv_upper_static if static else _lib.tboa_chol_inv_upper
        self._check(fn(self._h, H3.shape[1], H3.shape[0], _ptr(H3), damp, _ptr(U)))
        return U if (H.dim() == 3 or out is not None) else U[0]

    # ---- the method
    def build_hessians(self, X, X_fp, Wq, Wk, Wv, Wo, n_q_heads, n_kv_heads, head_dim, alpha=0.0, causal=True,
                       with_R_v=True, seq_chunk=0, parts="all", keep_fp_projections=False):
        """parts: "all", "qk" (H_in, R, H_out of W_Q and W_K, plus H_out of W_V) or "v" (H_in, R of W_V).
        keep_fp_projections: also returns "fp_cache", the buffer tboa_build_hessian_out_proj can reuse (None when the
        library has no use for one: fp32 inputs, or no R_v).  The buffer belongs to this context and is overwritten by its
        next call with keep_fp_projections."""
        S, L, d = X.shape
        dt = X.dtype
        for t in (X, Wq, Wk, Wv, Wo):
            _dev(t, dt)
        if X_fp is not None:
            _dev(X_fp, dt)
        desc = AttnDesc(d, n_q_heads, n_kv_heads, head_dim, S, L, _dtype_code(X), int(causal), alpha, seq_chunk)
        f = dict(dtype=torch.float32, device=X.device)
        dh = head_dim
        qk, v = parts in ("all", "qk"), parts in ("all", "v")
        out = dict(Hin_qk=None, Hout_q=None, Hout_k=None, Hin_v=None, Hout_v=None, R_qk=None, R_v=None)
        if qk:
            out.update(Hin_qk=torch.empty(d, d, **f), Hout_q=torch.empty(n_q_heads, dh, dh, **f),
                       Hout_k=torch.empty(n_kv_heads, dh, dh, **f), Hout_v=torch.empty(n_kv_heads, dh, dh, **f))
            if X_fp is not None:
                out["R_qk"] = torch.empty(d, d, **f)
        if v:
            out["Hin_v"] = torch.empty(n_kv_heads, d, d, **f)
            if X_fp is not None and with_R_v:
                out["R_v"] = torch.empty(n_kv_heads, d, d, **f)
        cache = None
        if keep_fp_projections and out["R_v"] is not None:
            nbytes = int(_lib.tboa_fp_cache_bytes(C.byref(desc)))
            cache = getattr(self, "_fp_cache", None)      # one buffer per context, reused from block to block
            if nbytes == 0:
                cache = None
            elif cache is None or cache.numel() != nbytes or cache.device != X.device:
                cache = self._fp_cache = torch.empty(nbytes, dtype=torch.uint8, device=X.device)
        self._check(_lib.tboa_build_hessians(self._h, C.byref(desc), _ptr(X), _ptr(X_fp if (qk or out["R_v"] is not None) else None),
                                             _ptr(Wq), _ptr(Wk), _ptr(Wv),
                                             _ptr(Wo), _ptr(out["Hin_qk"]), _ptr(out["R_qk"]), _ptr(out["Hout_q"]),
                                             _ptr(out["Hout_k"]), _ptr(out["Hin_v"]), _ptr(out["R_v"]), _ptr(out["Hout_v"]), _ptr(cache)))
        if keep_fp_projections:
            out["fp_cache"] = cache
        return out

    def build_hessian_out_proj(self, X, X_fp, Wq_deq, Wk_deq, Wv_deq, Wq, Wk, Wv, n_q_heads, n_kv_heads, head_dim,
                               alpha=0.0, causal=True, seq_chunk=0, fp_cache=None):
        S, L, d = X.shape
        for t in (Wq_deq, Wk_deq, Wv_deq):
            _dev(t, torch.float32)
        desc = AttnDesc(d, n_q_heads, n_kv_heads, head_dim, S, L, _dtype_code(X), int(causal), alpha, seq_chunk)
        dq = n_q_heads * head_dim
        Hin_o = torch.empty(dq, dq, dtype=torch.float32, device=X.device)
        R_o = torch.empty_like(Hin_o) if X_fp is not None else None
        self._check(_lib.tboa_build_hessian_out_proj(self._h, C.byref(desc), _ptr(_dev(X)), _ptr(X_fp), _ptr(Wq_deq),
                                                     _ptr(Wk_deq), _ptr(Wv_deq), _ptr(Wq), _ptr(Wk), _ptr(Wv),
                                                     _ptr(Hin_o), _ptr(R_o), _ptr(fp_cache)))
        return Hin_o, R_o

    def act_fakequant(self, X, bits, out=None):
        _dev(X)
        out = torch.empty_like(X) if out is None else out
        d = X.shape[-1]
        self._check(_lib.tboa_act_fakequant(self._h, X.numel() // d, d, bits, _dtype_code(X), _ptr(X), _ptr(out)))
        return out

    def hadamard_rotate(self, X, signs=None, out=None):
        _dev(X)
        if signs is not None:
            _dev(signs, torch.float32)
        out = torch.empty_like(X) if out is None else out
        d = X.shape[-1]
        self._check(_lib.tboa_hadamard_rotate(self._h, X.numel() // d, d, _dtype_code(X), _ptr(X), _ptr(signs), _ptr(out)))
        return out

    def build_hessian_linear(self, X, X_fp=None, alpha=0.0):
        """H_in = X^T X and R = alpha (X - X_fp)^T X of a plain linear layer; X [.., d_in]."""
        _dev(X)
        d = X.shape[-1]
        H = torch.empty(d, d, dtype=torch.float32, device=X.device)
        R = None
        if X_fp is not None:
            _dev(X_fp, X.dtype)
            R = torch.empty_like(H)
        self._check(_lib.tboa_build_hessian_linear(self._h, X.numel() // d, d, _dtype_code(X), alpha, _ptr(X), _ptr(X_fp), _ptr(H), _ptr(R)))
        return H, R

    def swiglu_forward(self, X, Wg, Wu):
        """silu(X Wg^T) * (X Wu^T); Wg, Wu [d_ff, d] in X's type or fp32 (dequantized)."""
        _dev(X); _dev(Wg); _dev(Wu, Wg.dtype)
        d = X.shape[-1]; dff = Wg.shape[0]
        out = torch.empty(*X.shape[:-1], dff, dtype=X.dtype, device=X.device)
        self._check(_lib.tboa_swiglu_forward(self._h, X.numel() // d, d, dff, _dtype_code(X), _ptr(X), _dtype_code(Wg), _ptr(Wg), _ptr(Wu), _ptr(out)))
        return out

    def build_hout(self, H_in, W, n_heads, rep, head_dim):
        """H_out[g] = sum over the rep heads of group g of W_h H_in W_h^T (fp32 [n_heads, dh, dh]); W in fp32 or bf16."""
        _dev(H_in, torch.float32); _dev(W)
        out = torch.empty(n_heads, head_dim, head_dim, dtype=torch.float32, device=W.device)
        self._check(_lib.tboa_build_hout(self._h, H_in.shape[0], n_heads, rep, head_dim, _ptr(H_in), _dtype_code(W), _ptr(W), _ptr(out)))
        return out

    def build_hout_q_kv_cache(self, X, Wk, n_q_heads, n_kv_heads, head_dim, kv_bits):
        """H_out of W_Q,h from the keys of a kv_bits-bit cache (fp32 [Hq, dh, dh]); X [S, L, d] and Wk in one type."""
        _dev(X); _dev(Wk, X.dtype)
        S, L, d = X.shape
        desc = AttnDesc(d, n_q_heads, n_kv_heads, head_dim, S, L, _dtype_code(X), 1, 0.0, 0)
        out = torch.empty(n_q_heads, head_dim, head_dim, dtype=torch.float32, device=X.device)
        self._check(_lib.tboa_build_hout_q_kv_cache(self._h, C.byref(desc), _ptr(X), _ptr(Wk), kv_bits, _ptr(out)))
        return out

    def attention_forward(self, X, Wq, Wk, Wv, n_q_heads, n_kv_heads, head_dim, causal=True):
        """concat_h(A_h V_h) [S, L, Hq dh] of X [S, L, d]; weights in X's type or fp32 (dequantized)."""
        _dev(X); _dev(Wq); _dev(Wk, Wq.dtype); _dev(Wv, Wq.dtype)
        S, L, d = X.shape
        desc = AttnDesc(d, n_q_heads, n_kv_heads, head_dim, S, L, _dtype_code(X), int(causal), 0.0, 0)
        out = torch.empty(S, L, n_q_heads * head_dim, dtype=X.dtype, device=X.device)
        self._check(_lib.tboa_attention_forward(self._h, C.byref(desc), _ptr(X), _dtype_code(Wq), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(out)))
        return out

    def linear_forward(self, X, W, residual=None):
        """X W^T (+ residual); W [d_out, d_in] in X's type or fp32 (dequantized)."""
        _dev(X); _dev(W)
        if residual is not None:
            _dev(residual, X.dtype)
        d_in = X.shape[-1]; d_out = W.shape[0]
        out = torch.empty(*X.shape[:-1], d_out, dtype=X.dtype, device=X.device)
        self._check(_lib.tboa_linear_forward(self._h, X.numel() // d_in, d_in, d_out, _dtype_code(X), _ptr(X), _dtype_code(W), _ptr(W),
                                             _ptr(residual), _ptr(out)))
        return out

    def pack_codes(self, codes, bits):
        """uint8 codes [d_out, d_in] -> int32 tensor [d_out, ceil(d_in * bits / 32)] holding the little-endian bit stream."""
        _dev(codes, torch.uint8)
        d_out, d_in = codes.shape
        wpr = int(_lib.tboa_packed_words_per_row(d_in, bits))
        packed = torch.empty(d_out, max(wpr, 1), dtype=torch.int32, device=codes.device)
        self._check(_lib.tboa_pack_codes(self._h, d_out, d_in, bits, _ptr(codes), _ptr(packed)))
        return packed

    def dequant_gemv(self, packed, scales, zeros, x, d_in, bits, group=0):
        _dev(packed, torch.int32); _dev(scales, torch.float32); _dev(zeros, torch.float32); _dev(x, torch.float32)
        d_out = packed.shape[0]
        y = torch.empty(d_out, dtype=torch.float32, device=x.device)
        self._check(_lib.tboa_dequant_gemv(self._h, d_out, d_in, bits, group, _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(x), _ptr(y)))
        return y

    def quantize_layer(self, W, H_in, H_out, R, n_heads, bits, block, group=0, cd_iters=1, adaptive_grid=True,
                       grid_points=100, max_shrink=0.8, damp=0.01, grid_guard=0.0):
        """grid_guard: see tboa_layer_desc (0: default; negative: fp64 costs for every grid candidate)."""
        _dev(W); _dev(H_in, torch.float32)
        d_out, d_in = W.shape
        ng = d_in // group if group else 1
        desc = self.layer_desc(W, H_in, n_heads, bits, block, group, cd_iters, adaptive_grid, grid_points, max_shrink, damp, grid_guard)
        dev = W.device
        codes = torch.empty(d_out, d_in, dtype=torch.uint8, device=dev)
        scales = torch.empty(d_out, ng, dtype=torch.float32, device=dev)
        zeros = torch.empty(d_out, ng, dtype=torch.float32, device=dev)
        W_deq = torch.empty(d_out, d_in, dtype=torch.float32, device=dev)
        loss = (C.c_double * 2)()
        lph = (C.c_double * (2 * n_heads))()
        if H_out is not None:
            _dev(H_out, torch.float32)
        if R is not None:
            _dev(R, torch.float32)
        self._check(_lib.tboa_quantize_layer(self._h, C.byref(desc), _ptr(W), _ptr(H_in), _ptr(H_out), _ptr(R),
                                             _ptr(codes), _ptr(scales), _ptr(zeros), _ptr(W_deq), loss, lph))
        terms = [(lph[2 * h], lph[2 * h + 1]) for h in range(n_heads)]
        return dict(codes=codes, scales=scales, zeros=zeros, W_deq=W_deq, loss_quad=loss[0], loss_cross=loss[1],
                    loss=loss[0] + loss[1], loss_per_head=[q + c for q, c in terms], loss_per_head_terms=terms)
