"""ctypes binding of libcassandra_hip.so: same names as include/cassandra.h, argument
marshalling only.  torch tensors provide device memory and the stream; every step of the
path runs in the HIP kernels.  Loading fails loudly if the library has not been built."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcassandra_hip.so")

CAS_OK, CAS_EINVAL, CAS_ENOTSUP, CAS_ENOMEM, CAS_EHIP = 0, -1, -2, -3, -4
CAS_EXP_RAW, CAS_EXP_SHARED = 0, 2   # cas_fmt.exp_mode


class CasError(RuntimeError):
    def __init__(self, code, what, hip=0):
        super().__init__(f"{what}: error {code} ({_lib().cas_strerror(code).decode()})"
                         + (f", hip error {hip}" if hip else ""))
        self.code = code


class cas_fmt(C.Structure):
    _fields_ = [("keep_permille", C.c_int32), ("trunc_bits", C.c_int32), ("exp_mode", C.c_int32)]


class cas_wdesc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("K", C.c_int32), ("t", C.c_int32),
                ("bw", C.c_int32), ("sw", C.c_int32), ("lw", C.c_int32), ("pw", C.c_int32),
                ("off_bitmap", C.c_int64), ("off_spec", C.c_int64),
                ("off_lo", C.c_int64), ("off_pruned", C.c_int64),
                ("spec_bytes", C.c_int64), ("verif_bytes", C.c_int64)]


class cas_udesc(C.Structure):
    _fields_ = [("base", cas_wdesc), ("smw", C.c_int32), ("reserved", C.c_int32),
                ("off_bitmap", C.c_int64), ("off_sm", C.c_int64), ("off_table", C.c_int64),
                ("off_rowoff", C.c_int64), ("off_ue", C.c_int64), ("ue_words", C.c_int64),
                ("spec_bytes", C.c_int64), ("exp_of_rank", C.c_uint8 * 256)]


class cas_kv_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_tokens", C.c_int32), ("n_pages", C.c_int32), ("max_seqs", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("fmt", cas_fmt),
                ("K", C.c_int32), ("sw", C.c_int32), ("lw", C.c_int32), ("pw", C.c_int32),
                ("tile_spec_bytes", C.c_int64), ("tile_verif_bytes", C.c_int64),
                ("spec_pool_bytes", C.c_int64), ("verif_pool_bytes", C.c_int64)]


class cas_model_cfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_layers", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("max_cols", C.c_int32), ("max_pos", C.c_int32), ("rms_eps", C.c_float), ("max_seqs", C.c_int32)]


class cas_tensor(C.Structure):
    _fields_ = [("desc", cas_wdesc), ("d_spec", C.c_void_p), ("d_verif", C.c_void_p)]


class cas_mxdesc(C.Structure):
    _fields_ = [("base", cas_wdesc), ("fw", C.c_int32), ("ew", C.c_int32),
                ("off_bitmap", C.c_int64), ("off_sexp", C.c_int64), ("off_field", C.c_int64),
                ("off_lo", C.c_int64), ("off_pruned", C.c_int64),
                ("spec_bytes", C.c_int64), ("verif_bytes", C.c_int64)]


class cas_layer_weights(C.Structure):
    _fields_ = [("wqkv", cas_tensor), ("wo", cas_tensor), ("wgu", cas_tensor), ("wd", cas_tensor),
                ("d_g_attn", C.c_void_p), ("d_g_ffn", C.c_void_p)]


class cas_model_weights(C.Structure):
    _fields_ = [("layers", C.POINTER(cas_layer_weights)), ("lm_head", cas_tensor), ("d_embed", C.c_void_p),
                ("d_g_final", C.c_void_p), ("d_rope", C.c_void_p)]


_LIB = None

_SIGNATURES = {
    "cas_ctx_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_size_t]),
    "cas_ctx_destroy": (C.c_int, [C.c_void_p]),
    "cas_strerror": (C.c_char_p, [C.c_int]),
    "cas_last_hip_error": (C.c_int, [C.c_void_p]),
    "cas_prof_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "cas_prof_read": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                C.POINTER(C.c_double)]),
    "cas_prof_reset": (C.c_int, [C.c_void_p]),
    "cas_weight_desc": (C.c_int, [C.c_int64, C.c_int64, C.POINTER(cas_fmt), C.POINTER(cas_wdesc)]),
    "cas_encode_weight": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(cas_wdesc),
                                    C.c_void_p, C.c_void_p]),
    "cas_decode_weight": (C.c_int, [C.c_void_p, C.POINTER(cas_wdesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_int64]),
    "cas_gemv_draft": (C.c_int, [C.c_void_p, C.POINTER(cas_wdesc), C.c_void_p, C.c_void_p, C.c_int,
                                 C.c_void_p]),
    "cas_gemv_draft_fused": (C.c_int, [C.c_void_p, C.POINTER(cas_wdesc), C.c_void_p, C.c_void_p, C.c_int,
                                       C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_void_p]),
    "cas_gemm_verify": (C.c_int, [C.c_void_p, C.POINTER(cas_wdesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_int, C.c_void_p]),
    "cas_kv_desc_init": (C.c_int, [C.POINTER(cas_kv_desc)]),
    "cas_kv_create": (C.c_int, [C.POINTER(cas_kv_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                C.POINTER(C.c_void_p)]),
    "cas_kv_destroy": (C.c_int, [C.c_void_p]),
    "cas_kv_append": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int]),
    "cas_kv_set_len": (C.c_int, [C.c_void_p, C.c_int, C.c_int32]),
    "cas_kv_len": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int32)]),
    "cas_kv_read": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                              C.c_void_p, C.c_void_p]),
    "cas_attention": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int,
                                C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]),
    "cas_attention_multi": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int32), C.c_int,
                                      C.POINTER(C.c_void_p), C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_void_p),
                                      C.POINTER(C.c_void_p), C.POINTER(C.c_int32), C.POINTER(C.c_void_p)]),
    "cas_attention_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int,
                                       C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]),
    "cas_attention_static_capacity": (C.c_size_t, []),
    "cas_model_act_bytes": (C.c_int, [C.POINTER(cas_model_cfg), C.POINTER(C.c_size_t)]),
    "cas_model_create": (C.c_int, [C.POINTER(cas_model_cfg), C.POINTER(cas_model_weights), C.c_void_p, C.c_size_t,
                                   C.POINTER(C.c_void_p)]),
    "cas_model_destroy": (C.c_int, [C.c_void_p]),
    "cas_draft_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                 C.c_void_p]),
    "cas_verify_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                  C.c_void_p]),
    "cas_commit": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]),
    "cas_draft_step_multi": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]),
    "cas_verify_step_multi": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]),
    "cas_spec_round": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int,
                                 C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "cas_spec_round_multi": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "cas_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int]),
    "cas_accept_sampling": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int,
                                      C.POINTER(C.c_int32)]),
    "cas_accept": (C.c_int, [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32),
                             C.POINTER(C.c_int32)]),
    "cas_objective": (C.c_int, [C.c_double, C.c_double, C.c_int, C.c_int, C.c_double, C.c_int, C.c_int, C.c_int,
                                C.POINTER(C.c_double)]),
    "cas_tune_grid": (C.c_int, [C.POINTER(C.c_double), C.c_int, C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32),
                                C.c_double, C.c_double, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32),
                                C.POINTER(C.c_int32)]),
    "cas_speed_model": (C.c_int, [C.c_double, C.c_int, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double),
                                  C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "cas_tune_measured": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int,
                                    C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.POINTER(C.c_double)]),
    "cas_dense_decode_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_void_p]),
    "cas_token_probs": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "cas_spec_round_sampling_scratch_floats": (C.c_size_t, [C.c_int, C.c_int]),
    "cas_spec_round_sampling": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int,
                                          C.POINTER(C.c_double), C.c_void_p, C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "cas_unary_plan": (C.c_int, [C.c_void_p, C.POINTER(cas_wdesc), C.c_void_p, C.POINTER(cas_udesc)]),
    "cas_unary_encode": (C.c_int, [C.c_void_p, C.POINTER(cas_udesc), C.c_void_p, C.c_void_p]),
    "cas_unary_decode": (C.c_int, [C.c_void_p, C.POINTER(cas_udesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]),
    "cas_gemv_draft_unary": (C.c_int, [C.c_void_p, C.POINTER(cas_udesc), C.c_void_p, C.c_void_p, C.c_void_p]),
    "cas_model_use_unary": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(cas_udesc), C.c_void_p]),
    "cas_gemm_verify_unary": (C.c_int, [C.c_void_p, C.POINTER(cas_udesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                      C.c_void_p]),
    "cas_gemv_bf16": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "cas_mx_plan": (C.c_int, [C.POINTER(cas_wdesc), C.POINTER(cas_mxdesc)]),
    "cas_mx_encode": (C.c_int, [C.c_void_p, C.POINTER(cas_mxdesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "cas_mx_decode": (C.c_int, [C.c_void_p, C.POINTER(cas_mxdesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]),
    "cas_gemv_draft_mx": (C.c_int, [C.c_void_p, C.POINTER(cas_mxdesc), C.c_void_p, C.c_void_p, C.c_void_p]),
    "cas_gemm_verify_mx": (C.c_int, [C.c_void_p, C.POINTER(cas_mxdesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                   C.c_void_p]),
    "cas_model_use_mx": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(cas_mxdesc), C.c_void_p, C.c_void_p]),
}


def exported_names():
    return sorted(_SIGNATURES)


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -c 'import __graft_entry__ as g; g.build()'` (no CPU fallback exists)")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


class Context:
    """Owns a cas_ctx bound to the current torch stream."""

    def __init__(self, workspace=None):
        import torch
        self._torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("the Cassandra HIP path needs a GPU; there is no CPU fallback")
        self.workspace = workspace
        h = C.c_void_p()
        stream = torch.cuda.current_stream().cuda_stream
        ws_ptr = _ptr(workspace)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        rc = _lib().cas_ctx_create(C.byref(h), C.c_void_p(stream), ws_ptr, ws_bytes)
        if rc != CAS_OK:
            raise CasError(rc, "cas_ctx_create")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            _lib().cas_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != CAS_OK:
            raise CasError(rc, what, _lib().cas_last_hip_error(self.h))


PROF_GEMV_DRAFT, PROF_GEMM_VERIFY, PROF_ATTN_DRAFT, PROF_ATTN_VERIFY = 0, 1, 2, 3


def cas_prof_enable(ctx: Context, on: bool):
    ctx._check(_lib().cas_prof_enable(ctx.h, 1 if on else 0), "cas_prof_enable")


def cas_prof_read(ctx: Context, kernel_class: int):
    n, ms, by = C.c_int64(), C.c_double(), C.c_double()
    ctx._check(_lib().cas_prof_read(ctx.h, kernel_class, C.byref(n), C.byref(ms), C.byref(by)), "cas_prof_read")
    return n.value, ms.value, by.value


def cas_prof_reset(ctx: Context):
    ctx._check(_lib().cas_prof_reset(ctx.h), "cas_prof_reset")


def cas_weight_desc(rows, cols, keep_permille, trunc_bits, exp_mode=0):
    fmt = cas_fmt(keep_permille, trunc_bits, exp_mode)
    d = cas_wdesc()
    rc = _lib().cas_weight_desc(rows, cols, C.byref(fmt), C.byref(d))
    if rc != CAS_OK:
        raise CasError(rc, "cas_weight_desc")
    return d


class EncodedWeight:
    """Descriptor + the two device buffers (uint8 torch tensors) of one encoded matrix."""

    def __init__(self, desc, spec, verif):
        self.desc, self.spec, self.verif = desc, spec, verif


def cas_encode_weight(ctx: Context, W, keep_permille, trunc_bits, act_norm=None) -> EncodedWeight:
    """W: torch int16/uint16/bfloat16 [rows, cols] on the GPU (bf16 bit patterns)."""
    torch = ctx._torch
    assert W.is_cuda and W.dim() == 2 and W.element_size() == 2 and W.stride(1) == 1
    rows, cols = W.shape
    d = cas_weight_desc(rows, cols, keep_permille, trunc_bits)
    spec = torch.empty(d.spec_bytes, dtype=torch.uint8, device=W.device)
    verif = torch.empty(d.verif_bytes, dtype=torch.uint8, device=W.device)
    ctx._check(_lib().cas_encode_weight(ctx.h, _ptr(W), W.stride(0), _ptr(act_norm), C.byref(d), _ptr(spec),
                                        _ptr(verif)), "cas_encode_weight")
    return EncodedWeight(d, spec, verif)


def cas_objective(alpha, s_w, w_keep_permille, w_trunc_bits, s_kv, kv_keep_permille, kv_trunc_bits, b_bits=16):
    j = C.c_double()
    rc = _lib().cas_objective(alpha, s_w, w_keep_permille, w_trunc_bits, s_kv, kv_keep_permille, kv_trunc_bits, b_bits,
                              C.byref(j))
    if rc != CAS_OK:
        raise CasError(rc, "cas_objective")
    return j.value


def cas_tune_grid(alpha, keep_permille, trunc_bits, s_w, s_kv, kv_keep_permille, kv_trunc_bits, b_bits=16):
    """alpha: [len(keep_permille)][len(trunc_bits)] nested sequence; returns (keep index, trunc index)."""
    nk, nt = len(keep_permille), len(trunc_bits)
    flat = (C.c_double * (nk * nt))(*[float(alpha[i][j]) for i in range(nk) for j in range(nt)])
    kp = (C.c_int32 * nk)(*keep_permille)
    tb = (C.c_int32 * nt)(*trunc_bits)
    bi, bj = C.c_int32(), C.c_int32()
    rc = _lib().cas_tune_grid(flat, nk, kp, nt, tb, s_w, s_kv, kv_keep_permille, kv_trunc_bits, b_bits,
                              C.byref(bi), C.byref(bj))
    if rc != CAS_OK:
        raise CasError(rc, "cas_tune_grid")
    return bi.value, bj.value


def cas_speed_model(alpha, gamma, t_draft, t_verify, t_plain=0.0):
    """Returns (tokens per round, tokens per second, speedup over plain decoding)."""
    n, r, sp = C.c_double(), C.c_double(), C.c_double()
    rc = _lib().cas_speed_model(float(alpha), int(gamma), float(t_draft), float(t_verify), float(t_plain),
                                C.byref(n), C.byref(r), C.byref(sp))
    if rc != CAS_OK:
        raise CasError(rc, "cas_speed_model")
    return n.value, r.value, sp.value


def cas_tune_measured(alpha, t_draft, t_verify, gamma):
    """alpha, t_draft, t_verify: [n_keep][n_trunc] nested sequences; returns
    ((keep index, trunc index), tokens per second of every grid point as nested lists)."""
    nk, nt = len(alpha), len(alpha[0])
    flat = lambda a: (C.c_double * (nk * nt))(*[float(a[i][j]) for i in range(nk) for j in range(nt)])
    rates = (C.c_double * (nk * nt))()
    bi, bj = C.c_int32(), C.c_int32()
    rc = _lib().cas_tune_measured(flat(alpha), flat(t_draft), flat(t_verify), nk, nt, int(gamma), C.byref(bi),
                                  C.byref(bj), rates)
    if rc != CAS_OK:
        raise CasError(rc, "cas_tune_measured")
    return (bi.value, bj.value), [[rates[i * nt + j] for j in range(nt)] for i in range(nk)]


class UnaryWeight:
    """Unary-exponent form of an encoded matrix: descriptor, the unary speculation buffer and
    the (shared) verification buffer."""

    def __init__(self, desc, uspec, verif):
        self.desc, self.uspec, self.verif = desc, uspec, verif


def cas_unary_plan(ctx: Context, ew: EncodedWeight) -> cas_udesc:
    u = cas_udesc()
    ctx._check(_lib().cas_unary_plan(ctx.h, C.byref(ew.desc), _ptr(ew.spec), C.byref(u)), "cas_unary_plan")
    return u


def cas_unary_encode(ctx: Context, ew: EncodedWeight, udesc=None) -> UnaryWeight:
    torch = ctx._torch
    u = udesc if udesc is not None else cas_unary_plan(ctx, ew)
    uspec = torch.empty(u.spec_bytes, dtype=torch.uint8, device=ew.spec.device)
    ctx._check(_lib().cas_unary_encode(ctx.h, C.byref(u), _ptr(ew.spec), _ptr(uspec)), "cas_unary_encode")
    return UnaryWeight(u, uspec, ew.verif)


def cas_unary_decode(ctx: Context, uw: UnaryWeight, full: bool):
    torch = ctx._torch
    d = uw.desc.base
    out = torch.empty((d.rows, d.cols), dtype=torch.int16, device=uw.uspec.device)
    ctx._check(_lib().cas_unary_decode(ctx.h, C.byref(uw.desc), _ptr(uw.uspec), _ptr(uw.verif) if full else None,
                                       _ptr(out), d.cols), "cas_unary_decode")
    return out


def cas_gemv_draft_unary(ctx: Context, uw: UnaryWeight, x, out=None):
    """x: bf16 bits [cols] or [1, cols] -> float32 [rows]."""
    torch = ctx._torch
    d = uw.desc.base
    assert x.numel() == d.cols and x.is_contiguous() and x.element_size() == 2
    if out is None:
        out = torch.empty(d.rows, dtype=torch.float32, device=x.device)
    ctx._check(_lib().cas_gemv_draft_unary(ctx.h, C.byref(uw.desc), _ptr(uw.uspec), _ptr(x), _ptr(out)),
               "cas_gemv_draft_unary")
    return out


def cas_gemm_verify_unary(ctx: Context, uw: UnaryWeight, X, out=None):
    """X: bf16 bits [ncols, cols] -> float32 [ncols, rows], W exact, read from the unary form."""
    torch = ctx._torch
    d = uw.desc.base
    assert X.dim() == 2 and X.shape[1] == d.cols and X.is_contiguous() and X.element_size() == 2
    if out is None:
        out = torch.empty((X.shape[0], d.rows), dtype=torch.float32, device=X.device)
    ctx._check(_lib().cas_gemm_verify_unary(ctx.h, C.byref(uw.desc), _ptr(uw.uspec), _ptr(uw.verif), _ptr(X),
                                            X.shape[0], _ptr(out)), "cas_gemm_verify_unary")
    return out


def cas_gemv_bf16(ctx: Context, W, x, out=None):
    """Dense baseline: W bf16 bits [rows, cols] (row-major), x bf16 bits [cols] -> float32 [rows]."""
    torch = ctx._torch
    assert W.dim() == 2 and W.is_contiguous() and W.element_size() == 2 and x.numel() == W.shape[1]
    if out is None:
        out = torch.empty(W.shape[0], dtype=torch.float32, device=W.device)
    ctx._check(_lib().cas_gemv_bf16(ctx.h, _ptr(W), W.shape[0], W.shape[1], W.shape[1], _ptr(x), _ptr(out)),
               "cas_gemv_bf16")
    return out


class MxWeight:
    """Shared-exponent form of an encoded matrix: descriptor and its two buffers."""

    def __init__(self, desc, spec, verif):
        self.desc, self.spec, self.verif = desc, spec, verif


def cas_mx_plan(desc: cas_wdesc) -> cas_mxdesc:
    m = cas_mxdesc()
    rc = _lib().cas_mx_plan(C.byref(desc), C.byref(m))
    if rc != CAS_OK:
        raise CasError(rc, "cas_mx_plan")
    return m


def cas_mx_encode(ctx: Context, ew: EncodedWeight) -> MxWeight:
    torch = ctx._torch
    m = cas_mx_plan(ew.desc)
    spec = torch.empty(m.spec_bytes, dtype=torch.uint8, device=ew.spec.device)
    verif = torch.empty(m.verif_bytes, dtype=torch.uint8, device=ew.spec.device)
    ctx._check(_lib().cas_mx_encode(ctx.h, C.byref(m), _ptr(ew.spec), _ptr(ew.verif), _ptr(spec), _ptr(verif)),
               "cas_mx_encode")
    return MxWeight(m, spec, verif)


def cas_mx_decode(ctx: Context, mw: MxWeight, full: bool):
    torch = ctx._torch
    d = mw.desc.base
    out = torch.empty((d.rows, d.cols), dtype=torch.int16, device=mw.spec.device)
    ctx._check(_lib().cas_mx_decode(ctx.h, C.byref(mw.desc), _ptr(mw.spec), _ptr(mw.verif) if full else None,
                                    _ptr(out), d.cols), "cas_mx_decode")
    return out


def cas_gemv_draft_mx(ctx: Context, mw: MxWeight, x, out=None):
    """x: bf16 bits [cols] or [1, cols] -> float32 [rows]."""
    torch = ctx._torch
    d = mw.desc.base
    assert x.numel() == d.cols and x.is_contiguous() and x.element_size() == 2
    if out is None:
        out = torch.empty(d.rows, dtype=torch.float32, device=x.device)
    ctx._check(_lib().cas_gemv_draft_mx(ctx.h, C.byref(mw.desc), _ptr(mw.spec), _ptr(x), _ptr(out)),
               "cas_gemv_draft_mx")
    return out


def cas_gemm_verify_mx(ctx: Context, mw: MxWeight, X, out=None):
    """X: bf16 bits [ncols, cols] -> float32 [ncols, rows]; the weight is the converted matrix."""
    torch = ctx._torch
    d = mw.desc.base
    assert X.dim() == 2 and X.shape[1] == d.cols and X.is_contiguous() and X.element_size() == 2
    if out is None:
        out = torch.empty((X.shape[0], d.rows), dtype=torch.float32, device=X.device)
    ctx._check(_lib().cas_gemm_verify_mx(ctx.h, C.byref(mw.desc), _ptr(mw.spec), _ptr(mw.verif), _ptr(X), X.shape[0],
                                         _ptr(out)), "cas_gemm_verify_mx")
    return out


def cas_decode_weight(ctx: Context, ew: EncodedWeight, full: bool):
    torch = ctx._torch
    out = torch.empty((ew.desc.rows, ew.desc.cols), dtype=torch.int16, device=ew.spec.device)
    ctx._check(_lib().cas_decode_weight(ctx.h, C.byref(ew.desc), _ptr(ew.spec), _ptr(ew.verif) if full else None,
                                        _ptr(out), ew.desc.cols), "cas_decode_weight")
    return out


def cas_gemv_draft(ctx: Context, ew: EncodedWeight, x, out=None):
    """x: bf16 bits [batch, cols] -> float32 [batch, rows]."""
    torch = ctx._torch
    assert x.dim() == 2 and x.shape[1] == ew.desc.cols and x.is_contiguous() and x.element_size() == 2
    if out is None:
        out = torch.empty((x.shape[0], ew.desc.rows), dtype=torch.float32, device=x.device)
    ctx._check(_lib().cas_gemv_draft(ctx.h, C.byref(ew.desc), _ptr(ew.spec), _ptr(x), x.shape[0], _ptr(out)),
               "cas_gemv_draft")
    return out


def cas_gemv_draft_fused(ctx: Context, ew: EncodedWeight, x, y=None, gain=None, eps=0.0, epilogue=0, out16=None):
    """Fused form: optional RMSNorm of x (gain), epilogue 0 = fp32 y, 1 = residual into out16,
    2 = SwiGLU of row pairs into out16."""
    ctx._check(_lib().cas_gemv_draft_fused(ctx.h, C.byref(ew.desc), _ptr(ew.spec), _ptr(x), x.shape[0], _ptr(y),
                                           _ptr(gain), eps, epilogue, _ptr(out16)), "cas_gemv_draft_fused")
    return y if epilogue == 0 else out16


def cas_gemm_verify(ctx: Context, ew: EncodedWeight, X, out=None):
    """X: bf16 bits [ncols, cols] -> float32 [ncols, rows]."""
    torch = ctx._torch
    assert X.dim() == 2 and X.shape[1] == ew.desc.cols and X.is_contiguous() and X.element_size() == 2
    if out is None:
        out = torch.empty((X.shape[0], ew.desc.rows), dtype=torch.float32, device=X.device)
    ctx._check(_lib().cas_gemm_verify(ctx.h, C.byref(ew.desc), _ptr(ew.spec), _ptr(ew.verif), _ptr(X), X.shape[0],
                                      _ptr(out)), "cas_gemm_verify")
    return out


def cas_accept_sampling(p, q, r):
    g = len(r)
    arr = lambda v: (C.c_double * max(g, 1))(*[float(x) for x in v])
    n = C.c_int32()
    rc = _lib().cas_accept_sampling(arr(p), arr(q), arr(r), g, C.byref(n))
    if rc != CAS_OK:
        raise CasError(rc, "cas_accept_sampling")
    return n.value


def cas_accept(draft, target):
    k = len(draft)
    d = (C.c_int32 * max(k, 1))(*[int(v) for v in draft])
    t = (C.c_int32 * (k + 1))(*[int(v) for v in target])
    n = C.c_int32()
    out = (C.c_int32 * (k + 1))()
    rc = _lib().cas_accept(d, t, k, C.byref(n), out)
    if rc != CAS_OK:
        raise CasError(rc, "cas_accept")
    return n.value, [out[i] for i in range(n.value + 1)]


class KVCache:
    """Pools, page table and the cas_kv handle of a compressed paged cache."""

    def __init__(self, ctx: Context, n_layers, n_kv_heads, n_pages, max_seqs, max_pages_per_seq,
                 keep_permille=600, trunc_bits=4, head_dim=128, page_tokens=64, page_table=None, exp_mode=0):
        torch = ctx._torch
        d = cas_kv_desc()
        d.n_layers, d.n_kv_heads, d.head_dim, d.page_tokens = n_layers, n_kv_heads, head_dim, page_tokens
        d.n_pages, d.max_seqs, d.max_pages_per_seq = n_pages, max_seqs, max_pages_per_seq
        d.fmt = cas_fmt(keep_permille, trunc_bits, exp_mode)   # CAS_EXP_RAW or CAS_EXP_SHARED
        rc = _lib().cas_kv_desc_init(C.byref(d))
        if rc != CAS_OK:
            raise CasError(rc, "cas_kv_desc_init")
        self.desc = d
        self.ctx = ctx
        self.spec_pool = torch.empty(d.spec_pool_bytes, dtype=torch.uint8, device="cuda")
        self.verif_pool = torch.empty(d.verif_pool_bytes, dtype=torch.uint8, device="cuda")
        if page_table is None:
            assert max_seqs * max_pages_per_seq <= n_pages
            page_table = torch.arange(max_seqs * max_pages_per_seq, dtype=torch.int32).reshape(
                max_seqs, max_pages_per_seq)
        self.page_table = page_table.to(device="cuda", dtype=torch.int32).contiguous()
        h = C.c_void_p()
        rc = _lib().cas_kv_create(C.byref(d), _ptr(self.spec_pool), _ptr(self.verif_pool), _ptr(self.page_table),
                                  C.byref(h))
        if rc != CAS_OK:
            raise CasError(rc, "cas_kv_create")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            _lib().cas_kv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cas_kv_append(ctx: Context, kv: KVCache, layer, seq, K, V):
    """K, V: bf16 bits [n_tok, n_kv_heads, head_dim]."""
    assert K.is_contiguous() and V.is_contiguous() and K.shape == V.shape
    ctx._check(_lib().cas_kv_append(ctx.h, kv.h, layer, seq, _ptr(K), _ptr(V), K.shape[0]), "cas_kv_append")


def cas_kv_set_len(kv: KVCache, seq, length):
    rc = _lib().cas_kv_set_len(kv.h, seq, length)
    if rc != CAS_OK:
        raise CasError(rc, "cas_kv_set_len")


def cas_kv_len(kv: KVCache, seq):
    n = C.c_int32()
    rc = _lib().cas_kv_len(kv.h, seq, C.byref(n))
    if rc != CAS_OK:
        raise CasError(rc, "cas_kv_len")
    return n.value


def cas_kv_read(ctx: Context, kv: KVCache, layer, seq, pos0, n_tok, full):
    torch = ctx._torch
    shp = (n_tok, kv.desc.n_kv_heads, kv.desc.head_dim)
    K = torch.empty(shp, dtype=torch.int16, device="cuda")
    V = torch.empty(shp, dtype=torch.int16, device="cuda")
    ctx._check(_lib().cas_kv_read(ctx.h, kv.h, layer, seq, pos0, n_tok, 1 if full else 0, _ptr(K), _ptr(V)),
               "cas_kv_read")
    return K, V


def cas_attention(ctx: Context, kv: KVCache, layer, seq, full, Q, Knew, Vnew, out=None):
    """Q: bf16 bits [ncols, n_q_heads, 128]; Knew/Vnew: [n_new, n_kv_heads, 128]."""
    torch = ctx._torch
    assert Q.is_contiguous() and Knew.is_contiguous() and Vnew.is_contiguous()
    if out is None:
        out = torch.empty_like(Q)
    ctx._check(_lib().cas_attention(ctx.h, kv.h, layer, seq, 1 if full else 0, _ptr(Q), Q.shape[0], Q.shape[1],
                                    _ptr(Knew), _ptr(Vnew), Knew.shape[0], _ptr(out)), "cas_attention")
    return out


def cas_attention_multi(ctx: Context, kv: KVCache, layer, seqs, full, Qs, Knews, Vnews):
    """One attention call for several sequences: lists of per-sequence tensors as in cas_attention."""
    torch = ctx._torch
    n = len(seqs)
    outs = [torch.empty_like(q) for q in Qs]
    for t in (*Qs, *Knews, *Vnews):
        assert t.is_contiguous()
    i32 = lambda v: (C.c_int32 * n)(*[int(x) for x in v])
    ptrs = lambda ts: (C.c_void_p * n)(*[t.data_ptr() for t in ts])
    ctx._check(_lib().cas_attention_multi(ctx.h, kv.h, layer, n, i32(seqs), 1 if full else 0, ptrs(Qs),
                                          i32([q.shape[0] for q in Qs]), Qs[0].shape[1], ptrs(Knews), ptrs(Vnews),
                                          i32([k.shape[0] for k in Knews]), ptrs(outs)), "cas_attention_multi")
    return outs


def cas_attention_static(ctx: Context, kv: KVCache, layer, seq, full, Q, Knew, Vnew, out):
    """cas_attention with the partial results in the library's fixed device array; `out` must be
    given (this wrapper allocates nothing either)."""
    assert Q.is_contiguous() and Knew.is_contiguous() and Vnew.is_contiguous() and out.is_contiguous()
    ctx._check(_lib().cas_attention_static(ctx.h, kv.h, layer, seq, 1 if full else 0, _ptr(Q), Q.shape[0], Q.shape[1],
                                           _ptr(Knew), _ptr(Vnew), Knew.shape[0], _ptr(out)), "cas_attention_static")
    return out


def cas_attention_static_capacity() -> int:
    return int(_lib().cas_attention_static_capacity())


def _tensor(ew: EncodedWeight) -> cas_tensor:
    return cas_tensor(ew.desc, ew.spec.data_ptr(), ew.verif.data_ptr())


class Model:
    """Holds the encoded weights (device tensors stay referenced here) and the cas_model handle.

    layers: list of dicts with EncodedWeight entries wqkv, wo, wgu, wd and bf16-bit tensors
    g_attn, g_ffn; lm_head: EncodedWeight; embed, g_final: bf16-bit tensors; rope: float32
    tensor [max_pos, 64, 2]."""

    def __init__(self, ctx: Context, shape, layers, lm_head, embed, g_final, rope, max_cols, max_seqs=1):
        torch = ctx._torch
        self.ctx, self.shape = ctx, shape
        self._keep = (layers, lm_head, embed, g_final, rope)
        cfg = cas_model_cfg(shape.hidden, len(layers), shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                            shape.ffn, shape.vocab, max_cols, rope.shape[0], shape.rms_eps, max_seqs)
        self.cfg = cfg
        nbytes = C.c_size_t()
        rc = _lib().cas_model_act_bytes(C.byref(cfg), C.byref(nbytes))
        if rc != CAS_OK:
            raise CasError(rc, "cas_model_act_bytes")
        self.act = torch.empty(nbytes.value, dtype=torch.uint8, device="cuda")
        arr = (cas_layer_weights * len(layers))()
        for i, L in enumerate(layers):
            arr[i] = cas_layer_weights(_tensor(L["wqkv"]), _tensor(L["wo"]), _tensor(L["wgu"]), _tensor(L["wd"]),
                                       L["g_attn"].data_ptr(), L["g_ffn"].data_ptr())
        w = cas_model_weights(arr, _tensor(lm_head), embed.data_ptr(), g_final.data_ptr(), rope.data_ptr())
        h = C.c_void_p()
        rc = _lib().cas_model_create(C.byref(cfg), C.byref(w), _ptr(self.act), nbytes.value, C.byref(h))
        if rc != CAS_OK:
            raise CasError(rc, "cas_model_create")
        self.h = h

    def use_unary(self, layer: int, which: int, uw=None):
        """Switch a linear layer (layer -1: the output head; which: 0 wqkv, 1 wo, 2 wgu, 3 wd) to the
        unary form `uw` of its speculation data (UnaryWeight), or back to the raw form (None)."""
        rc = _lib().cas_model_use_unary(self.h, layer, which, C.byref(uw.desc) if uw is not None else None,
                                        _ptr(uw.uspec) if uw is not None else None)
        if rc != CAS_OK:
            raise CasError(rc, "cas_model_use_unary")
        self._unary = getattr(self, "_unary", {})
        self._unary[(layer, which if layer >= 0 else 0)] = uw   # keeps the buffer alive

    def use_mx(self, layer: int, which: int, mw=None):
        """Switch a linear layer to the shared-exponent form `mw` (MxWeight): its weight becomes the
        converted matrix.  None switches back to the raw form."""
        rc = _lib().cas_model_use_mx(self.h, layer, which, C.byref(mw.desc) if mw is not None else None,
                                     _ptr(mw.spec) if mw is not None else None,
                                     _ptr(mw.verif) if mw is not None else None)
        if rc != CAS_OK:
            raise CasError(rc, "cas_model_use_mx")
        self._mx = getattr(self, "_mx", {})
        self._mx[(layer, which if layer >= 0 else 0)] = mw   # keeps the buffers alive

    def close(self):
        if getattr(self, "h", None):
            _lib().cas_model_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cas_draft_step(ctx, model: Model, kv: KVCache, seq, token_in, slot, token_out, logits=None):
    ctx._check(_lib().cas_draft_step(ctx.h, model.h, kv.h, seq, _ptr(token_in), slot, _ptr(token_out),
                                     _ptr(logits)), "cas_draft_step")


def cas_verify_step(ctx, model: Model, kv: KVCache, seq, tokens, k, target, logits=None):
    ctx._check(_lib().cas_verify_step(ctx.h, model.h, kv.h, seq, _ptr(tokens), k, _ptr(target), _ptr(logits)),
               "cas_verify_step")


def cas_draft_step_multi(ctx, model: Model, kv: KVCache, seqs, slots, tokens_in, tokens_out):
    n = len(seqs)
    ctx._check(_lib().cas_draft_step_multi(ctx.h, model.h, kv.h, n, (C.c_int32 * n)(*seqs), (C.c_int32 * n)(*slots),
                                           _ptr(tokens_in), _ptr(tokens_out)), "cas_draft_step_multi")


def cas_verify_step_multi(ctx, model: Model, kv: KVCache, seqs, ks, tokens, target):
    n = len(seqs)
    ctx._check(_lib().cas_verify_step_multi(ctx.h, model.h, kv.h, n, (C.c_int32 * n)(*seqs), (C.c_int32 * n)(*ks),
                                            _ptr(tokens), _ptr(target)), "cas_verify_step_multi")


def cas_commit(ctx, model: Model, kv: KVCache, seq, n_accepted):
    ctx._check(_lib().cas_commit(ctx.h, model.h, kv.h, seq, n_accepted), "cas_commit")


def cas_spec_round(ctx, model: Model, kv: KVCache, seq, pending, k):
    out = (C.c_int32 * (k + 1))()
    n = C.c_int32()
    ctx._check(_lib().cas_spec_round(ctx.h, model.h, kv.h, seq, int(pending), k, out, C.byref(n)), "cas_spec_round")
    return n.value, [out[i] for i in range(n.value + 1)]


class cas_dense_layer(C.Structure):
    _fields_ = [("d_wqkv", C.c_void_p), ("d_wo", C.c_void_p), ("d_wgu", C.c_void_p), ("d_wd", C.c_void_p)]


def cas_dense_decode_step(ctx, model: Model, layers, lm_head, kcache, vcache, length, token_in, token_out=None,
                          logits=None):
    """Plain bf16 decode step (baseline).  layers: list of dicts of int16 device tensors
    wqkv / wo / wgu / wd; kcache, vcache: int16 [n_layers][max_pos][n_kv_heads][128]."""
    arr = (cas_dense_layer * len(layers))()
    for i, L in enumerate(layers):
        for n in ("wqkv", "wo", "wgu", "wd"):
            assert L[n].is_contiguous()
            setattr(arr[i], "d_" + n, L[n].data_ptr())
    ctx._check(_lib().cas_dense_decode_step(ctx.h, model.h, arr, lm_head.data_ptr(), kcache.data_ptr(), vcache.data_ptr(),
                                            int(length), token_in.data_ptr(),
                                            None if token_out is None else token_out.data_ptr(),
                                            None if logits is None else logits.data_ptr()), "cas_dense_decode_step")


def cas_token_probs(ctx, logits, tokens, out=None):
    """logits: float32 [n][vocab]; tokens: int32 [n]; returns float32 [n] softmax probabilities."""
    torch = ctx._torch
    assert logits.is_contiguous() and logits.dtype == torch.float32 and tokens.dtype == torch.int32
    n, vocab = logits.shape
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=logits.device)
    ctx._check(_lib().cas_token_probs(ctx.h, logits.data_ptr(), vocab, n, tokens.data_ptr(), out.data_ptr()),
               "cas_token_probs")
    return out


def cas_spec_round_sampling(ctx, model: Model, kv: KVCache, seq, pending, k, r, scratch=None):
    """One round with the acceptance rule of Eq. 1; r: k uniform numbers.  Returns
    (n_accepted, emitted tokens, p, q)."""
    torch = ctx._torch
    need = _lib().cas_spec_round_sampling_scratch_floats(model.shape.vocab, k)
    if scratch is None:
        scratch = torch.empty(max(need, 1), dtype=torch.float32, device="cuda")
    assert scratch.numel() >= need and scratch.dtype == torch.float32
    out = (C.c_int32 * (k + 1))()
    n = C.c_int32()
    p, q = (C.c_double * max(k, 1))(), (C.c_double * max(k, 1))()
    rr = (C.c_double * max(k, 1))(*[float(x) for x in r])
    ctx._check(_lib().cas_spec_round_sampling(ctx.h, model.h, kv.h, seq, int(pending), k, rr, scratch.data_ptr(), out,
                                              C.byref(n), p, q), "cas_spec_round_sampling")
    return n.value, [out[i] for i in range(n.value + 1)], [p[i] for i in range(k)], [q[i] for i in range(k)]


def cas_spec_round_multi(ctx, model: Model, kv: KVCache, seqs, pending, k):
    """Returns a list of (n_accepted, emitted tokens) per sequence."""
    n = len(seqs)
    out = (C.c_int32 * (n * (k + 1)))()
    acc = (C.c_int32 * n)()
    ctx._check(_lib().cas_spec_round_multi(ctx.h, model.h, kv.h, n, (C.c_int32 * n)(*seqs),
                                           (C.c_int32 * n)(*[int(p) for p in pending]), k, out, acc),
               "cas_spec_round_multi")
    return [(acc[s], [out[s * (k + 1) + i] for i in range(acc[s] + 1)]) for s in range(n)]


def cas_prefill(ctx, model: Model, kv: KVCache, seq, tokens):
    ctx._check(_lib().cas_prefill(ctx.h, model.h, kv.h, seq, _ptr(tokens), tokens.numel()), "cas_prefill")
