"""ctypes binding of libgoose.so: argument marshalling only, every step runs in the HIP kernels.

Method names mirror the C ABI (include/goose.h).  Tensors are torch tensors living on the GPU;
the binding passes their data pointers and the current torch stream.  There is no fallback: if the
library is missing, loading raises.
"""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))

EXPORTS = [
    "goose_strerror", "goose_last_hip_error", "goose_create", "goose_create_batched", "goose_destroy", "goose_check_parent",
    "goose_packed_layer_bytes", "goose_pack_layer", "goose_packed_lm_head_bytes", "goose_pack_lm_head",
    "goose_build_mask", "goose_embed", "goose_verify_layer", "goose_lm_head_argmax",
    "goose_accept", "goose_compact_kv", "goose_verify_step", "goose_device_flags",
    "goose_packed_matrix_bytes", "goose_pack_matrix", "goose_gemm_packed", "goose_gemm_swiglu_packed",
    "goose_profile_enable", "goose_profile_kinds", "goose_profile_kind_name", "goose_profile_read",
    "goose_copy_probe", "goose_harvest_topk",
    "goose_context_match", "goose_spine_budget", "goose_build_spine_tree", "goose_spine_ratio_tier", "goose_ema_update",
    "goose_cycle_mode", "goose_verify_step_batched",
    "goose_split_operand", "goose_gemm_packed_ex", "goose_gemm_swiglu_packed_ex",
    "goose_lm_head_argmax_static", "goose_plan_cycle",
]

GOOSE_DTYPE_BF16, GOOSE_DTYPE_F32, GOOSE_DTYPE_F16 = 0, 1, 2
DTYPE_CODES = {"bf16": GOOSE_DTYPE_BF16, "f32": GOOSE_DTYPE_F32, "f16": GOOSE_DTYPE_F16}


class GooseError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: status {status} ({_strerror(status)})")
        self.status = status


class _Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("vocab", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32), ("n_kv_heads", C.c_int32), ("qk_norm", C.c_int32), ("act_mode", C.c_int32)]


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2", "gq", "gk")]


class _ModelPtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("d_embed", "d_packed_layers", "d_packed_head", "d_kcache_all",
                                          "d_vcache_all")]


class _StepIO(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("d_tokens", "d_parent", "d_is_spine", "d_P", "d_argmax", "d_accept_len",
                                          "d_path", "d_bonus", "d_next_root_or_null", "d_logits_or_null",
                                          "d_margin_or_null", "d_succ_ids_or_null", "d_succ_scores_or_null")] + \
               [("harvest_k", C.c_int32)]


class _Request(C.Structure):
    _fields_ = [("d_tokens", C.c_void_p), ("d_parent", C.c_void_p), ("d_is_spine", C.c_void_p), ("B", C.c_int32),
                ("P_max", C.c_int32), ("d_kcache_all", C.c_void_p), ("d_vcache_all", C.c_void_p), ("d_P", C.c_void_p),
                ("d_accept_len", C.c_void_p), ("d_path", C.c_void_p), ("d_bonus", C.c_void_p),
                ("d_next_root_or_null", C.c_void_p), ("d_succ_ids_or_null", C.c_void_p),
                ("d_succ_scores_or_null", C.c_void_p), ("harvest_k", C.c_int32)]


@dataclass
class ModelDesc:
    n_layers: int
    hidden: int
    n_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"
    n_kv_heads: int = 0
    qk_norm: bool = False
    act_mode: int = 0      # GOOSE_ACT_F16 (0) or GOOSE_ACT_TWO_TERM (1): see goose.h

    @property
    def kv_heads(self):
        return self.n_kv_heads or self.n_heads

    @classmethod
    def from_shape(cls, s):
        return cls(s.n_layers, s.hidden, s.n_heads, s.head_dim, s.ffn, s.vocab, s.rope_base, s.rms_eps, s.dtype,
                   getattr(s, "n_kv_heads", 0), getattr(s, "qk_norm", False), getattr(s, "act_mode", 0))

    def _c(self):
        return _Desc(self.n_layers, self.hidden, self.n_heads, self.head_dim, self.ffn, self.vocab,
                     self.rope_base, self.rms_eps, DTYPE_CODES[self.dtype],
                     self.n_kv_heads, int(self.qk_norm), int(self.act_mode))


_lib = None


def lib_path():
    return os.path.join(_PKG, "libgoose.so")


def load_library():
    """Loads libgoose.so built in-tree (python -m paper_2604_02047_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built; run `python -m paper_2604_02047_amd.build`")
    lib = C.CDLL(path)
    lib.goose_strerror.restype = C.c_char_p
    lib.goose_strerror.argtypes = [C.c_int]
    lib.goose_last_hip_error.restype = C.c_char_p
    lib.goose_last_hip_error.argtypes = []
    lib.goose_create.argtypes = [C.POINTER(_Desc), C.c_int, C.c_int, C.POINTER(C.c_void_p)]
    lib.goose_create_batched.argtypes = [C.POINTER(_Desc), C.c_int, C.c_int, C.c_int, C.POINTER(C.c_void_p)]
    lib.goose_destroy.argtypes = [C.c_void_p]
    lib.goose_destroy.restype = None
    lib.goose_check_parent.argtypes = [C.c_void_p, C.c_int]
    lib.goose_packed_layer_bytes.argtypes = [C.c_void_p]
    lib.goose_packed_layer_bytes.restype = C.c_size_t
    lib.goose_packed_lm_head_bytes.argtypes = [C.c_void_p]
    lib.goose_packed_lm_head_bytes.restype = C.c_size_t
    lib.goose_pack_layer.argtypes = [C.c_void_p, C.POINTER(_LayerWeights), C.c_void_p, C.c_void_p]
    lib.goose_pack_lm_head.argtypes = [C.c_void_p] * 5
    lib.goose_build_mask.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 5
    lib.goose_embed.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    lib.goose_verify_layer.argtypes = [C.c_void_p] * 5 + [C.c_int, C.c_void_p, C.c_int] + [C.c_void_p] * 3
    lib.goose_lm_head_argmax.argtypes = [C.c_void_p] * 3 + [C.c_int] + [C.c_void_p] * 4
    lib.goose_lm_head_argmax_static.argtypes = [C.c_void_p] * 3 + [C.c_int] + [C.c_void_p] * 3
    lib.goose_accept.argtypes = [C.c_void_p] * 5 + [C.c_int] + [C.c_void_p] * 4
    lib.goose_compact_kv.argtypes = [C.c_void_p] * 3 + [C.c_int] + [C.c_void_p] * 5
    lib.goose_verify_step.argtypes = [C.c_void_p, C.POINTER(_ModelPtrs), C.POINTER(_StepIO), C.c_int, C.c_int,
                                      C.c_void_p]
    lib.goose_device_flags.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
    lib.goose_verify_step_batched.argtypes = [C.c_void_p, C.POINTER(_ModelPtrs), C.POINTER(_Request), C.c_int,
                                              C.c_void_p, C.c_void_p]
    lib.goose_packed_matrix_bytes.argtypes = [C.c_int, C.c_int]
    lib.goose_packed_matrix_bytes.restype = C.c_size_t
    lib.goose_pack_matrix.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.goose_gemm_packed.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_void_p] + [C.c_int] * 5 + [C.c_void_p, C.c_void_p]
    lib.goose_gemm_swiglu_packed.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_void_p] + [C.c_int] * 4 + [C.c_void_p, C.c_int,
                                                                                                C.c_void_p]
    lib.goose_split_operand.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    lib.goose_gemm_packed_ex.argtypes = ([C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p] + [C.c_int] * 5 +
                                         [C.c_float, C.c_void_p, C.c_void_p])
    lib.goose_gemm_swiglu_packed_ex.argtypes = ([C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p] + [C.c_int] * 4 +
                                                [C.c_float, C.c_void_p, C.c_int, C.c_void_p])
    lib.goose_profile_enable.argtypes = [C.c_void_p, C.c_int]
    lib.goose_profile_kinds.argtypes = []
    lib.goose_profile_kind_name.argtypes = [C.c_int]
    lib.goose_profile_kind_name.restype = C.c_char_p
    lib.goose_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.goose_context_match.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 3
    lib.goose_spine_budget.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double] + [C.c_void_p] * 3
    lib.goose_build_spine_tree.argtypes = [C.c_int32, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                           C.c_int, C.c_double, C.c_double, C.c_int, C.c_double] + [C.c_void_p] * 4
    lib.goose_spine_ratio_tier.argtypes = [C.c_double]
    lib.goose_plan_cycle.argtypes = ([C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_int, C.c_int, C.c_int, C.c_double, C.c_double, C.c_int, C.c_double, C.c_int]
                                     + [C.c_void_p] * 5)
    lib.goose_spine_ratio_tier.restype = C.c_double
    lib.goose_ema_update.argtypes = [C.c_double, C.c_int, C.c_int, C.c_double]
    lib.goose_ema_update.restype = C.c_double
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name in ("goose_spine_ratio_tier", "goose_ema_update"):
            continue
        if name not in ("goose_strerror", "goose_last_hip_error", "goose_destroy", "goose_packed_layer_bytes", "goose_packed_lm_head_bytes",
                        "goose_profile_kind_name", "goose_packed_matrix_bytes"):
            fn.restype = C.c_int
    _lib = lib
    return lib


def _strerror(status):
    try:
        lib = load_library()
        msg = lib.goose_strerror(int(status)).decode()
        if status == -5:
            msg += ": " + lib.goose_last_hip_error().decode()
        return msg
    except Exception:  # pragma: no cover
        return "?"


def _check(status, what):
    if status != 0:
        raise GooseError(status, what)


def goose_check_parent(parent) -> int:
    """Host-side validation of a parent array; returns the C status code (0 = ok)."""
    if parent is None:
        return load_library().goose_check_parent(None, 0)
    a = np.ascontiguousarray(np.asarray(parent, dtype=np.int32))
    return load_library().goose_check_parent(a.ctypes.data_as(C.c_void_p), int(a.shape[0]))


def _np_i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def goose_context_match(seq, lens=(3, 4, 5), max_len=20):
    """Host n-gram lookup; returns (draft chain as an int32 array, consensus flag)."""
    seq, lens = _np_i32(seq), _np_i32(lens)
    draft = np.zeros(max_len, np.int32)
    m, cons = C.c_int32(0), C.c_int32(0)
    _check(load_library().goose_context_match(seq.ctypes.data, len(seq), lens.ctypes.data, len(lens), max_len,
                                              draft.ctypes.data, C.addressof(m), C.addressof(cons)),
           "goose_context_match")
    return draft[:m.value].copy(), bool(cons.value)


def goose_spine_budget(B, m, r, rho):
    out = (C.c_int32 * 3)()
    base = C.addressof(out)
    _check(load_library().goose_spine_budget(B, m, r, rho, base, base + 4, base + 8), "goose_spine_budget")
    return out[0], out[1], out[2]


def goose_build_spine_tree(anchor, draft, succ_ids, succ_scores, B, r, rho=0.5, D=6, min_score=0.01):
    """Host tree builder on host tables (numpy int32 [V][K], float32 [V][K]); returns (tokens, parent, is_spine)."""
    draft = _np_i32(draft)
    assert succ_ids.dtype == np.int32 and succ_scores.dtype == np.float32
    assert succ_ids.flags.c_contiguous and succ_scores.flags.c_contiguous and succ_ids.shape == succ_scores.shape
    V, K = succ_ids.shape
    tok, par, spn = np.zeros(B, np.int32), np.zeros(B, np.int32), np.zeros(B, np.uint8)
    n = C.c_int32(0)
    _check(load_library().goose_build_spine_tree(int(anchor), draft.ctypes.data, len(draft), succ_ids.ctypes.data,
                                                 succ_scores.ctypes.data, V, K, B, r, rho, D, min_score,
                                                 tok.ctypes.data, par.ctypes.data, spn.ctypes.data, C.addressof(n)),
           "goose_build_spine_tree")
    return tok[:n.value].copy(), par[:n.value].copy(), spn[:n.value].copy()


MODE_AR, MODE_TREE, MODE_BYPASS = 0, 1, 2
GOOSE_FLAG_BAD_PARENT, GOOSE_FLAG_CAPACITY, GOOSE_FLAG_RANGE, GOOSE_FLAG_WEIGHT_RANGE = 1, 2, 4, 8   # goose_device_flags
GOOSE_ACT_F16, GOOSE_ACT_TWO_TERM = 0, 1
GOOSE_ERR_CAPACITY, GOOSE_ERR_NOT_TOPOLOGICAL = -3, -4


def goose_cycle_mode(m, consensus, bypass_len, anchor_has_successors) -> int:
    return int(load_library().goose_cycle_mode(int(m), int(bool(consensus)), int(bypass_len),
                                               int(bool(anchor_has_successors))))


def goose_plan_cycle(seq, lens, max_spine, anchor, succ_ids, succ_scores, B, p_hat, rho=0.5, D=6, min_score=0.01,
                     bypass_len=8):
    """Host side of a cycle in one call: returns (tokens, parent, is_spine, mode)."""
    seq, lens = _np_i32(seq), _np_i32(lens)
    assert succ_ids.dtype == np.int32 and succ_scores.dtype == np.float32
    assert succ_ids.flags.c_contiguous and succ_scores.flags.c_contiguous and succ_ids.shape == succ_scores.shape
    V, K = succ_ids.shape
    tok, par, spn = np.zeros(B, np.int32), np.zeros(B, np.int32), np.zeros(B, np.uint8)
    n, mode = C.c_int32(0), C.c_int32(0)
    _check(load_library().goose_plan_cycle(seq.ctypes.data, len(seq), lens.ctypes.data, len(lens), int(max_spine),
                                           int(anchor), succ_ids.ctypes.data, succ_scores.ctypes.data, V, K, int(B),
                                           float(p_hat), float(rho), int(D), float(min_score), int(bypass_len),
                                           tok.ctypes.data, par.ctypes.data, spn.ctypes.data, C.addressof(n),
                                           C.addressof(mode)), "goose_plan_cycle")
    return tok[:n.value].copy(), par[:n.value].copy(), spn[:n.value].copy(), int(mode.value)


def goose_spine_ratio_tier(p_hat):
    return float(load_library().goose_spine_ratio_tier(p_hat))


def goose_ema_update(p_hat, accepted_spine, offered_spine, alpha=0.3):
    return float(load_library().goose_ema_update(p_hat, accepted_spine, offered_spine, alpha))


def goose_packed_matrix_bytes(N: int, K: int) -> int:
    return int(load_library().goose_packed_matrix_bytes(N, K))


def goose_pack_matrix(w, N, K, packed):
    _check(load_library().goose_pack_matrix(_ptr(w), N, K, _ptr(packed), _stream()), "goose_pack_matrix")


def _dtype_code(t):
    import torch
    return {torch.bfloat16: GOOSE_DTYPE_BF16, torch.float16: GOOSE_DTYPE_F16}[t.dtype]


def goose_gemm_packed(a, lda, packed, N, K, B, nw, ksplit, partials):
    """a: bf16 or fp16 tensor (its dtype selects the kernel); packed: goose_pack_matrix of weights of the same type."""
    _check(load_library().goose_gemm_packed(_dtype_code(a), _ptr(a), lda, _ptr(packed), N, K, B, nw, ksplit,
                                            _ptr(partials), _stream()), "goose_gemm_packed")


def goose_gemm_swiglu_packed(a, lda, packed, N, K, B, nw, h, ldh):
    _check(load_library().goose_gemm_swiglu_packed(_dtype_code(a), _ptr(a), lda, _ptr(packed), N, K, B, nw, _ptr(h), ldh,
                                                   _stream()), "goose_gemm_swiglu_packed")


def goose_split_operand(src, rows, cols, ld_src, dst, ld_dst):
    """fp32 rows -> the two-term operand layout (dst's dtype selects bf16 or fp16)."""
    _check(load_library().goose_split_operand(_dtype_code(dst), _ptr(src), rows, cols, ld_src, _ptr(dst), ld_dst,
                                              _stream()), "goose_split_operand")


def goose_gemm_packed_ex(a, lda, terms, packed, N, K, B, nw, ksplit, partials, out_scale=1.0):
    _check(load_library().goose_gemm_packed_ex(_dtype_code(a), _ptr(a), lda, terms, _ptr(packed), N, K, B, nw, ksplit,
                                               out_scale, _ptr(partials), _stream()), "goose_gemm_packed_ex")


def goose_gemm_swiglu_packed_ex(a, lda, terms, packed, N, K, B, nw, h, ldh, out_scale=1.0):
    _check(load_library().goose_gemm_swiglu_packed_ex(_dtype_code(a), _ptr(a), lda, terms, _ptr(packed), N, K, B, nw,
                                                      out_scale, _ptr(h), ldh, _stream()), "goose_gemm_swiglu_packed_ex")


def goose_copy_probe(src, dst, nbytes):
    _check(load_library().goose_copy_probe(_ptr(src), _ptr(dst), C.c_size_t(nbytes), _stream()), "goose_copy_probe")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def goose_lm_head_argmax_static(desc: ModelDesc, packed_head, x, B, argmax, margin=None):
    """goose_lm_head_argmax without a context and without any allocation (static device workspace)."""
    cd = desc._c()
    _check(load_library().goose_lm_head_argmax_static(C.byref(cd), _ptr(packed_head), _ptr(x), B, _ptr(argmax),
                                                      _ptr(margin), _stream()), "goose_lm_head_argmax_static")


class GooseContext:
    """Owns a goose_ctx.  Methods are the C entry points with torch tensors as arguments."""

    def __init__(self, desc: ModelDesc, max_B: int, cap: int, max_rows: int = 0):
        """max_rows > 0: workspace for batched passes of that many stacked rows (goose_create_batched)."""
        self.lib = load_library()
        self.desc = desc
        self.max_B, self.cap, self.max_rows = max_B, cap, max_rows or (max_B + 31) // 32 * 32
        h = C.c_void_p()
        cd = desc._c()
        if max_rows:
            _check(self.lib.goose_create_batched(C.byref(cd), max_B, max_rows, cap, C.byref(h)), "goose_create_batched")
        else:
            _check(self.lib.goose_create(C.byref(cd), max_B, cap, C.byref(h)), "goose_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self.lib.goose_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- sizes
    def goose_packed_layer_bytes(self) -> int:
        return int(self.lib.goose_packed_layer_bytes(self._h))

    def goose_packed_lm_head_bytes(self) -> int:
        return int(self.lib.goose_packed_lm_head_bytes(self._h))

    # ---- packing
    def goose_pack_layer(self, raw: dict, packed_layer):
        w = _LayerWeights(*[(raw[n].data_ptr() if n in raw else None)
                            for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2", "gq", "gk")])
        _check(self.lib.goose_pack_layer(self._h, C.byref(w), _ptr(packed_layer), _stream()), "goose_pack_layer")

    def goose_pack_lm_head(self, gf, wlm, packed_head):
        _check(self.lib.goose_pack_lm_head(self._h, _ptr(gf), _ptr(wlm), _ptr(packed_head), _stream()),
               "goose_pack_lm_head")

    # ---- the verification path
    def goose_build_mask(self, parent, B, P, mask, depth, pos, d_P=None):
        _check(self.lib.goose_build_mask(self._h, _ptr(parent), B, P, _ptr(d_P), _ptr(mask), _ptr(depth), _ptr(pos),
                                         _stream()), "goose_build_mask")

    def goose_embed(self, embed, tokens, B, x):
        _check(self.lib.goose_embed(self._h, _ptr(embed), _ptr(tokens), B, _ptr(x), _stream()), "goose_embed")

    def goose_verify_layer(self, packed_layer, x, kcache, vcache, P, B, mask, pos, d_P=None):
        _check(self.lib.goose_verify_layer(self._h, _ptr(packed_layer), _ptr(x), _ptr(kcache), _ptr(vcache), P,
                                           _ptr(d_P), B, _ptr(mask), _ptr(pos), _stream()), "goose_verify_layer")

    def goose_lm_head_argmax(self, packed_head, x, B, argmax, logits=None, margin=None):
        _check(self.lib.goose_lm_head_argmax(self._h, _ptr(packed_head), _ptr(x), B, _ptr(argmax), _ptr(logits),
                                             _ptr(margin), _stream()), "goose_lm_head_argmax")

    def goose_harvest_topk(self, logits, ld, tokens, B, K, succ_ids, succ_scores):
        _check(self.lib.goose_harvest_topk(self._h, _ptr(logits), C.c_size_t(ld), _ptr(tokens), B, K, _ptr(succ_ids),
                                           _ptr(succ_scores), _stream()), "goose_harvest_topk")

    def goose_accept(self, parent, tokens, is_spine, argmax, B, accept_len, path, bonus):
        _check(self.lib.goose_accept(self._h, _ptr(parent), _ptr(tokens), _ptr(is_spine), _ptr(argmax), B,
                                     _ptr(accept_len), _ptr(path), _ptr(bonus), _stream()), "goose_accept")

    def goose_compact_kv(self, kcache_all, vcache_all, P, path, accept_len, new_P=None, d_P=None):
        _check(self.lib.goose_compact_kv(self._h, _ptr(kcache_all), _ptr(vcache_all), P, _ptr(d_P), _ptr(path),
                                         _ptr(accept_len), _ptr(new_P), _stream()), "goose_compact_kv")

    def goose_verify_step(self, model: dict, io: dict, B, P_max):
        m = _ModelPtrs(*[model[n].data_ptr() for n in ("embed", "packed_layers", "packed_head", "kcache", "vcache")])
        names = ("tokens", "parent", "is_spine", "P", "argmax", "accept_len", "path", "bonus", "next_root", "logits",
                 "margin", "succ_ids", "succ_scores")
        s = _StepIO(*[(io[n].data_ptr() if io.get(n) is not None else None) for n in names],
                    int(io.get("harvest_k") or 0))
        _check(self.lib.goose_verify_step(self._h, C.byref(m), C.byref(s), B, P_max, _stream()), "goose_verify_step")

    def goose_verify_step_batched(self, model: dict, requests: list, argmax_all):
        """requests: dicts with tokens, parent, is_spine (or None), B, P_max, kcache, vcache, P, accept_len, path,
        bonus, next_root (or None), succ_ids / succ_scores (or None: no harvest) -- device tensors / ints."""
        m = _ModelPtrs(model["embed"].data_ptr(), model["packed_layers"].data_ptr(), model["packed_head"].data_ptr(),
                       None, None)
        arr = (_Request * len(requests))()
        for i, q in enumerate(requests):
            def p(name):
                t = q.get(name)
                return None if t is None else t.data_ptr()
            arr[i] = _Request(p("tokens"), p("parent"), p("is_spine"), int(q["B"]), int(q["P_max"]), p("kcache"),
                              p("vcache"), p("P"), p("accept_len"), p("path"), p("bonus"), p("next_root"),
                              p("succ_ids"), p("succ_scores"),
                              0 if q.get("succ_ids") is None else int(q["succ_ids"].shape[1]))
        _check(self.lib.goose_verify_step_batched(self._h, C.byref(m), arr, len(requests), _ptr(argmax_all),
                                                  _stream()), "goose_verify_step_batched")

    def goose_device_flags(self) -> int:
        out = C.c_int32(0)
        _check(self.lib.goose_device_flags(self._h, _stream(), C.byref(out)), "goose_device_flags")
        return out.value

    def goose_profile_enable(self, enable: bool):
        _check(self.lib.goose_profile_enable(self._h, 1 if enable else 0), "goose_profile_enable")

    def goose_profile_read(self) -> dict:
        """{kernel kind: (total ms, launches)} since the last read."""
        n = self.lib.goose_profile_kinds()
        ms = (C.c_double * n)()
        cnt = (C.c_int32 * n)()
        _check(self.lib.goose_profile_read(self._h, _stream(), ms, cnt), "goose_profile_read")
        return {self.lib.goose_profile_kind_name(k).decode(): (ms[k], cnt[k]) for k in range(n)}
