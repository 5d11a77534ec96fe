"""ctypes binding of liblsq.so: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class LsqError(RuntimeError):
    pass


class DBG:
    LOGITS, SCORE, TOKENS, LEN, FINISHED, PARENT, CAND_SCORE, CAND_IDX, HIDDEN, MEMORY = range(10)
    CROSS_KV, CACHE_K, CACHE_V = 100, 200, 300


def library_path() -> str:
    return os.path.join(_HERE, "liblsq.so")


def load_library() -> C.CDLL:
    """Loads the in-tree liblsq.so; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise LsqError(f"{path} is missing: build it with `python -m paper_2010_13887_amd.build` "
                       "(or __graft_entry__.build()); there is no fallback path")
    # PyTorch ships its own HIP runtime; whichever copy is loaded first serves the whole process, and
    # the workspace tensor and this library must talk to the same one (loaded the other way round,
    # the library's first runtime call reports that there is no device)
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, sz, i32, f32 = C.c_void_p, C.c_size_t, C.c_int, C.c_float
    sig = {
        "lsq_workspace_bytes": [vp, sz, i32, i32, i32, C.POINTER(sz)],
        "lsq_set_workspace": [vp, sz, vp],
        "lsq_init": [vp, sz, i32, i32, i32],
        "lsq_encode": [vp, vp, i32, i32],
        "lsq_decode_step": [],
        "lsq_decode_steps": [i32],
        "lsq_get_beams": [vp, vp, vp],
        "lsq_step_index": [],
        "lsq_set_graphs": [i32],
        "lsq_set_cache_refresh": [i32],
        "lsq_set_diversity": [i32, f32],
        "lsq_set_layernorm_fusion": [i32],
        "lsq_set_attention_blocks": [i32],
        "lsq_set_topk_statistics": [i32],
        "lsq_set_canaries": [i32],
        "lsq_debug_check_canaries": [],
        "lsq_k_layernorm_gemm": [i32, vp, i32, vp, vp, vp, vp, vp, C.c_float, vp, vp, vp, i32, i32, i32, i32, vp],
        "lsq_k_layernorm_cross_attention": [vp, i32, vp, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, vp, vp, i32, i32, i32,
                                            i32, vp],
        "lsq_k_cross_attention_q": [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp],
        "lsq_k_gemm_logits": [vp, vp, vp, vp, i32, i32, i32, vp],
        "lsq_k_gemm_logits_supported": [i32, i32, i32],
        "lsq_k_row_topk_groups": [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp],
        "lsq_k_self_attention_block": [vp, i32, vp, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, vp, vp, i32, vp, i32, i32, i32,
                                       i32, i32, i32, vp],
        "lsq_k_cross_attention_block": [vp, i32, vp, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32,
                                        vp],
        "lsq_debug_read": [i32, vp, sz],
        "lsq_profile_enable": [i32],
        "lsq_profile_classes": [],
        "lsq_profile_read": [vp, vp, i32],
        "lsq_k_gemm": [i32, vp, vp, vp, vp, i32, i32, i32, i32, vp],
        "lsq_k_pack_weights": [vp, vp, i32, i32, vp],
        "lsq_k_gemm_add_layernorm": [i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp, vp],
        "lsq_k_gemm_add_layernorm_static": [i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp],
        "lsq_k_self_attention": [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
        "lsq_k_encoder_attention": [i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp],
        "lsq_k_self_attention_table": [i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp],
        "lsq_k_cross_attention": [i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
        "lsq_k_row_topk": [i32, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp],
        "lsq_k_beam_refine": [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp],
        "lsq_k_beam_refine_table": [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp],
        "lsq_k_cache_reorder": [i32, vp, vp, i32, i32, i32, i32, i32, i32, vp],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.lsq_k_gemm_add_layernorm_scratch.argtypes = [i32, i32, i32, i32]
    lib.lsq_k_gemm_add_layernorm_scratch.restype = C.c_size_t
    lib.lsq_k_gemm_add_layernorm_static_limit.argtypes = []
    lib.lsq_k_gemm_add_layernorm_static_limit.restype = C.c_size_t
    lib.lsq_k_packed_weight_bytes.argtypes = [i32, i32]
    lib.lsq_k_packed_weight_bytes.restype = C.c_size_t
    lib.lsq_free.argtypes = []
    lib.lsq_free.restype = None
    lib.lsq_profile_class_name.argtypes = [i32]
    lib.lsq_profile_class_name.restype = C.c_char_p
    lib.lsq_last_error.argtypes = []
    lib.lsq_last_error.restype = C.c_char_p
    _LIB = lib
    return lib


def lsq_last_error() -> str:
    return load_library().lsq_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise LsqError(f"lsq error {rc}: {lsq_last_error()}")
    return rc


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


# ---- the C calls, same names ---------------------------------------------------------------
def lsq_workspace_bytes(blob: bytes, max_batch: int, beam: int, max_len: int) -> int:
    n = C.c_size_t()
    _check(load_library().lsq_workspace_bytes(blob, len(blob), max_batch, beam, max_len, C.byref(n)))
    return n.value


def lsq_set_workspace(dev_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(load_library().lsq_set_workspace(dev_ptr, nbytes, stream))


def lsq_init(blob: bytes, max_batch: int, beam: int, max_len: int) -> None:
    _check(load_library().lsq_init(blob, len(blob), max_batch, beam, max_len))


def lsq_encode(src_ids, src_lens) -> None:
    ids, lens = _host_i32(src_ids), _host_i32(src_lens)
    if ids.ndim != 2 or lens.ndim != 1 or ids.shape[0] != lens.shape[0]:
        raise LsqError("src_ids must be [batch, stride] and src_lens [batch]")
    _check(load_library().lsq_encode(ids.ctypes.data, lens.ctypes.data, ids.shape[0], ids.shape[1]))


def lsq_decode_step() -> int:
    return _check(load_library().lsq_decode_step())


def lsq_decode_steps(n: int) -> int:
    return _check(load_library().lsq_decode_steps(n))


def lsq_set_graphs(on: bool) -> None:
    _check(load_library().lsq_set_graphs(int(on)))


def lsq_set_layernorm_fusion(on: bool) -> None:
    """LayerNorm inside the consuming product when at most 8 rows are alive (default on)."""
    _check(load_library().lsq_set_layernorm_fusion(int(on)))


def lsq_set_attention_blocks(max_rows: int) -> None:
    """Attention sublayers as one launch each while at most max_rows rows are alive (0: off; default 64)."""
    _check(load_library().lsq_set_attention_blocks(int(max_rows)))


def lsq_set_topk_statistics(mode: int) -> None:
    """Retrieve stage from the logit product's group statistics: 1 (default) in one launch with the re-rank stage,
    2 as a launch of its own, 0 off (every row read in full)."""
    _check(load_library().lsq_set_topk_statistics(int(mode)))


def lsq_set_canaries(on: bool) -> None:
    """Red zones behind every region of the workspace, from the next lsq_workspace_bytes / lsq_init on (debug aid)."""
    _check(load_library().lsq_set_canaries(int(on)))


def lsq_debug_check_canaries() -> int:
    """How many red zones have been written to (0 = none)."""
    return _check(load_library().lsq_debug_check_canaries())


def lsq_set_diversity(groups: int = 1, strength: float = 0.0) -> None:
    """Diverse beam search from the next encode on: `groups` groups per sentence, Hamming penalty `strength`."""
    _check(load_library().lsq_set_diversity(int(groups), float(strength)))


REFRESH_MOVE, REFRESH_TABLE = 0, 1


def lsq_set_cache_refresh(mode: int) -> None:
    """How the K/V cache follows the beams from the next encode on: REFRESH_MOVE copies cache rows,
    REFRESH_TABLE (default) keeps a table of which row holds which position."""
    _check(load_library().lsq_set_cache_refresh(int(mode)))


def lsq_step_index() -> int:
    return _check(load_library().lsq_step_index())


def lsq_get_beams(batch: int, beam: int, max_len: int):
    ids = np.empty((batch, beam, max_len), np.int32)
    lens = np.empty((batch, beam), np.int32)
    scores = np.empty((batch, beam), np.float32)
    _check(load_library().lsq_get_beams(ids.ctypes.data, lens.ctypes.data, scores.ctypes.data))
    return ids, lens, scores


def lsq_free() -> None:
    load_library().lsq_free()


def lsq_debug_read(what: int, shape, dtype=np.float32) -> np.ndarray:
    out = np.empty(shape, dtype)
    _check(load_library().lsq_debug_read(what, out.ctypes.data, out.nbytes))
    return out


def lsq_profile_enable(on: bool) -> None:
    _check(load_library().lsq_profile_enable(int(on)))


def lsq_profile_read() -> dict:
    """{class name: (summed milliseconds, launches)} since the last read."""
    lib = load_library()
    n = lib.lsq_profile_classes()
    ms = np.zeros(n, np.float64)
    cnt = np.zeros(n, np.int64)
    _check(lib.lsq_profile_read(ms.ctypes.data, cnt.ctypes.data, n))
    return {lib.lsq_profile_class_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


# ---- single-kernel entry points on torch tensors ----------------------------------------------
def _dt(t) -> int:
    import torch
    if t.dtype == torch.float16:
        return 1
    if t.dtype == torch.float32:
        return 0
    raise LsqError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _p(t) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def k_gemm(A, B, bias, C_out, relu: bool = False, gelu: bool = False, packed: bool = False) -> None:
    """C_out = act(A . B^T + bias), act = ReLU, tanh-GELU or none; a float32 C_out with float16 inputs
    keeps the accumulators unrounded.  packed: B is the output of k_pack_weights (N and K from C_out and A)."""
    import torch
    M, K = A.shape
    N = C_out.shape[1]
    assert packed or (tuple(B.shape) == (N, K))
    assert C_out.shape[0] == M and not (relu and gelu)
    flags = int(relu) | (4 if gelu else 0) | (2 if (A.dtype == torch.float16 and C_out.dtype == torch.float32) else 0)
    flags |= 16 if packed else 0
    assert flags & 2 or C_out.dtype == A.dtype
    _check(load_library().lsq_k_gemm(_dt(A), _p(A), _p(B), _p(bias), _p(C_out), M, N, K, flags, _stream()))


def k_pack_weights(W):
    """The float16 matrix W [N, K] in fragment order (see lsq_k_pack_weights): a flat float16 tensor."""
    import torch
    N, K = W.shape
    lib = load_library()
    nbytes = lib.lsq_k_packed_weight_bytes(N, K)
    if nbytes == 0:
        raise LsqError("K must be a multiple of 16")
    out = torch.empty(nbytes // 2, dtype=torch.float16, device=W.device)
    _check(lib.lsq_k_pack_weights(_p(W), _p(out), N, K, _stream()))
    return out


def k_gemm_add_layernorm(inp, W, bias, x, gamma, beta, eps: float) -> None:
    """x <- LayerNorm(x + inp . W^T + bias) * gamma + beta, in place on x."""
    import torch
    M, K = inp.shape
    d = W.shape[0]
    assert W.shape[1] == K and tuple(x.shape) == (M, d)
    lib = load_library()
    scratch = torch.empty(max(16, lib.lsq_k_gemm_add_layernorm_scratch(_dt(x), M, d, K)), dtype=torch.uint8,
                          device=x.device)
    _check(lib.lsq_k_gemm_add_layernorm(_dt(x), _p(inp), _p(W), _p(bias), _p(x), _p(gamma), _p(beta), M, d, K, eps,
                                        _p(scratch), _stream()))


def k_gemm_add_layernorm_static(inp, W, bias, x, gamma, beta, eps: float) -> None:
    """k_gemm_add_layernorm with the partial sums in the library's built-in buffer: nothing is allocated."""
    M, K = inp.shape
    d = W.shape[0]
    assert W.shape[1] == K and tuple(x.shape) == (M, d)
    _check(load_library().lsq_k_gemm_add_layernorm_static(_dt(x), _p(inp), _p(W), _p(bias), _p(x), _p(gamma), _p(beta),
                                                          M, d, K, eps, _stream()))


def k_gemm_add_layernorm_static_limit() -> int:
    return load_library().lsq_k_gemm_add_layernorm_static_limit()


def k_layernorm_gemm(P, ln_bias, gamma, beta, x_old, x_new, eps: float, W, bias, C_out, relu: bool = False) -> None:
    """C_out = act(LN(x_old + sum of the slabs P + ln_bias) . W^T + bias); x_new receives the normalised rows."""
    import torch
    splits, M, K = P.shape
    N = W.shape[0]
    flags = int(relu) | (2 if C_out.dtype == torch.float32 else 0)
    _check(load_library().lsq_k_layernorm_gemm(_dt(x_old), _p(P), splits, _p(ln_bias), _p(gamma), _p(beta), _p(x_old),
                                               _p(x_new), eps, _p(W), _p(bias), _p(C_out), M, N, K, flags, _stream()))


def k_layernorm_cross_attention(P, ln_bias, gamma, beta, x_old, x_new, eps: float, Wq_packed, bq, kv, src_off, src_len,
                                out, batch: int, beam: int, heads: int) -> None:
    """out = cross-attention of q = LN(x_old + sum of the slabs P + ln_bias) . Wq^T + bq; x_new receives the normalised
    rows.  Wq_packed: k_pack_weights(Wq)."""
    splits, M, d = P.shape
    assert M == batch * beam
    _check(load_library().lsq_k_layernorm_cross_attention(_p(P), splits, _p(ln_bias), _p(gamma), _p(beta), _p(x_old),
                                                          _p(x_new), eps, _p(Wq_packed), _p(bq), _p(kv), _p(src_off),
                                                          _p(src_len), _p(out), batch, beam, heads, d, _stream()))


def k_self_attention_block(P, ln_bias, gamma, beta, x_old, x_new, eps: float, Wqkv_packed, bqkv, Wo_packed, Kc, Vc,
                           slab_table, nkeys: int, P_out, batch: int, beam: int, heads: int, pre_ln: bool = False) -> None:
    """Self-attention sublayer up to the output projection's per-head partial sums P_out [heads, rows, d]; P None: the
    rows are x_old as they are (pre_ln: LayerNorm(x_old)).  Kc, Vc [rows, T, d] receive the new position at index nkeys."""
    M, d = x_old.shape
    splits = 0 if P is None else P.shape[0]
    assert M == batch * beam and tuple(P_out.shape) == (heads, M, d)
    _check(load_library().lsq_k_self_attention_block(_p(P), splits, _p(ln_bias), _p(gamma), _p(beta), _p(x_old), _p(x_new),
                                                     eps, _p(Wqkv_packed), _p(bqkv), _p(Wo_packed), _p(Kc), _p(Vc),
                                                     _p(slab_table), nkeys, _p(P_out), batch, beam, heads, d, Kc.shape[1],
                                                     int(bool(pre_ln)), _stream()))


def k_cross_attention_block(P, ln_bias, gamma, beta, x_old, x_new, eps: float, Wq_packed, bq, Wo_packed, kv, src_off,
                            src_len, P_out, batch: int, beam: int, heads: int) -> None:
    """Cross-attention sublayer up to the output projection's per-head partial sums P_out [heads, rows, d]."""
    splits, M, d = P.shape
    assert M == batch * beam and tuple(P_out.shape) == (heads, M, d)
    _check(load_library().lsq_k_cross_attention_block(_p(P), splits, _p(ln_bias), _p(gamma), _p(beta), _p(x_old), _p(x_new),
                                                      eps, _p(Wq_packed), _p(bq), _p(Wo_packed), _p(kv), _p(src_off),
                                                      _p(src_len), _p(P_out), batch, beam, heads, d, _stream()))


def k_gemm_logits(A, B, C_out, stats) -> None:
    """C_out [M,N] float32 = A . B^T with (largest, sum of exp(value - largest)) of every (row, 32-column group) in
    stats [M, ceil(N/32), 2]."""
    M, K = A.shape
    N = B.shape[0]
    assert tuple(stats.shape) == (M, (N + 31) // 32, 2)
    _check(load_library().lsq_k_gemm_logits(_p(A), _p(B), _p(C_out), _p(stats), M, N, K, _stream()))


def k_gemm_logits_supported(M: int, N: int, K: int) -> bool:
    return bool(load_library().lsq_k_gemm_logits_supported(M, N, K))


def k_row_topk_groups(logits, stats, score, finished, k: int, eos: int, out_score, out_idx, raw: bool = False) -> None:
    M, V = logits.shape
    _check(load_library().lsq_k_row_topk_groups(_p(logits), _p(stats), _p(score), _p(finished), M, V, k, eos, int(raw),
                                                _p(out_score), _p(out_idx), _stream()))


def k_cross_attention_q(x, Wq_packed, bq, kv, src_off, src_len, out, batch: int, beam: int, heads: int) -> None:
    """out = cross-attention of q = x . Wq^T + bq (more than 64 rows); Wq_packed: k_pack_weights(Wq)."""
    M, d = x.shape
    assert M == batch * beam
    _check(load_library().lsq_k_cross_attention_q(_p(x), _p(Wq_packed), _p(bq), _p(kv), _p(src_off), _p(src_len), _p(out),
                                                  batch, beam, heads, d, _stream()))


def k_self_attention(q, Kc, Vc, out, heads: int, nkeys: int) -> None:
    rows, d = q.shape
    T = Kc.shape[1]
    _check(load_library().lsq_k_self_attention(_dt(q), _p(q), _p(Kc), _p(Vc), _p(out), rows, heads, d, T, nkeys,
                                               _stream()))


def k_self_attention_table(q, Kc, Vc, slab, out, beam: int, heads: int, nkeys: int) -> None:
    """Self-attention where position j of row r is read from cache row (r - r % beam) + slab[r, j]."""
    rows, d = q.shape
    T = Kc.shape[1]
    assert tuple(slab.shape) == (rows, T + 1)
    _check(load_library().lsq_k_self_attention_table(_dt(q), _p(q), _p(Kc), _p(Vc), _p(slab), _p(out), rows, beam,
                                                     heads, d, T, nkeys, _stream()))


def k_encoder_attention(qkv, row_seq, seq_off, seq_len, out, heads: int, causal: bool = False) -> None:
    """Self-attention inside packed sequences; qkv [rows, 3d] = [Q | K | V]."""
    rows, d3 = qkv.shape
    _check(load_library().lsq_k_encoder_attention(_dt(qkv), _p(qkv), _p(row_seq), _p(seq_off), _p(seq_len), _p(out),
                                                  rows, heads, d3 // 3, int(causal), _stream()))


def k_cross_attention(q, kv, src_off, src_len, out, batch: int, beam: int, heads: int, max_src_len: int) -> None:
    d = q.shape[1]
    _check(load_library().lsq_k_cross_attention(_dt(q), _p(q), _p(kv), _p(src_off), _p(src_len), _p(out), batch,
                                                beam, heads, d, max_src_len, _stream()))


def k_row_topk(logits, score, finished, k: int, eos: int, out_score, out_idx) -> None:
    M, V = logits.shape
    _check(load_library().lsq_k_row_topk(_dt(logits), _p(logits), _p(score), _p(finished), M, V, k, eos,
                                         _p(out_score), _p(out_idx), _stream()))


def k_beam_refine(cand_score, cand_idx, score, tokens, length, finished, parent, cap, active, batch: int, k: int,
                  V: int, T: int, t: int, eos: int, slab=None) -> None:
    """slab: optional int32 [batch*k, T+1] table gathered by parent along with the token histories."""
    lib = load_library()
    if slab is None:
        _check(lib.lsq_k_beam_refine(_p(cand_score), _p(cand_idx), _p(score), _p(tokens), _p(length), _p(finished),
                                     _p(parent), _p(cap), _p(active), batch, k, V, T, t, eos, _stream()))
    else:
        assert tuple(slab.shape) == (batch * k, T + 1)
        _check(lib.lsq_k_beam_refine_table(_p(cand_score), _p(cand_idx), _p(score), _p(tokens), _p(length),
                                           _p(finished), _p(parent), _p(cap), _p(active), _p(slab), batch, k, V, T,
                                           t, eos, _stream()))


def k_cache_reorder(cache, parent, layers: int, batch: int, k: int, T: int, d: int, npos: int) -> None:
    _check(load_library().lsq_k_cache_reorder(_dt(cache), _p(cache), _p(parent), layers, batch, k, T, d, npos,
                                              _stream()))


# ---- convenience: one object that owns the workspace -------------------------------------------
class Engine:
    """Owns the device workspace (a torch uint8 tensor) for one loaded model.  One per process."""

    def __init__(self, blob: bytes, max_batch: int, beam: int, max_len: int, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise LsqError("no GPU visible; this library has no CPU path")
        load_library()
        self.max_batch, self.beam, self.max_len = max_batch, beam, max_len
        nbytes = lsq_workspace_bytes(blob, max_batch, beam, max_len)
        torch.cuda.set_device(device)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        # a stream of its own (default priority): the default stream cannot be captured into graphs
        self.torch_stream = torch.cuda.Stream(device=device)
        self.stream = self.torch_stream.cuda_stream
        torch.cuda.current_stream().synchronize()
        lsq_set_workspace(self.workspace.data_ptr(), nbytes, self.stream)
        try:
            lsq_init(blob, max_batch, beam, max_len)
        except Exception:
            lsq_free()
            raise
        self.batch = 0

    def encode(self, src_ids, src_lens) -> None:
        lsq_encode(src_ids, src_lens)
        self.batch = len(src_lens)

    def decode_step(self) -> int:
        return lsq_decode_step()

    def decode_steps(self, n: int) -> int:
        return lsq_decode_steps(n)

    def get_beams(self):
        return lsq_get_beams(self.batch, self.beam, self.max_len)

    def debug(self, what: int, shape, dtype=np.float32):
        return lsq_debug_read(what, shape, dtype)

    def translate(self, src_ids, src_lens, sync_every: int = 1):
        self.encode(src_ids, src_lens)
        while self.decode_steps(sync_every) > 0:
            pass
        return self.get_beams()

    def close(self) -> None:
        lsq_free()
        self.workspace = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
