"""Kernel-level parity: every HIP kernel against the oracle's function of the same operation on
seeded tensors, through the C ABI (needs an MI355X).  Sizes span several tiles and ragged tails."""
import numpy as np
import pytest

from oracle import lsq_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    return lib, torch


def _dev(torch, a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def _h(a):       # round to fp16 and widen: the values an fp16 tensor holds
    return np.asarray(a, np.float32).astype(np.float16).astype(np.float32)


@pytest.mark.parametrize("M,N,K", [(8, 192, 64), (33, 1000, 72), (130, 520, 256), (512, 1024, 1024),
                                   (512, 3072, 1024), (100, 1003, 264), (512, 32000, 1024), (1, 64, 8),
                                   (700, 136, 4096),
                                   # more than 256 tiles of 64x64, k a multiple of 64: tiles loaded straight into LDS;
                                   # ragged rows and columns, fewer k-tiles than stages, unaligned output rows
                                   (300, 4100, 128), (321, 3071, 64), (450, 2500, 1024), (257, 4224, 320)])
@pytest.mark.parametrize("relu", [False, True])
def test_gemm_fp16(env, M, N, K, relu):
    lsq, torch = env
    rng = np.random.default_rng(M * 7 + N)
    A, B, bias = _h(rng.standard_normal((M, K))), _h(rng.standard_normal((N, K)) * 0.05), _h(rng.standard_normal(N))
    ref = A.astype(np.float64) @ B.astype(np.float64).T + bias
    if relu:
        ref = np.maximum(ref, 0)
    dA, dB, db = _dev(torch, A, torch.float16), _dev(torch, B, torch.float16), _dev(torch, bias, torch.float16)
    C32 = torch.empty(M, N, dtype=torch.float32, device="cuda")
    lsq.k_gemm(dA, dB, db, C32, relu)
    got = C32.cpu().numpy()
    scale = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64).T + np.abs(bias)
    assert (np.abs(got - ref) <= 2e-6 * scale + 1e-7).all()        # fp32 accumulation of exact products
    C16 = torch.empty(M, N, dtype=torch.float16, device="cuda")
    lsq.k_gemm(dA, dB, db, C16, relu)
    got16 = C16.float().cpu().numpy()
    np.testing.assert_allclose(got16, ref, rtol=1e-3, atol=2e-6 * scale.max() + 1e-6)
    # no bias
    lsq.k_gemm(dA, dB, None, C32, False)
    assert (np.abs(C32.cpu().numpy() - (ref_nb := A.astype(np.float64) @ B.astype(np.float64).T)) <= 2e-6 * scale + 1e-7).all()


@pytest.mark.parametrize("M,N,K", [(8, 192, 64), (33, 1000, 71), (130, 77, 256), (2, 3000, 64), (33, 1000, 72),
                                   (512, 1024, 1024), (100, 1003, 264), (1, 64, 8), (700, 136, 4096), (64, 50, 40),
                                   (65, 32000, 512)])
@pytest.mark.parametrize("relu", [False, True])
def test_gemm_fp32(env, M, N, K, relu):
    """fp32 models: streamed through the fp32 matrix cores when K is a multiple of 8, the plain tile
    kernel otherwise; fp32 accumulation in both."""
    lsq, torch = env
    rng = np.random.default_rng(M + N)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    C = torch.full((M, N), 7.0, dtype=torch.float32, device="cuda")
    lsq.k_gemm(_dev(torch, A), _dev(torch, B), _dev(torch, bias), C, relu)
    ref = A.astype(np.float64) @ B.astype(np.float64).T + bias
    if relu:
        ref = np.maximum(ref, 0)
    scale = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64).T + np.abs(bias)
    assert (np.abs(C.cpu().numpy() - ref) <= 3e-6 * scale + 1e-6).all()
    lsq.k_gemm(_dev(torch, A), _dev(torch, B), None, C, False)                       # no bias
    assert (np.abs(C.cpu().numpy() - A.astype(np.float64) @ B.astype(np.float64).T) <= 3e-6 * scale + 1e-6).all()


@pytest.mark.parametrize("M,N,K", [(5, 264, 128), (32, 3072, 768), (200, 520, 72), (600, 3072, 768)])
@pytest.mark.parametrize("half", [False, True])
def test_gemm_gelu(env, M, N, K, half):
    """tanh-GELU epilogue (decoder-only model's feed-forward) against the oracle's gelu_tanh in float64."""
    lsq, torch = env
    rng = np.random.default_rng(M + N + K)
    cast = _h if half else (lambda a: np.asarray(a, np.float32))
    A, B, bias = cast(rng.standard_normal((M, K))), cast(rng.standard_normal((N, K)) * 0.1), cast(rng.standard_normal(N))
    ref = O.gelu_tanh(A.astype(np.float64) @ B.astype(np.float64).T + bias)
    td = torch.float16 if half else torch.float32
    C = torch.empty(M, N, dtype=torch.float32, device="cuda")
    lsq.k_gemm(_dev(torch, A, td), _dev(torch, B, td), _dev(torch, bias, td), C, gelu=True)
    np.testing.assert_allclose(C.cpu().numpy(), ref, rtol=2e-5, atol=2e-5)


@pytest.mark.parametrize("rows,d,K", [(1, 64, 64), (5, 512, 2048), (513, 1024, 1024), (512, 1024, 4096),
                                      (37, 2048, 264), (64, 1024, 4096), (9, 72, 40), (4, 100, 16), (3, 4104, 128)])
@pytest.mark.parametrize("half", [False, True])
def test_gemm_add_layernorm(env, rows, d, K, half):
    """x <- LN(x + in . W^T + bias): split-K partial sums, bias, residual and LayerNorm."""
    lsq, torch = env
    rng = np.random.default_rng(rows + d + K)
    cast = _h if half else (lambda a: np.asarray(a, np.float32))
    x, inp = cast(rng.standard_normal((rows, d)) * 2), cast(rng.standard_normal((rows, K)))
    W, bias = cast(rng.standard_normal((d, K)) * 0.05), cast(rng.standard_normal(d) * 0.3)
    g, b = cast(1 + 0.3 * rng.standard_normal(d)), cast(0.3 * rng.standard_normal(d))
    a = inp.astype(np.float64) @ W.astype(np.float64).T + bias
    ref = O.layer_norm(x.astype(np.float64) + a, g.astype(np.float64), b.astype(np.float64), 1e-5)
    td = torch.float16 if half else torch.float32
    dx = _dev(torch, x, td)
    lsq.k_gemm_add_layernorm(_dev(torch, inp, td), _dev(torch, W, td), _dev(torch, bias, td), dx, _dev(torch, g, td),
                             _dev(torch, b, td), 1e-5)
    got = dx.float().cpu().numpy()
    if half:
        np.testing.assert_allclose(got, ref, rtol=1.1e-3, atol=1e-3)
        assert np.abs(got - _h(ref)).max() <= 4e-3 and (got != _h(ref)).mean() < 0.02
    else:
        np.testing.assert_allclose(got, ref, rtol=3e-5, atol=3e-5)


@pytest.mark.parametrize("M,N,K", [(1, 32, 16), (4, 3072, 1024), (32, 1000, 512), (33, 96, 768), (64, 50257, 64),
                                   (7, 37, 48), (64, 2304, 768), (17, 31, 1024)])
@pytest.mark.parametrize("f32_out", [False, True])
def test_gemm_with_fragment_ordered_weights(env, M, N, K, f32_out):
    """lsq_k_pack_weights lays the matrix out exactly as documented, and a product that reads it gives
    the same bits as the product that reads the row-major matrix (same fragments, same order) wherever the
    latter runs the same kernel: from 33 rows on it runs a tiled kernel when k >= 768 or the product is vocabulary-sized
    (another summation order)."""
    lsq, torch = env
    rng = np.random.default_rng(M + N + K)
    A, W, bias = _h(rng.standard_normal((M, K))), _h(rng.standard_normal((N, K)) * 0.1), _h(rng.standard_normal(N))
    h = torch.float16
    dA, dW, dbias = _dev(torch, A, h), _dev(torch, W, h), _dev(torch, bias, h)
    packed = lsq.k_pack_weights(dW)
    nb = (N + 31) // 32
    Wp = np.zeros((nb * 32, K), np.float16)
    Wp[:N] = W
    # [block][row in block][k-step][half of the step][8] -> [block][k-step][half][row][8]: lane = half * 32 + row
    ref = Wp.reshape(nb, 32, K // 16, 2, 8).transpose(0, 2, 3, 1, 4).reshape(-1)
    assert np.array_equal(packed.cpu().numpy(), ref)
    C1 = torch.full((M, N), 7.0, dtype=torch.float32 if f32_out else h, device="cuda")
    C2 = torch.full_like(C1, 9.0)
    lsq.k_gemm(dA, dW, dbias, C1, relu=True)
    lsq.k_gemm(dA, packed, dbias, C2, relu=True, packed=True)
    if M <= 32 or (K < 768 and (N + 127) // 128 < 125):      # where the row-major product runs the skinny kernel too
        assert torch.equal(C1, C2)
    else:
        np.testing.assert_allclose(C1.double().cpu().numpy(), C2.double().cpu().numpy(), rtol=2e-3 if not f32_out else 1e-5,
                                   atol=(2e-3 if not f32_out else 1e-5) * (1 + float(C2.abs().max())))
    want = np.maximum(A.astype(np.float64) @ W.astype(np.float64).T + bias, 0)
    np.testing.assert_allclose(C2.double().cpu().numpy(), want, rtol=2e-3 if not f32_out else 1e-5,
                               atol=(2e-3 if not f32_out else 1e-5) * (1 + np.abs(want).max()))


@pytest.mark.parametrize("rows,d,N,splits", [(1, 64, 96, 1), (4, 1024, 3072, 4), (8, 1024, 1000, 4), (5, 512, 2048, 2),
                                             (7, 768, 50, 3), (8, 1024, 32000, 4), (3, 48, 40, 1)])
@pytest.mark.parametrize("f32_out", [False, True])
def test_layernorm_inside_product(env, rows, d, N, splits, f32_out):
    """Product that normalises its own input: x_new is bit-identical to the stand-alone LayerNorm
    kernel's rows, and C equals the plain product of those rows."""
    lsq, torch = env
    rng = np.random.default_rng(rows + d + N)
    x = _h(rng.standard_normal((rows, d)) * 2)
    P = (rng.standard_normal((splits, rows, d)) * 0.5).astype(np.float32)
    lb, g, b = _h(rng.standard_normal(d) * 0.3), _h(1 + 0.3 * rng.standard_normal(d)), _h(0.3 * rng.standard_normal(d))
    W, bias = _h(rng.standard_normal((N, d)) * 0.05), _h(rng.standard_normal(N))
    h = torch.float16
    dx, dP = _dev(torch, x, h), _dev(torch, P)
    dlb, dg, db, dW, dbias = (_dev(torch, a, h) for a in (lb, g, b, W, bias))
    x_new = torch.full((rows, d), 7.0, dtype=h, device="cuda")
    C = torch.full((rows, N), 7.0, dtype=torch.float32 if f32_out else h, device="cuda")
    lsq.k_layernorm_gemm(dP, dlb, dg, db, dx, x_new, 1e-5, dW, dbias, C, relu=True)
    assert torch.equal(dx, _dev(torch, x, h))                       # the residual input is left alone
    # the same rows from the oracle (float64), and the product of the rows the kernel actually made
    a = P.astype(np.float64).sum(0) + lb
    ref_rows = O.layer_norm(x.astype(np.float64) + a, g.astype(np.float64), b.astype(np.float64), 1e-5)
    got_rows = x_new.float().cpu().numpy()
    np.testing.assert_allclose(got_rows, ref_rows, rtol=1.1e-3, atol=1e-3)
    assert np.abs(got_rows - _h(ref_rows)).max() <= 4e-3 and (got_rows != _h(ref_rows)).mean() < 0.02
    C2 = torch.empty_like(C)
    lsq.k_gemm(x_new, dW, dbias, C2, relu=True)
    assert torch.equal(C, C2)                                        # same fragments, same order of accumulation


@pytest.mark.parametrize("rows,H,dh,T,nkeys", [(3, 4, 16, 8, 1), (9, 4, 16, 8, 8), (32, 8, 64, 110, 77),
                                               (5, 2, 128, 40, 33), (7, 3, 32, 50, 50), (130, 16, 64, 178, 41),
                                               (300, 8, 64, 60, 60), (2, 2, 16, 200, 199), (5, 2, 16, 1, 1),
                                               (600, 4, 32, 3, 2)])
@pytest.mark.parametrize("half", [False, True])
def test_self_attention(env, rows, H, dh, T, nkeys, half):
    lsq, torch = env
    rng = np.random.default_rng(rows * 3 + nkeys)
    d = H * dh
    cast = _h if half else (lambda a: np.asarray(a, np.float32))
    q = cast(rng.standard_normal((rows, d)))
    Kc, Vc = cast(rng.standard_normal((rows, T, d))), cast(rng.standard_normal((rows, T, d)))
    Kc[:, nkeys:] = np.nan                                 # positions past the history may be read, and must not matter
    Vc[:, nkeys:] = np.inf
    td = torch.float16 if half else torch.float32
    out = torch.full((rows, d), 7.0, dtype=td, device="cuda")
    lsq.k_self_attention(_dev(torch, q, td), _dev(torch, Kc, td), _dev(torch, Vc, td), out, H, nkeys)
    ref = np.stack([O.attention(q[r:r + 1].astype(np.float64), Kc[r, :nkeys].astype(np.float64),
                                Vc[r, :nkeys].astype(np.float64), H)[0] for r in range(rows)])
    tol = 1.5e-3 if half else 2e-5
    np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=tol, atol=tol)


@pytest.mark.parametrize("B,k,H,dh,T,nkeys", [(2, 4, 4, 16, 8, 1), (3, 4, 8, 64, 110, 77), (5, 3, 2, 32, 50, 50),
                                              (75, 4, 8, 64, 60, 41), (2, 8, 2, 128, 40, 33), (4, 1, 4, 16, 9, 9),
                                              (3, 4, 2, 16, 1, 1), (140, 4, 4, 32, 2, 1)])
@pytest.mark.parametrize("half", [False, True])
def test_self_attention_through_slab_table(env, B, k, H, dh, T, nkeys, half):
    """Position j of row r is read from cache row (r - r % k) + slab[r, j]: equals attention over the
    gathered history."""
    lsq, torch = env
    rng = np.random.default_rng(B * 7 + k + nkeys)
    rows, d = B * k, H * dh
    cast = _h if half else (lambda a: np.asarray(a, np.float32))
    q = cast(rng.standard_normal((rows, d)))
    Kc, Vc = cast(rng.standard_normal((rows, T, d))), cast(rng.standard_normal((rows, T, d)))
    slab = rng.integers(0, k, size=(rows, T + 1)).astype(np.int32)
    slab[:, nkeys:] = rng.choice([1 << 20, -5, k, -(1 << 30)], size=(rows, T + 1 - nkeys))   # entries past the history
    Kc[:, nkeys:] = np.nan                                 # and cache positions past it may be read (the first request
    Vc[:, nkeys:] = np.nan                                 # does not wait for the length), and must not matter
    td = torch.float16 if half else torch.float32
    out = torch.full((rows, d), 7.0, dtype=td, device="cuda")
    lsq.k_self_attention_table(_dev(torch, q, td), _dev(torch, Kc, td), _dev(torch, Vc, td), _dev(torch, slab), out, k, H, nkeys)
    j = np.arange(nkeys)
    ref = np.stack([O.attention(q[r:r + 1].astype(np.float64), Kc[r - r % k + slab[r, :nkeys], j].astype(np.float64),
                                Vc[r - r % k + slab[r, :nkeys], j].astype(np.float64), H)[0] for r in range(rows)])
    tol = 1.5e-3 if half else 2e-5
    np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=tol, atol=tol)


@pytest.mark.parametrize("lens,H,dh", [([5, 8], 4, 16), ([1, 60, 17, 33], 8, 64), ([128, 3], 16, 64), ([9], 2, 128),
                                       ([40] * 7, 3, 32),
                                       # matrix-core kernel (float16, heads of 32 / 64 / 128): sentences longer than several
                                       # key blocks, blocks of 32 rows that hold many one-token sentences, a last block of
                                       # one row, a sentence ending exactly on a block boundary
                                       ([300, 2, 257], 2, 64), ([1] * 70 + [3], 4, 64), ([32, 32, 1], 2, 32),
                                       ([31, 33, 64, 2], 2, 128), ([700], 1, 64)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("half", [False, True])
def test_encoder_attention(env, lens, H, dh, causal, half):
    """Packed sequences: every row attends its own sequence (all of it, or up to itself)."""
    lsq, torch = env
    rng = np.random.default_rng(sum(lens) + H)
    d, R = H * dh, sum(lens)
    cast = _h if half else (lambda a: np.asarray(a, np.float32))
    qkv = cast(rng.standard_normal((R, 3 * d)))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    row_seq = np.repeat(np.arange(len(lens)), lens).astype(np.int32)
    td = torch.float16 if half else torch.float32
    out = torch.full((R, d), 7.0, dtype=td, device="cuda")
    lsq.k_encoder_attention(_dev(torch, qkv, td), _dev(torch, row_seq), _dev(torch, off[:-1].copy()),
                            _dev(torch, np.array(lens, np.int32)), out, H, causal)
    ref = np.empty((R, d))
    for b, n in enumerate(lens):
        blk = qkv[off[b]:off[b] + n].astype(np.float64)
        mask = np.tril(np.ones((n, n), bool)) if causal else None
        ref[off[b]:off[b] + n] = O.attention(blk[:, :d], blk[:, d:2 * d], blk[:, 2 * d:], H, mask)
    tol = 1.5e-3 if half else 2e-5
    np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=tol, atol=tol)


@pytest.mark.parametrize("lens,beam,H,dh", [([5, 8], 4, 4, 16), ([1, 60, 17, 33], 4, 8, 64), ([9, 2, 31], 3, 2, 32),
                                            ([4, 4, 128, 7, 1], 8, 16, 64), ([3], 1, 2, 128), ([6, 11], 5, 4, 16),
                                            ([300, 2, 257], 4, 2, 64), ([256, 40], 2, 4, 32), ([33, 64, 65], 4, 2, 128),
                                            ([700], 3, 2, 16)])
@pytest.mark.parametrize("half", [False, True])
def test_cross_attention(env, lens, beam, H, dh, half):
    lsq, torch = env
    rng = np.random.default_rng(sum(lens) + beam)
    d, B = H * dh, len(lens)
    cast = _h if half else (lambda a: np.asarray(a, np.float32))
    q = cast(rng.standard_normal((B * beam, d)))
    kv = cast(rng.standard_normal((sum(lens), 2 * d)))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    td = torch.float16 if half else torch.float32
    out = torch.full((B * beam, d), 7.0, dtype=td, device="cuda")
    lsq.k_cross_attention(_dev(torch, q, td), _dev(torch, kv, td), _dev(torch, off), _dev(torch, np.array(lens, np.int32)),
                          out, B, beam, H, max(lens))
    ref = np.concatenate([O.attention(q[b * beam:(b + 1) * beam].astype(np.float64),
                                      kv[off[b]:off[b + 1], :d].astype(np.float64),
                                      kv[off[b]:off[b + 1], d:].astype(np.float64), H) for b in range(B)])
    tol = 1.5e-3 if half else 2e-5
    np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=tol, atol=tol)


@pytest.mark.parametrize("lens,beam,H,splits", [([5], 4, 16, 4), ([130, 7], 4, 16, 2), ([33, 60], 3, 8, 1), ([1, 2, 90, 49], 2, 4, 4),
                                               ([257], 1, 1, 3), ([40, 40, 41, 200, 9, 64, 64, 3], 1, 16, 4),
                                               ([7, 50, 33, 3, 90, 12, 28, 28, 61, 5, 17, 44, 2, 130, 29, 30], 4, 16, 2)])
def test_cross_attention_that_makes_its_queries(env, lens, beam, H, splits):
    """LayerNorm + query product + attention in one kernel: the normalised rows are bit-identical to those of
    the product kernel that normalises its input, the queries are the same bits too, so the output equals
    attention over those queries (up to the order in which the keys are summed), and the oracle's."""
    lsq, torch = env
    rng = np.random.default_rng(sum(lens) * 7 + beam + H)
    d, B = H * 64, len(lens)
    rows = B * beam
    x = _h(rng.standard_normal((rows, d)) * 2)
    P = (rng.standard_normal((splits, rows, d)) * 0.5).astype(np.float32)
    lb, g, b = _h(rng.standard_normal(d) * 0.3), _h(1 + 0.3 * rng.standard_normal(d)), _h(0.3 * rng.standard_normal(d))
    Wq, bq = _h(rng.standard_normal((d, d)) * 0.05), _h(rng.standard_normal(d) * 0.5)
    kv = _h(rng.standard_normal((sum(lens), 2 * d)))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    h = torch.float16
    dx, dP, dkv = _dev(torch, x, h), _dev(torch, P), _dev(torch, kv, h)
    dlb, dg, db, dW, dbq = (_dev(torch, a, h) for a in (lb, g, b, Wq, bq))
    doff, dlen = _dev(torch, off), _dev(torch, np.array(lens, np.int32))
    packed = lsq.k_pack_weights(dW)
    x_new = torch.full((rows, d), 7.0, dtype=h, device="cuda")
    out = torch.full((rows, d), 7.0, dtype=h, device="cuda")
    lsq.k_layernorm_cross_attention(dP, dlb, dg, db, dx, x_new, 1e-5, packed, dbq, dkv, doff, dlen, out, B, beam, H)
    assert torch.equal(dx, _dev(torch, x, h))                       # the residual input is left alone
    # the separate kernels: product that normalises its input, then attention
    x_new2 = torch.full_like(x_new, 9.0)
    q2 = torch.empty((rows, d), dtype=h, device="cuda")
    for r0 in range(0, rows, 8):                                    # that kernel takes 8 rows at most; rows are independent
        r1 = min(rows, r0 + 8)
        xn, qq = torch.empty((r1 - r0, d), dtype=h, device="cuda"), torch.empty((r1 - r0, d), dtype=h, device="cuda")
        lsq.k_layernorm_gemm(dP[:, r0:r1].contiguous(), dlb, dg, db, dx[r0:r1].contiguous(), xn, 1e-5, dW, dbq, qq)
        x_new2[r0:r1], q2[r0:r1] = xn, qq
    assert torch.equal(x_new, x_new2)
    out2 = torch.empty_like(out)
    lsq.k_cross_attention(q2, dkv, doff, dlen, out2, B, beam, H, max(lens))
    np.testing.assert_allclose(out.float().cpu().numpy(), out2.float().cpu().numpy(), rtol=2e-3, atol=2e-3)
    # the oracle, from the queries the kernels made (their rounding to float16 is part of the path)
    qf = q2.float().cpu().numpy()
    ref = np.concatenate([O.attention(qf[i * beam:(i + 1) * beam].astype(np.float64),
                                      kv[off[i]:off[i + 1], :d].astype(np.float64),
                                      kv[off[i]:off[i + 1], d:].astype(np.float64), H) for i in range(B)])
    np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=1.5e-3, atol=1.5e-3)
    # and the queries themselves against the oracle's rows
    a = P.astype(np.float64).sum(0) + lb
    rows_ref = O.layer_norm(x.astype(np.float64) + a, g.astype(np.float64), b.astype(np.float64), 1e-5)
    np.testing.assert_allclose(qf, _h(rows_ref) @ Wq.astype(np.float64).T + bq, rtol=4e-3, atol=4e-3 * (1 + np.abs(qf).max()))


def _ln_rows(x, P, lb, g, b):
    """The oracle's LayerNorm of x + (slabs + bias), float64."""
    return O.layer_norm(x.astype(np.float64) + (P.astype(np.float64).sum(0) + lb), g.astype(np.float64), b.astype(np.float64), 1e-5)


@pytest.mark.parametrize("B,beam,H,T,nkeys,splits,table,pre", [
    (1, 4, 16, 60, 0, 0, True, False),       # first step: no history, rows taken as they are
    (1, 4, 16, 180, 171, 4, True, False),    # one sentence of the big model deep into a translation
    (3, 4, 8, 70, 33, 2, True, False),       # base model shape
    (16, 4, 16, 50, 17, 1, True, False),     # the most rows the kernel takes
    (5, 3, 4, 40, 39, 3, False, False),      # the cache's last position, rows that keep their own slab, beam 3
    (7, 2, 12, 90, 64, 4, True, False),      # four wavefronts per row
    (9, 1, 8, 130, 129, 2, False, False),    # beam 1
    (16, 2, 12, 192, 100, 4, False, True),   # pre-LN model, GPT-2-small shape: rows in pairs
    (8, 4, 12, 192, 63, 0, False, True),     # ... first layer: LayerNorm of the rows as they are
    (31, 1, 8, 80, 79, 2, False, True),      # ... an odd row count
    (16, 4, 4, 70, 0, 1, False, True),       # ... no history
])
def test_self_attention_block(env, B, beam, H, T, nkeys, splits, table, pre):
    """[LayerNorm +] QKV slice + cache append + self-attention + per-head output projection in one launch: every
    stage against the oracle, stage by stage from the values the kernel itself stored before it.  pre: the
    arithmetic of pre-LN models (the residual sum is stored, its LayerNorm is multiplied)."""
    lsq, torch = env
    rng = np.random.default_rng(B * 131 + beam * 17 + H + nkeys)
    d, rows = H * 64, B * beam
    h = torch.float16
    x = _h(rng.standard_normal((rows, d)) * (2 if splits else 1))
    lb, g, b = _h(rng.standard_normal(d) * 0.3), _h(1 + 0.3 * rng.standard_normal(d)), _h(0.3 * rng.standard_normal(d))
    P = (rng.standard_normal((max(splits, 1), rows, d)) * 0.5).astype(np.float32)
    Wqkv, bqkv = _h(rng.standard_normal((3 * d, d)) * 0.05), _h(rng.standard_normal(3 * d) * 0.5)
    Wo = _h(rng.standard_normal((d, d)) * 0.05)
    Kc, Vc = _h(rng.standard_normal((rows, T, d))), _h(rng.standard_normal((rows, T, d)))
    Kc[:, nkeys:], Vc[:, nkeys:] = np.nan, np.nan           # what lies beyond the history may be read, and must not matter
    slab = rng.integers(0, beam, size=(rows, T + 1)).astype(np.int32)
    slab[:, nkeys:] = rng.choice([1 << 20, -5, beam, -(1 << 30)], size=(rows, T + 1 - nkeys))
    dK, dV = _dev(torch, Kc, h), _dev(torch, Vc, h)
    dx, dP = _dev(torch, x, h), _dev(torch, P)
    x_new = torch.full((rows, d), 7.0, dtype=h, device="cuda")
    P_out = torch.full((H, rows, d), 7.0, dtype=torch.float32, device="cuda")
    dWqkv, dWo = _dev(torch, Wqkv, h), _dev(torch, Wo, h)
    lsq.k_self_attention_block(dP if splits else None, _dev(torch, lb, h), _dev(torch, g, h), _dev(torch, b, h), dx,
                               x_new if splits else None, 1e-5, lsq.k_pack_weights(dWqkv), _dev(torch, bqkv, h),
                               lsq.k_pack_weights(dWo), dK, dV, _dev(torch, slab) if table else None, nkeys, P_out, B, beam, H,
                               pre_ln=pre)
    assert torch.equal(dx, _dev(torch, x, h))
    # 1. the normalised rows
    if pre:
        stream = x
        if splits:   # the residual stream, stored; its LayerNorm is what the products see
            stream = x_new.float().cpu().numpy()
            np.testing.assert_allclose(stream, x.astype(np.float64) + (P[:splits].astype(np.float64).sum(0) + lb), rtol=1e-3, atol=1e-3)
        got_rows = _h(O.layer_norm(stream.astype(np.float64), g.astype(np.float64), b.astype(np.float64), 1e-5))
    elif splits:
        got_rows = x_new.float().cpu().numpy()
        np.testing.assert_allclose(got_rows, _ln_rows(x, P[:splits], lb, g, b), rtol=2e-3, atol=2e-3)
    else:
        got_rows = x
    # 2. k and v of the new position, written to the cache at index nkeys and nowhere else
    qkv = got_rows.astype(np.float64) @ Wqkv.astype(np.float64).T + bqkv
    gK, gV = dK.float().cpu().numpy(), dV.float().cpu().numpy()
    tol = 4e-3 * (1 + np.abs(qkv).max())
    np.testing.assert_allclose(gK[:, nkeys], qkv[:, d:2 * d], rtol=4e-3, atol=tol)
    np.testing.assert_allclose(gV[:, nkeys], qkv[:, 2 * d:], rtol=4e-3, atol=tol)
    keep = np.ones(T, bool)
    keep[nkeys] = False
    assert np.array_equal(gK[:, keep], Kc[:, keep], equal_nan=True) and np.array_equal(gV[:, keep], Vc[:, keep], equal_nan=True)
    # 3. attention over the history (through the table) plus the new position, with the kernel's own k and v there
    q = _h(qkv[:, :d])
    j = np.arange(nkeys)
    ctx = np.empty((rows, d))
    for r in range(rows):
        src = (r - r % beam + slab[r, :nkeys]) if table else np.full(nkeys, r)
        Kr = np.concatenate([Kc[src, j], gK[r:r + 1, nkeys]]).astype(np.float64)
        Vr = np.concatenate([Vc[src, j], gV[r:r + 1, nkeys]]).astype(np.float64)
        ctx[r] = O.attention(q[r:r + 1].astype(np.float64), Kr, Vr, H)[0]
    # 4. the heads' shares of the output projection: each slab and their sum
    got = P_out.cpu().numpy().astype(np.float64)
    ref = np.stack([ctx[:, hh * 64:(hh + 1) * 64] @ Wo[:, hh * 64:(hh + 1) * 64].astype(np.float64).T for hh in range(H)])
    scale = np.abs(ref).max()
    # (a query that rounds to the neighbouring float16 value moves a score by up to 1e-3 * |k|)
    np.testing.assert_allclose(got, ref, rtol=0, atol=6e-3 * scale)
    np.testing.assert_allclose(got.sum(0), ctx @ Wo.astype(np.float64).T, rtol=0, atol=6e-3 * np.abs(ref.sum(0)).max())


@pytest.mark.parametrize("lens,beam,H,splits", [([5], 4, 16, 16), ([130, 7], 4, 16, 16), ([33, 60, 2], 3, 8, 8), ([1, 2, 90, 49], 2, 4, 4),
                                               ([257], 1, 12, 12), ([40, 40, 41, 200, 9, 64, 64, 3], 1, 16, 1),
                                               ([7, 50, 33, 3, 90, 12, 28, 28, 61, 5, 17, 44, 2, 130, 29, 30], 4, 16, 16)])
def test_cross_attention_block(env, lens, beam, H, splits):
    """LayerNorm over per-head slabs + query slice + cross-attention + per-head output projection in one launch."""
    lsq, torch = env
    rng = np.random.default_rng(sum(lens) * 5 + beam + H)
    d, B = H * 64, len(lens)
    rows = B * beam
    h = torch.float16
    x = _h(rng.standard_normal((rows, d)) * 2)
    P = (rng.standard_normal((splits, rows, d)) * 0.3).astype(np.float32)
    lb, g, b = _h(rng.standard_normal(d) * 0.3), _h(1 + 0.3 * rng.standard_normal(d)), _h(0.3 * rng.standard_normal(d))
    Wq, bq = _h(rng.standard_normal((d, d)) * 0.05), _h(rng.standard_normal(d) * 0.5)
    Wo = _h(rng.standard_normal((d, d)) * 0.05)
    kv = _h(rng.standard_normal((sum(lens), 2 * d)))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    dx = _dev(torch, x, h)
    x_new = torch.full((rows, d), 7.0, dtype=h, device="cuda")
    P_out = torch.full((H, rows, d), 7.0, dtype=torch.float32, device="cuda")
    lsq.k_cross_attention_block(_dev(torch, P), _dev(torch, lb, h), _dev(torch, g, h), _dev(torch, b, h), dx, x_new, 1e-5,
                                lsq.k_pack_weights(_dev(torch, Wq, h)), _dev(torch, bq, h),
                                lsq.k_pack_weights(_dev(torch, Wo, h)), _dev(torch, kv, h), _dev(torch, off),
                                _dev(torch, np.array(lens, np.int32)), P_out, B, beam, H)
    assert torch.equal(dx, _dev(torch, x, h))
    got_rows = x_new.float().cpu().numpy()
    np.testing.assert_allclose(got_rows, _ln_rows(x, P, lb, g, b), rtol=2e-3, atol=2e-3)
    q = _h(got_rows.astype(np.float64) @ Wq.astype(np.float64).T + bq)
    ctx = np.concatenate([O.attention(q[i * beam:(i + 1) * beam].astype(np.float64),
                                      kv[off[i]:off[i + 1], :d].astype(np.float64),
                                      kv[off[i]:off[i + 1], d:].astype(np.float64), H) for i in range(B)])
    got = P_out.cpu().numpy().astype(np.float64)
    ref = np.stack([ctx[:, hh * 64:(hh + 1) * 64] @ Wo[:, hh * 64:(hh + 1) * 64].astype(np.float64).T for hh in range(H)])
    np.testing.assert_allclose(got, ref, rtol=0, atol=6e-3 * np.abs(ref).max())
    np.testing.assert_allclose(got.sum(0), ctx @ Wo.astype(np.float64).T, rtol=0, atol=6e-3 * np.abs(ref.sum(0)).max())


def _oracle_row_topk(logits, score, finished, k, eos):
    """Per row: the oracle's candidate scores and a full sort."""
    M, V = logits.shape
    os_, oi = np.full((M, k), -np.inf, np.float32), np.full((M, k), -1, np.int32)
    logp = O.log_softmax(logits.astype(np.float32))
    for r in range(M):
        if finished[r]:
            os_[r, 0], oi[r, 0] = score[r], eos
            continue
        c = (score[r] + logp[r]).astype(np.float32)
        best = O.topk_by_full_sort(c, np.arange(V), k)
        os_[r, :len(best)], oi[r, :len(best)] = c[best], best
    return os_, oi


@pytest.mark.parametrize("lens,beam,H", [([7] * 17, 4, 2), (list(range(1, 130)), 4, 4), ([33, 1, 64, 2] * 8 + [5], 2, 16),
                                         ([3] * 70, 1, 1), ([9, 140, 2] * 9, 3, 8)])
def test_cross_attention_that_makes_its_queries_many_rows(env, lens, beam, H):
    """Query product + cross-attention in one kernel for more than 64 rows (groups of sentences per
    workgroup, a last group that is not full, sentences of 1 to 140 keys): against the oracle's attention
    over q = x . Wq^T + bq rounded to float16, and against the two separate kernels."""
    lsq, torch = env
    rng = np.random.default_rng(sum(lens) + beam * 3 + H)
    d, B = H * 64, len(lens)
    rows = B * beam
    assert rows > 64
    x = _h(rng.standard_normal((rows, d)))
    Wq, bq = _h(rng.standard_normal((d, d)) * 0.05), _h(rng.standard_normal(d) * 0.5)
    kv = _h(rng.standard_normal((sum(lens), 2 * d)))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    h = torch.float16
    dx, dkv, dW, dbq = _dev(torch, x, h), _dev(torch, kv, h), _dev(torch, Wq, h), _dev(torch, bq, h)
    doff, dlen = _dev(torch, off), _dev(torch, np.array(lens, np.int32))
    out = torch.full((rows, d), 7.0, dtype=h, device="cuda")
    lsq.k_cross_attention_q(dx, lsq.k_pack_weights(dW), dbq, dkv, doff, dlen, out, B, beam, H)
    q2 = torch.empty((rows, d), dtype=h, device="cuda")
    lsq.k_gemm(dx, dW, dbq, q2)
    out2 = torch.empty_like(out)
    lsq.k_cross_attention(q2, dkv, doff, dlen, out2, B, beam, H, max(lens))
    got = out.float().cpu().numpy()
    np.testing.assert_allclose(got, out2.float().cpu().numpy(), rtol=2e-3, atol=2e-3)
    qref = _h(x.astype(np.float64) @ Wq.astype(np.float64).T + bq).astype(np.float64)
    ref = np.concatenate([O.attention(qref[i * beam:(i + 1) * beam], kv[off[i]:off[i + 1], :d].astype(np.float64),
                                      kv[off[i]:off[i + 1], d:].astype(np.float64), H) for i in range(B)])
    np.testing.assert_allclose(got, ref, rtol=2.5e-3, atol=2.5e-3)


@pytest.mark.parametrize("M,V,k", [(8, 1000, 4), (5, 12, 3), (33, 32000, 4), (6, 50257, 8), (4, 8192, 1),
                                   (3, 8200, 5), (2, 65536, 4), (7, 2048, 4), (9, 5, 5), (5, 1000, 32), (4, 32000, 16),
                                   (3, 50257, 32), (6, 40, 32), (2, 20, 32), (3, 50257, 16)])
@pytest.mark.parametrize("case", ["random", "ties", "all_equal", "dead_and_finished"])
def test_row_topk(env, M, V, k, case):
    lsq, torch = env
    rng = np.random.default_rng(M + V + k)
    logits = (rng.standard_normal((M, V)) * 0.7).astype(np.float32)
    score = -(rng.random(M) * 50).astype(np.float32)
    fin = np.zeros(M, np.int32)
    if case == "ties":
        logits = np.round(logits * 2) / 2            # heavy duplication: order decided by token id
    elif case == "all_equal":
        logits[:] = 0.125
    elif case == "dead_and_finished":
        score[::2] = -np.inf
        fin[1::3] = 1
    eos = 2
    os_ = torch.zeros(M, k, dtype=torch.float32, device="cuda")
    oi = torch.zeros(M, k, dtype=torch.int32, device="cuda")
    lsq.k_row_topk(_dev(torch, logits), _dev(torch, score), _dev(torch, fin), k, eos, os_, oi)
    got_s, got_i = os_.cpu().numpy(), oi.cpu().numpy()
    ref_s, ref_i = _oracle_row_topk(logits, score, fin, k, eos)
    if case == "random":
        # distinct logits: indices are unique wherever neighbouring candidates differ by more than rounding
        c = np.sort(-(score[:, None] + O.log_softmax(logits.astype(np.float64))), axis=1)[:, :k + 1]
        clear = (np.diff(c, axis=1) > 1e-4).all(axis=1) | ~np.isfinite(c).all(axis=1)
        assert clear.mean() > 0.5
        assert np.array_equal(got_i[clear], ref_i[clear])
    else:
        assert np.array_equal(got_i, ref_i)          # bit-exact indices on identical scores
    both = np.isfinite(ref_s)
    assert np.array_equal(np.isfinite(got_s), both)
    np.testing.assert_allclose(got_s[both], ref_s[both], rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("M,N,K", [(4, 1000, 64), (33, 32000, 512), (64, 5000, 1024), (8, 37, 16), (65, 32000, 1024),
                                   (512, 32000, 1024), (130, 26000, 64), (300, 50257, 768 - 768 % 64), (1, 32, 16),
                                   # the tiled kernels: ragged columns and k, vocabulary-sized products of few rows,
                                   # a shape that would otherwise go to the kernel without statistics
                                   (100, 1003, 72), (48, 32000, 512), (20, 26000, 520), (300, 4100, 128), (32, 50257, 768)])
def test_logit_product_group_statistics(env, M, N, K):
    """The logit product's (largest, sum of exponentials) per row and 32-column group, against numpy on the logits
    the same launch wrote (which are checked against the float64 product)."""
    lsq, torch = env
    assert lsq.k_gemm_logits_supported(M, N, K)
    rng = np.random.default_rng(M + N + K)
    A, B = _h(rng.standard_normal((M, K))), _h(rng.standard_normal((N, K)) * 0.2)
    G = (N + 31) // 32
    C = torch.full((M, N), 7.0, dtype=torch.float32, device="cuda")
    st = torch.full((M, G, 2), 7.0, dtype=torch.float32, device="cuda")
    lsq.k_gemm_logits(_dev(torch, A, torch.float16), _dev(torch, B, torch.float16), C, st)
    got, gst = C.cpu().numpy(), st.cpu().numpy()
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    np.testing.assert_allclose(got, ref, rtol=0, atol=2e-6 * (np.abs(A) @ np.abs(B).T).max())
    pad = np.full((M, G * 32), -np.inf)
    pad[:, :N] = got
    grp = pad.reshape(M, G, 32)
    gmax = grp.max(-1)
    assert np.array_equal(gst[..., 0], gmax.astype(np.float32))              # the stored logits' own maxima, bit for bit
    np.testing.assert_allclose(gst[..., 1], np.exp(grp - gmax[..., None]).sum(-1), rtol=2e-6)


@pytest.mark.parametrize("M,V,k", [(8, 1000, 4), (5, 12, 3), (33, 32000, 4), (6, 50257, 8), (4, 8192, 1), (3, 8200, 5),
                                   (2, 65536, 4), (7, 2048, 4), (9, 5, 5), (130, 32000, 4), (3, 33, 2)])
@pytest.mark.parametrize("case", ["random", "ties", "all_equal", "dead_and_finished", "one_group_holds_all"])
def test_row_topk_from_group_statistics(env, M, V, k, case):
    """The retrieve kernel that works from the logit product's group statistics: the same candidates as the kernel
    that reads the whole row, and the oracle's."""
    lsq, torch = env
    rng = np.random.default_rng(M + V + k)
    logits = (rng.standard_normal((M, V)) * 0.7).astype(np.float32)
    score = -(rng.random(M) * 50).astype(np.float32)
    fin = np.zeros(M, np.int32)
    if case == "ties":
        logits = np.round(logits * 2) / 2
    elif case == "all_equal":
        logits[:] = 0.125                              # every group reaches the threshold: the exact fallback
    elif case == "dead_and_finished":
        score[::2] = -np.inf
        fin[1::3] = 1
    elif case == "one_group_holds_all":
        at = (V // 2) // 32 * 32
        logits[:, at:at + min(32, V - at)] += 9.0      # the k best of every row sit in one group
    eos = 2
    G = (V + 31) // 32
    pad = np.full((M, G * 32), -np.inf, np.float32)
    pad[:, :V] = logits
    grp = pad.reshape(M, G, 32)
    gmax = grp.max(-1)
    stats = np.stack([gmax, np.exp(grp - gmax[..., None]).sum(-1)], axis=-1).astype(np.float32)
    dl, ds, df = _dev(torch, logits), _dev(torch, score), _dev(torch, fin)
    os_ = torch.zeros(M, k, dtype=torch.float32, device="cuda")
    oi = torch.zeros(M, k, dtype=torch.int32, device="cuda")
    lsq.k_row_topk_groups(dl, _dev(torch, stats), ds, df, k, eos, os_, oi)
    os2 = torch.zeros(M, k, dtype=torch.float32, device="cuda")
    oi2 = torch.zeros(M, k, dtype=torch.int32, device="cuda")
    lsq.k_row_topk(dl, ds, df, k, eos, os2, oi2)
    got_s, got_i = os_.cpu().numpy(), oi.cpu().numpy()
    ref_s, ref_i = _oracle_row_topk(logits, score, fin, k, eos)
    if case in ("random", "one_group_holds_all"):
        c = np.sort(-(score[:, None] + O.log_softmax(logits.astype(np.float64))), axis=1)[:, :k + 1]
        clear = (np.diff(c, axis=1) > 1e-4).all(axis=1) | ~np.isfinite(c).all(axis=1)
        assert clear.mean() > 0.5
        assert np.array_equal(got_i[clear], ref_i[clear]) and np.array_equal(got_i[clear], oi2.cpu().numpy()[clear])
    else:
        assert np.array_equal(got_i, ref_i) and np.array_equal(got_i, oi2.cpu().numpy())
    both = np.isfinite(ref_s)
    assert np.array_equal(np.isfinite(got_s), both)
    np.testing.assert_allclose(got_s[both], ref_s[both], rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(got_s[both], os2.cpu().numpy()[both], rtol=2e-6, atol=2e-6)


@pytest.mark.parametrize("M,V,k", [(32, 50257, 8), (32, 32000, 32), (5, 1000, 32), (6, 40, 32), (3, 50257, 1), (70, 8200, 16)])
@pytest.mark.parametrize("case", ["random", "ties", "all_equal"])
def test_largest_logits_from_group_statistics(env, M, V, k, case):
    """Sampling's candidates (the k largest logits, value descending, token ascending) from the group statistics."""
    lsq, torch = env
    rng = np.random.default_rng(M + V + k + 1)
    logits = (rng.standard_normal((M, V)) * 0.7).astype(np.float32)
    if case == "ties":
        logits = np.round(logits * 2) / 2
    elif case == "all_equal":
        logits[:] = -0.5
    G = (V + 31) // 32
    pad = np.full((M, G * 32), -np.inf, np.float32)
    pad[:, :V] = logits
    grp = pad.reshape(M, G, 32)
    gmax = grp.max(-1)
    stats = np.stack([gmax, np.exp(grp - gmax[..., None]).sum(-1)], axis=-1).astype(np.float32)
    os_ = torch.zeros(M, k, dtype=torch.float32, device="cuda")
    oi = torch.zeros(M, k, dtype=torch.int32, device="cuda")
    lsq.k_row_topk_groups(_dev(torch, logits), _dev(torch, stats), None, None, k, 2, os_, oi, raw=True)
    got_s, got_i = os_.cpu().numpy(), oi.cpu().numpy()
    kk = min(k, V)
    order = np.lexsort((np.broadcast_to(np.arange(V), (M, V)), -logits), axis=1)[:, :kk]
    assert np.array_equal(got_i[:, :kk], order)
    assert np.array_equal(got_s[:, :kk], np.take_along_axis(logits, order, 1))
    assert (got_i[:, kk:] == -1).all() and np.isneginf(got_s[:, kk:]).all()


def _state(rng, B, k, V, T, t, eos, finished_frac):
    M = B * k
    tokens = rng.integers(4, V, size=(M, T + 1)).astype(np.int32)
    tokens[:, 0] = 1
    fin = (rng.random(M) < finished_frac)
    length = np.where(fin, rng.integers(1, t + 1, size=M) if t >= 1 else 0, t).astype(np.int32)
    if t == 0:
        fin[:] = False
    score = np.sort(-(rng.random((B, k)) * 5).astype(np.float32), axis=1)[:, ::-1].copy()
    cap = rng.integers(t + 1, T + 1, size=B).astype(np.int32)
    return tokens, length, fin, score, cap


@pytest.mark.parametrize("B,k,V,T,t", [(2, 4, 1000, 8, 0), (5, 3, 12, 11, 4), (128, 4, 32000, 178, 40),
                                       (3, 8, 50, 9, 8), (4, 1, 100, 6, 2), (6, 5, 37, 12, 7)])
@pytest.mark.parametrize("ties", [False, True])
def test_row_topk_then_refine_matches_oracle_step(env, B, k, V, T, t, ties):
    """retrieve + re-rank on seeded logits and beam state == the oracle's softmax + full sort +
    bookkeeping, including finished hypotheses, caps, -inf beams and exact ties."""
    lsq, torch = env
    rng = np.random.default_rng(B * 31 + V + t)
    M = B * k
    import lsq_synth as S
    hp = S.HParams(n_enc=1, n_dec=1, d_model=8, n_heads=1, d_ffn=8, vocab=V, max_pos=8)
    m = O.Model(S.make_blob(hp))
    tokens, length, fin, score, cap = _state(rng, B, k, V, T, t, m.eos, 0.0 if t == 0 else 0.3)
    if t == 0:
        score[:, 1:] = -np.inf
        score[:, 0] = 0
    logits = (rng.standard_normal((M, V)) * 0.7).astype(np.float32)
    if ties:
        logits = np.round(logits * 2) / 2
        score = np.round(score * 2) / 2                      # equal beam scores too: flat index decides
    # oracle step
    st = O.DecodeState(m, np.ones(B, np.int32), k, T)
    st.tokens, st.len, st.finished, st.score, st.cap, st.t = tokens.copy(), length.copy(), fin.copy(), score.copy(), cap.copy(), t
    st.Kc, st.Vc = [], []
    tok, par, sc, margin = O.beam_select(m, st, logits)
    active_ref = O.beam_advance(m, st, tok, par, sc)
    # library
    d_score = _dev(torch, score.reshape(-1))
    d_tokens, d_len, d_fin = _dev(torch, tokens), _dev(torch, length), _dev(torch, fin.astype(np.int32))
    cs = torch.zeros(M, k, dtype=torch.float32, device="cuda")
    ci = torch.zeros(M, k, dtype=torch.int32, device="cuda")
    parent = torch.zeros(M, dtype=torch.int32, device="cuda")
    active = torch.zeros(1, dtype=torch.int32, device="cuda")
    lsq.k_row_topk(_dev(torch, logits), d_score, d_fin, k, m.eos, cs, ci)
    slab0 = rng.integers(0, k, size=(M, T + 1)).astype(np.int32)
    slab0[:, t + 1:] = -7                                   # not yet meaningful
    d_slab = _dev(torch, slab0)
    lsq.k_beam_refine(cs, ci, d_score, d_tokens, d_len, d_fin, parent, _dev(torch, cap), active, B, k, V, T, t, m.eos,
                      slab=d_slab)
    ok = (margin > 1e-4) | ties        # with exact ties both sides see identical scores per row
    g_par = parent.cpu().numpy().reshape(B, k)
    # the slab table follows the library's own parents exactly: history gathered, next position = own row
    g_slab = d_slab.cpu().numpy()
    src_row = (np.arange(M) // k) * k + g_par.reshape(-1)
    assert np.array_equal(g_slab[:, :t + 1], slab0[src_row, :t + 1])
    assert np.array_equal(g_slab[:, t + 1], np.arange(M) % k)
    assert (g_slab[:, t + 2:] == -7).all()
    g_tok, g_len, g_fin = d_tokens.cpu().numpy(), d_len.cpu().numpy(), d_fin.cpu().numpy()
    g_score = d_score.cpu().numpy().reshape(B, k)
    assert ok.mean() > 0.5
    for b in np.nonzero(ok)[0]:
        r = slice(b * k, (b + 1) * k)
        assert np.array_equal(g_par[b], par[b])
        assert np.array_equal(g_len[r], st.len[r]) and np.array_equal(g_fin[r] != 0, st.finished[r])
        for j in range(k):
            n = st.len[b * k + j]
            assert np.array_equal(g_tok[b * k + j, :n + 1], st.tokens[b * k + j, :n + 1])
        f = np.isfinite(sc[b])
        assert np.array_equal(np.isfinite(g_score[b]), f)
        np.testing.assert_allclose(g_score[b][f], sc[b][f], rtol=1e-5, atol=1e-5)
    if ok.all():
        assert int(active.item()) == active_ref


@pytest.mark.parametrize("layers,B,k,T,d,npos", [(2, 3, 4, 8, 64, 8), (12, 16, 4, 60, 1024, 41), (4, 5, 3, 9, 32, 1),
                                                 (2, 2, 8, 20, 128, 13), (3, 4, 1, 6, 64, 6), (2, 7, 5, 33, 72 * 8, 20)])
@pytest.mark.parametrize("half", [False, True])
def test_cache_reorder(env, layers, B, k, T, d, npos, half):
    lsq, torch = env
    rng = np.random.default_rng(layers + B + d)
    M = B * k
    cache = rng.standard_normal((layers, M, T, d)).astype(np.float16 if half else np.float32)
    parent = rng.integers(0, k, size=(B, k)).astype(np.int32)
    parent[0] = np.arange(k)                               # one sentence whose beams do not move
    if B > 1:
        parent[1] = np.roll(np.arange(k), 1)               # a pure permutation (cycle)
    dc = _dev(torch, cache)
    lsq.k_cache_reorder(dc, _dev(torch, parent.reshape(-1)), layers, B, k, T, d, npos)
    rows = (np.arange(B)[:, None] * k + parent).reshape(-1)
    ref = cache.copy()
    ref[:, :, :npos] = cache[:, rows, :npos]               # positions beyond npos are untouched
    assert np.array_equal(dc.cpu().numpy(), ref)
