"""GPU parity of the kernel-level entry points against the oracle's pieces, called
through the C ABI.  Sizes span several tiles and ragged tails."""
import math

import numpy as np
import pytest

from oracle import stage_oracle as O
from paper_2007_01045_amd import binding as B
from paper_2007_01045_amd import inputs as I
from tests.stage_util import rel_l2, to_np

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def dev(a, dtype):
    return torch.as_tensor(np.ascontiguousarray(a)).to(dtype).cuda().contiguous()


def rnd(tag, shape, scale=1.0, bf16=True):
    v = scale * I.normal(77, tag, int(np.prod(shape))).reshape(shape)
    return I.round_to_bf16(v).astype(np.float64) if bf16 else v.astype(np.float32).astype(np.float64)


TOL = {B.DTYPE_BF16: 6e-3, B.DTYPE_F32: 2e-5}
TD = {B.DTYPE_BF16: torch.bfloat16, B.DTYPE_F32: torch.float32}


def gemm_case(dtype, M, N, K, akS, bkS, epi, batch=1, nseg=1, expect_mfma=None, tile=0):
    bf = dtype == B.DTYPE_BF16
    td = TD[dtype]
    ks = K // nseg
    # logical operands per batch and segment
    A = rnd("A", (batch, nseg, M, ks), bf16=bf)
    Bm = rnd("B", (batch, nseg, N, ks), bf16=bf)
    bias = rnd("bias", (batch, N), bf16=bf)
    aux = rnd("aux", (batch, M, N), bf16=bf and not (epi & B.EPI_AUX32))
    C0 = rnd("C0", (batch, M, N), bf16=False)
    acc = np.stack([sum(A[z, i] @ Bm[z, i].T for i in range(nseg)) for z in range(batch)])
    t = acc.copy()
    if epi & B.EPI_BIAS:
        t += bias[:, None, :]
    if epi & B.EPI_ADD:
        t += aux
    if epi & B.EPI_MUL:
        t *= aux
    A_mem = A.transpose(0, 1, 3, 2) if akS else A        # k-strided: [k][rows]
    B_mem = Bm.transpose(0, 1, 3, 2) if bkS else Bm
    dA, dB = dev(A_mem, td), dev(B_mem, td)
    dbias, daux = dev(bias, td), dev(aux, torch.float32 if epi & B.EPI_AUX32 else td)
    d = B.dapple_gemm_desc()
    d.A, d.B, d.bias, d.aux = dA.data_ptr(), dB.data_ptr(), dbias.data_ptr(), daux.data_ptr()
    d.M, d.N, d.K = M, N, K
    d.lda, d.ldb = (M if akS else ks), (N if bkS else ks)
    d.ldc = d.ldaux = N
    d.a_kstrided, d.b_kstrided = int(akS), int(bkS)
    d.kseg_len, d.segA, d.segB = ks, M * ks, N * ks
    d.batch, d.sA, d.sB, d.sC, d.sBias = batch, nseg * M * ks, nseg * N * ks, M * N, N
    d.epi = epi
    d.tile = tile
    if epi & B.EPI_ACC32:
        dC = dev(C0, torch.float32)
        want = [C0 + t]
    elif epi & B.EPI_GELU:
        dC, dC2 = torch.empty(batch, M, N, dtype=td, device="cuda"), torch.empty(batch, M, N, dtype=td, device="cuda")
        d.C2 = dC2.data_ptr()
        want = [O.gelu(t), O.gelu_grad(t)]
    else:
        dC = torch.empty(batch, M, N, dtype=td, device="cuda")
        want = [t]
    d.C = dC.data_ptr()
    if epi & B.EPI_BSUM:          # column sums of B over k, added to what the vector holds
        bs0 = rnd("bs0", (N,), bf16=False)
        dbs = dev(bs0, torch.float32)
        d.bsum = dbs.data_ptr()
    if epi & B.EPI_ROWDOT:        # per row and block of 32 columns: sum of (stored output) * aux
        nblk = (N + 31) // 32
        drd = torch.full((nblk, M), float("nan"), dtype=torch.float32, device="cuda")
        d.rowdot = drd.data_ptr()
    used = B.dapple_gemm(dtype, d)
    torch.cuda.synchronize()
    if expect_mfma is not None:
        assert used == int(expect_mfma)
    if epi & B.EPI_ROWDOT:
        stored = to_np(dC)[0].astype(np.float64)
        prod = stored * aux[0].astype(np.float64)
        want_rd = np.stack([prod[:, 32 * j:32 * j + 32].sum(axis=1) for j in range(nblk)])
        got_rd = to_np(drd)
        assert np.isfinite(got_rd).all(), "a row sum was not written"
        assert rel_l2(got_rd, want_rd) < 1e-5, (M, N, K, rel_l2(got_rd, want_rd))
        assert np.abs(got_rd - want_rd).max() < 1e-4 * max(np.abs(want_rd).max(), 1.0)
    if epi & B.EPI_BSUM:
        want_bs = bs0 + sum(Bm[0, i].sum(axis=1) for i in range(nseg))
        assert rel_l2(to_np(dbs), want_bs) < (1e-5 if bf else 2e-5), (M, N, K, rel_l2(to_np(dbs), want_bs))
    got = [to_np(dC)] + ([to_np(dC2)] if epi & B.EPI_GELU else [])
    for g, w in zip(got, want):
        assert rel_l2(g, w) < TOL[dtype], (M, N, K, akS, bkS, epi, rel_l2(g, w))
        # element-wise: no element may be off by more than a few roundings of the largest value
        assert np.abs(g - w).max() < (3e-2 if bf else 1e-4) * max(np.abs(w).max(), 1.0)


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6])
def test_gemm_mfma_every_tile_shape_and_ring_depth(tile):
    # K = 64 * (1, 2, 3, 5, 7, 8): shorter than the ring, a multiple of no ring depth, and longer;
    # ragged M and N; both operand layouts; a segmented K
    for K in (64, 128, 192, 320, 448, 512):
        gemm_case(B.DTYPE_BF16, 328, 200, K, False, True, B.EPI_BIAS, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_BF16, 264, 136, 320, True, True, B.EPI_ACC32, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_BF16, 264, 136, 448, False, False, B.EPI_ADD, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_BF16, 200, 264, 3 * 192, False, False, B.EPI_ADD, nseg=3, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_BF16, 136, 264, 320, True, False, 0, batch=3, expect_mfma=True, tile=tile)


@pytest.mark.parametrize("tile", [0, 3, 4, 5])
def test_gemm_weight_gradient_with_bias_column_sums(tile):
    # C += A^T-layout product and bsum += column sums of B in one launch; ragged M, N; K = 64 * (1, 5, 32);
    # enough tiles for the 128x128 choice and few enough for the 128x64 one; the plain kernel for fp32
    for (M, N, K) in ((264, 136, 64), (264, 136, 320), (1024, 2048 + 8, 2048), (72, 40, 192)):
        gemm_case(B.DTYPE_BF16, M, N, K, True, True, B.EPI_ACC32 | B.EPI_BSUM, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_F32, 70, 52, 33, True, True, B.EPI_ACC32 | B.EPI_BSUM, expect_mfma=False, tile=tile)


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 6])
def test_gemm_row_sums_of_output_times_second_operand(tile):
    # ragged M and N (N not a multiple of 32: the last block is short), bf16 and fp32 second operand
    gemm_case(B.DTYPE_BF16, 328, 200, 192, False, False, B.EPI_ROWDOT | B.EPI_AUX32, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_BF16, 264, 136, 320, False, True, B.EPI_ROWDOT | B.EPI_BIAS, expect_mfma=True, tile=tile)
    gemm_case(B.DTYPE_BF16, 512, 256, 128, False, False, B.EPI_ROWDOT | B.EPI_AUX32, expect_mfma=True, tile=tile)


def test_gemm_row_sums_need_the_mfma_kernel():
    d = B.dapple_gemm_desc()
    x = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    d.A = d.B = d.C = d.aux = d.rowdot = x.data_ptr()
    d.M = d.N = d.K = 48
    d.lda = d.ldb = d.ldc = d.ldaux = 48
    def code(dtype):
        with pytest.raises(B.StageError) as e:
            B.dapple_gemm(dtype, d)
        return e.value.code
    d.epi = B.EPI_ROWDOT
    assert code(B.DTYPE_F32) == B.STAGE_E_CONFIG          # fp32: the plain kernel
    assert code(B.DTYPE_BF16) == B.STAGE_E_CONFIG         # K = 48: the plain kernel
    d.epi = B.EPI_ROWDOT | B.EPI_ADD
    assert code(B.DTYPE_BF16) == B.STAGE_E_CONFIG         # nothing else may use aux
    d.epi = B.EPI_ROWDOT
    d.rowdot = None
    assert code(B.DTYPE_BF16) == B.STAGE_E_NULL


@pytest.mark.parametrize("akS", [False, True])
@pytest.mark.parametrize("bkS", [False, True])
def test_gemm_mfma_layouts_ragged(akS, bkS):
    # 128x128 tiles with ragged M and N (multiples of 8 for k-strided operands)
    gemm_case(B.DTYPE_BF16, 328, 200, 192, akS, bkS, 0, expect_mfma=True)
    # enough tiles for the 256x128 and 256x256 variants
    gemm_case(B.DTYPE_BF16, 2048 + 64, 3720, 128, akS, bkS, B.EPI_BIAS, expect_mfma=True)
    gemm_case(B.DTYPE_BF16, 4096, 4096 + 16, 64, akS, bkS, 0, expect_mfma=True)


@pytest.mark.parametrize("epi", [B.EPI_BIAS, B.EPI_BIAS | B.EPI_ADD, B.EPI_MUL, B.EPI_ADD,
                                 B.EPI_BIAS | B.EPI_GELU, B.EPI_ACC32])
def test_gemm_mfma_epilogues(epi):
    gemm_case(B.DTYPE_BF16, 300, 264, 256, False, True, epi, expect_mfma=True)
    gemm_case(B.DTYPE_BF16, 264, 136, 128, True, True, epi, batch=3, expect_mfma=True)


def test_gemm_mfma_segments_and_batch():
    gemm_case(B.DTYPE_BF16, 272, 192, 3 * 128, False, False, B.EPI_ADD, nseg=3, expect_mfma=True)
    gemm_case(B.DTYPE_BF16, 136, 128, 64, False, True, B.EPI_BIAS, batch=3, expect_mfma=True)


def test_gemm_ragged_n_not_multiple_of_4():
    gemm_case(B.DTYPE_BF16, 130, 124, 64, False, False, B.EPI_BIAS, expect_mfma=True)
    gemm_case(B.DTYPE_BF16, 130, 122, 64, False, False, B.EPI_BIAS, expect_mfma=False)   # ldc % 4 != 0


@pytest.mark.parametrize("dtype", [B.DTYPE_F32, B.DTYPE_BF16])
def test_gemm_plain_kernel(dtype):
    for akS in (False, True):
        for bkS in (False, True):
            gemm_case(dtype, 37, 50, 24, akS, bkS, B.EPI_BIAS | B.EPI_ADD, expect_mfma=False)
    gemm_case(dtype, 33, 20, 36, False, False, B.EPI_ACC32, nseg=3, batch=2, expect_mfma=False)
    gemm_case(dtype, 19, 28, 16, False, True, B.EPI_BIAS | B.EPI_GELU, expect_mfma=False)


def attention_case(dtype, b, s, A, d):
    bf = dtype == B.DTYPE_BF16
    td = TD[dtype]
    H = A * d
    q, k, v, dctx = (rnd(t, (b, s, H), bf16=bf) for t in ("q", "k", "v", "dctx"))
    split = lambda t: t.reshape(b, s, A, d).transpose(0, 2, 1, 3)
    merge = lambda t: t.transpose(0, 2, 1, 3).reshape(b, s, H)
    ctx_ref, P = O.attention_fwd(split(q), split(k), split(v))
    dq_r, dk_r, dv_r = O.attention_bwd(split(dctx), split(q), split(k), split(v), P)
    dq, dk, dv, dc = dev(q, td), dev(k, td), dev(v, td), dev(dctx, td)
    ctx = torch.empty(b * s, H, dtype=td, device="cuda")
    lse = torch.empty(b, A, s, dtype=torch.float32, device="cuda")
    B.dapple_attention_fwd(dtype, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ctx.data_ptr(), lse.data_ptr(),
                           b, s, A, H)
    gq, gk, gv = (torch.empty(b * s, H, dtype=td, device="cuda") for _ in range(3))
    delta = torch.empty(b, A, s, dtype=torch.float32, device="cuda")
    B.dapple_attention_bwd(dtype, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ctx.data_ptr(), lse.data_ptr(),
                           dc.data_ptr(), gq.data_ptr(), gk.data_ptr(), gv.data_ptr(), delta.data_ptr(), b, s, A, H)
    torch.cuda.synchronize()
    tol = 1.2e-2 if bf else 2e-5
    assert rel_l2(to_np(ctx).reshape(b, s, H), merge(ctx_ref)) < tol
    # logsumexp of the scaled logits, log2 domain
    S = split(q) @ split(k).transpose(0, 1, 3, 2) / math.sqrt(d)
    lse_ref = (np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)) / math.log(2.0)
    assert np.abs(to_np(lse) - lse_ref).max() < (2e-2 if bf else 1e-4)
    for got, ref, n in ((gq, dq_r, "dq"), (gk, dk_r, "dk"), (gv, dv_r, "dv")):
        e = rel_l2(to_np(got).reshape(b, s, H), merge(ref))
        assert e < tol, (n, e)


def test_attention_mfma():
    attention_case(B.DTYPE_BF16, 2, 192, 3, 64)      # ragged: 192 = 128 + 64 rows
    attention_case(B.DTYPE_BF16, 1, 512, 2, 64)


@pytest.mark.parametrize("dtype", [B.DTYPE_F32, B.DTYPE_BF16])
def test_attention_plain(dtype):
    attention_case(dtype, 2, 16, 4, 16)
    attention_case(dtype, 1, 37, 3, 8)


@pytest.mark.parametrize("dtype,H", [(B.DTYPE_F32, 64), (B.DTYPE_F32, 1000), (B.DTYPE_BF16, 1024),
                                     (B.DTYPE_BF16, 264)])
def test_layernorm(dtype, H):
    bf = dtype == B.DTYPE_BF16
    td = TD[dtype]
    rows, eps = 77, 1e-5
    fix = (lambda a: I.round_to_bf16(a).astype(np.float64)) if bf else (lambda a: a.astype(np.float32).astype(np.float64))
    z = fix(rnd("z", (rows, H), 2.0, bf16=bf) + 0.5)
    g = fix(1 + rnd("g", (H,), 0.1, bf16=bf))
    be = rnd("be", (H,), 0.1, bf16=bf)
    dy = rnd("dy", (rows, H), bf16=bf)
    y_ref, cache = O.layernorm_fwd(z, g, be, eps)
    dz_ref, dg_ref, db_ref = O.layernorm_bwd(dy, cache, g)
    dz_, dg_, dbe = dev(z, td), dev(g, td), dev(be, td)
    y = torch.empty(rows, H, dtype=td, device="cuda")
    stats = torch.empty(rows, 2, dtype=torch.float32, device="cuda")
    B.dapple_layernorm_fwd(dtype, dz_.data_ptr(), dg_.data_ptr(), dbe.data_ptr(), y.data_ptr(), stats.data_ptr(),
                           rows, H, eps)
    ddy = dev(dy, td)
    dz = torch.empty(rows, H, dtype=td, device="cuda")
    partial = torch.empty(((rows + 7) // 8) * 3 * H, dtype=torch.float32, device="cuda")
    acc = torch.ones(3, H, dtype=torch.float32, device="cuda")       # accumulates on top of what is there
    B.dapple_layernorm_bwd(dtype, ddy.data_ptr(), dz_.data_ptr(), stats.data_ptr(), dg_.data_ptr(), dz.data_ptr(),
                           partial.data_ptr(), acc[0].data_ptr(), acc[1].data_ptr(), acc[2].data_ptr(), rows, H)
    torch.cuda.synchronize()
    tol = 5e-3 if bf else 1e-5
    assert rel_l2(to_np(y), y_ref) < tol
    assert np.abs(to_np(stats)[:, 0] - z.mean(-1)).max() < 1e-4
    assert rel_l2(to_np(stats)[:, 1], cache[1][:, 0]) < 1e-5
    assert rel_l2(to_np(dz), dz_ref) < tol
    a = to_np(acc) - 1.0
    assert rel_l2(a[0], dg_ref) < tol and rel_l2(a[1], db_ref) < tol
    assert rel_l2(a[2], dz_ref.sum(0)) < (3e-2 if bf else 1e-4)


@pytest.mark.parametrize("dtype", [B.DTYPE_F32, B.DTYPE_BF16])
def test_colsum(dtype):
    bf = dtype == B.DTYPE_BF16
    rows, cols, ld = 203, 1032, 1040
    X = rnd("X", (rows, ld), bf16=bf)
    dX = dev(X, TD[dtype])
    partial = torch.empty(((rows + 63) // 64) * cols, dtype=torch.float32, device="cuda")
    out = torch.full((cols,), 2.0, dtype=torch.float32, device="cuda")
    B.dapple_colsum(dtype, dX.data_ptr(), rows, cols, ld, partial.data_ptr(), out.data_ptr())
    torch.cuda.synchronize()
    assert rel_l2(to_np(out) - 2.0, X[:, :cols].sum(0)) < 1e-5


@pytest.mark.parametrize("seed", [5, 6])
def test_gemm_random_shapes(seed):
    """Random M, N, K (ragged against every tile size), layouts, epilogues, batches, K segments and tile
    choices, bf16 and fp32: whichever kernel takes the problem must agree with the float64 product."""
    import random
    rng = random.Random(seed)
    epis = [0, B.EPI_BIAS, B.EPI_BIAS | B.EPI_ADD, B.EPI_MUL, B.EPI_ADD, B.EPI_BIAS | B.EPI_GELU, B.EPI_ACC32]
    for case in range(30):
        dtype = rng.choice([B.DTYPE_BF16, B.DTYPE_BF16, B.DTYPE_F32])
        M = rng.choice([rng.randint(1, 64), rng.randint(65, 700), 8 * rng.randint(1, 80)])
        N = rng.choice([4 * rng.randint(1, 150), 8 * rng.randint(1, 70), rng.randint(1, 300)])
        nseg = rng.choice([1, 1, 2, 3])
        K = nseg * 8 * rng.randint(1, 40)
        akS, bkS = rng.random() < 0.5, rng.random() < 0.5
        epi = rng.choice(epis)
        batch = rng.choice([1, 1, 2, 3])
        tile = rng.randint(0, 6)
        print(f"case {case}: dtype={dtype} M={M} N={N} K={K} akS={akS} bkS={bkS} epi={epi} batch={batch} nseg={nseg} "
              f"tile={tile}", flush=True)
        gemm_case(dtype, M, N, K, akS, bkS, epi, batch=batch, nseg=nseg, tile=tile)


def test_attention_random_shapes():
    import random
    rng = random.Random(9)
    for case in range(16):
        dtype = rng.choice([B.DTYPE_BF16, B.DTYPE_F32])
        d = rng.choice([64, 64, 32, 16, 8])
        A, b = rng.randint(1, 4), rng.randint(1, 3)
        s = rng.choice([64, 128, 192, 320, 8, 24, 100])
        print(f"case {case}: dtype={dtype} b={b} s={s} A={A} d={d}", flush=True)
        attention_case(dtype, b, s, A, d)
