"""GPU parity: every stage of the HIP path against the CPU oracle, through the C ABI.

Bar: permutation, mask, statistics, compressed values and metadata bit-exact; products within a
normwise relative error per output row of 2e-3 (fp16) / 1e-2 (bf16).
"""
import hashlib
import json
import math
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import esparse_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {torch.float16: 2e-3, torch.bfloat16: 1e-2}


@pytest.fixture(scope="module")
def esp():
    import paper_2310_15929_amd as esp
    esp.load_library()
    return esp


@pytest.fixture(scope="module")
def ctx(esp):
    assert torch.cuda.is_available()
    return esp.Context(0)


def _np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.float().numpy()
    return t.numpy()


def _bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _rand(shape, dtype, seed, scale=1.0, col_scale=None):
    return wl.normal_matrix(shape[0], shape[1], wl.stream_id("test", seed), scale=scale, col_scale=col_scale,
                            dtype=dtype)


def _sha(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


# ---------------------------------------------------------------- channel statistics
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("T,K", [(256, 512), (1000, 70), (37, 2)])
def test_channel_stats_bit_exact(ctx, dtype, T, K):
    scales = np.exp(np.random.default_rng(T + K).standard_normal(K) * 2.0)
    Xc = _rand((T, K), dtype, 11, col_scale=scales)
    if K >= 4:
        Xc[:, 1] = 0.75          # constant channel
        Xc[:, 3] = 0.0           # all-zero channel
    print(f"stats T={T} K={K} {dtype}", flush=True)
    ir, am = ctx.channel_stats(Xc.cuda(), 100)
    x = _np(Xc)
    assert (ir == orc.channel_entropy(x, 100)).all()
    assert (am == orc.channel_amplitude(x)).all()


def test_channel_stats_other_bin_counts(ctx):
    Xc = _rand((512, 16), torch.float16, 12)
    for bins in (1, 7, 256):
        ir, _ = ctx.channel_stats(Xc.cuda(), bins)
        assert (ir == orc.channel_entropy(_np(Xc), bins)).all()


# ---------------------------------------------------------------- prune
def _prune_case(esp, ctx, N, K, T, B, n, m, dtype, flags, seed, max_swaps=0):
    scales = wl.channel_scales("lognormal", K, wl.stream_id("ps", seed))
    W = _rand((N, K), dtype, seed, scale=K ** -0.5)
    Xc = _rand((T, K), dtype, seed + 1, col_scale=scales)
    alpha = wl.default_alpha(T)
    opts = esp.PruneOpts(n_keep=n, m_group=m, block=B, bins=100, alpha=alpha, flags=flags, max_swaps=max_swaps)
    print(f"prune N={N} K={K} T={T} B={B} {n}:{m} {dtype} flags={flags} max_swaps={max_swaps}", flush=True)
    res = ctx.prune(Xc.cuda(), W.cuda(), opts, want_retained=True)
    torch.cuda.synchronize()
    theta, mask, s, swaps = orc.prune(_np(Xc), _np(W), n, m, B, alpha, 100,
                                      use_entropy=bool(flags & esp.USE_ENTROPY), use_norm=bool(flags & esp.USE_NORM),
                                      use_gns=bool(flags & esp.USE_GNS), use_lbs=bool(flags & esp.USE_LBS),
                                      max_swaps=max_swaps)
    assert (res.score == s).all(), "scores differ"
    assert (res.perm.cpu().numpy() == theta).all(), "theta differs"
    if flags & esp.USE_LBS:
        assert (res.swaps == swaps).all(), "swap counts differ"
    assert (res.mask.cpu().numpy() == mask).all(), "mask differs"
    # a float64 sum of N * K / m terms: the device adds them in its own order (eq. 5 fixes none)
    assert res.retained == pytest.approx(orc.retained_metric(_np(W), s, theta, n, m), rel=1e-12)
    return res, W, Xc, theta, mask, s


@pytest.mark.parametrize("n,m,B", [(2, 4, 32), (2, 4, 64), (4, 8, 32)])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_prune_bit_exact(esp, ctx, n, m, B, dtype):
    _prune_case(esp, ctx, 96, 128, 200, B, n, m, dtype, esp.USE_ALL, 21)


def test_prune_ablation_switches(esp, ctx):
    for flags in (esp.USE_NORM, esp.USE_NORM | esp.USE_ENTROPY, esp.USE_NORM | esp.USE_ENTROPY | esp.USE_GNS,
                  esp.USE_ENTROPY | esp.USE_LBS):
        _prune_case(esp, ctx, 64, 64, 128, 32, 2, 4, torch.float16, flags, 22)


def test_prune_max_swaps_and_ties(esp, ctx):
    _prune_case(esp, ctx, 48, 64, 64, 32, 2, 4, torch.float16, esp.USE_ALL, 23, max_swaps=3)
    # heavy ties: weights on a coarse grid, scores given
    N, K, B = 40, 64, 32
    rng = np.random.default_rng(5)
    W = torch.tensor(rng.integers(-3, 4, size=(N, K)) * 0.25, dtype=torch.float16)
    s = rng.integers(1, 4, size=K).astype(np.float64)
    opts = esp.PruneOpts(block=B, alpha=1.0)
    res = ctx.prune(None, W.cuda(), opts, score=s)
    theta0 = orc.global_naive_shuffle(W.numpy(), s, 4)
    theta, swaps = orc.local_block_shuffle_vectorised(W.numpy(), s, theta0, 2, 4, B)
    assert (res.perm.cpu().numpy() == theta).all() and (res.swaps == swaps).all()
    assert (res.mask.cpu().numpy() == orc.nm_mask(W.numpy(), s, theta, 2, 4)).all()


def test_config1_against_stored_oracle_results(esp, ctx):
    """Workload configuration 1, complete, against results the oracle wrote to tests/golden."""
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "cfg1_oracle.json")))
    W = wl.weights(1, "linear")
    Xc = wl.calibration(1, "linear")
    X = wl.activations(1, "linear", 16)
    assert _sha(W.numpy()) == gold["inputs_sha256"]["W"] and _sha(Xc.numpy()) == gold["inputs_sha256"]["Xc"]
    opts = esp.PruneOpts(block=64, alpha=gold["alpha"])
    print("config 1 prune", flush=True)
    res = ctx.prune(Xc.cuda(), W.cuda(), opts, want_retained=True)
    assert res.perm.cpu().tolist() == gold["theta"]
    assert res.swaps.tolist() == gold["swaps"]
    assert _sha(res.score) == gold["score_sha256"]
    assert _sha(res.mask.cpu().numpy()) == gold["mask_sha256"]
    assert res.retained == pytest.approx(gold["retained"], rel=1e-12)
    comp = ctx.compress(W.cuda(), res.mask, res.perm)
    assert _sha(_bits(comp.values)) == gold["values_sha256"]
    assert _sha(comp.meta.cpu().numpy()) == gold["meta_sha256"]
    Np_Kp = 512 * 512
    nat = comp.native.cpu().numpy()
    assert _sha(nat[:Np_Kp]) == gold["native_values_sha256"] and _sha(nat[Np_Kp:]) == gold["native_meta_sha256"]
    theta = np.array(gold["theta"])
    mask = res.mask.cpu().numpy()
    Yref = orc.spmm_ref(X.numpy(), W.numpy(), theta, mask)
    for v in range(esp.num_variants()):
        try:
            Y = ctx.spmm(X.cuda(), comp, res.perm, variant=v)
        except esp.EsparseError as e:
            assert e.code == -2                      # variant not applicable to this M
            continue
        err = orc.rowwise_rel_error(_np(Y), Yref)
        assert err.max() <= 2e-3, (esp.variant_name(v), err.max())


# ---------------------------------------------------------------- compression
@pytest.mark.parametrize("N,K", [(24, 320), (16, 256), (5, 36), (130, 1040), (33, 36864), (3, 81920)])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_compress_2_4_bit_exact(esp, ctx, N, K, dtype):
    W = _rand((N, K), dtype, 31)
    rng = np.random.default_rng(N * K)
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), s, theta, 2, 4)
    print(f"compress N={N} K={K} {dtype}", flush=True)
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), torch.tensor(theta, dtype=torch.int32).cuda())
    Wb = _bits(W).reshape(N, K)
    values, meta = orc.compress_vectorised(Wb, theta, mask, 2, 4)        # on raw 16-bit patterns
    assert (_bits(comp.values).reshape(values.shape) == values).all()
    assert (comp.meta.cpu().numpy().view(np.uint32).reshape(meta.shape) == meta).all()
    nv, nm = orc.native_tiling(values, meta, N, K)
    nat = comp.native.cpu().numpy()
    assert nat.size == esp.compressed_size(N, K, 2, 4)[2]
    assert (nat[:nv.nbytes].view(np.uint16) == nv).all()
    assert (nat[nv.nbytes:].view(np.uint16) == nm).all()


def test_compress_4_8_and_derived_mask_and_errors(esp, ctx):
    N, K = 20, 64
    W = _rand((N, K), torch.float16, 32)
    rng = np.random.default_rng(9)
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), s, theta, 4, 8)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, 4, 8)
    values, meta = orc.compress_vectorised(_bits(W).reshape(N, K), theta, mask, 4, 8)
    assert (_bits(comp.values).reshape(values.shape) == values).all()
    assert (comp.meta.cpu().numpy().reshape(meta.shape) == meta).all()
    nv, nm = orc.native_tiling_4_8(values, meta, N, K)
    nat = comp.native.cpu().numpy()
    assert nat.size == esp.compressed_size(N, K, 4, 8)[2] == nv.nbytes + nm.nbytes
    assert (nat[:nv.nbytes].view(np.uint16) == nv).all() and (nat[nv.nbytes:] == nm).all()
    # mask = NULL: the mask is read off the zeros of an already pruned weight
    for n, m in ((2, 4), (4, 8)):
        mk = orc.nm_mask_vectorised(_np(W), s, theta, n, m)
        Wz = torch.tensor(_np(W) * orc.mask_to_original_order(mk, theta), dtype=torch.float16)
        comp = ctx.compress(Wz.cuda(), None, th, n, m)
        values, meta = orc.compress_vectorised(_bits(Wz).reshape(N, K), theta, mk, n, m)
        assert (_bits(comp.values).reshape(values.shape) == values).all()
        assert (comp.meta.cpu().numpy().view(meta.dtype).reshape(meta.shape) == meta).all()
    # a dense weight has more than n non-zeros per group
    with pytest.raises(esp.EsparseError) as e:
        ctx.compress(W.cuda(), None, th, 2, 4)
    assert e.value.code == -5
    bad = mask.copy()
    bad[3, 8:16] = 1
    with pytest.raises(esp.EsparseError) as e:
        ctx.compress(W.cuda(), torch.tensor(bad).cuda(), th, 4, 8)
    assert e.value.code == -5
    th_bad = th.clone()
    th_bad[5] = th_bad[6]
    with pytest.raises(esp.EsparseError) as e:
        ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th_bad, 4, 8)
    assert e.value.code == -6


# ---------------------------------------------------------------- products
def _spmm_case(esp, ctx, M, N, K, dtype, seed, use_perm=True):
    rng = np.random.default_rng(seed)
    scales = wl.channel_scales("lognormal", K, wl.stream_id("xs", seed))
    W = _rand((N, K), dtype, seed, scale=K ** -0.5)
    X = _rand((M, K), dtype, seed + 7, col_scale=scales)
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K) if use_perm else np.arange(K)
    mask = orc.nm_mask_vectorised(_np(W), s, theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda() if use_perm else None
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, canonical=False)
    Yref = orc.spmm_ref(_np(X), _np(W), theta, mask)
    Ydref = orc.dense_ref(_np(X), _np(W))
    packed = ctx.dense_pack(W.cuda())
    Xd = X.cuda()
    for v in range(esp.num_variants()):
        print(f"spmm M={M} N={N} K={K} {dtype} perm={use_perm} variant={esp.variant_name(v)}", flush=True)
        try:
            Y = ctx.spmm(Xd, comp, th, variant=v)
            torch.cuda.synchronize()
            err = orc.rowwise_rel_error(_np(Y), Yref)
            assert err.max() <= TOL[dtype], ("sparse", esp.variant_name(v), err.max())
        except esp.EsparseError as e:
            assert e.code == -2                      # not for this shape, or a variant of the dense product only
        try:
            Yd = ctx.dense_gemm(Xd, packed, N, variant=v)
            torch.cuda.synchronize()
            err = orc.rowwise_rel_error(_np(Yd), Ydref)
            assert err.max() <= TOL[dtype], ("dense", esp.variant_name(v), err.max())
        except esp.EsparseError as e:
            assert e.code == -2                      # not for this shape, or a variant of the 2:4 product only
    # default variant
    Y = ctx.spmm(Xd, comp, th)
    assert orc.rowwise_rel_error(_np(Y), Yref).max() <= TOL[dtype]


@pytest.mark.parametrize("M", [1, 8, 16, 33, 130])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_spmm_small_ragged(esp, ctx, M, dtype):
    _spmm_case(esp, ctx, M, 72, 576, dtype, 41)


@pytest.mark.parametrize("M", [2, 3, 5, 9, 15, 17])
def test_spmm_few_tokens_compact_staging(esp, ctx, M):
    """Up to 16 tokens the decode kernels read the compact copy of the staged activations (token count rounded up
    to a power of two, the padding tokens zero); 17 is the first size that does not."""
    _spmm_case(esp, ctx, M, 88, 832, torch.float16, 46 + M)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_spmm_decode_step_pairs(esp, ctx, dtype):
    """K = 2048: 16 step pairs divide among 8 and 16 waves, so the decode kernels with two or four token tiles take
    the steps pairwise and read one index word per pair."""
    _spmm_case(esp, ctx, 33, 80, 2048, dtype, 52)
    _spmm_case(esp, ctx, 20, 48, 2048, dtype, 53)


def test_spmm_stream_spans(esp, ctx):
    """Stream kernels cut the steps of all row blocks into equal spans: a span inside one row block (partial
    pieces), a span across a row block boundary, and spans holding several whole row blocks (stored directly)."""
    _spmm_case(esp, ctx, 70, 400, 768, torch.float16, 44)        # 12 steps per row block, spans of 8
    _spmm_case(esp, ctx, 40, 65536 + 48, 256, torch.bfloat16, 45)  # 4 steps per row block, spans of 8 or more


def test_spmm_identity_perm_and_multi_tile(esp, ctx):
    _spmm_case(esp, ctx, 16, 512, 2048, torch.float16, 42, use_perm=False)
    _spmm_case(esp, ctx, 200, 272, 1280, torch.float16, 43)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_spmm_k_split_over_workgroups(esp, ctx, dtype):
    # K long enough (64 stages of 64 channels) for the split-K variants to really split; ragged M and N
    _spmm_case(esp, ctx, 100, 300, 4096, dtype, 49)
    _spmm_case(esp, ctx, 64, 144, 2304, dtype, 50)
    _spmm_case(esp, ctx, 300, 272, 4096, dtype, 51)   # 128 < M <= 512: up to four splits


def test_spmm_many_tokens_row_staging(esp, ctx):
    """Long inputs are staged by workgroups that hold 2 to 16 whole rows of X; the workgroups of one token tile are
    numbered 8 apart.  8 and 16 rows per workgroup need thousands of tokens; the tile counts (257, 513) are not
    multiples of 8 and the last tile is ragged."""
    _spmm_case(esp, ctx, 4100, 32, 512, torch.float16, 54)
    _spmm_case(esp, ctx, 8200, 32, 320, torch.bfloat16, 55)


def test_spmm_banded_tile_order(esp, ctx):
    """More than 8 token blocks per row block: the tile kernels number their macro tiles in bands of 8 row blocks
    (token blocks outermost within a band).  11 row blocks of 256 (22 of 128) leave a ragged last band; 2400 tokens are
    10 blocks of 256 (19 of 128), the last one ragged."""
    _spmm_case(esp, ctx, 2400, 2816, 256, torch.float16, 56)


def test_stacked_matrices_share_one_theta(esp, ctx):
    """Matrices that read the same input (q/k/v, gate/up) pruned as one stacked matrix: one theta, one mask;
    the product of the stack is the concatenation of the products of its slices (bitwise: rows are independent)
    and matches the oracle on the stack."""
    K, T, M = 256, 128, 20
    Ws = [_rand((n, K), torch.float16, 60 + i, scale=K ** -0.5) for i, n in enumerate((48, 32, 80))]
    Wcat = torch.cat(Ws, dim=0)
    Xc = _rand((T, K), torch.float16, 63, col_scale=wl.channel_scales("lognormal", K, wl.stream_id("st", 1)))
    X = _rand((M, K), torch.float16, 64)
    alpha = wl.default_alpha(T)
    res = ctx.prune(Xc.cuda(), Wcat.cuda(), esp.PruneOpts(block=64, alpha=alpha))
    theta, mask, s, _ = orc.prune(_np(Xc), _np(Wcat), 2, 4, 64, alpha, 100)
    assert (res.perm.cpu().numpy() == theta).all() and (res.mask.cpu().numpy() == mask).all()
    comp = ctx.compress(Wcat.cuda(), res.mask, res.perm, canonical=False)
    Y = ctx.spmm(X.cuda(), comp, res.perm)
    assert orc.rowwise_rel_error(_np(Y), orc.spmm_ref(_np(X), _np(Wcat), theta, mask)).max() <= 2e-3
    lo = 0
    for W in Ws:
        n = W.shape[0]
        part = ctx.compress(W.cuda(), res.mask[lo:lo + n].contiguous(), res.perm, canonical=False)
        Yp = ctx.spmm(X.cuda(), part, res.perm)
        assert (_bits(Yp) == _bits(Y[:, lo:lo + n])).all()
        lo += n


def test_spmm_one_hot_reads_back_weights_through_theta(esp, ctx):
    N, K = 48, 256
    rng = np.random.default_rng(3)
    W = _rand((N, K), torch.float16, 44)
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), s, theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th)
    X = torch.eye(K, dtype=torch.float16)
    Y = ctx.spmm(X.cuda(), comp, th)                      # [K, N]: row c = masked W[:, c]
    ref = (_np(W) * orc.mask_to_original_order(mask, theta)).T
    assert (_np(Y) == ref).all()
    ones = torch.ones((1, K), dtype=torch.float16)
    Y1 = ctx.spmm(ones.cuda(), comp, th)
    assert np.allclose(_np(Y1)[0], ref.sum(axis=0), rtol=2e-3, atol=1e-3)


def test_spmm_repeat_is_bitwise_identical_and_m0(esp, ctx):
    N, K, M = 64, 1024, 24
    W = _rand((N, K), torch.float16, 45, scale=K ** -0.5)
    X = _rand((M, K), torch.float16, 46)
    theta = np.random.default_rng(1).permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), np.ones(K), theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, canonical=False)
    for v in range(esp.num_variants()):
        try:
            a = _bits(ctx.spmm(X.cuda(), comp, th, variant=v))
        except esp.EsparseError as e:
            assert e.code == -2                      # variant not applicable to this M
            continue
        b = _bits(ctx.spmm(X.cuda(), comp, th, variant=v))
        assert (a == b).all()
    Y0 = ctx.spmm(X[:0].cuda(), comp, th)
    assert Y0.shape == (0, N)


@pytest.mark.parametrize("M,K", [(1, 832), (2, 832), (1, 11008), (2, 4096), (1, 36864), (3, 832)])
def test_spmm_theta_gathered_in_the_kernel_equals_staged(esp, ctx, M, K):
    """With one or two tokens the decode kernels apply the channel re-ordering themselves (no staged copy, no staging
    launch) where the gathered row fits the LDS; the result is bitwise the one of the two-step path (activations staged
    through theta by a launch of their own, then multiplied) and within tolerance of the oracle.  K = 36864 at one token
     (and 11008) and three tokens are beyond what is gathered in the kernel (both calls then take the staged path)."""
    N = 80
    rng = np.random.default_rng(M * 7 + K)
    W = _rand((N, K), torch.float16, 61, scale=K ** -0.5)
    X = _rand((M, K), torch.float16, 62, col_scale=wl.channel_scales("lognormal", K, wl.stream_id("xs", 62)))
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), np.abs(rng.standard_normal(K)) + 0.1, theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, canonical=False)
    Yref = orc.spmm_ref(_np(X), _np(W), theta, mask)
    Xd = X.cuda()
    ran = 0
    for perm in (th, None):
        ref = Yref if perm is not None else orc.spmm_ref(_np(X), _np(W[:, theta]), np.arange(K), mask)
        comp_p = comp if perm is not None else ctx.compress(W[:, theta].contiguous().cuda(), torch.tensor(mask).cuda(), None, canonical=False)
        for v in range(esp.num_variants()):
            print(f"fold M={M} K={K} perm={'theta' if perm is not None else 'identity'} variant={esp.variant_name(v)}", flush=True)
            try:
                Y = ctx.spmm(Xd, comp_p, perm, variant=v)
            except esp.EsparseError as e:
                assert e.code == -2
                continue
            ws = ctx.stage_activations(Xd, perm, N)
            Y2 = torch.empty_like(Y)
            ctx.spmm_staged(M, comp_p, ws, Y2, variant=v)
            torch.cuda.synchronize()
            assert (_bits(Y) == _bits(Y2)).all(), esp.variant_name(v)
            assert orc.rowwise_rel_error(_np(Y), ref).max() <= 2e-3
            ran += 1
    assert ran > 4


@pytest.mark.parametrize("M", [8, 100, 300])
def test_spmm_replayed_from_a_hip_graph(esp, ctx, M):
    """The calls enqueue kernels only (no allocation, no memset, no synchronisation), so a caller may capture them
    into a HIP graph: every variant, staging included, captured once on a side stream and replayed three times with
    new activations and eager work of the same context between the replays, must reproduce the eager result bit
    for bit (decode, K-split, stream and tile kernels with their reduction launches)."""
    N, K = 272, 2048
    W = _rand((N, K), torch.float16, 61, scale=K ** -0.5)
    theta = np.random.default_rng(2).permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), np.ones(K), theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, canonical=False)
    Xs = [_rand((M, K), torch.float16, 62 + i).cuda() for i in range(3)]
    other = _rand((M + 5, K), torch.float16, 70).cuda()
    side = torch.cuda.Stream()
    for v in range(esp.num_variants()):
        try:
            eager = [_bits(ctx.spmm(x, comp, th, variant=v)) for x in Xs]
        except esp.EsparseError as e:
            assert e.code == -2
            continue
        print(f"graph replay M={M} variant={esp.variant_name(v)}", flush=True)
        xin = Xs[0].clone()
        yout = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        ws = torch.empty(esp.spmm_workspace(M, N, K) + 256, dtype=torch.uint8, device="cuda")
        ws = ws[(-ws.data_ptr()) % 256:]
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            ctx.stage_activations(xin, th, N, ws)
            ctx.spmm_staged(M, comp, ws, yout, variant=v)       # warm-up on the side stream
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=side):
                ctx.stage_activations(xin, th, N, ws)
                ctx.spmm_staged(M, comp, ws, yout, variant=v)
        torch.cuda.synchronize()
        for i in (1, 2, 0):
            xin.copy_(Xs[i])
            yout.zero_()
            ctx.spmm(other, comp, th, variant=v)                # eager work between the replays (own workspace)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert (_bits(yout) == eager[i]).all(), (esp.variant_name(v), i)
        del g


def test_workspace_too_small_and_bad_variant(esp, ctx):
    import ctypes as C
    N, K, M = 32, 256, 4
    W = _rand((N, K), torch.float16, 47)
    comp = ctx.compress(torch.tensor(_np(W) * np.tile([1, 1, 0, 0], (N, K // 4)), dtype=torch.float16).cuda(), None, None)
    X = _rand((M, K), torch.float16, 48).cuda()
    Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    ws = ctx.workspace(1024)
    lib = esp.load_library()
    rc = lib.esparse_spmm(ctx._h, X.data_ptr(), M, comp.native.data_ptr(), None, N, K, 0, 2, 4, Y.data_ptr(),
                          ws.data_ptr(), 1024, -1)
    assert rc == -7
    with pytest.raises(esp.EsparseError) as e:
        ctx.spmm(X, comp, None, variant=999)
    assert e.value.code == -1


@pytest.mark.parametrize("M,N,K", [(33, 80, 2048), (130, 272, 1024), (600, 528, 768)])
def test_named_variant_stays_inside_the_workspace_size_reported_for_it(esp, ctx, M, N, K):
    # esparse_spmm_workspace(M, N, K, variant): a call naming that variant accepts exactly that many bytes, touches
    # nothing behind them (a guard pattern follows the workspace) and gives the product of the full-size workspace
    W = _rand((N, K), torch.float16, 81)
    comp = ctx.compress(torch.tensor(_np(W) * np.tile([1, 0, 1, 0], (N, K // 4)), dtype=torch.float16).cuda(), None, None)
    X = _rand((M, K), torch.float16, 82).cuda()
    th = torch.tensor(np.random.default_rng(83).permutation(K), dtype=torch.int32).cuda()
    lib = esp.load_library()
    guard = 1 << 20
    for v in range(esp.num_variants()):
        try:
            ref = _bits(ctx.spmm(X, comp, th, variant=v))
        except esp.EsparseError as e:
            assert e.code == -2
            continue
        need = esp.spmm_workspace(M, N, K, v)
        assert need <= esp.spmm_workspace(M, N, K)
        buf = torch.full((need + guard + 256,), 0xA5, dtype=torch.uint8, device="cuda")
        off = (-buf.data_ptr()) % 256
        Y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        print(f"workspace of variant {esp.variant_name(v)}: {need} bytes", flush=True)
        rc = lib.esparse_spmm(ctx._h, X.data_ptr(), M, comp.native.data_ptr(), th.data_ptr(), N, K, 0, 2, 4, Y.data_ptr(),
                              buf.data_ptr() + off, need, v)
        assert rc == 0, (esp.variant_name(v), lib.esparse_last_error(ctx._h).decode())
        torch.cuda.synchronize()
        assert (_bits(Y) == ref).all(), esp.variant_name(v)
        assert bool((buf[off + need:] == 0xA5).all()), esp.variant_name(v)
        rc = lib.esparse_spmm(ctx._h, X.data_ptr(), M, comp.native.data_ptr(), th.data_ptr(), N, K, 0, 2, 4, Y.data_ptr(),
                              buf.data_ptr() + off, need - 256, v)
        assert rc == -7


def test_matrix_rate_is_plausible(esp, ctx):
    # register-resident operands: below the published peaks (5.0 PFLOP/s effective for 2:4, 2.5 dense; 3 % for the
    # clock's tolerance), well above what any product kernel reaches, zeros not slower than random data, and the 2:4
    # instruction about twice the dense one
    sr = ctx.matrix_rate(True, esp.F16, True)
    sz = ctx.matrix_rate(True, esp.F16, False)
    dr = ctx.matrix_rate(False, esp.F16, True)
    br = ctx.matrix_rate(True, esp.BF16, True)
    m1 = ctx.matrix_rate(True, esp.F16, True, mix=1)
    m2 = ctx.matrix_rate(True, esp.F16, True, mix=2)
    print(f"matrix rate TFLOP/s: 2:4 fp16 random {sr:.0f}, zeros {sz:.0f}, bf16 random {br:.0f}, dense fp16 random {dr:.0f}; "
          f"with a stage's LDS reads {m1:.0f}, and its DMA, wait and barrier {m2:.0f}", flush=True)
    assert 1500 < sr <= 5150 and 1500 < br <= 5150 and sr * 0.95 <= sz <= 5150
    assert 750 < dr <= 2575 and 1.6 < sr / dr < 2.4
    assert 1000 < m2 <= m1 * 1.05 and m1 <= sr * 1.05


def test_read_rate_is_plausible(esp, ctx):
    # cold plain reads: below the published 8 TB/s, rising with the bytes per launch (launch, ramp-up and drain are fixed)
    small, mid, big = ctx.read_rate(16 << 20), ctx.read_rate(100 << 20), ctx.read_rate(1 << 30)
    print(f"plain read GB/s: 16 MiB {small:.0f}, 100 MiB {mid:.0f}, 1 GiB {big:.0f}", flush=True)
    assert 1000 < small < mid < big * 1.05 and big < 8000


def test_tune_picks_a_variant_and_persists(esp, ctx, tmp_path):
    best, ms = ctx.tune(16, 512, 1024, esp.F16, sparse=True)
    assert 0 <= best < esp.num_variants() and ms > 0
    p = str(tmp_path / "tuned.txt")
    ctx.tune_save(p)
    c2 = esp.Context(0)
    c2.tune_load(p)
    assert esp.variant_name(best) in open(p).read()
    # a choice for launches of three products of the shape is kept beside the single one and survives the file
    bg, msg = ctx.tune_group(3, 16, 512, 1024, esp.F16, sparse=True)
    assert 0 <= bg < esp.num_variants() and msg > 0
    ctx.tune_save(p)
    lines = [l.split() for l in open(p).read().splitlines() if not l.startswith("#")]
    assert ["1", "0", "16", "512", "1024", esp.variant_name(best)] in lines
    assert ["1", "0", "16", "512", "1024", esp.variant_name(bg), "3"] in lines
    c3 = esp.Context(0)
    c3.tune_load(p)
    q = str(tmp_path / "again.txt")
    c3.tune_save(q)
    assert sorted(open(q).read().splitlines()) == sorted(open(p).read().splitlines())


# ---------------------------------------------------------------- eq. 4 report
def test_output_error_report_for_the_ablation_settings(esp, ctx):
    """Relative output error of eq. (4) on held-out activations for the four settings of the paper's ablation
    (norm; + entropy; + global shuffle; + local block shuffle), device against oracle."""
    N, K, T, M = 96, 128, 200, 64
    scales = wl.channel_scales("lognormal", K, wl.stream_id("oe", 1))
    W = _rand((N, K), torch.float16, 70, scale=K ** -0.5)
    Xc = _rand((T, K), torch.float16, 71, col_scale=scales)
    X = _rand((M, K), torch.float16, 72, col_scale=scales)
    alpha = wl.default_alpha(T)
    packed = ctx.dense_pack(W.cuda())
    Yd = ctx.dense_gemm(X.cuda(), packed, N)
    for flags in (esp.USE_NORM, esp.USE_NORM | esp.USE_ENTROPY, esp.USE_NORM | esp.USE_ENTROPY | esp.USE_GNS, esp.USE_ALL):
        res = ctx.prune(Xc.cuda(), W.cuda(), esp.PruneOpts(block=32, alpha=alpha, flags=flags))
        comp = ctx.compress(W.cuda(), res.mask, res.perm, canonical=False)
        Ys = ctx.spmm(X.cuda(), comp, res.perm)
        num, den = ctx.output_error(Yd, Ys)
        # the entry point itself, against float64 numpy on the same two outputs
        a, b = _np(Yd).astype(np.float64), _np(Ys).astype(np.float64)
        assert abs(num - ((a - b) ** 2).sum()) <= 1e-12 * num and abs(den - (a ** 2).sum()) <= 1e-12 * den
        # the report, against the oracle's eq. (4) on exact products (the device outputs are rounded to 16 bits)
        theta, mask, _, _ = orc.prune(_np(Xc), _np(W), 2, 4, 32, alpha, 100, use_entropy=bool(flags & esp.USE_ENTROPY),
                                      use_norm=True, use_gns=bool(flags & esp.USE_GNS), use_lbs=bool(flags & esp.USE_LBS))
        ref = orc.output_error(_np(X), _np(W), theta, mask)
        assert abs(num / den - ref) <= 1e-2 * ref, (flags, num / den, ref)
    n0, d0 = ctx.output_error(Yd[:0], Yd[:0])
    assert (n0, d0) == (0.0, 0.0)


# ---------------------------------------------------------------- 4:8 product (bitmaps expanded in registers)
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("M,N,K", [(1, 72, 576), (8, 40, 256), (33, 72, 576), (40, 72, 1024), (64, 144, 2304), (150, 48, 512),
                                   (300, 520, 768), (200, 100, 264)])
def test_spmm_4_8(esp, ctx, M, N, K, dtype):
    rng = np.random.default_rng(M * N + K)
    scales = wl.channel_scales("lognormal", K, wl.stream_id("x48", M))
    W = _rand((N, K), dtype, 80, scale=K ** -0.5)
    X = _rand((M, K), dtype, 81, col_scale=scales)
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), s, theta, 4, 8)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, 4, 8)
    values, meta = orc.compress_vectorised(_bits(W).reshape(N, K), theta, mask, 4, 8)
    nv, nm = orc.native_tiling_4_8(values, meta, N, K)
    nat = comp.native.cpu().numpy()
    assert (nat[:nv.nbytes].view(np.uint16) == nv).all() and (nat[nv.nbytes:] == nm).all()
    Yref = orc.spmm_ref(_np(X), _np(W), theta, mask)
    ran = 0
    for v in [-1] + list(range(esp.num_variants())):
        print(f"4:8 spmm M={M} N={N} K={K} {dtype} variant={v}", flush=True)
        try:
            Y = ctx.spmm(X.cuda(), comp, th, variant=v)
        except esp.EsparseError as e:
            assert e.code == -2 and v >= 0          # not a decode, four-slot stream or 4:8 tile kernel, or not for this M
            continue
        torch.cuda.synchronize()
        err = orc.rowwise_rel_error(_np(Y), Yref)
        assert err.max() <= TOL[dtype], (v, err.max())
        ran += 1
    assert ran >= 3


def test_products_on_seeded_random_shapes(esp, ctx):
    """Shapes drawn from a seeded generator (ragged tails in every dimension, token counts on both sides of every
    kernel family's boundary), both weight formats and the dense product, each through the kernel the library
    chooses by itself, against the oracle."""
    rng = np.random.default_rng(20231015)
    boundaries = [1, 2, 3, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 300]
    for case in range(18):
        M = int(boundaries[case])
        N = int(rng.integers(1, 700))
        K = int(rng.integers(1, 200)) * 8
        dtype = torch.float16 if case % 3 else torch.bfloat16
        W = _rand((N, K), dtype, 300 + case, scale=K ** -0.5)
        X = _rand((M, K), dtype, 400 + case, col_scale=wl.channel_scales("lognormal", K, wl.stream_id("rs", case)))
        s = np.abs(rng.standard_normal(K)) + 0.1
        theta = rng.permutation(K)
        th = torch.tensor(theta, dtype=torch.int32).cuda()
        print(f"random shape {case}: M={M} N={N} K={K} {dtype}", flush=True)
        for n, m in ((2, 4), (4, 8)):
            mask = orc.nm_mask_vectorised(_np(W), s, theta, n, m)
            comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, n, m, canonical=False)
            Y = ctx.spmm(X.cuda(), comp, th)
            torch.cuda.synchronize()
            err = orc.rowwise_rel_error(_np(Y), orc.spmm_ref(_np(X), _np(W), theta, mask))
            assert err.max() <= TOL[dtype], (case, n, m, err.max())
        Yd = ctx.dense_gemm(X.cuda(), ctx.dense_pack(W.cuda()), N)
        torch.cuda.synchronize()
        assert orc.rowwise_rel_error(_np(Yd), orc.dense_ref(_np(X), _np(W))).max() <= TOL[dtype], case


def test_spmm_4_8_one_hot_reads_back_weights(esp, ctx):
    N, K = 32, 256
    rng = np.random.default_rng(48)
    W = _rand((N, K), torch.float16, 82)
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(_np(W), s, theta, 4, 8)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, 4, 8, canonical=False)
    Y = ctx.spmm(torch.eye(K, dtype=torch.float16).cuda(), comp, th)         # [K, N]: row c = masked W[:, c]
    assert (_np(Y) == (_np(W) * orc.mask_to_original_order(mask, theta)).T).all()


# ---------------------------------------------------------------- several products of one shape in one call
@pytest.mark.parametrize("n,m", [(2, 4), (4, 8)])
@pytest.mark.parametrize("M", [1, 20, 64, 100])
def test_spmm_group_equals_single_products(esp, ctx, M, n, m):
    N, K = 80, 512
    rng = np.random.default_rng(M + n)
    X = _rand((M, K), torch.float16, 90).cuda()
    X2 = _rand((M, K), torch.float16, 91).cuda()
    comps, perms, refs = [], [], []
    for i in range(3):
        W = _rand((N, K), torch.float16, 92 + i, scale=K ** -0.5)
        s = np.abs(rng.standard_normal(K)) + 0.1
        theta = rng.permutation(K)
        mask = orc.nm_mask_vectorised(_np(W), s, theta, n, m)
        th = torch.tensor(theta, dtype=torch.int32).cuda()
        comps.append(ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, n, m, canonical=False))
        perms.append(th)
        refs.append(orc.spmm_ref(_np(X2 if i == 2 else X), _np(W), theta, mask))
    Xs = [X, X, X2]                                   # two members share their input, like q/k/v
    print(f"group M={M} {n}:{m}", flush=True)
    Ys = ctx.spmm_group(Xs, comps, perms)
    torch.cuda.synchronize()
    for i in range(3):
        assert orc.rowwise_rel_error(_np(Ys[i]), refs[i]).max() <= 2e-3
        single = ctx.spmm(Xs[i], comps[i], perms[i])
        assert (_bits(single) == _bits(Ys[i])).all()
    if n == 2:
        Ws = [_rand((N, K), torch.float16, 92 + i, scale=K ** -0.5).cuda() for i in range(3)]
        packed = [ctx.dense_pack(W) for W in Ws]
        Yd = ctx.dense_gemm_group(Xs, packed, N)
        for i in range(3):
            assert (_bits(Yd[i]) == _bits(ctx.dense_gemm(Xs[i], packed[i], N))).all()
            assert orc.rowwise_rel_error(_np(Yd[i]), orc.dense_ref(_np(Xs[i]), _np(Ws[i]))).max() <= 2e-3
    if M <= 32:
        # the two halves as separate calls (they exist where a decode kernel is the default: M <= 32)
        ws = ctx.workspace(4 * esp.spmm_workspace(M, N, K))
        ctx.stage_activations_group(Xs, perms, comps[0], ws)
        outs = [torch.empty_like(y) for y in Ys]
        ctx.spmm_group_staged(M, comps, ws, outs)
        for i in range(3):
            assert (_bits(outs[i]) == _bits(Ys[i])).all()
    # identity permutation for all members, one member only
    Y1 = ctx.spmm_group([X], comps[:1], None)
    assert (_bits(Y1[0]) == _bits(ctx.spmm(X, comps[0], None))).all()
