"""esparse_spmm_static (the entry point that allocates nothing: its scratch is a fixed array in the library's
device image) against esparse_spmm, through the C ABI: two calls in a row, the second with a smaller input, so
that the second runs on whatever the first left in the array.  Bar: bitwise equal outputs (same kernels, same
variant), and the product within the tolerance of the oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import esparse_oracle as orc

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _case(esp, ctx, M, N, K, seed, variant=-1):
    rng = np.random.default_rng(seed)
    W = wl.normal_matrix(N, K, wl.stream_id("na-w", seed), scale=K ** -0.5)
    X = wl.normal_matrix(M, K, wl.stream_id("na-x", seed), col_scale=wl.channel_scales("lognormal", K, wl.stream_id("na-s", seed)))
    s = np.abs(rng.standard_normal(K)) + 0.1
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(W.numpy(), s, theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, canonical=False)
    Yref = orc.spmm_ref(X.numpy(), W.numpy(), theta, mask)
    return X.cuda(), comp, th, Yref


def test_static_scratch_product_equals_workspace_product(capfd):
    import paper_2310_15929_amd as esp
    lib = esp.load_library()
    ctx = esp.Context(0)
    # first a large input (prefill kernel, 300 tokens), then smaller ones (stream kernel with partial tiles; decode
    # kernel with the compact staging of a few tokens), all through the same static array
    for M, N, K, seed in [(300, 528, 2304, 1), (70, 400, 768, 2), (5, 88, 832, 3), (1, 88, 832, 4)]:
        X, comp, th, Yref = _case(esp, ctx, M, N, K, seed)
        print(f"static scratch M={M} N={N} K={K}", flush=True)
        Y0 = ctx.spmm(X, comp, th)
        Y1 = torch.full_like(Y0, float("nan"))
        before = torch.cuda.memory_allocated()
        ctx.spmm_static(X, comp, th, out=Y1)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert (_bits(Y0) == _bits(Y1)).all()
        assert orc.rowwise_rel_error(Y1.float().cpu().numpy(), Yref).max() <= 2e-3
    # every variant that accepts a shape, twice in a row on the same array
    X, comp, th, Yref = _case(esp, ctx, 33, 80, 2048, 5)
    for v in range(esp.num_variants()):
        try:
            Y0 = ctx.spmm(X, comp, th, variant=v)
        except esp.EsparseError as e:
            assert e.code == -2
            continue
        for _ in range(2):
            Y1 = torch.full_like(Y0, float("nan"))
            ctx.spmm_static(X, comp, th, variant=v, out=Y1)
            torch.cuda.synchronize()
            assert (_bits(Y0) == _bits(Y1)).all(), esp.variant_name(v)
    # a shape whose built-in choice (a stream kernel) keeps more partial tiles than the array holds: the call takes the
    # built-in choice among the kernels without partial tiles instead
    M, N, K = 100, 9600, 256
    vs = {esp.variant_name(v): v for v in range(esp.num_variants())}
    assert esp.spmm_workspace(M, N, K) > (64 << 20) > esp.spmm_workspace(M, N, K, vs["tile32_w8_t128"])
    X, comp, th, Yref = _case(esp, ctx, M, N, K, 6)
    Y1 = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    ctx.spmm_static(X, comp, th, out=Y1)
    torch.cuda.synchronize()
    assert orc.rowwise_rel_error(Y1.float().cpu().numpy(), Yref).max() <= 2e-3
    assert (_bits(ctx.spmm(X, comp, th, variant=vs["tile32_w8_t128"])) == _bits(Y1)).all()
    # beyond the fixed size: a clear error, nothing launched, the output untouched
    M, N, K = 4096, 256, 16384          # 128 MiB of staged activations
    Y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    Xbig = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    wbytes = esp.compressed_size(N, K, 2, 4)[2]
    comp_big = esp.Compressed(None, None, torch.zeros(wbytes, dtype=torch.uint8, device="cuda"), N, K, 2, 4, esp.F16)
    with pytest.raises(esp.EsparseError) as e:
        ctx.spmm_static(Xbig, comp_big, None, out=Y)
    assert e.value.code == -7 and "static scratch" in str(e.value)
    assert int(Y.count_nonzero()) == 0
    # M = 0 is a no-op
    rc = lib.esparse_spmm_static(ctx._h, None, 0, None, None, 16, 16, 0, 2, 4, None, -1)
    assert rc == 0


@pytest.mark.parametrize("M", [1, 2, 8, 70])
def test_static_scratch_call_captured_in_a_hip_graph(M):
    """The callers this entry point exists for: the whole call (theta gathered in the kernel for one or two tokens, the
    staging launch into the library's scratch otherwise) is captured into a HIP graph once and replayed with new
    activations, eager work of the same context between the replays; every replay reproduces the eager result of
    esparse_spmm bit for bit."""
    import paper_2310_15929_amd as esp
    ctx = esp.Context(0)
    N, K = 272, 2048
    rng = np.random.default_rng(M)
    W = wl.normal_matrix(N, K, wl.stream_id("nag-w", M), scale=K ** -0.5)
    theta = rng.permutation(K)
    mask = orc.nm_mask_vectorised(W.numpy(), np.ones(K), theta, 2, 4)
    th = torch.tensor(theta, dtype=torch.int32).cuda()
    comp = ctx.compress(W.cuda(), torch.tensor(mask).cuda(), th, canonical=False)
    Xs = [wl.normal_matrix(M, K, wl.stream_id("nag-x", M, i)).cuda() for i in range(3)]
    other = wl.normal_matrix(M + 3, K, wl.stream_id("nag-o", M)).cuda()
    eager = [_bits(ctx.spmm(x, comp, th)) for x in Xs]
    xin = Xs[0].clone()
    yout = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    print(f"static scratch under graph capture M={M}", flush=True)
    with torch.cuda.stream(side):
        ctx.spmm_static(xin, comp, th, out=yout)                # warm-up on the side stream (looks the scratch address up)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            ctx.spmm_static(xin, comp, th, out=yout)
    torch.cuda.synchronize()
    for i in (1, 2, 0):
        xin.copy_(Xs[i])
        yout.zero_()
        ctx.spmm(other, comp, th)                               # eager work between the replays (its own workspace)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert (_bits(yout) == eager[i]).all(), i
    del g
