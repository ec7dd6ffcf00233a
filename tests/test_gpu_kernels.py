"""Parity of each HIP kernel, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import flover_synth as synth
from oracle import oracle as orc

pytestmark = pytest.mark.gpu

fl = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global fl
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2305_13484_amd as m
    fl = m
    m.load_library()


TDT = synth.TORCH_DTYPE


# ---------------------------------------------------------------- weight GEMM

@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16, synth.DT_F32])
@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (5, 100, 96), (16, 256, 512), (17, 1000, 256), (33, 130, 1024),
                                   (70, 320, 2048), (128, 192, 4096), (200, 64, 160), (300, 320, 1024),
                                   (513, 130, 512), (48, 200, 512), (90, 130, 1024), (100, 320, 512)])
def test_gemm_matches_oracle(dtype, M, N, K):
    print("gemm", dtype, M, N, K, flush=True)
    g = torch.Generator().manual_seed(100 + M + N)
    x = torch.randn((M, K), generator=g).to(TDT[dtype])
    W = (torch.randn((N, K), generator=g) * 0.05).to(TDT[dtype])
    ref = orc.gemm(dtype, x, W)
    got = fl.k_gemm(x.cuda(), W.cuda()).cpu().double().numpy()
    bound = (x.double().abs() @ W.double().abs().T).numpy()       # sum of |terms| per output
    assert np.all(np.abs(got - ref) <= 4e-6 * bound + 1e-30)


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
def test_gemm_row_result_does_not_depend_on_other_rows(dtype):
    g = torch.Generator().manual_seed(5)
    K, N = 1024, 448
    x = torch.randn((600, K), generator=g).to(TDT[dtype]).cuda()
    W = (torch.randn((N, K), generator=g) * 0.05).to(TDT[dtype]).cuda()
    tw = fl.binding.TiledWeight(W)
    full = fl.k_gemm(x, tw)
    for M in (1, 16, 17, 32, 48, 64, 65, 81, 96, 100, 112, 128, 129, 256, 257, 400, 513):   # every count of 16-row tiles up to 8
        part = fl.k_gemm(x[:M].contiguous(), tw)
        assert torch.equal(part, full[:M]), M
    alone = fl.k_gemm(x[77:78].contiguous(), tw)
    assert torch.equal(alone[0], full[77])


@pytest.mark.parametrize("M", [8, 24, 48, 72, 96, 112, 128, 600])
def test_gemm_full_size_sampled_columns(M):
    """The 7B shapes the benchmark runs, at row counts that select each kernel variant (<=16 direct, <=32 / <=64 / <=128
    LDS-staged with 4 or 8 waves, above that the 256-row blocks of a context pass with a ragged last block); sampled
    output columns from the oracle."""
    dtype = synth.DT_BF16
    for (N, K) in [(12288, 4096), (4096, 11008), (22016, 4096), (32000, 4096)]:
        print("gemm full", M, N, K, flush=True)
        g = torch.Generator(device="cuda").manual_seed(N + M)
        x = torch.randn((M, K), generator=g, device="cuda").to(TDT[dtype])
        W = (torch.randn((N, K), generator=g, device="cuda") * 0.02).to(TDT[dtype])
        got = fl.k_gemm(x, W)
        cols = np.random.default_rng(N).choice(N, size=24, replace=False)
        cols = np.concatenate([cols, [0, N - 1]]).astype(np.int32)
        xh, Wh = x.cpu(), W[torch.as_tensor(cols, device="cuda").long()].cpu().contiguous()
        ref = orc.gemm(dtype, xh, Wh)
        bound = (xh.double().abs() @ Wh.double().abs().T).numpy()
        err = np.abs(got[:, torch.as_tensor(cols, device="cuda").long()].cpu().double().numpy() - ref)
        assert np.all(err <= 4e-6 * bound)
        del W


# ---------------------------------------------------------------- gated MLP input (contraction + activation, one launch)

def _gated_reference(dtype, x, Wg, Wu):
    """fp64 silu(g) * u before the final rounding, and a bound on what fp32 accumulation may move it by."""
    g, u = orc.gemm(dtype, x, Wg), orc.gemm(dtype, x, Wu)
    eg = 4e-6 * (x.double().abs() @ Wg.double().abs().T).numpy()
    eu = 4e-6 * (x.double().abs() @ Wu.double().abs().T).numpy()
    sg = g / (1.0 + np.exp(-g))
    ref = sg * u
    slack = 1.1 * np.abs(u) * eg + np.abs(sg) * eu          # |d silu / dg| <= 1.1
    return ref, slack


def _gated_check(dtype, got, ref, slack):
    half_ulp = 2.0 ** -8 if dtype == synth.DT_BF16 else 2.0 ** -11       # relative, of the rounding to the model dtype
    tiny = 0.0 if dtype == synth.DT_BF16 else 2.0 ** -25                  # fp16 subnormal spacing
    assert np.all(np.abs(got - ref) <= half_ulp * np.abs(ref) * 1.001 + slack * (1 + half_ulp) + tiny + 1e-30)


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
@pytest.mark.parametrize("M,F,K", [(1, 32, 512), (7, 96, 512), (16, 352, 1024), (17, 64, 1024), (32, 160, 512),
                                   (33, 96, 2048), (64, 224, 512), (65, 128, 1024), (128, 96, 512), (129, 64, 512),
                                   (300, 160, 1024), (48, 96, 512), (90, 160, 1024), (110, 64, 512)])
def test_gated_mlp_matches_oracle(dtype, M, F, K):
    print("gated", dtype, M, F, K, flush=True)
    g = torch.Generator().manual_seed(300 + M + F)
    x = torch.randn((M, K), generator=g).to(TDT[dtype])
    Wg = (torch.randn((F, K), generator=g) * 0.05).to(TDT[dtype])
    Wu = (torch.randn((F, K), generator=g) * 0.05).to(TDT[dtype])
    ref, slack = _gated_reference(dtype, x, Wg, Wu)
    gw = fl.binding.GatedWeight(Wg.cuda(), Wu.cuda())
    got = fl.k_gated_mlp(x.cuda(), gw).cpu().double().numpy()
    _gated_check(dtype, got, ref, slack)


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
def test_gated_mlp_row_result_does_not_depend_on_other_rows(dtype):
    g = torch.Generator().manual_seed(6)
    K, F = 1024, 416
    x = torch.randn((300, K), generator=g).to(TDT[dtype]).cuda()
    gw = fl.binding.GatedWeight((torch.randn((F, K), generator=g) * 0.05).to(TDT[dtype]).cuda(),
                                (torch.randn((F, K), generator=g) * 0.05).to(TDT[dtype]).cuda())
    full = fl.k_gated_mlp(x, gw)
    for M in (1, 16, 17, 32, 33, 48, 64, 65, 81, 96, 100, 112, 128, 129, 200, 257):   # every count of 16-row tiles up to 8
        part = fl.k_gated_mlp(x[:M].contiguous(), gw)
        assert torch.equal(part, full[:M]), M
    alone = fl.k_gated_mlp(x[77:78].contiguous(), gw)
    assert torch.equal(alone[0], full[77])


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
@pytest.mark.parametrize("M,F,K", [(40, 96, 512), (130, 352, 1024), (300, 160, 1024), (600, 224, 512)])
def test_gated_mlp_of_a_context_pass_matches_oracle(dtype, M, F, K):
    g = torch.Generator().manual_seed(400 + M + F)
    x = torch.randn((M, K), generator=g).to(TDT[dtype])
    Wg = (torch.randn((F, K), generator=g) * 0.05).to(TDT[dtype])
    Wu = (torch.randn((F, K), generator=g) * 0.05).to(TDT[dtype])
    ref, slack = _gated_reference(dtype, x, Wg, Wu)
    gw = fl.binding.GatedWeight(Wg.cuda(), Wu.cuda())
    got = fl.k_gated_mlp(x.cuda(), gw, context_pass=True).cpu().double().numpy()
    _gated_check(dtype, got, ref, slack)


@pytest.mark.parametrize("M,context", [(8, False), (24, False), (48, False), (64, False), (72, False), (96, False),
                                       (112, False), (128, False), (300, True), (513, True), (1024, True)])
def test_gated_mlp_full_size_sampled_columns(M, context):
    """The 7B gate|up shape at row counts that select each variant of the one-launch form (1 to 8 row tiles); as a
    context pass: one slice with the activation as the 256-row-block kernel's epilogue (300, 513 and
    1024 rows, incl. ragged last blocks) -- sampled MLP columns from the oracle."""
    dtype, F, K = synth.DT_BF16, 11008, 4096
    print("gated full", M, context, flush=True)
    if context:
        from paper_2305_13484_amd.binding import k_gemm_plan
        # the plan of the plain 2F-column matrix is a lower bound of how attractive one slice is for the paired one
        print("slices of a plain matrix of this shape:", k_gemm_plan(dtype, 2 * F, K, M))
    g = torch.Generator(device="cuda").manual_seed(F + M)
    x = torch.randn((M, K), generator=g, device="cuda").to(TDT[dtype])
    Wg = (torch.randn((F, K), generator=g, device="cuda") * 0.02).to(TDT[dtype])
    Wu = (torch.randn((F, K), generator=g, device="cuda") * 0.02).to(TDT[dtype])
    got = fl.k_gated_mlp(x, fl.binding.GatedWeight(Wg, Wu), context_pass=context)
    cols = np.concatenate([np.random.default_rng(M).choice(F, size=24, replace=False), [0, 15, 16, F - 1]])
    ci = torch.as_tensor(cols, device="cuda").long()
    ref, slack = _gated_reference(dtype, x.cpu(), Wg[ci].cpu().contiguous(), Wu[ci].cpu().contiguous())
    _gated_check(dtype, got[:, ci].cpu().double().numpy(), ref, slack)


def test_gated_mlp_at_the_30b_shape_sampled_columns_and_row_invariance():
    """F = 17920, K = 6656: more 128-column blocks than compute units, so 33-64 rows take the 256-column blocks of 16
    waves; sampled MLP columns from the oracle, and every row count gives the same bits for a row."""
    dtype, F, K = synth.DT_BF16, 17920, 6656
    g = torch.Generator(device="cuda").manual_seed(30)
    x = torch.randn((100, K), generator=g, device="cuda").to(TDT[dtype])
    Wg = (torch.randn((F, K), generator=g, device="cuda") * 0.02).to(TDT[dtype])
    Wu = (torch.randn((F, K), generator=g, device="cuda") * 0.02).to(TDT[dtype])
    gw = fl.binding.GatedWeight(Wg, Wu)
    full = fl.k_gated_mlp(x, gw)
    for M in (8, 24, 48, 64, 65, 100):       # 65 and 100 rows: two launches at this shape
        print("gated 30b", M, flush=True)
        assert torch.equal(fl.k_gated_mlp(x[:M].contiguous(), gw), full[:M]), M
    cols = np.concatenate([np.random.default_rng(3).choice(F, size=20, replace=False), [0, 16, F - 1]])
    ci = torch.as_tensor(cols, device="cuda").long()
    ref, slack = _gated_reference(dtype, x[:48].cpu(), Wg[ci].cpu().contiguous(), Wu[ci].cpu().contiguous())
    _gated_check(dtype, full[:48, ci].cpu().double().numpy(), ref, slack)


def test_gated_mlp_rejects_shapes_it_does_not_serve():
    lib = fl.load_library()
    assert lib.flover_k_gated_mlp(2, None, None, 4, 48, 512, 0, None, None, 0, None) == -1       # F not a multiple of 32
    assert lib.flover_k_gated_mlp(2, None, None, 4, 64, 256, 0, None, None, 0, None) == -1       # K not a multiple of 512
    assert lib.flover_k_gated_mlp(0, None, None, 4, 64, 512, 0, None, None, 0, None) == -1       # fp32


# ---------------------------------------------------------------- ragged decode attention

ATT_TOL = {synth.DT_F32: 2e-5, synth.DT_F16: 1.5e-3, synth.DT_BF16: 1e-2}   # |err| / max|ref row|: rounding of the output
                                                                            # to dtype (2^-11, 2^-8 half-ulps) + fp32 softmax


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16, synth.DT_F32])
@pytest.mark.parametrize("d", [64, 128])
def test_attention_matches_oracle(dtype, d):
    print("attention", dtype, d, flush=True)
    M, Cn, nh, S = 11, 14, 8, 700
    q, k, v, slots, lens = synth.attention_case(17 + d, M, Cn, nh, d, S, dtype, 1, S)
    lens[:5] = [1, 2, 255, 256, 257]       # single row, chunk boundaries
    lens[5] = S
    # rows at or beyond len hold garbage that must not be read into the result
    for s_, n_ in zip(slots.tolist(), lens.tolist()):
        k[s_, :, n_:] = float("nan")
        v[s_, :, n_:] = float("nan")
    pairs = [(m, h) for m in range(M) for h in range(nh)]
    ref = orc.attention(dtype, q, k, v, slots, lens, pairs).reshape(M, nh, d)
    got = fl.k_decode_attention(q.cuda(), k.cuda(), v.cuda(), slots, lens).cpu().double().numpy()
    assert np.isfinite(got).all()
    scale = np.abs(ref).max(axis=2, keepdims=True)
    assert (np.abs(got - ref) / scale).max() <= ATT_TOL[dtype]


def test_attention_row_result_does_not_depend_on_other_rows():
    dtype, d = synth.DT_BF16, 128
    M, Cn, nh, S = 9, 12, 4, 600
    q, k, v, slots, lens = synth.attention_case(3, M, Cn, nh, d, S, dtype, 1, S)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    full = fl.k_decode_attention(qd, kd, vd, slots, lens)
    for m in range(M):
        one = fl.k_decode_attention(qd[m:m + 1].contiguous(), kd, vd, slots[m:m + 1], lens[m:m + 1])
        assert torch.equal(one[0], full[m])


def test_attention_benchmark_shape_sampled_pairs():
    """Config 2's shape (256 live, 32 heads, head_dim 128, lengths U{1..4096}, bf16): sampled (row, head) outputs."""
    dtype, M, Cn, nh, d, S = synth.DT_BF16, 256, 256, 32, 128, 4096
    print("attention full size", flush=True)
    q, k, v, slots, lens = synth.attention_case(2, M, Cn, nh, d, S, dtype, 1, S, device="cuda", fill="all")
    got = fl.k_decode_attention(q, k, v, slots, lens)
    rng = np.random.default_rng(0)
    rows = np.concatenate([rng.choice(M, size=10, replace=False), [int(np.argmax(lens)), int(np.argmin(lens))]])
    heads = rng.integers(0, nh, size=len(rows))
    # a compact host cache holding just the sampled (slot, head) planes
    kk = torch.stack([k[slots[r], h] for r, h in zip(rows, heads)]).unsqueeze(1).cpu().contiguous()
    vv = torch.stack([v[slots[r], h] for r, h in zip(rows, heads)]).unsqueeze(1).cpu().contiguous()
    qq = torch.stack([q[r, h] for r, h in zip(rows, heads)]).unsqueeze(1).cpu().contiguous()
    ref = orc.attention(dtype, qq, kk, vv, np.arange(len(rows)), lens[rows], [(i, 0) for i in range(len(rows))])
    g = torch.stack([got[r, h] for r, h in zip(rows, heads)]).cpu().double().numpy()
    scale = np.abs(ref).max(axis=1, keepdims=True)
    assert (np.abs(g - ref) / scale).max() <= ATT_TOL[dtype]
    del k, v
    torch.cuda.empty_cache()


def test_attention_rejects_bad_arguments():
    q, k, v, slots, lens = synth.attention_case(1, 2, 3, 4, 64, 32, synth.DT_BF16, 1, 32)
    bad = lens.copy()
    bad[0] = 33
    with pytest.raises(fl.FloverError):
        fl.k_decode_attention(q.cuda(), k.cuda(), v.cuda(), slots, bad)
    bad = slots.copy()
    bad[1] = 3
    with pytest.raises(fl.FloverError):
        fl.k_decode_attention(q.cuda(), k.cuda(), v.cuda(), bad, lens)
    out = fl.k_decode_attention(q.cuda()[:0].contiguous(), k.cuda(), v.cuda(), slots[:0], lens[:0])   # empty batch
    assert out.shape[0] == 0


# ---------------------------------------------------------------- memory shuffle copy

@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F32])
def test_compact_is_bit_exact(dtype):
    L, Cn, nh, S, d = 3, 10, 4, 300, 64
    g = torch.Generator().manual_seed(9)
    cache = torch.randn((L, 2, Cn, nh, S, d), generator=g).to(TDT[dtype])
    src, dst, ln = [7, 9, 0, 8], [2, 3, 5, 4], [300, 1, 129, 0]
    ref = cache.clone()
    orc.compact(ref, L, Cn, nh, S, d, cache.element_size(), src, dst, ln)
    dev = cache.cuda()
    fl.k_compact(dev, src, dst, ln)
    assert torch.equal(dev.cpu().view(torch.uint8), ref.view(torch.uint8))
    # rows >= len of the destination and all other slots stay untouched
    assert torch.equal(dev.cpu()[:, :, 3, :, 1:], cache[:, :, 3, :, 1:])
    assert torch.equal(dev.cpu()[:, :, 1], cache[:, :, 1])


def test_compact_rejects_overlapping_sets_and_empty_list():
    cache = torch.zeros((1, 2, 4, 4, 8, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fl.FloverError):
        fl.k_compact(cache, [0, 1], [1, 2], [4, 4])
    with pytest.raises(fl.FloverError):
        fl.k_compact(cache, [0], [5], [4])
    fl.k_compact(cache, [], [], [])


def test_compact_benchmark_shape():
    """Config 2's cache (1 layer, 256 slots, 32 heads, 4096 x 128 bf16 = 16 GiB): 26 moves, checked by equality with
    the sources' snapshots and by checksums of every untouched slot."""
    print("compact full size", flush=True)
    L, Cn, nh, S, d = 1, 256, 32, 4096, 128
    cache = torch.empty((L, 2, Cn, nh, S, d), dtype=torch.bfloat16, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(4)
    for c in range(Cn):
        cache[0, :, c].copy_(torch.randn((2, nh, S, d), generator=gen, device="cuda"))
    rng = np.random.default_rng(4)
    perm = rng.permutation(Cn)
    src, dst = perm[:26].tolist(), perm[26:52].tolist()
    ln = rng.integers(1, S + 1, size=26).tolist()
    ln[0], ln[1] = S, 1
    before = [cache[:, :, s, :, :n].clone() for s, n in zip(src, ln)]
    tails = [cache[:, :, t, :, n:].clone() for t, n in zip(dst, ln)]
    sums = cache.view(torch.int16).to(torch.int32).sum(dim=(0, 1, 3, 4, 5))
    fl.k_compact(cache, src, dst, ln)
    for i, (s, t, n) in enumerate(zip(src, dst, ln)):
        assert torch.equal(cache[:, :, t, :, :n], before[i])
        assert torch.equal(cache[:, :, t, :, n:], tails[i])
    after = cache.view(torch.int16).to(torch.int32).sum(dim=(0, 1, 3, 4, 5))
    untouched = np.setdiff1d(np.arange(Cn), dst)
    assert torch.equal(after[untouched], sums[untouched])
    del cache
    torch.cuda.empty_cache()


def test_copy_probe_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    fl.k_copy_probe(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
