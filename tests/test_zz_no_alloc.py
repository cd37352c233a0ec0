"""moe_permute_static (the entry point for callers that cannot allocate: fixed device scratch inside the library, no
context) against moe_permute on the same inputs, bit for bit: two calls in a row, the second on a smaller problem,
then a third at the largest size the fixed scratch admits for this expert count; and the refusal beyond it."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _inputs(T, k, h, E, seed, skip_frac=0.05):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    idx = torch.randint(0, E, (T, k), dtype=torch.int32, device="cuda", generator=g)
    drop = torch.rand((T, k), device="cuda", generator=g) < skip_frac      # "not on this GPU" slots
    idx = torch.where(drop, torch.full_like(idx, -1), idx)
    X = (torch.randn((T, h), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    return idx, X


def _run(fn, X, idx, T, k, h, E, align):
    i32 = torch.int32
    Rcap = T * k + E * (align - 1)
    # canaries: rows beyond offsets[E] must stay untouched, padding rows must be zeroed
    Xp = torch.full((Rcap, h), 7.0, dtype=torch.bfloat16, device="cuda")
    row_of = torch.full((T, k), -7, dtype=i32, device="cuda")
    src_of = torch.full((Rcap,), -7, dtype=i32, device="cuda")
    offsets = torch.full((E + 1,), -7, dtype=i32, device="cuda")
    counts = torch.full((E,), -7, dtype=i32, device="cuda")
    fn(X, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts)
    torch.cuda.synchronize()
    return [t.cpu().numpy() if t.dtype != torch.bfloat16 else t.view(torch.int16).cpu().numpy()
            for t in (Xp, row_of, src_of, offsets, counts)]


def test_permute_static_matches_permute():
    from paper_2603_07685_amd import binding as B
    B.lib()
    torch.cuda.set_device(0)
    ctx = B.Context(16384, 8, 256, 1024, 256)

    def with_ctx(X, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts):
        B.moe_permute(ctx, X, B.BF16, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts)

    def static(X, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts):
        B.moe_permute_static(X, B.BF16, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts)

    # the second call is smaller than the first (the shared scratch still holds the first call's histograms), the
    # third is the router-wide shape of the DeepSeek-V3-style config (256 experts)
    for (T, k, h, E, align, seed) in [(4099, 8, 512, 96, 1, 11), (517, 2, 256, 8, 128, 12), (16384, 8, 64, 256, 16, 13)]:
        idx, X = _inputs(T, k, h, E, seed)
        ref = _run(with_ctx, X, idx, T, k, h, E, align)
        got = _run(static, X, idx, T, k, h, E, align)
        for name, a, b in zip(("Xp", "row_of", "src_of", "offsets", "counts"), got, ref):
            assert np.array_equal(a, b), (name, T, k, E)
        assert int(ref[4].sum()) == int((idx >= 0).sum().item())
    # maps only (X = Xp = NULL), as the fused-quantisation layers call it
    T, k, h, E, align = 1000, 4, 128, 16, 32
    idx, X = _inputs(T, k, h, E, 14)
    Rcap = T * k + E * (align - 1)
    outs = []
    for fn in (lambda *a: B.moe_permute(ctx, None, B.BF16, idx, T, k, h, E, align, None, Rcap, *a),
               lambda *a: B.moe_permute_static(None, B.BF16, idx, T, k, h, E, align, None, Rcap, *a)):
        bufs = [torch.full(s, -7, dtype=torch.int32, device="cuda") for s in ((T, k), (Rcap,), (E + 1,), (E,))]
        fn(*bufs)
        torch.cuda.synchronize()
        outs.append([b.cpu().numpy() for b in bufs])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_permute_static_refuses_sizes_beyond_its_scratch():
    from paper_2603_07685_amd import binding as B
    B.lib()
    torch.cuda.set_device(0)
    T, k, E = 262144 + 1024, 1, 1024          # 257 chunks x 1024 experts x 4 B > 1 MiB
    i32 = torch.int32
    idx = torch.zeros((T, k), dtype=i32, device="cuda")
    row_of = torch.full((T, k), -7, dtype=i32, device="cuda")
    src_of = torch.full((T * k,), -7, dtype=i32, device="cuda")
    offsets = torch.full((E + 1,), -7, dtype=i32, device="cuda")
    counts = torch.full((E,), -7, dtype=i32, device="cuda")
    with pytest.raises(B.MoeError, match="exceeds the fixed scratch"):
        B.moe_permute_static(None, B.BF16, idx, T, k, 8, E, 1, None, T * k, row_of, src_of, offsets, counts)
    torch.cuda.synchronize()
    assert int(row_of.min().item()) == -7 and int(offsets.max().item()) == -7   # nothing was launched
    # exactly at the limit it runs
    T = 262144
    B.moe_permute_static(None, B.BF16, idx[:T], T, k, 8, E, 1, None, T * k, row_of[:T], src_of[:T], offsets, counts)
    torch.cuda.synchronize()
    assert int(counts[0].item()) == T and int(offsets[E].item()) == T
