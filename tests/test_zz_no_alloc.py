"""The entry point that allocates nothing (lags_sparsify_layer_noalloc) against
lags_sparsify_layer, bit for bit, through the C ABI: pairs of calls in a row on one stream, the
second with a smaller input, over layers of every route; capacity errors enqueue nothing."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.cpu().numpy().view(np.uint32)


def test_noalloc_matches_sparsify_layer():
    import torch
    from paper_1911_08727_amd import lags
    dev = torch.device("cuda:0")
    ctx = lags.Context(0)
    gen = torch.Generator(device=dev).manual_seed(77)
    # (d, rho): multi-workgroup finish, one-workgroup finish (large and small workgroups, short and
    # full sample), the two one-workgroup classes, a layer
    # too dense to sample (multi-pass route), an all-zero layer (rejected guess)
    cases = [(3_000_001, 0.001), (700_000, 0.004), (16_000_000, 0.0015), (8_000_000, 0.004), (1 << 20, 0.001), (30_000, 0.01),
             (5_000, 0.002), (600, 0.01), (300_000, 0.5), (250_000, 0.001), (41_000, 0.003), (40, 1.0)]
    lr = 0.25
    for n, (d, rho) in enumerate(cases):
        k = lags.lags_topk_count(d, rho)
        print("[gpu-case] noalloc d=%d k=%d" % (d, k), flush=True)
        g = torch.empty(d, dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=gen)
        if d == 250_000:
            g.zero_()
        r0 = torch.empty(d, dtype=torch.float32, device=dev).normal_(0.0, 0.3, generator=gen)
        if d == 250_000:
            r0.zero_()
        g_before = g.clone()
        res_a, res_b = r0.clone(), r0.clone()
        oi_a = torch.full((k,), -7, dtype=torch.int32, device=dev)
        ov_a = torch.full((k,), float("nan"), dtype=torch.float32, device=dev)
        oi_b, ov_b = oi_a.clone(), ov_a.clone()
        ctx.lags_sparsify_layer(g, res_a, lr, k, oi_a, ov_a)
        lags.lags_sparsify_layer_noalloc(0, g, res_b, lr, k, oi_b, ov_b)
        torch.cuda.synchronize()
        assert np.array_equal(oi_a.cpu().numpy(), oi_b.cpu().numpy()), (d, k)
        assert np.array_equal(_bits(ov_a), _bits(ov_b)), (d, k)
        assert np.array_equal(_bits(res_a), _bits(res_b)), (d, k)
        assert np.array_equal(_bits(g), _bits(g_before)), "grad was written"
    ctx.destroy()


def test_noalloc_rejects_what_does_not_fit():
    import torch
    from paper_1911_08727_amd import lags
    dev = torch.device("cuda:0")
    assert lags.lags_noalloc_max_elements() == 16_777_216
    d = lags.lags_noalloc_max_elements() + 4096
    g = torch.zeros(d, dtype=torch.float32, device=dev)
    r = torch.zeros(d, dtype=torch.float32, device=dev)
    k = 1000
    oi = torch.full((k,), -7, dtype=torch.int32, device=dev)
    ov = torch.full((k,), 3.0, dtype=torch.float32, device=dev)
    with pytest.raises(lags.LagsError) as e:
        lags.lags_sparsify_layer_noalloc(0, g, r, 0.1, k, oi, ov)
    assert e.value.code == lags.LAGS_ECAPACITY
    # dense enough to need 1024 slots per tile: 3907 tiles x 1024 > 2^19
    d2 = 16_000_000
    k2 = lags.lags_topk_count(d2, 0.03)
    oi2 = torch.full((k2,), -7, dtype=torch.int32, device=dev)
    ov2 = torch.full((k2,), 3.0, dtype=torch.float32, device=dev)
    with pytest.raises(lags.LagsError) as e:
        lags.lags_sparsify_layer_noalloc(0, g[:d2], r[:d2], 0.1, k2, oi2, ov2)
    assert e.value.code == lags.LAGS_ECAPACITY
    with pytest.raises(lags.LagsError) as e:
        lags.lags_sparsify_layer_noalloc(0, g[:100], r[:100], float("nan"), 5, oi[:5], ov[:5])
    assert e.value.code == lags.LAGS_EINVAL
    torch.cuda.synchronize()
    assert bool((oi == -7).all()) and bool((ov == 3.0).all()) and bool((oi2 == -7).all())
