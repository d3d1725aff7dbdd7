"""The allocation-free correction scan (snlp_correction_scan_static: probe partials in a fixed device array inside
the library instead of a caller workspace) against snlp_correction_scan, through the C ABI (-m gpu).

Same kernels, same order: the written trace and the probe must be bit-identical.  Two calls in a row share the one
array, the second with a smaller input (fewer partial blocks and fewer layers than the entries the first call left
behind); then a larger 256-thread-block shape, a shape beyond the array's limit (must be refused without a launch),
and the allocator's counters around the calls."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def reference(snlp, mode, n, L, M, d, old, g, Hres, pre, post, with_probe):
    hd = d if d <= 256 and d % 2 == 0 else 4
    m = snlp.Snlp(L=L, d=d, n_heads=d // hd, head_dim=hd, d_mlp=64, B=1, T=M, n_streams=n, dtype=snlp.F32)
    if n > 1:
        m.set_hc(Hres, pre, post)
    tr = m.bind_trace()
    tr.copy_(old)
    probe = torch.zeros((2, L), dtype=torch.float32, device=tr.device) if with_probe else None
    m.correction_scan(mode, g, probe)
    torch.cuda.synchronize()
    out = tr.clone()
    m.close()
    return out, probe


def run_case(snlp, seed, mode, n, L, M, d, with_probe=True):
    print("[case] static scan mode=%d n=%d L=%d M=%d d=%d probe=%s" % (mode, n, L, M, d, with_probe), flush=True)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed)
    Hres = rng.uniform(0, 1, (L, n, n)).astype(np.float32)
    post = rng.uniform(0.5, 2, (L, n)).astype(np.float32)
    pre = rng.uniform(0, 1, (L, n)).astype(np.float32)
    old = torch.from_numpy(rng.standard_normal((L + 1, M, n, d)).astype(np.float32)).to(dev)
    g = torch.from_numpy(rng.standard_normal((L, M, d)).astype(np.float32)).to(dev)
    ref, ref_probe = reference(snlp, mode, n, L, M, d, old, g, Hres, pre, post, with_probe)
    tr = old.clone()
    probe = torch.full((2, L), -1.0, dtype=torch.float32, device=dev) if with_probe else None
    Hd = torch.from_numpy(Hres).to(dev) if n > 1 else None
    pd = torch.from_numpy(post).to(dev) if n > 1 else None
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
    snlp.correction_scan_static(mode, tr, g, Hd, pd, probe)
    after = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before                                   # no torch allocation inside the call
    assert torch.equal(tr.view(torch.int32), ref.view(torch.int32))
    if with_probe:
        assert torch.equal(probe.view(torch.int32), ref_probe.view(torch.int32))
        assert bool((probe[0] > 0).all())


def test_static_scratch_correction_scan_matches_workspace_version():
    import paper_2605_17842_amd as snlp
    run_case(snlp, 1, snlp.HCN, 4, 9, 300, 256)              # 64-thread blocks, 300 partial blocks x 18 entries
    run_case(snlp, 2, snlp.IDN, 1, 5, 37, 132)               # right after it, smaller: 20 blocks x 10 entries
    run_case(snlp, 3, snlp.IDN, 4, 3, 8, 64)                 # IDN on a 4-stream state
    run_case(snlp, 4, snlp.IDN, 1, 12, 2048, 768)            # 256-thread blocks (M d > 2^20), 1536 blocks x 24
    run_case(snlp, 5, snlp.HCN, 2, 6, 100, 128, with_probe=False)
    run_case(snlp, 6, snlp.HCN, 4, 9, 300, 256)              # the first case again after the others


def test_static_scratch_limit_and_argument_errors():
    import paper_2605_17842_amd as snlp
    dev = torch.device("cuda:0")
    # 2^20 / 4 / 64 = 4096 blocks of 64 threads; x 2 x L = 160 floats each -> 655360 fits, L = 200 does not
    M, d = 1024, 1024
    for L, ok in ((80, True), (200, False)):
        tr = torch.zeros((L + 1, M, 1, d), dtype=torch.float32, device=dev)
        g = torch.zeros((L, M, d), dtype=torch.float32, device=dev)
        probe = torch.full((2, L), -1.0, dtype=torch.float32, device=dev)
        if ok:
            snlp.correction_scan_static(snlp.IDN, tr, g, None, None, probe)
            torch.cuda.synchronize()
            assert bool((probe == 0).all())
        else:
            with pytest.raises(snlp.SnlpError, match="static scratch"):
                snlp.correction_scan_static(snlp.IDN, tr, g, None, None, probe)
            torch.cuda.synchronize()
            assert bool((probe == -1).all())                 # nothing was launched
            snlp.correction_scan_static(snlp.IDN, tr, g, None, None, None)   # without a probe no scratch is needed
            torch.cuda.synchronize()
        del tr, g
    tr = torch.zeros((3, 4, 2, 8), dtype=torch.float32, device=dev)
    g = torch.zeros((2, 4, 8), dtype=torch.float32, device=dev)
    with pytest.raises(snlp.SnlpError):
        snlp.correction_scan_static(snlp.HCN, tr, g, None, None, None)        # n > 1 without post / Hres
    with pytest.raises(snlp.SnlpError):
        snlp.correction_scan_static(snlp.HCN, tr[:, :, :1].contiguous(), g, None, None, None)   # HCN on one stream
