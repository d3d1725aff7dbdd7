"""Parity of the HIP path against the CPU oracle, through the C ABI (needs an MI355X: -m gpu).

Tolerances (per layer state, relative Frobenius error, maximum over layers and over the K values of a
case): 1e-5 for the fp32 operand path, 2e-2 for the bf16 operand path; the correction scan on given
branch outputs is bit-exact; squared-norm probes agree to 1e-5 relative on given branch outputs.
"""
import sys

import numpy as np
import pytest
import torch

import snlp_inputs as si
from oracle import snlp_oracle as oc
from oracle.harness import oracle_model, per_layer_rel_err, rel_err

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gh():
    from paper_2605_17842_amd import harness
    return harness


def np_trace(m):
    torch.cuda.synchronize()
    return m.trace.cpu().numpy()


def check_iterates(gh, shp, t, mode, Ks, tol, check_seq=True, check_probe=True):
    """GPU iterate from the h0 initialisation against the oracle at every K in Ks; optionally the sequential
    forward and the probe.  Returns the worst relative error seen."""
    md = oracle_model(shp, t, widen=True)
    m = gh.gpu_model(shp, t)
    worst = 0.0
    Kmax = max(Ks)
    say("%s oracle iterate K<=%d" % (shp.name, Kmax))
    _, oprobe, kept = oc.iterate(md, oc.init_trace(md, t["h0"]), mode, Kmax, keep=True)
    say("%s gpu iterate" % shp.name)
    m.init_trace(m.h0)
    probe = torch.zeros((Kmax, 2, shp.L), dtype=torch.float32, device=m.device)
    done = 0
    for K in sorted(Ks):
        m.iterate(mode, K - done, probe[done:])
        done = K
        err = per_layer_rel_err(np_trace(m), kept[K - 1])
        say("%s K=%d max rel err %.3e" % (shp.name, K, err.max()))
        assert err.max() < tol, (K, err)
        worst = max(worst, float(err.max()))
    if check_probe:
        gp = probe.cpu().numpy().astype(np.float64)
        ref = oprobe
        # The probe entries are norms of differences of states; their error is set by the error of the
        # states (tol relative to the state / branch scale), not by their own size.  Compare the norms
        # with an absolute bound tied to the largest one (the first round's, of the order of ||g||).
        bound = 4 * tol * np.sqrt(ref.max())
        assert np.all(np.abs(np.sqrt(gp) - np.sqrt(ref)) <= bound), (gp, ref)
        assert np.array_equal(gp == 0, ref == 0)        # converged layers: exactly zero on both sides
    if check_seq:
        say("%s sequential forward" % shp.name)
        seq = oc.sequential_forward(md, t["h0"], mode)
        gseq = m.sequential_forward(mode, m.h0)
        torch.cuda.synchronize()
        err = per_layer_rel_err(gseq.cpu().numpy(), seq)
        say("%s sequential max rel err %.3e" % (shp.name, err.max()))
        assert err.max() < tol, err
        worst = max(worst, float(err.max()))
    m.close()
    return worst


# ------------------------------------------------------------------ correction scan: bit-exact

# Small batches (M d <= 2^20): one wave per block, operands through the caches -- k_scan<N, U, ., ., 64, false>.
SCAN_SMALL = [(1, oc.IDN, 5, 37, 132), (4, oc.HCN, 6, 19, 260), (4, oc.IDN, 3, 8, 64), (2, oc.HCN, 9, 300, 128),
              (3, oc.HCN, 4, 5, 16), (8, oc.HCN, 3, 7, 32), (1, oc.IDN, 26, 64, 1664)]
# The sizes the prefill workloads run (M d > 2^20).  There snlp_correction_scan, like a round of snlp_iterate, runs the
# row-per-workgroup kernel that also prepares the next round's normalised inputs (k_scan_norm<N, U, PROBE, OutT, STREAM>;
# a launch whose trace exceeds 128 MB streams its operands with non-temporal loads); the 256-thread k_scan variants
# remain for the read-only probe, the one-shot-forward initialisation and the allocation-free entry point
# (test_zz_no_alloc.py, test_prefill_size_scan_variants_agree below).
SCAN_PREFILL = [
    (4, oc.HCN, 20, 2048, 1280),   # d20 HCN workload: 839 MB of trace -> k_scan_norm<4, 2, ., float, false> (fp32 context: never streamed)
    (1, oc.IDN, 26, 4096, 1664),   # d26 long prefill: 709 MB            -> k_scan_norm<1, 4, ...>
    (1, oc.IDN, 12, 2048, 768),    # d12 prefill: 75 MB
    (4, oc.HCN, 5, 1024, 1280),
    (4, oc.IDN, 3, 1024, 1280),    # H = I block on four streams, mode IDN
    (2, oc.HCN, 7, 2048, 1280),
]


@pytest.mark.parametrize("n,mode,L,M,d", SCAN_SMALL + SCAN_PREFILL)
def test_correction_scan_bit_exact_and_probe(gh, n, mode, L, M, d):
    say("scan n=%d mode=%d L=%d M=%d d=%d" % (n, mode, L, M, d))
    rng = np.random.default_rng(100 + n + L)
    shp = si.Shape("scan", L=L, d=d, n_heads=1, head_dim=d if d <= 256 and d % 2 == 0 else 4, d_mlp=64, B=1, T=M,
                   n_streams=n, bf16=False)
    shp = shp.with_(n_heads=d // shp.head_dim)
    import paper_2605_17842_amd as snlp
    m = snlp.Snlp(L=L, d=d, n_heads=shp.n_heads, head_dim=shp.head_dim, d_mlp=64, B=1, T=M, n_streams=n, dtype=snlp.F32)
    Hres = rng.uniform(0, 1, (L, n, n)).astype(np.float32)
    post = rng.uniform(0.5, 2, (L, n)).astype(np.float32)
    pre = rng.uniform(0, 1, (L, n)).astype(np.float32)
    if n > 1:
        m.set_hc(Hres, pre, post)
    md = oc.Model(L=L, d=d, n_heads=1, head_dim=d, d_mlp=1, B=1, T=M, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                  n_streams=n, Hres=Hres, pre=pre, post=post)
    old = rng.standard_normal((L + 1, M, n, d)).astype(np.float32)
    g = rng.standard_normal((L, M, d)).astype(np.float32)
    tr = m.bind_trace()
    tr.copy_(torch.from_numpy(old))
    probe = torch.zeros((2, L), dtype=torch.float32, device=tr.device)
    m.correction_scan(mode, torch.from_numpy(g).to(tr.device), probe)
    torch.cuda.synchronize()
    ref = oc.correction_scan(md, old[0], g, mode)
    got = tr.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    r_ref = oc.residual_sq(md, old, g, mode)
    d_ref = np.sum((ref[1:].astype(np.float64) - old[1:].astype(np.float64)) ** 2, axis=(1, 2, 3))
    gp = probe.cpu().numpy().astype(np.float64)
    assert np.allclose(gp[0], r_ref, rtol=1e-5, atol=0)
    assert np.allclose(gp[1], d_ref, rtol=1e-5, atol=0)
    # without a probe the written trace is the same
    tr.copy_(torch.from_numpy(old))
    m.correction_scan(mode, torch.from_numpy(g).to(tr.device), None)
    torch.cuda.synchronize()
    assert np.array_equal(tr.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    m.close()


@pytest.mark.parametrize("n,mode,L,M,d", [(4, oc.HCN, 20, 2048, 1280), (1, oc.IDN, 26, 4096, 1664), (1, oc.IDN, 12, 2048, 768),
                                          (4, oc.IDN, 3, 1024, 1280)])
def test_prefill_size_scan_variants_agree(gh, n, mode, L, M, d):
    """The 256-thread k_scan variants at prefill sizes (streamed above 128 MB of trace: k_scan<N, U, ., ., 256, true / false>),
    reached through the allocation-free entry point, against the oracle bit for bit, probe included."""
    import paper_2605_17842_amd as snlp
    say("static scan n=%d mode=%d L=%d M=%d d=%d" % (n, mode, L, M, d))
    rng = np.random.default_rng(400 + n + L)
    Hres = rng.uniform(0, 1, (L, n, n)).astype(np.float32)
    post = rng.uniform(0.5, 2, (L, n)).astype(np.float32)
    md = oc.Model(L=L, d=d, n_heads=1, head_dim=d, d_mlp=1, B=1, T=M, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                  n_streams=n, Hres=Hres, pre=np.ones((L, n), np.float32), post=post)
    old = rng.standard_normal((L + 1, M, n, d)).astype(np.float32)
    g = rng.standard_normal((L, M, d)).astype(np.float32)
    dev = torch.device("cuda:0")
    tr = torch.from_numpy(old).to(dev)
    probe = torch.zeros((2, L), dtype=torch.float32, device=dev)
    snlp.correction_scan_static(mode, tr, torch.from_numpy(g).to(dev), torch.from_numpy(Hres).to(dev) if n > 1 else None,
                                torch.from_numpy(post).to(dev) if n > 1 else None, probe)
    torch.cuda.synchronize()
    ref = oc.correction_scan(md, old[0], g, mode)
    assert np.array_equal(tr.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    gp = probe.cpu().numpy().astype(np.float64)
    assert np.allclose(gp[0], oc.residual_sq(md, old, g, mode), rtol=1e-5, atol=0)
    assert np.allclose(gp[1], np.sum((ref[1:].astype(np.float64) - old[1:].astype(np.float64)) ** 2, axis=(1, 2, 3)), rtol=1e-5, atol=0)


@pytest.mark.parametrize("n,bf16", [(1, True), (4, True), (2, False)])
def test_correction_leaves_next_rounds_normalised_inputs(gh, n, bf16):
    """Large batches: the correction kernel also writes the (pre-mixed and) normalised branch inputs of the next round.
    They must be the bits the stand-alone norm pass computes from the new trace, the rounds that use them must equal
    rounds that do not, and K = L must still be the sequential trace bit for bit."""
    import paper_2605_17842_amd as snlp
    shp = si.Shape("next_inputs", L=3, d=1280, n_heads=10, head_dim=128, d_mlp=1280, B=2, T=448, P=0, n_streams=n, bf16=bf16,
                   seed=210 + n)      # M d = 1.15M > 2^20: one token row per workgroup in the correction
    t = si.generate(shp)
    if n > 1:                         # distinct streams, so that the pre-mix matters
        t["h0"] = (t["h0"] + np.random.default_rng(3).standard_normal(t["h0"].shape).astype(np.float32)).astype(np.float32)
    mode = oc.HCN if n > 1 else oc.IDN
    m = gh.gpu_model(shp, t)
    m.h0 = torch.from_numpy(t["h0"]).to(m.device)
    m.init_trace(m.h0)
    m.iterate(mode, 1, None)
    torch.cuda.synchronize()
    left_x, left_u = m.stage_buffer("xhat"), (m.stage_buffer("u") if n > 1 else None)
    after1 = m.trace.clone()
    m.bind_trace(m.trace)                              # forget the cached inputs: the next evaluation recomputes them
    m.evaluate_branches()
    torch.cuda.synchronize()
    fresh_x, fresh_u = m.stage_buffer("xhat"), (m.stage_buffer("u") if n > 1 else None)
    per = shp.M * shp.d
    assert torch.equal(left_x.view(torch.int16 if bf16 else torch.int32)[per:], fresh_x.view(torch.int16 if bf16 else torch.int32)[per:])
    if n > 1:
        assert torch.equal(left_u.view(torch.int32)[per:], fresh_u.view(torch.int32)[per:])
    # two more rounds with and without the cached inputs
    m.iterate(mode, 2, None)
    a = m.trace.clone()
    m.trace.copy_(after1)
    m.bind_trace(m.trace)
    m.iterate(mode, 1, None)
    m.bind_trace(m.trace)
    m.iterate(mode, 1, None)
    torch.cuda.synchronize()
    assert torch.equal(a, m.trace)
    assert torch.equal(a, m.sequential_forward(mode, m.h0))          # L = 3 rounds in all
    md = oracle_model(shp, t, widen=True)
    ref, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), mode, 2)
    m.init_trace(m.h0)
    m.iterate(mode, 2, None)
    assert per_layer_rel_err(np_trace(m), ref).max() < (TOL_BF16 if bf16 else TOL_F32)
    m.close()


# ------------------------------------------------------------------ config 1: fp32 operand path

def test_config1_tiny_idn_fp32(gh):
    shp = si.config(1)
    t = si.generate(shp)
    worst = check_iterates(gh, shp, t, oc.IDN, [1, 2, 3, 4], TOL_F32)
    say("config1 worst %.3e" % worst)


def test_config1_gpu_invariants(gh):
    """On the GPU itself: after k rounds layers 1..k equal the GPU sequential trace bit for bit, K = L recovers
    it, converged layers have zero residual, and snlp_residual_norm agrees with the probe."""
    shp = si.config(1)
    t = si.generate(shp)
    m = gh.gpu_model(shp, t)
    seq = m.sequential_forward(0, m.h0).clone()
    m.init_trace(m.h0)
    probe = torch.zeros((shp.L, 2, shp.L), dtype=torch.float32, device=m.device)
    for k in range(1, shp.L + 1):
        m.iterate(0, 1, probe[k - 1:])
        torch.cuda.synchronize()
        assert torch.equal(m.trace[: k + 1], seq[: k + 1]), k
        rn = m.residual_norm(0)
        torch.cuda.synchronize()
        assert torch.all(rn[:k] == 0)
    assert torch.equal(m.trace, seq)
    pr = probe.cpu().numpy()
    for k in range(shp.L):
        assert np.all(pr[k, 0, :k] == 0) and np.all(pr[k, 1, :k] == 0) and np.all(pr[k, 0, k:] > 0)
    # residual_norm of the K = 1 trace equals sqrt of the probe row entering round 2
    m.init_trace(m.h0)
    m.iterate(0, 1)
    rn = m.residual_norm(0).cpu().numpy()
    assert np.allclose(rn, np.sqrt(pr[1, 0]), rtol=1e-5)
    m.close()


@pytest.mark.parametrize("P,T,B,n", [(0, 9, 2, 1), (13, 7, 2, 1), (5, 70, 1, 1), (11, 6, 2, 3)])
def test_fp32_path_ragged_shapes(gh, P, T, B, n):
    shp = si.Shape("f32_ragged", L=3, d=96, n_heads=3, head_dim=32, d_mlp=200, B=B, T=T, P=P, n_streams=n,
                   bf16=False, seed=50 + P + T)
    t = si.generate(shp)
    for k in ("Wqkv", "Wo", "Wfc", "Wproj"):
        t[k] = t[k] * np.float32(6.0)      # branch outputs comparable to the state
    mode = oc.HCN if n > 1 else oc.IDN
    check_iterates(gh, shp, t, mode, [1, 2, 3], TOL_F32)


# ------------------------------------------------------------------ bf16 MFMA path, small and ragged

@pytest.mark.parametrize("name,P,T,B,n,L", [
    ("block_T40", 0, 40, 2, 1, 3),          # one ragged query tile, no prefix
    ("block_T200_P37", 37, 200, 1, 1, 2),   # two query tiles, prefix not a multiple of the key tile
    ("decode_T5_P70", 70, 5, 3, 1, 3),      # decode kernel, ragged prefix
    ("decode_T1_P0", 0, 1, 2, 1, 2),        # softmax over a single key
    ("decode_T16_P2048", 2048, 16, 1, 1, 2),
    ("hcn_T33", 0, 33, 2, 4, 3),
    ("hcn_n2_T9_P20", 20, 9, 2, 2, 3),      # two and eight residual streams
    ("hcn_n8_T21", 0, 21, 1, 8, 2),
])
def test_bf16_path_small_shapes(gh, name, P, T, B, n, L):
    shp = si.Shape(name, L=L, d=256, n_heads=2, head_dim=128, d_mlp=512, B=B, T=T, P=P, n_streams=n, bf16=True,
                   seed=70 + P + T)
    t = si.generate(shp)
    mode = oc.HCN if n > 1 else oc.IDN
    check_iterates(gh, shp, t, mode, [1, 2, L], TOL_BF16)


@pytest.mark.parametrize("name,P,T,B,n,L", [
    ("graph_decode_T8_P600", 600, 8, 2, 1, 3),      # decode attention with its own rotation, skinny GEMMs, two-kernel scan
    ("graph_block_hcn_T40", 0, 40, 2, 4, 3),        # block attention, 128 x 128 GEMM tiles, 4 streams
    # M d > 2^20: the eager rounds after the first take their branch inputs from the previous correction, the
    # replayed round (captured after the initialisation) recomputes them -- the two must agree bit for bit
    ("graph_prefill_T2060", 0, 2060, 2, 1, 2),
])
def test_rounds_replayed_from_a_hip_graph_equal_eager_rounds(gh, name, P, T, B, n, L):
    """One round (evaluate + correct + probe) captured in a HIP graph and replayed L times, with eager work and
    synchronisations of the same context between the replays, gives the eager trace and probe bit for bit after every
    replay: the round enqueues kernels only (no allocation, no memset node), and a round captured directly after an
    initialisation recomputes every branch input, so it does not depend on what ran between the replays."""
    shp = si.Shape(name, L=L, d=256, n_heads=2, head_dim=128, d_mlp=512, B=B, T=T, P=P, n_streams=n, bf16=True, seed=77 + T)
    t = si.generate(shp)
    mode = oc.HCN if n > 1 else oc.IDN
    m = gh.gpu_model(shp, t)
    eager_tr, eager_pr = [], []
    m.init_trace(m.h0)
    for _ in range(L):
        pr = torch.zeros((1, 2, L), dtype=torch.float32, device=m.trace.device)
        m.iterate(mode, 1, pr)
        torch.cuda.synchronize()
        eager_tr.append(m.trace.clone()); eager_pr.append(pr.clone())
    probe = torch.zeros((1, 2, L), dtype=torch.float32, device=m.trace.device)
    cap = torch.cuda.Stream(device=m.trace.device)
    cap.wait_stream(torch.cuda.current_stream(m.trace.device))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(cap):
        m.init_trace(m.h0)
        m.iterate(mode, 1, probe)                 # warm-up on the capture stream
        cap.synchronize()
        m.init_trace(m.h0)
        cap.synchronize()
        with torch.cuda.graph(g, stream=cap):
            m.iterate(mode, 1, probe)
    torch.cuda.synchronize()
    scratch = torch.empty_like(m.trace)
    for k in range(L):
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(m.trace, eager_tr[k]), "%s: trace after replay %d differs from eager round %d" % (name, k + 1, k + 1)
        assert torch.equal(probe, eager_pr[k]), "%s: probe after replay %d differs" % (name, k + 1)
        # eager work of the same context between replays (its own output buffer; the bound trace is left alone)
        m.sequential_forward(mode, m.h0, scratch)
        torch.cuda.synchronize()
    assert torch.equal(scratch, eager_tr[L - 1])     # K = L rounds equal the sequential trace, and both paths still agree
    m.close()


def test_bf16_gpu_invariants_and_hcn_identity(gh):
    """K = L recovers the GPU sequential trace bit for bit (batch-invariant kernels); HCN with H = I equals
    IDN bit for bit on the same model."""
    shp = si.Shape("inv", L=4, d=256, n_heads=2, head_dim=128, d_mlp=512, B=2, T=24, P=40, n_streams=1, seed=91)
    t = si.generate(shp)
    m = gh.gpu_model(shp, t)
    seq = m.sequential_forward(0, m.h0).clone()
    m.init_trace(m.h0)
    for k in range(1, shp.L + 1):
        m.iterate(0, 1)
        torch.cuda.synchronize()
        assert torch.equal(m.trace[: k + 1], seq[: k + 1]), k
    m.close()
    shp = shp.with_(n_streams=4, P=0, T=48)
    t = si.generate(shp, identity_mixing=True)
    m = gh.gpu_model(shp, t)
    m.init_trace(m.h0)
    m.iterate(1, 2)
    a = m.trace.clone()
    m.init_trace(m.h0)
    m.iterate(0, 2)
    torch.cuda.synchronize()
    assert torch.equal(a, m.trace)
    assert torch.equal(m.sequential_forward(1, m.h0), m.sequential_forward(0, m.h0))
    m.close()


def test_error_paths(gh):
    import paper_2605_17842_amd as snlp
    with pytest.raises(snlp.SnlpError):
        snlp.Snlp(L=2, d=256, n_heads=2, head_dim=128, d_mlp=100, B=1, T=4, dtype=snlp.BF16)   # d_mlp % 64
    with pytest.raises(snlp.SnlpError):
        snlp.Snlp(L=2, d=128, n_heads=2, head_dim=64, d_mlp=128, B=1, T=4, dtype=snlp.BF16)    # head_dim != 128
    m = snlp.Snlp(L=2, d=64, n_heads=2, head_dim=32, d_mlp=64, B=1, T=4, dtype=snlp.F32)
    m.bind_trace()
    with pytest.raises(snlp.SnlpError):
        m.iterate(0, 1)                      # weights not bound
    with pytest.raises(snlp.SnlpError):
        m.correction_scan(1, torch.zeros((2, 4, 64), device="cuda"))   # HCN on a single-stream model
    m.close()


# ------------------------------------------------------------------ sequential prefix and one-shot-forward initialisation

@pytest.mark.parametrize("bf16,n,S,init", [(False, 1, 2, 0), (False, 1, 0, 1), (True, 1, 2, 1), (True, 4, 3, 0), (True, 4, 1, 1)])
def test_prefix_and_fwd_initialisation(gh, bf16, n, S, init):
    import paper_2605_17842_amd as snlp
    if bf16:
        shp = si.Shape("pre_bf16", L=5, d=256, n_heads=2, head_dim=128, d_mlp=512, B=2, T=20, P=24, n_streams=n, seed=120 + S)
        t = si.generate(shp)
        tol = TOL_BF16
    else:
        shp = si.Shape("pre_f32", L=5, d=96, n_heads=3, head_dim=32, d_mlp=200, B=2, T=9, P=5, n_streams=n, bf16=False, seed=130 + S)
        t = si.generate(shp)
        for k in ("Wqkv", "Wo", "Wfc", "Wproj"):
            t[k] = t[k] * np.float32(6.0)
        tol = TOL_F32
    mode = oc.HCN if n > 1 else oc.IDN
    say("%s n=%d S=%d init=%d" % (shp.name, n, S, init))
    md = oracle_model(shp, t, widen=True)
    m = gh.gpu_model(shp, t)
    m.set_prefix(S)
    m.init_trace_ex(mode, init, m.h0)
    ref0 = oc.init_trace(md, t["h0"], S=S, mode=mode, init=init)
    assert per_layer_rel_err(np_trace(m), ref0).max() < tol
    gseq = m.sequential_forward(mode, m.h0).clone()
    torch.cuda.synchronize()
    exact = S + (1 if init else 0)            # layers exact before the first round
    assert torch.equal(m.trace[: exact + 1], gseq[: exact + 1])
    K = 2
    probe = torch.zeros((K, 2, shp.L), dtype=torch.float32, device=m.device)
    m.iterate(mode, K, probe)
    ref, oprobe, _ = oc.iterate(md, ref0, mode, K, S=S)
    err = per_layer_rel_err(np_trace(m), ref)
    say("  K=%d max rel err %.3e" % (K, err.max()))
    assert err.max() < tol
    gp = probe.cpu().numpy().astype(np.float64)
    assert np.all(gp[:, :, :S] == 0.0)
    assert np.all(np.abs(np.sqrt(gp) - np.sqrt(oprobe)) <= 4 * tol * np.sqrt(oprobe.max()))
    rn = m.residual_norm(mode).cpu().numpy()
    assert np.all(rn[: min(exact + K, shp.L)] == 0.0)
    m.iterate(mode, shp.L - exact - K, None)          # finite termination from the shifted start
    torch.cuda.synchronize()
    assert torch.equal(m.trace, gseq)
    m.close()


# ------------------------------------------------------------------ diagonal surrogate with supplied diagonals

@pytest.mark.parametrize("L,M,d", [(5, 37, 132), (26, 64, 1664), (3, 300, 128),
                                   (12, 2048, 768), (26, 4096, 1664)])   # the last two: prefill sizes, every block full
def test_diag_correction_scan_bit_exact(gh, L, M, d):
    import paper_2605_17842_amd as snlp
    rng = np.random.default_rng(300 + L)
    hd = d if d <= 256 and d % 2 == 0 else 4
    m = snlp.Snlp(L=L, d=d, n_heads=d // hd, head_dim=hd, d_mlp=64, B=1, T=M, dtype=snlp.F32)
    old = rng.standard_normal((L + 1, M, 1, d)).astype(np.float32)
    g = rng.standard_normal((L, M, d)).astype(np.float32)
    a = rng.uniform(-1, 1.5, (L, M, d)).astype(np.float32)
    tr = m.bind_trace()
    tr.copy_(torch.from_numpy(old))
    probe = torch.zeros((2, L), dtype=torch.float32, device=tr.device)
    m.correction_scan_diag(torch.from_numpy(g).to(tr.device), torch.from_numpy(a).to(tr.device), probe)
    torch.cuda.synchronize()
    ref = oc.correction_scan_diag(old, g, a)
    assert np.array_equal(tr.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    md = oc.Model(L=L, d=d, n_heads=1, head_dim=d, d_mlp=1, B=1, T=M, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[])
    gp = probe.cpu().numpy().astype(np.float64)
    assert np.allclose(gp[0], oc.residual_sq(md, old, g, oc.IDN), rtol=1e-5)
    assert np.allclose(gp[1], np.sum((ref[1:].astype(np.float64) - old[1:].astype(np.float64)) ** 2, axis=(1, 2, 3)), rtol=1e-5)
    tr.copy_(torch.from_numpy(old))
    m.correction_scan_diag(torch.from_numpy(g).to(tr.device), torch.from_numpy(a).to(tr.device), None)
    torch.cuda.synchronize()
    assert np.array_equal(tr.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    m.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_iterate_diag_against_oracle_and_termination(gh, bf16):
    if bf16:
        shp = si.Shape("diag_bf16", L=4, d=256, n_heads=2, head_dim=128, d_mlp=512, B=2, T=12, P=20, seed=140)
        t, tol = si.generate(shp), TOL_BF16
    else:
        shp = si.Shape("diag_f32", L=4, d=96, n_heads=3, head_dim=32, d_mlp=200, B=2, T=9, P=5, bf16=False, seed=141)
        t, tol = si.generate(shp), TOL_F32
        for k in ("Wqkv", "Wo", "Wfc", "Wproj"):
            t[k] = t[k] * np.float32(6.0)
    rng = np.random.default_rng(7)
    diag = rng.uniform(0.5, 1.2, (shp.L, shp.M, shp.d)).astype(np.float32)
    md = oracle_model(shp, t, widen=True)
    m = gh.gpu_model(shp, t)
    dg = torch.from_numpy(diag).to(m.device)
    m.init_trace(m.h0)
    probe = torch.zeros((2, 2, shp.L), dtype=torch.float32, device=m.device)
    m.iterate_diag(2, dg, probe)
    ref, oprobe = oc.iterate_diag(md, oc.init_trace(md, t["h0"]), diag, 2)
    err = per_layer_rel_err(np_trace(m), ref)
    say("%s iterate_diag K=2 max rel err %.3e" % (shp.name, err.max()))
    assert err.max() < tol
    gp = probe.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(np.sqrt(gp) - np.sqrt(oprobe)) <= 4 * tol * np.sqrt(oprobe.max()))
    gseq = m.sequential_forward(0, m.h0).clone()
    m.iterate_diag(shp.L - 2, dg, None)
    torch.cuda.synchronize()
    assert torch.equal(m.trace, gseq)          # any diagonals: K = L recovers the sequential trace bit for bit
    m.close()


# ------------------------------------------------------------------ chunkwise fused layers N x F

@pytest.mark.parametrize("bf16,L,F,P,T,B", [(False, 6, 2, 5, 9, 2), (False, 6, 6, 0, 12, 1), (True, 6, 3, 24, 6, 2),
                                            (True, 4, 2, 0, 150, 1), (True, 4, 4, 40, 8, 2)])
def test_fused_chunks(gh, bf16, L, F, P, T, B):
    if bf16:
        shp = si.Shape("fused_bf16", L=L, d=256, n_heads=2, head_dim=128, d_mlp=512, B=B, T=T, P=P, seed=150 + F)
        t, tol = si.generate(shp), TOL_BF16
    else:
        shp = si.Shape("fused_f32", L=L, d=96, n_heads=3, head_dim=32, d_mlp=200, B=B, T=T, P=P, bf16=False, seed=160 + F)
        t, tol = si.generate(shp), TOL_F32
        for k in ("Wqkv", "Wo", "Wfc", "Wproj"):
            t[k] = t[k] * np.float32(6.0)
    N = L // F
    say("%s %dxF%d" % (shp.name, N, F))
    md = oracle_model(shp, t, widen=True)
    m = gh.gpu_model(shp, t)
    m.set_fusion(F)
    m.bind_trace()
    assert tuple(m.trace.shape) == (N + 1, shp.M, 1, shp.d)
    seq = oc.fused_sequential_forward(md, t["h0"], F)
    gseq = m.sequential_forward(0, m.h0).clone()
    torch.cuda.synchronize()
    err = per_layer_rel_err(gseq.cpu().numpy(), seq)
    say("  fused sequential max rel err %.3e" % err.max())
    assert err.max() < tol
    m.init_trace(m.h0)
    K = min(2, N)
    probe = torch.zeros((K, 2, N), dtype=torch.float32, device=m.device)
    m.iterate(0, K, probe)
    tr0 = np.ascontiguousarray(np.broadcast_to(t["h0"], (N + 1,) + t["h0"].shape)).copy()
    ref, oprobe, _ = oc.fused_iterate(md, tr0, F, K)
    err = per_layer_rel_err(np_trace(m), ref)
    say("  fused K=%d max rel err %.3e" % (K, err.max()))
    assert err.max() < tol
    gp = probe.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(np.sqrt(gp) - np.sqrt(oprobe)) <= 4 * tol * np.sqrt(oprobe.max()))
    m.iterate(0, N - K, None)
    torch.cuda.synchronize()
    assert torch.equal(m.trace, gseq)            # K = N recovers the fused sequential trace bit for bit
    # F = 1 is the plain model, bit for bit
    m.set_fusion(1)
    m.bind_trace()
    plain = m.sequential_forward(0, m.h0).clone()
    m.init_trace(m.h0)
    m.iterate(0, 2, None)
    a = m.trace.clone()
    m2 = gh.gpu_model(shp, t)
    m2.init_trace(m2.h0)
    m2.iterate(0, 2, None)
    torch.cuda.synchronize()
    assert torch.equal(a, m2.trace) and torch.equal(plain, m2.sequential_forward(0, m2.h0))
    m.close(); m2.close()


# ------------------------------------------------------------------ degenerate cases and determinism

def test_degenerate_cases_and_determinism(gh):
    # L = 1: one round is the sequential forward; K = 0 is a no-op; calls compose; two runs are bit-identical
    shp = si.Shape("L1", L=1, d=256, n_heads=2, head_dim=128, d_mlp=512, B=1, T=3, P=0, seed=170)
    t = si.generate(shp)
    m = gh.gpu_model(shp, t)
    m.init_trace(m.h0)
    before = m.trace.clone()
    m.iterate(0, 0, None)
    torch.cuda.synchronize()
    assert torch.equal(m.trace, before)
    m.iterate(0, 1, None)
    assert torch.equal(m.trace, m.sequential_forward(0, m.h0))
    m.close()

    shp = si.Shape("det", L=5, d=256, n_heads=2, head_dim=128, d_mlp=512, B=3, T=7, P=45, seed=171)
    t = si.generate(shp)
    m = gh.gpu_model(shp, t)
    probe = torch.zeros((3, 2, shp.L), dtype=torch.float32, device=m.device)
    m.init_trace(m.h0)
    m.iterate(0, 3, probe)
    a, pa = m.trace.clone(), probe.clone()
    m.init_trace(m.h0)
    probe.zero_()
    m.iterate(0, 1, probe)
    m.iterate(0, 2, probe[1:])
    torch.cuda.synchronize()
    assert torch.equal(a, m.trace) and torch.equal(pa, probe)        # iterate(1) + iterate(2) == iterate(3), bit for bit
    m2 = gh.gpu_model(shp, t)                                         # a second context, fresh workspace
    m2.init_trace(m2.h0)
    m2.iterate(0, 3, None)
    torch.cuda.synchronize()
    assert torch.equal(a, m2.trace)
    m.close(); m2.close()


@pytest.mark.gpu
@pytest.mark.parametrize("n,S,init", [(1, 0, 0), (1, 2, 1), (3, 0, 0), (3, 1, 1)])
def test_leaving_converged_layers_out(gh, n, S, init):
    """Rounds restricted to the layers that can still change: bit-identical trace and probes to full rounds, within
    tolerance of the oracle's restricted rounds, and every call that could invalidate the count of exact layers
    resets it."""
    import paper_2605_17842_amd as snlp
    shp = si.Shape("skip", L=6, d=256, n_heads=2, head_dim=128, d_mlp=512, B=2, T=11, P=19, n_streams=n, seed=180 + n + S)
    t = si.generate(shp)
    mode = oc.HCN if n > 1 else oc.IDN
    say("skip converged n=%d S=%d init=%d" % (n, S, init))
    md = oracle_model(shp, t, widen=True)
    m = gh.gpu_model(shp, t)
    m.set_prefix(S)
    K = shp.L
    pf = torch.zeros((K, 2, shp.L), dtype=torch.float32, device=m.device)
    ps = torch.full((K, 2, shp.L), -1.0, dtype=torch.float32, device=m.device)
    m.init_trace_ex(mode, init, m.h0)
    m.iterate(mode, K, pf)
    full = m.trace.clone()
    m.set_skip_converged(True)
    m.init_trace_ex(mode, init, m.h0)
    m.iterate(mode, 2, ps)
    m.iterate(mode, K - 2, ps[2:])                       # the count carries over between calls
    torch.cuda.synchronize()
    assert torch.equal(full, m.trace) and torch.equal(pf, ps)
    ref0 = oc.init_trace(md, t["h0"], S=S, mode=mode, init=init)
    ref, oprobe = oc.iterate_skipping_converged(md, ref0, mode, K, S=S, exact=S + init)
    assert per_layer_rel_err(np_trace(m), ref).max() < TOL_BF16
    gp = ps.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(np.sqrt(gp) - np.sqrt(oprobe)) <= 4 * TOL_BF16 * np.sqrt(oprobe.max()))

    # a new h0 through init_trace resets the count; so does rebinding the trace (nothing is then left out)
    h1 = (m.h0 * 0.5).contiguous()
    m.init_trace_ex(mode, init, h1)
    m.iterate(mode, 2, None)
    a = m.trace.clone()
    m.set_skip_converged(False)
    m.init_trace_ex(mode, init, h1)
    m.iterate(mode, 2, None)
    torch.cuda.synchronize()
    assert torch.equal(a, m.trace)
    m.set_skip_converged(True)
    m.init_trace_ex(mode, init, h1)
    m.iterate(mode, 1, None)
    m.trace[S + 1].mul_(1.25)                            # the caller edits an "exact" slot, then says so by rebinding
    edited = m.trace.clone()
    m.bind_trace(m.trace)
    m.iterate(mode, 1, None)
    b = m.trace.clone()
    m.set_skip_converged(False)
    m.trace.copy_(edited)
    m.bind_trace(m.trace)                                # the caller wrote into the bound trace: bind it again
    m.iterate(mode, 1, None)
    torch.cuda.synchronize()
    assert torch.equal(b, m.trace)
    if n > 1:                                            # a round in the other mode on an n-stream model resets too
        m.set_skip_converged(True)
        m.init_trace_ex(oc.HCN, 0, m.h0)
        m.iterate(oc.HCN, 2, None)
        m.iterate(oc.IDN, 1, None)
        c1 = m.trace.clone()
        m.set_skip_converged(False)
        m.init_trace_ex(oc.HCN, 0, m.h0)
        m.iterate(oc.HCN, 2, None)
        m.iterate(oc.IDN, 1, None)
        torch.cuda.synchronize()
        assert torch.equal(c1, m.trace)
    m.close()


@pytest.mark.gpu
def test_leaving_converged_layers_out_diag_and_fused(gh):
    shp = si.Shape("skipd", L=6, d=256, n_heads=2, head_dim=128, d_mlp=512, B=2, T=9, P=13, seed=190)
    t = si.generate(shp)
    m = gh.gpu_model(shp, t)
    rng = np.random.default_rng(5)
    diag = torch.from_numpy(rng.uniform(0.2, 1.1, size=(shp.L, shp.M, shp.d)).astype(np.float32)).to(m.device)
    pf = torch.zeros((4, 2, shp.L), dtype=torch.float32, device=m.device)
    ps = torch.full_like(pf, -1.0)
    m.init_trace(m.h0)
    m.iterate_diag(4, diag, pf)
    full = m.trace.clone()
    m.set_skip_converged(True)
    m.init_trace(m.h0)
    m.iterate_diag(4, diag, ps)
    torch.cuda.synchronize()
    assert torch.equal(full, m.trace) and torch.equal(pf, ps)
    m.close()

    m = gh.gpu_model(shp, t)                             # fused chunks: units are chunks
    m.set_fusion(2)
    m.bind_trace()
    tr = m.trace
    m.init_trace(m.h0)
    m.iterate(0, 3, None)
    full = tr.clone()
    m.set_skip_converged(True)
    m.init_trace(m.h0)
    m.iterate(0, 3, None)
    torch.cuda.synchronize()
    assert torch.equal(full, tr)
    m.close()


@pytest.mark.gpu
@pytest.mark.parametrize("name,d,F,B", [
    ("wide_tn3", 512, 1408, 16),      # 50 layers: QKV (N = 1536) and FC (N = 1408, ragged last tile) take 3 column blocks per wave
    ("wide_tn2_tn4", 384, 1920, 16),  # QKV (N = 1152, ragged) takes 2, FC (N = 1920, ragged) takes the 512-column tile
    ("wide_tn3_m56", 512, 1408, 7),   # 56 rows: two row blocks per wave, the second ragged
])
def test_decode_gemm_wide_column_tiles(gh, name, d, F, B):
    """Decode-shaped GEMMs pick their column-tile width from the launch size.  A deep, narrow model makes the
    batched launches take the wide tiles while the one-layer launches of the sequential path take the narrow
    one: parity with the oracle, and K = L must still equal the sequential trace bit for bit."""
    shp = si.Shape(name, L=50, d=d, n_heads=d // 128, head_dim=128, d_mlp=F, B=B, T=8, P=40, seed=200 + d + B)
    t = si.generate(shp)
    say("%s L=50 d=%d F=%d M=%d" % (name, d, F, shp.M))
    md = oracle_model(shp, t, widen=True)
    m = gh.gpu_model(shp, t)
    m.init_trace(m.h0)
    m.iterate(0, 2, None)
    ref, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), oc.IDN, 2)
    err = per_layer_rel_err(np_trace(m), ref)
    say("  K=2 max rel err %.3e" % err.max())
    assert err.max() < TOL_BF16
    seq = m.sequential_forward(0, m.h0).clone()
    m.set_skip_converged(True)            # rounds of shrinking size cross the tile-width thresholds on the way
    m.init_trace(m.h0)
    m.iterate(0, shp.L, None)
    torch.cuda.synchronize()
    assert torch.equal(m.trace, seq)
    m.close()


@pytest.mark.gpu
def test_prefill_gemm_tail_pieces_equal_whole_tiles(gh):
    """Prefill GEMM launches cut the last, incomplete round of 256 x 256 tiles into smaller pieces, by the launch
    size.  On a deep, narrow model with ragged rows and columns (600 rows; widths of 2.5, 7.5 and 5.25 tiles), K = L
    rounds that leave converged layers out run launches of 34, 33, ... 1 layers, whose remainders pass through every
    piece shape and the plain form; the one-layer launches of the sequential path use other tile shapes again.  Every
    output element is the same k-ordered sum in all of them, so the two traces must agree bit for bit (parity of the
    pieces with the oracle: the stage test on the same shape)."""
    shp = si.Shape("gemm_tail_L34", L=34, d=640, n_heads=5, head_dim=128, d_mlp=1344, B=3, T=200, P=0, seed=941)
    t = si.generate(shp)
    say("gemm_tail_L34 M=%d" % shp.M)
    m = gh.gpu_model(shp, t)
    seq = m.sequential_forward(0, m.h0).clone()
    m.set_skip_converged(True)
    m.init_trace(m.h0)
    m.iterate(0, shp.L, None)
    torch.cuda.synchronize()
    assert torch.equal(m.trace, seq)
    m.close()
