"""Pins of the CPU oracle: what the paper and the mathematics fix, checked without any GPU.

Each test names the statement it pins.  Paper locations: Eq. (1)-(2) residual formulation,
Eq. (4)-(5) SNLP evaluation and update, Eq. (6)-(7) IDN, Eq. (8) HCN, Alg. 1-2 (Appendix
"Algorithm"), Appendix "Variance Reduction Derivation" (one-step closed form), Appendix
"Connection to Hyper-Connections and mHC".
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import snlp_inputs as si
from oracle import snlp_oracle as oc
from oracle.harness import oracle_model, rel_err

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small(n_streams=1, bf16=False, P=0, L=4, T=6, B=2, seed=7, identity=False, d=32, H=2, dh=16, Fm=64):
    shp = si.Shape("small", L=L, d=d, n_heads=H, head_dim=dh, d_mlp=Fm, B=B, T=T, P=P,
                   n_streams=n_streams, bf16=bf16, seed=seed)
    t = si.generate(shp, identity_mixing=identity)
    # N(0, 0.02) weights make branches tiny next to h_0 ~ N(0,1); scale them up so that every
    # invariant below is exercised with branch outputs of the same order as the state.
    if not bf16:
        for k in ("Wqkv", "Wo", "Wfc", "Wproj"):
            t[k] = t[k] * np.float32(8.0)
    return shp, t, oracle_model(shp, t)


def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split(":")
            vals[k.strip()] = np.array([float(x) for x in v.split()], dtype=np.float32)
    return vals


# ---------------------------------------------------------------- hand-worked fixtures

def test_golden_hcn_scan_matches_hand_computation():
    g = read_golden("hcn_scan_small.txt")
    md = oc.Model(L=2, d=1, n_heads=1, head_dim=1, d_mlp=1, B=1, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                  n_streams=2, Hres=np.stack([g["H1"].reshape(2, 2), g["H2"].reshape(2, 2)]),
                  pre=np.ones((2, 2), np.float32), post=np.stack([g["p1"], g["p2"]]))
    X0 = g["X0"].reshape(1, 2, 1)
    tr = oc.correction_scan(md, X0, g["g"].reshape(2, 1, 1), oc.HCN)
    assert np.array_equal(tr[1].ravel(), g["expect_X1"])
    assert np.array_equal(tr[2].ravel(), g["expect_X2"])


def _stub_branch(model, l, u):
    """F(u) = a + m with a = 2 u, m = 0.5 * reverse_channels(u + a) (the stub of hc_sublayer_premix_small.txt)."""
    u = np.asarray(u, dtype=np.float64)
    a = 2.0 * u
    return a, 0.5 * (u + a)[:, ::-1]


def _hc_sublayer_fixture_holds(mod) -> bool:
    """The hand-worked two-layer hyper-connection fixture through mod.premix and mod.sequential_forward, the
    branch replaced by the fixture's stub."""
    g = read_golden("hc_sublayer_premix_small.txt")
    md = mod.Model(L=2, d=2, n_heads=1, head_dim=2, d_mlp=1, B=1, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                   n_streams=2, Hres=np.stack([g["H1"].reshape(2, 2), g["H2"].reshape(2, 2)]),
                   pre=np.stack([g["pre1"], g["pre2"]]), post=np.stack([g["post1"], g["post2"]]))
    X0 = g["X0"].reshape(1, 2, 2)
    real = mod.branch
    mod.branch = _stub_branch
    try:
        tr = mod.sequential_forward(md, X0, mod.HCN)
        u1 = mod.premix(md, 1, tr[0])
        u2 = mod.premix(md, 2, tr[1])
    finally:
        mod.branch = real
    return (np.array_equal(u1.ravel(), g["expect_u1"]) and np.array_equal(u2.ravel(), g["expect_u2"])
            and np.array_equal(tr[1].ravel(), g["expect_X1"]) and np.array_equal(tr[2].ravel(), g["expect_X2"]))


def test_golden_hc_sublayer_with_premix_matches_hand_computation():
    assert _hc_sublayer_fixture_holds(oc)


def test_premix_one_hot_selects_a_stream_and_matches_scalar_loop():
    """u = sum_j pre[j] X[:, j]: a one-hot pre returns that stream exactly; a general pre equals the scalar loop."""
    rng = np.random.default_rng(5)
    L, n, M, d = 3, 4, 5, 6
    X = rng.standard_normal((M, n, d)).astype(np.float32)              # distinct streams
    for j in range(n):
        pre = np.zeros((L, n), np.float32)
        pre[:, j] = 1.0
        md = oc.Model(L=L, d=d, n_heads=1, head_dim=d, d_mlp=1, B=M, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                      n_streams=n, Hres=None, pre=pre, post=np.ones((L, n), np.float32))
        assert np.array_equal(oc.premix(md, 2, X), X[:, j, :].astype(np.float64))
    pre = rng.uniform(-1, 1, (L, n)).astype(np.float32)
    md = oc.Model(L=L, d=d, n_heads=1, head_dim=d, d_mlp=1, B=M, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                  n_streams=n, Hres=None, pre=pre, post=rng.uniform(-1, 1, (L, n)).astype(np.float32))
    for l in (1, 3):
        u = oc.premix(md, l, X)
        for m in range(M):
            for c in range(d):
                want = sum(float(pre[l - 1, j]) * float(X[m, j, c]) for j in range(n))
                assert abs(u[m, c] - want) < 1e-12
    # single-stream models: the branch input is the state itself
    md1 = oc.Model(L=1, d=d, n_heads=1, head_dim=d, d_mlp=1, B=M, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[])
    assert np.array_equal(oc.premix(md1, 1, X[:, :1, :]), X[:, 0, :].astype(np.float64))


def test_golden_idn_prefix_matches_hand_computation():
    g = read_golden("idn_prefix_small.txt")
    md = oc.Model(L=3, d=1, n_heads=1, head_dim=1, d_mlp=1, B=1, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[])
    tr = oc.correction_scan(md, g["h0"].reshape(1, 1, 1), g["g"].reshape(3, 1, 1), oc.IDN)
    assert np.array_equal(tr[1:].ravel(), g["expect"])


# ---------------------------------------------------------------- branch pieces vs library routines / closed forms

def test_rmsnorm_matches_torch_and_closed_form():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 48))
    ref = F.rms_norm(torch.from_numpy(x), (48,), eps=1e-6).numpy()
    assert np.allclose(oc.rmsnorm(x, 1e-6), ref, rtol=1e-12, atol=1e-14)
    c = np.full((1, 10), -3.0)
    assert np.allclose(oc.rmsnorm(c, 1e-6), -1.0 / np.sqrt(1.0 + 1e-6 / 9.0))


def test_rope_is_complex_rotation_with_half_split_pairs():
    rng = np.random.default_rng(1)
    dh, T, base = 16, 9, 1.0e4
    x = rng.standard_normal((2, 3, T, dh))
    pos = 5 + np.arange(T)
    cos, sin = oc.rope_cos_sin(pos, dh, base)
    y = oc.apply_rope(x, cos, sin)
    # independent statement: pair (c, c+dh/2) is the complex number x_c + i x_{c+dh/2}, multiplied by
    # exp(i p theta_c), theta_c = base^(-2c/dh)
    z = torch.complex(torch.from_numpy(x[..., : dh // 2]), torch.from_numpy(x[..., dh // 2:]))
    theta = torch.tensor([base ** (-2.0 * c / dh) for c in range(dh // 2)], dtype=torch.float64)
    rot = torch.polar(torch.ones(T, dh // 2, dtype=torch.float64), torch.from_numpy(pos.astype(np.float64))[:, None] * theta)
    zr = z * rot
    ref = torch.cat([zr.real, zr.imag], dim=-1).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-13)
    # position 0 is the identity; rotations keep each head vector's norm
    c0, s0 = oc.rope_cos_sin(np.array([0]), dh, base)
    assert np.array_equal(oc.apply_rope(x[..., :1, :], c0, s0), x[..., :1, :])
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(2)
    dh = 32
    q = rng.standard_normal((1, dh))
    k = rng.standard_normal((1, dh))

    def score(pq, pk):
        cq, sq = oc.rope_cos_sin(np.array([pq]), dh, 1e4)
        ck, sk = oc.rope_cos_sin(np.array([pk]), dh, 1e4)
        return float((oc.apply_rope(q, cq, sq) @ oc.apply_rope(k, ck, sk).T)[0, 0])

    assert abs(score(7, 3) - score(104, 100)) < 1e-10
    assert abs(score(7, 3) - score(3, 7)) > 1e-3       # a sign error in the rotation would make these equal


@pytest.mark.parametrize("P", [0, 5])
def test_attention_matches_torch_sdpa_with_explicit_mask(P):
    rng = np.random.default_rng(3)
    B, H, T, dh = 2, 3, 7, 16
    q, k, v = (rng.standard_normal((B, H, T, dh)) for _ in range(3))
    kp = rng.standard_normal((B, H, P, dh)) if P else None
    vp = rng.standard_normal((B, H, P, dh)) if P else None
    out = oc.attention(q, k, v, kp, vp)
    keys = np.concatenate([kp, k], axis=2) if P else k
    vals = np.concatenate([vp, v], axis=2) if P else v
    mask = torch.ones(T, P + T, dtype=torch.bool)
    mask[:, P:] = torch.tril(torch.ones(T, T, dtype=torch.bool))
    ref = F.scaled_dot_product_attention(torch.from_numpy(q), torch.from_numpy(keys), torch.from_numpy(vals),
                                         attn_mask=mask).numpy()
    assert np.allclose(out, ref, rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(4)
    # T = 1, no prefix: softmax over one key, output is v
    q, k, v = (rng.standard_normal((1, 2, 1, 8)) for _ in range(3))
    assert np.allclose(oc.attention(q, k, v, None, None), v)
    # equal keys: uniform softmax, output = running mean of the visible values
    T = 5
    k = np.broadcast_to(rng.standard_normal((1, 1, 1, 8)), (1, 1, T, 8)).copy()
    q, v = rng.standard_normal((1, 1, T, 8)), rng.standard_normal((1, 1, T, 8))
    out = oc.attention(q, k, v, None, None)
    means = np.cumsum(v[0, 0], axis=0) / np.arange(1, T + 1)[:, None]
    assert np.allclose(out[0, 0], means)


def test_branch_matches_torch_library_composition():
    shp, t, md = small(P=5)
    rng = np.random.default_rng(5)
    u = rng.standard_normal((shp.M, shp.d))
    a, m = oc.branch(md, 2, u)
    # the same layer assembled from torch's library routines in fp64
    B, T, H, dh, d, P = shp.B, shp.T, shp.n_heads, shp.head_dim, shp.d, shp.P
    W = {k: torch.from_numpy(t[k][1].astype(np.float64)) for k in ("Wqkv", "Wo", "Wfc", "Wproj")}
    ut = torch.from_numpy(u)
    x = F.rms_norm(ut, (d,), eps=shp.rms_eps)
    q, k, v = (x @ W["Wqkv"]).view(B, T, 3 * d).split(d, dim=-1)
    q, k, v = (z.reshape(B, T, H, dh).transpose(1, 2) for z in (q, k, v))
    theta = shp.rope_base ** (-2.0 * torch.arange(dh // 2, dtype=torch.float64) / dh)
    rot = torch.polar(torch.ones(T, dh // 2, dtype=torch.float64),
                      (P + torch.arange(T, dtype=torch.float64))[:, None] * theta)

    def rope(z):
        zc = torch.complex(z[..., : dh // 2], z[..., dh // 2:]) * rot
        return torch.cat([zc.real, zc.imag], dim=-1)

    q = F.rms_norm(rope(q), (dh,), eps=shp.rms_eps)
    k = F.rms_norm(rope(k), (dh,), eps=shp.rms_eps)
    kp = torch.from_numpy(si.as_float(t["Kpre"][1]).astype(np.float64))
    vp = torch.from_numpy(si.as_float(t["Vpre"][1]).astype(np.float64))
    mask = torch.ones(T, P + T, dtype=torch.bool)
    mask[:, P:] = torch.tril(torch.ones(T, T, dtype=torch.bool))
    o = F.scaled_dot_product_attention(q, torch.cat([kp, k], 2), torch.cat([vp, v], 2), attn_mask=mask)
    a_ref = o.transpose(1, 2).reshape(B * T, d) @ W["Wo"]
    x2 = F.rms_norm(ut + a_ref, (d,), eps=shp.rms_eps)
    m_ref = torch.relu(x2 @ W["Wfc"]).square() @ W["Wproj"]
    assert rel_err(a, a_ref.numpy()) < 1e-12
    assert rel_err(m, m_ref.numpy()) < 1e-12
    assert np.linalg.norm(a) > 1e-3 and np.linalg.norm(m) > 1e-3


def test_mlp_with_nonpositive_preactivations_is_zero():
    shp, t, md = small()
    md.Wfc = [-np.abs(w) for w in md.Wfc]
    u = np.abs(np.random.default_rng(6).standard_normal((shp.M, shp.d))) + 0.1
    md.Wo = [np.zeros_like(w) for w in md.Wo]          # a = 0, so norm(u + a) stays positive
    a, m = oc.branch(md, 1, u)
    assert np.all(a == 0) and np.all(m == 0)


def test_causality_and_prefix_visibility():
    shp, t, md = small(P=4, B=1, T=6)
    rng = np.random.default_rng(8)
    u = rng.standard_normal((shp.M, shp.d))
    a0, m0 = oc.branch(md, 1, u)
    u2 = u.copy()
    u2[4] += 1.0                                         # change block token 4
    a1, m1 = oc.branch(md, 1, u2)
    assert np.array_equal(a0[:4], a1[:4]) and np.array_equal(m0[:4], m1[:4])
    assert not np.allclose(a0[4:], a1[4:])
    md.Kpre[0] = md.Kpre[0].copy()
    md.Kpre[0][0, :, 2, :] += 0.5                        # change one prefix row: every token sees it
    a2, _ = oc.branch(md, 1, u)
    assert all(not np.allclose(a0[i], a2[i]) for i in range(shp.T))


# ---------------------------------------------------------------- invariants of the iteration

@pytest.mark.parametrize("n,mode", [(1, oc.IDN), (3, oc.HCN), (3, oc.IDN)])
def test_finite_termination_and_prefix_stability_bitwise(n, mode):
    """After k rounds layers 1..k equal the sequential trace (bitwise: same fp32 operations on the same
    inputs); K = L recovers it; residuals of those layers are exactly zero."""
    shp, t, md = small(n_streams=n, P=3)
    seq = oc.sequential_forward(md, t["h0"], mode)
    tr = oc.init_trace(md, t["h0"])
    final, probe, kept = oc.iterate(md, tr, mode, shp.L, keep=True)
    for k, trk in enumerate(kept, start=1):
        assert np.array_equal(trk[: k + 1], seq[: k + 1])
        if k < shp.L:
            assert not np.array_equal(trk[k + 1], seq[k + 1])
    assert np.array_equal(final, seq)
    for k in range(shp.L):
        assert np.all(probe[k, 0, :k] == 0.0)            # converged layers have zero residual
        assert np.all(probe[k, 0, k:] > 0.0)
        assert np.all(probe[k, 1, :k] == 0.0)            # and do not move any more
    assert np.all(oc.residual_norm(md, seq, mode) == 0.0)   # G(h) = 0 <=> sequential trace
    assert np.all(oc.residual_norm(md, kept[0], mode)[1:] > 0.0)


def test_initial_residual_is_branch_norm_at_h0():
    shp, t, md = small()
    tr = oc.init_trace(md, t["h0"])
    r = oc.residual_norm(md, tr)
    for l in range(1, shp.L + 1):
        a, m = oc.branch(md, l, t["h0"][:, 0, :])
        assert abs(r[l - 1] - np.linalg.norm(a + m)) < 1e-5 * np.linalg.norm(a + m)


def test_one_step_idn_closed_form():
    """K = 1 from the h0 initialisation: h_L = h_0 + sum_l g_l(h_0)."""
    shp, t, md = small(P=2)
    tr, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), oc.IDN, 1)
    u = t["h0"][:, 0, :].astype(np.float64)
    total = u.copy()
    for l in range(1, shp.L + 1):
        a, m = oc.branch(md, l, u)
        total = total + a + m
    assert rel_err(tr[shp.L][:, 0, :], total) < 1e-6
    assert rel_err(tr[shp.L][:, 0, :], u) > 1e-2


@pytest.mark.parametrize("n,mode", [(1, oc.IDN), (4, oc.HCN)])
def test_prefix_form_equals_literal_update(n, mode):
    """The affine/prefix form used by the oracle and the literal Eq. (5) update agree to rounding."""
    shp, t, md = small(n_streams=n)
    tr0 = oc.init_trace(md, t["h0"])
    for K in (1, 2, 3):
        pf, _, _ = oc.iterate(md, tr0, mode, K)
        df = oc.iterate_delta_form(md, tr0, mode, K)
        assert rel_err(pf, df) < 2e-6


@pytest.mark.parametrize("n,mode", [(1, oc.IDN), (4, oc.HCN)])
def test_update_is_scan_of_residuals(n, mode):
    """Newton on the block lower-bidiagonal system: delta_l = -G_l + A_l delta_{l-1}."""
    shp, t, md = small(n_streams=n)
    tr1, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), mode, 1)
    tr2, _, _ = oc.iterate(md, tr1, mode, 1)
    delta = tr2.astype(np.float64) - tr1.astype(np.float64)
    prev = np.zeros_like(delta[0])
    for l in range(1, shp.L + 1):
        G = tr1[l].astype(np.float64) - oc.full_layer(md, l, tr1[l - 1], mode)
        A = np.eye(n) if mode == oc.IDN else md.Hres[l - 1].astype(np.float64)
        prev = -G + np.einsum("ij,mjc->mic", A, prev)
        assert np.linalg.norm(delta[l] - prev) < 1e-5 * max(np.linalg.norm(tr1[l]), 1.0)


def test_hcn_with_identity_mixing_equals_idn_bitwise():
    shp, t, md = small(n_streams=4, identity=True)
    assert np.array_equal(md.Hres[0], np.eye(4, dtype=np.float32))
    tr0 = oc.init_trace(md, t["h0"])
    for K in (1, 2, shp.L):
        a, pa, _ = oc.iterate(md, tr0, oc.HCN, K)
        b, pb, _ = oc.iterate(md, tr0, oc.IDN, K)
        assert np.array_equal(a, b)
        assert np.array_equal(pa, pb)
    assert np.array_equal(oc.sequential_forward(md, t["h0"], oc.HCN), oc.sequential_forward(md, t["h0"], oc.IDN))


def test_hcn_scan_against_python_unroll_and_affine_composition():
    rng = np.random.default_rng(11)
    L, n, M, d = 4, 3, 2, 5
    Hres = rng.uniform(0.0, 1.0, (L, n, n)).astype(np.float32)
    post = rng.uniform(0.5, 2.0, (L, n)).astype(np.float32)
    md = oc.Model(L=L, d=d, n_heads=1, head_dim=d, d_mlp=1, B=M, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                  n_streams=n, Hres=Hres, pre=np.ones((L, n), np.float32), post=post)
    X0 = rng.standard_normal((M, n, d)).astype(np.float32)
    g = rng.standard_normal((L, M, d)).astype(np.float32)
    tr = oc.correction_scan(md, X0, g, oc.HCN)
    # (1) scalar loops, one fp32 operation at a time in the documented order: must match bit for bit
    for m in range(M):
        for c in range(d):
            x = [X0[m, j, c] for j in range(n)]
            for l in range(L):
                new = []
                for i in range(n):
                    acc = np.float32(post[l, i] * g[l, m, c])
                    for j in range(n):
                        acc = np.float32(acc + np.float32(Hres[l, i, j] * x[j]))
                    new.append(acc)
                x = new
                for i in range(n):
                    assert x[i] == tr[l + 1, m, i, c]
    # (2) composed affine maps (A, b) <- (H_l A, H_l b + p_l g_l) in fp64: equal to rounding
    A = np.eye(n)
    b = np.zeros((M, n, d))
    for l in range(L):
        Hl = Hres[l].astype(np.float64)
        A = Hl @ A
        b = np.einsum("ij,mjc->mic", Hl, b) + post[l].astype(np.float64)[None, :, None] * g[l].astype(np.float64)[:, None, :]
        full = np.einsum("ij,mjc->mic", A, X0.astype(np.float64)) + b
        assert rel_err(tr[l + 1], full) < 1e-6


def test_stream_sum_follows_prefix_sum_when_columns_sum_to_one():
    shp, t, md = small(n_streams=4)
    assert np.allclose(md.Hres.sum(axis=1), 1.0, atol=1e-6)       # columns normalised last by the recipe
    assert np.allclose(md.Hres.sum(axis=2), 1.0, atol=1e-3)
    tr0 = oc.init_trace(md, t["h0"])
    g = oc.evaluate_branches(md, tr0)
    tr1 = oc.correction_scan(md, tr0[0], g, oc.HCN)
    acc = tr0[0].astype(np.float64).sum(axis=1)
    for l in range(1, shp.L + 1):
        acc = acc + md.post[l - 1].astype(np.float64).sum() * g[l - 1].astype(np.float64)
        assert rel_err(tr1[l].astype(np.float64).sum(axis=1), acc) < 1e-5


def test_correction_propagates_in_one_round_but_plain_fixed_point_does_not():
    shp, t, md = small(L=5)
    shp2, t2, md2 = small(L=5)
    md2.Wo[0] = md2.Wo[0] * np.float32(1.5)                       # perturb layer 1 only
    tr0 = oc.init_trace(md, t["h0"])
    a, _, _ = oc.iterate(md, tr0, oc.IDN, 1)
    b, _, _ = oc.iterate(md2, tr0, oc.IDN, 1)
    assert rel_err(a[5], b[5]) > 1e-4                             # reaches the last layer at K = 1
    for K in (1, 2, 3):
        ja = oc.iterate_no_correction(md, tr0, oc.IDN, K)
        jb = oc.iterate_no_correction(md2, tr0, oc.IDN, K)
        for l in range(K + 1, 6):
            assert np.array_equal(ja[l], jb[l])                   # staircase: layers > K not reached
        assert not np.array_equal(ja[K], jb[K])
    assert rel_err(oc.iterate_no_correction(md, tr0, oc.IDN, 5), oc.sequential_forward(md, t["h0"])) < 1e-6


def test_single_layer_iteration_is_sequential():
    shp, t, md = small(L=1)
    tr, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), oc.IDN, 1)
    assert np.array_equal(tr, oc.sequential_forward(md, t["h0"]))


def test_iterates_stay_bounded():
    shp, t, md = small(P=3)
    tr = oc.init_trace(md, t["h0"])
    gmax = 0.0
    for k in range(3):
        g = oc.evaluate_branches(md, tr)
        gmax = max(gmax, max(np.linalg.norm(g[l]) for l in range(shp.L)))
        tr, _, _ = oc.iterate(md, tr, oc.IDN, 1)
        for l in range(shp.L + 1):
            assert np.linalg.norm(tr[l]) <= np.linalg.norm(t["h0"]) + l * gmax * (1 + 1e-6)


def test_iterate_calls_compose():
    shp, t, md = small(n_streams=2)
    tr0 = oc.init_trace(md, t["h0"])
    a, pa, _ = oc.iterate(md, tr0, oc.HCN, 3)
    b1, p1, _ = oc.iterate(md, tr0, oc.HCN, 1)
    b2, p2, _ = oc.iterate(md, b1, oc.HCN, 2)
    assert np.array_equal(a, b2)
    assert np.array_equal(pa, np.concatenate([p1, p2]))
    c, pc, _ = oc.iterate(md, tr0, oc.HCN, 0)
    assert np.array_equal(c, tr0) and pc.shape == (0, 2, shp.L)


# ---------------------------------------------------------------- the bf16-operand test aid

def test_bf16_rounding_aid_matches_torch_and_changes_no_formula():
    """round_bf16 only rounds stored operands: bf16_round is torch's float32 -> bfloat16 conversion; the rounded branch
    equals the same composition written with torch bfloat16 casts; switched off, nothing changes."""
    rng = np.random.default_rng(9)
    x = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096), [0.0, -0.0, 1.0, 3.0e38, 1.0e-40]])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oc.bf16_round(x), want)
    assert np.array_equal(oc.bf16_round(x), si.bf16_bits_to_f32(si.f32_to_bf16_bits(x.astype(np.float32))).astype(np.float64))

    shp, t, md = small(P=3, L=2, T=5, B=1)
    u = t["h0"][:, 0, :].astype(np.float64)
    exact_a, exact_m = oc.branch(md, 1, u)
    mdr = oc.Model(**{**md.__dict__, "round_bf16": True})
    ra, rm = oc.branch(mdr, 1, u)
    assert 1e-4 < rel_err(ra, exact_a) < 2e-2 and 1e-4 < rel_err(rm, exact_m) < 2e-2      # operand rounding only
    bf = lambda z: z.to(torch.bfloat16).to(torch.float64)
    tt = lambda z: torch.from_numpy(np.ascontiguousarray(z, dtype=np.float64))
    eps, dh, H, T = md.rms_eps, md.head_dim, md.n_heads, md.T
    norm = lambda z: z / torch.sqrt((z * z).mean(-1, keepdim=True) + eps)
    xh = bf(norm(tt(u)).float())
    qkv = bf((xh @ tt(md.Wqkv[0])).float()).reshape(T, 3, H, dh)
    cos, sin = [tt(z) for z in oc.rope_cos_sin(md.P + np.arange(T), dh, md.rope_base)]
    def rot(z):                                                   # z [T, H, dh]
        z1, z2 = z[..., : dh // 2], z[..., dh // 2:]
        return torch.cat([z1 * cos[:, None] - z2 * sin[:, None], z2 * cos[:, None] + z1 * sin[:, None]], -1)
    q = bf(norm(rot(qkv[:, 0])).float()).transpose(0, 1)         # [H, T, dh]
    k = bf(norm(rot(qkv[:, 1])).float()).transpose(0, 1)
    v = qkv[:, 2].transpose(0, 1)
    keys = torch.cat([tt(md.Kpre[0][0]), k], 1)
    vals = torch.cat([tt(md.Vpre[0][0]), v], 1)
    sc = q @ keys.transpose(1, 2) / np.sqrt(dh)
    vis = torch.cat([torch.ones(T, md.P, dtype=torch.bool), torch.tril(torch.ones(T, T, dtype=torch.bool))], 1)
    sc = sc.masked_fill(~vis, float("-inf"))
    e = torch.exp(sc - sc.max(-1, keepdim=True).values)
    o = bf(((bf(e.float()) @ vals) / e.sum(-1, keepdim=True)).float()).transpose(0, 1).reshape(T, H * dh)
    a = o @ tt(md.Wo[0])
    assert rel_err(ra, a.numpy()) < 1e-12
    x2 = bf(norm(tt(u) + a).float())
    hid = bf((torch.relu(x2 @ tt(md.Wfc[0])) ** 2).float())
    assert rel_err(rm, (hid @ tt(md.Wproj[0])).numpy()) < 1e-12


# ---------------------------------------------------------------- the pins notice planted mistakes

def _pins_hold(mod) -> bool:
    """A condensed run of the pins above against module-like `mod` (used with planted mistakes)."""
    try:
        g = read_golden("hcn_scan_small.txt")
        md = mod.Model(L=2, d=1, n_heads=1, head_dim=1, d_mlp=1, B=1, T=1, P=0, Wqkv=[], Wo=[], Wfc=[], Wproj=[],
                       n_streams=2, Hres=np.stack([g["H1"].reshape(2, 2), g["H2"].reshape(2, 2)]),
                       pre=np.ones((2, 2), np.float32), post=np.stack([g["p1"], g["p2"]]))
        tr = mod.correction_scan(md, g["X0"].reshape(1, 2, 1), g["g"].reshape(2, 1, 1), mod.HCN)
        if not (np.array_equal(tr[1].ravel(), g["expect_X1"]) and np.array_equal(tr[2].ravel(), g["expect_X2"])):
            return False
        shp, t, md = small(n_streams=3, P=3)
        seq = mod.sequential_forward(md, t["h0"], mod.HCN)
        fin, _, _ = mod.iterate(md, mod.init_trace(md, t["h0"]), mod.HCN, shp.L)
        if not np.array_equal(fin, seq):
            return False
        df = mod.iterate_delta_form(md, mod.init_trace(md, t["h0"]), mod.HCN, 2)
        pf, _, _ = mod.iterate(md, mod.init_trace(md, t["h0"]), mod.HCN, 2)
        if rel_err(pf, df) > 2e-6:
            return False
        test_branch_matches_torch_library_composition()
        test_rope_is_complex_rotation_with_half_split_pairs()
        test_one_step_idn_closed_form()
        if not _hc_sublayer_fixture_holds(mod):
            return False
        return True
    except AssertionError:
        return False


def test_pins_catch_planted_mistakes(monkeypatch):
    assert _pins_hold(oc)
    # transposed mixing matrix
    orig = oc.layer_step

    def transposed(model, l, X_prev, g, mode):
        if model.Hres is None:
            return orig(model, l, X_prev, g, mode)
        sw = oc.Model(**{**model.__dict__, "Hres": np.ascontiguousarray(np.swapaxes(model.Hres, 1, 2))})
        return orig(sw, l, X_prev, g, mode)

    monkeypatch.setattr(oc, "layer_step", transposed)
    assert not _pins_hold(oc)
    monkeypatch.setattr(oc, "layer_step", orig)
    # rotation with the wrong sign
    orig_rope = oc.apply_rope
    monkeypatch.setattr(oc, "apply_rope", lambda x, c, s: orig_rope(x, c, -s))
    assert not _pins_hold(oc)
    monkeypatch.setattr(oc, "apply_rope", orig_rope)
    # branch output that drops the MLP update
    orig_bo = oc.branch_output

    def no_mlp(model, l, X_prev):
        a, m = oc.branch(model, l, oc.premix(model, l, X_prev))
        return a.astype(np.float32)

    monkeypatch.setattr(oc, "branch_output", no_mlp)
    assert not _pins_hold(oc)
    monkeypatch.setattr(oc, "branch_output", orig_bo)
    # layers reading their own state instead of the previous one (off-by-one in the trace index)
    orig_eval = oc.evaluate_branches
    monkeypatch.setattr(oc, "evaluate_branches",
                        lambda model, trace, S=0: np.stack([oc.branch_output(model, l, trace[l]) for l in range(1, model.L + 1)]))
    assert not _pins_hold(oc)
    monkeypatch.setattr(oc, "evaluate_branches", orig_eval)
    # stream pre-mix weighted by post instead of pre, and with the stream axis reversed
    orig_premix = oc.premix

    def premix_with(pick):
        def wrong(model, l, X):
            X = np.asarray(X, dtype=np.float64)
            if model.n_streams == 1:
                return X[:, 0, :]
            return np.einsum("j,mjc->mc", np.asarray(pick(model, l), dtype=np.float64), X)
        return wrong

    monkeypatch.setattr(oc, "premix", premix_with(lambda model, l: model.post[l - 1]))
    assert not _pins_hold(oc)
    monkeypatch.setattr(oc, "premix", premix_with(lambda model, l: model.pre[l - 1][::-1]))
    assert not _pins_hold(oc)
    monkeypatch.setattr(oc, "premix", orig_premix)
    assert _pins_hold(oc)


# ---------------------------------------------------------------- input recipe

def test_inputs_are_seeded_and_shaped():
    shp = si.config(3, L=2, B=2, T=4, P=16)
    a, b = si.generate(shp), si.generate(shp)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert a["h0"].shape == (8, 1, 1280) and a["Wqkv"].shape == (2, 1280, 3840) and a["Wqkv"].dtype == np.uint16
    assert a["Kpre"].shape == (2, 2, 10, 16, 128)
    k = si.as_float(a["Kpre"]).astype(np.float64)
    assert np.allclose(np.sqrt(np.mean(k * k, axis=-1)), 1.0, atol=5e-3)
    w = si.as_float(a["Wfc"])
    assert abs(float(w.std()) - 0.02) < 5e-4
    # round to nearest even on the 8th mantissa bit: 1 + 2^-8 ties to 1, 1 + 3*2^-8 ties to 1 + 2^-6
    assert si.bf16_bits_to_f32(si.f32_to_bf16_bits(np.array([1.00390625], np.float32)))[0] == 1.0
    assert si.bf16_bits_to_f32(si.f32_to_bf16_bits(np.array([1.01171875], np.float32)))[0] == 1.015625
    tb = torch.tensor(w[0, :4, :4]).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(tb, w[0, :4, :4])                    # already bf16-representable
    r = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    assert np.array_equal(si.bf16_bits_to_f32(si.f32_to_bf16_bits(r)),
                          torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy())


# ---------------------------------------------------------------- sequential prefix and one-shot-forward initialisation

@pytest.mark.parametrize("n,mode", [(1, oc.IDN), (3, oc.HCN)])
def test_prefix_and_fwd_initialisation_terminate_early(n, mode):
    """Alg. 2 with a sequential prefix of S layers: slots 0..S are exact from the start, each round makes one
    more layer exact, K = L - S recovers the sequential trace bit for bit.  The one-shot-forward initialisation
    makes layer S+1 exact before the first round, so K = L - S - 1 suffices."""
    shp, t, md = small(n_streams=n, L=5, P=2)
    seq = oc.sequential_forward(md, t["h0"], mode)
    for S in (0, 2, 4):
        tr = oc.init_trace(md, t["h0"], S=S, mode=mode)
        assert np.array_equal(tr[: S + 1], seq[: S + 1])
        assert all(np.array_equal(tr[l], seq[S]) for l in range(S + 1, 6))
        _, probe, kept = oc.iterate(md, tr, mode, 5 - S, keep=True, S=S)
        for k, trk in enumerate(kept, start=1):
            assert np.array_equal(trk[: S + k + 1], seq[: S + k + 1])
            if S + k < 5:
                assert not np.array_equal(trk[S + k + 1], seq[S + k + 1])
        assert np.all(probe[:, :, :S] == 0.0)
        trf = oc.init_trace(md, t["h0"], S=S, mode=mode, init=oc.INIT_FWD)
        assert np.array_equal(trf[: S + 2], seq[: S + 2])
        if S < 3:
            assert not np.array_equal(trf[S + 2], seq[S + 2])
        fin, _, _ = oc.iterate(md, trf, mode, 5 - S - 1, S=S)
        assert np.array_equal(fin, seq)


@pytest.mark.parametrize("n,mode", [(1, oc.IDN), (3, oc.HCN), (3, oc.IDN)])
def test_leaving_converged_layers_out_changes_nothing(n, mode):
    """Rounds that work only on the layers that can still change give the same trace and the same probes, bit for
    bit, as full rounds: for both initialisations, with and without a sequential prefix, up to K = L."""
    shp, t, md = small(n_streams=n, L=5, P=2)
    for S, init in ((0, oc.INIT_H0), (2, oc.INIT_H0), (0, oc.INIT_FWD), (1, oc.INIT_FWD)):
        tr0 = oc.init_trace(md, t["h0"], S=S, mode=mode, init=init)
        full, pfull, _ = oc.iterate(md, tr0, mode, 5, S=S)
        exact = S + (1 if init == oc.INIT_FWD else 0)
        skip, pskip = oc.iterate_skipping_converged(md, tr0, mode, 5, S=S, exact=exact)
        assert np.array_equal(full, skip) and np.array_equal(pfull, pskip)
        # the probes of the layers left out are exactly zero in the full rounds too
        for k in range(5):
            assert np.all(pfull[k, :, : min(exact + k, 5)] == 0.0)
    # overstating the number of exact layers does change the result: the count is what makes it safe
    tr0 = oc.init_trace(md, t["h0"], mode=mode)
    wrong, _ = oc.iterate_skipping_converged(md, tr0, mode, 2, exact=2)
    right, _, _ = oc.iterate(md, tr0, mode, 2)
    assert not np.array_equal(wrong, right)


def test_fwd_initialisation_is_one_uncorrected_round():
    shp, t, md = small(L=4)
    trf = oc.init_trace(md, t["h0"], init=oc.INIT_FWD)
    jac = oc.iterate_no_correction(md, oc.init_trace(md, t["h0"]), oc.IDN, 1)
    assert rel_err(trf, jac) < 1e-6
    # and differs from the h0 initialisation followed by one corrected round beyond layer 1
    one, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), oc.IDN, 1)
    assert np.array_equal(one[1], trf[1]) and not np.array_equal(one[3], trf[3])


# ---------------------------------------------------------------- diagonal surrogate with supplied diagonals

def test_diag_correction_special_cases_and_termination():
    shp, t, md = small(L=5, P=2)
    rng = np.random.default_rng(21)
    seq = oc.sequential_forward(md, t["h0"])
    tr0 = oc.init_trace(md, t["h0"])
    ones = np.ones((shp.L, shp.M, shp.d), np.float32)
    # a = 1 is IDN (to rounding: the additions associate differently)
    a1, _ = oc.iterate_diag(md, tr0, ones, 2)
    b1, _, _ = oc.iterate(md, tr0, oc.IDN, 2)
    assert rel_err(a1, b1) < 1e-6
    # a = 0 is the uncorrected fixed point h_l = f_l(h_{l-1}^k), exactly
    a0, _ = oc.iterate_diag(md, tr0, 0 * ones, 2)
    j0 = oc.iterate_no_correction(md, tr0, oc.IDN, 2)
    assert rel_err(a0, j0) < 1e-6
    # any diagonals: after k rounds layers 1..k are exact, K = L recovers the sequential trace bit for bit
    diag = rng.uniform(-0.5, 1.5, (shp.L, shp.M, shp.d)).astype(np.float32)
    tr = tr0
    for k in range(1, shp.L + 1):
        tr, probe = oc.iterate_diag(md, tr, diag, 1)
        assert np.array_equal(tr[: k + 1], seq[: k + 1])
        assert np.all(probe[0, 0, : k - 1] == 0.0)
    assert np.array_equal(tr, seq)


def test_diag_correction_is_exact_newton_on_elementwise_affine_layers():
    """If every layer is f_l(x) = c_l x + e_l elementwise, the true Jacobian is diag(c_l); with a_l = c_l the
    correction is exact Newton on a linear system and reaches the sequential trace in ONE round from any
    starting trace (Methods: "If A = J, this recovers the exact DEER/Newton update")."""
    rng = np.random.default_rng(22)
    L, M, d = 6, 3, 7
    c = rng.uniform(-1.2, 1.2, (L, M, d))
    e = rng.standard_normal((L, M, d))
    h0 = rng.standard_normal((M, 1, d)).astype(np.float32)
    seq = np.empty((L + 1, M, 1, d))
    seq[0] = h0
    for l in range(1, L + 1):
        seq[l][:, 0, :] = c[l - 1] * seq[l - 1][:, 0, :] + e[l - 1]
    start = rng.standard_normal((L + 1, M, 1, d)).astype(np.float32)
    start[0] = h0
    g = np.stack([(c[l] - 1.0) * start[l][:, 0, :] + e[l] for l in range(L)]).astype(np.float32)   # g_l(h_{l-1}^k)
    new = oc.correction_scan_diag(start, g, c.astype(np.float32))
    assert rel_err(new, seq) < 1e-5
    wrong = oc.correction_scan_diag(start, g, (0.5 * c).astype(np.float32))
    assert rel_err(wrong, seq) > 1e-2


def test_diag_scan_against_scalar_loops_and_affine_composition():
    rng = np.random.default_rng(23)
    L, M, d = 4, 2, 3
    old = rng.standard_normal((L + 1, M, 1, d)).astype(np.float32)
    g = rng.standard_normal((L, M, d)).astype(np.float32)
    a = rng.uniform(-1, 1, (L, M, d)).astype(np.float32)
    new = oc.correction_scan_diag(old, g, a)
    for m in range(M):
        for ch in range(d):
            x = old[0, m, 0, ch]
            A, Bc = 1.0, 0.0
            for l in range(1, L + 1):
                tilde = np.float32(old[l - 1, m, 0, ch] + g[l - 1, m, ch])
                x = np.float32(tilde + np.float32(a[l - 1, m, ch] * np.float32(x - old[l - 1, m, 0, ch])))
                assert x == new[l, m, 0, ch]                     # scalar loop, same fp32 order: bit for bit
                # Alg. 3: h_l = a_l h_{l-1} + b_l with b_l = h~_l - a_l h_{l-1}^k, composed associatively
                al = float(a[l - 1, m, ch])
                bl = float(old[l - 1, m, 0, ch]) + float(g[l - 1, m, ch]) - al * float(old[l - 1, m, 0, ch])
                A, Bc = al * A, al * Bc + bl
                assert abs(A * float(old[0, m, 0, ch]) + Bc - float(x)) < 1e-5 * max(1.0, abs(float(x)))


# ---------------------------------------------------------------- chunkwise fused layers

def test_fused_chunks_special_cases():
    shp, t, md = small(L=6, P=2)
    h0 = t["h0"]
    # F = 1 is the plain model, bit for bit
    assert np.array_equal(oc.fused_sequential_forward(md, h0, 1), oc.sequential_forward(md, h0))
    a, pa, _ = oc.fused_iterate(md, oc.init_trace(md, h0), 1, 3)
    b, pb, _ = oc.iterate(md, oc.init_trace(md, h0), oc.IDN, 3)
    assert np.array_equal(a, b) and np.array_equal(pa, pb)
    # finite termination over chunks: K = L / F recovers the fused sequential trace bit for bit
    for F in (2, 3, 6):
        N = shp.L // F
        seq = oc.fused_sequential_forward(md, h0, F)
        tr0 = np.ascontiguousarray(np.broadcast_to(h0, (N + 1,) + h0.shape)).copy()
        fin, probe, kept = oc.fused_iterate(md, tr0, F, N, keep=True)
        for k, trk in enumerate(kept, start=1):
            assert np.array_equal(trk[: k + 1], seq[: k + 1])
        assert np.array_equal(fin, seq)
    # fusing changes the computation: every MLP branch sees the aggregate post-attention state (coupling term)
    assert rel_err(oc.fused_sequential_forward(md, h0, 2)[3], oc.sequential_forward(md, h0)[6]) > 1e-3


def test_fused_chunk_without_attention_output_is_one_step_idn():
    """With Wo = 0 every a_l vanishes, u_C = h, and a chunk over all layers gives h + sum_l m_l(h): the one-step
    IDN result (Appendix "Variance Reduction Derivation") of the same model."""
    shp, t, md = small(L=4)
    md.Wo = [np.zeros_like(w) for w in md.Wo]
    fused = oc.fused_sequential_forward(md, t["h0"], 4)
    idn1, _, _ = oc.iterate(md, oc.init_trace(md, t["h0"]), oc.IDN, 1)
    assert rel_err(fused[1], idn1[4]) < 1e-6
    assert rel_err(fused[1], t["h0"]) > 1e-3


def test_fused_chunk_matches_concatenated_weight_form():
    """The fused layer as the paper states it: Q, K, V and MLP-up weights concatenated along the output dimension,
    O and MLP-down weights along the input dimension (one wide matmul + sum-reduction)."""
    shp, t, md = small(L=2, P=0, B=1, T=5)
    h = t["h0"][:, 0, :].astype(np.float64)
    g = oc.fused_chunk_output(md, 1, 2, h)
    x = oc.rmsnorm(h, md.rms_eps)
    heads = []
    for l in (1, 2):                                              # attention per layer on the shared input
        qkv = (x @ md.Wqkv[l - 1].astype(np.float64)).reshape(1, 5, 3, md.n_heads, md.head_dim).transpose(2, 0, 3, 1, 4)
        cos, sin = oc.rope_cos_sin(np.arange(5), md.head_dim, md.rope_base)
        q = oc.rmsnorm(oc.apply_rope(qkv[0], cos, sin), md.rms_eps)
        k = oc.rmsnorm(oc.apply_rope(qkv[1], cos, sin), md.rms_eps)
        heads.append(oc.attention(q, k, np.ascontiguousarray(qkv[2]), None, None).transpose(0, 2, 1, 3).reshape(5, md.d))
    Ocat = np.concatenate([md.Wo[0], md.Wo[1]], axis=0).astype(np.float64)          # [2d, d]: input-dim concat
    a_C = np.concatenate(heads, axis=1) @ Ocat
    Wcat = np.concatenate([md.Wfc[0], md.Wfc[1]], axis=1).astype(np.float64)        # [d, 2F]: output-dim concat
    Pcat = np.concatenate([md.Wproj[0], md.Wproj[1]], axis=0).astype(np.float64)    # [2F, d]
    m_C = (np.maximum(oc.rmsnorm(h + a_C, md.rms_eps) @ Wcat, 0.0) ** 2) @ Pcat
    assert rel_err(g, a_C + m_C) < 1e-6
