"""The stage-by-stage GPU parity checks (test_gpu_stages.py) can fail: shown on the CPU with the oracle alone.

Each planted mistake is put into a copy of the ORACLE's own pieces (never into GPU code); the wrong stage outputs are
compared with the right ones through the same row-wise metric and the same cases the GPU test uses, and must exceed
the GPU test's tolerance in at least one case.  So a kernel making that mistake would fail the GPU test.  For
contrast the old whole-state metric is evaluated too: it does not notice most of them."""
import numpy as np
import pytest

from oracle import snlp_oracle as oc
from oracle.harness import per_layer_rel_err
import stage_checks as sc

CASES = [c for c in sc.SMALL_CASES]


def stages_all_layers(case, md, trace):
    return [sc.oracle_stages(md, l, trace[l - 1]) for l in range(1, case.shape.L + 1)]


def worst_errors(case, md, trace, right):
    """Row-wise stage errors of the (patched) oracle against `right`, worst over layers."""
    fused_rope = case.shape.T <= 16 and case.shape.P >= 512
    worst = {}
    for l, ref in enumerate(right, start=1):
        got = sc.oracle_stages(md, l, trace[l - 1])
        for k, e in sc.compare_stages(got, ref, case.shape.n_streams, rotated_qk=not fused_rope).items():
            worst[k] = max(worst.get(k, 0.0), e)
    return worst


# ---- planted mistakes: each returns a context manager-like (enter, exit) pair patching the oracle module

def plant_no_rotation_on_k(mp):
    real = oc.apply_rope
    calls = {"n": 0}
    def wrong(x, cos, sin):
        calls["n"] += 1
        return x if calls["n"] % 2 == 0 else real(x, cos, sin)      # q is rotated (odd calls), k is not
    mp.setattr(oc, "apply_rope", wrong)


def plant_block_keys_masked_out(mp):
    real = oc.attention
    def wrong(q, k, v, kpre, vpre):
        if kpre is None or kpre.shape[2] == 0:
            return real(q, k, v, kpre, vpre)
        # prefix only: the block's own rows never enter the softmax (except each query's own row when there is no prefix)
        B, H, T, dh = q.shape
        out = np.empty_like(q)
        for b in range(B):
            for h in range(H):
                s = (q[b, h] @ np.asarray(kpre[b, h], dtype=np.float64).T) / np.sqrt(float(dh))
                e = np.exp(s - s.max(axis=-1, keepdims=True))
                out[b, h] = (e / e.sum(axis=-1, keepdims=True)) @ np.asarray(vpre[b, h], dtype=np.float64)
        return out
    mp.setattr(oc, "attention", wrong)


def plant_prefix_tile_dropped(mp):
    real = oc.attention
    def wrong(q, k, v, kpre, vpre):
        if kpre is None or kpre.shape[2] < 64:
            return real(q, k, v, kpre, vpre)
        keep = np.ones(kpre.shape[2], dtype=bool)
        keep[32:64] = False                                       # one 32-key tile of the prefix is skipped
        return real(q, k, v, np.asarray(kpre)[:, :, keep], np.asarray(vpre)[:, :, keep])
    mp.setattr(oc, "attention", wrong)


def plant_no_causal_mask(mp):
    def wrong(q, k, v, kpre, vpre):
        B, H, T, dh = q.shape
        out = np.empty_like(q)
        for b in range(B):
            for h in range(H):
                keys, vals = k[b, h], v[b, h]
                if kpre is not None and kpre.shape[2] > 0:
                    keys = np.concatenate([np.asarray(kpre[b, h], dtype=np.float64), keys])
                    vals = np.concatenate([np.asarray(vpre[b, h], dtype=np.float64), vals])
                s = (q[b, h] @ keys.T) / np.sqrt(float(dh))      # every block row visible to every query
                e = np.exp(s - s.max(axis=-1, keepdims=True))
                out[b, h] = (e / e.sum(axis=-1, keepdims=True)) @ vals
        return out
    mp.setattr(oc, "attention", wrong)


def plant_positions_without_prefix_offset(mp):
    real = oc.rope_cos_sin
    def wrong(positions, head_dim, base):
        positions = np.asarray(positions)
        return real(positions - positions[0], head_dim, base)     # angle t instead of P + t
    mp.setattr(oc, "rope_cos_sin", wrong)


def plant_no_score_scale(mp):
    real = oc.attention
    def wrong(q, k, v, kpre, vpre):
        return real(q * np.sqrt(float(q.shape[-1])), k, v, kpre, vpre)   # cancels the 1 / sqrt(dh)
    mp.setattr(oc, "attention", wrong)


def plant_attention_zeroed(mp):
    mp.setattr(oc, "attention", lambda q, k, v, kpre, vpre: np.zeros_like(q))


def plant_pre_swapped_for_post(mp):
    def wrong(model, l, X):
        X = np.asarray(X, dtype=np.float64)
        if model.n_streams == 1:
            return X[:, 0, :]
        return np.einsum("j,mjc->mc", np.asarray(model.post[l - 1], dtype=np.float64), X)
    mp.setattr(oc, "premix", wrong)


def plant_streams_reversed_in_premix(mp):
    def wrong(model, l, X):
        X = np.asarray(X, dtype=np.float64)
        if model.n_streams == 1:
            return X[:, 0, :]
        return np.einsum("j,mjc->mc", np.asarray(model.pre[l - 1], dtype=np.float64)[::-1], X)
    mp.setattr(oc, "premix", wrong)


def plant_relu_instead_of_relu_squared(mp):
    def wrong(model, l, u_mid):
        x2 = oc.rmsnorm(np.asarray(u_mid, dtype=np.float64), model.rms_eps)
        hid = np.maximum(x2 @ np.asarray(model.Wfc[l - 1], dtype=np.float64), 0.0)
        return hid @ np.asarray(model.Wproj[l - 1], dtype=np.float64)
    mp.setattr(oc, "mlp_update", wrong)


MISTAKES = [
    ("no rotation on the block's k rows", plant_no_rotation_on_k, ("k", "attn")),
    ("block keys masked out", plant_block_keys_masked_out, ("attn",)),
    ("one prefix tile dropped", plant_prefix_tile_dropped, ("attn",)),
    ("no causal mask inside the block", plant_no_causal_mask, ("attn",)),
    ("rotation angle t instead of P + t", plant_positions_without_prefix_offset, ("attn",)),
    ("scores not scaled by 1 / sqrt(dh)", plant_no_score_scale, ("attn",)),
    ("attention output zeroed", plant_attention_zeroed, ("attn", "a")),
    ("pre swapped for post in the stream pre-mix", plant_pre_swapped_for_post, ("u",)),
    ("stream axis reversed in the pre-mix", plant_streams_reversed_in_premix, ("u",)),
    ("ReLU instead of ReLU^2", plant_relu_instead_of_relu_squared, ("m",)),
]


@pytest.fixture(scope="module")
def right_answers():
    out = {}
    for case in CASES:
        t = case.tensors()
        md = sc.model_of(case, t)
        mode = oc.HCN if case.shape.n_streams > 1 else oc.IDN
        tr0 = oc.init_trace(md, t["h0"])
        tr1, _, _ = oc.iterate(md, tr0, mode, 1)
        out[case.name] = (case, md, tr1, stages_all_layers(case, md, tr1))
    return out


@pytest.mark.parametrize("name,plant,stages", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_exceeds_stage_tolerance(right_answers, monkeypatch, name, plant, stages):
    tol = sc.tolerances()
    caught = []
    state_metric = []
    for cname, (case, md, tr1, right) in right_answers.items():
        with monkeypatch.context() as mp:
            plant(mp)
            worst = worst_errors(case, md, tr1, right)
            # the old metric: relative Frobenius error of whole hidden states after one more round
            mode = oc.HCN if case.shape.n_streams > 1 else oc.IDN
            wrong_next, _, _ = oc.iterate(md, tr1, mode, 1)
        right_next, _, _ = oc.iterate(md, tr1, mode, 1)
        state_metric.append(float(per_layer_rel_err(wrong_next, right_next).max()))
        hit = [k for k in stages if k in worst and worst[k] > tol[k]]
        if hit:
            caught.append((cname, {k: worst[k] for k in hit}))
    print("%s: caught by %d case(s): %s; whole-state metric at most %.2e" %
          (name, len(caught), "; ".join("%s %s" % (c, {k: "%.1e" % v for k, v in w.items()}) for c, w in caught[:4]), max(state_metric)))
    assert caught, "no stage check notices: " + name
    # every stage error that counts is far beyond the tolerance, not marginally above it
    assert max(max(w.values()) for _, w in caught) > 5 * sc.TOL_ATTN or stages == ("u",)


def test_decode_specific_mistakes_are_caught_by_the_fused_rotation_cases(right_answers, monkeypatch):
    """The three mistakes the decode kernel's own rotation path could make are each noticed by a case with P >= 512
    and T <= 16 (the shapes on which that path runs)."""
    tol = sc.TOL_ATTN
    fused = [n for n, (c, _, _, _) in right_answers.items() if c.shape.P >= 512 and c.shape.T <= 16]
    assert len(fused) >= 6
    for name, plant in (("no rotation on the block's k rows", plant_no_rotation_on_k),
                        ("block keys masked out", plant_block_keys_masked_out),
                        ("one prefix tile dropped", plant_prefix_tile_dropped),
                        ("no causal mask inside the block", plant_no_causal_mask)):
        hits = []
        for cname in fused:
            case, md, tr1, right = right_answers[cname]
            with monkeypatch.context() as mp:
                plant(mp)
                worst = worst_errors(case, md, tr1, right)
            if worst["attn"] > tol:
                hits.append((cname, worst["attn"]))
        print(name, "->", hits)
        assert hits, name


def test_whole_state_metric_misses_attention_mistakes(right_answers, monkeypatch):
    """Why the per-stage checks exist: on the decode shape behind a long prefix the relative Frobenius error of the hidden
    states stays under 2e-2 even with the attention output zeroed."""
    case, md, tr1, right = right_answers["decode_P999_T16"]
    right_next, _, _ = oc.iterate(md, tr1, oc.IDN, 1)
    with monkeypatch.context() as mp:
        plant_no_rotation_on_k(mp)
        wrong_next, _, _ = oc.iterate(md, tr1, oc.IDN, 1)
    assert per_layer_rel_err(wrong_next, right_next).max() < 2e-2


def test_row_metric_definition():
    ref = np.array([[3.0, 4.0], [0.0, 0.0], [1.0, 0.0]])
    x = np.array([[3.0, 4.5], [0.0, 0.0], [1.0, 0.0]])
    assert np.isclose(sc.row_rel_err(x, ref), 0.1)
    x[1, 0] = 1e-9
    assert sc.row_rel_err(x, ref) == float("inf")
