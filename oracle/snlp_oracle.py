"""CPU oracle for the SNLP iteration.  TEST INFRASTRUCTURE, not a product path.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file; the HIP library never calls it and shares no code with it.

What it computes, and where the paper defines it
------------------------------------------------
* hidden-state trace h_0..h_L and layer maps h_l = f_l(h_{l-1}): Methods,
  "Layer traces as residual equations", Eq. (1).
* residual G_l(h) = h_l - f_l(h_{l-1}): Eq. (2).
* sequential execution: Appendix "Algorithm", Alg. 1.
* SNLP iteration = parallel evaluation of every layer on the current trace
  (Eq. (4)) followed by the structured correction (Eq. (5)); the loop with
  h0 initialisation is Alg. 2.
* IDN surrogate A = I (Eq. (6)-(7)): with f_l(x) = x + g_l(x) (Appendix
  "Variance Reduction Derivation") the correction becomes
  h_l^{k+1} = h_{l-1}^{k+1} + g_l(h_{l-1}^k), a prefix sum over depth.
* HCN surrogate A_l = residual stream-mixing matrix (Eq. (8); Appendix
  "Connection to Hyper-Connections and mHC", simplified HC sublayer
  x_{l+1} = H^res x_l + H^post F(H^pre x_l)).

Notation.  The paper's f_l is the FULL layer; g_l is its non-residual branch
(attention + MLP update).  Here `branch` returns the pair (a, m) with
g = a + m.  The branch itself (pre-norm RMSNorm without gain, QKV, rotary
embedding, per-head QK RMSNorm, causal softmax attention over a read-only
KV prefix plus the block, ReLU^2 MLP) is fixed by the benchmark shapes, the
paper naming only rotary embeddings for its Nanochat models (Experiments,
setup paragraph).

Arithmetic.  The trace and the branch outputs a, m are stored in fp32.  A
branch is evaluated in fp64 on the upcast trace and its two outputs are
rounded to fp32 once.  The correction is strict fp32 in a fixed order, so a
same-order fp32 implementation must match it bit for bit:
    g   = a (+) m
    IDN (one stream):  h_l = h_{l-1} (+) g_l
    HC model, stream i:  acc = p_l[i] (*) g;  for j = 0..n-1: acc = acc (+) (H_l[i][j] (*) X_{l-1}[j])
    (IDN on an HC model: X_l[i] = X_{l-1}[i] (+) (p_l[i] (*) g))
where (+), (*) are single IEEE fp32 operations (no fused multiply-add).
Residual norms accumulate in fp64.

There is no blocking, fusion or reordering here: every function is the
definition written out with numpy, loops over layers, batch and heads.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

IDN = 0
HCN = 1

f32 = np.float32
f64 = np.float64


@dataclass
class Model:
    """Weights and sizes of an L-layer stack.  Arrays may be any float dtype; they
    are widened to fp64 where used.  y = x @ W for every weight."""
    L: int
    d: int
    n_heads: int
    head_dim: int
    d_mlp: int
    B: int
    T: int
    P: int
    Wqkv: Sequence[np.ndarray]            # [L][d, 3d], columns q | k | v, head h at h*dh..(h+1)*dh-1
    Wo: Sequence[np.ndarray]              # [L][d, d]
    Wfc: Sequence[np.ndarray]             # [L][d, F]
    Wproj: Sequence[np.ndarray]           # [L][F, d]
    Kpre: Optional[Sequence[np.ndarray]] = None   # [L][B, H, P, dh], used as given
    Vpre: Optional[Sequence[np.ndarray]] = None
    n_streams: int = 1
    Hres: Optional[np.ndarray] = None     # [L, n, n] fp32
    pre: Optional[np.ndarray] = None      # [L, n] fp32  (H^pre, a row vector: n streams -> 1)
    post: Optional[np.ndarray] = None     # [L, n] fp32  (H^post, a column vector: 1 -> n streams)
    rope_base: float = 1.0e4
    rms_eps: float = 1.0e-6
    # Test aid, off by default (the definition above is then evaluated in fp64 throughout): round to bfloat16 at the
    # points where a bf16-operand implementation stores an operand -- the normalised inputs, q / k / v, the rotated
    # and normalised q and k, the softmax probabilities that multiply v, the heads' outputs, the hidden activations.
    # It changes no formula; it lets a comparison with such an implementation use a tolerance set by accumulation
    # order instead of by operand rounding.
    round_bf16: bool = False

    @property
    def M(self) -> int:
        return self.B * self.T


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to bfloat16 (via fp32), returned as fp64."""
    u = np.ascontiguousarray(x, dtype=f32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return r.astype(np.uint32).view(f32).astype(f64)


def _operand(model: "Model", x: np.ndarray) -> np.ndarray:
    return bf16_round(x) if model.round_bf16 else x


# ----------------------------------------------------------------------------
# Pieces of the branch g_l
# ----------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) over the last axis, no gain (fp64)."""
    x = np.asarray(x, dtype=f64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope_cos_sin(positions: np.ndarray, head_dim: int, base: float) -> Tuple[np.ndarray, np.ndarray]:
    """cos/sin of p * base^(-2c/dh) for c = 0..dh/2-1; shape [len(positions), dh/2] (fp64)."""
    c = np.arange(head_dim // 2, dtype=f64)
    theta = np.power(f64(base), -2.0 * c / head_dim)
    ang = np.asarray(positions, dtype=f64)[:, None] * theta[None, :]
    return np.cos(ang), np.sin(ang)


def apply_rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate channel pairs (c, c + dh/2) of x[..., T, dh] by the angle of row t."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
              kpre: Optional[np.ndarray], vpre: Optional[np.ndarray], round_p=None) -> np.ndarray:
    """Softmax attention of one layer; q, k, v are [B, H, T, dh], prefix [B, H, P, dh].

    Query t sees every prefix row and block rows t' <= t; scores are
    q.k / sqrt(dh); softmax over the visible keys; output sum_j p_j v_j.
    """
    B, H, T, dh = q.shape
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(f64(dh))
    causal = np.tril(np.ones((T, T), dtype=bool))
    for b in range(B):
        for h in range(H):
            if kpre is not None and kpre.shape[2] > 0:
                keys = np.concatenate([np.asarray(kpre[b, h], dtype=f64), k[b, h]], axis=0)
                vals = np.concatenate([np.asarray(vpre[b, h], dtype=f64), v[b, h]], axis=0)
                P = kpre.shape[2]
            else:
                keys, vals, P = k[b, h], v[b, h], 0
            s = (q[b, h] @ keys.T) * scale                       # [T, P+T]
            visible = np.concatenate([np.ones((T, P), dtype=bool), causal], axis=1)
            s = np.where(visible, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            e = np.exp(s)
            if round_p is None:
                p = e / e.sum(axis=-1, keepdims=True)
                out[b, h] = p @ vals
            else:       # test aid: the probabilities multiply v as rounded operands, their sum stays unrounded
                out[b, h] = (round_p(e) @ vals) / e.sum(axis=-1, keepdims=True)
    return out


def qkv_heads(model: Model, l: int, u: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q, k, v of layer l (1-based) at input u [M, d], each [B, H, T, dh] (fp64): norm(u) Wqkv split into
    heads, q and k rotated at positions P + t and then normalised per head."""
    md = model
    B, T, H, dh = md.B, md.T, md.n_heads, md.head_dim
    u = np.asarray(u, dtype=f64)
    x = _operand(md, rmsnorm(u, md.rms_eps))
    qkv = _operand(md, x @ np.asarray(md.Wqkv[l - 1], dtype=f64))          # [M, 3d]
    qkv = qkv.reshape(B, T, 3, H, dh).transpose(2, 0, 3, 1, 4)             # [3, B, H, T, dh]
    q, k, v = qkv[0], qkv[1], qkv[2]
    cos, sin = rope_cos_sin(md.P + np.arange(T), dh, md.rope_base)
    q = _operand(md, rmsnorm(apply_rope(q, cos, sin), md.rms_eps))
    k = _operand(md, rmsnorm(apply_rope(k, cos, sin), md.rms_eps))
    return q, k, np.ascontiguousarray(v)


def attn_heads(model: Model, l: int, u: np.ndarray) -> np.ndarray:
    """Attn_l(norm(u)): the heads' outputs of layer l side by side, [M, d] (fp64), before the output projection."""
    md = model
    q, k, v = qkv_heads(md, l, u)
    kpre = md.Kpre[l - 1] if md.Kpre is not None else None
    vpre = md.Vpre[l - 1] if md.Vpre is not None else None
    if md.round_bf16:
        o = _operand(md, attention(q, k, v, kpre, vpre, round_p=bf16_round))
    else:
        o = attention(q, k, v, kpre, vpre)                                 # [B, H, T, dh]
    return o.transpose(0, 2, 1, 3).reshape(md.B * md.T, md.d)


def attn_update(model: Model, l: int, u: np.ndarray) -> np.ndarray:
    """a_l(u) = Attn_l(norm(u)) Wo_l for layer l (1-based) at input u [M, d]; fp64."""
    return attn_heads(model, l, u) @ np.asarray(model.Wo[l - 1], dtype=f64)


def mlp_update(model: Model, l: int, u_mid: np.ndarray) -> np.ndarray:
    """m_l(u') = relu(norm(u') Wfc_l)^2 Wproj_l at the post-attention state u' [M, d]; fp64."""
    x2 = _operand(model, rmsnorm(np.asarray(u_mid, dtype=f64), model.rms_eps))
    hid = _operand(model, np.maximum(x2 @ np.asarray(model.Wfc[l - 1], dtype=f64), 0.0) ** 2)
    return hid @ np.asarray(model.Wproj[l - 1], dtype=f64)


def branch(model: Model, l: int, u: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(a, m) = the attention update and the MLP update of layer l (1-based) at input u [M, d].

    a = Attn_l(norm(u)) Wo;  m = relu(norm(u + a) Wfc)^2 Wproj;  g_l(u) = a + m
    (the per-layer case of the Appendix "Fused Cross-Layer Coupling" formulas).
    All in fp64; returns fp64.
    """
    u = np.asarray(u, dtype=f64)
    a = attn_update(model, l, u)
    return a, mlp_update(model, l, u + a)


def premix(model: Model, l: int, X: np.ndarray) -> np.ndarray:
    """Branch input of layer l from the n-stream state X [M, n, d]: sum_j pre_l[j] X[:, j] (fp64)."""
    X = np.asarray(X, dtype=f64)
    if model.n_streams == 1:
        return X[:, 0, :]
    w = np.asarray(model.pre[l - 1], dtype=f64)
    return np.einsum("j,mjc->mc", w, X)


def branch_output(model: Model, l: int, X_prev: np.ndarray) -> np.ndarray:
    """g_l evaluated at the state X_prev [M, n, d], as the fp32 quantity the correction consumes:
    a and m rounded to fp32 once each, then g = a (+) m in fp32."""
    a, m = branch(model, l, premix(model, l, X_prev))
    return a.astype(f32) + m.astype(f32)


# ----------------------------------------------------------------------------
# One layer step and the two corrections, strict fp32
# ----------------------------------------------------------------------------

def layer_step(model: Model, l: int, X_prev: np.ndarray, g: np.ndarray, mode: int) -> np.ndarray:
    """X_l from X_{l-1} [M, n, d] fp32 and the branch output g [M, d] fp32 (strict fp32).

    n = 1:            X_l = X_{l-1} (+) g
    n > 1, HCN:       X_l[i] = p[i] (*) g, then (+) H[i][j] (*) X_{l-1}[j] for j = 0..n-1 in order
    n > 1, IDN:       X_l[i] = X_{l-1}[i] (+) (p[i] (*) g)      (the H = I block)
    """
    X_prev = np.asarray(X_prev, dtype=f32)
    g = np.asarray(g, dtype=f32)
    n = model.n_streams
    if n == 1:
        return X_prev + g[:, None, :]
    p = np.asarray(model.post[l - 1], dtype=f32)
    out = np.empty_like(X_prev)
    for i in range(n):
        t = p[i] * g
        if mode == IDN:
            out[:, i, :] = X_prev[:, i, :] + t
        else:
            Hm = np.asarray(model.Hres[l - 1], dtype=f32)
            acc = t
            for j in range(n):
                acc = acc + Hm[i, j] * X_prev[:, j, :]
            out[:, i, :] = acc
    return out


def correction_scan(model: Model, X0: np.ndarray, g_all: np.ndarray, mode: int,
                    S: int = 0, prefix: Optional[np.ndarray] = None) -> np.ndarray:
    """The structured correction in prefix / affine form (Eq. (5) with f_l = residual-mix + branch).

    X0 [M, n, d] fp32, g_all [L, M, d] fp32 -> new trace [L+1, M, n, d] fp32,
    X_l = layer_step(X_{l-1}, g_l), l = S+1..L, left to right, starting from the fixed prefix state
    (h_S^{k+1} = h_S).  With S > 0, `prefix` [S+1, M, n, d] holds slots 0..S, which are copied.
    """
    L = g_all.shape[0]
    tr = np.empty((L + 1,) + X0.shape, dtype=f32)
    tr[0] = X0
    if S > 0:
        tr[: S + 1] = prefix[: S + 1]
    for l in range(S + 1, L + 1):
        tr[l] = layer_step(model, l, tr[l - 1], g_all[l - 1], mode)
    return tr


def correction_scan_diag(trace_old: np.ndarray, g_all: np.ndarray, diag: np.ndarray, S: int = 0) -> np.ndarray:
    """Diagonal-surrogate correction (Methods, "Diagonal Newton (DiagN)"; Appendix "Algorithm", Alg. 3 with the
    diagonals a_l supplied by the caller), single-stream models:
        h~_l = h_{l-1}^k (+) g_l;   h_l^{k+1} = h~_l (+) a_l (*) (h_{l-1}^{k+1} (-) h_{l-1}^k)
    i.e. Eq. (5) with A_l = diag(a_l), which is the elementwise affine recurrence h_l = a_l h_{l-1} + b_l,
    b_l = h~_l - a_l h_{l-1}^k of Alg. 3, walked left to right in strict fp32 (each operation rounded once).
    trace_old [L+1, M, 1, d], g_all [L, M, d], diag [L, M, d] fp32 -> new trace."""
    old = np.asarray(trace_old, dtype=f32)
    new = old.copy()
    for l in range(S + 1, old.shape[0]):
        tilde = old[l - 1][:, 0, :] + np.asarray(g_all[l - 1], dtype=f32)
        delta = new[l - 1][:, 0, :] - old[l - 1][:, 0, :]
        new[l][:, 0, :] = tilde + np.asarray(diag[l - 1], dtype=f32) * delta
    return new


def iterate_diag(model: Model, trace: np.ndarray, diag: np.ndarray, K: int, S: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """K rounds of (parallel evaluation, diagonal correction) with the same supplied diagonals every round.
    Returns (trace, probe [K, 2, L]) with the probe defined as in `iterate`."""
    trace = np.asarray(trace, dtype=f32)
    probe = np.zeros((K, 2, model.L), dtype=f64)
    for k in range(K):
        g_all = evaluate_branches(model, trace, S)
        probe[k, 0] = residual_sq(model, trace, g_all, IDN, S)
        new = correction_scan_diag(trace, g_all, diag, S)
        dlt = new[1:].astype(f64) - trace[1:].astype(f64)
        probe[k, 1] = np.sum(dlt * dlt, axis=(1, 2, 3))
        trace = new
    return trace, probe


# ----------------------------------------------------------------------------
# Sequential forward (Alg. 1), SNLP iteration (Alg. 2), residual (Eq. (2))
# ----------------------------------------------------------------------------

def default_mode(model: Model) -> int:
    return HCN if model.n_streams > 1 else IDN


def sequential_forward(model: Model, X0: np.ndarray, mode: Optional[int] = None) -> np.ndarray:
    """Alg. 1: h_l = f_l(h_{l-1}), l = 1..L.  Returns the trace [L+1, M, n, d] fp32.
    `mode` selects the layer map on an HC model (HCN: mixing by H_l; IDN: H_l = I)."""
    mode = default_mode(model) if mode is None else mode
    X0 = np.asarray(X0, dtype=f32)
    tr = np.empty((model.L + 1,) + X0.shape, dtype=f32)
    tr[0] = X0
    for l in range(1, model.L + 1):
        g = branch_output(model, l, tr[l - 1])
        tr[l] = layer_step(model, l, tr[l - 1], g, mode)
    return tr


INIT_H0 = 0
INIT_FWD = 1


def init_trace(model: Model, X0: np.ndarray, S: int = 0, mode: Optional[int] = None, init: int = INIT_H0) -> np.ndarray:
    """Alg. 2 up to the start of the solver loop: the first S layers are evaluated sequentially
    (h_l = f_l(h_{l-1}), l = 1..S), then every suffix state is initialised
      INIT_H0:  h_{S+j} = h_S                       (the "h0" configurations of Alg. 2)
      INIT_FWD: h_{S+j} = f_{S+j}(h_S)              (one-shot parallel forward from the prefix state;
                                                     Methods, "Inference With Fusion and Chunking")."""
    mode = default_mode(model) if mode is None else mode
    X0 = np.asarray(X0, dtype=f32)
    tr = np.empty((model.L + 1,) + X0.shape, dtype=f32)
    tr[0] = X0
    for l in range(1, S + 1):
        tr[l] = layer_step(model, l, tr[l - 1], branch_output(model, l, tr[l - 1]), mode)
    for l in range(S + 1, model.L + 1):
        if init == INIT_H0:
            tr[l] = tr[S]
        else:
            tr[l] = layer_step(model, l, tr[S], branch_output(model, l, tr[S]), mode)
    return tr


def evaluate_branches(model: Model, trace: np.ndarray, S: int = 0) -> np.ndarray:
    """Eq. (4): every suffix layer l = S+1..L evaluated on the current estimate of its input;
    g_all [L, M, d] fp32 (rows of the prefix layers are zero and unused)."""
    g = np.zeros((model.L,) + (trace.shape[1], trace.shape[3]), dtype=f32)
    for l in range(S + 1, model.L + 1):
        g[l - 1] = branch_output(model, l, trace[l - 1])
    return g


def residual_sq(model: Model, trace: np.ndarray, g_all: np.ndarray, mode: int, S: int = 0) -> np.ndarray:
    """r_l^2 = || X_l - f_l(X_{l-1}) ||_F^2 for l = S+1..L (Eq. (2)), with f_l applied as layer_step
    (fp32) to the given branch outputs and the squares accumulated in fp64 (prefix entries are 0)."""
    r = np.zeros(model.L, dtype=f64)
    for l in range(S + 1, model.L + 1):
        f = layer_step(model, l, trace[l - 1], g_all[l - 1], mode)
        diff = trace[l].astype(f64) - f.astype(f64)
        r[l - 1] = np.sum(diff * diff)
    return r


def iterate(model: Model, trace: np.ndarray, mode: int, K: int,
            keep: bool = False, S: int = 0) -> Tuple[np.ndarray, np.ndarray, List[np.ndarray]]:
    """K rounds of (parallel evaluation, structured correction) on `trace` (Alg. 2 inner loop) over
    the suffix layers S+1..L; slots 0..S stay fixed.

    Returns (new trace, probe [K, 2, L] fp64, [trace after each round] if keep).
    probe[k, 0, l-1] = r_l^2 of the trace ENTERING round k (free: its branch outputs are the ones
    the round evaluates); probe[k, 1, l-1] = || X_l^{k+1} - X_l^{k} ||_F^2.
    """
    trace = np.asarray(trace, dtype=f32)
    probe = np.zeros((K, 2, model.L), dtype=f64)
    kept: List[np.ndarray] = []
    for k in range(K):
        g_all = evaluate_branches(model, trace, S)
        probe[k, 0] = residual_sq(model, trace, g_all, mode, S)
        new = correction_scan(model, trace[0], g_all, mode, S, trace)
        dlt = new[1:].astype(f64) - trace[1:].astype(f64)
        probe[k, 1] = np.sum(dlt * dlt, axis=(1, 2, 3))
        trace = new
        if keep:
            kept.append(new)
    return trace, probe, kept


def iterate_skipping_converged(model: Model, trace: np.ndarray, mode: int, K: int, S: int = 0,
                               exact: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """The same K rounds with the layers that are already exact left out.  By induction on Eq. (5) a layer whose
    input equals the sequential state gets a zero correction and becomes exact, and never changes afterwards: k rounds
    after an initialisation make layers S+1..S+k exact (`exact` = number of leading exact layers of `trace`, S for the
    "h0" initialisation, S+1 after the one-shot forward).  Round k is therefore a round of `iterate` with the prefix
    moved to the exact layers (at least the last layer is always worked on).  Returns (trace, probe [K, 2, L])."""
    trace = np.asarray(trace, dtype=f32)
    exact = S if exact is None else exact
    probe = np.zeros((K, 2, model.L), dtype=f64)
    for k in range(K):
        trace, pr, _ = iterate(model, trace, mode, 1, S=min(max(exact, S), model.L - 1))
        probe[k] = pr[0]
        exact = min(max(exact, S) + 1, model.L)
    return trace, probe


def residual_norm(model: Model, trace: np.ndarray, mode: Optional[int] = None) -> np.ndarray:
    """r_l = || G_l(trace) ||_F, l = 1..L, at the cost of one evaluation of every branch."""
    mode = default_mode(model) if mode is None else mode
    trace = np.asarray(trace, dtype=f32)
    return np.sqrt(residual_sq(model, trace, evaluate_branches(model, trace), mode))


# ----------------------------------------------------------------------------
# Chunkwise fused layers (Methods, "Layer fusion" / "Chunkwise strategy"; Appendix "Fused Cross-Layer Coupling")
# ----------------------------------------------------------------------------

def fused_chunk_output(model: Model, c: int, F: int, h: np.ndarray) -> np.ndarray:
    """g_C(h) for chunk c (1-based) of F consecutive layers that all read the same input h [M, d]:
        a_C = sum_{l in C} O_l Attn_l(Q_l h, K_l h, V_l h);   u_C = h + a_C;
        m_C = sum_{l in C} P_l phi(W_l Norm(u_C));            F_C(h) = u_C + m_C = h + g_C(h).
    Evaluated in fp64; a_C and m_C are rounded to fp32 once each and g_C = a_C (+) m_C in fp32.
    Single-stream models."""
    h = np.asarray(h, dtype=f64)
    layers = range((c - 1) * F + 1, c * F + 1)
    a_C = np.zeros_like(h)
    for l in layers:
        a_C = a_C + attn_update(model, l, h)
    m_C = np.zeros_like(h)
    for l in layers:
        m_C = m_C + mlp_update(model, l, h + a_C)
    return a_C.astype(f32) + m_C.astype(f32)


def fused_sequential_forward(model: Model, X0: np.ndarray, F: int) -> np.ndarray:
    """The fused model executed chunk after chunk: h_c = h_{c-1} (+) g_C(h_{c-1}); trace [L/F + 1, M, 1, d]."""
    N = model.L // F
    X0 = np.asarray(X0, dtype=f32)
    tr = np.empty((N + 1,) + X0.shape, dtype=f32)
    tr[0] = X0
    for c in range(1, N + 1):
        tr[c] = tr[c - 1] + fused_chunk_output(model, c, F, tr[c - 1][:, 0, :])[:, None, :]
    return tr


def fused_iterate(model: Model, trace: np.ndarray, F: int, K: int, keep: bool = False):
    """Chunkwise SNLP with the identity surrogate: all chunks evaluated on the current chunk-input estimates,
    then h_c^{k+1} = F_C(h_{c-1}^k) + (h_{c-1}^{k+1} - h_{c-1}^k), in prefix form h_c = h_{c-1} (+) g_C.
    trace [L/F + 1, M, 1, d].  Returns (trace, probe [K, 2, L/F], kept)."""
    N = model.L // F
    trace = np.asarray(trace, dtype=f32)
    probe = np.zeros((K, 2, N), dtype=f64)
    kept = []
    for k in range(K):
        g = np.stack([fused_chunk_output(model, c, F, trace[c - 1][:, 0, :]) for c in range(1, N + 1)])
        new = np.empty_like(trace)
        new[0] = trace[0]
        for c in range(1, N + 1):
            f = trace[c - 1] + g[c - 1][:, None, :]
            probe[k, 0, c - 1] = np.sum((trace[c].astype(f64) - f.astype(f64)) ** 2)
            new[c] = new[c - 1] + g[c - 1][:, None, :]
        probe[k, 1] = np.sum((new[1:].astype(f64) - trace[1:].astype(f64)) ** 2, axis=(1, 2, 3))
        trace = new
        if keep:
            kept.append(new)
    return trace, probe, kept


# ----------------------------------------------------------------------------
# Cross-checks used only by the oracle's own tests
# ----------------------------------------------------------------------------

def full_layer(model: Model, l: int, X_prev: np.ndarray, mode: int) -> np.ndarray:
    """f_l(X_{l-1}) in fp64 (no fp32 rounding): residual mixing plus post-weighted branch."""
    X = np.asarray(X_prev, dtype=f64)
    a, m = branch(model, l, premix(model, l, X))
    g = a + m
    n = model.n_streams
    if n == 1:
        return X + g[:, None, :]
    p = np.asarray(model.post[l - 1], dtype=f64)
    Hm = np.eye(n) if mode == IDN else np.asarray(model.Hres[l - 1], dtype=f64)
    return np.einsum("ij,mjc->mic", Hm, X) + p[None, :, None] * g[:, None, :]


def iterate_delta_form(model: Model, trace: np.ndarray, mode: int, K: int) -> np.ndarray:
    """The literal update of Alg. 2 / Eq. (5) in fp64:
    h_l^{k+1} = f_l(h_{l-1}^k) + A_l (h_{l-1}^{k+1} - h_{l-1}^k), with A = I or H_l."""
    cur = np.asarray(trace, dtype=f64)
    n = model.n_streams
    for _ in range(K):
        tilde = [full_layer(model, l, cur[l - 1], mode) for l in range(1, model.L + 1)]
        new = np.empty_like(cur)
        new[0] = cur[0]
        for l in range(1, model.L + 1):
            delta = new[l - 1] - cur[l - 1]
            if n > 1 and mode == HCN:
                delta = np.einsum("ij,mjc->mic", np.asarray(model.Hres[l - 1], dtype=f64), delta)
            new[l] = tilde[l - 1] + delta
        cur = new
    return cur


def iterate_no_correction(model: Model, trace: np.ndarray, mode: int, K: int) -> np.ndarray:
    """Naive parallel fixed point h_l^{k+1} = f_l(h_{l-1}^k) (no correction), fp64; it advances
    information by one layer per round (Methods, "Effect of the correction")."""
    cur = np.asarray(trace, dtype=f64)
    for _ in range(K):
        new = np.empty_like(cur)
        new[0] = cur[0]
        for l in range(1, model.L + 1):
            new[l] = full_layer(model, l, cur[l - 1], mode)
        cur = new
    return cur
