"""Per-stage parity metric and cases, shared by the GPU stage tests and by the CPU test that shows these checks
notice planted mistakes.  Oracle side only: nothing here touches the HIP library.

Why per stage: with weights N(0, 0.02^2) the attention update is a few percent of the hidden state, so a bound on
the state cannot see the attention kernels.  Each stage output of one batched evaluation (Eq. (4)) is therefore
compared with the oracle RELATIVE TO ITS OWN NORM, token row by token row, and the maximum over rows is bounded by

    u     branch input sum_j pre[j] X[j] (n > 1), fp32 on both sides                       1e-6
    qk    rotated + normalised q and k rows per head (where the rotation is a pass of its own)  1e-2
    v     value rows per head                                                                  1e-2
    attn  heads' outputs before the output projection                                          2e-2
    a     attention update (fp32 out)                                                          2e-2
    m     MLP update g - a (fp32 out)                                                          1e-2

Where the bf16 bounds come from.  Every operand the kernels round to bf16 carries a relative error of at most 2^-9
per element (about 1.1e-3 rms; a 128-long row of such errors measures 2.7e-3 at worst over the rows of a case).
q / k / v rows, and an MLP update (normalised input, hidden activations, two long contractions in which the
errors add in quadrature) stay at 3e-3..4e-3 per row: bound 1e-2.  A head's output does not average when few keys
carry it (the first block rows behind a prefix whose values are zero; a single key): the error of a score,
sigma = 2.2e-3 from the two roundings each of q and k (after the QKV GEMM, after rotation + norm), enters the
probability as a relative error common to all 128 channels, as does the probability's own rounding (<= 3.9e-3), on
top of the roundings of v and of the output (3.8e-3 together): 4 sigma + 3.9e-3 + 3.8e-3 = 1.65e-2, bound 2e-2
(observed: up to 1.2e-2 on such rows, 4e-3..5e-3 where many keys contribute).  The attention update inherits the
row error of the heads' outputs through the output projection.  Every planted indexing, masking or rotation mistake
moves the same quantities by 4e-2 to 10 (test_stage_check_teeth.py)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, Optional, Sequence

import numpy as np

import snlp_inputs as si
from oracle import snlp_oracle as oc
from oracle.harness import oracle_model

TOL_STAGE = 1e-2
TOL_ATTN = 2e-2
TOL_U = 1e-6


def row_rel_err(x: np.ndarray, ref: np.ndarray) -> float:
    """max over rows (last axis = one row) of ||x - ref|| / ||ref||, fp64.  Rows whose reference is exactly zero
    must be exactly zero."""
    x = np.asarray(x, dtype=np.float64).reshape(-1, x.shape[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, ref.shape[-1])
    num = np.linalg.norm(x - ref, axis=-1)
    den = np.linalg.norm(ref, axis=-1)
    zero = den == 0
    if np.any(zero & (num != 0)):
        return float("inf")
    return float(np.max(num[~zero] / den[~zero])) if np.any(~zero) else 0.0


@dataclass
class StageCase:
    name: str
    shape: si.Shape
    zero_vpre: bool = False            # output carried by the block's own keys only
    distinct_streams: bool = False     # n > 1: perturb h0 per stream so that the pre-mix is visible
    layers: Optional[Sequence[int]] = None   # 1-based layers to compare (None: all)
    second_state: bool = True          # also evaluate at the oracle's K = 1 trace (distinct layer inputs)

    def tensors(self) -> Dict[str, np.ndarray]:
        t = si.generate(self.shape)
        if self.zero_vpre:
            t["Vpre"] = np.zeros_like(t["Vpre"])
        if self.distinct_streams:
            rng = np.random.default_rng(self.shape.seed + 77)
            t["h0"] = (t["h0"] + rng.standard_normal(t["h0"].shape).astype(np.float32)).astype(np.float32)
        return t


def small(name, **kw) -> si.Shape:
    base = dict(L=2, d=256, n_heads=2, head_dim=128, d_mlp=512, B=2, T=8, P=0, n_streams=1, bf16=True, seed=900)
    base.update(kw)
    return si.Shape(name, **base)


# Small cases: every decode-kernel and block-kernel path, cheap enough for the CPU-only teeth test as well.
SMALL_CASES = [
    StageCase("block_T200_P37", small("block_T200_P37", B=1, T=200, P=37, seed=901)),
    StageCase("block_T40_P0", small("block_T40_P0", T=40, seed=902)),
    # 8 query tiles per stream: the stream-major workgroup order, a ragged last tile, a prefix that ends inside a key step
    StageCase("block_T1000_P37", small("block_T1000_P37", B=1, T=1000, P=37, seed=911), layers=(2,), second_state=False),
    # prefix and block both made of whole key steps (the linear-address load paths)
    StageCase("block_T130_P96", small("block_T130_P96", T=130, P=96, seed=912)),
    StageCase("decode_T1_P0", small("decode_T1_P0", T=1, seed=903)),
    StageCase("decode_T5_P70", small("decode_T5_P70", B=3, T=5, P=70, seed=904)),
    # decode kernel with its own rotation of q and of the block's k rows (P >= 512, T <= 16)
    StageCase("decode_P512_T16", small("decode_P512_T16", T=16, P=512, seed=905)),
    StageCase("decode_P512_T16_v0", small("decode_P512_T16_v0", T=16, P=512, seed=905), zero_vpre=True),
    StageCase("decode_P523_T5", small("decode_P523_T5", T=5, P=523, seed=906)),                      # P mod 32 = 11
    StageCase("decode_P523_T5_v0", small("decode_P523_T5_v0", T=5, P=523, seed=906), zero_vpre=True),
    StageCase("decode_P999_T16", small("decode_P999_T16", B=1, T=16, P=999, seed=907)),              # P mod 32 = 7: block rows straddle two tiles
    StageCase("decode_P999_T16_v0", small("decode_P999_T16_v0", B=1, T=16, P=999, seed=907), zero_vpre=True),
    StageCase("decode_P2048_T8_v0", small("decode_P2048_T8_v0", T=8, P=2048, seed=908), zero_vpre=True),
    # 81 key tiles, the last one made of block rows 1..15 only: query row 0 sees none of its keys
    StageCase("decode_P2559_T16", small("decode_P2559_T16", B=1, T=16, P=2559, seed=910)),
    StageCase("decode_P2559_T16_v0", small("decode_P2559_T16_v0", B=1, T=16, P=2559, seed=910), zero_vpre=True),
    StageCase("hcn_n4_T33", small("hcn_n4_T33", T=33, n_streams=4, L=3, seed=909), distinct_streams=True),
]

# Block lengths and prefix lengths around the block kernel's step (32 keys), query tile (128 rows) and load paths
# (GPU test only; one layer each).
def _edge(T, P, seed):
    name = "block_T%d_P%d" % (T, P)
    return StageCase(name, small(name, L=1, B=1, T=T, P=P, seed=seed), second_state=False)


EDGE_CASES = [_edge(T, P, 920 + i) for i, (T, P) in enumerate([
    (17, 0), (31, 1), (32, 32), (33, 31), (63, 64), (64, 33), (65, 95), (127, 0), (128, 64), (129, 63), (255, 1), (257, 160)])]

# Deep, narrow prefill models whose layer-batched GEMM launches end in an incomplete round of 256 x 256 tiles, with
# M = 600 rows (2.3 row tiles) and output widths of 2.5, 7.5 and 5.25 column tiles: d = 640, d_mlp = 1344, so O / PROJ
# have 9 tiles per layer, QKV 24, FC 18.  30 layers: O / PROJ 270 tiles and FC 540, remainders 14 and 28 (cut into
# 128 x 64 pieces; QKV 720, remainder 208, stays whole).  34 layers: O / PROJ 306 and QKV 816, remainders 50 and 48
# (128 x 128 pieces), FC 612, remainder 100 (256 x 128 halves, and the half-empty last column tile runs as a half).
# The remainder's tiles are the last in launch order, so the last two layers are compared, and the first.
def _tail(name, L, seed):
    shp = si.Shape(name, L=L, d=640, n_heads=5, head_dim=128, d_mlp=1344, B=3, T=200, P=0, n_streams=1, bf16=True, seed=seed)
    return StageCase(name, shp, layers=(1, L - 1, L), second_state=False)


TAIL_CASES = [_tail("gemm_tail_L30", 30, 940), _tail("gemm_tail_L34", 34, 941)]

# Decode launches of more than 512 (layer, sequence, head) items, where the workgroups of the first round also touch
# the block rows of later ones: 576 and 1300 items (neither a multiple of 512), 5 and 16 block rows, prefixes that do
# not end on a tile boundary (GPU test only; the layers whose items are touched, and the first, are compared).
def _touch(name, L, B, T, P, seed, layers):
    return StageCase(name, small(name, L=L, B=B, T=T, P=P, seed=seed), layers=layers, second_state=False)


DECODE_MANY_ITEMS_CASES = [
    _touch("decode_576_items_T5_P523", 24, 12, 5, 523, 950, (1, 22, 24)),
    _touch("decode_1300_items_T16_P70", 50, 13, 16, 70, 951, (1, 21, 41, 50)),
]

# The benchmark workloads at full size (GPU test only).
FULL_CASES = [
    StageCase("d20_decode_T8", si.config(3, T=8)),
    StageCase("d20_decode_T4", si.config(3, T=4), second_state=False),
    StageCase("d20_decode_T1", si.config(3, T=1), second_state=False),
    StageCase("d20_hcn", si.config(4), distinct_streams=True, layers=(1, 7, 20), second_state=False),
]


def oracle_stages(md: oc.Model, l: int, X_prev: np.ndarray) -> Dict[str, np.ndarray]:
    """The stage outputs of layer l (1-based) at the state X_prev [M, n, d], in fp64:
    u [M, d]; q, k, v [M, H, dh] (q, k rotated and normalised); attn [M, d]; a [M, d]; m [M, d]."""
    u = oc.premix(md, l, X_prev)
    q, k, v = oc.qkv_heads(md, l, u)
    rows = lambda x: x.transpose(0, 2, 1, 3).reshape(md.B * md.T, md.n_heads, md.head_dim)
    attn = oc.attn_heads(md, l, u)
    a = attn @ np.asarray(md.Wo[l - 1], dtype=np.float64)
    m = oc.mlp_update(md, l, u + a)
    return {"u": u, "q": rows(q), "k": rows(k), "v": rows(v), "attn": attn, "a": a, "m": m}


def fro_rel_err(x: np.ndarray, ref: np.ndarray) -> float:
    """|| x - ref ||_F / || ref ||_F over the whole stage output, fp64."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


def compare_stages(got: Dict[str, np.ndarray], ref: Dict[str, np.ndarray], n_streams: int, rotated_qk: bool,
                   metric: Callable = None) -> Dict[str, float]:
    """Relative errors of the stage outputs present in `got` (same keys as oracle_stages); row-wise maximum by default."""
    metric = metric or row_rel_err
    out = {}
    if n_streams > 1 and "u" in got:
        out["u"] = metric(got["u"], ref["u"])
    if rotated_qk:
        out["q"] = metric(got["q"], ref["q"])
        out["k"] = metric(got["k"], ref["k"])
    out["v"] = metric(got["v"], ref["v"])
    for key in ("attn", "a", "m"):
        out[key] = metric(got[key], ref[key])
    return out


def tolerances() -> Dict[str, float]:
    return {"u": TOL_U, "q": TOL_STAGE, "k": TOL_STAGE, "v": TOL_STAGE, "attn": TOL_ATTN, "a": TOL_ATTN, "m": TOL_STAGE}


def tolerances_rounded() -> Dict[str, float]:
    """Bounds on the relative Frobenius error of a stage against the oracle run with round_bf16 (operands rounded to
    bf16 where the kernels round them).  q, k and v then differ only where fp32 and fp64 accumulation fall on two sides
    of a rounding boundary (observed: 0 to 2e-4), which makes this the tight check of the projection, the rotation
    and the norm.  The heads' outputs stay at 2e-3..4e-3: the kernels round the probabilities relative to a running
    reference exponent, which no oracle can reproduce, and the output's own bf16 rounding then differs by whole ulps."""
    return {"u": TOL_U, "q": 5e-4, "k": 5e-4, "v": 5e-4, "attn": 6e-3, "a": 6e-3, "m": 4e-3}


def model_of(case: StageCase, t: Dict[str, np.ndarray]) -> oc.Model:
    return oracle_model(case.shape, t, widen=case.shape.L * case.shape.d <= 4096)
