"""CPU oracle for block-wise predictive FFN sparsity in LLM prefill.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check
and the benchmark's CPU-baseline leg may import it; the GPU library never does
and shares no code, table or helper with it.

It is a plain, slow, fp64 numpy transcription of what the paper defines, one
block of prompt tokens at a time, in the paper's order of steps:

  Sec. 3.1            the prompt is cut into blocks of N_block tokens
  Sec. 3.2, Eq. 12    a = Softmax(q_pred X^T / sqrt(d_model)) X     (pooling)
  Sec. 3.2, Eq. 13    s = ReLU(a W_pred1) W_pred2                   (scores)
  Sec. 3.2, Eq. 14    M_j = 1 iff s_j is among the top-K scores     (mask)
  Sec. 3.2, Eq. 15-17 SelectRows / SelectCols of the FFN weights    (gather)
  Sec. 3.2, Eq. 18    FFN^ = W^down (sigma(W^gate X) * (W^up X))    (sparse FFN)
  Sec. 3.3, Eq. 20-21 Y = FFN^ + W_comp2 sigma(W_comp1 X)           (compensation)
  Sec. 2,   Eq. 10    Y = [sigma(X W_gate) * (X W_up)] W_down       (dense FFN)
  Sec. 3.4, Alg. 1    layer-wise budget allocation                  (schedule)

All arithmetic is float64 on the exact values of the (bf16) inputs; there is no
blocking, fusion or reordering beyond what those equations state.  A numpy
matmul or sort serves as a step where the equation is a matmul or a ranking.

Readings taken where the paper is silent (each is also listed in the design
notes of the repository):
  * tokens are rows (x_t is 1 x d_model); Eq. 18/20 are written column-style in
    the paper, Eq. 10/13 row-style - the same maps.
  * W_gate, W_up are d_ffn x d_model and W_down is d_model x d_ffn, as Eq. 15-17
    select rows of the first two and columns of the third.
  * sigma of the FFN is SiLU (the Llama/Qwen gated FFN); sigma of the
    compensator is SiLU unless another activation is asked for.
  * q_pred = None means mean pooling, which is Eq. 12 at q_pred = 0.
  * top-K ties go to the lower neuron index; the selected set is returned in
    ascending index order.
  * K = clamp(floor((1 - sparsity) * d_ffn + 0.5), 1, d_ffn).
  * a prompt whose length is not a multiple of the block size ends in a short
    block.

Pins (tests/test_oracle_pins.py): every function here is pinned to something
other than itself - closed forms, brute force on tiny inputs, hand-worked
examples, library routines (torch fp64, scipy) on tie-free data, invariants.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

F64 = np.float64


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------
# scalar helpers
# --------------------------------------------------------------------------

def k_from_sparsity(d_ffn: int, sparsity: float) -> int:
    """Number of neurons kept at a given sparsity (reading: round half up,
    at least one neuron, at most all)."""
    k = int(np.floor((1.0 - float(sparsity)) * d_ffn + 0.5))
    return max(1, min(int(d_ffn), k))


def silu(v: np.ndarray) -> np.ndarray:
    """SiLU(v) = v / (1 + exp(-v)), the gate activation of a SwiGLU FFN."""
    v = _f64(v)
    with np.errstate(over="ignore"):
        return v / (1.0 + np.exp(-v))


def activation(name: str, v: np.ndarray) -> np.ndarray:
    if name == "silu":
        return silu(v)
    if name == "relu":
        return np.maximum(_f64(v), 0.0)
    if name == "identity":
        return _f64(v)
    raise ValueError(f"unknown activation {name!r}")


def bf16_round(v: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bf16, returned as float64 values (used only
    where the layer stack stores activations as bf16 between layers)."""
    f = np.ascontiguousarray(v, dtype=np.float32)
    u = f.view(np.uint32)
    u = (u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(F64)


# --------------------------------------------------------------------------
# Sec. 3.2: expert neuron predictor
# --------------------------------------------------------------------------

def pool_block(xb: np.ndarray, q_pred: Optional[np.ndarray]) -> np.ndarray:
    """Eq. 12: single-query attention pooling of one block.

    xb is N_block x d_model.  Tokens are keys and values, q_pred the query.
    q_pred None = mean pooling (softmax of a constant)."""
    xb = _f64(xb)
    n, d_model = xb.shape
    if q_pred is None:
        p = np.full(n, 1.0 / n, dtype=F64)
    else:
        z = (xb @ _f64(q_pred)) / np.sqrt(F64(d_model))
        e = np.exp(z - z.max())
        p = e / e.sum()
    return p @ xb


def predictor_scores(xb, q_pred, w1, w2) -> np.ndarray:
    """Eq. 12-13: s = ReLU(a W_pred1) W_pred2 for one block, a from Eq. 12.
    w1 is d_model x r, w2 is r x d_ffn."""
    a = pool_block(xb, q_pred)
    hidden = np.maximum(a @ _f64(w1), 0.0)
    return hidden @ _f64(w2)


def select_topk(scores: np.ndarray, k: int) -> np.ndarray:
    """Eq. 14: indices j with M_j = 1, i.e. the K highest scores; equal scores
    are ranked by lower index first.  Returned ascending (int32).

    Brute force: rank all neurons by (score descending, index ascending) with a
    full sort and keep the first K."""
    s = _f64(scores)
    d_ffn = s.shape[0]
    if not 1 <= k <= d_ffn:
        raise ValueError("k out of range")
    neg = -s
    neg = neg + 0.0                      # -0.0 and +0.0 rank as equal
    order = np.lexsort((np.arange(d_ffn), neg))   # primary key: -score, then index
    return np.sort(order[:k]).astype(np.int32)


def selection_margin(scores: np.ndarray, k: int) -> float:
    """s_(K) - s_(K+1) of the descending-sorted scores (inf when K = d_ffn):
    how far the selection is from a tie at the threshold."""
    s = np.sort(_f64(scores))[::-1]
    if k >= s.shape[0]:
        return float("inf")
    return float(s[k - 1] - s[k])


# --------------------------------------------------------------------------
# Sec. 3.2 / 3.3: sparse FFN and compensator, Sec. 2: dense FFN
# --------------------------------------------------------------------------

def sparse_ffn_block(xb, w_gate, w_up, w_down, idx) -> np.ndarray:
    """Eq. 15-18 for one block: gather rows idx of W_gate, W_up (d_ffn x
    d_model) and columns idx of W_down (d_model x d_ffn), then
    FFN^(X) = (SiLU(X W^gate^T) * (X W^up^T)) W^down^T."""
    xb = _f64(xb)
    idx = np.asarray(idx, dtype=np.int64)
    wg_hat = _f64(np.asarray(w_gate)[idx, :])        # Eq. 16, K x d_model
    wu_hat = _f64(np.asarray(w_up)[idx, :])          # Eq. 15, K x d_model
    wd_hat = _f64(np.asarray(w_down)[:, idx])        # Eq. 17, d_model x K
    act = silu(xb @ wg_hat.T) * (xb @ wu_hat.T)      # N_block x K
    return act @ wd_hat.T                            # N_block x d_model


def compensator_block(xb, wc1, wc2, act: str = "silu") -> np.ndarray:
    """Eq. 20: Y_comp = sigma(X W_comp1) W_comp2, wc1 d_model x r', wc2 r' x
    d_model.  Does not see the mask."""
    return activation(act, _f64(xb) @ _f64(wc1)) @ _f64(wc2)


def dense_ffn(x, w_gate, w_up, w_down) -> np.ndarray:
    """Eq. 10: Y = [SiLU(X W_gate) * (X W_up)] W_down with every neuron, written
    with the same operand shapes as the sparse form (W_gate, W_up: d_ffn x
    d_model, applied as X W^T; W_down: d_model x d_ffn)."""
    x = _f64(x)
    g = x @ _f64(w_gate).T
    u = x @ _f64(w_up).T
    return (silu(g) * u) @ _f64(w_down).T


# --------------------------------------------------------------------------
# one layer over a whole prompt
# --------------------------------------------------------------------------

@dataclass
class LayerResult:
    y: Optional[np.ndarray]            # T x d_model float64 (None if ffn skipped)
    indices: List[np.ndarray]          # per block, ascending int32
    margins: List[float]               # per block selection margin
    score_absmax: List[float]          # per block max |s|
    macs_predictor: int = 0
    macs_ffn: int = 0
    macs_comp: int = 0
    scores: Optional[List[np.ndarray]] = None


def block_ranges(n_tokens: int, block: int):
    """Sec. 3.1: consecutive blocks of `block` tokens; the last may be short."""
    return [(t0, min(n_tokens, t0 + block)) for t0 in range(0, n_tokens, block)]


def fastforward_layer(x, w_gate, w_up, w_down, w1, w2, block: int,
                      k_per_block: Sequence[int], q_pred=None,
                      wc1=None, wc2=None, comp_act: str = "silu",
                      indices_override: Optional[Sequence[np.ndarray]] = None,
                      compute_ffn: bool = True, blocks: Optional[Sequence[int]] = None,
                      keep_scores: bool = False) -> LayerResult:
    """Sec. 3.1-3.3 on one layer: for every block predict -> top-K -> sparse FFN
    -> + compensation.  `blocks` restricts the FFN part to some blocks (the
    selection is always done for all); rows of y for the others stay NaN."""
    x = np.asarray(x)
    n_tokens, d_model = x.shape
    ranges = block_ranges(n_tokens, block)
    if len(k_per_block) != len(ranges):
        raise ValueError("k_per_block must have one entry per block")
    res = LayerResult(y=None, indices=[], margins=[], score_absmax=[],
                      scores=[] if keep_scores else None)
    if compute_ffn:
        res.y = np.full((n_tokens, d_model), np.nan, dtype=F64)
    r = np.asarray(w1).shape[1]
    d_ffn = np.asarray(w2).shape[1]
    for b, (t0, t1) in enumerate(ranges):
        xb = _f64(x[t0:t1])
        k = int(k_per_block[b])
        if indices_override is None:
            s = predictor_scores(xb, q_pred, w1, w2)
            idx = select_topk(s, k)
            res.margins.append(selection_margin(s, k))
            res.score_absmax.append(float(np.abs(s).max()))
            if keep_scores:
                res.scores.append(s)
            res.macs_predictor += (t1 - t0) * d_model + d_model * r + r * d_ffn
        else:
            idx = np.asarray(indices_override[b], dtype=np.int32)
        res.indices.append(idx)
        if not compute_ffn or (blocks is not None and b not in blocks):
            continue
        yb = sparse_ffn_block(xb, w_gate, w_up, w_down, idx)
        res.macs_ffn += 3 * (t1 - t0) * d_model * len(idx)
        if wc1 is not None:
            yb = yb + compensator_block(xb, wc1, wc2, comp_act)      # Eq. 21
            res.macs_comp += 2 * (t1 - t0) * d_model * np.asarray(wc1).shape[1]
        res.y[t0:t1] = yb
    return res


# --------------------------------------------------------------------------
# layer stack glue (pre-norm residual stack around the FFN path)
# --------------------------------------------------------------------------

def rmsnorm_rows(h, eps: float) -> np.ndarray:
    """x_t = h_t / sqrt(mean_c(h_t,c^2) + eps), gain 1."""
    h = _f64(h)
    return h / np.sqrt((h * h).mean(axis=1, keepdims=True) + eps)


def stack_layer(h, layer_weights: dict, block: int, k_per_block, eps: float,
                comp_act: str = "silu", blocks=None):
    """One layer of the stack: x = bf16(RMSNorm(h)); y = layer(x);
    h' = bf16(h + y).  Activations between layers are stored as bf16."""
    x = bf16_round(rmsnorm_rows(h, eps))
    res = fastforward_layer(x, block=block, k_per_block=k_per_block,
                            comp_act=comp_act, blocks=blocks, **layer_weights)
    h_next = bf16_round(_f64(h) + res.y)
    return x, res, h_next


# --------------------------------------------------------------------------
# Sec. 3.4, Alg. 1: layer-wise budget allocation
# --------------------------------------------------------------------------

def layerwise_budgets(importance: Sequence[float], budget: float) -> np.ndarray:
    """Alg. 1: the total budget B*L is handed out layer by layer in proportion
    to the importance still unassigned, each layer's share capped at 1.
    b_i is the fraction of neurons layer i keeps (sparsity_i = 1 - b_i)."""
    s = [float(v) for v in importance]
    n_layers = len(s)
    total = float(budget) * n_layers
    s_total = float(sum(s))
    out = []
    for i in range(n_layers):
        b_i = min(1.0, s[i] / s_total * total)
        total -= b_i
        s_total -= s[i]
        out.append(b_i)
    return np.array(out, dtype=F64)
