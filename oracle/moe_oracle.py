"""CPU oracle for one Mixture-of-Experts layer. TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module. The GPU library never does, and the two share no code.

What it computes is the MoE layer as the paper states it (Section 2.2): a gating
step scores every expert for every token, each token goes to its top-k experts,
every expert is a feed-forward network, and the layer output is the weighted sum
of the selected experts' outputs. The steps between (per-expert token counts,
normalised token weights, scattering tokens to their experts) are the ones the
paper's implementation section lists for its fused gating kernel (Section 6,
"Fused kernels"), and the expert FFN is the pair of GEMMs "FFN Input" and
"FFN Output" of the paper's GEMM table (Section 4.2, Table 3).

The method is exact (no approximation), so each function below is the plain
definition written out with numpy, in float64. Inputs are taken at their storage
precision: float arrays are used as they are; uint16 arrays are bfloat16 bit
patterns and are widened exactly. Nothing is rounded between steps.

Readings where the paper is silent (each is also pinned by a test):
  * top-k ties go to the lower expert index; a token's k picks are listed in
    descending-logit order
  * "normalised token weights" = softmax over the k selected logits
  * rows inside one expert's segment keep ascending flat assignment order t*k+j
  * experts are SwiGLU FFNs: y = (silu(x Wg^T) * (x Wu^T)) Wd^T, no biases;
    the paper's "FFN Input" GEMM is read as the fused [gate | up] projection
  * no capacity limit: every assignment is processed
Precondition: logits hold no NaN.

Parity pins: every function here is pinned by tests/test_oracle_pins.py against
brute force, closed forms, library routines and invariants. The paper prints no
activations or outputs, so beyond those pins the FFN values are not pinned by
paper-printed numbers.
"""
from __future__ import annotations

import numpy as np


def widen(a: np.ndarray) -> np.ndarray:
    """Storage type -> float64, exactly. uint16 is read as bfloat16 bits."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def gate_logits(x: np.ndarray, w_r: np.ndarray) -> np.ndarray:
    """Gating scores (Section 2.2): logits[t, e] = <x[t, :], W_r[e, :]>, rounded once to float32.

    The router consumes float32 logits; both the oracle and the GPU path route the
    same logits bytes, which is what makes bit-exact routing well defined.
    """
    return (widen(x) @ widen(w_r).T).astype(np.float32)


def route(logits: np.ndarray, k: int):
    """Top-k selection, normalised weights and per-expert counts (Section 2.2; Section 6 "Fused kernels").

    Returns
      topk_idx[T, k] int32   the k experts with the largest logits, largest first,
                             equal logits ordered by ascending expert index
      topk_w[T, k]  float64  softmax over those k logits
      counts[E]     int32    assignments per expert
      offsets[E+1]  int32    exclusive prefix sum of counts; offsets[E] = T*k
    """
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    # The definition of "k largest, ties to the lower index, in descending order":
    # a stable sort by descending value keeps equal values in index order.
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")
    topk_idx = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(logits.astype(np.float64), topk_idx.astype(np.int64), axis=1)
    p = np.exp(sel - sel[:, :1])          # the first pick is the row maximum
    topk_w = p / p.sum(axis=1, keepdims=True)
    counts = np.zeros(E, dtype=np.int32)
    for e in topk_idx.reshape(-1):
        counts[e] += 1
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    return topk_idx, topk_w, counts, offsets


def dispatch(x: np.ndarray, topk_idx: np.ndarray, offsets: np.ndarray):
    """Put every token's row into an expert-contiguous buffer, once per expert it was routed to
    (Section 2.2: tokens go to their experts; Section 6 "Fused kernels": the scatter step).

    Assignments are visited in flat order i = t*k + j; each takes the next free row of
    its expert's segment [offsets[e], offsets[e+1]).

    Returns
      xp[A, d]   row r is a copy (same storage type) of the token that owns row r
      pos[T, k]  int32  row of assignment (t, j)
      src[A]     int32  flat assignment index t*k+j that owns row r
    """
    x = np.asarray(x)
    topk_idx = np.asarray(topk_idx)
    T, k = topk_idx.shape
    A = T * k
    cursor = [int(v) for v in offsets[:-1]]
    pos = np.zeros((T, k), dtype=np.int32)
    src = np.zeros(A, dtype=np.int32)
    xp = np.zeros((A, x.shape[1]), dtype=x.dtype)
    for i in range(A):
        t, j = divmod(i, k)
        e = int(topk_idx[t, j])
        r = cursor[e]
        cursor[e] = r + 1
        pos[t, j] = r
        src[r] = i
        xp[r, :] = x[t, :]
    return xp, pos, src


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float64 values rounded to the nearest bfloat16 (ties to even) via float32, returned as float64.
    Diagnostic only (see expert_ffn's `store_bf16`): it mimics where a bf16 implementation stores."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def expert_ffn(xp: np.ndarray, offsets: np.ndarray, expert_weights, return_h: bool = False, store_bf16: bool = False):
    """Per-expert SwiGLU FFN over the expert-contiguous rows (Section 4.2, Table 3: "FFN Input"
    (b_e, h) x (h, h') and "FFN Output" (b_e, h') x (h', h), with tensor-parallel degree 1).

    expert_weights(e) -> (W_gate[f, d], W_up[f, d], W_down[d, f]) for expert e, or a sequence
    indexed by e. Experts with no rows are never asked for their weights.

      h[r, :] = silu(xp[r, :] W_gate_e^T) * (xp[r, :] W_up_e^T)
      y[r, :] = h[r, :] W_down_e^T              for r in expert e's segment

    store_bf16=True is a diagnostic, not the definition: h and y are rounded to bfloat16 where a bf16
    implementation stores them, so that what is left of a comparison is accumulation order alone.

    Returns y[A, d] float64 (and h[A, f] float64 if return_h).
    """
    get = expert_weights if callable(expert_weights) else (lambda e: expert_weights[e])
    E = len(offsets) - 1
    A, d = xp.shape
    y = np.zeros((A, d), dtype=np.float64)
    h_all = None
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        w_gate, w_up, w_down = get(e)
        rows = widen(xp[lo:hi])
        g = rows @ widen(w_gate).T
        u = rows @ widen(w_up).T
        h = silu(g) * u
        if store_bf16:
            h = round_to_bf16(h)
        y[lo:hi] = round_to_bf16(h @ widen(w_down).T) if store_bf16 else h @ widen(w_down).T
        if return_h:
            if h_all is None:
                h_all = np.zeros((A, h.shape[1]), dtype=np.float64)
            h_all[lo:hi] = h
    return (y, h_all) if return_h else y


def expert_ffn_segments(xp: np.ndarray, seg_begin, seg_end, seg_expert, expert_weights, y=None):
    """The same per-expert FFN over explicit row ranges: slot s applies expert seg_expert[s] to
    rows [seg_begin[s], seg_end[s]). This is what one expert node runs when popular experts have
    several copies, each taking part of the expert's rows (Section 6, "Load balance").
    Rows outside every range are left as they are in `y` (zeros if y is None). Returns y float64."""
    get = expert_weights if callable(expert_weights) else (lambda e: expert_weights[e])
    A, d = xp.shape
    if y is None:
        y = np.zeros((A, d), dtype=np.float64)
    for lo, hi, e in zip(seg_begin, seg_end, seg_expert):
        lo, hi = int(lo), int(hi)
        if hi <= lo:
            continue
        w_gate, w_up, w_down = get(int(e))
        rows = widen(xp[lo:hi])
        h = silu(rows @ widen(w_gate).T) * (rows @ widen(w_up).T)
        y[lo:hi] = h @ widen(w_down).T
    return y


def combine(y: np.ndarray, pos: np.ndarray, topk_w: np.ndarray) -> np.ndarray:
    """Weighted sum of each token's k expert outputs (Section 2.2):
    out[t, :] = sum_j topk_w[t, j] * y[pos[t, j], :]. Returns float64 [T, d]."""
    y = widen(y)
    T, k = pos.shape
    out = np.zeros((T, y.shape[1]), dtype=np.float64)
    for j in range(k):
        out += np.asarray(topk_w, dtype=np.float64)[:, j:j + 1] * y[pos[:, j].astype(np.int64)]
    return out


def moe_layer(x: np.ndarray, logits: np.ndarray, k: int, expert_weights):
    """The whole layer: route -> dispatch -> expert FFN -> combine. Returns a dict of every
    intermediate so tests can compare step by step."""
    topk_idx, topk_w, counts, offsets = route(logits, k)
    xp, pos, src = dispatch(x, topk_idx, offsets)
    y = expert_ffn(xp, offsets, expert_weights)
    out = combine(y, pos, topk_w)
    return dict(topk_idx=topk_idx, topk_w=topk_w, counts=counts, offsets=offsets,
                xp=xp, pos=pos, src=src, y=y, out=out)


def token_outputs(x: np.ndarray, topk_idx: np.ndarray, topk_w: np.ndarray, tokens, expert_weights):
    """Layer output for a chosen subset of tokens, given their routing.

    Each token's output depends only on its own row of x and its own k experts, so the full
    layer can be checked on a sample. Tokens are grouped by expert so each expert's weights
    are widened once. Returns float64 [len(tokens), d].
    """
    get = expert_weights if callable(expert_weights) else (lambda e: expert_weights[e])
    tokens = [int(t) for t in tokens]
    k = topk_idx.shape[1]
    xs = widen(np.asarray(x)[tokens])
    out = np.zeros_like(xs)
    experts = sorted({int(e) for t in tokens for e in topk_idx[t]})
    for e in experts:
        members = [(n, j) for n, t in enumerate(tokens) for j in range(k) if int(topk_idx[t, j]) == e]
        w_gate, w_up, w_down = get(e)
        rows = xs[[n for n, _ in members]]
        h = silu(rows @ widen(w_gate).T) * (rows @ widen(w_up).T)
        ye = h @ widen(w_down).T
        for m, (n, j) in enumerate(members):
            out[n] += float(topk_w[tokens[n], j]) * ye[m]
    return out
