"""CPU oracle for the dropless-MoE (dMoE) expert layer.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; the product
(the HIP library and its Python binding) never does and shares no code with it.

What is computed, and from where in the paper:

* Router (Section 2.1): tokens are projected from hidden_size to num_experts scores with a learned matrix,
  scores are normalised with a softmax, and the top_k experts are taken greedily per token.
* Permutation (Sections 2.2 and 5.2): tokens are grouped by expert; each group is zero-padded to the next
  multiple of the 128-row block.
* Topology (Figure 3C, Sections 5.1.3 and 5.1.4, Figure 5 caption): the block-diagonal, variable-height
  block-sparse matrix in blocked-CSR form, with per-block row indices (the hybrid blocked-CSR-COO encoding)
  and the transpose indices (metadata of the transposed matrix plus the offset of each nonzero block).
* Expert computation (Sections 2.3, 4.1, 5.1, Figure 6): a block-diagonal block-sparse product equals one
  dense product per expert on exactly the tokens routed to it, and zero padding adds nothing, so the oracle
  is that plain definition: per expert, two dense matmuls around the activation.  No padding, no drops.
* Un-permutation (Section 2.4): expert outputs are scaled by the router's confidence and summed over top_k.
* Backward (Section 5.1 lists the four backward products): the chain rule on the forward definition, with
  the expert assignments held constant.

Precision: the router logits are accumulated in float32 in ascending order of the hidden index, one
multiply-add at a time, because they decide integers (the expert assignment) and both sides must take that
decision in the same arithmetic.  Everything else is float64 on the bf16 inputs widened exactly.

Readings where the paper is silent (the full list lives in the design notes): activation = exact (erf)
GELU; no expert biases; flat assignment index f = token * top_k + slot; ties in top-k go to the lowest
expert index; tokens keep ascending f inside an expert group; an empty expert owns no rows and no blocks;
indices are 32-bit; confidence weights are the softmax probabilities of the chosen experts, optionally
divided by their sum over the k slots.

Pins (tests/test_oracle_*.py): dense all-experts-masked float64 brute force, torch float64 autograd on that
dense formulation, central finite differences, the single-expert case against two library GEMMs, routing
against a float64 stable argsort where the margin is clear, GELU special values, and the structural
invariants of the permutation and of the sparse-matrix encoding.
"""
from __future__ import annotations

import math
import numpy as np
from scipy.special import erf as _erf

BLOCK = 128


# ----------------------------------------------------------------------------- helpers
def widen_bf16(bits: np.ndarray, dtype=np.float64) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float (exact)."""
    f32 = (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    return f32.astype(dtype, copy=False)


def gelu(v: np.ndarray) -> np.ndarray:
    """Exact GELU  v * Phi(v),  Phi the standard normal CDF."""
    return 0.5 * v * (1.0 + _erf(v / math.sqrt(2.0)))


def gelu_grad(v: np.ndarray) -> np.ndarray:
    """d/dv [v Phi(v)] = Phi(v) + v phi(v)."""
    return 0.5 * (1.0 + _erf(v / math.sqrt(2.0))) + v * np.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)


def gelu_tanh(v: np.ndarray) -> np.ndarray:
    """The tanh form of GELU:  0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3)))  (activation = 1)."""
    return 0.5 * v * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))


def gelu_tanh_grad(v: np.ndarray) -> np.ndarray:
    """Derivative of the tanh form: with u = sqrt(2/pi)(v + 0.044715 v^3) and t = tanh u,
    0.5 (1 + t) + 0.5 v (1 - t^2) sqrt(2/pi) (1 + 3 * 0.044715 v^2)."""
    t = np.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3))
    return 0.5 * (1.0 + t) + 0.5 * v * (1.0 - t * t) * math.sqrt(2.0 / math.pi) * (1.0 + 3.0 * 0.044715 * v * v)


def activation_pair(activation: int):
    """(act, act') for the configuration's `activation` field: 0 exact GELU, 1 tanh form."""
    if activation == 0:
        return gelu, gelu_grad
    if activation == 1:
        return gelu_tanh, gelu_tanh_grad
    raise ValueError("activation must be 0 or 1")


# ----------------------------------------------------------------------------- router (Section 2.1)
def router_logits(x_bits: np.ndarray, wr_bits: np.ndarray, bias: np.ndarray | None) -> np.ndarray:
    """float32 scores[t,e] = sum_i x[t,i] * Wr[i,e], accumulated for i = 0, 1, ... in that order
    (a bf16 x bf16 product is exact in float32, so each step is one rounding), then + bias[e]."""
    x = widen_bf16(x_bits, np.float32)
    wr = widen_bf16(wr_bits, np.float32)
    T, d = x.shape
    acc = np.zeros((T, wr.shape[1]), dtype=np.float32)
    for i in range(d):
        acc += x[:, i, None] * wr[i, None, :]
    if bias is not None:
        acc += np.asarray(bias, dtype=np.float32)[None, :]
    return acc


def top_k_greedy(logits: np.ndarray, top_k: int) -> np.ndarray:
    """expert_idx[t,s]: for s = 0..k-1 the highest-scoring expert not taken yet; ties -> lowest index.
    Selection on the scores equals selection on their softmax (monotone)."""
    T, E = logits.shape
    work = logits.astype(np.float32, copy=True)
    idx = np.empty((T, top_k), dtype=np.int32)
    rows = np.arange(T)
    for s in range(top_k):
        best = np.argmax(work, axis=1)          # first maximum = lowest expert index
        idx[:, s] = best
        work[rows, best] = -np.inf
    return idx


def softmax_probs(logits: np.ndarray) -> np.ndarray:
    """float64 softmax over experts of the float32 scores."""
    z = logits.astype(np.float64)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def route(x_bits, wr_bits, bias, top_k: int, normalize_topk: int):
    """Returns logits f32 [T,E], expert_idx i32 [T,k], weights f64 [T,k], probs f64 [T,E]."""
    logits = router_logits(x_bits, wr_bits, bias)
    idx = top_k_greedy(logits, top_k)
    p = softmax_probs(logits)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if normalize_topk:
        w = w / w.sum(axis=1, keepdims=True)
    return logits, idx, w, p


# ----------------------------------------------------------------------------- permutation (Sections 2.2, 5.2)
def permutation(expert_idx: np.ndarray, num_experts: int, block: int = BLOCK):
    """Group the flat assignments f = t*k + s by expert (ascending f inside a group), pad each group to the
    next multiple of `block`.

    Returns tokens_per_expert [E], padded_offsets [E+1] (rows), row_of [T*k] (padded row of f),
    token_of [P] (f for each padded row, -1 on padding rows)."""
    flat = np.asarray(expert_idx, dtype=np.int64).reshape(-1)
    n = np.zeros(num_experts, dtype=np.int32)
    members = []
    for e in range(num_experts):
        S_e = np.flatnonzero(flat == e)         # ascending f
        members.append(S_e)
        n[e] = S_e.size
    padded = ((n.astype(np.int64) + block - 1) // block) * block
    offsets = np.zeros(num_experts + 1, dtype=np.int64)
    for e in range(num_experts):
        offsets[e + 1] = offsets[e] + padded[e]
    P = int(offsets[-1])
    row_of = np.full(flat.size, -1, dtype=np.int32)
    token_of = np.full(P, -1, dtype=np.int32)
    for e in range(num_experts):
        for j, f in enumerate(members[e]):
            row_of[f] = offsets[e] + j
            token_of[offsets[e] + j] = f
    return n, offsets.astype(np.int32), row_of, token_of


# ----------------------------------------------------------------------------- token dropping (Section 2.2)
def expert_capacity(num_tokens: int, num_experts: int, capacity_factor: float, top_k: int = 1) -> int:
    """Section 2.2: expert_capacity = num_tokens / num_experts x capacity_factor, the number of assignments an
    expert may take.  With top_k choices per token there are num_tokens*top_k assignments to share out (reading:
    the paper writes the top-1 case).  Rounded down, at least 1."""
    return max(1, int(math.floor(num_tokens * top_k / num_experts * capacity_factor)))


def capacity_keep_mask(expert_idx: np.ndarray, num_experts: int, capacity: int) -> np.ndarray:
    """bool [T,k]: assignment f = t*k + s is kept iff fewer than `capacity` assignments with a smaller f went to the
    same expert (Section 2.2: tokens beyond an expert's capacity are dropped; reading: in flat order, the first
    ones stay).  capacity <= 0 keeps everything (the dropless layer)."""
    flat = np.asarray(expert_idx, dtype=np.int64).reshape(-1)
    keep = np.ones(flat.size, dtype=bool)
    if capacity > 0:
        taken = np.zeros(num_experts, dtype=np.int64)
        for f in range(flat.size):
            e = flat[f]
            keep[f] = taken[e] < capacity
            taken[e] += 1
    return keep.reshape(np.asarray(expert_idx).shape)


def permutation_capacity(expert_idx: np.ndarray, num_experts: int, capacity: int, pad_to_capacity: bool = False,
                         block: int = BLOCK):
    """permutation() for the token-dropping layer: an expert's group holds its kept assignments only (ascending f);
    dropped assignments have row_of = -1.  A group is padded to the next multiple of `block`, or, with
    pad_to_capacity, every expert owns ceil(capacity/block)*block rows (unused capacity is padding, Section 2.2).

    Returns tokens_per_expert (kept) [E], padded_offsets [E+1], row_of [T*k], token_of [P]."""
    flat = np.asarray(expert_idx, dtype=np.int64).reshape(-1)
    keep = capacity_keep_mask(expert_idx, num_experts, capacity).reshape(-1)
    n = np.zeros(num_experts, dtype=np.int32)
    members = []
    for e in range(num_experts):
        S_e = np.flatnonzero((flat == e) & keep)
        members.append(S_e)
        n[e] = S_e.size
    if pad_to_capacity:
        padded = np.full(num_experts, ((capacity + block - 1) // block) * block, dtype=np.int64)
    else:
        padded = -(-n.astype(np.int64) // block) * block           # next multiple of the block
    offsets = np.zeros(num_experts + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(padded)
    row_of = np.full(flat.size, -1, dtype=np.int32)
    token_of = np.full(int(offsets[-1]), -1, dtype=np.int32)
    for e in range(num_experts):
        for j, f in enumerate(members[e]):
            row_of[f] = offsets[e] + j
            token_of[offsets[e] + j] = f
    return n, offsets.astype(np.int32), row_of, token_of


# ----------------------------------------------------------------------------- topology (Fig. 3C, 5.1.3, 5.1.4)
def block_mask(padded_offsets: np.ndarray, hb: int, block: int = BLOCK) -> np.ndarray:
    """Dense 0/1 map of nonzero blocks, R x (E*hb): block-row r of expert e is nonzero exactly on that
    expert's hb block-columns (the variable-height block diagonal of Figure 3C)."""
    E = len(padded_offsets) - 1
    R = int(padded_offsets[-1]) // block
    m = np.zeros((R, E * hb), dtype=np.uint8)
    for e in range(E):
        r0, r1 = int(padded_offsets[e]) // block, int(padded_offsets[e + 1]) // block
        m[r0:r1, e * hb:(e + 1) * hb] = 1
    return m


def encode_mask(mask: np.ndarray) -> dict:
    """Hybrid blocked-CSR-COO encoding of a block mask plus its transpose indices.

    Primary (row-wise) order numbers the nonzero blocks 0..nnz-1; block b's values live at offset b.
      row_offsets[r], column_indices[b]   -- blocked CSR
      row_indices[b]                      -- the COO row of each block (Section 5.1.3)
    Transposed order (Section 5.1.4) is the blocked CSR of the transposed mask:
      column_offsets_t[c], row_indices_t[i], and block_offsets_t[i] = primary number of that block."""
    R, C = mask.shape
    row_offsets = np.zeros(R + 1, dtype=np.int32)
    column_indices, row_indices = [], []
    number = -np.ones((R, C), dtype=np.int64)
    for r in range(R):
        cols = np.flatnonzero(mask[r])
        for c in cols:
            number[r, c] = len(column_indices)
            column_indices.append(c)
            row_indices.append(r)
        row_offsets[r + 1] = len(column_indices)
    column_offsets_t = np.zeros(C + 1, dtype=np.int32)
    row_indices_t, block_offsets_t = [], []
    for c in range(C):
        rows = np.flatnonzero(mask[:, c])
        for r in rows:
            row_indices_t.append(r)
            block_offsets_t.append(number[r, c])
        column_offsets_t[c + 1] = len(row_indices_t)
    as_i32 = lambda a: np.asarray(a, dtype=np.int32).reshape(-1)
    return {
        "row_offsets": row_offsets, "column_indices": as_i32(column_indices), "row_indices": as_i32(row_indices),
        "column_offsets_t": column_offsets_t, "row_indices_t": as_i32(row_indices_t),
        "block_offsets_t": as_i32(block_offsets_t),
    }


def topology(padded_offsets: np.ndarray, ffn_hidden: int, block: int = BLOCK) -> dict:
    """make_topology of Figure 6: the encoding of the block-diagonal mask, plus the counts P, R, nnz."""
    hb = ffn_hidden // block
    enc = encode_mask(block_mask(padded_offsets, hb, block))
    P = int(padded_offsets[-1])
    enc["counts"] = np.array([P, P // block, (P // block) * hb, 0], dtype=np.int32)
    return enc


def topology_closed_form(padded_offsets: np.ndarray, ffn_hidden: int, block: int = BLOCK) -> dict:
    """The same arrays written as closed forms of the block-diagonal structure (cross-check only)."""
    hb = ffn_hidden // block
    E = len(padded_offsets) - 1
    first = np.asarray(padded_offsets, dtype=np.int64) // block
    rows = first[1:] - first[:-1]
    R = int(first[-1])
    owner = np.repeat(np.arange(E), rows)
    b = np.arange(R * hb)
    out = {
        "row_offsets": (np.arange(R + 1) * hb).astype(np.int32),
        "column_indices": (owner[b // hb] * hb + b % hb).astype(np.int32) if R else np.zeros(0, np.int32),
        "row_indices": (b // hb).astype(np.int32),
    }
    col_rows = np.repeat(rows, hb)
    out["column_offsets_t"] = np.concatenate([[0], np.cumsum(col_rows)]).astype(np.int32)
    rit, bot = [], []
    for c in range(E * hb):
        e = c // hb
        for j in range(int(rows[e])):
            r = first[e] + j
            rit.append(r)
            bot.append(r * hb + c % hb)
    out["row_indices_t"] = np.asarray(rit, dtype=np.int32).reshape(-1)
    out["block_offsets_t"] = np.asarray(bot, dtype=np.int32).reshape(-1)
    return out


# ----------------------------------------------------------------------------- expert computation + un-permute
def _members(expert_idx: np.ndarray, e: int) -> np.ndarray:
    return np.flatnonzero(np.asarray(expert_idx).reshape(-1) == e)


def forward(x_bits, w1_bits, w2_bits, expert_idx, weights, ffn_hidden: int, keep: bool = False, activation: int = 0,
            keep_mask=None):
    """y[t] = sum_s weights[t,s] * FFN_{e(t,s)}(x[t]),  FFN_e(v) = gelu(v W1_e) W2_e   (Sections 2.3-2.4, Fig. 6).

    keep_mask (bool [T,k], optional): the token-dropping layer of Section 2.2 -- assignments whose entry is False
    are dropped: they reach no expert and add nothing to y.

    Returns y float64 [T,d]; with keep=True also the per-expert intermediates for backward()."""
    if keep_mask is not None:
        expert_idx = np.where(np.asarray(keep_mask, dtype=bool), expert_idx, -1)      # -1 is no expert's group
    T, d = x_bits.shape
    k = expert_idx.shape[1]
    E = w1_bits.shape[1] // ffn_hidden
    h = ffn_hidden
    x = widen_bf16(x_bits)
    w_flat = np.asarray(weights, dtype=np.float64).reshape(-1)
    y = np.zeros((T, d), dtype=np.float64)
    saved = {}
    for e in range(E):
        S_e = _members(expert_idx, e)
        if S_e.size == 0:
            continue
        tok = S_e // k
        W1_e = widen_bf16(w1_bits[:, e * h:(e + 1) * h])
        W2_e = widen_bf16(w2_bits[e * h:(e + 1) * h, :])
        X_e = x[tok]
        H_e = X_e @ W1_e
        A_e = activation_pair(activation)[0](H_e)
        O_e = A_e @ W2_e
        np.add.at(y, tok, w_flat[S_e, None] * O_e)
        if keep:
            saved[e] = (S_e, X_e, H_e, A_e, O_e)
    return (y, saved) if keep else y


def backward(x_bits, wr_bits, w1_bits, w2_bits, dy_bits, expert_idx, weights, probs, ffn_hidden: int,
             normalize_topk: int, activation: int = 0, keep_mask=None):
    """Gradients of  L = <dy, y>  with the expert assignments held constant.

    keep_mask: as in forward().  A dropped assignment's confidence does not appear in y, so its dweights entry is
    zero; the confidences themselves (and their renormalisation over the k slots) are those of the router.

    Returns dx [T,d], dw_router [d,E], dw1 [d,E*h], dw2 [E*h,d] (float64), and dweights [T,k]."""
    T, d = x_bits.shape
    k = expert_idx.shape[1]
    h = ffn_hidden
    E = w1_bits.shape[1] // h
    x = widen_bf16(x_bits)
    wr = widen_bf16(wr_bits)
    dy = widen_bf16(dy_bits)
    w_flat = np.asarray(weights, dtype=np.float64).reshape(-1)
    _, saved = forward(x_bits, w1_bits, w2_bits, expert_idx, weights, h, keep=True, activation=activation,
                       keep_mask=keep_mask)

    dx = np.zeros((T, d))
    dw1 = np.zeros((d, E * h))
    dw2 = np.zeros((E * h, d))
    dwt = np.zeros(T * k)
    for e in range(E):
        if e not in saved:
            continue                               # empty expert: its weight gradients stay exactly zero
        S_e, X_e, H_e, A_e, O_e = saved[e]
        tok = S_e // k
        W1_e = widen_bf16(w1_bits[:, e * h:(e + 1) * h])
        W2_e = widen_bf16(w2_bits[e * h:(e + 1) * h, :])
        dO_e = w_flat[S_e, None] * dy[tok]
        dwt[S_e] = np.einsum("ij,ij->i", dy[tok], O_e)
        dw2[e * h:(e + 1) * h, :] = A_e.T @ dO_e
        dA_e = dO_e @ W2_e.T
        dH_e = dA_e * activation_pair(activation)[1](H_e)
        dw1[:, e * h:(e + 1) * h] = X_e.T @ dH_e
        np.add.at(dx, tok, dH_e @ W1_e.T)

    # router: weights = softmax(scores)[chosen] (optionally renormalised over the k slots)
    dwt = dwt.reshape(T, k)
    w = np.asarray(weights, dtype=np.float64).reshape(T, k)
    p = np.asarray(probs, dtype=np.float64)
    idx = expert_idx.astype(np.int64)
    if normalize_topk:
        Z = np.take_along_axis(p, idx, axis=1).sum(axis=1, keepdims=True)
        dsel = (dwt - (dwt * w).sum(axis=1, keepdims=True)) / Z
    else:
        dsel = dwt
    dp = np.zeros_like(p)
    np.put_along_axis(dp, idx, dsel, axis=1)
    dlogits = p * (dp - (dp * p).sum(axis=1, keepdims=True))
    dw_router = x.T @ dlogits
    dx += dlogits @ wr.T
    return {"dx": dx, "dw_router": dw_router, "dw1": dw1, "dw2": dw2, "dweights": dwt, "dlogits": dlogits}


# ----------------------------------------------------------------------------- slices for very large layers
def forward_rows(x_bits, w1_bits, w2_bits, expert_idx, weights, ffn_hidden: int, tokens) -> np.ndarray:
    """y[t] for the listed tokens only (each row is an independent dense computation)."""
    h = ffn_hidden
    k = expert_idx.shape[1]
    out = np.zeros((len(tokens), x_bits.shape[1]))
    for i, t in enumerate(tokens):
        v = widen_bf16(x_bits[t])
        for s in range(k):
            e = int(expert_idx[t, s])
            hid = gelu(v @ widen_bf16(w1_bits[:, e * h:(e + 1) * h]))
            out[i] += float(weights[t, s]) * (hid @ widen_bf16(w2_bits[e * h:(e + 1) * h, :]))
    return out


def backward_rows(x_bits, wr_bits, w1_bits, w2_bits, dy_bits, expert_idx, weights, probs, ffn_hidden: int,
                  normalize_topk: int, tokens):
    """dx[t], dweights[t,:] and dlogits[t,:] for the listed tokens only."""
    h = ffn_hidden
    k = expert_idx.shape[1]
    wr = widen_bf16(wr_bits)
    dxs = np.zeros((len(tokens), x_bits.shape[1]))
    dws = np.zeros((len(tokens), k))
    dls = np.zeros((len(tokens), probs.shape[1]))
    for i, t in enumerate(tokens):
        v = widen_bf16(x_bits[t])
        g = widen_bf16(dy_bits[t])
        for s in range(k):
            e = int(expert_idx[t, s])
            W1_e = widen_bf16(w1_bits[:, e * h:(e + 1) * h])
            W2_e = widen_bf16(w2_bits[e * h:(e + 1) * h, :])
            hid = v @ W1_e
            o = gelu(hid) @ W2_e
            dws[i, s] = g @ o
            dh = ((float(weights[t, s]) * g) @ W2_e.T) * gelu_grad(hid)
            dxs[i] += dh @ W1_e.T
        p = np.asarray(probs[t], dtype=np.float64)
        w = np.asarray(weights[t], dtype=np.float64)
        idx = expert_idx[t].astype(np.int64)
        if normalize_topk:
            dsel = (dws[i] - (dws[i] * w).sum()) / p[idx].sum()
        else:
            dsel = dws[i]
        dp = np.zeros_like(p)
        dp[idx] = dsel
        dl = p * (dp - (dp * p).sum())
        dls[i] = dl
        dxs[i] += dl @ wr.T
    return dxs, dws, dls


def weight_grad_panel(x_bits, w1_bits, w2_bits, dy_bits, expert_idx, weights, ffn_hidden: int, e: int, cols):
    """For expert e and a list of its hidden units `cols` (0..h-1): dW1[:, e*h+cols] ([d,|cols|]) and
    dW2[e*h+cols, :] ([|cols|,d]).  Both depend only on those columns of H_e."""
    h = ffn_hidden
    k = expert_idx.shape[1]
    cols = np.asarray(cols, dtype=np.int64)
    d = x_bits.shape[1]
    S_e = _members(expert_idx, e)
    if S_e.size == 0:
        return np.zeros((d, cols.size)), np.zeros((cols.size, d))
    tok = S_e // k
    X_e = widen_bf16(x_bits[tok])
    dO_e = np.asarray(weights, dtype=np.float64).reshape(-1)[S_e, None] * widen_bf16(dy_bits[tok])
    H_c = X_e @ widen_bf16(w1_bits[:, e * h + cols])
    dW2_c = gelu(H_c).T @ dO_e
    dH_c = (dO_e @ widen_bf16(w2_bits[e * h + cols, :]).T) * gelu_grad(H_c)
    dW1_c = X_e.T @ dH_c
    return dW1_c, dW2_c
