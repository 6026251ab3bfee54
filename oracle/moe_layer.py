"""Oracle for one GPU's share of an expert-parallel MoE layer (TEST INFRASTRUCTURE).

The paper describes the layer only in words (Sec. 2.1): a Gate picks the experts
of each token, a first all-to-all carries each token to its experts' GPUs, the
expert FFNs process what they receive, a second all-to-all (the reverse of the
first, same sizes) brings the results back and Aggregation forms the weighted
output.  Everything numerical below is therefore a stated reading of that
passage; each function names the reading it implements.

All floating point is fp64 on the inputs as given (inputs are already rounded to
their storage dtype by the caller); nothing is rounded in between.  Integer
results (indices, counts, permutations) are exact.

Pins (tests/test_oracle_layer.py): exhaustive top-k against a full sort, tie and
duplicate-row cases, probability mass invariants, brute-force recount of traffic,
permutation invariants for every destination order, hand-built capacity case,
identity / K = 1 FFN special cases, SwiGLU reducing to the SiLU MLP, closed-form
scalars, and the step-wise pipeline run over an emulated cluster against the
per-token definition `layer_dense`.
"""
from __future__ import annotations

import numpy as np

ACT_SILU_MLP, ACT_GELU_MLP, ACT_SWIGLU = 0, 1, 2


# --------------------------------------------------------------------------- Gate (Sec. 2.1)
def gate_logits(x, w_gate, gate_bias=None):
    """logit[t, e] = sum_h x[t, h] * Wg[e, h] (+ bias[e]), accumulated in fp64."""
    z = np.asarray(x, dtype=np.float64) @ np.asarray(w_gate, dtype=np.float64).T
    if gate_bias is not None:
        z = z + np.asarray(gate_bias, dtype=np.float64)[None, :]
    return z


def route(x, w_gate, gate_bias, k, renorm):
    """Gate of Sec. 2.1 read as: linear logits, softmax over the E experts, top-k.

    Selection is on the logits (softmax is monotone): the k largest, listed by
    descending logit, equal logits resolved towards the lower expert index.  The
    combine weight of choice j is the softmax probability of the chosen expert;
    with ``renorm`` the k weights are divided by their sum.
    Returns (idx[T, k] int32, w[T, k] float64, logits[T, E] float64).
    """
    z = gate_logits(x, w_gate, gate_bias)
    T, E = z.shape
    # stable argsort of -z keeps the lower index first among equals
    order = np.argsort(-z, axis=1, kind="stable")
    idx = order[:, :k].astype(np.int32)
    zmax = z.max(axis=1, keepdims=True)
    ez = np.exp(z - zmax)
    p = ez / ez.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return idx, w, z


def route_margin(z, k):
    """Gap between the k-th and (k+1)-th largest logit of every token (inf if k == E).

    Not part of the method: the parity harness uses it to state that the chosen
    indices do not depend on summation order for the seed in use.
    """
    s = -np.sort(-z, axis=1)
    if k >= z.shape[1]:
        return np.full(z.shape[0], np.inf)
    gaps = [s[:, j] - s[:, j + 1] for j in range(k)]
    return np.min(np.stack(gaps, axis=1), axis=1)


# ------------------------------------------------- traffic row (Sec. 4, Table 1: d_ij)
def traffic(idx, expert_to_gpu, G, capacity=0):
    """Row g of the first all-to-all's traffic matrix, in token-slots.

    A slot is a (token, choice) pair with id t * k + j.  With a capacity C > 0 a
    slot is kept iff fewer than C slots with a smaller id chose the same expert.
    expert_count[e] counts kept slots of expert e, dest_count[d] sums them over
    the experts placed on GPU d (self traffic included: those rows are real work
    for the local FFN; the diagonal is ignored only when communication time is
    computed).  Returns (expert_count[E], dest_count[G], n_dropped, keep[T*k]).
    """
    idx = np.asarray(idx)
    E = len(expert_to_gpu)
    flat = idx.reshape(-1)
    keep = np.ones(flat.shape[0], dtype=bool)
    expert_count = np.zeros(E, dtype=np.int64)
    for s, e in enumerate(flat):
        if capacity > 0 and expert_count[e] >= capacity:
            keep[s] = False
        else:
            expert_count[e] += 1
    dest_count = np.zeros(G, dtype=np.int64)
    for e in range(E):
        dest_count[expert_to_gpu[e]] += expert_count[e]
    return expert_count, dest_count, int((~keep).sum()), keep


# ------------------------------- buffer layer in the scheduled order (Sec. 3, Comm. scheduling)
def segment_order(expert_to_gpu, dest_order):
    """Experts in send order: destinations as listed in dest_order, and within one
    destination its experts by ascending id."""
    segs = []
    for d in dest_order:
        for e in range(len(expert_to_gpu)):
            if expert_to_gpu[e] == d:
                segs.append(e)
    return segs


def dispatch(x, idx, expert_to_gpu, dest_order, capacity=0):
    """Send buffer of one GPU.

    Kept slots are laid out destination by destination in ``dest_order``; inside
    a destination expert by expert (ascending id); inside an expert by ascending
    slot id.  Row r of the buffer is a copy of the token row of the slot placed
    there.  Returns dict(send_buf, slot_to_row (-1 = dropped), row_to_slot,
    seg_offset[E+1], seg_expert[E], n_rows).
    """
    x = np.asarray(x)
    idx = np.asarray(idx)
    T, k = idx.shape
    E = len(expert_to_gpu)
    _, _, _, keep = traffic(idx, expert_to_gpu, int(max(expert_to_gpu)) + 1, capacity)
    flat = idx.reshape(-1)
    seg_expert = segment_order(expert_to_gpu, dest_order)
    slot_to_row = np.full(T * k, -1, dtype=np.int32)
    row_to_slot = []
    seg_offset = [0]
    for e in seg_expert:
        for s in np.nonzero(keep & (flat == e))[0]:      # ascending slot id
            slot_to_row[s] = len(row_to_slot)
            row_to_slot.append(int(s))
        seg_offset.append(len(row_to_slot))
    row_to_slot = np.asarray(row_to_slot, dtype=np.int32)
    send_buf = x[row_to_slot // k] if len(row_to_slot) else np.zeros((0, x.shape[1]), x.dtype)
    return {"send_buf": send_buf, "slot_to_row": slot_to_row, "row_to_slot": row_to_slot,
            "seg_offset": np.asarray(seg_offset, dtype=np.int32),
            "seg_expert": np.asarray(seg_expert, dtype=np.int32), "n_rows": len(row_to_slot)}


def dispatch_chunks(x, idx, expert_to_gpu, chunks, capacity=0):
    """Send buffer of one GPU laid out for a preemptive schedule (Appendix A: in every
    time slot a GPU sends to one GPU, and a flow may be served in several slots).

    The kept slots of a destination form one sequence: expert by expert (ascending
    id), inside an expert by ascending slot id - the order `dispatch` uses.
    ``chunks`` is a list of (dest, rows): chunk c carries the next ``rows`` slots of
    its destination's sequence, fewer (possibly none) if the sequence runs out; a
    chunk whose dest is no GPU is empty.  What the plan did not cover follows after
    the last chunk, destination by destination in ascending GPU id.  The buffer is
    the concatenation of the chunks.  A piece is a maximal run of rows of one chunk
    and one expert; pieces are listed in buffer order.
    Returns dict(send_buf, slot_to_row (-1 = dropped), row_to_slot, chunk_offset
    [len(chunks)+G+1], piece_offset[P+1], piece_expert[P], n_rows).
    """
    x = np.asarray(x)
    idx = np.asarray(idx)
    T, k = idx.shape
    G = int(max(expert_to_gpu)) + 1
    _, _, _, keep = traffic(idx, expert_to_gpu, G, capacity)
    flat = idx.reshape(-1)
    seq = [[] for _ in range(G)]                            # per destination: its slots in order
    for e in range(len(expert_to_gpu)):
        seq[expert_to_gpu[e]].extend(int(s) for s in np.nonzero(keep & (flat == e))[0])
    taken = [0] * G
    row_to_slot, chunk_offset = [], [0]
    for dest, rows in list(chunks) + [(d, None) for d in range(G)]:
        if 0 <= dest < G:
            hi = len(seq[dest]) if rows is None else min(len(seq[dest]), taken[dest] + max(int(rows), 0))
            row_to_slot.extend(seq[dest][taken[dest]:hi])
            taken[dest] = hi
        chunk_offset.append(len(row_to_slot))
    slot_to_row = np.full(T * k, -1, dtype=np.int32)
    for r, s in enumerate(row_to_slot):
        slot_to_row[s] = r
    piece_start, piece_expert = [], []
    for c in range(len(chunk_offset) - 1):
        for r in range(chunk_offset[c], chunk_offset[c + 1]):
            e = int(flat[row_to_slot[r]])
            if r == chunk_offset[c] or e != piece_expert[-1]:
                piece_start.append(r)
                piece_expert.append(e)
    piece_offset = piece_start + [len(row_to_slot)]
    row_to_slot = np.asarray(row_to_slot, dtype=np.int32)
    send_buf = x[row_to_slot // k] if len(row_to_slot) else np.zeros((0, x.shape[1]), x.dtype)
    return {"send_buf": send_buf, "slot_to_row": slot_to_row, "row_to_slot": row_to_slot,
            "chunk_offset": np.asarray(chunk_offset, dtype=np.int32),
            "piece_offset": np.asarray(piece_offset, dtype=np.int32),
            "piece_expert": np.asarray(piece_expert, dtype=np.int32), "n_rows": len(row_to_slot)}


# ----------------------------------------------------------------- expert FFN (Sec. 2.1)
def _silu(a):
    return a / (1.0 + np.exp(-a))


def _gelu_tanh(a):
    return 0.5 * a * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (a + 0.044715 * a ** 3)))


def ffn(rows, w1, w_up, w_down, act):
    """One expert applied to rows[R, H]; weights stored [out, in].

    act 0: Wd . silu(W1 . x);  act 1: Wd . gelu(W1 . x) with the tanh form of GELU;
    act 2: Wd . (silu(W1 . x) * (Wu . x)).  No biases.  fp64 throughout.
    """
    r = np.asarray(rows, dtype=np.float64)
    a = r @ np.asarray(w1, dtype=np.float64).T
    if act == ACT_SILU_MLP:
        h = _silu(a)
    elif act == ACT_GELU_MLP:
        h = _gelu_tanh(a)
    elif act == ACT_SWIGLU:
        h = _silu(a) * (r @ np.asarray(w_up, dtype=np.float64).T)
    else:
        raise ValueError(act)
    return h @ np.asarray(w_down, dtype=np.float64).T


def expert_ffn(recv, seg_offset, seg_expert, experts, act):
    """Grouped FFN: rows [seg_offset[i], seg_offset[i+1]) go through local expert seg_expert[i]."""
    recv = np.asarray(recv)
    out = np.zeros((recv.shape[0], np.asarray(experts[0]["w_down"]).shape[0]), dtype=np.float64)
    for i, e in enumerate(seg_expert):
        lo, hi = int(seg_offset[i]), int(seg_offset[i + 1])
        if hi > lo:
            w = experts[int(e)]
            out[lo:hi] = ffn(recv[lo:hi], w["w1"], w.get("w_up"), w["w_down"], act)
    return out


# ---------------------------------------------------------------- Aggregation (Sec. 2.1)
def combine(ret, slot_to_row, w, shared_out=None):
    """y[t] = sum_j w[t, j] * ret[slot_to_row[t*k + j]] over kept slots (+ shared_out[t]).

    ``ret`` is in send-buffer row order: the second all-to-all is the reverse of
    the first with the same sizes (Sec. 2.2), so results come back where the
    tokens were sent from.
    """
    ret = np.asarray(ret, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    T, k = w.shape
    y = np.zeros((T, ret.shape[1]), dtype=np.float64)
    for t in range(T):
        for j in range(k):
            r = slot_to_row[t * k + j]
            if r >= 0:
                y[t] += w[t, j] * ret[r]
    if shared_out is not None:
        y += np.asarray(shared_out, dtype=np.float64)
    return y


# ------------------------------------------- the plain definition the whole path must reach
def layer_dense(x, w_gate, gate_bias, k, renorm, experts, act, capacity=0, shared=None):
    """y_t = sum over kept choices j of w_tj * FFN_{e_tj}(x_t)  (+ sum_s FFN_shared_s(x_t)).

    Per-token loop over the definition; no buffers, no permutation.  ``experts``
    is the list of ALL E experts' weights.  A choice is dropped by the capacity
    rule of `traffic` (ascending slot id, per expert, on this GPU's tokens).
    """
    x = np.asarray(x, dtype=np.float64)
    idx, w, _ = route(x, w_gate, gate_bias, k, renorm)
    T = x.shape[0]
    H_out = np.asarray(experts[0]["w_down"]).shape[0]
    y = np.zeros((T, H_out), dtype=np.float64)
    seen = {}
    for t in range(T):
        for j in range(k):
            e = int(idx[t, j])
            c = seen.get(e, 0)
            if capacity > 0 and c >= capacity:
                continue
            seen[e] = c + 1
            we = experts[e]
            y[t] += w[t, j] * ffn(x[t:t + 1], we["w1"], we.get("w_up"), we["w_down"], act)[0]
        if shared:
            for ws in shared:
                y[t] += ffn(x[t:t + 1], ws["w1"], ws.get("w_up"), ws["w_down"], act)[0]
    return y
