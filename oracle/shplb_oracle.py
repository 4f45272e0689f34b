"""CPU oracle for head-adaptive block-sparse causal prefill (S-HPLB hot path).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is
checked against.  It may be imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path; it shares no code with
the HIP kernels or their Python binding and imports neither.

Everything is fp64 on inputs given as bf16 bit patterns (so the oracle and the GPU
see identical input values).  Nothing is blocked, fused or reordered beyond what
each definition states.

What the paper fixes and what it leaves open
  * Attention itself is Eq. 1 (Section 2.1): A = softmax(Q K^T / sqrt(d)), O = A V,
    per head, K/V shared by the G consecutive query heads of a GQA group.
  * Sparse attention computes only a chosen subset of query-key pairs under a
    per-head budget (Sections 2.3, 3.1); the head-adaptive budget is applied as a
    top-k, which needs only ordinal information (Section 2.4).
  * The head-to-device assignment is the greedy of Section 3.3: sort heads by
    budget descending, give each to the currently least-loaded device; the
    objective is Eq. 2, I = max_d L_d / mean_d L_d with L_d the sum of budgets.
  * The paper does not define the block-importance estimator or the selection
    rule (Section 4: its kernels come from another framework).  The readings used
    here: importance of key block j for query block i = dot product of the
    mean-pooled query block and mean-pooled key block, times 1/sqrt(d); every row
    keeps block 0 (sink) and its own diagonal block and fills the rest of its
    budget with the highest-scoring earlier blocks, ties to the lower index; the
    budget is per head, in blocks, and applies to every query-block row of the head.

  * Budgets come from max-min budget shifting (Section 3.2): start from equal budgets
    and move budget from the head with the highest recovery ratio to the head with the
    lowest until the giver has become the minimum or nobody above the lower bound is
    left to give.  The paper states neither the step nor the exact test; readings:
    one step of `step` units per move; the receiver is the lowest-recovery head, the
    giver the highest-recovery other head that can still give (ties to the lower
    index); a move that would lower the minimum recovery is not made and ends the
    iteration; a move that is made and leaves the giver as the (possibly tied)
    minimum ends it too; an indivisible total gives its remainder to the first heads.

  * The recovery ratio of Section 2.4 (cumulative attention weight of the top-k keys) is
    taken at block granularity: the mass of key block j for query block i is the
    attention weight that the queries of block i put on the keys of block j, averaged
    over the block's queries; a head's recovery at budget b is the mass of the b
    heaviest blocks of a row, averaged over all queries of the head (rows with fewer
    than b visible blocks recover everything).  The paper profiles tokens (k = 4096);
    blocks are what the path's budgets count.
  * The same ratio at the paper's own granularity (token_recovery): for every query
    token the sum of its k largest attention weights, Eq. 1 weights under the causal
    mask; a query that sees no more than k keys recovers 1; a head's figure is the mean
    over its queries (the paper plots one number per head and does not say how the
    queries are combined).

Pins (tests/test_oracle_*.py): dense special case vs a textbook attention routine,
row sums, constant-V, sink+diagonal special case, selection-order invariance,
closed-form pooled scores, brute-force top-k, constructed ties, hand-worked greedy
instance, exhaustive optimum on tiny partitions, cost closed form; budget shifting:
hand-worked instance, identical curves, exhaustive max-min optimum for two heads,
invariants on random monotone curves; block mass: rows sum to one, closed form for
constant keys, block sums of a textbook softmax; recovery curves: closed forms for
uniform and one-hot rows, monotone and concave in the budget; token recovery: closed form
for constant keys, top-k sums of a textbook softmax, best subset by exhaustive search,
k = 1 is the largest weight, whole blocks of equal keys against the block profile.
Parity unpinned: how well pooled-score selection tracks true attention mass (needs
the paper's models and data); only self-consistency is checked.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- inputs
def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64 values (exact)."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def blocks_per_sequence(cu_seqlens: Sequence[int], block: int) -> List[int]:
    cu = [int(x) for x in cu_seqlens]
    return [-(-(cu[s + 1] - cu[s]) // block) for s in range(len(cu) - 1)]


# --------------------------------------------------------------------------- a1 / a2
def pool_blocks(x_bits: np.ndarray, cu_seqlens: Sequence[int], block: int) -> List[np.ndarray]:
    """Mean over the valid tokens of each block.  x_bits: [T, H, D] bf16 bits.
    Returns one [H, nb_s, D] fp64 array per sequence."""
    out = []
    nbs = blocks_per_sequence(cu_seqlens, block)
    for s, nb in enumerate(nbs):
        t_begin, t_end = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        h, d = x_bits.shape[1], x_bits.shape[2]
        pooled = np.zeros((h, nb, d), np.float64)
        for b in range(nb):
            t0 = t_begin + b * block
            t1 = min(t_end, t0 + block)
            xb = decode_bf16(x_bits[t0:t1])              # [cnt, H, D]
            pooled[:, b, :] = xb.sum(axis=0) / float(t1 - t0)
        out.append(pooled)
    return out


def block_scores(q_bits: np.ndarray, k_bits: np.ndarray, cu_seqlens: Sequence[int], block: int,
                 scale: Optional[float] = None) -> List[np.ndarray]:
    """Pooled block-importance logits, one [Hq, nb_s, nb_s] fp64 array per sequence.
    s[h, i, j] = (Qbar[h, i] . Kbar[h // G, j]) * scale for j <= i; entries with
    j > i are NaN (undefined, never read).  scale defaults to 1/sqrt(d) (Eq. 1)."""
    hq, d = q_bits.shape[1], q_bits.shape[2]
    hkv = k_bits.shape[1]
    g = hq // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    qbar = pool_blocks(q_bits, cu_seqlens, block)
    kbar = pool_blocks(k_bits, cu_seqlens, block)
    out = []
    for qs, ks in zip(qbar, kbar):
        nb = qs.shape[1]
        sc = np.full((hq, nb, nb), np.nan, np.float64)
        for h in range(hq):
            full = (qs[h] @ ks[h // g].T) * scale
            tri = np.tril_indices(nb)
            sc[h][tri] = full[tri]
        out.append(sc)
    return out


# --------------------------------------------------------------------------- a3
def n_selected(budget: int, nb: int, i: int) -> int:
    """Blocks selected by row i of a head with this budget: the budget, at least
    the two forced blocks, at most the sequence's blocks and the causal-visible i+1."""
    k_eff = min(max(int(budget), 2), nb)
    return min(k_eff, i + 1)


def sel_row_ptr(cu_seqlens: Sequence[int], block: int, n_q_heads: int,
                budgets: Sequence[int]) -> np.ndarray:
    """CSR row pointer of the selection.  Row order: sequence, then head, then query
    block.  budgets: [n_seq * n_q_heads] in blocks."""
    nbs = blocks_per_sequence(cu_seqlens, block)
    counts = []
    for s, nb in enumerate(nbs):
        for h in range(n_q_heads):
            for i in range(nb):
                counts.append(n_selected(budgets[s * n_q_heads + h], nb, i))
    ptr = np.zeros(len(counts) + 1, np.int64)
    ptr[1:] = np.cumsum(np.asarray(counts, np.int64))
    return ptr


def select_row(scores_row: np.ndarray, i: int, n: int) -> np.ndarray:
    """One row's selection.  scores_row[j] valid for j <= i.  Forced {0, i}; then the
    best-scoring of blocks 1..i-1, ties to the lower index, until n blocks are held.
    Comparisons are made in the dtype of scores_row.  Returns ascending indices."""
    chosen = {0, i}
    want = n - len(chosen)
    if want > 0:
        cand = np.arange(1, i)
        # stable sort on descending score keeps equal scores in ascending index order
        order = np.argsort(-scores_row[1:i], kind="stable")
        chosen.update(int(c) for c in cand[order[:want]])
    return np.array(sorted(chosen), np.int32)


def select_blocks(scores: List[np.ndarray], budgets: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Selection for every row.  scores: per-sequence [Hq, nb, nb] arrays (any float
    dtype; the ordering decision is taken in that dtype).  Returns (sel_ptr int64
    [rows+1], sel_idx int32) in CSR form."""
    idx = []
    ptr = [0]
    for s, sc in enumerate(scores):
        hq, nb, _ = sc.shape
        for h in range(hq):
            for i in range(nb):
                n = n_selected(budgets[s * hq + h], nb, i)
                row = select_row(sc[h, i], i, n)
                assert len(row) == n
                idx.append(row)
                ptr.append(ptr[-1] + n)
    return np.asarray(ptr, np.int64), (np.concatenate(idx).astype(np.int32) if idx else np.zeros(0, np.int32))


# --------------------------------------------------------------------------- a5
def sparse_attention_row(q_bits: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray,
                         cu_seqlens: Sequence[int], block: int, s: int, h: int, i: int,
                         sel: Sequence[int], scale: Optional[float] = None
                         ) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1 restricted to the key blocks in sel, with the token-level causal mask,
    for the query tokens of block i of head h of sequence s.
    Returns (O [n_tokens, D] fp64, lse [n_tokens] fp64 natural log)."""
    hq, d = q_bits.shape[1], q_bits.shape[2]
    g = hq // k_bits.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    t_begin, t_end = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
    q0 = t_begin + i * block
    q1 = min(t_end, q0 + block)
    q = decode_bf16(q_bits[q0:q1, h, :])                          # [nq, D]
    key_tok = np.concatenate([np.arange(t_begin + j * block, min(t_end, t_begin + (j + 1) * block))
                              for j in sel])
    k = decode_bf16(k_bits[key_tok, h // g, :])
    v = decode_bf16(v_bits[key_tok, h // g, :])
    logits = (q @ k.T) * scale                                    # [nq, nk]
    q_tok = np.arange(q0, q1)
    logits = np.where(key_tok[None, :] <= q_tok[:, None], logits, -np.inf)
    m = logits.max(axis=1, keepdims=True)
    p = np.exp(logits - m)
    l = p.sum(axis=1, keepdims=True)
    out = (p @ v) / l
    lse = (m + np.log(l))[:, 0]
    return out, lse


def sparse_attention(q_bits, k_bits, v_bits, cu_seqlens, block, sel_ptr, sel_idx,
                     scale: Optional[float] = None, rows: Optional[Sequence[int]] = None
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """All (or the given) rows.  Returns O [T, Hq, D] fp64 and lse [Hq, T] fp64; tokens
    of rows that were not requested are NaN."""
    total, hq, d = q_bits.shape
    nbs = blocks_per_sequence(cu_seqlens, block)
    out = np.full((total, hq, d), np.nan, np.float64)
    lse = np.full((hq, total), np.nan, np.float64)
    want = None if rows is None else set(int(r) for r in rows)
    r = 0
    for s, nb in enumerate(nbs):
        for h in range(hq):
            for i in range(nb):
                if want is None or r in want:
                    sel = sel_idx[sel_ptr[r]:sel_ptr[r + 1]]
                    o, l = sparse_attention_row(q_bits, k_bits, v_bits, cu_seqlens, block, s, h, i, sel, scale)
                    t0 = int(cu_seqlens[s]) + i * block
                    out[t0:t0 + o.shape[0], h, :] = o
                    lse[h, t0:t0 + o.shape[0]] = l
                r += 1
    return out, lse


def row_index(cu_seqlens: Sequence[int], block: int, n_q_heads: int, s: int, h: int, i: int) -> int:
    nbs = blocks_per_sequence(cu_seqlens, block)
    return sum(nbs[:s]) * n_q_heads + h * nbs[s] + i


def row_decode(cu_seqlens: Sequence[int], block: int, n_q_heads: int, row: int) -> Tuple[int, int, int]:
    nbs = blocks_per_sequence(cu_seqlens, block)
    for s, nb in enumerate(nbs):
        if row < nb * n_q_heads:
            return s, row // nb, row % nb
        row -= nb * n_q_heads
    raise IndexError(row)


# --------------------------------------------------------------------------- a6
def balance_heads(costs: Sequence[int], n_parts: int, max_per_part: int = 0
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """Greedy multiway partition (Section 3.3): visit units by descending cost (equal
    costs in ascending index), give each to the part with the smallest load so far
    (equal loads: lowest part index).  max_per_part > 0 additionally skips parts that
    already hold that many units (an extension for equal-sized GQA shares; 0 is the
    paper's algorithm).  Returns (part_of int32 [n], loads int64 [n_parts])."""
    n = len(costs)
    order = sorted(range(n), key=lambda x: (-int(costs[x]), x))
    loads = [0] * n_parts
    counts = [0] * n_parts
    part_of = [-1] * n
    for x in order:
        best = None
        for p in range(n_parts):
            if max_per_part > 0 and counts[p] >= max_per_part:
                continue
            if best is None or loads[p] < loads[best]:
                best = p
        if best is None:
            raise ValueError("max_per_part * n_parts < number of units")
        part_of[x] = best
        loads[best] += int(costs[x])
        counts[best] += 1
    return np.asarray(part_of, np.int32), np.asarray(loads, np.int64)


def imbalance(loads: Sequence[float]) -> float:
    """Eq. 2 objective: max load over mean load."""
    loads = [float(x) for x in loads]
    return max(loads) / (sum(loads) / len(loads))


# --------------------------------------------------------------------------- budgets (Section 3.2)
def shift_budgets(recovery: np.ndarray, total: int, lower: int, step: int = 1) -> Tuple[np.ndarray, int]:
    """Max-min sparsity budget shifting (Section 3.2).

    recovery[h][b]: attention-weight recovery ratio of head h under a budget of b units,
    b = 0 .. n_levels-1, non-decreasing in b.  `total` units are shared out, no head
    below `lower`.  Returns (budgets int64 [n_heads], number of moves made).

    The steps, in the paper's order: equal budgets; repeatedly move `step` units from
    the head with the highest recovery ratio (highest sparsity) to the head with the
    lowest; stop when (i) the giver has become the new minimum, i.e. further moves
    cannot help, or (ii) nobody above the lower bound is left to give.
    """
    rec = np.asarray(recovery, dtype=np.float64)
    n_heads, n_levels = rec.shape
    if n_heads < 1 or step < 1 or lower < 0:
        raise ValueError("bad arguments")
    if np.any(np.diff(rec, axis=1) < 0):
        raise ValueError("recovery curves must be non-decreasing")
    base, extra = divmod(int(total), n_heads)
    b = [base + (1 if h < extra else 0) for h in range(n_heads)]        # equal budgets
    if min(b) < lower or max(b) > n_levels - 1:
        raise ValueError("total does not fit between the lower bound and the curves' range")
    moves = 0
    while True:
        now = [rec[h][b[h]] for h in range(n_heads)]
        recv = min(range(n_heads), key=lambda h: (now[h], h))           # lowest recovery, then lowest index
        givers = [h for h in range(n_heads) if h != recv and b[h] - step >= lower]
        if not givers or b[recv] + step > n_levels - 1:
            break                                                       # (ii): nothing left to move
        give = min(givers, key=lambda h: (-now[h], h))                  # highest recovery, then lowest index
        after = list(now)
        after[give] = rec[give][b[give] - step]
        after[recv] = rec[recv][b[recv] + step]
        if min(after) < min(now):
            break                                                       # (i): the move would not help
        b[give] -= step
        b[recv] += step
        moves += 1
        if after[give] <= min(after):
            break                                                       # (i): the giver is the new minimum
    return np.asarray(b, dtype=np.int64), moves


# --------------------------------------------------------------------------- recovery profile (Section 2.4)
def block_mass(q_bits: np.ndarray, k_bits: np.ndarray, cu_seqlens: Sequence[int], block: int,
               softmax_scale: Optional[float] = None, rows: Optional[Sequence[int]] = None
               ) -> List[np.ndarray]:
    """Attention weight per (query block, key block), Eq. 1 weights under the causal mask:
    mass[s][h, i, j] = mean over the valid queries t of block i of sum over the keys u of
    block j (u <= t) of softmax_t(q_t . k_u * scale).  One [Hq, nb, nb] fp64 array per
    sequence, NaN where j > i and on rows not asked for (`rows`: global row indices as in
    row_index(); None = all)."""
    q = decode_bf16(q_bits)
    k = decode_bf16(k_bits)
    n_q_heads, n_kv_heads, d = q.shape[1], k.shape[1], q.shape[2]
    group = n_q_heads // n_kv_heads
    scale = 1.0 / math.sqrt(d) if softmax_scale is None else float(softmax_scale)
    cu = [int(x) for x in cu_seqlens]
    nbs = blocks_per_sequence(cu, block)
    want = None if rows is None else set(int(r) for r in rows)
    out = []
    for s, nb in enumerate(nbs):
        m = np.full((n_q_heads, nb, nb), np.nan)
        for h in range(n_q_heads):
            kh = k[cu[s]:cu[s + 1], h // group, :]
            for i in range(nb):
                if want is not None and row_index(cu, block, n_q_heads, s, h, i) not in want:
                    continue
                t0, t1 = cu[s] + i * block, min(cu[s] + (i + 1) * block, cu[s + 1])
                logits = q[t0:t1, h, :] @ kh[:t1 - cu[s]].T * scale              # [queries, keys so far]
                pos_q = np.arange(t0, t1)[:, None] - cu[s]
                pos_k = np.arange(t1 - cu[s])[None, :]
                logits = np.where(pos_k <= pos_q, logits, -np.inf)
                w = np.exp(logits - logits.max(axis=1, keepdims=True))
                w /= w.sum(axis=1, keepdims=True)
                for j in range(i + 1):
                    m[h, i, j] = w[:, j * block:(j + 1) * block].sum() / (t1 - t0)
        out.append(m)
    return out


def recovery_curves(mass: List[np.ndarray], cu_seqlens: Sequence[int], block: int) -> np.ndarray:
    """Recovery ratio per head and budget (Section 2.4, at block granularity):
    curves[h][b] = mean over all queries of head h (all sequences) of the mass of the b
    heaviest key blocks of the query's row; b = 0 .. max blocks.  A row with fewer than b
    visible blocks recovers its whole mass."""
    cu = [int(x) for x in cu_seqlens]
    nbs = blocks_per_sequence(cu, block)
    n_heads, n_levels = mass[0].shape[0], max(nbs) + 1
    curves = np.zeros((n_heads, n_levels))
    n_queries = 0
    for s, nb in enumerate(nbs):
        for i in range(nb):
            n_valid = min(block, cu[s + 1] - cu[s] - i * block)
            n_queries += n_valid
            for h in range(n_heads):
                heaviest_first = np.sort(mass[s][h, i, :i + 1])[::-1]
                cum = np.concatenate([[0.0], np.cumsum(heaviest_first)])
                row = np.full(n_levels, cum[-1])
                row[:i + 2] = cum
                curves[h] += n_valid * row
    return curves / n_queries


def selection_recovery(mass: List[np.ndarray], cu_seqlens: Sequence[int], block: int,
                       sel_ptr: np.ndarray, sel_idx: np.ndarray) -> np.ndarray:
    """Mean over all queries of a head of the mass its selected blocks hold: [n_heads]."""
    cu = [int(x) for x in cu_seqlens]
    nbs = blocks_per_sequence(cu, block)
    n_heads = mass[0].shape[0]
    got = np.zeros(n_heads)
    n_queries = 0
    for s, nb in enumerate(nbs):
        for i in range(nb):
            n_valid = min(block, cu[s + 1] - cu[s] - i * block)
            n_queries += n_valid
            for h in range(n_heads):
                r = row_index(cu, block, n_heads, s, h, i)
                got[h] += n_valid * mass[s][h, i, sel_idx[sel_ptr[r]:sel_ptr[r + 1]]].sum()
    return got / n_queries


def token_recovery(q_bits: np.ndarray, k_bits: np.ndarray, cu_seqlens: Sequence[int],
                   budgets: Sequence[int], softmax_scale: Optional[float] = None,
                   tokens: Optional[Sequence[int]] = None) -> np.ndarray:
    """Recovery ratio of Section 2.4 at token granularity: out[b, h, t] = sum of the budgets[b]
    largest attention weights (Eq. 1, causal) of query token t of head h; a query that sees at
    most budgets[b] keys recovers 1.  fp64 [len(budgets), Hq, T]; NaN at tokens not asked for
    (`tokens`: global token indices; None = all)."""
    q = decode_bf16(q_bits)
    k = decode_bf16(k_bits)
    n_q_heads, n_kv_heads, d = q.shape[1], k.shape[1], q.shape[2]
    group = n_q_heads // n_kv_heads
    scale = 1.0 / math.sqrt(d) if softmax_scale is None else float(softmax_scale)
    cu = [int(x) for x in cu_seqlens]
    out = np.full((len(budgets), n_q_heads, cu[-1]), np.nan)
    want = range(cu[-1]) if tokens is None else sorted(set(int(t) for t in tokens))
    for t in want:
        s = max(x for x in range(len(cu) - 1) if cu[x] <= t)
        for h in range(n_q_heads):
            logits = k[cu[s]:t + 1, h // group, :] @ q[t, h, :] * scale          # the keys the query sees
            w = np.exp(logits - logits.max())
            w /= w.sum()
            largest_first = np.sort(w)[::-1]
            for b, budget in enumerate(budgets):
                out[b, h, t] = 1.0 if budget >= len(w) else largest_first[:int(budget)].sum()
    return out


def token_recovery_heads(recovery: np.ndarray) -> np.ndarray:
    """Per-head figure: mean over the queries (all sequences) of token_recovery's output,
    [Hq, len(budgets)]; tokens not asked for (NaN) are left out."""
    return np.nanmean(recovery, axis=2).T
