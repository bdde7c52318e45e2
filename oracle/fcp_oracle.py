"""CPU oracle for one worker's block-level attention (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
HIP library must compute.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does, and this file
imports nothing from the product package.

What it follows (all from the paper):

* Attention definition (section "Attention Computation", the unnumbered
  equation): O = Softmax(Q K^T / sqrt(D), masked) V per head, causal or
  non-causal.  The printed equation writes the mask as an element-wise product
  inside the softmax; it is read here in the universal sense: masked entries are
  left out of the softmax.
* Context-parallel associativity (section "Context Parallelism"): results
  computed over slices of the context are reduced to the final output.  The
  partial oracle restricts the definition to a subset of key columns; the merge
  oracle is the log-sum-exp weighted combination, which restores the
  whole-sequence result exactly.
* Sharding policy (section "Block Distributor"): every sequence is cut into
  fixed-size blocks, the last one ragged; block dependencies follow from the
  mask (Fig. "Zig-Zag packing" caption, Fig. "congestion-free solver").
* Bottom-up coalescer (section "Communication Planner"): c consecutive
  KV blocks of a query block form one stage; here one stage = one partial slot.
* Backward: the paper states that the backward pass is implemented but prints
  no formula; the oracle is the analytic gradient of the forward definition.

Readings where the paper is silent (GQA mapping, LSE base, canonical table
order, empty slots) are stated beside the code that takes them.

Pinned by tests/test_oracle_pins.py (brute-force softmax, closed forms, a
library attention routine, finite differences, gradient invariants, the
block+merge == whole invariant, the Fig. "Zig-Zag packing" block counts).
"""
from __future__ import annotations

import numpy as np

FULL = 0   # every (row, col) of the pair is attended
DIAG = 1   # same block on both sides under a causal mask: col <= row
PACKED_FULL = 2   # same packed block on both sides: FULL restricted to (row, col) of one member sequence
PACKED_DIAG = 3   # same packed block on both sides: DIAG restricted to (row, col) of one member sequence


# --------------------------------------------------------------------------
# bf16 bit patterns -> fp64 (exact)
# --------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# S1 + S2: block table, pair list, slots (integer work)
# --------------------------------------------------------------------------
def plan_blocks(seq_lens, block_size, causal=1, coalesce=0, q_owned=None):
    """Sharding policy G plus the worker's dependency list.

    Every sequence of length L becomes ceil(L / block_size) blocks, the last of
    length L - (n-1)*block_size (section "Block Distributor", sharding policy);
    a zero-length sequence yields no block.  KV blocks of all sequences are
    resident; the worker owns the query side of `q_owned` ((seq, idx) rows; None
    = every block).

    Dependencies (mask-derived, as in the Zig-Zag figure's caption: under a
    causal mask the i-th query block computes with KV blocks 0..i of its own
    sequence): causal -> (i, j, FULL) for j < i and (i, i, DIAG); non-causal ->
    (i, j, FULL) for every j of the sequence.

    Reading (paper silent): tables are in canonical order -- blocks by (seq,
    idx); pairs by (q block, kv block); the r-th pair of a query block falls in
    that block's local slot r // c (c = coalesce, 0 = one slot for all); slots
    are numbered globally in that order, and slot k of a query block with
    `tok_len` rows owns rows [row_start, row_start + tok_len) of the partial
    buffers.

    Returns int32 arrays:
      kv_blocks [n, 4] = (seq, idx, tok_start in the KV buffer, tok_len)
      q_blocks  [n, 4] = (seq, idx, tok_start in the Q buffer, tok_len)
      pairs     [n, 4] = (q_blk, kv_blk, kind, slot)      (indices into the tables)
      slots     [n, 4] = (q_blk, pair_begin, n_pairs, row_start)
      n_slot_rows
    """
    seq_lens = [int(x) for x in np.asarray(seq_lens).reshape(-1)]
    bs = int(block_size)
    c = int(coalesce)
    if bs <= 0 or c < 0 or any(L < 0 for L in seq_lens):
        raise ValueError("invalid argument")
    kv_blocks = []
    first_blk = []          # index of block 0 of each sequence in kv_blocks
    nblk = []
    tok = 0
    for s, L in enumerate(seq_lens):
        n = -(-L // bs)
        first_blk.append(len(kv_blocks))
        nblk.append(n)
        for i in range(n):
            ln = min(bs, L - i * bs)
            kv_blocks.append((s, i, tok, ln))
            tok += ln
    if q_owned is None:
        owned = [(b[0], b[1]) for b in kv_blocks]
    else:
        owned = [(int(a), int(b)) for a, b in np.asarray(q_owned).reshape(-1, 2)]
        for s, i in owned:
            if not (0 <= s < len(seq_lens)) or not (0 <= i < nblk[s]):
                raise ValueError("owned block out of range")
        if any(owned[t] >= owned[t + 1] for t in range(len(owned) - 1)):
            raise ValueError("q_owned must be strictly increasing in (seq, idx)")
    q_blocks = []
    qtok = 0
    for s, i in owned:
        ln = kv_blocks[first_blk[s] + i][3]
        q_blocks.append((s, i, qtok, ln))
        qtok += ln
    pairs, slots = [], []
    row = 0
    for qb, (s, i, _, ln) in enumerate(q_blocks):
        js = range(i + 1) if causal else range(nblk[s])
        for r, j in enumerate(js):
            opens_slot = (r == 0) if c == 0 else (r % c == 0)
            if opens_slot:
                slots.append([qb, len(pairs), 0, row])
                row += ln
            kind = DIAG if (causal and j == i) else FULL
            pairs.append((qb, first_blk[s] + j, kind, len(slots) - 1))
            slots[-1][2] += 1
    mk = lambda rows: np.asarray(rows, dtype=np.int32).reshape(-1, 4)
    return dict(kv_blocks=mk(kv_blocks), q_blocks=mk(q_blocks), pairs=mk(pairs), slots=mk(slots),
                n_slot_rows=int(row))


def plan_blocks_packed(seq_lens, block_size, causal=1, coalesce=0, q_owned=None, unit_of_block=None):
    """plan_blocks with the short sequences of a scheduling unit sharing one block (section "Block
    Distributor", sharding policy: sequences shorter than the block size are packed into as few
    blocks as possible and go through the variable-length path).

    `unit_of_block` names the unit of every block of the unpacked table (fcp_sched_oracle.pack_units
    writes it).  Reading (paper silent on the layout): a unit of two or more blocks -- each a whole
    sequence shorter than a block, together at most block_size tokens -- becomes ONE block that
    stands where its lowest member stood, holds its members in ascending order of their unpacked
    block index and carries that member's seq with idx 0; it has one pair, with itself
    (PACKED_DIAG under a causal mask, else PACKED_FULL), hence one slot.  Everything else is planned
    as by plan_blocks.  A unit is owned as a whole or not at all.

    Returns the plan_blocks tables plus
      segments [n, 4] = (kv_blk, seq, tok_off, tok_len): the members of every packed block.
    """
    seq_lens = [int(x) for x in np.asarray(seq_lens).reshape(-1)]
    bs = int(block_size)
    c = int(coalesce)
    if bs <= 0 or c < 0 or any(L < 0 for L in seq_lens):
        raise ValueError("invalid argument")
    flat = []               # unpacked blocks: (seq, idx, len)
    for s, L in enumerate(seq_lens):
        for i in range(-(-L // bs)):
            flat.append((s, i, min(bs, L - i * bs)))
    unit = list(range(len(flat))) if unit_of_block is None else [int(u) for u in np.asarray(unit_of_block).reshape(-1)]
    if len(unit) != len(flat):
        raise ValueError("unit_of_block must have one entry per unpacked block")
    members = {}
    for b, u in enumerate(unit):
        members.setdefault(u, []).append(b)
    for u, bl in members.items():
        if len(bl) >= 2:
            if any(flat[b][1] != 0 or flat[b][2] >= bs or seq_lens[flat[b][0]] != flat[b][2] for b in bl):
                raise ValueError("a packed unit may only hold whole sequences shorter than a block")
            if sum(flat[b][2] for b in bl) > bs:
                raise ValueError("a packed unit does not fit into one block")
    if q_owned is None:
        owned = set(range(len(flat)))
    else:
        rows = [(int(a), int(b)) for a, b in np.asarray(q_owned).reshape(-1, 2)]
        if any(rows[t] >= rows[t + 1] for t in range(len(rows) - 1)):
            raise ValueError("q_owned must be strictly increasing in (seq, idx)")
        index = {(s, i): b for b, (s, i, _) in enumerate(flat)}
        if any(r not in index for r in rows):
            raise ValueError("owned block out of range")
        owned = set(index[r] for r in rows)
    kv_blocks, q_blocks, segments, pairs, slots = [], [], [], [], []
    kv_of_flat = {}          # unpacked block -> index in kv_blocks (lowest member for a packed block)
    tok = 0
    for b, (s, i, ln) in enumerate(flat):
        bl = members[unit[b]]
        if len(bl) >= 2:
            if b != bl[0]:
                continue
            off = 0
            for m in bl:
                segments.append((len(kv_blocks), flat[m][0], off, flat[m][2]))
                off += flat[m][2]
            ln = off
        kv_of_flat[b] = len(kv_blocks)
        kv_blocks.append((s, 0 if len(bl) >= 2 else i, tok, ln))
        tok += ln
    nblk = {}
    first = {}
    for b, (s, i, _) in enumerate(flat):
        nblk[s] = nblk.get(s, 0) + 1
        first.setdefault(s, b)
    row = qtok = 0
    for b, (s, i, _) in enumerate(flat):
        bl = members[unit[b]]
        packed = len(bl) >= 2
        if packed:
            own = [m in owned for m in bl]
            if any(own) and not all(own):
                raise ValueError("a packed unit must be owned as a whole")
            if b != bl[0]:
                continue
        if b not in owned:
            continue
        kb = kv_of_flat[b]
        ln = kv_blocks[kb][3]
        qb = len(q_blocks)
        q_blocks.append((kv_blocks[kb][0], kv_blocks[kb][1], qtok, ln))
        qtok += ln
        if packed:
            slots.append([qb, len(pairs), 1, row])
            row += ln
            pairs.append((qb, kb, PACKED_DIAG if causal else PACKED_FULL, len(slots) - 1))
            continue
        js = range(i + 1) if causal else range(nblk[s])
        for r, j in enumerate(js):
            if (r == 0) if c == 0 else (r % c == 0):
                slots.append([qb, len(pairs), 0, row])
                row += ln
            pairs.append((qb, kv_of_flat[first[s] + j], DIAG if (causal and j == i) else FULL, len(slots) - 1))
            slots[-1][2] += 1
    mk = lambda rows: np.asarray(rows, dtype=np.int32).reshape(-1, 4)
    return dict(kv_blocks=mk(kv_blocks), q_blocks=mk(q_blocks), pairs=mk(pairs), slots=mk(slots),
                n_slot_rows=int(row), segments=mk(segments))


def packed_row_maps(plan, seq_lens, block_size, q_owned=None):
    """Where the rows of a packed plan's buffers sit in the sequence-major layout that worker_fwd /
    worker_bwd use: kv_src[r] = row of the sequence-major K / V buffer held by row r of the plan's
    K / V buffer; q_src[r] likewise for the Q buffers (sequence-major Q = the owned rows by sequence
    and position, as _owned_positions orders them)."""
    seq_lens = [int(x) for x in np.asarray(seq_lens).reshape(-1)]
    bs = int(block_size)
    seq_off = np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int64)
    seg_of = {}
    for kb, s, off, ln in plan.get("segments", np.zeros((0, 4), np.int32)):
        seg_of.setdefault(int(kb), []).append((int(s), int(off), int(ln)))
    kv_index = {(int(b[0]), int(b[1])): n for n, b in enumerate(plan["kv_blocks"])}

    def block_tokens(s, i, ln, kb):
        """(seq, position) of every token of a block, in buffer order"""
        if kb in seg_of:
            return [(ms, p) for ms, _, mlen in seg_of[kb] for p in range(mlen)]
        return [(s, i * bs + p) for p in range(ln)]

    kv_src = []
    for kb, (s, i, _, ln) in enumerate(plan["kv_blocks"]):
        kv_src += [seq_off[ms] + p for ms, p in block_tokens(int(s), int(i), int(ln), kb)]
    # sequence-major Q row of (seq, position): rank among the owned rows
    pos = _owned_positions(seq_lens, bs, q_owned)
    q_row = {}
    n = 0
    for s, pp in enumerate(pos):
        for p in pp:
            q_row[(s, int(p))] = n
            n += 1
    q_src = []
    for s, i, _, ln in plan["q_blocks"]:
        kb = kv_index[(int(s), int(i))]
        q_src += [q_row[t] for t in block_tokens(int(s), int(i), int(ln), kb)]
    return np.asarray(kv_src, dtype=np.int64), np.asarray(q_src, dtype=np.int64)


def pair_nnz(plan) -> int:
    """Number of unmasked score entries over all pairs (per query head).
    FULL m x n -> m*n; DIAG m x m -> m(m+1)/2; the PACKED kinds: the same, member by member."""
    seg_of = {}
    for kb, _, _, ln in plan.get("segments", np.zeros((0, 4), np.int32)):
        seg_of.setdefault(int(kb), []).append(int(ln))
    tot = 0
    for qb, kb, kind, _ in plan["pairs"]:
        m = int(plan["q_blocks"][qb][3])
        n = int(plan["kv_blocks"][kb][3])
        if kind in (PACKED_FULL, PACKED_DIAG):
            tot += sum(x * (x + 1) // 2 if kind == PACKED_DIAG else x * x for x in seg_of[int(kb)])
        else:
            tot += m * (m + 1) // 2 if kind == DIAG else m * n
    return tot


# --------------------------------------------------------------------------
# The definition, one sequence at a time
# --------------------------------------------------------------------------
def _kv_head(h, n_q_heads, n_kv_heads):
    # Reading (paper silent on the GQA mapping): contiguous groups.
    return (h * n_kv_heads) // n_q_heads


def _scores(qh, kh, scale, q_pos, k_pos, causal):
    """scale * q k^T with excluded entries set to -inf.  q_pos/k_pos are token
    positions inside the sequence; causal: key j is visible to query i iff
    pos_j <= pos_i (section "Attention Computation")."""
    s = (qh @ kh.T) * scale
    if causal:
        s = np.where(k_pos[None, :] <= q_pos[:, None], s, -np.inf)
    return s


def _softmax_rows(s):
    """Row-wise one-shot softmax and its log-sum-exp (natural log of the sum of
    exp of the scaled scores).  A row with no visible key gets P = 0, LSE = -inf."""
    m = np.max(s, axis=1, keepdims=True) if s.shape[1] else np.full((s.shape[0], 1), -np.inf)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    p = np.exp(s - m_safe)
    l = np.sum(p, axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(l > 0, m_safe + np.log(l), -np.inf)
        p = np.where(l > 0, p / np.where(l > 0, l, 1.0), 0.0)
    return p, lse[:, 0]


def attention_fwd_seq(q, k, v, causal=True, scale=None, q_pos=None, k_pos=None, row_chunk=1024):
    """O and LSE of query rows `q` [Lq, Hq, d] against keys/values `k`, `v`
    [Lk, Hkv, d] of the same sequence (fp64).  q_pos / k_pos default to
    0..L-1.  Restricting k, v, k_pos to a subset of the columns gives a
    *partial* result over that subset (normalised over the subset)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    Lq, Hq, d = q.shape
    Lk, Hkv, _ = k.shape
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    q_pos = np.arange(Lq) if q_pos is None else np.asarray(q_pos)
    k_pos = np.arange(Lk) if k_pos is None else np.asarray(k_pos)
    o = np.zeros((Lq, Hq, d))
    lse = np.full((Lq, Hq), -np.inf)
    for h in range(Hq):
        g = _kv_head(h, Hq, Hkv)
        kh = np.ascontiguousarray(k[:, g, :])
        vh = np.ascontiguousarray(v[:, g, :])
        for r0 in range(0, Lq, row_chunk):
            r1 = min(Lq, r0 + row_chunk)
            s = _scores(q[r0:r1, h, :], kh, scale, q_pos[r0:r1], k_pos, causal)
            p, l = _softmax_rows(s)
            o[r0:r1, h, :] = p @ vh
            lse[r0:r1, h] = l
    return o, lse


def attention_bwd_seq(q, k, v, d_o, causal=True, scale=None, q_pos=None, k_pos=None, row_chunk=1024):
    """Gradients of sum(O * d_o) w.r.t. q, k, v for the forward above.
    With P the softmax matrix of a head: dV = P^T dO; dP = dO V^T;
    D_i = sum_c dO_ic O_ic; dS = P o (dP - D); dQ = scale dS K; dK = scale dS^T Q;
    dK, dV are summed over the query heads that share a KV head."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    Lq, Hq, d = q.shape
    Lk, Hkv, _ = k.shape
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    q_pos = np.arange(Lq) if q_pos is None else np.asarray(q_pos)
    k_pos = np.arange(Lk) if k_pos is None else np.asarray(k_pos)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for h in range(Hq):
        g = _kv_head(h, Hq, Hkv)
        kh = np.ascontiguousarray(k[:, g, :])
        vh = np.ascontiguousarray(v[:, g, :])
        for r0 in range(0, Lq, row_chunk):
            r1 = min(Lq, r0 + row_chunk)
            qh = q[r0:r1, h, :]
            doh = d_o[r0:r1, h, :]
            p, _ = _softmax_rows(_scores(qh, kh, scale, q_pos[r0:r1], k_pos, causal))
            oh = p @ vh
            dv[:, g, :] += p.T @ doh
            dp = doh @ vh.T
            dd = np.sum(doh * oh, axis=1, keepdims=True)
            ds = p * (dp - dd)
            dq[r0:r1, h, :] = scale * (ds @ kh)
            dk[:, g, :] += scale * (ds.T @ qh)
    return dq, dk, dv


# --------------------------------------------------------------------------
# The worker's share on the packed buffers (whole sequences, no blocks)
# --------------------------------------------------------------------------
def _owned_positions(seq_lens, block_size, q_owned):
    """For each sequence: token positions of the worker's query rows, in the
    order they sit in the packed Q buffer (owned blocks in (seq, idx) order)."""
    per_seq = [[] for _ in seq_lens]
    if q_owned is None:
        for s, L in enumerate(seq_lens):
            per_seq[s] = np.arange(int(L))
        return per_seq
    for s, i in np.asarray(q_owned).reshape(-1, 2):
        L = int(seq_lens[s])
        lo = int(i) * block_size
        per_seq[int(s)].append(np.arange(lo, min(L, lo + block_size)))
    return [np.concatenate(p) if len(p) else np.arange(0) for p in per_seq]


def worker_fwd(q_bits, k_bits, v_bits, seq_lens, block_size, causal=1, q_owned=None, scale=None):
    """Whole-sequence attention for every owned query row.
    q_bits [Tq, Hq, d], k_bits/v_bits [Tkv, Hkv, d] are bf16 bit patterns in
    the packed token-major layout.  Returns O [Tq, Hq, d], LSE [Tq, Hq] in fp64."""
    pos = _owned_positions(seq_lens, block_size, q_owned)
    Tq, Hq, d = q_bits.shape
    o = np.zeros((Tq, Hq, d))
    lse = np.full((Tq, Hq), -np.inf)
    qoff = koff = 0
    for s, L in enumerate(seq_lens):
        L = int(L)
        n = len(pos[s])
        if n:
            qs = bf16_to_f64(q_bits[qoff:qoff + n])
            ks = bf16_to_f64(k_bits[koff:koff + L])
            vs = bf16_to_f64(v_bits[koff:koff + L])
            o[qoff:qoff + n], lse[qoff:qoff + n] = attention_fwd_seq(
                qs, ks, vs, bool(causal), scale, q_pos=pos[s], k_pos=np.arange(L))
        qoff += n
        koff += L
    return o, lse


def worker_bwd(q_bits, k_bits, v_bits, do_bits, seq_lens, block_size, causal=1, q_owned=None, scale=None):
    """Gradients for the worker's share: dQ for owned rows; dK, dV = the owned
    rows' contribution to every resident KV row (what the worker would push back
    to the KV owners).  Returns dq [Tq,Hq,d], dk, dv [Tkv,Hkv,d] in fp64."""
    pos = _owned_positions(seq_lens, block_size, q_owned)
    dq = np.zeros(q_bits.shape)
    dk = np.zeros(k_bits.shape)
    dv = np.zeros(v_bits.shape)
    qoff = koff = 0
    for s, L in enumerate(seq_lens):
        L = int(L)
        n = len(pos[s])
        if n:
            a, b, c = attention_bwd_seq(
                bf16_to_f64(q_bits[qoff:qoff + n]), bf16_to_f64(k_bits[koff:koff + L]),
                bf16_to_f64(v_bits[koff:koff + L]), bf16_to_f64(do_bits[qoff:qoff + n]),
                bool(causal), scale, q_pos=pos[s], k_pos=np.arange(L))
            dq[qoff:qoff + n] = a
            dk[koff:koff + L] = b
            dv[koff:koff + L] = c
        qoff += n
        koff += L
    return dq, dk, dv


def rows_fwd(q_bits, k_bits, v_bits, seq_lens, block_size, plan, q_rows, causal=1, scale=None):
    """O, LSE for a sample of Q-buffer rows only (each against all visible keys
    of its sequence).  `plan` is this module's plan_blocks output (used only to
    find the sequence and position of a Q-buffer row)."""
    qb_tab = plan["q_blocks"]
    starts = qb_tab[:, 2]
    seq_off = np.concatenate([[0], np.cumsum(np.asarray(seq_lens, dtype=np.int64))])
    Hq, d = q_bits.shape[1:]
    o = np.zeros((len(q_rows), Hq, d))
    lse = np.zeros((len(q_rows), Hq))
    for t, r in enumerate(q_rows):
        b = int(np.searchsorted(starts, r, side="right") - 1)
        s, i, st, _ = (int(x) for x in qb_tab[b])
        p = i * block_size + (int(r) - st)
        L = int(seq_lens[s])
        hi = p + 1 if causal else L
        k0 = int(seq_off[s])
        o[t], lse[t] = (x[0] for x in attention_fwd_seq(
            bf16_to_f64(q_bits[r:r + 1]), bf16_to_f64(k_bits[k0:k0 + hi]), bf16_to_f64(v_bits[k0:k0 + hi]),
            False, scale))
    return o, lse


# --------------------------------------------------------------------------
# Partials per slot, and their merge
# --------------------------------------------------------------------------
def partial_fwd(q_bits, k_bits, v_bits, plan, block_size, causal=1, scale=None):
    """The definition restricted, slot by slot, to the slot's KV columns.
    Returns O_part [n_slot_rows, Hq, d] and LSE_part [n_slot_rows, Hq] (fp64);
    each partial is normalised over its own columns.  An empty slot cannot
    arise from plan_blocks; a row with no visible column gets O = 0, LSE = -inf."""
    Hq, d = q_bits.shape[1:]
    o = np.zeros((plan["n_slot_rows"], Hq, d))
    lse = np.full((plan["n_slot_rows"], Hq), -np.inf)
    for qb, p0, npairs, row0 in plan["slots"]:
        _, qi, qst, qln = (int(x) for x in plan["q_blocks"][qb])
        cols = []
        kpos = []
        for _, kb, _, _ in plan["pairs"][p0:p0 + npairs]:
            _, kj, kst, kln = (int(x) for x in plan["kv_blocks"][kb])
            cols.append(np.arange(kst, kst + kln))
            kpos.append(kj * block_size + np.arange(kln))
        cols = np.concatenate(cols)
        kpos = np.concatenate(kpos)
        o[row0:row0 + qln], lse[row0:row0 + qln] = attention_fwd_seq(
            bf16_to_f64(q_bits[qst:qst + qln]), bf16_to_f64(k_bits[cols]), bf16_to_f64(v_bits[cols]),
            bool(causal), scale, q_pos=qi * block_size + np.arange(qln), k_pos=kpos)
    return o, lse


def merge_partials(o_part, lse_part, plan):
    """Reduce the partials of every query block (section "Context Parallelism":
    intermediate results over slices are reduced to the final output):
      LSE = ln sum_p exp(LSE_p),  O = sum_p exp(LSE_p - LSE) O_p.
    exp(-inf) counts as 0; a row whose partials are all empty gets O = 0,
    LSE = -inf.  Returns O [Tq, Hq, d], LSE [Tq, Hq] (fp64)."""
    o_part = np.asarray(o_part, dtype=np.float64)
    lse_part = np.asarray(lse_part, dtype=np.float64)
    qb_tab = plan["q_blocks"]
    Tq = int(np.sum(qb_tab[:, 3], dtype=np.int64))
    Hq, d = o_part.shape[1:]
    o = np.zeros((Tq, Hq, d))
    lse = np.full((Tq, Hq), -np.inf)
    by_q = {}
    for qb, _, _, row0 in plan["slots"]:
        by_q.setdefault(int(qb), []).append(int(row0))
    for qb, rows in by_q.items():
        _, _, qst, qln = (int(x) for x in qb_tab[qb])
        ls = np.stack([lse_part[r:r + qln] for r in rows])          # [P, qln, Hq]
        os_ = np.stack([o_part[r:r + qln] for r in rows])           # [P, qln, Hq, d]
        m = np.max(ls, axis=0)
        m_safe = np.where(np.isfinite(m), m, 0.0)
        w = np.exp(ls - m_safe[None])
        tot = np.sum(w, axis=0)
        with np.errstate(divide="ignore", invalid="ignore"):
            lse[qst:qst + qln] = np.where(tot > 0, m_safe + np.log(tot), -np.inf)
            wn = np.where(tot[None] > 0, w / np.where(tot > 0, tot, 1.0)[None], 0.0)
        o[qst:qst + qln] = np.sum(wn[..., None] * os_, axis=0)
    return o, lse


def stage_tables(plan, stage):
    """The tables of one execution stage (section "Communication Planner": a worker runs its
    stages one after the other and reduces each stage's result into what it has so far).  Stage
    k = the k-th slot of every query block that has one; its slots are renumbered, its pairs
    point at them, and a slot's rows are the rows of its query block in the Q buffer (a partial
    buffer of one stage has the layout of the final output).  Returns (pairs [n,4], slots [n,4],
    n_stages) with n_stages = the largest number of slots of any query block."""
    pairs, slots = [], []
    local = {}
    most = 0
    for qb, p0, npairs, _ in (tuple(int(x) for x in row) for row in plan["slots"]):
        k = local.get(qb, 0)
        local[qb] = k + 1
        most = max(most, k + 1)
        if k != stage:
            continue
        slots.append((qb, len(pairs), npairs, int(plan["q_blocks"][qb][2])))
        for q, kv, kind, _ in plan["pairs"][p0:p0 + npairs]:
            pairs.append((int(q), int(kv), int(kind), len(slots) - 1))
    return (np.asarray(pairs, dtype=np.int32).reshape(-1, 4), np.asarray(slots, dtype=np.int32).reshape(-1, 4), most)


# --------------------------------------------------------------------------
# FLOP model used for the reported throughput
# --------------------------------------------------------------------------
def flops(plan, n_q_heads, head_dim):
    """Causal-adjusted FLOPs: forward 4 d per unmasked score entry per query
    head (two contractions), backward 10 d (five contractions)."""
    nnz = pair_nnz(plan)
    return 4 * head_dim * n_q_heads * nnz, 10 * head_dim * n_q_heads * nnz
