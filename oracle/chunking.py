"""ORACLE -- test infrastructure only: chunk construction and chunk scheduling in plain Python.

Follows the paper's Algorithm 1 (section 4.1) and Algorithm 2 (section 4.2) step by step.  Where the
paper leaves a choice open the reading is stated at the step that takes it.

Pins: the paper's worked examples (lengths {1,1,2,4} Units with ChunkSize 2 and 4 Units give 4 and 2 chunks),
validity invariants on random lists, exhaustive minimum bin counts on tiny inputs, and the counts
section 4.2 states for Algorithm 2.  PARITY UNPINNED by the paper: WHICH valid packing Algorithm 1's
'try binpacking' step produces (the paper names no heuristic and prints no packing), and the whole
merge_tails variant (the paper prints no such chunking); both are pinned only by those invariants and by
hand-worked examples of the reading taken here.

A chunk is a dict:
    tokens      number of tokens in the chunk (<= chunk_size)
    prefix_len  tokens of the same long sequence that lie in earlier chunks (0 for packed chunks
                that hold no slice of a split sequence)
    group       id of its dependency group; idx_in_group its 0-based position there
    segments    list of (seq_id, seq_start, length): which tokens of which input sequence
A group is a dict: seq_id (the long sequence, or -1 for a packed chunk) and chunks (ids, ascending
dependency order = forward order).
"""


def _try_pack(order, n_bins, cap):
    """One bin-packing attempt (Algorithm 1, the 'try binpacking into BinCnt bins' step).

    order: items (seq_id, seq_start, length, is_tail), longest first.
    The paper names no heuristic.  Reading: each item goes to the bin with the smallest load (ties:
    lowest bin number), which keeps the chunks about equally full as section 1 asks; the attempt
    fails as soon as an item does not fit there.  With merged tails (see build_chunks) a tail only
    considers bins that hold no tail yet, and fails when there is none.
    """
    load = [0] * n_bins
    tails = [0] * n_bins
    members = [[] for _ in range(n_bins)]
    for item in order:
        length, is_tail = item[2], item[3]
        allowed = [x for x in range(n_bins) if not (is_tail and tails[x])]
        if not allowed:
            return None
        b = min(allowed, key=lambda x: (load[x], x))
        if load[b] + length > cap:           # limit is inclusive: a bin may be exactly full
            return None
        load[b] += length
        tails[b] += is_tail
        members[b].append(item)
    return members


def build_chunks(seq_lens, chunk_size, merge_tails=False):
    """Algorithm 1.  Returns (chunks, groups).

    merge_tails: a variant the algorithm leaves open (its listing appends every slice of a split
    sequence as a chunk of its own).  The last slice of a split sequence, when shorter than
    ChunkSize, becomes one more item of the bin-packing instead, so that it shares a chunk with
    short sequences; a chunk takes at most one tail, and the chunk that holds it is the last chunk
    of that sequence's dependency group.
    """
    lens = [int(x) for x in seq_lens]
    cap = int(chunk_size)
    if cap < 1 or any(x < 1 for x in lens):
        raise ValueError("chunk_size and every length must be >= 1")

    # 'longer than ChunkSize' are split; a sequence of exactly ChunkSize tokens is one full
    # standalone chunk (the paper's example: a 2-Unit sequence with ChunkSize 2 Units).
    long_ids = [i for i, x in enumerate(lens) if x > cap]
    items = [(i, 0, x, False) for i, x in enumerate(lens) if x <= cap]

    chunks, groups = [], []
    tail_group = {}
    for i in long_ids:                       # input order
        gid = len(groups)
        groups.append({"seq_id": i, "chunks": []})
        start, m = 0, 0
        while start < lens[i]:
            n = min(cap, lens[i] - start)
            if merge_tails and n < cap:
                items.append((i, start, n, True))
                tail_group[i] = (gid, m)
                break
            groups[gid]["chunks"].append(len(chunks))
            chunks.append({"tokens": n, "prefix_len": start, "group": gid, "idx_in_group": m,
                           "segments": [(i, start, n)]})
            start += n
            m += 1

    if items:
        order = sorted(items, key=lambda it: (-it[2], it[0]))
        bins = None
        for n_bins in range(1, len(items) + 1):         # first bin count that works wins
            bins = _try_pack(order, n_bins, cap)
            if bins is not None:
                break
        for members in bins:
            if not members:
                continue
            members = sorted(members)                    # input order inside a chunk
            segs = [(i, start, n) for (i, start, n, _) in members]
            tail = [it for it in members if it[3]]
            if tail:
                gid, m = tail_group[tail[0][0]]
                groups[gid]["chunks"].append(len(chunks))
                prefix = tail[0][1]
            else:
                gid, m, prefix = len(groups), 0, 0
                groups.append({"seq_id": -1, "chunks": [len(chunks)]})
            chunks.append({"tokens": sum(s[2] for s in segs), "prefix_len": prefix, "group": gid,
                           "idx_in_group": m, "segments": segs})
    return chunks, groups


FWD_KEEP, FWD_DISCARD, BWD = 0, 1, 2


def schedule_group(chunk_ids, K):
    """Algorithm 2 for one dependency group: list of (op, chunk_id).

    Readings of the printed listing, both forced by section 4.2's prose: the chunks whose
    activations are kept are the LAST K (the first N-K run forward twice), and the final loop
    visits the first N-K chunks in DESCENDING order (a chunk's key/value gradient needs every
    later chunk's contribution first).
    """
    if K < 1:
        raise ValueError("K must be >= 1")
    n = len(chunk_ids)
    ops = []
    if n <= K:
        ops += [(FWD_KEEP, c) for c in chunk_ids]
        ops += [(BWD, c) for c in reversed(chunk_ids)]
        return ops
    for m, c in enumerate(chunk_ids):
        ops.append((FWD_KEEP if m >= n - K else FWD_DISCARD, c))
    for c in reversed(chunk_ids[n - K:]):
        ops.append((BWD, c))
    for c in reversed(chunk_ids[:n - K]):
        ops.append((FWD_KEEP, c))
        ops.append((BWD, c))
    return ops


def build_schedule(groups, K):
    """Algorithm 2 applied to every group in group order; each group's ops are contiguous."""
    ops = []
    for g in groups:
        ops += schedule_group(list(g["chunks"]), K)
    return ops


def schedule_stats(chunks, groups, K):
    """Replay of Algorithm 2's schedule (section 4.2): how many passes it takes and how much it keeps.

    A FWD_KEEP op keeps its chunk's activations until that chunk's BWD op; FWD_DISCARD keeps nothing.
    Section 4.2 states the two facts this measures: the first N-K chunks of a group run forward
    twice, and the kept activations never exceed K chunks (memory governed by K * ChunkSize).
    The key/value state of a split sequence lives as long as its group is being processed.
    """
    tokens = {i: c["tokens"] for i, c in enumerate(chunks)}
    st = dict(n_forward=0, n_backward=0, n_reforward=0, peak_kept_chunks=0, peak_kept_tokens=0, state_tokens=0)
    kept = set()
    for op, c in build_schedule(groups, K):
        if op == BWD:
            st["n_backward"] += 1
            kept.remove(c)
        else:
            st["n_forward"] += 1
            if op == FWD_KEEP:
                kept.add(c)
                st["peak_kept_chunks"] = max(st["peak_kept_chunks"], len(kept))
                st["peak_kept_tokens"] = max(st["peak_kept_tokens"], sum(tokens[x] for x in kept))
    assert not kept
    st["n_reforward"] = st["n_forward"] - len(chunks)
    for g in groups:
        if g["seq_id"] >= 0:     # the split sequence's own tokens (a chunk with a merged tail also holds others)
            own = sum(n for c in g["chunks"] for (sid, _, n) in chunks[c]["segments"] if sid == g["seq_id"])
            st["state_tokens"] = max(st["state_tokens"], own)
    return st
