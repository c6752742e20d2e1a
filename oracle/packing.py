"""Host step that turns a list of samples into packed micro-batches (oracle).

A sample whose length for this section is zero does not activate the section
and is dropped (a text-only sample bypasses the vision encoder: paper Sec. 2.1
and the worked example of Sec. 3.4, where a zero time before the critical
section marks such a sample).  The remaining samples are taken in the given
order, or longest first, and packed greedily under a per-section token budget
(each section has its own micro-batch size: Sec. 3.2).
"""


def pack_microbatches(lengths, token_budget, policy=0):
    """Returns (order, mb_offsets, cu_seqlens_per_mb).

    order: indices of the kept samples in execution order.
    mb_offsets: micro-batch m holds order[mb_offsets[m]:mb_offsets[m+1]].
    cu_seqlens_per_mb: one prefix-sum list (starting at 0) per micro-batch.
    A sample that does not fit into the open micro-batch closes it; a sample
    longer than the budget is placed alone.
    """
    kept = [i for i, n in enumerate(lengths) if n > 0]
    if policy == 1:
        kept = sorted(kept, key=lambda i: -lengths[i])  # stable: ties keep input order
    order, mb_offsets, cus = [], [0], []
    cur, tokens = [0], 0
    for i in kept:
        if tokens > 0 and tokens + lengths[i] > token_budget:
            cus.append(cur)
            mb_offsets.append(len(order))
            cur, tokens = [0], 0
        order.append(i)
        tokens += lengths[i]
        cur.append(tokens)
    if tokens > 0:
        cus.append(cur)
        mb_offsets.append(len(order))
    return order, mb_offsets, cus
