"""TEST INFRASTRUCTURE: token-based micro-batching, the paper's "TB" baseline.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module; it shares no
code with the product and never imports it.

Section "Motivation" (micro-batching methods figure: "micro-batches of the same token count, so that
there are fewer samples in micro-batches of larger sequence lengths") and section "Evaluation",
ablation of micro-batching ("TB ... splits micro-batches so that each micro-batch contains roughly
the same number of tokens", with the number of tokens per micro-batch found by search).

Plain definition taken here (the paper gives no more than the two sentences above):
  * samples are ordered as for the dynamic programme (ascending length; encoder-decoder: input
    length, then target length; equal keys keep their original order);
  * the ordered list is cut from the front; a micro-batch takes samples as long as
        (number of samples) x (longest sample in it)  <=  token budget,
    i.e. its PADDED token count stays within the budget, and is closed as soon as one more sample
    would exceed it.  For an encoder-decoder batch the count is that of the input stream (the
    same quantity the memory cap limits);
  * a single sample longer than the budget cannot be placed: no partition (None).

parity pins (tests/test_oracle_token_based.py): an example worked by hand; brute force over all
contiguous partitions (the result has the fewest micro-batches any admissible partition can have, and
its cut list is the lexicographically largest admissible one); every micro-batch admissible and not
extensible; closed forms for equal lengths and for budgets that bind nowhere / everywhere.
"""


def order(lengths, lengths_tgt=None):
    n = len(lengths)
    if lengths_tgt is None:
        return sorted(range(n), key=lambda i: (int(lengths[i]), i))
    return sorted(range(n), key=lambda i: (int(lengths[i]), int(lengths_tgt[i]), i))


def plan(lengths, budget, lengths_tgt=None):
    """-> dict(perm, cuts) or None when some sample alone exceeds the budget."""
    perm = order(lengths, lengths_tgt)
    ls = [int(lengths[i]) for i in perm]
    n = len(ls)
    cuts = [0]
    start = 0
    while start < n:
        if ls[start] > budget:
            return None
        end = start + 1
        while end < n and (end + 1 - start) * max(ls[start:end + 1]) <= budget:
            end += 1
        cuts.append(end)
        start = end
    return {"perm": perm, "cuts": cuts}
