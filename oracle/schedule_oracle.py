"""CPU oracle for one epoch of a pack whose members use different batch sizes.  TEST
INFRASTRUCTURE ONLY: nothing in the product path may import, call or link this file.

What it computes (paper Section 3.2, second half, and Section 3.3).  The members of a pack share
one input stream.  At every step the shared batch has the size of the LARGEST batch among the
members still training, and a member with a smaller batch trains on the leading rows of it, so
after the largest-batch member has seen the whole dataset the others have seen only a fraction
(batch 50 next to batch 100: one half; batch 80: four fifths).  The usage of the dataset is
therefore recorded per member.  When the member with the largest batch has finished it leaves the
pack; the largest batch among the remaining members becomes the shared batch size, and the shared
batches are now cut from the samples THAT member has not used yet.  Those are, by construction,
unused by every other remaining member too.  This repeats until every member has used every
sample exactly once.

The oracle is that description carried out with sets of sample indices, one set per member, in
the order the text gives.  It contains no arithmetic beyond counting.

Readings where the text is silent:
  * the dataset is visited in index order (a shuffle is a permutation applied by the caller);
  * within a phase the pool of samples is cut into consecutive shared batches; when the pool does
    not divide by the batch size the last shared batch of the phase is short, and a member takes
    min(own batch size, rows available) rows of it - dropping the short batch would lose samples,
    which the text rules out;
  * members with equal batch size finish together; among them the lowest index names the phase.
"""
from __future__ import annotations


def epoch_schedule(n_samples, batch):
    """Schedule of one epoch over samples 0 .. n_samples-1 for members with batch sizes `batch`.

    Returns a list of steps.  Each step is a dict
      idx    list of dataset indices: row r of the shared batch is sample idx[r]
      rows   list over members: how many leading rows of the shared batch the member trains on
             (0: the member has finished and left the pack)
      lead   the member whose batch size is the shared batch size in this phase
    """
    K = len(batch)
    if K == 0 or n_samples < 1 or any(int(b) < 1 for b in batch):
        raise ValueError("need at least one member, one sample and positive batch sizes")
    unused = [set(range(n_samples)) for _ in range(K)]      # dataset usage, recorded per member
    finished = [False] * K
    steps = []
    while not all(finished):
        live = [k for k in range(K) if not finished[k]]
        lead = live[0]
        for k in live:                                      # largest batch, lowest index on ties
            if batch[k] > batch[lead]:
                lead = k
        pool = sorted(unused[lead])                         # what the leading member has not seen
        for s in range(0, len(pool), batch[lead]):
            shared = pool[s:s + batch[lead]]
            rows = [0] * K
            for k in live:
                take = shared[:batch[k]]
                if not set(take) <= unused[k]:
                    raise AssertionError("a member would see a sample twice")
                unused[k] -= set(take)
                rows[k] = len(take)
            steps.append({"idx": list(shared), "rows": rows, "lead": lead})
        for k in live:
            if not unused[k]:
                finished[k] = True
        if not finished[lead]:
            raise AssertionError("the leading member must finish its phase")
    return steps


def progress_after(steps, n_samples, K, upto):
    """Fraction of the dataset each member has used after the first `upto` steps."""
    used = [0] * K
    for st in steps[:upto]:
        for k in range(K):
            used[k] += st["rows"][k]
    return [u / float(n_samples) for u in used]
