"""Request-granular best-effort selection -- TEST INFRASTRUCTURE ONLY.

Paper section 4.4: under the best-effort policy the policy manager drops requests
from observation instead of stalling.  Drop-recent: the most recently added
requests go first (observability is retained on the requests closest to
finishing).  Keep-by-pattern: requests matching the user's predicate are
prioritised; when capacity is insufficient the others are dropped first.

Written out as the definition: rank the requests, keep the longest prefix of the
ranking whose cost fits the budget.

Pins (tests/test_policy_select.py, applied to this function directly): drop-recent keeps the
oldest requests, keep-by-pattern drops non-matching requests first, the kept set is a maximal
prefix of the ranking (adding the next request would exceed the budget).  Parity unpinned: tie-breaking and "prefix, not
best fit" are this build's readings of a strategy the paper describes in a sentence each.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

DROP_RECENT, KEEP_BY_PATTERN = 0, 1


def select(strategy: int, reqs: Sequence[Tuple[int, int, int, int]], bytes_per_row: int,
           budget_bytes: int) -> List[int]:
    """reqs: (req_id, rows, admit_order, matches) in batch order -> keep flag per request."""
    def rank(i):
        _, _, admit, matches = reqs[i]
        cls = 0 if (strategy == KEEP_BY_PATTERN and matches) else (1 if strategy == KEEP_BY_PATTERN else 0)
        return (cls, admit, i)

    keep = [0] * len(reqs)
    used = 0
    for i in sorted(range(len(reqs)), key=rank):
        cost = reqs[i][1] * bytes_per_row
        if used + cost > budget_bytes:
            break
        used += cost
        keep[i] = 1
    return keep
