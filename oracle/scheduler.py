"""Plain statement of RServe's request bookkeeping (TEST INFRASTRUCTURE ONLY): the per-request embedding tracker
(section 3.1), encoder batching (Algorithm 1, section 3.2) and the schedulable-token scheduler (Algorithm 2,
section 3.3).  Pure-Python, token by token where that is the clearest statement; it shares no code with the library.

Readings of the paper taken here (the same as the library's header states):
  * "|buffer| >= C" in Algorithm 1 counts multimodal TOKENS (section 3.2: "batches containing at least C multimodal
    tokens"), and an item is never split.
  * Algorithm 2, a request with t > B schedulable tokens runs B of them (the listing sets B to 0 without saying so).
  * Algorithm 2's "t < p" is read as "tokens of the request remain un-prefilled after this round".
  * A request with t = 0 is still visited and joins S with zero tokens, as the listing adds every dequeued request.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple


@dataclass
class TrackedRequest:
    """Section 3.1: one readiness tag per token (True for text, False for multimodal until encoded) and a cursor."""
    request_id: int
    segments: List[Tuple[bool, int]]                 # (is_multimodal, n_tokens) in prompt order
    ready: List[bool] = field(default_factory=list)  # per token
    prefilled: int = 0

    def __post_init__(self):
        self.ready = []
        for is_mm, n in self.segments:
            self.ready += [not is_mm] * n

    @property
    def prompt_length(self) -> int:
        return len(self.ready)

    def mark_ready(self, segment: int) -> None:
        first = sum(n for _, n in self.segments[:segment])
        for tkn in range(first, first + self.segments[segment][1]):
            self.ready[tkn] = True

    def schedulable_tokens(self) -> int:
        """Section 3.3: a token is schedulable once its embedding is ready and every earlier token is prefilled or
        schedulable: count ready tokens from the cursor up to the first one that is not ready."""
        t = 0
        while self.prefilled + t < len(self.ready) and self.ready[self.prefilled + t]:
            t += 1
        return t


def encoder_batches(segments: Sequence[Tuple[bool, int]], c: int) -> List[List[int]]:
    """Algorithm 1 for one request: lists of segment indices, one list per Encode(buffer) call."""
    calls: List[List[int]] = []
    buffer: List[int] = []
    for idx, (is_mm, _) in enumerate(segments):
        if is_mm:
            buffer.append(idx)
            if sum(segments[i][1] for i in buffer) >= c:
                calls.append(buffer)
                buffer = []
    if buffer:
        calls.append(buffer)
    return calls


def schedule_round(queue: List[TrackedRequest], budget: int):
    """Algorithm 2, one iteration.  Returns (S, new_queue) with S = [(request, first_token, n_tokens)]; the requests'
    cursors are advanced (BatchExecute is the caller's business)."""
    q = list(queue)
    s = []
    u = []
    b = budget
    while q and b > 0:
        r = q.pop(0)
        t = r.schedulable_tokens()
        n = t if t <= b else b
        b = b - t if t <= b else 0
        s.append((r, r.prefilled, n))
        r.prefilled += n
        if r.prefilled < r.prompt_length:
            u.append(r)
    return s, u + q
