"""Score-free simulator of TreeKV's span structure (test helper).

Every cache slot stands for a contiguous span of original positions and keeps
exactly one of them.  Which one depends on the scores; the spans themselves do
not: an eviction in scope (idx, idx+1) merges the two slots' spans (Section 4.1,
"Eviction Scope", with idx cycling left to right).  This file knows nothing of
attention; it only tracks [lo, hi] intervals.
"""


class SpanSim:
    def __init__(self, c, n_sink=0, n_recent=0):
        self.c, self.n_sink = c, n_sink
        self.m = c - n_sink - n_recent
        self.spans = []  # [lo, hi] inclusive, cache order
        self.idx0 = 0    # 0-based scope index inside the tree region
        self.t = 0

    def step(self):
        """Append token t.  Returns None, or (left_span, right_span) of the scope that merged."""
        self.spans.append([self.t, self.t])
        self.t += 1
        if len(self.spans) <= self.c:
            return None
        i = self.n_sink + self.idx0
        left, right = self.spans[i], self.spans[i + 1]
        scope = (tuple(left), tuple(right))
        self.spans[i:i + 2] = [[left[0], right[1]]]
        self.idx0 = (self.idx0 + 1) % self.m
        return scope

    def sizes(self):
        return [hi - lo + 1 for lo, hi in self.spans]
