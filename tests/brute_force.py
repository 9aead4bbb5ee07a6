"""Independent re-simulation of TreeKV on tiny inputs, used only to pin the oracle.

Pure Python: one list of dict records per stream, `list.pop` for eviction,
`math.fsum` for every sum.  Written from Algorithm 1 of the paper (Section 4.1),
separately from the C++ oracle: it shares nothing with it.
"""
import cmath
import math


def _softmax(xs):
    mx = max(xs)
    es = [math.exp(x - mx) for x in xs]
    tot = math.fsum(es)
    return [e / tot for e in es]


def _dot(a, b):
    return math.fsum(x * y for x, y in zip(a, b))


class BruteTreeKV:
    def __init__(self, c, G, d, n_sink=0, n_recent=0, scale=None, keep_left=False, literal_idx=False,
                 accumulated=False, rerank_base=None):
        self.c, self.G, self.d = c, G, d
        self.n_sink, self.m = n_sink, c - n_sink - n_recent
        self.scale = 1.0 / math.sqrt(d) if scale is None else scale
        self.keep_left, self.literal_idx, self.accumulated = keep_left, literal_idx, accumulated
        self.rerank_base = rerank_base   # not None: positions re-assigned to cache ranks, rotary encoding
        self.cache = []   # records: pos, k, v, S, C
        self.idx = 1      # 1-based, as printed in Algorithm 1
        self.t = 0

    def _logit(self, q, k, distance):
        if self.rerank_base is None:
            return _dot(q, k)
        # rotary encoding in its relative form: plane i contributes Re(q_i conj(k_i) e^{1j distance theta_i})
        total = []
        for i in range(self.d // 2):
            theta = self.rerank_base ** (-2.0 * i / self.d)
            total.append((complex(q[2 * i], q[2 * i + 1]) * complex(k[2 * i], -k[2 * i + 1])
                          * cmath.exp(1j * distance * theta)).real)
        return math.fsum(total)

    def _attend(self, q, visible):
        outs, probs = [], []
        n = len(visible)
        for g in range(self.G):
            a = _softmax([self.scale * self._logit(q[g], rec["k"], n - 1 - j) for j, rec in enumerate(visible)])
            outs.append([math.fsum(a[j] * visible[j]["v"][e] for j in range(len(visible)))
                         for e in range(self.d)])
            probs.append(a)
        return outs, probs

    def _maybe_evict(self, seq, sbar_of):
        """seq: list of records in cache order; returns evicted position or -1."""
        if len(seq) <= self.c:
            return -1
        i = self.n_sink + self.idx - 1
        left, right = seq[i], seq[i + 1]
        if self.keep_left or sbar_of(left) > sbar_of(right):
            gone = seq.pop(i + 1)
        else:
            gone = seq.pop(i)
        if self.literal_idx:
            self.idx = (self.idx + 1) % self.m + 1
        else:
            self.idx = self.idx % self.m + 1
        return gone["pos"]

    def decode_step(self, q, k, v):
        self.cache.append(dict(pos=self.t, k=list(k), v=list(v), S=0.0, C=0))
        outs, probs = self._attend(q, self.cache)
        for j, rec in enumerate(self.cache):
            rec["C"] += 1
            rec["S"] = math.fsum([rec["S"]] + [probs[g][j] for g in range(self.G)])
        ev = self._maybe_evict(self.cache, (lambda r: r["S"]) if self.accumulated else (lambda r: r["S"] / r["C"]))
        self.t += 1
        return outs, ev

    def prefill_chunk(self, Q, K, V):
        L = len(K)
        n0 = len(self.cache)
        full = self.cache + [dict(pos=self.t + i, k=list(K[i]), v=list(V[i]), S=0.0, C=0) for i in range(L)]
        outs = []
        for i in range(L):
            vis = full[: n0 + i + 1]
            o, probs = self._attend(Q[i], vis)
            outs.append(o)
            for j, rec in enumerate(vis):
                rec["C"] += 1
                rec["S"] = math.fsum([rec["S"]] + [probs[g][j] for g in range(self.G)])
        frozen = {id(rec): rec["S"] if self.accumulated else rec["S"] / rec["C"] for rec in full}
        seq = full[:n0]
        evs = []
        for i in range(L):
            seq.append(full[n0 + i])
            evs.append(self._maybe_evict(seq, lambda r: frozen[id(r)]))
        self.cache = seq
        self.t += L
        return outs, evs

    def prefill_prompt(self, Qw, K, V, b):
        """Section 4.2 on an empty cache: blocks of b tokens, the last block's queries score the prompt."""
        T = len(K)
        N = T // b
        toks = [dict(pos=j, k=list(K[j]), v=list(V[j]), parts=[], C=0) for j in range(T)]
        for i in range(b):
            vis = toks[: T - b + i + 1]
            _, probs = self._attend(Qw[i], vis)
            for j, rec in enumerate(vis):
                rec["C"] += 1
                rec["parts"] += [probs[g][j] for g in range(self.G)]
        sbar = [math.fsum(rec["parts"]) / (1 if self.accumulated else rec["C"]) for rec in toks]
        beta = [math.fsum(sbar[k * b:(k + 1) * b]) / b for k in range(N)]
        # Algorithm 1 with blocks for tokens
        cb, sink_b = self.c // b, -(-self.n_sink // b)
        recent_b = -(-(self.c - self.n_sink - self.m) // b)
        m_b = cb - sink_b - recent_b
        idx, seq, gone = 1, [], []
        for k in range(N):
            seq.append(k)
            if len(seq) <= cb:
                gone.append(-1)
                continue
            i = sink_b + idx - 1
            if self.keep_left or beta[seq[i]] > beta[seq[i + 1]]:
                gone.append(seq.pop(i + 1))
            else:
                gone.append(seq.pop(i))
            idx = idx % m_b + 1
        self.cache = []
        for k in seq:
            for j in range(k * b, (k + 1) * b):
                self.cache.append(dict(pos=j, k=toks[j]["k"], v=toks[j]["v"], S=sbar[j] * (1 if self.accumulated else T - j), C=T - j))
        self.t, self.idx = T, 1
        return gone, sbar, beta

    def positions(self):
        return [rec["pos"] for rec in self.cache]

    def scores(self):
        return [rec["S"] for rec in self.cache], [rec["C"] for rec in self.cache]
