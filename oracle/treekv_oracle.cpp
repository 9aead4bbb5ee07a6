// TreeKV CPU oracle: TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, slow, scalar fp64 implementation of the TreeKV cache step for ONE
// (batch, kv-head) stream, written from the paper (Algorithm 1 "Compression by
// TreeKV", Section 4.1; attention of Section 3.1).  Only tests, the smoke check
// and the benchmark's cpu_baseline leg may build, load or call it.  It shares
// no code, header, table or helper with the HIP library.
//
// What it follows, step by step (Algorithm 1, one loop iteration):
//   K, V grow by the new row                                   (the append step)
//   a = SoftMax(q K^T * scale) over the whole cache, o = a V   (the attention step, Sec. 3.1)
//   C = (C u {0}) + 1,  S = (S u {0}) + a                      (the C and S updates)
//   if length > c:  Sbar = S / C; compare Sbar[idx], Sbar[idx+1];
//                   evict idx+1 if Sbar[idx] > Sbar[idx+1], else evict idx;
//                   advance idx                                (the eviction block)
// Eviction is a std::vector erase on every per-token array; nothing is blocked,
// fused or reordered.
//
// Readings of the paper taken here (each also listed in the design notes):
//  * idx advance.  The printed update "(idx+1) mod c + 1" skips every other
//    scope, contradicting Section 4.1, whose example has idx take 1, 2, 3, 4 in turn.
//    Default: idx <- (idx mod m) + 1.  The printed form is kept behind
//    TKO_IDX_LITERAL.
//  * Layout.  Section 5.2 keeps 4 initial and 508 recent tokens next to 512
//    method-selected ones.  The cache is [n_sink | m tree slots | n_recent]
//    with m = c - n_sink - n_recent; Algorithm 1's scope indexes the tree
//    region, i.e. logical slots (n_sink+idx, n_sink+idx+1), and its cycle
//    length is m.  n_sink = n_recent = 0 is Algorithm 1 verbatim.
//  * Grouped queries (paper silent).  The G query heads that share this KV
//    head all attend; S adds the sum of their probabilities, C adds 1.
//  * Ties.  The comparison is a strict ">", so equal scores evict idx.
//  * Ablation of Section 5.4 (always keep the left token): TKO_KEEP_LEFT.
//  * Importance criterion.  Section 4.1 names the averaged attention weight Sbar = S / C as the
//    criterion of choice and mentions that accumulated weights were tried too: with
//    TKO_SCORE_ACCUMULATED the averaging step is skipped and the comparison is on S itself.  (In the
//    one-shot prompt compression a token's importance is then its summed, not averaged, window
//    attention, and S is handed over as it is.)
//  * Chunked prefill (not in the paper, whose prefill works on blocks with an
//    observation window; Section 4.2 only says scores and scopes are computed
//    ahead of the selection).  A chunk of L tokens attends the cache as it
//    was before the chunk plus the chunk's own tokens up to and including
//    itself; S and C are updated with every row; Sbar is then frozen and
//    Algorithm 1's append / compare / evict / advance is replayed for the L
//    tokens in order.  L = 1 is exactly a decode step.
//
//  * One-shot prompt compression (Section 4.2, "Prefilling Stage").  The prompt is cut into
//    blocks of b tokens; the queries of the last block (the observation window) attend the
//    whole prompt causally; a token's importance is its attention averaged over the window
//    queries that see it (S / C of Algorithm 1 restricted to those queries, summed over the
//    group's heads); a block's importance is the mean over its b tokens; Algorithm 1
//    (append, then the eviction block) then runs with blocks in the place of tokens, the block scores frozen,
//    a capacity of c / b blocks and ceil(n_sink / b) sink and ceil(n_recent / b) recent
//    blocks.  The paper does not say how decoding takes over; here the kept tokens keep their
//    window average as Sbar: C becomes the number of prompt queries since the token arrived
//    (T - position) and S = Sbar * C, and token-level eviction starts at idx = 1.
//  * Position re-assignment (Section 4.1, "Position Encoding").  With TKO_POSITION_RERANK the
//    stream holds keys WITHOUT positional encoding; at every step the cached tokens, in cache
//    order and including the new one, are given the positions 0, 1, .., n-1 (the paper's
//    example: tokens {0,1,2,3,7,8,9} and the 10th get {0,..,7}), and the rotary encoding of
//    those positions is applied to the keys and (position n-1) to the query before the attention step.
//    The rotary encoding is the one of its defining paper (RoFormer, eq. 15/34): dimensions
//    (2i, 2i+1) form a plane rotated by position * base^(-2i/d), base 10000 unless set.  The
//    paper does not say which flavour its models use; a model that pairs (i, i + d/2) instead
//    permutes the head dimension of q and k accordingly.  In the one-shot prompt compression
//    nothing has been evicted yet when the window scores the prompt, so the positions are the
//    original ones (key j at j, window query i at T - W + i); the cache it leaves holds the keys
//    unencoded, as decoding expects.  A prefill chunk (this build's own call, see above) is scored
//    before any of its tokens is evicted: the n0 cached tokens are at positions 0 .. n0-1 and chunk
//    token i at n0 + i, which for a chunk of one token is the decode step's rule.
//
//  * Wavelet analysis of Sections 3.2-3.3 (tko_wavelet_components, stateless): the signal is
//    s[n] = a[n] * v[n] (one row per position, d columns); every column is decomposed along the
//    sequence by L levels of the Haar filter pair (filtering, then down-sampling by two), and
//    Rec(D_l) is rebuilt from the level-l detail coefficients alone by l single-level
//    reconstructions, the first with a zero approximation, the others with zero details.
//    Positions and coefficients are counted from 1 as in the printed reconstruction formula, so
//    coefficient n belongs to the signal pair (2n-1, 2n).  "Magnitude" is |Rec(D_l)[n]| averaged
//    over the d columns (the paper averages over layers, heads and samples; the columns
//    are averaged too, the figure showing one curve per level).  The sequence length must be a
//    multiple of 2^L (the paper's 512 with L = 5 is; it says nothing about other lengths).
//
// Near-tie handling for parity runs: every decision reports its relative
// margin |Sbar_l - Sbar_r| / max(Sbar_l, Sbar_r).  A caller may pass the
// position another implementation evicted; the oracle adopts it only when
// that position is the other member of the scope AND the margin is below the
// caller's threshold; otherwise it keeps its own choice and reports the
// disagreement.
//
// parity unpinned: model quality (perplexity, task scores) of the heuristic;
// it needs datasets and weights that are not available.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum : int { TKO_KEEP_LEFT = 1, TKO_IDX_LITERAL = 2, TKO_SCORE_ACCUMULATED = 4, TKO_POSITION_RERANK = 8 };

struct Stream {
  int c = 0, n_sink = 0, n_recent = 0, m = 0, G = 1, d = 0, flags = 0;
  double scale = 1.0;
  double rope_base = 10000.0;
  long long t = 0;  // tokens processed so far == position of the next token
  int idx = 1;      // the paper's 1-based idx (Algorithm 1, initialisation)
  std::vector<std::vector<double>> K, V;  // one row per cached token
  std::vector<double> S;                  // accumulated attention weight
  std::vector<long long> C;               // number of queries that attended the token
  std::vector<long long> pos;             // original 0-based stream position
};

struct Decision {
  long long evicted_pos = -1;
  double margin = -1.0;     // -1: no eviction at this step
  int adopted = 0;          // 1: took the caller's choice at a near-tie
  int disagreed = 0;        // 1: caller's choice differed and was NOT adopted
};

void softmax_row(const std::vector<double>& logits, size_t n, std::vector<double>& a) {
  double mx = -INFINITY;
  for (size_t j = 0; j < n; ++j) mx = logits[j] > mx ? logits[j] : mx;
  double sum = 0.0;
  for (size_t j = 0; j < n; ++j) { a[j] = std::exp(logits[j] - mx); sum += a[j]; }
  for (size_t j = 0; j < n; ++j) a[j] /= sum;
}

// Rotary position encoding of one row x [d] at position p: every plane (2i, 2i+1) is turned by
// the angle p * base^(-2i/d).
std::vector<double> rotary(const double* x, int d, long long p, double base) {
  std::vector<double> y(x, x + d);
  for (int i = 0; 2 * i + 1 < d; ++i) {
    const double angle = (double)p * std::pow(base, -2.0 * (double)i / (double)d);
    const double co = std::cos(angle), si = std::sin(angle);
    y[2 * i] = x[2 * i] * co - x[2 * i + 1] * si;
    y[2 * i + 1] = x[2 * i] * si + x[2 * i + 1] * co;
  }
  return y;
}

// Single-level decomposition (Section 3.2): A[n] = sum_k s[k] g[2n-k], D[n] = sum_k s[k] h[2n-k], indices from 1,
// with the Haar pair g = (r, r), h = (-r, r) on taps 0 and 1, r = sqrt(2)/2.
void haar_decompose(const std::vector<double>& s, std::vector<double>& A, std::vector<double>& D) {
  const double r = std::sqrt(2.0) / 2.0;
  const double g[2] = {r, r}, h[2] = {-r, r};
  const size_t half = s.size() / 2;
  A.assign(half, 0.0);
  D.assign(half, 0.0);
  for (size_t n = 1; n <= half; ++n)
    for (size_t k = 1; k <= s.size(); ++k) {
      const long long tap = 2 * (long long)n - (long long)k;
      if (tap == 0 || tap == 1) { A[n - 1] += s[k - 1] * g[tap]; D[n - 1] += s[k - 1] * h[tap]; }
    }
}

// Single-level reconstruction R(A, D)[n], n from 1: odd n takes (A + D) of coefficient (n+1)/2, even n (A - D) of n/2.
std::vector<double> haar_reconstruct(const std::vector<double>& A, const std::vector<double>& D) {
  const double r = std::sqrt(2.0) / 2.0;
  std::vector<double> out(2 * A.size());
  for (size_t n = 1; n <= out.size(); ++n)
    out[n - 1] = (n % 2 == 1) ? r * (A[(n + 1) / 2 - 1] + D[(n + 1) / 2 - 1]) : r * (A[n / 2 - 1] - D[n / 2 - 1]);
  return out;
}

// The eviction block of Algorithm 1 on a list of token handles `order` whose scores are sbar[handle].
// Returns the index (into `order`) that is to be erased, or -1 when length <= c.
int choose_eviction(Stream& s, const std::vector<int>& order, const std::vector<double>& sbar,
                    const std::vector<long long>& pos_of, long long forced_pos, double follow_thresh,
                    Decision& dec) {
  if ((long long)order.size() <= (long long)s.c) return -1;
  const int l = s.n_sink + (s.idx - 1);  // 0-based logical slot of the paper's idx
  const int r = l + 1;
  const double sl = sbar[order[l]], sr = sbar[order[r]];
  int victim;
  if (s.flags & TKO_KEEP_LEFT) victim = r;
  else victim = (sl > sr) ? r : l;
  const double big = sl > sr ? sl : sr;
  dec.margin = big > 0.0 ? std::fabs(sl - sr) / big : 0.0;
  if (forced_pos >= 0 && forced_pos != pos_of[order[victim]]) {
    const int other = victim == l ? r : l;
    if (forced_pos == pos_of[order[other]] && dec.margin < follow_thresh && !(s.flags & TKO_KEEP_LEFT)) {
      victim = other;
      dec.adopted = 1;
    } else {
      dec.disagreed = 1;
    }
  }
  dec.evicted_pos = pos_of[order[victim]];
  if (s.flags & TKO_IDX_LITERAL) s.idx = (s.idx + 1) % s.m + 1;
  else s.idx = s.idx % s.m + 1;
  return victim;
}

}  // namespace

extern "C" {

void* tko_new(int budget, int n_sink, int n_recent, int G, int d, double scale, int flags) {
  if (budget < 1 || n_sink < 0 || n_recent < 0 || G < 1 || d < 1) return nullptr;
  if (budget - n_sink - n_recent < 1) return nullptr;
  Stream* s = new Stream;
  s->c = budget; s->n_sink = n_sink; s->n_recent = n_recent; s->m = budget - n_sink - n_recent;
  s->G = G; s->d = d; s->scale = scale; s->flags = flags;
  return s;
}

void tko_free(void* h) { delete static_cast<Stream*>(h); }

// An independent copy of a stream's whole state (for callers that may want to take a call back).
void* tko_clone(void* h) { return new Stream(*static_cast<Stream*>(h)); }

void tko_set_rope_base(void* h, double base) { static_cast<Stream*>(h)->rope_base = base; }

int tko_len(void* h) { return (int)static_cast<Stream*>(h)->pos.size(); }
long long tko_t(void* h) { return static_cast<Stream*>(h)->t; }
int tko_idx(void* h) { return static_cast<Stream*>(h)->idx; }

// Copies the per-token state in cache order; any pointer may be null.
void tko_state(void* h, long long* pos, double* S, long long* C) {
  Stream& s = *static_cast<Stream*>(h);
  for (size_t j = 0; j < s.pos.size(); ++j) {
    if (pos) pos[j] = s.pos[j];
    if (S) S[j] = s.S[j];
    if (C) C[j] = s.C[j];
  }
}

// Copies the cached K and V rows (cache order), [len][d] each.
void tko_kv(void* h, double* K, double* V) {
  Stream& s = *static_cast<Stream*>(h);
  for (size_t j = 0; j < s.K.size(); ++j)
    for (int e = 0; e < s.d; ++e) { K[j * s.d + e] = s.K[j][e]; V[j * s.d + e] = s.V[j][e]; }
}

// One decode step (one iteration of Algorithm 1's loop without the projections).
//   q [G][d], k [d], v [d]  ->  out [G][d]
//   forced_pos: -1, or the position another implementation evicted at this step.
//   result[0] = evicted position or -1, result[1] = adopted, result[2] = disagreed.
//   commit == 0: report what the step would do (out, margin, result) and leave the
//   state untouched.
void tko_decode_step(void* h, const double* q, const double* k, const double* v, double* out,
                     long long forced_pos, double follow_thresh, int commit,
                     long long* result, double* margin) {
  Stream& s = *static_cast<Stream*>(h);
  const Stream backup = commit ? Stream() : s;
  // the append step, and the "u {0}" of the C and S updates
  s.K.emplace_back(k, k + s.d);
  s.V.emplace_back(v, v + s.d);
  s.S.push_back(0.0);
  s.C.push_back(0);
  s.pos.push_back(s.t);
  const size_t n = s.K.size();
  // the attention step and o = a V, once per query head of the group
  // with position re-assignment: the token at cache index j is at position j, the query at n - 1
  const bool rerank = (s.flags & TKO_POSITION_RERANK) != 0;
  std::vector<std::vector<double>> Kpos;
  if (rerank)
    for (size_t j = 0; j < n; ++j) Kpos.push_back(rotary(s.K[j].data(), s.d, (long long)j, s.rope_base));
  const std::vector<std::vector<double>>& Katt = rerank ? Kpos : s.K;
  std::vector<double> logits(n), a(n), asum(n, 0.0);
  for (int g = 0; g < s.G; ++g) {
    std::vector<double> qg(q + g * s.d, q + (g + 1) * s.d);
    if (rerank) qg = rotary(qg.data(), s.d, (long long)n - 1, s.rope_base);
    for (size_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int e = 0; e < s.d; ++e) acc += qg[e] * Katt[j][e];
      logits[j] = acc * s.scale;
    }
    softmax_row(logits, n, a);
    for (int e = 0; e < s.d; ++e) {
      double acc = 0.0;
      for (size_t j = 0; j < n; ++j) acc += a[j] * s.V[j][e];
      out[g * s.d + e] = acc;
    }
    for (size_t j = 0; j < n; ++j) asum[j] += a[j];
  }
  // C and S updates
  for (size_t j = 0; j < n; ++j) { s.C[j] += 1; s.S[j] += asum[j]; }
  // the eviction block
  Decision dec;
  std::vector<int> order(n);
  std::vector<double> sbar(n);
  const bool accumulated = (s.flags & TKO_SCORE_ACCUMULATED) != 0;
  for (size_t j = 0; j < n; ++j) { order[j] = (int)j; sbar[j] = accumulated ? s.S[j] : s.S[j] / (double)s.C[j]; }
  const int victim = choose_eviction(s, order, sbar, s.pos, forced_pos, follow_thresh, dec);
  if (victim >= 0) {
    s.K.erase(s.K.begin() + victim);
    s.V.erase(s.V.begin() + victim);
    s.S.erase(s.S.begin() + victim);
    s.C.erase(s.C.begin() + victim);
    s.pos.erase(s.pos.begin() + victim);
  }
  s.t += 1;
  if (result) { result[0] = dec.evicted_pos; result[1] = dec.adopted; result[2] = dec.disagreed; }
  if (margin) *margin = dec.margin;
  if (!commit) s = backup;
}

// T decode steps in a row: the loop of Algorithm 1 over a whole stream.
//   q [T][G][d], k [T][d], v [T][d]; out [T][G][d] or null; forced [T] or null;
//   evicted [T], margins [T] or null; counts[0] += adopted, counts[1] += disagreed.
void tko_decode_stream(void* h, const double* q, const double* k, const double* v, int T, double* out,
                       const long long* forced, double follow_thresh, long long* evicted, double* margins,
                       long long* counts) {
  Stream& s = *static_cast<Stream*>(h);
  std::vector<double> o((size_t)s.G * s.d);
  for (int i = 0; i < T; ++i) {
    long long res[3];
    double mg;
    tko_decode_step(h, q + (size_t)i * s.G * s.d, k + (size_t)i * s.d, v + (size_t)i * s.d,
                    out ? out + (size_t)i * s.G * s.d : o.data(), forced ? forced[i] : -1, follow_thresh, 1,
                    res, &mg);
    if (evicted) evicted[i] = res[0];
    if (margins) margins[i] = mg;
    if (counts) { counts[0] += res[1]; counts[1] += res[2]; }
  }
}

// One prefill chunk of L tokens (see the header for the definition).
//   Q [L][G][d], K [L][d], V [L][d]  ->  out [L][G][d]
//   forced_pos: null, or [L] positions another implementation evicted at each of the
//   chunk's tokens (-1 where it evicted nothing).
//   evicted [L], margins [L], adopted [L], disagreed [L]: per-token decision records
//   (any may be null).
// With position re-assignment the chunk is scored before anything of it is evicted, so the positions are the
// ranks at that moment: the n0 cached tokens are at 0 .. n0-1, chunk token i (and its query) at n0 + i.
// Returns 0.
int tko_prefill_chunk(void* h, const double* Q, const double* K, const double* V, int L, double* out,
                       const long long* forced_pos, double follow_thresh,
                       long long* evicted, double* margins, int* adopted, int* disagreed) {
  Stream& s = *static_cast<Stream*>(h);
  const size_t n0 = s.K.size();
  for (int i = 0; i < L; ++i) {
    s.K.emplace_back(K + (size_t)i * s.d, K + (size_t)(i + 1) * s.d);
    s.V.emplace_back(V + (size_t)i * s.d, V + (size_t)(i + 1) * s.d);
    s.S.push_back(0.0);
    s.C.push_back(0);
    s.pos.push_back(s.t + i);
  }
  const size_t n = s.K.size();
  const bool rerank = (s.flags & TKO_POSITION_RERANK) != 0;
  std::vector<std::vector<double>> Kpos;
  if (rerank)
    for (size_t j = 0; j < n; ++j) Kpos.push_back(rotary(s.K[j].data(), s.d, (long long)j, s.rope_base));
  const std::vector<std::vector<double>>& Katt = rerank ? Kpos : s.K;
  std::vector<double> logits(n), a(n), asum(n);
  for (int i = 0; i < L; ++i) {
    const size_t vis = n0 + (size_t)i + 1;  // the cache before the chunk, plus chunk tokens <= i
    for (size_t j = 0; j < vis; ++j) asum[j] = 0.0;
    for (int g = 0; g < s.G; ++g) {
      std::vector<double> qv(Q + ((size_t)i * s.G + g) * s.d, Q + ((size_t)i * s.G + g + 1) * s.d);
      if (rerank) qv = rotary(qv.data(), s.d, (long long)(n0 + (size_t)i), s.rope_base);
      const double* q = qv.data();
      for (size_t j = 0; j < vis; ++j) {
        double acc = 0.0;
        for (int e = 0; e < s.d; ++e) acc += q[e] * Katt[j][e];
        logits[j] = acc * s.scale;
      }
      softmax_row(logits, vis, a);
      double* o = out + ((size_t)i * s.G + g) * s.d;
      for (int e = 0; e < s.d; ++e) {
        double acc = 0.0;
        for (size_t j = 0; j < vis; ++j) acc += a[j] * s.V[j][e];
        o[e] = acc;
      }
      for (size_t j = 0; j < vis; ++j) asum[j] += a[j];
    }
    for (size_t j = 0; j < vis; ++j) { s.C[j] += 1; s.S[j] += asum[j]; }
  }
  // frozen scores, then the replay of the append step and the eviction block token by token
  const bool accumulated = (s.flags & TKO_SCORE_ACCUMULATED) != 0;
  std::vector<double> sbar(n);
  for (size_t j = 0; j < n; ++j) sbar[j] = accumulated ? s.S[j] : s.S[j] / (double)s.C[j];
  std::vector<int> order;
  order.reserve(n);
  for (size_t j = 0; j < n0; ++j) order.push_back((int)j);
  for (int i = 0; i < L; ++i) {
    order.push_back((int)(n0 + i));
    Decision dec;
    const int victim = choose_eviction(s, order, sbar, s.pos, forced_pos ? forced_pos[i] : -1,
                                       follow_thresh, dec);
    if (victim >= 0) order.erase(order.begin() + victim);
    if (evicted) evicted[i] = dec.evicted_pos;
    if (margins) margins[i] = dec.margin;
    if (adopted) adopted[i] = dec.adopted;
    if (disagreed) disagreed[i] = dec.disagreed;
  }
  // keep the survivors, in order
  std::vector<std::vector<double>> K2, V2;
  std::vector<double> S2;
  std::vector<long long> C2, P2;
  for (int hnd : order) {
    K2.push_back(s.K[hnd]); V2.push_back(s.V[hnd]);
    S2.push_back(s.S[hnd]); C2.push_back(s.C[hnd]); P2.push_back(s.pos[hnd]);
  }
  s.K.swap(K2); s.V.swap(V2); s.S.swap(S2); s.C.swap(C2); s.pos.swap(P2);
  s.t += L;
  return 0;
}

// One-shot block-level compression of a whole prompt (Section 4.2).  The stream must be empty.
//   Qw [b][G][d]: queries of the prompt's last b tokens; K, V [T][d]: the whole prompt.
//   forced_block: null, or [T/b] the block another implementation evicted when block i was
//   appended (-1 where it evicted none); adopted only at near-ties, as in tko_decode_step.
//   evicted_block, margins [T/b]; counts[0] += adopted, counts[1] += disagreed;
//   token_sbar [T], block_score [T/b] (any may be null).
// Returns 0, or -1 if the arguments do not fit (non-empty stream, T or c not a multiple of b,
// no tree block left).
int tko_prefill_prompt(void* h, const double* Qw, const double* K, const double* V, int T, int b,
                       const long long* forced_block, double follow_thresh, long long* evicted_block,
                       double* margins, long long* counts, double* token_sbar, double* block_score) {
  Stream& s = *static_cast<Stream*>(h);
  if (!s.pos.empty() || s.t != 0 || b < 1 || T < b || T % b != 0 || s.c % b != 0) return -1;
  const int N = T / b, W = b;
  Stream blk;                                     // Algorithm 1's scalars, counted in blocks
  blk.c = s.c / b;
  blk.n_sink = (s.n_sink + b - 1) / b;
  blk.n_recent = (s.n_recent + b - 1) / b;
  blk.m = blk.c - blk.n_sink - blk.n_recent;
  blk.flags = s.flags;
  if (blk.m < 1) return -1;
  // the observation window queries the entire sequence (causally); attention, C and S updates for those queries only
  std::vector<double> Ssum((size_t)T, 0.0), logits((size_t)T), a((size_t)T);
  std::vector<long long> Cnt((size_t)T, 0);
  // with position re-assignment the keys carry no positional encoding: key j is at position j here
  const bool rerank = (s.flags & TKO_POSITION_RERANK) != 0;
  std::vector<double> Kpos;
  if (rerank) {
    Kpos.resize((size_t)T * s.d);
    for (int j = 0; j < T; ++j) {
      const std::vector<double> kr = rotary(K + (size_t)j * s.d, s.d, j, s.rope_base);
      for (int e = 0; e < s.d; ++e) Kpos[(size_t)j * s.d + e] = kr[e];
    }
  }
  const double* Katt = rerank ? Kpos.data() : K;
  for (int i = 0; i < W; ++i) {
    const size_t vis = (size_t)(T - W + i) + 1;
    for (int g = 0; g < s.G; ++g) {
      std::vector<double> qv(Qw + ((size_t)i * s.G + g) * s.d, Qw + ((size_t)i * s.G + g + 1) * s.d);
      if (rerank) qv = rotary(qv.data(), s.d, (long long)(T - W + i), s.rope_base);
      const double* q = qv.data();
      for (size_t j = 0; j < vis; ++j) {
        double acc = 0.0;
        for (int e = 0; e < s.d; ++e) acc += q[e] * Katt[j * s.d + e];
        logits[j] = acc * s.scale;
      }
      softmax_row(logits, vis, a);
      for (size_t j = 0; j < vis; ++j) Ssum[j] += a[j];
    }
    for (size_t j = 0; j < vis; ++j) Cnt[j] += 1;
  }
  // the average S / C per token, then the block's score: the average over its b tokens
  std::vector<double> sbar((size_t)T), beta((size_t)N);
  const bool accumulated = (s.flags & TKO_SCORE_ACCUMULATED) != 0;
  for (int j = 0; j < T; ++j) sbar[j] = accumulated ? Ssum[j] : Ssum[j] / (double)Cnt[j];
  for (int k = 0; k < N; ++k) {
    double acc = 0.0;
    for (int x = 0; x < b; ++x) acc += sbar[(size_t)k * b + x];
    beta[k] = acc / (double)b;
  }
  if (token_sbar) for (int j = 0; j < T; ++j) token_sbar[j] = sbar[j];
  if (block_score) for (int k = 0; k < N; ++k) block_score[k] = beta[k];
  // Algorithm 1's append step and eviction block, one block at a time
  std::vector<long long> block_id((size_t)N);
  for (int k = 0; k < N; ++k) block_id[k] = k;
  std::vector<int> order;
  for (int k = 0; k < N; ++k) {
    order.push_back(k);
    Decision dec;
    const int victim = choose_eviction(blk, order, beta, block_id, forced_block ? forced_block[k] : -1,
                                       follow_thresh, dec);
    if (victim >= 0) order.erase(order.begin() + victim);
    if (evicted_block) evicted_block[k] = dec.evicted_pos;
    if (margins) margins[k] = dec.margin;
    if (counts) { counts[0] += dec.adopted; counts[1] += dec.disagreed; }
  }
  // the kept blocks' tokens are the cache that decoding starts from
  for (int kb : order) {
    for (int x = 0; x < b; ++x) {
      const long long j = (long long)kb * b + x;
      s.K.emplace_back(K + (size_t)j * s.d, K + (size_t)(j + 1) * s.d);
      s.V.emplace_back(V + (size_t)j * s.d, V + (size_t)(j + 1) * s.d);
      s.C.push_back((long long)T - j);
      s.S.push_back(accumulated ? sbar[(size_t)j] : sbar[(size_t)j] * (double)((long long)T - j));
      s.pos.push_back(j);
    }
  }
  s.t = T;
  s.idx = 1;
  return 0;
}

// Wavelet analysis of Sections 3.2-3.3 for one head at one generation step.
//   a [t]: attention weights; V [t][d]; levels L >= 1 with 2^L dividing t.
//   magnitude [L][t]: row l-1 holds |Rec(D_l)[n]| averaged over the d columns.
//   coeffs (may be null) [d][t]: per column the list [A_L, D_L, D_{L-1}, .., D_1] (lengths t/2^L, t/2^L, .., t/2).
//   rec_sum (may be null) [d][t]: per column Rec(A_L) + sum_l Rec(D_l), which must give the signal back.
// Returns 0, or -1 if the sizes do not fit.
int tko_wavelet_components(const double* a, const double* V, int t, int d, int levels, double* magnitude,
                           double* coeffs, double* rec_sum) {
  if (t < 1 || d < 1 || levels < 1 || levels > 30 || t % (1 << levels) != 0) return -1;
  for (size_t i = 0; i < (size_t)levels * t; ++i) magnitude[i] = 0.0;
  for (int e = 0; e < d; ++e) {
    std::vector<double> sig((size_t)t);
    for (int n = 0; n < t; ++n) sig[n] = a[n] * V[(size_t)n * d + e];       // s = a^T o V, column e
    std::vector<std::vector<double>> D((size_t)levels + 1);
    std::vector<double> A = sig, A_next;
    for (int l = 1; l <= levels; ++l) { haar_decompose(A, A_next, D[l]); A.swap(A_next); }
    if (coeffs) {
      double* c = coeffs + (size_t)e * t;
      size_t o = 0;
      for (double x : A) c[o++] = x;
      for (int l = levels; l >= 1; --l) for (double x : D[l]) c[o++] = x;
    }
    std::vector<double> total((size_t)t, 0.0);
    for (int l = 0; l <= levels; ++l) {       // l = 0 stands for Rec(A_L)
      const int depth = l == 0 ? levels : l;
      std::vector<double> rec;
      if (l == 0) rec = haar_reconstruct(A, std::vector<double>(A.size(), 0.0));
      else rec = haar_reconstruct(std::vector<double>(D[l].size(), 0.0), D[l]);
      for (int up = depth - 1; up >= 1; --up) rec = haar_reconstruct(rec, std::vector<double>(rec.size(), 0.0));
      for (int n = 0; n < t; ++n) {
        total[n] += rec[n];
        if (l >= 1) magnitude[(size_t)(l - 1) * t + n] += std::fabs(rec[n]) / (double)d;
      }
    }
    if (rec_sum) for (int n = 0; n < t; ++n) rec_sum[(size_t)e * t + n] = total[n];
  }
  return 0;
}

}  // extern "C"
