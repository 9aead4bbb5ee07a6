// Runs every entry point of the CPU oracle on small seeded inputs under AddressSanitizer / UBSan: decode streams
// with evictions (all flags, follow mode, dry runs), prefill chunks, one-shot prompt compression followed by decode
// steps, re-assigned positions, the wavelet analysis.  Only memory safety and defined behaviour are checked here;
// the values are checked by the pins.  Test infrastructure.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
void* tko_new(int budget, int n_sink, int n_recent, int G, int d, double scale, int flags);
void tko_free(void* h);
void tko_set_rope_base(void* h, double base);
int tko_len(void* h);
long long tko_t(void* h);
int tko_idx(void* h);
void tko_state(void* h, long long* pos, double* S, long long* C);
void tko_kv(void* h, double* K, double* V);
void tko_decode_step(void* h, const double* q, const double* k, const double* v, double* out, long long forced_pos,
                     double follow_thresh, int commit, long long* result, double* margin);
void tko_decode_stream(void* h, const double* q, const double* k, const double* v, int T, double* out,
                       const long long* forced, double follow_thresh, long long* evicted, double* margins, long long* counts);
int tko_prefill_chunk(void* h, const double* Q, const double* K, const double* V, int L, double* out,
                      const long long* forced_pos, double follow_thresh, long long* evicted, double* margins,
                      int* adopted, int* disagreed);
int tko_prefill_prompt(void* h, const double* Qw, const double* K, const double* V, int T, int b,
                       const long long* forced_block, double follow_thresh, long long* evicted_block, double* margins,
                       long long* counts, double* token_sbar, double* block_score);
int tko_wavelet_components(const double* a, const double* V, int t, int d, int levels, double* magnitude, double* coeffs,
                           double* rec_sum);
}

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: CHECK failed: %s\n", __FILE__, __LINE__, #cond); exit(1); } } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd() {                       // uniform in (-1, 1), xorshift
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / (double)(1ull << 52) - 1.0;
}
static std::vector<double> fill(size_t n) { std::vector<double> x(n); for (double& e : x) e = 2.0 * rnd(); return x; }

int main() {
  const int layouts[][3] = {{1, 0, 0}, {2, 0, 0}, {5, 0, 0}, {9, 2, 3}, {16, 4, 4}, {6, 0, 5}, {6, 5, 0}};
  for (const auto& lay : layouts) for (int G : {1, 3}) for (int flags : {0, 1, 2, 4, 8, 5, 12}) {
    const int c = lay[0], d = 6, T = 5 * c + 7;
    void* s = tko_new(c, lay[1], lay[2], G, d, 0.4, flags);
    CHECK(s);
    tko_set_rope_base(s, 100.0);
    const auto q = fill((size_t)T * G * d), k = fill((size_t)T * d), v = fill((size_t)T * d);
    std::vector<double> out((size_t)T * G * d), mg(T);
    std::vector<long long> ev(T), forced(T, -1);
    long long counts[2] = {0, 0};
    tko_decode_stream(s, q.data(), k.data(), v.data(), T, out.data(), nullptr, 0.0, ev.data(), mg.data(), counts);
    CHECK(tko_len(s) == (T < c ? T : c) && tko_t(s) == T && tko_idx(s) >= 1);
    std::vector<long long> pos(c), C(c);
    std::vector<double> S(c), K((size_t)c * d), V((size_t)c * d);
    tko_state(s, pos.data(), S.data(), C.data());
    tko_kv(s, K.data(), V.data());
    tko_free(s);
    // the same stream again, following itself and a wrong choice now and then, with dry runs in between
    s = tko_new(c, lay[1], lay[2], G, d, 0.4, flags);
    tko_set_rope_base(s, 100.0);
    for (int t = 0; t < T; ++t) {
      long long res[3]; double m;
      tko_decode_step(s, &q[(size_t)t * G * d], &k[(size_t)t * d], &v[(size_t)t * d], out.data(), t % 3 ? ev[t] : t / 2, 0.5, 0, res, &m);
      tko_decode_step(s, &q[(size_t)t * G * d], &k[(size_t)t * d], &v[(size_t)t * d], out.data(), ev[t], 1e-4, 1, res, &m);
      CHECK(res[0] == ev[t]);
    }
    tko_free(s);
    // chunks and single steps mixed
    s = tko_new(c, lay[1], lay[2], G, d, 0.4, flags);
    int t = 0;
    for (int L : {3, 1, 2 * c + 1, 7, 1, c}) {
      if (t + L > T) break;
      std::vector<long long> e(L); std::vector<double> m(L); std::vector<int> ad(L), di(L);
      const int rc = tko_prefill_chunk(s, &q[(size_t)t * G * d], &k[(size_t)t * d], &v[(size_t)t * d], L, out.data(), nullptr, 0.0,
                                       e.data(), m.data(), ad.data(), di.data());
      CHECK(rc == 0);
      t += L;
    }
    tko_free(s);
  }
  // one-shot prompt compression, then decoding
  for (int flags : {0, 1, 4, 8}) for (int b : {1, 4}) {
    const int c = 16, G = 2, d = 4, T = 12 * b * 3, steps = 9;
    void* s = tko_new(c, 3, 5, G, d, 0.5, flags);
    const auto qw = fill((size_t)b * G * d), K = fill((size_t)T * d), V = fill((size_t)T * d);
    std::vector<long long> evb(T / b); std::vector<double> mg(T / b), tok(T), blk(T / b);
    long long counts[2] = {0, 0};
    CHECK(tko_prefill_prompt(s, qw.data(), K.data(), V.data(), T, b, nullptr, 0.0, evb.data(), mg.data(), counts, tok.data(), blk.data()) == 0);
    CHECK(tko_prefill_prompt(s, qw.data(), K.data(), V.data(), T, b, nullptr, 0.0, nullptr, nullptr, nullptr, nullptr, nullptr) == -1);
    for (int i = 0; i < steps; ++i) {
      const auto q = fill((size_t)G * d), k = fill(d), v = fill(d);
      std::vector<double> o((size_t)G * d); long long res[3]; double m;
      tko_decode_step(s, q.data(), k.data(), v.data(), o.data(), -1, 0.0, 1, res, &m);
    }
    CHECK(tko_len(s) == c);
    tko_free(s);
  }
  // wavelet analysis
  for (int levels : {1, 3, 5}) {
    const int t = 64, d = 5;
    const auto a = fill(t), V = fill((size_t)t * d);
    std::vector<double> mag((size_t)levels * t), co((size_t)d * t), rs((size_t)d * t);
    CHECK(tko_wavelet_components(a.data(), V.data(), t, d, levels, mag.data(), co.data(), rs.data()) == 0);
    CHECK(tko_wavelet_components(a.data(), V.data(), t, d, levels, mag.data(), nullptr, nullptr) == 0);
    CHECK(tko_wavelet_components(a.data(), V.data(), t - 1, d, levels, mag.data(), nullptr, nullptr) == -1);
  }
  CHECK(tko_new(4, 3, 1, 1, 4, 1.0, 0) == nullptr);
  puts("oracle clean");
  return 0;
}
