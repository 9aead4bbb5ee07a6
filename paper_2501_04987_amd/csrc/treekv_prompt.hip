// TreeKV one-shot prompt compression on gfx950 (Section 4.2, "Prefilling Stage").
//
// The prompt is cut into blocks of b tokens.  The queries of the last block (the observation window)
// attend the whole prompt causally; a token's importance is its attention weight averaged over the
// window queries that see it (Algorithm 1's S / C restricted to those queries, summed over the query
// heads of the group); a block's importance is the mean over its b tokens; Algorithm 1 (append,
// then its eviction block) then runs with blocks in the place of tokens and the block scores frozen.  The kept blocks'
// rows become the cache and decoding takes over from there.
//
// Four launches:
//   stats    grid (splits, units): every workgroup streams its slice of the prompt's keys once and
//            leaves, per window query, the (max, sum) of the scaled logits it saw.
//   scores   same grid: merges the slices' (max, sum), streams the same keys again, turns logits into
//            probabilities and adds them up per key over the window queries: the token scores.
//   blocks   grid (units): block means, then Algorithm 1 over blocks.  With frozen scores the scopes of
//            one pass of idx over the tree region are disjoint pairs of the sequence at the pass's
//            start followed by the blocks that enter during the pass, so a pass is one parallel step.
//   handoff  grid (row groups, units): copies the kept rows into slots 0.., and writes the scores, the
//            order arrays, the bookkeeping words and the retained list that decoding starts from.
//
// Both streaming kernels are bound by the read of K (twice 2*T*d bytes per unit): the logits of b queries
// against T keys are [b x d].[d x T], a contraction with b*G <= 128 rows, done on the matrix pipe with
// the keys read straight from global memory in operand order (S^T = K Q^T, 16 keys x 32 dims per
// instruction; the window queries sit in registers as the other operand), so the vector ALU is left with
// one exponential per logit.
//
// With positions re-assigned (TREEKV_POSITION_RERANK) the keys and queries come without positional encoding and
// nothing has been evicted yet, so key j is at position j and window query i at T - W + i.  The keys are turned
// in registers (fp32, angles from the table) right after they arrive and split into two bf16 parts, hi + lo; the
// window's queries are turned and split once per call by a small kernel and sit in LDS; a logit is then
// k_hi.q_hi + k_lo.q_hi + k_hi.q_lo (the missing lo.lo term is 2^-18 of the product).  Same four launches after that.

#include "treekv_internal.h"

namespace tkv {

namespace {

constexpr int PP_THREADS = 512;
constexpr int PP_WAVES = PP_THREADS / 64;
constexpr int PP_TILE = 32;                      // keys per wave iteration (two operand blocks of 16)
constexpr int PP_STEP = PP_WAVES * PP_TILE;
constexpr float NEG_BIG = -1.0e30f;

template <bool B> struct BoolTag { static constexpr bool value = B; };

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ inline f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ inline unsigned pack_bf16(float a, float b) {       // (a in the low half), round to nearest even
  f32x2_t v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
// One plane (two adjacent dims, packed as bf16 in `w`) turned by the angle whose (cos, sin) are given:
// the bf16 pair nearest to the result, and the bf16 pair nearest to what that rounding lost.
__device__ inline void turn_pair(unsigned w, float c, float s, unsigned& hi, unsigned& lo) {
  const float x0 = __uint_as_float(w << 16), x1 = __uint_as_float(w & 0xffff0000u);
  const float r0 = fmaf(x0, c, -(x1 * s)), r1 = fmaf(x0, s, x1 * c);
  hi = pack_bf16(r0, r1);
  lo = pack_bf16(r0 - __uint_as_float(hi << 16), r1 - __uint_as_float(hi & 0xffff0000u));
}
__device__ inline int q_swz(int D, int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }

template <int CTRL>
__device__ inline float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
  return v + __int_as_float(moved);
}
// Sum over the 16 lanes of a DPP row; every lane gets the total.
__device__ inline float row16_sum(float v) {
  v = dpp_add<0x128>(v);
  v = dpp_add<0x124>(v);
  v = dpp_add<0x122>(v);
  v = dpp_add<0x121>(v);
  return v;
}

// What the two streaming kernels share: the window queries as MFMA operands, the slice of keys a
// workgroup owns, and the loop that turns 32 keys into NB x 2 accumulators of scaled logits.
//   query row qr = i * G + g (window query i, head g of the group), padded with rows that see nothing to NB * 16;
//   row qr sees the keys below T - W + i + 1.
template <int D, int NB, bool ROPE>
struct PromptStream {
  static constexpr int KS = D / 32;
  static constexpr int Q_LDS_BYTES = ROPE ? 2 * NB * 16 * D * 2 : 0;
  // one operand block of keys in flight: 16 keys x this lane's 8 dims of every k-step, and (ROPE) the (cos, sin)
  // pairs of those dims at the keys' positions
  struct KB { uint4 k[KS]; uint4 t[ROPE ? 2 * KS : 1]; };
  uint4 qa[ROPE ? 1 : NB][KS];
  const uint16_t* sq;          // ROPE: LDS [hi, lo][NB * 16 rows][D], 16-byte pieces swizzled by row
  const float2* tab;           // ROPE: (cos, sin) of position * theta_i
  int lim[NB];                 // first key this lane's query of block nb does not see, capped at the slice's end
  const uint16_t* Ku;          // key 0 of the unit
  size_t row_stride;           // elements between consecutive keys of the unit
  int begin, end, T;
  int lane, wave, lr, q4;

  __device__ inline void init(const Params& p, const uint16_t* Qw, const uint16_t* K, int T_, int W, int unit,
                              int split, int rows_per_split, uint16_t* sm_q) {
    const int tid = threadIdx.x;
    sq = sm_q;
    tab = p.rope_tab;
    lane = tid & 63; wave = tid >> 6; lr = lane & 15; q4 = lane >> 4;
    T = T_;
    const int kvh = unit % p.Hkv, b = unit / p.Hkv;
    Ku = K + ((size_t)b * T * p.Hkv + kvh) * D;
    row_stride = (size_t)p.Hkv * D;
    begin = split * rows_per_split;
    end = min(T, begin + rows_per_split);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int qr = nb * 16 + lr;
      const bool live = qr < W * p.G;
      const int i = qr / p.G, g = qr % p.G;
      lim[nb] = live ? min(end, T - W + i + 1) : 0;
      // (a padding row repeats the window's last query: it sees no key, lim = 0, so what it holds does not matter,
      // and a load on every path lets the key requests go out without waiting for these)
      const int iq = live ? i : W - 1, gq = live ? g : 0;
      if constexpr (!ROPE) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          qa[nb][ks] = *reinterpret_cast<const uint4*>(Qw + (((size_t)b * W + iq) * p.H + (size_t)kvh * p.G + gq) * D + ks * 32 + q4 * 8);
      }
    }
    if constexpr (ROPE) {
      // the turned queries of this unit (hi rows, then lo rows) -> LDS; the caller's barrier publishes them
      constexpr int PIECES = D / 8;
      const uint4* src = reinterpret_cast<const uint4*>(p.pp_qrot + (size_t)unit * 2 * 128 * D);
      for (int x = tid; x < 2 * NB * 16 * PIECES; x += PP_THREADS) {
        const int piece = x % PIECES, row = (x / PIECES) % (NB * 16), half = x / (PIECES * NB * 16);
        *reinterpret_cast<uint4*>(sm_q + ((size_t)(half * NB * 16 + row) * D + ((piece ^ q_swz(D, row)) * 8))) =
            src[((size_t)half * 128 + row) * PIECES + piece];
      }
    }
  }
  // One operand block: keys base + lr (clamped into the prompt), this lane's 8 dims of every k-step.
  // The callers request blocks past their slice rather than branch around the request: with every load on
  // every path the compiler's count of outstanding loads is exact and a wait covers the block it needs only.
  __device__ inline void load_block(KB& kb, int base) const {
    const int row = max(0, min(base + lr, T - 1));
    const uint16_t* r = Ku + (size_t)row * row_stride + q4 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kb.k[ks] = *reinterpret_cast<const uint4*>(r + ks * 32);
    if constexpr (ROPE) {
      const uint4* tr = reinterpret_cast<const uint4*>(tab + (size_t)row * (D / 2) + q4 * 4);   // key `row` is at position `row`
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) { kb.t[2 * ks] = tr[ks * 8]; kb.t[2 * ks + 1] = tr[ks * 8 + 1]; }
    }
  }
  // scaled-logit accumulators of one operand block: acc[nb][i] = <key base + q4*4 + i, query nb*16 + lr>
  // (STEPWISE, ROPE only: the scheduler may not fetch a later k-step's query operands before the current one
  // is done - for the kernel that would otherwise run out of registers)
  template <bool STEPWISE = false>
  __device__ inline void logits(const KB& kb, f32x4_t (&acc)[NB]) const {
    if constexpr (!ROPE) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc[nb] = mfma16(kb.k[ks], qa[nb][ks], acc[nb]);
      }
    } else {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      // one k-step at a time: its 8 dims are turned and split, used against every query block, and forgotten
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 t0 = kb.t[2 * ks], t1 = kb.t[2 * ks + 1];
        uint4 kh, kl;
        turn_pair(kb.k[ks].x, __uint_as_float(t0.x), __uint_as_float(t0.y), kh.x, kl.x);
        turn_pair(kb.k[ks].y, __uint_as_float(t0.z), __uint_as_float(t0.w), kh.y, kl.y);
        turn_pair(kb.k[ks].z, __uint_as_float(t1.x), __uint_as_float(t1.y), kh.z, kl.z);
        turn_pair(kb.k[ks].w, __uint_as_float(t1.z), __uint_as_float(t1.w), kh.w, kl.w);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int row = nb * 16 + lr;
          const int off = ((ks * 4 + q4) ^ q_swz(D, row)) * 8;
          const uint4 bh = *reinterpret_cast<const uint4*>(sq + (size_t)row * D + off);
          const uint4 bl = *reinterpret_cast<const uint4*>(sq + (size_t)(NB * 16 + row) * D + off);
          acc[nb] = mfma16(kh, bh, acc[nb]);
          acc[nb] = mfma16(kl, bh, acc[nb]);
          acc[nb] = mfma16(kh, bl, acc[nb]);
        }
        if constexpr (STEPWISE) __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
};

// The window's queries turned to their positions (query i of the window at T - W + i) and split into bf16 hi and
// lo parts: pp_qrot [unit][hi, lo][128 rows][D], row i * G + g, rows past W * G zero.
template <int D>
__global__ void prompt_turn_queries_kernel(Params p, const uint16_t* __restrict__ Qw, int T, int W) {
  const int unit = blockIdx.y, kvh = unit % p.Hkv, b = unit / p.Hkv;
  unsigned* dst = reinterpret_cast<unsigned*>(p.pp_qrot + (size_t)unit * 2 * 128 * D);
  for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < 128 * (D / 2); x += gridDim.x * blockDim.x) {
    const int pair = x % (D / 2), row = x / (D / 2);
    unsigned hi = 0, lo = 0;
    if (row < W * p.G) {
      const int i = row / p.G, g = row % p.G;
      const unsigned w = reinterpret_cast<const unsigned*>(Qw + (((size_t)b * W + i) * p.H + (size_t)kvh * p.G + g) * D)[pair];
      const float2 cs = p.rope_tab[(size_t)(T - W + i) * (D / 2) + pair];
      turn_pair(w, cs.x, cs.y, hi, lo);
    }
    dst[(size_t)row * (D / 2) + pair] = hi;
    dst[(size_t)(128 + row) * (D / 2) + pair] = lo;
  }
}

// ---------------------------------------------------------------------------------------------
// stats: per (unit, slice, query row) the maximum and the sum of exp2(logit - maximum) over the slice
// ---------------------------------------------------------------------------------------------
template <int D, int NB, bool ROPE>
__global__ __launch_bounds__(PP_THREADS) void prompt_stats_kernel(Params p, const uint16_t* __restrict__ Qw,
                                                                  const uint16_t* __restrict__ K, int T, int W,
                                                                  int rows_per_split, int nsplit) {
  using PS = PromptStream<D, NB, ROPE>;
  using KB = typename PS::KB;
  __shared__ float sm_m[PP_WAVES][NB * 16], sm_l[PP_WAVES][NB * 16];
  extern __shared__ __attribute__((aligned(16))) uint16_t stats_q[];   // ROPE: the turned queries
  PS st;
  const int split = blockIdx.x, unit = blockIdx.y;
  st.init(p, Qw, K, T, W, unit, split, rows_per_split, stats_q);
  const float sc = p.scale_log2e;
  const int lim_all = min(st.end, T - W + 1);      // every query sees the keys below this

  float m_run[NB], l_run[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) { m_run[nb] = NEG_BIG; l_run[nb] = 0.f; }

  // two tiles of 32 keys in flight per wave: (k0, k1) and (k2, k3); a block is requested again, two tiles on,
  // as soon as its logits are out
  // (one tile with all eight operand blocks of queries: the registers do not hold more)
  // (and with the rotary angles travelling with the keys)
  constexpr int AHEAD = (NB < 8 && !ROPE) ? 2 : 1;
  KB k0, k1, k2, k3;
  int base = st.begin + st.wave * PP_TILE;
  st.load_block(k0, base); st.load_block(k1, base + 16);
  if (AHEAD == 2) { st.load_block(k2, base + PP_STEP); st.load_block(k3, base + PP_STEP + 16); }
  if constexpr (ROPE) __syncthreads();               // the queries are in LDS
  // One operand block of 16 keys at a time: its accumulators are consumed before the next block's exist.
  // `ragged` (a type, so that the common case carries no masking code): some query does not see some key.
  auto block = [&](auto ragged, KB& k, int tile, int h) {
    constexpr bool RAGGED = decltype(ragged)::value;
    f32x4_t a[NB];
    st.template logits<true>(k, a);
    if constexpr (!ROPE) st.load_block(k, tile + AHEAD * PP_STEP + h * 16);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float r[4];                                    // raw logits; the scale is positive, so max commutes with it
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        r[i] = a[nb][i];
        if (RAGGED) r[i] = (tile + h * 16 + st.q4 * 4 + i < st.lim[nb]) ? r[i] : NEG_BIG;
      }
      const float mx = fmaxf(m_run[nb], fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3])) * sc);
      float add = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float pe = fast_exp2(fmaf(r[i], sc, -mx));
        if (RAGGED) pe = r[i] > 0.5f * NEG_BIG ? pe : 0.f;
        add += pe;
      }
      l_run[nb] = fmaf(l_run[nb], fast_exp2(m_run[nb] - mx), add);
      m_run[nb] = mx;
    }
    // (with the angles in tow a block takes too many registers to be requested while its predecessor is in use)
    if constexpr (ROPE) st.load_block(k, tile + AHEAD * PP_STEP + h * 16);
  };
  auto tile = [&](KB& ka, KB& kb, int t) {
    if (t + PP_TILE > lim_all) { block(BoolTag<true>{}, ka, t, 0); block(BoolTag<true>{}, kb, t, 1); }
    else { block(BoolTag<false>{}, ka, t, 0); block(BoolTag<false>{}, kb, t, 1); }
  };
  for (; base < st.end; base += AHEAD * PP_STEP) {
    tile(k0, k1, base);
    if (AHEAD == 2) tile(k2, k3, base + PP_STEP);     // past the slice's end every key is masked
  }
  // the four lane groups of a wave hold different keys of the same query; then the waves
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int off = 16; off < 64; off <<= 1) {
      const float mo = __shfl_xor(m_run[nb], off, 64), lo = __shfl_xor(l_run[nb], off, 64);
      const float mx = fmaxf(m_run[nb], mo);
      l_run[nb] = l_run[nb] * fast_exp2(m_run[nb] - mx) + lo * fast_exp2(mo - mx);
      m_run[nb] = mx;
    }
    if (st.q4 == 0) { sm_m[st.wave][nb * 16 + st.lr] = m_run[nb]; sm_l[st.wave][nb * 16 + st.lr] = l_run[nb]; }
  }
  __syncthreads();
  const int tid = threadIdx.x;
  if (tid < NB * 16) {
    float mx = NEG_BIG, l = 0.f;
#pragma unroll
    for (int w = 0; w < PP_WAVES; ++w) mx = fmaxf(mx, sm_m[w][tid]);
#pragma unroll
    for (int w = 0; w < PP_WAVES; ++w) l += sm_l[w][tid] * fast_exp2(sm_m[w][tid] - mx);
    float* dst = p.pp_stat + (((size_t)unit * nsplit + split) * 128 + tid) * 2;
    dst[0] = mx; dst[1] = l;
  }
}

// ---------------------------------------------------------------------------------------------
// scores: token score = (sum over the window queries that see the key of its probability) / (their number)
// ---------------------------------------------------------------------------------------------
template <int D, int NB, bool ROPE>
__global__ __launch_bounds__(PP_THREADS) void prompt_scores_kernel(Params p, const uint16_t* __restrict__ Qw,
                                                                   const uint16_t* __restrict__ K, int T, int W,
                                                                   int rows_per_split, int nsplit, int block_means) {
  using PS = PromptStream<D, NB, ROPE>;
  using KB = typename PS::KB;
  __shared__ float sm_ML[NB * 16];
  extern __shared__ __attribute__((aligned(16))) uint16_t scores_q[];   // ROPE: the turned queries; then sm_tok
  float* sm_tok = reinterpret_cast<float*>(scores_q + PS::Q_LDS_BYTES / 2);   // [rows_per_split] when block_means
  PS st;
  const int split = blockIdx.x, unit = blockIdx.y, tid = threadIdx.x;
  st.init(p, Qw, K, T, W, unit, split, rows_per_split, scores_q);
  const float sc = p.scale_log2e;
  const int lim_all = min(st.end, T - W + 1);

  // This pass walks its slice from the end to the start: what the first pass read last is what the
  // memory-side cache still holds, so most of a prompt that is not much larger than that cache is not
  // fetched from HBM a second time.
  KB k0, k1;
  const int first = st.begin + st.wave * PP_TILE;
  int base = first < st.end ? first + (st.end - 1 - first) / PP_STEP * PP_STEP : first - PP_STEP;
  st.load_block(k0, base); st.load_block(k1, base + 16);

  if (tid < NB * 16) {                 // the slices' (max, sum) of this query row -> the row's max and 1 / sum
    const float* src = p.pp_stat + ((size_t)unit * nsplit * 128 + tid) * 2;
    float mx = NEG_BIG, l = 0.f;
    for (int s = 0; s < nsplit; ++s) mx = fmaxf(mx, src[(size_t)s * 256]);
    for (int s = 0; s < nsplit; ++s) l += src[(size_t)s * 256 + 1] * fast_exp2(src[(size_t)s * 256] - mx);
    // probability = exp2(logit * scale - (max + log2 sum)); padding rows add nothing
    sm_ML[tid] = (tid < W * p.G && l > 0.f) ? -(mx + __builtin_amdgcn_logf(l)) : -INFINITY;
  }
  __syncthreads();
  float negML[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) negML[nb] = sm_ML[nb * 16 + st.lr];
  const float inv_w = 1.0f / (float)W;
  const bool averaged = !(p.flags & TREEKV_SCORE_ACCUMULATED);

  float* tok = p.pp_tok + (size_t)unit * T;
  auto block = [&](auto ragged, KB& k, int tile, int h) {
    constexpr bool RAGGED = decltype(ragged)::value;
    f32x4_t a[NB];
    st.logits(k, a);
    st.load_block(k, tile - PP_STEP + h * 16);
    float col[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float pe = fast_exp2(fmaf(a[nb][i], sc, negML[nb]));
        if (RAGGED) pe = (tile + h * 16 + st.q4 * 4 + i < st.lim[nb]) ? pe : 0.f;
        col[i] += pe;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) col[i] = row16_sum(col[i]);
    if (st.lr == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = tile + h * 16 + st.q4 * 4 + i;
        if (!RAGGED || j < st.end) {
          // every window query sees a key before the window; the key T - x is seen by x of them
          // (with accumulated weights as the criterion the sum itself is the score)
          const float sj = !averaged ? col[i] : RAGGED ? col[i] / (float)min(W, T - j) : col[i] * inv_w;
          tok[j] = sj;
          if (block_means) sm_tok[j - st.begin] = sj;
        }
      }
    }
  };
  for (; base >= first; base -= PP_STEP) {
    if (base + PP_TILE > lim_all) { block(BoolTag<true>{}, k0, base, 0); block(BoolTag<true>{}, k1, base, 1); }
    else { block(BoolTag<false>{}, k0, base, 0); block(BoolTag<false>{}, k1, base, 1); }
  }
  // a block's score is the mean over its W tokens (the blocks of this slice lie wholly inside it)
  if (block_means) {
    __syncthreads();
    float* beta = p.pp_beta + (size_t)unit * (T / W);
    for (int k = tid; k < (st.end - st.begin) / W; k += PP_THREADS) {
      float acc = 0.f;
      for (int x = 0; x < W; ++x) acc += sm_tok[k * W + x];
      beta[st.begin / W + k] = acc / (float)W;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// token scores for fp32 storage: plain vector arithmetic, one window query at a time
// ---------------------------------------------------------------------------------------------
// The matrix pipe takes bf16; with fp32 storage the scores are held to the precision of fp32 sums, so this instance
// works through the window's queries one after the other: LPR lanes share a key (16 bytes each, summed by shuffles),
// the scaled logits of the query sit in LDS, then become probabilities, and every thread adds those of the keys it
// owns to the unit's token scores.  One workgroup per unit; not a fast path (the one configuration with fp32
// storage has no prompt to compress).
constexpr int PF_THREADS = 256;

// ROPE (positions re-assigned): key j is turned to position j as it is read, window query i to T - W + i as it is
// staged, with the (cos, sin) table's rows for those positions.
template <int D, bool ROPE>
__global__ __launch_bounds__(PF_THREADS) void prompt_scores_f32_kernel(Params p, const float* __restrict__ Qw,
                                                                       const float* __restrict__ K, int T, int W) {
  constexpr int LPR = D / 4, KPP = PF_THREADS / LPR;
  extern __shared__ float pf_smem[];
  float* sp = pf_smem;                  // [T] scaled logits, then exponentials
  float* sred = sp + T;                 // [PF_THREADS / 64]
  float* sq = sred + PF_THREADS / 64;   // [D]
  const int unit = blockIdx.x, tid = threadIdx.x, kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int grp = tid / LPR, piece = tid % LPR;
  float* tok = p.pp_tok + (size_t)unit * T;
  const float* Ku = K + ((size_t)b * T * p.Hkv + kvh) * D;
  const size_t kstride = (size_t)p.Hkv * D;
  for (int j = tid; j < T; j += PF_THREADS) tok[j] = 0.f;      // a thread only ever touches the keys j = tid mod PF_THREADS
  auto block_reduce = [&](float v, bool take_max) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float o = __shfl_xor(v, off, 64);
      v = take_max ? fmaxf(v, o) : v + o;
    }
    __syncthreads();
    if ((tid & 63) == 0) sred[tid >> 6] = v;
    __syncthreads();
    float r = sred[0];
#pragma unroll
    for (int w = 1; w < PF_THREADS / 64; ++w) r = take_max ? fmaxf(r, sred[w]) : r + sred[w];
    __syncthreads();
    return r;
  };
  for (int i = 0; i < W; ++i) {
    const int nvis = T - W + i + 1;                             // window query i sees the keys up to its own
    for (int g = 0; g < p.G; ++g) {
      if (tid < D) {
        const float* qrow = Qw + (((size_t)b * W + i) * p.H + kvh * p.G + g) * D;
        float qx = qrow[tid];
        if constexpr (ROPE) {
          const float2 cs = p.rope_tab[(size_t)(T - W + i) * (D / 2) + tid / 2];
          const float other = qrow[tid ^ 1];
          qx = (tid & 1) ? other * cs.y + qx * cs.x : qx * cs.x - other * cs.y;
        }
        sq[tid] = qx;
      }
      __syncthreads();
      const float4 qv = *reinterpret_cast<const float4*>(sq + piece * 4);
      for (int j0 = 0; j0 < nvis; j0 += KPP) {
        const int j = j0 + grp;
        float acc = 0.f;
        if (j < nvis) {
          float4 kv = *reinterpret_cast<const float4*>(Ku + (size_t)j * kstride + piece * 4);
          if constexpr (ROPE) {
            const float4 cs = *reinterpret_cast<const float4*>(p.rope_tab + (size_t)j * (D / 2) + piece * 2);
            kv = make_float4(kv.x * cs.x - kv.y * cs.y, kv.x * cs.y + kv.y * cs.x, kv.z * cs.z - kv.w * cs.w,
                             kv.z * cs.w + kv.w * cs.z);
          }
          acc = kv.x * qv.x;
          acc = fmaf(kv.y, qv.y, acc);
          acc = fmaf(kv.z, qv.z, acc);
          acc = fmaf(kv.w, qv.w, acc);
        }
#pragma unroll
        for (int off = LPR / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (j < nvis && piece == 0) sp[j] = acc * p.scale_log2e;
      }
      __syncthreads();
      float mx = NEG_BIG;
      for (int j = tid; j < nvis; j += PF_THREADS) mx = fmaxf(mx, sp[j]);
      mx = block_reduce(mx, true);
      float sum = 0.f;
      for (int j = tid; j < nvis; j += PF_THREADS) {
        const float e = fast_exp2(sp[j] - mx);
        sp[j] = e;
        sum += e;
      }
      sum = block_reduce(sum, false);
      const float inv = 1.0f / sum;
      for (int j = tid; j < nvis; j += PF_THREADS) tok[j] += sp[j] * inv;
      __syncthreads();
    }
  }
  // the key T - x is seen by x of the window's queries, every key before the window by all W of them
  if (!(p.flags & TREEKV_SCORE_ACCUMULATED))
    for (int j = tid; j < T; j += PF_THREADS) tok[j] /= (float)min(W, T - j);
}

// ---------------------------------------------------------------------------------------------
// blocks: block means, Algorithm 1 over blocks with frozen scores, the kept blocks in ascending order
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prompt_blocks_kernel(Params p, int T, int b, int cb, int sink_b, int recent_b,
                                                            int have_means, int32_t* __restrict__ evicted_blocks) {
  extern __shared__ __attribute__((aligned(16))) float pb_smem[];
  const int unit = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int N = T / b, m_b = cb - sink_b - recent_b;
  float* beta = pb_smem;                                  // [N]
  // the tree region as (block, score bits) pairs, so that a pass reads a scope's two entries and nothing else
  int2* cur = reinterpret_cast<int2*>(pb_smem + ((N + 1) & ~1));   // [m_b]
  int2* nxt = cur + m_b;
  const float* tok = p.pp_tok + (size_t)unit * T;
  int* kept = p.pp_kept + (size_t)unit * p.budget;
  int32_t* evu = evicted_blocks ? evicted_blocks + (size_t)unit * N : nullptr;

  for (int k = tid; k < N; k += nt) {
    if (have_means) {
      beta[k] = p.pp_beta[(size_t)unit * N + k];
    } else {
      float acc = 0.f;
      for (int x = 0; x < b; ++x) acc += tok[(size_t)k * b + x];
      beta[k] = acc / (float)b;
    }
    if (evu && k < cb) evu[k] = -1;                       // blocks that arrive while the cache still has room
  }
  if (N <= cb) {                                          // nothing to evict
    for (int k = tid; k < N; k += nt) kept[k] = k;
    return;
  }
  __syncthreads();
  // One pass of idx over the tree region: the sequence is the region at the pass's start followed by the blocks
  // that enter during the pass; the block entering at eviction step e is block sink_b + m_b + e (the one that
  // just left the recent window, or the arriving block itself without one), the block arriving then is cb + e.
  const int n_ev = N - cb;
  if (m_b <= 64) {
    // A region that fits one wave stays in that wave's registers, one entry per lane, and a pass is a handful of
    // lane exchanges: no barrier between the passes (there are (N - cb) / m_b of them, 32 at 32768 tokens in blocks
    // of 64 into 2048 slots, and a workgroup barrier each was most of this kernel's time).
    if (tid < 64) {
      const int k = tid;
      int2 c = k < m_b ? make_int2(sink_b + k, __float_as_int(beta[sink_b + k])) : make_int2(0, 0);
      for (int e0 = 0; e0 < n_ev; e0 += m_b) {
        const int cnt = min(m_b, n_ev - e0);
        // entry `i` of the pass's sequence; every lane takes part in the exchanges, whatever its own i
        auto seq = [&](int i) {
          const int from = min(i, 63);
          int2 v = make_int2(__shfl(c.x, from, 64), __shfl(c.y, from, 64));
          if (i >= m_b && k < m_b) v = make_int2(sink_b + e0 + i, __float_as_int(beta[sink_b + e0 + i]));
          return v;
        };
        const bool scope = k < cnt;
        const int2 l = seq(scope ? 2 * k : k + cnt), r = seq(scope ? 2 * k + 1 : k + cnt);
        const bool drop_right = (p.flags & TREEKV_KEEP_LEFT) || (__int_as_float(l.y) > __int_as_float(r.y));   // a tie evicts the left block
        if (scope && evu) evu[cb + e0 + k] = drop_right ? r.x : l.x;
        c = (!scope || drop_right) ? l : r;
      }
      if (k < m_b) cur[k] = c;
    }
    __syncthreads();
  } else {
  for (int k = tid; k < m_b; k += nt) cur[k] = make_int2(sink_b + k, __float_as_int(beta[sink_b + k]));
  __syncthreads();
  for (int e0 = 0; e0 < n_ev; e0 += m_b) {
    const int cnt = min(m_b, n_ev - e0);
    auto seq = [&](int k) { return k < m_b ? cur[k] : make_int2(sink_b + e0 + k, __float_as_int(beta[sink_b + e0 + k])); };
    for (int k = tid; k < m_b; k += nt) {
      int2 v;
      if (k < cnt) {
        const int2 l = seq(2 * k), r = seq(2 * k + 1);
        const bool drop_right = (p.flags & TREEKV_KEEP_LEFT) || (__int_as_float(l.y) > __int_as_float(r.y));   // a tie evicts the left block
        v = drop_right ? l : r;
        if (evu) evu[cb + e0 + k] = drop_right ? r.x : l.x;
      } else {
        v = seq(k + cnt);
      }
      nxt[k] = v;
    }
    __syncthreads();
    int2* t = cur; cur = nxt; nxt = t;
  }
  }
  for (int i = tid; i < cb; i += nt) {
    int v;
    if (i < sink_b) v = i;
    else if (i < sink_b + m_b) v = cur[i - sink_b].x;
    else v = N - recent_b + (i - sink_b - m_b);
    kept[i] = v;
  }
}

// ---------------------------------------------------------------------------------------------
// handoff: the kept rows become slots 0 .. n-1 (logical order = slot order), and decoding's state is set
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prompt_handoff_kernel(Params p, const uint4* __restrict__ Kp,
                                                             const uint4* __restrict__ Vp, int T, int b, int n,
                                                             int row_vec, int32_t* __restrict__ retained,
                                                             int32_t* __restrict__ n_retained) {
  const int per_wg = 256 / row_vec;
  const int unit = blockIdx.y, tid = threadIdx.x;
  const int i = blockIdx.x * per_wg + tid / row_vec, e = tid % row_vec;
  const int kvh = unit % p.Hkv, bq = unit / p.Hkv;
  if (blockIdx.x == 0) {
    int* meta = p.meta + (size_t)unit * META_STRIDE;
    if (tid == 0) {
      meta[META_N] = n;
      meta[META_FREE] = n;             // n < budget: the next slot; n == budget: the spare slot
      meta[META_J] = 0;                // token-level eviction starts at the first scope
      meta[META_RHEAD] = 0;
      meta[META_T] = T;
      if (n_retained) n_retained[unit] = n;
    }
    int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
    for (int x = tid; x < p.n_recent; x += 256) Ru[x] = p.n_sink + p.m + x;
    int* Eu = p.E + (size_t)unit * 2 * p.m;
    int* PEu = p.PE + (size_t)unit * 2 * p.m;
    for (int k = p.m + tid; k < 2 * p.m; k += 256) Eu[k] = PEu[k] = 0;
  }
  if (i >= p.budget) return;
  int pos = -1;
  if (i < n) {
    const int kb = p.pp_kept[(size_t)unit * p.budget + i / b];
    pos = kb * b + i % b;
    const size_t src = (((size_t)bq * T + pos) * p.Hkv + kvh) * row_vec + e;
    const size_t dst = ((size_t)unit * p.cap + i) * row_vec + e;
    // streamed through: read once, and not read again before the caches have turned over (measured: with ordinary
    // stores the next call's first pass over the keys takes 6 us longer, the dirty rows being written back under it)
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u kk = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(Kp) + src);
    const v4u vv = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(Vp) + src);
    __builtin_nontemporal_store(kk, reinterpret_cast<v4u*>(p.K) + dst);
    __builtin_nontemporal_store(vv, reinterpret_cast<v4u*>(p.V) + dst);
  }
  if (e != 0) return;
  retained[(size_t)unit * p.budget + i] = pos;
  // Sbar stays the window average: C = T - pos queries of the prompt could attend the token, S = Sbar * C
  // (with accumulated weights as the criterion, S is the window's sum as it is)
  if (i < n) {
    const float sj = p.pp_tok[(size_t)unit * T + pos];
    p.S[(size_t)unit * p.cap + i] = (p.flags & TREEKV_SCORE_ACCUMULATED) ? sj : sj * (float)(T - pos);
  }
  const int k = i - p.n_sink;
  if (k >= 0 && k < p.m) {
    p.E[(size_t)unit * 2 * p.m + k] = i;
    p.PE[(size_t)unit * 2 * p.m + k] = i < n ? pos : i;
  }
}

template <int D, int NB, bool ROPE>
int launch_streams(const Params& p, const uint16_t* Qw, const uint16_t* K, int T, int W, int rows_per_split,
                   int nsplit, int block_means, hipStream_t s) {
  constexpr size_t q_lds = PromptStream<D, NB, ROPE>::Q_LDS_BYTES;
  const size_t lds = q_lds + (block_means ? (size_t)rows_per_split * 4 : 0);
  if (q_lds > 48 * 1024 && hip_failed(hipFuncSetAttribute((const void*)prompt_stats_kernel<D, NB, ROPE>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)q_lds)))
    return TREEKV_EHIP;
  if (lds > 48 * 1024 && hip_failed(hipFuncSetAttribute((const void*)prompt_scores_kernel<D, NB, ROPE>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
    return TREEKV_EHIP;
  if constexpr (ROPE) hipLaunchKernelGGL((prompt_turn_queries_kernel<D>), dim3(128 * (D / 2) / 256, p.U), dim3(256), 0, s, p, Qw, T, W);
  hipLaunchKernelGGL((prompt_stats_kernel<D, NB, ROPE>), dim3(nsplit, p.U), dim3(PP_THREADS), q_lds, s, p, Qw, K, T, W,
                     rows_per_split, nsplit);
  hipLaunchKernelGGL((prompt_scores_kernel<D, NB, ROPE>), dim3(nsplit, p.U), dim3(PP_THREADS), lds, s, p, Qw, K, T, W,
                     rows_per_split, nsplit, block_means);
  return TREEKV_OK;
}

template <int D, bool ROPE>
int launch_streams_r(const Params& p, const uint16_t* Qw, const uint16_t* K, int T, int W, int rows_per_split,
                     int nsplit, int block_means, hipStream_t s) {
  const int nb = (W * p.G + 15) / 16;
  if (nb <= 2) return launch_streams<D, 2, ROPE>(p, Qw, K, T, W, rows_per_split, nsplit, block_means, s);
  if (nb <= 4) return launch_streams<D, 4, ROPE>(p, Qw, K, T, W, rows_per_split, nsplit, block_means, s);
  return launch_streams<D, 8, ROPE>(p, Qw, K, T, W, rows_per_split, nsplit, block_means, s);
}

template <int D>
int launch_streams_d(const Params& p, const uint16_t* Qw, const uint16_t* K, int T, int W, int rows_per_split,
                     int nsplit, int block_means, hipStream_t s) {
  if (p.flags & TREEKV_POSITION_RERANK) return launch_streams_r<D, true>(p, Qw, K, T, W, rows_per_split, nsplit, block_means, s);
  return launch_streams_r<D, false>(p, Qw, K, T, W, rows_per_split, nsplit, block_means, s);
}

}  // namespace

// Slices per unit: one workgroup per compute unit (measured: 256 workgroups 51 us, 512: 60, 1024: 73 for the
// statistics pass over a 32k prompt of 32 heads), a slice a multiple of what a workgroup
// takes per iteration, at most PROMPT_MAX_SPLITS of them.
int prompt_splits(const Params& p, int T, int* rows_per_split) {
  int ns = (256 + p.U - 1) / p.U;
  const int by_len = (T + PP_STEP - 1) / PP_STEP;
  if (ns > by_len) ns = by_len;
  if (ns > PROMPT_MAX_SPLITS) ns = PROMPT_MAX_SPLITS;
  if (ns < 1) ns = 1;
  int rows = ((T + ns - 1) / ns + PP_STEP - 1) / PP_STEP * PP_STEP;
  ns = (T + rows - 1) / rows;
  *rows_per_split = rows;
  return ns;
}

size_t prompt_blocks_lds(int T, int b, int cb, int sink_b, int recent_b) {
  return ((size_t)(T / b) + 1 + 4 * (size_t)(cb - sink_b - recent_b)) * 4;
}

int launch_prompt(const Params& p, const void* Qw, const void* K, const void* V, int T, int b, int32_t* retained,
                  int32_t* n_retained, int32_t* evicted_blocks, float* token_scores, hipStream_t s) {
  const int cb = p.budget / b, sink_b = (p.n_sink + b - 1) / b, recent_b = (p.n_recent + b - 1) / b;
  int block_means = 0;
  if (p.dtype == TREEKV_F32) {
    // fp32 storage: the vector-ALU instance (a query's logits must fit in LDS)
    if (T > 32768) return TREEKV_EUNSUPPORTED;
    const size_t lds = ((size_t)T + PF_THREADS / 64 + p.D) * sizeof(float);
    const bool rope = (p.flags & TREEKV_POSITION_RERANK) != 0;
    auto kern = p.D == 128 ? (rope ? prompt_scores_f32_kernel<128, true> : prompt_scores_f32_kernel<128, false>)
                           : (rope ? prompt_scores_f32_kernel<64, true> : prompt_scores_f32_kernel<64, false>);
    if (lds > 48 * 1024 && hip_failed(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
      return TREEKV_EHIP;
    hipLaunchKernelGGL(kern, dim3(p.U), dim3(PF_THREADS), lds, s, p, (const float*)Qw, (const float*)K, T, b);
  } else {
    int rows_per_split = 0;
    const int nsplit = prompt_splits(p, T, &rows_per_split);
    // the scores kernel also takes the block means when no block straddles two slices and a slice's scores fit
    // in 40 KB of LDS (slices start at multiples of what a workgroup takes per iteration)
    block_means = (PP_STEP % b == 0 && (size_t)rows_per_split * 4 <= 40 * 1024) ? 1 : 0;
    const int rc = p.D == 128 ? launch_streams_d<128>(p, (const uint16_t*)Qw, (const uint16_t*)K, T, b, rows_per_split, nsplit, block_means, s)
                              : launch_streams_d<64>(p, (const uint16_t*)Qw, (const uint16_t*)K, T, b, rows_per_split, nsplit, block_means, s);
    if (rc != TREEKV_OK) return rc;
  }
  const size_t lds = prompt_blocks_lds(T, b, cb, sink_b, recent_b);
  if (lds > 48 * 1024 &&
      hip_failed(hipFuncSetAttribute((const void*)prompt_blocks_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
    return TREEKV_EHIP;
  const int blocks_threads = 256;
  hipLaunchKernelGGL(prompt_blocks_kernel, dim3(p.U), dim3(blocks_threads), lds, s, p, T, b, cb, sink_b, recent_b,
                     block_means, evicted_blocks);
  const int row_vec = p.D * (p.dtype == TREEKV_BF16 ? 2 : 4) / 16, per_wg = 256 / row_vec;
  const int n = T < p.budget ? T : p.budget;
  hipLaunchKernelGGL(prompt_handoff_kernel, dim3((p.budget + per_wg - 1) / per_wg, p.U), dim3(256), 0, s, p,
                     (const uint4*)K, (const uint4*)V, T, b, n, row_vec, retained, n_retained);
  if (token_scores &&
      hip_failed(hipMemcpyAsync(token_scores, p.pp_tok, (size_t)p.U * T * sizeof(float), hipMemcpyDeviceToDevice, s)))
    return TREEKV_EHIP;
  return finish_launch();
}

}  // namespace tkv
