// Chunked prefill of TreeKV for gfx950.
//
// A chunk of L tokens attends the cache as it was before the chunk plus the chunk's own tokens
// up to and including itself; every row's probabilities are added to the scores; the averaged
// scores are then frozen and Algorithm 1's append / compare / evict / advance (lines 4-5, 9-17)
// is replayed for the L tokens.  L = 1 gives the decode step.
//
// Three launches per chunk:
//   attend   grid row tiles x G x U (ids remapped so that a unit's row tiles share an XCD's L2).  Two passes
//            over all visible columns with MFMA (16x16x32 bf16): the first finds the row statistics, the
//            second forms the final probabilities, O^T += V^T P^T with P split into two bf16 halves
//            (hi + lo) so that rounding P costs 2^-16, not 2^-9, and the probabilities' sums down the
//            workgroup's rows, one part per row group.  Writes O and the column-sum parts.
//   replay   grid U.  Adds the column-sum parts to the scores (Algorithm 1, line 8; fixed order, no
//            atomics), then Algorithm 1's eviction for the chunk's tokens with frozen scores.  Inside one
//            sweep of idx over the tree region the scopes are disjoint pairs, so a sweep is one
//            parallel pass; sweeps run one after the other.  Then surviving chunk tokens are
//            matched with freed slots (prefix sums), the order arrays are rewritten and the
//            retained positions emitted.
//   scatter  grid (L, U).  Copies the surviving chunk rows into their slots.
//
// Token ids during the replay: a slot number (< cap) for a cached token, cap + i for chunk
// token i that has no slot yet.

#include "treekv_internal.h"

namespace tkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int ROW_TILE = 64;     // query rows per attend workgroup
constexpr float NEG_BIG = -1.0e30f;

__device__ inline f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

struct ChunkInfo {
  int n;        // tokens cached before the chunk
  int fslot;    // the free slot (a hole among slots [0, n] once the cache is full)
  int t0;       // position of the chunk's first token
};

__device__ inline ChunkInfo load_chunk_info(const int* meta) {
  ChunkInfo c;
  c.n = meta[META_N];
  c.fslot = meta[META_FREE];
  c.t0 = meta[META_T];
  return c;
}

// ---------------------------------------------------------------------------------------------
// attend
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

// two floats -> two bf16 (round to nearest even) packed in one dword, first value in the low half
__device__ inline unsigned pack_bf16(float a, float b) {
  f32x2_t v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

constexpr int AT_THREADS = 512;   // 8 waves
constexpr int AT_COLS = 128;      // columns per staged tile of the attend kernel

template <int D>
struct AttendLds {
  static constexpr int KSTRIDE = D + 8;          // bf16 elements per staged K row (padded: conflict-free b128 reads)
  static constexpr int VSTRIDE = AT_COLS + 8;    // bf16 elements per staged V^T row
  static constexpr int K_ELEMS = AT_COLS * KSTRIDE;
  static constexpr int V_ELEMS = D * VSTRIDE;
  static constexpr size_t BYTES = 2 * (size_t)(K_ELEMS + V_ELEMS) * sizeof(uint16_t);   // two stages
};

// One workgroup owns 64 query rows of one head and passes over the visible columns twice.
//
// Sweep 1 finds every row's softmax statistics (max, sum).  No LDS and no barriers: wave w takes the
// 16-column block w of every 128-column tile against all 64 rows, its K rows loaded straight from
// global memory in MFMA operand order (every K row is read once per workgroup).  Each lane keeps a
// running (max, sum) for its own columns of its four rows; lanes and waves are merged once, at the end.
//
// Sweep 2 recomputes the logits and, knowing the statistics, forms the normalised probabilities
// directly: p = exp2(s*scale - max - log2(sum)), no running maximum and nothing to rescale.  They feed
// O^T += V^T P^T and, summed down the rows, the per-column score increments (Algorithm 1, line 8).
// Here K and V^T tiles are staged through LDS, double buffered, and the 8 waves are 2 row groups (32 rows
// = two 16-row MFMA blocks) x 4 column quarters (32 columns of every tile): each K / V^T operand read
// from LDS feeds the MFMAs of two row blocks, and two waves share a SIMD so that one's exp / convert
// work overlaps the other's MFMAs.  The four quarters of a row group add their O through LDS at the end.
// Threads 0-255 stage V (transposing), threads 256-511 stage K.
//
// Column sums: a wave adds its two row blocks, reduces over the 16 lanes that hold the 16 rows and
// writes the 32 sums of its columns to part row_tile*2 + row_group of the head's partial array;
// the replay kernel adds the parts in a fixed order.  A workgroup writes every column of every tile it
// visits (masked entries as zeros) and nothing else.
//
// Staged V^T layout.  Row d holds the tile's columns in the order the P^T operand uses them: inside
// quarter c, column j sits at position c*32 + ((j%16)/4)*8 + ((j%32)/16)*4 + j%4, so that the 8 k-slots of
// lane group q4 (columns c*32 + q4*4 + {0..3} and c*32 + 16 + q4*4 + {0..3}) are the 16 contiguous
// bytes of "pair" c*4 + q4.  Pairs are XOR-swizzled with (d/16)%8: the 16 lanes of an operand read share
// d/16, so reads stay conflict free, while the transposing 8-byte writes of 16 lanes (same columns, rows 8
// apart) spread over the banks.
template <int CTRL>
__device__ inline float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
  return v + __int_as_float(moved);
}
// max of three.  This file is compiled with -fno-honor-nans: otherwise every fmaxf operand that comes out of
// an MFMA costs an extra instruction that quiets signalling NaNs, and the pair is not fused into v_max3_f32.
__device__ inline float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
template <bool B> struct BoolTag { static constexpr bool value = B; };

// Sum over the 16 lanes of a DPP row; every lane gets the total.
__device__ inline float row16_sum(float v) {
  v = dpp_add<0x128>(v);           // row_ror:8
  v = dpp_add<0x124>(v);           // row_ror:4
  v = dpp_add<0x122>(v);           // row_ror:2
  v = dpp_add<0x121>(v);           // row_ror:1
  return v;
}

template <int D>
__global__ __launch_bounds__(AT_THREADS) void prefill_attend_kernel(Params p, const uint16_t* __restrict__ Q,
                                                                    const uint16_t* __restrict__ Kc,
                                                                    const uint16_t* __restrict__ Vc, int L,
                                                                    int row_tiles, float* __restrict__ out) {
  using Lds = AttendLds<D>;
  constexpr int KS = D / 32;          // k-steps of the q.k contraction
  constexpr int DB = D / 16;          // 16-wide blocks of the head dimension
  constexpr int PARTS = D / 8;        // 16-byte pieces per row
  constexpr int KCH = AT_COLS * PARTS / 256;           // K pieces per K-staging thread (4 or 8)
  constexpr int VBL = (AT_COLS / 4) * PARTS / 256;     // 4-column x 8-dim V blocks per V-staging thread (1 or 2)
  static_assert((KCH == 4 || KCH == 8) && (VBL == 1 || VBL == 2), "staging is written for head_dim 64 and 128");
  constexpr int KROWS_PER_X = 256 / PARTS;             // rows between a K thread's consecutive pieces
  constexpr int VJG_PER_X = 256 / PARTS;               // column groups between a V thread's two blocks
  extern __shared__ __attribute__((aligned(16))) uint16_t pf_smem[];
  uint16_t* sK = pf_smem;                               // [2][K_ELEMS]
  uint16_t* sVt = pf_smem + 2 * Lds::K_ELEMS;           // [2][V_ELEMS]

  // Workgroups are dealt to the 8 XCDs round robin by their linear id, and each XCD has its own L2.
  // The row tiles of one unit read the same K and V, so give them ids that land on one XCD:
  // workgroup w works on item (w % 8) * (n/8) + w / 8 of the (row tile fastest) item list.
  const int n_items = row_tiles * p.G * p.U, per_xcd = (n_items + 7) / 8;
  const int item = ((int)blockIdx.x % 8) * per_xcd + (int)blockIdx.x / 8;
  if (item >= n_items) return;
  const int row_tile = item % row_tiles, g = (item / row_tiles) % p.G, unit = item / (row_tiles * p.G);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, q4 = lane >> 4;
  const int rg = wave & 1;                                 // sweep 2: rows 32*rg .. +31 of the workgroup's 64
  const int cq = wave >> 1;                                // sweep 2: column quarter of every tile
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int h = kvh * p.G + g;
  const ChunkInfo ci = load_chunk_info(p.meta + (size_t)unit * META_STRIDE);
  const int rbase = row_tile * ROW_TILE;                   // first chunk row of the workgroup

  // B operands: the Q rows of the four 16-row blocks (rows past the chunk repeat its last row)
  uint4 qa[4][KS];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    const uint16_t* qp = Q + (((size_t)b * L + min(rbase + rb * 16 + lr, L - 1)) * p.H + h) * D + q4 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qa[rb][ks] = *reinterpret_cast<const uint4*>(qp + ks * 32);
  }

  const uint16_t* Ku = (const uint16_t*)p.K + (size_t)unit * p.cap * D;
  const uint16_t* Vu = (const uint16_t*)p.V + (size_t)unit * p.cap * D;
  const int chunk_row_stride = p.Hkv * D;
  const uint16_t* Kcu = Kc + ((size_t)b * L * p.Hkv + kvh) * D;
  const uint16_t* Vcu = Vc + ((size_t)b * L * p.Hkv + kvh) * D;

  const int cache_tiles = (ci.n + 1 + AT_COLS - 1) / AT_COLS;          // slots [0, n], the free one masked
  const int last_row = min(rbase + ROW_TILE, L) - 1;                   // last chunk row of the workgroup
  const int chunk_tiles = last_row / AT_COLS + 1;                      // causal: columns <= last_row
  const int ntiles = cache_tiles + chunk_tiles;
  const float sc = p.scale_log2e;
  const int n_cached = ci.n, fslot = ci.fslot;
  const int cache_lim = p.cap - 1, chunk_lim = L - 1;                   // last row that exists

  // ------------------------------------------------------------------------------------------
  // sweep 1: row statistics
  // ------------------------------------------------------------------------------------------
  float neg_ml0, neg_ml1;              // -(max + log2(sum)) in the scaled log2 domain, rows of the two sweep-2 blocks
  {
    float m_run[4], l_run[4];          // this lane's columns of row rb*16 + lr: max of the scaled logits, sum of exp2
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) { m_run[rb] = NEG_BIG; l_run[rb] = 0.f; }
    // K tiles go through LDS here too (two stages): 16 lanes fetch one row with 16-byte loads, which the memory
    // pipeline coalesces; MFMA operand order (consecutive lanes = consecutive rows) straight from global does not.
    constexpr int RPP = AT_THREADS / PARTS;          // rows per pass of the 512 threads
    constexpr int NPASS = AT_COLS / RPP;             // passes per tile (4 at d=128, 2 at d=64)
    const int s_row = tid / PARTS, s_part = tid % PARTS;
    uint4 kr0, kr1, kr2, kr3;
    kr0 = kr1 = kr2 = kr3 = make_uint4(0, 0, 0, 0);
    auto load_k = [&](int tile) {
      const bool is_cache = tile < cache_tiles;
      const int col0 = is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS;
      const uint16_t* base = (is_cache ? Ku : Kcu) + s_part * 8;
      const int rstride = is_cache ? D : chunk_row_stride;
      const int lim = is_cache ? cache_lim : chunk_lim;
      auto ld = [&](int x) { return *reinterpret_cast<const uint4*>(base + (size_t)min(col0 + s_row + x * RPP, lim) * rstride); };
      kr0 = ld(0); kr1 = ld(1);
      if constexpr (NPASS > 2) { kr2 = ld(2); kr3 = ld(3); }
    };
    auto store_k = [&](int buf) {
      uint16_t* dst = sK + buf * Lds::K_ELEMS + s_row * Lds::KSTRIDE + s_part * 8;
      *reinterpret_cast<uint4*>(dst) = kr0;
      *reinterpret_cast<uint4*>(dst + RPP * Lds::KSTRIDE) = kr1;
      if constexpr (NPASS > 2) {
        *reinterpret_cast<uint4*>(dst + 2 * RPP * Lds::KSTRIDE) = kr2;
        *reinterpret_cast<uint4*>(dst + 3 * RPP * Lds::KSTRIDE) = kr3;
      }
    };
    // S^T of this wave's 16 columns of a staged tile against the 64 rows
    const int k1_off = (wave * 16 + lr) * Lds::KSTRIDE + q4 * 8;
    auto qk = [&](f32x4_t (&s)[4], int buf) {
      const uint16_t* kp = sK + buf * Lds::K_ELEMS + k1_off;
      uint4 k[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) k[ks] = *reinterpret_cast<const uint4*>(kp + ks * 32);
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) s[rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) s[rb] = mfma16(k[ks], qa[rb][ks], s[rb]);
    };
    // Masked logits become -inf: their exp2 is 0 against any finite running max, and a lane that has seen
    // nothing yet keeps its (finite) initial max, so no probability needs a guard.
    auto stats = [&](f32x4_t (&s)[4], int tile) {
      const bool is_cache = tile < cache_tiles;
      const int c0 = (is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS) + wave * 16;   // this wave's 16 columns
      // only tiles that touch the end of the cache, the free slot or the causal diagonal need a mask (wave uniform)
      const bool need_mask = is_cache ? (c0 + 15 > n_cached || (fslot >= c0 && fslot < c0 + 16)) : (c0 + 15 > rbase);
      if (need_mask) {
        const int excl = is_cache ? fslot : -1;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
          const int lim = is_cache ? n_cached : rbase + rb * 16 + lr;      // last visible column of this lane's row
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int col = c0 + q4 * 4 + i;
            s[rb][i] = (col <= lim && col != excl) ? s[rb][i] : -INFINITY;
          }
        }
      }
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        // The running max lives in the scaled domain: exp2(m_run - m_new) is then exactly 1 when the max stays.
        const float m_new = fmaxf(m_run[rb], max3(s[rb][0], s[rb][1], fmaxf(s[rb][2], s[rb][3])) * sc);
        const float e0 = fast_exp2(fmaf(s[rb][0], sc, -m_new)), e1 = fast_exp2(fmaf(s[rb][1], sc, -m_new));
        const float e2 = fast_exp2(fmaf(s[rb][2], sc, -m_new)), e3 = fast_exp2(fmaf(s[rb][3], sc, -m_new));
        l_run[rb] = fmaf(l_run[rb], fast_exp2(m_run[rb] - m_new), (e0 + e1) + (e2 + e3));
        m_run[rb] = m_new;
      }
    };
    // Software pipeline: while the statistics of tile t are updated (vector ALU), the logits of tile t+1 are
    // formed (matrix pipe) and tile t+2 is on its way from global memory.  One barrier per tile.
    f32x4_t sa[4], sb[4];
    load_k(0);
    store_k(0);
    if (ntiles > 1) { load_k(1); store_k(1); }
    __syncthreads();
    qk(sa, 0);
    __syncthreads();                    // stage 0 is overwritten below
    auto step = [&](f32x4_t (&cur)[4], f32x4_t (&nxt)[4], int t) {
      if (t + 2 < ntiles) load_k(t + 2);
      if (t + 1 < ntiles) qk(nxt, (t + 1) & 1);
      stats(cur, t);
      if (t + 2 < ntiles) store_k(t & 1);        // tile t's stage: last read one barrier ago
      __syncthreads();
    };
    for (int t = 0; t < ntiles; t += 2) {
      step(sa, sb, t);
      if (t + 1 < ntiles) step(sb, sa, t + 1);
    }
    // merge the four lanes that share a row, then the eight waves through LDS
    float* st = reinterpret_cast<float*>(pf_smem);       // [8 waves][64 rows][2]
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {
        const float mo = __shfl_xor(m_run[rb], off, 64), lo = __shfl_xor(l_run[rb], off, 64);
        const float mn = fmaxf(m_run[rb], mo);
        l_run[rb] = l_run[rb] * fast_exp2(m_run[rb] - mn) + lo * fast_exp2(mo - mn);
        m_run[rb] = mn;
      }
      if (q4 == 0) {
        st[(wave * 64 + rb * 16 + lr) * 2] = m_run[rb];
        st[(wave * 64 + rb * 16 + lr) * 2 + 1] = l_run[rb];
      }
    }
    __syncthreads();
    auto final_of = [&](int r) {       // r: row inside the workgroup's 64
      float mx = NEG_BIG;
#pragma unroll
      for (int w = 0; w < 8; ++w) mx = fmaxf(mx, st[(w * 64 + r) * 2]);
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) l += st[(w * 64 + r) * 2 + 1] * fast_exp2(st[(w * 64 + r) * 2] - mx);
      // rows past the chunk get probabilities of zero: they must not reach the column sums
      return rbase + r < L ? -(mx + __log2f(l)) : NEG_BIG;
    };
    neg_ml0 = final_of(rg * 32 + lr);
    neg_ml1 = final_of(rg * 32 + 16 + lr);
    __syncthreads();                   // the staging below reuses this LDS
  }

  // ------------------------------------------------------------------------------------------
  // sweep 2: outputs and column sums
  // ------------------------------------------------------------------------------------------
  const int row0 = rbase + rg * 32;                        // first chunk row of this wave
  const int my_row0 = row0 + lr, my_row1 = row0 + 16 + lr; // the query rows this lane's results belong to
  uint4 qa0[KS], qa1[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const uint4 a0 = qa[0][ks], a1 = qa[1][ks], a2 = qa[2][ks], a3 = qa[3][ks];   // values, not addresses, into the select
    qa0[ks] = rg ? a2 : a0;
    qa1[ks] = rg ? a3 : a1;
  }

  // ---- staging: global -> registers -> LDS (named registers: arrays here end up in scratch memory) ----
  uint4 g0, g1, g2, g3, g4, g5, g6, g7;
  g0 = g1 = g2 = g3 = g4 = g5 = g6 = g7 = make_uint4(0, 0, 0, 0);
  const bool v_role = tid < 256;
  const int st = tid & 255;
  // V role: blocks of columns (v_jg + x*VJG_PER_X)*4..+3, dims v_part*8..+7.  K role: pieces st + x*256.
  const int v_part = st % PARTS, v_jg = st / PARTS;
  const int k_r0 = st / PARTS, k_part = st % PARTS;
  const uint16_t* cache_base = (v_role ? Vu : Ku) + (v_role ? v_part : k_part) * 8;
  const uint16_t* chunk_base = (v_role ? Vcu : Kcu) + (v_role ? v_part : k_part) * 8;
  auto load_regs = [&](int tile) {
    const bool is_cache = tile < cache_tiles;
    const int col0 = is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS;
    const uint16_t* base = is_cache ? cache_base : chunk_base;
    const int rstride = is_cache ? D : chunk_row_stride;
    const int lim = is_cache ? cache_lim : chunk_lim;
    auto ld = [&](int r) { return *reinterpret_cast<const uint4*>(base + (size_t)min(col0 + r, lim) * rstride); };
    if (v_role) {
      const int r = v_jg * 4;
      g0 = ld(r); g1 = ld(r + 1); g2 = ld(r + 2); g3 = ld(r + 3);
      if constexpr (VBL > 1) {
        const int r2 = r + VJG_PER_X * 4;
        g4 = ld(r2); g5 = ld(r2 + 1); g6 = ld(r2 + 2); g7 = ld(r2 + 3);
      }
    } else {
      g0 = ld(k_r0); g1 = ld(k_r0 + KROWS_PER_X); g2 = ld(k_r0 + 2 * KROWS_PER_X); g3 = ld(k_r0 + 3 * KROWS_PER_X);
      if constexpr (KCH > 4) {
        g4 = ld(k_r0 + 4 * KROWS_PER_X); g5 = ld(k_r0 + 5 * KROWS_PER_X);
        g6 = ld(k_r0 + 6 * KROWS_PER_X); g7 = ld(k_r0 + 7 * KROWS_PER_X);
      }
    }
  };
  // LDS destinations do not depend on the tile: byte offsets inside one stage
  const int k_dst = (k_r0 * Lds::KSTRIDE + k_part * 8) * 2;
  auto v_dst_of = [&](int jg) {        // column group jg (4 columns) of the tile, this thread's 8 dims
    const int c = jg / 8, jq = jg % 8;                                  // quarter, group inside the quarter
    const int pair = (c * 4 + (jq % 4)) ^ ((v_part >> 1) & 7);          // (d/16)%8 == v_part/2 for all 8 dims
    return ((v_part * 8) * Lds::VSTRIDE + pair * 8 + (jq / 4) * 4) * 2;
  };
  const int v_dst0 = v_dst_of(v_jg), v_dst1 = v_dst_of(v_jg + VJG_PER_X);
  auto store_lds = [&](int buf) {
    if (!v_role) {
      char* k = reinterpret_cast<char*>(sK + buf * Lds::K_ELEMS) + k_dst;
      constexpr int step = KROWS_PER_X * Lds::KSTRIDE * 2;
      *reinterpret_cast<uint4*>(k) = g0;
      *reinterpret_cast<uint4*>(k + step) = g1;
      *reinterpret_cast<uint4*>(k + 2 * step) = g2;
      *reinterpret_cast<uint4*>(k + 3 * step) = g3;
      if constexpr (KCH > 4) {
        *reinterpret_cast<uint4*>(k + 4 * step) = g4;
        *reinterpret_cast<uint4*>(k + 5 * step) = g5;
        *reinterpret_cast<uint4*>(k + 6 * step) = g6;
        *reinterpret_cast<uint4*>(k + 7 * step) = g7;
      }
    } else {
      char* vb = reinterpret_cast<char*>(sVt + buf * Lds::V_ELEMS);
      // dword w of the four rows holds dims 2w, 2w+1 of columns +0..+3: regroup into one 8-byte word per dim
      auto emit = [&](char* v, unsigned a0, unsigned a1, unsigned a2, unsigned a3, int e_even) {
#pragma unroll
        for (int odd = 0; odd < 2; ++odd) {
          const unsigned sel = odd ? 0x07060302u : 0x05040100u;       // the odd / even bf16 of both dwords
          uint2 o;
          o.x = __builtin_amdgcn_perm(a1, a0, sel);                   // columns +0, +1
          o.y = __builtin_amdgcn_perm(a3, a2, sel);                   // columns +2, +3
          *reinterpret_cast<uint2*>(v + (e_even + odd) * Lds::VSTRIDE * 2) = o;
        }
      };
      char* v0 = vb + v_dst0;
      emit(v0, g0.x, g1.x, g2.x, g3.x, 0); emit(v0, g0.y, g1.y, g2.y, g3.y, 2);
      emit(v0, g0.z, g1.z, g2.z, g3.z, 4); emit(v0, g0.w, g1.w, g2.w, g3.w, 6);
      if constexpr (VBL > 1) {
        char* v1 = vb + v_dst1;
        emit(v1, g4.x, g5.x, g6.x, g7.x, 0); emit(v1, g4.y, g5.y, g6.y, g7.y, 2);
        emit(v1, g4.z, g5.z, g6.z, g7.z, 4); emit(v1, g4.w, g5.w, g6.w, g7.w, 6);
      }
    }
  };

  // operand read offsets (bytes inside one stage), tile independent
  const int ka_off = ((cq * 32 + lr) * Lds::KSTRIDE + q4 * 8) * 2;                     // + bk*16 rows, + ks*64 bytes
  const int va_row = (lr * Lds::VSTRIDE) * 2;
  const int va_pair = cq * 4 + q4;                                                     // swizzled with d & 7 per read

  f32x4_t o0[DB], o1[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) { o0[d] = f32x4_t{0.f, 0.f, 0.f, 0.f}; o1[d] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }

  // the part of the head's column-sum array this wave writes: [cache columns rounded up to a tile | chunk columns]
  const int cap_cols = (p.cap + AT_COLS - 1) / AT_COLS * AT_COLS;
  const int cs_stride = cap_cols + (p.max_chunk + AT_COLS - 1) / AT_COLS * AT_COLS;
  const int n_parts = 2 * ((p.max_chunk + ROW_TILE - 1) / ROW_TILE);
  float* cs_part = p.pf_colpart + (((size_t)unit * p.G + g) * n_parts + row_tile * 2 + rg) * cs_stride + cq * 32 + q4 * 4;

  // probabilities of one row block's 8 logits: the packed hi / lo P^T operands; the values themselves in place of s
  auto soft = [&](f32x4_t (&s)[2], float neg_ml, uint4& phi, uint4& plo) {
    unsigned hi[4], lo[4];                    // k-slots 0-3 = block 0, i = 0..3; k-slots 4-7 = block 1
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const float p0 = fast_exp2(fmaf(s[e2 >> 1][(e2 & 1) * 2], sc, neg_ml));
      const float p1 = fast_exp2(fmaf(s[e2 >> 1][(e2 & 1) * 2 + 1], sc, neg_ml));
      s[e2 >> 1][(e2 & 1) * 2] = p0;
      s[e2 >> 1][(e2 & 1) * 2 + 1] = p1;
      hi[e2] = pack_bf16(p0, p1);
      lo[e2] = pack_bf16(p0 - __uint_as_float(hi[e2] << 16), p1 - __uint_as_float(hi[e2] & 0xffff0000u));
    }
    phi = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    plo = make_uint4(lo[0], lo[1], lo[2], lo[3]);
  };

  load_regs(0);
  store_lds(0);
  __syncthreads();
  for (int tile = 0; tile < ntiles; ++tile) {
    if (tile + 1 < ntiles) load_regs(tile + 1);            // in flight while this tile is computed
    const bool is_cache = tile < cache_tiles;
    const int col0 = is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS;
    const char* k = reinterpret_cast<const char*>(sK + (tile & 1) * Lds::K_ELEMS) + ka_off;
    const char* v = reinterpret_cast<const char*>(sVt + (tile & 1) * Lds::V_ELEMS);

    // S^T blocks: rows = columns col0 + cq*32 + bk*16 + q4*4 + i, column = the lane's query row of block 0 / 1
    f32x4_t s0[2], s1[2];
#pragma unroll
    for (int bk = 0; bk < 2; ++bk) {
      s0[bk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      s1[bk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 a = *reinterpret_cast<const uint4*>(k + bk * 16 * Lds::KSTRIDE * 2 + ks * 64);
        s0[bk] = mfma16(a, qa0[ks], s0[bk]);
        s1[bk] = mfma16(a, qa1[ks], s1[bk]);
      }
    }
    // only tiles that touch the end of the cache, the free slot or the causal diagonal need a mask (wave uniform)
    const bool need_mask = is_cache ? (col0 + AT_COLS - 1 > n_cached || (fslot >= col0 && fslot < col0 + AT_COLS))
                                    : (col0 + AT_COLS - 1 > row0);
    if (need_mask) {
      const int cbase = col0 + cq * 32 + q4 * 4;
      const int excl = is_cache ? fslot : -1;
      const int lim0 = is_cache ? n_cached : my_row0, lim1 = is_cache ? n_cached : my_row1;   // last visible column
#pragma unroll
      for (int bk = 0; bk < 2; ++bk)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int col = cbase + bk * 16 + i;
          s0[bk][i] = (col <= lim0 && col != excl) ? s0[bk][i] : -INFINITY;   // exp2 gives exactly 0
          s1[bk][i] = (col <= lim1 && col != excl) ? s1[bk][i] : -INFINITY;
        }
    }
    uint4 phi0, plo0, phi1, plo1;
    soft(s0, neg_ml0, phi0, plo0);
    soft(s1, neg_ml1, phi1, plo1);
    // O^T += V^T P^T : A = V^T[d][the quarter's 8 k-slot columns of this lane group], B = P^T (hi and lo parts)
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      const uint4 a = *reinterpret_cast<const uint4*>(v + va_row + ((va_pair ^ (d & 7)) * 16) + d * 16 * Lds::VSTRIDE * 2);
      o0[d] = mfma16(a, phi0, o0[d]);
      o1[d] = mfma16(a, phi1, o1[d]);
      o0[d] = mfma16(a, plo0, o0[d]);
      o1[d] = mfma16(a, plo1, o1[d]);
    }
    // column sums over this wave's 32 rows
    {
      float* dst = cs_part + (is_cache ? col0 : cap_cols + col0);
#pragma unroll
      for (int bk = 0; bk < 2; ++bk) {
        float4 c;
        c.x = row16_sum(s0[bk][0] + s1[bk][0]);
        c.y = row16_sum(s0[bk][1] + s1[bk][1]);
        c.z = row16_sum(s0[bk][2] + s1[bk][2]);
        c.w = row16_sum(s0[bk][3] + s1[bk][3]);
        if (lr == 0) *reinterpret_cast<float4*>(dst + bk * 16) = c;
      }
    }
    if (tile + 1 < ntiles) store_lds((tile + 1) & 1);      // the other stage: last read one barrier ago
    __syncthreads();
  }

  // ---- add the four column quarters of every row group through LDS ----
  float* xch = reinterpret_cast<float*>(pf_smem);           // [6 waves][2 blocks][DB*4][64 lanes]
  constexpr int XN = DB * 4;
  if (cq > 0) {
    float* dst = xch + (((cq - 1) * 2 + rg) * 2 * XN) * 64 + lane;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i) { dst[(d * 4 + i) * 64] = o0[d][i]; dst[(XN + d * 4 + i) * 64] = o1[d][i]; }
  }
  __syncthreads();
  if (cq > 0) return;
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const float* src = xch + ((c * 2 + rg) * 2 * XN) * 64 + lane;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i) { o0[d][i] += src[(d * 4 + i) * 64]; o1[d][i] += src[(XN + d * 4 + i) * 64]; }
  }
  auto finish = [&](int my_row, const f32x4_t (&oacc)[DB]) {
    if (my_row < L) {
      float* op = out + (((size_t)b * L + my_row) * p.H + h) * D;
#pragma unroll
      for (int d = 0; d < DB; ++d)
        *reinterpret_cast<float4*>(op + d * 16 + q4 * 4) = make_float4(oacc[d][0], oacc[d][1], oacc[d][2], oacc[d][3]);
    }
  };
  finish(my_row0, o0);
  finish(my_row1, o1);
}

// ---------------------------------------------------------------------------------------------
// replay
// ---------------------------------------------------------------------------------------------
constexpr int RP_THREADS = 512;

// Inclusive prefix sum of one int per thread over the workgroup (RP_THREADS threads).
__device__ inline int block_scan_inclusive(int v, int* sm_wave) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(v, off, 64);
    if (lane >= off) v += o;
  }
  __syncthreads();
  if (lane == 63) sm_wave[wave] = v;
  __syncthreads();
  int add = 0;
  for (int w = 0; w < wave; ++w) add += sm_wave[w];
  return v + add;
}

// Words of LDS the replay needs to keep a unit's order arrays, scores and flags on chip.
__host__ __device__ inline size_t replay_lds_words(int m, int cap, int r, int L) {
  return (size_t)4 * m + cap + L + (cap + L) + (L + 2) + (r > 0 ? r : 1);
}

// IN_LDS: the unit's E, PE, R, S, the chunk's S, the flags and the free list are copied into LDS up
// front, the replay runs on those copies (generic pointers, so the code below is the same either way) and
// the live parts are written back at the end.  Without it (budgets too large for LDS) it runs in place.
template <bool IN_LDS>
__global__ __launch_bounds__(RP_THREADS) void prefill_replay_kernel(Params p, int L, int32_t* __restrict__ retained,
                                                                    int32_t* __restrict__ n_retained,
                                                                    int32_t* __restrict__ evicted) {
  __shared__ int sm_wave[RP_THREADS / 64];
  __shared__ int sm_carry;
  extern __shared__ __attribute__((aligned(16))) int rp_smem[];
  const int unit = blockIdx.x, tid = threadIdx.x;
  int* meta = p.meta + (size_t)unit * META_STRIDE;
  float* Sg = p.S + (size_t)unit * p.cap;
  int* Eg = p.E + (size_t)unit * 2 * p.m;
  int* PEg = p.PE + (size_t)unit * 2 * p.m;
  int* Rg = p.R + (size_t)unit * max(p.n_recent, 1);
  float* snew_w = p.pf_snew + (size_t)unit * p.max_chunk;    // the chunk tokens' scores (moved into LDS below)
  int* flag_g = p.pf_flag + (size_t)unit * (p.cap + p.max_chunk);
  int32_t* evu = evicted ? evicted + (size_t)unit * L : nullptr;

  float* Su = Sg;
  int *Eu = Eg, *PEu = PEg, *Ru = Rg;
  int* flag = flag_g;              // [0,cap): slot freed; [cap, cap+L): chunk token dead -> later its destination slot
  int* free_list = p.pf_list + (size_t)unit * (p.cap + p.max_chunk);
  if constexpr (IN_LDS) {
    int* w = rp_smem;
    Eu = w; w += 2 * p.m;
    PEu = w; w += 2 * p.m;
    Su = reinterpret_cast<float*>(w); w += p.cap;
    float* sn = reinterpret_cast<float*>(w); w += L;
    flag = w; w += p.cap + L;
    free_list = w; w += L + 2;
    Ru = w;
    for (int i = tid; i < 2 * p.m; i += RP_THREADS) { Eu[i] = Eg[i]; PEu[i] = PEg[i]; }
    for (int i = tid; i < p.n_recent; i += RP_THREADS) Ru[i] = Rg[i];
    snew_w = sn;
  }

  const int n0 = meta[META_N], f0 = meta[META_FREE], j0 = meta[META_J], rhead0 = meta[META_RHEAD], t0 = meta[META_T];

  // ---- Algorithm 1, line 8 for the whole chunk: add the attend kernel's column-sum parts, in a fixed order ----
  {
    const int cap_cols = (p.cap + AT_COLS - 1) / AT_COLS * AT_COLS;
    const int cs_stride = cap_cols + (p.max_chunk + AT_COLS - 1) / AT_COLS * AT_COLS;
    const int n_parts = 2 * ((p.max_chunk + ROW_TILE - 1) / ROW_TILE);
    const int used = 2 * ((L + ROW_TILE - 1) / ROW_TILE);          // parts the attend kernel wrote
    const float* cp = p.pf_colpart + (size_t)unit * p.G * n_parts * cs_stride;
    // four columns per thread and step, so that all the parts' loads are in flight together
    for (int i4 = tid * 4; i4 < p.cap; i4 += RP_THREADS * 4) {
      float4 add = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int g = 0; g < p.G; ++g)
        for (int part = 0; part < used; ++part) {
          const float4 x = *reinterpret_cast<const float4*>(cp + ((size_t)g * n_parts + part) * cs_stride + i4);
          add.x += x.x; add.y += x.y; add.z += x.z; add.w += x.w;
        }
      const float a[4] = {add.x, add.y, add.z, add.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = i4 + e;
        if (i < p.cap) {
          float v = Sg[i];
          if (i <= n0 && i != f0) {                                  // the columns every row tile visited
            v += a[e];
            Sg[i] = v;
          }
          if constexpr (IN_LDS) Su[i] = v;
        }
      }
    }
    for (int i4 = tid * 4; i4 < L; i4 += RP_THREADS * 4) {
      // chunk columns of column tile i4 / 128 are visited by row tiles 2 * (i4 / 128) and up (causal)
      float4 add = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int g = 0; g < p.G; ++g)
        for (int part = 4 * (i4 / AT_COLS); part < used; ++part) {
          const float4 x = *reinterpret_cast<const float4*>(cp + ((size_t)g * n_parts + part) * cs_stride + cap_cols + i4);
          add.x += x.x; add.y += x.y; add.z += x.z; add.w += x.w;
        }
      const float a[4] = {add.x, add.y, add.z, add.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (i4 + e < L) snew_w[i4 + e] = a[e];
    }
    __syncthreads();
  }
  const float* snew = snew_w;
  const int cap = p.cap, c = p.budget, m = p.m, r = p.n_recent;
  const int F = min(L, c - n0);            // tokens that still fit without eviction (they take slots n0 ..)
  const int Lev = L - F;                   // tokens that each trigger one eviction
  const int t_end = t0 + L - 1;            // every count C is t_end - position + 1 once the chunk is in
  const int tev = t0 + F;                  // position of the first evicting token

  // ---- phase 0: flags, scores of the tokens that got slots while filling ----
  for (int i = tid; i < cap + L; i += RP_THREADS) flag[i] = 0;
  for (int i = tid; i < F; i += RP_THREADS) {
    Su[n0 + i] = snew[i];
    if constexpr (IN_LDS) Sg[n0 + i] = snew[i];
  }
  for (int i = tid; i < F; i += RP_THREADS) if (evu) evu[i] = -1;
  __syncthreads();

  int j_final = j0, rhead_final = rhead0, f_final = n0 + F, n_final = n0 + F;
  if (Lev > 0) {
    n_final = c;
    const int fstart = F > 0 ? c : f0;     // the one free slot when the evictions start
    auto score_of = [&](int id) -> float { return id < cap ? Su[id] : snew[id - cap]; };
    auto chunk_id = [&](int i) -> int { return i < F ? n0 + i : cap + i; };   // id of chunk token i

    // sweeps of idx over the tree region: eviction steps [e_a, e_b) share one sweep
    int e_a = 0;
    while (e_a < Lev) {
      const int j_a = (j0 + e_a) % m;
      const int e_b = min(Lev, e_a + (m - j_a));
      const int cnt = e_b - e_a;
      // (1) the tokens that enter the tree region at these steps
      for (int x = tid; x < cnt; x += RP_THREADS) {
        const int e = e_a + x;
        const int pos_nc = tev + e - r;    // r == 0: the new token itself
        int id;
        if (pos_nc >= t0) id = chunk_id(pos_nc - t0);
        else id = Ru[(rhead0 + e) % r];    // still the ring's entry from before the chunk (e < r here)
        Eu[m + j_a + x] = id;
        PEu[m + j_a + x] = pos_nc;
      }
      __syncthreads();
      // (2) all scopes of the sweep are disjoint pairs: decide them in parallel, then write
      for (int x0 = 0; x0 < cnt; x0 += RP_THREADS) {
        const int x = x0 + tid;
        int surv_id = 0, surv_pos = 0, lose_id = 0, lose_pos = 0;
        if (x < cnt) {
          const int j = j_a + x;
          const int idl = Eu[2 * j], idr = Eu[2 * j + 1];
          const int pl = PEu[2 * j], pr = PEu[2 * j + 1];
          const float bl = score_of(idl) / (float)(t_end - pl + 1);
          const float br = score_of(idr) / (float)(t_end - pr + 1);
          const bool drop_right = (p.flags & TREEKV_KEEP_LEFT) || (bl > br);
          surv_id = drop_right ? idl : idr; surv_pos = drop_right ? pl : pr;
          lose_id = drop_right ? idr : idl; lose_pos = drop_right ? pr : pl;
        }
        __syncthreads();
        if (x < cnt) {
          const int j = j_a + x;
          Eu[j] = surv_id; PEu[j] = surv_pos;
          flag[lose_id] = 1;               // a slot that is free now, or a chunk token that is gone
          if (evu) evu[F + e_a + x] = lose_pos;
        }
        __syncthreads();
      }
      e_a = e_b;
    }
    j_final = (j0 + Lev) % m;

    // ---- the recent window: the last r chunk tokens (or fewer) take over ring entries ----
    if (r > 0) {
      for (int x = tid; x < r; x += RP_THREADS) {
        // ring index (rhead0 + e) % r is written by steps e = x, x + r, ...; the last one below Lev stays
        if (x < Lev) {
          const int e_last = x + ((Lev - 1 - x) / r) * r;
          Ru[(rhead0 + x) % r] = chunk_id(F + e_last);
        }
      }
      rhead_final = (rhead0 + Lev) % r;
    }
    __syncthreads();

    // ---- match surviving slot-less chunk tokens with free slots ----
    if (tid == 0) flag[fstart] = 1;
    __syncthreads();
    // rank of every free slot among the free slots (ascending slot number)
    int carry = 0;
    for (int s0 = 0; s0 < cap; s0 += RP_THREADS) {
      const int s = s0 + tid;
      const int isf = s < cap ? flag[s] : 0;
      const int inc = block_scan_inclusive(isf, sm_wave) + carry;
      if (isf) free_list[inc - 1] = s;       // the free slots in ascending order
      if (tid == RP_THREADS - 1) sm_carry = inc;
      __syncthreads();
      carry = sm_carry;
      __syncthreads();
    }
    const int n_free = carry;
    // rank of every surviving slot-less chunk token (ascending chunk index)
    carry = 0;
    for (int i0 = F; i0 < L; i0 += RP_THREADS) {
      const int i = i0 + tid;
      const int alive = (i < L) ? (flag[cap + i] == 0) : 0;
      const int inc = block_scan_inclusive(alive, sm_wave) + carry;
      if (i < L) flag[cap + i] = alive ? free_list[inc - 1] : -1;   // now: its slot, or -1
      if (tid == RP_THREADS - 1) sm_carry = inc;
      __syncthreads();
      carry = sm_carry;
      __syncthreads();
    }
    const int n_alive = carry;                       // n_free == n_alive + 1: one slot stays free
    f_final = free_list[n_alive < n_free ? n_alive : n_free - 1];

    // ---- rewrite ids that still name chunk tokens, hand their scores to their slots ----
    for (int k = tid; k < m; k += RP_THREADS) {
      const int x = tree_index(k, j_final);
      const int id = Eu[x];
      if (id >= cap) Eu[x] = flag[id];
    }
    for (int x = tid; x < r; x += RP_THREADS) {
      const int id = Ru[x];
      if (id >= cap) Ru[x] = flag[id];
    }
    for (int i = F + tid; i < L; i += RP_THREADS) {
      const int slot = flag[cap + i];
      if (slot >= 0) Sg[slot] = snew[i];
    }
  }
  // tokens that arrived while filling sit in slots n0 + i unless the chunk also evicted them;
  // flag[cap + i] is now every chunk token's destination slot (or -1) for the scatter
  for (int i = tid; i < F; i += RP_THREADS) flag[cap + i] = flag[n0 + i] ? -1 : n0 + i;
  __syncthreads();
  if constexpr (IN_LDS) {          // write back what later kernels and later calls read
    for (int i = tid; i < L; i += RP_THREADS) flag_g[cap + i] = flag[cap + i];
    if (Lev > 0) {
      for (int i = tid; i < 2 * m; i += RP_THREADS) { Eg[i] = Eu[i]; PEg[i] = PEu[i]; }
      for (int i = tid; i < r; i += RP_THREADS) Rg[i] = Ru[i];
    }
  }

  // ---- retained positions, bookkeeping words ----
  int32_t* ret = retained + (size_t)unit * c;
  for (int i = tid; i < c; i += RP_THREADS) {
    int pv = -1;
    if (i < n_final) {
      pv = i;
      if (n_final == c) {
        const int k = i - p.n_sink;
        if (k >= 0 && k < m) pv = PEu[tree_index(k, j_final)];
        else if (k >= m) pv = t_end + 1 - r + (k - m);
      }
    }
    ret[i] = pv;
  }
  if (tid == 0) {
    meta[META_N] = n_final;
    meta[META_FREE] = f_final;
    meta[META_J] = j_final;
    meta[META_RHEAD] = rhead_final;
    meta[META_T] = t0 + L;
    if (n_retained) n_retained[unit] = n_final;
  }
}

// ---------------------------------------------------------------------------------------------
// scatter: chunk rows that survived go to their slots
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void prefill_scatter_kernel(Params p, const uint4* __restrict__ Kc,
                                                             const uint4* __restrict__ Vc, int L, int row_vec) {
  const int i = blockIdx.x, unit = blockIdx.y;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int slot = p.pf_flag[(size_t)unit * (p.cap + p.max_chunk) + p.cap + i];
  if (slot < 0) return;
  const size_t src = (((size_t)b * L + i) * p.Hkv + kvh) * row_vec;
  const size_t dst = ((size_t)unit * p.cap + slot) * row_vec;
  for (int e = threadIdx.x; e < row_vec; e += 64) {
    reinterpret_cast<uint4*>(p.K)[dst + e] = Kc[src + e];
    reinterpret_cast<uint4*>(p.V)[dst + e] = Vc[src + e];
  }
}

template <int D>
int launch_prefill_d(const Params& p, const void* Q, const void* K, const void* V, int L, float* out,
                     int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  const uint16_t* q = (const uint16_t*)Q;
  const uint16_t* k = (const uint16_t*)K;
  const uint16_t* v = (const uint16_t*)V;
  const int row_tiles = (L + ROW_TILE - 1) / ROW_TILE;
  auto attend = prefill_attend_kernel<D>;
  const size_t lds = AttendLds<D>::BYTES;
  if (lds > 48 * 1024 &&
      hipFuncSetAttribute((const void*)attend, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return TREEKV_EHIP;
  const int n_items = row_tiles * p.G * p.U;
  hipLaunchKernelGGL(attend, dim3((n_items + 7) / 8 * 8), dim3(AT_THREADS), lds, s, p, q, k, v, L, row_tiles, out);
  const size_t rp_lds = replay_lds_words(p.m, p.cap, p.n_recent, L) * sizeof(int);
  if (rp_lds <= 140 * 1024) {
    auto replay = prefill_replay_kernel<true>;
    if (rp_lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)replay, hipFuncAttributeMaxDynamicSharedMemorySize, (int)rp_lds) != hipSuccess)
      return TREEKV_EHIP;
    hipLaunchKernelGGL(replay, dim3(p.U), dim3(RP_THREADS), rp_lds, s, p, L, retained, n_retained, evicted);
  } else {
    hipLaunchKernelGGL(prefill_replay_kernel<false>, dim3(p.U), dim3(RP_THREADS), 0, s, p, L, retained, n_retained,
                       evicted);
  }
  hipLaunchKernelGGL(prefill_scatter_kernel, dim3(L, p.U), dim3(64), 0, s, p, (const uint4*)K, (const uint4*)V, L,
                     D * 2 / 16);
  return hipGetLastError() == hipSuccess ? TREEKV_OK : TREEKV_EHIP;
}

}  // namespace

int launch_prefill(const Params& p, const void* Q, const void* K, const void* V, int len, float* out,
                   int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  if (p.dtype != TREEKV_BF16) return TREEKV_EUNSUPPORTED;      // the MFMA path is bf16
  if (p.D == 128) return launch_prefill_d<128>(p, Q, K, V, len, out, retained, n_retained, evicted, s);
  if (p.D == 64) return launch_prefill_d<64>(p, Q, K, V, len, out, retained, n_retained, evicted, s);
  return TREEKV_EUNSUPPORTED;
}

}  // namespace tkv
