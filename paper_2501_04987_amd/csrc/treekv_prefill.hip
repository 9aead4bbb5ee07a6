// Chunked prefill of TreeKV for gfx950.
//
// A chunk of L tokens attends the cache as it was before the chunk plus the chunk's own tokens
// up to and including itself; every row's probabilities are added to the scores; the averaged
// scores are then frozen and Algorithm 1's append / compare / evict / advance (lines 4-5, 9-17)
// is replayed for the L tokens.  L = 1 gives the decode step.
//
// Four launches per chunk:
//   attend   grid row tiles x G x U (ids remapped so that a unit's row tiles share an XCD's L2).  Flash-style pass over all visible columns with MFMA:
//            S^T = K Q^T (16x16x32 bf16), online softmax in registers, O^T += V^T P^T with P
//            split into two bf16 halves (hi + lo) so that rounding P costs 2^-16, not 2^-9.
//            Writes O and the final row statistics (max, 1/sum).
//   colsum   grid (column tiles, U).  Recomputes S = Q K^T for one 64-column tile against every
//            row that sees it, normalises with the final row statistics and sums down the rows:
//            a workgroup owns its columns, so the sums need no atomics and have a fixed order.
//            Cache columns add to S in place (Algorithm 1, line 8), chunk columns get their S.
//   replay   grid U.  Algorithm 1's eviction for the chunk's tokens with frozen scores.  Inside one
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

constexpr int PF_THREADS = 256;
constexpr int ROW_TILE = 64;     // query rows per attend workgroup (16 per wave)
constexpr int COL_TILE = 64;     // columns per step
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

// Work split.  A workgroup owns 64 query rows of one head and walks over the visible columns in
// tiles of 128.  Its 8 waves are 2 row groups (32 rows = two 16-row MFMA blocks) x 4 column quarters
// (32 columns of every tile): each K / V^T operand read from LDS feeds the MFMAs of two row blocks,
// and two waves share a SIMD so that one's exp / convert work overlaps the other's MFMAs.  Every wave
// keeps its own online-softmax state per row block; the four quarters of a row group are merged through
// LDS at the end.  Threads 0-255 stage V (transposing), threads 256-511 stage K.
//
// Staged V^T layout.  Row d holds the tile's columns in the order the P^T operand uses them: inside
// quarter c, column j sits at position c*32 + ((j%16)/4)*8 + ((j%32)/16)*4 + j%4, so that the 8 k-slots of
// lane group q4 (columns c*32 + q4*4 + {0..3} and c*32 + 16 + q4*4 + {0..3}) are the 16 contiguous
// bytes of "pair" c*4 + q4.  Pairs are XOR-swizzled with (d/16)%8: the 16 lanes of an operand read share
// d/16, so reads stay conflict free, while the transposing 8-byte writes of 16 lanes (same columns, rows 8
// apart) spread over the banks.
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
  const int rg = wave & 1;                                 // row group: rows 32*rg .. +31 of the workgroup's 64
  const int cq = wave >> 1;                                // column quarter of every tile
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int h = kvh * p.G + g;
  const ChunkInfo ci = load_chunk_info(p.meta + (size_t)unit * META_STRIDE);

  const int row0 = row_tile * ROW_TILE + rg * 32;          // first chunk row of this wave
  const int my_row0 = row0 + lr, my_row1 = row0 + 16 + lr; // the query rows this lane's results belong to
  uint4 qa0[KS], qa1[KS];                                  // B operands: Q rows of the two row blocks
  {
    const uint16_t* q0p = Q + (((size_t)b * L + min(my_row0, L - 1)) * p.H + h) * D + q4 * 8;
    const uint16_t* q1p = Q + (((size_t)b * L + min(my_row1, L - 1)) * p.H + h) * D + q4 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qa0[ks] = *reinterpret_cast<const uint4*>(q0p + ks * 32);
      qa1[ks] = *reinterpret_cast<const uint4*>(q1p + ks * 32);
    }
  }

  const uint16_t* Ku = (const uint16_t*)p.K + (size_t)unit * p.cap * D;
  const uint16_t* Vu = (const uint16_t*)p.V + (size_t)unit * p.cap * D;
  const int chunk_row_stride = p.Hkv * D;
  const uint16_t* Kcu = Kc + ((size_t)b * L * p.Hkv + kvh) * D;
  const uint16_t* Vcu = Vc + ((size_t)b * L * p.Hkv + kvh) * D;

  const int cache_tiles = (ci.n + 1 + AT_COLS - 1) / AT_COLS;          // slots [0, n], the free one masked
  const int last_row = min(row_tile * ROW_TILE + ROW_TILE, L) - 1;     // last chunk row of the workgroup
  const int chunk_tiles = last_row / AT_COLS + 1;                      // causal: columns <= last_row
  const int ntiles = cache_tiles + chunk_tiles;

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
  const int cache_lim = p.cap - 1, chunk_lim = L - 1;                   // last row that exists
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

  float m0 = NEG_BIG, m1 = NEG_BIG;    // running row max of the raw logits over this wave's columns, per row block
  float l0 = 0.f, l1 = 0.f;
  f32x4_t o0[DB], o1[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) { o0[d] = f32x4_t{0.f, 0.f, 0.f, 0.f}; o1[d] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }
  const float sc = p.scale_log2e;
  const int n_cached = ci.n, fslot = ci.fslot;

  // softmax of one row block's 8 logits against its running state; returns the packed hi / lo P^T operands
  auto soft = [&](f32x4_t (&s)[2], float& m_run, float& l_part, f32x4_t (&oacc)[DB], bool need_mask, uint4& phi, uint4& plo) {
    float mx = m_run;
#pragma unroll
    for (int bk = 0; bk < 2; ++bk)
#pragma unroll
      for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[bk][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (__any(mx != m_run)) {                 // the running max moved for some row of the block: rescale
      const float corr = fast_exp2((m_run - mx) * sc);
      l_part *= corr;
#pragma unroll
      for (int d = 0; d < DB; ++d) oacc[d] *= corr;
      m_run = mx;
    }
    const float neg_ms = -mx * sc;
    unsigned hi[4], lo[4];                    // k-slots 0-3 = block 0, i = 0..3; k-slots 4-7 = block 1
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const float s0 = s[e2 >> 1][(e2 & 1) * 2], s1 = s[e2 >> 1][(e2 & 1) * 2 + 1];
      float p0 = fast_exp2(fmaf(s0, sc, neg_ms)), p1 = fast_exp2(fmaf(s1, sc, neg_ms));
      if (need_mask) {                        // a row with nothing visible yet has max == NEG_BIG: exp2(0) must not count
        p0 = s0 > 0.5f * NEG_BIG ? p0 : 0.f;
        p1 = s1 > 0.5f * NEG_BIG ? p1 : 0.f;
      }
      l_part += p0 + p1;
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
#pragma unroll
      for (int bk = 0; bk < 2; ++bk)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int col = col0 + cq * 32 + bk * 16 + q4 * 4 + i;
          const bool cvis = is_cache ? (col <= n_cached && col != fslot) : true;
          s0[bk][i] = (cvis && (is_cache || col <= my_row0)) ? s0[bk][i] : NEG_BIG;
          s1[bk][i] = (cvis && (is_cache || col <= my_row1)) ? s1[bk][i] : NEG_BIG;
        }
    }
    uint4 phi0, plo0, phi1, plo1;
    soft(s0, m0, l0, o0, need_mask, phi0, plo0);
    soft(s1, m1, l1, o1, need_mask, phi1, plo1);
    // O^T += V^T P^T : A = V^T[d][the quarter's 8 k-slot columns of this lane group], B = P^T (hi and lo parts)
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      const uint4 a = *reinterpret_cast<const uint4*>(v + va_row + ((va_pair ^ (d & 7)) * 16) + d * 16 * Lds::VSTRIDE * 2);
      o0[d] = mfma16(a, phi0, o0[d]);
      o1[d] = mfma16(a, phi1, o1[d]);
      o0[d] = mfma16(a, plo0, o0[d]);
      o1[d] = mfma16(a, plo1, o1[d]);
    }
    if (tile + 1 < ntiles) store_lds((tile + 1) & 1);      // the other stage: last read one barrier ago
    __syncthreads();
  }

  // ---- merge the four column quarters of every row group through LDS ----
  float* xch = reinterpret_cast<float*>(pf_smem);           // [6 waves][2 blocks][2 + DB*4][64 lanes]
  constexpr int XN = 2 + DB * 4;
  if (cq > 0) {
    float* dst = xch + (((cq - 1) * 2 + rg) * 2 * XN) * 64 + lane;
    dst[0] = m0; dst[64] = l0;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[(2 + d * 4 + i) * 64] = o0[d][i];
    dst += XN * 64;
    dst[0] = m1; dst[64] = l1;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[(2 + d * 4 + i) * 64] = o1[d][i];
  }
  __syncthreads();
  if (cq > 0) return;
  auto merge_in = [&](const float* src, float& m_run, float& l_part, f32x4_t (&oacc)[DB]) {
    const float mo = src[0], lo2 = src[64];
    const float mx = fmaxf(m_run, mo);
    const float ca = fast_exp2((m_run - mx) * sc), cb = fast_exp2((mo - mx) * sc);
    l_part = l_part * ca + lo2 * cb;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i) oacc[d][i] = oacc[d][i] * ca + src[(2 + d * 4 + i) * 64] * cb;
    m_run = mx;
  };
  for (int c = 0; c < 3; ++c) {
    const float* src = xch + ((c * 2 + rg) * 2 * XN) * 64 + lane;
    merge_in(src, m0, l0, o0);
    merge_in(src + XN * 64, m1, l1, o1);
  }
  auto finish = [&](int my_row, float m_run, float l_part, const f32x4_t (&oacc)[DB]) {
    float l_row = l_part + __shfl_xor(l_part, 16, 64);
    l_row += __shfl_xor(l_row, 32, 64);
    const float inv = 1.0f / l_row;
    if (my_row < L) {
      float* op = out + (((size_t)b * L + my_row) * p.H + h) * D;
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        float4 o = make_float4(oacc[d][0] * inv, oacc[d][1] * inv, oacc[d][2] * inv, oacc[d][3] * inv);
        *reinterpret_cast<float4*>(op + d * 16 + q4 * 4) = o;
      }
      if (q4 == 0) {
        float* rs = p.pf_rowstat + (((size_t)unit * p.G + g) * p.max_chunk + my_row) * 2;
        rs[0] = m_run * sc;                   // row max in the scaled log2 domain
        rs[1] = inv;
      }
    }
  };
  finish(my_row0, m0, l0, o0);
  finish(my_row1, m1, l1, o1);
}

// ---------------------------------------------------------------------------------------------
// colsum
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(PF_THREADS) void prefill_colsum_kernel(Params p, const uint16_t* __restrict__ Q,
                                                                    const uint16_t* __restrict__ Kc, int L) {
  constexpr int KS = D / 32;
  constexpr int WAVES = PF_THREADS / 64;
  constexpr int QSTRIDE = D + 8;                    // bf16 elements per staged Q row (padded: conflict-free b128 reads)
  constexpr int LPR = D / 8;                        // lanes that cover one Q row with 16-byte loads
  constexpr int QLOADS = 16 * LPR / 64;             // loads per lane for a 16-row tile (4 at d=128, 2 at d=64)
  __shared__ float sm_cs[WAVES][COL_TILE];
  __shared__ __attribute__((aligned(16))) uint16_t sm_q[WAVES][16 * QSTRIDE];   // one 16-row Q tile per wave

  const int unit = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, q4 = lane >> 4;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  const ChunkInfo ci = load_chunk_info(p.meta + (size_t)unit * META_STRIDE);

  const int max_cache_tiles = (p.cap + COL_TILE - 1) / COL_TILE;
  const bool is_cache = (int)blockIdx.x < max_cache_tiles;
  const int col0 = is_cache ? blockIdx.x * COL_TILE : ((int)blockIdx.x - max_cache_tiles) * COL_TILE;
  if (is_cache ? col0 > ci.n : col0 >= L) return;          // nothing visible in this tile (uniform)

  // the tile's K rows as B operands, held in registers for the whole kernel
  uint4 kb[4][KS];
  bool colvis[4];                                           // validity of this lane's column in each block
#pragma unroll
  for (int bk = 0; bk < 4; ++bk) {
    const int col = col0 + bk * 16 + lr;
    const uint16_t* ks = is_cache ? (const uint16_t*)p.K + ((size_t)unit * p.cap + min(col, p.cap - 1)) * D
                                  : Kc + (((size_t)b * L + min(col, L - 1)) * p.Hkv + kvh) * D;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) kb[bk][kk] = *reinterpret_cast<const uint4*>(ks + kk * 32 + q4 * 8);
    colvis[bk] = is_cache ? (col <= ci.n && col != ci.fslot) : (col < L);
  }

  float cs0 = 0.f, cs1 = 0.f, cs2 = 0.f, cs3 = 0.f;
  const int first_rt = is_cache ? 0 : col0 / 16;            // causal: rows below the tile's first column see none of it
  const int n_rt = (L + 15) / 16;
  const float sc = p.scale_log2e;
  const int Lm1 = L - 1;
  const size_t q_row_stride = (size_t)p.H * D;

  // One item = one 16-row tile of one query head against the 64 columns.  Items are dealt round robin
  // to the waves.  Q rows are 8 KB apart in the caller's [B, L, H, d] layout, so they are fetched as whole
  // rows (16 lanes per row), parked in a wave-private LDS tile and read back in MFMA operand order.
  const int q_lrow = lane / LPR, q_lpart = lane % LPR;      // this lane's row (of each group of 64/LPR rows) and piece
  uint16_t* myq = sm_q[wave];
  auto fetch = [&](uint4& iq0, uint4& iq1, uint4& iq2, uint4& iq3, float4& is01, float4& is23, int g, int rt) {
    const uint16_t* qp = Q + ((size_t)b * L) * q_row_stride + (size_t)(kvh * p.G + g) * D + q_lpart * 8;
    auto row = [&](int x) { return qp + (size_t)min(rt * 16 + q_lrow + x * (64 / LPR), Lm1) * q_row_stride; };
    iq0 = *reinterpret_cast<const uint4*>(row(0));
    iq1 = *reinterpret_cast<const uint4*>(row(1));
    if constexpr (QLOADS > 2) {
      iq2 = *reinterpret_cast<const uint4*>(row(2));
      iq3 = *reinterpret_cast<const uint4*>(row(3));
    }
    // results land on rows rt*16 + q4*4 + {0..3}: their (max, 1/sum) pairs are 32 contiguous bytes
    // (rows past L hold stale values; the array is padded and those rows are masked out below)
    const float* rs = p.pf_rowstat + (((size_t)unit * p.G + g) * p.max_chunk + rt * 16 + q4 * 4) * 2;
    is01 = *reinterpret_cast<const float4*>(rs);
    is23 = *reinterpret_cast<const float4*>(rs + 4);
  };
  auto compute = [&](const uint4& iq0, const uint4& iq1, const uint4& iq2, const uint4& iq3, const float4& is01,
                     const float4& is23, int rt) {
    // rows of the tile past L, or the causal diagonal
    const bool special = (rt * 16 + 15 > Lm1) || (!is_cache && col0 + COL_TILE - 1 > rt * 16);
    const float m0 = is01.x, i0 = is01.y, m1 = is01.z, i1 = is01.w;
    const float m2 = is23.x, i2 = is23.y, m3 = is23.z, i3 = is23.w;
    // rows -> LDS -> A operands (row lr, k = ks*32 + q4*8 ..)
    uint16_t* wq = myq + q_lrow * QSTRIDE + q_lpart * 8;
    *reinterpret_cast<uint4*>(wq) = iq0;
    *reinterpret_cast<uint4*>(wq + (64 / LPR) * QSTRIDE) = iq1;
    if constexpr (QLOADS > 2) {
      *reinterpret_cast<uint4*>(wq + 2 * (64 / LPR) * QSTRIDE) = iq2;
      *reinterpret_cast<uint4*>(wq + 3 * (64 / LPR) * QSTRIDE) = iq3;
    }
    __builtin_amdgcn_wave_barrier();
    const uint16_t* rq = myq + lr * QSTRIDE + q4 * 8;
    const uint4 a0 = *reinterpret_cast<const uint4*>(rq);
    const uint4 a1 = *reinterpret_cast<const uint4*>(rq + 32);
    uint4 a2 = a0, a3 = a1;
    if constexpr (KS > 2) {
      a2 = *reinterpret_cast<const uint4*>(rq + 64);
      a3 = *reinterpret_cast<const uint4*>(rq + 96);
    }
    __builtin_amdgcn_wave_barrier();
    auto block = [&](int bk, float& cs) {
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(a0, kb[bk][0], acc);
      acc = mfma16(a1, kb[bk][1], acc);
      if constexpr (KS > 2) {
        acc = mfma16(a2, kb[bk][2], acc);
        acc = mfma16(a3, kb[bk][3], acc);
      }
      float p0 = fast_exp2(fmaf(acc[0], sc, -m0)) * i0;
      float p1 = fast_exp2(fmaf(acc[1], sc, -m1)) * i1;
      float p2 = fast_exp2(fmaf(acc[2], sc, -m2)) * i2;
      float p3 = fast_exp2(fmaf(acc[3], sc, -m3)) * i3;
      if (special) {
        const int col = col0 + bk * 16 + lr, row = rt * 16 + q4 * 4;
        p0 = (row + 0 <= Lm1 && (is_cache || col <= row + 0)) ? p0 : 0.f;
        p1 = (row + 1 <= Lm1 && (is_cache || col <= row + 1)) ? p1 : 0.f;
        p2 = (row + 2 <= Lm1 && (is_cache || col <= row + 2)) ? p2 : 0.f;
        p3 = (row + 3 <= Lm1 && (is_cache || col <= row + 3)) ? p3 : 0.f;
      }
      cs += (p0 + p1) + (p2 + p3);
    };
    block(0, cs0); block(1, cs1); block(2, cs2); block(3, cs3);
  };
  const uint4 z4 = make_uint4(0, 0, 0, 0);
  const float4 zf = make_float4(0.f, 0.f, 0.f, 0.f);
  // One Q tile in flight per wave: with the K tile held in registers, a second buffered tile costs more in
  // occupancy than it hides in latency (measured).
  for (int g = 0; g < p.G; ++g) {
    uint4 aq0 = z4, aq1 = z4, aq2 = z4, aq3 = z4;
    float4 as01 = zf, as23 = zf;
    for (int rt = first_rt + wave; rt < n_rt; rt += WAVES) {
      fetch(aq0, aq1, aq2, aq3, as01, as23, g, rt);
      compute(aq0, aq1, aq2, aq3, as01, as23, rt);
    }
  }
  float cs[4] = {colvis[0] ? cs0 : 0.f, colvis[1] ? cs1 : 0.f, colvis[2] ? cs2 : 0.f, colvis[3] ? cs3 : 0.f};
#pragma unroll
  for (int bk = 0; bk < 4; ++bk) {
    cs[bk] += __shfl_xor(cs[bk], 16, 64);
    cs[bk] += __shfl_xor(cs[bk], 32, 64);
    if (q4 == 0) sm_cs[wave][bk * 16 + lr] = cs[bk];
  }
  __syncthreads();
  if (tid < COL_TILE) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) tot += sm_cs[w][tid];
    const int col = col0 + tid;
    if (is_cache) {
      if (col <= ci.n && col != ci.fslot) p.S[(size_t)unit * p.cap + col] += tot;
    } else if (col < L) {
      p.pf_snew[(size_t)unit * p.max_chunk + col] = tot;
    }
  }
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
  const float* snew_g = p.pf_snew + (size_t)unit * p.max_chunk;
  int* flag_g = p.pf_flag + (size_t)unit * (p.cap + p.max_chunk);
  int32_t* evu = evicted ? evicted + (size_t)unit * L : nullptr;

  float* Su = Sg;
  int *Eu = Eg, *PEu = PEg, *Ru = Rg;
  const float* snew = snew_g;
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
    for (int i = tid; i < p.cap; i += RP_THREADS) Su[i] = Sg[i];
    for (int i = tid; i < L; i += RP_THREADS) sn[i] = snew_g[i];
    for (int i = tid; i < p.n_recent; i += RP_THREADS) Ru[i] = Rg[i];
    snew = sn;
    __syncthreads();
  }

  const int n0 = meta[META_N], f0 = meta[META_FREE], j0 = meta[META_J], rhead0 = meta[META_RHEAD], t0 = meta[META_T];
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
  const int col_tiles = (p.cap + COL_TILE - 1) / COL_TILE + (L + COL_TILE - 1) / COL_TILE;
  hipLaunchKernelGGL((prefill_colsum_kernel<D>), dim3(col_tiles, p.U), dim3(PF_THREADS), 0, s, p, q, k, L);
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
