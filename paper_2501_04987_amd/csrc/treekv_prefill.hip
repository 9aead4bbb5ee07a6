// Chunked prefill of TreeKV for gfx950.
//
// A chunk of L tokens attends the cache as it was before the chunk plus the chunk's own tokens
// up to and including itself; every row's probabilities are added to the scores; the averaged
// scores are then frozen and Algorithm 1's append / compare / evict / advance
// is replayed for the L tokens.  L = 1 gives the decode step.
//
// Two launches per chunk:
//   attend   grid row tiles x G x U (ids remapped so that a unit's row tiles share an XCD's L2).  Two passes
//            over all visible columns with MFMA (16x16x32 bf16): the first finds the row statistics, the
//            second forms the final probabilities, O^T += V^T P^T with P split into two bf16 halves
//            (hi + lo) so that rounding P costs 2^-16, not 2^-9, and the probabilities' sums down the
//            workgroup's rows.  Writes O; the column sums go, as 64-bit fixed point, into one accumulator
//            per column of the unit with integer atomic adds (which commute exactly: whatever order the
//            workgroups arrive in, the sum is the same to the bit).
//   replay   grid U.  Adds the accumulated column sums to the scores (Algorithm 1's S update) and clears the
//            accumulators, then Algorithm 1's eviction for the chunk's tokens with frozen scores.  Inside one
//            sweep of idx over the tree region the scopes are disjoint pairs, so a sweep is one
//            parallel pass; sweeps run one after the other.  Then surviving chunk tokens are
//            matched with freed slots (ballot ranks), the order arrays are rewritten, the retained
//            positions emitted and the surviving chunk rows copied into their slots.
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
constexpr float COLSUM_FIX = 1099511627776.0f;      // 2^40: column sums cross kernels as 64-bit fixed point

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

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) short4_t lds_short4_t;

// LDS of the attend kernel: K and V tiles exactly as they lie in memory (row-major, 128 rows each),
// two stages of each; the 16-byte pieces of a row are XOR-swizzled (see the kernel).
template <int D>
struct AttendLds {
  static constexpr int TILE_ELEMS = AT_COLS * D;                 // bf16 elements of one staged tile
  static constexpr int COLBUF_FLOATS = 2 * 2 * AT_COLS;          // column sums on their way out: [2 tiles][2 row groups][128]
  static constexpr size_t BYTES = 4 * (size_t)TILE_ELEMS * sizeof(uint16_t) + COLBUF_FLOATS * sizeof(float);
};

template <int CTRL>
__device__ inline float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
  return v + __int_as_float(moved);
}
// Sum over the 16 lanes of a DPP row; every lane gets the total.
__device__ inline float row16_sum(float v) {
  v = dpp_add<0x128>(v);           // row_ror:8
  v = dpp_add<0x124>(v);           // row_ror:4
  v = dpp_add<0x122>(v);           // row_ror:2
  v = dpp_add<0x121>(v);           // row_ror:1
  return v;
}
// max of three.  This file is compiled with -fno-honor-nans: otherwise every fmaxf operand that comes out of
// an MFMA costs an extra instruction that quiets signalling NaNs, and the pair is not fused into v_max3_f32.
__device__ inline float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <bool B> struct BoolTag { static constexpr bool value = B; };

// s_waitcnt vmcnt(N) alone (the other counters not waited for), N < 16.  A statement the compiler moves no memory
// access across: LDS reads that follow it read what the awaited copies wrote.
template <int N>
__device__ inline void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// Asynchronous copy of 16 bytes per lane from global memory into LDS: lane i's bytes land at
// lds_base + 16 * i (lds_base: wave-uniform LDS byte address, taken from M0).  Written as assembly on
// purpose: issued through the compiler's builtin, every later LDS read is preceded by a wait for all
// outstanding copies (it cannot tell which LDS bytes they fill), which would undo the prefetching.
// Completion is tracked by vmcnt like any load; the callers wait explicitly (wait_vmcnt) before the
// barrier that publishes a tile.
__device__ inline void async_copy16(const void* src, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(src), "s"(lds_base) : "memory");   // M0 is reserved: the compiler keeps nothing in it across statements
}
// The same with the source given as a wave-uniform base and a per-lane byte offset.
__device__ inline void async_copy16_offset(const void* uniform_base, unsigned lane_offset, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_offset), "s"(uniform_base), "s"(lds_base) : "memory");
}
// A run of copies whose sources and LDS images are both contiguous, 1 KB apart: one M0 write, and the instruction
// offset (which is added to the global and to the LDS address alike) steps both sides.  One statement, so that
// nothing can come between the M0 write and its readers.
__device__ inline void async_copy16_run(const void* uniform_base, unsigned lds_base, unsigned off0, unsigned off1) {
  asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %0, %2\n\t"
               "global_load_lds_dwordx4 %1, %2 offset:1024"
               :: "v"(off0), "v"(off1), "s"(uniform_base), "s"(lds_base) : "memory");
}
__device__ inline void async_copy16_run(const void* uniform_base, unsigned lds_base, unsigned off0, unsigned off1,
                                        unsigned off2, unsigned off3) {
  asm volatile("s_mov_b32 m0, %5\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %0, %4\n\t"
               "global_load_lds_dwordx4 %1, %4 offset:1024\n\t"
               "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
               "global_load_lds_dwordx4 %3, %4 offset:3072"
               :: "v"(off0), "v"(off1), "v"(off2), "v"(off3), "s"(uniform_base), "s"(lds_base) : "memory");
}
__device__ inline unsigned lds_address(const void* shared_ptr) {
  return (unsigned)(uintptr_t)(lds_void_t*)shared_ptr;
}

// One workgroup owns 64 query rows of one head and passes over the visible columns twice, in tiles of 128.
//
// Staging.  Tiles go from global memory into LDS with asynchronous 16-byte loads (global_load_lds): no
// registers, no LDS store instructions, and the next tiles are in flight while the current one is used.
// One such instruction fills 1 KB of LDS in lane order, so a staged tile is row-major like the source; what
// a lane is free to choose is which 16-byte piece of its row it fetches, and that gives the swizzle: slot s
// of row r holds piece s ^ KSWZ(r) (K tiles) or s ^ VSWZ(r) (V tiles), chosen so that the operand reads
// below touch every LDS bank once.
//
// Sweep 1 finds every row's softmax statistics (max, sum).  Wave w takes the 16-column block w of every
// tile against all 64 rows (four 16-row MFMA blocks): S^T = K Q^T, K rows from LDS as A operands.  Each
// lane keeps a running (max, sum) for its own columns of its four rows; lanes and waves are merged once,
// at the end.  Four K stages, so tiles are requested three iterations before they are used.
//
// Sweep 2 recomputes the logits and, knowing the statistics, forms the normalised probabilities
// directly: p = exp2(s*scale - max - log2(sum)), no running maximum and nothing to rescale.  They feed
// O^T += V^T P^T and, summed down the rows, the per-column score increments (Algorithm 1's S update).
// The 8 waves are 2 row groups (32 rows = two 16-row MFMA blocks) x 4 column quarters (32 columns of
// every tile).  S^T comes out of the MFMA with a lane holding 8 columns of one row, which is the B
// operand layout of P^T, so P never leaves the registers; it is split into two bf16 halves (hi + lo) so that
// rounding P costs 2^-16, not 2^-9.  The A operand V^T[d][8 columns] is read from the row-major V tile with
// the transposing LDS read (ds_read_b64_tr_b16: 16 lanes fetch a 4 x 16 block and each gets one column).
// Both sweeps are software pipelined: the logits of tile t+1 are formed (matrix pipe) while the
// probabilities of tile t are worked out (vector ALU).  The four quarters of a row group add their O through
// LDS at the end.
//
// Column sums: a wave adds its two row blocks, reduces over the 16 lanes that hold the 16 rows and
// leaves the 32 sums of its columns in LDS.  During the next tile two of the waves add the two row groups
// and add the tile's 128 sums to the unit's accumulators (the atomics then have a whole iteration to
// complete before anything waits on the memory counter).  A workgroup touches the accumulators of the columns
// of the tiles it visits (masked entries add zero; cache columns past the last cached token are left alone).
//
// ROPE (positions re-assigned to cache ranks): queries and keys come, already turned to their ranks and split into
// two bf16 parts each, from the scratch prefill_turn_kernel fills (pf_qrot, pf_krot; the chunk's own keys lie behind
// the cache rows there), and a logit is k_hi.q_hi + k_lo.q_hi + k_hi.q_lo (what is left out, lo.lo, is 2^-18 of the
// product).  The staging memory then holds one tile pair (hi, lo) where the plain kernel holds two tiles: sweep 1
// requests one tile ahead instead of three, and sweep 2 has a second barrier per tile (the K pair is requested once
// every wave has formed its logits from it).  Everything after the logits is unchanged.
template <int D, bool ROPE>
__global__ __launch_bounds__(AT_THREADS) void prefill_attend_kernel(Params p, const uint16_t* __restrict__ Q,
                                                                    const uint16_t* __restrict__ Kc,
                                                                    const uint16_t* __restrict__ Vc, int L,
                                                                    int row_tiles, float* __restrict__ out) {
  using Lds = AttendLds<D>;
  constexpr int KS = D / 32;          // k-steps of the q.k contraction
  constexpr int DB = D / 16;          // 16-wide blocks of the head dimension
  constexpr int PARTS = D / 8;        // 16-byte pieces per row
  constexpr int ROWB = D * 2;         // bytes per row
  constexpr int RPC = 1024 / ROWB;    // rows per 1 KB async-load instruction (4 at d=128, 8 at d=64)
  constexpr int CPW = AT_COLS / RPC / 8;               // such instructions per wave and tile (4 or 2)
  static_assert(D == 64 || D == 128, "swizzles are written for head_dim 64 and 128");
  extern __shared__ __attribute__((aligned(1024))) uint16_t pf_smem[];
  uint16_t* sK = pf_smem;                               // sweep 2: [2][TILE_ELEMS]; sweep 1: all four stages
  uint16_t* sV = pf_smem + 2 * Lds::TILE_ELEMS;         // [2][TILE_ELEMS]
  float* sC = reinterpret_cast<float*>(pf_smem + 4 * Lds::TILE_ELEMS);   // [2][2][128]

  // swizzles of the 16-byte slots of tile row r
  auto kswz = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  auto vswz = [](int r) { return D == 128 ? ((r & 7) << 1) : (((r >> 1) & 3) << 1); };

  // Workgroups are dealt to the 8 XCDs round robin by their linear id, and each XCD has its own L2.
  // The row tiles of one unit read the same K and V, so give them ids that land on one XCD:
  // workgroup w works on item (w % 8) * (n/8) + w / 8 of the (row tile fastest) item list.
  const int n_items = row_tiles * p.G * p.U, per_xcd = (n_items + 7) / 8;
  const int item = ((int)blockIdx.x % 8) * per_xcd + (int)blockIdx.x / 8;
  if (item >= n_items) return;
  const int row_tile = item % row_tiles, g = (item / row_tiles) % p.G, unit = item / (row_tiles * p.G);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, q4 = lane >> 4;
  const int rg = wave & 1;                                 // sweep 2: rows 32*rg .. +31 of the workgroup's 64
  const int cq = wave >> 1;                                // sweep 2: column quarter of every tile
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int h = kvh * p.G + g;
  const ChunkInfo ci = load_chunk_info(p.meta + (size_t)unit * META_STRIDE);
  const int rbase = row_tile * ROW_TILE;                   // first chunk row of the workgroup

  // B operands: the Q rows of the four 16-row blocks (rows past the chunk repeat its last row)
  constexpr int QL = ROPE ? KS : 1;          // the second bf16 part of the queries exists only with ROPE
  uint4 qa[4][KS], qlo[4][QL];
  const uint16_t* Qsrc = ROPE ? p.pf_qrot : Q;
  const size_t q_part = (size_t)p.B * p.max_chunk * p.H * D;      // pf_qrot: [hi, lo][B][max_chunk][H][D]
  const int q_rows = ROPE ? p.max_chunk : L;
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    const uint16_t* qp = Qsrc + (((size_t)b * q_rows + min(rbase + rb * 16 + lr, L - 1)) * p.H + h) * D + q4 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qa[rb][ks] = *reinterpret_cast<const uint4*>(qp + ks * 32);
    if constexpr (ROPE) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qlo[rb][ks] = *reinterpret_cast<const uint4*>(qp + q_part + ks * 32);
    }
  }

  const size_t krot_rows = (size_t)p.cap + p.max_chunk;            // pf_krot: [U][hi, lo][cap + max_chunk][D]
  const uint16_t* Ku = ROPE ? p.pf_krot + (size_t)unit * 2 * krot_rows * D : (const uint16_t*)p.K + (size_t)unit * p.cap * D;
  const uint16_t* Vu = (const uint16_t*)p.V + (size_t)unit * p.cap * D;
  const int chunk_row_stride = p.Hkv * D;
  const int kchunk_row_stride = ROPE ? D : chunk_row_stride;
  const uint16_t* Kcu = ROPE ? Ku + (size_t)p.cap * D : Kc + ((size_t)b * L * p.Hkv + kvh) * D;
  const uint16_t* Vcu = Vc + ((size_t)b * L * p.Hkv + kvh) * D;
  const size_t klo_off = krot_rows * D;                            // from a key's hi part to its lo part (ROPE)

  // Cache columns are the n cached tokens' slots in slot order with the free slot left out: column j is slot
  // j + (j >= fslot).  (Walking slots [0, n] and masking the free one would cost a full cache of 2048 a 17th tile
  // for its one last slot.)
  const int cache_tiles = (ci.n + AT_COLS - 1) / AT_COLS;
  const int last_row = min(rbase + ROW_TILE, L) - 1;                   // last chunk row of the workgroup
  const int chunk_tiles = last_row / AT_COLS + 1;                      // causal: columns <= last_row
  const int ntiles = cache_tiles + chunk_tiles;
  const float sc = p.scale_log2e;
  const int last_cached = ci.n - 1, fslot = ci.fslot;                   // last visible cache column
  const int cache_lim = p.cap - 1, chunk_lim = L - 1;                   // last row that exists

  // ---- asynchronous tile loads: this wave's CPW instructions of 1 KB each ----
  // Instruction x of wave w fills LDS block c = w*CPW + x, i.e. tile rows c*RPC + a_lrow.  w*CPW*RPC is a
  // multiple of 16 rows, so the swizzle of a lane's row depends on x and a_lrow only.
  static_assert(CPW * RPC == 16, "a wave covers 16 rows of every tile");
  const int a_lrow = lane / PARTS, a_slot = lane % PARTS;
  auto issue_tile = [&](const uint16_t* cache_src, const uint16_t* chunk_src, int chunk_stride, int tile, uint16_t* stage,
                        auto swz) {
    const bool is_cache = tile < cache_tiles;
    const int col0 = is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS;
    const uint16_t* base = is_cache ? cache_src : chunk_src;
    const int rstride = is_cache ? D : chunk_stride;
    const int lim = is_cache ? cache_lim : chunk_lim;
    const int col_w = col0 + wave * 16;                   // first column of this wave's 16 (wave uniform)
    // cache columns at and after the free slot sit one row further on
    const int shift = (is_cache && col_w >= fslot) ? 1 : 0;
    const bool straddles = is_cache && col_w < fslot && fslot <= col_w + 15;
    const int row_w = col_w + shift;                      // first source row, unless the wave straddles the free slot
    if (row_w + 15 <= lim && is_cache && !straddles) {
      // Cache rows are contiguous, like their LDS image: one scalar base and one M0 for the run of requests;
      // the per-lane offsets differ only in the swizzled piece.
      const unsigned lane_row = (unsigned)(a_lrow * D) * 2;
      const uint16_t* sbase = base + (size_t)row_w * D;
      const unsigned m0 = __builtin_amdgcn_readfirstlane(lds_address(stage + wave * CPW * 512));
      auto voff = [&](int x) { return lane_row + ((a_slot ^ swz(x * RPC + a_lrow)) * 16); };
      if constexpr (CPW == 4) async_copy16_run(sbase, m0, voff(0), voff(1), voff(2), voff(3));
      else async_copy16_run(sbase, m0, voff(0), voff(1));
    } else if (row_w + 15 <= lim && !straddles) {
      // every row exists: a scalar base per instruction plus a per-lane byte offset
      const unsigned lane_row = (unsigned)(a_lrow * rstride) * 2;
#pragma unroll
      for (int x = 0; x < CPW; ++x) {
        const unsigned voff = lane_row + ((a_slot ^ swz(x * RPC + a_lrow)) * 16);
        const uint16_t* sbase = base + (size_t)(row_w + x * RPC) * rstride;
        async_copy16_offset(sbase, voff, __builtin_amdgcn_readfirstlane(lds_address(stage + (wave * CPW + x) * 512)));
      }
    } else {
      // rows past the last one repeat it (they are masked later; what they must not be is unreadable)
#pragma unroll
      for (int x = 0; x < CPW; ++x) {
        const int r = x * RPC + a_lrow;
        const int col = col_w + r;
        const int row = col + ((is_cache && col >= fslot) ? 1 : 0);
        const uint16_t* src = base + (size_t)min(row, lim) * rstride + (a_slot ^ swz(r)) * 8;
        async_copy16(src, __builtin_amdgcn_readfirstlane(lds_address(stage + (wave * CPW + x) * 512)));
      }
    }
  };

  // ------------------------------------------------------------------------------------------
  // sweep 1: row statistics
  // ------------------------------------------------------------------------------------------
  float neg_ml0, neg_ml1;              // -(max + log2(sum)) in the scaled log2 domain, rows of the two sweep-2 blocks
  {
    float m_run[4], l_run[4];          // this lane's columns of row rb*16 + lr: max of the scaled logits, sum of exp2
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) { m_run[rb] = NEG_BIG; l_run[rb] = 0.f; }
    // S^T of this wave's 16 columns of a staged tile against the 64 rows
    const int k1_row = wave * 16 + lr;
    const int k1_off = k1_row * D;
    const int k1_swz = kswz(k1_row);
    auto qk = [&](f32x4_t (&s)[4], int stage) {
      const uint16_t* kp = sK + stage * Lds::TILE_ELEMS + k1_off;
      uint4 k[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) k[ks] = *reinterpret_cast<const uint4*>(kp + ((ks * 4 + q4) ^ k1_swz) * 8);
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) s[rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) s[rb] = mfma16(k[ks], qa[rb][ks], s[rb]);
      if constexpr (ROPE) {          // stage holds the keys' hi parts, stage + 1 their lo parts
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) s[rb] = mfma16(k[ks], qlo[rb][ks], s[rb]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) k[ks] = *reinterpret_cast<const uint4*>(kp + Lds::TILE_ELEMS + ((ks * 4 + q4) ^ k1_swz) * 8);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) s[rb] = mfma16(k[ks], qa[rb][ks], s[rb]);
      }
    };
    // Masked logits become -inf: their exp2 is 0 against any finite running max, and a lane that has seen
    // nothing yet keeps its (finite) initial max, so no probability needs a guard.
    auto stats = [&](f32x4_t (&s)[4], int tile) {
      const bool is_cache = tile < cache_tiles;
      const int c0 = (is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS) + wave * 16;   // this wave's 16 columns
      // only tiles that touch the end of the cache, the free slot or the causal diagonal need a mask (wave uniform)
      const bool need_mask = is_cache ? (c0 + 15 > last_cached) : (c0 + 15 > rbase);
      if (need_mask) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
          const int lim = is_cache ? last_cached : rbase + rb * 16 + lr;   // last visible column of this lane's row
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int col = c0 + q4 * 4 + i;
            s[rb][i] = col <= lim ? s[rb][i] : -INFINITY;
          }
        }
      }
      // The reference m_run of a lane's sums only has to keep exp2 in range, so it is raised lazily: when some
      // lane of the wave meets a logit more than 16 (log2 units) above its reference.  After the first tiles that
      // is rare, and the common path has no rescaling and one exp2 per logit.
      float tmax[4];
      bool grow = false;
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        tmax[rb] = max3(s[rb][0], s[rb][1], fmaxf(s[rb][2], s[rb][3])) * sc;
        grow |= tmax[rb] - 16.0f > m_run[rb];
      }
      if (__any(grow)) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
          const float m_new = fmaxf(m_run[rb], tmax[rb]);     // scaled domain: exp2(0) is exactly 1 where nothing changes
          l_run[rb] *= fast_exp2(m_run[rb] - m_new);
          m_run[rb] = m_new;
        }
      }
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const float e0 = fast_exp2(fmaf(s[rb][0], sc, -m_run[rb])), e1 = fast_exp2(fmaf(s[rb][1], sc, -m_run[rb]));
        const float e2 = fast_exp2(fmaf(s[rb][2], sc, -m_run[rb])), e3 = fast_exp2(fmaf(s[rb][3], sc, -m_run[rb]));
        l_run[rb] += (e0 + e1) + (e2 + e3);
      }
    };
    // Iteration t: request tile t+3, form the logits of tile t+1 while the statistics of tile t are updated.
    // Stage (t+3)&3 held tile t-1, last read in iteration t-2.  In this sweep a wave reads exactly the 16 rows
    // of every tile that it requested itself, so the waves need no barrier between tiles: each runs on its own
    // count of outstanding requests.
    f32x4_t sa[4], sb[4];
    // ROPE: tile t sits in the stage pair (t & 1) * 2 (hi), + 1 (lo) and is requested two tiles ahead
    auto issue_k1 = [&](int t) {
      if constexpr (ROPE) {
        issue_tile(Ku, Kcu, kchunk_row_stride, t, sK + ((t & 1) * 2) * Lds::TILE_ELEMS, kswz);
        issue_tile(Ku + klo_off, Kcu + klo_off, kchunk_row_stride, t, sK + ((t & 1) * 2 + 1) * Lds::TILE_ELEMS, kswz);
      } else {
        issue_tile(Ku, Kcu, kchunk_row_stride, t, sK + (t & 3) * Lds::TILE_ELEMS, kswz);
      }
    };
    constexpr int AHEAD = ROPE ? 2 : 3;     // how many tiles ahead of the one being finished the requests run
#pragma unroll
    for (int t = 0; t < AHEAD; ++t)
      if (t < ntiles) issue_k1(t);
    wait_vmcnt<0>();
    __syncthreads();
    qk(sa, 0);
    auto step = [&](f32x4_t (&cur)[4], f32x4_t (&nxt)[4], int t) {
      const bool more = t + AHEAD < ntiles;
      if constexpr (ROPE) {
        // the pair of tile t+2 goes where tile t was (its logits were formed in iteration t-1) and is read in the
        // next iteration: everything must have landed by then
        if (more) issue_k1(t + 2);
        if (t + 1 < ntiles) qk(nxt, ((t + 1) & 1) * 2);
        stats(cur, t);
        wait_vmcnt<0>();
      } else {
        if (more) issue_k1(t + 3);
        if (t + 1 < ntiles) qk(nxt, (t + 1) & 3);
        stats(cur, t);
        // tile t+2 must have landed before the next iteration reads it; only this iteration's requests may stay out
        if (more) wait_vmcnt<CPW>(); else wait_vmcnt<0>();
      }
    };
    for (int t = 0; t < ntiles; t += 2) {
      step(sa, sb, t);
      if (t + 1 < ntiles) step(sb, sa, t + 1);
    }
    __syncthreads();                   // the statistics below reuse the staging memory other waves may still read
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
  uint4 qa0[KS], qa1[KS], ql0[QL], ql1[QL];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const uint4 a0 = qa[0][ks], a1 = qa[1][ks], a2 = qa[2][ks], a3 = qa[3][ks];   // values, not addresses, into the select
    qa0[ks] = rg ? a2 : a0;
    qa1[ks] = rg ? a3 : a1;
  }
  if constexpr (ROPE) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint4 a0 = qlo[0][ks], a1 = qlo[1][ks], a2 = qlo[2][ks], a3 = qlo[3][ks];
      ql0[ks] = rg ? a2 : a0;
      ql1[ks] = rg ? a3 : a1;
    }
  }

  // operand read offsets inside one stage (bf16 elements), tile independent
  // K: row cq*32 + bk*16 + lr, piece ks*4 + q4
  const int k2_off = (cq * 32 + lr) * D;                                 // + bk*16 rows
  const int k2_swz0 = kswz(cq * 32 + lr), k2_swz1 = kswz(cq * 32 + 16 + lr);
  // V: the lane hands the transposing read the address of 4 dims of one row: row cq*32 + hh*16 + q4*4 + lr/4,
  // dims db*16 + (lr%4)*4 .. +3, i.e. half (lr%4)%2 of piece db*2 + (lr%4)/2
  const int v_row0 = cq * 32 + q4 * 4 + (lr >> 2), v_row1 = v_row0 + 16;
  const int v_off0 = v_row0 * D + (lr & 1) * 4, v_off1 = v_row1 * D + (lr & 1) * 4;
  const int v_swz0 = vswz(v_row0) ^ ((lr >> 1) & 1), v_swz1 = vswz(v_row1) ^ ((lr >> 1) & 1);   // piece db*2 ^ this

  f32x4_t o0[DB], o1[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) { o0[d] = f32x4_t{0.f, 0.f, 0.f, 0.f}; o1[d] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }

  // the unit's column-sum accumulators: [cache columns rounded up to a tile | chunk columns]
  const int cap_cols = (p.cap + AT_COLS - 1) / AT_COLS * AT_COLS;
  const int cs_stride = cap_cols + (p.max_chunk + AT_COLS - 1) / AT_COLS * AT_COLS;
  unsigned long long* cs_acc = p.pf_colacc + (size_t)unit * cs_stride;
  float* cs_lds = sC + rg * AT_COLS + cq * 32 + q4 * 4;                  // + (tile & 1) * 2 * AT_COLS, + bk * 16
  // the waves of column quarter t & 3 pass tile t's sums on (during tile t+1): thread j of the pair owns column j
  auto drain = [&](int tile) {
    const bool is_cache = tile < cache_tiles;
    const int col0 = is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS;
    const float* src = sC + (tile & 1) * 2 * AT_COLS + (tid & 127);
    // Integer adds commute exactly, so the row tiles (and query heads) of a unit can meet in one accumulator per
    // column in any order and the result is still the same to the bit.  A tile's sum is below 64; 2^-40 resolves it
    // far finer than fp32 does.
    const long long fix = (long long)((src[0] + src[AT_COLS]) * COLSUM_FIX + 0.5f);
    const int col = col0 + (tid & 127);
    if (is_cache) {             // the accumulators are indexed by slot
      if (col <= last_cached) atomicAdd(cs_acc + col + (col >= fslot ? 1 : 0), (unsigned long long)fix);
    } else {
      atomicAdd(cs_acc + cap_cols + col, (unsigned long long)fix);
    }
  };

  // S^T blocks of a staged K tile: rows = columns cq*32 + bk*16 + q4*4 + i, column = the lane's query row of block 0 / 1
  auto qk2 = [&](f32x4_t (&s0)[2], f32x4_t (&s1)[2], int stage) {
    const uint16_t* kp = sK + stage * Lds::TILE_ELEMS + k2_off;
    uint4 ka[2][KS];
#pragma unroll
    for (int bk = 0; bk < 2; ++bk)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        ka[bk][ks] = *reinterpret_cast<const uint4*>(kp + bk * 16 * D + ((ks * 4 + q4) ^ (bk ? k2_swz1 : k2_swz0)) * 8);
#pragma unroll
    for (int bk = 0; bk < 2; ++bk) { s0[bk] = f32x4_t{0.f, 0.f, 0.f, 0.f}; s1[bk] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int bk = 0; bk < 2; ++bk) {
        s0[bk] = mfma16(ka[bk][ks], qa0[ks], s0[bk]);
        s1[bk] = mfma16(ka[bk][ks], qa1[ks], s1[bk]);
      }
    if constexpr (ROPE) {            // `stage` holds the keys' hi parts, the stage after it their lo parts
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int bk = 0; bk < 2; ++bk) {
          s0[bk] = mfma16(ka[bk][ks], ql0[ks], s0[bk]);
          s1[bk] = mfma16(ka[bk][ks], ql1[ks], s1[bk]);
        }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int bk = 0; bk < 2; ++bk) {
          const uint4 kl = *reinterpret_cast<const uint4*>(kp + Lds::TILE_ELEMS + bk * 16 * D +
                                                           ((ks * 4 + q4) ^ (bk ? k2_swz1 : k2_swz0)) * 8);
          s0[bk] = mfma16(kl, qa0[ks], s0[bk]);
          s1[bk] = mfma16(kl, qa1[ks], s1[bk]);
        }
    }
  };
  // bf16 pairs (-1, 0) and (0, -1).  Kept opaque in scalar registers: as immediates, the second has the bit
  // pattern of the fp32 inline constant -1.0, which a packed 16-bit operand does not read as these two halves.
  unsigned minus_one_lo = 0x0000BF80u, minus_one_hi = 0xBF800000u;
  asm volatile("" : "+s"(minus_one_lo), "+s"(minus_one_hi));
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
      // p - hi in one instruction each: a bf16 dot product against (-1, 0) / (0, -1) added to p
      const bf16x2_t hv = __builtin_bit_cast(bf16x2_t, hi[e2]);
      const float l0 = __builtin_amdgcn_fdot2_f32_bf16(hv, __builtin_bit_cast(bf16x2_t, minus_one_lo), p0, false);
      const float l1 = __builtin_amdgcn_fdot2_f32_bf16(hv, __builtin_bit_cast(bf16x2_t, minus_one_hi), p1, false);
      lo[e2] = pack_bf16(l0, l1);
    }
    phi = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    plo = make_uint4(lo[0], lo[1], lo[2], lo[3]);
  };
  // what follows the logits of tile t, in three pieces: mask + probabilities, O^T += V^T P^T, column sums
  auto mask_tile = [&](f32x4_t (&s0)[2], f32x4_t (&s1)[2], int tile) {
    const bool is_cache = tile < cache_tiles;
    const int col0 = is_cache ? tile * AT_COLS : (tile - cache_tiles) * AT_COLS;
    // only tiles that touch the end of the cache or the causal diagonal need a mask (wave uniform)
    const bool need_mask = is_cache ? (col0 + AT_COLS - 1 > last_cached) : (col0 + AT_COLS - 1 > row0);
    if (need_mask) {
      const int cbase = col0 + cq * 32 + q4 * 4;
      const int lim0 = is_cache ? last_cached : my_row0, lim1 = is_cache ? last_cached : my_row1;   // last visible column
#pragma unroll
      for (int bk = 0; bk < 2; ++bk)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int col = cbase + bk * 16 + i;
          s0[bk][i] = col <= lim0 ? s0[bk][i] : -INFINITY;   // exp2 gives exactly 0
          s1[bk][i] = col <= lim1 ? s1[bk][i] : -INFINITY;
        }
    }
  };
  // O^T += V^T P^T : A = V^T[d][the quarter's 8 k-slot columns of this lane group], B = P^T (hi and lo parts)
  auto pv = [&](int tile, const uint4& phi0, const uint4& plo0, const uint4& phi1, const uint4& plo1) {
    const uint16_t* vp = sV + (tile & 1) * Lds::TILE_ELEMS;
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      const short4_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(vp + v_off0 + ((d * 2) ^ v_swz0) * 8));
      const short4_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(vp + v_off1 + ((d * 2) ^ v_swz1) * 8));
      const uint2 a0 = __builtin_bit_cast(uint2, t0), a1 = __builtin_bit_cast(uint2, t1);
      const uint4 a = make_uint4(a0.x, a0.y, a1.x, a1.y);
      o0[d] = mfma16(a, phi0, o0[d]);
      o1[d] = mfma16(a, phi1, o1[d]);
      o0[d] = mfma16(a, plo0, o0[d]);
      o1[d] = mfma16(a, plo1, o1[d]);
    }
  };
  // column sums over this wave's 32 rows (s0 / s1 hold the probabilities by now)
  auto colsums = [&](const f32x4_t (&s0)[2], const f32x4_t (&s1)[2], int tile) {
    float* dst = cs_lds + (tile & 1) * 2 * AT_COLS;
#pragma unroll
    for (int bk = 0; bk < 2; ++bk) {
      float4 c;
      c.x = row16_sum(s0[bk][0] + s1[bk][0]);
      c.y = row16_sum(s0[bk][1] + s1[bk][1]);
      c.z = row16_sum(s0[bk][2] + s1[bk][2]);
      c.w = row16_sum(s0[bk][3] + s1[bk][3]);
      if (lr == 0) *reinterpret_cast<float4*>(dst + bk * 16) = c;
    }
  };

  f32x4_t sa0[2], sa1[2], sb0[2], sb1[2];
  if constexpr (!ROPE) {
  // Iteration t: request K of tile t+2 and V of tile t+1, form the logits of tile t+1, finish tile t.
  // K stage t&1 held tile t, whose logits were formed in iteration t-1; V stage (t+1)&1 held tile t-1.
  issue_tile(Ku, Kcu, kchunk_row_stride, 0, sK, kswz);
  issue_tile(Vu, Vcu, chunk_row_stride, 0, sV, vswz);
  if (ntiles > 1) issue_tile(Ku, Kcu, kchunk_row_stride, 1, sK + Lds::TILE_ELEMS, kswz);
  wait_vmcnt<0>();
  __syncthreads();
  qk2(sa0, sa1, 0);
  __syncthreads();                     // K stage 0 is requested again right below
  auto step2 = [&](f32x4_t (&c0)[2], f32x4_t (&c1)[2], f32x4_t (&n0)[2], f32x4_t (&n1)[2], int t, auto matrix_first) {
    if (t > 0 && cq == ((t - 1) & 3)) drain(t - 1);
    // Requests of this iteration: K of tile t+2 into K stage t&1, V of tile t+1 into V stage (t+1)&1.
    const bool more_k = t + 2 < ntiles, more_v = t + 1 < ntiles;
    uint16_t* k_stage = sK + (t & 1) * Lds::TILE_ELEMS;
    uint16_t* v_stage = sV + ((t + 1) & 1) * Lds::TILE_ELEMS;
    if (more_k) issue_tile(Ku, Kcu, kchunk_row_stride, t + 2, k_stage, kswz);
    if (more_v) issue_tile(Vu, Vcu, chunk_row_stride, t + 1, v_stage, vswz);
    // The two waves that share a SIMD take the four pieces in different orders, so that one is on the matrix pipe
    // while the other is on the vector ALU instead of both wanting the same unit at the same time:
    //   waves 0-3: logits(t+1)  probabilities(t)  PV(t)  column sums(t)
    //   waves 4-7: probabilities(t)  column sums(t)  logits(t+1)  PV(t)
    uint4 phi0, plo0, phi1, plo1;
    if constexpr (decltype(matrix_first)::value) {
      if (t + 1 < ntiles) qk2(n0, n1, (t + 1) & 1);
      mask_tile(c0, c1, t);
      soft(c0, neg_ml0, phi0, plo0);
      soft(c1, neg_ml1, phi1, plo1);
      pv(t, phi0, plo0, phi1, plo1);
      colsums(c0, c1, t);
    } else {
      mask_tile(c0, c1, t);
      soft(c0, neg_ml0, phi0, plo0);
      soft(c1, neg_ml1, phi1, plo1);
      colsums(c0, c1, t);
      if (t + 1 < ntiles) qk2(n0, n1, (t + 1) & 1);
      pv(t, phi0, plo0, phi1, plo1);
    }
    wait_vmcnt<0>();                   // this iteration's requests are the next one's operands
    __syncthreads();
  };
  if (wave < 4) {                      // (the choice is made outside the loop: inside, the two bodies would share registers badly)
    for (int t = 0; t < ntiles; t += 2) {
      step2(sa0, sa1, sb0, sb1, t, BoolTag<true>{});
      if (t + 1 < ntiles) step2(sb0, sb1, sa0, sa1, t + 1, BoolTag<true>{});
    }
  } else {
    for (int t = 0; t < ntiles; t += 2) {
      step2(sa0, sa1, sb0, sb1, t, BoolTag<false>{});
      if (t + 1 < ntiles) step2(sb0, sb1, sa0, sa1, t + 1, BoolTag<false>{});
    }
  }
  } else {
  // ROPE: one K pair (hi in K stage 0, lo in K stage 1) and two V stages.  Iteration t: with the pair of tile t+1
  // landed, form its logits; once every wave has done so, request the pair of tile t+2 into the same two stages and
  // finish tile t while it is on its way.  V of tile t+1 goes into V stage (t+1)&1, which held tile t-1.
  auto issue_k2 = [&](int t) {
    issue_tile(Ku, Kcu, kchunk_row_stride, t, sK, kswz);
    issue_tile(Ku + klo_off, Kcu + klo_off, kchunk_row_stride, t, sK + Lds::TILE_ELEMS, kswz);
  };
  issue_k2(0);
  issue_tile(Vu, Vcu, chunk_row_stride, 0, sV, vswz);
  wait_vmcnt<0>();
  __syncthreads();
  qk2(sa0, sa1, 0);
  __syncthreads();                     // the pair is requested again right below
  if (ntiles > 1) issue_k2(1);
  auto step2 = [&](f32x4_t (&c0)[2], f32x4_t (&c1)[2], f32x4_t (&n0)[2], f32x4_t (&n1)[2], int t) {
    wait_vmcnt<0>();                   // the pair of tile t+1 and V of tile t
    __syncthreads();                   // ... for every wave; and every wave is done with V of tile t-1 and tile t-1's sums
    if (t + 1 < ntiles) issue_tile(Vu, Vcu, chunk_row_stride, t + 1, sV + ((t + 1) & 1) * Lds::TILE_ELEMS, vswz);
    if (t > 0 && cq == ((t - 1) & 3)) drain(t - 1);
    if (t + 1 < ntiles) qk2(n0, n1, 0);
    __syncthreads();                   // every wave has read the pair
    if (t + 2 < ntiles) issue_k2(t + 2);
    uint4 phi0, plo0, phi1, plo1;
    mask_tile(c0, c1, t);
    soft(c0, neg_ml0, phi0, plo0);
    soft(c1, neg_ml1, phi1, plo1);
    pv(t, phi0, plo0, phi1, plo1);
    colsums(c0, c1, t);
  };
  for (int t = 0; t < ntiles; t += 2) {
    step2(sa0, sa1, sb0, sb1, t);
    if (t + 1 < ntiles) step2(sb0, sb1, sa0, sa1, t + 1);
  }
  __syncthreads();                     // the last tile's sums are in LDS
  }
  if (cq == ((ntiles - 1) & 3)) drain(ntiles - 1);     // the last tile's sums (its barrier has passed)

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
// attend for fp32 storage: plain vector arithmetic, one query row at a time
// ---------------------------------------------------------------------------------------------
// The matrix pipe takes bf16; with fp32 storage the results are held to 1e-5, so this instance does the same
// four steps (logits, row softmax, output, column sums) with fp32 multiply-adds.  A workgroup takes F32_ROWS
// consecutive rows of one head: per row, LPR lanes share a key (16 bytes each, summed by shuffles), the scaled
// logits and then the probabilities sit in LDS, the output is added up by (piece of the head dimension, stripe
// of keys) and the stripes are merged through LDS; every thread keeps the column sums of the columns it owns and
// adds them, as 2^-40 fixed point, to the unit's accumulators at the end (integer adds: order does not matter).
// Not a fast path: the one configuration with fp32 storage decodes.
constexpr int F32_THREADS = 256;
constexpr int F32_ROWS = 16;

// ROPE (positions re-assigned to cache ranks): queries and keys are read, already turned to their ranks, from the scratch
// prefill_turn_f32_kernel fills (the same memory the bf16 path keeps its two-part copies in).
template <int D, bool ROPE>
__global__ __launch_bounds__(F32_THREADS) void prefill_attend_f32_kernel(Params p, const float* __restrict__ Q,
                                                                         const float* __restrict__ Kc,
                                                                         const float* __restrict__ Vc, int L,
                                                                         float* __restrict__ out) {
  constexpr int LPR = D / 4;                       // lanes per row (16 bytes each)
  constexpr int KPP = F32_THREADS / LPR;           // keys per pass
  extern __shared__ float f32_smem[];
  const int unit = blockIdx.z, g = blockIdx.y, tid = threadIdx.x;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv, h = kvh * p.G + g;
  const ChunkInfo ci = load_chunk_info(p.meta + (size_t)unit * META_STRIDE);
  const int ncache = ci.n + 1;                     // slots [0, n], the free one masked
  const int r0 = blockIdx.x * F32_ROWS, r1 = min(L, r0 + F32_ROWS);
  const int ncols = ncache + r1;                   // columns any of this workgroup's rows can see
  float* sp = f32_smem;                            // [ncols] scaled logits, then probabilities
  float* sred = sp + ncols;                        // [F32_THREADS] reductions, then [KPP][D] output stripes
  float* sq = sred + (KPP * D > F32_THREADS ? KPP * D : F32_THREADS);    // [D] the query row
  const size_t krot_rows = (size_t)p.cap + p.max_chunk;          // turned keys: [U][cap + max_chunk][D] fp32
  const float* Ku = ROPE ? reinterpret_cast<const float*>(p.pf_krot) + (size_t)unit * krot_rows * D
                         : (const float*)p.K + (size_t)unit * p.cap * D;
  const float* Vu = (const float*)p.V + (size_t)unit * p.cap * D;
  const float* Kcu = ROPE ? Ku + (size_t)p.cap * D : Kc + ((size_t)b * L * p.Hkv + kvh) * D;
  const float* Vcu = Vc + ((size_t)b * L * p.Hkv + kvh) * D;
  const size_t cstride = (size_t)p.Hkv * D;
  const size_t kcstride = ROPE ? (size_t)D : cstride;
  const float* Qsrc = ROPE ? reinterpret_cast<const float*>(p.pf_qrot) : Q;   // turned queries: [B][max_chunk][H][D] fp32
  const int q_rows = ROPE ? p.max_chunk : L;
  const int grp = tid / LPR, piece = tid % LPR;
  constexpr int OWN = 40;                          // columns a thread owns: ncols <= OWN * F32_THREADS (checked by the host)
  float csum[OWN];
#pragma unroll
  for (int x = 0; x < OWN; ++x) csum[x] = 0.f;
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
    for (int w = 1; w < F32_THREADS / 64; ++w) r = take_max ? fmaxf(r, sred[w]) : r + sred[w];
    __syncthreads();
    return r;
  };
  for (int i = r0; i < r1; ++i) {
    const int nvis = ncache + i + 1;
    if (tid < D) sq[tid] = Qsrc[(((size_t)b * q_rows + i) * p.H + h) * D + tid];
    __syncthreads();
    const float4 qv = *reinterpret_cast<const float4*>(sq + piece * 4);
    // logits
    for (int j0 = 0; j0 < nvis; j0 += KPP) {
      const int j = j0 + grp;
      float acc = 0.f;
      if (j < nvis) {
        const float* row = j < ncache ? Ku + (size_t)j * D : Kcu + (size_t)(j - ncache) * kcstride;
        const float4 kv = *reinterpret_cast<const float4*>(row + piece * 4);
        acc = kv.x * qv.x;
        acc = fmaf(kv.y, qv.y, acc);
        acc = fmaf(kv.z, qv.z, acc);
        acc = fmaf(kv.w, qv.w, acc);
      }
#pragma unroll
      for (int off = LPR / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
      if (j < nvis && piece == 0) sp[j] = (j == ci.fslot && j < ncache) ? -INFINITY : acc * p.scale_log2e;
    }
    __syncthreads();
    // row softmax
    float mx = NEG_BIG;
    for (int j = tid; j < nvis; j += F32_THREADS) mx = fmaxf(mx, sp[j]);
    mx = block_reduce(mx, true);
    float sum = 0.f;
    for (int j = tid; j < nvis; j += F32_THREADS) {
      const float e = fast_exp2(sp[j] - mx);
      sp[j] = e;
      sum += e;
    }
    sum = block_reduce(sum, false);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int x = 0; x < OWN; ++x) {
      const int j = tid + x * F32_THREADS;
      if (j < nvis) {
        const float pj = sp[j] * inv;
        sp[j] = pj;
        csum[x] += pj;
      }
    }
    __syncthreads();
    // output: this thread's 4 dimensions over its stripe of keys
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = grp; j < nvis; j += KPP) {
      const float* row = j < ncache ? Vu + (size_t)j * D : Vcu + (size_t)(j - ncache) * cstride;
      const float4 vv = *reinterpret_cast<const float4*>(row + piece * 4);
      const float pj = sp[j];
      o.x = fmaf(pj, vv.x, o.x); o.y = fmaf(pj, vv.y, o.y); o.z = fmaf(pj, vv.z, o.z); o.w = fmaf(pj, vv.w, o.w);
    }
    *reinterpret_cast<float4*>(sred + grp * D + piece * 4) = o;
    __syncthreads();
    if (tid < D) {
      float a = 0.f;
#pragma unroll
      for (int w = 0; w < KPP; ++w) a += sred[w * D + tid];
      out[(((size_t)b * L + i) * p.H + h) * D + tid] = a;
    }
    __syncthreads();
  }
  // the column sums of this workgroup's rows
  const int cap_cols = (p.cap + AT_COLS - 1) / AT_COLS * AT_COLS;
  const int cs_stride = cap_cols + (p.max_chunk + AT_COLS - 1) / AT_COLS * AT_COLS;
  unsigned long long* cs_acc = p.pf_colacc + (size_t)unit * cs_stride;
#pragma unroll
  for (int x = 0; x < OWN; ++x) {
    const int j = tid + x * F32_THREADS;
    if (j < ncols && csum[x] != 0.f) {
      const long long fix = (long long)(csum[x] * COLSUM_FIX + 0.5f);
      atomicAdd(cs_acc + (j < ncache ? j : cap_cols + (j - ncache)), (unsigned long long)fix);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// positions re-assigned to cache ranks: the chunk's queries and every key it attends, turned and split
// ---------------------------------------------------------------------------------------------
// A chunk is scored before anything of it is evicted, so the n0 cached tokens are at the positions 0 .. n0-1 of
// their logical order and chunk token i (and its query) at n0 + i.  The rotary encoding turns plane (2i, 2i+1) of
// a row by position * base^(-2i/d); here that is done once per call, in fp32 with the (cos, sin) table, and the
// result is left as two bf16 parts (hi = the rounded value, lo = the rounded remainder) for the matrix pipe.
// One thread turns 8 dimensions (4 planes, one 16-byte piece) of one row.  Rows of a unit: n0 cached keys (by
// logical index, written at their slot), L chunk keys (written behind the cache rows), L * G queries.
template <int D>
__global__ __launch_bounds__(256) void prefill_turn_kernel(Params p, const uint16_t* __restrict__ Q,
                                                           const uint16_t* __restrict__ Kc, int L) {
  constexpr int PARTS = D / 8;
  const int unit = blockIdx.y, kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int n0 = meta[META_N], j = meta[META_J], rhead = meta[META_RHEAD];
  const int rows = n0 + L + L * p.G;
  const int x = blockIdx.x * 256 + threadIdx.x;
  const int row = x / PARTS, part = x % PARTS;
  if (row >= rows) return;
  const size_t krot_rows = (size_t)p.cap + p.max_chunk;
  uint16_t* khi = p.pf_krot + (size_t)unit * 2 * krot_rows * D;
  const uint16_t* src;
  uint16_t* dst;
  size_t lo_off;
  int pos;
  if (row < n0) {                                   // cached key at logical index `row`
    const int* Eu = p.E + (size_t)unit * 2 * p.m;
    const int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
    const int slot = n0 < p.budget ? row : logical_to_slot(p, Eu, Ru, rhead, j, row);
    src = (const uint16_t*)p.K + ((size_t)unit * p.cap + slot) * D;
    dst = khi + (size_t)slot * D;
    lo_off = krot_rows * D;
    pos = row;
  } else if (row < n0 + L) {                        // the chunk's own key i
    const int i = row - n0;
    src = Kc + (((size_t)b * L + i) * p.Hkv + kvh) * D;
    dst = khi + ((size_t)p.cap + i) * D;
    lo_off = krot_rows * D;
    pos = row;
  } else {                                          // query i of head g of the group
    const int i = (row - n0 - L) / p.G, g = (row - n0 - L) % p.G;
    const int h = kvh * p.G + g;
    src = Q + (((size_t)b * L + i) * p.H + h) * D;
    dst = p.pf_qrot + (((size_t)b * p.max_chunk + i) * p.H + h) * D;
    lo_off = (size_t)p.B * p.max_chunk * p.H * D;
    pos = n0 + i;
  }
  const uint4 raw = *reinterpret_cast<const uint4*>(src + part * 8);
  const float4* cs = reinterpret_cast<const float4*>(p.rope_tab + (size_t)pos * (D / 2) + part * 4);
  const float4 c01 = cs[0], c23 = cs[1];            // (cos, sin) of planes 4 part .. 4 part + 3
  const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
  const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
  unsigned hi[4], lo[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float x0 = __uint_as_float(w[e] << 16), x1 = __uint_as_float(w[e] & 0xffff0000u);
    const float y0 = x0 * co[e] - x1 * si[e], y1 = x0 * si[e] + x1 * co[e];
    hi[e] = pack_bf16(y0, y1);
    lo[e] = pack_bf16(y0 - __uint_as_float(hi[e] << 16), y1 - __uint_as_float(hi[e] & 0xffff0000u));
  }
  *reinterpret_cast<uint4*>(dst + part * 8) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  *reinterpret_cast<uint4*>(dst + lo_off + part * 8) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// ---------------------------------------------------------------------------------------------
// replay (and the copy of the surviving chunk rows into their slots)
// ---------------------------------------------------------------------------------------------
constexpr int RP_THREADS = 1024;
constexpr int RP_WAVES = RP_THREADS / 64;

// Rank of this thread's flag among the set flags of the threads before it, and the number of set flags in the
// workgroup: one ballot per wave, the waves' counts through LDS.
__device__ inline int block_rank(bool flag, int* sm_wave, int& total) {
  const unsigned long long b = __ballot(flag);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int within = __popcll(b & ((1ull << lane) - 1ull));
  if (lane == 0) sm_wave[wave] = __popcll(b);
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < RP_WAVES; ++w) {
    const int c = sm_wave[w];
    before += w < wave ? c : 0;
    tot += c;
  }
  __syncthreads();                 // sm_wave is free again
  total = tot;
  return before + within;
}

// Words of LDS the replay needs to keep a unit's order arrays, scores, the chunk's scores, flags and lists on chip.
__host__ __device__ inline size_t replay_lds_words(int m, int cap, int r, int L) {
  return (size_t)4 * m + cap + 4 * (size_t)L + 4 + (r > 0 ? r : 1);
}

// One workgroup per unit.  IN_LDS: the unit's E, PE, R, S and the chunk's scores, flags and lists live in LDS (generic
// pointers, so the code below is the same either way) and the live parts are written back at the end.  Without it
// (budgets too large for LDS) the replay runs in place, with its lists in the workspace's prefill scratch.
//
// Tokens that lose a scope: a cached token frees its slot, a chunk token that has no slot yet just disappears.  The
// k-th slot freed (in the order of the eviction steps, the slot that was free before the chunk first) goes to the
// k-th surviving chunk token without a slot (in chunk order); the one slot left over is the next call's free slot.
template <bool IN_LDS>
__global__ __launch_bounds__(RP_THREADS) void prefill_replay_kernel(Params p, int L, const uint4* __restrict__ Kc,
                                                                    const uint4* __restrict__ Vc, int row_vec,
                                                                    int32_t* __restrict__ retained,
                                                                    int32_t* __restrict__ n_retained,
                                                                    int32_t* __restrict__ evicted) {
  __shared__ int sm_wave[RP_WAVES];
  extern __shared__ __attribute__((aligned(16))) int rp_smem[];
  const int unit = blockIdx.x, tid = threadIdx.x;
  int* meta = p.meta + (size_t)unit * META_STRIDE;
  float* Sg = p.S + (size_t)unit * p.cap;
  int* Eg = p.E + (size_t)unit * 2 * p.m;
  int* PEg = p.PE + (size_t)unit * 2 * p.m;
  int* Rg = p.R + (size_t)unit * max(p.n_recent, 1);
  int32_t* evu = evicted ? evicted + (size_t)unit * L : nullptr;
  const int cap = p.cap, c = p.budget, m = p.m, r = p.n_recent;

  float* Su = Sg;
  int *Eu = Eg, *PEu = PEg, *Ru = Rg;
  float* snew = p.pf_snew + (size_t)unit * p.max_chunk;                  // [L] the chunk tokens' scores
  int* dest = p.pf_flag + (size_t)unit * (cap + p.max_chunk) + cap;     // [L] 1: the token lost a scope; later: its slot or -1
  int* loser = p.pf_list + (size_t)unit * (cap + p.max_chunk);          // [L] slot freed at eviction step e, or -1
  int* free_list = loser + L;                                           // [L + 1] freed slots in the order they are handed out
  if constexpr (IN_LDS) {
    int* w = rp_smem;
    Eu = w; w += 2 * m;
    PEu = w; w += 2 * m;
    Su = reinterpret_cast<float*>(w); w += cap;
    snew = reinterpret_cast<float*>(w); w += L;
    dest = w; w += L;
    loser = w; w += L;
    free_list = w; w += L + 1;
    Ru = w;
  }

  // Everything the kernel reads from global memory is requested here in one go (what a unit's replay costs is
  // memory round trips: its data was last touched a whole chunk ago): the bookkeeping words, the old scores and
  // the chunk's column sums of the first PRE * 1024 columns, and, for the LDS variant, the order arrays.
  const int cap_cols = (cap + AT_COLS - 1) / AT_COLS * AT_COLS;
  const int cs_stride = cap_cols + (p.max_chunk + AT_COLS - 1) / AT_COLS * AT_COLS;
  unsigned long long* acc = p.pf_colacc + (size_t)unit * cs_stride;
  constexpr int PRE = 3;
  const int n0 = meta[META_N], f0 = meta[META_FREE], j0 = meta[META_J], rhead0 = meta[META_RHEAD], t0 = meta[META_T];
  float s_pre[PRE];
  unsigned long long a_pre[PRE], n_pre[PRE];
#pragma unroll
  for (int u = 0; u < PRE; ++u) {
    const int x = u * RP_THREADS + tid;
    s_pre[u] = Sg[min(x, cap - 1)];
    a_pre[u] = acc[min(x, cap - 1)];
    n_pre[u] = acc[cap_cols + min(x, L - 1)];
  }
  if constexpr (IN_LDS) {
    // only the live entries: after j0 evictions of the sweep in progress the region reads E[0, j0) and E[2 j0, m + j0)
    for (int i0 = 0; i0 < m; i0 += 4 * RP_THREADS) {
      int e[4], pe[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { const int x = tree_index(min(i0 + u * RP_THREADS + tid, m - 1), j0); e[u] = Eg[x]; pe[u] = PEg[x]; }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int k = i0 + u * RP_THREADS + tid;
        if (k < m) { Eu[tree_index(k, j0)] = e[u]; PEu[tree_index(k, j0)] = pe[u]; }
      }
    }
    for (int i = tid; i < r; i += RP_THREADS) Ru[i] = Rg[i];
  }

  // ---- Algorithm 1's S update for the whole chunk: add the column sums the attend kernel left in the accumulators ----
  {
    // every accumulator that is read is also cleared for the next chunk (the others only ever received zeros)
    auto cache_col = [&](int x, float v, unsigned long long a) {
      if (x <= n0 && x != f0) {                                      // the columns every row tile visited
        v += (float)(long long)a * (1.0f / COLSUM_FIX);
        Sg[x] = v;
        acc[x] = 0;
      }
      if constexpr (IN_LDS) Su[x] = v;
    };
    auto chunk_col = [&](int x, unsigned long long a) {
      snew[x] = (float)(long long)a * (1.0f / COLSUM_FIX);
      acc[cap_cols + x] = 0;
    };
#pragma unroll
    for (int u = 0; u < PRE; ++u) {
      const int x = u * RP_THREADS + tid;
      if (x < cap) cache_col(x, s_pre[u], a_pre[u]);
      if (x < L) chunk_col(x, n_pre[u]);
    }
    for (int x = PRE * RP_THREADS + tid; x < cap; x += RP_THREADS) cache_col(x, Sg[x], acc[x]);
    for (int x = PRE * RP_THREADS + tid; x < L; x += RP_THREADS) chunk_col(x, acc[cap_cols + x]);
  }
  const int F = min(L, c - n0);            // tokens that still fit without eviction (they take slots n0 ..)
  const int Lev = L - F;                   // tokens that each trigger one eviction
  const int t_end = t0 + L - 1;            // every count C is t_end - position + 1 once the chunk is in
  const int tev = t0 + F;                  // position of the first evicting token
  for (int i = tid; i < L; i += RP_THREADS) { dest[i] = 0; loser[i] = -1; }
  __syncthreads();

  // ---- tokens that got slots while filling ----
  for (int i = tid; i < F; i += RP_THREADS) {
    Su[n0 + i] = snew[i];
    if constexpr (IN_LDS) Sg[n0 + i] = snew[i];
    if (evu) evu[i] = -1;
  }
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
          const bool averaged = !(p.flags & TREEKV_SCORE_ACCUMULATED);
          const float bl = averaged ? score_of(idl) / (float)(t_end - pl + 1) : score_of(idl);
          const float br = averaged ? score_of(idr) / (float)(t_end - pr + 1) : score_of(idr);
          const bool drop_right = (p.flags & TREEKV_KEEP_LEFT) || (bl > br);
          surv_id = drop_right ? idl : idr; surv_pos = drop_right ? pl : pr;
          lose_id = drop_right ? idr : idl; lose_pos = drop_right ? pr : pl;
        }
        __syncthreads();
        if (x < cnt) {
          const int j = j_a + x;
          Eu[j] = surv_id; PEu[j] = surv_pos;
          if (lose_id >= cap) dest[lose_id - cap] = 1;                       // a chunk token without a slot is gone
          else {
            loser[e_a + x] = lose_id;                                        // a slot that is free now
            if (lose_id >= n0 && lose_id < n0 + F) dest[lose_id - n0] = 1;   // ... which a token of this chunk had taken
          }
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

    // ---- freed slots in the order they are handed out: the slot free before the chunk, then by eviction step ----
    if (tid == 0) free_list[0] = fstart;
    int n_free = 1;
    for (int e0 = 0; e0 < Lev; e0 += RP_THREADS) {
      const int e = e0 + tid;
      const int slot = e < Lev ? loser[e] : -1;
      int total;
      const int rank = block_rank(slot >= 0, sm_wave, total);
      if (slot >= 0) free_list[n_free + rank] = slot;
      n_free += total;
    }
    __syncthreads();
    // ---- surviving chunk tokens without a slot take them in chunk order ----
    int n_alive = 0;
    for (int i0 = F; i0 < L; i0 += RP_THREADS) {
      const int i = i0 + tid;
      const bool alive = i < L && dest[i] == 0;
      int total;
      const int rank = block_rank(alive, sm_wave, total);
      if (i < L) dest[i] = alive ? free_list[n_alive + rank] : -1;
      n_alive += total;
    }
    f_final = free_list[n_alive < n_free ? n_alive : n_free - 1];      // n_free == n_alive + 1: one slot stays free
    __syncthreads();

    // ---- rewrite ids that still name chunk tokens, hand their scores to their slots ----
    for (int k = tid; k < m; k += RP_THREADS) {
      const int x = tree_index(k, j_final);
      const int id = Eu[x];
      if (id >= cap) Eu[x] = dest[id - cap];
    }
    for (int x = tid; x < r; x += RP_THREADS) {
      const int id = Ru[x];
      if (id >= cap) Ru[x] = dest[id - cap];
    }
    for (int i = F + tid; i < L; i += RP_THREADS) {
      const int slot = dest[i];
      if (slot >= 0) Sg[slot] = snew[i];
    }
  }
  // tokens that arrived while filling sit in slots n0 + i unless the chunk also evicted them
  for (int i = tid; i < F; i += RP_THREADS) dest[i] = dest[i] ? -1 : n0 + i;
  __syncthreads();
  if constexpr (IN_LDS) {          // write back what later calls read: the live entries
    if (Lev > 0) {
      for (int k = tid; k < m; k += RP_THREADS) { const int x = tree_index(k, j_final); Eg[x] = Eu[x]; PEg[x] = PEu[x]; }
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

  if constexpr (IN_LDS) {
    int* dest_g = p.pf_flag + (size_t)unit * (cap + p.max_chunk) + cap;
    for (int i = tid; i < L; i += RP_THREADS) dest_g[i] = dest[i];
  }
}

// ---------------------------------------------------------------------------------------------
// scatter: chunk rows that survived go to their slots
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_scatter_kernel(Params p, const uint4* __restrict__ Kc,
                                                              const uint4* __restrict__ Vc, int L, int row_vec) {
  // row_vec lanes (16-byte pieces of a row: 16 at d=128, 8 at d=64) per token, 256 / row_vec tokens per workgroup
  const int per_wg = 256 / row_vec;
  const int i = blockIdx.x * per_wg + threadIdx.x / row_vec, e = threadIdx.x % row_vec, unit = blockIdx.y;
  if (i >= L) return;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int slot = p.pf_flag[(size_t)unit * (p.cap + p.max_chunk) + p.cap + i];
  if (slot < 0) return;
  const size_t src = (((size_t)b * L + i) * p.Hkv + kvh) * row_vec + e;
  const size_t dst = ((size_t)unit * p.cap + slot) * row_vec + e;
  reinterpret_cast<uint4*>(p.K)[dst] = Kc[src];
  reinterpret_cast<uint4*>(p.V)[dst] = Vc[src];
}

// What follows the attend kernel, whatever the storage type: replay, then the surviving rows' copy.
int launch_replay(const Params& p, const void* K, const void* V, int L, int32_t* retained, int32_t* n_retained,
                  int32_t* evicted, hipStream_t s) {
  const size_t rp_lds = replay_lds_words(p.m, p.cap, p.n_recent, L) * sizeof(int);
  const int row_vec = p.D * (p.dtype == TREEKV_BF16 ? 2 : 4) / 16;
  if (rp_lds <= 140 * 1024) {
    auto replay = prefill_replay_kernel<true>;
    if (rp_lds > 48 * 1024 &&
        hip_failed(hipFuncSetAttribute((const void*)replay, hipFuncAttributeMaxDynamicSharedMemorySize, (int)rp_lds)))
      return TREEKV_EHIP;
    hipLaunchKernelGGL(replay, dim3(p.U), dim3(RP_THREADS), rp_lds, s, p, L, (const uint4*)K, (const uint4*)V, row_vec,
                       retained, n_retained, evicted);
  } else {
    if (2 * (size_t)L + 1 > (size_t)p.cap + p.max_chunk) return TREEKV_EUNSUPPORTED;   // its lists live in pf_list
    hipLaunchKernelGGL(prefill_replay_kernel<false>, dim3(p.U), dim3(RP_THREADS), 0, s, p, L, (const uint4*)K,
                       (const uint4*)V, row_vec, retained, n_retained, evicted);
  }
  hipLaunchKernelGGL(prefill_scatter_kernel, dim3((L + 256 / row_vec - 1) / (256 / row_vec), p.U), dim3(256), 0, s, p, (const uint4*)K, (const uint4*)V, L, row_vec);
  return finish_launch();
}

template <int D>
int launch_prefill_d(const Params& p, const void* Q, const void* K, const void* V, int L, float* out,
                     int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  const uint16_t* q = (const uint16_t*)Q;
  const uint16_t* k = (const uint16_t*)K;
  const uint16_t* v = (const uint16_t*)V;
  const int row_tiles = (L + ROW_TILE - 1) / ROW_TILE;
  const bool rope = (p.flags & TREEKV_POSITION_RERANK) != 0;
  if (rope) {
    const int rows = p.budget + L + L * p.G;           // at most: every cached key, the chunk's keys and queries
    hipLaunchKernelGGL(prefill_turn_kernel<D>, dim3((rows * (D / 8) + 255) / 256, p.U), dim3(256), 0, s, p, q, k, L);
  }
  auto attend = rope ? prefill_attend_kernel<D, true> : prefill_attend_kernel<D, false>;
  const size_t lds = AttendLds<D>::BYTES;
  if (lds > 48 * 1024 &&
      hip_failed(hipFuncSetAttribute((const void*)attend, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
    return TREEKV_EHIP;
  const int n_items = row_tiles * p.G * p.U;
  hipLaunchKernelGGL(attend, dim3((n_items + 7) / 8 * 8), dim3(AT_THREADS), lds, s, p, q, k, v, L, row_tiles, out);
  return launch_replay(p, K, V, L, retained, n_retained, evicted, s);
}

// The same for fp32 storage: one thread turns 4 dimensions (2 planes) of one row and stores them as fp32; the keys go
// to [U][cap + max_chunk][D] (cache rows at their slot, the chunk's behind them), the queries to [B][max_chunk][H][D].
template <int D>
__global__ __launch_bounds__(256) void prefill_turn_f32_kernel(Params p, const float* __restrict__ Q,
                                                               const float* __restrict__ Kc, int L) {
  constexpr int PARTS = D / 4;
  const int unit = blockIdx.y, kvh = unit % p.Hkv, b = unit / p.Hkv;
  const int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int n0 = meta[META_N], j = meta[META_J], rhead = meta[META_RHEAD];
  const int rows = n0 + L + L * p.G;
  const int x = blockIdx.x * 256 + threadIdx.x;
  const int row = x / PARTS, part = x % PARTS;
  if (row >= rows) return;
  const size_t krot_rows = (size_t)p.cap + p.max_chunk;
  float* kturned = reinterpret_cast<float*>(p.pf_krot) + (size_t)unit * krot_rows * D;
  const float* src;
  float* dst;
  int pos;
  if (row < n0) {                                   // cached key at logical index `row`
    const int* Eu = p.E + (size_t)unit * 2 * p.m;
    const int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
    const int slot = n0 < p.budget ? row : logical_to_slot(p, Eu, Ru, rhead, j, row);
    src = (const float*)p.K + ((size_t)unit * p.cap + slot) * D;
    dst = kturned + (size_t)slot * D;
    pos = row;
  } else if (row < n0 + L) {                        // the chunk's own key i
    const int i = row - n0;
    src = Kc + (((size_t)b * L + i) * p.Hkv + kvh) * D;
    dst = kturned + ((size_t)p.cap + i) * D;
    pos = row;
  } else {                                          // query i of head g of the group
    const int i = (row - n0 - L) / p.G, g = (row - n0 - L) % p.G;
    const int h = kvh * p.G + g;
    src = Q + (((size_t)b * L + i) * p.H + h) * D;
    dst = reinterpret_cast<float*>(p.pf_qrot) + (((size_t)b * p.max_chunk + i) * p.H + h) * D;
    pos = n0 + i;
  }
  const float4 xv = *reinterpret_cast<const float4*>(src + part * 4);
  const float4 cs = *reinterpret_cast<const float4*>(p.rope_tab + (size_t)pos * (D / 2) + part * 2);   // (cos, sin) x 2 planes
  float4 y;
  y.x = xv.x * cs.x - xv.y * cs.y;
  y.y = xv.x * cs.y + xv.y * cs.x;
  y.z = xv.z * cs.z - xv.w * cs.w;
  y.w = xv.z * cs.w + xv.w * cs.z;
  *reinterpret_cast<float4*>(dst + part * 4) = y;
}

// fp32 storage: the vector-arithmetic attend, then the same replay.
template <int D>
int launch_prefill_f32(const Params& p, const void* Q, const void* K, const void* V, int L, float* out,
                       int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  const size_t ncols = (size_t)p.cap + L;
  if (ncols > 40 * (size_t)F32_THREADS) return TREEKV_EUNSUPPORTED;      // a thread owns at most 40 columns' sums
  constexpr int KPP = F32_THREADS / (D / 4);
  const size_t lds = (ncols + (KPP * D > F32_THREADS ? KPP * D : F32_THREADS) + D) * sizeof(float);
  const bool rope = (p.flags & TREEKV_POSITION_RERANK) != 0;
  if (rope) {
    const int rows = p.budget + L + L * p.G;           // at most: every cached key, the chunk's keys and queries
    hipLaunchKernelGGL(prefill_turn_f32_kernel<D>, dim3((rows * (D / 4) + 255) / 256, p.U), dim3(256), 0, s, p,
                       (const float*)Q, (const float*)K, L);
  }
  auto attend = rope ? prefill_attend_f32_kernel<D, true> : prefill_attend_f32_kernel<D, false>;
  if (lds > 48 * 1024 &&
      hip_failed(hipFuncSetAttribute((const void*)attend, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
    return TREEKV_EHIP;
  hipLaunchKernelGGL(attend, dim3((L + F32_ROWS - 1) / F32_ROWS, p.G, p.U), dim3(F32_THREADS), lds, s, p, (const float*)Q,
                     (const float*)K, (const float*)V, L, out);
  return launch_replay(p, K, V, L, retained, n_retained, evicted, s);
}

}  // namespace

int launch_prefill(const Params& p, const void* Q, const void* K, const void* V, int len, float* out,
                   int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  if (p.dtype == TREEKV_F32) {
    if (p.D == 128) return launch_prefill_f32<128>(p, Q, K, V, len, out, retained, n_retained, evicted, s);
    if (p.D == 64) return launch_prefill_f32<64>(p, Q, K, V, len, out, retained, n_retained, evicted, s);
    return TREEKV_EUNSUPPORTED;
  }
  if (p.D == 128) return launch_prefill_d<128>(p, Q, K, V, len, out, retained, n_retained, evicted, s);
  if (p.D == 64) return launch_prefill_d<64>(p, Q, K, V, len, out, retained, n_retained, evicted, s);
  return TREEKV_EUNSUPPORTED;
}

}  // namespace tkv
