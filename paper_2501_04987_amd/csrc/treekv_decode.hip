// Decode step of TreeKV for gfx950: one iteration of Algorithm 1's loop after the projections, for every (batch, KV head) unit.
// HBM-bound: per unit it must read every K and V row once (Section 3.1).
//
// Two launch shapes share the streaming code and the epilogue:
//   FUSED  one kernel, grid = U workgroups of 512 threads (measured best of 256..1024).  One workgroup owns a unit end to end; logits stay
//          in LDS, scores and tree positions are prefetched into registers before the streaming
//          starts, so the epilogue (score update, eviction, retained list) waits for no global
//          load.  Used when U alone fills the chip.
//   SPLIT  two kernels.  grid = (nsplit, U) workgroups of 512 threads each stream a slice of the
//          unit's slots and write a partial (output accumulator, max, sum) plus the slice's
//          logits to scratch; a second kernel with one workgroup per unit merges the slices and
//          runs the same epilogue.  The kernel boundary is the only synchronisation.
//
// Streaming.  Rows are 16-byte lane loads: LPR lanes cover one row, a wave load covers 64/LPR
// whole rows, a tile is KU wave loads of K and of V, double buffered.  q.k is reduced inside
// each lane group with DPP; every lane group keeps an online-softmax state (running max, sum,
// output accumulator) in registers, so K and V stream together and no barrier sits inside the
// loop.  Scaled logits are parked in LDS for the score update.  The first tile is requested
// before the unit's bookkeeping words have arrived (cache rows are always initialised memory);
// the new token's k and v are read from the caller's buffers wherever the free slot's index
// comes up, and copied into the cache at the end.

#include "treekv_internal.h"

namespace tkv {

namespace {

// 16-byte row piece with the non-temporal hint: a cache row is read once per step.
__device__ inline uint4 ld_row16(const void* ptr) {
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  const v4u r = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(ptr));
  return make_uint4(r.x, r.y, r.z, r.w);
}
// Measured best of 256 .. 1024 threads per workgroup, for both shapes.
constexpr int FUSED_THREADS = 512;
// position re-assignment in the streaming kernels: off; the angles' (cos, sin) from two small tables in LDS; from the
// context's full table in memory (budgets whose small tables would not fit)
enum : int { ROPE_OFF = 0, ROPE_LDS = 1, ROPE_MEM = 2 };
constexpr int SPLIT_THREADS = 512;
constexpr int MERGE_THREADS = 1024;
constexpr int KU = 2;                  // wave loads of K (and of V) per tile (4: measured slower)
constexpr float NEG_BIG = -1.0e30f;
// Iteration (of n) of the streaming loop at which a workgroup issues its mid-stream stores.  Measured: the
// later they go the better, as long as they are out before the epilogue; early ones interrupt the reads.
__device__ inline int mid_point(int n) { return n * 3 / 4; }
constexpr size_t LDS_LIMIT = 150 * 1024;   // of the 160 KB a workgroup can have

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

template <int CTRL>
__device__ inline float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
  return v + __int_as_float(moved);
}

// Sum over the LPR consecutive lanes that hold one row; every lane of the group gets the total.
template <int LPR>
__device__ inline float group_sum(float v) {
  if constexpr (LPR == 8) {
    v = dpp_add<0x141>(v);           // row_half_mirror: i <-> 7-i
    v = dpp_add<0x1B>(v);            // quad_perm [3,2,1,0]
    v = dpp_add<0xB1>(v);            // quad_perm [1,0,3,2]
  } else {
    v = dpp_add<0x128>(v);           // row_ror:8 (rotate inside each 16-lane row)
    v = dpp_add<0x124>(v);           // row_ror:4
    v = dpp_add<0x122>(v);           // row_ror:2
    v = dpp_add<0x121>(v);           // row_ror:1
    if constexpr (LPR == 32) v += __shfl_xor(v, 16, 64);
  }
  return v;
}

// q.k over one lane's 16 bytes.
template <typename T> struct Dot;
template <> struct Dot<uint16_t> {
  __device__ static inline float run(const uint4& k, const uint4& q) {
    float d = 0.f;
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), d, false);
    return d;
  }
};
template <> struct Dot<float> {
  __device__ static inline float run(const uint4& k, const uint4& q) {
    float d = __uint_as_float(k.x) * __uint_as_float(q.x);
    d = fmaf(__uint_as_float(k.y), __uint_as_float(q.y), d);
    d = fmaf(__uint_as_float(k.z), __uint_as_float(q.z), d);
    d = fmaf(__uint_as_float(k.w), __uint_as_float(q.w), d);
    return d;
  }
};

// What one decode step does to a unit's bookkeeping; known before any score is.
struct Step {
  int n1;            // slots [0, n1) take part in the attention
  int fslot;         // slot of the new token
  int j0;            // eviction index of this step (the paper's idx - 1)
  int t;             // position of the new token
  int rhead;
  bool evict;
  int n_new;         // tokens retained once the step is over
  int j_done;        // evictions of the round done once the step is over
  int newcomer;      // slot that enters the tree region at this step
  int newcomer_pos;
  int scope_l, scope_r, pos_l, pos_r;   // the eviction scope {idx, idx+1}: slots and positions
};

// The five bookkeeping words: everything the streaming and the retained list need.
__device__ inline Step load_meta(const Params& p, const int* meta) {
  Step s;
  s.n1 = meta[META_N] + 1;
  s.fslot = meta[META_FREE];
  s.j0 = meta[META_J];
  s.t = meta[META_T];
  s.rhead = meta[META_RHEAD];
  s.evict = s.n1 > p.budget;
  s.n_new = s.evict ? p.budget : s.n1;
  s.j_done = s.evict ? s.j0 + 1 : s.j0;
  s.newcomer = s.fslot;
  s.newcomer_pos = s.t - p.n_recent;     // the recent window holds the last n_recent positions
  s.scope_l = s.scope_r = -1;
  s.pos_l = s.pos_r = 0;
  return s;
}

// The eviction scope: loads that depend on the bookkeeping words and are first needed in the
// epilogue, so they are requested while the rows stream.
__device__ inline void load_scope(const Params& p, Step& s, const int* Eu, const int* PEu, const int* Ru) {
  if (!s.evict) return;
  if (p.n_recent > 0) s.newcomer = Ru[s.rhead];     // the window's oldest member moves into the tree region
  s.scope_l = Eu[2 * s.j0];
  s.pos_l = PEu[2 * s.j0];
  if (2 * s.j0 + 1 == p.m + s.j0) { s.scope_r = s.newcomer; s.pos_r = s.newcomer_pos; }
  else { s.scope_r = Eu[2 * s.j0 + 1]; s.pos_r = PEu[2 * s.j0 + 1]; }
}

// Position of logical index i once the step is over.  The two tree entries the step itself
// writes are taken from `surv_pos` / the newcomer when `patched`, else read as they were.
__device__ inline int position_of(const Params& p, const Step& s, const int* PEu, int i, int surv_pos, bool patched) {
  if (i >= s.n_new) return -1;
  if (s.n_new < p.budget) return i;        // still filling: token i sits at index i
  const int k = i - p.n_sink;
  if (k < 0) return i;
  if (k >= p.m) return s.t + 1 - p.n_recent + (k - p.m);
  if (s.evict && patched) {
    if (k == s.j0) return surv_pos;
    if (k == p.m - 1) return s.newcomer_pos;
  }
  return PEu[tree_index(k, s.j_done)];
}

// ---------------------------------------------------------------------------------------------
// Streaming: online softmax over slots [begin, end) of one unit by one workgroup.
// Leaves per-wave (max, sum, accumulator) in LDS and the scaled logits in sm_s[g][row - begin].
// ---------------------------------------------------------------------------------------------
// ROPE (position re-assignment, Section 4.1 "Position Encoding"): the cache holds keys without positional
// encoding; a key's position is its rank in the cache's logical order, the query's the rank of the new token, and
// the rotary encoding enters the logit in its relative form: with (c, s) = (cos, sin) of distance * theta_i from a
// table, plane i of the key is turned back by that angle and then multiplied with the query's plane.  The ranks of
// the slots a workgroup streams are laid out in LDS (behind the logits) from the order arrays before the first
// tile is consumed; the (cos, sin) pairs come from two small tables in LDS (see TAB_STEP below), looked up one
// tile ahead of their use.
template <typename T, int D, int G, int THREADS, int ROPE = ROPE_OFF>
struct Stream {
  static constexpr int WAVES = THREADS / 64;
  static constexpr int EPL = Storage<T>::EPL;   // elements per 16-byte lane load
  static constexpr int LPR = D / EPL;           // lanes per row
  static constexpr int RPL = 64 / LPR;          // rows per wave load
  static constexpr int TILE = RPL * KU;         // rows per wave iteration
  static constexpr int STEP = WAVES * TILE;     // rows per workgroup iteration
  static constexpr int LDS_FLOATS_FIXED = WAVES * G * (D + 2);
  static constexpr int LDS_WORDS_PER_ROW = G + (ROPE ? 1 : 0);     // logits, and the slot's rank
  static constexpr int TV = EPL / 4;            // 16-byte pieces of a lane's (cos, sin) pairs
  // ROPE: the angles' (cos, sin) come from two small tables in LDS, rows 0, 64, 128, .. and rows 0 .. 63 of the
  // context's table, multiplied as complex numbers: (cos, sin)(n theta) = (cos, sin)(64 a theta) x (cos, sin)(b theta)
  // for n = 64 a + b.  Read from the full table in memory, the pairs are as many bytes per row as K and V together and
  // cost the launch 6 us at 256 units x 2048 slots.
  static constexpr int TAB_STEP = 64;
  __host__ __device__ static inline int tab_rows(int cap) { return (cap - 1) / TAB_STEP + 1 + TAB_STEP; }
  // budgets whose two tables would take more than 80 KB of LDS (more than 6144 slots at head_dim 128, twice that
  // at 64) read the pairs from the full table in memory instead
  __host__ __device__ static inline bool tab_in_lds(int cap) { return (size_t)tab_rows(cap) * D * sizeof(float) <= 80 * 1024; }
  __host__ __device__ static inline size_t tab_offset(int rows) {     // in floats from the start of the dynamic LDS
    return ((size_t)LDS_FLOATS_FIXED + (size_t)LDS_WORDS_PER_ROW * rows + 3) & ~(size_t)3;
  }
  // floats of dynamic LDS for `rows` streamed rows of a cache of `cap` slots
  __host__ __device__ static inline size_t lds_floats(int cap, int rows) {
    return ROPE == ROPE_LDS ? tab_offset(rows) + (size_t)tab_rows(cap) * D
                            : (size_t)LDS_FLOATS_FIXED + (size_t)LDS_WORDS_PER_ROW * rows;
  }

  // sm_acc [WAVES][G][D], sm_wm [WAVES][G], sm_wl [WAVES][G].  `after_meta(st)` runs once the
  // bookkeeping words are known, after the first tile has been requested.
  // `mid_stream()` runs once, three quarters of the way through the loop: the place for stores that should
  // be out of the way before the epilogue.
  template <class AfterMeta, class MidStream>
  __device__ static inline void run(const Params& p, int unit, int begin_spec, const T* __restrict__ q_in,
                                    const T* __restrict__ knew, const T* __restrict__ vnew, const int* meta,
                                    float* sm_s, int lds_rows, float* sm_acc, float* sm_wm, float* sm_wl,
                                    Step& st, int& begin, int& end, bool fused, AfterMeta after_meta,
                                    MidStream mid_stream) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane % LPR, ri = lane / LPR;
    const int kvh = unit % p.Hkv, b = unit / p.Hkv;
    const T* Ku = (const T*)p.K + (size_t)unit * p.cap * D;
    const T* Vu = (const T*)p.V + (size_t)unit * p.cap * D;

    // first two tiles, requested before the bookkeeping words are known (rows clamped to the allocation)
    uint4 ka[KU], va[KU], kb[KU], vb[KU];
    int base = begin_spec + wave * TILE;
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const int row = min(base + u * RPL + ri, p.cap - 1);
      ka[u] = ld_row16(Ku + (size_t)row * D + li * EPL);
      va[u] = ld_row16(Vu + (size_t)row * D + li * EPL);
    }
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const int row = min(base + STEP + u * RPL + ri, p.cap - 1);
      kb[u] = ld_row16(Ku + (size_t)row * D + li * EPL);
      vb[u] = ld_row16(Vu + (size_t)row * D + li * EPL);
    }
    uint4 qr[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
      qr[g] = *reinterpret_cast<const uint4*>(q_in + ((size_t)b * p.H + (size_t)kvh * G + g) * D + li * EPL);

    // ROPE: the two small tables, copied while the first rows are on their way.  A table row is laid out so that
    // the LPR lanes of a row read consecutive 16-byte pieces: piece x of lane l at [x][l].
    uint4* sm_tab = reinterpret_cast<uint4*>(sm_s - LDS_FLOATS_FIXED + tab_offset(lds_rows));
    const int tab_a = (p.cap - 1) / TAB_STEP + 1;         // rows 0, 64, .. come first, rows 0 .. 63 after them
    constexpr bool lds_tab = ROPE == ROPE_LDS;
    if constexpr (lds_tab) {
      constexpr int RV = D / 4;                           // 16-byte pieces of a table row
      for (int e = tid; e < tab_rows(p.cap) * RV; e += THREADS) {
        const int r = e / RV, c = e % RV;
        const int pos = min(r < tab_a ? r * TAB_STEP : r - tab_a, p.cap - 1);   // rows past cap - 1 are never looked up
        sm_tab[r * RV + (c % TV) * LPR + c / TV] = reinterpret_cast<const uint4*>(p.rope_tab + (size_t)pos * (D / 2))[c];
      }
    }

    st = load_meta(p, meta);
    begin = begin_spec;
    end = fused ? st.n1 : min(st.n1, begin + p.rows_per_split);
    const int fslot = st.fslot;
    after_meta(st);

    // position re-assignment: rank of every streamed slot, then the table rows of the two tiles in flight
    int* sm_rank = reinterpret_cast<int*>(sm_s + (size_t)G * lds_rows);
    uint4 ta[ROPE ? KU : 1][ROPE ? TV : 1], tb2[ROPE ? KU : 1][ROPE ? TV : 1];
    auto load_tab = [&](uint4 (&td)[ROPE ? KU : 1][ROPE ? TV : 1], int tb) {
      if constexpr (ROPE) {
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          const int row = max(min(tb + u * RPL + ri, end - 1), begin);
          const int dist = min(max(st.n1 - 1 - sm_rank[row - begin], 0), p.cap - 1);
          if constexpr (!lds_tab) {
            const uint4* src = reinterpret_cast<const uint4*>(p.rope_tab + (size_t)dist * (D / 2) + li * (EPL / 2));
#pragma unroll
            for (int x = 0; x < TV; ++x) td[u][x] = src[x];
          } else {
          const uint4* ra = sm_tab + (dist / TAB_STEP) * (D / 4) + li;
          const uint4* rb = sm_tab + (tab_a + dist % TAB_STEP) * (D / 4) + li;
#pragma unroll
          for (int x = 0; x < TV; ++x) {
            const uint4 a = ra[x * LPR], c = rb[x * LPR];
            const float ac0 = __uint_as_float(a.x), as0 = __uint_as_float(a.y), ac1 = __uint_as_float(a.z), as1 = __uint_as_float(a.w);
            const float bc0 = __uint_as_float(c.x), bs0 = __uint_as_float(c.y), bc1 = __uint_as_float(c.z), bs1 = __uint_as_float(c.w);
            td[u][x] = make_uint4(__float_as_uint(fmaf(ac0, bc0, -(as0 * bs0))), __float_as_uint(fmaf(as0, bc0, ac0 * bs0)),
                                  __float_as_uint(fmaf(ac1, bc1, -(as1 * bs1))), __float_as_uint(fmaf(as1, bc1, ac1 * bs1)));
          }
          }
        }
      }
    };
    if constexpr (ROPE) {
      const int n = st.n1 - 1;                  // cached tokens; the new one takes rank n
      if (n < p.budget) {                       // still filling: token i sits in slot i
        for (int r = begin + tid; r < end; r += THREADS) sm_rank[r - begin] = r;
      } else {
        const int* Eu = p.E + (size_t)unit * 2 * p.m;
        const int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
        for (int i = tid; i < n; i += THREADS) {
          const int slot = logical_to_slot(p, Eu, Ru, st.rhead, st.j0, i);
          if (slot >= begin && slot < end) sm_rank[slot - begin] = i;
        }
        if (tid == 0 && fslot >= begin && fslot < end) sm_rank[fslot - begin] = n;
      }
      __syncthreads();
      if (base < end) load_tab(ta, base);
      if (base + STEP < end) load_tab(tb2, base + STEP);
    }

    auto load_tile = [&](uint4 (&kd)[KU], uint4 (&vd)[KU], int tb) {
      const bool has_new = fslot >= tb && fslot < tb + TILE;       // wave uniform
#pragma unroll
      for (int u = 0; u < KU; ++u) {
        const int row = min(tb + u * RPL + ri, end - 1);
        const T* ks = Ku + (size_t)row * D;
        const T* vs = Vu + (size_t)row * D;
        if (has_new && row == fslot) { ks = knew; vs = vnew; }
        kd[u] = ld_row16(ks + li * EPL);
        vd[u] = ld_row16(vs + li * EPL);
      }
    };
    // a speculative tile read the free slot's stale row if it covers it: fetch the real one
    auto patch_new = [&](uint4 (&kd)[KU], uint4 (&vd)[KU], int tb) {
      if (fslot >= tb && fslot < tb + TILE) {
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          if (tb + u * RPL + ri == fslot) {
            kd[u] = *reinterpret_cast<const uint4*>(knew + li * EPL);
            vd[u] = *reinterpret_cast<const uint4*>(vnew + li * EPL);
          }
        }
      }
    };
    patch_new(ka, va, base);
    patch_new(kb, vb, base + STEP);

    float m_run[G], l_run[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m_run[g] = NEG_BIG; l_run[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    // the query as floats, up front unless that would not fit the registers
    constexpr bool Q_WIDE = ROPE && G * EPL <= 32;
    float qf[Q_WIDE ? G : 1][EPL];
    if constexpr (Q_WIDE) {
#pragma unroll
      for (int g = 0; g < G; ++g) Storage<T>::widen(qr[g], qf[g]);
    }
    auto tile = [&](const uint4 (&kr)[KU], const uint4 (&vr)[KU], const uint4 (&tr)[ROPE ? KU : 1][ROPE ? TV : 1], int tb) {
      float s[KU][G];
      bool ok[KU];
#pragma unroll
      for (int u = 0; u < KU; ++u) {
        const int row = tb + u * RPL + ri;
        ok[u] = row < end;
        float kt[EPL];                          // ROPE: the key's planes turned back by distance * theta
        if constexpr (ROPE) {
          float kf[EPL], cs[EPL];
          Storage<T>::widen(kr[u], kf);
#pragma unroll
          for (int x = 0; x < TV; ++x) {
            cs[4 * x] = __uint_as_float(tr[u][x].x); cs[4 * x + 1] = __uint_as_float(tr[u][x].y);
            cs[4 * x + 2] = __uint_as_float(tr[u][x].z); cs[4 * x + 3] = __uint_as_float(tr[u][x].w);
          }
#pragma unroll
          for (int e = 0; e < EPL; e += 2) {
            kt[e] = fmaf(kf[e], cs[e], kf[e + 1] * cs[e + 1]);
            kt[e + 1] = fmaf(kf[e + 1], cs[e], -(kf[e] * cs[e + 1]));
          }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float part;
          if constexpr (ROPE) {
            part = 0.f;
            if constexpr (Q_WIDE) {
#pragma unroll
              for (int e = 0; e < EPL; ++e) part = fmaf(qf[g][e], kt[e], part);
            } else {
              float qg[EPL];
              Storage<T>::widen(qr[g], qg);
#pragma unroll
              for (int e = 0; e < EPL; ++e) part = fmaf(qg[e], kt[e], part);
            }
          } else {
            part = Dot<T>::run(kr[u], qr[g]);
          }
          float d = group_sum<LPR>(part) * p.scale_log2e;
          d = ok[u] ? d : NEG_BIG;
          s[u][g] = d;
          if (li == 0 && ok[u]) sm_s[(size_t)g * lds_rows + (row - begin)] = d;
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mxv = m_run[g];
#pragma unroll
        for (int u = 0; u < KU; ++u) mxv = fmaxf(mxv, s[u][g]);
        const float corr = fast_exp2(m_run[g] - mxv);
        m_run[g] = mxv;
        l_run[g] *= corr;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          const float pr = ok[u] ? fast_exp2(s[u][g] - mxv) : 0.f;
          s[u][g] = pr;
          l_run[g] += pr;
        }
      }
#pragma unroll
      for (int u = 0; u < KU; ++u) {
        float vf[EPL];
        Storage<T>::widen(vr[u], vf);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(s[u][g], vf[e], acc[g][e]);
      }
    };

    const int mid_iter = mid_point((end - begin + 2 * STEP - 1) / (2 * STEP));
    int iter = 0;
    for (; base < end; base += 2 * STEP, ++iter) {
      if (iter > 0 && base + STEP < end) { load_tile(kb, vb, base + STEP); load_tab(tb2, base + STEP); }
      tile(ka, va, ta, base);
      if (base + 2 * STEP < end) { load_tile(ka, va, base + 2 * STEP); load_tab(ta, base + 2 * STEP); }
      if (base + STEP < end) tile(kb, vb, tb2, base + STEP);
      if (iter == mid_iter) mid_stream();
    }
    if (iter <= mid_iter) mid_stream();

    // merge the RPL lane groups of the wave
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float mo = __shfl_xor(m_run[g], off, 64);
        const float lo = __shfl_xor(l_run[g], off, 64);
        const float mxv = fmaxf(m_run[g], mo);
        const float ca = fast_exp2(m_run[g] - mxv), cb = fast_exp2(mo - mxv);
        l_run[g] = l_run[g] * ca + lo * cb;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const float ao = __shfl_xor(acc[g][e], off, 64);
          acc[g][e] = acc[g][e] * ca + ao * cb;
        }
        m_run[g] = mxv;
      }
    }
    if (ri == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm_acc[(wave * G + g) * D + li * EPL + e] = acc[g][e];
        if (li == 0) { sm_wm[wave * G + g] = m_run[g]; sm_wl[wave * G + g] = l_run[g]; }
      }
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Streaming for grouped queries (bf16, G >= 2).  With G query heads per KV head the per-row work
// is a small contraction, [G x d] . [d x rows] and [G x rows] . [rows x d], and doing it on the
// vector ALU costs G times the instructions of the G = 1 stream: the kernel turns ALU bound.  Here the two
// contractions go to the matrix pipe (16x16x32 bf16 MFMA with the G heads in 16 columns), which is
// otherwise idle; the stream itself (every K and V row read once, 16-byte lane loads) is unchanged.
//   S^T = K Q^T   A = 16 K rows read straight from global in operand order, B = Q (columns >= G are padding)
//   O^T += V^T P^T  A = V^T: the wave's 32 V rows are transposed in registers (v_perm) into a wave-private
//                   LDS tile; B = P^T, which is exactly the accumulator layout of S^T (no lane movement).
// P is split into two bf16 parts (hi + lo) so that rounding it costs 2^-16, not 2^-9.
// Same outputs as Stream::run: per-wave (max, sum, accumulator) in LDS, scaled logits in sm_s.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

__device__ inline f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
__device__ inline unsigned pack_bf16(float a, float b) {
  f32x2_t v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

template <int D, int G, int THREADS>
struct StreamMfma {
  using T = uint16_t;
  static constexpr int WAVES = THREADS / 64;
  static constexpr int TILE = 32;                 // rows per wave iteration (one k-step of the P.V contraction)
  static constexpr int STEP = WAVES * TILE;
  static constexpr int KS = D / 32, DB = D / 16, PARTS = D / 8;
  static constexpr int VSTRIDE = TILE + 8;        // bf16 elements per staged V^T row (80 bytes: conflict-free b128 reads)
  static constexpr int VT_FLOATS = D * VSTRIDE / 2;
  static constexpr int LDS_FLOATS_FIXED = WAVES * G * (D + 2) + WAVES * VT_FLOATS;
  static constexpr int LDS_WORDS_PER_ROW = G;
  __host__ __device__ static inline size_t lds_floats(int, int rows) {
    return (size_t)LDS_FLOATS_FIXED + (size_t)LDS_WORDS_PER_ROW * rows;
  }
  static constexpr int VLOADS = TILE * PARTS / 64;        // 16-byte V pieces per lane and tile (8 at d=128, 4 at d=64)
  static_assert(G >= 2 && G <= 16 && (VLOADS == 8 || VLOADS == 4), "written for head_dim 64 / 128");

  template <class AfterMeta, class MidStream>
  __device__ static inline void run(const Params& p, int unit, int begin_spec, const T* __restrict__ q_in,
                                    const T* __restrict__ knew, const T* __restrict__ vnew, const int* meta,
                                    float* sm_s, int lds_rows, float* sm_acc, float* sm_wm, float* sm_wl,
                                    Step& st, int& begin, int& end, bool fused, AfterMeta after_meta,
                                    MidStream mid_stream) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, q4 = lane >> 4;
    const int kvh = unit % p.Hkv, b = unit / p.Hkv;
    const T* Ku = (const T*)p.K + (size_t)unit * p.cap * D;
    const T* Vu = (const T*)p.V + (size_t)unit * p.cap * D;
    uint16_t* vt = reinterpret_cast<uint16_t*>(sm_acc + WAVES * G * (D + 2)) + (size_t)wave * (VT_FLOATS * 2);

    // B operand of S^T = K Q^T: column lr is query head lr of the group (zero beyond G)
    uint4 qa[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qa[ks] = make_uint4(0, 0, 0, 0);
      if (lr < G) qa[ks] = *reinterpret_cast<const uint4*>(q_in + ((size_t)b * p.H + (size_t)kvh * G + lr) * D + ks * 32 + q4 * 8);
    }

    st = load_meta(p, meta);
    begin = begin_spec;
    end = fused ? st.n1 : min(st.n1, begin + p.rows_per_split);
    const int fslot = st.fslot;
    after_meta(st);

    // K rows arrive in operand order: lane (lr, q4) holds K[row + lr][ks*32 + q4*8 ..] of two 16-row blocks.
    // V rows arrive as whole rows: 16 lanes per row, lane group q4 takes rows q4*4 + {0..3} of each block.
    uint4 k00, k01, k02, k03, k10, k11, k12, k13;            // [block][k-step]
    uint4 v00, v01, v02, v03, v10, v11, v12, v13;            // [block][row q4*4 + x], this lane's 8 dims
    k00 = k01 = k02 = k03 = k10 = k11 = k12 = k13 = make_uint4(0, 0, 0, 0);
    v00 = v01 = v02 = v03 = v10 = v11 = v12 = v13 = make_uint4(0, 0, 0, 0);
    auto row_ptr = [&](const T* cache, const T* fresh, int row) -> const T* {
      const int r = min(row, end - 1);
      return r == fslot ? fresh : cache + (size_t)r * D;
    };
    auto load_k = [&](int tb) {
      const T* r0 = row_ptr(Ku, knew, tb + lr) + q4 * 8;
      const T* r1 = row_ptr(Ku, knew, tb + 16 + lr) + q4 * 8;
      k00 = ld_row16(r0); k01 = ld_row16(r0 + 32);
      k10 = ld_row16(r1); k11 = ld_row16(r1 + 32);
      if constexpr (KS > 2) {
        k02 = ld_row16(r0 + 64); k03 = ld_row16(r0 + 96);
        k12 = ld_row16(r1 + 64); k13 = ld_row16(r1 + 96);
      }
    };
    // V pieces: piece index = lane + 64*x; row = piece / PARTS, part = piece % PARTS.  With PARTS = 16 a lane keeps
    // part = lr and rows q4 + 4x; the transposition below wants rows q4*4 + {0..3}, so rows are dealt that way.
    const int v_part = lane % PARTS, v_rg = lane / PARTS;    // v_rg: 0..3 (d=128) or 0..7 (d=64)
    auto load_v = [&](int tb) {
      if constexpr (PARTS == 16) {
        const int r = tb + v_rg * 4;
        v00 = ld_row16(row_ptr(Vu, vnew, r) + v_part * 8);
        v01 = ld_row16(row_ptr(Vu, vnew, r + 1) + v_part * 8);
        v02 = ld_row16(row_ptr(Vu, vnew, r + 2) + v_part * 8);
        v03 = ld_row16(row_ptr(Vu, vnew, r + 3) + v_part * 8);
        v10 = ld_row16(row_ptr(Vu, vnew, r + 16) + v_part * 8);
        v11 = ld_row16(row_ptr(Vu, vnew, r + 17) + v_part * 8);
        v12 = ld_row16(row_ptr(Vu, vnew, r + 18) + v_part * 8);
        v13 = ld_row16(row_ptr(Vu, vnew, r + 19) + v_part * 8);
      } else {                                               // d = 64: 8 row groups of 4 rows cover the 32 rows
        const int r = tb + v_rg * 4;
        v00 = ld_row16(row_ptr(Vu, vnew, r) + v_part * 8);
        v01 = ld_row16(row_ptr(Vu, vnew, r + 1) + v_part * 8);
        v02 = ld_row16(row_ptr(Vu, vnew, r + 2) + v_part * 8);
        v03 = ld_row16(row_ptr(Vu, vnew, r + 3) + v_part * 8);
      }
    };
    // staged V^T: row d, the tile's rows in k-slot order: row (blk*16 + q*4 + i) at position q*8 + blk*4 + i;
    // the 16-byte pair q is XOR-swizzled with (d/16)%4 (reads of an operand share d/16; writes spread out)
    auto put_v = [&](const uint4& a, const uint4& b2, const uint4& c, const uint4& d4, int blk, int q) {
      auto emit = [&](unsigned a0, unsigned a1, unsigned a2, unsigned a3, int e_even) {
#pragma unroll
        for (int odd = 0; odd < 2; ++odd) {
          const unsigned sel = odd ? 0x07060302u : 0x05040100u;
          uint2 o;
          o.x = __builtin_amdgcn_perm(a1, a0, sel);
          o.y = __builtin_amdgcn_perm(a3, a2, sel);
          const int dd = v_part * 8 + e_even + odd;
          *reinterpret_cast<uint2*>(&vt[dd * VSTRIDE + ((q ^ ((dd >> 4) & 3)) * 8) + blk * 4]) = o;
        }
      };
      emit(a.x, b2.x, c.x, d4.x, 0); emit(a.y, b2.y, c.y, d4.y, 2);
      emit(a.z, b2.z, c.z, d4.z, 4); emit(a.w, b2.w, c.w, d4.w, 6);
    };

    float m_run = NEG_BIG, l_part = 0.f;           // this lane's query head (lr): running max, partial sum
    f32x4_t oacc[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d) oacc[d] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const float sc = p.scale_log2e;

    int base = begin + wave * TILE;
    if (base < end) { load_k(base); load_v(base); }
    const int mid_iter = mid_point((end - begin + STEP - 1) / STEP);
    int iter = 0;
    for (; base < end; base += STEP, ++iter) {
      const int nb = base + STEP;
      // ---- S^T: two 16-row blocks ----
      f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
      s0 = mfma16(k00, qa[0], s0); s1 = mfma16(k10, qa[0], s1);
      s0 = mfma16(k01, qa[1], s0); s1 = mfma16(k11, qa[1], s1);
      if constexpr (KS > 2) {
        s0 = mfma16(k02, qa[2], s0); s1 = mfma16(k12, qa[2], s1);
        s0 = mfma16(k03, qa[3], s0); s1 = mfma16(k13, qa[3], s1);
      }
      if (nb < end) load_k(nb);                                       // next tile's K behind this tile's softmax
      // ---- V rows -> V^T tile (wave private) ----
      if constexpr (PARTS == 16) {
        put_v(v00, v01, v02, v03, 0, v_rg);
        put_v(v10, v11, v12, v13, 1, v_rg);
      } else {
        put_v(v00, v01, v02, v03, v_rg >> 2, v_rg & 3);
      }
      if (nb < end) load_v(nb);
      // ---- logits of rows base + blk*16 + q4*4 + i for head lr ----
      float sv[8];
      const bool tail = base + TILE > end;
#pragma unroll
      for (int i = 0; i < 4; ++i) { sv[i] = s0[i] * sc; sv[4 + i] = s1[i] * sc; }
      if (tail) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sv[e] = (base + (e >> 2) * 16 + q4 * 4 + (e & 3) < end) ? sv[e] : NEG_BIG;
      }
      if (lr < G) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int row = base + (e >> 2) * 16 + q4 * 4 + (e & 3);
          if (!tail || row < end) sm_s[(size_t)lr * lds_rows + (row - begin)] = sv[e];
        }
      }
      float mx = m_run;
#pragma unroll
      for (int e = 0; e < 8; ++e) mx = fmaxf(mx, sv[e]);
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (__any(mx != m_run)) {
        const float corr = fast_exp2(m_run - mx);
        l_part *= corr;
#pragma unroll
        for (int d = 0; d < DB; ++d) oacc[d] *= corr;
        m_run = mx;
      }
      unsigned hi[4], lo[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        float p0 = fast_exp2(sv[2 * e2] - mx), p1 = fast_exp2(sv[2 * e2 + 1] - mx);
        if (tail) {
          p0 = sv[2 * e2] > 0.5f * NEG_BIG ? p0 : 0.f;
          p1 = sv[2 * e2 + 1] > 0.5f * NEG_BIG ? p1 : 0.f;
        }
        l_part += p0 + p1;
        hi[e2] = pack_bf16(p0, p1);
        lo[e2] = pack_bf16(p0 - __uint_as_float(hi[e2] << 16), p1 - __uint_as_float(hi[e2] & 0xffff0000u));
      }
      const uint4 phi = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      const uint4 plo = make_uint4(lo[0], lo[1], lo[2], lo[3]);
      // ---- O^T += V^T P^T ----
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        const uint4 a = *reinterpret_cast<const uint4*>(&vt[(d * 16 + lr) * VSTRIDE + ((q4 ^ (d & 3)) * 8)]);
        oacc[d] = mfma16(a, phi, oacc[d]);
        oacc[d] = mfma16(a, plo, oacc[d]);
      }
      __builtin_amdgcn_wave_barrier();
      if (iter == mid_iter) mid_stream();
    }
    if (iter <= mid_iter) mid_stream();

    float l_row = l_part + __shfl_xor(l_part, 16, 64);
    l_row += __shfl_xor(l_row, 32, 64);
    if (lr < G) {
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int i = 0; i < 4; ++i) sm_acc[(wave * G + lr) * D + d * 16 + q4 * 4 + i] = oacc[d][i];
      if (q4 == 0) { sm_wm[wave * G + lr] = m_run; sm_wl[wave * G + lr] = l_row; }
    }
  }
};

// The stream to use for a storage type and group size.
template <typename T, int D, int G, int THREADS, int ROPE> struct PickStream { using type = Stream<T, D, G, THREADS, ROPE>; };
// which instance a context's decode steps take
template <typename T, int D>
inline int rope_mode(const Params& p) {
  if (!(p.flags & TREEKV_POSITION_RERANK)) return ROPE_OFF;
  return Stream<T, D, 1, FUSED_THREADS, ROPE_LDS>::tab_in_lds(p.cap) ? ROPE_LDS : ROPE_MEM;
}
template <int D, int THREADS> struct PickStream<uint16_t, D, 2, THREADS, ROPE_OFF> { using type = StreamMfma<D, 2, THREADS>; };
template <int D, int THREADS> struct PickStream<uint16_t, D, 4, THREADS, ROPE_OFF> { using type = StreamMfma<D, 4, THREADS>; };
template <int D, int THREADS> struct PickStream<uint16_t, D, 8, THREADS, ROPE_OFF> { using type = StreamMfma<D, 8, THREADS>; };

// Global (max, sum) over the parts' (max, sum) pairs, identical in every thread that calls it.
__device__ inline void merge_stats(const float* pm, const float* pl, int nparts, int stride, float& M, float& L) {
  float mx = NEG_BIG;
  for (int w = 0; w < nparts; ++w) mx = fmaxf(mx, pm[w * stride]);
  float l = 0.f;
  for (int w = 0; w < nparts; ++w) l += pl[w * stride] * fast_exp2(pm[w * stride] - mx);
  M = mx; L = l;
}

// ---------------------------------------------------------------------------------------------
// Epilogue shared by both shapes: Algorithm 1's score update and eviction block, the retained
// list, and the append of the new row.  `logit(g, slot)` returns the scaled logit; M, invL per g.
// EP > 0: the first EP old scores per thread come in registers, and the caller has already written
// the retained list except for the one entry this step's decision fills in.
// With EP > 0, `park` (LDS, may alias the logits of head 0) receives every new score and the decision reads
// its two operands from there; with EP == 0 the two owners leave them in sm_sc.
// A wave issues an instruction every five cycles or so and nothing else runs at this point, so this code is
// laid out for a short instruction stream per wave: uniform exits from the unrolled loops, and the dozen
// bookkeeping stores dealt to lane 0 of different waves.  The k, v rows are held by the last LPR threads.
// ---------------------------------------------------------------------------------------------
template <typename T, int D, int G, int THREADS, int EP, class LogitFn>
__device__ inline void epilogue(const Params& p, int unit, const Step& st, const float (&M)[G], const float (&invL)[G],
                                LogitFn logit, const float* s_old, uint4 knew_r, uint4 vnew_r, float* sm_sc, float* park,
                                int32_t* __restrict__ retained, int32_t* __restrict__ n_retained,
                                int32_t* __restrict__ evicted, int* meta, int ret_patch_tid) {
  constexpr int LPR = D / Storage<T>::EPL;
  static_assert(THREADS >= 256 && LPR <= 64, "the bookkeeping stores are dealt to four waves");
  const int tid = threadIdx.x;
  float* Su = p.S + (size_t)unit * p.cap;
  int* Eu = p.E + (size_t)unit * 2 * p.m;
  int* PEu = p.PE + (size_t)unit * 2 * p.m;
  int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);

  auto prob = [&](int slot) -> float {
    float a = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) a += fast_exp2(logit(g, slot) - M[g]) * invL[g];
    return a;
  };
  auto put_score = [&](int slot, float sn) {
    __builtin_nontemporal_store(sn, Su + slot);    // read again only a whole step later
    if constexpr (EP > 0) park[slot] = sn;
    else {
      if (slot == st.scope_l) sm_sc[0] = sn;
      if (slot == st.scope_r) sm_sc[1] = sn;
    }
  };
#pragma unroll
  for (int x = 0; x < EP; ++x) {
    if (x * THREADS >= st.n1) break;                 // uniform
    const int slot = tid + x * THREADS;
    if (slot < st.n1) put_score(slot, s_old[x] + prob(slot));
  }
  for (int slot = tid + EP * THREADS; slot < st.n1; slot += THREADS)
    put_score(slot, (slot == st.fslot ? 0.f : Su[slot]) + prob(slot));
  // the new token's k, v become cache rows
  if (tid >= THREADS - LPR) {
    T* Kw = (T*)p.K + ((size_t)unit * p.cap + st.fslot) * D;
    T* Vw = (T*)p.V + ((size_t)unit * p.cap + st.fslot) * D;
    reinterpret_cast<uint4*>(Kw)[tid - (THREADS - LPR)] = knew_r;
    reinterpret_cast<uint4*>(Vw)[tid - (THREADS - LPR)] = vnew_r;
  }
  __syncthreads();

  // lane 0 of the first four waves and the owner of the open retained entry take the same decision from the
  // same two numbers; everyone else is done
  if (EP > 0 && !((tid & 63) == 0 && tid < 256) && tid != ret_patch_tid) return;
  bool drop_right = false;
  if (st.evict) {
    const float sl = EP > 0 ? park[st.scope_l] : sm_sc[0], sr = EP > 0 ? park[st.scope_r] : sm_sc[1];
    const bool averaged = !(p.flags & TREEKV_SCORE_ACCUMULATED);
    const float bl = averaged ? sl / (float)(st.t - st.pos_l + 1) : sl;
    const float br = averaged ? sr / (float)(st.t - st.pos_r + 1) : sr;
    drop_right = (p.flags & TREEKV_KEEP_LEFT) || (bl > br);     // strict: a tie evicts the left slot
  }
  const int surv_pos = drop_right ? st.pos_l : st.pos_r;
  if (tid == 0) {                                    // the tree entry the survivor moves up to
    if (st.evict) {
      Eu[st.j0] = drop_right ? st.scope_l : st.scope_r;
      PEu[st.j0] = surv_pos;
    }
  } else if (tid == 64) {                            // the five bookkeeping words
    int f_new = st.n1, j = st.j0, rhead = st.rhead;
    if (st.evict) {
      if (p.n_recent > 0) rhead = rhead + 1 == p.n_recent ? 0 : rhead + 1;
      f_new = drop_right ? st.scope_r : st.scope_l;
      j = st.j0 + 1 == p.m ? 0 : st.j0 + 1;
    }
    meta[META_N] = st.n_new;
    meta[META_FREE] = f_new;
    meta[META_J] = j;
    meta[META_RHEAD] = rhead;
    meta[META_T] = st.t + 1;
  } else if (tid == 128) {                           // what the caller asked to be told
    if (evicted) evicted[unit] = st.evict ? (drop_right ? st.pos_r : st.pos_l) : -1;
    if (n_retained) n_retained[unit] = st.n_new;
  } else if (tid == 192) {                           // the newcomer's tree entry and the ring
    if (st.evict) {
      if (p.n_recent > 0) Ru[st.rhead] = st.fslot;   // the new token takes the ring entry of the one that left
      Eu[p.m + st.j0] = st.newcomer;
      PEu[p.m + st.j0] = st.newcomer_pos;
    }
  }

  // retained positions in ascending order
  int32_t* ret = retained + (size_t)unit * p.budget;
  if constexpr (EP > 0) {
    // the rest was written up front; the same thread that wrote this entry's old value patches it
    if (st.evict && tid == ret_patch_tid) ret[p.n_sink + st.j0] = surv_pos;
  } else {
    for (int i = tid; i < p.budget; i += THREADS) ret[i] = position_of(p, st, PEu, i, surv_pos, true);
  }
}

// ---------------------------------------------------------------------------------------------
template <typename T, int D, int G, int ROPE>
__global__ __launch_bounds__(FUSED_THREADS) void decode_fused_kernel(Params p, const T* __restrict__ q_in,
                                                                     const T* __restrict__ k_in,
                                                                     const T* __restrict__ v_in,
                                                                     float* __restrict__ out,
                                                                     int32_t* __restrict__ retained,
                                                                     int32_t* __restrict__ n_retained,
                                                                     int32_t* __restrict__ evicted) {
  constexpr int THREADS = FUSED_THREADS;
  using St = typename PickStream<T, D, G, THREADS, ROPE>::type;
  constexpr int WAVES = St::WAVES;
  constexpr int EP = 5 * 1024 / THREADS;       // covers budgets up to 5119 from registers
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* sm_acc = smem;
  float* sm_wm = sm_acc + WAVES * G * D;
  float* sm_wl = sm_wm + WAVES * G;
  float* sm_s = smem + St::LDS_FLOATS_FIXED;   // [G][cap]
  __shared__ float sm_sc[2];

  const int unit = blockIdx.x, tid = threadIdx.x;
  int* meta = p.meta + (size_t)unit * META_STRIDE;
  const T* knew = k_in + (size_t)unit * D;
  const T* vnew = v_in + (size_t)unit * D;
  const float* Su = p.S + (size_t)unit * p.cap;
  const int* PEu = p.PE + (size_t)unit * 2 * p.m;

  // Right after the first tile is requested: the old scores (held in registers until the epilogue),
  // the new row, and the retained list, which is known up front except for the one entry the
  // eviction decides (patched in the epilogue).
  float s_old[EP];
  constexpr int EP4 = (EP + 3) / 4;            // each thread writes runs of four retained entries
  int4 pe_pre[EP4];
  uint4 knew_r = make_uint4(0, 0, 0, 0), vnew_r = knew_r;
  Step st;
  int begin, end;
  St::run(p, unit, 0, q_in, knew, vnew, meta, sm_s, p.cap, sm_acc, sm_wm, sm_wl, st, begin, end, true,
          [&](const Step& s0) {
            constexpr int LPR = D / Storage<T>::EPL;
            if (tid >= THREADS - LPR) {
              knew_r = reinterpret_cast<const uint4*>(knew)[tid - (THREADS - LPR)];
              vnew_r = reinterpret_cast<const uint4*>(vnew)[tid - (THREADS - LPR)];
            }
#pragma unroll
            for (int x = 0; x < EP; ++x) {
              const int slot = tid + x * THREADS;
              s_old[x] = (slot < s0.n1 && slot != s0.fslot) ? Su[slot] : 0.f;
            }
#pragma unroll
            for (int x = 0; x < EP4; ++x) {
              const int i = 4 * (tid + x * THREADS);
              pe_pre[x] = make_int4(position_of(p, s0, PEu, i, -1, true), position_of(p, s0, PEu, i + 1, -1, true),
                                    position_of(p, s0, PEu, i + 2, -1, true), position_of(p, s0, PEu, i + 3, -1, true));
            }
          },
          [&]() {
            load_scope(p, st, p.E + (size_t)unit * 2 * p.m, PEu, p.R + (size_t)unit * max(p.n_recent, 1));
            int32_t* ret = retained + (size_t)unit * p.budget;
            const bool quads = (p.budget & 3) == 0 && (reinterpret_cast<uintptr_t>(retained) & 15) == 0;
#pragma unroll
            for (int x = 0; x < EP4; ++x) {
              const int i = 4 * (tid + x * THREADS);
              if (quads) {
                if (i < p.budget) *reinterpret_cast<int4*>(ret + i) = pe_pre[x];
              } else {
                if (i < p.budget) ret[i] = pe_pre[x].x;
                if (i + 1 < p.budget) ret[i + 1] = pe_pre[x].y;
                if (i + 2 < p.budget) ret[i + 2] = pe_pre[x].z;
                if (i + 3 < p.budget) ret[i + 3] = pe_pre[x].w;
              }
            }
            for (int i = tid + 4 * EP4 * THREADS; i < p.budget; i += THREADS)
              ret[i] = position_of(p, st, PEu, i, -1, true);
          });
  __syncthreads();

  float M[G], invL[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float L;
    merge_stats(sm_wm + g, sm_wl + g, WAVES, G, M[g], L);
    invL[g] = 1.0f / L;
  }
  // the thread that wrote the retained entry the decision fills in
  const int ret_i = p.n_sink + st.j0;
  const int ret_owner = (ret_i < 4 * EP4 * THREADS ? ret_i / 4 : ret_i) % THREADS;
  epilogue<T, D, G, THREADS, EP>(p, unit, st, M, invL, [&](int g, int slot) { return sm_s[(size_t)g * p.cap + slot]; },
                                 s_old, knew_r, vnew_r, sm_sc, sm_s, retained, n_retained, evicted, meta, ret_owner);
  // the attention output: last, and by the highest threads, whose waves have no bookkeeping stores to issue
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  for (int i = THREADS - 1 - tid; i < G * D; i += THREADS) {
    const int g = i / D, col = i % D;
    float a = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) a += sm_acc[(w * G + g) * D + col] * fast_exp2(sm_wm[w * G + g] - M[g]);
    out[((size_t)b * p.H + (size_t)kvh * G + g) * D + col] = a * invL[g];
  }
}

template <typename T, int D, int G, int ROPE>
__global__ __launch_bounds__(SPLIT_THREADS) void decode_split_kernel(Params p, const T* __restrict__ q_in,
                                                                     const T* __restrict__ k_in,
                                                                     const T* __restrict__ v_in) {
  constexpr int THREADS = SPLIT_THREADS;
  using St = typename PickStream<T, D, G, THREADS, ROPE>::type;
  constexpr int WAVES = St::WAVES;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* sm_acc = smem;
  float* sm_wm = sm_acc + WAVES * G * D;
  float* sm_wl = sm_wm + WAVES * G;
  float* sm_s = smem + St::LDS_FLOATS_FIXED;   // [G][rows_per_split]

  const int split = blockIdx.x, unit = blockIdx.y, tid = threadIdx.x;
  const int* meta = p.meta + (size_t)unit * META_STRIDE;
  Step st;
  int begin, end;
  St::run(p, unit, split * p.rows_per_split, q_in, k_in + (size_t)unit * D, v_in + (size_t)unit * D, meta, sm_s,
          p.rows_per_split, sm_acc, sm_wm, sm_wl, st, begin, end, false, [](const Step&) {}, []() {});
  __syncthreads();
  float* part = p.partial + ((size_t)unit * p.nsplit + split) * G * (D + 2);
  for (int i = tid; i < G * D; i += THREADS) {
    const int g = i / D, col = i % D;
    float M, L;
    merge_stats(sm_wm + g, sm_wl + g, WAVES, G, M, L);
    float a = 0.f;
    for (int w = 0; w < WAVES; ++w) a += sm_acc[(w * G + g) * D + col] * fast_exp2(sm_wm[w * G + g] - M);
    part[(size_t)g * (D + 2) + col] = a;
    if (col == 0) { part[(size_t)g * (D + 2) + D] = M; part[(size_t)g * (D + 2) + D + 1] = L; }
  }
  float* lg = p.logits + (size_t)unit * G * p.cap;
  for (int g = 0; g < G; ++g)
    for (int r = tid; r < end - begin; r += THREADS) lg[(size_t)g * p.cap + begin + r] = sm_s[(size_t)g * p.rows_per_split + r];
}

// Second kernel of the SPLIT shape: one workgroup per unit.  Latency is all that matters here, so
// everything the epilogue needs (the slices' logits, the old scores, the tree positions) is requested in one
// go right after the bookkeeping words, the logits are parked in LDS, and from there on the kernel is the
// tail of the fused one.
template <typename T, int D, int G, bool LOGITS_IN_LDS>
__global__ __launch_bounds__(MERGE_THREADS) void decode_merge_kernel(Params p, const T* __restrict__ k_in,
                                                                     const T* __restrict__ v_in,
                                                                     float* __restrict__ out,
                                                                     int32_t* __restrict__ retained,
                                                                     int32_t* __restrict__ n_retained,
                                                                     int32_t* __restrict__ evicted) {
  constexpr int THREADS = MERGE_THREADS;
  // slots / list entries per thread served from registers (none when the logits do not fit in LDS: huge budgets)
  constexpr int EP = LOGITS_IN_LDS ? 5 * 1024 / THREADS : 0;
  constexpr int LPR = D / Storage<T>::EPL;
  extern __shared__ __attribute__((aligned(16))) float smem[];              // [G][cap] logits
  __shared__ float sm_sc[2];
  const int unit = blockIdx.x, tid = threadIdx.x;
  int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int* PEu = p.PE + (size_t)unit * 2 * p.m;
  const float* Su = p.S + (size_t)unit * p.cap;
  const float* lg = p.logits + (size_t)unit * G * p.cap;
  Step st = load_meta(p, meta);

  float s_old[EP > 0 ? EP : 1], lreg[EP > 0 ? EP : 1][G];
  int pe_pre[EP > 0 ? EP : 1];
#pragma unroll
  for (int x = 0; x < EP; ++x) {
    const int slot = tid + x * THREADS;
    const bool live = slot < st.n1;
    s_old[x] = (live && slot != st.fslot) ? Su[slot] : 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) lreg[x][g] = live ? lg[(size_t)g * p.cap + slot] : 0.f;
    pe_pre[x] = position_of(p, st, PEu, slot, -1, true);
  }
  uint4 knew_r = make_uint4(0, 0, 0, 0), vnew_r = knew_r;
  if (tid >= THREADS - LPR) {
    knew_r = reinterpret_cast<const uint4*>(k_in + (size_t)unit * D)[tid - (THREADS - LPR)];
    vnew_r = reinterpret_cast<const uint4*>(v_in + (size_t)unit * D)[tid - (THREADS - LPR)];
  }
  load_scope(p, st, p.E + (size_t)unit * 2 * p.m, PEu, p.R + (size_t)unit * max(p.n_recent, 1));

  const float* parts = p.partial + (size_t)unit * p.nsplit * G * (D + 2);
  float M[G], invL[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float L;
    merge_stats(parts + (size_t)g * (D + 2) + D, parts + (size_t)g * (D + 2) + D + 1, p.nsplit, G * (D + 2), M[g], L);
    invL[g] = 1.0f / L;
  }
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  for (int i = tid; i < G * D; i += THREADS) {
    const int g = i / D, col = i % D;
    float a = 0.f;
    for (int s = 0; s < p.nsplit; ++s) {
      const float* ps = parts + ((size_t)s * G + g) * (D + 2);
      a += ps[col] * fast_exp2(ps[D] - M[g]);
    }
    out[((size_t)b * p.H + (size_t)kvh * G + g) * D + col] = a * invL[g];
  }
  // logits -> LDS, retained list (all but the entry the decision fills)
  int32_t* ret = retained + (size_t)unit * p.budget;
#pragma unroll
  for (int x = 0; x < EP; ++x) {
    const int slot = tid + x * THREADS;
    if (slot < p.cap) {
#pragma unroll
      for (int g = 0; g < G; ++g) smem[(size_t)g * p.cap + slot] = lreg[x][g];
    }
    if (slot < p.budget) ret[slot] = pe_pre[x];
  }
  if constexpr (LOGITS_IN_LDS) {
    for (int slot = tid + EP * THREADS; slot < st.n1; slot += THREADS)
      for (int g = 0; g < G; ++g) smem[(size_t)g * p.cap + slot] = lg[(size_t)g * p.cap + slot];
    for (int i = tid + EP * THREADS; i < p.budget; i += THREADS) ret[i] = position_of(p, st, PEu, i, -1, true);
    __syncthreads();
    epilogue<T, D, G, THREADS, EP>(p, unit, st, M, invL, [&](int g, int slot) { return smem[(size_t)g * p.cap + slot]; },
                                   s_old, knew_r, vnew_r, sm_sc, smem, retained, n_retained, evicted, meta,
                                   (p.n_sink + st.j0) % THREADS);
  } else {
    (void)ret;
    epilogue<T, D, G, THREADS, 0>(p, unit, st, M, invL, [&](int g, int slot) { return lg[(size_t)g * p.cap + slot]; },
                                  nullptr, knew_r, vnew_r, sm_sc, nullptr, retained, n_retained, evicted, meta, -1);
  }
}

template <typename T, int D, int G, int ROPE>
int launch_decode_g(const Params& p, const void* q, const void* k, const void* v, float* out, int32_t* retained,
                    int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  const T* qt = (const T*)q;
  const T* kt = (const T*)k;
  const T* vt = (const T*)v;
  if (p.nsplit == 1) {
    using St = typename PickStream<T, D, G, FUSED_THREADS, ROPE>::type;
    const size_t lds = St::lds_floats(p.cap, p.cap) * sizeof(float);
    if (lds > LDS_LIMIT) return TREEKV_EUNSUPPORTED;
    auto kern = decode_fused_kernel<T, D, G, ROPE>;
    if (lds > 48 * 1024 &&
        hip_failed(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
      return TREEKV_EHIP;
    hipLaunchKernelGGL(kern, dim3(p.U), dim3(FUSED_THREADS), lds, s, p, qt, kt, vt, out, retained, n_retained, evicted);
  } else {
    using St = typename PickStream<T, D, G, SPLIT_THREADS, ROPE>::type;
    const size_t lds = St::lds_floats(p.cap, p.rows_per_split) * sizeof(float);
    if (lds > LDS_LIMIT) return TREEKV_EUNSUPPORTED;
    auto kern = decode_split_kernel<T, D, G, ROPE>;
    if (lds > 48 * 1024 &&
        hip_failed(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)))
      return TREEKV_EHIP;
    hipLaunchKernelGGL(kern, dim3(p.nsplit, p.U), dim3(SPLIT_THREADS), lds, s, p, qt, kt, vt);
    const size_t mlds = (size_t)G * p.cap * sizeof(float);
    if (mlds <= LDS_LIMIT) {
      auto merge = decode_merge_kernel<T, D, G, true>;
      if (mlds > 48 * 1024 &&
          hip_failed(hipFuncSetAttribute((const void*)merge, hipFuncAttributeMaxDynamicSharedMemorySize, (int)mlds)))
        return TREEKV_EHIP;
      hipLaunchKernelGGL(merge, dim3(p.U), dim3(MERGE_THREADS), mlds, s, p, kt, vt, out, retained, n_retained, evicted);
    } else {
      hipLaunchKernelGGL((decode_merge_kernel<T, D, G, false>), dim3(p.U), dim3(MERGE_THREADS), 0, s, p, kt, vt, out,
                         retained, n_retained, evicted);
    }
  }
  return finish_launch();
}

template <typename T, int D>
int launch_decode_d(const Params& p, const void* q, const void* k, const void* v, float* out, int32_t* retained,
                    int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  const int mode = rope_mode<T, D>(p);
#define TKV_LAUNCH_G(G_)                                                                                              \
  case G_:                                                                                                            \
    return mode == ROPE_LDS   ? launch_decode_g<T, D, G_, ROPE_LDS>(p, q, k, v, out, retained, n_retained, evicted, s) \
           : mode == ROPE_MEM ? launch_decode_g<T, D, G_, ROPE_MEM>(p, q, k, v, out, retained, n_retained, evicted, s) \
                              : launch_decode_g<T, D, G_, ROPE_OFF>(p, q, k, v, out, retained, n_retained, evicted, s);
  switch (p.G) {
    TKV_LAUNCH_G(1)
    TKV_LAUNCH_G(2)
    TKV_LAUNCH_G(4)
    TKV_LAUNCH_G(8)
    default: return TREEKV_EUNSUPPORTED;
  }
#undef TKV_LAUNCH_G
}

// LDS bytes the streaming kernel of the current shape (fused when nsplit == 1) asks for; 0 if no kernel exists.
template <typename T, int D, int G, int ROPE>
size_t stream_lds_g(const Params& p) {
  using Sf = typename PickStream<T, D, G, FUSED_THREADS, ROPE>::type;
  using Ss = typename PickStream<T, D, G, SPLIT_THREADS, ROPE>::type;
  return (p.nsplit == 1 ? Sf::lds_floats(p.cap, p.cap) : Ss::lds_floats(p.cap, p.rows_per_split)) * sizeof(float);
}
template <typename T, int D>
size_t stream_lds_d(const Params& p) {
  const int mode = rope_mode<T, D>(p);
#define TKV_LDS_G(G_)                                                   \
  case G_:                                                              \
    return mode == ROPE_LDS   ? stream_lds_g<T, D, G_, ROPE_LDS>(p)     \
           : mode == ROPE_MEM ? stream_lds_g<T, D, G_, ROPE_MEM>(p)     \
                              : stream_lds_g<T, D, G_, ROPE_OFF>(p);
  switch (p.G) {
    TKV_LDS_G(1)
    TKV_LDS_G(2)
    TKV_LDS_G(4)
    TKV_LDS_G(8)
    default: return 0;
  }
#undef TKV_LDS_G
}

}  // namespace

bool decode_shape_fits(const Params& p) {
  size_t b = 0;
  if (p.dtype == TREEKV_BF16) b = p.D == 128 ? stream_lds_d<uint16_t, 128>(p) : p.D == 64 ? stream_lds_d<uint16_t, 64>(p) : 0;
  else if (p.dtype == TREEKV_F32) b = p.D == 128 ? stream_lds_d<float, 128>(p) : p.D == 64 ? stream_lds_d<float, 64>(p) : 0;
  return b != 0 && b <= LDS_LIMIT;
}

int launch_decode(const Params& p, const void* q, const void* k, const void* v, float* out, int32_t* retained,
                  int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  if (p.dtype == TREEKV_BF16) {
    if (p.D == 128) return launch_decode_d<uint16_t, 128>(p, q, k, v, out, retained, n_retained, evicted, s);
    if (p.D == 64) return launch_decode_d<uint16_t, 64>(p, q, k, v, out, retained, n_retained, evicted, s);
  } else if (p.dtype == TREEKV_F32) {
    if (p.D == 128) return launch_decode_d<float, 128>(p, q, k, v, out, retained, n_retained, evicted, s);
    if (p.D == 64) return launch_decode_d<float, 64>(p, q, k, v, out, retained, n_retained, evicted, s);
  }
  return TREEKV_EUNSUPPORTED;
}

}  // namespace tkv
