// Decode step of TreeKV for gfx950: one launch does Algorithm 1, lines 4-17, for every
// (batch, KV head) unit.
//
// Work split.  grid = (nsplit, U).  Workgroup (s, u) streams a contiguous range of unit u's
// cache slots: K rows for the logits, V rows for the output, both as 16-byte lane loads
// (a wave covers 64/LPR whole rows per load instruction, LPR lanes per row).  Each lane group
// keeps an online-softmax state (running max, sum, output accumulator) in registers, so the
// K and V streams interleave and no barrier sits inside the loop.  The scaled logits go to a
// small scratch array; the group states are merged per wave (shuffles), per workgroup (LDS)
// and written as one partial per workgroup.
//
// The last workgroup of a unit to finish (ticket counter) merges the partials, writes the
// output, turns the stored logits into normalised probabilities and adds them to the slot
// scores (lines 7-8), takes the eviction decision (lines 9-17) and writes the retained
// positions.  Nothing waits on another workgroup, so every wave exits.
//
// The new token's k and v are read from the caller's buffers by whichever workgroup owns
// the free slot's index; the last workgroup copies them into the cache afterwards.

#include "treekv_internal.h"

namespace tkv {

namespace {

constexpr int DEC_THREADS = 256;
constexpr int DEC_WAVES = DEC_THREADS / 64;
constexpr int DEC_UNROLL = 4;
constexpr float NEG_BIG = -1.0e30f;

template <typename T, int D, int G>
__global__ __launch_bounds__(DEC_THREADS) void decode_kernel(Params p, const T* __restrict__ q_in,
                                                             const T* __restrict__ k_in,
                                                             const T* __restrict__ v_in,
                                                             float* __restrict__ out,
                                                             int32_t* __restrict__ retained,
                                                             int32_t* __restrict__ n_retained,
                                                             int32_t* __restrict__ evicted) {
  constexpr int EPL = Storage<T>::EPL;       // elements per lane load
  constexpr int LPR = D / EPL;               // lanes per row
  constexpr int RPL = 64 / LPR;              // rows per wave load
  constexpr int TILE = RPL * DEC_UNROLL;     // rows per wave iteration
  static_assert(LPR >= 1 && LPR <= 64 && (64 % LPR) == 0, "row must fit a wave");

  const int split = blockIdx.x, unit = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane % LPR, ri = lane / LPR;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;

  int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int n = meta[META_N];
  const int fslot = meta[META_FREE];
  const int n1 = n + 1;                      // slots [0, n1) take part; slot fslot is the new token

  const T* Ku = (const T*)p.K + (size_t)unit * p.cap * D;
  const T* Vu = (const T*)p.V + (size_t)unit * p.cap * D;
  const T* knew = k_in + (size_t)unit * D;
  const T* vnew = v_in + (size_t)unit * D;
  float* lg = p.logits + (size_t)unit * G * p.cap;

  // this lane's slice of the G query vectors
  float qf[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const T* qp = q_in + ((size_t)b * p.H + (size_t)kvh * G + g) * D + li * EPL;
    Storage<T>::widen(*reinterpret_cast<const uint4*>(qp), qf[g]);
  }

  // row range of this workgroup, a multiple of RPL so that lane groups stay aligned
  int per = (n1 + p.nsplit - 1) / p.nsplit;
  per = (per + RPL - 1) / RPL * RPL;
  const int begin = split * per;
  const int end = min(n1, begin + per);

  float m_run[G], l_run[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = NEG_BIG; l_run[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  for (int base = begin + wave * TILE; base < end; base += DEC_WAVES * TILE) {
    uint4 kr[DEC_UNROLL], vr[DEC_UNROLL];
    bool ok[DEC_UNROLL];
    int rows[DEC_UNROLL];
#pragma unroll
    for (int u = 0; u < DEC_UNROLL; ++u) {
      const int row = base + u * RPL + ri;
      ok[u] = row < end;
      const int rr = ok[u] ? row : begin;    // begin < end here, so this is a live row
      rows[u] = row;
      const T* kp = (rr == fslot) ? knew : Ku + (size_t)rr * D;
      const T* vp = (rr == fslot) ? vnew : Vu + (size_t)rr * D;
      kr[u] = *reinterpret_cast<const uint4*>(kp + li * EPL);
      vr[u] = *reinterpret_cast<const uint4*>(vp + li * EPL);
    }
    float s[DEC_UNROLL][G];
#pragma unroll
    for (int u = 0; u < DEC_UNROLL; ++u) {
      float kf[EPL];
      Storage<T>::widen(kr[u], kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d = fmaf(kf[e], qf[g][e], d);
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off, 64);
        d *= p.scale_log2e;
        s[u][g] = d;
        if (li == 0 && ok[u]) lg[(size_t)g * p.cap + rows[u]] = d;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mx = m_run[g];
#pragma unroll
      for (int u = 0; u < DEC_UNROLL; ++u) mx = ok[u] ? fmaxf(mx, s[u][g]) : mx;
      const float corr = fast_exp2(m_run[g] - mx);
      m_run[g] = mx;
      l_run[g] *= corr;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
#pragma unroll
      for (int u = 0; u < DEC_UNROLL; ++u) {
        const float pr = ok[u] ? fast_exp2(s[u][g] - mx) : 0.f;
        s[u][g] = pr;
        l_run[g] += pr;
      }
    }
#pragma unroll
    for (int u = 0; u < DEC_UNROLL; ++u) {
      float vf[EPL];
      Storage<T>::widen(vr[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(s[u][g], vf[e], acc[g][e]);
    }
  }

  // merge the RPL lane groups of the wave
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = __shfl_xor(m_run[g], off, 64);
      const float lo = __shfl_xor(l_run[g], off, 64);
      const float mx = fmaxf(m_run[g], mo);
      const float ca = fast_exp2(m_run[g] - mx), cb = fast_exp2(mo - mx);
      l_run[g] = l_run[g] * ca + lo * cb;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float ao = __shfl_xor(acc[g][e], off, 64);
        acc[g][e] = acc[g][e] * ca + ao * cb;
      }
      m_run[g] = mx;
    }
  }

  // merge the waves of the workgroup through LDS
  __shared__ float sm_acc[DEC_WAVES][G][D];
  __shared__ float sm_m[DEC_WAVES][G], sm_l[DEC_WAVES][G];
  __shared__ float sm_M[G], sm_invL[G];
  __shared__ int sm_i[8];
  __shared__ float sm_sc[2];
  if (ri == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_acc[wave][g][li * EPL + e] = acc[g][e];
      if (li == 0) { sm_m[wave][g] = m_run[g]; sm_l[wave][g] = l_run[g]; }
    }
  }
  __syncthreads();
  float* part = p.partial + ((size_t)unit * p.nsplit + split) * G * (D + 2);
  for (int i = tid; i < G * D; i += DEC_THREADS) {
    const int g = i / D, col = i % D;
    float mx = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < DEC_WAVES; ++w) mx = fmaxf(mx, sm_m[w][g]);
    float a = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < DEC_WAVES; ++w) {
      const float cw = fast_exp2(sm_m[w][g] - mx);
      a += sm_acc[w][g][col] * cw;
      l += sm_l[w][g] * cw;
    }
    part[(size_t)g * (D + 2) + col] = a;
    if (col == 0) { part[(size_t)g * (D + 2) + D] = mx; part[(size_t)g * (D + 2) + D + 1] = l; }
  }

  // ticket: the last workgroup of the unit carries on
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const unsigned ticket = atomicAdd(&p.counter[unit], 1u);
    sm_i[0] = (ticket == (unsigned)p.nsplit - 1u);
  }
  __syncthreads();
  if (!sm_i[0]) return;
  __threadfence();

  // ---- merge the partials: output, global max and sum per query head ----
  const float* parts = p.partial + (size_t)unit * p.nsplit * G * (D + 2);
  for (int i = tid; i < G * D; i += DEC_THREADS) {
    const int g = i / D, col = i % D;
    float mx = NEG_BIG;
    for (int sidx = 0; sidx < p.nsplit; ++sidx)
      mx = fmaxf(mx, ld_agent(parts + ((size_t)sidx * G + g) * (D + 2) + D));
    float a = 0.f, l = 0.f;
    for (int sidx = 0; sidx < p.nsplit; ++sidx) {
      const float* ps = parts + ((size_t)sidx * G + g) * (D + 2);
      const float cw = fast_exp2(ld_agent(ps + D) - mx);
      a += ld_agent(ps + col) * cw;
      l += ld_agent(ps + D + 1) * cw;
    }
    out[((size_t)b * p.H + (size_t)kvh * G + g) * D + col] = a / l;
    if (col == 0) { sm_M[g] = mx; sm_invL[g] = 1.0f / l; }
  }

  // ---- bookkeeping that does not depend on the scores (one thread) ----
  float* Su = p.S + (size_t)unit * p.cap;
  int* posu = p.pos + (size_t)unit * p.cap;
  int* Eu = p.E + (size_t)unit * 2 * p.m;
  int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
  const int t = meta[META_T];
  const bool evict = n1 > p.budget;
  if (tid == 0) {
    int j = meta[META_J], rhead = meta[META_RHEAD];
    int sl = -1, sr = -1;
    if (evict) {
      int newcomer = fslot;
      if (p.n_recent > 0) {                  // the new token enters the recent window; its oldest
        newcomer = Ru[rhead];                // member moves into the tree region
        Ru[rhead] = fslot;
        rhead = rhead + 1 == p.n_recent ? 0 : rhead + 1;
      }
      Eu[p.m + j] = newcomer;
      sl = Eu[2 * j];
      sr = Eu[2 * j + 1];
    }
    sm_i[1] = sl; sm_i[2] = sr; sm_i[3] = j; sm_i[4] = rhead;
    posu[fslot] = t;
  }
  __syncthreads();

  // ---- lines 7-8: S = (S u {0}) + a, with a = exp2(logit - M) / L summed over the group ----
  const int scope_l = sm_i[1], scope_r = sm_i[2];
  for (int jj = tid; jj < n1; jj += DEC_THREADS) {
    float a = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) a += fast_exp2(ld_agent(lg + (size_t)g * p.cap + jj) - sm_M[g]) * sm_invL[g];
    const float sn = (jj == fslot ? 0.f : Su[jj]) + a;
    Su[jj] = sn;
    if (jj == scope_l) sm_sc[0] = sn;
    if (jj == scope_r) sm_sc[1] = sn;
  }
  // the new token's k, v become cache rows
  {
    T* Kw = (T*)p.K + ((size_t)unit * p.cap + fslot) * D;
    T* Vw = (T*)p.V + ((size_t)unit * p.cap + fslot) * D;
    for (int i = tid; i < D; i += DEC_THREADS) { Kw[i] = knew[i]; Vw[i] = vnew[i]; }
  }
  __syncthreads();

  // ---- lines 9-17: compare the scope's averaged scores, evict, advance ----
  if (tid == 0) {
    int j = sm_i[3];
    int n_new = n1, f_new = n1, ev_pos = -1;
    if (evict) {
      const int pl = posu[scope_l], pr = posu[scope_r];
      const float bl = sm_sc[0] / (float)(t - pl + 1);
      const float br = sm_sc[1] / (float)(t - pr + 1);
      const bool drop_right = (p.flags & TREEKV_KEEP_LEFT) || (bl > br);
      const int loser = drop_right ? scope_r : scope_l;
      Eu[j] = drop_right ? scope_l : scope_r;
      ev_pos = drop_right ? pr : pl;
      f_new = loser;
      n_new = p.budget;
      j = j + 1 == p.m ? 0 : j + 1;
    }
    meta[META_N] = n_new;
    meta[META_FREE] = f_new;
    meta[META_J] = j;
    meta[META_RHEAD] = sm_i[4];
    meta[META_T] = t + 1;
    p.counter[unit] = 0;
    sm_i[5] = n_new; sm_i[6] = j;
    if (evicted) evicted[unit] = ev_pos;
    if (n_retained) n_retained[unit] = n_new;
  }
  __syncthreads();

  // ---- retained positions in ascending order ----
  {
    const int n_new = sm_i[5], j_done = sm_i[6], rhead = sm_i[4];
    int32_t* ret = retained + (size_t)unit * p.budget;
    if (n_new < p.budget) {
      for (int i = tid; i < p.budget; i += DEC_THREADS) ret[i] = i < n_new ? i : -1;
    } else {
      // after the round's last eviction META_J wraps to 0, which reads the same as m done
      for (int i = tid; i < p.budget; i += DEC_THREADS)
        ret[i] = posu[logical_to_slot(p, Eu, Ru, rhead, j_done, i)];
    }
  }
}

template <typename T, int D>
int launch_decode_g(const Params& p, const void* q, const void* k, const void* v, float* out, int32_t* retained,
                    int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  dim3 grid(p.nsplit, p.U), block(DEC_THREADS);
#define TKV_LAUNCH(GV)                                                                                 \
  hipLaunchKernelGGL((decode_kernel<T, D, GV>), grid, block, 0, s, p, (const T*)q, (const T*)k,        \
                     (const T*)v, out, retained, n_retained, evicted)
  switch (p.G) {
    case 1: TKV_LAUNCH(1); break;
    case 2: TKV_LAUNCH(2); break;
    case 4: TKV_LAUNCH(4); break;
    case 8: TKV_LAUNCH(8); break;
    default: return TREEKV_EUNSUPPORTED;
  }
#undef TKV_LAUNCH
  return hipGetLastError() == hipSuccess ? TREEKV_OK : TREEKV_EHIP;
}

}  // namespace

int launch_decode(const Params& p, const void* q, const void* k, const void* v, float* out, int32_t* retained,
                  int32_t* n_retained, int32_t* evicted, hipStream_t s) {
  if (p.dtype == TREEKV_BF16) {
    if (p.D == 128) return launch_decode_g<uint16_t, 128>(p, q, k, v, out, retained, n_retained, evicted, s);
    if (p.D == 64) return launch_decode_g<uint16_t, 64>(p, q, k, v, out, retained, n_retained, evicted, s);
  } else if (p.dtype == TREEKV_F32) {
    if (p.D == 128) return launch_decode_g<float, 128>(p, q, k, v, out, retained, n_retained, evicted, s);
    if (p.D == 64) return launch_decode_g<float, 64>(p, q, k, v, out, retained, n_retained, evicted, s);
  }
  return TREEKV_EUNSUPPORTED;
}

}  // namespace tkv
