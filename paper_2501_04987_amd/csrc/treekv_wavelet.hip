// Wavelet analysis behind the method (Sections 3.2-3.3): how much of the information gathered by attention,
// s[n] = a[n] * v[n], sits in each Haar frequency band, position by position.
//
// For the Haar pair the reconstruction from one level's detail coefficients alone has a closed form: over a block
// of 2^l positions Rec(D_l) is +-2^-l * (sum of the block's first half - sum of its second half), so its magnitude
// is one number per block and column.  The multi-level decomposition is therefore a tree of pairwise sums over 32
// consecutive rows (five levels), and the kernel is one streaming read of V: a wave takes 32 rows, a lane 16 bytes
// of a few consecutive rows (the low levels stay inside the lane, the top ones cross lanes by shuffles), the
// magnitudes are averaged over the d columns (lane-local, then across the lanes that share a row) and leave
// through a small LDS tile as whole rows of the output.
//
//   wavelet_components_kernel   grid (ceil(t / 512), heads) x 256 threads -> per_head [heads][levels][t]
//   wavelet_mean_kernel         grid ceil(levels * t / 32) x 1024 threads -> mean [levels][t], heads added in a fixed order

#include "treekv_internal.h"

namespace tkv {
namespace {

constexpr int WV_THREADS = 256;
constexpr int WV_WAVES = WV_THREADS / 64;
constexpr int WV_BLOCK = 32;          // rows per wave pass = 2^5, the deepest level
constexpr int WV_LEVELS = 5;
constexpr int WV_ITERS = 4;           // 32-row blocks a wave takes, 128 rows apart

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

template <typename T, int D>
__global__ __launch_bounds__(WV_THREADS) void wavelet_components_kernel(const float* __restrict__ a,
                                                                        const T* __restrict__ V, int t, int levels,
                                                                        float* __restrict__ per_head) {
  constexpr int EPL = Storage<T>::EPL;
  constexpr int LPR = D / EPL;            // lanes that share a row
  constexpr int RG = 64 / LPR;            // row groups of a wave
  constexpr int RPLN = WV_BLOCK / RG;     // consecutive rows of one lane
  constexpr int IN = ilog2(RPLN);         // levels that stay inside a lane
  static_assert(RG * RPLN == WV_BLOCK && (1 << IN) == RPLN && IN >= 1 && IN < WV_LEVELS, "shape");
  __shared__ float tile[WV_WAVES][WV_LEVELS][WV_BLOCK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane % LPR, ri = lane / LPR;
  const int head = blockIdx.y;
  const T* Vh = V + (size_t)head * t * D;
  const float* ah = a + (size_t)head * t;
  constexpr int STRIDE = WV_WAVES * WV_BLOCK;                      // rows a workgroup covers per iteration
  const int first = blockIdx.x * WV_ITERS * STRIDE + wave * WV_BLOCK;   // wave uniform

  // the rows of one block: 16 bytes of V and the weight per row, requested one block ahead of their use
  uint4 raw[RPLN], raw_next[RPLN];
  float w[RPLN], w_next[RPLN];
  auto request = [&](uint4 (&r)[RPLN], float (&wt)[RPLN], int base) {
#pragma unroll
    for (int j = 0; j < RPLN; ++j) {
      const int row = base + ri * RPLN + j;
      const int rc = min(row, t - 1);
      r[j] = *reinterpret_cast<const uint4*>(Vh + (size_t)rc * D + li * EPL);
      wt[j] = row < t ? ah[rc] : 0.f;                            // rows past the end count as zero
    }
  };
  if (first < t) request(raw, w, first);
#pragma unroll
  for (int it = 0; it < WV_ITERS; ++it) {
    const int base = first + it * STRIDE;
    const bool live = base < t;                                    // wave uniform
    if (it + 1 < WV_ITERS && base + STRIDE < t) request(raw_next, w_next, base + STRIDE);
    if (live) {
      // s = a o V for this lane's rows and columns
      float x[RPLN][EPL];
#pragma unroll
      for (int j = 0; j < RPLN; ++j) {
        float vf[EPL];
        Storage<T>::widen(raw[j], vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) x[j][e] = w[j] * vf[e];
      }
      // levels inside the lane: pairwise differences and sums; |difference| added over the lane's columns
      float mag_in[RPLN];                 // RPLN >> l entries per level l = 1.., one level after the other
#pragma unroll
      for (int i = 0; i < RPLN; ++i) mag_in[i] = 0.f;
      float top[EPL];                     // sum of the lane's rows, per column
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        float s[RPLN];
#pragma unroll
        for (int j = 0; j < RPLN; ++j) s[j] = x[j][e];
        int off = 0;
#pragma unroll
        for (int l = 1; l <= IN; ++l) {
          const int n = RPLN >> l;
#pragma unroll
          for (int m = 0; m < n; ++m) {
            const float lo = s[2 * m], hi = s[2 * m + 1];
            mag_in[off + m] += fabsf(lo - hi);
            s[m] = lo + hi;
          }
          off += n;
        }
        top[e] = s[0];
      }
      // levels across row groups
      float mag_x[WV_LEVELS - IN];
#pragma unroll
      for (int l = 0; l < WV_LEVELS - IN; ++l) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const float other = __shfl_xor(top[e], LPR << l, 64);
          acc += fabsf(top[e] - other);
          top[e] += other;
        }
        mag_x[l] = acc;
      }
      // add over the lanes that share the rows
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) {
#pragma unroll
        for (int i = 0; i < RPLN - 1; ++i) mag_in[i] += __shfl_xor(mag_in[i], o, 64);
#pragma unroll
        for (int l = 0; l < WV_LEVELS - IN; ++l) mag_x[l] += __shfl_xor(mag_x[l], o, 64);
      }
      // |Rec(D_l)| = 2^-l |first half - second half|, the same for all 2^l rows of the block; mean over the D columns
      if (li == 0) {
        int off = 0;
#pragma unroll
        for (int l = 1; l <= IN; ++l) {
          const int n = RPLN >> l;
          const float f = 1.0f / (float)((1 << l) * D);
#pragma unroll
          for (int m = 0; m < n; ++m)
#pragma unroll
            for (int r = 0; r < (1 << l); ++r) tile[wave][l - 1][ri * RPLN + (m << l) + r] = mag_in[off + m] * f;
          off += n;
        }
#pragma unroll
        for (int l = 0; l < WV_LEVELS - IN; ++l) {
          const float f = 1.0f / (float)((1 << (IN + 1 + l)) * D);
#pragma unroll
          for (int r = 0; r < RPLN; ++r) tile[wave][IN + l][ri * RPLN + r] = mag_x[l] * f;
        }
      }
      // the tile is this wave's own: written and read by the same wave, in program order
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      for (int i = lane; i < levels * WV_BLOCK; i += 64) {
        const int l = i / WV_BLOCK, r = i % WV_BLOCK;
        if (base + r < t) per_head[((size_t)head * levels + l) * t + base + r] = tile[wave][l][r];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    if (it + 1 < WV_ITERS) {
#pragma unroll
      for (int j = 0; j < RPLN; ++j) { raw[j] = raw_next[j]; w[j] = w_next[j]; }
    }
  }
}

// Mean over the heads: a workgroup owns 32 adjacent outputs (whole 128-byte lines); 32 head lanes each add every 32nd head, then a fixed
// tree over the lanes: the order of the additions depends on nothing but `heads`.
constexpr int MEAN_COLS = 32, MEAN_LANES = 32;
__global__ __launch_bounds__(MEAN_COLS * MEAN_LANES) void wavelet_mean_kernel(const float* __restrict__ per_head,
                                                                              int heads, int n, float* __restrict__ mean) {
  __shared__ float red[MEAN_LANES][MEAN_COLS];
  const int tx = threadIdx.x % MEAN_COLS, ty = threadIdx.x / MEAN_COLS;
  const int i = blockIdx.x * MEAN_COLS + tx;
  float acc = 0.f;
  if (i < n)
#pragma unroll 8
    for (int h = ty; h < heads; h += MEAN_LANES) acc += per_head[(size_t)h * n + i];
  red[ty][tx] = acc;
  __syncthreads();
  for (int half = MEAN_LANES / 2; half >= 1; half >>= 1) {
    if (ty < half) red[ty][tx] += red[ty + half][tx];
    __syncthreads();
  }
  if (ty == 0 && i < n) mean[i] = red[0][tx] / (float)heads;
}

template <typename T, int D>
void launch_components(const float* a, const void* V, int heads, int t, int levels, float* per_head, hipStream_t s) {
  const int rows = WV_BLOCK * WV_WAVES * WV_ITERS;
  const int blocks = (t + rows - 1) / rows;
  hipLaunchKernelGGL((wavelet_components_kernel<T, D>), dim3(blocks, heads), dim3(WV_THREADS), 0, s, a, (const T*)V, t,
                     levels, per_head);
}

}  // namespace

int launch_wavelet(const float* a, const void* V, int dtype, int heads, int t, int d, int levels, float* per_head,
                   float* mean, hipStream_t s) {
  if (dtype == TREEKV_BF16 && d == 128) launch_components<uint16_t, 128>(a, V, heads, t, levels, per_head, s);
  else if (dtype == TREEKV_BF16 && d == 64) launch_components<uint16_t, 64>(a, V, heads, t, levels, per_head, s);
  else if (dtype == TREEKV_F32 && d == 128) launch_components<float, 128>(a, V, heads, t, levels, per_head, s);
  else if (dtype == TREEKV_F32 && d == 64) launch_components<float, 64>(a, V, heads, t, levels, per_head, s);
  else return TREEKV_EUNSUPPORTED;
  if (mean) {
    const int n = levels * t;
    hipLaunchKernelGGL(wavelet_mean_kernel, dim3((n + MEAN_COLS - 1) / MEAN_COLS), dim3(MEAN_COLS * MEAN_LANES), 0, s, per_head, heads, n, mean);
  }
  return finish_launch();
}

}  // namespace tkv
