// Host side of the TreeKV C ABI: configuration checks, workspace carving, launches.
// Also the three small utility kernels (reset, score read-out, K/V gather).

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "treekv_internal.h"

// Scratch of treekv_decode_step_static: the split shape's logits and partial results, in the library's own image
// instead of the caller's workspace.  Every GPU the library runs on holds its own copy, at its own address, until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[TREEKV_STATIC_SCRATCH_BYTES];

struct treekv_ctx {
  treekv_config cfg;
  tkv::Params p;
  size_t ws_bytes;
  bool bound;
  char hip_err[256];
};

namespace tkv {
namespace {

constexpr size_t ALIGN = 256;
size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

size_t rope_rows(const Params& p) {
  const size_t chunk = (size_t)p.cap + p.max_chunk;
  return chunk > (size_t)p.max_prompt ? chunk : (size_t)p.max_prompt;
}

// Walks the workspace layout; with base == nullptr it only measures.
size_t carve(Params& p, char* base) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* ptr = base ? base + off : nullptr;
    off += align_up(bytes);
    return ptr;
  };
  const size_t esz = p.dtype == TREEKV_BF16 ? 2 : 4;
  const size_t U = p.U, cap = p.cap, ext = (size_t)p.cap + p.max_chunk;
  p.K = take(U * cap * p.D * esz);
  p.V = take(U * cap * p.D * esz);
  p.S = (float*)take(U * cap * 4);
  p.E = (int*)take(U * 2 * p.m * 4);
  p.PE = (int*)take(U * 2 * p.m * 4);
  p.R = (int*)take(U * (size_t)(p.n_recent > 0 ? p.n_recent : 1) * 4);
  p.meta = (int*)take(U * META_STRIDE * 4);
  p.logits = (float*)take(U * p.G * cap * 4);
  p.partial = (float*)take(U * p.nsplit * p.G * (size_t)(p.D + 2) * 4);
  const size_t cs_cols = (cap + 127) / 128 * 128 + ((size_t)p.max_chunk + 127) / 128 * 128;
  p.pf_colacc = (unsigned long long*)take(U * cs_cols * 8);
  p.pf_snew = (float*)take(U * (size_t)p.max_chunk * 4);
  p.pf_flag = (int*)take(U * ext * 4);
  p.pf_list = (int*)take(U * ext * 4);
  if (p.max_prompt > 0) {
    p.pp_tok = (float*)take(U * (size_t)p.max_prompt * 4);
    p.pp_beta = (float*)take(U * (size_t)p.max_prompt * 4);
    p.pp_stat = (float*)take(U * (size_t)PROMPT_MAX_SPLITS * 128 * 2 * 4);
    p.pp_kept = (int*)take(U * (size_t)p.budget * 4);
  }
  if (p.flags & TREEKV_POSITION_RERANK) {
    p.rope_tab = (float2*)take(rope_rows(p) * (size_t)(p.D / 2) * sizeof(float2));
    if (p.max_prompt > 0) p.pp_qrot = (uint16_t*)take(U * 2 * 128 * (size_t)p.D * 2);
    p.pf_krot = (uint16_t*)take(U * 2 * ext * p.D * 2);
    p.pf_qrot = (uint16_t*)take(2 * (size_t)p.B * p.max_chunk * p.H * p.D * 2);
  }
  return off;
}

__global__ void reset_kernel(Params p) {
  const int unit = blockIdx.x;
  int* meta = p.meta + (size_t)unit * META_STRIDE;
  int* Eu = p.E + (size_t)unit * 2 * p.m;
  int* PEu = p.PE + (size_t)unit * 2 * p.m;
  int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
  // While the cache fills, token i sits in slot i, so at the first eviction the tree region
  // is slots (and positions) n_sink .. n_sink+m-1 and the recent window the slots after it.
  for (int i = threadIdx.x; i < 2 * p.m; i += blockDim.x) Eu[i] = PEu[i] = i < p.m ? p.n_sink + i : 0;
  for (int i = threadIdx.x; i < p.n_recent; i += blockDim.x) Ru[i] = p.n_sink + p.m + i;
  for (int i = threadIdx.x; i < p.cap; i += blockDim.x) p.S[(size_t)unit * p.cap + i] = 0.f;
  const size_t cs_cols = (size_t)(p.cap + 127) / 128 * 128 + (size_t)(p.max_chunk + 127) / 128 * 128;
  for (size_t i = threadIdx.x; i < cs_cols; i += blockDim.x) p.pf_colacc[(size_t)unit * cs_cols + i] = 0;
  // Cache rows are always initialised memory: the decode kernel requests its first rows before it
  // knows how many are live, and multiplies what it did not need by zero.
  const size_t vecs = (size_t)p.cap * p.D * (p.dtype == TREEKV_BF16 ? 2 : 4) / 16;
  uint4* Kz = reinterpret_cast<uint4*>(p.K) + (size_t)unit * vecs;
  uint4* Vz = reinterpret_cast<uint4*>(p.V) + (size_t)unit * vecs;
  for (size_t i = threadIdx.x; i < vecs; i += blockDim.x) Kz[i] = Vz[i] = make_uint4(0, 0, 0, 0);
  if (threadIdx.x < META_STRIDE) meta[threadIdx.x] = 0;
}

// (cos, sin) of distance * base^(-2i/D) for every distance two cached tokens can have, in double precision.
__global__ void rope_table_kernel(Params p) {
  const size_t rows = (size_t)p.cap + p.max_chunk > (size_t)p.max_prompt ? (size_t)p.cap + p.max_chunk : (size_t)p.max_prompt;
  const size_t n = rows * (p.D / 2);
  for (size_t x = blockIdx.x * (size_t)blockDim.x + threadIdx.x; x < n; x += (size_t)gridDim.x * blockDim.x) {
    const int dist = (int)(x / (p.D / 2)), i = (int)(x % (p.D / 2));
    const double angle = (double)dist * pow((double)p.rope_base, -2.0 * (double)i / (double)p.D);
    p.rope_tab[x] = make_float2((float)cos(angle), (float)sin(angle));
  }
}

__global__ void scores_kernel(Params p, float* __restrict__ scores) {
  const int unit = blockIdx.x;
  const int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int n = meta[META_N], j = meta[META_J], rhead = meta[META_RHEAD];
  const int* Eu = p.E + (size_t)unit * 2 * p.m;
  const int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
  for (int i = threadIdx.x; i < p.budget; i += blockDim.x) {
    float s = 0.f;
    if (i < n) {
      const int slot = n < p.budget ? i : logical_to_slot(p, Eu, Ru, rhead, j, i);
      s = p.S[(size_t)unit * p.cap + slot];
    }
    scores[(size_t)unit * p.budget + i] = s;
  }
}

__global__ void gather_kv_kernel(Params p, uint4* __restrict__ Kout, uint4* __restrict__ Vout, int row_vec) {
  const int unit = blockIdx.y, i = blockIdx.x;   // one block per logical row
  const int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int n = meta[META_N], j = meta[META_J], rhead = meta[META_RHEAD];
  const int* Eu = p.E + (size_t)unit * 2 * p.m;
  const int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
  const size_t dst = ((size_t)unit * p.budget + i) * row_vec;
  if (i >= n) {
    for (int e = threadIdx.x; e < row_vec; e += blockDim.x) Kout[dst + e] = Vout[dst + e] = make_uint4(0, 0, 0, 0);
    return;
  }
  const int slot = n < p.budget ? i : logical_to_slot(p, Eu, Ru, rhead, j, i);
  const size_t src = ((size_t)unit * p.cap + slot) * row_vec;
  for (int e = threadIdx.x; e < row_vec; e += blockDim.x) {
    Kout[dst + e] = reinterpret_cast<const uint4*>(p.K)[src + e];
    Vout[dst + e] = reinterpret_cast<const uint4*>(p.V)[src + e];
  }
}

// ---- snapshots of a context's state (treekv_export_state / treekv_import_state) -------------------
// Byte offsets of the snapshot's arrays; every array starts on a 256-byte boundary.
treekv_state_layout state_layout(const Params& p) {
  treekv_state_layout l;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += align_up(bytes); return at; };
  const size_t esz = p.dtype == TREEKV_BF16 ? 2 : 4, U = p.U, c = p.budget;
  l.header = take(U * 4 * 4);
  l.positions = take(U * c * 4);
  l.slots = take(U * c * 4);
  l.S = take(U * c * 4);
  l.K = take(U * c * p.D * esz);
  l.V = take(U * c * p.D * esz);
  l.bytes = off;
  return l;
}

// Header, positions, slots and S of every unit, in position order (the K and V rows go through gather_kv_kernel).
__global__ void export_state_kernel(Params p, int* __restrict__ hdr, int* __restrict__ pos, int* __restrict__ slots,
                                    float* __restrict__ S) {
  const int unit = blockIdx.x;
  const int* meta = p.meta + (size_t)unit * META_STRIDE;
  const int n = meta[META_N], j = meta[META_J], rhead = meta[META_RHEAD], t = meta[META_T];
  const int* Eu = p.E + (size_t)unit * 2 * p.m;
  const int* PEu = p.PE + (size_t)unit * 2 * p.m;
  const int* Ru = p.R + (size_t)unit * max(p.n_recent, 1);
  if (threadIdx.x < 4) {
    const int h[4] = {n, t, j + 1, 0};
    hdr[(size_t)unit * 4 + threadIdx.x] = h[threadIdx.x];
  }
  for (int i = threadIdx.x; i < p.budget; i += blockDim.x) {
    int po = -1, sl = -1;
    float sc = 0.f;
    if (i < n) {
      po = sl = i;                        // while the cache fills, token i sits in slot i
      if (n == p.budget) {
        sl = logical_to_slot(p, Eu, Ru, rhead, j, i);
        const int k = i - p.n_sink;
        if (k >= p.m) po = t - p.n_recent + (k - p.m);
        else if (k >= 0) po = PEu[tree_index(k, j)];
      }
      sc = p.S[(size_t)unit * p.cap + sl];
    }
    const size_t o = (size_t)unit * p.budget + i;
    pos[o] = po; slots[o] = sl; S[o] = sc;
  }
}

// Checks one unit's snapshot and, if it describes a state Algorithm 1 can be in, rebuilds the unit's bookkeeping
// from it; a unit whose snapshot does not pass is left empty (as after a reset).  The slot every token's rows go to
// is left in pf_list[unit][0 .. budget) for import_rows_kernel (-1: no row to copy).
__global__ __launch_bounds__(256) void import_state_kernel(Params p, const int* __restrict__ hdr,
                                                           const int* __restrict__ pos, const int* __restrict__ slots,
                                                           const float* __restrict__ S, int32_t* __restrict__ status) {
  const int unit = blockIdx.x, tid = threadIdx.x;
  const int n = hdr[(size_t)unit * 4], t = hdr[(size_t)unit * 4 + 1], j = hdr[(size_t)unit * 4 + 2] - 1;
  const int c = p.budget, m = p.m, r = p.n_recent, sink = p.n_sink, cap = p.cap;
  const int* po = pos + (size_t)unit * c;
  const int* sl = slots + (size_t)unit * c;
  int* meta = p.meta + (size_t)unit * META_STRIDE;
  int* Eu = p.E + (size_t)unit * 2 * m;
  int* PEu = p.PE + (size_t)unit * 2 * m;
  int* Ru = p.R + (size_t)unit * max(r, 1);
  float* Su = p.S + (size_t)unit * cap;
  int* mark = p.pf_flag + (size_t)unit * (cap + p.max_chunk);       // [cap] scratch: which token claims a slot
  int* dest = p.pf_list + (size_t)unit * (cap + p.max_chunk);       // [budget] slot of token i
  __shared__ int sm_free;

  // the scalars, then the arrays
  int bad = (n < 0 || n > c || t < n || j < 0 || j >= m) ? 1 : 0;
  const bool full = n == c;
  if (!bad && !full && (t != n || j != 0)) bad = 1;                  // nothing has been evicted while the cache fills
  const bool own_slots = !bad && full && sl[0] >= 0;                 // else: token i goes to slot i
  if (!bad) {
    for (int i = tid; i < n; i += 256) {
      const int x = po[i];
      if (!full) { if (x != i) bad = 1; continue; }
      const int k = i - sink;
      if (x < 0 || x >= t || (i > 0 && po[i - 1] >= x)) bad = 1;     // ascending positions below t
      if (k < 0 && x != i) bad = 1;                                  // the sinks are the first tokens
      if (k >= m && x != t - r + (k - m)) bad = 1;                   // the recent window is the last r tokens
      if (own_slots && (sl[i] < 0 || sl[i] >= cap)) bad = 1;
    }
  }
  bad = __syncthreads_or(bad);
  if (!bad && own_slots) {                                           // every slot claimed once
    for (int s = tid; s < cap; s += 256) mark[s] = -1;
    __syncthreads();
    for (int i = tid; i < n; i += 256) mark[sl[i]] = i;
    __syncthreads();
    for (int i = tid; i < n; i += 256) if (mark[sl[i]] != i) bad = 1;
    bad = __syncthreads_or(bad);
  }
  if (status && tid == 0) status[unit] = bad ? TREEKV_EINVAL : TREEKV_OK;
  const int n_eff = bad ? 0 : n;

  int free_slot = n_eff;                                             // filling, or token i in slot i: the next slot
  if (!bad && own_slots) {
    for (int s = tid; s < cap; s += 256) if (mark[s] < 0) sm_free = s;   // cap = n + 1 slots: exactly one is unclaimed
    __syncthreads();
    free_slot = sm_free;
  }
  const bool use_slots = own_slots && !bad, use_pos = full && !bad;
  auto slot_of = [&](int i) { return use_slots ? sl[i] : i; };
  auto pos_of = [&](int i) { return use_pos ? po[i] : i; };
  const int jd = bad ? 0 : j;
  for (int i = tid; i < 2 * m; i += 256) Eu[i] = PEu[i] = 0;
  for (int s = tid; s < cap; s += 256) Su[s] = 0.f;
  __syncthreads();
  for (int k = tid; k < m; k += 256) {
    const int x = tree_index(k, jd);
    Eu[x] = slot_of(sink + k);
    PEu[x] = pos_of(sink + k);
  }
  for (int k = tid; k < r; k += 256) Ru[k] = slot_of(sink + m + k);
  for (int i = tid; i < c; i += 256) {
    dest[i] = i < n_eff ? slot_of(i) : -1;
    if (i < n_eff) Su[slot_of(i)] = S[(size_t)unit * c + i];
  }
  if (tid < META_STRIDE) {
    int w = 0;
    if (tid == META_N) w = n_eff;
    else if (tid == META_FREE) w = free_slot;
    else if (tid == META_J) w = jd;
    else if (tid == META_T) w = bad ? 0 : t;
    meta[tid] = w;
  }
}

__global__ void import_rows_kernel(Params p, const uint4* __restrict__ Kin, const uint4* __restrict__ Vin, int row_vec) {
  const int unit = blockIdx.y, i = blockIdx.x;   // one block per snapshot row
  const int slot = p.pf_list[(size_t)unit * (p.cap + p.max_chunk) + i];
  if (slot < 0) return;
  const size_t src = ((size_t)unit * p.budget + i) * row_vec;
  const size_t dst = ((size_t)unit * p.cap + slot) * row_vec;
  for (int e = threadIdx.x; e < row_vec; e += blockDim.x) {
    reinterpret_cast<uint4*>(p.K)[dst + e] = Kin[src + e];
    reinterpret_cast<uint4*>(p.V)[dst + e] = Vin[src + e];
  }
}

thread_local hipError_t tl_hip_error = hipSuccess;

int check_launch() { return finish_launch(); }

}  // namespace

bool hip_failed(hipError_t e) {
  if (e == hipSuccess) return false;
  tl_hip_error = e;
  return true;
}
int finish_launch() { return hip_failed(hipGetLastError()) ? TREEKV_EHIP : TREEKV_OK; }
hipError_t take_hip_error() {
  const hipError_t e = tl_hip_error;
  tl_hip_error = hipSuccess;
  return e;
}

int launch_export_state(const Params& p, char* dst, hipStream_t s) {
  const treekv_state_layout l = state_layout(p);
  const int row_vec = p.D * (p.dtype == TREEKV_BF16 ? 2 : 4) / 16;
  hipLaunchKernelGGL(export_state_kernel, dim3(p.U), dim3(256), 0, s, p, (int*)(dst + l.header), (int*)(dst + l.positions),
                     (int*)(dst + l.slots), (float*)(dst + l.S));
  hipLaunchKernelGGL(gather_kv_kernel, dim3(p.budget, p.U), dim3(64), 0, s, p, (uint4*)(dst + l.K), (uint4*)(dst + l.V), row_vec);
  return finish_launch();
}

int launch_import_state(const Params& p, const char* src, int32_t* status, hipStream_t s) {
  const treekv_state_layout l = state_layout(p);
  const int row_vec = p.D * (p.dtype == TREEKV_BF16 ? 2 : 4) / 16;
  hipLaunchKernelGGL(import_state_kernel, dim3(p.U), dim3(256), 0, s, p, (const int*)(src + l.header),
                     (const int*)(src + l.positions), (const int*)(src + l.slots), (const float*)(src + l.S), status);
  hipLaunchKernelGGL(import_rows_kernel, dim3(p.budget, p.U), dim3(64), 0, s, p, (const uint4*)(src + l.K),
                     (const uint4*)(src + l.V), row_vec);
  return finish_launch();
}

int launch_reset(const Params& p, hipStream_t s) {
  hipLaunchKernelGGL(reset_kernel, dim3(p.U), dim3(256), 0, s, p);
  if (p.flags & TREEKV_POSITION_RERANK)
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((rope_rows(p) * (p.D / 2) + 255) / 256)), dim3(256), 0, s, p);
  return check_launch();
}

int launch_scores(const Params& p, float* scores, hipStream_t s) {
  hipLaunchKernelGGL(scores_kernel, dim3(p.U), dim3(256), 0, s, p, scores);
  return check_launch();
}

int launch_gather_kv(const Params& p, void* K_out, void* V_out, hipStream_t s) {
  const int row_vec = p.D * (p.dtype == TREEKV_BF16 ? 2 : 4) / 16;
  hipLaunchKernelGGL(gather_kv_kernel, dim3(p.budget, p.U), dim3(64), 0, s, p, (uint4*)K_out, (uint4*)V_out, row_vec);
  return check_launch();
}

}  // namespace tkv

// --------------------------------------------------------------------------------------
// C ABI
// --------------------------------------------------------------------------------------
namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Every entry point that launches calls fresh() first: an error an earlier, unrelated HIP call of this thread
// left behind is dropped there, so it is not taken for a failure of this library's launches.
void fresh() {
  (void)hipGetLastError();
  (void)tkv::take_hip_error();
}

int record_hip(treekv_ctx* ctx, int rc) {
  const hipError_t e = tkv::take_hip_error();
  if (rc == TREEKV_EHIP) snprintf(ctx->hip_err, sizeof(ctx->hip_err), "%s", hipGetErrorString(e));
  return rc;
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES];
std::mutex scratch_mutex;

int static_scratch(void** out) {
  int dev = -1;
  if (tkv::hip_failed(hipGetDevice(&dev))) return TREEKV_EHIP;
  if (dev < 0 || dev >= MAX_DEVICES) return TREEKV_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (tkv::hip_failed(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return TREEKV_EHIP;
    scratch_ptr[dev] = ptr;
  }
  *out = scratch_ptr[dev];
  return TREEKV_OK;
}

int pick_splits(const treekv_config& c) {
  // With about 200 units or more, one 512-thread workgroup per unit fills the 256 compute units and
  // keeps the whole step in one kernel.  Below that, split every unit's slots over a few 512-thread
  // workgroups (measured best: about 160 workgroups in all; 128 units -> 2 slices, 32 units -> 5), but keep
  // a slice at 128 slots or more (below that the merge costs more than the streaming it spreads).
  const int units = c.batch * c.kv_heads;
  if (units >= 192) return 1;
  int splits = (160 + units - 1) / units;
  const int max_by_len = (c.budget + 1 + 127) / 128;
  if (splits > max_by_len) splits = max_by_len;
  if (splits > 32) splits = 32;
  if (splits < 1) splits = 1;
  return splits;
}

}  // namespace

extern "C" {

int treekv_init_ex(treekv_ctx** out, const treekv_config* cfg_in) {
  if (!out || !cfg_in) return TREEKV_EINVAL;
  treekv_config c = *cfg_in;
  if (c.budget < 1 || c.q_heads < 1 || c.kv_heads < 1 || c.batch < 1) return TREEKV_EINVAL;
  if (c.q_heads % c.kv_heads != 0) return TREEKV_EINVAL;
  if (c.n_sink == TREEKV_DEFAULT_LAYOUT && c.n_recent == TREEKV_DEFAULT_LAYOUT) {
    // Section 5.2's 4 initial + 512 selected + 508 recent tokens of 1024, scaled to the budget
    if (c.budget < 16) return TREEKV_EINVAL;
    c.n_sink = 4;
    c.n_recent = c.budget - c.budget / 2 - 4;
  }
  if (c.n_sink < 0 || c.n_recent < 0 || c.budget - c.n_sink - c.n_recent < 1) return TREEKV_EINVAL;
  if (c.dtype != TREEKV_BF16 && c.dtype != TREEKV_F32) return TREEKV_EINVAL;
  if (c.flags & ~(TREEKV_KEEP_LEFT | TREEKV_SCORE_ACCUMULATED | TREEKV_POSITION_RERANK)) return TREEKV_EINVAL;
  if (!(c.rope_base >= 0.0f) || isinf(c.rope_base)) return TREEKV_EINVAL;
  if (c.rope_base == 0.0f) c.rope_base = 10000.0f;
  if (c.max_chunk < 0 || c.kv_splits < 0 || c.kv_splits > 64) return TREEKV_EINVAL;
  if (!(c.softmax_scale >= 0.0f) || isinf(c.softmax_scale)) return TREEKV_EINVAL;
  if (c.head_dim != 64 && c.head_dim != 128) return TREEKV_EUNSUPPORTED;
  const int G = c.q_heads / c.kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return TREEKV_EUNSUPPORTED;
  if ((long long)c.budget > (1 << 24) || (long long)c.batch * c.kv_heads > 65535) return TREEKV_EUNSUPPORTED;
  if (c.max_chunk == 0) c.max_chunk = 512;
  if (c.max_chunk > 4096) return TREEKV_EUNSUPPORTED;
  if (c.max_prompt < 0) return TREEKV_EINVAL;
  if (c.max_prompt > (1 << 24)) return TREEKV_EUNSUPPORTED;
  if (c.softmax_scale == 0.0f) c.softmax_scale = 1.0f / sqrtf((float)c.head_dim);
  if (c.kv_splits == 0) c.kv_splits = pick_splits(c);

  treekv_ctx* ctx = new (std::nothrow) treekv_ctx;
  if (!ctx) return TREEKV_EINVAL;
  memset(ctx, 0, sizeof(*ctx));
  ctx->cfg = c;
  tkv::Params& p = ctx->p;
  p.budget = c.budget; p.cap = c.budget + 1; p.n_sink = c.n_sink; p.n_recent = c.n_recent;
  p.m = c.budget - c.n_sink - c.n_recent;
  p.B = c.batch; p.H = c.q_heads; p.Hkv = c.kv_heads; p.G = G; p.D = c.head_dim; p.U = c.batch * c.kv_heads;
  p.dtype = c.dtype; p.flags = c.flags; p.nsplit = c.kv_splits; p.max_chunk = c.max_chunk;
  p.max_prompt = c.max_prompt;
  p.rope_base = c.rope_base;
  p.scale_log2e = c.softmax_scale * 1.4426950408889634f;
  // a unit whose logits do not fit one workgroup's LDS is split further
  for (;;) {
    p.rows_per_split = ((p.cap + p.nsplit - 1) / p.nsplit + 63) / 64 * 64;
    if (tkv::decode_shape_fits(p) || p.nsplit >= 64) break;
    p.nsplit = p.nsplit < 2 ? 2 : p.nsplit + (p.nsplit + 1) / 2;
    if (p.nsplit > 64) p.nsplit = 64;
  }
  if (!tkv::decode_shape_fits(p)) { delete ctx; return TREEKV_EUNSUPPORTED; }
  ctx->cfg.kv_splits = p.nsplit;
  ctx->ws_bytes = tkv::carve(p, nullptr);
  *out = ctx;
  return TREEKV_OK;
}

int treekv_init(treekv_ctx** out, int budget, int heads, int head_dim) {
  if (budget < 16) return TREEKV_EINVAL;
  treekv_config c;
  memset(&c, 0, sizeof(c));
  c.budget = budget; c.q_heads = heads; c.kv_heads = heads; c.head_dim = head_dim; c.batch = 1;
  c.dtype = TREEKV_BF16;
  c.n_sink = c.n_recent = TREEKV_DEFAULT_LAYOUT;
  return treekv_init_ex(out, &c);
}

void treekv_destroy(treekv_ctx* ctx) { delete ctx; }

int treekv_get_config(const treekv_ctx* ctx, treekv_config* out) {
  if (!ctx || !out) return TREEKV_EINVAL;
  *out = ctx->cfg;
  return TREEKV_OK;
}

size_t treekv_workspace_bytes(const treekv_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }

int treekv_bind_workspace(treekv_ctx* ctx, void* dev_ptr, size_t bytes) {
  if (!ctx || !dev_ptr) return TREEKV_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dev_ptr) & (tkv::ALIGN - 1)) != 0 || bytes < ctx->ws_bytes) return TREEKV_ENOWS;
  tkv::carve(ctx->p, static_cast<char*>(dev_ptr));
  ctx->bound = true;
  return TREEKV_OK;
}

int treekv_reset(treekv_ctx* ctx, void* stream) {
  if (!ctx) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_reset(ctx->p, (hipStream_t)stream));
}

int treekv_decode_step(treekv_ctx* ctx, const void* q, const void* k, const void* v, void* out, int32_t* retained,
                       int32_t* n_retained, int32_t* evicted, void* stream) {
  if (!ctx || !q || !k || !v || !out || !retained) return TREEKV_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_decode(ctx->p, q, k, v, (float*)out, retained, n_retained, evicted,
                                            (hipStream_t)stream));
}

int treekv_decode_step_static(treekv_ctx* ctx, const void* q, const void* k, const void* v, void* out,
                              int32_t* retained, int32_t* n_retained, int32_t* evicted, void* stream) {
  if (!ctx || !q || !k || !v || !out || !retained) return TREEKV_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  tkv::Params p = ctx->p;
  size_t lg = 0;
  if (p.nsplit > 1) {                       // the one-kernel shape keeps its logits in LDS and needs no scratch
    lg = tkv::align_up((size_t)p.U * p.G * p.cap * sizeof(float));
    const size_t pt = tkv::align_up((size_t)p.U * p.nsplit * p.G * (size_t)(p.D + 2) * sizeof(float));
    if (lg + pt > (size_t)TREEKV_STATIC_SCRATCH_BYTES) return TREEKV_ESCRATCH;
  }
  fresh();
  if (p.nsplit > 1) {
    void* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc != TREEKV_OK) return record_hip(ctx, rc);
    p.logits = static_cast<float*>(base);
    p.partial = reinterpret_cast<float*>(static_cast<char*>(base) + lg);
  }
  return record_hip(ctx, tkv::launch_decode(p, q, k, v, (float*)out, retained, n_retained, evicted, (hipStream_t)stream));
}

int treekv_prefill_chunk(treekv_ctx* ctx, const void* Q, const void* K, const void* V, int len, void* out,
                         int32_t* retained, int32_t* n_retained, int32_t* evicted, void* stream) {
  if (!ctx || !Q || !K || !V || !out || !retained) return TREEKV_EINVAL;
  if (len < 1 || len > ctx->cfg.max_chunk) return TREEKV_EINVAL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(out)) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_prefill(ctx->p, Q, K, V, len, (float*)out, retained, n_retained, evicted,
                                             (hipStream_t)stream));
}

int treekv_prefill_prompt(treekv_ctx* ctx, const void* Qw, const void* K, const void* V, int len, int block,
                          int32_t* retained, int32_t* n_retained, int32_t* evicted_blocks, float* token_scores,
                          void* stream) {
  if (!ctx || !Qw || !K || !V || !retained) return TREEKV_EINVAL;
  const treekv_config& c = ctx->cfg;
  if (block < 1 || len < block || len > c.max_prompt || len % block != 0 || c.budget % block != 0) return TREEKV_EINVAL;
  const int cb = c.budget / block, sink_b = (c.n_sink + block - 1) / block, recent_b = (c.n_recent + block - 1) / block;
  if (cb - sink_b - recent_b < 1) return TREEKV_EINVAL;
  if (!aligned16(Qw) || !aligned16(K) || !aligned16(V)) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  // the window's queries of one KV head's group are the rows of one matrix operand set
  if (block * (c.q_heads / c.kv_heads) > 128) return TREEKV_EUNSUPPORTED;
  if (tkv::prompt_blocks_lds(len, block, cb, sink_b, recent_b) > 150 * 1024) return TREEKV_EUNSUPPORTED;
  fresh();
  return record_hip(ctx, tkv::launch_prompt(ctx->p, Qw, K, V, len, block, retained, n_retained, evicted_blocks,
                                            token_scores, (hipStream_t)stream));
}

size_t treekv_state_bytes(const treekv_ctx* ctx) { return ctx ? tkv::state_layout(ctx->p).bytes : 0; }

int treekv_get_state_layout(const treekv_ctx* ctx, treekv_state_layout* out) {
  if (!ctx || !out) return TREEKV_EINVAL;
  *out = tkv::state_layout(ctx->p);
  return TREEKV_OK;
}

int treekv_export_state(treekv_ctx* ctx, void* dst, size_t bytes, void* stream) {
  if (!ctx || !dst) return TREEKV_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dst) & (tkv::ALIGN - 1)) != 0 || bytes < tkv::state_layout(ctx->p).bytes) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_export_state(ctx->p, static_cast<char*>(dst), (hipStream_t)stream));
}

int treekv_import_state(treekv_ctx* ctx, const void* src, size_t bytes, int32_t* status, void* stream) {
  if (!ctx || !src) return TREEKV_EINVAL;
  if ((reinterpret_cast<uintptr_t>(src) & (tkv::ALIGN - 1)) != 0 || bytes < tkv::state_layout(ctx->p).bytes) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_import_state(ctx->p, static_cast<const char*>(src), status, (hipStream_t)stream));
}

int treekv_scores(treekv_ctx* ctx, float* scores, void* stream) {
  if (!ctx || !scores) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_scores(ctx->p, scores, (hipStream_t)stream));
}

int treekv_gather_kv(treekv_ctx* ctx, void* K_out, void* V_out, void* stream) {
  if (!ctx || !K_out || !V_out) return TREEKV_EINVAL;
  if (!aligned16(K_out) || !aligned16(V_out)) return TREEKV_EINVAL;
  if (!ctx->bound) return TREEKV_ENOWS;
  fresh();
  return record_hip(ctx, tkv::launch_gather_kv(ctx->p, K_out, V_out, (hipStream_t)stream));
}

int treekv_wavelet_components(const float* a, const void* V, int dtype, int heads, int t, int d, int levels,
                              float* per_head, float* mean, void* stream) {
  if (!a || !V || !per_head) return TREEKV_EINVAL;
  if (dtype != TREEKV_BF16 && dtype != TREEKV_F32) return TREEKV_EINVAL;
  if (heads < 1 || t < 1 || levels < 1 || levels > 30 || t % (1 << levels) != 0) return TREEKV_EINVAL;
  if (!aligned16(V)) return TREEKV_EINVAL;
  if (levels > 5 || (d != 64 && d != 128) || heads > 65535 || (long long)levels * t > (1ll << 30)) return TREEKV_EUNSUPPORTED;
  fresh();
  const int rc = tkv::launch_wavelet(a, V, dtype, heads, t, d, levels, per_head, mean, (hipStream_t)stream);
  (void)tkv::take_hip_error();
  return rc;
}

const char* treekv_strerror(int status) {
  switch (status) {
    case TREEKV_OK: return "ok";
    case TREEKV_EINVAL: return "invalid argument";
    case TREEKV_ENOWS: return "workspace not bound, misaligned or too small";
    case TREEKV_EHIP: return "HIP call failed";
    case TREEKV_EUNSUPPORTED: return "configuration not supported by this build";
    case TREEKV_ESCRATCH: return "needs more scratch than the library's fixed array holds";
    default: return "unknown status";
  }
}

const char* treekv_last_hip_error(const treekv_ctx* ctx) { return ctx ? ctx->hip_err : ""; }

}  // extern "C"
