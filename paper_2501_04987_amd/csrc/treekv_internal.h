// Internal declarations shared by the host library and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "treekv.h"

namespace tkv {

// Per-unit bookkeeping words (unit = one (batch, KV head) stream).
enum MetaField : int {
  META_N = 0,      // tokens currently retained
  META_FREE = 1,   // physical slot the next token is written to
  META_J = 2,      // 0-based eviction index inside the tree region (the paper's idx - 1)
  META_RHEAD = 3,  // oldest entry of the recent-window ring
  META_T = 4,      // tokens processed so far == position of the next token
  META_STRIDE = 8
};

// Everything a kernel needs to find its way through the workspace.
//
// Physical layout.  A unit owns cap = budget + 1 cache rows ("slots").  A token
// stays in the slot it was written to until it is evicted; the evicted slot is
// the next token's slot.  Attention ignores order, so rows never move.
// Logical (position) order is kept in small index arrays:
//   sinks   : slots 0 .. n_sink-1 hold positions 0 .. n_sink-1 (written while filling)
//   tree    : E[2m] (slots) and PE[2m] (the positions they hold).  During a round of m
//             evictions, E[0..m) is the tree region at the round's start and E[m+j] the
//             token that entered the tree region at the round's j-th step.  Eviction j
//             compares E[2j] and E[2j+1] and stores the survivor in E[j].  After
//             eviction j the region reads E[0..j] then E[2j+2 .. m+j].
//   recent  : ring R[n_recent] of slots, oldest at META_RHEAD; it always holds the last
//             n_recent positions, so their positions need no array.
struct Params {
  int budget, cap, n_sink, n_recent, m;
  int B, H, Hkv, G, D, U;   // U = B * Hkv units
  int dtype, flags, nsplit, max_chunk;
  int rows_per_split;       // decode: slots one workgroup streams (a multiple of 64)
  float scale_log2e;        // softmax_scale * log2(e): probabilities are exp2 of scaled logits
  void* K;                  // [U][cap][D] storage dtype
  void* V;                  // [U][cap][D]
  float* S;                 // [U][cap] accumulated attention weight per slot
  int* E;                   // [U][2m] slots of the tree region
  int* PE;                  // [U][2m] positions of the tree region
  int* R;                   // [U][max(n_recent,1)]
  int* meta;                // [U][META_STRIDE]
  float* logits;            // [U][G][cap]   decode scratch: scaled logits (log2 domain)
  float* partial;           // [U][nsplit][G][D+2] decode scratch: split-KV partial (acc, max, sum)
  // prefill scratch
  unsigned long long* pf_colacc;   // [U][cache columns | chunk columns, each rounded up to 128] column sums of the chunk in flight, fixed point
  float* pf_snew;           // [U][max_chunk] accumulated S of the chunk's tokens
  int* pf_flag;             // [U][cap + max_chunk] freed slots / dead chunk tokens, then destinations
  int* pf_list;             // [U][cap + max_chunk] free slots in ascending order
  // one-shot prompt compression scratch
  int max_prompt;           // longest prompt treekv_prefill_prompt accepts (0: none)
  float* pp_tok;            // [U][T] token scores of the prompt in flight (dense, stride T <= max_prompt)
  float* pp_beta;           // [U][T / block] block scores of the prompt in flight
  float* pp_stat;           // [U][PROMPT_MAX_SPLITS][128][2] per slice and window query row: max, sum
  int* pp_kept;             // [U][budget] kept blocks, ascending
  // position re-assignment (only with TREEKV_POSITION_RERANK)
  float rope_base;
  float2* rope_tab;         // [max(cap + max_chunk, max_prompt)][D/2] (cos, sin) of n * rope_base^(-2i/D): n a distance between
                            // two cached tokens (decode), a rank (prefill chunk) or a prompt position (prompt compression)
  uint16_t* pp_qrot;        // [U][hi, lo][128][D] bf16: the window's queries turned to their positions (max_prompt > 0)
  uint16_t* pf_krot;        // [U][hi, lo][cap + max_chunk][D] bf16: a prefill chunk's keys (cache rows by slot, then the
                            // chunk's own) turned to their ranks, split into two bf16 parts
  uint16_t* pf_qrot;        // [hi, lo][B][max_chunk][H][D] bf16: the chunk's queries, likewise
};
constexpr int PROMPT_MAX_SPLITS = 64;

// HIP errors.  A launch_* function ends with finish_launch(), which takes HIP's last error (and so clears
// it); hip_failed(e) is true for e != hipSuccess.  Either way the error is remembered, per host thread,
// until the C entry point that ran the launch copies its text into the context (take_hip_error).
int finish_launch();
bool hip_failed(hipError_t e);
hipError_t take_hip_error();

// true if the decode kernels of the current shape (p.nsplit, p.rows_per_split) fit in LDS
bool decode_shape_fits(const Params& p);
int launch_reset(const Params& p, hipStream_t s);
int launch_decode(const Params& p, const void* q, const void* k, const void* v, float* out,
                  int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s);
int launch_prefill(const Params& p, const void* Q, const void* K, const void* V, int len, float* out,
                   int32_t* retained, int32_t* n_retained, int32_t* evicted, hipStream_t s);
int launch_prompt(const Params& p, const void* Qw, const void* K, const void* V, int T, int b, int32_t* retained,
                  int32_t* n_retained, int32_t* evicted_blocks, float* token_scores, hipStream_t s);
size_t prompt_blocks_lds(int T, int b, int cb, int sink_b, int recent_b);
int launch_wavelet(const float* a, const void* V, int dtype, int heads, int t, int d, int levels, float* per_head,
                   float* mean, hipStream_t s);
int launch_scores(const Params& p, float* scores, hipStream_t s);
int launch_gather_kv(const Params& p, void* K_out, void* V_out, hipStream_t s);
int launch_export_state(const Params& p, char* dst, hipStream_t s);
int launch_import_state(const Params& p, const char* src, int32_t* status, hipStream_t s);

// ---- device helpers shared by the kernels ---------------------------------
#if defined(__HIPCC__)

template <typename T> struct Storage;
template <> struct Storage<uint16_t> {   // bfloat16 bit patterns
  static constexpr int EPL = 8;          // elements in one 16-byte lane load
  __device__ static inline void widen(const uint4& r, float (&f)[8]) {
    const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <> struct Storage<float> {
  static constexpr int EPL = 4;
  __device__ static inline void widen(const uint4& r, float (&f)[4]) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Tree-region index k (0 <= k < m) -> index into E / PE, after j_done evictions of the
// current round (0 <= j_done <= m; a round that just ended reads the same either way).
__device__ inline int tree_index(int k, int j_done) { return k < j_done ? k : k + j_done; }

// Logical index i (0 <= i < budget) -> physical slot, for a unit whose cache is full.
__device__ inline int logical_to_slot(const Params& p, const int* E, const int* R, int rhead, int j_done, int i) {
  if (i < p.n_sink) return i;
  int k = i - p.n_sink;
  if (k < p.m) return E[tree_index(k, j_done)];
  k -= p.m;
  int r = rhead + k;
  if (r >= p.n_recent) r -= p.n_recent;
  return R[r];
}

#endif  // __HIPCC__

}  // namespace tkv
