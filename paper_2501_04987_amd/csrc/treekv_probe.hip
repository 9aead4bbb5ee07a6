// Measurement kernels behind treekv_probe.h: streaming read, plain copy, matrix-pipe issue rate.

#include "treekv_internal.h"
#include "treekv_probe.h"

namespace {

typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
constexpr int RD_THREADS = 512;
constexpr size_t WG_BYTES = (size_t)1 << 20;

template <int UN>
__global__ __launch_bounds__(RD_THREADS) void probe_read_kernel(const v4u* __restrict__ src, size_t wg_vecs,
                                                                float* __restrict__ sink) {
  const v4u* p = src + (size_t)blockIdx.x * wg_vecs;
  unsigned acc = 0;
  for (size_t i = threadIdx.x; i < wg_vecs; i += RD_THREADS * UN) {
    v4u r[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) r[u] = __builtin_nontemporal_load(p + i + (size_t)u * RD_THREADS);
#pragma unroll
    for (int u = 0; u < UN; ++u) acc += r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
  }
  if (acc == 0x12345678u) sink[0] = 1.f;
}

__global__ __launch_bounds__(RD_THREADS) void probe_copy_kernel(v4u* __restrict__ dst, const v4u* __restrict__ src) {
  const size_t base = (size_t)blockIdx.x * (WG_BYTES / 16);
  constexpr int UN = 4;
  for (size_t i = threadIdx.x; i < WG_BYTES / 16; i += RD_THREADS * UN) {
    v4u r[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) r[u] = src[base + i + (size_t)u * RD_THREADS];
#pragma unroll
    for (int u = 0; u < UN; ++u) dst[base + i + (size_t)u * RD_THREADS] = r[u];
  }
}

// 8 independent accumulator chains per wave, so consecutive instructions never wait for each other's result.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
  f32x4_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const v4u a = {0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u}, b = a;   // eight bf16 values near 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[m]) : "v"(a), "v"(b));
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  if (s == 1.2345f) sink[0] = s;
}

bool mib_multiple(size_t bytes) { return bytes >= WG_BYTES && bytes % WG_BYTES == 0 && bytes / WG_BYTES <= 0x7fffffffu; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int treekv_probe_read(const void* src, size_t bytes, int kib_per_workgroup, int loads_in_flight, float* sink, void* stream) {
  if (!src || !sink || !aligned16(src) || !mib_multiple(bytes)) return TREEKV_EINVAL;
  if (kib_per_workgroup < 32 || kib_per_workgroup > 1024 || (kib_per_workgroup & (kib_per_workgroup - 1))) return TREEKV_EINVAL;
  const size_t wg_bytes = (size_t)kib_per_workgroup << 10, wg_vecs = wg_bytes / 16;
  const dim3 grid((unsigned)(bytes / wg_bytes)), block(RD_THREADS);
  hipStream_t st = (hipStream_t)stream;
  // a workgroup's share is a multiple of 512 threads x 16 bytes x the loads in flight (32 KiB at 4)
  if (loads_in_flight == 2) hipLaunchKernelGGL(probe_read_kernel<2>, grid, block, 0, st, (const v4u*)src, wg_vecs, sink);
  else if (loads_in_flight == 4) hipLaunchKernelGGL(probe_read_kernel<4>, grid, block, 0, st, (const v4u*)src, wg_vecs, sink);
  else if (loads_in_flight == 8 && kib_per_workgroup >= 64) hipLaunchKernelGGL(probe_read_kernel<8>, grid, block, 0, st, (const v4u*)src, wg_vecs, sink);
  else return TREEKV_EINVAL;
  const int rc = tkv::finish_launch();
  (void)tkv::take_hip_error();
  return rc;
}

int treekv_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || !mib_multiple(bytes)) return TREEKV_EINVAL;
  hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)(bytes / WG_BYTES)), dim3(RD_THREADS), 0, (hipStream_t)stream,
                     (v4u*)dst, (const v4u*)src);
  const int rc = tkv::finish_launch();
  (void)tkv::take_hip_error();
  return rc;
}

int treekv_probe_mfma(float* sink, int workgroups, int waves_per_simd, int iters, double* flops, void* stream) {
  if (!sink || workgroups < 1 || workgroups > 65535 || iters < 1 || (waves_per_simd != 1 && waves_per_simd != 2))
    return TREEKV_EINVAL;
  if (waves_per_simd == 1)
    hipLaunchKernelGGL((probe_mfma_kernel<256>), dim3(workgroups), dim3(256), 0, (hipStream_t)stream, sink, iters);
  else
    hipLaunchKernelGGL((probe_mfma_kernel<512>), dim3(workgroups), dim3(512), 0, (hipStream_t)stream, sink, iters);
  if (flops) *flops = (double)workgroups * 4 * waves_per_simd * (double)iters * 8 * (2.0 * 16 * 16 * 32);
  const int rc = tkv::finish_launch();
  (void)tkv::take_hip_error();
  return rc;
}

}  // extern "C"
