// Key centering vector mu = (1/n) sum_i k_i per (batch, KV head) (Sec. 4.3 "Data
// pre-processing").  HBM-bound streaming read of the K cache: each thread sums up to
// rows_per_chunk/16 rows of one 8-element column group in float32, the workgroup and the
// chunks are combined in float64 in a fixed order, so the result is reproducible.
#include "mp_common.h"
#include "device_utils.h"

namespace mp {

template <int ET>
__global__ __launch_bounds__(256) void key_mean_partial_kernel(MeanArgs a) {
  __shared__ double red[16][kHeadDim];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  const int cg = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int64_t base = (int64_t)(unit / a.n_kv_heads) * a.stride_b + (int64_t)(unit % a.n_kv_heads) * a.stride_h;
  const int64_t r0 = (int64_t)chunk * a.rows_per_chunk;
  const int64_t r1 = r0 + a.rows_per_chunk < a.n ? r0 + a.rows_per_chunk : a.n;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
  for (int64_t i = r0 + rl; i < r1; i += 16) {
    float v[8];
    load8<ET>(a.Kc, base + i * a.stride_n + cg * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rl][cg * 8 + e] = (double)acc[e];
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    double s = 0.0;
    for (int r = 0; r < 16; ++r) s += red[r][threadIdx.x];
    a.partial[((int64_t)unit * a.nchunk + chunk) * kHeadDim + threadIdx.x] = s;
  }
}

// Sums the chunk partials of one (batch, KV head) in a fixed order: eight groups of 128
// threads take every eighth chunk (independent loads), LDS joins the groups.
__global__ __launch_bounds__(1024) void key_mean_final_kernel(MeanArgs a) {
  __shared__ double red[8][kHeadDim];
  const int unit = blockIdx.x;
  const int d = threadIdx.x & (kHeadDim - 1), grp = threadIdx.x >> 7;
  double s = 0.0;
#pragma unroll 4
  for (int c = grp; c < a.nchunk; c += 8) s += a.partial[((int64_t)unit * a.nchunk + c) * kHeadDim + d];
  red[grp][d] = s;
  __syncthreads();
  if (grp == 0) {
    double t = 0.0;
#pragma unroll
    for (int r = 0; r < 8; ++r) t += red[r][d];
    a.mu[(int64_t)unit * kHeadDim + d] = a.n > 0 ? (float)(t / (double)a.n) : 0.f;
  }
}

hipError_t launch_key_mean(const MeanArgs& a, hipStream_t s) {
  if (a.units <= 0) return hipSuccess;
  if (a.nchunk > 0) {
    dim3 grid((unsigned)a.nchunk, (unsigned)a.units);
    if (a.is_fp32) hipLaunchKernelGGL(key_mean_partial_kernel<kFP32>, grid, dim3(256), 0, s, a);
    else if (a.kv_fp8) hipLaunchKernelGGL(key_mean_partial_kernel<kFP8>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(key_mean_partial_kernel<kBF16>, grid, dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(key_mean_final_kernel, dim3((unsigned)a.units), dim3(1024), 0, s, a);
  return hipGetLastError();
}

}  // namespace mp
