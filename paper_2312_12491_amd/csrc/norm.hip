// GroupNorm (+SiLU) over one or two concatenated NHWC sources, and LayerNorm over token rows.
// Statistics are accumulated in double and applied in fp32, whatever the storage type.
#include "common.h"

namespace {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// one block per (sample, group, split): partial sums -> atomics-free two-level reduce through `part`
template <typename T>
__global__ __launch_bounds__(256) void gn_stats_kernel(GroupNormParams p) {
  const int g = blockIdx.x % p.groups, n = blockIdx.x / p.groups;
  const int C = p.C1 + p.C2, cg = C / p.groups;
  const T* s1 = (const T*)p.src1;
  const T* s2 = (const T*)p.src2;
  const long long total = (long long)p.HW * cg;
  double sum = 0.0, sq = 0.0;
  for (long long i = threadIdx.x; i < total; i += blockDim.x) {
    int px = (int)(i / cg);
    int c = g * cg + (int)(i - (long long)px * cg);
    long long pix = (long long)n * p.HW + px;
    float v = c < p.C1 ? to_f32<T>(s1[pix * p.C1 + c]) : to_f32<T>(s2[pix * p.C2 + (c - p.C1)]);
    sum += v;
    sq += (double)v * v;
  }
  __shared__ double red[2][4];
  sum = wave_sum(sum);
  sq = wave_sum(sq);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][w] = sum; red[1][w] = sq; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    double q = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    double mean = s / (double)total;
    double var = q / (double)total - mean * mean;
    if (var < 0) var = 0;
    p.stats[2 * blockIdx.x] = (float)mean;
    p.stats[2 * blockIdx.x + 1] = (float)(1.0 / sqrt(var + (double)p.eps));
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gn_apply_kernel(GroupNormParams p, long long total) {
  const int C = p.C1 + p.C2, cg = C / p.groups;
  const T* s1 = (const T*)p.src1;
  const T* s2 = (const T*)p.src2;
  T* out = (T*)p.out;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    long long pix = i / C;
    int c = (int)(i - pix * C);
    int n = (int)(pix / p.HW);
    float v = c < p.C1 ? to_f32<T>(s1[pix * p.C1 + c]) : to_f32<T>(s2[pix * p.C2 + (c - p.C1)]);
    const float* st = p.stats + 2 * ((long long)n * p.groups + c / cg);
    float y = (v - st[0]) * st[1] * p.gamma[c] + p.beta[c];
    if (p.silu) y = y / (1.0f + expf(-y));
    out[i] = from_f32<T>(y);
  }
}

// one wave per token row
template <typename T>
__global__ __launch_bounds__(256) void layer_norm_kernel(LayerNormParams p) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= p.rows) return;
  const T* x = (const T*)p.src + (long long)row * p.C;
  T* y = (T*)p.out + (long long)row * p.C;
  float sum = 0.f;
  for (int c = lane; c < p.C; c += 64) sum += to_f32<T>(x[c]);
  const float mean = wave_sum(sum) / (float)p.C;
  float sq = 0.f;
  for (int c = lane; c < p.C; c += 64) {
    float d = to_f32<T>(x[c]) - mean;
    sq += d * d;
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)p.C + p.eps);
  for (int c = lane; c < p.C; c += 64)
    y[c] = from_f32<T>((to_f32<T>(x[c]) - mean) * rstd * p.gamma[c] + p.beta[c]);
}

}  // namespace

template <typename T> void launch_group_norm(const GroupNormParams& p, hipStream_t s) {
  hipLaunchKernelGGL(gn_stats_kernel<T>, dim3(p.samples * p.groups), dim3(256), 0, s, p);
  long long total = (long long)p.samples * p.HW * (p.C1 + p.C2);
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(gn_apply_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, p, total);
}
template void launch_group_norm<float>(const GroupNormParams&, hipStream_t);
template void launch_group_norm<bf16_t>(const GroupNormParams&, hipStream_t);

template <typename T> void launch_layer_norm(const LayerNormParams& p, hipStream_t s) {
  hipLaunchKernelGGL(layer_norm_kernel<T>, dim3((p.rows + 3) / 4), dim3(256), 0, s, p);
}
template void launch_layer_norm<float>(const LayerNormParams&, hipStream_t);
template void launch_layer_norm<bf16_t>(const LayerNormParams&, hipStream_t);
