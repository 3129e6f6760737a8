// softmax(q k^T / sqrt(d)) v on the vector ALU in fp32 with an online softmax: the float32 path and the
// fallback of the bf16 path.  One block = 64 queries of one (sample, head); four lanes share a query, each
// owning a quarter of the head width; K/V tiles of 32 keys are staged in LDS as fp32.
#include "common.h"

namespace {

constexpr int BQ = 64, KT = 32;

template <typename T, int DP>  // DP = ceil(d / 4) upper bound (register slice per lane)
__global__ __launch_bounds__(256) void attn_generic_kernel(AttnParams p) {
  constexpr int DMAX = DP * 4;
  __shared__ float Ks[KT][DMAX + 4];
  __shared__ float Vs[KT][DMAX + 4];
  const int tid = threadIdx.x;
  const int head = blockIdx.y, sample = blockIdx.z;
  const int qi = blockIdx.x * BQ + (tid >> 2);
  const int part = tid & 3;
  const int dp = p.d / 4;  // d is a multiple of 4
  const int c0 = head * p.d;
  const T* Q = (const T*)p.q;
  const T* K = (const T*)p.k;
  const T* V = (const T*)p.v;
  long long kvoff = p.kv_select ? (long long)p.kv_select[sample] * p.kv_select_stride
                                : (long long)sample * p.kv_sample_stride;
  int Skv = p.Skv;
  if (p.kv_group > 1 && sample < p.kv_group_rows) {  // keys / values of the whole stream batch, in batch order
    kvoff = (long long)(sample - sample % p.kv_group) * p.kv_sample_stride;
    Skv = p.Skv * p.kv_group;
  }
  const bool q_ok = qi < p.Sq;

  float q[DP], o[DP];
#pragma unroll
  for (int e = 0; e < DP; ++e) {
    o[e] = 0.f;
    q[e] = (q_ok && e < dp)
               ? to_f32<T>(Q[((long long)sample * p.Sq + qi) * p.ldq + c0 + part * dp + e]) * p.scale
               : 0.f;
  }
  float mrun = -INFINITY, lrun = 0.f;

  for (int j0 = 0; j0 < Skv; j0 += KT) {
    __syncthreads();
    for (int i = tid; i < KT * p.d; i += 256) {
      int r = i / p.d, c = i - r * p.d;
      int j = j0 + r;
      float kv = 0.f, vv = 0.f;
      if (j < Skv) {
        kv = to_f32<T>(K[kvoff + (long long)j * p.ldk + c0 + c]);
        vv = to_f32<T>(V[kvoff + (long long)j * p.ldv + c0 + c]);
      }
      Ks[r][c] = kv;
      Vs[r][c] = vv;
    }
    __syncthreads();
    const int jn = min(KT, Skv - j0);
    for (int r = 0; r < jn; ++r) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < DP; ++e)
        if (e < dp) s = fmaf(q[e], Ks[r][part * dp + e], s);
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      float mnew = fmaxf(mrun, s);
      float corr = expf(mrun - mnew);  // exp(-inf) = 0 on the first key
      float pj = expf(s - mnew);
      lrun = lrun * corr + pj;
#pragma unroll
      for (int e = 0; e < DP; ++e)
        if (e < dp) o[e] = fmaf(pj, Vs[r][part * dp + e], o[e] * corr);
      mrun = mnew;
    }
  }
  if (q_ok) {
    T* O = (T*)p.out;
    float inv = 1.0f / lrun;
#pragma unroll
    for (int e = 0; e < DP; ++e)
      if (e < dp) O[((long long)sample * p.Sq + qi) * p.ldo + c0 + part * dp + e] = from_f32<T>(o[e] * inv);
  }
}

}  // namespace

template <typename T> void launch_attention_generic(const AttnParams& p, hipStream_t s) {
  dim3 grid((p.Sq + BQ - 1) / BQ, p.heads, p.samples);
  if (p.d <= 32)
    hipLaunchKernelGGL((attn_generic_kernel<T, 8>), grid, dim3(256), 0, s, p);
  else if (p.d <= 64)
    hipLaunchKernelGGL((attn_generic_kernel<T, 16>), grid, dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((attn_generic_kernel<T, 40>), grid, dim3(256), 0, s, p);
}
template void launch_attention_generic<float>(const AttnParams&, hipStream_t);
template void launch_attention_generic<bf16_t>(const AttnParams&, hipStream_t);
