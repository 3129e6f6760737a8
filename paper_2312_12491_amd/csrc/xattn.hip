// Cross-attention against a fixed prompt, folded into two GEMMs (bf16 path).
//
// The keys and values of the prompt are constants between prompt changes (appendix, pre-computation), so per head h
//   scores   = LN(x) Wq_h^T K_h^T / sqrt(d)      = LN(x) (K_h Wq_h)^T / sqrt(d)
//   out     += softmax(scores) V_h Wo_h^T        = softmax(scores) (Wo_h V_h^T)^T
// and the products in parentheses can be made once per prompt:
//   QK [heads*Lp][C] : row h*Lp + j = log2(e)/sqrt(d) * sum_e K[j][h d + e] Wq[h d + e][:]      (rows j >= L zero)
//   VO [C][heads*Lp] : column h*Lp + j = sum_e V[j][h d + e] Wo[:][h d + e]                      (columns j >= L zero)
// with Lp = L rounded up to the softmax segment of the GEMM epilogue.  A cross-attention is then
// GEMM (rows x QK, per-head softmax over Lp columns in the epilogue) -> GEMM (probabilities x VO + bias + residual)
// instead of projection, attention kernel and projection.  The LayerNorm in front is folded into QK like into any
// other consuming layer (scale into the columns, row sums and shift product as vectors).
#include "common.h"

namespace {

// one thread per (n, c) of QK: fp32 value into `raw` (unscaled by the norm), bf16(value * gamma[c]) into the packed matrix
__global__ void xattn_qk_kernel(const bf16_t* __restrict__ kv, int ld_kv, const float* __restrict__ wq,
                                const float* __restrict__ gamma, float* __restrict__ raw, bf16_t* __restrict__ packed,
                                int C, int heads, int d, int L, int Lp, int Npad, float scale) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)Npad * C) return;
  const int n = (int)(idx / C), c = (int)(idx - (long long)n * C);
  const int h = n / Lp, j = n - h * Lp;
  float acc = 0.f;
  if (h < heads && j < L) {
    for (int e = 0; e < d; ++e) acc = fmaf((float)kv[(long long)j * ld_kv + h * d + e], wq[(long long)(h * d + e) * C + c], acc);
    acc *= scale;
  }
  raw[idx] = acc;
  const int ntile = n >> 4, kstep = c >> 5, lane = (n & 15) + 16 * ((c & 31) >> 3), jj = c & 7;
  packed[((((long long)ntile * (C >> 5) + kstep) * 64 + lane) << 3) + jj] = (bf16_t)(acc * gamma[c]);
}

// one thread per row n of QK: wsum[n] = sum_c bf16(raw * gamma), lnb[n] = sum_c raw * beta
__global__ void xattn_qk_vectors_kernel(const float* __restrict__ raw, const float* __restrict__ gamma,
                                        const float* __restrict__ beta, float* __restrict__ wsum, float* __restrict__ lnb,
                                        int C, int Npad) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= Npad) return;
  double ws = 0.0, lb = 0.0;
  for (int c = 0; c < C; ++c) {
    const float v = raw[(long long)n * C + c];
    ws += (double)(float)(bf16_t)(v * gamma[c]);
    lb += (double)v * (double)beta[c];
  }
  wsum[n] = (float)ws;
  lnb[n] = (float)lb;
}

// one thread per (c, k) of VO, written packed as a [C][Npad] matrix
__global__ void xattn_vo_kernel(const bf16_t* __restrict__ kv, int ld_kv, int v_off, const float* __restrict__ wo,
                                bf16_t* __restrict__ packed, int C, int heads, int d, int L, int Lp, int Npad) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)C * Npad) return;
  const int c = (int)(idx / Npad), k = (int)(idx - (long long)c * Npad);
  const int h = k / Lp, j = k - h * Lp;
  float acc = 0.f;
  if (h < heads && j < L)
    for (int e = 0; e < d; ++e) acc = fmaf((float)kv[(long long)j * ld_kv + v_off + h * d + e], wo[(long long)c * C + h * d + e], acc);
  const int ntile = c >> 4, kstep = k >> 5, lane = (c & 15) + 16 * ((k & 31) >> 3), jj = k & 7;
  packed[((((long long)ntile * (Npad >> 5) + kstep) * 64 + lane) << 3) + jj] = (bf16_t)acc;
}

}  // namespace

void launch_xattn_fold(const void* kv, int ld_kv, const float* wq, const float* wo, const float* gamma, const float* beta,
                       float* raw, void* qk_packed, float* wsum, float* lnb, void* vo_packed, int C, int heads, int d,
                       int L, int Lp, int Npad, hipStream_t s) {
  const float scale = (float)(1.4426950408889634 / sqrt((double)d));
  const long long total = (long long)Npad * C;
  hipLaunchKernelGGL(xattn_qk_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)kv, ld_kv, wq,
                     gamma, raw, (bf16_t*)qk_packed, C, heads, d, L, Lp, Npad, scale);
  hipLaunchKernelGGL(xattn_qk_vectors_kernel, dim3((Npad + 63) / 64), dim3(64), 0, s, (const float*)raw, gamma, beta, wsum,
                     lnb, C, Npad);
  hipLaunchKernelGGL(xattn_vo_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)kv, ld_kv, C,
                     wo, (bf16_t*)vo_packed, C, heads, d, L, Lp, Npad);
}
