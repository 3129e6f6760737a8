// Implicit-GEMM convolution / linear layer on the vector ALU with fp32 accumulation.
// This is the float32 path of the library and the fallback of the bf16 path for shapes the MFMA kernel
// does not take.  64x64 output tile per 256-thread block, 16-deep K slices staged through LDS.
#include "common.h"

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float silu(float x) { return x / (1.0f + expf(-x)); }

template <typename T>
__global__ __launch_bounds__(256) void igemm_generic_kernel(IgemmParams p) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Ws[TK][TN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.x * TM, n0 = blockIdx.y * TN;
  const int Ct = p.C1 + p.C2;
  const int pad = p.ksize / 2;
  const int HWo = p.Hout * p.Wout;
  const int Hs = p.upsample ? p.Hin * 2 : p.Hin, Wsz = p.upsample ? p.Win * 2 : p.Win;  // logical input size

  // loader mapping: thread -> (row lr, k group lk*4..+4) for A and (col lr, k group) for W
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  const int am = m0 + lr;
  int a_n = 0, a_y = 0, a_x = 0;
  const bool a_ok = am < p.M;
  if (a_ok) {
    a_n = am / HWo;
    int r = am - a_n * HWo;
    a_y = r / p.Wout;
    a_x = r - a_y * p.Wout;
  }
  const T* s1 = (const T*)p.src1;
  const T* s2 = (const T*)p.src2;
  const T* W = (const T*)p.W;
  const int wn = n0 + lr;

  const int tx = tid & 15, ty = tid >> 4;  // compute mapping: rows ty*4.., cols tx*4..
  float acc[4][4] = {};

  for (int k0 = 0; k0 < p.K; k0 += TK) {
    float av[4], wv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int k = k0 + lk + j;
      float a = 0.f;
      if (a_ok && k < p.K) {
        int tap = k / Ct, c = k - tap * Ct;
        int ky = tap / p.ksize, kx = tap - ky * p.ksize;
        int iy = a_y * p.stride + ky - pad, ix = a_x * p.stride + kx - pad;
        if (iy >= 0 && iy < Hs && ix >= 0 && ix < Wsz) {
          if (p.upsample) { iy >>= 1; ix >>= 1; }
          long long pix = ((long long)a_n * p.Hin + iy) * p.Win + ix;
          a = c < p.C1 ? to_f32<T>(s1[pix * p.C1 + c]) : to_f32<T>(s2[pix * p.C2 + (c - p.C1)]);
        }
      }
      av[j] = a;
      wv[j] = (wn < p.N && k < p.K) ? to_f32<T>(W[(long long)wn * p.K + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      As[lk + j][lr] = av[j];
      Ws[lk + j][lr] = wv[j];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; w[i] = Ws[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
  }

  T* out = (T*)p.out;
  const T* res = (const T*)p.residual;
  const int Nout = p.epilogue == EPI_GEGLU ? p.N / 2 : p.N;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= p.M) continue;
    int sample = m / HWo;
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      float x = acc[i][j];
      if (n < p.N) {
        if (p.bias) x += p.bias[n];
        if (p.rowbias) x += p.rowbias[(long long)sample * p.rowbias_ld + n];
      }
      v[j] = x;
    }
    if (p.epilogue == EPI_GEGLU) {
#pragma unroll
      for (int j = 0; j < 4; j += 2) {
        int n = n0 + tx * 4 + j;
        if (n + 1 < p.N) out[(long long)m * Nout + (n >> 1)] = from_f32<T>(v[j] * gelu_erf(v[j + 1]));
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int n = n0 + tx * 4 + j;
        if (n >= p.N) continue;
        float x = v[j];
        if (p.epilogue == EPI_SILU) x = silu(x);
        if (res) x += to_f32<T>(res[(long long)m * Nout + n]);
        if (p.epilogue == EPI_RELU) x = fmaxf(x, 0.f);
        out[(long long)m * Nout + n] = from_f32<T>(x);
      }
    }
  }
}

}  // namespace

template <typename T> void launch_igemm_generic(const IgemmParams& p, hipStream_t s) {
  dim3 grid((p.M + TM - 1) / TM, (p.N + TN - 1) / TN);
  hipLaunchKernelGGL(igemm_generic_kernel<T>, grid, dim3(256), 0, s, p);
}
template void launch_igemm_generic<float>(const IgemmParams&, hipStream_t);
template void launch_igemm_generic<bf16_t>(const IgemmParams&, hipStream_t);
