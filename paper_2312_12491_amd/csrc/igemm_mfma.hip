// bf16 implicit-GEMM convolution / linear layer on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16).
//
//   out[m][n] = sum_k A[m][k] W[n][k]     m = (sample, oy, ox), k = tap*(C1+C2) + c
//
// Work split: one 256-thread block (4 waves, 2x2) owns a BM x BN output tile.  The activation tile
// (implicit im2col rows, gathered from NHWC with zero padding, stride, nearest-2x upsample and a second
// concatenated source folded into the indexing) is staged through double-buffered LDS; the weights are
// stored pre-packed in MFMA fragment order and go from global memory straight into registers, one coalesced
// 1 KB read per fragment, prefetched one stage ahead.  The MFMA is issued with the weight fragment as the
// row operand, so every lane ends up with 4 consecutive output channels of one pixel: bias, time-embedding
// bias, GEGLU and the residual are applied on registers and stored as 8-byte vectors.
// Optional split-K (grid.z) accumulates fp32 partials with atomics into a zeroed workspace that a small
// finalize kernel turns into the output (and zeroes again).
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

template <int BM, int BN, int KS>
__global__ __launch_bounds__(256) void igemm_mfma_kernel(IgemmParams p, int mtiles, int ksteps_total,
                                                         int stages_per_split) {
  constexpr int WM = 2, WN = 2;
  constexpr int KC = 32 * KS;
  constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 16, NT = WTN / 16;
  constexpr int ROWB = KC * 2 + 16;   // LDS row pitch in bytes (pad keeps 16-lane b128 reads conflict-free)
  constexpr int CPR = KC / 8;         // 16-byte chunks per row
  constexpr int NLD = BM * CPR / 256; // chunks each thread stages
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][BM * ROWB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int mtile = blockIdx.x % mtiles, ntile = blockIdx.x / mtiles;
  const int m0 = mtile * BM, n0 = ntile * BN;
  const int Ct = p.C1 + p.C2;
  const int pad = p.ksize >> 1;
  const int HWo = p.Hout * p.Wout;
  const int Hs = p.upsample ? p.Hin * 2 : p.Hin, Wsz = p.upsample ? p.Win * 2 : p.Win;
  const bf16_t* s1 = (const bf16_t*)p.src1;
  const bf16_t* s2 = (const bf16_t*)p.src2;
  const bf16_t* Wp = (const bf16_t*)p.W;

  // ---- loader slots of this thread
  int ld_y[NLD], ld_x[NLD], ld_row[NLD];
  long long ld_base[NLD];
  bool ld_ok[NLD];
  const int cq = tid % CPR;
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    int row = (tid + i * 256) / CPR;
    ld_row[i] = row;
    int m = m0 + row;
    ld_ok[i] = m < p.M;
    int mm = ld_ok[i] ? m : 0;
    int n = mm / HWo;
    int r = mm - n * HWo;
    int oy = r / p.Wout, ox = r - oy * p.Wout;
    ld_y[i] = oy * p.stride - pad;
    ld_x[i] = ox * p.stride - pad;
    ld_base[i] = (long long)n * p.Hin * p.Win;
  }

  // ---- K range of this split
  const int stage0 = blockIdx.z * stages_per_split;
  const int total_stages = ksteps_total / KS;
  int nstages = total_stages - stage0;
  if (nstages > stages_per_split) nstages = stages_per_split;
  int kk = stage0 * KC;
  int tap = kk / Ct, cch = kk - tap * Ct;
  int ky = tap / p.ksize, kx = tap - ky * p.ksize;

  // weight fragments of this wave: global n-tile index gnt0 + nt
  const int gnt0 = (n0 + wn * WTN) >> 4;
  const int ntiles_total = p.N >> 4;

  uint4 areg[NLD];
  bf16x8 bcur[KS][NT], bnxt[KS][NT];

  auto load_a = [&]() {
    const bf16_t* src;
    int Cs, c = cch;
    if (c < p.C1) { src = s1; Cs = p.C1; } else { src = s2; Cs = p.C2; c -= p.C1; }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      int iy = ld_y[i] + ky, ix = ld_x[i] + kx;
      bool ok = ld_ok[i] && iy >= 0 && iy < Hs && ix >= 0 && ix < Wsz;
      if (p.upsample) { iy >>= 1; ix >>= 1; }
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *(const uint4*)(src + (ld_base[i] + (long long)iy * p.Win + ix) * Cs + c + cq * 8);
      areg[i] = v;
    }
  };
  auto load_b = [&](bf16x8 (&b)[KS][NT], int kstep) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        int g = gnt0 + nt;
        if (g < ntiles_total)
          b[ks][nt] = *(const bf16x8*)(Wp + (((long long)g * ksteps_total + kstep + ks) * 64 + lane) * 8);
        else
          b[ks][nt] = bf16x8{};
      }
  };
  auto advance = [&]() {
    kk += KC;
    cch += KC;
    if (cch >= Ct) {
      cch = 0;
      if (++kx == p.ksize) { kx = 0; ++ky; }
    }
  };

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (nstages > 0) {
    load_a();
    load_b(bcur, kk / 32);
  }
  int buf = 0;
  for (int s = 0; s < nstages; ++s) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) *(uint4*)(&lds[buf][ld_row[i] * ROWB + cq * 16]) = areg[i];
    __syncthreads();
    if (s + 1 < nstages) {
      advance();
      load_a();
      load_b(bnxt, kk / 32);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 af[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        af[mt] = *(const bf16x8*)(&lds[buf][(wm * WTM + mt * 16 + (lane & 15)) * ROWB + (ks * 32 + (lane >> 4) * 8) * 2]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bcur[ks][nt], af[mt], acc[mt][nt], 0, 0, 0);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bcur[ks][nt] = bnxt[ks][nt];
    buf ^= 1;
  }

  // ---- epilogue: lane holds channels n..n+3 of pixel m
  const int Nout = p.epilogue == EPI_GEGLU ? p.N >> 1 : p.N;
  bf16_t* out = (bf16_t*)p.out;
  const bf16_t* res = (const bf16_t*)p.residual;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m0 + wm * WTM + mt * 16 + (lane & 15);
    if (m >= p.M) continue;
    const int sample = m / HWo;
    if (p.splitk > 1) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int n = (gnt0 + nt) * 16 + (lane >> 4) * 4;
        if (n >= p.N) continue;
        float* w = p.workspace + (long long)m * p.N + n;
#pragma unroll
        for (int v = 0; v < 4; ++v) atomicAdd(w + v, acc[mt][nt][v]);
      }
      continue;
    }
    if (p.epilogue == EPI_GEGLU) {
#pragma unroll
      for (int nt = 0; nt < NT; nt += 2) {
        const int n = (gnt0 + nt) * 16 + (lane >> 4) * 4;
        if (n >= p.N) continue;
        f32x4 a = acc[mt][nt], g = acc[mt][nt + 1];
        if (p.bias) {
          a += *(const f32x4*)(p.bias + n);
          g += *(const f32x4*)(p.bias + n + 16);
        }
        bf16x4 o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = (bf16_t)(a[v] * gelu_erf(g[v]));
        const int oc = ((gnt0 + nt) >> 1) * 16 + (lane >> 4) * 4;
        *(bf16x4*)(out + (long long)m * Nout + oc) = o;
      }
    } else {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int n = (gnt0 + nt) * 16 + (lane >> 4) * 4;
        if (n >= p.N) continue;
        f32x4 x = acc[mt][nt];
        if (p.bias) x += *(const f32x4*)(p.bias + n);
        if (p.rowbias) x += *(const f32x4*)(p.rowbias + (long long)sample * p.rowbias_ld + n);
        if (res) {
          bf16x4 r = *(const bf16x4*)(res + (long long)m * Nout + n);
#pragma unroll
          for (int v = 0; v < 4; ++v) x[v] += (float)r[v];
        }
        bf16x4 o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = (bf16_t)x[v];
        *(bf16x4*)(out + (long long)m * Nout + n) = o;
      }
    }
  }
}

// split-K finalize: workspace (fp32 [M][N]) -> out with the epilogue of the main kernel; re-zeroes the workspace
__global__ __launch_bounds__(256) void igemm_finalize_kernel(IgemmParams p) {
  const long long idx4 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total4 = (long long)p.M * p.N / 4;
  if (idx4 >= total4) return;
  const long long e = idx4 * 4;
  const int m = (int)(e / p.N), n = (int)(e - (long long)m * p.N);
  f32x4 x = *(f32x4*)(p.workspace + e);
  *(f32x4*)(p.workspace + e) = f32x4{0.f, 0.f, 0.f, 0.f};
  if (p.bias) x += *(const f32x4*)(p.bias + n);
  if (p.rowbias) x += *(const f32x4*)(p.rowbias + (long long)(m / (p.Hout * p.Wout)) * p.rowbias_ld + n);
  if (p.residual) {
    bf16x4 r = *(const bf16x4*)((const bf16_t*)p.residual + e);
#pragma unroll
    for (int v = 0; v < 4; ++v) x[v] += (float)r[v];
  }
  bf16x4 o;
#pragma unroll
  for (int v = 0; v < 4; ++v) o[v] = (bf16_t)x[v];
  *(bf16x4*)((bf16_t*)p.out + e) = o;
}

template <int BM, int BN, int KS> void launch_cfg(const IgemmParams& p, hipStream_t s) {
  const int mtiles = (p.M + BM - 1) / BM, ntiles = (p.N + BN - 1) / BN;
  const int ksteps_total = p.K / 32;
  const int total_stages = ksteps_total / KS;
  const int splitk = p.splitk > 1 ? p.splitk : 1;
  const int sps = (total_stages + splitk - 1) / splitk;
  dim3 grid(mtiles * ntiles, 1, splitk);
  hipLaunchKernelGGL((igemm_mfma_kernel<BM, BN, KS>), grid, dim3(256), 0, s, p, mtiles, ksteps_total, sps);
  if (splitk > 1) {
    long long total4 = (long long)p.M * p.N / 4;
    hipLaunchKernelGGL(igemm_finalize_kernel, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s, p);
  }
}

}  // namespace

bool igemm_mfma_available() { return true; }

bool igemm_mfma_supported(const IgemmParams& p) {
  if (p.C1 % 32 || p.C2 % 32 || p.N % 16) return false;
  if (p.epilogue == EPI_GEGLU && p.N % 128) return false;
  if (p.epilogue == EPI_SILU) return false;
  if (p.splitk > 1 && p.epilogue != EPI_NONE) return false;
  return true;
}

void launch_igemm_mfma(const IgemmParams& p, hipStream_t s) {
  const bool k64 = (p.C1 % 64 == 0) && (p.C2 % 64 == 0);
  int bn;
  if (p.epilogue == EPI_GEGLU) bn = 128;
  else if (p.N % 160 == 0) bn = 160;
  else if (p.N % 128 == 0) bn = 128;
  else bn = 64;
  if (bn == 160) { if (k64) launch_cfg<128, 160, 2>(p, s); else launch_cfg<128, 160, 1>(p, s); }
  else if (bn == 128) { if (k64) launch_cfg<128, 128, 2>(p, s); else launch_cfg<128, 128, 1>(p, s); }
  else { if (k64) launch_cfg<128, 64, 2>(p, s); else launch_cfg<128, 64, 1>(p, s); }
}
