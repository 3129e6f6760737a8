// bf16 implicit-GEMM convolution / linear layer on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16).
//
//   out[m][n] = sum_k A[m][k] W[n][k]     m = (sample, oy, ox), k = tap*(C1+C2) + c
//
// Work split: one 256-thread block (4 waves, 2x2) owns a BM x BN output tile.  The activation tile (implicit
// im2col rows gathered from NHWC, with zero padding, stride, nearest-2x upsample and a second, concatenated
// source folded into the indexing) and the weight tile (stored pre-packed in MFMA fragment order) are staged
// through LDS buffers.  Three kernels: the main one (igemm_dma_kernel) moves both operands global -> LDS directly in
// 64-deep K stages (channels a multiple of 64), in one of three pipeline shapes (launch_ring); igemm_mfma_kernel
// stages activations through registers in 32-deep stages and reads weight fragments straight into registers
// (channels a multiple of 32); igemm_rows_kernel, for 1x1 layers with K <= 640 on many rows, keeps a block's input
// rows in LDS for the whole launch and streams the weights through registers, without barriers.  The MFMA is issued with the
// weight fragment as the row operand, so every lane ends up with 4 consecutive output channels of one pixel:
// bias, time-embedding bias, GEGLU and the residual are applied on registers and stored as 8-byte vectors.
// Optional split-K writes fp32 partial tiles to a workspace that a small finalize kernel sums and turns into
// the output.  (Summing them in the last block to finish instead was measured and is slower here: the blocks of
// a tile sit on different XCDs, and both a device-scope fence per block - a write-back of the whole L2 - and
// cache-bypassing accesses to the partials cost more than the extra launch.)
#include "common.h"

#include <stdio.h>
#include <stdlib.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// GELU(x) = x/2 (1 + erf(x/sqrt 2)) for the bf16 path.  erfc(|z|) from the rational approximation 7.1.26 of
// Abramowitz & Stegun (absolute error of erf below 1.5e-7, far under bf16 resolution): E = poly(t) exp(-z^2),
// t = 1/(1 + p|z|); 1 + erf(z) is E for z < 0 (no cancellation in the tail) and 2 - E otherwise.  About a third
// of the instructions of erff, which made the GEGLU epilogue the longest phase of the short-K feed-forward GEMMs.
__device__ __forceinline__ float gelu_erf(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float e = poly * t * __builtin_amdgcn_exp2f(z * z * -1.4426950408889634f);
  return 0.5f * x * (x < 0.f ? e : 2.0f - e);
}

template <int I> struct IC { static constexpr int value = I; };

// sum over the four lanes {l, l^16, l^32, l^48} (the lanes that hold one output row), on the vector ALU:
// v_permlane16_swap / v_permlane32_swap with both operands equal leave (x[l], x[l^16]) resp. (x[l], x[l^32]) in a lane
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float quad_max(float x) {
  u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float quad_sum(float x) {
  u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// sum over the 16 lanes of a DPP row (lanes that differ in lane % 16), left in every lane: four rotate-and-add steps
template <int CTRL> __device__ __forceinline__ float dpp_rot(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float row16_sum(float x) {
  x += dpp_rot<0x128>(x);   // row_ror:8
  x += dpp_rot<0x124>(x);   // row_ror:4
  x += dpp_rot<0x122>(x);   // row_ror:2
  x += dpp_rot<0x121>(x);   // row_ror:1
  return x;
}

// mean and 1/std of the block's input rows for a folded LayerNorm, from the partial sums the producing layer left:
// thread r < BM folds the parts of row m0 + r and leaves (mean, rstd) in LDS for the epilogue.  (Requesting the
// parts before the main loop and folding them after it, which takes the wait out of the prologue, was measured: it
// needs the parts in registers across the loop, and with the part count capped to keep that affordable the
// producing layers lose their best tile width - 7.03 ms per step against 6.94.)
__device__ __forceinline__ void ln_rows_to_lds(const IgemmParams& p, int m0, int BM, float* lnrow) {
  const int r = threadIdx.x;
  if (p.ln_stats == nullptr || r >= BM) return;
#ifdef SDSTREAM_DEVHOOKS
  if (p.dev_exp & 8) { lnrow[r * 2] = 0.f; lnrow[r * 2 + 1] = 1.f; return; }
#endif
  const int m = min(m0 + r, p.M - 1);
  const float2* src = (const float2*)p.ln_stats + (long long)m * p.ln_parts;
  // all parts requested at once (one memory round trip instead of one per part); surplus slots re-read the last part
  float2 v[LN_MAX_PARTS];
#pragma unroll
  for (int i = 0; i < LN_MAX_PARTS; ++i) v[i] = src[min(i, p.ln_parts - 1)];
  float s = 0.f, q = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAX_PARTS; ++i) {
    if (i < p.ln_parts) {
      s += v[i].x;
      q += v[i].y;
    }
  }
  const float inv = 1.0f / (float)p.K;
  const float mean = s * inv;
  const float var = fmaxf(q * inv - mean * mean, 0.f);
  lnrow[r * 2] = mean;
  lnrow[r * 2 + 1] = 1.0f / sqrtf(var + p.ln_eps);
}

// Block -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  In the natural
// order (m-tile fastest) an XCD therefore sees every 8th m-tile of every weight column: the activations are split
// over the L2s and the weights are fetched by all eight - right when the activations are the larger operand.  When
// the weights are larger (the deep levels), `chunked` gives physical block p the logical index
// (p % 8) * (grid / 8) + p / 8 (grid padded to a multiple of 8): every XCD then owns a contiguous run of the order,
// i.e. whole weight columns, and a weight slab is fetched into one L2 instead of eight.
struct TileId { int mtile, ntile, split; bool valid; };
__device__ __forceinline__ TileId tile_of_block(const FastDiv& mtiles, const FastDiv& ntiles, int splitk, int chunked) {
  const int per = gridDim.x >> 3;
  const int logical = chunked ? (blockIdx.x & 7) * per + (blockIdx.x >> 3) : (int)blockIdx.x;
  TileId t;
  t.valid = logical < (int)(mtiles.d * ntiles.d) * splitk;
  const int r = fast_div(logical, mtiles);
  t.mtile = logical - r * (int)mtiles.d;
  t.split = fast_div(r, ntiles);
  t.ntile = r - t.split * (int)ntiles.d;
  return t;
}

// Epilogue shared by the kernels: lane holds channels n..n+3 (n = (gnt0+nt)*16 + 4*(lane/16)) of pixel
// m = mbase + mt*16 + lane%16 in acc[mt][nt].
// Everything the epilogue reads (bias, time-embedding bias, residual) is requested in one go by epilogue_load,
// before the first use: with a load and its wait inside the (mt, nt) loops the epilogue was a chain of up to
// 3*MT*NT memory round trips.  The 64-row kernels call epilogue_load before their main loop, so that on the
// short-K layers those round trips overlap the loop instead of following it.
template <int MT, int NT> struct EpilogueIn {
  f32x4 biasv[NT];       // bias; loaded values are not touched before epilogue_store (a use would wait for them)
  f32x4 rbv[NT];         // time-embedding bias when all rows of the wave belong to one sample
  f32x4 wsv[NT];         // folded LayerNorm: row sums of the scaled weights
  bf16x4 rv[MT][NT];     // residual
  bool one_sample;
};

template <int MT, int NT>
__device__ __forceinline__ void epilogue_load(const IgemmParams& p, EpilogueIn<MT, NT>& in, int mbase, int gnt0,
                                              int lane, int HWo) {
  in.one_sample = false;
  if (p.splitk > 1) return;   // partial tiles take nothing in
  const int Nout = p.epilogue == EPI_GEGLU ? p.N >> 1 : p.N;
  const bf16_t* res = (const bf16_t*)p.residual;
  const int ncol = (lane >> 4) * 4;
  const int m_last = min(mbase + MT * 16, p.M) - 1;
  const int sample0 = fast_div(mbase, p.fd_hw);
  in.one_sample = p.rowbias != nullptr && m_last >= mbase && sample0 == fast_div(m_last, p.fd_hw);   // wave-uniform
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int n = min((gnt0 + nt) * 16 + ncol, p.N - 4);   // clamped: columns past N are never stored
    // absent terms are read from the zero page: a select on the loaded value would be a use
    const long long voff = (p.slot_m > 0 && mbase >= p.slot_m) ? p.slot_v_bytes / 4 : 0;   // wave-uniform
    const float* bsrc = p.bias ? p.bias + voff + n : (const float*)p.zeros;
    const float* rsrc = in.one_sample ? p.rowbias + (long long)sample0 * p.rowbias_ld + n : (const float*)p.zeros;
    in.biasv[nt] = *(const f32x4*)bsrc;
    in.rbv[nt] = *(const f32x4*)rsrc;
    in.wsv[nt] = *(const f32x4*)(p.ln_wsum ? p.ln_wsum + voff + n : (const float*)p.zeros);
  }
#ifdef SDSTREAM_DEVHOOKS
  if (p.dev_exp & 16384) res = nullptr;
#endif
  if (res && p.epilogue != EPI_GEGLU) {   // (plain and ReLU epilogues)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = max(min(mbase + mt * 16 + (lane & 15), p.M - 1), 0);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int n = min((gnt0 + nt) * 16 + ncol, p.N - 4);
        in.rv[mt][nt] = *(const bf16x4*)(res + (long long)m * Nout + n);
      }
    }
  }
}

// per lane: sum and sum of squares, over the wave's rows, of what is stored in each of the lane's 4 NT columns
template <int NT> struct ColStats { float s[NT][4], q[NT][4]; };

// lnrow / red: LDS, [rows of the block][2], already offset to this wave's first row; wn: the wave's column half;
// ntile, ntiles: the block's column tile and their number (index of the row statistics it writes);
// cst: where the plain epilogue adds up the column statistics of the stored values (null: nowhere)
template <int MT, int NT, bool CS>
__device__ __forceinline__ void epilogue_store_cs(const IgemmParams& p, f32x4 (&acc)[MT][NT],
                                                  const EpilogueIn<MT, NT>& in, int mbase, int gnt0, int lane, int HWo,
                                                  int split, const float* lnrow, float* red, int wn, int ntile,
                                                  int ntiles, ColStats<NT>& cst) {
  const int Nout = p.epilogue == EPI_GEGLU ? p.N >> 1 : p.N;
  if (p.ln_stats) {   // folded LayerNorm: rstd (x W'^T - mean wsum)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const float mean = lnrow[(mt * 16 + (lane & 15)) * 2], rstd = lnrow[(mt * 16 + (lane & 15)) * 2 + 1];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (acc[mt][nt] - mean * in.wsv[nt]) * rstd;
    }
  }
  bf16_t* out = (bf16_t*)p.out;
  const bool has_res = p.residual != nullptr;
  const int ncol = (lane >> 4) * 4;
  if (p.splitk > 1) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mbase + mt * 16 + (lane & 15);
      if (m >= p.M) continue;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int n = (gnt0 + nt) * 16 + ncol;
        if (n >= p.N) continue;
        *(f32x4*)(p.workspace + ((long long)split * p.M + m) * p.N + n) = acc[mt][nt];
      }
    }
    return;
  }
  f32x4 addv[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) addv[nt] = in.biasv[nt] + in.rbv[nt];
  if (p.epilogue == EPI_GEGLU) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mbase + mt * 16 + (lane & 15);
      if (m >= p.M) continue;
#pragma unroll
      for (int nt = 0; nt < NT; nt += 2) {
        const int n = (gnt0 + nt) * 16 + ncol;
        if (n >= p.N) continue;
        const f32x4 a = acc[mt][nt] + addv[nt], g = acc[mt][nt + 1] + addv[nt + 1];
        bf16x4 o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = (bf16_t)(a[v] * gelu_erf(g[v]));
        const int oc = ((gnt0 + nt) >> 1) * 16 + ncol;
#ifdef SDSTREAM_DEVHOOKS
        if (p.dev_exp & 1) {
#pragma unroll
          for (int v = 0; v < 4; ++v) o[v] = (bf16_t)(a[v] * g[v]);
        }
        if ((p.dev_exp & 2) && a[0] != 12345.678f) continue;
#endif
        *(bf16x4*)(out + (long long)m * Nout + oc) = o;
      }
    }
    return;
  }
  if (p.epilogue == EPI_SOFTMAX) {
    // A wave's 16*NT columns are whole segments of SEG n-tiles (NT n-tiles = one 80-column head, or 16-column heads):
    // a row's segment lives in the four lanes that share the row, 4*SEG values each.
    auto softmax_rows = [&](auto segc) {
      constexpr int SEG = decltype(segc)::value;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mbase + mt * 16 + (lane & 15);
#pragma unroll
        for (int s0 = 0; s0 + SEG <= NT; s0 += SEG) {
          float e[SEG][4];
          bool ok[SEG][4];
          float mx = -3.0e38f;
#pragma unroll
          for (int t = 0; t < SEG; ++t) {
            const f32x4 x = acc[mt][s0 + t] + addv[s0 + t];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int col = (gnt0 + s0 + t) * 16 + ncol + v;
              ok[t][v] = t * 16 + ncol + v < p.sm_len && col < p.sm_cols;
              e[t][v] = x[v];
              if (ok[t][v]) mx = fmaxf(mx, x[v]);
            }
          }
          mx = quad_max(mx);
          float sum = 0.f;
#pragma unroll
          for (int t = 0; t < SEG; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              e[t][v] = ok[t][v] ? __builtin_amdgcn_exp2f(e[t][v] - mx) : 0.f;
              sum += e[t][v];
            }
          sum = quad_sum(sum);
          const float inv = sum > 0.f ? 1.0f / sum : 0.f;
          if (m < p.M) {
#pragma unroll
            for (int t = 0; t < SEG; ++t) {
              const int n = (gnt0 + s0 + t) * 16 + ncol;
              if (n >= p.N) continue;
              bf16x4 o;
#pragma unroll
              for (int v = 0; v < 4; ++v) o[v] = (bf16_t)(e[t][v] * inv);
              *(bf16x4*)(out + (long long)m * Nout + n) = o;
            }
          }
        }
      }
    };
    if constexpr (NT == 5) {
      if (p.sm_lp == 80) softmax_rows(IC<5>{}); else softmax_rows(IC<1>{});
    }
    return;
  }
  float ssum[MT], ssq[MT];   // per output row: sum and sum of squares of what is stored (for a LayerNorm folded into the next layer)
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    ssum[mt] = 0.f;
    ssq[mt] = 0.f;
    const int m = mbase + mt * 16 + (lane & 15);
    if (m >= p.M) continue;
    const int sample = fast_div(m, p.fd_hw);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int n = (gnt0 + nt) * 16 + ncol;
      if (n >= p.N) continue;
      f32x4 x = acc[mt][nt] + addv[nt];
      if (p.rowbias && !in.one_sample) x += *(const f32x4*)(p.rowbias + (long long)sample * p.rowbias_ld + n);
      if (has_res) {
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] += (float)in.rv[mt][nt][v];
      }
      if (p.epilogue == EPI_RELU) {
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = fmaxf(x[v], 0.f);
      }
      bf16x4 o;
#pragma unroll
      for (int v = 0; v < 4; ++v) o[v] = (bf16_t)x[v];
#ifdef SDSTREAM_DEVHOOKS
      if (!((p.dev_exp & 8192) && x[0] != 12345.678f))
#endif
      *(bf16x4*)(out + (long long)m * Nout + n) = o;
      if (p.stats_out) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float r = (float)o[v];
          ssum[mt] += r;
          ssq[mt] = fmaf(r, r, ssq[mt]);
        }
      }
      if constexpr (CS) {
        if (p.gn_stats) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float r = (float)o[v];
            cst.s[nt][v] += r;
            cst.q[nt][v] = fmaf(r, r, cst.q[nt][v]);
          }
        }
      }
    }
  }
  if (p.stats_out) {   // block-uniform: the two waves that share rows add up through LDS, one part per column tile
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      ssum[mt] = quad_sum(ssum[mt]);
      ssq[mt] = quad_sum(ssq[mt]);
    }
    __syncthreads();   // every wave is done with the tiles in LDS
    if (wn == 1 && lane < 16) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        red[(mt * 16 + lane) * 2] = ssum[mt];
        red[(mt * 16 + lane) * 2 + 1] = ssq[mt];
      }
    }
    __syncthreads();
    if (wn == 0 && lane < 16) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mbase + mt * 16 + lane;
        if (m >= p.M) continue;
        float2 o;
        o.x = ssum[mt] + red[(mt * 16 + lane) * 2];
        o.y = ssq[mt] + red[(mt * 16 + lane) * 2 + 1];
        *((float2*)p.stats_out + (long long)m * ntiles + ntile) = o;
      }
    }
  }
}

template <int MT, int NT>
__device__ __forceinline__ void epilogue_store(const IgemmParams& p, f32x4 (&acc)[MT][NT],
                                               const EpilogueIn<MT, NT>& in, int mbase, int gnt0, int lane, int HWo,
                                               int split, const float* lnrow, float* red, int wn, int ntile,
                                               int ntiles) {
  ColStats<NT> none;
  epilogue_store_cs<MT, NT, false>(p, acc, in, mbase, gnt0, lane, HWo, split, lnrow, red, wn, ntile, ntiles, none);
}

template <int BM, int BN, int NSETS>
__global__ __launch_bounds__(256, 2) void igemm_mfma_kernel(IgemmParams p, FastDiv mtiles, FastDiv ntiles, int ksteps_total,
                                                         int stages_per_split) {
  constexpr int WM = 2, WN = 2;
  constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 16, NT = WTN / 16;
  constexpr int ROWB = 80;             // LDS row pitch: 32 bf16 + 16 bytes pad (16-lane b128 reads hit 64 distinct banks)
  constexpr int CPR = 4;               // 16-byte chunks per row
  constexpr int NLD = BM * CPR / 256;  // chunks each thread stages
  constexpr int D = NSETS - 1;         // prefetch distance in 32-deep K stages
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][BM * ROWB];
  __shared__ float lnrow[BM * 2], red[BM * 2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const TileId tile = tile_of_block(mtiles, ntiles, p.splitk > 1 ? p.splitk : 1, p.xcd_chunked);
  if (!tile.valid) return;  // padding block (uniform for the whole block, before any barrier)
  const int mtile = tile.mtile, ntile = tile.ntile;
  const int m0 = mtile * BM, n0 = ntile * BN;
  ln_rows_to_lds(p, m0, BM, lnrow);   // read by the epilogue, after the barriers of the main loop
  const int Ct = p.C1 + p.C2;
  const int pad = p.ksize >> 1;
  const int HWo = p.Hout * p.Wout;
  const int Hs = p.upsample ? p.Hin * 2 : p.Hin, Wsz = p.upsample ? p.Win * 2 : p.Win;
  const int ups = p.upsample;
  const char* s1 = (const char*)p.src1;
  const char* s2 = (const char*)p.src2;
  const char* Wp = (const char*)p.W + ((p.slot_m > 0 && m0 >= p.slot_m) ? p.slot_w_bytes : 0);

  // ---- loader slots of this thread: output pixel of the row, top-left tap position, LDS address
  int ld_y[NLD], ld_x[NLD], ld_lds[NLD];
  unsigned ld_pix0[NLD];
  bool ld_ok[NLD];
  const int cq = tid & (CPR - 1);
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    int row = (tid + i * 256) / CPR;
    ld_lds[i] = row * ROWB + cq * 16;
    int m = m0 + row;
    ld_ok[i] = m < p.M;
    int mm = ld_ok[i] ? m : 0;
    int n = fast_div(mm, p.fd_hw);
    int r = mm - n * HWo;
    int oy = fast_div(r, p.fd_w), ox = r - oy * p.Wout;
    ld_y[i] = oy * p.stride - pad;
    ld_x[i] = ox * p.stride - pad;
    ld_pix0[i] = (unsigned)n * (unsigned)(p.Hin * p.Win);
  }

  // ---- K range of this split, and the cursor of the next stage to load
  const int stage0 = tile.split * stages_per_split;
  int nstages = ksteps_total - stage0;
  if (nstages > stages_per_split) nstages = stages_per_split;
  int l_k32 = stage0;
  const int k32_last = ksteps_total - 1;
  int l_c, l_ky, l_kx;
  {
    int kk = stage0 * 32;
    int tap = fast_div(kk, p.fd_ct);
    l_c = kk - tap * Ct;
    l_ky = fast_div(tap, p.fd_ks);
    l_kx = tap - l_ky * p.ksize;
  }

  // weight fragments of this wave: global n-tile index gnt0 + nt, 1 KB per (n-tile, k-step)
  const int gnt0 = (n0 + wn * WTN) >> 4;
  const int ntiles_total = p.N >> 4;
  unsigned boff[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int g = gnt0 + nt;
    if (g >= ntiles_total) g = ntiles_total - 1;  // columns past N are computed on valid data and dropped
    boff[nt] = ((unsigned)g * (unsigned)ksteps_total * 64u + (unsigned)lane) * 16u;
  }

  u32x4 areg[NSETS][NLD];
  bf16x8 breg[NSETS][NT];
  unsigned okm[NSETS];

  // issues the global loads of the cursor's stage into register set `set` (no waits, no branches):
  // rows in the padding read a clamped in-range pixel and are zeroed when they are written to LDS
  auto load = [&](auto setc) {
    constexpr int set = decltype(setc)::value;
    const char* src;
    int Cs, c = l_c;
    if (c < p.C1) { src = s1; Cs = p.C1; } else { src = s2; Cs = p.C2; c -= p.C1; }
    unsigned m = 0;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      int iy = ld_y[i] + l_ky, ix = ld_x[i] + l_kx;
      bool ok = ld_ok[i] && (unsigned)iy < (unsigned)Hs && (unsigned)ix < (unsigned)Wsz;
      iy = min(max(iy, 0), Hs - 1) >> ups;
      ix = min(max(ix, 0), Wsz - 1) >> ups;
      unsigned off = ((ld_pix0[i] + (unsigned)(iy * p.Win + ix)) * (unsigned)Cs + (unsigned)(c + cq * 8)) * 2u;
      areg[set][i] = *(const u32x4*)(src + off);
      m |= (ok ? 1u : 0u) << i;
    }
    okm[set] = m;
    const unsigned kb = (unsigned)min(l_k32, k32_last) * 1024u;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) breg[set][nt] = *(const bf16x8*)(Wp + (boff[nt] + kb));
    ++l_k32;
    l_c += 32;
    if (l_c >= Ct) {
      l_c = 0;
      if (++l_kx == p.ksize) { l_kx = 0; ++l_ky; }
    }
  };

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  int buf = 0;
  // one 32-deep stage: stage the activations loaded D stages ago, sync, prefetch D stages ahead, multiply
  auto stage = [&](auto setc) {
    constexpr int set = decltype(setc)::value;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      u32x4 v = areg[set][i];
      if (!((okm[set] >> i) & 1u)) v = u32x4{0u, 0u, 0u, 0u};
      *(u32x4*)(&lds[buf][ld_lds[i]]) = v;
    }
    __syncthreads();
    load(IC<(set + D) % NSETS>{});  // unconditional: past the end the cursor re-reads in-range data that is never used
    bf16x8 af[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      af[mt] = *(const bf16x8*)(&lds[buf][(wm * WTM + mt * 16 + (lane & 15)) * ROWB + (lane >> 4) * 16]);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(breg[set][nt], af[mt], acc[mt][nt], 0, 0, 0);
    buf ^= 1;
  };

  load(IC<0>{});
  if constexpr (D > 1) load(IC<1>{});
  if constexpr (D > 2) load(IC<2>{});
  for (int base = 0; base < nstages; base += NSETS) {
    stage(IC<0>{});
    if (base + 1 >= nstages) break;
    stage(IC<1>{});
    if constexpr (NSETS > 2) {
      if (base + 2 >= nstages) break;
      stage(IC<2>{});
    }
    if constexpr (NSETS > 3) {
      if (base + 3 >= nstages) break;
      stage(IC<3>{});
    }
  }

  EpilogueIn<MT, NT> epi_in;
  epilogue_load<MT, NT>(p, epi_in, m0 + wm * WTM, gnt0, lane, HWo);
  epilogue_store<MT, NT>(p, acc, epi_in, m0 + wm * WTM, gnt0, lane, HWo, tile.split, lnrow + wm * WTM * 2,
                         red + wm * WTM * 2, wn, ntile, (int)ntiles.d);
}

// ---------------------------------------------------------------------------------------------------
// Kernel with direct global -> LDS loads (global_load_lds_dwordx4): no staging registers, no ds_write
// phase.  One wave-wide load moves 1 KB: lane l's 16 bytes land at (wave-uniform LDS base) + 16 l, while the
// global address is free per lane.  Weights: one load per packed fragment (already in ds_read order).
// Activations: one load covers 8 rows of 128 bytes (64 channels); rows are unpadded, so lane (row r, slot j)
// fetches the row's 16-byte chunk j ^ ((r >> 1) & 7) and the fragment reads apply the same XOR, which spreads
// the 16 rows of a fragment over all banks.  Rows outside the image or past M read the zero page instead.
//
// Pipeline, three shapes (launch_ring picks one per launch):
//  * NBUF = 2, two barriers per stage: a wave reads ALL fragments of stage s into registers, the block synchronises,
//    and the buffer is immediately refilled with stage s+2 while the MFMAs of stage s run.  For launches with two
//    blocks per compute unit (three buffers would leave room for one).
//  * NBUF = 3, ONEBAR: loads run two stages ahead into the buffer whose stage was multiplied before the last
//    barrier, so the barrier that publishes stage s also frees the buffer of stage s-1: one barrier per stage.
//    -10 % on the launches with one block per unit; a fourth buffer (three stages ahead) gains nothing more.
//  * KG = 2: eight waves, two groups with two buffers each; group g multiplies stages g, g+2, ... of the block's
//    range and the groups swap halves of their accumulators through LDS before the epilogue.
// 256-row tiles on 8 waves (weight columns fetched once for twice the rows) were slower: 121 us against 105 us on
// the 16384x640x5760 layer.  The loads are issued from inline assembly and
// waited for with explicit vmcnt values (every wave issues the same number per stage), because the compiler
// would otherwise drain all outstanding loads before each LDS read.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_dma16(const void* gsrc, unsigned lds_base) {
  // m0 = wave-uniform LDS byte address of lane 0's destination; saved and restored around the load
  unsigned keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, off\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(keep)
      : "s"(lds_base), "v"(gsrc)
      : "memory");
}

// waits until at most min(ahead, NBUF-1) * NLOADS of this wave's loads are outstanding (s_waitcnt takes an immediate)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
template <int NBUF, int NLOADS> __device__ __forceinline__ void wait_stages_ahead(int ahead) {
  if constexpr (NBUF > 1) {
    if (ahead >= NBUF - 1) { wait_vmcnt<(NBUF - 1) * NLOADS>(); return; }
    wait_stages_ahead<NBUF - 1, NLOADS>(ahead);
  } else {
    wait_vmcnt<0>();
  }
}

template <int BM, int BN, int NBUF, bool ONEBAR, int KG>
__global__ __launch_bounds__(256 * KG, KG == 1 ? 2 : 1) void igemm_dma_kernel(IgemmParams p, FastDiv mtiles,
                                                                             FastDiv ntiles, int ksteps_total,
                                                                             int stages_per_split) {
  static_assert(KG == 1 || (KG == 2 && NBUF == 2 && !ONEBAR), "two wave groups: two buffers each");
  constexpr int WM = 2, WN = 2, NW = 4;
  constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 16, NT = WTN / 16;
  constexpr int NLA = BM / 8 / NW, NLB = BN / 8 / NW;   // 1 KB loads per wave and stage: activation row groups, weight fragments
  static_assert(BM % 32 == 0 && BN % 32 == 0, "loads must divide evenly over the waves");
  constexpr int NLOADS = NLA + NLB;
  constexpr int ABYTES = BM * 128, BBYTES = BN * 128, STAGE = ABYTES + BBYTES;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // NBUF stages of [A | B]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6) & 3;   // within its group
  const int grp = KG == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 8);
  const int wm = wave & 1, wn = wave >> 1;
  const TileId tile = tile_of_block(mtiles, ntiles, p.splitk > 1 ? p.splitk : 1, p.xcd_chunked);
  if (!tile.valid) return;  // padding block (uniform for the whole block, before any barrier)
  const int m0 = tile.mtile * BM, n0 = tile.ntile * BN;
  const int Ct = p.C1 + p.C2;
  const int pad = p.ksize >> 1;
  const int HWo = p.Hout * p.Wout;
  const int Hs = p.upsample ? p.Hin * 2 : p.Hin, Wsz = p.upsample ? p.Win * 2 : p.Win;
  const int ups = p.upsample;
  const char* s1 = (const char*)p.src1;
  const char* s2 = (const char*)p.src2;
  const char* Wp = (const char*)p.W + ((p.slot_m > 0 && m0 >= p.slot_m) ? p.slot_w_bytes : 0);
  const char* zeros = (const char*)p.zeros;
  unsigned char* ring = lds + grp * (NBUF * STAGE);   // this group's stage buffers
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) void*)ring;
  float* lnrow = (float*)(lds + KG * NBUF * STAGE);   // [BM][2] mean, rstd of the input rows (folded LayerNorm)
  float* red = lnrow + BM * 2;                   // [BM][2] row statistics of the other column half

  // A loads of this lane: load i of wave w fills LDS rows (i*NW + w)*8 .. +7
  int ld_y[NLA], ld_x[NLA];
  unsigned ld_pix0[NLA], ld_ch[NLA];
  bool ld_ok[NLA];
#pragma unroll
  for (int i = 0; i < NLA; ++i) {
    const int row = (i * NW + wave) * 8 + (lane >> 3);
    ld_ch[i] = (unsigned)(((lane & 7) ^ ((row >> 1) & 7)) * 8);   // first channel of the chunk this lane fetches
    const int m = m0 + row;
    ld_ok[i] = m < p.M;
    const int mm = ld_ok[i] ? m : 0;
    const int n = fast_div(mm, p.fd_hw);
    const int r = mm - n * HWo;
    const int oy = fast_div(r, p.fd_w), ox = r - oy * p.Wout;
    ld_y[i] = oy * p.stride - pad;
    ld_x[i] = ox * p.stride - pad;
    ld_pix0[i] = (unsigned)n * (unsigned)(p.Hin * p.Win);
  }
  // B loads: load i of wave w is fragment f = i*NW + w of the stage: n-tile f/2, k-step f%2
  const int gnt_blk = n0 >> 4, ntiles_total = p.N >> 4;
  const int total_stages = ksteps_total >> 1;
  const int stage0 = tile.split * stages_per_split;
  int nstages = total_stages - stage0;
  if (nstages > stages_per_split) nstages = stages_per_split;
  const int nstages_all = nstages;
  if constexpr (KG > 1) nstages = (nstages - grp + KG - 1) / KG;   // group g takes stages g, g + KG, ... of the block's range
  int l_stage = stage0 + grp;
  const int stage_last = total_stages - 1;
  const char* bptr[NLB];   // this lane's 16 bytes of fragment i in the cursor's stage
#pragma unroll
  for (int i = 0; i < NLB; ++i) {
    const int f = i * NW + wave;
    int g = gnt_blk + (f >> 1);
    if (g >= ntiles_total) g = ntiles_total - 1;  // columns past N are computed on valid data and dropped
    bptr[i] = Wp + ((unsigned)g * (unsigned)ksteps_total * 64u + (unsigned)((f & 1) * 64 + lane)) * 16u +
              (unsigned)min(l_stage, stage_last) * 2048u;
  }

  // The K axis may carry a second segment behind the ksize x ksize taps: a 1x1 convolution over src3 | src4 (the
  // skip path of a ResBlock, summed into the same accumulators).  cur_* describe the segment the cursor is in.
  int l_c, l_ky, l_kx;
  const char* cur_s1 = s1;
  const char* cur_s2 = s2;
  int cur_C1 = p.C1, cur_Ct = Ct, cur_ks = p.ksize, cur_off = 0;   // cur_off: added to the tap offsets (pad of segment 1)
  bool seg2 = false;
  auto enter_seg2 = [&]() {
    seg2 = true;
    cur_s1 = (const char*)p.src3;
    cur_s2 = (const char*)p.src4;
    cur_C1 = p.C3;
    cur_Ct = p.C3 + p.C4;
    cur_ks = 1;
    cur_off = pad;
    l_ky = 0;
    l_kx = 0;
  };
  {
    int kk = (stage0 + grp) * 64;
    const int k_seg1 = p.ksize * p.ksize * Ct;
    if (p.C3 > 0 && kk >= k_seg1) {
      enter_seg2();
      l_c = kk - k_seg1;
    } else {
      int tap = fast_div(kk, p.fd_ct);
      l_c = kk - tap * Ct;
      l_ky = fast_div(tap, p.fd_ks);
      l_kx = tap - l_ky * p.ksize;
    }
  }

  // Per-lane source address and validity of every A load for the cursor's position.  Inside a tap and a source
  // the address just advances by 64 channels per stage; it is rebuilt when the tap or the source changes.
  // (The cursor is advanced once more after the last stage is issued: there the tap index leaves the kernel
  // window and the rebuilt entries are marked invalid; they are never used.)
  const char* aptr[NLA];   // meaningless (and unused) where !okv
  bool okv[NLA];
  auto set_tap = [&]() {
    const bool live = l_ky < cur_ks;
    const char* src;
    int Cs, c = l_c;
    if (c < cur_C1) { src = cur_s1; Cs = cur_C1; } else { src = cur_s2; Cs = cur_Ct - cur_C1; c -= cur_C1; }
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
      const int iy = ld_y[i] + l_ky + cur_off, ix = ld_x[i] + l_kx + cur_off;
      okv[i] = live && ld_ok[i] && (unsigned)iy < (unsigned)Hs && (unsigned)ix < (unsigned)Wsz;
      const unsigned lin = ld_pix0[i] + (unsigned)((iy >> ups) * p.Win + (ix >> ups));
      aptr[i] = src + (lin * (unsigned)Cs + (unsigned)c + ld_ch[i]) * 2u;
    }
  };
  set_tap();

  // issues the NLOADS loads of the cursor's stage into LDS buffer `buf` and advances the cursor
  auto advance = [&]() {
#pragma unroll
    for (int i = 0; i < NLA; ++i) aptr[i] += 128;
    const int bstep = l_stage < stage_last ? 2048 : 0;   // the pointer never leaves the packed weights
#pragma unroll
    for (int i = 0; i < NLB; ++i) bptr[i] += bstep;
    ++l_stage;
    l_c += 64;
    if (l_c == cur_C1 || l_c >= cur_Ct) {       // next source of a concatenation, next tap, or next segment
      if (l_c >= cur_Ct) {
        l_c = 0;
        if (++l_kx == cur_ks) { l_kx = 0; ++l_ky; }
        if (l_ky == cur_ks && !seg2 && p.C3 > 0) enter_seg2();
      }
      set_tap();
    }
  };
  auto issue = [&](int buf) {
    const unsigned sa = lds0 + buf * STAGE;
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
      const char* g = okv[i] ? aptr[i] : zeros;
#ifdef SDSTREAM_DEVHOOKS
      if (p.dev_exp & 256) g = zeros;
      if (p.dev_exp & 4096) continue;
#endif
      lds_dma16(g, sa + (i * NW + wave) * 1024);
    }
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
      const char* g = bptr[i];
#ifdef SDSTREAM_DEVHOOKS
      if (p.dev_exp & 512) g = zeros;
      if (p.dev_exp & 2048) continue;
#endif
      lds_dma16(g, sa + ABYTES + (i * NW + wave) * 1024);
    }
#pragma unroll
    for (int g = 0; g < KG; ++g) advance();
  };

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // fragment read addresses of this lane (row and XOR term are the same for both k-steps)
  int a_row[MT], a_x[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int r = wm * WTM + mt * 16 + (lane & 15);
    a_row[mt] = r * 128;
    a_x[mt] = (r >> 1) & 7;
  }

  // 64-row tiles (the short-K layers): what the epilogue reads is requested ahead of the main loop.  These
  // loads are older than every LDS load below, so the first stage's vmcnt wait covers them.
  EpilogueIn<MT, NT> epi_in;
  if constexpr (BM == 64 && KG == 1) epilogue_load<MT, NT>(p, epi_in, m0 + wm * WTM, (n0 + wn * WTN) >> 4, lane, HWo);
  constexpr int PRE = ONEBAR ? NBUF - 1 : NBUF;   // stages in flight ahead of the one being multiplied
#pragma unroll
  for (int b = 0; b < PRE; ++b)
    if (b < nstages) issue(b);
  // after the first stages are on their way: the wait for these loads also waits for those, which the loop would do next anyway
  ln_rows_to_lds(p, m0, BM, lnrow);

  // Rotated loop: the MFMAs of a stage's second k-step are issued together with the fragment reads of the next
  // stage's first k-step, so half of the LDS read latency sits in the shadow of the matrix cores.
  bf16x8 af[2][MT], bfr[2][NT];
  auto read_frags = [&](int ks, int buf) {
#ifdef SDSTREAM_DEVHOOKS
    if ((p.dev_exp & 1024) && (ks | buf) != 0) return;
#endif
    const unsigned char* sa = ring + buf * STAGE;
    const unsigned char* sb = sa + ABYTES;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      af[ks][mt] = *(const bf16x8*)(sa + a_row[mt] + (((ks * 4 + (lane >> 4)) ^ a_x[mt]) << 4));
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) bfr[ks][nt] = *(const bf16x8*)(sb + ((wn * NT + nt) * 2 + ks) * 1024 + lane * 16);
  };
  auto mfmas = [&](int ks) {
#ifdef SDSTREAM_DEVHOOKS
    if (p.dev_exp & 4) return;
#endif
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[ks][nt], af[ks][mt], acc[mt][nt], 0, 0, 0);
  };
  static_assert((NBUF - 1) * NLOADS < 64, "vmcnt is a 6-bit counter");
  static_assert(!ONEBAR || NBUF >= 3, "one barrier per stage needs a buffer nobody reads");
  int buf = 0;
  if constexpr (KG == 2) {
    // Two wave groups split the block's K range stage by stage (in-block split-K: a compute unit with one block
    // still has two waves per SIMD, and no partial tile leaves the unit).  Both run the two-barrier loop, the
    // second group half an iteration behind: while one group reads fragments the other issues its loads, and
    // every barrier is passed by all eight waves (each group uses every other one).
    const int iters = (nstages_all + 1) >> 1;   // of the first group; the second has as many or one less
    if (grp == 1) __syncthreads();
    for (int s = 0; s < iters; ++s) {
      const bool live = s < nstages;
      if (live) wait_stages_ahead<NBUF, NLOADS>(nstages - 1 - s);
      __syncthreads();
      if (live) {
        read_frags(0, buf);
        if (s > 0) {
          mfmas(1);
#pragma unroll
          for (int i = 0; i < MT + NT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
          }
        }
        read_frags(1, buf);
      }
      __syncthreads();
      if (live) {
        if (s + NBUF < nstages) issue(buf);
        mfmas(0);
        buf ^= 1;
      }
    }
    if (grp == 0) __syncthreads();
  } else {
  for (int s = 0; s < nstages; ++s) {
    // all but this wave's loads of the stages after s (NBUF-1 of them, fewer at the end: nothing is loaded past
    // the last stage - on the short-K layers two more stages would be a third of the traffic) have landed
    wait_stages_ahead<PRE, NLOADS>(nstages - 1 - s);
    __syncthreads();                     // ... and everyone else's part of stage s too
    read_frags(0, buf);
    if (s > 0) {
      mfmas(1);                          // second k-step of stage s-1
#pragma unroll
      for (int i = 0; i < MT + NT; ++i) {   // one fragment read per two MFMAs, as long as both last
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      }
    }
    read_frags(1, buf);
    if constexpr (ONEBAR) {
      // every wave has passed this stage's barrier, so it holds its fragments of stage s-1: that buffer is free
      if (s + PRE < nstages) issue(buf == 0 ? NBUF - 1 : buf - 1);   // stage s+NBUF-1
    } else {
      __syncthreads();                     // every wave holds its fragments: the buffer can be refilled
      if (s + NBUF < nstages) issue(buf);  // stage s+NBUF
    }
    mfmas(0);
    buf = buf + 1 == NBUF ? 0 : buf + 1;
  }
  }
  if (nstages > 0) mfmas(1);
  if constexpr (KG == 2) {
    // The groups swap halves of their accumulators through LDS: each ends up with the sums of 32 of the wave
    // tile's 64 rows and runs the epilogue on those.
    constexpr int MH = MT / 2;
    const int row0 = wm * WTM + grp * (MH * 16);
    EpilogueIn<MH, NT> hin;
    epilogue_load<MH, NT>(p, hin, m0 + row0, (n0 + wn * WTN) >> 4, lane, HWo);
    f32x4 fin[MH][NT];
    f32x4* xch = (f32x4*)lds;   // [group][wave][MH * NT][lane]
    __syncthreads();            // both groups are done with the stage buffers
    f32x4* mine = xch + ((grp * NW + wave) * (MH * NT)) * 64 + lane;
    const f32x4* theirs = xch + (((grp ^ 1) * NW + wave) * (MH * NT)) * 64 + lane;
    if (grp == 0) {
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) mine[(i * NT + j) * 64] = acc[MH + i][j];
    } else {
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) mine[(i * NT + j) * 64] = acc[i][j];
    }
    __syncthreads();
    if (grp == 0) {
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) fin[i][j] = acc[i][j] + theirs[(i * NT + j) * 64];
    } else {
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) fin[i][j] = theirs[(i * NT + j) * 64] + acc[MH + i][j];
    }
    ColStats<NT> cst;
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) { cst.s[j][v] = 0.f; cst.q[j][v] = 0.f; }
    epilogue_store_cs<MH, NT, true>(p, fin, hin, m0 + row0, (n0 + wn * WTN) >> 4, lane, HWo, tile.split,
                                    lnrow + row0 * 2, red + row0 * 2, wn, tile.ntile, (int)ntiles.d, cst);
    if (p.gn_stats) {
      // GroupNorm statistics of the block's 128 rows x BN columns for the norm that follows (block-uniform branch;
      // the launcher has checked that the rows lie in one sample and that groups do not straddle column tiles):
      // columns over the 16 lanes of a row, then over the four waves that share the columns, then channels to groups.
      // Every sum is taken in a fixed order.
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          cst.s[j][v] = row16_sum(cst.s[j][v]);
          cst.q[j][v] = row16_sum(cst.q[j][v]);
        }
      float* cred = (float*)lds;   // [4 row groups][BN columns][2]
      __syncthreads();             // the accumulator exchange above is read
      if ((lane & 15) == 0) {
        const int rg = grp * 2 + wm;
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int col = wn * WTN + j * 16 + (lane >> 4) * 4 + v;
            cred[(rg * BN + col) * 2] = cst.s[j][v];
            cred[(rg * BN + col) * 2 + 1] = cst.q[j][v];
          }
      }
      __syncthreads();
      const int cg = p.gn_cg, gtile = BN / cg;
      if (tid < gtile * 2) {   // one thread per (group, sum | sum of squares)
        const int gi = tid >> 1, st = tid & 1;
        float a = 0.f;
        for (int c = gi * cg; c < (gi + 1) * cg; ++c)
          a += (cred[(0 * BN + c) * 2 + st] + cred[(1 * BN + c) * 2 + st]) +
               (cred[(2 * BN + c) * 2 + st] + cred[(3 * BN + c) * 2 + st]);
        const int smp = fast_div(m0, p.fd_hw);
        const int sp = (m0 - smp * HWo) / BM, nsp = HWo / BM;
        p.gn_stats[(((long long)smp * nsp + sp) * p.gn_groups + n0 / cg + gi) * 2 + st] = a;
      }
    }
  } else {
    if constexpr (BM != 64) epilogue_load<MT, NT>(p, epi_in, m0 + wm * WTM, (n0 + wn * WTN) >> 4, lane, HWo);
    epilogue_store<MT, NT>(p, acc, epi_in, m0 + wm * WTM, (n0 + wn * WTN) >> 4, lane, HWo, tile.split,
                           lnrow + wm * WTM * 2, red + wm * WTM * 2, wn, tile.ntile, (int)ntiles.d);
  }
}

// Kernel for 1x1 layers with a short K on many rows (K = 32 KSTEPS channels): the block's BM input rows stay in LDS
// for the whole launch (loaded once, against once per column tile in the kernel above), and the weights never touch
// LDS - every wave owns 32-column slices of the block's column range and reads its two packed fragments per k-step
// straight from global memory into a ring of registers five k-steps deep.  After the prologue nothing synchronises:
// the waves (two or more per SIMD) run at their own pace, so one wave's epilogue overlaps the others' MFMAs.
// Two shapes: 128 rows x 8 waves walking many slices each (GEGLU input, fused q/k/v of the first level), and
// 64 rows x 10 waves with one slice each for N = 320 (the projections around the attentions of the first level),
// where the waves meet once at the end to add up the row statistics a following folded LayerNorm reads.
template <int KSTEPS, int BM, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 1) void igemm_rows_kernel(IgemmParams p, int nsplit, int slices_per_block) {
  constexpr int MT = BM / 16, NT = 2, RING = 5;
  static_assert(KSTEPS % RING == 0 && KSTEPS % 2 == 0, "the ring keeps its phase from slice to slice");
  constexpr int STAGES = KSTEPS / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [STAGES][BM rows of 128 bytes, chunks XOR-swizzled]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mtile = blockIdx.x / nsplit, ns = blockIdx.x - mtile * nsplit;
  const int m0 = mtile * BM;
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) void*)lds;
  float* lnrow = (float*)(lds + STAGES * BM * 128);   // [BM][2] mean, rstd of the input rows (folded LayerNorm)
  float* red = lnrow + BM * 2;                        // [WAVES][BM][2] row statistics per wave
  const int K = KSTEPS * 32;
  const bool slot1 = p.slot_m > 0 && m0 >= p.slot_m;  // rows of the second prompt: second set of weights and vectors
  const long long voff = slot1 ? p.slot_v_bytes / 4 : 0;

  // the rows: STAGES x BM/8 loads of 1 KB (8 rows of 64 channels each), dealt over the waves
  {
    const char* A = (const char*)p.src1;
    const char* zeros = (const char*)p.zeros;
    for (int i = wave; i < STAGES * (BM / 8); i += WAVES) {
      const int st = i / (BM / 8), rg = i - st * (BM / 8);
      const int row = rg * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      const int m = m0 + row;
      const char* g = m < p.M ? A + ((long long)m * K + st * 64 + chunk * 8) * 2 : zeros;
      lds_dma16(g, lds0 + st * (BM * 128) + rg * 1024);
    }
  }
  ln_rows_to_lds(p, m0, BM, lnrow);

  // this wave's slices: s_lo + wave, s_lo + wave + WAVES, ... below s_hi; slice = 32 columns = two packed n-tiles
  const int s_lo = ns * slices_per_block;
  const int s_hi = min(s_lo + slices_per_block, p.N >> 5);
  const char* W = (const char*)p.W + (slot1 ? p.slot_w_bytes : 0);
  auto frag_ptr = [&](int slice, int t, int ks) {
    return (const bf16x8*)(W + (((long long)(slice * 2 + t) * KSTEPS + ks) * 64 + lane) * 16);
  };
  bf16x8 bq[RING][NT];
  int slice = s_lo + wave;
  if (slice < s_hi) {
#pragma unroll
    for (int r = 0; r < RING; ++r)
#pragma unroll
      for (int t = 0; t < NT; ++t) bq[r][t] = *frag_ptr(slice, t, r);
  }
  int a_off[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) a_off[mt] = (mt * 16 + (lane & 15)) * 128;
  const int a_x = ((lane & 15) >> 1) & 7;   // (row >> 1) & 7 with row = mt * 16 + lane % 16
  __builtin_amdgcn_s_waitcnt(0x0F70 | 0 | (0 << 14));   // vmcnt(0): the rows (and the first fragments) have landed
  __syncthreads();
  if constexpr (BM == 64) {
    if (p.gn_in_stats) {
      // GroupNorm of the input rows, in place in LDS, with the arithmetic of the norm's own apply pass (partial sums
      // folded in double in a fixed order, y = fma(x, rstd gamma, beta - mean rstd gamma), rounded to bf16): what
      // this layer multiplies is bit for bit what that pass would have written.  The block's rows lie in one sample.
      float* gmr = red;   // [groups][2] mean, rstd (the row-statistics area is not in use yet)
      const int HWo = p.Hout * p.Wout, smp = m0 / HWo;
      const int groups = p.gn_in_groups, cg = K / groups, nsp = p.gn_in_splits;
      for (int idx = tid; idx < groups * 8; idx += 64 * WAVES) {
        const int gi = idx >> 3, part = idx & 7;
        double ss = 0.0, qq = 0.0;
        for (int k = part; k < nsp; k += 8) {
          const float* src = p.gn_in_stats + (((long long)smp * nsp + k) * groups + gi) * 2;
          ss += src[0];
          qq += src[1];
        }
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) {
          ss += __shfl_xor(ss, o);
          qq += __shfl_xor(qq, o);
        }
        if (part == 0) {
          const double cnt = (double)HWo * cg;
          const double mean = ss / cnt;
          double var = qq / cnt - mean * mean;
          if (var < 0) var = 0;
          gmr[gi * 2] = (float)mean;
          gmr[gi * 2 + 1] = (float)(1.0 / sqrt(var + (double)p.gn_in_eps));
        }
      }
      __syncthreads();
      float* scsh = gmr + groups * 2;   // [K][2] scale, shift per channel
      for (int ch = tid; ch < K; ch += 64 * WAVES) {
        const int gi = ch / cg;
        const float rs = gmr[gi * 2 + 1] * p.gn_in_gamma[ch];
        scsh[ch * 2] = rs;
        scsh[ch * 2 + 1] = p.gn_in_beta[ch] - gmr[gi * 2] * rs;
      }
      __syncthreads();
      constexpr int CHUNKS = KSTEPS * 4;   // 16-byte chunks per row
      for (int i = tid; i < BM * CHUNKS; i += 64 * WAVES) {
        const int r = i / CHUNKS, c = i - r * CHUNKS;
        bf16x8* cell = (bf16x8*)(lds + (c >> 3) * (BM * 128) + r * 128 + (((c & 7) ^ ((r >> 1) & 7)) << 4));
        bf16x8 v = *cell;
        const f32x4* ss = (const f32x4*)(scsh + c * 16);   // (scale, shift) of the chunk's 8 channels
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const f32x4 t = ss[e >> 1];
          v[e] = (bf16_t)fmaf((float)v[e], t[0], t[1]);
          v[e + 1] = (bf16_t)fmaf((float)v[e + 1], t[2], t[3]);
        }
        *cell = v;
      }
      __syncthreads();
    }
  }

  const int ncol = (lane >> 4) * 4;
  const float* zf = (const float*)p.zeros;
  bf16_t* out = (bf16_t*)p.out;
  const bf16_t* res = (const bf16_t*)p.residual;
  for (; slice < s_hi; slice += WAVES) {
    f32x4 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int next = slice + WAVES;
    const int n0 = slice * 32 + ncol, n1 = n0 + 16;
    // what the epilogue reads is requested ahead of the loop: bias and weight row sums (16 registers), and the
    // residual of the short shape (16 more; the tall shape has none)
    const f32x4 bias0 = *(const f32x4*)(p.bias ? p.bias + voff + n0 : zf), bias1 = *(const f32x4*)(p.bias ? p.bias + voff + n1 : zf);
    f32x4 ws0 = {0.f, 0.f, 0.f, 0.f}, ws1 = ws0;
    if constexpr (BM == 128) {   // (only the tall shape takes layers with a folded LayerNorm)
      ws0 = *(const f32x4*)(p.ln_wsum ? p.ln_wsum + voff + n0 : zf);
      ws1 = *(const f32x4*)(p.ln_wsum ? p.ln_wsum + voff + n1 : zf);
    }
    bf16x4 r0[MT], r1[MT];
    if constexpr (BM == 64) {
      if (res) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int m = min(m0 + mt * 16 + (lane & 15), p.M - 1);
          r0[mt] = *(const bf16x4*)(res + (long long)m * p.N + n0);
          r1[mt] = *(const bf16x4*)(res + (long long)m * p.N + n1);
        }
      }
    }
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      bf16x8 af[MT];
      const unsigned char* sa = lds + (ks >> 1) * (BM * 128);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) af[mt] = *(const bf16x8*)(sa + a_off[mt] + (((((ks & 1) * 4) + (lane >> 4)) ^ a_x) << 4));
      bf16x8 b0 = bq[ks % RING][0], b1 = bq[ks % RING][1];
      // refill the ring slot with the k-step RING ahead: of this slice, or of the wave's next one
      if (ks + RING < KSTEPS) {
        bq[ks % RING][0] = *frag_ptr(slice, 0, ks + RING);
        bq[ks % RING][1] = *frag_ptr(slice, 1, ks + RING);
      } else if (next < s_hi) {
        bq[ks % RING][0] = *frag_ptr(next, 0, ks + RING - KSTEPS);
        bq[ks % RING][1] = *frag_ptr(next, 1, ks + RING - KSTEPS);
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0, af[mt], acc[mt][0], 0, 0, 0);
        acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1, af[mt], acc[mt][1], 0, 0, 0);
      }
      // Keeps the scheduler from hoisting every k-step's row fragments (spills).  A second fragment set, read under
      // the previous k-step's MFMAs, was slower (37 against 33 us per launch): with two waves per SIMD the other
      // wave already fills the wait.
      __builtin_amdgcn_sched_barrier(0);
    }
    // epilogue of this kernel's layers: folded LayerNorm, bias, then GEGLU (value and gate tiles side by side) or
    // residual and plain store, with the row sums of what is stored for a LayerNorm folded into the next layer
    ColStats<NT> cst;   // short shape: column sums of what is stored, for a GroupNorm that follows
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) { cst.s[j][v] = 0.f; cst.q[j][v] = 0.f; }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int r = mt * 16 + (lane & 15), m = m0 + r;
      f32x4 x0 = acc[mt][0], x1 = acc[mt][1];
      if constexpr (BM == 128) {
        if (p.ln_stats) {
          const float mean = lnrow[r * 2], rstd = lnrow[r * 2 + 1];
          x0 = (x0 - mean * ws0) * rstd;
          x1 = (x1 - mean * ws1) * rstd;
        }
      }
      x0 += bias0;
      x1 += bias1;
      float ssum = 0.f, ssq = 0.f;
      if (m < p.M) {
        if (p.epilogue == EPI_GEGLU) {
          bf16x4 o;
#pragma unroll
          for (int v = 0; v < 4; ++v) o[v] = (bf16_t)(x0[v] * gelu_erf(x1[v]));
#ifdef SDSTREAM_DEVHOOKS
          if (p.dev_exp & 1) {
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = (bf16_t)(x0[v] * x1[v]);
          }
          if ((p.dev_exp & 2) && x0[0] != 12345.678f) continue;
#endif
          *(bf16x4*)(out + (long long)m * (p.N >> 1) + slice * 16 + ncol) = o;
        } else {
          if constexpr (BM == 64) {
            if (res) {
#pragma unroll
              for (int v = 0; v < 4; ++v) { x0[v] += (float)r0[mt][v]; x1[v] += (float)r1[mt][v]; }
            }
          }
          bf16x4 o0, o1;
#pragma unroll
          for (int v = 0; v < 4; ++v) { o0[v] = (bf16_t)x0[v]; o1[v] = (bf16_t)x1[v]; }
          *(bf16x4*)(out + (long long)m * p.N + n0) = o0;
          *(bf16x4*)(out + (long long)m * p.N + n1) = o1;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float a = (float)o0[v], b = (float)o1[v];
            ssum += a + b;
            ssq = fmaf(a, a, fmaf(b, b, ssq));
            if constexpr (BM == 64) {
              cst.s[0][v] += a; cst.q[0][v] = fmaf(a, a, cst.q[0][v]);
              cst.s[1][v] += b; cst.q[1][v] = fmaf(b, b, cst.q[1][v]);
            }
          }
        }
      }
      if constexpr (BM == 64) {
        if (p.stats_out) {   // block-uniform
          ssum = quad_sum(ssum);
          ssq = quad_sum(ssq);
          if (lane < 16) {
            red[(wave * BM + r) * 2] = ssum;
            red[(wave * BM + r) * 2 + 1] = ssq;
          }
        }
      }
    }
    if constexpr (BM == 64) {
      if (p.gn_stats) {   // block-uniform: this wave's 32 channel sums over the block's rows, into LDS
        float* cred = red + WAVES * BM * 2;   // [N columns][2]
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float a = row16_sum(cst.s[j][v]), b = row16_sum(cst.q[j][v]);
            if ((lane & 15) == 0) {
              const int col = slice * 32 + j * 16 + ncol + v;
              cred[col * 2] = a;
              cred[col * 2 + 1] = b;
            }
          }
      }
    }
  }
  if constexpr (BM == 64) {
    // every wave of the short shape has exactly one slice (the launcher sees to it), so all of them arrive here
    if (p.gn_stats) {   // channels to groups: one thread per (group, sum | sum of squares); the rows lie in one sample
      __syncthreads();
      const float* cred = red + WAVES * BM * 2;
      const int cg = p.gn_cg;
      if (tid < p.gn_groups * 2) {
        const int gi = tid >> 1, st = tid & 1;
        float a = 0.f;
        for (int c = gi * cg; c < (gi + 1) * cg; ++c) a += cred[c * 2 + st];
        const int HWo = p.Hout * p.Wout;
        const int smp = m0 / HWo, sp = (m0 - smp * HWo) / BM, nsp = HWo / BM;
        p.gn_stats[(((long long)smp * nsp + sp) * p.gn_groups + gi) * 2 + st] = a;
      }
    }
    if (p.stats_out) {
      __syncthreads();
      if (tid < BM && m0 + tid < p.M) {
        float2 o = {0.f, 0.f};
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
          o.x += red[(w * BM + tid) * 2];
          o.y += red[(w * BM + tid) * 2 + 1];
        }
        *((float2*)p.stats_out + (m0 + tid)) = o;   // one part per row
      }
    }
  }
}

// split-K finalize: sum of the partials (fp32 [splitk][M][N]) -> out with the epilogue of the main kernel
__global__ __launch_bounds__(256) void igemm_finalize_kernel(IgemmParams p) {
  const long long idx4 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total4 = (long long)p.M * p.N / 4;
  if (idx4 >= total4) return;
  const long long e = idx4 * 4;   // < 2^31 (checked by igemm_mfma_supported)
  const int m = fast_div((int)e, p.fd_n), n = (int)e - m * p.N;
  // the kernel is one latency chain per thread: issue every independent load before the first add
  const long long plane = (long long)p.M * p.N;
  f32x4 add = {0.f, 0.f, 0.f, 0.f};
  if (p.bias) add = *(const f32x4*)(p.bias + n);
  if (p.rowbias) add += *(const f32x4*)(p.rowbias + (long long)fast_div(m, p.fd_hw) * p.rowbias_ld + n);
  bf16x4 r = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
  if (p.residual) r = *(const bf16x4*)((const bf16_t*)p.residual + e);
  f32x4 x = *(const f32x4*)(p.workspace + e);
  int z = 1;
  for (; z + 4 <= p.splitk; z += 4) {   // same order of additions as one by one
    const f32x4 a = *(const f32x4*)(p.workspace + (long long)z * plane + e);
    const f32x4 b = *(const f32x4*)(p.workspace + (long long)(z + 1) * plane + e);
    const f32x4 c = *(const f32x4*)(p.workspace + (long long)(z + 2) * plane + e);
    const f32x4 d = *(const f32x4*)(p.workspace + (long long)(z + 3) * plane + e);
    x += a; x += b; x += c; x += d;
  }
  for (; z < p.splitk; ++z) x += *(const f32x4*)(p.workspace + (long long)z * plane + e);
  x += add;
#pragma unroll
  for (int v = 0; v < 4; ++v) x[v] += (float)r[v];
  bf16x4 o;
#pragma unroll
  for (int v = 0; v < 4; ++v) o[v] = (bf16_t)x[v];
  *(bf16x4*)((bf16_t*)p.out + e) = o;
}

template <int BM, int BN, int NSETS> void launch_cfg(const IgemmParams& p, hipStream_t s) {
  const int mtiles = (p.M + BM - 1) / BM, ntiles = (p.N + BN - 1) / BN;
  const int ksteps_total = p.K / 32;
  const int splitk = p.splitk > 1 ? p.splitk : 1;
  const int sps = (ksteps_total + splitk - 1) / splitk;
  dim3 grid((mtiles * ntiles * splitk + 7) & ~7);
  hipLaunchKernelGGL((igemm_mfma_kernel<BM, BN, NSETS>), grid, dim3(256), 0, s, p, make_fastdiv(mtiles),
                     make_fastdiv(ntiles), ksteps_total, sps);
  if (splitk > 1) {
    long long total4 = (long long)p.M * p.N / 4;
    hipLaunchKernelGGL(igemm_finalize_kernel, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s, p);
  }
}

template <int BM, int BN, int NBUF, bool ONEBAR = false, int KG = 1> void launch_dma(const IgemmParams& p, hipStream_t s) {
  constexpr int LDS = KG * NBUF * (BM + BN) * 128 + BM * 16;   // stages, then two [BM][2] float arrays of row statistics
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)igemm_dma_kernel<BM, BN, NBUF, ONEBAR, KG>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    attr_set = true;
  }
  const int mtiles = (p.M + BM - 1) / BM, ntiles = (p.N + BN - 1) / BN;
  const int ksteps_total = p.K / 32;
  const int total_stages = ksteps_total / 2;
  const int splitk = p.splitk > 1 ? p.splitk : 1;
  const int sps = (total_stages + splitk - 1) / splitk;
  dim3 grid((mtiles * ntiles * splitk + 7) & ~7);
  hipLaunchKernelGGL((igemm_dma_kernel<BM, BN, NBUF, ONEBAR, KG>), grid, dim3(256 * KG), LDS, s, p, make_fastdiv(mtiles),
                     make_fastdiv(ntiles), ksteps_total, sps);
  if (splitk > 1) {
    long long total4 = (long long)p.M * p.N / 4;
    hipLaunchKernelGGL(igemm_finalize_kernel, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s, p);
  }
}

// The layers igemm_rows_kernel takes: plain rows (1x1, one source), enough of them that 256 blocks have work, and
//  tall shape: K = 320 and N >= 960 on >= 4096 rows, no residual, no row statistics to leave (GEGLU input, fused q/k/v);
//  short shape: K = 320 or 640 and N = 320 (ten waves, one 32-column slice each).
// Returns 0, or the shape (1 tall, 2 short).  Must not depend on the row range or the weight slot of a launch: a
// layer launched on sub-ranges of its rows keeps the kernel chosen for the whole range (force_variant).
int rows_kernel_shape(const IgemmParams& p) {
  if (p.ksize != 1 || p.stride != 1 || p.upsample || p.C2 != 0 || p.C3 != 0 || p.rowbias || p.N % 32) return 0;
  if (p.epilogue == EPI_GEGLU || (p.epilogue == EPI_NONE && p.N >= 960)) {
    if (p.C1 != 320 || p.stats_out || p.residual) return 0;
    return (p.M + 127) / 128 >= 32 ? 1 : 0;   // (from one 64 x 64 sample on: 23 -> 15 us per launch there)
  }
  if (p.epilogue == EPI_NONE && p.N == 320 && (p.C1 == 320 || p.C1 == 640) && !p.ln_stats)
    return (p.M + 63) / 64 >= 200 ? 2 : 0;
  return 0;
}

template <int KSTEPS, int BM, int WAVES> void launch_rows_t(const IgemmParams& p, int nsplit, hipStream_t s) {
  constexpr int LDS = (KSTEPS / 2) * BM * 128 + BM * 8 + WAVES * BM * 8 + (BM == 64 ? 320 * 8 : 0);
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)igemm_rows_kernel<KSTEPS, BM, WAVES>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    attr_set = true;
  }
  const int mtiles = (p.M + BM - 1) / BM;
  const int slices = p.N / 32;
  const int spb = (slices + nsplit - 1) / nsplit;
  hipLaunchKernelGGL((igemm_rows_kernel<KSTEPS, BM, WAVES>), dim3(mtiles * nsplit), dim3(64 * WAVES), LDS, s, p, nsplit, spb);
}

void launch_rows(const IgemmParams& p, hipStream_t s) {
  if (p.N == 320 && p.epilogue == EPI_NONE) {   // short shape: ten slices, one per wave
    if (p.C1 == 320) launch_rows_t<10, 64, 10>(p, 1, s); else launch_rows_t<20, 64, 10>(p, 1, s);
    return;
  }
  const int mtiles = (p.M + 127) / 128;
  launch_rows_t<10, 128, 8>(p, mtiles >= 256 ? 1 : 256 / mtiles, s);
}

struct Choice { int variant, bn, splitk; };  // variant 0: 32-deep stages, weights through registers (any C % 32 == 0);
                                             // 1: direct-to-LDS kernel with 128-row tiles, 2: with 64-row tiles,
                                             // 3: row-resident kernel (bn = N: one part of row statistics per row)

// Tile / kernel / split-K selection, from per-layer timings of the SD-shaped net on MI355X (256 compute units).
// What the timings say: a layer runs best with about one 128-row tile per compute unit - 256 blocks beat 512 blocks
// of half the size or half the K range (fewer fetches of each operand across L2 -> LDS, fewer partial tiles) -
// until a block's share of K passes ~100 stages, where a second block per unit pays again.  Layers with fewer tiles
// than that split K if K is long, and otherwise fall back to 64-row tiles.
Choice choose(const IgemmParams& p) {
  Choice c;
  const bool k64 = p.C1 % 64 == 0 && p.C2 % 64 == 0 && p.C3 % 64 == 0 && p.C4 % 64 == 0;
  const bool geglu = p.epilogue == EPI_GEGLU;
  const bool softmax = p.epilogue == EPI_SOFTMAX;   // its segments need the 80-column wave tile
  const int bn0 = softmax ? 160 : geglu ? 128 : p.N % 160 == 0 ? 160 : p.N % 128 == 0 ? 128 : 64;
  c.bn = bn0;
  c.splitk = 1;
  if (!k64) {
    c.variant = 0;
    if (p.stats_out && (p.N + c.bn - 1) / c.bn > LN_MAX_PARTS) c.bn = 160;
    return c;
  }
  if (!p.force_bn) {
    bool rows_ok = true;
#ifdef SDSTREAM_DEVHOOKS
    static const bool no_rows = getenv("SDSTREAM_NO_ROWS") != nullptr;   // (read here: the engine asks for plans too)
    static const bool no_rows_short = getenv("SDSTREAM_NO_ROWS_SHORT") != nullptr;
    rows_ok = !no_rows;
#endif
    int shape = rows_ok ? rows_kernel_shape(p) : 0;
#ifdef SDSTREAM_DEVHOOKS
    if (shape == 2 && no_rows_short) shape = 0;
#endif
    if (shape) {
      c.variant = 3;
      c.bn = shape == 2 ? p.N : bn0;
      return c;
    }
  }
  const int stages = p.K / 64;
  const bool may_split = p.epilogue == EPI_NONE && p.workspace != nullptr && !p.no_splitk;
  const long long mn = (long long)p.M * p.N;
  auto blocks = [&](int bm, int bn) { return ((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn); };
  // K splits for a grid of nb tiles: up to one block per compute unit, two where a block would walk > 100 stages
  auto split_for = [&](int nb) {
    int k = nb >= 200 ? 1 : (256 + nb / 2) / nb;
    if (stages / k > 100) k *= 2;
    const int most = stages / 8 > 1 ? stages / 8 : 1;
    return k < most ? k : most;
  };
  // 128-row tiles: of the widths that divide N, the one that fills whole rounds of one block per compute unit best
  int bn6 = bn0;
  if (!geglu && p.N % 160 == 0 && p.N % 128 == 0) {
    auto fill = [&](int bn) { const int nb = blocks(128, bn); return (double)nb / (double)(((nb + 255) / 256) * 256); };
    if (fill(128) > fill(160) + 1e-3) bn6 = 128;
  }
  int sk = 1;
  const int nb6 = blocks(128, bn6);
  // below 48 stages, where 64-row tiles alone fill the chip, they beat a two-way K split of 128-row tiles and its
  // finalize pass (26 against 30 us on the 4096 x 640 x 2560 layers)
  const bool no_split_64 = stages < 48 && blocks(64, bn0) >= 200;
  if (nb6 >= 200 && stages >= 5) {
    c.variant = 1;
    c.bn = bn6;
    sk = split_for(nb6);
  } else if (stages >= 32 && !no_split_64) {
    // long K, few tiles: split K; full tiles as long as enough blocks remain
    const int s1 = split_for(blocks(128, bn0));
    bool tall = may_split && blocks(128, bn0) * s1 >= 150;
    // ... unless they leave a fifth of the units idle where 64-row tiles with their split fill them (the 1024-row
    // layers of a one-row step: 160 against 256 blocks, 19.5 -> 16.7 us with the finalize pass)
    if (tall && blocks(128, bn0) * s1 < 200 && blocks(64, bn0) * split_for(blocks(64, bn0)) >= 240) tall = false;
    if (tall) {
      c.variant = 1;
      sk = s1;
    } else {
      c.variant = 2;
      sk = split_for(blocks(64, bn0));
    }
  } else {
    // short K, few tiles (most 1x1 layers of the deeper levels): narrower 64-row tiles rather than a split
    c.variant = 2;
    if (blocks(64, c.bn) < 256) {
      if (!geglu && p.N % 128 == 0 && blocks(64, 128) >= 200) c.bn = 128;
      else if (p.N % 64 == 0) c.bn = 64;
    }
    const int nb = blocks(64, c.bn);
    if (nb < 64 && stages >= 16) sk = split_for(nb);
  }
  // a layer that leaves row statistics writes one part per column tile, and the reader takes at most LN_MAX_PARTS
  if (p.stats_out && (p.N + c.bn - 1) / c.bn > LN_MAX_PARTS) c.bn = 160;
  if (softmax) c.bn = 160;
  if (p.force_bn) {   // a launch on a sub-range of rows keeps the tile shape chosen for the whole range
    c.variant = p.force_variant;
    c.bn = p.force_bn;
    sk = 1;
  }
  if (!may_split) sk = 1;
  if ((long long)sk * mn > p.workspace_floats) sk = (int)(p.workspace_floats / mn);
  c.splitk = sk > 1 ? sk : 1;
#ifdef SDSTREAM_DEVHOOKS
  static const char* const tune = getenv("SDSTREAM_TUNE");
  if (const char* t = tune) {  // "variant,bn,splitk" for sweeps; unsupported combinations are ignored
    int v = -1, bn = 0, sk = 0;
    if (sscanf(t, "%d,%d,%d", &v, &bn, &sk) == 3) {
      if (v >= 0 && v <= 2 && (k64 || v == 0)) c.variant = v;
      if ((bn == 160 || bn == 128 || bn == 64) && !(p.epilogue == EPI_GEGLU && bn == 160)) c.bn = bn;
      if (sk >= 1 && may_split && (long long)sk * p.M * p.N <= p.workspace_floats &&
          sk <= (c.variant == 0 ? p.K / 32 : p.K / 64))
        c.splitk = sk;
    }
  }
#endif
  return c;
}

template <int BM, int BN> int dma_blocks(const IgemmParams& p) {
  return ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN) * (p.splitk > 1 ? p.splitk : 1);
}

// Pipeline shape per launch.  With more than one block per compute unit: two LDS buffers and two barriers per stage
// (two co-resident blocks overlap each other's waits).  With at most one block per unit, or when two blocks of three
// buffers still fit a unit's LDS (registers allow two): three buffers and one barrier per stage.  With at most one
// block per unit and a long K range per block: eight waves in two groups that split the block's stages (in-block
// split-K), which gives the unit two waves per SIMD; below ~24 stages the exchange of the accumulators at the end
// costs more than that brings (per-layer timings inside the step: -2 to -9 us on the 3x3 layers of 40-75 us,
// +1 us on the 13-19 us layers).  Launches of two blocks per unit stay as they are: two independent blocks beat
// one grouped block after the other (48 -> 58 us); launches of 16-160 blocks on the deep levels and the 64-row
// launches of one block per unit gain nothing from groups either (+-0.5 us: their 12-19 us are launch, prologue
// and epilogue latency, not the loop).
constexpr int kGroupSplitMinStages = 24;
template <int BM, int BN> void launch_ring(const IgemmParams& p, hipStream_t s) {
  constexpr int LDS3 = 3 * (BM + BN) * 128 + BM * 16;
  const bool one_per_unit = dma_blocks<BM, BN>(p) <= 256;
  bool three = 2 * LDS3 <= 160 * 1024 || one_per_unit;
  int group_min = kGroupSplitMinStages;
#ifdef SDSTREAM_DEVHOOKS
  if (p.dev_exp & 16) three = false;
  if (p.dev_exp & 32) three = true;
  static const char* const kg = getenv("SDSTREAM_KGMIN");
  if (kg) group_min = atoi(kg);
#endif
  if constexpr (BM == 128) {
    const int splitk = p.splitk > 1 ? p.splitk : 1;
    const int stages = (p.K / 64 + splitk - 1) / splitk;
    // (a launch that is to leave GroupNorm statistics was planned as a grouped one: only that kernel writes them)
    if ((one_per_unit && stages >= group_min) || p.gn_stats) { launch_dma<BM, BN, 2, false, 2>(p, s); return; }
  }
  if (three) launch_dma<BM, BN, 3, true>(p, s);
  else launch_dma<BM, BN, 2, false>(p, s);
}

template <int BN> void launch_bn(const IgemmParams& p, int variant, hipStream_t s) {
  switch (variant) {
    case 1: launch_ring<128, BN>(p, s); break;
    case 2: launch_ring<64, BN>(p, s); break;
    default: launch_cfg<128, BN, 3>(p, s); break;
  }
}

}  // namespace

bool igemm_mfma_available() { return true; }

IgemmPlan igemm_mfma_plan(const IgemmParams& p) {
  const Choice c = choose(p);
  IgemmPlan r;
  r.variant = c.variant;
  r.bm = c.variant == 2 || (c.variant == 3 && p.N == 320 && p.epilogue == EPI_NONE) ? 64 : 128;
  r.bn = c.bn;
  r.splitk = c.splitk;
  if (r.splitk > 1) {  // drop splits that the rounding of stages per split leaves empty
    const int stages = c.variant == 0 ? p.K / 32 : p.K / 64;
    const int sps = (stages + r.splitk - 1) / r.splitk;
    r.splitk = (stages + sps - 1) / sps;
  }
  r.grouped = false;
  if (r.variant == 1) {   // (the rule of launch_ring)
    const int blocks = ((p.M + 127) / 128) * ((p.N + r.bn - 1) / r.bn) * r.splitk;
    const int stages = (p.K / 64 + r.splitk - 1) / r.splitk;
    r.grouped = blocks <= 256 && stages >= kGroupSplitMinStages;
  }
  return r;
}

bool igemm_mfma_supported(const IgemmParams& p) {
  if (p.C1 % 32 || p.C2 % 32 || p.N % 16) return false;
  if (p.C3 > 0 && (p.C1 % 64 || p.C2 % 64 || p.C3 % 64 || p.C4 % 64 || p.upsample || p.stride != 1)) return false;
  if (p.epilogue == EPI_GEGLU && p.N % 128) return false;
  if (p.epilogue == EPI_SILU) return false;
  // the kernel addresses activations and weights with 32-bit byte offsets
  const long long samples = (p.M + (long long)p.Hout * p.Wout - 1) / ((long long)p.Hout * p.Wout);
  const long long cmax = p.C1 > p.C2 ? p.C1 : p.C2;
  if (samples * p.Hin * p.Win * cmax * 2 >= (1LL << 32)) return false;
  if ((long long)p.N * p.K * 2 >= (1LL << 32)) return false;
  if ((long long)p.M * p.N >= (1LL << 31)) return false;   // output element indices are divided as 31-bit values
  return true;
}

void launch_igemm_mfma(const IgemmParams& p0, hipStream_t s) {
  IgemmParams p = p0;
#ifdef SDSTREAM_DEVHOOKS
  static const int dev_exp = getenv("SDSTREAM_EXP") ? atoi(getenv("SDSTREAM_EXP")) : 0;
  p.dev_exp = dev_exp;
#endif
  const IgemmPlan c = igemm_mfma_plan(p);
  p.splitk = c.splitk;
  p.xcd_chunked = (long long)p.N * p.K > (long long)p.M * (p.C1 + p.C2) ? 1 : 0;
  p.fd_hw = make_fastdiv((unsigned)(p.Hout * p.Wout));
  p.fd_w = make_fastdiv((unsigned)p.Wout);
  p.fd_ct = make_fastdiv((unsigned)(p.C1 + p.C2));
  p.fd_ks = make_fastdiv((unsigned)p.ksize);
  p.fd_n = make_fastdiv((unsigned)p.N);
  if (c.variant == 3) launch_rows(p, s);
  else if (c.bn == 160) launch_bn<160>(p, c.variant, s);
  else if (c.bn == 128) launch_bn<128>(p, c.variant, s);
  else launch_bn<64>(p, c.variant, s);
}
