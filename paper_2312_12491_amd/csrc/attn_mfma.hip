// bf16 flash attention on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16), online softmax in fp32.
//
// One 256-thread block = 128 queries of one (sample, head); each wave owns 2 tiles of 16 queries.  K/V tiles
// of 64 keys are staged in LDS (K as [key][d], V transposed as [d][key]) and shared by the four waves.
// Scores are computed transposed, S^T = K Q^T, so a lane holds 16 keys of ONE query per tile: the running
// max / sum / rescale factor are per-lane scalars and the probabilities feed the second MFMA (O^T = V^T P^T)
// straight from registers.  The contraction order of that MFMA is a fixed permutation of the keys, applied
// identically to P (register order) and to the V^T fragment read.
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int QT = 2;     // query tiles (of 16) per wave
constexpr int BQ = 4 * QT * 16;
constexpr int BKV = 64;

template <int DK, int DT>  // DK = ceil(d/32) contraction steps of Q K^T; DT = ceil(d/16) output tiles of P V
__global__ __launch_bounds__(256) void attn_mfma_kernel(AttnParams p) {
  constexpr int KPITCH = DK * 64 + 16;   // bytes per key row of the K tile
  constexpr int VPITCH = BKV * 2 + 16;   // bytes per d row of the V^T tile
  constexpr int DPAD = DT * 16;
  __shared__ __attribute__((aligned(16))) unsigned char Ks[BKV * KPITCH];
  __shared__ __attribute__((aligned(16))) unsigned char Vs[DPAD * VPITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, li = lane & 15;
  const int head = blockIdx.y, sample = blockIdx.z;
  const int d = p.d, c0 = head * d;
  const int dchunks = d >> 3;  // 16-byte chunks per row
  const bf16_t* Q = (const bf16_t*)p.q;
  const bf16_t* K = (const bf16_t*)p.k;
  const bf16_t* V = (const bf16_t*)p.v;
  const long long kvoff = p.kv_select ? (long long)p.kv_select[sample] * p.kv_select_stride
                                      : (long long)sample * p.kv_sample_stride;
  const int q0 = blockIdx.x * BQ + wave * (QT * 16);

  // zero both tiles once: padding columns / rows are never written again
  for (int i = tid; i < (BKV * KPITCH) / 16; i += 256) ((uint4*)Ks)[i] = make_uint4(0, 0, 0, 0);
  for (int i = tid; i < (DPAD * VPITCH) / 16; i += 256) ((uint4*)Vs)[i] = make_uint4(0, 0, 0, 0);

  // Q fragments (B operand: column = query li, 8 consecutive d)
  bf16x8 qf[QT][DK];
#pragma unroll
  for (int t = 0; t < QT; ++t)
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      int q = q0 + t * 16 + li, dd = ks * 32 + g * 8;
      bf16x8 v = bf16x8{};
      if (q < p.Sq && dd < d) v = *(const bf16x8*)(Q + ((long long)sample * p.Sq + q) * p.ldq + c0 + dd);
      qf[t][ks] = v;
    }

  f32x4 o[QT][DT];
  float mrun[QT], lrun[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    mrun[t] = -1e30f;
    lrun[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float sc = p.scale * 1.44269504088896341f;  // scores are exponentiated in base 2

  // loader slots: K chunk (row, c) ; V chunk (key = tid%64, c = tid/64 + 4*i)
  constexpr int KSLOTS = (BKV * DK * 4 + 255) / 256;  // upper bound on 16-byte chunks per thread
  constexpr int VSLOTS = (DT * 2 + 3) / 4;
  uint4 kreg[KSLOTS], vreg[VSLOTS];
  const int nkchunks = BKV * dchunks;

  auto load_tiles = [&](int j0) {
#pragma unroll
    for (int i = 0; i < KSLOTS; ++i) {
      int ch = tid + i * 256;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ch < nkchunks) {
        int r = ch / dchunks, c = ch - r * dchunks;
        if (j0 + r < p.Skv) v = *(const uint4*)(K + kvoff + (long long)(j0 + r) * p.ldk + c0 + c * 8);
      }
      kreg[i] = v;
    }
#pragma unroll
    for (int i = 0; i < VSLOTS; ++i) {
      int c = (tid >> 6) + 4 * i, r = tid & 63;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (c < dchunks && j0 + r < p.Skv) v = *(const uint4*)(V + kvoff + (long long)(j0 + r) * p.ldv + c0 + c * 8);
      vreg[i] = v;
    }
  };
  auto store_tiles = [&]() {
#pragma unroll
    for (int i = 0; i < KSLOTS; ++i) {
      int ch = tid + i * 256;
      if (ch < nkchunks) {
        int r = ch / dchunks, c = ch - r * dchunks;
        *(uint4*)(Ks + r * KPITCH + c * 16) = kreg[i];
      }
    }
#pragma unroll
    for (int i = 0; i < VSLOTS; ++i) {
      int c = (tid >> 6) + 4 * i, r = tid & 63;
      if (c < dchunks) {
        const unsigned short* h = (const unsigned short*)&vreg[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) *(unsigned short*)(Vs + (c * 8 + e) * VPITCH + r * 2) = h[e];
      }
    }
  };

  load_tiles(0);
  for (int j0 = 0; j0 < p.Skv; j0 += BKV) {
    __syncthreads();  // previous tile fully consumed (also orders the initial zero fill)
    store_tiles();
    __syncthreads();
    if (j0 + BKV < p.Skv) load_tiles(j0 + BKV);

#pragma unroll
    for (int t = 0; t < QT; ++t) {
      // S^T tiles: rows = keys 16*kt + 4g + v, column = query li
      f32x4 s[4];
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) {
        s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < DK; ++ks) {
          bf16x8 kf = *(const bf16x8*)(Ks + (kt * 16 + li) * KPITCH + (ks * 32 + g * 8) * 2);
          s[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[t][ks], s[kt], 0, 0, 0);
        }
      }
      float mx = -1e30f;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float x = (j0 + kt * 16 + g * 4 + v < p.Skv) ? s[kt][v] * sc : -1e30f;
          s[kt][v] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun[t], mx);
      const float alpha = __builtin_amdgcn_exp2f(mrun[t] - mnew);
      mrun[t] = mnew;
      float sum = 0.f;
      bf16x8 pf[2];
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float e = __builtin_amdgcn_exp2f(s[kt][v] - mnew);
          sum += e;
          pf[kt >> 1][(kt & 1) * 4 + v] = (bf16_t)e;
        }
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      lrun[t] = lrun[t] * alpha + sum;
      // O^T += V^T P^T : rows = d (16*dt + 4g + v), column = query li
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        f32x4 acc = o[t][dt] * alpha;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const unsigned char* row = Vs + (dt * 16 + li) * VPITCH + (kk * 32 + g * 4) * 2;
          bf16x4 lo = *(const bf16x4*)row;
          bf16x4 hi = *(const bf16x4*)(row + 32);
          bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[kk], acc, 0, 0, 0);
        }
        o[t][dt] = acc;
      }
    }
  }

  bf16_t* O = (bf16_t*)p.out;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int q = q0 + t * 16 + li;
    if (q >= p.Sq) continue;
    const float inv = 1.0f / lrun[t];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int dd = dt * 16 + g * 4;
      if (dd >= d) continue;
      bf16x4 w;
#pragma unroll
      for (int v = 0; v < 4; ++v) w[v] = (bf16_t)(o[t][dt][v] * inv);
      *(bf16x4*)(O + ((long long)sample * p.Sq + q) * p.ldo + c0 + dd) = w;
    }
  }
}

template <int DK, int DT> void launch_cfg(const AttnParams& p, hipStream_t s) {
  dim3 grid((p.Sq + BQ - 1) / BQ, p.heads, p.samples);
  hipLaunchKernelGGL((attn_mfma_kernel<DK, DT>), grid, dim3(256), 0, s, p);
}

}  // namespace

bool attention_mfma_supported(const AttnParams& p) {
  if (p.d % 8 || p.ldq % 8 || p.ldk % 8 || p.ldv % 8 || p.ldo % 4) return false;
  switch (p.d) {
    case 8: case 16: case 32: case 40: case 64: case 80: case 160: return true;
    default: return false;
  }
}

void launch_attention_mfma(const AttnParams& p, hipStream_t s) {
  switch (p.d) {
    case 8: case 16: launch_cfg<1, 1>(p, s); break;
    case 32: launch_cfg<1, 2>(p, s); break;
    case 40: launch_cfg<2, 3>(p, s); break;
    case 64: launch_cfg<2, 4>(p, s); break;
    case 80: launch_cfg<3, 5>(p, s); break;
    case 160: launch_cfg<5, 10>(p, s); break;
    default: break;
  }
}
