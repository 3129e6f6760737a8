// bf16 flash attention on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16), online softmax in fp32.
//
// One 256-thread block = 64*QT queries of one (sample, head); each wave owns QT tiles of 16 queries.  K/V tiles
// of 64 keys are staged in double-buffered LDS (K as [key][d], V transposed as [d][key]) and shared by the waves;
// every K / V fragment read from LDS is used for all QT query tiles of the wave.
// Scores are computed transposed, S^T = K Q^T, so a lane holds 16 keys of ONE query per tile: the running
// max / sum / rescale factor are per-lane scalars and the probabilities feed the second MFMA (O^T = V^T P^T)
// straight from registers.  The contraction order of that MFMA is a fixed permutation of the keys, applied
// identically to P (register order) and to V^T (the order in which the keys of a tile are stored in LDS).
#include "common.h"

#include <stdlib.h>

#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BKV = 64;

// Reductions over the four lanes {li, li+16, li+32, li+48} that share a query, on the vector ALU:
// v_permlane16_swap / v_permlane32_swap with both operands equal leave (x[l], x[l^16]) resp. (x[l], x[l^32]) in a lane.
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

// DK = ceil(d/32) contraction steps of Q K^T; DT = ceil(d/16) output tiles of P V; QT = query tiles (of 16) per wave.
// ONES (head sizes with d % 16 == 8, i.e. padding rows in the last output tile): row d of the V^T tile is set to
// one, so row d of O^T accumulates the softmax denominator in the matrix core - from the same bf16-rounded
// probabilities as the numerator, rescaled with it - and the per-tile sum on the vector ALU, which bounds this
// kernel at small d, goes away.
template <int DK, int DT, int QT, bool ONES, int PIPE>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(AttnParams p) {
  constexpr int BQ = 4 * QT * 16;
  constexpr int KPITCH = DK * 64 + 16;   // bytes per key row of the K tile
  constexpr int VPITCH = BKV * 2 + 16;   // bytes per d row of the V^T tile
  constexpr int DPAD = DT * 16;
  constexpr int KBYTES = BKV * KPITCH, VBYTES = DPAD * VPITCH, TILE = KBYTES + VBYTES;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // two [K | V^T] tiles

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, li = lane & 15;
  const int head = blockIdx.y, sample = blockIdx.z;
  const int d = p.d, c0 = head * d;
  const int dchunks = d >> 3;  // 16-byte chunks per row
  const bf16_t* Q = (const bf16_t*)p.q;
  const bf16_t* K = (const bf16_t*)p.k;
  const bf16_t* V = (const bf16_t*)p.v;
  long long kvoff = p.kv_select ? (long long)p.kv_select[sample] * p.kv_select_stride
                                : (long long)sample * p.kv_sample_stride;
  int Skv = p.Skv;
  if (p.kv_group > 1 && sample < p.kv_group_rows) {  // keys / values of the whole stream batch, in batch order
    kvoff = (long long)(sample - sample % p.kv_group) * p.kv_sample_stride;
    Skv = p.Skv * p.kv_group;
  }
  const int q0 = blockIdx.x * BQ + wave * (QT * 16);

  // zero both buffers once: padding columns / rows are never written again
  for (int i = tid; i < (2 * TILE) / 16; i += 256) ((uint4*)smem)[i] = make_uint4(0, 0, 0, 0);

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
  // Everything about a slot that does not depend on the key tile is worked out once: the loaders run per tile and
  // were, with their index arithmetic, longer than the tile's MFMA and softmax work at one query tile per wave.
  const bf16_t* kptr[KSLOTS];   // row r, chunk c of key tile 0
  int krow[KSLOTS], klds[KSLOTS];   // row (BKV when the slot is unused: never below Skv - j0), LDS byte offset
#pragma unroll
  for (int i = 0; i < KSLOTS; ++i) {
    const int ch = tid + i * 256;
    const int r = ch / dchunks, c = ch - r * dchunks;
    const bool used = ch < nkchunks;
    krow[i] = used ? r : (1 << 30);
    klds[i] = r * KPITCH + c * 16;
    kptr[i] = K + kvoff + (long long)r * p.ldk + c0 + c * 8;
  }
  const int vkey = tid & 63;
  const bf16_t* vptr[VSLOTS];
  bool vuse[VSLOTS];
#pragma unroll
  for (int i = 0; i < VSLOTS; ++i) {
    const int c = (tid >> 6) + 4 * i;
    vuse[i] = c < dchunks;
    vptr[i] = V + kvoff + (long long)vkey * p.ldv + c0 + c * 8;
  }

  auto load_tiles = [&](int j0) {
    const long long koff = (long long)j0 * p.ldk, voff = (long long)j0 * p.ldv;
    const int left = Skv - j0;   // keys from j0 on
#pragma unroll
    for (int i = 0; i < KSLOTS; ++i) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (krow[i] < left) v = *(const uint4*)(kptr[i] + koff);
      kreg[i] = v;
    }
#pragma unroll
    for (int i = 0; i < VSLOTS; ++i) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (vuse[i] && vkey < left) v = *(const uint4*)(vptr[i] + voff);
      vreg[i] = v;
    }
  };
  // Key r of a tile sits at position vpos in a V^T row: the 8 keys a lane multiplies in one MFMA (4 consecutive
  // from each half of a 32-key step, the order the probabilities have in registers) are then one 16-byte read.
  const int vpos = (vkey & 32) + ((vkey & 12) << 1) + ((vkey & 16) >> 2) + (vkey & 3);
  auto store_tiles = [&](int b) {
    unsigned char* Ks = smem + b * TILE;
    unsigned char* Vs = Ks + KBYTES;
#pragma unroll
    for (int i = 0; i < KSLOTS; ++i)
      if (krow[i] < BKV) *(uint4*)(Ks + klds[i]) = kreg[i];
#pragma unroll
    for (int i = 0; i < VSLOTS; ++i) {
      const int c = (tid >> 6) + 4 * i;
      if (vuse[i]) {
        const unsigned short* h = (const unsigned short*)&vreg[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) *(unsigned short*)(Vs + (c * 8 + e) * VPITCH + vpos * 2) = h[e];
      }
    }
  };

  load_tiles(0);
  __syncthreads();  // zero fill done
  if (ONES && tid < 2 * BKV) {
    const int b = tid / BKV, key = tid - b * BKV;
    *(bf16_t*)(smem + b * TILE + KBYTES + d * VPITCH + key * 2) = (bf16_t)1.0f;
  }
  store_tiles(0);
  __syncthreads();
  // One key tile.  Only the last tile can be ragged; it gets its own copy of the body, because the compiler
  // otherwise computes the per-key masks (about 50 vector instructions) for every tile.
  auto key_tile = [&](auto ragged_tag, int j0, int buf) {
    constexpr bool RAGGED = decltype(ragged_tag)::value;
    const unsigned char* Ks = smem + buf * TILE;
    const unsigned char* Vs = Ks + KBYTES;
    const bool more = j0 + BKV < Skv;
    if (more) load_tiles(j0 + BKV);  // in flight while this tile is multiplied

    if constexpr (PIPE != 0) {
      // Software pipeline over the wave's query tiles: the softmax of tile t (vector ALU, what bounds this kernel at
      // small d) is issued interleaved with the matrix-core work that does not depend on it - the scores of tile
      // t + 1 and the P V product of tile t - 1 - instead of three phases one after the other.  The tile's K fragments
      // are read once into registers (every one serves all QT query tiles); scores and probabilities alternate
      // between two register sets.
      bf16x8 kfr[4][DK];
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int ks = 0; ks < DK; ++ks) kfr[kt][ks] = *(const bf16x8*)(Ks + (kt * 16 + li) * KPITCH + (ks * 32 + g * 8) * 2);
      constexpr bool VPRE = DT * QT <= 12;
      bf16x8 vfr[VPRE ? DT : 1][2];
      if constexpr (VPRE) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int kk = 0; kk < 2; ++kk)
            vfr[dt][kk] = *(const bf16x8*)(Vs + (dt * 16 + li) * VPITCH + (kk * 32 + g * 8) * 2);
      }
      f32x4 sacc[2][4];
      bf16x8 pf[2][2];
      auto scores = [&](int t, f32x4 (&sa)[4]) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
          sa[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < DK; ++ks)
            sa[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr[kt][ks], qf[t][ks], sa[kt], 0, 0, 0);
        }
      };
      auto weighted_values = [&](int t, const bf16x8 (&pp)[2]) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            bf16x8 vf;
            if constexpr (VPRE) vf = vfr[dt][kk];
            else vf = *(const bf16x8*)(Vs + (dt * 16 + li) * VPITCH + (kk * 32 + g * 8) * 2);
            o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pp[kk], o[t][dt], 0, 0, 0);
          }
      };
      scores(0, sacc[0]);
      __builtin_amdgcn_sched_barrier(0);   // what follows is scheduled without these: they have nothing to hide behind
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        if (t + 1 < QT) scores(t + 1, sacc[(t + 1) & 1]);
        if (t > 0) weighted_values(t - 1, pf[(t - 1) & 1]);
        f32x4(&sa)[4] = sacc[t & 1];
        if constexpr (RAGGED) {
#pragma unroll
          for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (j0 + kt * 16 + g * 4 + v >= Skv) sa[kt][v] = -3.0e38f;
        }
        float mx = sa[0][0];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int v = 0; v < 4; ++v) mx = fmaxf(mx, sa[kt][v]);
        mx = quad_max(mx);
        const float mnew = fmaxf(mrun[t], mx * sc);
        const float alpha = __builtin_amdgcn_exp2f(mrun[t] - mnew);
        mrun[t] = mnew;
        float sum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float e = __builtin_amdgcn_exp2f(fmaf(sa[kt][v], sc, -mnew));
            if (!ONES) sum += e;
            pf[t & 1][kt >> 1][(kt & 1) * 4 + v] = (bf16_t)e;
          }
        if (!ONES) {
          sum = quad_sum(sum);
          lrun[t] = lrun[t] * alpha + sum;
        }
        // one matrix instruction per four vector instructions, as long as both last
#pragma unroll
        for (int i = 0; i < 4 * DK + 2 * DT; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, PIPE, 0);
        }
        if (__any(alpha != 1.0f)) {   // wave-uniform: some query of this tile moved its running max
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[t][dt] *= alpha;
        }
      }
      weighted_values(QT - 1, pf[(QT - 1) & 1]);
    } else {
    // S^T tiles: rows = keys 16*kt + 4g + v, column = query li; every K fragment serves all QT query tiles
    f32x4 sacc[QT][4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
      for (int t = 0; t < QT; ++t) sacc[t][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        bf16x8 kf = *(const bf16x8*)(Ks + (kt * 16 + li) * KPITCH + (ks * 32 + g * 8) * 2);
#pragma unroll
        for (int t = 0; t < QT; ++t)
          sacc[t][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[t][ks], sacc[t][kt], 0, 0, 0);
      }
    }
    // V^T fragments of the whole tile, requested before the softmax arithmetic that hides their latency - where
    // the registers are there (DT * QT <= 12: not d = 64 with 4 query tiles, not d = 160 with 2)
    constexpr bool VPRE = DT * QT <= 12;
    bf16x8 vfr[VPRE ? DT : 1][2];
    if constexpr (VPRE) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
          vfr[dt][kk] = *(const bf16x8*)(Vs + (dt * 16 + li) * VPITCH + (kk * 32 + g * 8) * 2);
    }
    bf16x8 pf[QT][2];
    float alpha[QT];
    bool rescale = false;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      f32x4(&s)[4] = sacc[t];
      if constexpr (RAGGED) {  // keys past the end must not win the max or add to the sum
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (j0 + kt * 16 + g * 4 + v >= Skv) s[kt][v] = -3.0e38f;
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) mx = fmaxf(mx, s[kt][v]);
      mx = quad_max(mx);
      const float mnew = fmaxf(mrun[t], mx * sc);   // running max of the scaled scores (base-2 exponent units)
      alpha[t] = __builtin_amdgcn_exp2f(mrun[t] - mnew);
      mrun[t] = mnew;
      float sum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float e = __builtin_amdgcn_exp2f(fmaf(s[kt][v], sc, -mnew));
          if (!ONES) sum += e;
          pf[t][kt >> 1][(kt & 1) * 4 + v] = (bf16_t)e;
        }
      if (!ONES) {
        sum = quad_sum(sum);
        lrun[t] = lrun[t] * alpha[t] + sum;
      }
      rescale = rescale || __any(alpha[t] != 1.0f);
    }
    // O^T += V^T P^T : rows = d (16*dt + 4g + v), column = query li.  The old sums are rescaled only when some
    // query of the wave moved its running max (wave-uniform test); every V fragment serves all QT query tiles.
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      if (rescale) {
#pragma unroll
        for (int t = 0; t < QT; ++t) o[t][dt] *= alpha[t];
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x8 vf;
        if constexpr (VPRE) vf = vfr[dt][kk];
        else vf = *(const bf16x8*)(Vs + (dt * 16 + li) * VPITCH + (kk * 32 + g * 8) * 2);
#pragma unroll
        for (int t = 0; t < QT; ++t)
          o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t][kk], o[t][dt], 0, 0, 0);
      }
    }
    }
    // the other buffer was last read one iteration ago, before the barrier every wave has passed since
    if (more) store_tiles(buf ^ 1);
    __syncthreads();
  };
  int buf = 0, j0 = 0;
  for (; j0 + BKV <= Skv; j0 += BKV, buf ^= 1) key_tile(std::false_type{}, j0, buf);
  if (j0 < Skv) key_tile(std::true_type{}, j0, buf);

  bf16_t* O = (bf16_t*)p.out;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    // ONES: the denominator of query li is element 0 of the last output tile in the lanes with g == 2 (row d)
    const float l = ONES ? __shfl(o[t][DT - 1][0], 32 + li) : lrun[t];
    const int q = q0 + t * 16 + li;
    if (q >= p.Sq) continue;
    const float inv = 1.0f / l;
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

template <int DK, int DT, int QT, bool ONES, int PIPE> void launch_qt_p(const AttnParams& p, hipStream_t s) {
  constexpr int BQ = 4 * QT * 16;
  constexpr int LDS = 2 * (BKV * (DK * 64 + 16) + DT * 16 * (BKV * 2 + 16));
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)attn_mfma_kernel<DK, DT, QT, ONES, PIPE>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    attr_set = true;
  }
  dim3 grid((p.Sq + BQ - 1) / BQ, p.heads, p.samples);
  hipLaunchKernelGGL((attn_mfma_kernel<DK, DT, QT, ONES, PIPE>), grid, dim3(256), LDS, s, p);
}

// With two or more query tiles per wave the tile loop is software-pipelined (one matrix instruction per four vector
// instructions: -4.5 % on the 4096-token, d = 40 self-attentions; ratios of 3 to 8 give the same).  Not at d = 160,
// where the second set of score registers spills.  (Key tiles of 128 instead of 64 keys per barrier, multiplied as
// two halves, were measured too: 149.4 against 147.7 us - the hand-over between tiles is not what is left.)
template <int DK, int DT, int QT, bool ONES> void launch_qt(const AttnParams& p, hipStream_t s) {
  constexpr int PIPE = QT >= 2 && DT <= 5 ? 4 : 0;
#ifdef SDSTREAM_DEVHOOKS
  static const bool no_pipe = getenv("SDSTREAM_ATTN_NOPIPE") != nullptr;
  if (no_pipe) { launch_qt_p<DK, DT, QT, ONES, 0>(p, s); return; }
#endif
  launch_qt_p<DK, DT, QT, ONES, PIPE>(p, s);
}

// more query tiles per wave amortise the K / V fragment reads; fewer keep small problems spread over the chip
template <int DK, int DT, bool ONES> void launch_cfg(const AttnParams& p, hipStream_t s) {
#ifdef SDSTREAM_DEVHOOKS
  static const int force = getenv("SDSTREAM_ATTN_QT") ? atoi(getenv("SDSTREAM_ATTN_QT")) : 0;
#else
  constexpr int force = 0;
#endif
  auto blocks = [&](int qt) { return (long long)((p.Sq + 64 * qt - 1) / (64 * qt)) * p.heads * p.samples; };
  int qt = 1;
  if (blocks(2) >= 512) qt = 2;
  if constexpr (DT <= 4) { if (blocks(4) >= 512) qt = 4; }
  if (force) qt = force;
  if constexpr (DT <= 4) { if (qt == 4) { launch_qt<DK, DT, 4, ONES>(p, s); return; } }
  if (qt == 1) launch_qt<DK, DT, 1, ONES>(p, s); else launch_qt<DK, DT, 2, ONES>(p, s);
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
    case 8: case 16: launch_cfg<1, 1, false>(p, s); break;
    case 32: launch_cfg<1, 2, false>(p, s); break;
    case 40: launch_cfg<2, 3, true>(p, s); break;   // 40 = 2 * 16 + 8: row 40 of the last tile is free
    case 64: launch_cfg<2, 4, false>(p, s); break;
    case 80: launch_cfg<3, 5, false>(p, s); break;
    case 160: launch_cfg<5, 10, false>(p, s); break;
    default: break;
  }
}
