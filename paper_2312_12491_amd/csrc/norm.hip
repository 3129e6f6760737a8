// GroupNorm (+SiLU) over one or two concatenated NHWC sources, and LayerNorm over token rows.
// The float32 kernels accumulate their statistics in double; the bf16 kernels sum in float32 per thread and per
// block and fold the block partials in double, in a fixed order.  Normalisation is applied in float32.
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

// ---------------------------------------------------------------------------------------------------
// bf16 fast path.  A block owns PPB pixels of one sample and all channels; a thread owns one 16-byte
// chunk (8 channels) and walks the pixels with its row of lanes, so every global access is a full
// coalesced row.  Pass 1 writes per-(sample, pixel-split, group) partial sums in a fixed order
// (deterministic); pass 2 folds the partials in double, then normalises, scales and applies SiLU.
// ---------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

__device__ __forceinline__ bf16x8 gn_load8(const GroupNormParams& p, long long pix, int c) {
  const bf16_t* src = c < p.C1 ? (const bf16_t*)p.src1 + pix * p.C1 + c : (const bf16_t*)p.src2 + pix * p.C2 + (c - p.C1);
  return *(const bf16x8*)src;
}

// group of channel c0 + e for e = 0..7 with one division instead of eight (a run-time integer division is ~30
// instructions; the kernels around here are a few microseconds long)
struct GroupWalk {
  int g, r, cg;
  __device__ __forceinline__ GroupWalk(int c0, int cg_) : g(c0 / cg_), r(c0 - (c0 / cg_) * cg_), cg(cg_) {}
  __device__ __forceinline__ int next() {   // group of the current channel, then advance by one channel
    const int cur = g;
    if (++r == cg) { r = 0; ++g; }
    return cur;
  }
};

// Both passes are latency chains, not streams (their time barely changes between 1 and 4 samples), so they are
// built to be short: blocks of up to 512 threads (more for rows wider than 512 chunks) so that a thread touches a
// few pixels with all its loads in flight at once, and reductions in three parallel steps (pixel lanes -> channel totals -> 8 threads per group
// with shuffles) instead of one thread per group walking LDS.
__global__ __launch_bounds__(1024) void gn_partial_bf16_kernel(GroupNormParams p, int ppb, int nsplit, int chunks,
                                                               int lanes) {
  extern __shared__ float sm[];  // [lanes][C][2] per-lane sums, then [C][2] channel totals
  const int C = p.C1 + p.C2, cg = C / p.groups;
  const int n = blockIdx.x / nsplit, sp = blockIdx.x - n * nsplit;
  const int chunk = threadIdx.x % chunks, ln = threadIdx.x / chunks;
  const int px0 = sp * ppb, px1 = min(p.HW, px0 + ppb);
  float s[8], q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s[e] = 0.f; q[e] = 0.f; }
  // four pixels per trip so that four loads are in flight per thread
  for (int px = px0 + ln; px < px1; px += 4 * lanes) {
    bf16x8 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int pu = px + u * lanes;
      v[u] = gn_load8(p, (long long)n * p.HW + (pu < px1 ? pu : px), chunk * 8);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (px + u * lanes >= px1) break;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = (float)v[u][e];
        s[e] += x;
        q[e] = fmaf(x, x, q[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sm[(ln * C + chunk * 8 + e) * 2] = s[e];
    sm[(ln * C + chunk * 8 + e) * 2 + 1] = q[e];
  }
  __syncthreads();
  float* tot = sm + (size_t)lanes * C * 2;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    float ss = 0.f, qq = 0.f;
#pragma unroll 8
    for (int l = 0; l < lanes; ++l) {
      ss += sm[(l * C + c) * 2];
      qq += sm[(l * C + c) * 2 + 1];
    }
    tot[c * 2] = ss;
    tot[c * 2 + 1] = qq;
  }
  __syncthreads();
  // blockDim is a multiple of 8 (launcher), so the 8 threads of a group are always in one wave and one trip
  for (int idx = threadIdx.x; idx < p.groups * 8; idx += blockDim.x) {
    const int g = idx >> 3, part = idx & 7;
    float ss = 0.f, qq = 0.f;
    for (int c = g * cg + part; c < (g + 1) * cg; c += 8) {
      ss += tot[c * 2];
      qq += tot[c * 2 + 1];
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
      ss += __shfl_xor(ss, o);
      qq += __shfl_xor(qq, o);
    }
    if (part == 0) {
      float* dst = p.stats + (((long long)n * nsplit + sp) * p.groups + g) * 2;
      dst[0] = ss;
      dst[1] = qq;
    }
  }
}

// Pass 2: every block first folds the pixel-split partials of its sample into mean / rstd per group (in double,
// fixed order, so all blocks of a sample agree bit for bit), then normalises its pixels.  `nsplit_p` is the split
// count of pass 1 (at most 64: 8 threads per group take up to 8 partials each).
__global__ __launch_bounds__(1024) void gn_apply_bf16_kernel(GroupNormParams p, int ppb, int nsplit, int chunks,
                                                             int lanes, int nsplit_p) {
  extern __shared__ float sm[];  // [groups][2]: mean, rstd
  const int C = p.C1 + p.C2, cg = C / p.groups;
  const int n = blockIdx.x / nsplit, sp = blockIdx.x - n * nsplit;
  const int chunk = threadIdx.x % chunks, ln = threadIdx.x / chunks;
  for (int idx = threadIdx.x; idx < p.groups * 8; idx += blockDim.x) {
    const int g = idx >> 3, part = idx & 7;
    double ss = 0.0, qq = 0.0;
#pragma unroll 8
    for (int k = part; k < nsplit_p; k += 8) {
      const float* src = p.stats + (((long long)n * nsplit_p + k) * p.groups + g) * 2;
      ss += src[0];
      qq += src[1];
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
      ss += __shfl_xor(ss, o);
      qq += __shfl_xor(qq, o);
    }
    if (part == 0) {
      const double cnt = (double)p.HW * cg;
      const double mean = ss / cnt;
      double var = qq / cnt - mean * mean;
      if (var < 0) var = 0;
      sm[g * 2] = (float)mean;
      sm[g * 2 + 1] = (float)(1.0 / sqrt(var + (double)p.eps));
    }
  }
  __syncthreads();
  float sc[8], sh[8];
  GroupWalk walk(chunk * 8, cg);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int c = chunk * 8 + e, g = walk.next();
    const float rs = sm[g * 2 + 1] * p.gamma[c];
    sc[e] = rs;
    sh[e] = p.beta[c] - sm[g * 2] * rs;
  }
  const int px0 = sp * ppb, px1 = min(p.HW, px0 + ppb);
  bf16_t* out = (bf16_t*)p.out;
  for (int px = px0 + ln; px < px1; px += 4 * lanes) {
    bf16x8 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int pu = px + u * lanes;
      v[u] = gn_load8(p, (long long)n * p.HW + (pu < px1 ? pu : px), chunk * 8);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int pu = px + u * lanes;
      if (pu >= px1) break;
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float y = fmaf((float)v[u][e], sc[e], sh[e]);
        if (p.silu) y *= __builtin_amdgcn_rcpf(1.0f + __expf(-y));   // 1 ulp reciprocal instead of the ~10-instruction division
        o[e] = (bf16_t)y;
      }
      *(bf16x8*)(out + ((long long)n * p.HW + pu) * C + chunk * 8) = o;
    }
  }
}

// Single-kernel variant for planes small enough to sit in registers: a block owns ALL pixels of one sample for a
// set of `gs` consecutive groups (gs * cg channels, a whole number of 16-byte chunks), so statistics and
// normalisation need no second launch - the two-pass pair above costs two launch latencies, which is most of
// its time on the small feature maps (measured inside the step: 7.5 - 8.5 us against 9 - 10 us at 8x8 and 16x16,
// 11 - 15 us against 15 - 16 us at 32x32).  A thread keeps up to R chunks (pixels ln, ln + lanes, ...), all loaded up front.
template <int R>
__global__ __launch_bounds__(1024) void gn_fused_bf16_kernel(GroupNormParams p, int gs, int chunks, int lanes) {
  extern __shared__ float sm[];  // [lanes][setC][2] per-lane sums | [setC][2] channel totals | [gs][2] mean, rstd
  const int C = p.C1 + p.C2, cg = C / p.groups, setC = gs * cg, nsets = p.groups / gs;
  const int n = blockIdx.x / nsets, set = blockIdx.x - n * nsets;
  const int c0 = set * setC;
  const int chunk = threadIdx.x % chunks, ln = threadIdx.x / chunks;
  bf16x8 v[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int px = ln + r * lanes;
    v[r] = gn_load8(p, (long long)n * p.HW + (px < p.HW ? px : 0), c0 + chunk * 8);
  }
  // scale / shift are requested now: after the statistics they would add a memory round trip to the chain
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const f32x4 ga0 = *(const f32x4*)(p.gamma + c0 + chunk * 8), ga1 = *(const f32x4*)(p.gamma + c0 + chunk * 8 + 4);
  const f32x4 be0 = *(const f32x4*)(p.beta + c0 + chunk * 8), be1 = *(const f32x4*)(p.beta + c0 + chunk * 8 + 4);
  float s[8], q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s[e] = 0.f; q[e] = 0.f; }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    if (ln + r * lanes >= p.HW) break;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (float)v[r][e];
      s[e] += x;
      q[e] = fmaf(x, x, q[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sm[(ln * setC + chunk * 8 + e) * 2] = s[e];
    sm[(ln * setC + chunk * 8 + e) * 2 + 1] = q[e];
  }
  __syncthreads();
  // channel totals: 8 threads per (channel, sum | square sum); blockDim is a multiple of 8 (launcher)
  float* tot = sm + (size_t)lanes * setC * 2;
  for (int idx = threadIdx.x; idx < setC * 2 * 8; idx += blockDim.x) {
    const int item = idx >> 3, part = idx & 7;
    float a = 0.f;
    for (int l = part; l < lanes; l += 8) a += sm[l * setC * 2 + item];
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) a += __shfl_xor(a, o);
    if (part == 0) tot[item] = a;
  }
  __syncthreads();
  float* mr = tot + setC * 2;
  for (int idx = threadIdx.x; idx < gs * 8; idx += blockDim.x) {
    const int g = idx >> 3, part = idx & 7;
    double ss = 0.0, qq = 0.0;
    for (int c = g * cg + part; c < (g + 1) * cg; c += 8) {
      ss += tot[c * 2];
      qq += tot[c * 2 + 1];
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
      ss += __shfl_xor(ss, o);
      qq += __shfl_xor(qq, o);
    }
    if (part == 0) {
      const double cnt = (double)p.HW * cg;
      const double mean = ss / cnt;
      double var = qq / cnt - mean * mean;
      if (var < 0) var = 0;
      mr[g * 2] = (float)mean;
      mr[g * 2 + 1] = (float)(1.0 / sqrt(var + (double)p.eps));
    }
  }
  __syncthreads();
  float sc[8], sh[8];
  GroupWalk walk(chunk * 8, cg);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int cl = chunk * 8 + e, g = walk.next();
    const float rs = mr[g * 2 + 1] * (e < 4 ? ga0[e & 3] : ga1[e & 3]);
    sc[e] = rs;
    sh[e] = (e < 4 ? be0[e & 3] : be1[e & 3]) - mr[g * 2] * rs;
  }
  bf16_t* out = (bf16_t*)p.out;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int px = ln + r * lanes;
    if (px >= p.HW) break;
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float y = fmaf((float)v[r][e], sc[e], sh[e]);
      if (p.silu) y *= __builtin_amdgcn_rcpf(1.0f + __expf(-y));   // 1 ulp reciprocal instead of the ~10-instruction division
      o[e] = (bf16_t)y;
    }
    *(bf16x8*)(out + ((long long)n * p.HW + px) * C + c0 + chunk * 8) = o;
  }
}

struct GnFusedPlan { int gs, chunks, lanes, R; size_t lds; };
// false when the plane does not fit the single-kernel variant
bool gn_fused_plan(const GroupNormParams& p, GnFusedPlan& f) {
  const int C = p.C1 + p.C2;
  if (p.groups <= 0 || C % p.groups) return false;
  const int cg = C / p.groups;
  int gs = 1;
  while (gs <= 8 && ((gs * cg) % 8 != 0 || p.groups % gs != 0)) ++gs;
  if (gs > 8) return false;
  f.gs = gs;
  f.chunks = gs * cg / 8;
  if (f.chunks > 32) return false;
  const int max_lanes = (1024 / f.chunks) & ~7;
  // pixels in parallel: a quarter of the plane, at least 64 (measured inside the step at 16x16: 64 lanes 8.8 us,
  // 200 lanes 10.1 us - the per-lane sums go through LDS; at 8x8: 64 lanes 6.4 us, 16 lanes 8 us)
  int lanes = ((p.HW + 3) / 4 + 7) & ~7;
  if (lanes < 64) lanes = 64;
  if (lanes > ((p.HW + 7) & ~7)) lanes = (p.HW + 7) & ~7;
  if (lanes > max_lanes) lanes = max_lanes;
  if (lanes < 8) lanes = 8;
  f.lanes = lanes;
  const int r = (p.HW + lanes - 1) / lanes;
  // beyond 8 chunks per thread the pair of kernels is faster (measured inside the step: 16 -> 32 us against 22 us,
  // 24 -> 62 us against 27 us; too few blocks, too many registers)
  if (r > 8) return false;
  f.R = r <= 4 ? 4 : 8;
  f.lds = ((size_t)lanes + 1) * gs * cg * 2 * sizeof(float) + (size_t)gs * 2 * sizeof(float);
  return f.lds <= 96 * 1024;
}

template <int R> void launch_gn_fused_r(const GroupNormParams& p, const GnFusedPlan& f, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)gn_fused_bf16_kernel<R>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    attr_set = true;
  }
  hipLaunchKernelGGL(gn_fused_bf16_kernel<R>, dim3(p.samples * (p.groups / f.gs)), dim3(f.chunks * f.lanes), f.lds, s,
                     p, f.gs, f.chunks, f.lanes);
}

// thread geometry of the fast path: `chunks` 16-byte chunks per pixel row x `lanes` pixels, a multiple of 8 threads
int gn_lanes(int chunks) {
  int lanes = 512 / chunks;   // 512-thread blocks measured best inside the step (1024: +8 %, 256: +15 %)
  if (lanes < 1) lanes = 1;
  if (lanes > 32) lanes = 32;
  if (chunks % 8 != 0) lanes &= ~7;
  return lanes;
}

bool gn_fast_ok(const GroupNormParams& p) {
  const int C = p.C1 + p.C2;
  return p.C1 % 8 == 0 && p.C2 % 8 == 0 && C / 8 <= 1024 && gn_lanes(C / 8) >= 1 &&
         ((size_t)gn_lanes(C / 8) + 1) * C * 2 * sizeof(float) <= 160 * 1024;
}

// pass 2: four pixels per thread, one trip of the loop (measured inside the step: 1 / 2 / 3 / 4 / 8 pixels ->
// 293 / 211 / 191 / 196 / 198 us over the 30 launches of a step)
void launch_gn_apply(const GroupNormParams& p, int nsplit_p, hipStream_t s) {
  const int C = p.C1 + p.C2, chunks = C / 8;
  const int lanes = gn_lanes(chunks);
  const int threads = chunks * lanes;
  const int ppb = 4 * lanes;
  const int nsplit = (p.HW + ppb - 1) / ppb;
  hipLaunchKernelGGL(gn_apply_bf16_kernel, dim3(p.samples * nsplit), dim3(threads), (size_t)p.groups * 2 * sizeof(float),
                     s, p, ppb, nsplit, chunks, lanes, nsplit_p);
}

void launch_gn_fast(const GroupNormParams& p, hipStream_t s) {
  GnFusedPlan f;
  if (gn_fused_plan(p, f)) {
    if (f.R == 4) launch_gn_fused_r<4>(p, f, s); else launch_gn_fused_r<8>(p, f, s);
    return;
  }
  const int C = p.C1 + p.C2, chunks = C / 8;
  const int lanes = gn_lanes(chunks);
  const int threads = chunks * lanes;
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)gn_partial_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    attr_set = true;
  }
  // pass 1: at most 64 pixel splits per sample, at most 4 pixels per thread
  int ppb_p = (p.HW + 63) / 64;
  if (ppb_p < lanes) ppb_p = lanes;
  const int nsplit_p = (p.HW + ppb_p - 1) / ppb_p;
  hipLaunchKernelGGL(gn_partial_bf16_kernel, dim3(p.samples * nsplit_p), dim3(threads),
                     ((size_t)lanes + 1) * C * 2 * sizeof(float), s, p, ppb_p, nsplit_p, chunks, lanes);
  launch_gn_apply(p, nsplit_p, s);
}

}  // namespace

bool group_norm_takes_partials(const GroupNormParams& p) {
  GnFusedPlan f;
  return gn_fast_ok(p) && !gn_fused_plan(p, f);
}
void launch_group_norm_apply(const GroupNormParams& p, int splits, hipStream_t s) { launch_gn_apply(p, splits, s); }

template <typename T> void launch_group_norm_generic(const GroupNormParams& p, hipStream_t s);

template <typename T> void launch_group_norm(const GroupNormParams& p, hipStream_t s) { launch_group_norm_generic<T>(p, s); }
template <> void launch_group_norm<bf16_t>(const GroupNormParams& p, hipStream_t s) {
  if (gn_fast_ok(p)) launch_gn_fast(p, s); else launch_group_norm_generic<bf16_t>(p, s);
}
template void launch_group_norm<float>(const GroupNormParams&, hipStream_t);

template <typename T> void launch_group_norm_generic(const GroupNormParams& p, hipStream_t s) {
  hipLaunchKernelGGL(gn_stats_kernel<T>, dim3(p.samples * p.groups), dim3(256), 0, s, p);
  long long total = (long long)p.samples * p.HW * (p.C1 + p.C2);
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(gn_apply_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, p, total);
}
template void launch_group_norm_generic<float>(const GroupNormParams&, hipStream_t);
template void launch_group_norm_generic<bf16_t>(const GroupNormParams&, hipStream_t);

namespace {
// bf16 fast path: a wave owns a row and keeps it in registers (16-byte chunks, up to 3 per lane: C <= 1536)
__global__ __launch_bounds__(256) void layer_norm_bf16_kernel(LayerNormParams p) {
  typedef __attribute__((ext_vector_type(8))) __bf16 v8;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= p.rows) return;
  const int chunks = p.C >> 3;
  const bf16_t* x = (const bf16_t*)p.src + (long long)row * p.C;
  bf16_t* y = (bf16_t*)p.out + (long long)row * p.C;
  v8 v[3];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ch = lane + i * 64;
    if (ch < chunks) {
      v[i] = *(const v8*)(x + ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += (float)v[i][e];
    }
  }
  const float mean = wave_sum(sum) / (float)p.C;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ch = lane + i * 64;
    if (ch < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float d = (float)v[i][e] - mean;
        sq = fmaf(d, d, sq);
      }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)p.C + p.eps);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ch = lane + i * 64;
    if (ch < chunks) {
      v8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        o[e] = (bf16_t)(((float)v[i][e] - mean) * rstd * p.gamma[ch * 8 + e] + p.beta[ch * 8 + e]);
      *(v8*)(y + ch * 8) = o;
    }
  }
}
}  // namespace

template <> void launch_layer_norm<bf16_t>(const LayerNormParams& p, hipStream_t s);

template <typename T> void launch_layer_norm(const LayerNormParams& p, hipStream_t s) {
  hipLaunchKernelGGL(layer_norm_kernel<T>, dim3((p.rows + 3) / 4), dim3(256), 0, s, p);
}
template void launch_layer_norm<float>(const LayerNormParams&, hipStream_t);
template <> void launch_layer_norm<bf16_t>(const LayerNormParams& p, hipStream_t s) {
  if (p.C % 8 == 0 && p.C <= 1536)
    hipLaunchKernelGGL(layer_norm_bf16_kernel, dim3((p.rows + 3) / 4), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(layer_norm_kernel<bf16_t>, dim3((p.rows + 3) / 4), dim3(256), 0, s, p);
}
