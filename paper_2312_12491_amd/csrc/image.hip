// First and last convolution of the latent <-> image stage (the tiny autoencoder around the U-Net): the two
// kernels that touch the u8 image.  Everything between them is 3x3 convolutions of one width on NHWC activations
// and runs on the implicit-GEMM kernels.
#include "common.h"

namespace {

// u8 image [N][H][W][3] -> T NHWC [N*H*W][C0]: x / 255, 3x3, pad 1, + bias.  A block owns 64 pixels; their
// 27-value patches and the transposed weights sit in LDS.  A lane owns an output channel with its 27 weights in
// registers and a wave walks 16 of the pixels: patch values are LDS broadcasts, stores are whole pixel rows.
constexpr int II_PIX = 64;
template <typename T>
__global__ __launch_bounds__(256) void image_in_kernel(const uint8_t* __restrict__ img, const float* __restrict__ w,
                                                       const float* __restrict__ b, T* __restrict__ out, int N, int H,
                                                       int W, int C0) {
  extern __shared__ float sm[];
  float* wt = sm;              // [27][C0]
  float* patch = sm + 27 * C0; // [II_PIX][28]
  const long long total_pix = (long long)N * H * W;
  const long long pix0 = (long long)blockIdx.x * II_PIX;
  for (int i = threadIdx.x; i < 27 * C0; i += 256) {
    const int co = i / 27, k = i - co * 27;   // OIHW = [co][ci][ky][kx]
    wt[k * C0 + co] = w[i];
  }
  for (int i = threadIdx.x; i < II_PIX * 27; i += 256) {
    const int p = i / 27, k = i - p * 27;
    const long long pix = pix0 + p;
    float v = 0.f;
    if (pix < total_pix) {
      const int xx = (int)(pix % W), yy = (int)((pix / W) % H), n = (int)(pix / ((long long)W * H));
      const int ci = k / 9, t = k - ci * 9;
      const int iy = yy + t / 3 - 1, ix = xx + t % 3 - 1;
      if (iy >= 0 && iy < H && ix >= 0 && ix < W)
        v = (float)img[(((long long)n * H + iy) * W + ix) * 3 + ci] * (1.0f / 255.0f);
    }
    patch[p * 28 + k] = v;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int co = lane; co < C0; co += 64) {
    float wr[27];
#pragma unroll
    for (int k = 0; k < 27; ++k) wr[k] = wt[k * C0 + co];
    const float bias = b[co];
    for (int p = wave; p < II_PIX; p += 4) {
      if (pix0 + p >= total_pix) break;
      float acc = bias;
#pragma unroll
      for (int k = 0; k < 27; ++k) acc = fmaf(wr[k], patch[p * 28 + k], acc);
      out[(pix0 + p) * C0 + co] = from_f32<T>(acc);
    }
  }
}

typedef __attribute__((ext_vector_type(8))) __bf16 img_bf16x8;
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8], bool aligned) {
  if (aligned) {
    const img_bf16x8 x = *(const img_bf16x8*)p;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)x[e];
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)p[e];
  }
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8], bool aligned) {
  if (aligned) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = p[e];
  }
}

// T NHWC [N*H*W][C0] -> 3 channels: 3x3, pad 1, + bias, clamp to [0,1]; written as float NCHW [N][3][H][W] and / or
// as u8 HWC [N][H][W][3] (round(255 v), half to even).  A thread owns a pixel; the 3 x 9 x C0 weights sit in LDS as
// float4 per (tap, input channel).  (C0 / 8 lanes per pixel, one 16-byte chunk of each tap per lane and a shuffle sum,
// makes the global loads contiguous but was three times slower at 512 x 512: 254 us against 82 us.)
template <typename T>
__global__ __launch_bounds__(256) void image_out_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                        const float* __restrict__ b, float* __restrict__ out_f32,
                                                        uint8_t* __restrict__ out_u8, int N, int H, int W, int C0) {
  extern __shared__ float4 wl[];   // [9][C0]: the three output channels' weights of one (tap, input channel), padded to 16 bytes
  for (int i = threadIdx.x; i < 9 * C0; i += 256) {   // w is [co][tap][c]
    wl[i] = make_float4(to_f32<T>(w[i]), to_f32<T>(w[9 * C0 + i]), to_f32<T>(w[18 * C0 + i]), 0.f);
  }
  __syncthreads();
  const long long total_pix = (long long)N * H * W;
  const long long pix = (long long)blockIdx.x * 256 + threadIdx.x;
  if (pix >= total_pix) return;
  const int xx = (int)(pix % W), yy = (int)((pix / W) % H), n = (int)(pix / ((long long)W * H));
  float acc[3] = {b[0], b[1], b[2]};
  for (int tap = 0; tap < 9; ++tap) {
    const int iy = yy + tap / 3 - 1, ix = xx + tap % 3 - 1;
    if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
    const T* src = x + (((long long)n * H + iy) * W + ix) * C0;
    const float4* wt = wl + tap * C0;
    int c = 0;
    for (; c + 8 <= C0; c += 8) {   // 16- or 32-byte loads (rows start 16-byte aligned when C0 is a multiple of 8)
      float v[8];
      load8(src + c, v, (C0 & 7) == 0);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float4 ww = wt[c + e];   // the same address in every lane: one broadcast read for three products
        acc[0] = fmaf(v[e], ww.x, acc[0]);
        acc[1] = fmaf(v[e], ww.y, acc[1]);
        acc[2] = fmaf(v[e], ww.z, acc[2]);
      }
    }
    for (; c < C0; ++c) {
      const float v = to_f32<T>(src[c]);
      const float4 ww = wt[c];
      acc[0] = fmaf(v, ww.x, acc[0]);
      acc[1] = fmaf(v, ww.y, acc[1]);
      acc[2] = fmaf(v, ww.z, acc[2]);
    }
  }
#pragma unroll
  for (int co = 0; co < 3; ++co) {
    const float v = fminf(fmaxf(acc[co], 0.f), 1.f);
    if (out_f32) out_f32[(((long long)n * 3 + co) * H + yy) * W + xx] = v;
    if (out_u8) out_u8[pix * 3 + co] = (uint8_t)__float2int_rn(v * 255.0f);
  }
}

}  // namespace

template <typename T>
void launch_image_in(const uint8_t* img, const float* w, const float* b, void* out, int N, int H, int W, int C0,
                     hipStream_t s) {
  const long long pix = (long long)N * H * W;
  const size_t lds = (size_t)(27 * C0 + II_PIX * 28) * sizeof(float);
  hipLaunchKernelGGL(image_in_kernel<T>, dim3((unsigned)((pix + II_PIX - 1) / II_PIX)), dim3(256), lds, s, img, w, b,
                     (T*)out, N, H, W, C0);
}
template void launch_image_in<float>(const uint8_t*, const float*, const float*, void*, int, int, int, int, hipStream_t);
template void launch_image_in<bf16_t>(const uint8_t*, const float*, const float*, void*, int, int, int, int, hipStream_t);

template <typename T>
void launch_image_out(const void* x, const void* w, const float* b, float* out_f32, uint8_t* out_u8, int N, int H, int W,
                      int C0, hipStream_t s) {
  const long long pix = (long long)N * H * W;
  hipLaunchKernelGGL(image_out_kernel<T>, dim3((unsigned)((pix + 255) / 256)), dim3(256), (size_t)9 * C0 * sizeof(float4),
                     s, (const T*)x, (const T*)w, b, out_f32, out_u8, N, H, W, C0);
}
template void launch_image_out<float>(const void*, const void*, const float*, float*, uint8_t*, int, int, int, int, hipStream_t);
template void launch_image_out<bf16_t>(const void*, const void*, const float*, float*, uint8_t*, int, int, int, int, hipStream_t);
