// sdstream_ssf_static: the measurement and decision of the stochastic similarity filter (Eq. 8-9) for callers
// that cannot allocate - code under HIP graph capture, serving loops and harnesses that forbid hipMalloc.  No
// handle, no allocation, no host synchronisation: the per-block partial sums live in a file-scope device array.
#include "common.h"
#include "sdstream.h"

#include <stdio.h>

#include <mutex>
#include <string>

extern thread_local std::string g_sdstream_create_error;   // the message sdstream_last_error(NULL) returns

namespace {

constexpr int kMaxBlocks = 1024;
constexpr int kMaxDevices = 64;

// Scratch of sdstream_ssf_static: [kMaxBlocks][3] partial sums (dot, |frame|^2, |reference|^2).  Every GPU the
// library runs on holds its own copy until the process ends.  A call overwrites exactly the entries it reads
// back, so nothing in it has to start at zero.
static __device__ __align__(256) unsigned long long scratch[kMaxBlocks * 3];

std::mutex g_mu;
unsigned long long* g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, null until first use

__global__ __launch_bounds__(256) void ssf_partial_kernel(const uint8_t* __restrict__ f, const uint8_t* __restrict__ r,
                                                          long long n, unsigned long long* __restrict__ partial) {
  unsigned long long dot = 0, nt = 0, nr = 0;
  const long long nvec = n / 16;
  const uint4* f4 = (const uint4*)f;
  const uint4* r4 = (const uint4*)r;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < nvec;
       i += (long long)gridDim.x * blockDim.x) {
    const uint4 a = f4[i];
    const uint4 b = r ? r4[i] : make_uint4(0, 0, 0, 0);
    unsigned d = 0, q = 0, w = 0;  // 16 products of at most 255*255 fit in 32 bits
    d = __builtin_amdgcn_udot4(a.x, b.x, d, false);
    d = __builtin_amdgcn_udot4(a.y, b.y, d, false);
    d = __builtin_amdgcn_udot4(a.z, b.z, d, false);
    d = __builtin_amdgcn_udot4(a.w, b.w, d, false);
    q = __builtin_amdgcn_udot4(a.x, a.x, q, false);
    q = __builtin_amdgcn_udot4(a.y, a.y, q, false);
    q = __builtin_amdgcn_udot4(a.z, a.z, q, false);
    q = __builtin_amdgcn_udot4(a.w, a.w, q, false);
    w = __builtin_amdgcn_udot4(b.x, b.x, w, false);
    w = __builtin_amdgcn_udot4(b.y, b.y, w, false);
    w = __builtin_amdgcn_udot4(b.z, b.z, w, false);
    w = __builtin_amdgcn_udot4(b.w, b.w, w, false);
    dot += d;
    nt += q;
    nr += w;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {  // ragged tail, byte by byte
    for (long long i = nvec * 16; i < n; ++i) {
      const unsigned a = f[i], b = r ? r[i] : 0;
      dot += a * b;
      nt += a * a;
      nr += b * b;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    dot += __shfl_xor(dot, o);
    nt += __shfl_xor(nt, o);
    nr += __shfl_xor(nr, o);
  }
  __shared__ unsigned long long red[3][4];
  if ((threadIdx.x & 63) == 0) {
    red[0][threadIdx.x >> 6] = dot;
    red[1][threadIdx.x >> 6] = nt;
    red[2][threadIdx.x >> 6] = nr;
  }
  __syncthreads();
  if (threadIdx.x < 3)
    partial[blockIdx.x * 3 + threadIdx.x] =
        red[threadIdx.x][0] + red[threadIdx.x][1] + red[threadIdx.x][2] + red[threadIdx.x][3];
}

__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {   // SplitMix64 output function
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

// one block: folds the partials of this call (integers: any order gives the same sums), then Eq. 8, Eq. 9 and the draw
__global__ __launch_bounds__(256) void ssf_finish_kernel(const unsigned long long* __restrict__ partial, int blocks,
                                                         int have_ref, double eta, unsigned long long seed,
                                                         unsigned long long frame_index,
                                                         unsigned long long* __restrict__ sums_out,
                                                         int* __restrict__ skip_out, double* __restrict__ prob_out) {
  unsigned long long s[3] = {0, 0, 0};
  for (int b = threadIdx.x; b < blocks; b += 256) {
    s[0] += partial[b * 3];
    s[1] += partial[b * 3 + 1];
    s[2] += partial[b * 3 + 2];
  }
  __shared__ unsigned long long red[3][4];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s[k] += __shfl_xor(s[k], o);
    if ((threadIdx.x & 63) == 0) red[k][threadIdx.x >> 6] = s[k];
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  const unsigned long long dot = red[0][0] + red[0][1] + red[0][2] + red[0][3];
  const unsigned long long nt = red[1][0] + red[1][1] + red[1][2] + red[1][3];
  const unsigned long long nr = red[2][0] + red[2][1] + red[2][2] + red[2][3];
  double p = 0.0;
  if (have_ref && nt != 0 && nr != 0 && eta < 1.0) {
    double sc = (double)dot / sqrt((double)nt * (double)nr);
    if (sc > 1.0) sc = 1.0;
    p = (sc - eta) / (1.0 - eta);
    if (p < 0.0) p = 0.0;
  }
  const double u = (double)(mix64(seed + (frame_index + 1) * 0x9E3779B97F4A7C15ULL) >> 11) * (1.0 / 9007199254740992.0);
  if (sums_out) { sums_out[0] = dot; sums_out[1] = nt; sums_out[2] = nr; }
  *skip_out = (have_ref && u < p) ? 1 : 0;
  if (prob_out) *prob_out = p;
}

int static_fail(int code, const char* msg) {
  g_sdstream_create_error = msg;
  return code;
}

}  // namespace

extern "C" int sdstream_ssf_static(const uint8_t* frame, const uint8_t* reference, int32_t height, int32_t width,
                                   double eta, uint64_t seed, uint64_t frame_index, uint64_t* sums_out,
                                   int32_t* skip_out, double* prob_out, void* hip_stream) {
  if (!frame || !skip_out) return static_fail(SDSTREAM_E_INVALID_ARG, "sdstream_ssf_static: null frame or skip_out");
  if (height < 1 || width < 1) return static_fail(SDSTREAM_E_SHAPE, "sdstream_ssf_static: empty frame");
  const long long n = (long long)height * width * 3;
  if (n > SDSTREAM_SSF_STATIC_MAX_BYTES)
    return static_fail(SDSTREAM_E_SHAPE, "sdstream_ssf_static: frame larger than SDSTREAM_SSF_STATIC_MAX_BYTES");
  if ((((uintptr_t)frame) | ((uintptr_t)reference)) & 15)
    return static_fail(SDSTREAM_E_INVALID_ARG, "sdstream_ssf_static: frame and reference must be 16-byte aligned");
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return static_fail(SDSTREAM_E_HIP, "sdstream_ssf_static: no current device");
  unsigned long long* part = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {   // first call on this device, which is current: this device's copy of the array
      void* sym = nullptr;
      const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !sym) return static_fail(SDSTREAM_E_HIP, "sdstream_ssf_static: hipGetSymbolAddress failed");
      g_scratch_ptr[dev] = (unsigned long long*)sym;
    }
    part = g_scratch_ptr[dev];
  }
  long long want = (n / 16 + 255) / 256;
  const int blocks = (int)(want < 1 ? 1 : want > kMaxBlocks ? kMaxBlocks : want);
  hipStream_t s = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(ssf_partial_kernel, dim3(blocks), dim3(256), 0, s, frame, reference, n, part);
  hipLaunchKernelGGL(ssf_finish_kernel, dim3(1), dim3(256), 0, s, (const unsigned long long*)part, blocks,
                     reference ? 1 : 0, eta, (unsigned long long)seed, (unsigned long long)frame_index,
                     (unsigned long long*)sums_out, skip_out, prob_out);
  if (hipGetLastError() != hipSuccess) return static_fail(SDSTREAM_E_HIP, "sdstream_ssf_static: kernel launch failed");
  return SDSTREAM_OK;
}
