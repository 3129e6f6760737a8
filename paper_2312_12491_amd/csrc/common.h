// Shared declarations of the sdstream HIP library: storage types, kernel parameter blocks, launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

enum { EPI_NONE = 0, EPI_GEGLU = 1, EPI_SILU = 2, EPI_RELU = 3, EPI_SOFTMAX = 4 };
// RELU is applied after the residual sum.  SOFTMAX (MFMA kernels, 160-column tiles): the columns come in segments of
// sm_lp (16 or 80) of which the first sm_len are real; the output is softmax in base 2 over each segment's real
// columns (the weights carry log2(e)), zero elsewhere and in columns >= sm_cols.

// Division by a launch-time constant through one multiply-high (the round-up method of Granlund and Montgomery):
// exact for 0 <= x < 2^31.  An integer division by a run-time value costs ~30 instructions on this target, and
// the index set-up of a GEMM block has a dozen of them.
struct FastDiv {
  unsigned d, m, sh1, sh2;
};
inline FastDiv make_fastdiv(unsigned d) {
  FastDiv f;
  unsigned l = 0;
  while ((1ull << l) < d) ++l;   // ceil(log2 d), 0 for d = 1
  f.d = d;
  f.m = (unsigned)(((((unsigned long long)1 << l) - d) << 32) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}
__device__ __forceinline__ int fast_div(int x, const FastDiv& f) {
  const unsigned t = __umulhi(f.m, (unsigned)x);
  return (int)((t + (((unsigned)x - t) >> f.sh1)) >> f.sh2);
}

// C[M,N] = gather(A)[M,K] * W[N,K]^T (+ bias, + per-sample bias, activation, + residual).
// A is the implicit im2col matrix of one or two NHWC activations (channel concat): row m = (sample, oy, ox),
// column k = tap * (C1+C2) + c with tap = ky*ksize + kx; source pixel (oy*stride + ky - pad, ox*stride + kx - pad)
// in the (optionally nearest-2x upsampled) input, zero outside.  Linear layers are ksize = 1 over "pixels" = tokens.
struct IgemmParams {
  const void* src1;
  const void* src2;
  int C1, C2;
  int Hin, Win;      // stored size of the sources
  int Hout, Wout;
  int ksize, stride, upsample;
  int M, N, K;
  const void* W;         // layout depends on the kernel (generic: [N][K]; MFMA: fragment-packed)
  const float* bias;     // [N] or null
  const float* rowbias;  // [samples][rowbias_ld] or null (time-embedding bias of a ResBlock)
  int rowbias_ld;
  const void* residual;  // [M][Nout] or null
  void* out;             // [M][Nout], Nout = N (N/2 for GEGLU)
  int epilogue;
  int splitk;            // set by the MFMA launcher: number of K splits, fp32 partials [splitk][M][N] in `workspace`
  float* workspace;      // MFMA kernel only: split-K scratch (null forbids split-K)
  long long workspace_floats;
  int xcd_chunked;       // set by the MFMA launcher: block -> tile order (see tile_of_block)
  const void* zeros;     // MFMA kernel only: >= 16 readable zero bytes (source of padded / out-of-range rows)
  FastDiv fd_hw, fd_w, fd_ct, fd_ks, fd_n;   // set by the MFMA launcher: Hout*Wout, Wout, C1+C2, ksize, N
  // MFMA kernels only.  A LayerNorm in front of a linear layer is folded into it: with W' = W diag(gamma),
  //   LN(x) W^T = rstd (x W'^T - mean wsum) + beta W^T,   wsum[n] = sum_k W'[n][k],
  // so the layer multiplies the un-normalised rows, and its epilogue applies mean / rstd of the row, which come from
  // partial sums that the layer PRODUCING the rows left behind (stats_out of that layer = ln_stats of this one).
  const float* ln_stats;   // [M][ln_parts][2]: partial (sum, sum of squares) of input row m over a range of its channels; null = no fold
  int ln_parts;
  const float* ln_wsum;    // [N]; `W` holds W' and `bias` holds bias + beta W^T
  float ln_eps;
  float* stats_out;        // [M][ceil(N/BN)][2] partial sums of this layer's bf16-rounded output rows, one part per column tile; null = none
  int no_splitk;           // layers with ln_stats or stats_out never split K (their epilogue must see whole sums)
  // GroupNorm statistics of this layer's output, left by its epilogue for the GroupNorm that follows (only the
  // eight-wave 128 x 160 kernel does it; the launcher decides with gn_stats_splits): partial sums per
  // (sample, row tile of the sample, group) in the layout the GroupNorm apply pass folds
  float* gn_stats;         // [samples][Hout*Wout/128][gn_groups][2], or null
  int gn_cg, gn_groups;    // channels per group (divides 160), groups of the whole output
  // GroupNorm (scale and shift, no activation) applied to this layer's INPUT rows as they sit in LDS (64-row
  // row-resident kernel only; the launcher decides): the partial sums of the norm's statistics, as above, and its vectors
  const float* gn_in_stats;   // [samples][gn_in_splits][gn_in_groups][2], or null
  const float* gn_in_gamma;
  const float* gn_in_beta;
  int gn_in_splits, gn_in_groups;
  float gn_in_eps;
  // MFMA direct-to-LDS kernels only: a second K segment behind the taps, a 1x1 convolution over the channel concat of
  // src3 | src4 (same pixels as the output: stride 1, no upsampling), K = ksize^2 (C1+C2) + C3 + C4.  All four
  // channel counts multiples of 64.  Used to sum a ResBlock's 1x1 skip convolution into its second 3x3 convolution.
  const void* src3;
  const void* src4;
  int C3, C4;
  int sm_lp, sm_len, sm_cols;   // EPI_SOFTMAX
  // MFMA kernels: rows from slot_m on (a multiple of the row tile) use a second set of weights / vectors, slot_w_bytes
  // behind W and slot_v_bytes behind bias and ln_wsum (the negative prompt's matrices of a folded cross-attention)
  int slot_m;
  long long slot_w_bytes, slot_v_bytes;
  int dev_exp;                  // development builds only: bit mask of timing experiments (results are wrong with any bit set)
  int force_variant, force_bn;  // force_bn != 0: kernel variant (1: 128-row, 2: 64-row direct-to-LDS; 0: register-staged) and tile width to use, no split-K
};

#define LN_MAX_PARTS 20   // most parts of row statistics a folded LayerNorm reads (column tiles of the producing layer)

// Tile geometry the MFMA launcher will pick for p (M set): BN is what stats_out is indexed by.
// grouped: the launch takes the eight-wave kernel (two wave groups splitting the block's K range)
struct IgemmPlan { int variant, bm, bn, splitk; bool grouped; };
IgemmPlan igemm_mfma_plan(const IgemmParams& p);

#define GN_MAX_SPLIT 64
struct GroupNormParams {
  const void* src1;
  const void* src2;
  int C1, C2, HW, groups, samples;
  float eps;
  int silu;
  const float* gamma;
  const float* beta;
  float* stats;  // scratch, [samples][GN_MAX_SPLIT][groups][2] floats: partial sums, or mean / rstd per (sample, group)
  void* out;     // [samples][HW][C1+C2]
};

struct LayerNormParams {
  const void* src;
  int rows, C;
  float eps;
  const float* gamma;
  const float* beta;
  void* out;
};

// softmax(q k^T / sqrt(d)) v per (sample, head).  q/k/v/out are row-major with their own leading dimensions
// so fused QKV buffers can be addressed in place; head h uses columns [h*d, (h+1)*d).
struct AttnParams {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int ldq, ldk, ldv, ldo;
  int Sq, Skv, heads, d, samples;
  long long kv_sample_stride;   // elements between samples in k/v (0 with kv_select: cached prompt K/V)
  const int* kv_select;         // per sample: which cached context (0 positive, 1 negative) or null
  long long kv_select_stride;   // elements between cached contexts
  int kv_group;                 // > 1: Stream Batch cross-frame attention (Sec. 3.2): samples [0, kv_group_rows) come in runs
  int kv_group_rows;            //   of kv_group consecutive samples that attend to the keys / values of the whole run
                                //   (k/v rows of consecutive samples must be contiguous: kv_sample_stride = Skv * ld)
  float scale;
};

template <typename T> void launch_igemm_generic(const IgemmParams& p, hipStream_t s);
void launch_igemm_mfma(const IgemmParams& p, hipStream_t s);
bool igemm_mfma_supported(const IgemmParams& p);
bool igemm_mfma_available();
template <typename T> void launch_group_norm(const GroupNormParams& p, hipStream_t s);
// bf16 GroupNorm whose statistics pass a producing layer can replace: true when the norm runs as the pair
// (partial sums, apply) rather than as the single kernel of the small planes
bool group_norm_takes_partials(const GroupNormParams& p);
// the apply pass alone: p.stats already holds `splits` partial sums per (sample, group)
void launch_group_norm_apply(const GroupNormParams& p, int splits, hipStream_t s);
template <typename T> void launch_layer_norm(const LayerNormParams& p, hipStream_t s);
template <typename T> void launch_attention_generic(const AttnParams& p, hipStream_t s);
void launch_attention_mfma(const AttnParams& p, hipStream_t s);
bool attention_mfma_supported(const AttnParams& p);

// conv_in: fp32 NCHW [N,Cin,H,W] -> T NHWC [N,HW,C0]; w fp32 OIHW, 3x3 pad 1.
// flags: CONV_IN_SQUASH applies 3 tanh(x / 3) to the input (the decoder's latent clamp), CONV_IN_RELU a ReLU to the output.
enum { CONV_IN_SQUASH = 1, CONV_IN_RELU = 2 };
template <typename T>
void launch_conv_in(const float* x, const float* w, const float* b, void* out, int N, int Cin, int H, int W, int C0,
                    int flags, hipStream_t s);
// conv_out: T NHWC [N,HW,C0] -> fp32 NCHW [N,Cout,H,W]; w T [Cout][9][C0] (tap-major), 3x3 pad 1.
template <typename T>
void launch_conv_out(const void* x, const void* w, const float* b, float* out, int N, int Cout, int H, int W, int C0,
                     hipStream_t s);

// Image side of the tiny autoencoder: u8 HWC image -> first convolution (3 -> C0, x/255, fp32 weights OIHW), and last
// convolution (C0 -> 3, weights T [3][9][C0]) -> clamp [0,1] -> float NCHW and / or u8 HWC (either may be null).
template <typename T>
void launch_image_in(const uint8_t* img, const float* w, const float* b, void* out, int N, int H, int W, int C0,
                     hipStream_t s);
template <typename T>
void launch_image_out(const void* x, const void* w, const float* b, float* out_f32, uint8_t* out_u8, int N, int H, int W,
                      int C0, hipStream_t s);

// Per-prompt matrices of a folded cross-attention (bf16 path), see xattn.hip.  kv: the prompt's [L][2C] keys | values
// (bf16, row pitch ld_kv elements); wq, wo: the site's q and output projections, fp32 row-major [C][C]; gamma, beta: the
// LayerNorm in front of q; raw: fp32 scratch [Npad][C]; outputs: QK packed [Npad][C] with wsum / lnb [Npad], VO packed [C][Npad].
void launch_xattn_fold(const void* kv, int ld_kv, const float* wq, const float* wo, const float* gamma, const float* beta,
                       float* raw, void* qk_packed, float* wsum, float* lnb, void* vo_packed, int C, int heads, int d,
                       int L, int Lp, int Npad, hipStream_t s);

// e[row] = [cos(t f_j) ; sin(t f_j)], f_j = exp(-ln(1e4) j/half), evaluated in double.
void launch_time_embedding(const int* t, float* out, int rows, int C0, hipStream_t s);

struct StreamParams {
  int S, n, E;           // streams, denoising steps, elements per latent
  int mode, scheduler;
  float gamma, delta;
  const float* a;        // [n] sqrt(alpha), device
  const float* b;        // [n] sqrt(beta), device
  const float* cskip;    // [n] c_skip(tau_i), c_out(tau_i) of the consistency parameterisation (scheduler 2)
  const float* cout;
  const float* noise;    // [n][S][E]
  const float* x0_in;    // [S][E]
  float* xcur;           // [rows][E] U-Net input batch of this call
  float* xnext;          // the next call's batch (rows i+1 written by the tail)
  float* rcur;           // [S*n][E] reference latents, same row order
  float* rnext;
  const float* eps;      // [rows][E] U-Net output
  float* out;            // [S][E]
};
void launch_stream_head(const StreamParams& p, hipStream_t s);
void launch_stream_tail(const StreamParams& p, hipStream_t s);

// SSF: dot(frame, ref) and |frame|^2 as exact 64-bit integers into sums[0..1]; copies frame to spare.
void launch_ssf_reduce(const uint8_t* frame, const uint8_t* ref, uint8_t* spare, long long n, unsigned long long* sums,
                       hipStream_t s);

// Weight repacking from the canonical fp32 layouts.  All run on device from a staging copy.
//  conv OIHW [O][I][kh][kw] -> T [O][kh*kw][I] (tap-major K), optionally GEGLU row interleave
template <typename T>
void launch_repack_rowmajor(const float* src, void* dst, int O, int I, int taps, int geglu_block, hipStream_t s);
//  `in_scale` (may be null): per input channel factor applied before rounding (the scale of a folded LayerNorm)
//  `ksteps_total` / `kstep0`: the matrix is one K segment of a wider packed matrix (0 / 0: it stands alone)
void launch_repack_mfma(const float* src, void* dst, int O, int I, int taps, int geglu_block, const float* in_scale,
                        int ksteps_total, int kstep0, hipStream_t s);
// Vectors of a LayerNorm (gamma, beta over the I input channels) folded into the [O][I] matrix `src`, in the row order
// of the packed matrix: wsum[n] = sum_i bf16(gamma_i w[n][i]) (what the matrix core multiplies), lnb[n] = sum_i beta_i w[n][i]
void launch_ln_fold_vectors(const float* src, const float* gamma, const float* beta, float* wsum, float* lnb, int O, int I,
                            int geglu_block, hipStream_t s);
void launch_add_f32(float* dst, const float* src, int n, hipStream_t s);
void launch_permute_bias(const float* src, float* dst, int O, int geglu_block, hipStream_t s);
template <typename T> void launch_convert(const float* src, void* dst, long long n, hipStream_t s);
void launch_fill_u32(void* dst, unsigned v, long long n_words, hipStream_t s);
void launch_copy_rows_f32(const float* src, float* dst, long long n, hipStream_t s);

// blocks of 4 waves running `iters` rounds of 8 register-only MFMAs each; `sink` is never written
void launch_mfma_ceiling(int iters, int blocks, float* sink, hipStream_t s);
