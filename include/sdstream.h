/*
 * sdstream - the Stream Batch denoising step of StreamDiffusion (arXiv 2312.12491) for AMD MI355X (gfx950).
 *
 * One handle owns one static-shape denoising engine: the weights of a latent-diffusion U-Net, the rolling
 * latent queue of Sec. 3.1, the per-slot reference latents needed by residual classifier-free guidance
 * (Sec. 3.3), the pre-computed caches of the appendix "Pre-computation" (per-step noise, sqrt(alpha)/sqrt(beta),
 * time-embedding biases, cross-attention K/V of the prompt) and the reference image of the stochastic
 * similarity filter (Sec. 3.4).  Shapes are fixed at creation, as the paper fixes them per engine (appendix,
 * "Model Acceleration"): a new shape needs a new handle.
 *
 * Conventions
 *   - Every function returns SDSTREAM_OK (0) or a negative SDSTREAM_E_* code; nothing throws or aborts.  After a
 *     failure sdstream_last_error() gives a message.  A call that fails its argument checks leaves the handle as
 *     it was; sdstream_step with a new timestep list clears the queue before it launches anything, so a HIP
 *     error reported after that point leaves an empty queue.
 *   - "host" / "device" on a pointer says where the memory lives.  The library never keeps, frees or writes a
 *     caller's input pointer after the call returns (device inputs must stay valid until the stream has run).
 *   - Tensors at the boundary are float32, latents NCHW [.,C,H,W], contexts row-major [L,D].
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls enqueue work and return
 *     without synchronising unless stated otherwise.
 *   - A handle may be used by one thread at a time.
 */
#ifndef SDSTREAM_H
#define SDSTREAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SDSTREAM_OK 0
#define SDSTREAM_E_INVALID_ARG (-1)
#define SDSTREAM_E_NOT_READY (-2)
#define SDSTREAM_E_SHAPE (-3)
#define SDSTREAM_E_NOMEM (-4)
#define SDSTREAM_E_HIP (-5)

#define SDSTREAM_MAX_LEVELS 8

/* cfg_mode: which noise the scheduler update sees */
#define SDSTREAM_CFG_NONE 0    /* eps_c                                                        */
#define SDSTREAM_CFG_FULL 1    /* Eq. 2, 2n U-Net rows per frame                               */
#define SDSTREAM_CFG_SELF 2    /* Eq. 5-6 with the input latent as reference, n rows           */
#define SDSTREAM_CFG_ONETIME 3 /* Eq. 5-7, reference from one negative-prompt row, n+1 rows    */

typedef struct sdstream sdstream_t;

typedef struct {
  int32_t in_channels;                          /* latent channels (4)                                         */
  int32_t n_levels;                             /* resolution levels of the U-Net                              */
  int32_t block_channels[SDSTREAM_MAX_LEVELS];  /* width per level, e.g. 320,640,1280,1280                     */
  int32_t layers_per_block;                     /* ResBlocks per level on the way down (one more on the way up)*/
  uint32_t attn_level_mask;                     /* bit l: a transformer follows every ResBlock of level l      */
  int32_t num_heads;                            /* exactly one of num_heads / head_dim is > 0                  */
  int32_t head_dim;
  int32_t mid_attention;                        /* transformer between the two middle ResBlocks                */
  int32_t context_len, context_dim;             /* prompt embedding [L,D]                                      */
  int32_t norm_groups;                          /* GroupNorm groups                                            */
  int32_t latent_h, latent_w;
  int32_t dtype;                                /* 0: float32 storage and arithmetic; 1: bf16 storage, MFMA    */
  int32_t n_denoise;                            /* n = Stream Batch size = denoising steps                     */
  int32_t n_streams;                            /* S independent streams sharing weights, noise and prompt     */
  int32_t cfg_mode;                             /* SDSTREAM_CFG_*                                              */
  int32_t scheduler;                            /* 0: LCM re-noising with the cached noise; 1: DDIM (eta = 0); */
                                                /* 2: as 0 with x0 = c_skip(tau) x + c_out(tau) (x - b eps)/a,  */
                                                /*    the appendix's parameterisation instead of its (0,1) form */
  int32_t cross_frame;                          /* 1: Stream Batch cross-frame attention (Sec. 3.2, K_Batch /  */
                                                /*    V_Batch): every self-attention of a row uses the keys and */
                                                /*    values of all n rows of its stream (and prompt branch);   */
                                                /*    0: rows independent                                       */
  int32_t image_width;                          /* > 0: the engine also owns the latent <-> image stage (a tiny */
                                                /*    convolutional autoencoder of this width, 64 in the         */
                                                /*    workloads; needs in_channels = 4); 0: latents only         */
} sdstream_config;

/* Creates an engine on the current HIP device and allocates all device state.  No weights yet. */
int sdstream_create(const sdstream_config* cfg, sdstream_t** out);
void sdstream_destroy(sdstream_t* h);
const char* sdstream_last_error(const sdstream_t* h); /* h may be NULL: message of the last failed create */

/* Weight manifest: the order, names, shapes (conv OIHW, linear [out,in]) and kinds
 * (0 weight, 1 bias, 2 norm scale, 3 norm shift) of the tensors in the blob load_weights expects. */
int64_t sdstream_param_count(const sdstream_t* h);
int32_t sdstream_manifest_size(const sdstream_t* h);
int sdstream_manifest_entry(const sdstream_t* h, int32_t index, char* name, size_t name_cap, int32_t shape[4],
                            int32_t* ndim, int32_t* kind);

/* host_blob: host, float32, all tensors of the manifest back to back; `bytes` must equal 4 * param_count.
 * The library copies, converts (bf16 round-to-nearest-even when dtype = 1) and repacks; synchronous. */
int sdstream_load_weights(sdstream_t* h, const void* host_blob, size_t bytes);

/* alphas_cumprod: host, [1000] (alpha of Eq. 1 per timestep); NULL restores the built-in scaled-linear table.
 * Resets the queue. */
int sdstream_set_schedule(sdstream_t* h, const float* alphas_cumprod);

/* The pre-sampled noise of the appendix: host, [n][S][C][H][W], fixed for the session.  Waits for all work on
 * the device, copies, then does what sdstream_reset does (queue and reference latents zeroed). */
int sdstream_set_noise(sdstream_t* h, const float* host_noise);

/* One pass of Sec. 3.1: takes one clean latent per stream, advances every queued latent one denoising step
 * (noise-in Eq. 1, batched U-Net, guidance Eq. 2 / Eq. 5-7, update Eq. 4, re-noise, queue shift) and writes the
 * latent that has finished its n-th step.
 *   x0_in        device [S,C,H,W]
 *   context      device [L,D] prompt embedding; neg_context likewise, required for CFG_FULL and CFG_ONETIME
 *   context_epoch the cross-attention K/V cache is rebuilt only when this value differs from the last call's
 *   timesteps    host [n], strictly decreasing, each in [0,999]; a change recomputes the caches, resets the queue
 *   gamma, delta guidance scale and residual-noise scale of Eq. 6 (ignored for CFG_NONE)
 *   out_latent   device [S,C,H,W]: x0-prediction of the frame given n-1 calls earlier
 *   out_valid    host, may be NULL: 0 during the first n-1 calls after a reset, else 1 */
int sdstream_step(sdstream_t* h, const float* x0_in, const float* context, const float* neg_context,
                  uint64_t context_epoch, const int32_t* timesteps, float gamma, float delta, float* out_latent,
                  int32_t* out_valid, void* hip_stream);

/* The U-Net alone (the eps_theta of Sec. 3.1), for checking it apart from the queue:
 *   x device [N,C,H,W], t host [N] in [0,999], ctx device [L,D], eps_out device [N,C,H,W];
 *   1 <= N <= sdstream_max_batch(h).  Does not touch the queue.
 *   With cross_frame = 1 (Sec. 3.2) every complete run of n_denoise consecutive rows is one stream batch whose rows
 *   share self-attention keys and values; rows left over at the end stay alone.  (In sdstream_step the batches are
 *   the n rows of a stream, the positive- and, under CFG_FULL, the negative-prompt rows each among themselves.) */
int sdstream_unet_forward(sdstream_t* h, const float* x, const int32_t* t, const float* ctx, int32_t n,
                          float* eps_out, void* hip_stream);
int32_t sdstream_max_batch(const sdstream_t* h);

/* Stochastic similarity filter (Eq. 8-9) on one raw frame: device, uint8 [h*w*3].  Computes the cosine
 * similarity with the stored reference frame from exact integer sums, the skip probability for threshold eta
 * and the decision u_k < P with u_k the counter-based uniform of (seed, frame_index) (see sdstream_ssf_decide).
 * A frame that is not skipped becomes the reference.  The first frame after create/reset is never skipped.
 * Synchronises the stream (it returns a decision).  skip: host; prob: host, may be NULL. */
int sdstream_ssf(sdstream_t* h, const uint8_t* frame, int32_t height, int32_t width, double eta, uint64_t seed,
                 uint64_t frame_index, int32_t* skip, double* prob, void* hip_stream);

/* The host half of the filter, usable without a GPU: given dot = I_t.I_ref, n_t = |I_t|^2, n_ref = |I_ref|^2,
 * returns 1 to skip, 0 to process.  S_C = min(1, dot / sqrt(n_t * n_ref)) in double; P = max(0,(S_C-eta)/(1-eta)),
 * P = 0 when eta >= 1 or a norm is zero; u = (mix(seed + (frame_index+1)*0x9E3779B97F4A7C15) >> 11) * 2^-53 with
 * mix the SplitMix64 output function; skip iff u < P. */
int sdstream_ssf_decide(uint64_t dot, uint64_t n_t, uint64_t n_ref, double eta, uint64_t seed, uint64_t frame_index,
                        double* prob);

/* The hard-threshold filter the paper compares the sampled one with (note at the end of Sec. 3.4; Table 3): skip
 * exactly when S_C > eta, i.e. when Eq. 9 gives a positive probability; nothing is drawn.  Same reduction kernel,
 * same reference-frame rule (only a frame that is let through becomes the reference; the first frame always is).
 * *similarity gets S_C (0 while there is no reference).  The two filters share the engine's reference frame: use
 * one of them per engine, or call sdstream_reset in between. */
int sdstream_ssf_decide_hard(uint64_t dot, uint64_t n_t, uint64_t n_ref, double eta, double* similarity);
int sdstream_ssf_hard(sdstream_t* h, const uint8_t* frame, int32_t height, int32_t width, double eta, int32_t* skip,
                      double* similarity, void* hip_stream);

/* Run statistics of the similarity filters (either kind) since create / the last reset, for the duty-cycle
 * comparison of Sec. 3.4 and Table 3: frames seen, frames let through (= denoising steps that still run; the
 * paper's power figure follows this share), and the longest run of consecutive skips (how long the output stayed
 * stuck).  Host pointers, each may be NULL. */
int sdstream_ssf_run_stats(const sdstream_t* h, int64_t* frames, int64_t* processed, int64_t* longest_skip_run);

/* The latent <-> image stage (appendix: the pipeline wraps a tiny autoencoder around the U-Net; the paper names it
 * and gives no layers, so these are this library's): all convolutions 3x3 with zero padding, one width w,
 *   Block(x) = ReLU(conv_c(ReLU(conv_b(ReLU(conv_a(x))))) + x)
 *   encoder : u8 image / 255 -> conv(3 -> w) -> Block -> 3 x [conv stride 2, no bias -> 3 Blocks] -> conv(w -> 4)
 *   decoder : 3 tanh(latent / 3) -> ReLU(conv(4 -> w)) -> 3 x [3 Blocks -> nearest 2x -> conv, no bias] -> Block
 *             -> conv(w -> 3) -> clamp to [0,1]; u8 image = round(255 x), ties to even
 * Images are device u8 [S][8 latent_h][8 latent_w][3] (one per stream), latents device float32 [S][4][h][w].
 * The stage has its own weight manifest and blob (same conventions as the U-Net's, encoder first).
 * Only engines created with image_width > 0 have it; the others return SDSTREAM_E_NOT_READY. */
int64_t sdstream_image_param_count(const sdstream_t* h);
int32_t sdstream_image_manifest_size(const sdstream_t* h);
int sdstream_image_manifest_entry(const sdstream_t* h, int32_t index, char* name, size_t name_cap, int32_t shape[4],
                                  int32_t* ndim, int32_t* kind);
int sdstream_load_image_weights(sdstream_t* h, const void* host_blob, size_t bytes);
int sdstream_encode(sdstream_t* h, const uint8_t* image, float* latent_out, void* hip_stream);
/* image_out (u8) and image_f32_out (float32 [S][3][H][W], the image before quantisation) may each be NULL, not both */
int sdstream_decode(sdstream_t* h, const float* latent, uint8_t* image_out, float* image_f32_out, void* hip_stream);
/* sdstream_step with the boundary at the image: encoder -> one Stream Batch step -> decoder, the latents staying in
 * the engine.  frame: the stream's next input image; image_out: the image of the frame given n-1 calls earlier.
 * Other arguments, validity and queue behaviour as in sdstream_step.  Replayed as ONE HIP graph per call when the
 * caller passes the same two image buffers (and gamma, delta) as on the previous call with the same queue parity;
 * otherwise the graph is captured again first.  (The similarity filter is a host decision taken before this call:
 * a skipped frame is simply not submitted.) */
int sdstream_step_image(sdstream_t* h, const uint8_t* frame, const float* context, const float* neg_context,
                        uint64_t context_epoch, const int32_t* timesteps, float gamma, float delta, uint8_t* image_out,
                        int32_t* out_valid, void* hip_stream);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The measurement and decision of sdstream_ssf with no handle, no allocation (no hipMalloc / hipFree /
 * allocating routine, on any call) and no host synchronisation: the caller keeps the reference frame, everything is
 * enqueued on `hip_stream`, results land in device memory.
 *   frame      device, uint8 [height*width*3], 16-byte aligned
 *   reference  device, same size and alignment, or NULL (no reference yet: never skipped, P = 0)
 *   sums_out   device [3] or NULL: dot = I_t.I_ref, |I_t|^2, |I_ref|^2 as exact integers
 *   skip_out   device int32: 1 to skip, 0 to process (then the caller makes `frame` its reference)
 *   prob_out   device double or NULL: P of Eq. 9
 * Same arithmetic and the same draw u(seed, frame_index) as sdstream_ssf_decide.
 * The per-block partial sums sit in a file-scope device array of 24 KiB that each GPU the library runs on holds
 * until the process ends; every call on a GPU shares it, so calls that overlap on one GPU (two streams, two
 * threads) race - serialise them.  Frames larger than SDSTREAM_SSF_STATIC_MAX_BYTES are rejected with
 * SDSTREAM_E_SHAPE; the message is read with sdstream_last_error(NULL). */
#define SDSTREAM_SSF_STATIC_MAX_BYTES (1LL << 28)
int sdstream_ssf_static(const uint8_t* frame, const uint8_t* reference, int32_t height, int32_t width, double eta,
                        uint64_t seed, uint64_t frame_index, uint64_t* sums_out, int32_t* skip_out, double* prob_out,
                        void* hip_stream);

/* Waits for the device, then zeroes the queue and the reference latents and clears the filter's reference frame,
 * the filter's run statistics and the warm-up counter. */
int sdstream_reset(sdstream_t* h);

/* Multiply-add work of one U-Net row as 2*M*N*K summed over every convolution, linear layer and attention
 * product that runs per step (cached K/V projections and the time-embedding path excluded). */
double sdstream_flops_per_row(const sdstream_t* h);

/* Per-kernel-class timing.  While enabled, sdstream_step / sdstream_unet_forward launch kernel by kernel with
 * HIP events around each launch on the caller's stream (no graph replay) and accumulate per class.
 * sdstream_profile_read synchronises and copies up to `cap` classes: name (<= 31 chars), launches, total
 * milliseconds, algorithmic flops and algorithmic bytes; returns the number of classes. */
typedef struct {
  char name[32];
  int64_t launches;
  double ms;
  double flops;
  double bytes;
} sdstream_profile_entry;
int sdstream_profile_enable(sdstream_t* h, int32_t on);
int sdstream_profile_reset(sdstream_t* h);
int32_t sdstream_profile_read(sdstream_t* h, sdstream_profile_entry* out, int32_t cap);

/* 0: launch kernels one by one; 1 (default): replay the step as a HIP graph captured on first use. */
int sdstream_use_graph(sdstream_t* h, int32_t on);

/* Measurement aid: the practical bf16 matrix-core ceiling of the device the handle lives on.  Runs a kernel that
 * does nothing but dependent-free v_mfma_f32_16x16x32_bf16 chains from registers (8 waves per compute unit, `iters`
 * rounds of 8 MFMAs per wave) on `hip_stream`, synchronises, and returns the achieved rate in *tflops_out
 * (host).  Says what clock the chip holds under matrix load; no step of the hot path uses it.
 * iters must be in [1, 1 << 20]. */
int sdstream_mfma_ceiling(sdstream_t* h, int32_t iters, double* tflops_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SDSTREAM_H */
