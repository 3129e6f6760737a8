// Host side of libsdstream: configuration, weight manifest and repacking, the static U-Net plan,
// the Stream Batch state machine and the C ABI declared in include/sdstream.h.
#include "common.h"
#include "sdstream.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <string>
#include <vector>

// message of the last failed call that had no handle to keep it in (sdstream_last_error(NULL)); per thread
thread_local std::string g_sdstream_create_error;
#define g_create_error g_sdstream_create_error

namespace {

// ------------------------------------------------------------------------------------------------
// plan-time interval allocator (first fit, coalescing).  Offsets are in bytes for ONE sample; the
// arena holds max_batch times that, sample-major per buffer, so a smaller batch uses a prefix.
// ------------------------------------------------------------------------------------------------
struct Interval {
  size_t off, size;
  bool free;
};
struct PlanAllocator {
  std::vector<Interval> iv;
  size_t peak = 0;
  size_t alloc(size_t bytes) {
    bytes = (bytes + 255) & ~(size_t)255;
    for (size_t i = 0; i < iv.size(); ++i) {
      if (iv[i].free && iv[i].size >= bytes) {
        if (iv[i].size > bytes) {
          Interval rest{iv[i].off + bytes, iv[i].size - bytes, true};
          iv[i].size = bytes;
          iv.insert(iv.begin() + i + 1, rest);
        }
        iv[i].free = false;
        return iv[i].off;
      }
    }
    // grow: extend a trailing free interval or append
    if (!iv.empty() && iv.back().free) {
      iv.back().size = bytes;
      iv.back().free = false;
      peak = iv.back().off + bytes;
      return iv.back().off;
    }
    Interval n{peak, bytes, false};
    iv.push_back(n);
    peak += bytes;
    return n.off;
  }
  void release(size_t off) {
    for (size_t i = 0; i < iv.size(); ++i) {
      if (iv[i].off == off && !iv[i].free) {
        iv[i].free = true;
        if (i + 1 < iv.size() && iv[i + 1].free) {
          iv[i].size += iv[i + 1].size;
          iv.erase(iv.begin() + i + 1);
        }
        if (i > 0 && iv[i - 1].free) {
          iv[i - 1].size += iv[i].size;
          iv.erase(iv.begin() + i);
        }
        return;
      }
    }
  }
};

// split-K is used only for GEMMs with few output tiles; splits * M * N never exceeds this
constexpr size_t kSplitKWorkspaceFloats = (size_t)16 << 20;

enum OpKind { OP_IGEMM, OP_GN, OP_LN, OP_ATTN, OP_CONV_IN, OP_CONV_OUT, OP_IMAGE_IN, OP_IMAGE_OUT };
enum ProfClass {
  PC_IGEMM_MFMA, PC_IGEMM_VALU, PC_ATTN_MFMA, PC_ATTN_VALU, PC_GROUP_NORM, PC_LAYER_NORM, PC_CONV_IN, PC_CONV_OUT,
  PC_STREAM_HEAD, PC_STREAM_TAIL, PC_COUNT
};
const char* kProfNames[PC_COUNT] = {"igemm_mfma", "igemm_valu", "attn_mfma", "attn_valu", "group_norm",
                                    "layer_norm", "conv_in", "conv_out", "stream_head", "stream_tail"};

struct Op {
  OpKind kind;
  int cls;
  bool mfma;
  IgemmParams g;
  GroupNormParams gn;
  LayerNormParams ln;
  AttnParams at;
  int rows_per_sample;   // output pixels / tokens per sample
  double flops_per_row;  // algorithmic multiply-add work per sample
  double bytes_per_row;  // algorithmic bytes per sample (activations in + out)
  double bytes_fixed;    // weights
  int ln_src_op;         // >= 0: index of the op whose stats_out this op's folded LayerNorm reads
  int xattn_site;        // >= 0: a GEMM of a folded cross-attention: its weights belong to the prompt slot of each row
  int xattn_role;        //   1: rows x QK with softmax; 2: probabilities x VO
  int gn_dst_plus1;      // GEMM op: 1 + index of the GroupNorm op that reads only this op's output, right after it (0: none)
  int gn_src_plus1;      // GroupNorm op: 1 + index of that GEMM op (0: none)
  int gn_in_plus1;       // GEMM op: 1 + index of the GroupNorm op right before it whose output only this op reads (0: none)
  int gn_out_plus1;      // GroupNorm op: 1 + index of that GEMM op (0: none)
  // conv_in / conv_out (fp32 NCHW <-> NHWC activations) and image_in / image_out (u8 HWC image <-> NHWC activations)
  const float* cw_f32;
  const void* cw;
  const float* cb;
  const void* cin;
  void* cout_;
  int cH, cW, cCin, cC0, cflags;   // spatial size, channels on the NCHW / image side, channels on the NHWC side
  float* img_f32;                  // image_out: float NCHW image or null
  uint8_t* img_u8;                 // image_out: u8 HWC image or null
};

enum LoadAction { LA_F32, LA_ROWMAJOR, LA_MFMA, LA_BIAS_PERM };
struct Entry {
  std::string name;
  int shape[4];
  int ndim;
  int kind;  // 0 weight 1 bias 2 gamma 3 beta
  size_t count;
  int action;
  size_t dst_off;  // bytes into the weight arena
  int O, I, taps, geglu;
  // a LayerNorm folded into this matrix (LA_MFMA only): byte offsets of the norm's scale / shift and of the two
  // derived vectors (row sums of the scaled weights, shift times weights) for this entry's rows
  bool ln_fold = false;
  size_t ln_g = 0, ln_b = 0, ln_wsum = 0, ln_lnb = 0;
  // LA_MFMA only: the matrix is one K segment of a wider packed matrix (pk_total k-steps of 32 in all, this one from pk_off)
  int pk_total = 0, pk_off = 0;
  bool raw_copy = false;   // also keep the fp32 tensor as it is, at raw_off
  size_t raw_off = 0;
};
struct BiasFix { size_t lnb, bias; int n; bool copy = false; };   // after loading: lnb[0..n) += bias[0..n) (copy: =)

struct LinW {
  size_t w = 0, b = 0;  // byte offsets into the weight arena (b: fp32)
  int N = 0, K = 0;
  bool mfma = false;
  bool has_bias = false;
};

struct KVSite {
  LinW w;        // fused [2C][D]
  size_t cache;  // byte offset in the persistent arena: [2][L][2C] T
  int C;
  // cross-attention folded into two GEMMs (bf16 matrix-core path): per prompt slot, in the persistent arena
  bool xfold = false;
  int heads = 0, d = 0, Lp = 0, Npad = 0;
  size_t wq_raw = 0, wo_raw = 0, ln_g = 0, ln_b = 0;   // weight arena: fp32 copies of q / output projection, the norm in front of q
  size_t qk = 0, vo = 0, wsum = 0, lnb = 0;            // persistent arena, slot 0; slot 1 follows at the *_stride
  size_t mat_stride = 0, vec_stride = 0;
};

}  // namespace

struct sdstream {
  sdstream_config cfg;
  std::string err;
  int elt = 4;  // bytes per activation element
  int max_batch = 0;
  int E = 0;  // elements per latent
  bool use_mfma = false;

  std::vector<Entry> manifest;
  std::vector<BiasFix> bias_fixes;
  int64_t n_params = 0;
  size_t weight_bytes = 0;
  char* weights = nullptr;
  bool weights_loaded = false;

  // activations
  PlanAllocator act;
  char* act_base = nullptr;
  size_t act_bytes = 0;
  // persistent buffers (temb biases, kv caches, state), plain bump allocation in bytes
  size_t persist_bytes = 0;
  char* persist = nullptr;

  std::vector<Op> ops;       // the U-Net
  std::vector<Op> temb_ops;  // time-embedding path (float32)
  std::vector<KVSite> kv_sites;
  size_t off_emb = 0, off_h1 = 0, off_h2 = 0, off_tdev = 0, off_ctxT = 0;
  size_t off_sel_zero = 0, off_sel_step = 0;
  size_t off_xraw = 0;     // fp32 scratch of the cross-attention fold
  size_t xraw_floats = 0;
  int neg_from = 0;        // rows from this index on use the negative prompt (set per U-Net call)
  size_t off_x[2] = {0, 0}, off_r[2] = {0, 0}, off_eps = 0, off_noise = 0, off_ab = 0;
  size_t off_unet_x = 0;  // fp32 input batch for unet_forward
  size_t off_zeros = 0;   // 256 bytes that stay zero
  size_t off_splitk = 0;  // fp32 [splits][M][N] partial tiles of a split-K GEMM (every launch overwrites what it reads back)
  double flops_per_row = 0;

  // state
  std::vector<int> temb_cached;  // timesteps the temb buffers hold
  std::vector<int> timesteps;    // of the stream
  bool have_noise = false;
  bool kv_valid = false;
  bool kv_for_step = false;
  uint64_t kv_epoch = 0;
  int cur = 0;
  long long calls = 0;
  double alphas[1000];

  // latent <-> image stage (cfg.image_width > 0): its own manifest, weights, activation arena and op lists
  std::vector<Entry> img_manifest;
  int64_t img_n_params = 0;
  size_t img_weight_bytes = 0;
  char* img_weights = nullptr;
  bool img_weights_loaded = false;
  PlanAllocator img_act;
  char* img_act_base = nullptr;
  size_t img_act_bytes = 0;
  std::vector<Op> img_enc_ops, img_dec_ops;
  size_t off_img_lat_in = 0, off_img_lat_out = 0;   // fp32 [S][C][h][w] latents between the stage and the step
  struct ImageGraph { hipGraphExec_t exec = nullptr; const void* frame = nullptr; void* image = nullptr; float gamma = 0, delta = 0; };
  ImageGraph img_graph[2];   // sdstream_step_image: one captured graph per queue buffer

  // ssf
  uint8_t* ssf_buf[2] = {nullptr, nullptr};
  unsigned long long* ssf_sums = nullptr;  // device [4]
  unsigned long long* ssf_host = nullptr;  // pinned [4]
  long long ssf_n = 0;
  int ssf_ref = -1;
  uint64_t ssf_ref_norm = 0;
  // run statistics of the filter since the last reset (Sec. 3.4: the share of frames that still reach the U-Net)
  long long ssf_frames = 0, ssf_processed = 0, ssf_skip_run = 0, ssf_longest_skip_run = 0;

  // graph
  bool graph_enabled = true;
  hipStream_t cap_stream = nullptr;
  std::map<int, hipGraphExec_t> graphs;

  // profiling
  bool profiling = false;
  struct ProfRec { int cls; hipEvent_t a, b; double flops, bytes; int op; int N; };
  std::vector<ProfRec> prof_pending;
  sdstream_profile_entry prof[PC_COUNT];
};

namespace {

int fail(sdstream* h, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (h) h->err = buf; else g_create_error = buf;
  return code;
}

#define HIP_TRY(h, expr)                                                                       \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(h, SDSTREAM_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// ------------------------------------------------------------------------------------------------
// builder: walks the U-Net once, registering weights (manifest + device layout) and emitting ops
// ------------------------------------------------------------------------------------------------
struct Builder {
  sdstream& e;
  bool dry;  // first pass: sizes only (pointers are offsets from null)
  size_t wbytes = 0, pbytes = 0;
  int temb_dim;

  explicit Builder(sdstream& eng, bool dry_) : e(eng), dry(dry_) { temb_dim = 4 * eng.cfg.block_channels[0]; }

  // ---- weights
  size_t walloc(size_t bytes) {
    size_t off = wbytes;
    wbytes += (bytes + 255) & ~(size_t)255;
    return off;
  }
  size_t palloc(size_t bytes) {
    size_t off = pbytes;
    pbytes += (bytes + 255) & ~(size_t)255;
    return off;
  }
  void add_entry(const std::string& name, std::initializer_list<int> shape, int kind, int action, size_t dst_off, int O,
                 int I, int taps, int geglu) {
    Entry en;
    en.name = name;
    en.ndim = (int)shape.size();
    en.count = 1;
    int i = 0;
    for (int s : shape) { en.shape[i++] = s; en.count *= (size_t)s; }
    for (; i < 4; ++i) en.shape[i] = 1;
    en.kind = kind;
    en.action = action;
    en.dst_off = dst_off;
    en.O = O; en.I = I; en.taps = taps; en.geglu = geglu;
    if (dry) e.manifest.push_back(en);
  }
  size_t fvec_off(const std::string& name, int n, int kind) {
    size_t off = walloc((size_t)n * 4);
    add_entry(name, {n}, kind, LA_F32, off, n, 1, 1, 0);
    return off;
  }
  float* fvec(const std::string& name, int n, int kind) { return (float*)(e.weights + fvec_off(name, n, kind)); }
  // LayerNorm (scale at g_off, shift at b_off) folded into `count` stacked matrices of rows_each rows whose weight
  // entries are the manifest's entries [size - back, size - back + count)
  struct LnVec { size_t wsum, lnb; };
  LnVec fold_ln(int count, int rows_each, int back, size_t g_off, size_t b_off) {
    LnVec v;
    v.wsum = walloc((size_t)count * rows_each * 4);
    v.lnb = walloc((size_t)count * rows_each * 4);
    if (dry) {
      for (int j = 0; j < count; ++j) {
        Entry& en = e.manifest[e.manifest.size() - back + j];
        en.ln_fold = true;
        en.ln_g = g_off;
        en.ln_b = b_off;
        en.ln_wsum = v.wsum + (size_t)j * rows_each * 4;
        en.ln_lnb = v.lnb + (size_t)j * rows_each * 4;
      }
    }
    return v;
  }
  void* aalloc_bytes(size_t bytes_per_sample) {
    size_t off = e.act.alloc(bytes_per_sample);
    return e.act_base + off * (size_t)e.max_batch;
  }
  bool mfma_ok(int C1, int C2, int N, bool geglu) const {
    if (!e.use_mfma || !igemm_mfma_available()) return false;
    if (C1 % 32 || C2 % 32) return false;
    if (N % 16) return false;
    if (geglu && N % 128) return false;
    return true;
  }
  // a conv / linear weight in the activation dtype; `ksz` 1 or 3; canonical shape OIHW or [O,I]
  LinW matw(const std::string& name, int O, int I, int ksz, bool conv_shape, bool bias, bool geglu, int C1, int C2) {
    LinW w;
    int taps = ksz * ksz;
    w.N = O;
    w.K = I * taps;
    w.mfma = mfma_ok(C1, C2, O, geglu);
    w.w = walloc((size_t)O * w.K * e.elt);
    int blk = geglu ? (w.mfma ? 16 : 1) : 0;
    if (conv_shape)
      add_entry(name + ".w", {O, I, ksz, ksz}, 0, w.mfma ? LA_MFMA : LA_ROWMAJOR, w.w, O, I, taps, blk);
    else
      add_entry(name + ".w", {O, I}, 0, w.mfma ? LA_MFMA : LA_ROWMAJOR, w.w, O, I, taps, blk);
    if (bias) {
      w.b = walloc((size_t)O * 4);
      w.has_bias = true;
      add_entry(name + ".b", {O}, 1, geglu ? LA_BIAS_PERM : LA_F32, w.b, O, 1, 1, blk);
    }
    return w;
  }
  // several [C,I] matrices stacked along the output dimension (fused q/k/v), no bias
  LinW fused(const std::vector<std::string>& names, int C, int I) {
    LinW w;
    int n = (int)names.size();
    w.N = n * C;
    w.K = I;
    w.mfma = mfma_ok(I, 0, C, false);
    w.w = walloc((size_t)w.N * I * e.elt);
    for (int j = 0; j < n; ++j)
      add_entry(names[j] + ".w", {C, I}, 0, w.mfma ? LA_MFMA : LA_ROWMAJOR, w.w + (size_t)j * C * I * e.elt, C, I, 1, 0);
    return w;
  }
  // fp32 [O][I] matrix + bias for the time-embedding path
  LinW f32w(const std::string& name, int O, int I) {
    LinW w;
    w.N = O; w.K = I; w.mfma = false; w.has_bias = true;
    w.w = walloc((size_t)O * I * 4);
    add_entry(name + ".w", {O, I}, 0, LA_F32, w.w, O, I, 1, 0);
    w.b = walloc((size_t)O * 4);
    add_entry(name + ".b", {O}, 1, LA_F32, w.b, O, 1, 1, 0);
    return w;
  }

  // ---- activations
  void* aalloc(size_t elems_per_sample) {
    size_t off = e.act.alloc(elems_per_sample * e.elt);
    return e.act_base + off * (size_t)e.max_batch;
  }
  void afree(void* p) { e.act.release((size_t)((char*)p - e.act_base) / (size_t)e.max_batch); }

  // ---- ops
  bool norm_only_here = false;   // set around the emission of a layer that is the only reader of the norm before it
  void* conv(const void* s1, int C1, const void* s2, int C2, int Hin, int Win, int Hout, int Wout, int ks, int stride,
             int ups, const LinW& w, const float* rowbias, int rowbias_ld, const void* residual, int epi) {
    Op op{};
    op.kind = OP_IGEMM;
    op.mfma = w.mfma;
    op.cls = w.mfma ? PC_IGEMM_MFMA : PC_IGEMM_VALU;
    IgemmParams& g = op.g;
    g.src1 = s1; g.src2 = s2; g.C1 = C1; g.C2 = C2;
    g.Hin = Hin; g.Win = Win; g.Hout = Hout; g.Wout = Wout;
    g.ksize = ks; g.stride = stride; g.upsample = ups;
    g.N = w.N; g.K = ks * ks * (C1 + C2);
    g.W = e.weights + w.w;
    g.bias = w.has_bias ? (const float*)(e.weights + w.b) : nullptr;
    g.rowbias = rowbias; g.rowbias_ld = rowbias_ld;
    g.residual = residual;
    g.epilogue = epi;
    g.splitk = 1;
    op.ln_src_op = -1;
    op.xattn_site = -1;
    // the layer reads the output of the norm just emitted, and nothing else does (the caller says so by passing
    // norm_only_here): the norm may be applied to this layer's input rows on load instead (launch_op decides)
    if (norm_only_here && !s2 && !e.ops.empty() && e.ops.back().kind == OP_GN && e.ops.back().gn.out == s1 && w.mfma) {
      op.gn_in_plus1 = (int)e.ops.size();
      e.ops.back().gn_out_plus1 = (int)e.ops.size() + 1;
    }
    int Nout = epi == EPI_GEGLU ? w.N / 2 : w.N;
    g.out = aalloc((size_t)Hout * Wout * Nout);
    op.rows_per_sample = Hout * Wout;
    op.flops_per_row = 2.0 * Hout * Wout * (double)w.N * g.K;
    op.bytes_per_row = ((double)Hin * Win * (C1 + C2) + (double)Hout * Wout * Nout * (residual ? 2 : 1)) * e.elt;
    op.bytes_fixed = (double)w.N * g.K * e.elt;
    e.ops.push_back(op);
    return g.out;
  }
  void* gn(const void* s1, int C1, const void* s2, int C2, int HW, float eps, int silu, const float* gamma,
           const float* beta, float* stats) {
    Op op{};
    op.kind = OP_GN;
    op.cls = PC_GROUP_NORM;
    GroupNormParams& p = op.gn;
    p.src1 = s1; p.src2 = s2; p.C1 = C1; p.C2 = C2; p.HW = HW; p.groups = e.cfg.norm_groups;
    p.eps = eps; p.silu = silu; p.gamma = gamma; p.beta = beta; p.stats = stats;
    p.out = aalloc((size_t)HW * (C1 + C2));
    op.rows_per_sample = HW;
    op.bytes_per_row = 2.0 * HW * (C1 + C2) * e.elt;
    // a norm over the output of the layer just emitted: that layer's epilogue may leave the statistics (launch_op decides)
    if (!s2 && !e.ops.empty() && e.ops.back().kind == OP_IGEMM && e.ops.back().mfma && e.ops.back().g.out == s1 &&
        e.ops.back().xattn_site < 0) {
      op.gn_src_plus1 = (int)e.ops.size();
      e.ops.back().gn_dst_plus1 = (int)e.ops.size() + 1;
    }
    e.ops.push_back(op);
    return p.out;
  }
  void* ln(const void* src, int rows, int C, const float* gamma, const float* beta) {
    Op op{};
    op.kind = OP_LN;
    op.cls = PC_LAYER_NORM;
    LayerNormParams& p = op.ln;
    p.src = src; p.C = C; p.eps = 1e-5f; p.gamma = gamma; p.beta = beta;
    p.out = aalloc((size_t)rows * C);
    op.rows_per_sample = rows;
    op.bytes_per_row = 2.0 * rows * C * e.elt;
    e.ops.push_back(op);
    return p.out;
  }
  void* attn(const void* q, int ldq, const void* k, const void* v, int ldkv, int Sq, int Skv, int heads, int d,
             bool cached, size_t cache_stride_elems) {
    Op op{};
    op.kind = OP_ATTN;
    AttnParams& p = op.at;
    p.q = q; p.k = k; p.v = v; p.ldq = ldq; p.ldk = ldkv; p.ldv = ldkv; p.ldo = heads * d;
    p.Sq = Sq; p.Skv = Skv; p.heads = heads; p.d = d;
    p.scale = (float)(1.0 / sqrt((double)d));
    if (cached) {
      p.kv_select = (const int*)(e.persist + e.off_sel_zero);  // patched per launch
      p.kv_select_stride = (long long)cache_stride_elems;
      p.kv_sample_stride = 0;
    } else {
      p.kv_select = nullptr;
      p.kv_sample_stride = (long long)Skv * ldkv;
    }
    p.out = aalloc((size_t)Sq * heads * d);
    op.mfma = e.use_mfma && attention_mfma_supported(p);
    op.cls = op.mfma ? PC_ATTN_MFMA : PC_ATTN_VALU;
    op.rows_per_sample = Sq;
    // with cross-frame attention a self-attention row sees the keys of all n rows of its stream batch
    const double kv_rows = (!cached && e.cfg.cross_frame && e.cfg.n_denoise > 1) ? e.cfg.n_denoise : 1;
    op.flops_per_row = 4.0 * Sq * (double)Skv * kv_rows * d * heads;
    op.bytes_per_row = (2.0 * Sq * heads * d + (cached ? 0.0 : 2.0 * Skv * heads * d)) * e.elt;
    e.ops.push_back(op);
    return p.out;
  }

  // ---- blocks
  struct ResW {
    float *g1, *b1, *g2, *b2;
    LinW c1, c2, skip, temb;
    bool has_skip, fused_skip;
    size_t rowbias;  // persist offset, [max_batch][cout] fp32
  };
  ResW res_weights(const std::string& p, int c1in, int c2in, int cout) {
    ResW r;
    int cin = c1in + c2in;
    r.g1 = fvec(p + ".norm1.g", cin, 2);
    r.b1 = fvec(p + ".norm1.b", cin, 3);
    r.c1 = matw(p + ".conv1", cout, cin, 3, true, true, false, cin, 0);
    r.temb = f32w(p + ".temb", cout, temb_dim);
    r.g2 = fvec(p + ".norm2.g", cout, 2);
    r.b2 = fvec(p + ".norm2.b", cout, 3);
    r.has_skip = cin != cout;
    // With the direct-to-LDS matrix-core kernels the 1x1 skip convolution is summed into conv2 as a second K segment:
    // one packed matrix [conv2 taps | skip], one bias vector (the sum of the two), one launch instead of two.
    r.fused_skip = r.has_skip && mfma_ok(cout, 0, cout, false) && cout % 64 == 0 && c1in % 64 == 0 && c2in % 64 == 0;
#ifdef SDSTREAM_DEVHOOKS
    if (getenv("SDSTREAM_NO_SKIPFUSE")) r.fused_skip = false;
#endif
    if (r.fused_skip) {
      const int k1 = 9 * cout, kt = k1 + cin;
      LinW w;
      w.N = cout; w.K = kt; w.mfma = true; w.has_bias = true;
      w.w = walloc((size_t)cout * kt * e.elt);
      add_entry(p + ".conv2.w", {cout, cout, 3, 3}, 0, LA_MFMA, w.w, cout, cout, 9, 0);
      if (dry) { e.manifest.back().pk_total = kt / 32; e.manifest.back().pk_off = 0; }
      const size_t b2 = walloc((size_t)cout * 4);
      add_entry(p + ".conv2.b", {cout}, 1, LA_F32, b2, cout, 1, 1, 0);
      add_entry(p + ".skip.w", {cout, cin, 1, 1}, 0, LA_MFMA, w.w, cout, cin, 1, 0);
      if (dry) { e.manifest.back().pk_total = kt / 32; e.manifest.back().pk_off = k1 / 32; }
      const size_t bs = walloc((size_t)cout * 4);
      add_entry(p + ".skip.b", {cout}, 1, LA_F32, bs, cout, 1, 1, 0);
      w.b = walloc((size_t)cout * 4);   // conv2.b + skip.b
      if (dry) {
        BiasFix f1{w.b, b2, cout, true}, f2{w.b, bs, cout, false};
        e.bias_fixes.push_back(f1);
        e.bias_fixes.push_back(f2);
      }
      r.c2 = w;
    } else {
      r.c2 = matw(p + ".conv2", cout, cout, 3, true, true, false, cout, 0);
      if (r.has_skip) r.skip = matw(p + ".skip", cout, cin, 1, true, true, false, c1in, c2in);
    }
    r.rowbias = palloc((size_t)e.max_batch * cout * 4);
    return r;
  }

  float* stats_buf() { return (float*)(e.persist + stats_off); }
  size_t stats_off = 0;

  // x = concat(x1, x2) (x2 may be null); consumes nothing, returns a new buffer
  void* res_block(const std::string& name, const void* x1, int c1in, const void* x2, int c2in, int cout, int H, int W) {
    ResW r = res_weights(name, c1in, c2in, cout);
    int HW = H * W;
    // time-embedding bias of this block: Linear(SiLU(temb)) per batch row
    {
      Op op{};
      op.kind = OP_IGEMM;
      op.cls = PC_IGEMM_VALU;
      IgemmParams& g = op.g;
      g.src1 = e.persist + e.off_h2; g.C1 = temb_dim; g.C2 = 0;
      g.Hin = g.Win = g.Hout = g.Wout = 1; g.ksize = 1; g.stride = 1;
      g.N = cout; g.K = temb_dim;
      g.W = e.weights + r.temb.w;
      g.bias = (const float*)(e.weights + r.temb.b);
      g.out = e.persist + r.rowbias;
      g.splitk = 1;
      op.rows_per_sample = 1;
      e.temb_ops.push_back(op);
    }
    void* t1 = gn(x1, c1in, x2, c2in, HW, 1e-5f, 1, r.g1, r.b1, stats_buf());
    void* t2 = conv(t1, c1in + c2in, nullptr, 0, H, W, H, W, 3, 1, 0, r.c1, (const float*)(e.persist + r.rowbias), cout,
                    nullptr, EPI_NONE);
    afree(t1);
    void* t3 = gn(t2, cout, nullptr, 0, HW, 1e-5f, 1, r.g2, r.b2, stats_buf());
    afree(t2);
    const void* skip = x1;
    void* sk = nullptr;
    if (r.fused_skip) {
      skip = nullptr;
    } else if (r.has_skip) {
      sk = conv(x1, c1in, x2, c2in, H, W, H, W, 1, 1, 0, r.skip, nullptr, 0, nullptr, EPI_NONE);
      skip = sk;
    }
    void* out = conv(t3, cout, nullptr, 0, H, W, H, W, 3, 1, 0, r.c2, nullptr, 0, skip, EPI_NONE);
    if (r.fused_skip) {   // second K segment: the block's input through the 1x1 weights
      IgemmParams& g = e.ops.back().g;
      g.src3 = x1; g.C3 = c1in;
      g.src4 = x2; g.C4 = c2in;
      g.K += c1in + c2in;
      e.ops.back().flops_per_row += 2.0 * HW * (double)cout * (c1in + c2in);
      e.ops.back().bytes_per_row += (double)HW * (c1in + c2in) * e.elt;
      e.ops.back().bytes_fixed += (double)cout * (c1in + c2in) * e.elt;
    }
    afree(t3);
    if (sk) afree(sk);
    return out;
  }

  void* transformer(const std::string& p, void* x, int C, int H, int W) {
    const int HW = H * W, L = e.cfg.context_len, D = e.cfg.context_dim;
    const int heads = e.cfg.num_heads > 0 ? e.cfg.num_heads : C / e.cfg.head_dim;
    const int d = C / heads;
    float* gng = fvec(p + ".norm.g", C, 2);
    float* gnb = fvec(p + ".norm.b", C, 3);
    LinW pin = matw(p + ".proj_in", C, C, 1, false, true, false, C, 0);
    bool fold = mfma_ok(C, 0, C, false) && mfma_ok(C, 0, 8 * C, true) && (C + 159) / 160 <= LN_MAX_PARTS;
#ifdef SDSTREAM_DEVHOOKS
    if (getenv("SDSTREAM_NO_LNFOLD")) fold = false;
#endif
    const size_t l1g_off = fvec_off(p + ".ln1.g", C, 2), l1b_off = fvec_off(p + ".ln1.b", C, 3);
    float* l1g = (float*)(e.weights + l1g_off);
    float* l1b = (float*)(e.weights + l1b_off);
    LinW qkv = fused({p + ".attn1.q", p + ".attn1.k", p + ".attn1.v"}, C, C);
    LnVec v1{}, v2{}, v3{};
    if (fold) v1 = fold_ln(3, C, 3, l1g_off, l1b_off);
    LinW o1 = matw(p + ".attn1.o", C, C, 1, false, true, false, C, 0);
    const size_t l2g_off = fvec_off(p + ".ln2.g", C, 2), l2b_off = fvec_off(p + ".ln2.b", C, 3);
    float* l2g = (float*)(e.weights + l2g_off);
    float* l2b = (float*)(e.weights + l2b_off);
    LinW q2 = fused({p + ".attn2.q"}, C, C);
    if (fold) v2 = fold_ln(1, C, 1, l2g_off, l2b_off);
    // cross-attention folded into two GEMMs: prompt length padded to the softmax segment of the GEMM epilogue
    const int Lp = L <= 16 ? 16 : (L > 64 && L <= 80 ? 80 : 0);
    const int Npad = (heads * Lp + 63) / 64 * 64;
    bool xfold = fold && Lp > 0 && heads * d == C && mfma_ok(C, 0, Npad, false) && mfma_ok(Npad, 0, C, false);
#ifdef SDSTREAM_DEVHOOKS
    if (getenv("SDSTREAM_NO_XFOLD")) xfold = false;
#endif
    size_t wq_raw = 0, wo_raw = 0;
    if (xfold) {
      wq_raw = walloc((size_t)C * C * 4);
      if (dry) { e.manifest.back().raw_copy = true; e.manifest.back().raw_off = wq_raw; }
    }
    KVSite site;
    site.w = fused({p + ".attn2.k", p + ".attn2.v"}, C, D);
    site.C = C;
    site.cache = palloc((size_t)2 * L * 2 * C * e.elt);
    e.kv_sites.push_back(site);
    LinW o2 = matw(p + ".attn2.o", C, C, 1, false, true, false, C, 0);
    if (xfold) {
      wo_raw = walloc((size_t)C * C * 4);
      if (dry) { Entry& en = e.manifest[e.manifest.size() - 2]; en.raw_copy = true; en.raw_off = wo_raw; }   // (attn2.o.w, attn2.o.b)
      KVSite& st = e.kv_sites.back();
      st.xfold = true;
      st.heads = heads; st.d = d; st.Lp = Lp; st.Npad = Npad;
      st.wq_raw = wq_raw; st.wo_raw = wo_raw; st.ln_g = l2g_off; st.ln_b = l2b_off;
      st.mat_stride = ((size_t)Npad * C * e.elt + 255) & ~(size_t)255;
      st.vec_stride = ((size_t)Npad * 4 + 255) & ~(size_t)255;
      st.qk = palloc(2 * st.mat_stride);
      st.vo = palloc(2 * st.mat_stride);
      st.wsum = palloc(2 * st.vec_stride);
      st.lnb = palloc(2 * st.vec_stride);
      if ((size_t)Npad * C > e.xraw_floats) e.xraw_floats = (size_t)Npad * C;
    }
    const size_t l3g_off = fvec_off(p + ".ln3.g", C, 2), l3b_off = fvec_off(p + ".ln3.b", C, 3);
    float* l3g = (float*)(e.weights + l3g_off);
    float* l3b = (float*)(e.weights + l3b_off);
    LinW ffi = matw(p + ".ff.in", 8 * C, C, 1, false, true, true, C, 0);
    if (fold) {
      v3 = fold_ln(1, 8 * C, 2, l3g_off, l3b_off);   // (entries: ff.in.w, ff.in.b)
      if (dry) e.bias_fixes.push_back(BiasFix{v3.lnb, ffi.b, 8 * C});
    }
    LinW ffo = matw(p + ".ff.out", C, 4 * C, 1, false, true, false, 4 * C, 0);
    LinW pout = matw(p + ".proj_out", C, C, 1, false, true, false, C, 0);

    void* t = gn(x, C, nullptr, 0, HW, 1e-6f, 0, gng, gnb, stats_buf());
    norm_only_here = true;   // (t is read by proj_in alone; x stays allocated as the block's residual)
    void* h = conv(t, C, nullptr, 0, H, W, H, W, 1, 1, 0, pin, nullptr, 0, nullptr, EPI_NONE);
    norm_only_here = false;
    // With the matrix-core kernels the three LayerNorms are folded into the layers that consume them: the producer of
    // the rows (proj_in, the two attention output projections) leaves per-row partial sums, the consumer (q/k/v, the
    // cross-attention q, the feed-forward input) multiplies the raw rows by weights pre-scaled with the norm's scale.
    const size_t stat_bytes = (size_t)HW * ((C + 63) / 64) * 2 * sizeof(float);
    // (the statistics buffer is taken while the inputs of the op are still allocated: it must not alias them)
    auto emit_stats = [&]() {   // the op just emitted also writes row statistics; returns (buffer, op index)
      void* sb = aalloc_bytes(stat_bytes);
      e.ops.back().g.stats_out = (float*)sb;
      e.ops.back().g.no_splitk = 1;
      return std::make_pair(sb, (int)e.ops.size() - 1);
    };
    auto read_stats = [&](std::pair<void*, int> st, const LnVec& v) {   // the op just emitted has the LayerNorm folded in
      IgemmParams& g = e.ops.back().g;
      g.ln_stats = (const float*)st.first;
      g.ln_wsum = (const float*)(e.weights + v.wsum);
      g.bias = (const float*)(e.weights + v.lnb);
      g.ln_eps = 1e-5f;
      g.no_splitk = 1;
      e.ops.back().ln_src_op = st.second;
    };
    if (fold) {
      auto st1 = emit_stats();
      afree(t);
      void* qk = conv(h, C, nullptr, 0, H, W, H, W, 1, 1, 0, qkv, nullptr, 0, nullptr, EPI_NONE);
      read_stats(st1, v1);
      afree(st1.first);
      char* qkb = (char*)qk;
      void* a1 = attn(qkb, 3 * C, qkb + (size_t)C * e.elt, qkb + (size_t)2 * C * e.elt, 3 * C, HW, HW, heads, d, false, 0);
      afree(qk);
      void* h2 = conv(a1, C, nullptr, 0, H, W, H, W, 1, 1, 0, o1, nullptr, 0, h, EPI_NONE);
      auto st2 = emit_stats();
      afree(a1);
      afree(h);
      void* h3;
      std::pair<void*, int> st3;
      if (xfold) {
        const KVSite& ks = e.kv_sites.back();
        const int site_index = (int)e.kv_sites.size() - 1;
        const double attn_flops = 4.0 * HW * (double)L * d * heads, lin_flops = 2.0 * HW * (double)C * C;
        LinW wa;   // rows x QK^T, per-head softmax in the epilogue
        wa.N = Npad; wa.K = C; wa.mfma = true;
        void* pr = conv(h2, C, nullptr, 0, H, W, H, W, 1, 1, 0, wa, nullptr, 0, nullptr, EPI_SOFTMAX);
        {
          Op& op = e.ops.back();
          op.g.W = e.persist + ks.qk;
          op.g.ln_stats = (const float*)st2.first;
          op.g.ln_wsum = (const float*)(e.persist + ks.wsum);
          op.g.bias = (const float*)(e.persist + ks.lnb);
          op.g.ln_eps = 1e-5f;
          op.g.no_splitk = 1;
          op.g.sm_lp = Lp; op.g.sm_len = L; op.g.sm_cols = heads * Lp;
          op.ln_src_op = st2.second;
          op.xattn_site = site_index;
          op.xattn_role = 1;
          op.flops_per_row = lin_flops + attn_flops / 2;   // algorithmic work of what it replaces: q projection, scores
          op.bytes_fixed = (double)Npad * C * e.elt;
        }
        afree(st2.first);
        LinW wb;   // probabilities x VO^T + bias + residual
        wb.N = C; wb.K = Npad; wb.mfma = true; wb.has_bias = true; wb.b = o2.b;
        h3 = conv(pr, Npad, nullptr, 0, H, W, H, W, 1, 1, 0, wb, nullptr, 0, h2, EPI_NONE);
        {
          Op& op = e.ops.back();
          op.g.W = e.persist + ks.vo;
          op.xattn_site = site_index;
          op.xattn_role = 2;
          op.flops_per_row = lin_flops + attn_flops / 2;   // output projection, probabilities x values
          op.bytes_fixed = (double)Npad * C * e.elt;
        }
        st3 = emit_stats();
        afree(pr);
        afree(h2);
      } else {
      void* qc = conv(h2, C, nullptr, 0, H, W, H, W, 1, 1, 0, q2, nullptr, 0, nullptr, EPI_NONE);
      read_stats(st2, v2);
      afree(st2.first);
      char* cache = e.persist + site.cache;
      void* a2 = attn(qc, C, cache, cache + (size_t)C * e.elt, 2 * C, HW, L, heads, d, true, (size_t)L * 2 * C);
      afree(qc);
      h3 = conv(a2, C, nullptr, 0, H, W, H, W, 1, 1, 0, o2, nullptr, 0, h2, EPI_NONE);
      st3 = emit_stats();
      afree(a2);
      afree(h2);
      }
      void* u = conv(h3, C, nullptr, 0, H, W, H, W, 1, 1, 0, ffi, nullptr, 0, nullptr, EPI_GEGLU);
      read_stats(st3, v3);
      afree(st3.first);
      void* h4 = conv(u, 4 * C, nullptr, 0, H, W, H, W, 1, 1, 0, ffo, nullptr, 0, h3, EPI_NONE);
      afree(u);
      afree(h3);
      void* out = conv(h4, C, nullptr, 0, H, W, H, W, 1, 1, 0, pout, nullptr, 0, x, EPI_NONE);
      afree(h4);
      return out;
    }
    afree(t);
    // self-attention
    void* n1 = ln(h, HW, C, l1g, l1b);
    void* qk = conv(n1, C, nullptr, 0, H, W, H, W, 1, 1, 0, qkv, nullptr, 0, nullptr, EPI_NONE);
    afree(n1);
    char* qkb = (char*)qk;
    void* a1 = attn(qkb, 3 * C, qkb + (size_t)C * e.elt, qkb + (size_t)2 * C * e.elt, 3 * C, HW, HW, heads, d, false, 0);
    afree(qk);
    void* h2 = conv(a1, C, nullptr, 0, H, W, H, W, 1, 1, 0, o1, nullptr, 0, h, EPI_NONE);
    afree(a1);
    afree(h);
    // cross-attention with the cached K/V of the prompt
    void* n2 = ln(h2, HW, C, l2g, l2b);
    void* qc = conv(n2, C, nullptr, 0, H, W, H, W, 1, 1, 0, q2, nullptr, 0, nullptr, EPI_NONE);
    afree(n2);
    char* cache = e.persist + site.cache;
    void* a2 = attn(qc, C, cache, cache + (size_t)C * e.elt, 2 * C, HW, L, heads, d, true, (size_t)L * 2 * C);
    afree(qc);
    void* h3 = conv(a2, C, nullptr, 0, H, W, H, W, 1, 1, 0, o2, nullptr, 0, h2, EPI_NONE);
    afree(a2);
    afree(h2);
    // GEGLU feed-forward
    void* n3 = ln(h3, HW, C, l3g, l3b);
    void* u = conv(n3, C, nullptr, 0, H, W, H, W, 1, 1, 0, ffi, nullptr, 0, nullptr, EPI_GEGLU);
    afree(n3);
    void* h4 = conv(u, 4 * C, nullptr, 0, H, W, H, W, 1, 1, 0, ffo, nullptr, 0, h3, EPI_NONE);
    afree(u);
    afree(h3);
    void* out = conv(h4, C, nullptr, 0, H, W, H, W, 1, 1, 0, pout, nullptr, 0, x, EPI_NONE);
    afree(h4);
    return out;
  }

  void build() {
    const sdstream_config& c = e.cfg;
    const int nl = c.n_levels, c0 = c.block_channels[0];
    int H = c.latent_h, W = c.latent_w;
    e.ops.clear();
    e.temb_ops.clear();
    e.kv_sites.clear();
    e.act = PlanAllocator();

    // persistent small buffers
    e.off_tdev = palloc((size_t)e.max_batch * 4);
    e.off_emb = palloc((size_t)e.max_batch * c0 * 4);
    e.off_h1 = palloc((size_t)e.max_batch * temb_dim * 4);
    e.off_h2 = palloc((size_t)e.max_batch * temb_dim * 4);
    e.off_ctxT = palloc((size_t)2 * c.context_len * c.context_dim * e.elt);
    e.off_sel_zero = palloc((size_t)e.max_batch * 4);
    e.off_sel_step = palloc((size_t)e.max_batch * 4);
    stats_off = palloc((size_t)e.max_batch * GN_MAX_SPLIT * c.norm_groups * 2 * 4);
    const size_t rows_state = (size_t)c.n_streams * c.n_denoise;
    for (int i = 0; i < 2; ++i) {
      e.off_x[i] = palloc((size_t)e.max_batch * e.E * 4);
      e.off_r[i] = palloc(rows_state * e.E * 4);
    }
    e.off_eps = palloc((size_t)e.max_batch * e.E * 4);
    e.off_noise = palloc(rows_state * e.E * 4);
    e.off_ab = palloc((size_t)4 * c.n_denoise * 4);   // a, b, c_skip, c_out per slot
    e.off_unet_x = palloc((size_t)e.max_batch * e.E * 4);
    e.off_splitk = palloc(kSplitKWorkspaceFloats * 4);
    e.off_zeros = palloc(256);
    e.xraw_floats = 0;
    if (c.image_width > 0) {
      e.off_img_lat_in = palloc((size_t)c.n_streams * e.E * 4);
      e.off_img_lat_out = palloc((size_t)c.n_streams * e.E * 4);
    }

    // time embedding MLP (float32)
    LinW t1 = f32w("time.lin1", temb_dim, c0);
    LinW t2 = f32w("time.lin2", temb_dim, temb_dim);
    for (int j = 0; j < 2; ++j) {
      Op op{};
      op.kind = OP_IGEMM;
      op.cls = PC_IGEMM_VALU;
      IgemmParams& g = op.g;
      g.src1 = e.persist + (j == 0 ? e.off_emb : e.off_h1);
      g.C1 = j == 0 ? c0 : temb_dim;
      g.Hin = g.Win = g.Hout = g.Wout = 1; g.ksize = 1; g.stride = 1;
      g.N = temb_dim; g.K = g.C1;
      const LinW& w = j == 0 ? t1 : t2;
      g.W = e.weights + w.w;
      g.bias = (const float*)(e.weights + w.b);
      g.out = e.persist + (j == 0 ? e.off_h1 : e.off_h2);
      g.epilogue = EPI_SILU;  // every consumer of temb applies SiLU first
      g.splitk = 1;
      op.rows_per_sample = 1;
      e.temb_ops.push_back(op);
    }

    // conv_in (fp32 weights, canonical OIHW)
    size_t ciw = walloc((size_t)c0 * c.in_channels * 9 * 4);
    add_entry("conv_in.w", {c0, c.in_channels, 3, 3}, 0, LA_F32, ciw, c0, c.in_channels, 9, 0);
    float* cib = fvec("conv_in.b", c0, 1);
    void* h;
    {
      Op op{};
      op.kind = OP_CONV_IN;
      op.cls = PC_CONV_IN;
      op.cw_f32 = (const float*)(e.weights + ciw);
      op.cb = cib;
      op.cH = H; op.cW = W; op.cCin = c.in_channels; op.cC0 = c0; op.cflags = 0;
      op.cout_ = aalloc((size_t)H * W * c0);
      op.rows_per_sample = H * W;
      op.flops_per_row = 2.0 * H * W * c0 * c.in_channels * 9;
      op.bytes_per_row = (double)H * W * (c.in_channels * 4 + c0 * e.elt);
      e.ops.push_back(op);
      h = op.cout_;
    }
    std::vector<std::pair<void*, int>> skips;
    skips.push_back({h, c0});
    int ch = c0;
    for (int l = 0; l < nl; ++l) {
      const int cl = c.block_channels[l];
      const bool at = (c.attn_level_mask >> l) & 1;
      for (int j = 0; j < c.layers_per_block; ++j) {
        std::string p = "down." + std::to_string(l);
        void* r = res_block(p + ".res." + std::to_string(j), h, ch, nullptr, 0, cl, H, W);
        ch = cl;
        if (at) {
          void* t = transformer(p + ".attn." + std::to_string(j), r, ch, H, W);
          afree(r);
          r = t;
        }
        h = r;
        skips.push_back({h, ch});
      }
      if (l != nl - 1) {
        LinW dw = matw("down." + std::to_string(l) + ".downsample", ch, ch, 3, true, true, false, ch, 0);
        int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
        h = conv(h, ch, nullptr, 0, H, W, Ho, Wo, 3, 2, 0, dw, nullptr, 0, nullptr, EPI_NONE);
        H = Ho; W = Wo;
        skips.push_back({h, ch});
      }
    }
    {
      void* r = res_block("mid.res.0", h, ch, nullptr, 0, ch, H, W);
      if (c.mid_attention) {
        void* t = transformer("mid.attn", r, ch, H, W);
        afree(r);
        r = t;
      }
      h = res_block("mid.res.1", r, ch, nullptr, 0, ch, H, W);
      afree(r);
    }
    // (the last skip entry is the tensor the middle block started from; it is still needed by the up path)
    bool h_owned = true;
    for (int l = nl - 1; l >= 0; --l) {
      const int cl = c.block_channels[l];
      const bool at = (c.attn_level_mask >> l) & 1;
      for (int j = 0; j < c.layers_per_block + 1; ++j) {
        std::string p = "up." + std::to_string(l);
        auto sk = skips.back();
        skips.pop_back();
        void* r = res_block(p + ".res." + std::to_string(j), h, ch, sk.first, sk.second, cl, H, W);
        if (h_owned) afree(h);
        afree(sk.first);
        ch = cl;
        if (at) {
          void* t = transformer(p + ".attn." + std::to_string(j), r, ch, H, W);
          afree(r);
          r = t;
        }
        h = r;
        h_owned = true;
      }
      if (l != 0) {
        LinW uw = matw("up." + std::to_string(l) + ".upsample", ch, ch, 3, true, true, false, ch, 0);
        void* u = conv(h, ch, nullptr, 0, H, W, 2 * H, 2 * W, 3, 1, 1, uw, nullptr, 0, nullptr, EPI_NONE);
        afree(h);
        h = u;
        H *= 2; W *= 2;
      }
    }
    float* og = fvec("out.norm.g", ch, 2);
    float* ob = fvec("out.norm.b", ch, 3);
    void* t = gn(h, ch, nullptr, 0, H * W, 1e-5f, 1, og, ob, stats_buf());
    afree(h);
    // conv_out: T [Cout][9][C0]
    size_t cow = walloc((size_t)c.in_channels * 9 * ch * e.elt);
    add_entry("conv_out.w", {c.in_channels, ch, 3, 3}, 0, LA_ROWMAJOR, cow, c.in_channels, ch, 9, 0);
    float* cob = fvec("conv_out.b", c.in_channels, 1);
    {
      Op op{};
      op.kind = OP_CONV_OUT;
      op.cls = PC_CONV_OUT;
      op.cin = t;
      op.cw = e.weights + cow;
      op.cb = cob;
      op.cH = H; op.cW = W; op.cCin = c.in_channels; op.cC0 = ch; op.cflags = 0;
      op.rows_per_sample = H * W;
      op.flops_per_row = 2.0 * H * W * c.in_channels * ch * 9;
      op.bytes_per_row = (double)H * W * (c.in_channels * 4 + ch * e.elt);
      e.ops.push_back(op);
    }
    afree(t);
    e.off_xraw = palloc((e.xraw_floats ? e.xraw_floats : 64) * 4);
    e.flops_per_row = 0;
    for (const Op& op : e.ops) e.flops_per_row += op.flops_per_row;
  }
};

// ------------------------------------------------------------------------------------------------
// the latent <-> image stage: a tiny convolutional autoencoder of one width w around the U-Net
//   Block(x) = ReLU(conv_c(ReLU(conv_b(ReLU(conv_a(x))))) + x)
//   encoder : u8 image / 255 -> conv(3 -> w) -> Block -> 3 x [conv stride 2 (no bias) -> 3 Blocks] -> conv(w -> C)
//   decoder : 3 tanh(latent / 3) -> ReLU(conv(C -> w)) -> 3 x [3 Blocks -> nearest 2x -> conv (no bias)] -> Block
//             -> conv(w -> 3) -> clamp [0,1]
// (all convolutions 3x3, pad 1).  The paper's appendix only names its autoencoder; these layers are this library's.
// ------------------------------------------------------------------------------------------------
struct ImageBuilder {
  sdstream& e;
  bool dry;
  size_t wbytes = 0;
  std::vector<Op>* ops = nullptr;
  explicit ImageBuilder(sdstream& eng, bool dry_) : e(eng), dry(dry_) {}

  size_t walloc(size_t bytes) {
    size_t off = wbytes;
    wbytes += (bytes + 255) & ~(size_t)255;
    return off;
  }
  void add_entry(const std::string& name, std::initializer_list<int> shape, int kind, int action, size_t dst_off, int O,
                 int I, int taps) {
    Entry en;
    en.name = name;
    en.ndim = (int)shape.size();
    en.count = 1;
    int i = 0;
    for (int s : shape) { en.shape[i++] = s; en.count *= (size_t)s; }
    for (; i < 4; ++i) en.shape[i] = 1;
    en.kind = kind; en.action = action; en.dst_off = dst_off;
    en.O = O; en.I = I; en.taps = taps; en.geglu = 0;
    if (dry) e.img_manifest.push_back(en);
  }
  float* bias(const std::string& name, int n) {
    size_t off = walloc((size_t)n * 4);
    add_entry(name, {n}, 1, LA_F32, off, n, 1, 1);
    return (float*)(e.img_weights + off);
  }
  struct CW { const void* w; const float* b; bool mfma; };
  CW convw(const std::string& name, int O, int I, bool with_bias) {   // w -> w convolutions in the activation type
    CW c;
    c.mfma = e.use_mfma && igemm_mfma_available() && I % 32 == 0 && O % 16 == 0;
    size_t off = walloc((size_t)O * I * 9 * e.elt);
    add_entry(name + ".w", {O, I, 3, 3}, 0, c.mfma ? LA_MFMA : LA_ROWMAJOR, off, O, I, 9);
    c.w = e.img_weights + off;
    c.b = with_bias ? bias(name + ".b", O) : nullptr;
    return c;
  }
  void* aalloc(size_t elems) {
    size_t off = e.img_act.alloc(elems * e.elt);
    return e.img_act_base + off * (size_t)e.cfg.n_streams;
  }
  void afree(void* p) { e.img_act.release((size_t)((char*)p - e.img_act_base) / (size_t)e.cfg.n_streams); }

  void* conv(const void* src, int C, int Hin, int Win, int Hout, int Wout, int stride, int ups, const CW& w,
             const void* residual, int epi) {
    Op op{};
    op.kind = OP_IGEMM;
    op.mfma = w.mfma;
    op.cls = w.mfma ? PC_IGEMM_MFMA : PC_IGEMM_VALU;
    op.ln_src_op = -1;
    op.xattn_site = -1;
    IgemmParams& g = op.g;
    g.src1 = src; g.C1 = C; g.C2 = 0;
    g.Hin = Hin; g.Win = Win; g.Hout = Hout; g.Wout = Wout;
    g.ksize = 3; g.stride = stride; g.upsample = ups;
    g.N = C; g.K = 9 * C;
    g.W = w.w; g.bias = w.b;
    g.residual = residual;
    g.epilogue = epi;
    g.splitk = 1;
    g.out = aalloc((size_t)Hout * Wout * C);
    op.rows_per_sample = Hout * Wout;
    op.flops_per_row = 2.0 * Hout * Wout * (double)C * g.K;
    ops->push_back(op);
    return g.out;
  }
  void* block(const std::string& p, void* x, int C, int H, int W) {
    CW a = convw(p + ".a", C, C, true), b = convw(p + ".b", C, C, true), c = convw(p + ".c", C, C, true);
    void* t1 = conv(x, C, H, W, H, W, 1, 0, a, nullptr, EPI_RELU);
    void* t2 = conv(t1, C, H, W, H, W, 1, 0, b, nullptr, EPI_RELU);
    afree(t1);
    void* out = conv(t2, C, H, W, H, W, 1, 0, c, x, EPI_RELU);   // ReLU(conv_c(.) + x)
    afree(t2);
    afree(x);
    return out;
  }
  void build() {
    const sdstream_config& c = e.cfg;
    const int w = c.image_width, lc = c.in_channels;
    int H = c.latent_h * 8, W = c.latent_w * 8;
    e.img_enc_ops.clear();
    e.img_dec_ops.clear();
    e.img_act = PlanAllocator();
    // ---- encoder
    ops = &e.img_enc_ops;
    void* x;
    {
      size_t woff = walloc((size_t)w * 27 * 4);
      add_entry("enc.in.w", {w, 3, 3, 3}, 0, LA_F32, woff, w, 3, 9);
      Op op{};
      op.kind = OP_IMAGE_IN;
      op.cls = PC_CONV_IN;
      op.cw_f32 = (const float*)(e.img_weights + woff);
      op.cb = bias("enc.in.b", w);
      op.cH = H; op.cW = W; op.cCin = 3; op.cC0 = w;
      op.cout_ = aalloc((size_t)H * W * w);
      op.rows_per_sample = H * W;
      ops->push_back(op);
      x = op.cout_;
    }
    x = block("enc.0.block.0", x, w, H, W);
    for (int s = 1; s <= 3; ++s) {
      CW d = convw("enc." + std::to_string(s) + ".down", w, w, false);
      void* y = conv(x, w, H, W, H / 2, W / 2, 2, 0, d, nullptr, EPI_NONE);
      afree(x);
      x = y;
      H /= 2; W /= 2;
      for (int j = 0; j < 3; ++j) x = block("enc." + std::to_string(s) + ".block." + std::to_string(j), x, w, H, W);
    }
    {
      size_t woff = walloc((size_t)lc * 9 * w * e.elt);
      add_entry("enc.out.w", {lc, w, 3, 3}, 0, LA_ROWMAJOR, woff, lc, w, 9);
      Op op{};
      op.kind = OP_CONV_OUT;
      op.cls = PC_CONV_OUT;
      op.cin = x;
      op.cw = e.img_weights + woff;
      op.cb = bias("enc.out.b", lc);
      op.cH = H; op.cW = W; op.cCin = lc; op.cC0 = w;
      op.rows_per_sample = H * W;
      ops->push_back(op);   // cout_ (the latent) is set per call
    }
    afree(x);
    // ---- decoder
    ops = &e.img_dec_ops;
    {
      size_t woff = walloc((size_t)w * lc * 9 * 4);
      add_entry("dec.in.w", {w, lc, 3, 3}, 0, LA_F32, woff, w, lc, 9);
      Op op{};
      op.kind = OP_CONV_IN;
      op.cls = PC_CONV_IN;
      op.cw_f32 = (const float*)(e.img_weights + woff);
      op.cb = bias("dec.in.b", w);
      op.cH = H; op.cW = W; op.cCin = lc; op.cC0 = w; op.cflags = CONV_IN_SQUASH | CONV_IN_RELU;
      op.cout_ = aalloc((size_t)H * W * w);
      op.rows_per_sample = H * W;
      ops->push_back(op);   // cin (the latent) is set per call
      x = op.cout_;
    }
    for (int s = 0; s < 3; ++s) {
      for (int j = 0; j < 3; ++j) x = block("dec." + std::to_string(s) + ".block." + std::to_string(j), x, w, H, W);
      CW u = convw("dec." + std::to_string(s) + ".up", w, w, false);
      void* y = conv(x, w, H, W, 2 * H, 2 * W, 1, 1, u, nullptr, EPI_NONE);
      afree(x);
      x = y;
      H *= 2; W *= 2;
    }
    x = block("dec.3.block.0", x, w, H, W);
    {
      size_t woff = walloc((size_t)3 * 9 * w * e.elt);
      add_entry("dec.out.w", {3, w, 3, 3}, 0, LA_ROWMAJOR, woff, 3, w, 9);
      Op op{};
      op.kind = OP_IMAGE_OUT;
      op.cls = PC_CONV_OUT;
      op.cin = x;
      op.cw = e.img_weights + woff;
      op.cb = bias("dec.out.b", 3);
      op.cH = H; op.cW = W; op.cCin = 3; op.cC0 = w;
      op.rows_per_sample = H * W;
      ops->push_back(op);   // img_f32 / img_u8 are set per call
    }
    afree(x);
  }
};

int validate(const sdstream_config& c, std::string& why) {
  char buf[256];
#define BAD(...) do { snprintf(buf, sizeof buf, __VA_ARGS__); why = buf; return SDSTREAM_E_INVALID_ARG; } while (0)
  if (c.in_channels < 1 || c.in_channels > 64) BAD("in_channels %d out of range", c.in_channels);
  if (c.n_levels < 1 || c.n_levels > SDSTREAM_MAX_LEVELS) BAD("n_levels %d out of range", c.n_levels);
  if (c.layers_per_block < 1 || c.layers_per_block > 8) BAD("layers_per_block %d out of range", c.layers_per_block);
  if (c.norm_groups < 1) BAD("norm_groups %d", c.norm_groups);
  if ((c.num_heads > 0) == (c.head_dim > 0)) BAD("exactly one of num_heads / head_dim must be positive");
  if (c.context_len < 1 || c.context_dim < 1) BAD("context %dx%d", c.context_len, c.context_dim);
  if (c.latent_h < 1 || c.latent_w < 1) BAD("latent %dx%d", c.latent_h, c.latent_w);
  if (c.latent_h % (1 << (c.n_levels - 1)) || c.latent_w % (1 << (c.n_levels - 1)))
    BAD("latent %dx%d must be divisible by 2^(n_levels-1)", c.latent_h, c.latent_w);
  if (c.dtype != 0 && c.dtype != 1) BAD("dtype %d", c.dtype);
  if (c.n_denoise < 1 || c.n_denoise > 64) BAD("n_denoise %d out of range", c.n_denoise);
  if (c.n_streams < 1 || c.n_streams > 64) BAD("n_streams %d out of range", c.n_streams);
  if (c.cfg_mode < 0 || c.cfg_mode > 3) BAD("cfg_mode %d", c.cfg_mode);
  if (c.scheduler < 0 || c.scheduler > 2) BAD("scheduler %d", c.scheduler);
  if (c.cross_frame < 0 || c.cross_frame > 1) BAD("cross_frame %d", c.cross_frame);
  if (c.image_width < 0 || c.image_width > 256) BAD("image_width %d out of range", c.image_width);
  if (c.image_width > 0 && c.in_channels != 4) BAD("the image stage needs 4 latent channels");
  if (c.image_width > 0 && (long long)(27 * c.image_width + 64 * 28) * 4 > 65536) BAD("image_width %d: LDS tile too large", c.image_width);
  for (int l = 0; l < c.n_levels; ++l) {
    int ch = c.block_channels[l];
    if (ch < 1 || ch % c.norm_groups) BAD("block_channels[%d]=%d not a multiple of norm_groups", l, ch);
    if (l == 0 && ch % 2) BAD("block_channels[0] must be even");
    bool at = ((c.attn_level_mask >> l) & 1) || (l == c.n_levels - 1 && c.mid_attention);
    if (at) {
      int heads = c.num_heads > 0 ? c.num_heads : ch / c.head_dim;
      if (heads < 1 || ch % heads) BAD("level %d: %d channels do not split into heads", l, ch);
      int d = ch / heads;
      if (d % 4 || d > 160) BAD("level %d: head width %d must be a multiple of 4 and at most 160", l, d);
    }
  }
  if ((long long)c.in_channels * 9 * (c.block_channels[0] + 64) * 4 > 65536)
    BAD("in_channels %d x block_channels[0] %d: the first convolution's LDS tile exceeds 64 KB", c.in_channels, c.block_channels[0]);
  return SDSTREAM_OK;
#undef BAD
}

void default_schedule(double* alphas) {
  // scaled-linear: beta_t = (linspace(sqrt(.00085), sqrt(.012), 1000))^2, alpha = cumulative product of 1 - beta
  double s0 = sqrt(0.00085), s1 = sqrt(0.012), prod = 1.0;
  for (int t = 0; t < 1000; ++t) {
    double sb = s0 + (s1 - s0) * (double)t / 999.0;
    prod *= 1.0 - sb * sb;
    alphas[t] = prod;
  }
}

int rows_for_mode(const sdstream_config& c) {
  int base = c.n_streams * c.n_denoise;
  if (c.cfg_mode == SDSTREAM_CFG_FULL) return 2 * base;
  if (c.cfg_mode == SDSTREAM_CFG_ONETIME) return base + c.n_streams;
  return base;
}

void reset_state(sdstream* h) {
  h->cur = 0;
  h->calls = 0;
  h->ssf_ref = -1;
  h->ssf_ref_norm = 0;
  h->ssf_frames = h->ssf_processed = h->ssf_skip_run = h->ssf_longest_skip_run = 0;
}

void ssf_count(sdstream* h, bool skipped) {
  h->ssf_frames++;
  if (skipped) {
    if (++h->ssf_skip_run > h->ssf_longest_skip_run) h->ssf_longest_skip_run = h->ssf_skip_run;
  } else {
    h->ssf_processed++;
    h->ssf_skip_run = 0;
  }
}

// ------------------------------------------------------------------------------------------------
// launching
// ------------------------------------------------------------------------------------------------
// the parameter block of a matrix-core GEMM op as it is launched on N rows (also what its tile plan is asked with)
IgemmParams mfma_params(sdstream* h, const Op& op0, int N) {
  IgemmParams g = op0.g;
  g.M = N * op0.rows_per_sample;
  g.zeros = h->persist + h->off_zeros;
  g.workspace = (float*)(h->persist + h->off_splitk);
  g.workspace_floats = (long long)kSplitKWorkspaceFloats;
  return g;
}

// Row tiles per sample when the GEMM op `prod`, launched on N rows, leaves the GroupNorm statistics that the norm op
// `gnop` right after it needs (the norm then runs its apply pass only); 0 when it does not.  Both launches ask here.
int gn_stats_splits(sdstream* h, const Op& prod, const Op& gnop, int N) {
#ifdef SDSTREAM_DEVHOOKS
  static const bool off = getenv("SDSTREAM_NO_GNSTATS") != nullptr;
  if (off) return 0;
#endif
  if (h->cfg.dtype != 1 || !prod.mfma) return 0;
  GroupNormParams gp = gnop.gn;
  gp.samples = N;
  if (!group_norm_takes_partials(gp)) return 0;
  const IgemmParams g = mfma_params(h, prod, N);
  if (g.epilogue != EPI_NONE || g.stats_out || g.ln_stats) return 0;
  const IgemmPlan pl = igemm_mfma_plan(g);
  const int HW = prod.rows_per_sample, C = g.N;
  if (C % gp.groups) return 0;
  const int cg = C / gp.groups;
  if (pl.variant == 3 && pl.bm == 64) {   // row-resident kernel, 64 rows x all 320 columns per block
    if (HW % 64 || HW / 64 > GN_MAX_SPLIT || g.slot_m > 0) return 0;
    return HW / 64;
  }
  if (!pl.grouped || pl.bn != 160 || pl.splitk != 1) return 0;
  if (HW % 128 || HW / 128 > GN_MAX_SPLIT || C % 160 || 160 % cg) return 0;
  return HW / 128;
}

// Statistics splits when the norm op `gnop` is not launched at all on N rows: the layer before it leaves its
// statistics AND the layer after it (`cons`, the 64-row row-resident kernel) applies it to its input rows on load.
// 0 when the norm runs as a kernel.  Both the norm's and the consumer's launch ask here.
int gn_applied_on_load(sdstream* h, const Op& gnop, const Op& cons, int N) {
#ifdef SDSTREAM_DEVHOOKS
  static const bool off = getenv("SDSTREAM_NO_GNLOAD") != nullptr;
  if (off) return 0;
#endif
  if (!gnop.gn_src_plus1 || gnop.gn.silu || gnop.gn.src2) return 0;
  const int splits = gn_stats_splits(h, h->ops[gnop.gn_src_plus1 - 1], gnop, N);
  if (!splits) return 0;
  const IgemmParams g = mfma_params(h, cons, N);
  const IgemmPlan pl = igemm_mfma_plan(g);
  if (pl.variant != 3 || pl.bm != 64 || g.C1 != 320 || g.C1 != gnop.gn.C1 || g.C1 % gnop.gn.groups) return 0;
  if (cons.rows_per_sample % 64 || gnop.gn.HW != cons.rows_per_sample) return 0;
  return splits;
}

void launch_op(sdstream* h, const Op& op0, int N, const int* kv_select, int xframe_rows, hipStream_t s) {
  const bool bf = h->cfg.dtype == 1;
  switch (op0.kind) {
    case OP_IGEMM: {
      IgemmParams g = op0.g;
      g.M = N * op0.rows_per_sample;
      g.zeros = h->persist + h->off_zeros;
      if (op0.mfma) {
        g = mfma_params(h, op0, N);
        if (op0.ln_src_op >= 0) {   // one part of row statistics per column tile of the producing layer
          const IgemmParams pg = mfma_params(h, h->ops[op0.ln_src_op], N);
          const int bn = igemm_mfma_plan(pg).bn;
          g.ln_parts = (pg.N + bn - 1) / bn;
        }
        if (op0.gn_in_plus1) {
          const Op& gnop = h->ops[op0.gn_in_plus1 - 1];
          const int splits = gn_applied_on_load(h, gnop, op0, N);
          if (splits) {   // the norm was not launched: its input, statistics and vectors come here
            g.src1 = gnop.gn.src1;
            g.gn_in_stats = gnop.gn.stats;
            g.gn_in_gamma = gnop.gn.gamma;
            g.gn_in_beta = gnop.gn.beta;
            g.gn_in_splits = splits;
            g.gn_in_groups = gnop.gn.groups;
            g.gn_in_eps = gnop.gn.eps;
          }
        }
        if (op0.gn_dst_plus1) {
          const Op& gnop = h->ops[op0.gn_dst_plus1 - 1];
          if (gn_stats_splits(h, op0, gnop, N)) {
            g.gn_stats = gnop.gn.stats;
            g.gn_groups = gnop.gn.groups;
            g.gn_cg = g.N / gnop.gn.groups;
          }
        }
        if (op0.xattn_site >= 0) {
          // The weights are per prompt: the rows of the positive prompt and those of the negative prompt (from row
          // neg_from on) are two launches on row ranges, with the tile shape the whole range would get (the layer
          // after this one reads one part of row statistics per column tile).
          const KVSite& ks = h->kv_sites[op0.xattn_site];
          const IgemmPlan plan = igemm_mfma_plan(g);
          const int split = h->neg_from < N ? h->neg_from : N;
          const int parts_out = (g.N + plan.bn - 1) / plan.bn;
          const long long split_m = (long long)split * op0.rows_per_sample;
          if (split > 0 && split < N && split_m % plan.bm == 0) {   // no row tile straddles the two prompts: one launch
            g.slot_m = (int)split_m;
            g.slot_w_bytes = (long long)ks.mat_stride;
            g.slot_v_bytes = op0.xattn_role == 1 ? (long long)ks.vec_stride : 0;
            launch_igemm_mfma(g, s);
            break;
          }
          for (int slot = 0; slot < 2; ++slot) {
            const int r0 = slot == 0 ? 0 : split, r1 = slot == 0 ? split : N;
            if (r1 <= r0) continue;
            IgemmParams q = g;
            const long long m0 = (long long)r0 * op0.rows_per_sample;
            q.M = (r1 - r0) * op0.rows_per_sample;
            q.force_variant = plan.variant;
            q.force_bn = plan.bn;
            q.src1 = (const char*)g.src1 + m0 * g.C1 * h->elt;
            q.out = (char*)g.out + m0 * g.N * h->elt;
            if (g.residual) q.residual = (const char*)g.residual + m0 * g.N * h->elt;
            if (g.ln_stats) q.ln_stats = g.ln_stats + m0 * g.ln_parts * 2;
            if (g.stats_out) q.stats_out = g.stats_out + m0 * parts_out * 2;
            q.W = (const char*)g.W + (size_t)slot * ks.mat_stride;
            if (op0.xattn_role == 1) {
              q.ln_wsum = (const float*)((const char*)g.ln_wsum + (size_t)slot * ks.vec_stride);
              q.bias = (const float*)((const char*)g.bias + (size_t)slot * ks.vec_stride);
            }
            launch_igemm_mfma(q, s);
          }
          break;
        }
        launch_igemm_mfma(g, s);
      }
      else if (bf) launch_igemm_generic<bf16_t>(g, s);
      else launch_igemm_generic<float>(g, s);
      break;
    }
    case OP_GN: {
      GroupNormParams p = op0.gn;
      p.samples = N;
      if (op0.gn_out_plus1 && gn_applied_on_load(h, op0, h->ops[op0.gn_out_plus1 - 1], N)) break;   // nothing to launch
      const int splits = op0.gn_src_plus1 ? gn_stats_splits(h, h->ops[op0.gn_src_plus1 - 1], op0, N) : 0;
      if (splits) launch_group_norm_apply(p, splits, s);   // the layer before it left the partial sums
      else if (bf) launch_group_norm<bf16_t>(p, s);
      else launch_group_norm<float>(p, s);
      break;
    }
    case OP_LN: {
      LayerNormParams p = op0.ln;
      p.rows = N * op0.rows_per_sample;
      if (bf) launch_layer_norm<bf16_t>(p, s); else launch_layer_norm<float>(p, s);
      break;
    }
    case OP_ATTN: {
      AttnParams p = op0.at;
      p.samples = N;
      if (p.kv_select) {
        p.kv_select = kv_select;
      } else if (h->cfg.cross_frame && h->cfg.n_denoise > 1) {
        // Sec. 3.2: the n rows of a stream batch attend to the keys and values of all of them
        p.kv_group = h->cfg.n_denoise;
        p.kv_group_rows = xframe_rows;
      }
      if (op0.mfma) launch_attention_mfma(p, s);
      else if (bf) launch_attention_generic<bf16_t>(p, s);
      else launch_attention_generic<float>(p, s);
      break;
    }
    case OP_CONV_IN: {
      const float* x = (const float*)op0.cin;
      if (bf) launch_conv_in<bf16_t>(x, op0.cw_f32, op0.cb, op0.cout_, N, op0.cCin, op0.cH, op0.cW, op0.cC0, op0.cflags, s);
      else launch_conv_in<float>(x, op0.cw_f32, op0.cb, op0.cout_, N, op0.cCin, op0.cH, op0.cW, op0.cC0, op0.cflags, s);
      break;
    }
    case OP_CONV_OUT: {
      float* out = (float*)op0.cout_;
      if (bf) launch_conv_out<bf16_t>(op0.cin, op0.cw, op0.cb, out, N, op0.cCin, op0.cH, op0.cW, op0.cC0, s);
      else launch_conv_out<float>(op0.cin, op0.cw, op0.cb, out, N, op0.cCin, op0.cH, op0.cW, op0.cC0, s);
      break;
    }
    case OP_IMAGE_IN: {
      const uint8_t* img = (const uint8_t*)op0.cin;
      if (bf) launch_image_in<bf16_t>(img, op0.cw_f32, op0.cb, op0.cout_, N, op0.cH, op0.cW, op0.cC0, s);
      else launch_image_in<float>(img, op0.cw_f32, op0.cb, op0.cout_, N, op0.cH, op0.cW, op0.cC0, s);
      break;
    }
    case OP_IMAGE_OUT: {
      if (bf) launch_image_out<bf16_t>(op0.cin, op0.cw, op0.cb, op0.img_f32, op0.img_u8, N, op0.cH, op0.cW, op0.cC0, s);
      else launch_image_out<float>(op0.cin, op0.cw, op0.cb, op0.img_f32, op0.img_u8, N, op0.cH, op0.cW, op0.cC0, s);
      break;
    }
  }
}

int prof_begin(sdstream* h, int cls, double flops, double bytes, hipStream_t s, int op = -1, int N = 0) {
  sdstream::ProfRec r;
  r.cls = cls; r.flops = flops; r.bytes = bytes; r.op = op; r.N = N;
  HIP_TRY(h, hipEventCreate(&r.a));
  HIP_TRY(h, hipEventCreate(&r.b));
  HIP_TRY(h, hipEventRecord(r.a, s));
  h->prof_pending.push_back(r);
  return SDSTREAM_OK;
}
int prof_end(sdstream* h, hipStream_t s) {
  HIP_TRY(h, hipEventRecord(h->prof_pending.back().b, s));
  return SDSTREAM_OK;
}

// the U-Net on `N` rows: x (fp32 NCHW, device) -> eps (fp32 NCHW, device)
int run_unet(sdstream* h, const float* x, float* eps, int N, const int* kv_select, bool for_step, hipStream_t s) {
  const bool graph = h->graph_enabled && !h->profiling && for_step;
  // rows that come in stream batches of n for cross-frame attention: in a step the positive-prompt rows (and, with
  // full CFG, their negative-prompt copies; the onetime-negative rows stay alone); in a plain forward call every
  // complete run of n rows
  const int nd = h->cfg.n_denoise;
  const int xframe_rows = for_step ? (h->cfg.cfg_mode == SDSTREAM_CFG_FULL ? 2 : 1) * h->cfg.n_streams * nd : N / nd * nd;
  // the first and last op read / write caller-visible buffers
  h->ops.front().cin = x;
  h->ops.back().cout_ = eps;
  h->neg_from = for_step ? h->cfg.n_streams * nd : N;
  if (graph) {
    const int key = N * 2 + h->cur;  // the input batch alternates between two buffers
    auto it = h->graphs.find(key);
    if (it == h->graphs.end()) {
      if (!h->cap_stream) HIP_TRY(h, hipStreamCreateWithFlags(&h->cap_stream, hipStreamNonBlocking));
      HIP_TRY(h, hipStreamBeginCapture(h->cap_stream, hipStreamCaptureModeThreadLocal));
      for (const Op& op : h->ops) launch_op(h, op, N, kv_select, xframe_rows, h->cap_stream);
      hipGraph_t gph = nullptr;
      HIP_TRY(h, hipStreamEndCapture(h->cap_stream, &gph));
      hipGraphExec_t ex = nullptr;
      hipError_t er = hipGraphInstantiate(&ex, gph, nullptr, nullptr, 0);
      hipGraphDestroy(gph);
      if (er != hipSuccess) return fail(h, SDSTREAM_E_HIP, "hipGraphInstantiate: %s", hipGetErrorString(er));
      it = h->graphs.emplace(key, ex).first;
    }
    HIP_TRY(h, hipGraphLaunch(it->second, s));
  } else {
    for (size_t oi = 0; oi < h->ops.size(); ++oi) {
      const Op& op = h->ops[oi];
      if (h->profiling) {
        int rc = prof_begin(h, op.cls, op.flops_per_row * N, op.bytes_per_row * N + op.bytes_fixed, s, (int)oi, N);
        if (rc) return rc;
      }
      launch_op(h, op, N, kv_select, xframe_rows, s);
      if (h->profiling) {
        int rc = prof_end(h, s);
        if (rc) return rc;
      }
    }
  }
  HIP_TRY(h, hipGetLastError());
  return SDSTREAM_OK;
}

// time-embedding biases for the rows' timesteps (cached)
int ensure_temb(sdstream* h, const std::vector<int>& t, hipStream_t s) {
  if (t == h->temb_cached) return SDSTREAM_OK;
  const int N = (int)t.size();
  // rare path (timesteps changed): drain the stream, then a blocking upload
  HIP_TRY(h, hipStreamSynchronize(s));
  HIP_TRY(h, hipMemcpy(h->persist + h->off_tdev, t.data(), (size_t)N * 4, hipMemcpyHostToDevice));
  launch_time_embedding((const int*)(h->persist + h->off_tdev), (float*)(h->persist + h->off_emb), N,
                        h->cfg.block_channels[0], s);
  for (const Op& op : h->temb_ops) {
    IgemmParams g = op.g;
    g.M = N;
    launch_igemm_generic<float>(g, s);
  }
  HIP_TRY(h, hipGetLastError());
  h->temb_cached = t;
  return SDSTREAM_OK;
}

// K/V of the prompt for every cross-attention site; slot 0 positive, slot 1 negative
int build_kv(sdstream* h, const float* ctx, const float* neg, hipStream_t s) {
  const sdstream_config& c = h->cfg;
  const bool bf = c.dtype == 1;
  const long long n = (long long)c.context_len * c.context_dim;
  char* ctxT = h->persist + h->off_ctxT;
  for (int slot = 0; slot < 2; ++slot) {
    const float* src = slot == 0 ? ctx : neg;
    if (!src) continue;
    void* dst = ctxT + (size_t)slot * n * h->elt;
    if (bf) launch_convert<bf16_t>(src, dst, n, s); else launch_convert<float>(src, dst, n, s);
    for (const KVSite& site : h->kv_sites) {
      IgemmParams g{};
      g.src1 = dst; g.C1 = c.context_dim; g.C2 = 0;
      g.Hin = c.context_len; g.Win = 1; g.Hout = c.context_len; g.Wout = 1;
      g.ksize = 1; g.stride = 1;
      g.M = c.context_len; g.N = 2 * site.C; g.K = c.context_dim;
      g.W = h->weights + site.w.w;
      g.out = h->persist + site.cache + (size_t)slot * c.context_len * 2 * site.C * h->elt;
      g.splitk = 1;
      g.zeros = h->persist + h->off_zeros;
      if (site.w.mfma) launch_igemm_mfma(g, s);
      else if (bf) launch_igemm_generic<bf16_t>(g, s);
      else launch_igemm_generic<float>(g, s);
      if (site.xfold)   // the per-prompt matrices of the folded cross-attention, from the keys / values just made
        launch_xattn_fold(g.out, 2 * site.C, (const float*)(h->weights + site.wq_raw), (const float*)(h->weights + site.wo_raw),
                          (const float*)(h->weights + site.ln_g), (const float*)(h->weights + site.ln_b),
                          (float*)(h->persist + h->off_xraw), h->persist + site.qk + (size_t)slot * site.mat_stride,
                          (float*)(h->persist + site.wsum + (size_t)slot * site.vec_stride),
                          (float*)(h->persist + site.lnb + (size_t)slot * site.vec_stride),
                          h->persist + site.vo + (size_t)slot * site.mat_stride, site.C, site.heads, site.d, c.context_len,
                          site.Lp, site.Npad, s);
    }
  }
  HIP_TRY(h, hipGetLastError());
  return SDSTREAM_OK;
}

// copies the tensors of `entries` from a host blob (manifest order, float32) into the arena at `base`, converting and
// repacking each as its entry says; synchronous
int load_entries(sdstream* h, const std::vector<Entry>& entries, char* base, int64_t n_params,
                 const std::vector<BiasFix>& fixes, const void* host_blob, size_t bytes) {
  if (bytes != (size_t)n_params * 4)
    return fail(h, SDSTREAM_E_SHAPE, "blob has %zu bytes, the manifest needs %zu", bytes, (size_t)n_params * 4);
  size_t max_count = 0;
  for (const Entry& en : entries) max_count = en.count > max_count ? en.count : max_count;
  float* stage = nullptr;
  HIP_TRY(h, hipMalloc((void**)&stage, max_count * 4));
  const bool bf = h->cfg.dtype == 1;
  const float* src = (const float*)host_blob;
  hipStream_t s = nullptr;
  int rc = SDSTREAM_OK;
  for (const Entry& en : entries) {
    hipError_t er = hipMemcpy(stage, src, en.count * 4, hipMemcpyHostToDevice);
    if (er != hipSuccess) { rc = fail(h, SDSTREAM_E_HIP, "hipMemcpy: %s", hipGetErrorString(er)); break; }
    src += en.count;
    void* dst = base + en.dst_off;
    if (en.raw_copy) launch_copy_rows_f32(stage, (float*)(base + en.raw_off), (long long)en.count, s);
    switch (en.action) {
      case LA_F32: launch_copy_rows_f32(stage, (float*)dst, (long long)en.count, s); break;
      case LA_ROWMAJOR:
        if (bf) launch_repack_rowmajor<bf16_t>(stage, dst, en.O, en.I, en.taps, en.geglu, s);
        else launch_repack_rowmajor<float>(stage, dst, en.O, en.I, en.taps, en.geglu, s);
        break;
      case LA_MFMA:
        if (en.ln_fold) {
          launch_repack_mfma(stage, dst, en.O, en.I, en.taps, en.geglu, (const float*)(base + en.ln_g), 0, 0, s);
          launch_ln_fold_vectors(stage, (const float*)(base + en.ln_g), (const float*)(base + en.ln_b),
                                 (float*)(base + en.ln_wsum), (float*)(base + en.ln_lnb), en.O, en.I, en.geglu, s);
        } else {
          launch_repack_mfma(stage, dst, en.O, en.I, en.taps, en.geglu, nullptr, en.pk_total, en.pk_off, s);
        }
        break;
      case LA_BIAS_PERM: launch_permute_bias(stage, (float*)dst, en.O, en.geglu, s); break;
    }
    er = hipDeviceSynchronize();
    if (er != hipSuccess) { rc = fail(h, SDSTREAM_E_HIP, "repack: %s", hipGetErrorString(er)); break; }
  }
  hipFree(stage);
  if (rc) return rc;
  for (const BiasFix& f : fixes) {   // vectors made of two loaded ones (bias + shift-times-weights of a folded LayerNorm; two biases)
    if (f.copy) launch_copy_rows_f32((const float*)(base + f.bias), (float*)(base + f.lnb), f.n, s);
    else launch_add_f32((float*)(base + f.lnb), (const float*)(base + f.bias), f.n, s);
  }
  HIP_TRY(h, hipDeviceSynchronize());
  return SDSTREAM_OK;
}

uint64_t splitmix64_mix(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

}  // namespace

// ================================================================================================
// C ABI
// ================================================================================================
extern "C" {

const char* sdstream_last_error(const sdstream_t* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

int sdstream_create(const sdstream_config* cfg, sdstream_t** out) {
  if (!cfg || !out) return fail(nullptr, SDSTREAM_E_INVALID_ARG, "null argument");
  *out = nullptr;
  std::string why;
  int rc = validate(*cfg, why);
  if (rc) return fail(nullptr, rc, "%s", why.c_str());
  sdstream* h = new (std::nothrow) sdstream();
  if (!h) return fail(nullptr, SDSTREAM_E_NOMEM, "out of host memory");
  h->cfg = *cfg;
  h->elt = cfg->dtype == 1 ? 2 : 4;
  h->use_mfma = cfg->dtype == 1;
#ifdef SDSTREAM_DEVHOOKS
  if (getenv("SDSTREAM_NO_MFMA")) h->use_mfma = false;   // development build only: bf16 storage on the vector-ALU kernels
#endif
  h->E = cfg->in_channels * cfg->latent_h * cfg->latent_w;
  h->max_batch = rows_for_mode(*cfg);
  memset(h->prof, 0, sizeof h->prof);
  default_schedule(h->alphas);
  // pass 1: sizes and manifest
  {
    Builder b(*h, true);
    b.build();
    h->weight_bytes = b.wbytes;
    h->persist_bytes = b.pbytes;
    h->act_bytes = h->act.peak * (size_t)h->max_batch;
  }
  h->n_params = 0;
  for (const Entry& en : h->manifest) h->n_params += (int64_t)en.count;
  if (cfg->image_width > 0) {
    ImageBuilder ib(*h, true);
    ib.build();
    h->img_weight_bytes = ib.wbytes;
    h->img_act_bytes = h->img_act.peak * (size_t)cfg->n_streams;
    for (const Entry& en : h->img_manifest) h->img_n_params += (int64_t)en.count;
  }
  hipError_t e1 = hipMalloc((void**)&h->weights, h->weight_bytes);
  hipError_t e2 = e1 == hipSuccess ? hipMalloc((void**)&h->persist, h->persist_bytes) : e1;
  hipError_t e3 = e2 == hipSuccess ? hipMalloc((void**)&h->act_base, h->act_bytes ? h->act_bytes : 256) : e2;
  if (e3 != hipSuccess) {
    int code = fail(nullptr, e3 == hipErrorOutOfMemory ? SDSTREAM_E_NOMEM : SDSTREAM_E_HIP, "hipMalloc: %s",
                    hipGetErrorString(e3));
    sdstream_destroy(h);
    return code;
  }
  if (hipMemset(h->persist, 0, h->persist_bytes) != hipSuccess) {
    sdstream_destroy(h);
    return fail(nullptr, SDSTREAM_E_HIP, "hipMemset failed");
  }
  if (cfg->image_width > 0) {
    hipError_t i1 = hipMalloc((void**)&h->img_weights, h->img_weight_bytes);
    hipError_t i2 = i1 == hipSuccess ? hipMalloc((void**)&h->img_act_base, h->img_act_bytes) : i1;
    if (i2 != hipSuccess) {
      int code = fail(nullptr, i2 == hipErrorOutOfMemory ? SDSTREAM_E_NOMEM : SDSTREAM_E_HIP, "hipMalloc: %s",
                      hipGetErrorString(i2));
      sdstream_destroy(h);
      return code;
    }
    ImageBuilder ib(*h, false);
    ib.build();
  }
  // pass 2: real pointers
  {
    Builder b(*h, false);
    b.build();
  }
  reset_state(h);
  *out = h;
  return SDSTREAM_OK;
}

void sdstream_destroy(sdstream_t* h) {
  if (!h) return;
  hipDeviceSynchronize();
  for (auto& kv : h->graphs) hipGraphExecDestroy(kv.second);
  for (auto& ig : h->img_graph) if (ig.exec) hipGraphExecDestroy(ig.exec);
  if (h->img_weights) hipFree(h->img_weights);
  if (h->img_act_base) hipFree(h->img_act_base);
  if (h->cap_stream) hipStreamDestroy(h->cap_stream);
  for (auto& r : h->prof_pending) { hipEventDestroy(r.a); hipEventDestroy(r.b); }
  if (h->weights) hipFree(h->weights);
  if (h->persist) hipFree(h->persist);
  if (h->act_base) hipFree(h->act_base);
  for (int i = 0; i < 2; ++i) if (h->ssf_buf[i]) hipFree(h->ssf_buf[i]);
  if (h->ssf_sums) hipFree(h->ssf_sums);
  if (h->ssf_host) hipHostFree(h->ssf_host);
  delete h;
}

int64_t sdstream_param_count(const sdstream_t* h) { return h ? h->n_params : 0; }
int32_t sdstream_manifest_size(const sdstream_t* h) { return h ? (int32_t)h->manifest.size() : 0; }
int32_t sdstream_max_batch(const sdstream_t* h) { return h ? h->max_batch : 0; }
double sdstream_flops_per_row(const sdstream_t* h) { return h ? h->flops_per_row : 0.0; }

int sdstream_manifest_entry(const sdstream_t* h, int32_t index, char* name, size_t name_cap, int32_t shape[4],
                            int32_t* ndim, int32_t* kind) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  sdstream* hm = const_cast<sdstream*>(h);
  if (index < 0 || index >= (int32_t)h->manifest.size()) return fail(hm, SDSTREAM_E_INVALID_ARG, "index out of range");
  const Entry& en = h->manifest[index];
  if (name && name_cap) {
    strncpy(name, en.name.c_str(), name_cap - 1);
    name[name_cap - 1] = 0;
  }
  if (shape) for (int i = 0; i < 4; ++i) shape[i] = en.shape[i];
  if (ndim) *ndim = en.ndim;
  if (kind) *kind = en.kind;
  return SDSTREAM_OK;
}

int sdstream_load_weights(sdstream_t* h, const void* host_blob, size_t bytes) {
  if (!h || !host_blob) return h ? fail(h, SDSTREAM_E_INVALID_ARG, "null blob") : SDSTREAM_E_INVALID_ARG;
  int rc = load_entries(h, h->manifest, h->weights, h->n_params, h->bias_fixes, host_blob, bytes);
  if (rc) return rc;
  h->weights_loaded = true;
  h->temb_cached.clear();
  h->kv_valid = false;
  return SDSTREAM_OK;
}

int64_t sdstream_image_param_count(const sdstream_t* h) { return h ? h->img_n_params : 0; }
int32_t sdstream_image_manifest_size(const sdstream_t* h) { return h ? (int32_t)h->img_manifest.size() : 0; }

int sdstream_image_manifest_entry(const sdstream_t* h, int32_t index, char* name, size_t name_cap, int32_t shape[4],
                                  int32_t* ndim, int32_t* kind) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  sdstream* hm = const_cast<sdstream*>(h);
  if (index < 0 || index >= (int32_t)h->img_manifest.size()) return fail(hm, SDSTREAM_E_INVALID_ARG, "index out of range");
  const Entry& en = h->img_manifest[index];
  if (name && name_cap) {
    strncpy(name, en.name.c_str(), name_cap - 1);
    name[name_cap - 1] = 0;
  }
  if (shape) for (int i = 0; i < 4; ++i) shape[i] = en.shape[i];
  if (ndim) *ndim = en.ndim;
  if (kind) *kind = en.kind;
  return SDSTREAM_OK;
}

int sdstream_load_image_weights(sdstream_t* h, const void* host_blob, size_t bytes) {
  if (!h || !host_blob) return h ? fail(h, SDSTREAM_E_INVALID_ARG, "null blob") : SDSTREAM_E_INVALID_ARG;
  if (h->cfg.image_width <= 0) return fail(h, SDSTREAM_E_NOT_READY, "this engine was created without an image stage");
  static const std::vector<BiasFix> none;
  int rc = load_entries(h, h->img_manifest, h->img_weights, h->img_n_params, none, host_blob, bytes);
  if (rc) return rc;
  h->img_weights_loaded = true;
  return SDSTREAM_OK;
}

int sdstream_set_schedule(sdstream_t* h, const float* alphas_cumprod) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (alphas_cumprod) {
    for (int t = 0; t < 1000; ++t)
      if (!(alphas_cumprod[t] > 0.f && alphas_cumprod[t] <= 1.f))
        return fail(h, SDSTREAM_E_INVALID_ARG, "alphas_cumprod[%d] = %g not in (0,1]", t, (double)alphas_cumprod[t]);
    for (int t = 0; t < 1000; ++t) h->alphas[t] = alphas_cumprod[t];
  } else {
    default_schedule(h->alphas);
  }
  h->timesteps.clear();
  reset_state(h);
  return SDSTREAM_OK;
}

int sdstream_set_noise(sdstream_t* h, const float* host_noise) {
  if (!h || !host_noise) return h ? fail(h, SDSTREAM_E_INVALID_ARG, "null noise") : SDSTREAM_E_INVALID_ARG;
  size_t bytes = (size_t)h->cfg.n_denoise * h->cfg.n_streams * h->E * 4;
  // drains every stream of the device first: a step still in flight reads the cache
  HIP_TRY(h, hipDeviceSynchronize());
  HIP_TRY(h, hipMemcpy(h->persist + h->off_noise, host_noise, bytes, hipMemcpyHostToDevice));
  h->have_noise = true;
  return sdstream_reset(h);
}

int sdstream_reset(sdstream_t* h) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  HIP_TRY(h, hipDeviceSynchronize());
  for (int i = 0; i < 2; ++i) {
    HIP_TRY(h, hipMemset(h->persist + h->off_x[i], 0, (size_t)h->max_batch * h->E * 4));
    HIP_TRY(h, hipMemset(h->persist + h->off_r[i], 0, (size_t)h->cfg.n_streams * h->cfg.n_denoise * h->E * 4));
  }
  reset_state(h);
  return SDSTREAM_OK;
}

int sdstream_unet_forward(sdstream_t* h, const float* x, const int32_t* t, const float* ctx, int32_t n, float* eps_out,
                          void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!x || !t || !ctx || !eps_out) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  if (!h->weights_loaded) return fail(h, SDSTREAM_E_NOT_READY, "weights not loaded");
  if (n < 1 || n > h->max_batch) return fail(h, SDSTREAM_E_SHAPE, "batch %d outside [1,%d]", n, h->max_batch);
  std::vector<int> tv(t, t + n);
  for (int v : tv) if (v < 0 || v > 999) return fail(h, SDSTREAM_E_INVALID_ARG, "timestep %d outside [0,999]", v);
  hipStream_t s = (hipStream_t)hip_stream;
  int rc = ensure_temb(h, tv, s);
  if (rc) return rc;
  rc = build_kv(h, ctx, nullptr, s);
  if (rc) return rc;
  h->kv_valid = false;  // the step path must rebuild its own
  return run_unet(h, x, eps_out, n, (const int*)(h->persist + h->off_sel_zero), false, s);
}

}  // extern "C"

namespace {
// everything of a step that comes before its launches: argument checks, schedule constants and queue reset on new
// timesteps, time-embedding biases, the prompt's keys / values; fills the parameter block of head and tail
int step_prepare(sdstream* h, const float* x0_in, const float* context, const float* neg_context, uint64_t context_epoch,
                 const int32_t* timesteps, float gamma, float delta, float* out_latent, hipStream_t s, StreamParams* pp) {
  const sdstream_config& c = h->cfg;
  if (!x0_in || !context || !timesteps || !out_latent) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  if (!h->weights_loaded) return fail(h, SDSTREAM_E_NOT_READY, "weights not loaded");
  if (!h->have_noise) return fail(h, SDSTREAM_E_NOT_READY, "noise cache not set");
  const bool need_neg = c.cfg_mode == SDSTREAM_CFG_FULL || c.cfg_mode == SDSTREAM_CFG_ONETIME;
  if (need_neg && !neg_context) return fail(h, SDSTREAM_E_INVALID_ARG, "this cfg_mode needs neg_context");
  const int n = c.n_denoise, S = c.n_streams;
  for (int i = 0; i < n; ++i) {
    if (timesteps[i] < 0 || timesteps[i] > 999)
      return fail(h, SDSTREAM_E_INVALID_ARG, "timestep %d outside [0,999]", timesteps[i]);
    if (i && timesteps[i] >= timesteps[i - 1]) return fail(h, SDSTREAM_E_INVALID_ARG, "timesteps must strictly decrease");
  }
  std::vector<int> ts(timesteps, timesteps + n);
  const int rows = h->max_batch;
  if (ts != h->timesteps) {
    // new schedule points: constants, selection table, and a fresh queue
    std::vector<float> ab(4 * n);
    for (int i = 0; i < n; ++i) {
      ab[i] = (float)sqrt(h->alphas[ts[i]]);
      ab[n + i] = (float)sqrt(1.0 - h->alphas[ts[i]]);
      // consistency parameterisation of the appendix (sigma_data = 0.5, s = 10), in the form that has the limits the
      // text states: c_skip(0) = 1, c_out(0) = 0, and (0, 1) to fp32 accuracy at the timesteps the paper runs
      const double st = 10.0 * ts[i], sd2 = 0.25;
      ab[2 * n + i] = (float)(sd2 / (st * st + sd2));
      ab[3 * n + i] = (float)(st / sqrt(st * st + sd2));
    }
    std::vector<int> sel(rows, 0);
    for (int r = S * n; r < rows; ++r) sel[r] = 1;
    HIP_TRY(h, hipStreamSynchronize(s));
    HIP_TRY(h, hipMemcpy(h->persist + h->off_ab, ab.data(), ab.size() * 4, hipMemcpyHostToDevice));
    HIP_TRY(h, hipMemcpy(h->persist + h->off_sel_step, sel.data(), sel.size() * 4, hipMemcpyHostToDevice));
    int rc = sdstream_reset(h);
    if (rc) return rc;
    h->timesteps = ts;
  }
  std::vector<int> trow(rows);
  for (int r = 0; r < S * n; ++r) trow[r] = ts[r % n];
  for (int r = S * n; r < rows; ++r) trow[r] = c.cfg_mode == SDSTREAM_CFG_FULL ? ts[(r - S * n) % n] : ts[0];
  int rc = ensure_temb(h, trow, s);
  if (rc) return rc;
  if (!h->kv_valid || h->kv_epoch != context_epoch) {
    rc = build_kv(h, context, need_neg ? neg_context : nullptr, s);
    if (rc) return rc;
    h->kv_valid = true;
    h->kv_epoch = context_epoch;
  }

  StreamParams& p = *pp;
  p.S = S; p.n = n; p.E = h->E; p.mode = c.cfg_mode; p.scheduler = c.scheduler;
  p.gamma = gamma; p.delta = delta;
  p.a = (const float*)(h->persist + h->off_ab);
  p.b = p.a + n;
  p.cskip = p.a + 2 * n;
  p.cout = p.a + 3 * n;
  p.noise = (const float*)(h->persist + h->off_noise);
  p.x0_in = x0_in;
  p.xcur = (float*)(h->persist + h->off_x[h->cur]);
  p.xnext = (float*)(h->persist + h->off_x[h->cur ^ 1]);
  p.rcur = (float*)(h->persist + h->off_r[h->cur]);
  p.rnext = (float*)(h->persist + h->off_r[h->cur ^ 1]);
  p.eps = (const float*)(h->persist + h->off_eps);
  p.out = out_latent;
  return SDSTREAM_OK;
}
}  // namespace

extern "C" {

int sdstream_step(sdstream_t* h, const float* x0_in, const float* context, const float* neg_context,
                  uint64_t context_epoch, const int32_t* timesteps, float gamma, float delta, float* out_latent,
                  int32_t* out_valid, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  StreamParams p;
  int rc = step_prepare(h, x0_in, context, neg_context, context_epoch, timesteps, gamma, delta, out_latent, s, &p);
  if (rc) return rc;
  const int n = h->cfg.n_denoise, S = h->cfg.n_streams, rows = h->max_batch;
  const double head_bytes = (double)S * h->E * 4 * 3, tail_bytes = (double)S * n * h->E * 4 * 5;
  if (h->profiling) { rc = prof_begin(h, PC_STREAM_HEAD, 0, head_bytes, s); if (rc) return rc; }
  launch_stream_head(p, s);
  if (h->profiling) { rc = prof_end(h, s); if (rc) return rc; }
  rc = run_unet(h, p.xcur, (float*)(h->persist + h->off_eps), rows, (const int*)(h->persist + h->off_sel_step), true, s);
  if (rc) return rc;
  if (h->profiling) { rc = prof_begin(h, PC_STREAM_TAIL, 0, tail_bytes, s); if (rc) return rc; }
  launch_stream_tail(p, s);
  if (h->profiling) { rc = prof_end(h, s); if (rc) return rc; }
  HIP_TRY(h, hipGetLastError());
  if (out_valid) *out_valid = h->calls >= n - 1 ? 1 : 0;
  h->calls++;
  h->cur ^= 1;
  return SDSTREAM_OK;
}

int sdstream_encode(sdstream_t* h, const uint8_t* image, float* latent_out, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!image || !latent_out) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  if (!h->img_weights_loaded) return fail(h, SDSTREAM_E_NOT_READY, "image-stage weights not loaded");
  hipStream_t s = (hipStream_t)hip_stream;
  h->img_enc_ops.front().cin = image;
  h->img_enc_ops.back().cout_ = latent_out;
  for (const Op& op : h->img_enc_ops) launch_op(h, op, h->cfg.n_streams, nullptr, 0, s);
  HIP_TRY(h, hipGetLastError());
  return SDSTREAM_OK;
}

int sdstream_decode(sdstream_t* h, const float* latent, uint8_t* image_out, float* image_f32_out, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!latent || (!image_out && !image_f32_out)) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  if (!h->img_weights_loaded) return fail(h, SDSTREAM_E_NOT_READY, "image-stage weights not loaded");
  hipStream_t s = (hipStream_t)hip_stream;
  h->img_dec_ops.front().cin = latent;
  h->img_dec_ops.back().img_u8 = image_out;
  h->img_dec_ops.back().img_f32 = image_f32_out;
  for (const Op& op : h->img_dec_ops) launch_op(h, op, h->cfg.n_streams, nullptr, 0, s);
  HIP_TRY(h, hipGetLastError());
  return SDSTREAM_OK;
}

int sdstream_step_image(sdstream_t* h, const uint8_t* frame, const float* context, const float* neg_context,
                        uint64_t context_epoch, const int32_t* timesteps, float gamma, float delta, uint8_t* image_out,
                        int32_t* out_valid, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!frame || !image_out) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  if (!h->img_weights_loaded) return fail(h, SDSTREAM_E_NOT_READY, "image-stage weights not loaded");
  hipStream_t s = (hipStream_t)hip_stream;
  float* lat_in = (float*)(h->persist + h->off_img_lat_in);
  float* lat_out = (float*)(h->persist + h->off_img_lat_out);
  StreamParams p;
  int rc = step_prepare(h, lat_in, context, neg_context, context_epoch, timesteps, gamma, delta, lat_out, s, &p);
  if (rc) return rc;
  const int n = h->cfg.n_denoise, S = h->cfg.n_streams, rows = h->max_batch;
  h->img_enc_ops.front().cin = frame;
  h->img_enc_ops.back().cout_ = lat_in;
  h->img_dec_ops.front().cin = lat_out;
  h->img_dec_ops.back().img_u8 = image_out;
  h->img_dec_ops.back().img_f32 = nullptr;
  h->ops.front().cin = p.xcur;
  h->ops.back().cout_ = (float*)(h->persist + h->off_eps);
  const int* sel = (const int*)(h->persist + h->off_sel_step);
  const int xframe_rows = (h->cfg.cfg_mode == SDSTREAM_CFG_FULL ? 2 : 1) * S * n;
  h->neg_from = S * n;
  auto launch_all = [&](hipStream_t st) {   // image -> latent -> one Stream Batch step -> latent -> image
    for (const Op& op : h->img_enc_ops) launch_op(h, op, S, nullptr, 0, st);
    launch_stream_head(p, st);
    for (const Op& op : h->ops) launch_op(h, op, rows, sel, xframe_rows, st);
    launch_stream_tail(p, st);
    for (const Op& op : h->img_dec_ops) launch_op(h, op, S, nullptr, 0, st);
  };
  if (h->graph_enabled && !h->profiling) {
    // One graph per queue buffer.  What a captured launch bakes in besides the engine's own buffers - the caller's two
    // image pointers and the guidance scalars - is remembered with the graph; a call that differs captures again, so a
    // caller that hands over the same device buffers every frame replays one graph per frame.
    sdstream::ImageGraph& ig = h->img_graph[h->cur];
    if (ig.exec && (ig.frame != frame || ig.image != image_out || ig.gamma != gamma || ig.delta != delta)) {
      hipGraphExecDestroy(ig.exec);
      ig.exec = nullptr;
    }
    if (!ig.exec) {
      if (!h->cap_stream) HIP_TRY(h, hipStreamCreateWithFlags(&h->cap_stream, hipStreamNonBlocking));
      HIP_TRY(h, hipStreamBeginCapture(h->cap_stream, hipStreamCaptureModeThreadLocal));
      launch_all(h->cap_stream);
      hipGraph_t gph = nullptr;
      HIP_TRY(h, hipStreamEndCapture(h->cap_stream, &gph));
      hipError_t er = hipGraphInstantiate(&ig.exec, gph, nullptr, nullptr, 0);
      hipGraphDestroy(gph);
      if (er != hipSuccess) { ig.exec = nullptr; return fail(h, SDSTREAM_E_HIP, "hipGraphInstantiate: %s", hipGetErrorString(er)); }
      ig.frame = frame; ig.image = image_out; ig.gamma = gamma; ig.delta = delta;
    }
    HIP_TRY(h, hipGraphLaunch(ig.exec, s));
  } else {
    launch_all(s);
  }
  HIP_TRY(h, hipGetLastError());
  if (out_valid) *out_valid = h->calls >= n - 1 ? 1 : 0;
  h->calls++;
  h->cur ^= 1;
  return SDSTREAM_OK;
}

int sdstream_ssf_decide(uint64_t dot, uint64_t n_t, uint64_t n_ref, double eta, uint64_t seed, uint64_t frame_index,
                        double* prob) {
  double p = 0.0;
  if (n_t != 0 && n_ref != 0 && eta < 1.0) {
    double sc = (double)dot / sqrt((double)n_t * (double)n_ref);
    if (sc > 1.0) sc = 1.0;
    p = (sc - eta) / (1.0 - eta);
    if (p < 0.0) p = 0.0;
  }
  uint64_t z = seed + (frame_index + 1) * 0x9E3779B97F4A7C15ULL;
  double u = (double)(splitmix64_mix(z) >> 11) * (1.0 / 9007199254740992.0);
  if (prob) *prob = p;
  return u < p ? 1 : 0;
}

int sdstream_ssf_decide_hard(uint64_t dot, uint64_t n_t, uint64_t n_ref, double eta, double* similarity) {
  double sc = 0.0;
  if (n_t != 0 && n_ref != 0) {
    sc = (double)dot / sqrt((double)n_t * (double)n_ref);
    if (sc > 1.0) sc = 1.0;
  }
  if (similarity) *similarity = sc;
  return (n_t != 0 && n_ref != 0 && sc > eta) ? 1 : 0;
}

}  // extern "C"

namespace {
// the device half of both filters: exact integer sums of the frame against the reference frame; the frame is
// copied into the spare buffer on the way, so letting it through afterwards is a pointer swap
int ssf_measure(sdstream* h, const uint8_t* frame, int32_t height, int32_t width, hipStream_t s, uint64_t* dot,
                uint64_t* nt, bool* have_ref, int* spare_out) {
  if (height < 1 || width < 1) return fail(h, SDSTREAM_E_SHAPE, "frame %dx%d", height, width);
  if (((uintptr_t)frame) & 15) return fail(h, SDSTREAM_E_INVALID_ARG, "frame must be 16-byte aligned");
  const long long n = (long long)height * width * 3;
  if (n != h->ssf_n) {
    HIP_TRY(h, hipDeviceSynchronize());
    for (int i = 0; i < 2; ++i) {
      if (h->ssf_buf[i]) hipFree(h->ssf_buf[i]);
      h->ssf_buf[i] = nullptr;
      HIP_TRY(h, hipMalloc((void**)&h->ssf_buf[i], (size_t)n + 16));
    }
    if (!h->ssf_sums) HIP_TRY(h, hipMalloc((void**)&h->ssf_sums, 4 * sizeof(unsigned long long)));
    if (!h->ssf_host) HIP_TRY(h, hipHostMalloc((void**)&h->ssf_host, 4 * sizeof(unsigned long long), hipHostMallocDefault));
    h->ssf_n = n;
    h->ssf_ref = -1;
  }
  const uint8_t* ref = h->ssf_ref >= 0 ? h->ssf_buf[h->ssf_ref] : nullptr;
  const int spare = h->ssf_ref >= 0 ? h->ssf_ref ^ 1 : 0;
  launch_ssf_reduce(frame, ref, h->ssf_buf[spare], n, h->ssf_sums, s);
  HIP_TRY(h, hipMemcpyAsync(h->ssf_host, h->ssf_sums, 2 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
  HIP_TRY(h, hipStreamSynchronize(s));
  *dot = h->ssf_host[0];
  *nt = h->ssf_host[1];
  *have_ref = ref != nullptr;
  *spare_out = spare;
  return SDSTREAM_OK;
}
}  // namespace

extern "C" {

int sdstream_ssf(sdstream_t* h, const uint8_t* frame, int32_t height, int32_t width, double eta, uint64_t seed,
                 uint64_t frame_index, int32_t* skip, double* prob, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!frame || !skip) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  uint64_t dot, nt;
  bool have_ref;
  int spare;
  int rc = ssf_measure(h, frame, height, width, (hipStream_t)hip_stream, &dot, &nt, &have_ref, &spare);
  if (rc) return rc;
  double p = 0.0;
  int sk = sdstream_ssf_decide(dot, nt, have_ref ? h->ssf_ref_norm : 0, eta, seed, frame_index, &p);
  if (!have_ref) { sk = 0; p = 0.0; }
  if (!sk) {
    h->ssf_ref = spare;
    h->ssf_ref_norm = nt;
  }
  ssf_count(h, sk != 0);
  *skip = sk;
  if (prob) *prob = p;
  return SDSTREAM_OK;
}

int sdstream_ssf_hard(sdstream_t* h, const uint8_t* frame, int32_t height, int32_t width, double eta, int32_t* skip,
                      double* similarity, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!frame || !skip) return fail(h, SDSTREAM_E_INVALID_ARG, "null argument");
  uint64_t dot, nt;
  bool have_ref;
  int spare;
  int rc = ssf_measure(h, frame, height, width, (hipStream_t)hip_stream, &dot, &nt, &have_ref, &spare);
  if (rc) return rc;
  double sc = 0.0;
  int sk = have_ref ? sdstream_ssf_decide_hard(dot, nt, h->ssf_ref_norm, eta, &sc) : 0;
  if (!sk) {
    h->ssf_ref = spare;
    h->ssf_ref_norm = nt;
  }
  ssf_count(h, sk != 0);
  *skip = sk;
  if (similarity) *similarity = sc;
  return SDSTREAM_OK;
}

int sdstream_ssf_run_stats(const sdstream_t* h, int64_t* frames, int64_t* processed, int64_t* longest_skip_run) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (frames) *frames = h->ssf_frames;
  if (processed) *processed = h->ssf_processed;
  if (longest_skip_run) *longest_skip_run = h->ssf_longest_skip_run;
  return SDSTREAM_OK;
}

int sdstream_profile_enable(sdstream_t* h, int32_t on) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  h->profiling = on != 0;
  return SDSTREAM_OK;
}

static int prof_drain(sdstream* h) {
  HIP_TRY(h, hipDeviceSynchronize());
  for (auto& r : h->prof_pending) {
    float ms = 0.f;
    hipEventElapsedTime(&ms, r.a, r.b);
#ifdef SDSTREAM_DEVHOOKS
    static const bool print_ops = getenv("SDSTREAM_PROFILE_OPS") != nullptr;
    if (r.op >= 0 && print_ops) {
      const Op& op = h->ops[r.op];
      if (op.kind == OP_IGEMM)
      {
        IgemmPlan pl{0, 0, 0, 0};
        if (op.mfma) pl = igemm_mfma_plan(mfma_params(h, op, r.N));
        fprintf(stderr, "op %3d %-11s M=%d N=%d K=%d ks=%d st=%d up=%d epi=%d res=%d v=%d bn=%d sk=%d  %.1f us  %.1f TF/s\n", r.op,
                kProfNames[r.cls], r.N * op.rows_per_sample, op.g.N, op.g.K, op.g.ksize, op.g.stride, op.g.upsample,
                op.g.epilogue, op.g.residual ? 1 : 0, pl.variant, pl.bn, pl.splitk, ms * 1e3, r.flops / (ms * 1e-3) / 1e12);
      }
      else if (op.kind == OP_ATTN)
        fprintf(stderr, "op %3d %-11s Sq=%d Skv=%d heads=%d d=%d  %.1f us  %.1f TF/s\n", r.op, kProfNames[r.cls],
                op.at.Sq, op.at.Skv, op.at.heads, op.at.d, ms * 1e3, r.flops / (ms * 1e-3) / 1e12);
      else
        fprintf(stderr, "op %3d %-11s rows=%d  %.1f us  %.1f GB/s\n", r.op, kProfNames[r.cls],
                r.N * op.rows_per_sample, ms * 1e3, r.bytes / (ms * 1e-3) / 1e9);
    }
#endif
    sdstream_profile_entry& e = h->prof[r.cls];
    e.launches += 1;
    e.ms += ms;
    e.flops += r.flops;
    e.bytes += r.bytes;
    hipEventDestroy(r.a);
    hipEventDestroy(r.b);
  }
  h->prof_pending.clear();
  return SDSTREAM_OK;
}

int sdstream_profile_reset(sdstream_t* h) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  int rc = prof_drain(h);
  if (rc) return rc;
  memset(h->prof, 0, sizeof h->prof);
  return SDSTREAM_OK;
}

int32_t sdstream_profile_read(sdstream_t* h, sdstream_profile_entry* out, int32_t cap) {
  if (!h || !out) return SDSTREAM_E_INVALID_ARG;
  int rc = prof_drain(h);
  if (rc) return rc;
  int n = 0;
  for (int c = 0; c < PC_COUNT && n < cap; ++c) {
    if (!h->prof[c].launches) continue;
    out[n] = h->prof[c];
    strncpy(out[n].name, kProfNames[c], sizeof out[n].name - 1);
    out[n].name[sizeof out[n].name - 1] = 0;
    ++n;
  }
  return n;
}

int sdstream_use_graph(sdstream_t* h, int32_t on) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  h->graph_enabled = on != 0;
  return SDSTREAM_OK;
}

int sdstream_mfma_ceiling(sdstream_t* h, int32_t iters, double* tflops_out, void* hip_stream) {
  if (!h) return SDSTREAM_E_INVALID_ARG;
  if (!tflops_out || iters < 1 || iters > (1 << 20)) return fail(h, SDSTREAM_E_INVALID_ARG, "mfma_ceiling: iters in [1, 2^20] and an output pointer are required");
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0, cus = 0;
  HIP_TRY(h, hipGetDevice(&dev));
  HIP_TRY(h, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  int blocks = cus * 2;   // two 4-wave blocks per compute unit: two waves per SIMD
#ifdef SDSTREAM_DEVHOOKS
  if (const char* e = getenv("SDSTREAM_CEIL_BPC")) blocks = cus * atoi(e);
#endif
  float* sink = (float*)h->persist;   // only ever compared against, never written or read
  hipEvent_t e0, e1;
  HIP_TRY(h, hipEventCreate(&e0));
  HIP_TRY(h, hipEventCreate(&e1));
  launch_mfma_ceiling(iters, blocks, sink, s);   // warm-up: clocks, code load
  HIP_TRY(h, hipEventRecord(e0, s));
  launch_mfma_ceiling(iters, blocks, sink, s);
  HIP_TRY(h, hipEventRecord(e1, s));
  HIP_TRY(h, hipEventSynchronize(e1));
  float ms = 0.f;
  HIP_TRY(h, hipEventElapsedTime(&ms, e0, e1));
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  const double flops = (double)blocks * 4.0 * (double)iters * 8.0 * (2.0 * 16 * 16 * 32);
  *tflops_out = flops / ((double)ms * 1e-3) / 1e12;
  return SDSTREAM_OK;
}

}  // extern "C"
