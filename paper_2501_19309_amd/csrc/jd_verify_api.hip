// C-ABI dispatcher of the verification head: argument validation, workspace, kernel
// selection by row count, optional per-kernel HIP-event timing.  See include/jd_verify.h
// for the contract of every entry point.
#include "../../include/jd_verify.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "jd_kernels.hpp"

using namespace jd;

struct jd_verify_ctx {
  jd_verify_config cfg;
  Geometry geo;
  const void* W;        // the caller's W_lm: kept (and read by every call) for fp32 weights only, else NULL
  const void* wj;
  void* Wp;             // re-tiled bf16 weights (bf16 weights only)
  void* Wp8;            // re-tiled one-byte codes (FP8 and INT8 weights)
  void* Wg8;            // re-tiled one-byte weights for the 352-row kernel (FP8 / INT8 weights, max_R > 176)
  const float* wscale;  // per-vocabulary-entry weight scale (FP8 and INT8 weights, may be NULL)
  float* L;             // [maxR][Vpad] fp32 logits
  float2* tpart;        // [maxR][nPartT]
  float2* dpart;        // [max_B*max_M][nPartD]
  float* t_max; float* t_sum; float* q_max; float* q_sum; float* g;
  double* chunk_mass;   // [max_B][nChunk] (the top-K rule reuses it as ints)
  int* rankpart;        // [max_B*max_M][kRankSplits], top-K rule only
  uint8_t* zflags;      // [maxR] per-slot test bits and error flags (row kernel -> sampler kernels)
  void* Xp;             // packed embeddings for the GEMM regime
  void* Xn;             // [max_R][d] normalised embeddings of the pre-norm entry point
  void* pool;           // one allocation behind tpart .. rankpart (see create)
  int nPartT, nPartD, nChunk;
  uint64_t bytes;
  float judge_threshold;
  // profiling
  bool prof_on;
  int prof_max, prof_n;
  std::vector<hipEvent_t> ev;  // (JD_NUM_KERNELS + 1) events per profiled call
};

static const int kDraftSplits = 16;   // column ranges per draft row in the statistics pass
static const int kF32Splits = 8;      // same for target logits on the fp32 path

// What the last failing HIP call of this thread was, for jd_verify_last_error_detail().
static thread_local char g_detail[320] = "";
static int hip_fail(const char* what, hipError_t e) {
  std::snprintf(g_detail, sizeof g_detail, "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
  (void)hipGetLastError();
  return e == hipErrorOutOfMemory ? JD_ERR_OOM : JD_ERR_HIP;
}
#define JD_HIP(expr) do { const hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_fail(#expr, e_); } while (0)
// Evaluates expr only while rc is still JD_OK: after a failed allocation nothing is launched on its (NULL) result.
#define JD_HIP_RC(expr) do { if (rc == JD_OK) { const hipError_t e_ = (expr); if (e_ != hipSuccess) rc = hip_fail(#expr, e_); } } while (0)

extern "C" const char* jd_verify_last_error_detail(void) { return g_detail; }

// ---- workspace of the entry point that allocates nothing (jd_verify_run_noalloc) ------------------
// Every device the library's code is loaded on holds its own copy of this array, at its own address, until
// the process ends.  On the host the name `scratch` is only a handle for hipGetSymbolAddress: the address a
// kernel can use is looked up once per device, with that device current, and kept in g_scratch[device].
// (No __attribute__((used)) here: the compiler keeps the array, and gives its device-side symbol the external
// linkage the runtime's look-up needs, because host code refers to it; with that attribute the symbol stays
// internal to the code object and the look-up ends the process.)
static __device__ __align__(256) unsigned char scratch[JD_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch[kMaxDevices];  // zero-initialised: not looked up yet

// Device address of `scratch` on `device`, which must be the calling thread's current device and a gfx950.
static int scratch_for_device(int device, unsigned char** out) {
  if (device < 0 || device >= kMaxDevices) return JD_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch[device]) {
    hipDeviceProp_t prop;
    JD_HIP(hipGetDeviceProperties(&prop, device));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
      std::snprintf(g_detail, sizeof g_detail, "device %d is %s; this library is built for gfx950 (MI355X) only",
                    device, prop.gcnArchName);
      return JD_ERR_HIP;
    }
    void* p = nullptr;
    JD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return hip_fail("hipGetSymbolAddress(scratch) returned NULL", hipErrorInvalidSymbol);
    g_scratch[device] = p;
  }
  *out = static_cast<unsigned char*>(g_scratch[device]);
  return JD_OK;
}

extern "C" const char* jd_verify_strerror(int code) {
  switch (code) {
    case JD_OK: return "ok";
    case JD_ERR_INVALID_ARG: return "invalid argument";
    case JD_ERR_SHAPE: return "shape out of range";
    case JD_ERR_UNSUPPORTED_DTYPE: return "unsupported dtype combination";
    case JD_ERR_OOM: return "out of device memory";
    case JD_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

extern "C" int jd_verify_validate_config(const jd_verify_config* c) {
  if (!c) return JD_ERR_INVALID_ARG;
  if (c->w_dtype != JD_F32 && c->w_dtype != JD_BF16 && c->w_dtype != JD_FP8_E4M3 && c->w_dtype != JD_INT8)
    return JD_ERR_INVALID_ARG;
  if (c->emb_dtype != JD_F32 && c->emb_dtype != JD_BF16) return JD_ERR_INVALID_ARG;
  if (c->w_layout != JD_W_VD && c->w_layout != JD_W_DV) return JD_ERR_INVALID_ARG;
  if (c->draft_kind != JD_DRAFT_LOGITS && c->draft_kind != JD_DRAFT_PROBS) return JD_ERR_INVALID_ARG;
  if (c->mode != JD_MODE_JUDGE && c->mode != JD_MODE_STANDARD) return JD_ERR_INVALID_ARG;
  if (!(c->temperature > 0.f) || !std::isfinite(c->temperature)) return JD_ERR_INVALID_ARG;
  if (!(c->delta >= 0.5f && c->delta <= 1.0f)) return JD_ERR_INVALID_ARG;
  if (!std::isfinite(c->judge_bias)) return JD_ERR_INVALID_ARG;
  if (c->device < 0) return JD_ERR_INVALID_ARG;
  if (c->rule != JD_RULE_SAMPLING && c->rule != JD_RULE_TOPK) return JD_ERR_INVALID_ARG;
  if (c->resample != JD_RESAMPLE_RESIDUAL && c->resample != JD_RESAMPLE_TARGET) return JD_ERR_INVALID_ARG;
  if (c->d <= 0 || c->V <= 0 || c->max_B <= 0 || c->max_M <= 0) return JD_ERR_SHAPE;
  if (c->max_M > 63) return JD_ERR_SHAPE;               // one wave64 ballot covers a sequence
  if (c->V > (1 << 30) || c->d > (1 << 20)) return JD_ERR_SHAPE;
  if ((int64_t)c->max_B * (c->max_M + 1) > (1 << 20)) return JD_ERR_SHAPE;
  if (c->rule == JD_RULE_TOPK && (c->top_k < 1 || c->top_k > c->V)) return JD_ERR_SHAPE;
  if (c->w_dtype == JD_FP8_E4M3 || c->w_dtype == JD_INT8) {
    if (c->emb_dtype != JD_BF16) return JD_ERR_UNSUPPORTED_DTYPE;
    if ((c->d % 16) != 0) return JD_ERR_SHAPE;
  } else if (c->w_dtype != c->emb_dtype) {
    return JD_ERR_UNSUPPORTED_DTYPE;
  }
  if (c->w_dtype == JD_BF16 && (c->d % 8) != 0) return JD_ERR_SHAPE;  // 128-bit operand loads
  return JD_OK;
}

// logit(delta) in double from the float the ABI carries, rounded once (near delta = 1 a float32 evaluation of
// delta / (1 - delta) is off by more than the judge logits' own precision); delta = 1 never accepts
static float judge_threshold_of(float delta) {
  return (delta >= 1.0f) ? INFINITY : (float)std::log((double)delta / (1.0 - (double)delta));
}

static void free_ctx(jd_verify_ctx* c) {
  if (!c) return;
  void* ptrs[] = {c->Wp, c->Wp8, c->Wg8, c->L, c->pool, c->Xp, c->Xn};  // tpart .. rankpart live inside pool
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  delete c;
}

template <typename T>
static int dev_alloc(jd_verify_ctx* c, T** p, size_t n) {
  const size_t bytes = (n ? n : 1) * sizeof(T);
  hipError_t e = hipMalloc(reinterpret_cast<void**>(p), bytes);
  if (e != hipSuccess) {
    *p = nullptr;
    return hip_fail("hipMalloc of workspace", e);
  }
  c->bytes += bytes;
  return JD_OK;
}

extern "C" int jd_verify_create(const jd_verify_config* cfg, const void* d_W_lm, const void* d_w_judge,
                                jd_verify_ctx** out_ctx) {
  return jd_verify_create_scaled(cfg, d_W_lm, nullptr, d_w_judge, out_ctx);
}

extern "C" int jd_verify_create_scaled(const jd_verify_config* cfg, const void* d_W_lm, const float* d_w_scale,
                                       const void* d_w_judge, jd_verify_ctx** out_ctx) {
  if (!out_ctx) return JD_ERR_INVALID_ARG;
  *out_ctx = nullptr;
  int rc = jd_verify_validate_config(cfg);
  if (rc != JD_OK) return rc;
  if (!d_W_lm || !d_w_judge) return JD_ERR_INVALID_ARG;
  if (d_w_scale && cfg->w_dtype != JD_FP8_E4M3 && cfg->w_dtype != JD_INT8) return JD_ERR_INVALID_ARG;

  int ndev = 0;
  JD_HIP(hipGetDeviceCount(&ndev));
  if (cfg->device >= ndev) return hip_fail("config.device is not a visible device", hipErrorInvalidDevice);
  JD_HIP(hipSetDevice(cfg->device));
  hipDeviceProp_t prop;
  JD_HIP(hipGetDeviceProperties(&prop, cfg->device));
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {   // the library holds gfx950 code only
    std::snprintf(g_detail, sizeof g_detail, "device %d is %s; this library is built for gfx950 (MI355X) only",
                  cfg->device, prop.gcnArchName);
    return JD_ERR_HIP;
  }
  {  // look up this device's copy of the no-allocation workspace now, so that a caller who has created a context
     // can use jd_verify_run_noalloc under stream capture; contexts themselves do not need it
    unsigned char* unused = nullptr;
    (void)scratch_for_device(cfg->device, &unused);
  }
  // The launchers report hipGetLastError(); a stale code left in this thread by an earlier, unrelated
  // runtime call of the caller (an event query that was "not ready", say) must not be taken for theirs.
  (void)hipGetLastError();

  jd_verify_ctx* c = new (std::nothrow) jd_verify_ctx();
  if (!c) return JD_ERR_OOM;
  c->cfg = *cfg;
  c->geo = make_geometry(cfg->d, cfg->V);
  c->W = d_W_lm; c->wj = d_w_judge; c->wscale = d_w_scale;
  c->judge_threshold = judge_threshold_of(cfg->delta);
  c->prof_on = false; c->prof_max = c->prof_n = 0;
  c->bytes = 0;

  const size_t maxR = (size_t)cfg->max_B * (cfg->max_M + 1);
  const size_t maxS = (size_t)cfg->max_B * cfg->max_M;
  const bool fp8 = cfg->w_dtype == JD_FP8_E4M3, int8 = cfg->w_dtype == JD_INT8;
  const bool bf16 = cfg->w_dtype == JD_BF16 || fp8 || int8;   // MFMA path (bf16 embeddings)
  c->nPartT = bf16 ? c->geo.nVG : kF32Splits;
  c->nPartD = kDraftSplits;
  c->nChunk = (cfg->V + kSamplerChunk - 1) / kSamplerChunk;

  rc = dev_alloc(c, &c->L, maxR * (size_t)c->geo.Vpad);
  if (rc == JD_OK) {
    // The small per-row arrays live side by side in ONE allocation: the kernels after the LM head are a
    // few microseconds each and walk chains of dependent loads, so every separate allocation they touch
    // is one more cold address translation on that chain.
    const bool topk = cfg->rule == JD_RULE_TOPK;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    const size_t o_tpart = take(maxR * (size_t)c->nPartT * sizeof(float2));
    const size_t o_dpart = take(maxS * (size_t)c->nPartD * sizeof(float2));
    const size_t o_tmax = take(maxR * sizeof(float)), o_tsum = take(maxR * sizeof(float));
    const size_t o_qmax = take(maxS * sizeof(float)), o_qsum = take(maxS * sizeof(float));
    const size_t o_g = take(maxS * sizeof(float));
    const size_t o_cm = take((size_t)cfg->max_B * c->nChunk * sizeof(double));
    const size_t o_rank = take(topk ? maxS * (size_t)kRankSplits * sizeof(int) : 0);
    const size_t o_zf = take(maxR);
    uint8_t* pool = nullptr;
    rc = dev_alloc(c, &pool, off);
    c->pool = pool;
    if (rc == JD_OK) {
      c->tpart = reinterpret_cast<float2*>(pool + o_tpart);
      c->dpart = reinterpret_cast<float2*>(pool + o_dpart);
      c->t_max = reinterpret_cast<float*>(pool + o_tmax); c->t_sum = reinterpret_cast<float*>(pool + o_tsum);
      c->q_max = reinterpret_cast<float*>(pool + o_qmax); c->q_sum = reinterpret_cast<float*>(pool + o_qsum);
      c->g = reinterpret_cast<float*>(pool + o_g);
      c->chunk_mass = reinterpret_cast<double*>(pool + o_cm);
      c->rankpart = topk ? reinterpret_cast<int*>(pool + o_rank) : nullptr;
      c->zflags = pool + o_zf;
    }
  }
  const bool w8 = fp8 || int8;
  if (rc == JD_OK && w8) {
    uint8_t* wp8 = nullptr;
    rc = dev_alloc(c, &wp8, c->geo.packed8_bytes());
    c->Wp8 = wp8;
    JD_HIP_RC(launch_pack_w8(d_W_lm, cfg->w_layout, c->geo, c->Wp8, nullptr));
    JD_HIP_RC(hipDeviceSynchronize());
  }
  // 8-bit contexts work from one-byte copies in every regime and hold no bf16 copy: Wp8 feeds the small-row and
  // the 176-row kernel, Wg8 (the same codes in the 352-row kernel's order) exists when that kernel can be chosen
  if (rc == JD_OK && bf16 && !w8) {
    uint8_t* wp = nullptr;
    rc = dev_alloc(c, &wp, c->geo.packed_bytes());
    c->Wp = wp;
    JD_HIP_RC(launch_pack_w(d_W_lm, cfg->w_layout, c->geo, c->Wp, nullptr));
    JD_HIP_RC(hipDeviceSynchronize());
  }
  if (rc == JD_OK && w8 && maxR > (size_t)kGemmRows) {
    uint8_t* wg8 = nullptr;
    rc = dev_alloc(c, &wg8, c->geo.packed8_bytes());
    c->Wg8 = wg8;
    JD_HIP_RC(launch_pack_w8g(d_W_lm, cfg->w_layout, c->geo, c->Wg8, nullptr));
    JD_HIP_RC(hipDeviceSynchronize());
  }
  if (rc == JD_OK && bf16 && maxR > 64) {
    JD_HIP_RC(init_lmhead_gemm());
    JD_HIP_RC(init_lmhead_gemm_dma());
  }
  if (rc == JD_OK && bf16 && maxR > 64) {
    uint8_t* xp = nullptr;
    rc = dev_alloc(c, &xp, gemm_xp_bytes((int)maxR, c->geo));
    c->Xp = xp;
  }
  if (rc == JD_OK) {
    uint8_t* xn = nullptr;
    rc = dev_alloc(c, &xn, maxR * (size_t)cfg->d * (cfg->emb_dtype == JD_BF16 ? 2 : 4));
    c->Xn = xn;
  }
  if (rc != JD_OK) { free_ctx(c); return rc; }
  // bf16 and 8-bit weights now live in the library's own re-tiled copies (the pack kernels have finished):
  // the caller's tensor is not read again and may be released
  if (bf16) c->W = nullptr;
  *out_ctx = c;
  return JD_OK;
}

extern "C" int jd_verify_destroy(jd_verify_ctx* ctx) {
  if (!ctx) return JD_OK;
  (void)hipSetDevice(ctx->cfg.device);
  (void)hipDeviceSynchronize();
  free_ctx(ctx);
  return JD_OK;
}

extern "C" int jd_verify_workspace_bytes(const jd_verify_ctx* ctx, uint64_t* out_bytes) {
  if (!ctx || !out_bytes) return JD_ERR_INVALID_ARG;
  *out_bytes = ctx->bytes;
  return JD_OK;
}

extern "C" int jd_verify_profile_begin(jd_verify_ctx* ctx, int32_t max_calls) {
  if (!ctx || max_calls <= 0 || max_calls > 4096) return JD_ERR_INVALID_ARG;
  const size_t need = (size_t)max_calls * (JD_NUM_KERNELS + 1);
  while (ctx->ev.size() < need) {
    hipEvent_t e;
    JD_HIP(hipEventCreate(&e));
    ctx->ev.push_back(e);
  }
  ctx->prof_on = true; ctx->prof_max = max_calls; ctx->prof_n = 0;
  return JD_OK;
}

extern "C" int jd_verify_profile_end(jd_verify_ctx* ctx, float* avg_ms, int32_t* n_calls) {
  if (!ctx || !avg_ms || !n_calls) return JD_ERR_INVALID_ARG;
  ctx->prof_on = false;
  double sum[JD_NUM_KERNELS] = {0, 0, 0, 0};
  for (int i = 0; i < ctx->prof_n; ++i) {
    hipEvent_t* e = &ctx->ev[(size_t)i * (JD_NUM_KERNELS + 1)];
    JD_HIP(hipEventSynchronize(e[JD_NUM_KERNELS]));
    for (int k = 0; k < JD_NUM_KERNELS; ++k) {
      float ms = 0.f;
      JD_HIP(hipEventElapsedTime(&ms, e[k], e[k + 1]));
      sum[k] += ms;
    }
  }
  for (int k = 0; k < JD_NUM_KERNELS; ++k) avg_ms[k] = ctx->prof_n ? (float)(sum[k] / ctx->prof_n) : 0.f;
  *n_calls = ctx->prof_n;
  ctx->prof_n = 0;
  return JD_OK;
}

// One verify call.  With d_hidden != NULL the LM-head input is the RMS-normalised d_hidden (written
// to the context's Xn) and the judge reads d_hidden itself; d_emb / d_emb_judge are then ignored.
static int run_impl(jd_verify_ctx* c, int32_t B, int32_t M, const void* d_emb, const void* d_emb_judge,
                    const void* d_hidden, const void* d_gamma, double rms_eps, const int32_t* d_draft_tokens,
                    const float* d_draft, int32_t draft_rows, const float* d_uniforms, const jd_verify_outputs* out,
                    void* hip_stream) {
  if (!c || (!d_emb && !d_hidden) || !d_draft_tokens || !d_draft || !d_uniforms || !out) return JD_ERR_INVALID_ARG;
  if (d_hidden && (!d_gamma || !(rms_eps >= 0.0) || !std::isfinite(rms_eps))) return JD_ERR_INVALID_ARG;
  if (!out->d_accept_len || !out->d_next_token || !out->d_status) return JD_ERR_INVALID_ARG;
  if (B < 1 || M < 1 || B > c->cfg.max_B || M > c->cfg.max_M) return JD_ERR_SHAPE;
  if (draft_rows != M && draft_rows != M + 1) return JD_ERR_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  (void)hipGetLastError();  // drop a stale code of the caller's own runtime calls (see create)
  const jd_verify_config& cfg = c->cfg;
  const Geometry& g = c->geo;
  const int R = B * (M + 1);
  const float invT = 1.0f / cfg.temperature;
  const bool fp8 = cfg.w_dtype == JD_FP8_E4M3, int8 = cfg.w_dtype == JD_INT8;
  const bool bf16 = cfg.w_dtype == JD_BF16 || fp8 || int8;
  const bool logits = cfg.draft_kind == JD_DRAFT_LOGITS;

  hipEvent_t* ev = nullptr;
  if (c->prof_on && c->prof_n < c->prof_max) ev = &c->ev[(size_t)(c->prof_n++) * (JD_NUM_KERNELS + 1)];
  if (ev) JD_HIP(hipEventRecord(ev[0], st));

  if (d_hidden) {  // pre-norm wiring: normalise for the LM head, judge on the hidden states as they are
    JD_HIP(launch_rmsnorm_rows(d_hidden, d_gamma, rms_eps, cfg.emb_dtype == JD_BF16, R, cfg.d, c->Xn, st));
    d_emb = c->Xn;
    d_emb_judge = d_hidden;
  }

  // Draft row statistics (first pass of the draft softmax) and the judge dot products do not
  // depend on the LM head.  In the small-row regime they ride in the LM-head launch as extra
  // workgroups; otherwise the statistics get a launch of their own and the judge dots are done
  // with the second softmax pass.
  const bool fused_side = bf16 && R <= 64;
  SideWork side;
  side.nStatBlocks = 0; side.nJudgeBlocks = 0;
  side.stats = make_rowstats_args(d_draft, M, (size_t)draft_rows * cfg.V, (size_t)cfg.V, cfg.V, c->nPartD, c->dpart);
  side.judge.emb_judge = d_emb_judge ? d_emb_judge : d_emb; side.judge.w_judge = c->wj;
  side.judge.emb_is_bf16 = cfg.emb_dtype == JD_BF16; side.judge.d = cfg.d; side.judge.M = M;
  side.judge.bias = cfg.judge_bias; side.judge.g = c->g;
  if (fused_side) {
    side.nStatBlocks = logits ? B * M * c->nPartD : 0;
    side.nJudgeBlocks = B * M;
  }

  // step 1: LM head (+ first softmax pass)
  if (bf16) {
    // 8-bit codes are converted to bf16 in registers by all three kernels (FP8: one instruction per two codes;
    // INT8: three, which the matrix-core-bound 352-row kernel cannot hide completely - it runs 4-8 % behind
    // the same kernel on bf16 weights and moves half the bytes)
    const bool w8 = fp8 || int8;
    const int wk = fp8 ? kWFp8 : int8 ? kWInt8 : kWBf16;
    if (R <= 64) {
      JD_HIP(launch_lmhead_skinny(w8 ? c->Wp8 : c->Wp, wk, c->wscale, d_emb, R, g, invT, c->L, c->tpart, side, st));
    } else if (gemm_uses_352(R)) {
      JD_HIP(launch_lmhead_gemm_dma(w8 ? c->Wg8 : c->Wp, wk, c->wscale, d_emb, R, g, invT, c->L, c->tpart, c->Xp, st));
    } else {
      JD_HIP(launch_lmhead_gemm(w8 ? c->Wp8 : c->Wp, wk, c->wscale, d_emb, R, g, invT, c->L, c->tpart, c->Xp, st));
    }
  } else {
    JD_HIP(launch_lmhead_f32(static_cast<const float*>(c->W), cfg.w_layout, static_cast<const float*>(d_emb), R,
                             cfg.d, cfg.V, invT, c->L, g.Vpad, st));
    JD_HIP(launch_rowstats(c->L, R, 1, (size_t)g.Vpad, 0, cfg.V, c->nPartT, c->tpart, st));
  }
  if (ev) JD_HIP(hipEventRecord(ev[1], st));

  // step 2: draft row statistics, when they did not ride beside the LM head
  if (logits && !fused_side)
    JD_HIP(launch_rowstats(d_draft, B * M, M, (size_t)draft_rows * cfg.V, (size_t)cfg.V, cfg.V, c->nPartD,
                           c->dpart, st));
  if (ev) JD_HIP(hipEventRecord(ev[2], st));

  // steps 3, 4 (and the second softmax pass): per-slot accept tests and judge
  const bool topk = cfg.rule == JD_RULE_TOPK;
  if (topk) JD_HIP(launch_rank(c->L, g.Vpad, d_draft_tokens, B, M, cfg.V, c->rankpart, st));
  AcceptArgs a;
  a.rule_topk = topk; a.top_k = cfg.top_k; a.rankpart = c->rankpart; a.nRankSplit = kRankSplits;
  a.B = B; a.M = M; a.d = cfg.d; a.V = cfg.V;
  a.emb_is_bf16 = cfg.emb_dtype == JD_BF16;
  a.draft_is_logits = logits; a.mode_judge = cfg.mode == JD_MODE_JUDGE;
  a.judge_done = fused_side;
  a.judge_threshold = c->judge_threshold; a.judge_bias = cfg.judge_bias;
  a.L = c->L; a.Lld = g.Vpad;
  a.tpart = c->tpart; a.nPartT = fused_side ? skinny_parts(g) : c->nPartT;  // the small-row launch hands over one partial per workgroup
  a.dpart = c->dpart; a.nPartD = c->nPartD;
  a.D = d_draft; a.draft_rows = draft_rows;
  a.tokens = d_draft_tokens; a.uniforms = d_uniforms;
  a.emb_judge = d_emb_judge ? d_emb_judge : d_emb; a.w_judge = c->wj;
  a.t_max = c->t_max; a.t_sum = c->t_sum; a.q_max = c->q_max; a.q_sum = c->q_sum; a.g = c->g;
  a.zflags = c->zflags;
  a.z_stand = out->d_z_stand; a.z_judge = out->d_z_judge;
  a.p_at = out->d_p_at_draft; a.q_at = out->d_q_at_draft; a.judge_logit = out->d_judge_logit;
  a.row_max = out->d_row_max; a.row_sumexp = out->d_row_sumexp;

  // steps 5-7: OR of the masks, accepted prefix, replacement / bonus token
  SamplerArgs s;
  s.B = B; s.M = M; s.V = cfg.V; s.draft_is_logits = logits;
  s.L = c->L; s.Lld = g.Vpad; s.D = d_draft; s.draft_rows = draft_rows; s.uniforms = d_uniforms;
  s.t_max = c->t_max; s.t_sum = c->t_sum; s.q_max = c->q_max; s.q_sum = c->q_sum;
  s.zflags = c->zflags; s.mode_judge = cfg.mode == JD_MODE_JUDGE;
  s.chunk_mass = c->chunk_mass; s.nChunk = c->nChunk;
  s.accept_len = out->d_accept_len; s.next_token = out->d_next_token; s.status = out->d_status;
  s.resample_target = cfg.resample == JD_RESAMPLE_TARGET;
  if (fused_side && !topk && M + 1 <= 16) {
    // Short drafts in the small-row regime: the row kernel and the sampler's first kernel as one launch (the judge
    // logits are in c->g).  Every sampler workgroup then recomputes the statistics of the sequence's M+1 rows,
    // 16 rows per pass: one pass is cheaper than a launch (M = 5: 7.9 us against 6.0 + 4.6 us and the gap
    // between them), two passes are not (M = 25: 11.1 us against 6.2 + 4.5 us).
    JD_HIP(launch_rows_mass(a, s, st));
    if (ev) JD_HIP(hipEventRecord(ev[3], st));
    JD_HIP(launch_sampler_pick(s, st));
  } else if (topk) {
    JD_HIP(launch_accept(a, st));
    if (ev) JD_HIP(hipEventRecord(ev[3], st));
    JD_HIP(launch_argmax(c->L, g.Vpad, c->t_max, c->zflags, s.mode_judge, out->d_accept_len, out->d_status, B, M, cfg.V,
                         reinterpret_cast<int*>(c->chunk_mass), c->nChunk, out->d_next_token, st));
  } else {
    JD_HIP(launch_accept(a, st));
    if (ev) JD_HIP(hipEventRecord(ev[3], st));
    JD_HIP(launch_sampler(s, st));
  }
  if (ev) JD_HIP(hipEventRecord(ev[4], st));

  if (out->d_probs) JD_HIP(launch_probs(c->L, g.Vpad, c->t_max, c->t_sum, R, cfg.V, out->d_probs, st));
  return JD_OK;
}

extern "C" int jd_verify_run(jd_verify_ctx* c, int32_t B, int32_t M, const void* d_emb, const void* d_emb_judge,
                             const int32_t* d_draft_tokens, const float* d_draft, int32_t draft_rows,
                             const float* d_uniforms, const jd_verify_outputs* out, void* hip_stream) {
  if (!d_emb) return JD_ERR_INVALID_ARG;
  return run_impl(c, B, M, d_emb, d_emb_judge, nullptr, nullptr, 0.0, d_draft_tokens, d_draft, draft_rows, d_uniforms,
                  out, hip_stream);
}

extern "C" int jd_verify_run_prenorm(jd_verify_ctx* c, int32_t B, int32_t M, const void* d_hidden, const void* d_gamma,
                                     double rms_eps, const int32_t* d_draft_tokens, const float* d_draft,
                                     int32_t draft_rows, const float* d_uniforms, const jd_verify_outputs* out,
                                     void* hip_stream) {
  if (!d_hidden) return JD_ERR_INVALID_ARG;
  return run_impl(c, B, M, nullptr, nullptr, d_hidden, d_gamma, rms_eps, d_draft_tokens, d_draft, draft_rows,
                  d_uniforms, out, hip_stream);
}

extern "C" int jd_verify_append_tokens(int32_t B, int32_t M, const int32_t* d_draft_tokens, const int32_t* d_accept_len,
                                       const int32_t* d_next_token, int32_t* d_token_buf, int32_t cap,
                                       int32_t* d_lengths, void* hip_stream) {
  if (!d_draft_tokens || !d_accept_len || !d_next_token || !d_token_buf || !d_lengths) return JD_ERR_INVALID_ARG;
  if (B < 1 || M < 1 || M > 63 || cap < 1) return JD_ERR_SHAPE;
  (void)hipGetLastError();  // drop a stale code of the caller's own runtime calls
  JD_HIP(launch_append_tokens(B, M, d_draft_tokens, d_accept_len, d_next_token, d_token_buf, cap, d_lengths,
                              static_cast<hipStream_t>(hip_stream)));
  return JD_OK;
}

// jd_verify_run for fp32 weights without a context: the workspace that jd_verify_create would allocate is laid
// out in the device's `scratch` array, the LM head reads the caller's W_lm in place, and the same kernels run.
extern "C" int jd_verify_run_noalloc(const jd_verify_config* cfg, const void* d_W_lm, const void* d_w_judge, int32_t B,
                                     int32_t M, const void* d_emb, const void* d_emb_judge,
                                     const int32_t* d_draft_tokens, const float* d_draft, int32_t draft_rows,
                                     const float* d_uniforms, const jd_verify_outputs* out, void* hip_stream) {
  int rc = jd_verify_validate_config(cfg);
  if (rc != JD_OK) return rc;
  if (!d_W_lm || !d_w_judge || !d_emb) return JD_ERR_INVALID_ARG;
  // bf16 and 8-bit weights are multiplied from a re-tiled copy, which only a context can hold
  if (cfg->w_dtype != JD_F32 || cfg->emb_dtype != JD_F32) return JD_ERR_UNSUPPORTED_DTYPE;
  if (B < 1 || M < 1 || B > cfg->max_B || M > cfg->max_M) return JD_ERR_SHAPE;

  // the workspace of THIS call (its B and M, not the config's maxima), carved out of the scratch array
  const Geometry geo = make_geometry(cfg->d, cfg->V);
  const size_t R = (size_t)B * (M + 1), S = (size_t)B * M;
  const int nChunk = (cfg->V + kSamplerChunk - 1) / kSamplerChunk;
  const bool topk = cfg->rule == JD_RULE_TOPK;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  const size_t o_L = take(R * (size_t)geo.Vpad * sizeof(float));
  const size_t o_tpart = take(R * (size_t)kF32Splits * sizeof(float2));
  const size_t o_dpart = take(S * (size_t)kDraftSplits * sizeof(float2));
  const size_t o_tmax = take(R * sizeof(float)), o_tsum = take(R * sizeof(float));
  const size_t o_qmax = take(S * sizeof(float)), o_qsum = take(S * sizeof(float));
  const size_t o_g = take(S * sizeof(float));
  const size_t o_cm = take((size_t)B * nChunk * sizeof(double));
  const size_t o_rank = take(topk ? S * (size_t)kRankSplits * sizeof(int) : 0);
  const size_t o_zf = take(R);
  if (off > (size_t)JD_NOALLOC_SCRATCH_BYTES) {
    std::snprintf(g_detail, sizeof g_detail, "jd_verify_run_noalloc: this call needs %zu bytes of workspace, the "
                  "static scratch array holds %zu", off, (size_t)JD_NOALLOC_SCRATCH_BYTES);
    return JD_ERR_SHAPE;
  }

  int cur = -1;
  JD_HIP(hipGetDevice(&cur));
  if (cur != cfg->device) {
    std::snprintf(g_detail, sizeof g_detail, "jd_verify_run_noalloc: current device is %d, config.device is %d", cur,
                  cfg->device);
    return JD_ERR_INVALID_ARG;
  }
  unsigned char* base = nullptr;
  rc = scratch_for_device(cfg->device, &base);
  if (rc != JD_OK) return rc;

  // a context on the host stack that owns nothing: run_impl only reads it
  jd_verify_ctx c;
  c.cfg = *cfg;
  c.cfg.max_B = B; c.cfg.max_M = M;
  c.geo = geo;
  c.W = d_W_lm; c.wj = d_w_judge; c.wscale = nullptr;
  c.Wp = c.Wp8 = c.Wg8 = c.Xp = c.Xn = c.pool = nullptr;
  c.L = reinterpret_cast<float*>(base + o_L);
  c.tpart = reinterpret_cast<float2*>(base + o_tpart);
  c.dpart = reinterpret_cast<float2*>(base + o_dpart);
  c.t_max = reinterpret_cast<float*>(base + o_tmax); c.t_sum = reinterpret_cast<float*>(base + o_tsum);
  c.q_max = reinterpret_cast<float*>(base + o_qmax); c.q_sum = reinterpret_cast<float*>(base + o_qsum);
  c.g = reinterpret_cast<float*>(base + o_g);
  c.chunk_mass = reinterpret_cast<double*>(base + o_cm);
  c.rankpart = topk ? reinterpret_cast<int*>(base + o_rank) : nullptr;
  c.zflags = base + o_zf;
  c.nPartT = kF32Splits; c.nPartD = kDraftSplits; c.nChunk = nChunk;
  c.bytes = 0;
  c.judge_threshold = judge_threshold_of(cfg->delta);
  c.prof_on = false; c.prof_max = c.prof_n = 0;
  return run_impl(&c, B, M, d_emb, d_emb_judge, nullptr, nullptr, 0.0, d_draft_tokens, d_draft, draft_rows, d_uniforms,
                  out, hip_stream);
}
