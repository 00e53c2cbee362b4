// Stand-alone caller of the C ABI (include/jd_verify.h): plain C++ and the HIP runtime, no Python, no
// torch in the process.  Reads one verify call's tensors from raw files, runs it through
// jd_verify_create / jd_verify_run (or jd_verify_run_prenorm) / jd_verify_destroy, writes the outputs
// back as raw files.  The GPU test-suite compares those with the float64 oracle.
//
//   jd_cabi_check <dir> B M d V w_dtype mode        mode 0: jd_verify_run, 1: jd_verify_run_prenorm,
//                                                   2: jd_verify_run_noalloc (fp32 only, no context at all)
//
// Inputs in <dir> (little endian, dense): emb.bin or hidden.bin + gamma.bin (bf16 or fp32, as w_dtype
// implies), W.bin, w_judge.bin, w_scale.bin (8-bit weights only), draft_logits.bin (fp32 [B][M+1][V]),
// draft_tokens.bin (int32 [B][M]), uniforms.bin (fp32 [B][M+1]).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "../include/jd_verify.h"

#define CK(x)                                                              \
  do {                                                                     \
    hipError_t e_ = (x);                                                   \
    if (e_ != hipSuccess) {                                                \
      std::printf("%s: %s\n", #x, hipGetErrorString(e_));                  \
      return 2;                                                            \
    }                                                                      \
  } while (0)
#define JD(x)                                                                                              \
  do {                                                                                                     \
    int rc_ = (x);                                                                                         \
    if (rc_ != JD_OK) {                                                                                    \
      std::printf("%s: %d %s | %s\n", #x, rc_, jd_verify_strerror(rc_), jd_verify_last_error_detail());    \
      return 3;                                                                                            \
    }                                                                                                      \
  } while (0)

static std::string g_dir;

static bool read_file(const char* name, size_t bytes, std::vector<unsigned char>* out) {
  const std::string path = g_dir + "/" + name;
  std::FILE* f = std::fopen(path.c_str(), "rb");
  if (!f) { std::printf("cannot open %s\n", path.c_str()); return false; }
  out->resize(bytes);
  const size_t got = std::fread(out->data(), 1, bytes, f);
  const bool at_end = std::fgetc(f) == EOF;
  std::fclose(f);
  if (got != bytes || !at_end) { std::printf("%s: expected %zu bytes\n", path.c_str(), bytes); return false; }
  return true;
}

// file -> device buffer (nullptr on failure)
static void* upload(const char* name, size_t bytes) {
  std::vector<unsigned char> h;
  if (!read_file(name, bytes, &h)) return nullptr;
  void* d = nullptr;
  if (hipMalloc(&d, bytes) != hipSuccess) return nullptr;
  if (hipMemcpy(d, h.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return nullptr;
  return d;
}

static void* device_zeros(size_t bytes) {
  void* d = nullptr;
  if (hipMalloc(&d, bytes) != hipSuccess) return nullptr;
  if (hipMemset(d, 0, bytes) != hipSuccess) return nullptr;
  return d;
}

static bool download(const char* name, const void* d, size_t bytes) {
  std::vector<unsigned char> h(bytes);
  if (hipMemcpy(h.data(), d, bytes, hipMemcpyDeviceToHost) != hipSuccess) return false;
  const std::string path = g_dir + "/" + name;
  std::FILE* f = std::fopen(path.c_str(), "wb");
  if (!f) return false;
  const bool ok = std::fwrite(h.data(), 1, bytes, f) == bytes;
  return std::fclose(f) == 0 && ok;
}

int main(int argc, char** argv) {
  std::setvbuf(stdout, nullptr, _IONBF, 0);
  if (argc != 8) { std::printf("usage: %s <dir> B M d V w_dtype mode\n", argv[0]); return 1; }
  g_dir = argv[1];
  const int B = std::atoi(argv[2]), M = std::atoi(argv[3]), d = std::atoi(argv[4]), V = std::atoi(argv[5]);
  const int wdt = std::atoi(argv[6]);
  const int mode = std::atoi(argv[7]);
  const bool prenorm = mode == 1, noalloc = mode == 2;

  jd_verify_config c = {};
  c.d = d; c.V = V; c.max_B = B; c.max_M = M;
  c.w_dtype = wdt; c.emb_dtype = (wdt == JD_F32) ? JD_F32 : JD_BF16;
  c.w_layout = JD_W_VD; c.draft_kind = JD_DRAFT_LOGITS; c.mode = JD_MODE_JUDGE;
  c.temperature = 1.0f; c.delta = 0.5f; c.judge_bias = 0.0f; c.device = 0;
  c.rule = JD_RULE_SAMPLING; c.resample = JD_RESAMPLE_RESIDUAL;
  JD(jd_verify_validate_config(&c));   // shapes are checked on the host before anything touches the device

  const size_t R = (size_t)B * (M + 1), S = (size_t)B * M;
  const size_t esz = (wdt == JD_F32) ? 4 : 2;                                // embeddings, w_judge, gamma
  const size_t wsz = (wdt == JD_F32) ? 4 : (wdt == JD_BF16 ? 2 : 1);         // W_lm
  const bool scaled = wdt == JD_FP8_E4M3 || wdt == JD_INT8;

  CK(hipSetDevice(0));
  void* dW = upload("W.bin", (size_t)V * d * wsz);
  void* dJ = upload("w_judge.bin", (size_t)d * esz);
  void* dScale = scaled ? upload("w_scale.bin", (size_t)V * 4) : nullptr;
  void* dE = upload(prenorm ? "hidden.bin" : "emb.bin", R * d * esz);
  void* dG = prenorm ? upload("gamma.bin", (size_t)d * esz) : nullptr;
  void* dD = upload("draft_logits.bin", R * V * 4);
  void* dT = upload("draft_tokens.bin", S * 4);
  void* dU = upload("uniforms.bin", R * 4);
  if (!dW || !dJ || !dE || !dD || !dT || !dU || (scaled && !dScale) || (prenorm && !dG)) return 4;

  jd_verify_outputs o = {};
  o.d_accept_len = static_cast<int32_t*>(device_zeros(B * 4));
  o.d_next_token = static_cast<int32_t*>(device_zeros(B * 4));
  o.d_status = static_cast<uint32_t*>(device_zeros(B * 4));
  o.d_z_stand = static_cast<uint8_t*>(device_zeros(S));
  o.d_z_judge = static_cast<uint8_t*>(device_zeros(S));
  o.d_p_at_draft = static_cast<float*>(device_zeros(S * 4));
  o.d_q_at_draft = static_cast<float*>(device_zeros(S * 4));
  o.d_judge_logit = static_cast<float*>(device_zeros(S * 4));
  o.d_row_max = static_cast<float*>(device_zeros(R * 4));
  o.d_row_sumexp = static_cast<float*>(device_zeros(R * 4));
  if (!o.d_accept_len || !o.d_next_token || !o.d_status || !o.d_z_stand || !o.d_z_judge || !o.d_p_at_draft ||
      !o.d_q_at_draft || !o.d_judge_logit || !o.d_row_max || !o.d_row_sumexp) return 4;

  jd_verify_ctx* ctx = nullptr;
  if (!noalloc) {
    if (scaled) JD(jd_verify_create_scaled(&c, dW, static_cast<const float*>(dScale), dJ, &ctx));
    else JD(jd_verify_create(&c, dW, dJ, &ctx));
  }

  hipStream_t st;
  CK(hipStreamCreate(&st));   // default priority
  if (noalloc)   // no context: the workspace is the library's static device array
    JD(jd_verify_run_noalloc(&c, dW, dJ, B, M, dE, nullptr, static_cast<const int32_t*>(dT), static_cast<const float*>(dD),
                             M + 1, static_cast<const float*>(dU), &o, st));
  else if (prenorm)
    JD(jd_verify_run_prenorm(ctx, B, M, dE, dG, 1e-5, static_cast<const int32_t*>(dT), static_cast<const float*>(dD),
                             M + 1, static_cast<const float*>(dU), &o, st));
  else
    JD(jd_verify_run(ctx, B, M, dE, nullptr, static_cast<const int32_t*>(dT), static_cast<const float*>(dD), M + 1,
                     static_cast<const float*>(dU), &o, st));
  CK(hipStreamSynchronize(st));

  bool ok = download("accept_len.bin", o.d_accept_len, B * 4) && download("next_token.bin", o.d_next_token, B * 4) &&
            download("status.bin", o.d_status, B * 4) && download("z_stand.bin", o.d_z_stand, S) &&
            download("z_judge.bin", o.d_z_judge, S) && download("p_at_draft.bin", o.d_p_at_draft, S * 4) &&
            download("q_at_draft.bin", o.d_q_at_draft, S * 4) && download("judge_logit.bin", o.d_judge_logit, S * 4) &&
            download("row_max.bin", o.d_row_max, R * 4) && download("row_sumexp.bin", o.d_row_sumexp, R * 4);
  uint64_t ws = 0;
  if (ctx) JD(jd_verify_workspace_bytes(ctx, &ws));
  JD(jd_verify_destroy(ctx));
  CK(hipStreamDestroy(st));
  void* all[] = {dW, dJ, dScale, dE, dG, dD, dT, dU, o.d_accept_len, o.d_next_token, o.d_status, o.d_z_stand,
                 o.d_z_judge, o.d_p_at_draft, o.d_q_at_draft, o.d_judge_logit, o.d_row_max, o.d_row_sumexp};
  for (void* p : all)
    if (p) CK(hipFree(p));
  std::printf("jd_cabi_check: B=%d M=%d d=%d V=%d w_dtype=%d mode=%d workspace=%llu bytes %s\n", B, M, d, V, wdt,
              mode, (unsigned long long)ws, ok ? "ok" : "FAILED to write outputs");
  return ok ? 0 : 5;
}
