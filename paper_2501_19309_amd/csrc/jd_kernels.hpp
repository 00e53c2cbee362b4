// Internal launcher interface between the C-ABI dispatcher and the gfx950 kernels.
// Not part of the public boundary (that is include/jd_verify.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jd {

// 128-bit load of data that is read once per launch (the weight stream of a launch with a single row tile, the draft
// logits): marked non-temporal, so that the caches do not keep lines nobody comes back for.  A streaming read of 4 GB
// runs at 6.8-7.0 TB/s with these loads against 6.0-6.2 TB/s with plain ones (measured, 128-bit loads per lane).
typedef unsigned int jd_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const jd_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const jd_u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
typedef float jd_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4* p) {
  const jd_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const jd_f32x4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
// 128-bit non-temporal store, for results that the storing launch does not read back.
__device__ __forceinline__ void store_stream(float4* p, float a, float b, float c, float d) {
  const jd_f32x4 v = {a, b, c, d};
  __builtin_nontemporal_store(v, reinterpret_cast<jd_f32x4*>(p));
}

// ---- packed W_lm geometry --------------------------------------------------------
// The bf16 LM-head weight is re-tiled once, at context creation, into MFMA operand
// order for v_mfma_f32_16x16x32_bf16:
//
//   Wp[ks / 4][vg][ks % 4][sub][lane][8]      (bf16)
//
//   vg   : vocabulary group of 64 consecutive rows            (V padded to 64)
//   ks   : K step of 32 consecutive hidden indices            (d padded to kKChunk)
//   sub  : 16-row block inside the group, 0..3
//   lane : 0..63; lane holds row  vg*64 + sub*16 + lane%16,
//                 hidden indices  ks*32 + (lane/16)*8 + 0..7
//
// One (vg, ks, sub) fragment is 1 KiB and is exactly what one wavefront loads with a
// single 128-bit-per-lane instruction.  A wavefront that owns a group reads 16 KiB of
// consecutive memory per four K steps; these K-step quads are the slowest index, so the
// wavefronts of the whole chip, which advance through K together, read one compact
// window of memory that moves linearly through Wp (measured 2-3 % faster on the
// 405B-shaped head than giving every group its own contiguous stream).
constexpr int kVocabGroup = 64;
constexpr int kKStep = 32;
constexpr int kKChunk = 256;                 // hidden indices per LDS-staged X chunk
constexpr int kStepsPerChunk = kKChunk / kKStep;
constexpr int kGroupAlloc = 8;               // Wp is allocated for a multiple of this many groups

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Position of fragment block (vg, ks) in Wp in units of 16 bytes (one block = 4 sub-fragments
// x 64 lanes = 256 units): group part + step part.
constexpr int kWpKG = 4;  // K steps kept adjacent per group (16 KiB per wavefront; 2 -> 4 gained 2.6 % at d = 16384)
__host__ __device__ __forceinline__ size_t wp_group_offset(int vg) { return (size_t)vg * (kWpKG * 256); }
__host__ __device__ __forceinline__ size_t wp_step_offset(int ks, int nVGalloc) {
  return (size_t)(ks / kWpKG) * nVGalloc * (kWpKG * 256) + (size_t)(ks % kWpKG) * 256;
}
__host__ __device__ __forceinline__ void wp_decode(size_t blk, int nVGalloc, int* vg, int* ks) {
  const int s = (int)(blk % kWpKG);
  const size_t t = blk / kWpKG;
  *vg = (int)(t % (size_t)nVGalloc);
  *ks = (int)(t / (size_t)nVGalloc) * kWpKG + s;
}

struct Geometry {
  int d, V;
  int dpad;      // d rounded up to kKChunk
  int Vpad;      // V rounded up to kVocabGroup; also the row stride of the fp32 logits scratch
  int nVG;       // Vpad / 64
  int nVGalloc;  // nVG rounded up to kGroupAlloc (zero-filled tail groups)
  size_t packed_bytes() const { return (size_t)nVGalloc * kVocabGroup * (size_t)dpad * 2; }
  size_t packed8_bytes() const { return (size_t)nVGalloc * kVocabGroup * (size_t)dpad; }
};

inline Geometry make_geometry(int d, int V) {
  Geometry g;
  g.d = d; g.V = V;
  g.dpad = round_up(d, kKChunk);
  g.Vpad = round_up(V, kVocabGroup);
  g.nVG = g.Vpad / kVocabGroup;
  g.nVGalloc = round_up(g.nVG, kGroupAlloc);
  return g;
}

// Storage of W_lm as the LM-head kernels see it.
enum WCode : int { kWBf16 = 0, kWFp8 = 1, kWInt8 = 2 };

// ---- packed FP8 W_lm --------------------------------------------------------------
// FP8 E4M3 weights (one byte per weight, one fp32 scale per vocabulary entry) are re-tiled into
//
//   Wp8[ks / 8][vg][(ks % 8) / 2][sub][lane][16]      (bytes)
//
// where the 16 bytes of a lane are its eight codes for K step 2*kp (hidden indices
// (2kp)*32 + (lane/16)*8 + 0..7) followed by its eight codes for K step 2*kp+1: one 128-bit load
// feeds the MFMA A operands of two K steps after conversion to bf16 (exact: every E4M3 value
// is a bf16 value).  Eight K steps are adjacent per group so that a wavefront still reads 16 KiB
// of consecutive memory, as in the bf16 layout.
constexpr int kW8KG = 8;  // K steps kept adjacent per group in Wp8
__host__ __device__ __forceinline__ size_t wp8_group_offset(int vg) { return (size_t)vg * (kW8KG / 2 * 256); }
__host__ __device__ __forceinline__ size_t wp8_pair_offset(int kp, int nVGalloc) {
  return (size_t)(kp / (kW8KG / 2)) * nVGalloc * (kW8KG / 2 * 256) + (size_t)(kp % (kW8KG / 2)) * 256;
}
__host__ __device__ __forceinline__ void wp8_decode(size_t blk, int nVGalloc, int* vg, int* kp) {
  const int s = (int)(blk % (kW8KG / 2));
  const size_t t = blk / (kW8KG / 2);
  *vg = (int)(t % (size_t)nVGalloc);
  *kp = (int)(t / (size_t)nVGalloc) * (kW8KG / 2) + s;
}

// ---- work that can ride beside the LM head -------------------------------------------
struct RowStatsArgs {   // first softmax pass over fp32 rows, see rowstats_block
  const float* base; int rowsUsed; size_t seqStride, rowStride;
  int V, nSplit, splitLen; float2* part;
};
struct JudgeArgs {      // judge dot products, see judge_block
  const void* emb_judge; const void* w_judge; int emb_is_bf16, d, M; float bias; float* g;
};
struct SideWork {
  RowStatsArgs stats; int nStatBlocks;   // nRows * nSplit workgroups (0 = none)
  JudgeArgs judge; int nJudgeBlocks;     // B * M workgroups (0 = none)
};
RowStatsArgs make_rowstats_args(const float* base, int rowsUsed, size_t seqStride, size_t rowStride, int V,
                                int nSplit, float2* part);

// ---- launchers (all asynchronous on `st`) -----------------------------------------

// Re-tile bf16 W_lm ([V][d] if layout==0, [d][V] if layout==1) into Wp, zero padded.
hipError_t launch_pack_w(const void* W, int layout, const Geometry& g, void* Wp, hipStream_t st);

// Re-tile one-byte codes of W_lm (FP8 E4M3 or INT8) into Wp8 (see above), zero padded.
hipError_t launch_pack_w8(const void* W8, int layout, const Geometry& g, void* Wp8, hipStream_t st);

// Small-row regime LM head (R <= 64): streams Wp once, MFMA, writes fp32 logits
// L[r*Lld + v] = (x_r . w_v) * invT for r < R, v < Vpad, and one softmax partial
// (max, sum exp) per (row, workgroup of four vocabulary groups): part[r*skinny_parts(g) + wg].
// `side` (may be empty) is executed by extra workgroups of the same launch.
// w_code kWFp8 / kWInt8: Wp is Wp8 and vscale (fp32 per vocabulary entry, or NULL = 1) multiplies the logits.
inline int skinny_parts(const Geometry& g) { return (g.nVG + 3) / 4; }   // partials per row of that launch
hipError_t launch_lmhead_skinny(const void* Wp, int w_code, const float* vscale, const void* X, int R,
                                const Geometry& g, float invT, float* L, float2* part, const SideWork& side,
                                hipStream_t st);

// LM head of calls of one 176-row tile (64 < R <= kGemmRows): all rows x 256 vocabulary entries per
// workgroup; same outputs as the skinny launcher.  Xp is scratch for the re-tiled embeddings,
// gemm_xp_bytes(R, g) bytes.
constexpr int kGemmRowBlocks = 11;                 // 16-row MFMA blocks per row tile
constexpr int kGemmRows = kGemmRowBlocks * 16;     // 176
constexpr int kGemmKChunk = 128;                   // hidden indices per LDS-staged chunk
constexpr int kDmaRowBlocks = 22;                  // row tiles of up to 352 rows (two halves of up to 11 row blocks)
constexpr int kDmaRows = kDmaRowBlocks * 16;
constexpr int kDmaMinHalfBlocks = 6;               // fewest row blocks per half the 352-row kernel is instantiated for
// 16-row blocks per row half that hold rows in the last 352-row tile of an R-row launch: its rows are spread over
// both halves (half 1 starts at row dma_half_blocks * 16 of the tile), so that both row halves of a workgroup
// run equally long K steps.
inline int dma_half_blocks(int R) {
  const int last = R - (R - 1) / kDmaRows * kDmaRows;  // 1 .. 352 rows in the last tile
  const int b = (last + 31) / 32;
  return b < kDmaMinHalfBlocks ? kDmaMinHalfBlocks : b;
}
inline size_t gemm_xp_bytes(int R, const Geometry& g) {  // enough for either tiling
  return (size_t)((R + kDmaRows - 1) / kDmaRows) * kDmaRows * (size_t)g.dpad * 2;
}
// w_code kWFp8 / kWInt8: W is Wp8 (the one-byte copy of the small-row kernel) and vscale holds the per-entry scales;
// kWBf16: W is the bf16 Wp.
hipError_t launch_lmhead_gemm(const void* W, int w_code, const float* vscale, const void* X, int R, const Geometry& g,
                              float invT, float* L, float2* part, void* Xp, hipStream_t st);
// The same projection on row tiles of up to 352 rows x 256 entries with both operands shared through LDS: the
// kernel of every call of more than 176 rows (gemm_uses_352); its row tiles are sized to the call.
// w_code kWFp8 / kWInt8: W is Wg8, the one-byte copy that launch_pack_w8g builds (Geometry::packed8_bytes() bytes),
// and vscale holds the per-entry scales; kWBf16: W is the bf16 Wp.
hipError_t launch_lmhead_gemm_dma(const void* W, int w_code, const float* vscale, const void* X, int R,
                                  const Geometry& g, float invT, float* L, float2* part, void* Xp, hipStream_t st);
hipError_t launch_pack_w8g(const void* W8, int layout, const Geometry& g, void* Wg8, hipStream_t st);
// Once per process before the first launch of either kernel (they use more dynamic LDS than the default limit).
hipError_t init_lmhead_gemm();
hipError_t init_lmhead_gemm_dma();
inline bool gemm_uses_352(int R) {
  return R > kGemmRows;  // every call of more than one 176-row tile (the 352-row kernel sizes its row tiles to the call)
}
// Re-tile bf16 embeddings X[R][d] into MFMA fragment order Xp[rt][chunk][xb][s][lane][8] (row tiles of
// rowBlocks*16 rows, chunks of `steps` K steps), zero padded.
// halfBlocks == 0: block position xb of row tile rt holds rows rt*tileRows + xb*16 .. +15 (176-row kernel).
// halfBlocks > 0: a row tile is two halves of rowBlocks/2 positions, of which the first halfBlocks (row tile splitRt:
// splitHalfBlocks) hold rows, half h starting at row h*halfBlocks*16 of the tile (352-row kernel).
hipError_t launch_pack_x(const void* X, int R, int d, int nRowTiles, int nChunks, int rowBlocks, int steps, int tileRows,
                         int halfBlocks, int splitRt, int splitHalfBlocks, void* Xp, hipStream_t st);

// fp32 LM head (any layout), plain FMA; writes logits only.
hipError_t launch_lmhead_f32(const float* W, int layout, const float* X, int R, int d, int V, float invT,
                             float* L, int Lld, hipStream_t st);

// Row statistics of an fp32 matrix: for each of nRows rows (row i lives at
// base + (i / rowsUsed) * seqStride + (i % rowsUsed) * rowStride, V columns) and each
// of nSplit column ranges, part[i*nSplit + s] = (max, sum exp(x - max)).
hipError_t launch_rowstats(const float* base, int nRows, int rowsUsed, size_t seqStride, size_t rowStride,
                           int V, int nSplit, float2* part, hipStream_t st);

struct AcceptArgs {
  int B, M, d, V;
  int emb_is_bf16;
  int draft_is_logits, mode_judge;
  int judge_done;          // g[] already holds the judge logits
  int rule_topk, top_k;    // top-K rule: z_stand = rank(c) < top_k, rank from rankpart
  const int* rankpart; int nRankSplit;  // [B*M][nRankSplit] partial rank counts
  float judge_threshold;   // logit(delta), +inf for delta == 1
  float judge_bias;
  const float* L; int Lld;             // target logits scratch
  const float2* tpart; int nPartT;     // target softmax partials [R][nPartT]
  const float2* dpart; int nPartD;     // draft partials [B*M][nPartD] (logits kind only)
  const float* D; int draft_rows;      // draft tensor [B][draft_rows][V]
  const int32_t* tokens;               // [B][M]
  const float* uniforms;               // [B][M+1]
  const void* emb_judge;               // [B][M+1][d]
  const void* w_judge;                 // [d]
  // workspace written for the sampler
  float* t_max; float* t_sum;          // [R]
  float* q_max; float* q_sum;          // [B*M]
  float* g;                            // [B*M] judge logits
  uint8_t* zflags;                     // [R] test bits and error flags of every slot, for the sampler kernels
  // outputs
  uint8_t* z_stand; uint8_t* z_judge;
  float* p_at; float* q_at; float* judge_logit; float* row_max; float* row_sumexp;
};
// Second softmax pass, judge, both accept tests per slot (one launch; the OR, the ballot and the prefix cut are
// done by the sampler / argmax kernels from zflags).
hipError_t launch_accept(const AcceptArgs& a, hipStream_t st);

struct SamplerArgs {
  int B, M, V;
  int draft_is_logits;
  int resample_target;   // draw the replacement from p itself, not from the residual
  const float* L; int Lld;
  const float* D; int draft_rows;
  const float* uniforms;
  const float* t_max; const float* t_sum; const float* q_max; const float* q_sum;
  const uint8_t* zflags; int mode_judge;   // per-slot test bits of launch_accept; z = stand OR (mode_judge AND judge)
  double* chunk_mass; int nChunk;      // [B][nChunk]
  int32_t* accept_len; int32_t* next_token; uint32_t* status;   // outputs: prefix, new token, JD_STATUS_* bits
};
constexpr int kSamplerChunk = 1024;     // tokens per sampler chunk
hipError_t launch_sampler(const SamplerArgs& a, hipStream_t st);
// Small-row regime with the judge logits already in a.g (sampling rule only): launch_accept and the first of the
// sampler's two kernels as ONE launch, followed by launch_sampler_pick.
hipError_t launch_rows_mass(const AcceptArgs& a, const SamplerArgs& s, hipStream_t st);
hipError_t launch_sampler_pick(const SamplerArgs& a, hipStream_t st);

// Top-K rule (Sec. 5): partial counts of the tokens that rank before the drafted one in its
// target row (larger logit, or equal logit and lower id): rankpart[(b*M+j)*nSplit + s].
constexpr int kRankSplits = 16;
hipError_t launch_rank(const float* L, int Lld, const int32_t* tokens, int B, int M, int V, int* rankpart,
                       hipStream_t st);

// Greedy new token for the top-K rule: accepted prefix from zflags (written to accept_len, status), then
// next_token[b] = lowest id attaining the maximum of that row of the target logits.  `chunk_arg` is
// [B][nChunk] ints of scratch.
hipError_t launch_argmax(const float* L, int Lld, const float* t_max, const uint8_t* zflags, int mode_judge,
                         int32_t* accept_len, uint32_t* status, int B, int M, int V, int* chunk_arg, int nChunk,
                         int32_t* next_token, hipStream_t st);

// Final RMS normalisation of R rows of d values (Sec. 4.1: the LM head reads the embedding after it):
// Xn[r][k] = round(H[r][k] * gamma[k] / sqrt(mean_k H[r][k]^2 + eps)), float64 arithmetic, one
// round-to-nearest-even to the storage type (bf16 bit patterns, or fp32 when !is_bf16).
hipError_t launch_rmsnorm_rows(const void* H, const void* gamma, double eps, int is_bf16, int R, int d, void* Xn,
                               hipStream_t st);

// Append the accepted draft tokens and the new token of every sequence to its token buffer
// (Sec. 3.1, after Eq. 4); one wavefront per sequence.
hipError_t launch_append_tokens(int B, int M, const int32_t* draft_tokens, const int32_t* accept_len,
                                const int32_t* next_token, int32_t* token_buf, int cap, int32_t* lengths,
                                hipStream_t st);

// probs[r*V + v] = exp(L[r*Lld + v] - t_max[r]) / t_sum[r]
hipError_t launch_probs(const float* L, int Lld, const float* t_max, const float* t_sum, int R, int V,
                        float* probs, hipStream_t st);

}  // namespace jd
