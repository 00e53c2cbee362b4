// LM-head projection for the small-row regime (R = B*(M+1) <= 64) on gfx950.
//
// Step 1 of verification (Sec. 3.1, Eq. 2): the target's final-layer embeddings of the
// M+1 positions go through the LM head; softmax of the result gives p_1..p_{M+1}.
// With a few dozen rows the contraction reads every weight once and reuses it R times:
// it is bound by streaming W_lm from HBM, so the kernel is organised around that stream.
//
//  * W_lm has been re-tiled (pack_w_kernel) so that one wavefront's operand fragment for
//    v_mfma_f32_16x16x32_bf16 is 1 KiB of consecutive memory: every load is a fully
//    coalesced 128-bit-per-lane load that lands directly in the MFMA A operand, with no
//    LDS round trip for the weights.
//  * A workgroup of NWAVES wavefronts owns NWAVES vocabulary groups of 64 rows; all of its
//    wavefronts share the embedding chunk, which is staged through LDS (XOR swizzled,
//    double buffered, one barrier per 256 hidden indices).
//  * Weight fragments are prefetched two K steps (8 KiB per wavefront) ahead into a
//    register double buffer.
//  * Epilogue: logits scaled by 1/T are written once as fp32 (the sampler needs one full
//    row per sequence later) and reduced on the fly to one (max, sum exp) partial per
//    (row, vocabulary group) - the first pass of the vocabulary softmax.
#include "jd_kernels.hpp"
#include "w8_frag.hpp"
#include "side_work.hpp"

namespace jd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#ifndef JD_PF
#define JD_PF 2
#endif
constexpr int kPF = JD_PF;  // K steps per weight prefetch group

// ------------------------------------------------------------------------------- pack

// One thread writes one 16-byte element of Wp (8 consecutive hidden indices of one row).
__global__ __launch_bounds__(256) void pack_w_kernel(const uint16_t* __restrict__ W, int layout, int V, int d, int KS,
                                                      int nVGalloc, size_t total, uint4* __restrict__ Wp) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int lane = (int)(idx & 63);
  int sub = (int)((idx >> 6) & 3);
  size_t t = idx >> 8;
  int ks, vg;
  wp_decode(t, nVGalloc, &vg, &ks);
  int v = vg * kVocabGroup + sub * 16 + (lane & 15);
  int k0 = ks * kKStep + (lane >> 4) * 8;
  union { uint4 q; uint16_t h[8]; } o;
  o.q = make_uint4(0u, 0u, 0u, 0u);
  if (v < V) {
    if (layout == 0) {
      if (k0 + 8 <= d && (d & 7) == 0) {
        o.q = *reinterpret_cast<const uint4*>(W + (size_t)v * d + k0);
      } else {
        for (int e = 0; e < 8; ++e)
          if (k0 + e < d) o.h[e] = W[(size_t)v * d + k0 + e];
      }
    } else {
      for (int e = 0; e < 8; ++e)
        if (k0 + e < d) o.h[e] = W[(size_t)(k0 + e) * V + v];
    }
  }
  Wp[idx] = o.q;
}

hipError_t launch_pack_w(const void* W, int layout, const Geometry& g, void* Wp, hipStream_t st) {
  if (!W || !Wp) return hipErrorInvalidValue;  // the kernel writes every element of Wp unconditionally
  const int KS = g.dpad / kKStep;
  const size_t total = (size_t)g.nVGalloc * KS * 256;
  const size_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_w_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint16_t*>(W), layout,
                     g.V, g.d, KS, g.nVGalloc, total, static_cast<uint4*>(Wp));
  return hipGetLastError();
}

// One thread writes one 16-byte element of Wp8: a row's codes for two consecutive K steps.
__global__ __launch_bounds__(256) void pack_w8_kernel(const uint8_t* __restrict__ W8, int layout, int V, int d,
                                                       int nVGalloc, size_t total, uint4* __restrict__ Wp8) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const int sub = (int)((idx >> 6) & 3);
  int vg, kp;
  wp8_decode(idx >> 8, nVGalloc, &vg, &kp);
  const int v = vg * kVocabGroup + sub * 16 + (lane & 15);
  union { uint4 q; uint8_t b[16]; } o;
  o.q = make_uint4(0u, 0u, 0u, 0u);
  if (v < V) {
    for (int s = 0; s < 2; ++s) {
      const int k0 = (2 * kp + s) * kKStep + (lane >> 4) * 8;
      for (int e = 0; e < 8; ++e)
        if (k0 + e < d) o.b[s * 8 + e] = (layout == 0) ? W8[(size_t)v * d + k0 + e] : W8[(size_t)(k0 + e) * V + v];
    }
  }
  Wp8[idx] = o.q;
}

hipError_t launch_pack_w8(const void* W8, int layout, const Geometry& g, void* Wp8, hipStream_t st) {
  if (!W8 || !Wp8) return hipErrorInvalidValue;
  const int KP = g.dpad / kKStep / 2;
  const size_t total = (size_t)g.nVGalloc * KP * 256;
  const size_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_w8_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint8_t*>(W8),
                     layout, g.V, g.d, g.nVGalloc, total, static_cast<uint4*>(Wp8));
  return hipGetLastError();
}

// ------------------------------------------------------------------------------- skinny

// LDS chunk layout: row-major [rows][32 x 16 B], 16-byte column index XOR (row & 15):
// conflict-free both for the staging writes (consecutive lanes, consecutive columns)
// and for the operand reads (consecutive lanes, consecutive rows, same column).
__device__ __forceinline__ int xs_index(int row, int c) { return row * (kKChunk / 8) + (c ^ (row & 15)); }

// WK = kWBf16: Wp holds bf16 fragments.  WK = kWFp8 / kWInt8: Wp holds one-byte codes (Wp8 layout), which
// are converted to bf16 in registers right before the MFMAs, and the logits are multiplied by the
// per-vocabulary-entry scale in the epilogue.  Everything else is shared.
template <int NXB, int NWAVES, int WK>
__global__ __launch_bounds__(NWAVES * 64) void lmhead_skinny_kernel(
    const uint4* __restrict__ Wp, const float* __restrict__ vscale, const uint16_t* __restrict__ X, int R, int d,
    int nChunks, int V, int nVG, int nVGalloc, float invT, float* __restrict__ L, int Lld,
    float2* __restrict__ part, int nLmBlocks, SideWork side) {
  constexpr int T = NWAVES * 64;
  constexpr int ROWS = NXB * 16;
  constexpr int ITEMS = ROWS * (kKChunk / 8);  // 16-byte items per staged chunk
  constexpr int IPT = ITEMS / T;               // items per thread
  static_assert(ITEMS % T == 0, "staging must divide evenly");
  // K steps per weight prefetch group: 2 for bf16 (8 KiB per wavefront in flight); 4 for FP8, whose
  // fragments are half the size, so that the same 8 KiB stay in flight
  constexpr bool W8 = WK != kWBf16;
  constexpr int PFS = W8 ? 2 * kPF : kPF;
  constexpr int GROUPS = kStepsPerChunk / PFS;
  static_assert(GROUPS % 2 == 0, "prefetch parity must be static");

  __shared__ uint4 xs[2][ITEMS];

  // Workgroups past the LM-head tiles carry the work that does not depend on the LM head
  // (draft row statistics, judge dot products); they fill slots the tiles leave free.
  if ((int)blockIdx.x >= nLmBlocks) {
    static_assert(NWAVES == 4, "side work is written for 256 threads");
    side_work_block(side, blockIdx.x - nLmBlocks, xs);
    return;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int n = lane & 15;   // MFMA column: embedding row inside a 16-row block
  const int gq = lane >> 4;  // MFMA K quarter / output row quad
  const int vg = blockIdx.x * NWAVES + wave;  // < nVGalloc by construction of the grid
  const int KS = nChunks * kStepsPerChunk;
  const int nGroupsTotal = KS / PFS;

  const uint4* wptr = Wp + (W8 ? wp8_group_offset(vg) : wp_group_offset(vg)) + lane;
  // 16-byte units: position of load i (of WS) of prefetch group g for sub-fragment `sub`.
  // bf16: one load per K step.  FP8: one load per pair of K steps (it carries both).
  constexpr int WS = W8 ? PFS / 2 : PFS;  // loads per (group, sub)
  auto w_offset = [&](int g, int i, int sub) -> size_t {
    if constexpr (W8) return wp8_pair_offset(g * WS + i, nVGalloc) + sub * 64;
    return wp_step_offset(g * PFS + i, nVGalloc) + sub * 64;
  };

  f32x4 acc[4][NXB];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int x = 0; x < NXB; ++x) acc[s][x] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 wbuf[2][WS][4];
  uint4 xreg[IPT];

  auto load_x = [&](int ch) {
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
      const int item = tid + i * T;
      const int row = item / (kKChunk / 8);
      const int c = item % (kKChunk / 8);
      const int k = ch * kKChunk + c * 8;
      // Branch-free on purpose: a load inside a branch makes the compiler's wait-count
      // tracking conservative and serialises the weight prefetch behind it.  Rows >= R
      // re-read row R-1 (their MFMA columns are never stored); hidden indices >= d
      // (padding of the last chunk) are zeroed when the registers are written to LDS.
      xreg[i] = *reinterpret_cast<const uint4*>(X + (size_t)min(row, R - 1) * d + min(k, d - 8));
    }
  };
  auto store_x = [&](int buf, int ch) {
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
      const int item = tid + i * T;
      const int c = item % (kKChunk / 8);
      const uint32_t keep = (ch * kKChunk + c * 8 < d) ? 0xffffffffu : 0u;
      const uint4 t = xreg[i];
      xs[buf][xs_index(item / (kKChunk / 8), c)] = make_uint4(t.x & keep, t.y & keep, t.z & keep, t.w & keep);
    }
  };

  // prologue: X chunk 0 into LDS, first weight group into registers
  load_x(0);
#pragma unroll
  for (int s = 0; s < WS; ++s)
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) wbuf[0][s][sub] = load_stream(wptr + w_offset(0, s, sub));
  store_x(0, 0);
  __syncthreads();

  for (int ch = 0; ch < nChunks; ++ch) {
    load_x(min(ch + 1, nChunks - 1));  // the last iteration re-stages its own chunk, unread
    __builtin_amdgcn_sched_barrier(0);
    const uint4* xcur = xs[ch & 1];
#pragma unroll
    for (int gi = 0; gi < GROUPS; ++gi) {
      // unconditional prefetch of the next group (the very last one re-reads itself)
      const int gnext = min(ch * GROUPS + gi + 1, nGroupsTotal - 1);
#pragma unroll
      for (int s = 0; s < WS; ++s)
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) wbuf[(gi + 1) & 1][s][sub] = load_stream(wptr + w_offset(gnext, s, sub));
      // keep the prefetch ahead of this group's MFMAs: without the fence the machine
      // scheduler sinks the loads next to their uses and the stream loses its depth
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < PFS; ++s) {
        const int c = (gi * PFS + s) * 4 + gq;
        bf16x8 bfrag[NXB];
#pragma unroll
        for (int x = 0; x < NXB; ++x) bfrag[x] = __builtin_bit_cast(bf16x8, xcur[xs_index(x * 16 + n, c)]);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          bf16x8 afrag;
          if constexpr (W8) {
            const uint4 w = wbuf[gi & 1][s / 2][sub];
            afrag = __builtin_bit_cast(bf16x8, (s & 1) == 0 ? w8x8_to_bf16x8<WK>(w.x, w.y) : w8x8_to_bf16x8<WK>(w.z, w.w));
          } else {
            afrag = __builtin_bit_cast(bf16x8, wbuf[gi & 1][s][sub]);
          }
#pragma unroll
          for (int x = 0; x < NXB; ++x)
            acc[sub][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag[x], acc[sub][x], 0, 0, 0);
        }
      }
    }
    store_x((ch + 1) & 1, min(ch + 1, nChunks - 1));
    __syncthreads();
  }

  // epilogue.  acc[sub][x][i] is logit of embedding row x*16 + n and vocabulary entry
  // vg*64 + sub*16 + gq*4 + i.  Every wavefront reduces its 64 vocabulary entries to one (max, sum exp) per
  // row; the four wavefronts' pairs are combined through LDS (the staging buffers are free: everybody is past
  // the last barrier of the loop), so that the launch hands over ONE softmax partial per (row, workgroup).
  const bool live = vg < nVG;  // a wavefront of padding groups contributes the empty partial
  float2* ps = reinterpret_cast<float2*>(&xs[0][0]);  // [NWAVES][ROWS]
  float osc[4][4];  // output scale of this lane's 16 vocabulary entries: (per-entry scale) / T
#pragma unroll
  for (int sub = 0; sub < 4; ++sub)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
      osc[sub][i] = (W8 && vscale != nullptr && v < V) ? vscale[v] * invT : invT;
    }
#pragma unroll
  for (int x = 0; x < NXB; ++x) {
    const int r = x * 16 + n;
    float vals[4][4];
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
        const float l = acc[sub][x][i] * osc[sub][i];
        vals[sub][i] = l;
        if (v < V) mx = fmaxf(mx, l);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    float sum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
        if (v < V) sum += __expf(vals[sub][i] - mx);
      }
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    if (live && r < R) {
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) {
        const int v0 = vg * kVocabGroup + sub * 16 + gq * 4;
        // non-temporal: the workgroups that finish early store while the others still stream weights, and
        // these stores disturb that stream least (4 us of 625 at d = 16384, 26 rows)
        store_stream(reinterpret_cast<float4*>(L + (size_t)r * Lld + v0), vals[sub][0], vals[sub][1], vals[sub][2], vals[sub][3]);
      }
    }
    if (gq == 0) ps[wave * ROWS + r] = live ? make_float2(mx, sum) : make_float2(-INFINITY, 0.f);
  }
  __syncthreads();
  if (tid < ROWS && tid < R) {
    MS st{-INFINITY, 0.f};
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {  // fixed order: the result does not depend on timing
      const float2 p = ps[w * ROWS + tid];
      st = ms_combine(st, MS{p.x, p.y});
    }
    part[(size_t)tid * nLmBlocks + blockIdx.x] = make_float2(st.m, st.s);
  }
}

template <int NXB, int NWAVES, int WK>
static hipError_t launch_skinny_t(const void* Wp, const float* vscale, const void* X, int R, const Geometry& g,
                                  float invT, float* L, float2* part, const SideWork& side, hipStream_t st) {
  const int nLm = (g.nVG + NWAVES - 1) / NWAVES;  // nLm*NWAVES <= nVGalloc since NWAVES divides kGroupAlloc
  const int grid = nLm + side.nStatBlocks + side.nJudgeBlocks;
  hipLaunchKernelGGL((lmhead_skinny_kernel<NXB, NWAVES, WK>), dim3(grid), dim3(NWAVES * 64), 0, st,
                     static_cast<const uint4*>(Wp), vscale, static_cast<const uint16_t*>(X), R, g.d,
                     g.dpad / kKChunk, g.V, g.nVG, g.nVGalloc, invT, L, g.Vpad, part, nLm, side);
  return hipGetLastError();
}

template <int WK>
static hipError_t launch_skinny_rows(const void* Wp, const float* vscale, const void* X, int R, const Geometry& g,
                                     float invT, float* L, float2* part, const SideWork& side, hipStream_t st) {
  if (R <= 16) return launch_skinny_t<1, 4, WK>(Wp, vscale, X, R, g, invT, L, part, side, st);
  if (R <= 32) return launch_skinny_t<2, 4, WK>(Wp, vscale, X, R, g, invT, L, part, side, st);
  if (R <= 48) return launch_skinny_t<3, 4, WK>(Wp, vscale, X, R, g, invT, L, part, side, st);
  return launch_skinny_t<4, 4, WK>(Wp, vscale, X, R, g, invT, L, part, side, st);
}

hipError_t launch_lmhead_skinny(const void* Wp, int w_code, const float* vscale, const void* X, int R,
                                const Geometry& g, float invT, float* L, float2* part, const SideWork& side,
                                hipStream_t st) {
  static_assert(kGroupAlloc % 4 == 0, "grid covers only allocated groups");
  if (R <= 0 || R > 64) return hipErrorInvalidValue;
  switch (w_code) {
    case kWBf16: return launch_skinny_rows<kWBf16>(Wp, nullptr, X, R, g, invT, L, part, side, st);
    case kWFp8: return launch_skinny_rows<kWFp8>(Wp, vscale, X, R, g, invT, L, part, side, st);
    case kWInt8: return launch_skinny_rows<kWInt8>(Wp, vscale, X, R, g, invT, L, part, side, st);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------------------- fp32

// One wavefront per vocabulary entry; lanes stride over the hidden dimension.
__global__ __launch_bounds__(256) void lmhead_f32_kernel(const float* __restrict__ W, int layout,
                                                          const float* __restrict__ X, int R, int d, int V,
                                                          float invT, float* __restrict__ L, int Lld) {
  const int lane = threadIdx.x & 63;
  const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (v >= V) return;
  for (int r0 = 0; r0 < R; r0 += 8) {
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int k = lane; k < d; k += 64) {
      const float w = (layout == 0) ? W[(size_t)v * d + k] : W[(size_t)k * V + v];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (r0 + i < R) acc[i] = fmaf(w, X[(size_t)(r0 + i) * d + k], acc[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float a = acc[i];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
      if (lane == 0 && r0 + i < R) L[(size_t)(r0 + i) * Lld + v] = a * invT;
    }
  }
}

hipError_t launch_lmhead_f32(const float* W, int layout, const float* X, int R, int d, int V, float invT, float* L,
                             int Lld, hipStream_t st) {
  hipLaunchKernelGGL(lmhead_f32_kernel, dim3((V + 3) / 4), dim3(256), 0, st, W, layout, X, R, d, V, invT, L, Lld);
  return hipGetLastError();
}

}  // namespace jd
