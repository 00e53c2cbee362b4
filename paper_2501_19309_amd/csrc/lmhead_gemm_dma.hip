// LM-head projection for calls of more than 176 rows, row tiles of up to 352 rows (Sec. 3.1, Eq. 2 for
// all rows of a batch), gfx950.  Same contract as the 176-row kernel next door.  704 rows (B=64, M=10) are two
// full tiles; other row counts get row tiles sized to the call (dma_plan below): a tile's rows are spread over
// its two row halves, and only the 16-row blocks that hold rows are loaded and multiplied.
//
// Why a second tiling.  With one 176 x 256 tile per workgroup the compute units request
// 27 KiB of operands from L2 per 704 matrix-core cycles, which is about what the
// texture/L1 path of a compute unit sustains for this access pattern (measured: 64 B/clk
// for pure L2 hits, about half of that when a quarter of the lines come from HBM) - the
// loads, not the MFMAs, set the pace.  Here a workgroup owns 352 rows x 256 vocabulary
// entries, both operands are fetched once per workgroup and shared through LDS, and the
// requests drop to 38 KiB per 1408 cycles (0.70 x per flop).
//
//   * 4 wavefronts (one per SIMD) as 2 (row halves) x 2 (vocabulary halves); each owns
//     176 x 128 = 11 x 8 accumulator tiles of v_mfma_f32_16x16x32_bf16 = 352 registers:
//     60 tiles live in accumulation registers, the other 28 in ordinary vector registers
//     (the MFMA takes either).
//   * operands travel HBM/L2 -> LDS by direct-to-LDS loads (global_load_lds_dwordx4: no
//     staging registers, no LDS-write instructions).  One K step (32 hidden indices) is
//     one stage of 38 KiB (22 KiB embeddings in fragment order + 16 KiB weights, which the
//     re-tiled W_lm already holds in fragment order); four stages = 152 KiB of LDS, so a
//     stage is requested three K steps (~2 us) before it is read.
//   * per K step a wavefront issues 88 MFMAs (8 per row block that holds rows), 19 conflict-free
//     ds_read_b128 (11 embedding fragments, refilled in place right after their row block, 8 weight
//     fragments into the other half of a double buffer), 9-10 direct-to-LDS loads and one barrier, each
//     placed alone behind an MFMA of its own.
//   * direct-to-LDS loads are written as inline assembly: the compiler then neither knows
//     nor waits for them, and the kernel counts them itself (they complete in issue order):
//     before the barrier of step k a wavefront waits until only its loads for steps k+2 and
//     k+3 are outstanding.  The barrier then says two things at once: every wavefront's
//     part of stage k+1 has landed, and nobody reads stage k any more (its operands are in
//     registers), so stage k is re-filled for step k+4.
#include <type_traits>

#include "w8_frag.hpp"
#include "jd_kernels.hpp"

namespace jd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;
constexpr int kDmaWaveRowBlocks = kDmaRowBlocks / 2;                    // 11 row blocks per wavefront
constexpr int kDmaStages = 4;
constexpr int kDmaXItems = kDmaRowBlocks * 64;                          // 16-byte items: 22 KiB of embeddings
// weights of one K step: 4 groups x 4 sub-blocks, 16 KiB as bf16 fragments, 8 KiB as FP8 fragments
template <bool W8> constexpr int kDmaWItems = W8 ? 8 * 64 : 16 * 64;
template <bool W8> constexpr int kDmaStageItems = kDmaXItems + kDmaWItems<W8>;      // 38 KiB (30 KiB) per K step
template <bool W8> constexpr size_t kDmaLdsBytes = (size_t)kDmaStages * kDmaStageItems<W8> * sizeof(uint4);  // 152 (120) KiB
// Tile (row block x, weight sub-block sb) lives in accumulation registers for the first 60 tiles (240 of the
// 256 registers) and in ordinary vector registers for the other 28.  Filling all 256 leaves the register
// allocator no room: it then parks values in scratch memory around the epilogue, reading tiles before the wait
// that protects them.
__host__ __device__ constexpr bool acc_in_agpr(int x, int sb) { return x < 7 || (x == 7 && sb < 4); }
static_assert(kDmaWaveRowBlocks == 11, "piece assignment and wait counts below assume 22 row blocks");

// acc += A * B in place; the accumulator is tied to an accumulation register (ACC) or to an
// ordinary vector register.  Inline assembly keeps all 88 tiles where they are (left to the
// register allocator they are copied around every iteration).  Hazards the compiler no longer
// sees: two MFMAs on one tile are 87 MFMAs apart, and the epilogue waits before reading.
template <bool ACC>
__device__ __forceinline__ void mfma_inplace(f32x4& acc, const uint4& a, const uint4& b) {
  const u32x4 av = __builtin_bit_cast(u32x4, a);
  const u32x4 bv = __builtin_bit_cast(u32x4, b);
  if constexpr (ACC)
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(av), "v"(bv));
  else
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(av), "v"(bv));
}

// f(integral_constant<int, I>) for I = 0 .. N-1, in order
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// One direct-to-LDS load: lane l of the wavefront copies 16 bytes from gsrc + l*16 to LDS byte
// address lds_byte + l*16 (M0 carries the wavefront's LDS base).  The compiler uses M0 for
// nothing else in this kernel.
__device__ __forceinline__ void dma_1k(const uint4* gsrc, unsigned lds_byte, unsigned lane16) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_byte), "v"(lane16), "s"(gsrc) : "memory");
}

// The same in two instructions that the caller places at least one instruction apart (a write of M0
// needs a wait state before the load that uses it).
__device__ __forceinline__ void set_m0(unsigned lds_byte) { asm volatile("s_mov_b32 m0, %0" ::"s"(lds_byte)); }
__device__ __forceinline__ void dma_issue(const uint4* gbase, unsigned lane_off) {
  asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(gbase) : "memory");
}

// WK = kWBf16: Wsrc is the re-tiled bf16 copy Wp.  WK = kWFp8, kWInt8: Wsrc is the one-byte copy Wg8 (see
// pack_w8g_kernel): half the weight bytes through L2, L1 and LDS; fragments are converted to bf16 in registers
// behind MFMAs that carry nothing else, one K step ahead (one instruction per two FP8 codes, three per two INT8
// codes); the per-entry scale is applied in the epilogue.
// Which weight sub-block (0..7) of the next K step a bf16 tile reads behind MFMA (row block x, sub-block sb); -1: none.
constexpr int dma_wf_slot(int x, int sb, int nlive) {
  if (sb == 3 && x >= 1 && x <= 8 && x <= nlive - 1) return x - 1;
  if (sb == 7 && x >= 1 && (nlive - 1) + (x - 1) < 8) return (nlive - 1) + (x - 1);
  return -1;
}
// Which direct-to-LDS piece has its M0 write (2*p) or its load (2*p + 1) behind MFMA (x, sb); -1: none.
constexpr int dma_piece_slot(int x, int sb, int nlive, int pieces) {
  if (x < 1) return -1;
  if ((sb == 5 || sb == 6) && x <= pieces && x <= nlive - 1) return 2 * (x - 1) + (sb == 6);
  if ((sb == 2 || sb == 4) && (nlive - 1) + (x - 1) < pieces) return 2 * ((nlive - 1) + (x - 1)) + (sb == 4);
  return -1;
}

// One tile: rows rt*tileRows .. and vocabulary entries vt*256 .. +255.  NLIVE = 16-row blocks per row half that hold
// rows (11 for a full tile of 352 rows; a smaller or ragged tile spreads its rows over both halves, NLIVE blocks each,
// half 1 starting at row NLIVE*16 of the tile).  Blocks beyond NLIVE are neither loaded nor multiplied: a K step is
// 8*NLIVE MFMAs long.  (Non-temporal weight loads for calls with a single row tile were measured: 0.376 -> 0.372 ms at
// 187 rows, within the noise elsewhere; not kept.)
template <int WK, int NLIVE>
__device__ __forceinline__ void dma_tile(
    const uint4* __restrict__ Wsrc, const float* __restrict__ vscale, const uint4* __restrict__ Xp, int R, int KS,
    int V, int nVG, int nVGalloc, float invT, float* __restrict__ L, int Lld, float2* __restrict__ part, const int rt,
    const int vt, const int tileRows) {
  constexpr bool W8 = WK != kWBf16;
  static_assert(NLIVE >= kDmaMinHalfBlocks && NLIVE <= kDmaWaveRowBlocks, "instantiated tiles");
  constexpr int kStageItems = kDmaStageItems<W8>;
  constexpr int kNW = W8 ? 2 : 4;            // direct-to-LDS loads of weights per wavefront and K step
  constexpr int PXhi = (NLIVE + 1) / 2;      // embedding row blocks per K step of wavefronts 0, 1 (2*NLIVE dealt to four)
  constexpr int PXlo = NLIVE / 2;            // ... of wavefronts 2, 3
  constexpr int kPieces = kNW + PXhi;
  extern __shared__ uint4 lds[];  // kDmaStages stages of [22 x 64 embedding items][weight items]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rh = wave >> 1, vh = wave & 1;  // row half, vocabulary half
  const int n = lane & 15;
  const int gq = lane >> 4;
  const unsigned lane16 = (unsigned)lane * 16u;
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)lds;

  // direct-to-LDS sources of this wavefront: the weights of vocabulary group vt*4 + wave (< nVGalloc,
  // allocated in multiples of 8 groups; 4 KiB per K step as bf16, 2 KiB as FP8), and the embedding row
  // blocks number wave, wave+4, .. of the 2*NLIVE that hold rows (block (rh, x) sits at position rh*11 + x
  // of a K step, in Xp and in the stage alike)
  const uint4* wsrc0 = W8 ? Wsrc + (size_t)(vt * 4 + wave) * 128 : Wsrc + wp_group_offset(vt * 4 + wave);
  const size_t wStep8 = (size_t)nVGalloc * 128;  // FP8: 16-byte items between consecutive K steps
  const uint4* xsrc0 = Xp + (size_t)rt * KS * kDmaRowBlocks * 64;
  const bool more = (NLIVE % 2 == 0) || wave < 2;  // NLIVE odd: wavefronts 0, 1 own one row block more than 2, 3
  const unsigned ldsW0 = lds0 + (unsigned)(kDmaXItems + wave * kNW * 64) * 16;
  unsigned xblk[PXhi];  // position of this wavefront's q-th row block (wave-uniform)
#pragma unroll
  for (int q = 0; q < PXhi; ++q) {
    const int li = min(wave + 4 * q, 2 * NLIVE - 1);
    xblk[q] = (unsigned)((li / NLIVE) * kDmaWaveRowBlocks + li % NLIVE);
  }

  // Wait until at most `groups` K steps of this wavefront's direct-to-LDS loads are outstanding and all
  // its LDS reads have returned.  With NLIVE odd, wavefronts 0, 1 issue one load more per step than 2, 3; loads
  // complete in issue order, so the count for the smaller number is right for both (0, 1 then also wait
  // for the first one or two loads of the following, much older, step).
  auto wait_groups = [&](auto gc) {
    constexpr int g = decltype(gc)::value;
    constexpr int outstanding = g * (kNW + PXlo);
    static_assert(outstanding < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(outstanding) : "memory");
  };
  static_assert(NLIVE != kDmaWaveRowBlocks || (3 * (kNW + PXlo) == (W8 ? 21 : 27) && 2 * (kNW + PXlo) == (W8 ? 14 : 18)),
                "full tiles: 27 / 18 loads (bf16), 21 / 14 (one-byte weights)");

  f32x4 acc[8][kDmaWaveRowBlocks];
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int x = 0; x < NLIVE; ++x) acc[s][x] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 xf[kDmaWaveRowBlocks];  // embedding fragments of the current K step, refilled in place
  uint4 wf[2][8];               // weight fragments (bf16): current step / next step
  uint2 raw[8];                 // FP8 only: codes of the next step's fragments on their way into wf

  // prologue: request K steps 0..3 (KS >= 8), wait for step 0, read its operands
#pragma unroll
  for (int s = 0; s < kDmaStages; ++s) {
    const unsigned dst = (unsigned)s * (kStageItems * 16);
    const uint4* wg = W8 ? wsrc0 + (size_t)s * wStep8 : wsrc0 + wp_step_offset(s, nVGalloc);
    const uint4* xg = xsrc0 + (size_t)s * (kDmaRowBlocks * 64);
#pragma unroll
    for (int p = 0; p < kNW; ++p) dma_1k(wg + p * 64, ldsW0 + dst + p * 1024, lane16);
#pragma unroll
    for (int q = 0; q < PXhi; ++q)
      if (q < PXlo || more) dma_1k(xg + xblk[q] * 64, lds0 + dst + xblk[q] * 1024, lane16);
  }
  wait_groups(std::integral_constant<int, 3>{});
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  {
    const uint4* xr = lds + rh * kDmaWaveRowBlocks * 64 + lane;
#pragma unroll
    for (int x = 0; x < NLIVE; ++x) xf[x] = xr[x * 64];
    if constexpr (W8) {
      const uint2* wr = reinterpret_cast<const uint2*>(lds + kDmaXItems) + vh * 8 * 64 + lane;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const uint2 c = wr[s * 64];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) set_dword(wf[0][s], jj, w8_frag_dword<WK>(c.x, c.y, jj));
      }
    } else {
      const uint4* wr = lds + kDmaXItems + vh * 8 * 64 + lane;
#pragma unroll
      for (int s = 0; s < 8; ++s) wf[0][s] = wr[s * 64];
    }
  }

  // K step k = 4*kk + ST; the stage index ST is a compile-time constant.  The wavefront's instruction
  // stream is written out MFMA by MFMA: with one wavefront per SIMD nothing else can fill the matrix
  // pipeline while this wavefront issues other instructions, and an MFMA leaves room for about three
  // of them, so every LDS read, M0 write, direct-to-LDS load and pair of conversion instructions sits
  // alone behind its own MFMA.
  auto k_step = [&](const uint4* wIter, const uint4* xIter, auto stc) {
    constexpr int ST = decltype(stc)::value;
    constexpr int cur = ST & 1, nxt = cur ^ 1;
    constexpr int RS = (ST + 1) % kDmaStages;  // stage of step k+1: read after the barrier
    constexpr unsigned stageByte = (unsigned)ST * (kStageItems * 16);
    const uint4* xr = lds + RS * kStageItems + rh * kDmaWaveRowBlocks * 64 + lane;
    const uint4* wr = lds + RS * kStageItems + kDmaXItems + vh * 8 * 64 + lane;                              // bf16
    const uint2* wr8 = reinterpret_cast<const uint2*>(lds + RS * kStageItems + kDmaXItems) + vh * 8 * 64 + lane;  // FP8
    // requested now: step k+4 into the stage this step frees (wIter, xIter: its group of four steps).
    // In the last group step k itself is requested again into its own, already consumed stage
    // (branch-free, unread).
    const uint4* wg = W8 ? wIter + (size_t)ST * wStep8 : wIter + ST * 256;
    const uint4* xg = xIter + ST * (kDmaRowBlocks * 64);
    static_for<0, 8 * NLIVE>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      constexpr int x = i / 8, sb = i % 8;  // row block, weight sub-block
      mfma_inplace<acc_in_agpr(x, sb)>(acc[sb][x], wf[cur][sb], xf[x]);
      if constexpr (i == 7) {
        // stage k+1 complete for this wavefront's part; after the barrier for everybody's,
        // and stage k (= ST) is free: all its fragments were read during step k-1
        wait_groups(std::integral_constant<int, 2>{});
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");  // no LDS read moves above the barrier
      }
      if constexpr (x >= 1 && sb == 1) xf[x - 1] = xr[(x - 1) * 64];  // row block x-1 of step k+1, in place
      if constexpr (i == 8 * NLIVE - 1) xf[x] = xr[x * 64];
      if constexpr (W8) {
        // weight sub-block x-1 of step k+1: codes read behind MFMA (x, 0), converted behind MFMAs (x+1, 2..5),
        // so that every MFMA of the step has at most one vector, LDS or memory instruction behind it
        if constexpr (NLIVE >= 10) {
          if constexpr (x >= 2 && x <= 9 && sb >= 2 && sb <= 5) set_dword(wf[nxt][x - 2], sb - 2, w8_frag_dword<WK>(raw[x - 2].x, raw[x - 2].y, sb - 2));
          if constexpr (x >= 1 && x <= 8 && sb == 0) raw[x - 1] = wr8[(x - 1) * 64];
        } else {
          // fewer than ten row blocks: codes of sub-blocks 2(x-1), 2(x-1)+1 read behind MFMAs (x, 0), (x, 7) for
          // x = 1..4, two fragment dwords converted behind each of MFMAs (x, 2..5) for x = 2..5
          if constexpr (x >= 1 && x <= 4 && sb == 0) raw[2 * (x - 1)] = wr8[(2 * (x - 1)) * 64];
          if constexpr (x >= 1 && x <= 4 && sb == 7) raw[2 * (x - 1) + 1] = wr8[(2 * (x - 1) + 1) * 64];
          if constexpr (x >= 2 && x <= 5 && sb >= 2 && sb <= 5) {
            constexpr int c0 = 2 * ((x - 2) * 4 + (sb - 2)), c1 = c0 + 1;
            set_dword(wf[nxt][c0 / 4], c0 % 4, w8_frag_dword<WK>(raw[c0 / 4].x, raw[c0 / 4].y, c0 % 4));
            set_dword(wf[nxt][c1 / 4], c1 % 4, w8_frag_dword<WK>(raw[c1 / 4].x, raw[c1 / 4].y, c1 % 4));
          }
        }
      } else {
        // weight sub-block s behind MFMA (s+1, 3); with fewer than nine row blocks the last ones behind (.., 7)
        constexpr int ws = dma_wf_slot(x, sb, NLIVE);
        if constexpr (ws >= 0) wf[nxt][ws] = wr[ws * 64];
      }
      {
        // direct-to-LDS piece p (weights first, then this wavefront's row blocks): M0 write and load behind
        // MFMAs (p+1, 5) and (p+1, 6); pieces that find no row block of their own there behind (.., 2) and (.., 4)
        constexpr int pp = dma_piece_slot(x, sb, NLIVE, kPieces);  // 2*p + (0: M0 write, 1: load), or -1
        if constexpr (pp >= 0) {
          constexpr int p = pp / 2, q = p - kNW;
          constexpr bool issue = (pp % 2) != 0;
          if constexpr (p < kNW) {
            if constexpr (!issue) set_m0(ldsW0 + stageByte + p * 1024);
            else dma_issue(wg, lane16 + p * 1024);
          } else if constexpr (q < PXlo) {
            if constexpr (!issue) set_m0(lds0 + stageByte + xblk[q] * 1024);
            else dma_issue(xg + xblk[q] * 64, lane16);
          } else if constexpr (issue) {
            if (more) dma_1k(xg + xblk[q] * 64, lds0 + stageByte + xblk[q] * 1024, lane16);  // wavefronts 0, 1 only
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);  // keep this dealing-out as written
    });
  };

  const int nKK = KS / 4;  // KS is a multiple of 8: d is padded to 256
  for (int kk = 0; kk < nKK; ++kk) {
    const int kn = min(kk + 1, nKK - 1);  // group of four steps requested during this one
    const uint4* wIter = W8 ? wsrc0 + (size_t)kn * 4 * wStep8 : wsrc0 + (size_t)kn * ((size_t)nVGalloc * (kWpKG * 256));
    const uint4* xIter = xsrc0 + (size_t)kn * (4 * kDmaRowBlocks * 64);
    k_step(wIter, xIter, std::integral_constant<int, 0>{});
    k_step(wIter, xIter, std::integral_constant<int, 1>{});
    k_step(wIter, xIter, std::integral_constant<int, 2>{});
    k_step(wIter, xIter, std::integral_constant<int, 3>{});
  }

  // every direct-to-LDS load must have landed before the workgroup gives its LDS back, and the
  // last MFMAs must have left the matrix pipeline before their tiles are read
  wait_groups(std::integral_constant<int, 0>{});
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);

  // epilogue: acc[s][x][i] = logit of row rt*tileRows + rh*NLIVE*16 + x*16 + n,
  //           vocabulary entry (vt*4 + vh*2 + s/4)*64 + (s%4)*16 + gq*4 + i
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int vg = vt * 4 + vh * 2 + half;
    if (vg >= nVG) continue;
    float osc[4][4];  // (per-entry weight scale, FP8 weights only) / T for this lane's 16 entries
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
        osc[sub][i] = (vscale != nullptr && v < V) ? vscale[v] * invT : invT;
      }
#pragma unroll
    for (int x = 0; x < NLIVE; ++x) {
      const int r = rt * tileRows + rh * (NLIVE * 16) + x * 16 + n;
      float vals[4][4];
      float mx = -INFINITY;
#pragma unroll
      for (int sub = 0; sub < 4; ++sub)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
          const float l = acc[half * 4 + sub][x][i] * osc[sub][i];
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
      if (r < R) {
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          const int v0 = vg * kVocabGroup + sub * 16 + gq * 4;
          *reinterpret_cast<float4*>(L + (size_t)r * Lld + v0) =
              make_float4(vals[sub][0], vals[sub][1], vals[sub][2], vals[sub][3]);
        }
        if (gq == 0) part[(size_t)r * nVG + vg] = make_float2(mx, sum);
      }
    }
  }
}

// One launch runs row tiles rt0 .. rt0 + nRowTiles - 1 (tile rt starts at row rt*tileRows), all with NLIVE row blocks
// per half: the equally sized row tiles of a call in one launch, or its full row tiles in one launch and a ragged last
// one in a launch of its own (one body per kernel: with a second body behind a branch the register allocator has
// to spill, and it does so around the MFMAs it cannot see into).
template <int WK, int NLIVE>
__global__ __launch_bounds__(256, 1) void lmhead_gemm_dma_kernel(
    const uint4* __restrict__ Wsrc, const float* __restrict__ vscale, const uint4* __restrict__ Xp, int R, int KS,
    int V, int nVG, int nVGalloc, int rt0, int nRowTiles, int tileRows, int nVocabTiles, float invT,
    float* __restrict__ L, int Lld, float2* __restrict__ part) {
  // XCD-aware tile id: the row tiles that stream the same 256 vocabulary rows get ids that the
  // hardware deals to one XCD, so W_lm crosses from HBM into one L2 only.
  const int bid = blockIdx.x;
  const int xcd = bid % kXcds;
  const int j = bid / kXcds;
  const int rt = rt0 + j % nRowTiles;
  const int vt = (j / nRowTiles) * kXcds + xcd;
  if (vt >= nVocabTiles) return;  // uniform for the whole workgroup, before any barrier
  dma_tile<WK, NLIVE>(Wsrc, vscale, Xp, R, KS, V, nVG, nVGalloc, invT, L, Lld, part, rt, vt, tileRows);
}

// Wg8[ks][vg][sub][lane][8 B]: the FP8 E4M3 codes of W_lm in MFMA fragment order for this kernel, one
// 512-byte fragment per (K step, vocabulary group, 16-row sub-block): lane holds row vg*64 + sub*16 + lane%16,
// hidden indices ks*32 + (lane/16)*8 + 0..7.  The four fragments of a group and the four groups of a
// workgroup's tile are adjacent, so a K step of a tile is 8 KiB of consecutive memory.  Zero padded.
__global__ __launch_bounds__(256) void pack_w8g_kernel(const uint8_t* __restrict__ W8, int layout, int V, int d,
                                                        int nVGalloc, size_t total, uint2* __restrict__ Wg8) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const int sub = (int)((idx >> 6) & 3);
  const size_t t = idx >> 8;
  const int vg = (int)(t % (size_t)nVGalloc);
  const int ks = (int)(t / (size_t)nVGalloc);
  const int v = vg * kVocabGroup + sub * 16 + (lane & 15);
  const int k0 = ks * kKStep + (lane >> 4) * 8;
  union { uint2 q; uint8_t b[8]; } o;
  o.q = make_uint2(0u, 0u);
  if (v < V)
    for (int e = 0; e < 8; ++e)
      if (k0 + e < d) o.b[e] = (layout == 0) ? W8[(size_t)v * d + k0 + e] : W8[(size_t)(k0 + e) * V + v];
  Wg8[idx] = o.q;
}

hipError_t launch_pack_w8g(const void* W8, int layout, const Geometry& g, void* Wg8, hipStream_t st) {
  if (!W8 || !Wg8) return hipErrorInvalidValue;
  const size_t total = (size_t)(g.dpad / kKStep) * g.nVGalloc * 256;
  const size_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_w8g_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint8_t*>(W8),
                     layout, g.V, g.d, g.nVGalloc, total, static_cast<uint2*>(Wg8));
  return hipGetLastError();
}

// More LDS than the default limit of a launch: raised once per process, at context creation (not in the
// launcher, which may run under stream capture).
template <int WK, int NLAST>
static hipError_t dma_lds_limit() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(lmhead_gemm_dma_kernel<WK, NLAST>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDmaLdsBytes<WK != kWBf16>);
}
template <int WK>
static hipError_t dma_lds_limits() {
  hipError_t e = dma_lds_limit<WK, 6>();
  if (e == hipSuccess) e = dma_lds_limit<WK, 7>();
  if (e == hipSuccess) e = dma_lds_limit<WK, 8>();
  if (e == hipSuccess) e = dma_lds_limit<WK, 9>();
  if (e == hipSuccess) e = dma_lds_limit<WK, 10>();
  if (e == hipSuccess) e = dma_lds_limit<WK, 11>();
  return e;
}

hipError_t init_lmhead_gemm_dma() {
  hipError_t e = dma_lds_limits<kWBf16>();
  if (e == hipSuccess) e = dma_lds_limits<kWFp8>();
  if (e == hipSuccess) e = dma_lds_limits<kWInt8>();
  return e;
}

template <int WK>
static void launch_dma(int nlive, int rt0, int nRt, int tileRows, int perRt, hipStream_t st, const void* W, const float* vscale,
                       const void* Xp, int R, int KS, const Geometry& g, int nVocabTiles, float invT, float* L,
                       float2* part) {
#define JD_DMA(NL_)                                                                                                \
  hipLaunchKernelGGL((lmhead_gemm_dma_kernel<WK, NL_>), dim3(perRt * nRt), dim3(256), kDmaLdsBytes<WK != kWBf16>, st, \
                     static_cast<const uint4*>(W), vscale, static_cast<const uint4*>(Xp), R, KS, g.V, g.nVG,          \
                     g.nVGalloc, rt0, nRt, tileRows, nVocabTiles, invT, L, g.Vpad, part)
  switch (nlive) {
    case 6: JD_DMA(6); break;
    case 7: JD_DMA(7); break;
    case 8: JD_DMA(8); break;
    case 9: JD_DMA(9); break;
    case 10: JD_DMA(10); break;
    default: JD_DMA(11); break;
  }
#undef JD_DMA
}

// How the rows of a call are cut into row tiles (measured at d = 8192, bf16: a tile with 6 .. 11 row blocks per half
// costs 0.37 / 0.40 / 0.44 / 0.47 / 0.51 / 0.55 ms in a launch of its own and about 5 % less next to the other row
// tiles of its vocabulary tiles, with which it shares the weights through L2):
//  * one row tile: as many blocks per half as its rows need;
//  * several: equally sized tiles if they need at most 9 blocks per half (363 rows = 2 x 6 blocks per half);
//  * else full tiles and the last one in a launch of its own, which streams the weights again, if that one needs at
//    most 8 blocks per half (880 rows = 2 full tiles + 6 blocks per half); else equally sized tiles of 10 blocks per
//    half if they hold the rows, else full tiles throughout.
struct DmaPlan { int tileRows, halfBlocks, lastHalfBlocks; };
static DmaPlan dma_plan(int R) {
  const int nRt = (R + kDmaRows - 1) / kDmaRows;
  if (nRt == 1) { const int n = dma_half_blocks(R); return {kDmaRows, n, n}; }
  const int nb = (R + 32 * nRt - 1) / (32 * nRt);  // blocks per half of equally sized tiles, 6 .. 11
  if (nb <= 9) return {32 * nb, nb, nb};
  const int nlast = dma_half_blocks(R);
  if (nlast <= 8) return {kDmaRows, kDmaWaveRowBlocks, nlast};
  if (nb == 10) return {32 * nb, nb, nb};
  return {kDmaRows, kDmaWaveRowBlocks, kDmaWaveRowBlocks};
}

hipError_t launch_lmhead_gemm_dma(const void* W, int w_code, const float* vscale, const void* X, int R,
                                  const Geometry& g, float invT, float* L, float2* part, void* Xp, hipStream_t st) {
  static_assert(kGroupAlloc % 4 == 0, "a vocabulary tile of 4 groups never leaves the allocation");
  static_assert(kWpKG * 256 == 4 * 256 && kKStep == 32, "a K step of one vocabulary group is 4 KiB, contiguous");
  static_assert(kDmaMinHalfBlocks == 6, "instantiations below");
  if (R <= 0 || !Xp || !W) return hipErrorInvalidValue;
  const int nRowTiles = (R + kDmaRows - 1) / kDmaRows;
  const int KS = g.dpad / kKStep;  // multiple of 8
  if (KS < 2 * kDmaStages) return hipErrorInvalidValue;
  const int nVocabTiles = (g.nVG + 3) / 4;
  const int perRt = ((nVocabTiles + kXcds - 1) / kXcds) * kXcds;  // workgroups per row tile
  auto go = [&](int nlive, int rt0, int nRt, int tileRows) {
    switch (w_code) {
      case kWFp8: launch_dma<kWFp8>(nlive, rt0, nRt, tileRows, perRt, st, W, vscale, Xp, R, KS, g, nVocabTiles, invT, L, part); break;
      case kWInt8: launch_dma<kWInt8>(nlive, rt0, nRt, tileRows, perRt, st, W, vscale, Xp, R, KS, g, nVocabTiles, invT, L, part); break;
      default: launch_dma<kWBf16>(nlive, rt0, nRt, tileRows, perRt, st, W, vscale, Xp, R, KS, g, nVocabTiles, invT, L, part); break;
    }
  };
  const DmaPlan plan = dma_plan(R);
  hipError_t e = launch_pack_x(X, R, g.d, nRowTiles, KS, kDmaRowBlocks, 1, plan.tileRows, plan.halfBlocks,
                               plan.lastHalfBlocks != plan.halfBlocks ? nRowTiles - 1 : -1, plan.lastHalfBlocks, Xp, st);
  if (e != hipSuccess) return e;
  if (plan.lastHalfBlocks == plan.halfBlocks) {
    go(plan.halfBlocks, 0, nRowTiles, plan.tileRows);       // equally sized row tiles, one launch
  } else {
    go(plan.halfBlocks, 0, nRowTiles - 1, plan.tileRows);   // the full row tiles
    go(plan.lastHalfBlocks, nRowTiles - 1, 1, plan.tileRows);  // the ragged last one
  }
  return hipGetLastError();
}

}  // namespace jd
