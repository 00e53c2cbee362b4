// LM-head projection for the large-row regime (R = B*(M+1) > 64, e.g. 64 sequences x 11
// rows = 704) on gfx950: here the contraction (Sec. 3.1, Eq. 2, for all rows of a batch)
// is dense enough to be bound by the matrix cores, not by the W_lm stream.
//
// Tiling.  One workgroup (4 wavefronts, one per SIMD, up to 512 registers each) owns
// 176 embedding rows x 256 vocabulary entries; each wavefront owns 176 x 64 of it as
// 11 x 4 accumulator tiles of v_mfma_f32_16x16x32_bf16 (176 registers).  704 rows are
// exactly four such row tiles, so the B=64, M=10 batch carries no padding rows.
//   * W_lm fragments go straight from the re-tiled global copy into MFMA A operands
//     (a wavefront's 64 vocabulary rows are its own - nothing to share through LDS),
//     prefetched two K steps ahead;
//   * the embedding tile is what the four wavefronts share: it is re-tiled once per call
//     into fragment order (pack_x_kernel) so that staging a 128-wide K chunk is a linear
//     44 KiB copy into LDS and every operand read is a conflict-free lane-linear
//     ds_read_b128; double buffered, one barrier per chunk;
//   * per K step a wavefront issues 44 MFMAs against 11 LDS reads and 4 global loads.
// Workgroup -> tile mapping is XCD aware: hardware deals consecutive workgroups round-robin
// to the 8 XCDs, so the four row tiles that stream the same 256 vocabulary rows are given
// ids that land on one XCD and share its L2: W_lm is fetched from HBM once.
// Epilogue as in the small-row kernel: fp32 logits / T and one (max, sum exp) softmax
// partial per (row, 64-entry vocabulary group).
#include <type_traits>

#include "jd_kernels.hpp"

namespace jd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;
constexpr int kGemmSteps = kGemmKChunk / kKStep;  // 4 K steps per staged chunk
constexpr int kGemmPF = 2;                        // K steps per weight prefetch group

// Xp[rt][chunk][xb][s][lane][8]: row rt*176 + xb*16 + lane%16, hidden index
// chunk*128 + s*32 + (lane/16)*8 + 0..7; zero for rows >= R and indices >= d.
__global__ __launch_bounds__(256) void pack_x_kernel(const uint16_t* __restrict__ X, int R, int d, int nChunks,
                                                      size_t total, uint4* __restrict__ Xp) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  size_t t = idx >> 6;
  const int s = (int)(t % kGemmSteps); t /= kGemmSteps;
  const int xb = (int)(t % kGemmRowBlocks); t /= kGemmRowBlocks;
  const int ch = (int)(t % (size_t)nChunks);
  const int rt = (int)(t / (size_t)nChunks);
  const int row = rt * kGemmRows + xb * 16 + (lane & 15);
  const int k = ch * kGemmKChunk + s * kKStep + (lane >> 4) * 8;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row < R && k < d) v = *reinterpret_cast<const uint4*>(X + (size_t)row * d + k);  // d % 8 == 0
  Xp[idx] = v;
}

__global__ __launch_bounds__(256, 1) void lmhead_gemm_kernel(
    const uint4* __restrict__ Wp, const uint4* __restrict__ Xp, int R, int nChunks, int V, int nVG, int nVGalloc,
    int nRowTiles, int nVocabTiles, float invT, float* __restrict__ L, int Lld, float2* __restrict__ part) {
  constexpr int NXB = kGemmRowBlocks;
  constexpr int ITEMS = NXB * kGemmSteps * 64;  // 16-byte items per staged chunk (44 KiB)
  constexpr int IPT = ITEMS / 256;              // = NXB
  constexpr int GROUPS = kGemmSteps / kGemmPF;
  static_assert(GROUPS % 2 == 0, "prefetch parity must be static");

  extern __shared__ uint4 xs_raw[];  // 2 x ITEMS x 16 B = 88 KiB (dynamic: above the static limit)
  uint4 (*xs)[ITEMS] = reinterpret_cast<uint4 (*)[ITEMS]>(xs_raw);

  // XCD-aware tile id: workgroups j = 0,1,2.. of one XCD walk row tiles fastest.
  const int bid = blockIdx.x;
  const int xcd = bid % kXcds;
  const int j = bid / kXcds;
  const int rt = j % nRowTiles;
  const int vt = (j / nRowTiles) * kXcds + xcd;
  if (vt >= nVocabTiles) return;  // uniform for the whole workgroup, before any barrier

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // wavefront-uniform values are made scalar explicitly so that addresses are formed as
  // (scalar base + lane offset) and do not occupy vector registers
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15;
  const int gq = lane >> 4;
  const int vg = vt * 4 + wave;  // < nVGalloc (allocated in multiples of 8 groups)
  const int KS = nChunks * kGemmSteps;
  const int nGroupsTotal = KS / kGemmPF;
  static_assert(kGemmPF == kWpKG, "one prefetch group = one contiguous 8 KiB block of Wp");
  const size_t wGroupStride = (size_t)nVGalloc * (kWpKG * 256);  // 16-byte units between K-step pairs

  const uint4* wbase = Wp + wp_group_offset(vg);
  const uint4* xbase = Xp + (size_t)rt * nChunks * ITEMS;

  f32x4 acc[4][NXB];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int x = 0; x < NXB; ++x) acc[s][x] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 wbuf[2][kGemmPF][4];

  // Staging of the next embedding chunk is spread over the K steps of the current one so that
  // only a few registers are live at a time: portion p (items 4p .. 4p+3 of this thread's 11)
  // is loaded during step p and written to the idle LDS buffer during step p+1.
  constexpr int kPortion = 4;
  constexpr int kPortions = (IPT + kPortion - 1) / kPortion;  // 3
  static_assert(kPortions < kGemmSteps, "every portion needs a later step to be stored in");
  static_assert(kPortion == 4 && IPT == 11, "portions are written out by hand below");
  uint4 xr0, xr1, xr2, xr3;  // named registers, not an array: keeps them off the stack

  // (portion and step numbers are compile-time constants so that every register array below
  // is indexed statically and stays in registers)
  auto load_portion = [&](const uint4* src, auto pc) {
    constexpr int p = decltype(pc)::value;
    xr0 = src[tid + (p * 4 + 0) * 256];
    xr1 = src[tid + (p * 4 + 1) * 256];
    xr2 = src[tid + (p * 4 + 2) * 256];
    if constexpr (p * 4 + 3 < IPT) xr3 = src[tid + (p * 4 + 3) * 256];
  };
  auto store_portion = [&](uint4* dst, auto pc) {
    constexpr int p = decltype(pc)::value;
    dst[tid + (p * 4 + 0) * 256] = xr0;
    dst[tid + (p * 4 + 1) * 256] = xr1;
    dst[tid + (p * 4 + 2) * 256] = xr2;
    if constexpr (p * 4 + 3 < IPT) dst[tid + (p * 4 + 3) * 256] = xr3;
  };
  auto load_wgroup = [&](const int buf, int g) {
    const uint4* src = wbase + (size_t)g * wGroupStride;
#pragma unroll
    for (int s2 = 0; s2 < kGemmPF; ++s2)
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) wbuf[buf][s2][sub] = src[s2 * 256 + sub * 64 + lane];
  };

  // prologue: chunk 0 into LDS buffer 0, first weight group into registers
  load_portion(xbase, std::integral_constant<int, 0>{}); store_portion(xs[0], std::integral_constant<int, 0>{});
  load_portion(xbase, std::integral_constant<int, 1>{}); store_portion(xs[0], std::integral_constant<int, 1>{});
  load_portion(xbase, std::integral_constant<int, 2>{}); store_portion(xs[0], std::integral_constant<int, 2>{});
  static_assert(kPortions == 3, "prologue and step schedule are written for three portions");
  load_wgroup(0, 0);
  __syncthreads();

  for (int ch = 0; ch < nChunks; ++ch) {
    // branch-free: the last iteration re-stages its own chunk into the idle buffer, unread
    const uint4* xnext = xbase + (size_t)min(ch + 1, nChunks - 1) * ITEMS;
    uint4* xdst = xs[(ch + 1) & 1];
    const uint4* xcur = xs[ch & 1] + lane;
    auto k_step = [&](auto ksc) {
      constexpr int ks = decltype(ksc)::value;
      constexpr int gi = ks / kGemmPF, s = ks % kGemmPF;
      if constexpr (ks > 0 && ks - 1 < kPortions) store_portion(xdst, std::integral_constant<int, (ks > 0 ? ks - 1 : 0)>{});
      if constexpr (ks < kPortions) load_portion(xnext, std::integral_constant<int, (ks < kPortions ? ks : 0)>{});
      // prefetch the next weight group (the very last one re-reads itself)
      if constexpr (s == 0) load_wgroup((gi + 1) & 1, min(ch * GROUPS + gi + 1, nGroupsTotal - 1));
      // keep the loads above ahead of this step's MFMAs
      __builtin_amdgcn_sched_barrier(0);
      // operand reads run two row blocks ahead of the MFMAs that consume them
      bf16x8 bfrag[3];
      bfrag[0] = __builtin_bit_cast(bf16x8, xcur[(0 * kGemmSteps + ks) * 64]);
      bfrag[1] = __builtin_bit_cast(bf16x8, xcur[(1 * kGemmSteps + ks) * 64]);
#pragma unroll
      for (int x = 0; x < NXB; ++x) {
        if (x + 2 < NXB) bfrag[(x + 2) % 3] = __builtin_bit_cast(bf16x8, xcur[((x + 2) * kGemmSteps + ks) * 64]);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub)
          acc[sub][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(bf16x8, wbuf[gi & 1][s][sub]), bfrag[x % 3], acc[sub][x], 0, 0, 0);
      }
      // pin that interleaving: 2 LDS reads, then (1 LDS read, 4 MFMA) per row block
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
      for (int x = 0; x < NXB; ++x) {
        if (x + 2 < NXB) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    k_step(std::integral_constant<int, 0>{});
    k_step(std::integral_constant<int, 1>{});
    k_step(std::integral_constant<int, 2>{});
    k_step(std::integral_constant<int, 3>{});
    static_assert(kGemmSteps == 4, "four K steps per staged chunk");
    __syncthreads();
  }

  // epilogue: acc[sub][x][i] = logit of row rt*176 + x*16 + n, entry vg*64 + sub*16 + gq*4 + i
  if (vg >= nVG) return;
#pragma unroll
  for (int x = 0; x < NXB; ++x) {
    const int r = rt * kGemmRows + x * 16 + n;
    float vals[4][4];
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
        const float l = acc[sub][x][i] * invT;
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

hipError_t launch_lmhead_gemm(const void* Wp, const void* X, int R, const Geometry& g, float invT, float* L,
                              float2* part, void* Xp, int /*num_cus*/, hipStream_t st) {
  static_assert(kGroupAlloc % 4 == 0, "a vocabulary tile of 4 groups never leaves the allocation");
  if (R <= 0 || !Xp) return hipErrorInvalidValue;
  const int nRowTiles = (R + kGemmRows - 1) / kGemmRows;
  const int nChunks = g.dpad / kGemmKChunk;
  const size_t total = (size_t)nRowTiles * nChunks * kGemmRowBlocks * kGemmSteps * 64;
  hipLaunchKernelGGL(pack_x_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint16_t*>(X), R, g.d, nChunks, total, static_cast<uint4*>(Xp));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int nVocabTiles = (g.nVG + 3) / 4;
  const int grid = ((nVocabTiles + kXcds - 1) / kXcds) * kXcds * nRowTiles;
  constexpr size_t kLds = 2 * (size_t)kGemmRowBlocks * kGemmSteps * 64 * sizeof(uint4);
  static bool attr_set = false;
  if (!attr_set) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(lmhead_gemm_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(lmhead_gemm_kernel, dim3(grid), dim3(256), kLds, st, static_cast<const uint4*>(Wp),
                     static_cast<const uint4*>(Xp), R, nChunks, g.V, g.nVG, g.nVGalloc, nRowTiles, nVocabTiles, invT,
                     L, g.Vpad, part);
  return hipGetLastError();
}

}  // namespace jd
