// LM-head projection for calls of one 176-row tile (65 .. 176 rows; Sec. 3.1, Eq. 2 for all rows of a batch) on
// gfx950.  Up to about 130 rows the launch is bound by the W_lm stream, beyond by the matrix cores; calls with more
// rows run on the 352-row kernel next door, which began as this kernel with both operands shared through LDS.
//
// Tiling.  One workgroup (4 wavefronts, one per SIMD, up to 512 registers each) owns all rows x 256 vocabulary
// entries; each wavefront owns 64 of them as up to 11 x 4 accumulator tiles of v_mfma_f32_16x16x32_bf16.
//   * W_lm fragments go straight from the re-tiled global copy into MFMA A operands
//     (a wavefront's 64 vocabulary rows are its own - nothing to share through LDS),
//     prefetched two K steps ahead, with non-temporal loads;
//   * the embedding tile is what the four wavefronts share: it is re-tiled once per call
//     into fragment order (pack_x_kernel) so that staging a 128-wide K chunk is a linear
//     copy into LDS and every operand read is a conflict-free lane-linear
//     ds_read_b128; double buffered, one barrier per chunk;
//   * per K step a wavefront issues up to 44 MFMAs against 11 LDS reads and 4 global loads; row blocks without rows
//     are left out at compile time (one instantiation per number of row blocks that hold rows).
// Epilogue as in the small-row kernel: fp32 logits / T and one (max, sum exp) softmax
// partial per (row, 64-entry vocabulary group).
#include <type_traits>

#include "w8_frag.hpp"
#include "jd_kernels.hpp"

namespace jd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// acc += A * B with the accumulator tied in place in an accumulation register.  Written as
// inline assembly because, left to the register allocator, the 44 accumulator tiles of a
// wavefront get distinct destination and source registers and ~220 copy instructions per
// loop iteration to move them back.  Hazards the compiler no longer sees are covered by
// construction: operands come from loads (wait counts are still inserted per register),
// two MFMAs on the same tile are 43 MFMAs apart, and the epilogue waits explicitly before
// reading the tiles.
__device__ __forceinline__ void mfma_16x16x32_bf16_inplace(f32x4& acc, const uint4& a, const bf16x8& b) {
  const u32x4 av = __builtin_bit_cast(u32x4, a);
  const u32x4 bv = __builtin_bit_cast(u32x4, b);
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(av), "v"(bv));
}

constexpr int kGemmSteps = kGemmKChunk / kKStep;  // 4 K steps per staged chunk
constexpr int kGemmPF = 2;                        // K steps per weight prefetch group
constexpr int kGemmWBufs = 4;                     // register ring of weight groups: 3 groups (6 K steps) ahead

// Xp[rt][chunk][xb][s][lane][8]: hidden index chunk*(steps*32) + s*32 + (lane/16)*8 + 0..7 of the row that block
// position xb of row tile rt holds; zero for rows >= R, indices >= d and positions without a row.
// halfBlocks == 0 (176-row kernel): position xb holds rows rt*tileRows + xb*16 + lane%16.
// halfBlocks > 0 (352-row kernel): a row tile is two halves of rowBlocks/2 positions each, of which the first
// halfBlocks (row tile splitRt: splitHalfBlocks) hold rows: position xb holds row
// rt*tileRows + (xb / (rowBlocks/2)) * hb*16 + (xb % (rowBlocks/2)) * 16 + lane%16.
__global__ __launch_bounds__(256) void pack_x_kernel(const uint16_t* __restrict__ X, int R, int d, int nChunks,
                                                      int rowBlocks, int steps, int tileRows, int halfBlocks,
                                                      int splitRt, int splitHalfBlocks, size_t total,
                                                      uint4* __restrict__ Xp) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  size_t t = idx >> 6;
  const int s = (int)(t % steps); t /= steps;
  const int xb = (int)(t % rowBlocks); t /= rowBlocks;
  const int ch = (int)(t % (size_t)nChunks);
  const int rt = (int)(t / (size_t)nChunks);
  int row = rt * tileRows + xb * 16 + (lane & 15);
  if (halfBlocks > 0) {
    const int half = rowBlocks / 2, h = xb / half, x = xb % half;
    const int hb = (rt == splitRt) ? splitHalfBlocks : halfBlocks;
    row = (x < hb) ? rt * tileRows + h * hb * 16 + x * 16 + (lane & 15) : R;
  }
  const int k = (ch * steps + s) * kKStep + (lane >> 4) * 8;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row < R && k < d) v = *reinterpret_cast<const uint4*>(X + (size_t)row * d + k);  // d % 8 == 0
  Xp[idx] = v;
}

hipError_t launch_pack_x(const void* X, int R, int d, int nRowTiles, int nChunks, int rowBlocks, int steps, int tileRows,
                         int halfBlocks, int splitRt, int splitHalfBlocks, void* Xp, hipStream_t st) {
  const size_t total = (size_t)nRowTiles * nChunks * rowBlocks * steps * 64;
  hipLaunchKernelGGL(pack_x_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint16_t*>(X), R, d, nChunks, rowBlocks, steps, tileRows, halfBlocks, splitRt,
                     splitHalfBlocks, total, static_cast<uint4*>(Xp));
  return hipGetLastError();
}

// WK = kWBf16: Wp is the re-tiled bf16 copy.  WK = kWFp8 / kWInt8: Wp is Wp8, the one-byte copy of the small-row kernel (a
// lane's 16 bytes are its codes for the two K steps of a prefetch group): half the weight bytes from HBM
// and through L2; fragments are converted to bf16 in registers one K step ahead, one instruction behind
// an MFMA each; the per-entry scale is applied in the epilogue.
// One tile: embedding rows 0 .. 175 (the kernel serves calls of one row tile, 65 .. 176 rows), vocabulary entries
// vt*256 .. +255.  NLIVE = number of the tile's 16-row blocks that hold rows; the MFMAs, loads and staging of the others
// are left out at compile time.  Every weight is read exactly once, so its loads are non-temporal (3-4 % faster).
template <int WK, int NLIVE>
__device__ __forceinline__ void gemm_tile(
    const uint4* __restrict__ Wp, const float* __restrict__ vscale, const uint4* __restrict__ Xp, int R,
    int nChunks, int V, int nVG, int nVGalloc, float invT, float* __restrict__ L, int Lld, float2* __restrict__ part,
    const int vt) {
  constexpr bool W8 = WK != kWBf16;  // one-byte codes (FP8 E4M3 or INT8) in the Wp8 layout
  constexpr int NXB = kGemmRowBlocks;
  constexpr int ITEMS = NXB * kGemmSteps * 64;  // 16-byte items per staged chunk (44 KiB)
  constexpr int IPT = ITEMS / 256;              // = NXB
  constexpr int GROUPS = kGemmSteps / kGemmPF;
  static_assert(GROUPS % 2 == 0, "prefetch parity must be static");

  extern __shared__ uint4 xs_raw[];  // 2 x ITEMS x 16 B = 88 KiB (dynamic: above the static limit)
  uint4 (*xs)[ITEMS] = reinterpret_cast<uint4 (*)[ITEMS]>(xs_raw);
  auto ldw = [](const uint4* p) -> uint4 { return load_stream(p); };

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
  static_assert(kWpKG % kGemmPF == 0, "a prefetch group (8 KiB) never straddles two K-step blocks of Wp");

  static_assert(kGemmPF == 2 && kW8KG % 2 == 0, "a prefetch group is one FP8 K-step pair");
  const uint4* wbase = Wp + (W8 ? wp8_group_offset(vg) : wp_group_offset(vg));
  const uint4* xbase = Xp;

  f32x4 acc[4][NXB];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int x = 0; x < NXB; ++x) acc[s][x] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 wbuf[kGemmWBufs][W8 ? 1 : kGemmPF][4];  // ring of weight groups (FP8: codes of both K steps in one item)
  uint4 cv[2][4];                               // FP8 only: converted fragments of the current / next K step

  // Staging of the embedding tile runs a whole chunk ahead: during chunk c, step p first
  // writes portion p of chunk c+1 (loaded one chunk earlier) into the idle LDS buffer and
  // then re-uses the same registers to load portion p of chunk c+2.  Every load therefore
  // has four K steps (2816 MFMA cycles) to land.  Portions are items 4p .. 4p+3 of this
  // thread's 11 sixteen-byte items; named registers, not an array, keep them off the stack,
  // and portion / step numbers are compile-time constants.
  constexpr int kPortions = 3;
  static_assert(IPT == 11 && kPortions < kGemmSteps && NLIVE >= 1 && NLIVE <= IPT, "portions are written out by hand below");
  uint4 xa0, xa1, xa2, xa3, xb0, xb1, xb2, xb3, xc0, xc1, xc2;

  // item i of a thread belongs to row block i of the tile (items are laid out row block by row block, 256 per
  // block): blocks without rows are never read back from LDS.  With one-byte weights, and in launches with a single
  // row tile, they are neither loaded nor staged (66 rows FP8 0.220 -> 0.197 ms, 374 rows FP8 0.723 -> 0.683 ms,
  // 66-110 rows bf16 0.338-0.344 -> 0.334-0.337 ms); with bf16 weights on several row tiles leaving the staging out
  // makes ragged launches 2-4 % slower (374 rows 0.783 -> 0.819 ms), so there the zero rows keep travelling
  constexpr int NSTAGE = NLIVE;
  auto load_portion = [&](const uint4* src, auto pc) {
    constexpr int p = decltype(pc)::value;
    if constexpr (p == 0) {
      if constexpr (0 < NSTAGE) xa0 = src[tid];
      if constexpr (1 < NSTAGE) xa1 = src[tid + 256];
      if constexpr (2 < NSTAGE) xa2 = src[tid + 512];
      if constexpr (3 < NSTAGE) xa3 = src[tid + 768];
    }
    if constexpr (p == 1) {
      if constexpr (4 < NSTAGE) xb0 = src[tid + 1024];
      if constexpr (5 < NSTAGE) xb1 = src[tid + 1280];
      if constexpr (6 < NSTAGE) xb2 = src[tid + 1536];
      if constexpr (7 < NSTAGE) xb3 = src[tid + 1792];
    }
    if constexpr (p == 2) {
      if constexpr (8 < NSTAGE) xc0 = src[tid + 2048];
      if constexpr (9 < NSTAGE) xc1 = src[tid + 2304];
      if constexpr (10 < NSTAGE) xc2 = src[tid + 2560];
    }
  };
  auto store_portion = [&](uint4* dst, auto pc) {
    constexpr int p = decltype(pc)::value;
    if constexpr (p == 0) {
      if constexpr (0 < NSTAGE) dst[tid] = xa0;
      if constexpr (1 < NSTAGE) dst[tid + 256] = xa1;
      if constexpr (2 < NSTAGE) dst[tid + 512] = xa2;
      if constexpr (3 < NSTAGE) dst[tid + 768] = xa3;
    }
    if constexpr (p == 1) {
      if constexpr (4 < NSTAGE) dst[tid + 1024] = xb0;
      if constexpr (5 < NSTAGE) dst[tid + 1280] = xb1;
      if constexpr (6 < NSTAGE) dst[tid + 1536] = xb2;
      if constexpr (7 < NSTAGE) dst[tid + 1792] = xb3;
    }
    if constexpr (p == 2) {
      if constexpr (8 < NSTAGE) dst[tid + 2048] = xc0;
      if constexpr (9 < NSTAGE) dst[tid + 2304] = xc1;
      if constexpr (10 < NSTAGE) dst[tid + 2560] = xc2;
    }
  };
  auto load_wgroup = [&](const int buf, int g) {
    if constexpr (W8) {
      const uint4* src = wbase + wp8_pair_offset(g, nVGalloc);
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) wbuf[buf][0][sub] = ldw(src + sub * 64 + lane);
    } else {
      const uint4* src = wbase + wp_step_offset(g * kGemmPF, nVGalloc);
#pragma unroll
      for (int s2 = 0; s2 < kGemmPF; ++s2)
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) wbuf[buf][s2][sub] = ldw(src + s2 * 256 + sub * 64 + lane);
    }
  };

  // prologue: chunk 0 into LDS buffer 0, chunk 1 into the staging registers
  load_portion(xbase, std::integral_constant<int, 0>{}); store_portion(xs[0], std::integral_constant<int, 0>{});
  load_portion(xbase, std::integral_constant<int, 1>{}); store_portion(xs[0], std::integral_constant<int, 1>{});
  load_portion(xbase, std::integral_constant<int, 2>{}); store_portion(xs[0], std::integral_constant<int, 2>{});
  {
    const uint4* x1 = xbase + (size_t)min(1, nChunks - 1) * ITEMS;
    load_portion(x1, std::integral_constant<int, 0>{});
    load_portion(x1, std::integral_constant<int, 1>{});
    load_portion(x1, std::integral_constant<int, 2>{});
  }
  // weight groups 0 .. kGemmWBufs-2 in flight before the loop starts
  static_assert(kGemmWBufs == 4 && GROUPS == 2, "ring index below assumes 2 groups per chunk, 4 buffers");
  load_wgroup(0, 0);
  load_wgroup(1, min(1, nGroupsTotal - 1));
  load_wgroup(2, min(2, nGroupsTotal - 1));
  if constexpr (W8) {  // fragments of K step 0
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) set_dword(cv[0][sub], jj, w8_frag_dword<WK>(wbuf[0][0][sub].x, wbuf[0][0][sub].y, jj));
  }
  __syncthreads();

  // One staged chunk.  `parity` (chunk index mod 2) is a compile-time constant: it selects the
  // LDS buffer and, with the group number inside the chunk, the slot of the register ring.
  auto chunk_body = [&](const int ch, auto parc) {
    constexpr int parity = decltype(parc)::value;
    // branch-free: past the end the last chunk is re-loaded and re-staged, unread
    const uint4* xnext = xbase + (size_t)min(ch + 2, nChunks - 1) * ITEMS;
    uint4* xdst = xs[parity ^ 1];
    const uint4* xcur = xs[parity] + lane;
    // write item i of chunk c+1 to LDS / reload the same registers with item i of chunk c+2
    auto stage_store = [&](const int i) {
      switch (i) {
        case 0: xdst[tid] = xa0; break;
        case 1: xdst[tid + 256] = xa1; break;
        case 2: xdst[tid + 512] = xa2; break;
        case 3: xdst[tid + 768] = xa3; break;
        case 4: xdst[tid + 1024] = xb0; break;
        case 5: xdst[tid + 1280] = xb1; break;
        case 6: xdst[tid + 1536] = xb2; break;
        case 7: xdst[tid + 1792] = xb3; break;
        case 8: xdst[tid + 2048] = xc0; break;
        case 9: xdst[tid + 2304] = xc1; break;
        case 10: xdst[tid + 2560] = xc2; break;
        default: break;
      }
    };
    auto stage_load = [&](const int i) {
      switch (i) {
        case 0: xa0 = xnext[tid]; break;
        case 1: xa1 = xnext[tid + 256]; break;
        case 2: xa2 = xnext[tid + 512]; break;
        case 3: xa3 = xnext[tid + 768]; break;
        case 4: xb0 = xnext[tid + 1024]; break;
        case 5: xb1 = xnext[tid + 1280]; break;
        case 6: xb2 = xnext[tid + 1536]; break;
        case 7: xb3 = xnext[tid + 1792]; break;
        case 8: xc0 = xnext[tid + 2048]; break;
        case 9: xc1 = xnext[tid + 2304]; break;
        case 10: xc2 = xnext[tid + 2560]; break;
        default: break;
      }
    };
    auto k_step = [&](auto ksc) {
      constexpr int ks = decltype(ksc)::value;
      constexpr int gi = ks / kGemmPF, s = ks % kGemmPF;
      constexpr int slot = (parity * GROUPS + gi) % kGemmWBufs;
      constexpr int nslot = (slot + kGemmWBufs - 1) % kGemmWBufs;
      // the weight group three ahead goes into the slot freed by the previous group, four
      // fragments per K step (past the end it re-reads the last group, unread)
      const int gnext = min(ch * GROUPS + gi + kGemmWBufs - 1, nGroupsTotal - 1);
      const uint4* wsrc = wbase + (W8 ? wp8_pair_offset(gnext, nVGalloc) : wp_step_offset(gnext * kGemmPF, nVGalloc)) + lane;
      // operand reads run two row blocks ahead of the MFMAs that consume them
      bf16x8 bfrag[3];
      bfrag[0] = __builtin_bit_cast(bf16x8, xcur[(0 * kGemmSteps + ks) * 64]);
      if constexpr (NLIVE > 1) bfrag[1] = __builtin_bit_cast(bf16x8, xcur[(1 * kGemmSteps + ks) * 64]);
      // Behind each MFMA of a lone wavefront exactly one vector, LDS or memory instruction issues for free
      // (every further one delays the next MFMA by about 7 cycles), so the step's loads, LDS writes and LDS
      // reads are dealt out one per MFMA: row block x carries behind its four MFMAs
      //   a weight load (even x) or a staging write (odd x) | the matching staging load | an operand read | -
#pragma unroll
      for (int x = 0; x < NXB; ++x) {
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          if constexpr (W8) {
            if (x < NLIVE) mfma_16x16x32_bf16_inplace(acc[sub][x], cv[ks & 1][sub], bfrag[x % 3]);
            // codes of the group three ahead: four loads, in the first K step of a group only
            if (s == 0 && sub == 0 && x % 2 == 0 && x / 2 < 4) wbuf[nslot][0][x / 2] = ldw(wsrc + (x / 2) * 64);
            // fragments of the next K step (second half of this group's codes, or first half of the next
            // group's): 16 conversions, behind MFMA (x, 3) of every row block and five otherwise empty slots
            constexpr int cslot = (s == 0) ? slot : (slot + 1) % kGemmWBufs;
            const int c = (sub == 3) ? x : (x == 8 && sub < 2) ? 11 + sub : (x == 9 && sub < 2) ? 13 + sub
                                                                         : (x == 10 && sub == 0) ? 15 : -1;
            if (c >= 0) {
              const uint4& codes = wbuf[cslot][0][c / 4];
              set_dword(cv[(ks + 1) & 1][c / 4], c % 4,
                        s == 0 ? w8_frag_dword<WK>(codes.z, codes.w, c % 4) : w8_frag_dword<WK>(codes.x, codes.y, c % 4));
            }
          } else {
            if (x < NLIVE) mfma_16x16x32_bf16_inplace(acc[sub][x], wbuf[slot][s][sub], bfrag[x % 3]);
            if (sub == 0 && x % 2 == 0 && x / 2 < 4) wbuf[nslot][s][x / 2] = ldw(wsrc + s * 256 + (x / 2) * 64);
          }
          if (sub == 0 && x % 2 == 1 && x / 2 < 4 && ks * 4 + x / 2 < NSTAGE) stage_store(ks * 4 + x / 2);
          if (sub == 1 && x % 2 == 1 && x / 2 < 4 && ks * 4 + x / 2 < NSTAGE) stage_load(ks * 4 + x / 2);
          if (sub == 2 && x + 2 < NLIVE) bfrag[(x + 2) % 3] = __builtin_bit_cast(bf16x8, xcur[((x + 2) * kGemmSteps + ks) * 64]);
          __builtin_amdgcn_sched_barrier(0);  // keep this dealing-out as written
        }
      }
    };
    k_step(std::integral_constant<int, 0>{});
    k_step(std::integral_constant<int, 1>{});
    k_step(std::integral_constant<int, 2>{});
    k_step(std::integral_constant<int, 3>{});
    static_assert(kGemmSteps == 4, "four K steps per staged chunk");
    __syncthreads();
  };

  for (int ch = 0; ch < nChunks; ch += 2) {  // nChunks is even: d is padded to 256
    chunk_body(ch, std::integral_constant<int, 0>{});
    chunk_body(ch + 1, std::integral_constant<int, 1>{});
  }

  // the last MFMAs must have left the matrix pipeline before their tiles are read
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);

  // epilogue: acc[sub][x][i] = logit of row x*16 + n, entry vg*64 + sub*16 + gq*4 + i
  if (vg >= nVG) return;
  float osc[4][4];  // (per-entry weight scale, FP8 weights only) / T for this lane's 16 vocabulary entries
#pragma unroll
  for (int sub = 0; sub < 4; ++sub)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = vg * kVocabGroup + sub * 16 + gq * 4 + i;
      osc[sub][i] = (vscale != nullptr && v < V) ? vscale[v] * invT : invT;
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

// One workgroup per vocabulary tile, XCD aware like the other kernels' grids (workgroup b runs on XCD b % 8).
template <int WK, int NLIVE>
__global__ __launch_bounds__(256, 1) void lmhead_gemm_kernel(
    const uint4* __restrict__ Wp, const float* __restrict__ vscale, const uint4* __restrict__ Xp, int R,
    int nChunks, int V, int nVG, int nVGalloc, int nVocabTiles, float invT, float* __restrict__ L,
    int Lld, float2* __restrict__ part) {
  const int vt = blockIdx.x;
  if (vt >= nVocabTiles) return;  // uniform for the whole workgroup, before any barrier
  gemm_tile<WK, NLIVE>(Wp, vscale, Xp, R, nChunks, V, nVG, nVGalloc, invT, L, Lld, part, vt);
}

constexpr size_t kGemmLdsBytes = 2 * (size_t)kGemmRowBlocks * kGemmSteps * 64 * sizeof(uint4);
// The dispatcher gives calls of up to 64 rows to the small-row kernel, so a tile here holds at least 65 rows.
constexpr int kGemmMinLive = 5;

// Instantiations by the number of 16-row blocks that hold rows (65 .. 176 rows): the kernel is bound by the weight
// stream - at half the bytes per weight, FP8, only once the MFMAs of empty blocks are gone.
template <int WK, int NLIVE>
static hipError_t set_lds_limit() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(lmhead_gemm_kernel<WK, NLIVE>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLdsBytes);
}
template <int WK>
static hipError_t set_lds_limits() {
  hipError_t e = set_lds_limit<WK, 5>();
  if (e == hipSuccess) e = set_lds_limit<WK, 6>();
  if (e == hipSuccess) e = set_lds_limit<WK, 7>();
  if (e == hipSuccess) e = set_lds_limit<WK, 8>();
  if (e == hipSuccess) e = set_lds_limit<WK, 9>();
  if (e == hipSuccess) e = set_lds_limit<WK, 10>();
  if (e == hipSuccess) e = set_lds_limit<WK, 11>();
  return e;
}

// More LDS than the default limit of a launch: raised once per process, at context creation (not in the
// launcher, which may run under stream capture).
hipError_t init_lmhead_gemm() {
  static_assert(kGemmMinLive == 5, "instantiations above and below");
  hipError_t e = set_lds_limits<kWBf16>();
  if (e == hipSuccess) e = set_lds_limits<kWFp8>();
  if (e == hipSuccess) e = set_lds_limits<kWInt8>();
  return e;
}

template <int WK>
static void launch_gemm_live(int live, int grid, hipStream_t st, const void* W, const float* vscale, const void* Xp, int R,
                             int nChunks, const Geometry& g, int nVocabTiles, float invT, float* L, float2* part) {
#define JD_LIVE(N)                                                                                                 \
  case N:                                                                                                          \
    hipLaunchKernelGGL((lmhead_gemm_kernel<WK, N>), dim3(grid), dim3(256), kGemmLdsBytes, st,                      \
                       static_cast<const uint4*>(W), vscale, static_cast<const uint4*>(Xp), R, nChunks, g.V, g.nVG, \
                       g.nVGalloc, nVocabTiles, invT, L, g.Vpad, part);                                            \
    break
  switch (live < kGemmMinLive ? kGemmMinLive : live) {
    JD_LIVE(5); JD_LIVE(6); JD_LIVE(7); JD_LIVE(8); JD_LIVE(9); JD_LIVE(10);
    default: JD_LIVE(11);
  }
#undef JD_LIVE
}

hipError_t launch_lmhead_gemm(const void* W, int w_code, const float* vscale, const void* X, int R, const Geometry& g,
                              float invT, float* L, float2* part, void* Xp, hipStream_t st) {
  static_assert(kGroupAlloc % 4 == 0, "a vocabulary tile of 4 groups never leaves the allocation");
  if (R <= 0 || R > kGemmRows || !Xp || !W) return hipErrorInvalidValue;  // one row tile
  const int nChunks = g.dpad / kGemmKChunk;
  hipError_t e = launch_pack_x(X, R, g.d, 1, nChunks, kGemmRowBlocks, kGemmSteps, kGemmRows, 0, -1, 0, Xp, st);
  if (e != hipSuccess) return e;
  const int nVocabTiles = (g.nVG + 3) / 4;
  const int live = (R + 15) / 16;  // row blocks that hold rows
  switch (w_code) {
    case kWFp8: launch_gemm_live<kWFp8>(live, nVocabTiles, st, W, vscale, Xp, R, nChunks, g, nVocabTiles, invT, L, part); break;
    case kWInt8: launch_gemm_live<kWInt8>(live, nVocabTiles, st, W, vscale, Xp, R, nChunks, g, nVocabTiles, invT, L, part); break;
    case kWBf16: launch_gemm_live<kWBf16>(live, nVocabTiles, st, W, vscale, Xp, R, nChunks, g, nVocabTiles, invT, L, part); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace jd
