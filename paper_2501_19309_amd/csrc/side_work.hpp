// Device code shared by the LM-head kernel and the tail kernels: the online-softmax state,
// the first softmax pass over one column range of one fp32 row, and one judge dot product.
// In the small-row regime these two pieces of work do not depend on the LM head, so they
// ride in the LM-head launch as extra workgroups ("side work") instead of launches of their own.
#pragma once

#include "jd_kernels.hpp"

namespace jd {

// Online-softmax state: m = running max, s = sum exp(x - m).
struct MS { float m, s; };

__device__ __forceinline__ MS ms_combine(MS a, MS b) {
  const float m = fmaxf(a.m, b.m);
  if (m == -INFINITY) return MS{m, a.s + b.s};  // both empty (keeps NaN sums visible)
  MS o;
  o.m = m;
  o.s = a.s * __expf(a.m - m) + b.s * __expf(b.m - m);
  return o;
}

// Fold one logit into the state.  A logit of -inf (a masked token) has probability zero and leaves
// the state alone; a NaN makes the sum NaN.
__device__ __forceinline__ MS ms_push(MS st, float x) {
  if (x != x) { st.s = NAN; return st; }
  if (x == -INFINITY) return st;
  if (x > st.m) { st.s *= __expf(st.m - x); st.m = x; }
  st.s += __expf(x - st.m);
  return st;
}

__device__ __forceinline__ MS ms_wave_reduce(MS v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    MS t;
    t.m = __shfl_xor(v.m, o);
    t.s = __shfl_xor(v.s, o);
    v = ms_combine(v, t);
  }
  return v;
}

__device__ __forceinline__ MS ms_block_reduce(MS st, MS* red /*[4]*/) {
  st = ms_wave_reduce(st);
  const int tid = threadIdx.x;
  if ((tid & 63) == 0) red[tid >> 6] = st;
  __syncthreads();
  return ms_combine(ms_combine(red[0], red[1]), ms_combine(red[2], red[3]));
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ float dot8_bf16(uint4 a, uint4 b, float acc) {
  acc = fmaf(bf16_lo(a.x), bf16_lo(b.x), acc); acc = fmaf(bf16_hi(a.x), bf16_hi(b.x), acc);
  acc = fmaf(bf16_lo(a.y), bf16_lo(b.y), acc); acc = fmaf(bf16_hi(a.y), bf16_hi(b.y), acc);
  acc = fmaf(bf16_lo(a.z), bf16_lo(b.z), acc); acc = fmaf(bf16_hi(a.z), bf16_hi(b.z), acc);
  acc = fmaf(bf16_lo(a.w), bf16_lo(b.w), acc); acc = fmaf(bf16_hi(a.w), bf16_hi(b.w), acc);
  return acc;
}

// First pass of the vocabulary softmax over columns [split*splitLen, (split+1)*splitLen) of one
// fp32 row (the draft logits, Sec. 3.1 Eq. 3 handed over as logits; also the target logits on
// the fp32 path).  256 threads; thread 0 writes part[row*nSplit + split] = (max, sum exp).
__device__ __forceinline__ void rowstats_block(const RowStatsArgs& a, int row, int split, MS* red /*[4]*/) {
  const float* p = a.base + (size_t)(row / a.rowsUsed) * a.seqStride + (size_t)(row % a.rowsUsed) * a.rowStride;
  const int c0 = split * a.splitLen;
  const int c1 = min(a.V, c0 + a.splitLen);
  MS st{-INFINITY, 0.f};
  const int tid = threadIdx.x;
  if (((reinterpret_cast<uintptr_t>(p) & 15) == 0)) {  // splitLen is a multiple of 4
    const int nvec = (c1 > c0) ? (c1 - c0) / 4 : 0;
    const float4* p4 = reinterpret_cast<const float4*>(p + c0);
    // four 128-bit loads per thread are in flight before any of them is used (non-temporal: of these rows only
    // single elements and one row per sequence are read again); a batch is folded in
    // around its own maximum (one rescale of the running sum, sixteen independent exps)
    constexpr int kBatch = 4;
    for (int i0 = 0; i0 < nvec; i0 += 256 * kBatch) {
      float4 x[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int i = i0 + u * 256 + tid;
        x[u] = (i < nvec) ? load_stream(p4 + i) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      }
      float mb = -INFINITY;
#pragma unroll
      for (int u = 0; u < kBatch; ++u) mb = fmaxf(mb, fmaxf(fmaxf(x[u].x, x[u].y), fmaxf(x[u].z, x[u].w)));
      if (mb == -INFINITY) {
        // padding or logits of -inf (probability zero) - or nothing but NaNs, which fmaxf drops: only this rare
        // case needs a look at every element.  With a finite maximum a NaN reaches the sum through its own exp.
        bool nan = false;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) nan = nan || (x[u].x != x[u].x) || (x[u].y != x[u].y) || (x[u].z != x[u].z) || (x[u].w != x[u].w);
        if (nan) st.s = NAN;
        continue;
      }
      if (mb > st.m) { st.s *= __expf(st.m - mb); st.m = mb; }
      float add = 0.f;
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        add += (__expf(x[u].x - st.m) + __expf(x[u].y - st.m)) + (__expf(x[u].z - st.m) + __expf(x[u].w - st.m));
      st.s += add;
    }
    for (int c = c0 + nvec * 4 + tid; c < c1; c += 256) st = ms_push(st, p[c]);
  } else {
    for (int c = c0 + tid; c < c1; c += 256) st = ms_push(st, p[c]);
  }
  const MS o = ms_block_reduce(st, red);
  if (tid == 0) a.part[(size_t)row * a.nSplit + split] = make_float2(o.m, o.s);
}

// Judge logit of draft slot blk = b*M + j:  g = w_judge . e[b, j+1, :] + bias  (Sec. 4.1; App. B.1).
// 256 threads; thread 0 writes a.g[blk] and returns it (other threads return 0).
__device__ __forceinline__ float judge_block(const JudgeArgs& a, int blk, float* redf /*[4]*/) {
  const int tid = threadIdx.x;
  const int b = blk / a.M, j = blk % a.M;
  const size_t e0 = ((size_t)b * (a.M + 1) + j + 1) * a.d;
  float acc = 0.f;
  if (a.emb_is_bf16) {  // d % 8 == 0 and 16-byte aligned rows on this path
    const uint4* w = reinterpret_cast<const uint4*>(a.w_judge);
    const uint4* e = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(a.emb_judge) + e0);
    for (int i = tid; i < a.d / 8; i += 256) acc = dot8_bf16(w[i], e[i], acc);
  } else {
    const float* w = reinterpret_cast<const float*>(a.w_judge);
    const float* e = reinterpret_cast<const float*>(a.emb_judge) + e0;
    for (int k = tid; k < a.d; k += 256) acc = fmaf(w[k], e[k], acc);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if ((tid & 63) == 0) redf[tid >> 6] = acc;
  __syncthreads();
  float g = 0.f;
  if (tid == 0) {
    g = (redf[0] + redf[1]) + (redf[2] + redf[3]) + a.bias;
    a.g[blk] = g;
  }
  return g;
}

// Workgroups [0, nStatBlocks) do row statistics, [nStatBlocks, nStatBlocks + nJudgeBlocks) judge dots.
__device__ __forceinline__ void side_work_block(const SideWork& w, int blk, void* smem16 /*>= 32 B*/) {
  if (blk < w.nStatBlocks) {
    rowstats_block(w.stats, blk / w.stats.nSplit, blk % w.stats.nSplit, static_cast<MS*>(smem16));
  } else if (blk - w.nStatBlocks < w.nJudgeBlocks) {
    (void)judge_block(w.judge, blk - w.nStatBlocks, static_cast<float*>(smem16));
  }
}

}  // namespace jd
