// Everything after the LM-head contraction: vocabulary-softmax statistics of the draft
// tensor, the accept tests, the judge, the mask combination, the accepted prefix and the
// residual / bonus-token sampler.  All of it is streaming or per-slot work (no MFMA).
#include "jd_kernels.hpp"
#include "side_work.hpp"

namespace jd {

// ------------------------------------------------------------------------------- row stats

// grid = nRows * nSplit, the column ranges of a row adjacent: workgroups that run at the same time stream
// neighbouring memory.  Each block reduces one contiguous column range of one row.
__global__ __launch_bounds__(256) void rowstats_kernel(RowStatsArgs a) {
  __shared__ MS red[4];
  rowstats_block(a, blockIdx.x / a.nSplit, blockIdx.x % a.nSplit, red);
}

RowStatsArgs make_rowstats_args(const float* base, int rowsUsed, size_t seqStride, size_t rowStride, int V,
                                int nSplit, float2* part) {
  RowStatsArgs a;
  a.base = base; a.rowsUsed = rowsUsed; a.seqStride = seqStride; a.rowStride = rowStride;
  a.V = V; a.nSplit = nSplit; a.part = part;
  int splitLen = (V + nSplit - 1) / nSplit;
  a.splitLen = (splitLen + 3) / 4 * 4;
  return a;
}

hipError_t launch_rowstats(const float* base, int nRows, int rowsUsed, size_t seqStride, size_t rowStride, int V,
                           int nSplit, float2* part, hipStream_t st) {
  const RowStatsArgs a = make_rowstats_args(base, rowsUsed, seqStride, rowStride, V, nSplit, part);
  hipLaunchKernelGGL(rowstats_kernel, dim3((unsigned)nRows * (unsigned)nSplit), dim3(256), 0, st, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------- accept

// Per-slot flags handed from the row kernel to the sampler kernels: zflags[b*(M+1) + r].
constexpr uint8_t kZStand = 1, kZJudge = 2, kZBadToken = 4, kZNan = 8;

// One thread's share (every 256th) of n (max, sum exp) partials.  The partials were written by another
// kernel and come from HBM, so eight loads are put in flight before anything is combined, and a batch
// is combined around its common maximum (independent exps, no serial chain).
__device__ __forceinline__ MS combine_partials(const float2* __restrict__ p, int n, int tid) {
  constexpr int kBatch = 8;
  MS st{-INFINITY, 0.f};
  for (int base = 0; base < n; base += 256 * kBatch) {
    float2 v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = base + u * 256 + tid;
      v[u] = (i < n) ? p[i] : make_float2(-INFINITY, 0.f);
    }
    float mx = st.m;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) mx = fmaxf(mx, v[u].x);
    if (mx == -INFINITY) {  // nothing but empty partials so far (keeps NaN sums visible)
#pragma unroll
      for (int u = 0; u < kBatch; ++u) st.s += v[u].y;
    } else {
      float sum = st.s * __expf(st.m - mx);
#pragma unroll
      for (int u = 0; u < kBatch; ++u) sum += v[u].y * __expf(v[u].x - mx);
      st.s = sum;
    }
    st.m = mx;
  }
  return st;
}

// Second pass of the two-pass vocabulary softmax, the judge head and the two accept tests, one workgroup per
// target row (b, r) so that the work spreads over the chip:
//   all rows      combine the LM-head partials of the row                     -> t_max, t_sum
//   rows r < M    (= draft slot j = r) combine the partials of draft row j    -> q_max, q_sum
//                 judge logit g = w_judge . e[b, j+1] + bias (Sec. 4.1; App. B.1), unless it was already
//                 computed beside the LM head
//                 standard test eps*q[c] < p[c] (Eq. 4; or the top-K rule of Sec. 5), judge test g > logit(delta)
// The two test bits and the slot's error flags go to zflags[b*(M+1) + r]; the sampler kernels OR them, ballot
// and cut the prefix.  The gathers of L[c] and D[c] are requested first, so that they travel while the
// partials are combined.
__global__ __launch_bounds__(256) void rows_kernel(AcceptArgs a) {
  __shared__ MS red[4];
  __shared__ float redf[4];
  const int tid = threadIdx.x;
  const int M = a.M, Mp1 = a.M + 1;
  const int row = blockIdx.x;          // b*(M+1) + r
  const int b = row / Mp1, r = row % Mp1;
  const int slot = b * M + r;          // meaningful for r < M
  const bool has_slot = r < M;

  int c = -1;
  float l_c = 0.f, d_c = 0.f, u = 0.f;
  bool tok_ok = false;
  if (has_slot && tid == 0) {
    c = a.tokens[slot];
    tok_ok = c >= 0 && c < a.V;
    if (tok_ok) {
      l_c = a.L[(size_t)row * a.Lld + c];
      d_c = a.D[((size_t)b * a.draft_rows + r) * a.V + c];
    }
    u = a.uniforms[b * Mp1 + r];
  }

  MS t = combine_partials(a.tpart + (size_t)row * a.nPartT, a.nPartT, tid);
  t = ms_block_reduce(t, red);
  if (tid == 0) {
    a.t_max[row] = t.m; a.t_sum[row] = t.s;
    if (a.row_max) a.row_max[row] = t.m;
    if (a.row_sumexp) a.row_sumexp[row] = t.s;
  }
  if (!has_slot) {
    if (tid == 0) a.zflags[row] = isnan(t.s) ? kZNan : 0;
    return;
  }

  MS q{0.f, 1.f};
  if (a.draft_is_logits) {
    __syncthreads();  // red is reused
    q = combine_partials(a.dpart + (size_t)slot * a.nPartD, a.nPartD, tid);
    q = ms_block_reduce(q, red);
    if (tid == 0) { a.q_max[slot] = q.m; a.q_sum[slot] = q.s; }
  }
  float g;
  if (a.judge_done) {
    g = (tid == 0) ? a.g[slot] : 0.f;  // computed beside the LM head
  } else {
    JudgeArgs ja;
    ja.emb_judge = a.emb_judge; ja.w_judge = a.w_judge; ja.emb_is_bf16 = a.emb_is_bf16;
    ja.d = a.d; ja.M = a.M; ja.bias = a.judge_bias; ja.g = a.g;
    g = judge_block(ja, slot, redf);   // valid on thread 0
  }
  if (tid != 0) return;

  bool zs = false, zj = false;
  float p_c = 0.f, q_c = 0.f;
  uint8_t flags = 0;
  if (tok_ok) {
    p_c = expf(l_c - t.m) / t.s;
    q_c = a.draft_is_logits ? expf(d_c - q.m) / q.s : d_c;
    if (a.rule_topk) {  // Sec. 5: among the top_k most probable tokens of p
      int rank = 0;
      for (int s = 0; s < a.nRankSplit; ++s) rank += a.rankpart[(size_t)slot * a.nRankSplit + s];
      zs = rank < a.top_k;
    } else {
      zs = u * q_c < p_c;   // Eq. 4, division-free and strict
    }
    zj = g > a.judge_threshold;
  } else {
    flags |= kZBadToken;
  }
  if (isnan(g) || isnan(t.s) || isnan(q.s) || isnan(q_c)) flags |= kZNan;
  a.zflags[row] = flags | (zs ? kZStand : 0) | (zj ? kZJudge : 0);
  if (a.z_stand) a.z_stand[slot] = zs;
  if (a.z_judge) a.z_judge[slot] = zj;
  if (a.p_at) a.p_at[slot] = p_c;
  if (a.q_at) a.q_at[slot] = q_c;
  if (a.judge_logit) a.judge_logit[slot] = g;
}

// z = z_stand OR z_judge (Sec. 4.1), one wavefront ballot whose trailing ones are the accepted prefix (Eq. 4;
// App. B.2, Fig. 8), and the OR of the sequence's error flags as JD_STATUS_* bits.  Every lane of the calling
// wavefront gets both results; M <= 63, so lanes 0..M hold the M slots and the bonus row.
__device__ __forceinline__ int prefix_from_flags(const uint8_t* __restrict__ zflags, int b, int M, int mode_judge,
                                                 uint32_t* status) {
  const int lane = threadIdx.x & 63;
  const uint8_t f = (lane <= M) ? zflags[b * (M + 1) + lane] : (uint8_t)0;
  const bool z = lane < M && ((f & kZStand) || (mode_judge && (f & kZJudge)));
  const unsigned long long mask = __ballot(z);
  uint32_t st = ((f & kZBadToken) ? 1u : 0u) | ((f & kZNan) ? 2u : 0u);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) st |= __shfl_xor(st, o);
  *status = st;
  return __ffsll((long long)~mask) - 1;  // lanes >= M vote 0, so the result is <= M
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(rows_kernel, dim3(a.B * (a.M + 1)), dim3(256), 0, st, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------- sampler

// Unnormalised mass of token v for sequence b given its accepted prefix m:
//   m <  M : max(0, p_{m+1}[v] - q_{m+1}[v])      (first rejected position)
//   m == M : p_{M+1}[v]                            (bonus token)
// (Sec. 3.1, paragraph after Eq. 4.)  `plain` forces the second form.
struct MassRow {
  const float* l; const float* dq;
  float tm, tinv, qm, qinv;
  int use_q, q_is_logits;
  __device__ __forceinline__ float operator()(int v) const {
    const float p = __expf(l[v] - tm) * tinv;
    if (!use_q) return p;
    const float q = q_is_logits ? __expf(dq[v] - qm) * qinv : dq[v];
    const float r = p - q;
    return (r < 0.f) ? 0.f : r;  // not fmaxf: a NaN must stay visible in the sum
  }
};

// Masses of the four consecutive tokens v0 .. v0+3 (v0 a multiple of 4; tokens >= V get 0).  When the row
// pointers allow it the logits come as one 128-bit load per tensor instead of four 32-bit ones; the values
// and everything computed from them are the same either way.
__device__ __forceinline__ void mass4(const MassRow& row, int v0, int V, double (&out)[4]) {
  const bool vec = v0 + 3 < V && ((reinterpret_cast<uintptr_t>(row.l + v0) | reinterpret_cast<uintptr_t>(row.dq + v0)) & 15) == 0;
  if (vec) {
    const float4 l = *reinterpret_cast<const float4*>(row.l + v0);
    const float lv[4] = {l.x, l.y, l.z, l.w};
    float qv[4] = {0.f, 0.f, 0.f, 0.f};
    if (row.use_q) {
      const float4 q = *reinterpret_cast<const float4*>(row.dq + v0);
      qv[0] = q.x; qv[1] = q.y; qv[2] = q.z; qv[3] = q.w;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float p = __expf(lv[i] - row.tm) * row.tinv;
      float m = p;
      if (row.use_q) {
        const float q = row.q_is_logits ? __expf(qv[i] - row.qm) * row.qinv : qv[i];
        const float r = p - q;
        m = (r < 0.f) ? 0.f : r;  // not fmaxf: a NaN must stay visible in the sum
      }
      out[i] = (double)m;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = (v0 + i < V) ? (double)row(v0 + i) : 0.0;
  }
}

__device__ __forceinline__ MassRow make_mass_row(const SamplerArgs& a, int b, int m, bool plain) {
  const int Mp1 = a.M + 1;
  MassRow r;
  r.l = a.L + (size_t)(b * Mp1 + m) * a.Lld;
  r.tm = a.t_max[b * Mp1 + m];
  r.tinv = 1.f / a.t_sum[b * Mp1 + m];
  r.use_q = (m < a.M) && !plain && !a.resample_target;
  r.q_is_logits = a.draft_is_logits;
  r.dq = a.D; r.qm = 0.f; r.qinv = 1.f;
  if (m < a.M) {
    r.dq = a.D + ((size_t)b * a.draft_rows + m) * a.V;
    if (a.draft_is_logits) { r.qm = a.q_max[b * a.M + m]; r.qinv = 1.f / a.q_sum[b * a.M + m]; }
  }
  return r;
}

// Sum of the masses of one chunk in float64, fixed order: each thread adds its 4
// consecutive tokens, then a fixed tree over the 256 threads.
__device__ __forceinline__ double chunk_sum(const MassRow& row, int chunk, int V, double* red /*[256]*/) {
  const int tid = threadIdx.x;
  const int v0 = chunk * kSamplerChunk + tid * 4;
  double m[4];
  mass4(row, v0, V, m);
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) s += m[i];
  red[tid] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  const double total = red[0];
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(256) void sampler_mass_kernel(SamplerArgs a) {
  __shared__ double red[256];
  const int b = blockIdx.x / a.nChunk, chunk = blockIdx.x % a.nChunk;  // 1-D grid: B is not bounded by 65535
  uint32_t status;
  const int m = prefix_from_flags(a.zflags, b, a.M, a.mode_judge, &status);  // steps 5, 6, in every wavefront
  if (chunk == 0 && threadIdx.x == 0) { a.accept_len[b] = m; a.status[b] = status; }
  const MassRow row = make_mass_row(a, b, m, false);
  const double s = chunk_sum(row, chunk, a.V, red);
  if (threadIdx.x == 0) a.chunk_mass[(size_t)b * a.nChunk + chunk] = s;
}

// Small-row regime (B*(M+1) <= 64, judge logits already computed beside the LM head): the row kernel and the
// sampler's first kernel in ONE launch.  Every workgroup (sequence b, chunk) first recomputes what the row
// kernel computes for its sequence - the M+1 target rows' softmax statistics from the LM head's partials (one
// per row and LM-head workgroup, so a few hundred), the M draft rows' statistics, both tests of every slot, the
// OR, the ballot and the prefix (steps 2-6) - and then sums its chunk of the sampler's masses (step 7).  The
// recomputation costs each workgroup about as much as its chunk; in exchange the call has one dependent launch
// fewer.  Workgroup 0 of a sequence writes the outputs and the statistics the pick kernel reads.
__global__ __launch_bounds__(256) void rows_mass_kernel(AcceptArgs a, SamplerArgs s) {
  __shared__ float2 tstat[64], qstat[64];  // (max, sum exp) of target rows 0..M and draft rows 0..M-1
  __shared__ double red[256];
  __shared__ int s_m;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int M = a.M, Mp1 = a.M + 1;
  const int b = blockIdx.x / s.nChunk, chunk = blockIdx.x % s.nChunk;

  // wavefront 0, lane j = slot j: the gathers travel while the partials are combined
  int c = -1;
  float l_c = 0.f, d_c = 0.f, u = 0.f, g = 0.f;
  bool tok_ok = false;
  if (wave == 0 && lane < M) {
    const int slot = b * M + lane;
    c = a.tokens[slot];
    tok_ok = c >= 0 && c < a.V;
    if (tok_ok) {
      l_c = a.L[(size_t)(b * Mp1 + lane) * a.Lld + c];
      d_c = a.D[((size_t)b * a.draft_rows + lane) * a.V + c];
    }
    u = a.uniforms[b * Mp1 + lane];
    g = a.g[slot];
  }

  // Statistics of the rows: groups of 16 lanes, one row per group and turn (16 rows per turn of the workgroup).
  // A lane's share of a row's partials (up to 32 at a time) is requested in one go and folded around its own
  // maximum - independent exps, one dependent step - then the 16 lanes are combined by four exchange steps.
  const int grp = tid >> 4, gl = tid & 15;
  auto group_reduce = [&](MS st) {
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
      MS t;
      t.m = __shfl_xor(st.m, o);
      t.s = __shfl_xor(st.s, o);
      st = ms_combine(st, t);
    }
    return st;
  };
  // One row per group and pass (two in flight at once were no faster at 26 rows and slower at 6: the folding,
  // not the second load latency, is what a pass costs).  The draft partials of the first 16 slots are requested
  // before the (longer) target rows are worked on.
  constexpr int kPer = 32, kTurns = 1;
  float2 dv[kTurns];
#pragma unroll
  for (int t = 0; t < kTurns; ++t) {
    const int j = 16 * t + grp;
    dv[t] = (a.draft_is_logits && j < M && gl < a.nPartD) ? a.dpart[(size_t)(b * M + j) * a.nPartD + gl]
                                                            : make_float2(-INFINITY, 0.f);
  }
  for (int r0 = 0; r0 <= M; r0 += 16 * kTurns) {
    MS st[kTurns];
    for (int i0 = 0; i0 < a.nPartT; i0 += 16 * kPer) {
      float2 v[kTurns][kPer];
#pragma unroll
      for (int t = 0; t < kTurns; ++t) {
        const int r = r0 + 16 * t + grp;
        const float2* p = a.tpart + (size_t)(b * Mp1 + min(r, M)) * a.nPartT;
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
          const int i = i0 + gl + 16 * e;
          v[t][e] = (r <= M && i < a.nPartT) ? p[i] : make_float2(-INFINITY, 0.f);
        }
      }
#pragma unroll
      for (int t = 0; t < kTurns; ++t) {
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < kPer; ++e) mx = fmaxf(mx, v[t][e].x);
        float sum = 0.f;
        if (mx == -INFINITY) {  // nothing but empty partials (keeps NaN sums visible)
#pragma unroll
          for (int e = 0; e < kPer; ++e) sum += v[t][e].y;
        } else {
#pragma unroll
          for (int e = 0; e < kPer; ++e) sum += v[t][e].y * __expf(v[t][e].x - mx);
        }
        st[t] = (i0 == 0) ? MS{mx, sum} : ms_combine(st[t], MS{mx, sum});
      }
    }
#pragma unroll
    for (int t = 0; t < kTurns; ++t) {
      const int r = r0 + 16 * t + grp;
      const MS o = group_reduce(st[t]);
      if (r <= M && gl == 0) tstat[r] = make_float2(o.m, o.s);
    }
  }
  // draft rows the same way: the nPartD (16) partials of a slot are one per lane of a group
  for (int j0 = 0; j0 < M; j0 += 16) {
    const int j = j0 + grp;
    const bool have = j < M;
    MS st{0.f, 1.f};
    if (a.draft_is_logits) {
      st = MS{-INFINITY, 0.f};
      if (j0 < 16 * kTurns) {
        const float2 x = dv[0];
        static_assert(kTurns == 1, "only the first 16 slots are prefetched");
        st = MS{x.x, x.y};
        for (int i = gl + 16; i < a.nPartD; i += 16) {  // more than 16 partials per slot
          const float2 y = have ? a.dpart[(size_t)(b * M + j) * a.nPartD + i] : make_float2(-INFINITY, 0.f);
          st = ms_combine(st, MS{y.x, y.y});
        }
      } else {
        for (int i = gl; i < a.nPartD; i += 16) {
          const float2 y = have ? a.dpart[(size_t)(b * M + j) * a.nPartD + i] : make_float2(-INFINITY, 0.f);
          st = ms_combine(st, MS{y.x, y.y});
        }
      }
      st = group_reduce(st);
    }
    if (have && gl == 0) qstat[j] = make_float2(st.m, st.s);
  }
  __syncthreads();

  if (wave == 0) {
    const bool first = chunk == 0;  // this workgroup writes the sequence's outputs
    bool zs = false, zj = false;
    float p_c = 0.f, q_c = 0.f;
    uint8_t flags = 0;
    if (lane < M) {
      const float2 t = tstat[lane], q = qstat[lane];
      if (tok_ok) {
        p_c = expf(l_c - t.x) / t.y;
        q_c = a.draft_is_logits ? expf(d_c - q.x) / q.y : d_c;
        zs = u * q_c < p_c;   // Eq. 4, division-free and strict
        zj = g > a.judge_threshold;
      } else {
        flags |= kZBadToken;
      }
      if (isnan(g) || isnan(t.y) || isnan(q.y) || isnan(q_c)) flags |= kZNan;
      flags |= (zs ? kZStand : 0) | (zj ? kZJudge : 0);
      if (first) {
        const int slot = b * M + lane;
        if (a.z_stand) a.z_stand[slot] = zs;
        if (a.z_judge) a.z_judge[slot] = zj;
        if (a.p_at) a.p_at[slot] = p_c;
        if (a.q_at) a.q_at[slot] = q_c;
        if (a.judge_logit) a.judge_logit[slot] = g;
        if (a.draft_is_logits) { a.q_max[slot] = q.x; a.q_sum[slot] = q.y; }
      }
    } else if (lane == M) {
      if (isnan(tstat[M].y)) flags |= kZNan;
    }
    if (lane <= M && first) {
      const float2 t = tstat[lane];
      const int row = b * Mp1 + lane;
      a.zflags[row] = flags;
      a.t_max[row] = t.x; a.t_sum[row] = t.y;
      if (a.row_max) a.row_max[row] = t.x;
      if (a.row_sumexp) a.row_sumexp[row] = t.y;
    }
    const bool z = lane < M && (zs || (s.mode_judge && zj));
    const unsigned long long mask = __ballot(z);
    uint32_t st = ((flags & kZBadToken) ? 1u : 0u) | ((flags & kZNan) ? 2u : 0u);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) st |= __shfl_xor(st, o);
    const int m = __ffsll((long long)~mask) - 1;  // lanes >= M vote 0, so m <= M
    if (lane == 0) {
      s_m = m;
      if (first) { s.accept_len[b] = m; s.status[b] = st; }
    }
  }
  __syncthreads();
  const int m = s_m;

  // step 7, first pass: this workgroup's chunk of the masses of row m
  MassRow row;
  row.l = s.L + (size_t)(b * Mp1 + m) * s.Lld;
  row.tm = tstat[m].x;
  row.tinv = 1.f / tstat[m].y;
  row.use_q = (m < M) && !s.resample_target;
  row.q_is_logits = s.draft_is_logits;
  row.dq = s.D; row.qm = 0.f; row.qinv = 1.f;
  if (m < M) {
    row.dq = s.D + ((size_t)b * s.draft_rows + m) * s.V;
    if (s.draft_is_logits) { row.qm = qstat[m].x; row.qinv = 1.f / qstat[m].y; }
  }
  const double sum = chunk_sum(row, chunk, s.V, red);
  if (tid == 0) s.chunk_mass[(size_t)b * s.nChunk + chunk] = sum;
}

// Block-wide helpers over 256 threads in float64 (fixed order, deterministic).
__device__ __forceinline__ double block_sum256(double v, double* red) {
  const int tid = threadIdx.x;
  red[tid] = v;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  const double total = red[0];
  __syncthreads();
  return total;
}

__device__ __forceinline__ double block_inclusive_scan256(double v, double* red) {
  const int tid = threadIdx.x;
  red[tid] = v;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const double add = (tid >= o) ? red[tid - o] : 0.0;
    __syncthreads();
    red[tid] += add;
    __syncthreads();
  }
  const double r = red[tid];
  __syncthreads();
  return r;
}

__device__ __forceinline__ double total_chunk_mass(const double* cm, int nChunk, double* red) {
  double v = 0.0;
  for (int i = threadIdx.x; i < nChunk; i += 256) v += cm[i];
  return block_sum256(v, red);
}

// Block-wide (256 threads) minimum of `lo` and maximum of `hi`: wavefront reductions, then the four
// wavefront results through LDS.  (LDS atomics on one address from every thread serialise: with them
// this step alone took 5 us of the kernel's 12.)
__device__ __forceinline__ void block_min_max256(int lo, int hi, int* s_lo /*[4]*/, int* s_hi /*[4]*/, int* out_lo,
                                                 int* out_hi) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = min(lo, __shfl_xor(lo, o));
    hi = max(hi, __shfl_xor(hi, o));
  }
  if ((threadIdx.x & 63) == 0) { s_lo[threadIdx.x >> 6] = lo; s_hi[threadIdx.x >> 6] = hi; }
  __syncthreads();
  *out_lo = min(min(s_lo[0], s_lo[1]), min(s_lo[2], s_lo[3]));
  *out_hi = max(max(s_hi[0], s_hi[1]), max(s_hi[2], s_hi[3]));
  __syncthreads();
}

// Inverse CDF in ascending token id: next = min{ v : cdf[v] > u_s * S }.
__global__ __launch_bounds__(256) void sampler_pick_kernel(SamplerArgs a) {
  __shared__ double red[256];
  __shared__ double s_base, s_carry;
  const int b = blockIdx.x, tid = threadIdx.x;
  double* cm = a.chunk_mass + (size_t)b * a.nChunk;

  // Requested before the first barrier, so that these two levels of dependent loads (the slot flags that give
  // the accepted prefix, then the statistics of its row) travel while the chunk masses are summed.
  uint32_t status_unused;
  const int m = prefix_from_flags(a.zflags, b, a.M, a.mode_judge, &status_unused);
  MassRow row = make_mass_row(a, b, m, false);
  const float u_s = a.uniforms[b * (a.M + 1) + a.M];

  double S = total_chunk_mass(cm, a.nChunk, red);
  const bool plain = !(S > 0.0);
  if (tid == 0 && S == 0.0 && m < a.M && !a.resample_target) atomicOr(&a.status[b], 4u);
  // a NaN in the sampled row (target or draft: with draft probabilities nothing else has looked at the
  // whole draft row) must not disappear behind the fallback to p below
  if (tid == 0 && !(S == S)) atomicOr(&a.status[b], 2u);
  if (plain) {
    // No residual mass (q == p at the cut), or NaN: recompute the chunk masses from p itself.
    const MassRow prow = make_mass_row(a, b, m, true);
    for (int ch = 0; ch < a.nChunk; ++ch) {
      const double s = chunk_sum(prow, ch, a.V, red);
      if (tid == 0) cm[ch] = s;
    }
    __syncthreads();
    S = total_chunk_mass(cm, a.nChunk, red);
    if (tid == 0 && !(S == S)) atomicOr(&a.status[b], 2u);
  }
  if (plain) row.use_q = 0;
  const double thresh = (double)u_s * S;

  // first chunk whose inclusive prefix exceeds the threshold
  __shared__ int s_lo[4], s_hi[4];
  int found = 0x7fffffff, lastchunk = -1;
  double carry = 0.0;
  for (int base = 0; base < a.nChunk; base += 256) {
    const int i = base + tid;
    const double val = (i < a.nChunk) ? cm[i] : 0.0;
    const double incl = carry + block_inclusive_scan256(val, red);
    const bool has = i < a.nChunk && val > 0.0;
    int lo, hi;
    block_min_max256((has && incl > thresh) ? i : 0x7fffffff, has ? i : -1, s_lo, s_hi, &lo, &hi);
    lastchunk = max(lastchunk, hi);
    if (lo != 0x7fffffff) {
      found = lo;
      if (i == lo) s_base = incl - val;
      break;
    }
    if (tid == 255) s_carry = incl;
    __syncthreads();
    carry = s_carry;
  }
  if (found == 0x7fffffff) {  // rounding left the threshold beyond the last edge (or S is NaN)
    found = lastchunk < 0 ? 0 : lastchunk;
    if (tid == 0) {
      double run = 0.0;
      for (int i = 0; i < found; ++i) run += cm[i];
      s_base = run;
    }
  }
  __syncthreads();
  const double s_thresh = thresh;

  // Scan inside the chosen chunk: thread t owns tokens 4t..4t+3 of the chunk.
  const int chunk = found;
  const int v0 = chunk * kSamplerChunk + tid * 4;
  double mv[4];
  mass4(row, v0, a.V, mv);
  double local = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) local += mv[i];
  red[tid] = local;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {  // inclusive scan over threads
    const double add = (tid >= o) ? red[tid - o] : 0.0;
    __syncthreads();
    red[tid] += add;
    __syncthreads();
  }
  const double before = s_base + ((tid > 0) ? red[tid - 1] : 0.0);
  // first token in this thread whose cumulative mass exceeds the threshold
  int cand = 0x7fffffff;
  double run = before;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    run += mv[i];
    if (cand == 0x7fffffff && mv[i] > 0.0 && run > s_thresh) cand = v0 + i;
  }
  // last token with mass (fallback when rounding leaves the threshold beyond the chunk)
  int lastpos = -1;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (mv[i] > 0.0) lastpos = v0 + i;
  int s_min, s_last;
  block_min_max256(cand, lastpos, s_lo, s_hi, &s_min, &s_last);
  if (tid == 0) {
    int tok = (s_min != 0x7fffffff) ? s_min : s_last;
    if (tok < 0) tok = 0;
    a.next_token[b] = tok;
  }
}

hipError_t launch_rows_mass(const AcceptArgs& a, const SamplerArgs& s, hipStream_t st) {
  if (a.M > 63 || !a.judge_done || a.rule_topk) return hipErrorInvalidValue;
  if ((size_t)s.nChunk * (size_t)s.B > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rows_mass_kernel, dim3((unsigned)(s.nChunk * s.B)), dim3(256), 0, st, a, s);
  return hipGetLastError();
}

hipError_t launch_sampler_pick(const SamplerArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(sampler_pick_kernel, dim3(a.B), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_sampler(const SamplerArgs& a, hipStream_t st) {
  if ((size_t)a.nChunk * (size_t)a.B > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(sampler_mass_kernel, dim3((unsigned)(a.nChunk * a.B)), dim3(256), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sampler_pick_kernel, dim3(a.B), dim3(256), 0, st, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------- top-K rule

// grid = (B*M, kRankSplits).  Counts, over one column range of target row j of sequence b, the
// tokens that rank before the drafted token c: larger logit, or equal logit and lower id.
__global__ __launch_bounds__(256) void rank_kernel(const float* __restrict__ L, int Lld,
                                                    const int32_t* __restrict__ tokens, int M, int V, int splitLen,
                                                    int* __restrict__ rankpart) {
  __shared__ int red[4];
  const int slot = blockIdx.x, split = blockIdx.y, tid = threadIdx.x;
  const int b = slot / M, j = slot % M;
  const int c = tokens[slot];
  int cnt = 0;
  if (c >= 0 && c < V) {
    const float* row = L + (size_t)(b * (M + 1) + j) * Lld;
    const float lc = row[c];
    // splitLen is a multiple of 4 and rows of L are 256-byte aligned: 128-bit loads, four per thread in
    // flight before anything is compared (the count is an integer: the order does not matter)
    const int c0 = split * splitLen, c1 = min(V, c0 + splitLen);
    const int nvec = (c1 > c0) ? (c1 - c0) / 4 : 0;
    const float4* row4 = reinterpret_cast<const float4*>(row + c0);
    constexpr int kBatch = 4;
    for (int i0 = 0; i0 < nvec; i0 += 256 * kBatch) {
      float4 x[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int i = i0 + u * 256 + tid;
        x[u] = (i < nvec) ? row4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (i0 + u * 256 + tid >= nvec) continue;
        const int v = c0 + (i0 + u * 256 + tid) * 4;
        cnt += (x[u].x > lc) || (x[u].x == lc && v < c);
        cnt += (x[u].y > lc) || (x[u].y == lc && v + 1 < c);
        cnt += (x[u].z > lc) || (x[u].z == lc && v + 2 < c);
        cnt += (x[u].w > lc) || (x[u].w == lc && v + 3 < c);
      }
    }
    for (int v = c0 + nvec * 4 + tid; v < c1; v += 256) {
      const float l = row[v];
      cnt += (l > lc) || (l == lc && v < c);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
  if ((tid & 63) == 0) red[tid >> 6] = cnt;
  __syncthreads();
  if (tid == 0) rankpart[(size_t)slot * gridDim.y + split] = red[0] + red[1] + red[2] + red[3];
}

hipError_t launch_rank(const float* L, int Lld, const int32_t* tokens, int B, int M, int V, int* rankpart,
                       hipStream_t st) {
  const int splitLen = ((V + kRankSplits - 1) / kRankSplits + 3) / 4 * 4;
  hipLaunchKernelGGL(rank_kernel, dim3(B * M, kRankSplits), dim3(256), 0, st, L, Lld, tokens, M, V, splitLen,
                     rankpart);
  return hipGetLastError();
}

// grid = (nChunk, B): lowest id in the chunk whose logit equals the row maximum (INT_MAX if none).
__global__ __launch_bounds__(256) void argmax_chunk_kernel(const float* __restrict__ L, int Lld,
                                                            const float* __restrict__ t_max,
                                                            const uint8_t* __restrict__ zflags, int mode_judge,
                                                            int32_t* __restrict__ accept_len,
                                                            uint32_t* __restrict__ status, int M, int V,
                                                            int nChunk, int* __restrict__ chunk_arg) {
  __shared__ int s_min;
  const int b = blockIdx.x / nChunk, chunk = blockIdx.x % nChunk, tid = threadIdx.x;  // 1-D grid, as the sampler's
  uint32_t st;
  const int m = prefix_from_flags(zflags, b, M, mode_judge, &st);
  if (chunk == 0 && tid == 0) { accept_len[b] = m; status[b] = st; }
  const int r = b * (M + 1) + m;
  const float tm = t_max[r];
  const float* row = L + (size_t)r * Lld;
  if (tid == 0) s_min = 0x7fffffff;
  __syncthreads();
  int cand = 0x7fffffff;
  const int v0 = chunk * kSamplerChunk + tid * 4;
#pragma unroll
  for (int i = 3; i >= 0; --i)
    if (v0 + i < V && row[v0 + i] == tm) cand = v0 + i;
  if (cand != 0x7fffffff) atomicMin(&s_min, cand);
  __syncthreads();
  if (tid == 0) chunk_arg[(size_t)b * nChunk + chunk] = s_min;
}

__global__ __launch_bounds__(256) void argmax_pick_kernel(const int* __restrict__ chunk_arg, int nChunk,
                                                           int32_t* __restrict__ next_token) {
  __shared__ int s_min;
  const int b = blockIdx.x, tid = threadIdx.x;
  if (tid == 0) s_min = 0x7fffffff;
  __syncthreads();
  int cand = 0x7fffffff;
  for (int i = tid; i < nChunk; i += 256) cand = min(cand, chunk_arg[(size_t)b * nChunk + i]);
  if (cand != 0x7fffffff) atomicMin(&s_min, cand);
  __syncthreads();
  if (tid == 0) next_token[b] = (s_min == 0x7fffffff) ? 0 : s_min;  // no finite maximum (NaN row): token 0
}

hipError_t launch_argmax(const float* L, int Lld, const float* t_max, const uint8_t* zflags, int mode_judge,
                         int32_t* accept_len, uint32_t* status, int B, int M, int V, int* chunk_arg, int nChunk,
                         int32_t* next_token, hipStream_t st) {
  if ((size_t)nChunk * (size_t)B > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(argmax_chunk_kernel, dim3((unsigned)(nChunk * B)), dim3(256), 0, st, L, Lld, t_max, zflags,
                     mode_judge, accept_len, status, M, V, nChunk, chunk_arg);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(argmax_pick_kernel, dim3(B), dim3(256), 0, st, chunk_arg, nChunk, next_token);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------- probs

__global__ __launch_bounds__(256) void probs_kernel(const float* __restrict__ L, int Lld,
                                                     const float* __restrict__ t_max,
                                                     const float* __restrict__ t_sum, int V, int nColBlocks,
                                                     float* __restrict__ probs) {
  const int r = blockIdx.x / nColBlocks;  // 1-D grid: the row count is not bounded by 65535
  const int v = (blockIdx.x % nColBlocks) * 256 + threadIdx.x;
  if (v >= V) return;
  probs[(size_t)r * V + v] = expf(L[(size_t)r * Lld + v] - t_max[r]) / t_sum[r];
}

hipError_t launch_probs(const float* L, int Lld, const float* t_max, const float* t_sum, int R, int V, float* probs,
                        hipStream_t st) {
  const int nColBlocks = (V + 255) / 256;
  if ((size_t)nColBlocks * (size_t)R > 0x7fffffffULL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(probs_kernel, dim3((unsigned)(nColBlocks * R)), dim3(256), 0, st, L, Lld, t_max, t_sum, V,
                     nColBlocks, probs);
  return hipGetLastError();
}

// ---- final RMS normalisation (pre-norm wiring) --------------------------------------------
// One workgroup per row.  float64 throughout: the products h*h and h*gamma are exact, the sum, the
// reciprocal square root and the last product round once each, so the value that is finally
// rounded to the storage type agrees with a float64 reference to ~1e-16 and the stored bits agree
// unless the value sits that close to a rounding tie.

constexpr int kNormThreads = 1024;

__device__ __forceinline__ double block_sum_f64(double v, double* sh) {  // kNormThreads threads
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < kNormThreads / 64; ++w) t += sh[w];
  __syncthreads();
  return t;
}

// float64 -> bfloat16, round to nearest even, through a float32 that is truncated and carries a
// sticky bit (round to odd), so that the two steps together round exactly once.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
  const float f = __double2float_rz(x);
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  if ((double)f != x) u |= 1u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ double bf16_to_f64(uint32_t bits16) { return (double)__uint_as_float(bits16 << 16); }

// bf16 rows, d % 8 == 0: 128-bit loads and stores, eight values per lane per trip.  The first
// kKeep trips of a lane (rows up to kKeep * 8192 values) stay in registers between the two passes,
// and the gain is fetched beside them, so that a row costs one trip to memory.
__global__ __launch_bounds__(kNormThreads) void rmsnorm_rows_bf16_kernel(const uint4* __restrict__ H,
                                                                         const uint4* __restrict__ G, double eps,
                                                                         int d, uint4* __restrict__ X) {
  constexpr int kKeep = 2;
  __shared__ double sh[kNormThreads / 64];
  const int nv = d / 8;
  const uint4* h = H + (size_t)blockIdx.x * nv;
  uint4* x = X + (size_t)blockIdx.x * nv;
  auto sum_sq = [](const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double lo = bf16_to_f64(w[i] & 0xffffu), hi = bf16_to_f64(w[i] >> 16);
      s += lo * lo;
      s += hi * hi;
    }
    return s;
  };
  auto scale = [](const uint4& v, const uint4& gv, double inv) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w}, gw[4] = {gv.x, gv.y, gv.z, gv.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo = f64_to_bf16_rne(bf16_to_f64(w[i] & 0xffffu) * bf16_to_f64(gw[i] & 0xffffu) * inv);
      const uint32_t hi = f64_to_bf16_rne(bf16_to_f64(w[i] >> 16) * bf16_to_f64(gw[i] >> 16) * inv);
      o[i] = lo | (hi << 16);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
  };
  uint4 hv[kKeep], gv[kKeep];
#pragma unroll
  for (int u = 0; u < kKeep; ++u) {
    const int k = threadIdx.x + u * kNormThreads;
    hv[u] = (k < nv) ? h[k] : make_uint4(0u, 0u, 0u, 0u);
    gv[u] = (k < nv) ? G[k] : make_uint4(0u, 0u, 0u, 0u);
  }
  double ss = 0.0;
#pragma unroll
  for (int u = 0; u < kKeep; ++u) ss += sum_sq(hv[u]);
  for (int k = threadIdx.x + kKeep * kNormThreads; k < nv; k += kNormThreads) ss += sum_sq(h[k]);
  ss = block_sum_f64(ss, sh);
  const double inv = 1.0 / sqrt(ss / (double)d + eps);
#pragma unroll
  for (int u = 0; u < kKeep; ++u) {
    const int k = threadIdx.x + u * kNormThreads;
    if (k < nv) x[k] = scale(hv[u], gv[u], inv);
  }
  for (int k = threadIdx.x + kKeep * kNormThreads; k < nv; k += kNormThreads) x[k] = scale(h[k], G[k], inv);
}

__global__ __launch_bounds__(kNormThreads) void rmsnorm_rows_f32_kernel(const float* __restrict__ H,
                                                                        const float* __restrict__ G, double eps,
                                                                        int d, float* __restrict__ X) {
  __shared__ double sh[kNormThreads / 64];
  const float* h = H + (size_t)blockIdx.x * d;
  float* x = X + (size_t)blockIdx.x * d;
  double ss = 0.0;
  for (int k = threadIdx.x; k < d; k += kNormThreads) {
    const double v = (double)h[k];
    ss += v * v;
  }
  ss = block_sum_f64(ss, sh);
  const double inv = 1.0 / sqrt(ss / (double)d + eps);
  for (int k = threadIdx.x; k < d; k += kNormThreads) x[k] = (float)((double)h[k] * (double)G[k] * inv);
}

hipError_t launch_rmsnorm_rows(const void* H, const void* gamma, double eps, int is_bf16, int R, int d, void* Xn,
                               hipStream_t st) {
  if (R <= 0 || d <= 0 || !H || !gamma || !Xn) return hipErrorInvalidValue;
  if (is_bf16) {
    if (d % 8 != 0) return hipErrorInvalidValue;  // the bf16 path requires it everywhere (128-bit rows)
    hipLaunchKernelGGL(rmsnorm_rows_bf16_kernel, dim3(R), dim3(kNormThreads), 0, st, static_cast<const uint4*>(H),
                       static_cast<const uint4*>(gamma), eps, d, static_cast<uint4*>(Xn));
  } else {
    hipLaunchKernelGGL(rmsnorm_rows_f32_kernel, dim3(R), dim3(kNormThreads), 0, st, static_cast<const float*>(H),
                       static_cast<const float*>(gamma), eps, d, static_cast<float*>(Xn));
  }
  return hipGetLastError();
}

// ---- the step after verification: grow each sequence's context ------------------------------
// One wavefront per sequence; lane i < n copies accepted draft token i, lane n writes the new token.
__global__ __launch_bounds__(256) void append_tokens_kernel(int B, int M, const int32_t* __restrict__ draft_tokens,
                                                            const int32_t* __restrict__ accept_len,
                                                            const int32_t* __restrict__ next_token,
                                                            int32_t* __restrict__ token_buf, int cap,
                                                            int32_t* __restrict__ lengths) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (b >= B) return;
  const int n = min(max(accept_len[b], 0), M);  // M <= 63: one lane per token
  const int len = min(max(lengths[b], 0), cap);
  if (lane <= n) {
    const int32_t t = lane < n ? draft_tokens[(size_t)b * M + lane] : next_token[b];
    if (len + lane < cap) token_buf[(size_t)b * cap + len + lane] = t;
  }
  if (lane == 0) lengths[b] = min(len + n + 1, cap);
}

hipError_t launch_append_tokens(int B, int M, const int32_t* draft_tokens, const int32_t* accept_len,
                                const int32_t* next_token, int32_t* token_buf, int cap, int32_t* lengths,
                                hipStream_t st) {
  if (B < 1 || M < 1 || M > 63 || cap < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(append_tokens_kernel, dim3((B + 3) / 4), dim3(256), 0, st, B, M, draft_tokens, accept_len,
                     next_token, token_buf, cap, lengths);
  return hipGetLastError();
}

}  // namespace jd
