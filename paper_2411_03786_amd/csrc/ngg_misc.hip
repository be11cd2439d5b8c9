// Small kernels of the verify step: embedding gather, RMSNorm, draft construction
// (Sections 4.1-4.3), greedy argmax + acceptance (introduction: keep a drafted token when the
// model would have predicted it) and the KV commit (Appendix D).  All integer work is exact.
#include "ngg_internal.h"

#include <algorithm>

namespace ngg {

// ---------------------------------------------------------------------------------------------
// block tokens + embedding gather.  A verify block (Section 3: input block (k, w+1)) in the
// shared-first-column layout: token 0 is the uncached last context token, token m >= 1 is drafted
// token m - 1 of the k x w draft batch (row-major: the same order).  In prefill mode token m is
// history token hist_base + m.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T *tok_emb, const int32_t *hist, const int32_t *drafts,
                                                    int32_t *block_tok, float *h, int d, int hist_base, int mode,
                                                    const int32_t *n_dev) {
  const int m = blockIdx.x;
  if (n_dev) hist_base = *n_dev - 1;
  // mode 0: a verify block whose rows share token 0 (the last context token), then the drafts row by row;
  // mode 1: consecutive history tokens; mode 2: single-column rows, every one the last context token
  const int tok = mode == 1 ? hist[hist_base + m] : (m == 0 || mode == 2 ? hist[hist_base] : drafts[m - 1]);
  if (threadIdx.x == 0) block_tok[m] = tok;
  const T *e = tok_emb + (size_t)tok * d;
  for (int i = 4 * threadIdx.x; i < d; i += 1024) {         // d is a multiple of 32: four elements per load
    float4 v;
    if constexpr (sizeof(T) == 2) {
      const bf16x4 q = *reinterpret_cast<const bf16x4 *>(e + i);
      v = float4{(float)q[0], (float)q[1], (float)q[2], (float)q[3]};
    } else {
      v = *reinterpret_cast<const float4 *>(e + i);
    }
    *reinterpret_cast<float4 *>(h + (size_t)m * d + i) = v;
  }
}

void launch_embed(int dtype, const void *tok_emb, const int32_t *hist, const int32_t *drafts, int32_t *block_tok,
                  float *h, int d, int M, int hist_base, int mode, hipStream_t s, const int32_t *n_dev) {
  if (dtype == 1)
    hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(M), dim3(256), 0, s, (const bf16_t *)tok_emb, hist, drafts, block_tok,
                       h, d, hist_base, mode, n_dev);
  else
    hipLaunchKernelGGL(embed_kernel<float>, dim3(M), dim3(256), 0, s, (const float *)tok_emb, hist, drafts, block_tok, h,
                       d, hist_base, mode, n_dev);
}

// ---------------------------------------------------------------------------------------------
// RMSNorm, split in two: this kernel adds the residual partials, stores the new residual stream and
// writes xg = h * gain (not yet divided by the root mean square) as the next GEMM's input, and the
// sum of squares of its part of the row; the GEMM multiplies its accumulators by
// 1 / sqrt(sum of squares / d + eps) in the epilogue (the GEMM is linear in its input rows).  That
// lets `segs` workgroups share a row: a single workgroup per row left one CU to pull the whole row
// and all its partials, with most CUs idle.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum_256(float v, float *sh) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const float t = sh[0] + sh[1] + sh[2] + sh[3];
  __syncthreads();
  return t;
}

// Every thread owns J groups of 4 consecutive features of segment blockIdx.y (group index
// tid + 256*j): all loads of the row and of its residual partials are issued before anything is
// used, so the kernel costs one memory round trip instead of one per feature.
// U: storage type of the gain (the user's weights); T: internal element type of xn.
template <typename U, typename T, int J>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float *__restrict__ h, const float *__restrict__ hpart, int n_part,
                                                      size_t part_stride, const U *__restrict__ gain, T *__restrict__ xn,
                                                      int d, int Mcap, float *__restrict__ row_ss) {
  __shared__ float sh[4];
  const int m = blockIdx.x, segs = gridDim.y;
  const int d4 = d / segs / 4, c4 = blockIdx.y * d4;       // float4 groups of this segment, first group
  float4 v[J];
  float4 gn[J];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int i4 = threadIdx.x + 256 * j;
    v[j] = float4{0.f, 0.f, 0.f, 0.f};
    gn[j] = float4{0.f, 0.f, 0.f, 0.f};
    if (i4 < d4) {
      v[j] = *reinterpret_cast<const float4 *>(h + (size_t)m * d + 4 * (c4 + i4));
      const U *gp = gain + 4 * (c4 + i4);
      gn[j] = float4{to_f32(gp[0]), to_f32(gp[1]), to_f32(gp[2]), to_f32(gp[3])};
    }
  }
  if constexpr (J > 4) {                                  // wide rows: too many registers to fetch every split at once
    for (int s = 0; s < n_part; ++s) {
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int i4 = threadIdx.x + 256 * j;
        if (i4 < d4) {
          const float4 p = *reinterpret_cast<const float4 *>(hpart + (size_t)s * part_stride + (size_t)m * d + 4 * (c4 + i4));
          v[j].x += p.x; v[j].y += p.y; v[j].z += p.z; v[j].w += p.w;
        }
      }
    }
  } else if (n_part > 0) {                                // residual add: partials in split order.  All splits
    float4 p[kMaxResidualSplits][J];                      // are fetched at once (a loop over n_part would pay
#pragma unroll                                            // one memory round trip per split); surplus slots
    for (int s = 0; s < kMaxResidualSplits; ++s) {        // repeat the last split and are not added
      const int sc = s < n_part ? s : n_part - 1;
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int i4 = threadIdx.x + 256 * j;
        p[s][j] = float4{0.f, 0.f, 0.f, 0.f};
        if (i4 < d4) p[s][j] = *reinterpret_cast<const float4 *>(hpart + (size_t)sc * part_stride + (size_t)m * d + 4 * (c4 + i4));
      }
    }
#pragma unroll
    for (int s = 0; s < kMaxResidualSplits; ++s) {
      if (s < n_part) {
#pragma unroll
        for (int j = 0; j < J; ++j) { v[j].x += p[s][j].x; v[j].y += p[s][j].y; v[j].z += p[s][j].z; v[j].w += p[s][j].w; }
      }
    }
  }
  float ss = 0.0f;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int i4 = threadIdx.x + 256 * j;
    ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
    if (i4 < d4) {
      if (n_part > 0) *reinterpret_cast<float4 *>(h + (size_t)m * d + 4 * (c4 + i4)) = v[j];
      T *o = xn + act_offset<T>(m, 4 * (c4 + i4), Mcap);   // 4 features stay inside one chunk
      store4(o, v[j].x * gn[j].x, v[j].y * gn[j].y, v[j].z * gn[j].z, v[j].w * gn[j].w);
    }
  }
  ss = block_sum_256(ss, sh);
  if (threadIdx.x == 0) row_ss[(size_t)m * kNormSegs + blockIdx.y] = ss;
}

// segments a row is split into: up to kNormSegs, each at least 1024 features wide
int rmsnorm_segments(int d) {
  int segs = d / 1024;
  segs = segs < 1 ? 1 : (segs > kNormSegs ? kNormSegs : segs);
  while (d % (segs * 4)) --segs;
  return segs;
}

template <typename U>
static void launch_rmsnorm_t(float *h, const float *hpart, int n_part, size_t part_stride, const void *gain, void *xn, int d,
                             int M, int Mcap, float *row_ss, hipStream_t s) {
  typedef typename Internal<U>::type T;
  const int segs = rmsnorm_segments(d);
  const int j = (d / segs / 4 + 255) / 256;
#define NGG_NORM(J)                                                                                                        \
  hipLaunchKernelGGL((rmsnorm_kernel<U, T, J>), dim3(M, segs), dim3(256), 0, s, h, hpart, n_part, part_stride, (const U *)gain, \
                     (T *)xn, d, Mcap, row_ss)
  if (j <= 1) NGG_NORM(1);
  else if (j <= 2) NGG_NORM(2);
  else if (j <= 4) NGG_NORM(4);
  else if (j <= 8) NGG_NORM(8);
  else NGG_NORM(16);
#undef NGG_NORM
}

void launch_rmsnorm(int dtype, float *h, const float *hpart, int n_part, size_t part_stride, const void *gain, void *xn,
                    int d, int M, int Mcap, float *row_ss, hipStream_t s) {
  if (dtype == 1) launch_rmsnorm_t<bf16_t>(h, hpart, n_part, part_stride, gain, xn, d, M, Mcap, row_ss, s);
  else launch_rmsnorm_t<float>(h, hpart, n_part, part_stride, gain, xn, d, M, Mcap, row_ss, s);
}

// rows of a row-major matrix of the user's weights -> chunk-major activation layout in the internal type
// (used to feed embedding rows to the GEMM); `centre` (fp32 [d], may be null) is subtracted first, then the
// value is multiplied by `scale` (a power of two that the GEMM's out_scale undoes)
template <typename U, typename T>
__global__ __launch_bounds__(256) void pack_rows_kernel(const U *src, T *dst, int d, int Mcap, const float *centre, float scale) {
  for (int i = threadIdx.x; i < d; i += 256) {
    const float v = to_f32(src[(size_t)blockIdx.x * d + i]);
    dst[act_offset<T>(blockIdx.x, i, Mcap)] = from_f32<T>((centre ? v - centre[i] : v) * scale);
  }
}

void launch_pack_rows(int dtype, const void *src, void *dst, int d, int M, int Mcap, hipStream_t s, float scale,
                      const float *centre) {
  if (dtype == 1)
    hipLaunchKernelGGL((pack_rows_kernel<bf16_t, half_t>), dim3(M), dim3(256), 0, s, (const bf16_t *)src, (half_t *)dst, d, Mcap, centre, scale);
  else
    hipLaunchKernelGGL((pack_rows_kernel<float, float>), dim3(M), dim3(256), 0, s, (const float *)src, (float *)dst, d, Mcap, centre, scale);
}

// largest magnitude of a matrix, left as an fp32 bit pattern (magnitudes order like unsigned integers)
template <typename U>
__global__ __launch_bounds__(256) void absmax_kernel(const U *src, size_t n, unsigned *out_bits) {
  __shared__ float sh[4];
  float m = 0.0f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) m = fmaxf(m, fabsf(to_f32(src[i])));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) atomicMax(out_bits, __float_as_uint(fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]))));
}

void launch_absmax(int dtype, const void *src, size_t n, unsigned *out_bits, hipStream_t s) {
  const unsigned blocks = (unsigned)std::min<size_t>(2048, (n + 255) / 256);
  if (dtype == 1) hipLaunchKernelGGL(absmax_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)src, n, out_bits);
  else hipLaunchKernelGGL(absmax_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)src, n, out_bits);
}

// mean[i] = (1/N) sum over rows of src[n][i]: one workgroup per 256 columns, rows summed in index
// order by every thread (deterministic); used once, for the mean output embedding of the unigram
template <typename T>
__global__ __launch_bounds__(256) void column_mean_kernel(const T *src, int N, int d, float *mean) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d) return;
  float acc = 0.0f;
  for (int n = 0; n < N; ++n) acc += to_f32(src[(size_t)n * d + i]);
  mean[i] = acc / (float)N;
}

void launch_column_mean(int dtype, const void *src, int N, int d, float *mean, hipStream_t s) {
  if (dtype == 1) hipLaunchKernelGGL(column_mean_kernel<bf16_t>, dim3((d + 255) / 256), dim3(256), 0, s, (const bf16_t *)src, N, d, mean);
  else hipLaunchKernelGGL(column_mean_kernel<float>, dim3((d + 255) / 256), dim3(256), 0, s, (const float *)src, N, d, mean);
}

// out[m] = -sum_v rows[m][v]^2 (the negated squared unigram distance: largest = nearest), one workgroup per row
__global__ __launch_bounds__(256) void neg_row_sumsq_kernel(const float *__restrict__ rows, int V, float *__restrict__ out) {
  __shared__ float sh[4];
  const float *row = rows + (size_t)blockIdx.x * V;
  float acc = 0.0f;
  for (int i = threadIdx.x; i < V; i += 256) acc += row[i] * row[i];
  acc = block_sum_256(acc, sh);
  if (threadIdx.x == 0) out[blockIdx.x] = -acc;
}

void launch_neg_row_sumsq(const float *rows, int M, int V, float *out, hipStream_t s) {
  hipLaunchKernelGGL(neg_row_sumsq_kernel, dim3(M), dim3(256), 0, s, rows, V, out);
}

// ---------------------------------------------------------------------------------------------
// Context N-gram matcher (Section 4.2), one workgroup of 1024 threads.
// For each query length q (q_max down to q_min): collect every window start i <= n-q-w whose
// first q tokens equal the last q context tokens; group equal w-token continuations; rank groups
// by (count desc, last start desc); append continuations not taken yet until k_ctx_max rows.
// Counts and last starts do not depend on the order in which matches were collected, so the
// result is deterministic although the lists are filled with atomics.
//
// Grouping and ranking take one of two routes that give the same groups:
//  * up to kSmallMatches matches: every match is compared with every other one, every group with
//    every other group (a few hundred compares per thread, no atomics on memory);
//  * more (a frequent last token on a long context; a periodic context makes every window a
//    match): the continuations go into an open-addressing hash table in the scratch memory, keyed
//    by a hash of the w tokens and resolved by comparing the tokens themselves, each slot holding
//    (a representative start, count, last start); the ranked prefix is then pulled out by
//    repeated selection, every wave over its share of the groups and wave 0 over the waves'
//    picks.  Linear in the number of matches.
// ---------------------------------------------------------------------------------------------
constexpr int kSmallMatches = 256;

__device__ __forceinline__ bool same_cont(const int32_t *x, int a, int b, int w) {
  for (int t = 0; t < w; ++t)
    if (x[a + t] != x[b + t]) return false;
  return true;
}

__device__ __forceinline__ unsigned cont_hash(const int32_t *x, int a, int w) {
  unsigned h = 0x811c9dc5u;
  for (int t = 0; t < w; ++t) h = (h ^ (unsigned)x[a + t]) * 0x01000193u;
  h ^= h >> 15;
  h *= 0x2c1b3c6du;
  h ^= h >> 12;
  return h;
}

// rank key of a group: count in the high word, last start in the low word (distinct groups have
// distinct last starts, so keys are unique); 0 = none
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned lo = __shfl_xor((unsigned)v, off), hi = __shfl_xor((unsigned)(v >> 32), off);
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    v = o > v ? o : v;
  }
  return v;
}

__global__ __launch_bounds__(1024) void ctx_match_kernel(const DraftArgs a) {
  constexpr int NWAVE = 16, WANT_MAX = 64;
  __shared__ int n_match, n_rep, n_taken;
  __shared__ int cand[WANT_MAX];                 // start of the continuation ranked r among this q's groups
  __shared__ unsigned long long wkey[NWAVE * WANT_MAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t *x = a.hist;
  const int n = a.n_dev ? *a.n_dev : a.n, w = a.w;
  const int kmax = min(a.k_ctx_max, a.k);
  if (tid == 0) n_taken = 0;
  __syncthreads();
  if (w >= 1 && kmax >= 1) {
    for (int q = a.q_max; q >= a.q_min; --q) {
      if (q < 1 || n < q + w) continue;                     // uniform
      if (tid == 0) { n_match = 0; n_rep = 0; }
      if (tid < WANT_MAX) cand[tid] = -1;
      __syncthreads();
      if (n_taken >= kmax) break;                           // uniform: read after the barrier
      const int last_start = n - q - w;
      for (int i = tid; i <= last_start; i += 1024) {
        bool eq = true;
        for (int t = 0; t < q; ++t) eq = eq && (x[i + t] == x[n - q + t]);
        if (eq) a.mlist[atomicAdd(&n_match, 1)] = i;
      }
      __syncthreads();
      const int nm = n_match;
      const int want = min(2 * kmax, WANT_MAX);
      if (nm <= kSmallMatches) {
        for (int t = tid; t < nm; t += 1024) {
          const int i = a.mlist[t];
          int cnt = 0, last = i;
          for (int u = 0; u < nm; ++u) {
            const int j = a.mlist[u];
            if (same_cont(x, i + q, j + q, w)) { ++cnt; last = max(last, j); }
          }
          if (last == i) {                                  // one representative per continuation
            const int slot = atomicAdd(&n_rep, 1);
            a.reps[2 * slot] = cnt;
            a.reps[2 * slot + 1] = i;
          }
        }
        __syncthreads();
        const int nr = n_rep;
        for (int t = tid; t < nr; t += 1024) {
          const int cnt = a.reps[2 * t], i = a.reps[2 * t + 1];
          int rank = 0;
          for (int u = 0; u < nr; ++u) {
            const int c2 = a.reps[2 * u], i2 = a.reps[2 * u + 1];
            rank += (c2 > cnt || (c2 == cnt && i2 > i)) ? 1 : 0;
          }
          if (rank < want) cand[rank] = i + q;
        }
      } else {
        // ---- hash grouping: T >= 2 nm slots of (representative start, count, last start) ----------
        int T = 128;
        while (T < 2 * nm) T <<= 1;                           // T <= a.gtab_slots: the launcher sized it for 2 n matches
        int *g_rep = a.gtab, *g_cnt = a.gtab + a.gtab_slots, *g_last = a.gtab + 2 * a.gtab_slots;
        for (int sl = tid; sl < T; sl += 1024) { g_rep[sl] = -1; g_cnt[sl] = 0; g_last[sl] = -1; }
        __syncthreads();
        for (int t = tid; t < nm; t += 1024) {
          const int i = a.mlist[t];
          unsigned sl = cont_hash(x, i + q, w) & (unsigned)(T - 1);
          for (int probe = 0; probe < T; ++probe) {         // the table is at most half full: an empty slot turns up
            const int r = atomicCAS(&g_rep[sl], -1, i);
            if (r == -1 || same_cont(x, r + q, i + q, w)) {
              atomicAdd(&g_cnt[sl], 1);
              atomicMax(&g_last[sl], i);
              break;
            }
            sl = (sl + 1) & (unsigned)(T - 1);
          }
        }
        __syncthreads();
        // groups -> reps[] as (count, last start); the table was written by atomics, which act on the L2:
        // read it there too (a plain load could hit a line the previous q left in this CU's L1)
        for (int sl = tid; sl < T; sl += 1024) {
          const int r = __hip_atomic_load(&g_rep[sl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (r != -1) {
            const int slot = atomicAdd(&n_rep, 1);
            a.reps[2 * slot] = __hip_atomic_load(&g_cnt[sl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            a.reps[2 * slot + 1] = __hip_atomic_load(&g_last[sl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
        __syncthreads();
        const int nr = n_rep;
        // ---- the `want` best groups in order: round r takes the largest key below the previous pick ----
        unsigned long long prev = ~0ull;
        for (int r = 0; r < want; ++r) {
          unsigned long long best = 0;
          for (int e = tid; e < nr; e += 1024) {
            const unsigned long long key = ((unsigned long long)(unsigned)a.reps[2 * e] << 32) | (unsigned)a.reps[2 * e + 1];
            if (key < prev && key > best) best = key;
          }
          best = wave_max_u64(best);
          if (lane == 0) wkey[wave * WANT_MAX + r] = best;
          prev = best;
          if (best == 0) {                                  // this wave's share ran out: the later rounds are empty too
            if (lane == 0)
              for (int r2 = r + 1; r2 < want; ++r2) wkey[wave * WANT_MAX + r2] = 0;
            break;
          }
        }
        __syncthreads();
        if (wave == 0) {
          unsigned long long prev0 = ~0ull;
          for (int r = 0; r < want; ++r) {
            unsigned long long best = 0;
            for (int e = lane; e < NWAVE * WANT_MAX; e += 64) {
              const unsigned long long key = (e % WANT_MAX) < want ? wkey[e] : 0;
              if (key < prev0 && key > best) best = key;
            }
            best = wave_max_u64(best);
            if (best == 0) break;
            if (lane == 0) cand[r] = (int)(unsigned)best + q;
            prev0 = best;
          }
        }
      }
      __syncthreads();
      if (tid == 0) {
        int taken = n_taken;
        for (int r = 0; r < want && taken < kmax; ++r) {
          const int c = cand[r];
          if (c < 0) break;
          bool dup = false;
          for (int p = 0; p < taken && !dup; ++p) {
            bool eq = true;
            for (int t = 0; t < w; ++t) eq = eq && (a.ctx_rows[p * w + t] == x[c + t]);
            dup = eq;
          }
          if (!dup) {
            for (int t = 0; t < w; ++t) a.ctx_rows[taken * w + t] = x[c + t];
            ++taken;
          }
        }
        n_taken = taken;
      }
      __syncthreads();
    }
  }
  if (tid == 0) *a.n_ctx = n_taken;
}

// ---------------------------------------------------------------------------------------------
// Model bigram scores z[v] = <unemb[v], tok_emb[x_last]> (Section 4.1).  The output embedding is
// read in operand order: a wave owns groups of 16 vocabulary rows and streams them as one flat
// sequence of 1 KB fragment loads, a ring of 8 ahead; the contraction runs on MFMA with the
// embedding of x_last as every column of the other operand (the matrix cores are idle anyway and
// this keeps the vector ALU out of the way of the loads).  fp32 accumulation.
// ---------------------------------------------------------------------------------------------
constexpr int kGemvBlocks = 256;     // workgroups of the bigram sweep; each keeps its own top-k candidates
constexpr int kCandStride = 32;      // candidate slots per workgroup (k <= 32)
constexpr int kGemvRing = 8;

__device__ __forceinline__ bool ranks_before(float v, int i, float ov, int oi) {   // (value desc, id asc)
  return v > ov || (v == ov && i < oi);
}

template <typename U, typename T>
__global__ __launch_bounds__(256) void bigram_gemv_kernel(const U *tok_emb, const T *unemb_t, const int32_t *hist, int n, const int32_t *n_dev,
                                                          int d, int vocab, int ksel, float *z, float *cand_val,
                                                          int *cand_idx, float emb_scale, float out_scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gemv_smem[];
  T *es = reinterpret_cast<T *>(gemv_smem);                  // [d] embedding of x_last (times emb_scale, internal type)
  float *zs = reinterpret_cast<float *>(gemv_smem + (size_t)d * sizeof(T));   // this block's scores
  if (n_dev) n = *n_dev;
  const int x = hist[n - 1];
  for (int i = threadIdx.x; i < d; i += 256) es[i] = from_f32<T>(to_f32(tok_emb[(size_t)x * d + i]) * emb_scale);
  __syncthreads();
  const int lane = threadIdx.x & 63, li = lane & 15, g = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_steps = d / 32, n_groups = vocab / 16;
  const int gpb = (n_groups + gridDim.x - 1) / gridDim.x;   // 16-row groups per workgroup
  const int g0 = blockIdx.x * gpb, g1 = min(n_groups, g0 + gpb);
  const int my_groups = g1 > g0 + wave ? (g1 - g0 - wave + 3) / 4 : 0;        // groups g0 + wave, + 4, ...
  const int total = my_groups * n_steps;                    // this wave's fragment loads, as one sequence
  int pg = 0, ps = 0;                                       // prefetch cursor: (group counter, step)
  auto next_frag = [&]() {                                  // past the end it repeats an in-bounds load
    const int grp = min(g0 + wave + 4 * pg, n_groups - 1);
    const Frag<T> f = load_frag_stream(tiled_block(unemb_t, grp, n_steps, lane) + (size_t)ps * 512);
    if (pg < my_groups && ++ps == n_steps) { ps = 0; ++pg; }
    return f;
  };
  Frag<T> ring[kGemvRing];
#pragma unroll
  for (int u = 0; u < kGemvRing; ++u) ring[u] = next_frag();
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  int s = 0, gi = 0;                                        // step inside the current group, group counter
  for (int t0 = 0; t0 < total; t0 += kGemvRing) {
#pragma unroll
    for (int u = 0; u < kGemvRing; ++u) {
      if (t0 + u < total) {                                  // uniform per wave
        mma(acc, ring[u], load_frag(es + s * 32 + g * 8));   // every column of the result is the same score
        if (++s == n_steps) {                               // group done: column 0 holds its 16 scores
          const int grp = g0 + wave + 4 * gi;
          if (li == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              z[grp * 16 + 4 * g + r] = acc[r] * out_scale;
              zs[(grp - g0) * 16 + 4 * g + r] = acc[r] * out_scale;
            }
          }
          acc = f32x4{0.f, 0.f, 0.f, 0.f};
          s = 0;
          ++gi;
        }
      }
      ring[u] = next_frag();
    }
  }
  __syncthreads();
  // this workgroup's ksel best scores, by (value desc, id asc): wave 0 pulls them out one by one; an entry
  // is "still in" when it ranks strictly after the last one taken
  if (wave == 0) {
    const int cnt = max(0, g1 - g0) * 16;
    float last_v = 0.0f;
    int last_i = -1;
    for (int r = 0; r < ksel; ++r) {
      float bv = kNegBig;
      int bi = 0x7fffffff;
      for (int j = lane; j < cnt; j += 64) {
        const float v = zs[j];
        const int id = g0 * 16 + j;
        if (r > 0 && !ranks_before(last_v, last_i, v, id)) continue;      // already taken
        if (ranks_before(v, id, bv, bi)) { bv = v; bi = id; }
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (ranks_before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      if (lane == 0) {
        cand_val[blockIdx.x * kCandStride + r] = bv;         // (kNegBig, INT_MAX) once the block ran out
        cand_idx[blockIdx.x * kCandStride + r] = bi;
      }
      last_v = bv;
      last_i = bi;
    }
  }
}

// One-off copy of a row-major matrix into operand order (see tiled_offset).  Destination row of
// source row n: row_map 0: row0 + n.  row_map 1 (q, k, v): inside every block of 2*half rows (a head)
// row i < half goes to 16*(i/8) + i%8 and row half + i to 16*(i/8) + 8 + i%8, so a 16-row fragment
// holds 8 rotary pairs (i, i + half).  row_map 2 / 3 (gate / up): row n goes to 16*(n/8) + n%8 (+ 8
// for up), so a fragment holds gate and up of 8 features.
__host__ __device__ inline int tile_dest_row(int n, int row_map, int half) {
  if (row_map == 1) {
    const int blk = n / (2 * half), i = n - blk * 2 * half;
    const int second = i >= half ? 1 : 0, ii = i - second * half;
    return blk * 2 * half + 16 * (ii / 8) + 8 * second + ii % 8;
  }
  if (row_map >= 2) return 16 * (n / 8) + 8 * (row_map - 2) + n % 8;
  return n;
}

template <typename U, typename T>
__global__ __launch_bounds__(256) void tile_weights_kernel(const U *src, T *dst, int N, int K, int row0, int row_map, int half,
                                                           float scale) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int pieces = K / 8;
  if (idx >= (size_t)N * pieces) return;
  const int n = (int)(idx / pieces), k = (int)(idx % pieces) * 8;
  const U *p = src + (size_t)n * K + k;
  T *q = dst + tiled_offset(row0 + tile_dest_row(n, row_map, half), k, K, (int)sizeof(T));
  if constexpr (sizeof(T) == 2) {
    // stored bf16 value times a power of two, rounded to fp16: exact unless it falls more than 2^31 below the matrix maximum
    const u32x4 raw = *reinterpret_cast<const u32x4 *>(p);
    const bf16_t *e = reinterpret_cast<const bf16_t *>(&raw);
    half8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = to_half(to_f32(e[i]) * scale);
    *reinterpret_cast<half8 *>(q) = o;
  } else {
    *reinterpret_cast<u32x4 *>(q) = *reinterpret_cast<const u32x4 *>(p);
    *reinterpret_cast<u32x4 *>(q + 256) = *reinterpret_cast<const u32x4 *>(p + 4);
  }
}

void launch_tile_weights(int dtype, const void *src, void *dst, int N, int K, int row0, hipStream_t s, float scale, int row_map,
                         int half) {
  const size_t total = (size_t)N * (K / 8);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dtype == 1)
    hipLaunchKernelGGL((tile_weights_kernel<bf16_t, half_t>), dim3(blocks), dim3(256), 0, s, (const bf16_t *)src, (half_t *)dst, N, K,
                       row0, row_map, half, scale);
  else
    hipLaunchKernelGGL((tile_weights_kernel<float, float>), dim3(blocks), dim3(256), 0, s, (const float *)src, (float *)dst, N, K,
                       row0, row_map, half, scale);
}

// Top-(k - n_ctx) of z by (score desc, id asc), chained extension through next1, and assembly of
// the k x w draft batch (Section 4.3: context rows first, the extended bigram fills the rest).
// Selection in two levels without a barrier per rank: every wave ranks its own 512 candidate slots
// (round r takes the best candidate that ranks after the wave's previous pick), then wave 0 ranks
// the 16 waves' survivors the same way.
__global__ __launch_bounds__(1024) void topk_assemble_kernel(const DraftArgs a) {
  constexpr int NWAVE = 16;
  __shared__ float wv[NWAVE * kCandStride];
  __shared__ int wi[NWAVE * kCandStride];
  __shared__ int top[kCandStride];
  constexpr int CPT = kGemvBlocks * kCandStride / 1024;     // candidate slots per thread
  constexpr int SPL = NWAVE * kCandStride / 64;             // survivor slots per lane of wave 0
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_ctx = *a.n_ctx;
  const int k_big = a.w >= 1 ? a.k - n_ctx : 0;
  // best of n values per lane that rank after (last_v, last_i), over the wave
  auto wave_pick = [&](const float *v, const int *id, int n, bool first, float last_v, int last_i, float &bv, int &bi) {
    bv = kNegBig;
    bi = 0x7fffffff;
    for (int j = 0; j < n; ++j) {
      const bool in = first || ranks_before(last_v, last_i, v[j], id[j]);
      if (in && ranks_before(v[j], id[j], bv, bi)) { bv = v[j]; bi = id[j]; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ranks_before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
  };
  if (k_big > 0) {
    // the candidates every workgroup of the sweep kept (its own top-k): the global top-k is among them
    float cv[CPT];
    int ci[CPT];
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int slot = tid + 1024 * j;
      const bool used = (slot % kCandStride) < a.k;
      cv[j] = used ? a.cand_val[slot] : kNegBig;
      ci[j] = used ? a.cand_idx[slot] : 0x7fffffff;
    }
    float last_v = 0.0f;
    int last_i = -1;
    for (int r = 0; r < k_big; ++r) {
      float bv;
      int bi;
      wave_pick(cv, ci, CPT, r == 0, last_v, last_i, bv, bi);
      last_v = bv;
      last_i = bi;
      if (lane == 0) { wv[wave * kCandStride + r] = bv; wi[wave * kCandStride + r] = bi; }
    }
  }
  __syncthreads();
  if (wave == 0 && k_big > 0) {
    float sv[SPL];
    int si[SPL];
#pragma unroll
    for (int j = 0; j < SPL; ++j) {
      const int e = lane + 64 * j;
      const bool used = (e % kCandStride) < k_big;
      sv[j] = used ? wv[e] : kNegBig;
      si[j] = used ? wi[e] : 0x7fffffff;
    }
    float last_v = 0.0f;
    int last_i = -1;
    for (int r = 0; r < k_big; ++r) {
      float bv;
      int bi;
      wave_pick(sv, si, SPL, r == 0, last_v, last_i, bv, bi);
      last_v = bv;
      last_i = bi;
      if (lane == 0) top[r] = bi;
    }
  }
  __syncthreads();
  if (tid < a.k && a.w >= 1) {
    const int r = tid;
    if (r < n_ctx) {
      for (int t = 0; t < a.w; ++t) a.drafts[r * a.w + t] = a.ctx_rows[r * a.w + t];
      a.row_src[r] = 0;
    } else {
      int t0 = top[r - n_ctx];
      for (int t = 0; t < a.w; ++t) {
        a.drafts[r * a.w + t] = t0;
        if (t + 1 < a.w) t0 = a.next1[t0];              // w - 1 dependent lookups
      }
      a.row_src[r] = 1;
    }
  } else if (tid < a.k) {
    a.row_src[tid] = 1;
  }
}

// The same assembly when the bigram comes from the precomputed full-model table (Section 4.1:
// the bigram and its extension are O(1) lookups): row i starts with the table's i-th ranked
// successor of the last token and continues with each token's top-ranked successor.
__global__ __launch_bounds__(64) void table_assemble_kernel(const DraftArgs a) {
  const int r = threadIdx.x;
  const int n_ctx = *a.n_ctx;
  if (r >= a.k) return;
  if (a.w < 1) { a.row_src[r] = 1; return; }
  if (r < n_ctx) {
    for (int t = 0; t < a.w; ++t) a.drafts[r * a.w + t] = a.ctx_rows[r * a.w + t];
    a.row_src[r] = 0;
  } else {
    // first token: the (r - n_ctx)-th ranked successor of the last token in the bigram table, or the
    // (r - n_ctx)-th nearest token of the unigram (context-free); then each token's top-ranked successor
    int t0 = a.uni_top ? a.uni_top[r - n_ctx] : a.bg_table[(size_t)a.hist[(a.n_dev ? *a.n_dev : a.n) - 1] * a.bg_K + (r - n_ctx)];
    for (int t = 0; t < a.w; ++t) {
      a.drafts[r * a.w + t] = t0;
      t0 = a.bg_table ? a.bg_table[(size_t)t0 * a.bg_K] : a.next1[t0];
    }
    a.row_src[r] = 1;
  }
}

void launch_ctx_match(const DraftArgs &a, hipStream_t s) { hipLaunchKernelGGL(ctx_match_kernel, dim3(1), dim3(1024), 0, s, a); }

void launch_build_drafts(int dtype, const DraftArgs &a, hipStream_t s) {
  if (a.bg_table || a.uni_top) {
    hipLaunchKernelGGL(ctx_match_kernel, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(table_assemble_kernel, dim3(1), dim3(64), 0, s, a);
    return;
  }
  // the sweep first: it is the long kernel, and while it runs the host gets the short ones queued
  // (a step starts with an idle queue, where every launch costs its full submission latency)
  if (a.w >= 1) {
    const int n_groups = a.vocab / 16, gpb = (n_groups + kGemvBlocks - 1) / kGemvBlocks;
    const size_t lds = (size_t)a.d * (dtype == 1 ? 2 : 4) + (size_t)gpb * 16 * sizeof(float);
    const float out_scale = 1.0f / (a.emb_scale * a.unemb_scale);       // powers of two: exact
    if (dtype == 1)
      hipLaunchKernelGGL((bigram_gemv_kernel<bf16_t, half_t>), dim3(kGemvBlocks), dim3(256), lds, s, (const bf16_t *)a.tok_emb,
                         (const half_t *)a.unemb_t, a.hist, a.n, a.n_dev, a.d, a.vocab, a.k, a.z, a.cand_val, a.cand_idx,
                         a.emb_scale, out_scale);
    else
      hipLaunchKernelGGL((bigram_gemv_kernel<float, float>), dim3(kGemvBlocks), dim3(256), lds, s, (const float *)a.tok_emb,
                         (const float *)a.unemb_t, a.hist, a.n, a.n_dev, a.d, a.vocab, a.k, a.z, a.cand_val, a.cand_idx,
                         a.emb_scale, out_scale);
  }
  hipLaunchKernelGGL(ctx_match_kernel, dim3(1), dim3(1024), 0, s, a);
  hipLaunchKernelGGL(topk_assemble_kernel, dim3(1), dim3(1024), 0, s, a);
}

// ---------------------------------------------------------------------------------------------
// Greedy argmax over the vocabulary (lowest id on ties) from the unembedding's per-tile partial
// maxima, accepted length of every row, winner (lowest row on ties) and the new tokens.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void wave_argmax(float &bv, int &bi) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(bv, off);
    const int oi = __shfl_xor(bi, off);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
}

// greedy[r*C + j] = argmax over the vocabulary after block token block_index(r, j), from the per-tile maxima; one
// workgroup per entry of the grid (in the shared-first-column layout the k entries of column 0 read the same token)
__global__ __launch_bounds__(256) void argmax_reduce_kernel(const float *__restrict__ pmax_val,
                                                            const int *__restrict__ pmax_idx, int tiles, int Mcap,
                                                            int32_t *greedy, int C, int shared0) {
  __shared__ float wv[4];
  __shared__ int wi[4];
  const int tid = threadIdx.x;
  const int m = block_index(blockIdx.x / C, blockIdx.x % C, C, shared0);
  float bv = kNegBig;
  int bi = 0x7fffffff;
  for (int t0 = tid; t0 < tiles; t0 += 1024) {              // four independent loads in flight
    float v[4];
    int ix[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = t0 + 256 * u;
      v[u] = t < tiles ? pmax_val[(size_t)t * Mcap + m] : kNegBig;
      ix[u] = t < tiles ? pmax_idx[(size_t)t * Mcap + m] : 0x7fffffff;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (v[u] > bv || (v[u] == bv && ix[u] < bi)) { bv = v[u]; bi = ix[u]; }
  }
  wave_argmax(bv, bi);
  if ((tid & 63) == 0) { wv[tid >> 6] = bv; wi[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int t = 1; t < 4; ++t)
      if (wv[t] > bv || (wv[t] == bv && wi[t] < bi)) { bv = wv[t]; bi = wi[t]; }
    greedy[blockIdx.x] = bi;
  }
}

__global__ __launch_bounds__(64) void accept_kernel(int k, int C, const int32_t *drafts, const int8_t *row_src,
                                                    const int32_t *n_ctx, int32_t *res, int greedy_off) {
  const int tid = threadIdx.x;
  const int32_t *greedy = res + greedy_off;
  const int w = C - 1;
  for (int r = tid; r < k; r += 64) {
    int acc = 0;
    while (acc < w && drafts[r * w + acc] == greedy[r * C + acc]) ++acc;
    res[RES_ACCEPT + r] = acc;
  }
  __syncthreads();
  if (tid == 0) {
    int win = 0, best = res[RES_ACCEPT];
    for (int r = 1; r < k; ++r)
      if (res[RES_ACCEPT + r] > best) { best = res[RES_ACCEPT + r]; win = r; }
    res[RES_WINNER] = win;
    res[RES_NACCEPT] = best;
    res[RES_NNEW] = best + 1;
    for (int i = 0; i < best; ++i) res[RES_NEWTOK + i] = drafts[win * w + i];
    res[RES_NEWTOK + best] = greedy[win * C + best];
    // what the draft builder left about these rows travels with the result
    res[RES_NCTX] = *n_ctx;
    res[RES_WINSRC] = row_src[win];
  }
}

void launch_argmax_accept(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int rows, int k, int C, int shared0,
                          const int32_t *drafts, const int8_t *row_src, const int32_t *n_ctx, int32_t *res, int greedy_off,
                          hipStream_t s) {
  hipLaunchKernelGGL(argmax_reduce_kernel, dim3(rows * C), dim3(256), 0, s, pmax_val, pmax_idx, tiles, Mcap, res + greedy_off, C,
                     shared0);
  if (k > 0) hipLaunchKernelGGL(accept_kernel, dim3(1), dim3(64), 0, s, k, C, drafts, row_src, n_ctx, res, greedy_off);
}

void launch_next1_finish(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int M, int32_t *next1_out,
                         hipStream_t s) {
  hipLaunchKernelGGL(argmax_reduce_kernel, dim3(M), dim3(256), 0, s, pmax_val, pmax_idx, tiles, Mcap, next1_out, 1, 0);
}

// ---------------------------------------------------------------------------------------------
// Top-K token ids of each logits row by (value desc, id asc): K rounds of a workgroup-wide
// selection, round i taking the best entry that ranks after round i-1's pick.  Used once per
// vocabulary entry when the full-model bigram table is built, never on the step.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void row_topk_kernel(const float *__restrict__ logits, int V, int K, int32_t *__restrict__ out) {
  __shared__ float wv[4];
  __shared__ int wi[4];
  __shared__ float sel_v;
  __shared__ int sel_i;
  const int m = blockIdx.x, tid = threadIdx.x;
  const float *row = logits + (size_t)m * V;
  float last_v = 0.0f;
  int last_i = -1;
  for (int r = 0; r < K; ++r) {
    float bv = kNegBig;
    int bi = 0x7fffffff;
    for (int i = tid; i < V; i += 256) {
      const float v = row[i];
      const bool in = r == 0 || ranks_before(last_v, last_i, v, i);
      if (in && ranks_before(v, i, bv, bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ranks_before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if ((tid & 63) == 0) { wv[tid >> 6] = bv; wi[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
      float fv = wv[0];
      int fi = wi[0];
      for (int t = 1; t < 4; ++t)
        if (ranks_before(wv[t], wi[t], fv, fi)) { fv = wv[t]; fi = wi[t]; }
      sel_v = fv; sel_i = fi;
      out[(size_t)m * K + r] = fi;
    }
    __syncthreads();
    last_v = sel_v;
    last_i = sel_i;
    __syncthreads();
  }
}

void launch_row_topk(const float *logits, int M, int V, int K, int32_t *out, hipStream_t s) {
  hipLaunchKernelGGL(row_topk_kernel, dim3(M), dim3(256), 0, s, logits, V, K, out);
}

__global__ void iota_kernel(int32_t *dst, int first, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = first + i;
}

// Streaming-read probe: every workgroup reads its contiguous share of the buffer once with 16-byte non-temporal
// loads, eight in flight per thread, and leaves one checksum word (so that nothing is optimised away).
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4 *__restrict__ src, size_t n16, unsigned *__restrict__ sink) {
  const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * per_wg, hi = lo + per_wg < n16 ? lo + per_wg : n16;
  unsigned acc = 0;
  size_t i = lo + threadIdx.x;
  for (; i + 7 * 256 < hi; i += 8 * 256) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < hi; i += 256) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (acc == 0x9e3779b9u) sink[blockIdx.x] = acc;           // practically never: the load results must stay live
}

void launch_read_probe(const void *src, size_t bytes, unsigned *sink, int blocks, hipStream_t s) {
  hipLaunchKernelGGL(read_probe_kernel, dim3(blocks), dim3(256), 0, s, (const u32x4 *)src, bytes / 16, sink);
}

__global__ void noop_kernel() {}

void launch_noop(hipStream_t s) { hipLaunchKernelGGL(noop_kernel, dim3(1), dim3(64), 0, s); }

void launch_iota(int32_t *dst, int first, int n, hipStream_t s) {
  hipLaunchKernelGGL(iota_kernel, dim3((n + 255) / 256), dim3(256), 0, s, dst, first, n);
}

// ---------------------------------------------------------------------------------------------
// Commit (Appendix D): the winner row's keys/values for block columns 0 .. n_new-1 become cache
// positions P .. P+n_new-1; the new tokens are appended to the history at P+1 ...
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void commit_kernel(T *kcache, T *vcache, const T *kscr, const T *vscr, int Hkv, int hd,
                                                     int Spad, int Mcap, int C, int shared0, int P, const int32_t *res, int fixed_row,
                                                     int fixed_n, int max_new, int32_t *hist, const int32_t *n_dev) {
  const int layer = blockIdx.y, hkv = blockIdx.x;
  if (n_dev) P = *n_dev - 1;
  int row = fixed_row, n_new = fixed_n;
  if (res) { row = res[RES_WINNER]; n_new = min(res[RES_NNEW], max_new); }
  const size_t lh = (size_t)layer * Hkv + hkv;
  const T *ks = kscr + lh * Mcap * hd;
  const T *vs = vscr + lh * hd * Mcap;
  T *kc = kcache + lh * Spad * hd;
  T *vc = vcache + lh * hd * Spad;
  for (int i = threadIdx.x; i < n_new * hd; i += 256) {
    const int j = i / hd, dd = i - j * hd;
    const int src = block_index(row, j, C, shared0), dst = P + j;   // both live in tiles of 32 positions, in operand order
    kc[k_offset(dst, dd, hd, (int)sizeof(T))] = ks[k_offset(src, dd, hd, (int)sizeof(T))];
    vc[v_offset(dst, dd, hd, (int)sizeof(T))] = vs[v_offset(src, dd, hd, (int)sizeof(T))];
  }
  if (res && layer == 0 && hkv == 0)
    for (int i = threadIdx.x; i < n_new; i += 256) hist[P + 1 + i] = res[RES_NEWTOK + i];
}

void launch_commit(int dtype, void *kcache, void *vcache, const void *kscr, const void *vscr, int L, int Hkv, int hd,
                   int Spad, int Mcap, int C, int shared0, int P, const int32_t *res, int fixed_row, int fixed_n, int max_new,
                   int32_t *hist, hipStream_t s, const int32_t *n_dev) {
  if (dtype == 1)
    hipLaunchKernelGGL(commit_kernel<half_t>, dim3(Hkv, L), dim3(256), 0, s, (half_t *)kcache, (half_t *)vcache,
                       (const half_t *)kscr, (const half_t *)vscr, Hkv, hd, Spad, Mcap, C, shared0, P, res, fixed_row, fixed_n,
                       max_new, hist, n_dev);
  else
    hipLaunchKernelGGL(commit_kernel<float>, dim3(Hkv, L), dim3(256), 0, s, (float *)kcache, (float *)vcache,
                       (const float *)kscr, (const float *)vscr, Hkv, hd, Spad, Mcap, C, shared0, P, res, fixed_row, fixed_n,
                       max_new, hist, n_dev);
}

__global__ void advance_kernel(int32_t *n_dev, const int32_t *res, int max_new) { *n_dev += min(res[RES_NNEW], max_new); }

void launch_advance(int32_t *n_dev, const int32_t *res, int max_new, hipStream_t s) {
  hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(1), 0, s, n_dev, res, max_new);
}

}  // namespace ngg
