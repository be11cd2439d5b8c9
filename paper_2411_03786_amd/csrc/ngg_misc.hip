// Small kernels of the verify step: embedding gather, RMSNorm, draft construction
// (Sections 4.1-4.3), greedy argmax + acceptance (introduction: keep a drafted token when the
// model would have predicted it) and the KV commit (Appendix D).  All integer work is exact.
#include "ngg_internal.h"

namespace ngg {

// ---------------------------------------------------------------------------------------------
// block tokens + embedding gather.  Block position m = r*C + j holds the uncached last context
// token for j = 0 and row r's drafted token j-1 otherwise (Section 3: input block (k, w+1)); in
// prefill mode it holds history token hist_base + m.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T *tok_emb, const int32_t *hist, const int32_t *drafts,
                                                    int32_t *block_tok, float *h, int d, int C, int w, int hist_base,
                                                    int from_hist) {
  const int m = blockIdx.x;
  int tok;
  if (from_hist) tok = hist[hist_base + m];
  else {
    const int r = m / C, j = m - r * C;
    tok = j == 0 ? hist[hist_base] : drafts[r * w + j - 1];
  }
  if (threadIdx.x == 0) block_tok[m] = tok;
  const T *e = tok_emb + (size_t)tok * d;
  for (int i = threadIdx.x; i < d; i += 256) h[(size_t)m * d + i] = to_f32(e[i]);
}

void launch_embed(int dtype, const void *tok_emb, const int32_t *hist, const int32_t *drafts, int32_t *block_tok,
                  float *h, int d, int M, int C, int w, int hist_base, int from_hist, hipStream_t s) {
  if (dtype == 1)
    hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(M), dim3(256), 0, s, (const bf16_t *)tok_emb, hist, drafts, block_tok,
                       h, d, C, w, hist_base, from_hist);
  else
    hipLaunchKernelGGL(embed_kernel<float>, dim3(M), dim3(256), 0, s, (const float *)tok_emb, hist, drafts, block_tok, h,
                       d, C, w, hist_base, from_hist);
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: xn = h * rsqrt(mean(h^2) + eps) * gain, one workgroup per row.
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

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *h, const T *gain, T *xn, int d, float eps) {
  __shared__ float sh[4];
  const float *row = h + (size_t)blockIdx.x * d;
  float ss = 0.0f;
  for (int i = threadIdx.x; i < d; i += 256) { const float v = row[i]; ss += v * v; }
  ss = block_sum_256(ss, sh);
  const float sc = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) xn[(size_t)blockIdx.x * d + i] = from_f32<T>(row[i] * sc * to_f32(gain[i]));
}

void launch_rmsnorm(int dtype, const float *h, const void *gain, void *xn, int d, int M, float eps, hipStream_t s) {
  if (dtype == 1)
    hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(M), dim3(256), 0, s, h, (const bf16_t *)gain, (bf16_t *)xn, d, eps);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(M), dim3(256), 0, s, h, (const float *)gain, (float *)xn, d, eps);
}

// ---------------------------------------------------------------------------------------------
// Context N-gram matcher (Section 4.2), one workgroup of 1024 threads.
// For each query length q (q_max down to q_min): collect every window start i <= n-q-w whose
// first q tokens equal the last q context tokens; group equal w-token continuations; rank groups
// by (count desc, last start desc); append continuations not taken yet until k_ctx_max rows.
// Counts and last starts do not depend on the order in which matches were collected, so the
// result is deterministic although the lists are filled with atomics.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ bool same_cont(const int32_t *x, int a, int b, int w) {
  for (int t = 0; t < w; ++t)
    if (x[a + t] != x[b + t]) return false;
  return true;
}

__global__ __launch_bounds__(1024) void ctx_match_kernel(const DraftArgs a) {
  __shared__ int n_match, n_rep, n_taken;
  __shared__ int cand[64];          // start of the continuation ranked r among this q's groups
  const int tid = threadIdx.x;
  const int32_t *x = a.hist;
  const int n = a.n, w = a.w;
  const int kmax = min(a.k_ctx_max, a.k);
  if (tid == 0) n_taken = 0;
  __syncthreads();
  if (w >= 1 && kmax >= 1) {
    for (int q = a.q_max; q >= a.q_min; --q) {
      if (q < 1 || n < q + w) continue;                     // uniform
      if (tid == 0) { n_match = 0; n_rep = 0; }
      if (tid < 64) cand[tid] = -1;
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
      for (int t = tid; t < nm; t += 1024) {
        const int i = a.mlist[t];
        int cnt = 0, last = i;
        for (int u = 0; u < nm; ++u) {
          const int j = a.mlist[u];
          if (same_cont(x, i + q, j + q, w)) { ++cnt; last = max(last, j); }
        }
        if (last == i) {                                    // one representative per continuation
          const int slot = atomicAdd(&n_rep, 1);
          a.reps[2 * slot] = cnt;
          a.reps[2 * slot + 1] = i;
        }
      }
      __syncthreads();
      const int nr = n_rep;
      const int want = min(2 * kmax, 64);
      for (int t = tid; t < nr; t += 1024) {
        const int cnt = a.reps[2 * t], i = a.reps[2 * t + 1];
        int rank = 0;
        for (int u = 0; u < nr; ++u) {
          const int c2 = a.reps[2 * u], i2 = a.reps[2 * u + 1];
          rank += (c2 > cnt || (c2 == cnt && i2 > i)) ? 1 : 0;
        }
        if (rank < want) cand[rank] = i + q;
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
// Model bigram scores z[v] = <unemb[v], tok_emb[x_last]> (Section 4.1), one wave per row of the
// output embedding, rows streamed once with 16-byte loads per lane; fp32 accumulation.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bigram_gemv_kernel(const T *tok_emb, const T *unemb, const int32_t *hist, int n,
                                                          int d, int vocab, float *z) {
  extern __shared__ float e[];
  const int x = hist[n - 1];
  for (int i = threadIdx.x; i < d; i += 256) e[i] = to_f32(tok_emb[(size_t)x * d + i]);
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = gridDim.x * 4;
  for (int v = wave; v < vocab; v += n_waves) {
    const T *row = unemb + (size_t)v * d;
    float acc = 0.0f;
    for (int c = lane * 8; c < d; c += 512) {
      const Frag<T> f = load_frag(row + c);
#pragma unroll
      for (int t = 0; t < 8; ++t) acc += to_f32(f.v[t]) * e[c + t];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) z[v] = acc;
  }
}

// Top-(k - n_ctx) of z by (score desc, id asc), chained extension through next1, and assembly of
// the k x w draft batch (Section 4.3: context rows first, the extended bigram fills the rest).
__global__ __launch_bounds__(1024) void topk_assemble_kernel(const DraftArgs a) {
  __shared__ float wv[16];
  __shared__ int wi[16];
  __shared__ float sel_v;
  __shared__ int sel_i;
  __shared__ int top[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_ctx = *a.n_ctx;
  const int k_big = a.w >= 1 ? a.k - n_ctx : 0;
  // this thread's best remaining candidate
  float bv = kNegBig;
  int bi = 0x7fffffff;
  auto rescan = [&](float lim_v, int lim_i, bool limited) {
    bv = kNegBig; bi = 0x7fffffff;
    for (int v = tid; v < a.vocab; v += 1024) {
      const float zv = a.z[v];
      if (limited && !(zv < lim_v || (zv == lim_v && v > lim_i))) continue;   // already selected
      if (zv > bv || (zv == bv && v < bi)) { bv = zv; bi = v; }
    }
  };
  rescan(0.f, 0, false);
  for (int r = 0; r < k_big; ++r) {
    float cv = bv;
    int ci = bi;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(cv, off);
      const int oi = __shfl_xor(ci, off);
      if (ov > cv || (ov == cv && oi < ci)) { cv = ov; ci = oi; }
    }
    if (lane == 0) { wv[wave] = cv; wi[wave] = ci; }
    __syncthreads();
    if (tid == 0) {
      float fv = wv[0];
      int fi = wi[0];
      for (int t = 1; t < 16; ++t)
        if (wv[t] > fv || (wv[t] == fv && wi[t] < fi)) { fv = wv[t]; fi = wi[t]; }
      sel_v = fv; sel_i = fi; top[r] = fi;
    }
    __syncthreads();
    if (bi == sel_i) rescan(sel_v, sel_i, true);           // only the owner of the winner looks again
    __syncthreads();
  }
  __syncthreads();
  if (tid < a.k && a.w >= 1) {
    const int r = tid;
    if (r < n_ctx) {
      for (int t = 0; t < a.w; ++t) a.drafts[r * a.w + t] = a.ctx_rows[r * a.w + t];
      a.row_src[r] = 0;
    } else {
      int t0 = top[r - n_ctx];
      for (int t = 0; t < a.w; ++t) { a.drafts[r * a.w + t] = t0; t0 = a.next1[t0]; }
      a.row_src[r] = 1;
    }
  } else if (tid < a.k) {
    a.row_src[tid] = 1;
  }
}

void launch_build_drafts(int dtype, const DraftArgs &a, hipStream_t s) {
  hipLaunchKernelGGL(ctx_match_kernel, dim3(1), dim3(1024), 0, s, a);
  if (a.w >= 1) {
    const int blocks = 1024;
    const size_t lds = (size_t)a.d * sizeof(float);
    if (dtype == 1)
      hipLaunchKernelGGL(bigram_gemv_kernel<bf16_t>, dim3(blocks), dim3(256), lds, s, (const bf16_t *)a.tok_emb,
                         (const bf16_t *)a.unemb, a.hist, a.n, a.d, a.vocab, a.z);
    else
      hipLaunchKernelGGL(bigram_gemv_kernel<float>, dim3(blocks), dim3(256), lds, s, (const float *)a.tok_emb,
                         (const float *)a.unemb, a.hist, a.n, a.d, a.vocab, a.z);
  }
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

__global__ __launch_bounds__(256) void argmax_accept_kernel(const float *pmax_val, const int *pmax_idx, int tiles,
                                                            int Mcap, int M, int k, int C, const int32_t *drafts,
                                                            int32_t *res, int greedy_off) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int32_t *greedy = res + greedy_off;
  for (int m = wave; m < M; m += 4) {
    float bv = kNegBig;
    int bi = 0x7fffffff;
    for (int t = lane; t < tiles; t += 64) {
      const float v = pmax_val[(size_t)t * Mcap + m];
      const int i = pmax_idx[(size_t)t * Mcap + m];
      if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
    wave_argmax(bv, bi);
    if (lane == 0) greedy[m] = bi;
  }
  __syncthreads();
  if (k <= 0) return;                                        // prefill / table mode: argmax only
  const int w = C - 1;
  for (int r = tid; r < k; r += 256) {
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
  }
}

void launch_argmax_accept(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int M, int k, int C,
                          const int32_t *drafts, int32_t *res, int greedy_off, hipStream_t s) {
  hipLaunchKernelGGL(argmax_accept_kernel, dim3(1), dim3(256), 0, s, pmax_val, pmax_idx, tiles, Mcap, M, k, C, drafts,
                     res, greedy_off);
}

__global__ __launch_bounds__(256) void next1_finish_kernel(const float *pmax_val, const int *pmax_idx, int tiles,
                                                           int Mcap, int M, int32_t *out) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= M) return;
  float bv = kNegBig;
  int bi = 0x7fffffff;
  for (int t = lane; t < tiles; t += 64) {
    const float v = pmax_val[(size_t)t * Mcap + m];
    const int i = pmax_idx[(size_t)t * Mcap + m];
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
  }
  wave_argmax(bv, bi);
  if (lane == 0) out[m] = bi;
}

void launch_next1_finish(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int M, int32_t *next1_out,
                         hipStream_t s) {
  hipLaunchKernelGGL(next1_finish_kernel, dim3((M + 3) / 4), dim3(256), 0, s, pmax_val, pmax_idx, tiles, Mcap, M,
                     next1_out);
}

// ---------------------------------------------------------------------------------------------
// Commit (Appendix D): the winner row's keys/values for block columns 0 .. n_new-1 become cache
// positions P .. P+n_new-1; the new tokens are appended to the history at P+1 ...
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void commit_kernel(T *kcache, T *vcache, const T *kscr, const T *vscr, int Hkv, int hd,
                                                     int Spad, int Mcap, int C, int P, const int32_t *res, int fixed_row,
                                                     int fixed_n, int max_new, int32_t *hist) {
  const int layer = blockIdx.y, hkv = blockIdx.x;
  int row = fixed_row, n_new = fixed_n;
  if (res) { row = res[RES_WINNER]; n_new = min(res[RES_NNEW], max_new); }
  const size_t lh = (size_t)layer * Hkv + hkv;
  const T *ks = kscr + lh * Mcap * hd;
  const T *vs = vscr + lh * hd * Mcap;
  T *kc = kcache + lh * Spad * hd;
  T *vc = vcache + lh * hd * Spad;
  for (int i = threadIdx.x; i < n_new * hd; i += 256) {
    const int j = i / hd, dd = i - j * hd;
    kc[(size_t)(P + j) * hd + dd] = ks[(size_t)(row * C + j) * hd + dd];
    vc[(size_t)dd * Spad + P + j] = vs[(size_t)dd * Mcap + row * C + j];
  }
  if (res && layer == 0 && hkv == 0)
    for (int i = threadIdx.x; i < n_new; i += 256) hist[P + 1 + i] = res[RES_NEWTOK + i];
}

void launch_commit(int dtype, void *kcache, void *vcache, const void *kscr, const void *vscr, int L, int Hkv, int hd,
                   int Spad, int Mcap, int C, int P, const int32_t *res, int fixed_row, int fixed_n, int max_new,
                   int32_t *hist, hipStream_t s) {
  if (dtype == 1)
    hipLaunchKernelGGL(commit_kernel<bf16_t>, dim3(Hkv, L), dim3(256), 0, s, (bf16_t *)kcache, (bf16_t *)vcache,
                       (const bf16_t *)kscr, (const bf16_t *)vscr, Hkv, hd, Spad, Mcap, C, P, res, fixed_row, fixed_n,
                       max_new, hist);
  else
    hipLaunchKernelGGL(commit_kernel<float>, dim3(Hkv, L), dim3(256), 0, s, (float *)kcache, (float *)vcache,
                       (const float *)kscr, (const float *)vscr, Hkv, hd, Spad, Mcap, C, P, res, fixed_row, fixed_n,
                       max_new, hist);
}

}  // namespace ngg
