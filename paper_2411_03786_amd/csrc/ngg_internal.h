// Internal declarations shared by the HIP translation units of libngg.
// Device code targets gfx950 (CDNA4) only: 64-wide wavefronts, MFMA 16x16 tiles.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ngg {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;   // "minus infinity" that stays finite under subtraction

// ---------------------------------------------------------------------------------------------
// MFMA operand fragments.  A fragment is the 8 consecutive contraction-index elements one lane
// feeds into a 16x16 matrix op: lane l supplies row/column (l % 16) and elements 8*(l/16) .. +8 of
// a 32-element slice of the contraction index.  bf16 uses one v_mfma_f32_16x16x32_bf16; fp32
// issues eight v_mfma_f32_16x16x4_f32 (element e of every lane goes into the e-th op, so both
// operands see the same permutation of the 32-element slice).  The 16x16 fp32 result holds, in
// lane l, column (l % 16) and rows 4*(l/16) .. +4.
// ---------------------------------------------------------------------------------------------
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { bf16x8 v; };
template <> struct Frag<float> { float v[8]; };

__device__ __forceinline__ Frag<bf16_t> load_frag(const bf16_t *p) {
  Frag<bf16_t> f;
  f.v = *reinterpret_cast<const bf16x8 *>(p);
  return f;
}
__device__ __forceinline__ Frag<float> load_frag(const float *p) {
  Frag<float> f;
  const float4 a = *reinterpret_cast<const float4 *>(p);
  const float4 b = *reinterpret_cast<const float4 *>(p + 4);
  f.v[0] = a.x; f.v[1] = a.y; f.v[2] = a.z; f.v[3] = a.w;
  f.v[4] = b.x; f.v[5] = b.y; f.v[6] = b.z; f.v[7] = b.w;
  return f;
}
template <typename T> __device__ __forceinline__ Frag<T> zero_frag();
template <> __device__ __forceinline__ Frag<bf16_t> zero_frag<bf16_t>() {
  Frag<bf16_t> f;
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = (bf16_t)0.0f;
  return f;
}
template <> __device__ __forceinline__ Frag<float> zero_frag<float>() {
  Frag<float> f;
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = 0.0f;
  return f;
}
__device__ __forceinline__ void pack_frag(Frag<bf16_t> &f, const float *p) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = (bf16_t)p[e];     // round to nearest even
}
__device__ __forceinline__ void pack_frag(Frag<float> &f, const float *p) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = p[e];
}

// acc[i][j] += sum_k a[i][k] * b[k][j]: a's lane index is the result row, b's the result column.
__device__ __forceinline__ void mma(f32x4 &acc, const Frag<bf16_t> &a, const Frag<bf16_t> &b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma(f32x4 &acc, const Frag<float> &a, const Frag<float> &b) {
#pragma unroll
  for (int e = 0; e < 8; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[e], b.v[e], acc, 0, 0, 0);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

template <typename T> __device__ __forceinline__ float fast_exp(float x);
template <> __device__ __forceinline__ float fast_exp<float>(float x) { return expf(x); }
template <> __device__ __forceinline__ float fast_exp<bf16_t>(float x) { return __expf(x); }

// ---------------------------------------------------------------------------------------------
// Launch descriptions (plain structs passed by value to the kernels).
// ---------------------------------------------------------------------------------------------
enum GemmEpilogue { EPI_QKV = 0, EPI_RESIDUAL = 1, EPI_GATEUP = 2, EPI_UNEMBED = 3 };

struct GemmArgs {
  const void *X;          // [M][ldx] activations, element type T
  int ldx;
  const void *W0, *W1, *W2;   // weight blocks, row-major [rows][K]
  int M, N, K;            // N = total logical output rows
  // EPI_RESIDUAL
  float *h;               // [M][N] fp32, updated in place
  // EPI_GATEUP
  void *act;              // [M][N] T  (N = d_ffn)
  // EPI_QKV
  void *q;                // [H][Mcap][hd] T
  void *kscr;             // this layer's [Hkv][Mcap][hd] T
  void *vscr;             // this layer's [Hkv][hd][Mcap] T (transposed)
  int H, Hkv, hd, Mcap, C, P;   // m = row*C + col sits at position P + col
  const float *rope_cos, *rope_sin;   // [Spad][hd/2]
  // EPI_UNEMBED
  float *logits;          // [M][N] fp32 or null
  float *pmax_val;        // [tiles][Mcap]
  int *pmax_idx;          // [tiles][Mcap]
};

struct AttnArgs {
  const void *q;          // [H][Mcap][hd]
  const void *kcache;     // this layer's [Hkv][Spad][hd]
  const void *vcache;     // this layer's [Hkv][hd][Spad]
  const void *kscr;       // this layer's [Hkv][Mcap][hd]
  const void *vscr;       // this layer's [Hkv][hd][Mcap]
  float *part_o;          // [H][n_splits+1][Mcap][hd]
  float *part_ml;         // [H][n_splits+1][Mcap][2]
  void *out;              // [M][H*hd] T
  int H, Hkv, Mcap, Spad, M, C, P, n_splits, span;
  float scale;
};

// launchers (host).  dtype: 0 = fp32, 1 = bf16.  Every launcher validates nothing: the API layer
// checks shapes before calling.
void launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t s);
int gemm_unembed_tiles(int N);
void launch_attention(int dtype, int hd, const AttnArgs &a, hipStream_t s);

void launch_embed(int dtype, const void *tok_emb, const int32_t *hist, const int32_t *drafts, int32_t *block_tok,
                  float *h, int d, int M, int C, int w, int hist_base, int from_hist, hipStream_t s);
void launch_rmsnorm(int dtype, const float *h, const void *gain, void *xn, int d, int M, float eps, hipStream_t s);

struct DraftArgs {
  const int32_t *hist; int n;
  int k, w, k_ctx_max, q_min, q_max;
  int32_t *mlist;         // [max_seq] scratch: matching window starts
  int32_t *reps;          // [2*max_seq] scratch: (count, last_start) of each distinct continuation
  int32_t *ctx_rows;      // [max_k][max_w]
  int32_t *n_ctx;         // [1]
  const void *tok_emb, *unemb; int d, vocab;
  float *z;               // [vocab]
  const int32_t *next1;   // [vocab]
  int32_t *drafts;        // [k][w]
  int8_t *row_src;        // [k]
};
void launch_build_drafts(int dtype, const DraftArgs &a, hipStream_t s);

// result block layout (int32 words)
enum { RES_WINNER = 0, RES_NACCEPT = 1, RES_NNEW = 2, RES_NCTX = 3, RES_NEWTOK = 8, RES_ACCEPT = 48 };
inline int res_greedy_off(int max_k) { return RES_ACCEPT + ((max_k + 7) / 8) * 8; }

void launch_argmax_accept(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int M, int k, int C,
                          const int32_t *drafts, int32_t *res, int greedy_off, hipStream_t s);
void launch_commit(int dtype, void *kcache, void *vcache, const void *kscr, const void *vscr, int L, int Hkv, int hd,
                   int Spad, int Mcap, int C, int P, const int32_t *res, int fixed_row, int fixed_n, int max_new,
                   int32_t *hist, hipStream_t s);
void launch_next1_finish(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int M, int32_t *next1_out,
                         hipStream_t s);

}  // namespace ngg
