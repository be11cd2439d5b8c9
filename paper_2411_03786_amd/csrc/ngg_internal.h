// Internal declarations shared by the HIP translation units of libngg.
// Device code targets gfx950 (CDNA4) only: 64-wide wavefronts, MFMA 16x16 tiles.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ngg {

// Element types.  A model stored in bf16 (ngg_dtype NGG_BF16) is computed with fp16 matrix operands: the
// library's operand-order copies of the weights are the stored bf16 values times a power of two chosen
// per matrix so that they are exact in fp16 (8 mantissa bits fit in 11; the scale brings the largest
// magnitude to [2^13, 2^14), so everything down to 2^-31 of it keeps all its bits), and activations,
// keys, values and probabilities are rounded to fp16 (11 mantissa bits) instead of bf16 (8).  The MFMA
// rate is the same, HBM bytes are the same, and the rounding noise per operand is 8 times smaller:
// with bf16 operands the logits of the 7B-width model drift past the 2e-2 logit tolerance between 8 and
// 16 layers.  bf16_t below is only the type user weights are READ in; half_t is the internal type.
typedef __bf16 bf16_t;
typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
template <typename U> struct Internal;                       // storage type of the user's weights -> internal element type
template <> struct Internal<float> { typedef float type; };
template <> struct Internal<bf16_t> { typedef half_t type; };
constexpr float kHalfMax = 65504.0f;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;   // "minus infinity" that stays finite under subtraction

// ---------------------------------------------------------------------------------------------
// MFMA operand fragments.  A fragment is the 8 consecutive contraction-index elements one lane
// feeds into a 16x16 matrix op: lane l supplies row/column (l % 16) and elements 8*(l/16) .. +8 of
// a 32-element slice of the contraction index.  fp16 uses one v_mfma_f32_16x16x32_f16; fp32
// issues eight v_mfma_f32_16x16x4_f32 (element e of every lane goes into the e-th op, so both
// operands see the same permutation of the 32-element slice).  The 16x16 fp32 result holds, in
// lane l, column (l % 16) and rows 4*(l/16) .. +4.
// ---------------------------------------------------------------------------------------------
template <typename T> struct Frag;
template <> struct Frag<half_t> { half8 v; };
template <> struct Frag<float> { float v[8]; };

__device__ __forceinline__ Frag<half_t> load_frag(const half_t *p) {
  Frag<half_t> f;
  f.v = *reinterpret_cast<const half8 *>(p);
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
// Operand-order ("tiled") weight storage.  A matrix [N][K] is cut into blocks of 16 rows x 32
// contraction elements, stored group-major: block (n/16, k/32) starts at element
// ((n/16) * (K/32) + k/32) * 512.  Inside a bf16 block lane l = ((k%32)/8)*16 + n%16 owns elements
// l*8 .. l*8+8 (its fragment; "bf16" = 2-byte elements, fp16 inside the library); an fp32 block is two 1 KB halves, half h holding elements 4h .. 4h+4
// of every lane's fragment at l*4.  A wave's load instruction therefore reads 1 KB contiguously.
__host__ __device__ __forceinline__ size_t tiled_offset(int n, int k, int K, int elem_size) {
  const size_t block = ((size_t)(n / 16) * (K / 32) + k / 32) * 512;
  const int l = ((k % 32) / 8) * 16 + n % 16, e = k % 8;
  return block + (elem_size == 2 ? l * 8 + e : (e / 4) * 256 + l * 4 + e % 4);
}
template <typename T>
__device__ __forceinline__ const T *tiled_block(const T *w, int group16, int n_steps, int lane) {
  return w + (size_t)group16 * n_steps * 512 + lane * (sizeof(T) == 2 ? 8 : 4);
}
__device__ __forceinline__ Frag<half_t> load_frag_tiled(const half_t *p) { return load_frag(p); }
__device__ __forceinline__ Frag<float> load_frag_tiled(const float *p) {
  Frag<float> f;
  const float4 a = *reinterpret_cast<const float4 *>(p);
  const float4 b = *reinterpret_cast<const float4 *>(p + 256);
  f.v[0] = a.x; f.v[1] = a.y; f.v[2] = a.z; f.v[3] = a.w;
  f.v[4] = b.x; f.v[5] = b.y; f.v[6] = b.z; f.v[7] = b.w;
  return f;
}
// The same fragment from global memory that is read once per launch (weights, cached keys and values):
// a non-temporal load, so the stream does not push the activations, which every workgroup re-reads,
// out of the L2 (measured on MI355X at the 7B shapes: gate/up 45.0 -> 42.2 us, q/k/v 24.2 -> 22.8,
// down 25.3 -> 23.4, unembedding 53 -> 49 at 60 block rows, and the same 2-3 us with one row).
__device__ __forceinline__ Frag<half_t> load_frag_stream(const half_t *p) {
  Frag<half_t> f;
  f.v = __builtin_nontemporal_load(reinterpret_cast<const half8 *>(p));
  return f;
}
__device__ __forceinline__ Frag<float> load_frag_stream(const float *p) {
  Frag<float> f;
  const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
  const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + 256));
  f.v[0] = a[0]; f.v[1] = a[1]; f.v[2] = a[2]; f.v[3] = a[3];
  f.v[4] = b[0]; f.v[5] = b[1]; f.v[6] = b[2]; f.v[7] = b[3];
  return f;
}

// Keys and values of one (layer, kv head) live in tiles of 32 positions, 32*hd elements each, both in
// operand order.  A key tile is the [32 keys][hd] matrix with its rows permuted (key 8a + 4f + b of
// the tile is row 16f + 4a + b: with that order the lane that holds a score fragment's column owns 8
// consecutive keys, which is what the probabilities' operand layout needs); a value tile is the
// transposed [hd][32 keys] matrix.
__host__ __device__ __forceinline__ int kv_key_row(int kk) { return ((kk >> 2) & 1) * 16 + (kk >> 3) * 4 + (kk & 3); }
__host__ __device__ __forceinline__ size_t k_offset(int pos, int dim, int hd, int elem_size) {
  return (size_t)(pos / 32) * 32 * hd + tiled_offset(kv_key_row(pos % 32), dim, hd, elem_size);
}
__host__ __device__ __forceinline__ size_t v_offset(int pos, int dim, int hd, int elem_size) {
  return (size_t)(pos / 32) * 32 * hd + tiled_offset(dim, pos % 32, 32, elem_size);
}

// Activation matrices that feed a GEMM (normalised hidden state, attention output, SwiGLU output)
// are stored chunk-major: [K / KC][Mcap][KC] with KC = 256 (bf16) or 128 (fp32) contraction
// elements, so that the slice of all block rows a workgroup stages per step of the GEMM is one
// contiguous region spread over every L2 channel (row-major rows lie a multiple of the channel
// interleave apart, which made all workgroups of a die hit the same few channels at once).
template <typename T> struct KChunk;
template <> struct KChunk<half_t> { static constexpr int value = 256; };
template <> struct KChunk<float> { static constexpr int value = 128; };
template <typename T>
__host__ __device__ __forceinline__ size_t act_offset(int m, int k, int Mcap) {
  constexpr int KC = KChunk<T>::value;
  return ((size_t)(k / KC) * Mcap + m) * KC + k % KC;
}
inline size_t act_elems(int dtype, int Mcap, int K) {
  const int kc = dtype == 1 ? KChunk<half_t>::value : KChunk<float>::value;
  return (size_t)((K + kc - 1) / kc) * Mcap * kc;
}

template <typename T> __device__ __forceinline__ Frag<T> zero_frag();
template <> __device__ __forceinline__ Frag<half_t> zero_frag<half_t>() {
  Frag<half_t> f;
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = (half_t)0.0f;
  return f;
}
template <> __device__ __forceinline__ Frag<float> zero_frag<float>() {
  Frag<float> f;
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = 0.0f;
  return f;
}
// fp32 -> fp16, round to nearest even; magnitudes beyond the fp16 range saturate instead of becoming infinite
__device__ __forceinline__ half_t to_half(float x) { return (half_t)fminf(fmaxf(x, -kHalfMax), kHalfMax); }
__device__ __forceinline__ void pack_frag(Frag<half_t> &f, const float *p) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = to_half(p[e]);
}
__device__ __forceinline__ void pack_frag(Frag<float> &f, const float *p) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = p[e];
}

// acc[i][j] += sum_k a[i][k] * b[k][j]: a's lane index is the result row, b's the result column.
__device__ __forceinline__ void mma(f32x4 &acc, const Frag<half_t> &a, const Frag<half_t> &b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.v, b.v, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma(f32x4 &acc, const Frag<float> &a, const Frag<float> &b) {
#pragma unroll
  for (int e = 0; e < 8; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[e], b.v[e], acc, 0, 0, 0);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
__device__ __forceinline__ float to_f32(half_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ half_t from_f32<half_t>(float x) { return to_half(x); }

// four consecutive elements in one store (8 bytes of fp16 or 16 bytes of fp32); dst is so aligned
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store4(half_t *dst, float a, float b, float c, float d) {
  half4 v;
  v[0] = to_half(a); v[1] = to_half(b); v[2] = to_half(c); v[3] = to_half(d);
  *reinterpret_cast<half4 *>(dst) = v;
}
__device__ __forceinline__ void store4(float *dst, float a, float b, float c, float d) {
  *reinterpret_cast<float4 *>(dst) = float4{a, b, c, d};
}

// Maximum / sum over the four lanes l, l^16, l^32, l^48 (one lane per 16-lane row of the wave); every
// lane gets the result.  The gfx950 row-swap instructions do this in the vector ALU (checked on the
// device: permlane16_swap(x, x) yields rows [x0 x0 x2 x2] and [x1 x1 x3 x3], permlane32_swap(x, x) the
// two halves [lo lo] and [hi hi]); a shuffle would go through the LDS pipeline and its latency.
__device__ __forceinline__ float rows_max(float x) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const unsigned v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// The value that the lane 32 lanes away holds.  In a 16x16 accumulator fragment lane (column, g) has
// rows 4g .. 4g+3, so rows 0..7 (g < 2) meet rows 8..15 of the same column this way.
__device__ __forceinline__ float other_half(float x) {
  const unsigned u = __float_as_uint(x);
  const auto b = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // b[0] = [lo lo], b[1] = [hi hi]
  return __uint_as_float((threadIdx.x & 32) ? b[0] : b[1]);
}

// x * sigmoid(x).  The 16-bit configuration rounds the product to 11 mantissa bits anyway, so it takes
// the hardware's base-2 exponential and reciprocal (about 1 ulp of fp32 each) in place of expf and
// an IEEE division, which cost ten times the instructions; overflow of the exponential gives x * 0.
template <typename T> __device__ __forceinline__ float silu(float x);
template <> __device__ __forceinline__ float silu<float>(float x) { return x / (1.0f + expf(-x)); }
template <> __device__ __forceinline__ float silu<half_t>(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// ---------------------------------------------------------------------------------------------
// Block token index.  The model call of Section 3 takes a block of R rows x C columns.  Plain layout
// (pieces of a prompt, table builds): m = r*C + j.  Shared-first-column layout (a verify block,
// C = w + 1 >= 2): column 0 of every row is the same token (the uncached last context token) at the same
// position and sees the same keys, so its activations, keys/values and logits are identical in every
// row and are computed once: m = 0 for column 0 and m = r*(C-1) + j for columns j >= 1, 1 + R*w distinct
// block tokens in all.  Token m sees the cached context, and of the block: itself, the earlier drafted
// tokens of its own row (indices block_row_start(m) .. m) and, in the shared layout, token 0.
// ---------------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ int block_index(int r, int j, int C, int shared0) {
  return shared0 ? (j == 0 ? 0 : r * (C - 1) + j) : r * C + j;
}
__host__ __device__ __forceinline__ int block_col(int m, int C, int shared0) {
  return shared0 ? (m == 0 ? 0 : (m - 1) % (C - 1) + 1) : m % C;
}
__host__ __device__ __forceinline__ int block_row_start(int m, int C, int shared0) {
  return shared0 ? (m == 0 ? 0 : m - (m - 1) % (C - 1)) : m - m % C;
}
__host__ __device__ __forceinline__ int block_tokens(int R, int C, int shared0) { return shared0 ? 1 + R * (C - 1) : R * C; }

// ---------------------------------------------------------------------------------------------
// Launch descriptions (plain structs passed by value to the kernels).
// ---------------------------------------------------------------------------------------------
enum GemmEpilogue { EPI_QKV = 0, EPI_RESIDUAL = 1, EPI_GATEUP = 2, EPI_UNEMBED = 3 };

struct GemmArgs {
  const void *X;          // activations, chunk-major [K/KC][Mcap][KC], element type T
  const void *W0;         // weight matrix in operand order (QKV: rows [q | k | v]; gate/up: rows [gate | up])
  int M, N, K;            // N = total logical output rows
  // q/k/v, gate/up, unembedding: X is h * gain; the epilogue multiplies row m by
  // 1 / sqrt((row_ss[m][0] + .. + row_ss[m][ss_segs-1]) / K + ss_eps).  Null: X is used as it is.
  const float *row_ss;
  int ss_segs;
  float ss_eps;
  float out_scale;        // every result is multiplied by this: 1 / (scale of the stored weights * scale of X); 1 for fp32 models
  int n_groups;           // residual, unembedding: pairs of 16-row fragments; q/k/v, gate/up: fragments (filled by the launcher)
  // EPI_RESIDUAL: split ks of KS stores its fp32 partial at hpart[ks][m][n]; the next RMSNorm adds them
  float *hpart;           // [KS][Mcap][N]
  int KS;
  // EPI_GATEUP
  void *act;              // chunk-major [N/KC][Mcap][KC] T  (N = d_ffn)
  // EPI_QKV
  void *q;                // [H][Mcap][hd] T
  void *kscr;             // this layer's block keys, [Hkv][kv_rows/32] tiles (k_offset)
  void *vscr;             // this layer's block values, [Hkv][kv_rows/32] tiles (v_offset)
  int kv_rows;            // positions per kv head of kscr/vscr: Mcap for the scratch; the cache's padded length when a
                          // prefill piece writes its keys and values straight to their cache tiles
  int H, Hkv, hd, Mcap, C, P;   // block token m sits at position P + block_col(m, C, shared0)
  const int32_t *n_dev;   // when set, P = *n_dev - 1 (see DraftArgs)
  int shared0;
  const float *rope_cos, *rope_sin;   // [Spad][hd/2]
  // EPI_UNEMBED
  float *logits;          // [M][N] fp32 or null
  float *pmax_val;        // [N/32][Mcap]
  int *pmax_idx;          // [N/32][Mcap]
};

constexpr int kMaxResidualSplits = 8;
constexpr int kNormSegs = 4;   // workgroups that may share a row of the RMSNorm; row_ss is [Mcap][kNormSegs]

struct AttnArgs {
  const void *q;          // [H][Mcap][hd]
  const void *kcache;     // this layer's cached keys, [Hkv][Spad/32] tiles of 32 positions (k_offset)
  const void *vcache;     // this layer's cached values, same tiling (v_offset)
  const void *kscr;       // this layer's block keys, [Hkv][kv_rows/32] tiles
  const void *vscr;       // this layer's block values, [Hkv][kv_rows/32] tiles
  int kv_rows;            // positions per kv head of kscr/vscr (Mcap, or the cache's padded length: see GemmArgs)
  float *part_o;          // [H][n_splits][Mpart/16][hd/16][64 lanes][4]: output fragments as the registers hold them
  float *part_ml;         // [H][n_splits][Mpart][2]
  int Mpart;              // rows per (head, slice) of the two partial buffers: M rounded up to 128
  void *out;              // chunk-major [H*hd/KC][Mcap][KC] T
  int H, Hkv, Mcap, Spad, M, C, P, n_splits;   // n_splits: workgroups that share a head's list of key tiles
  const int32_t *n_dev;   // when set, P = *n_dev - 1 (see DraftArgs)
  int shared0;            // block layout (block_index)
  float scale;
};

// launchers (host).  dtype: 0 = fp32, 1 = bf16.  Every launcher validates nothing: the API layer
// checks shapes before calling.
void launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t s);
int gemm_residual_splits(int dtype, int M, int N, int K);
void launch_attention(int dtype, int hd, const AttnArgs &a, hipStream_t s);
int attention_splits(int dtype, int hd, int H, int M, int P, int max_splits);
int attention_workgroups(int dtype, int hd, int H, int M, int n_splits);   // workgroups the main attention kernel is launched with

// mode 1: block token m is history token hist_base + m; mode 0: the verify block in the shared-first-column
// layout (token 0 is hist[hist_base], token m >= 1 is drafts[m - 1]); mode 2: a block of single-column rows (w = 0),
// every token hist[hist_base]
void launch_embed(int dtype, const void *tok_emb, const int32_t *hist, const int32_t *drafts, int32_t *block_tok,
                  float *h, int d, int M, int hist_base, int mode, hipStream_t s, const int32_t *n_dev = nullptr);   // n_dev: hist_base = *n_dev - 1
// h[m] += sum of n_part partials (hpart[s][m], stride part_stride floats between splits), then
// xn[m] = rmsnorm(h[m]) * gain, written chunk-major
// dst = (src - centre) * scale in the internal element type (src: the user's storage type)
void launch_pack_rows(int dtype, const void *src, void *dst, int d, int M, int Mcap, hipStream_t s, float scale,
                      const float *centre = nullptr);
// *out_bits = max(*out_bits, bit pattern of max |src[i]|) (fp32 bits; non-negative floats order like unsigned integers)
void launch_absmax(int dtype, const void *src, size_t n, unsigned *out_bits, hipStream_t s);
void launch_column_mean(int dtype, const void *src, int N, int d, float *mean, hipStream_t s);
void launch_neg_row_sumsq(const float *rows, int M, int V, float *out, hipStream_t s);
void launch_rmsnorm(int dtype, float *h, const float *hpart, int n_part, size_t part_stride, const void *gain, void *xn,
                    int d, int M, int Mcap, float *row_ss, hipStream_t s);
int rmsnorm_segments(int d);

struct DraftArgs {
  const int32_t *hist; int n;
  const int32_t *n_dev;   // when set, the kernels take n from here instead (a captured step replays with the same arguments)
  int k, w, k_ctx_max, q_min, q_max;
  int32_t *mlist;         // [max_seq] scratch: matching window starts
  int32_t *reps;          // [2*max_seq] scratch: (count, last_start) of each distinct continuation
  int32_t *gtab;          // [3][gtab_slots] scratch: grouping table (representative start | count | last start)
  int gtab_slots;         // a power of two >= 2 * max_seq
  int32_t *ctx_rows;      // [max_k][max_w]
  int32_t *n_ctx;         // [1]
  const void *tok_emb;    // row-major [vocab][d], the user's storage type
  float emb_scale;        // the embedding row is multiplied by this before it is rounded to the internal type
  const void *unemb_t;    // operand order, internal type, stored values times unemb_scale
  float unemb_scale;
  int d, vocab;
  float *z;               // [vocab]
  float *cand_val;        // [256][32] per-workgroup top-k candidates of the bigram sweep
  int *cand_idx;
  const int32_t *next1;   // [vocab]
  const int32_t *bg_table; // [vocab][bg_K] full-model bigram table, or null: bigram rows come from the sweep
  int bg_K;
  const int32_t *uni_top; // [>= k] tokens by ascending unigram distance, or null: first tokens come from the bigram
  int32_t *drafts;        // [k][w]
  int8_t *row_src;        // [k]
};
void launch_build_drafts(int dtype, const DraftArgs &a, hipStream_t s);
// the context matcher alone: reads hist, n, k, w, k_ctx_max, q_min, q_max and the three scratch arrays, writes ctx_rows, n_ctx
void launch_ctx_match(const DraftArgs &a, hipStream_t s);
// out[m][0..K) = ids of the K largest logits of row m by (value desc, id asc); logits [M][V] fp32
void launch_row_topk(const float *logits, int M, int V, int K, int32_t *out, hipStream_t s);
void launch_iota(int32_t *dst, int first, int n, hipStream_t s);
void launch_noop(hipStream_t s);
void launch_read_probe(const void *src, size_t bytes, unsigned *sink, int blocks, hipStream_t s);   // sink: >= blocks words
// copies src [N][K] (row-major) into rows row0 .. row0+N of the operand-order matrix dst
// row_map: 0 = row n goes to row0 + n; 1 = rotary pairing inside blocks of 2*half rows (row i < half of a block goes
// to 16*(i/8) + i%8, row half + i to 16*(i/8) + 8 + i%8); 2 / 3 = first / second member of interleaved 8-row halves
// (row n goes to 16*(n/8) + n%8, plus 8 for the second member)
// values are multiplied by `scale` (a power of two) on the way
void launch_tile_weights(int dtype, const void *src, void *dst, int N, int K, int row0, hipStream_t s, float scale,
                         int row_map = 0, int half = 0);

// result block layout (int32 words)
enum { RES_WINNER = 0, RES_NACCEPT = 1, RES_NNEW = 2, RES_NCTX = 3, RES_WINSRC = 4, RES_NEWTOK = 8, RES_ACCEPT = 48 };
inline int res_greedy_off(int max_k) { return RES_ACCEPT + ((max_k + 7) / 8) * 8; }

// greedy grid [rows][C] from the per-token partial maxima (token block_index(r, j, C, shared0)); k > 0: then the
// accepted lengths and the winner of the k x (C-1) drafts
void launch_argmax_accept(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int rows, int k, int C, int shared0,
                          const int32_t *drafts, const int8_t *row_src, const int32_t *n_ctx, int32_t *res, int greedy_off,
                          hipStream_t s);
// n_dev: P = *n_dev - 1 instead of the argument
void launch_commit(int dtype, void *kcache, void *vcache, const void *kscr, const void *vscr, int L, int Hkv, int hd,
                   int Spad, int Mcap, int C, int shared0, int P, const int32_t *res, int fixed_row, int fixed_n, int max_new,
                   int32_t *hist, hipStream_t s, const int32_t *n_dev = nullptr);
// *n_dev += min(res[RES_NNEW], max_new): the commit's bookkeeping on the device, after the commit kernel has read *n_dev
void launch_advance(int32_t *n_dev, const int32_t *res, int max_new, hipStream_t s);
void launch_next1_finish(const float *pmax_val, const int *pmax_idx, int tiles, int Mcap, int M, int32_t *next1_out,
                         hipStream_t s);

}  // namespace ngg
