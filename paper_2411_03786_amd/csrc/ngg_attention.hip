// Shared-prefix attention for the verify block.  Section 4.1 batches the k drafts by repeating
// the context into k identical rows, and the "Limitations" paragraph names the redundant prefix
// work as the method's cost; here the cached context is read ONCE for all k rows: every block token
// (row r, column j) is a query against the same cached keys, followed by the block's own keys (row
// r, columns <= j: a per-row causal mask).  Per head, the cached tiles and the block's tiles form
// one list that S workgroups split evenly; their partial (max, sum, output) triples are merged by a
// second kernel in list order (deterministic).
//
// Keys and values are kept in MFMA operand order (k_offset / v_offset in ngg_internal.h): a tile of
// 32 positions is 32*hd contiguous elements, cut into 1 KB blocks that are each exactly one
// wave-wide fragment load.  Two kernels use them:
//  * attn_shared_kernel (more than 16 block tokens): the four waves of a workgroup own different
//    groups of 16*QF queries and all need every tile, so the workgroup copies each tile into LDS once
//    (a linear copy: the tile already is in fragment order, so every fragment read is conflict-free)
//    and the waves read their MFMA operands from there.  No merge between waves.
//  * attn_stream_kernel (up to 16 block tokens, the single-token decode step): one group of queries,
//    so the four waves split the tiles instead and each tile goes from global memory straight into
//    the registers of the one wave that needs it; LDS only carries the final merge of the four waves.
#include "ngg_internal.h"

namespace ngg {

// Softmax arithmetic: the fp32 configuration uses expf on scores scaled by 1/sqrt(hd); the 16-bit
// configuration keeps scores, reference maxima and the stored partial maxima in the base-2 domain
// (scores times log2(e)/sqrt(hd)) so that each probability is one fused multiply-add and one v_exp_f32.
// There the probabilities are computed as 2^(s - ref + 10): the factor 2^10 is carried by the running
// sums and by the output alike and cancels in their quotient; it keeps probabilities down to 2^-24 of
// the reference in fp16's normal range (an fp16 matrix operand below 2^-14 may be flushed to zero,
// and thousands of such keys can add up to a visible share of a long context's softmax).
//
// The reference of a query is a maximum of its scores so far, brought up to date only when a tile holds a
// score more than `lazy` above it: softmax is invariant under the choice of reference as long as sums and
// output use the same one, so most tiles skip the cross-lane maximum, the rescaling factor and the rescaling
// of the output (16-bit: probabilities stay below 2^15; fp32: lazy = 0, the reference is the running maximum).
template <typename T> struct Softmax;
template <> struct Softmax<float> {
  static constexpr float lazy = 0.0f;
  static __device__ __forceinline__ float factor(float scale) { return scale; }
  static __device__ __forceinline__ float ex(float x) { return expf(x); }
  static __device__ __forceinline__ float bias(float ref) { return -ref; }
  static __device__ __forceinline__ float prob(float raw, float sfac, float bias) { return expf(fmaf(raw, sfac, bias)); }
};
template <> struct Softmax<half_t> {
  static constexpr float lazy = 5.0f;
  static __device__ __forceinline__ float factor(float scale) { return scale * 1.44269504088896f; }
  static __device__ __forceinline__ float ex(float x) { return __builtin_amdgcn_exp2f(x); }
  static __device__ __forceinline__ float bias(float ref) { return 10.0f - ref; }
  static __device__ __forceinline__ float prob(float raw, float sfac, float bias) { return __builtin_amdgcn_exp2f(fmaf(raw, sfac, bias)); }
};

// Probabilities are at most 2^15: no saturation needed on the way to fp16
__device__ __forceinline__ void pack_probs(Frag<half_t> &f, const float *p) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = (half_t)p[e];
}
__device__ __forceinline__ void pack_probs(Frag<float> &f, const float *p) { pack_frag(f, p); }

// One 16-query fragment against one 32-key tile, after the scores: the softmax part.  Returns the
// probabilities as the P operand of P.V, updates the query's reference maximum mref (the same in the four
// lanes of a query), this lane's share lsum of the running sum (the four lanes are added up once, at the end)
// and, when the reference moves, rescales the output so far.
// Sc: transposed raw scores (fragment f's row i is key 8*(i/4) + 4f + (i%4) of the tile, so this lane
// holds the 8 consecutive keys k0 .. k0+7 of its query); keys outside [lo, hi] are masked (except key 0
// when key0 is set: the block token every row shares) unless the whole tile is visible to every query (full).
template <typename T, int DF>
__device__ __forceinline__ Frag<T> softmax_tile(const f32x4 (&Sc)[2], float sfac, bool full, int k0, int lo, int hi, bool key0,
                                                float &mref, float &lsum, f32x4 (&O)[DF]) {
  float raw[8], p[8];
  unsigned vis = 0xffu;                                     // bit e: key k0 + e is visible to this lane's query
  float mx = kNegBig;
#pragma unroll
  for (int e = 0; e < 8; ++e) raw[e] = Sc[e >> 2][e & 3];
  if (full) {
#pragma unroll
    for (int e = 0; e < 8; ++e) mx = fmaxf(mx, raw[e]);
  } else {
    vis = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const bool v = (k0 + e >= lo && k0 + e <= hi) || (key0 && k0 + e == 0);
      vis |= v ? 1u << e : 0u;
      mx = fmaxf(mx, v ? raw[e] : kNegBig);
    }
  }
  mx = mx > 0.5f * kNegBig ? mx * sfac : kNegBig;           // sfac > 0: the maximum commutes with the scaling
  if (__ballot(mx > mref + Softmax<T>::lazy) != 0) {        // uniform; always taken on a query's first visible key
    const float mnew = fmaxf(mref, rows_max(mx));
    const float alpha = Softmax<T>::ex(mref - mnew);
    lsum *= alpha;
    // the output so far needs rescaling only if some query's reference moved, and not on the first
    // tile (the output is still zero)
    if (__ballot(mnew != mref && mref > 0.5f * kNegBig) != 0) {
#pragma unroll
      for (int df = 0; df < DF; ++df)
#pragma unroll
        for (int r = 0; r < 4; ++r) O[df][r] *= alpha;
    }
    mref = mnew;
  }
  const float bias = Softmax<T>::bias(mref);
  float ps = 0.0f;
  if (full) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = Softmax<T>::prob(raw[e], sfac, bias);
      ps += p[e];
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = (vis >> e & 1u) ? Softmax<T>::prob(raw[e], sfac, bias) : 0.0f;
      ps += p[e];
    }
  }
  lsum += ps;
  Frag<T> Pf;
  pack_probs(Pf, p);
  return Pf;
}

// One workgroup = 4 waves that take the tiles of one (head, list slice) round-robin, each against
// the same 16*QF queries.  With more than 16*QF block tokens, Z workgroups share a slice; the 1-D
// grid is laid out so that those Z get consecutive slots of one XCD (workgroup b goes to XCD b % 8):
// they run at about the same time on the same L2, and the slice comes from HBM once.
template <typename T, int HD, int QF>
__global__ __launch_bounds__(256) void attn_stream_kernel(const AttnArgs a, int Z, int n_units) {
  constexpr int DS = HD / 32;   // contraction slices of q.k
  constexpr int DF = HD / 16;   // 16-row groups of the transposed output
  constexpr int TILE = 32 * HD; // elements of a 32-position tile of keys (or values)
  constexpr int NW = 4;         // waves
  constexpr int GQ = 16 * QF;   // queries per workgroup
  constexpr int DUMP = QF * DF * 4 + 2 * QF;   // floats per lane handed over in the merge
  const int slot_b = blockIdx.x / 8, xcd = blockIdx.x % 8;
  const int unit = (slot_b / Z) * 8 + xcd;                  // (head, slice) pair
  if (unit >= n_units) return;                              // padding of the last row of 8
  const int S = a.n_splits;
  const int split = unit % S, h = unit / S;
  const int hkv = h / (a.H / a.Hkv);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: tile indices and their branches stay uniform
  const int li = lane & 15, g = lane >> 4;
  const int M = a.M, C = a.C, P = a.n_dev ? *a.n_dev - 1 : a.P;
  const int q0 = (slot_b % Z) * GQ;                         // first query of this workgroup
  const bool active = q0 < M;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *qs = reinterpret_cast<T *>(smem);                      // [QF][DS][64 lanes][8]: the queries as fragments
  float *red = reinterpret_cast<float *>(smem + (size_t)QF * DS * 512 * sizeof(T));   // [4 waves][DUMP][64]

  // ---- the tile list: NP cached tiles, then the NS tiles of the block's own keys that hold the draft
  //      rows of this workgroup's queries; this workgroup takes list entries [t_begin, t_end) -----------
  const int q_lo = min(q0, M - 1), q_hi = min(M, q0 + GQ) - 1;
  const int NP = (P + 31) / 32;
  const int sb = block_row_start(q_lo, C, a.shared0) / 32 * (a.shared0 ? 0 : 1);   // first block tile (tile 0 holds the shared token)
  const int NS = q_hi / 32 + 1 - sb;                        // no query sees a block key beyond itself
  const int TL = NP + NS;
  const int t_begin = (int)((long)TL * split / S), t_end = (int)((long)TL * (split + 1) / S);
  const int n_tiles = active ? t_end - t_begin : 0;
  const T *kc = (const T *)a.kcache + (size_t)hkv * a.Spad * HD, *vc = (const T *)a.vcache + (size_t)hkv * a.Spad * HD;
  const T *ksc = (const T *)a.kscr + (size_t)hkv * a.kv_rows * HD, *vsc = (const T *)a.vscr + (size_t)hkv * a.kv_rows * HD;

  // this lane's queries (result columns), one per group of 16: visible block keys are [qlo, qhi]
  int qlo[QF], qhi[QF];
  float mrun[QF], lrun[QF];
  f32x4 O[QF][DF];
#pragma unroll
  for (int qf = 0; qf < QF; ++qf) {
    const int mq = min(q0 + qf * 16 + li, M - 1);
    qlo[qf] = block_row_start(mq, C, a.shared0);
    qhi[qf] = mq;
    mrun[qf] = kNegBig;
    lrun[qf] = 0.0f;
#pragma unroll
    for (int df = 0; df < DF; ++df) O[qf][df] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // tile registers, two sets: K as 2 x DS fragments (rows = keys in the permuted order of
  // kv_key_row), V as DF fragments (rows = dims, contraction = the tile's 32 keys)
  Frag<T> kf[2][2][DS], vf[2][DF];
  auto load_tile = [&](Frag<T> (&kr)[2][DS], Frag<T> (&vr)[DF], int t) {
    const int ct = max(min(t_begin + t, t_end - 1), 0);     // clamped into the list: loads are unconditional
    const bool own = ct >= NP;
    const size_t off = (size_t)(own ? sb + ct - NP : ct) * TILE;
    const T *kp = tiled_block((own ? ksc : kc) + off, 0, DS, lane);
    const T *vp = tiled_block((own ? vsc : vc) + off, 0, 1, lane);
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) kr[f][ds] = load_frag_stream(kp + (f * DS + ds) * 512);
#pragma unroll
    for (int df = 0; df < DF; ++df) vr[df] = load_frag_stream(vp + df * 512);
  };

  const float sfac = Softmax<T>::factor(a.scale);
  constexpr int QG = QF >= 2 ? 2 : 1;                       // query groups in flight together (independent MFMA chains)
  auto compute = [&](const Frag<T> (&kr)[2][DS], const Frag<T> (&vr)[DF], int t) {
    if (t < n_tiles) {                                      // uniform per wave
      const int ct = t_begin + t;
      const bool own = ct >= NP;
      const int tile0 = (own ? sb + ct - NP : ct) * 32;
      const int k0 = tile0 + 8 * g;                         // this lane's first key of the tile
      const bool full = !own && tile0 + 32 <= P;            // every key visible to every query: no masks
#pragma unroll
      for (int q2 = 0; q2 < QF; q2 += QG) {
        __asm__ volatile("" ::: "memory");                  // keep the query fragments in LDS: re-read them here
        // scores, transposed: rows = keys, columns = queries.  Fragment f's row i is key
        // 8*(i/4) + 4f + (i%4) of the tile, so this lane ends up with 8 consecutive keys.
        f32x4 Sc[QG][2];
#pragma unroll
        for (int j = 0; j < QG; ++j)
#pragma unroll
          for (int f = 0; f < 2; ++f) Sc[j][f] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ds = 0; ds < DS; ++ds)
#pragma unroll
          for (int j = 0; j < QG; ++j) {
            const Frag<T> qfrag = load_frag(qs + (size_t)(((q2 + j) * DS + ds) * 64 + lane) * 8);
#pragma unroll
            for (int f = 0; f < 2; ++f) mma(Sc[j][f], kr[f][ds], qfrag);
          }
#pragma unroll
        for (int j = 0; j < QG; ++j) {
          const int qf = q2 + j;
          const Frag<T> Pf = softmax_tile<T, DF>(Sc[j], sfac, full, k0, own ? qlo[qf] : 0, own ? qhi[qf] : P - 1,
                                                 own && a.shared0, mrun[qf], lrun[qf], O[qf]);
#pragma unroll
          for (int df = 0; df < DF; ++df) mma(O[qf][df], vr[df], Pf);
        }
      }
    }
  };

  load_tile(kf[0], vf[0], wv);                              // on its way while the queries are staged

  // ---- queries into LDS, in operand order: entry (qf, ds, l) = query q0 + 16 qf + l%16, dims 32 ds + 8 (l/16) .. +8
  for (int e = tid; e < QF * DS * 64; e += 64 * NW) {
    const int l = e & 63, fd = e >> 6, qf = fd / DS, ds = fd - qf * DS;
    const int mq = min(q0 + qf * 16 + (l & 15), M - 1);
    const T *src = (const T *)a.q + ((size_t)h * a.Mcap + mq) * HD + ds * 32 + (l >> 4) * 8;
    T *dst = qs + (size_t)e * 8;
    if constexpr (sizeof(T) == 2) {
      *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<const u32x4 *>(src);
    } else {
      *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<const u32x4 *>(src);
      *reinterpret_cast<u32x4 *>(dst + 4) = *reinterpret_cast<const u32x4 *>(src + 4);
    }
  }
  __syncthreads();

  for (int t = wv; t < n_tiles; t += 2 * NW) {
    load_tile(kf[1], vf[1], t + NW);
    compute(kf[0], vf[0], t);
    load_tile(kf[0], vf[0], t + 2 * NW);
    compute(kf[1], vf[1], t + NW);
  }

  // ---- merge the four waves through LDS: every wave hands over its (max, sum, output) registers,
  //      then wave w combines items w, w + 4, ... of the QF*DF output fragments, always adding the
  //      waves in the order 0, 1, 2, 3, and stores them as this workgroup's partial -------------------
  {
    float *dst = red + (size_t)wv * DUMP * 64;
#pragma unroll
    for (int qf = 0; qf < QF; ++qf) {
#pragma unroll
      for (int df = 0; df < DF; ++df)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[((qf * DF + df) * 4 + r) * 64 + lane] = O[qf][df][r];
      dst[(QF * DF * 4 + 2 * qf) * 64 + lane] = mrun[qf];
      dst[(QF * DF * 4 + 2 * qf + 1) * 64 + lane] = lrun[qf];
    }
  }
  __syncthreads();
  if (!active) return;
  for (int item = wv; item < QF * DF; item += NW) {
    const int qf = item / DF, df = item - qf * DF;
    const int m = q0 + qf * 16 + li;
    float mw[NW], mstar = kNegBig;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      mw[w] = red[((size_t)w * DUMP + QF * DF * 4 + 2 * qf) * 64 + lane];
      mstar = fmaxf(mstar, mw[w]);
    }
    float l = 0.0f;
    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wgt = Softmax<T>::ex(mw[w] - mstar);
      l += red[((size_t)w * DUMP + QF * DF * 4 + 2 * qf + 1) * 64 + lane] * wgt;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] += red[((size_t)w * DUMP + item * 4 + r) * 64 + lane] * wgt;
    }
    l = rows_sum(l);                                        // the four lanes of a query each held a share of its sum
    // partial outputs keep the fragment order, [head][slice][16-query group][df][lane][4]: one store
    // instruction of the wave writes 1 KB contiguously
    const size_t blk = ((size_t)h * S + split) * (a.Mpart / 16) + (q0 / 16 + qf);
    *reinterpret_cast<float4 *>(a.part_o + ((blk * DF + df) * 64 + lane) * 4) = float4{o[0], o[1], o[2], o[3]};
    if (m < M && df == 0 && g == 0) {
      const size_t slot = ((size_t)h * S + split) * a.Mpart + m;
      a.part_ml[slot * 2 + 0] = mstar;
      a.part_ml[slot * 2 + 1] = l;
    }
  }
}

// Workgroup = (head, list slice, group of 64*QF queries); wave w owns queries q0 + 16*QF*w .. and
// reads every tile of the slice from the LDS copy.  Grid layout as in attn_stream_kernel.
template <typename T, int HD, int QF, bool NT>
__global__ __launch_bounds__(256, 2) void attn_shared_kernel(const AttnArgs a, int Z, int n_units) {
  constexpr int DS = HD / 32, DF = HD / 16;
  constexpr int TILE = 32 * HD;
  constexpr int GQ = 64 * QF;                               // queries per workgroup
  constexpr int PIECES = TILE * (int)sizeof(T) / 16;        // 16-byte pieces of a K (or V) tile
  constexpr int PPT = (PIECES + 255) / 256;                 // pieces per thread
  const int slot_b = blockIdx.x / 8, xcd = blockIdx.x % 8;
  const int unit = (slot_b / Z) * 8 + xcd;
  if (unit >= n_units) return;
  const int S = a.n_splits;
  const int split = unit % S, h = unit / S;
  const int hkv = h / (a.H / a.Hkv);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, g = lane >> 4;
  const int M = a.M, C = a.C, P = a.n_dev ? *a.n_dev - 1 : a.P;
  const int q0 = (slot_b % Z) * GQ;                         // first query of this workgroup (< M)
  const int qw = q0 + wv * 16 * QF;                         // first query of this wave
  const bool active = qw < M;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *kl = reinterpret_cast<T *>(smem);                      // [2][TILE] key tiles
  T *vl = kl + 2 * TILE;                                    // [2][TILE] value tiles

  const int q_hi = min(M, q0 + GQ) - 1;
  const int NP = (P + 31) / 32;
  const int sb = block_row_start(q0, C, a.shared0) / 32 * (a.shared0 ? 0 : 1);     // first block tile (tile 0 holds the shared token)
  const int NS = q_hi / 32 + 1 - sb;                        // no query sees a block key beyond itself
  const int TL = NP + NS;
  const int t_begin = (int)((long)TL * split / S), t_end = (int)((long)TL * (split + 1) / S);
  const int n_tiles = t_end - t_begin;
  const T *kc = (const T *)a.kcache + (size_t)hkv * a.Spad * HD, *vc = (const T *)a.vcache + (size_t)hkv * a.Spad * HD;
  const T *ksc = (const T *)a.kscr + (size_t)hkv * a.kv_rows * HD, *vsc = (const T *)a.vscr + (size_t)hkv * a.kv_rows * HD;

  // DEPTH register stages: tile t + DEPTH is requested when tile t is used (four stages measured slower than
  // two, at a 16K context and at 2K).  NT: the tiles are read with non-temporal loads (the launcher's choice).
  constexpr int DEPTH = 2;
  u32x4 kst[DEPTH][PPT], vst[DEPTH][PPT];
  auto stage_load = [&](u32x4 (&kr)[PPT], u32x4 (&vr)[PPT], int t) {
    const int ct = max(min(t_begin + t, t_end - 1), 0);     // clamped into the list: loads are unconditional
    const bool own = ct >= NP;
    const size_t off = (size_t)(own ? sb + ct - NP : ct) * TILE;
    const T *kp = (own ? ksc : kc) + off, *vp = (own ? vsc : vc) + off;
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      const int pc = min(tid + 256 * i, PIECES - 1);        // surplus threads repeat the last piece
      const u32x4 *ksrc = reinterpret_cast<const u32x4 *>(kp + (size_t)pc * (16 / sizeof(T)));
      const u32x4 *vsrc = reinterpret_cast<const u32x4 *>(vp + (size_t)pc * (16 / sizeof(T)));
      if constexpr (NT) { kr[i] = __builtin_nontemporal_load(ksrc); vr[i] = __builtin_nontemporal_load(vsrc); }
      else              { kr[i] = *ksrc; vr[i] = *vsrc; }
    }
  };
  auto stage_store = [&](const u32x4 (&kr)[PPT], const u32x4 (&vr)[PPT], int buf) {
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      const int pc = min(tid + 256 * i, PIECES - 1);
      *reinterpret_cast<u32x4 *>(kl + (size_t)buf * TILE + (size_t)pc * (16 / sizeof(T))) = kr[i];
      *reinterpret_cast<u32x4 *>(vl + (size_t)buf * TILE + (size_t)pc * (16 / sizeof(T))) = vr[i];
    }
  };
#pragma unroll
  for (int u = 0; u < DEPTH; ++u) stage_load(kst[u], vst[u], u);

  // this lane's queries (result columns), one per group of 16: visible block keys are [qlo, qhi]
  int qlo[QF], qhi[QF];
  float mrun[QF], lrun[QF];
  Frag<T> Q[QF][DS];
  f32x4 O[QF][DF];
#pragma unroll
  for (int qf = 0; qf < QF; ++qf) {
    const int mq = min(qw + qf * 16 + li, M - 1);
    qlo[qf] = block_row_start(mq, C, a.shared0);
    qhi[qf] = mq;
    mrun[qf] = kNegBig;
    lrun[qf] = 0.0f;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) Q[qf][ds] = load_frag((const T *)a.q + ((size_t)h * a.Mcap + mq) * HD + ds * 32 + g * 8);
#pragma unroll
    for (int df = 0; df < DF; ++df) O[qf][df] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float sfac = Softmax<T>::factor(a.scale);
  constexpr int LOFF = sizeof(T) == 2 ? 8 : 4;              // this lane's slice of a 1 KB (fp32: half-)block

  auto compute = [&](int t, int buf) {
    if (active && t < n_tiles) {                            // uniform per wave
      const int ct = t_begin + t;
      const bool own = ct >= NP;
      const int tile0 = (own ? sb + ct - NP : ct) * 32;
      const int k0 = tile0 + 8 * g;
      const bool full = !own && tile0 + 32 <= P;
      const T *kt = kl + (size_t)buf * TILE + lane * LOFF, *vt = vl + (size_t)buf * TILE + lane * LOFF;
      f32x4 Sc[QF][2];
#pragma unroll
      for (int qf = 0; qf < QF; ++qf)
#pragma unroll
        for (int f = 0; f < 2; ++f) Sc[qf][f] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ds = 0; ds < DS; ++ds)
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          const Frag<T> kfrag = load_frag_tiled(kt + (f * DS + ds) * 512);
#pragma unroll
          for (int qf = 0; qf < QF; ++qf) mma(Sc[qf][f], kfrag, Q[qf][ds]);
        }
      Frag<T> Pf[QF];
#pragma unroll
      for (int qf = 0; qf < QF; ++qf)
        Pf[qf] = softmax_tile<T, DF>(Sc[qf], sfac, full, k0, own ? qlo[qf] : 0, own ? qhi[qf] : P - 1, own && a.shared0,
                                     mrun[qf], lrun[qf], O[qf]);
#pragma unroll
      for (int df = 0; df < DF; ++df) {                     // every value fragment is read from LDS once for all query groups
        const Frag<T> vfrag = load_frag_tiled(vt + df * 512);
#pragma unroll
        for (int qf = 0; qf < QF; ++qf) mma(O[qf][df], vfrag, Pf[qf]);
      }
    }
  };

  // The query fragments must have landed before the loop: left pending, the compiler guards their first use
  // inside the loop body with a count that in later trips also waits for the tile requested one trip earlier,
  // and the loop runs one tile deep, at the memory latency (the first tile is needed right away anyway).
  __builtin_amdgcn_s_waitcnt(0x0F70);                       // vmcnt(0)
  for (int t = 0; t < n_tiles; t += DEPTH) {                // barriers are uniform; the tail of a round only loads
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      stage_store(kst[u], vst[u], u & 1);
      __syncthreads();
      stage_load(kst[u], vst[u], t + u + DEPTH);
      compute(t + u, u & 1);
    }
  }

  if (active) {
#pragma unroll
    for (int qf = 0; qf < QF; ++qf) {
      // partial outputs keep the fragment order, [head][slice][16-query group][df][lane][4]
      const size_t blk = ((size_t)h * S + split) * (a.Mpart / 16) + (qw / 16 + qf);
#pragma unroll
      for (int df = 0; df < DF; ++df)
        *reinterpret_cast<float4 *>(a.part_o + ((blk * DF + df) * 64 + lane) * 4) =
            float4{O[qf][df][0], O[qf][df][1], O[qf][df][2], O[qf][df][3]};
      const int m = qw + qf * 16 + li;
      const float l = rows_sum(lrun[qf]);                   // the four lanes of a query each held a share of its sum
      if (m < M && g == 0) {
        const size_t slot = ((size_t)h * S + split) * a.Mpart + m;
        a.part_ml[slot * 2 + 0] = mrun[qf];
        a.part_ml[slot * 2 + 1] = l;
      }
    }
  }
}

// out[m][h*HD + d] = sum_s o_s[d] e^{m_s - m*} / sum_s l_s e^{m_s - m*}, slices taken in index order,
// 8 at a time with a running maximum (one round of loads when there are at most 8 slices: the kernel
// is a chain of memory latencies, nothing else).  One workgroup per (16-query group, head); a thread
// owns one lane's 4 values of an output fragment (dims 16 df + 4 (lane/16) .. +4 of query lane%16).
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(const AttnArgs a) {
  constexpr int DF = HD / 16;
  const int qb = blockIdx.x, h = blockIdx.y;
  const int S = a.n_splits, MB = a.Mpart / 16;
  // two workgroups per (16-query group, head), one per half of the output fragments: more CUs pull the partials
  const int idx0 = blockIdx.z * (DF * 32), idx1 = idx0 + DF * 32;
  for (int idx = idx0 + threadIdx.x; idx < idx1; idx += 256) {
    const int df = idx >> 6, lane = idx & 63;
    const int m = qb * 16 + (lane & 15), d4 = df * 16 + 4 * (lane >> 4);
    if (m >= a.M) continue;
    const size_t slot0 = (size_t)h * S * a.Mpart + m;
    float mrun = kNegBig, l = 0.0f;
    float4 o{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < S; s0 += 8) {
      float4 v[8];
      float2 ml[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int sc = min(s0 + i, S - 1);
        v[i] = *reinterpret_cast<const float4 *>(a.part_o + (((((size_t)h * S + sc) * MB + qb) * DF + df) * 64 + lane) * 4);
        ml[i] = *reinterpret_cast<const float2 *>(a.part_ml + (slot0 + (size_t)sc * a.Mpart) * 2);
      }
      float mnew = mrun;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (s0 + i < S) mnew = fmaxf(mnew, ml[i].x);
      const float alpha = Softmax<T>::ex(mrun - mnew);
      l *= alpha; o.x *= alpha; o.y *= alpha; o.z *= alpha; o.w *= alpha;
      mrun = mnew;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (s0 + i < S) {
          const float wgt = Softmax<T>::ex(ml[i].x - mrun);
          l += ml[i].y * wgt;
          o.x += v[i].x * wgt; o.y += v[i].y * wgt; o.z += v[i].z * wgt; o.w += v[i].w * wgt;
        }
      }
    }
    const float inv = 1.0f / l;
    store4((T *)a.out + act_offset<T>(m, h * HD + d4, a.Mcap), o.x * inv, o.y * inv, o.z * inv, o.w * inv);
  }
}

template <typename T, int HD, int QF>
static void launch_stream(const AttnArgs &a, hipStream_t s) {
  const size_t lds = (size_t)QF * (HD / 32) * 512 * sizeof(T) + (size_t)4 * (QF * (HD / 16) * 4 + 2 * QF) * 64 * sizeof(float);
  const int Z = (a.M + 16 * QF - 1) / (16 * QF);
  const int n_units = a.n_splits * a.H;
  hipLaunchKernelGGL((attn_stream_kernel<T, HD, QF>), dim3((n_units + 7) / 8 * 8 * Z), dim3(256), lds, s, a, Z, n_units);
}

// query groups of 16 per wave in attn_shared_kernel: two once a block has more than 64 tokens,
// where the registers hold them (fp32 fragments are twice as large)
template <typename T, int HD> constexpr int attn_shared_qmax() { return sizeof(T) == 2 || HD <= 64 ? 2 : 1; }

template <typename T, int HD, int QF>
static void launch_shared(const AttnArgs &a, hipStream_t s) {
  const size_t lds = (size_t)4 * 32 * HD * sizeof(T);
  const int Z = (a.M + 64 * QF - 1) / (64 * QF);
  const int n_units = a.n_splits * a.H;
  // Slices of a dozen tiles or more that no other workgroup shares are read with non-temporal loads (measured on
  // MI355X, whole verify step: 7.07 -> 6.86 ms at a 16.4K context with 32 tiles per slice, 3.08 -> 3.06 ms at 13
  // tiles; 4.18 -> 4.19 ms at 8 tiles, where they stay ordinary loads)
  const int tiles = ((a.P + 31) / 32 + 1) / a.n_splits;
  const bool nt = Z == 1 && tiles >= 12;
  if (nt) hipLaunchKernelGGL((attn_shared_kernel<T, HD, QF, true>), dim3((n_units + 7) / 8 * 8 * Z), dim3(256), lds, s, a, Z, n_units);
  else hipLaunchKernelGGL((attn_shared_kernel<T, HD, QF, false>), dim3((n_units + 7) / 8 * 8 * Z), dim3(256), lds, s, a, Z, n_units);
}

template <typename T, int HD>
static void launch_hd(const AttnArgs &a, hipStream_t s) {
  if (a.M <= 16) launch_stream<T, HD, 1>(a, s);
  else if (a.M <= 64 || attn_shared_qmax<T, HD>() == 1) launch_shared<T, HD, 1>(a, s);
  else launch_shared<T, HD, attn_shared_qmax<T, HD>()>(a, s);
  hipLaunchKernelGGL((attn_merge_kernel<T, HD>), dim3((a.M + 15) / 16, a.H, 2), dim3(256), 0, s, a);
}

// Number of list slices per head: one workgroup per CU in total; two per CU for blocks of more than
// 64 tokens once every slice still has 16 tiles (measured at a 16K context: 74 -> 69 us; everywhere
// else one per CU was as fast or faster); never fewer than 4 tiles per slice.
int attention_splits(int dtype, int hd, int H, int M, int P, int max_splits) {
  const int qmax = dtype == 1 || hd <= 64 ? 2 : 1;
  const int per_wg = M <= 16 ? 16 : (M <= 64 ? 64 : 64 * qmax);
  const int Z = (M + per_wg - 1) / per_wg;
  const int tiles = (P + 31) / 32 + 1;
  const int one = 256 / (H * Z), two = M > 64 ? 512 / (H * Z) : one;
  int s = tiles / 16 > one ? tiles / 16 : one;
  s = s < two ? s : two;
  s = s < tiles / 4 ? s : tiles / 4;
  s = s < max_splits ? s : max_splits;
  return s < 1 ? 1 : s;
}

int attention_workgroups(int dtype, int hd, int H, int M, int n_splits) {
  const int qmax = dtype == 1 || hd <= 64 ? 2 : 1;
  const int per_wg = M <= 16 ? 16 : (M <= 64 ? 64 : 64 * qmax);
  return n_splits * H * ((M + per_wg - 1) / per_wg);
}

template <typename T>
static void launch_t(int hd, const AttnArgs &a, hipStream_t s) {
  if (hd == 32) launch_hd<T, 32>(a, s);
  else if (hd == 64) launch_hd<T, 64>(a, s);
  else launch_hd<T, 128>(a, s);
}

void launch_attention(int dtype, int hd, const AttnArgs &a, hipStream_t s) {
  if (dtype == 1) launch_t<half_t>(hd, a, s);
  else launch_t<float>(hd, a, s);
}

}  // namespace ngg
