// Shared-prefix attention for the verify block.  Section 4.1 batches the k drafts by repeating
// the context into k identical rows, and the "Limitations" paragraph names the redundant prefix
// work as the method's cost; here the cached context is read ONCE for all k rows: a workgroup
// owns (head, key span), and every block token (row r, column j) is a query against that span.
// The block's own keys (row r, columns <= j) form one more "span" with a per-row causal mask.
// Partial (max, sum, output) triples are merged by a second kernel in span order (deterministic).
//
// Layouts: keys [kv head][position][head_dim]; values in tiles of 32 positions, transposed inside
// the tile, [kv head][position/32][head_dim][32]: a tile of 32 keys and its 32 values are two
// contiguous regions, staged through LDS once per workgroup (double buffered) and read from there
// by the four waves (one group of 16 queries each) as MFMA row operands.
#include "ngg_internal.h"

namespace ngg {

// element (position, dim) of a value tensor stored in tiles of 32 positions: [position/32][dim][32]
template <int HD>
__host__ __device__ __forceinline__ size_t v_offset(int pos, int dim) {
  return ((size_t)(pos / 32) * HD + dim) * 32 + pos % 32;
}

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(const AttnArgs a) {
  constexpr int DS = HD / 32;   // contraction slices of q.k
  constexpr int DF = HD / 16;   // 16-row groups of the transposed output
  constexpr int PAD = 16 / (int)sizeof(T);
  constexpr int KROW = HD + PAD, VROW = 32 + PAD;           // padded LDS rows: conflict-free fragment reads
  constexpr int TILE_PIECES = 32 * HD * (int)sizeof(T) / 16;   // 16-byte pieces of a 32-key K (or V) tile
  constexpr int PPT = (TILE_PIECES + 255) / 256;            // pieces per thread
  constexpr int KPPR = HD * (int)sizeof(T) / 16;            // pieces per key row
  constexpr int VPPR = 32 * (int)sizeof(T) / 16;            // pieces per dim row
  const int split = blockIdx.x, h = blockIdx.y, mg = blockIdx.z;
  const int hkv = h / (a.H / a.Hkv);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int li = lane & 15, g = lane >> 4;
  const bool suffix = split == a.n_splits;
  const int M = a.M, C = a.C;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *ks = reinterpret_cast<T *>(smem);                      // [2][32][KROW], rows in fragment order
  T *vs = ks + 2 * 32 * KROW;                               // [2][HD][VROW]

  const T *kbase, *vbase;
  int key_begin, key_end, last_tile_key;
  if (!suffix) {
    kbase = (const T *)a.kcache + (size_t)hkv * a.Spad * HD;
    vbase = (const T *)a.vcache + (size_t)hkv * a.Spad * HD;
    key_begin = split * a.span;
    key_end = min(a.P, key_begin + a.span);
  } else {                                                  // the block's own keys: only the rows this group of
    kbase = (const T *)a.kscr + (size_t)hkv * a.Mcap * HD;  // 64 queries lives in
    vbase = (const T *)a.vscr + (size_t)hkv * a.Mcap * HD;
    const int q_lo = mg * 64, q_hi = min(M, q_lo + 64) - 1;
    key_begin = ((q_lo / C) * C) / 32 * 32;
    key_end = min(M, (q_hi / C + 1) * C);
  }
  const int n_tiles = (key_end - key_begin + 31) / 32;
  last_tile_key = key_begin + (n_tiles - 1) * 32;

  // staging: thread copies PPT pieces of the K tile and PPT pieces of the V tile
  int k_src[PPT], k_dst[PPT], v_src[PPT], v_dst[PPT];
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    int p = tid + 256 * i;
    p = p < TILE_PIECES ? p : TILE_PIECES - 1;              // duplicates write the same bytes
    const int kk = p / KPPR, kc = p - kk * KPPR;            // key inside the tile, 16-byte column
    k_src[i] = kk * HD + kc * PAD;
    k_dst[i] = (((kk >> 2) & 1) * 16 + (kk >> 3) * 4 + (kk & 3)) * KROW + kc * PAD;   // key 8a+4f+b -> row 16f+4a+b
    const int dd = p / VPPR, vc = p - dd * VPPR;
    v_src[i] = dd * 32 + vc * PAD;
    v_dst[i] = dd * VROW + vc * PAD;
  }
  // two register stages: the tile after next is already on its way while the current one is used
  u32x4 kst[2][PPT], vst[2][PPT];
  auto stage_load = [&](u32x4 (&kr)[PPT], u32x4 (&vr)[PPT], int t) {
    const int k0 = min(key_begin + t * 32, last_tile_key);  // clamped: loads are unconditional
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      kr[i] = *reinterpret_cast<const u32x4 *>(kbase + (size_t)k0 * HD + k_src[i]);
      vr[i] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)k0 * HD + v_src[i]);
    }
  };
  auto stage_store = [&](const u32x4 (&kr)[PPT], const u32x4 (&vr)[PPT], int buf) {
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      *reinterpret_cast<u32x4 *>(ks + buf * 32 * KROW + k_dst[i]) = kr[i];
      *reinterpret_cast<u32x4 *>(vs + buf * HD * VROW + v_dst[i]) = vr[i];
    }
  };

  const int mf = mg * 4 + wave;                             // this wave's group of 16 queries
  const bool active = mf * 16 < M;
  const int m0 = mf * 16;
  const int mq = min(m0 + li, M - 1);                       // this lane's query (result column)
  const int qrow = mq / C, qcol = mq - qrow * C;
  Frag<T> Q[DS];
#pragma unroll
  for (int ds = 0; ds < DS; ++ds) Q[ds] = load_frag((const T *)a.q + ((size_t)h * a.Mcap + mq) * HD + ds * 32 + g * 8);
  float mrun = kNegBig, lrun = 0.0f;
  f32x4 O[DF];
#pragma unroll
  for (int df = 0; df < DF; ++df) O[df] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int t, int buf) {
    if (active && t < n_tiles) {
      const int k0 = key_begin + t * 32;
      const T *kt = ks + buf * 32 * KROW + li * KROW + g * 8;
      const T *vt = vs + buf * HD * VROW + li * VROW + g * 8;
      // scores, transposed: rows = keys, columns = queries.  Fragment f's row i is key
      // k0 + 8*(i/4) + 4f + (i%4), so this lane ends up with the 8 consecutive keys k0 + 8g .. +8.
      f32x4 S[2];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        S[f] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) mma(S[f], load_frag(kt + f * 16 * KROW + ds * 32), Q[ds]);
      }
      float sv[8];
      bool vis[8];
      float mx = kNegBig;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = k0 + 8 * g + e;
        if (suffix) {
          const int kr = key / C;
          vis[e] = key < M && kr == qrow && (key - kr * C) <= qcol;
        } else {
          vis[e] = key < key_end;
        }
        sv[e] = vis[e] ? S[e >> 2][e & 3] * a.scale : kNegBig;
        mx = fmaxf(mx, sv[e]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun, mx);
      const float alpha = fast_exp<T>(mrun - mnew);
      float p[8], ps = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = vis[e] ? fast_exp<T>(sv[e] - mnew) : 0.0f;
        ps += p[e];
      }
      ps += __shfl_xor(ps, 16);
      ps += __shfl_xor(ps, 32);
      lrun = lrun * alpha + ps;
      mrun = mnew;
      Frag<T> Pf;
      pack_frag(Pf, p);
#pragma unroll
      for (int df = 0; df < DF; ++df) {
#pragma unroll
        for (int r = 0; r < 4; ++r) O[df][r] *= alpha;
        mma(O[df], load_frag(vt + df * 16 * VROW), Pf);
      }
    }
  };

  stage_load(kst[0], vst[0], 0);
  stage_load(kst[1], vst[1], 1);
  for (int t = 0; t < n_tiles; t += 2) {                    // barriers are uniform; the odd tail only loads
    stage_store(kst[0], vst[0], 0);
    __syncthreads();
    stage_load(kst[0], vst[0], t + 2);
    compute(t, 0);
    stage_store(kst[1], vst[1], 1);
    __syncthreads();
    stage_load(kst[1], vst[1], t + 3);
    compute(t + 1, 1);
  }

  const int m = m0 + li;
  if (active && m < M) {
    const size_t slot = ((size_t)h * (a.n_splits + 1) + split) * a.Mcap + m;
#pragma unroll
    for (int df = 0; df < DF; ++df) {
      float4 v{O[df][0], O[df][1], O[df][2], O[df][3]};
      *reinterpret_cast<float4 *>(a.part_o + slot * HD + df * 16 + 4 * g) = v;
    }
    if (g == 0) {
      a.part_ml[slot * 2 + 0] = mrun;
      a.part_ml[slot * 2 + 1] = lrun;
    }
  }
}

// out[m][h*HD + d] = sum_s o_s[d] e^{m_s - m*} / sum_s l_s e^{m_s - m*}, spans taken in index order.
template <typename T, int HD>
__global__ __launch_bounds__(HD) void attn_merge_kernel(const AttnArgs a) {
  const int m = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  const int S = a.n_splits + 1;
  const size_t slot0 = (size_t)h * S * a.Mcap + m;
  float mstar = kNegBig;
  for (int s = 0; s < S; ++s) mstar = fmaxf(mstar, a.part_ml[(slot0 + (size_t)s * a.Mcap) * 2]);
  float l = 0.0f, o = 0.0f;
  for (int s = 0; s < S; ++s) {
    const size_t slot = slot0 + (size_t)s * a.Mcap;
    const float wgt = fast_exp<T>(a.part_ml[slot * 2] - mstar);
    l += a.part_ml[slot * 2 + 1] * wgt;
    o += a.part_o[slot * HD + d] * wgt;
  }
  ((T *)a.out)[act_offset<T>(m, h * HD + d, a.Mcap)] = from_f32<T>(o / l);
}

template <typename T, int HD>
static void launch_hd(const AttnArgs &a, hipStream_t s) {
  constexpr int PAD = 16 / (int)sizeof(T);
  const size_t lds = (size_t)2 * (32 * (HD + PAD) + HD * (32 + PAD)) * sizeof(T);
  hipLaunchKernelGGL((attn_partial_kernel<T, HD>), dim3(a.n_splits + 1, a.H, (a.M + 63) / 64), dim3(256), lds, s, a);
  hipLaunchKernelGGL((attn_merge_kernel<T, HD>), dim3(a.M, a.H), dim3(HD), 0, s, a);
}

template <typename T>
static void launch_t(int hd, const AttnArgs &a, hipStream_t s) {
  if (hd == 32) launch_hd<T, 32>(a, s);
  else if (hd == 64) launch_hd<T, 64>(a, s);
  else launch_hd<T, 128>(a, s);
}

void launch_attention(int dtype, int hd, const AttnArgs &a, hipStream_t s) {
  if (dtype == 1) launch_t<bf16_t>(hd, a, s);
  else launch_t<float>(hd, a, s);
}

}  // namespace ngg
