// Shared-prefix attention for the verify block.  Section 4.1 batches the k drafts by repeating
// the context into k identical rows, and the "Limitations" paragraph names the redundant prefix
// work as the method's cost; here the cached context is read ONCE for all k rows: a workgroup
// owns (head, key span), and every block token (row r, column j) is a query against that span.
// The block's own keys (row r, columns <= j) form one more "span" with a per-row causal mask.
// Partial (max, sum, output) triples are merged by a second kernel in span order (deterministic).
//
// Layouts: keys [kv head][position][head_dim]; values transposed [kv head][head_dim][position],
// so both stream as MFMA row operands with the contraction index contiguous per lane.
#include "ngg_internal.h"

namespace ngg {

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(const AttnArgs a) {
  constexpr int DS = HD / 32;   // contraction slices of q.k
  constexpr int DF = HD / 16;   // 16-row groups of the transposed output
  const int split = blockIdx.x, h = blockIdx.y;
  const int hkv = h / (a.H / a.Hkv);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int li = lane & 15, g = lane >> 4;
  const bool suffix = split == a.n_splits;
  const int M = a.M, C = a.C;

  const T *kbase, *vbase;
  size_t v_ld;
  int key_begin, key_end;
  if (!suffix) {
    kbase = (const T *)a.kcache + (size_t)hkv * a.Spad * HD;
    vbase = (const T *)a.vcache + (size_t)hkv * HD * a.Spad;
    v_ld = a.Spad;
    key_begin = split * a.span;
    key_end = min(a.P, key_begin + a.span);
  } else {
    kbase = (const T *)a.kscr + (size_t)hkv * a.Mcap * HD;
    vbase = (const T *)a.vscr + (size_t)hkv * HD * a.Mcap;
    v_ld = a.Mcap;
    key_begin = 0;
    key_end = M;
  }

  const int n_mfrag = (M + 15) / 16;
  for (int mf = wave; mf < n_mfrag; mf += 4) {
    const int m0 = mf * 16;
    const int mq = min(m0 + li, M - 1);            // this lane's query (result column)
    const int qrow = mq / C, qcol = mq - qrow * C;
    Frag<T> Q[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) Q[ds] = load_frag((const T *)a.q + ((size_t)h * a.Mcap + mq) * HD + ds * 32 + g * 8);

    int kb = key_begin, ke = key_end;
    if (suffix) {                                  // only the rows this group of 16 queries lives in
      const int rlo = m0 / C, rhi = min(m0 + 15, M - 1) / C;
      kb = (rlo * C) / 32 * 32;
      ke = min(M, (rhi + 1) * C);
    }
    float mrun = kNegBig, lrun = 0.0f;
    f32x4 O[DF];
#pragma unroll
    for (int df = 0; df < DF; ++df) O[df] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int k0 = kb; k0 < ke; k0 += 32) {
      // scores, transposed: rows = keys, columns = queries.  Group f's row i is key
      // k0 + 8*(i/4) + 4f + (i%4), so this lane ends up with the 8 consecutive keys k0 + 8g .. +8.
      f32x4 S[2];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        S[f] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int key = k0 + 8 * (li >> 2) + 4 * f + (li & 3);
        const T *kp = kbase + (size_t)key * HD + g * 8;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) mma(S[f], load_frag(kp + ds * 32), Q[ds]);
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
        const T *vp = vbase + (size_t)(df * 16 + li) * v_ld + k0 + 8 * g;
        mma(O[df], load_frag(vp), Pf);
      }
    }

    const int m = m0 + li;
    if (m < M) {
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
  ((T *)a.out)[(size_t)m * (a.H * HD) + h * HD + d] = from_f32<T>(o / l);
}

template <typename T, int HD>
static void launch_hd(const AttnArgs &a, hipStream_t s) {
  hipLaunchKernelGGL((attn_partial_kernel<T, HD>), dim3(a.n_splits + 1, a.H), dim3(256), 0, s, a);
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
