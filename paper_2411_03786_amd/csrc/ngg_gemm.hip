// Skinny GEMM  Y[M x N] = X[M x K] . W[N x K]^T  for the k*(w+1) block rows of a verify call
// (Section 3: a model call on a (k, w+1) block is meant to stay memory-bound, so the kernel is
// built around streaming W once).  W rows are the MFMA "row" operand, X rows the "column"
// operand; each workgroup owns FN groups of 16 output features, its waves split the contraction
// index and reduce through LDS in a fixed order (deterministic).  Epilogues fuse rotary
// embedding + KV-scratch write, SwiGLU, the residual add and the per-position argmax partials.
#include "ngg_internal.h"

namespace ngg {

template <typename T, int FN, int FM>
struct Tile {
  Frag<T> a[FN];
  Frag<T> b[FM];
};

template <typename T, int EPI, int FN, int FM, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(const GemmArgs a) {
  const int tile = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int li = lane & 15, g = lane >> 4;
  const int K = a.K, M = a.M;

  // ---- which 16-row groups of W this workgroup owns ---------------------------------------------
  const T *wrow[FN];   // this lane's row of each group, offset to its 8-element slice
  int nbase[FN];       // logical output feature of each group's first row
  int head = 0, sub = 0, kind = 0;   // EPI_QKV: kind 0 = q, 1 = k, 2 = v
  if constexpr (EPI == EPI_QKV) {
    static_assert(FN == 2, "rotary pairs need two groups");
    const int tph = a.hd / 32;                       // tiles per head
    head = tile / tph;
    sub = tile - head * tph;
    const T *base;
    int hrow;                                        // first row of the head inside its matrix
    if (head < a.H) { kind = 0; base = (const T *)a.W0; hrow = head * a.hd; }
    else if (head < a.H + a.Hkv) { kind = 1; base = (const T *)a.W1; hrow = (head - a.H) * a.hd; head -= a.H; }
    else { kind = 2; base = (const T *)a.W2; hrow = (head - a.H - a.Hkv) * a.hd; head -= a.H + a.Hkv; }
#pragma unroll
    for (int f = 0; f < FN; ++f) {
      nbase[f] = f * (a.hd / 2) + sub * 16;          // element index inside the head
      wrow[f] = base + (size_t)(hrow + nbase[f] + li) * K + g * 8;
    }
  } else if constexpr (EPI == EPI_GATEUP) {
    static_assert(FN == 2, "gate and up rows travel together");
    nbase[0] = nbase[1] = tile * 16;
    wrow[0] = (const T *)a.W0 + (size_t)(tile * 16 + li) * K + g * 8;
    wrow[1] = (const T *)a.W1 + (size_t)(tile * 16 + li) * K + g * 8;
  } else {
#pragma unroll
    for (int f = 0; f < FN; ++f) {
      nbase[f] = (tile * FN + f) * 16;
      wrow[f] = (const T *)a.W0 + (size_t)(nbase[f] + li) * K + g * 8;
    }
  }

  const int steps = K / 32;
  const int s0 = (int)(((long)steps * wave) / WAVES);
  const int s1 = (int)(((long)steps * (wave + 1)) / WAVES);

  extern __shared__ float red[];   // [(WAVES-1)][FN*FM*4][64]

  for (int m0 = 0; m0 < M; m0 += 16 * FM) {
    const T *xrow[FM];
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
      int m = m0 + fm * 16 + li;
      m = m < M ? m : M - 1;                         // rows past M repeat the last one; never stored
      xrow[fm] = (const T *)a.X + (size_t)m * a.ldx + g * 8;
    }
    f32x4 acc[FN][FM];
#pragma unroll
    for (int f = 0; f < FN; ++f)
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) acc[f][fm] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto load_tile = [&](Tile<T, FN, FM> &t, int s) {
#pragma unroll
      for (int f = 0; f < FN; ++f) t.a[f] = load_frag(wrow[f] + (size_t)s * 32);
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) t.b[fm] = load_frag(xrow[fm] + (size_t)s * 32);
    };
    auto mma_tile = [&](const Tile<T, FN, FM> &t) {
#pragma unroll
      for (int f = 0; f < FN; ++f)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) mma(acc[f][fm], t.a[f], t.b[fm]);
    };

    Tile<T, FN, FM> t0, t1;
    int s = s0;
    if (s < s1) load_tile(t0, s);
    while (s < s1) {
      if (s + 1 < s1) load_tile(t1, s + 1);
      mma_tile(t0);
      ++s;
      if (s >= s1) break;
      if (s + 1 < s1) load_tile(t0, s + 1);
      mma_tile(t1);
      ++s;
    }

    // ---- reduce the waves' partial sums: wave 0 adds waves 1 .. WAVES-1 in that order ----------
    if constexpr (WAVES > 1) {
      if (wave > 0) {
        float *dst = red + (size_t)(wave - 1) * (FN * FM * 4 * 64);
#pragma unroll
        for (int f = 0; f < FN; ++f)
#pragma unroll
          for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[((f * FM + fm) * 4 + r) * 64 + lane] = acc[f][fm][r];
      }
      __syncthreads();
      if (wave == 0) {
        for (int wv = 1; wv < WAVES; ++wv) {
          const float *src = red + (size_t)(wv - 1) * (FN * FM * 4 * 64);
#pragma unroll
          for (int f = 0; f < FN; ++f)
#pragma unroll
            for (int fm = 0; fm < FM; ++fm)
#pragma unroll
              for (int r = 0; r < 4; ++r) acc[f][fm][r] += src[((f * FM + fm) * 4 + r) * 64 + lane];
        }
      }
    }

    // ---- epilogue (wave 0): lane holds, per group f and column block fm, column m = m0+fm*16+li
    //      and output features nbase[f] + 4g .. +4 -------------------------------------------------
    if (wave == 0) {
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) {
        const int m = m0 + fm * 16 + li;
        const bool live = m < M;
        if constexpr (EPI == EPI_RESIDUAL) {
          if (live) {
#pragma unroll
            for (int f = 0; f < FN; ++f) {
              float4 *p = reinterpret_cast<float4 *>(a.h + (size_t)m * a.N + nbase[f] + 4 * g);
              float4 v = *p;
              v.x += acc[f][fm][0]; v.y += acc[f][fm][1]; v.z += acc[f][fm][2]; v.w += acc[f][fm][3];
              *p = v;
            }
          }
        } else if constexpr (EPI == EPI_GATEUP) {
          if (live) {
            T *p = (T *)a.act + (size_t)m * a.N + nbase[0] + 4 * g;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float gt = acc[0][fm][r], up = acc[1][fm][r];
              const float sg = gt / (1.0f + fast_exp<float>(-gt));       // silu(gate)
              p[r] = from_f32<T>(sg * up);
            }
          }
        } else if constexpr (EPI == EPI_QKV) {
          if (live) {
            const int half = a.hd / 2;
            float lo[4], hi[4];
            if (kind < 2) {                                  // rotary embedding on q and k
              const int pos = a.P + (m % a.C);
              const float *cs = a.rope_cos + (size_t)pos * half + nbase[0] + 4 * g;
              const float *sn = a.rope_sin + (size_t)pos * half + nbase[0] + 4 * g;
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float x1 = acc[0][fm][r], x2 = acc[1][fm][r];
                lo[r] = x1 * cs[r] - x2 * sn[r];
                hi[r] = x2 * cs[r] + x1 * sn[r];
              }
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) { lo[r] = acc[0][fm][r]; hi[r] = acc[1][fm][r]; }
            }
            if (kind < 2) {
              T *dst = (kind == 0 ? (T *)a.q : (T *)a.kscr) + ((size_t)head * a.Mcap + m) * a.hd + nbase[0] + 4 * g;
#pragma unroll
              for (int r = 0; r < 4; ++r) { dst[r] = from_f32<T>(lo[r]); dst[half + r] = from_f32<T>(hi[r]); }
            } else {                                         // v is kept transposed: [dim][m]
              T *dst = (T *)a.vscr + ((size_t)head * a.hd + nbase[0] + 4 * g) * a.Mcap + m;
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                dst[(size_t)r * a.Mcap] = from_f32<T>(lo[r]);
                dst[(size_t)(half + r) * a.Mcap] = from_f32<T>(hi[r]);
              }
            }
          }
        } else {   // EPI_UNEMBED: optional logits, and this tile's best (value, id) per column
          float bv = kNegBig;
          int bi = 0x7fffffff;
#pragma unroll
          for (int f = 0; f < FN; ++f)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float v = acc[f][fm][r];
              const int n = nbase[f] + 4 * g + r;
              if (a.logits && live) a.logits[(size_t)m * a.N + n] = v;
              if (v > bv) { bv = v; bi = n; }                 // ascending n: the first maximum stays
            }
#pragma unroll
          for (int off = 16; off < 64; off <<= 1) {
            const float ov = __shfl_xor(bv, off);
            const int oi = __shfl_xor(bi, off);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
          }
          if (live && g == 0) {
            a.pmax_val[(size_t)tile * a.Mcap + m] = bv;
            a.pmax_idx[(size_t)tile * a.Mcap + m] = bi;
          }
        }
      }
    }
    if constexpr (WAVES > 1) __syncthreads();          // LDS is reused by the next column block
  }
}

template <typename T, int EPI, int FN, int FM, int WAVES>
static void launch_one(const GemmArgs &a, int tiles, hipStream_t s) {
  const size_t lds = (size_t)(WAVES - 1) * FN * FM * 4 * 64 * sizeof(float);
  hipLaunchKernelGGL((gemm_skinny_kernel<T, EPI, FN, FM, WAVES>), dim3(tiles), dim3(WAVES * 64), lds, s, a);
}

template <typename T, int EPI, int FN, int WAVES>
static void launch_fm(const GemmArgs &a, int tiles, hipStream_t s) {
  if (a.M <= 16) launch_one<T, EPI, FN, 1, WAVES>(a, tiles, s);
  else if (a.M <= 32) launch_one<T, EPI, FN, 2, WAVES>(a, tiles, s);
  else launch_one<T, EPI, FN, 4, WAVES>(a, tiles, s);
}

int gemm_unembed_tiles(int N) { return N / 32 * 32 == N ? N / 32 : N / 16; }

template <typename T>
static void launch_t(int epi, const GemmArgs &a, hipStream_t s) {
  switch (epi) {
    case EPI_QKV: launch_fm<T, EPI_QKV, 2, 4>(a, (a.H + 2 * a.Hkv) * (a.hd / 32), s); break;
    case EPI_GATEUP: launch_fm<T, EPI_GATEUP, 2, 4>(a, a.N / 16, s); break;
    case EPI_RESIDUAL: launch_fm<T, EPI_RESIDUAL, 1, 8>(a, a.N / 16, s); break;
    default:
      if (a.N % 32 == 0) launch_fm<T, EPI_UNEMBED, 2, 4>(a, a.N / 32, s);
      else launch_fm<T, EPI_UNEMBED, 1, 4>(a, a.N / 16, s);
  }
}

void launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t s) {
  if (dtype == 1) launch_t<bf16_t>(epi, a, s);
  else launch_t<float>(epi, a, s);
}

}  // namespace ngg
