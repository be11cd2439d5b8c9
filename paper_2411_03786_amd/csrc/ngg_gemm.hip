// Skinny GEMM  Y[M x N] = X[M x K] . W[N x K]^T  for the k*(w+1) block rows of a verify call
// (Section 3: a model call on a (k, w+1) block is meant to stay memory-bound, so the kernel is
// built around streaming W exactly once at HBM speed).
//
// W rows are the MFMA "row" operand.  The library keeps its own copy of every weight matrix in
// operand order (16 rows x 32 contraction elements per 1 KB block, lane-major), so one load
// instruction of a wave reads 1 KB of contiguous memory, a wave streams one contiguous region, and
// the data goes from global memory straight into MFMA registers (non-temporal loads: read once),
// prefetched RING steps ahead.  X rows are the "column" operand: the workgroup stages X[:, chunk] in LDS (double
// buffered, rows padded by 16 bytes so the 16 lanes of a quarter-wave hit distinct banks) and all
// waves read their fragments from there.  A workgroup has 4 waves arranged WN x WK: WN waves own
// different pairs of 16-row groups of W, WK waves split the steps of a chunk and are summed through
// LDS in a fixed order.  gridDim.y = KS splits the contraction across workgroups; only the
// residual epilogue supports it: every split stores its own fp32 partial, and the RMSNorm kernel
// that follows adds them in split order (deterministic, no atomics).
//
// Epilogues: rotary embedding + KV-scratch write (q, k, v), SwiGLU (gate, up), residual partial,
// and per-position argmax partials for the greedy choice (output embedding).
#include "ngg_internal.h"
#include <algorithm>
#include <type_traits>

namespace ngg {

// ---------------------------------------------------------------------------------------------
// Epilogues, shared by the skinny and the wide kernel.  `sum` is one complete 16x16 accumulator
// fragment: this lane holds column (block row) m and fragment rows 4g .. 4g+3.
// ---------------------------------------------------------------------------------------------

// q/k/v and gate/up: the fragment's rows 0..7 are the first members of 8 output pairs, rows 8..15 the
// second members (rotary pairs (i, i + hd/2) of one head; gate and up of 8 FFN features).  rs: the row's
// 1 / rms times the operand scales.  The caller has checked frag < n_groups; lanes g >= 2 only lend values.
// v: the first members (fragment rows 4g .. 4g+3, g < 2), x2: their partners (rows 8 + 4g ..), both already scaled
template <typename T, int EPI>
__device__ __forceinline__ void epi_paired_vals(const GemmArgs &a, int frag, int m, int M, int g, const float (&v)[4],
                                                const float (&x2)[4]) {
  if (m < M && g < 2) {
    if constexpr (EPI == EPI_GATEUP) {
      float o[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] = silu<T>(v[r]) * x2[r];
      store4((T *)a.act + act_offset<T>(m, frag * 8 + 4 * g, a.Mcap), o[0], o[1], o[2], o[3]);   // 4 features, one chunk
    } else {
      const int half = a.hd / 2, fph = a.hd / 16;    // fragments per head
      const int hh = frag / fph, sub = frag - hh * fph;                 // head over [q heads | k heads | v heads]
      const int kind = hh < a.H ? 0 : (hh < a.H + a.Hkv ? 1 : 2);
      const int head = kind == 0 ? hh : (kind == 1 ? hh - a.H : hh - a.H - a.Hkv);
      const int i0 = sub * 8 + 4 * g;                // dims i0 .. i0+3 and their partners i0 + half ..
      if (kind < 2) {                                // rotary embedding on q and k
        const int pos = (a.n_dev ? *a.n_dev - 1 : a.P) + block_col(m, a.C, a.shared0);
        const float *cs = a.rope_cos + (size_t)pos * half + i0;
        const float *sn = a.rope_sin + (size_t)pos * half + i0;
        float lo[4], hi[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          lo[r] = v[r] * cs[r] - x2[r] * sn[r];
          hi[r] = x2[r] * cs[r] + v[r] * sn[r];
        }
        if (kind == 0) {
          T *dst = (T *)a.q + ((size_t)head * a.Mcap + m) * a.hd + i0;
          store4(dst, lo[0], lo[1], lo[2], lo[3]);
          store4(dst + half, hi[0], hi[1], hi[2], hi[3]);
        } else {                                     // keys: tiles of 32 block positions in operand order
          T *kh = (T *)a.kscr + (size_t)head * a.kv_rows * a.hd;
          store4(kh + k_offset(m, i0, a.hd, (int)sizeof(T)), lo[0], lo[1], lo[2], lo[3]);
          store4(kh + k_offset(m, i0 + half, a.hd, (int)sizeof(T)), hi[0], hi[1], hi[2], hi[3]);
        }
      } else {                                       // values: the transposed tiles
        T *vh = (T *)a.vscr + (size_t)head * a.kv_rows * a.hd;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          vh[v_offset(m, i0 + r, a.hd, (int)sizeof(T))] = from_f32<T>(v[r]);
          vh[v_offset(m, i0 + half + r, a.hd, (int)sizeof(T))] = from_f32<T>(x2[r]);
        }
      }
    }
  }
}

template <typename T, int EPI>
__device__ __forceinline__ void epi_paired(const GemmArgs &a, int frag, int m, int M, int g, float rs, const f32x4 &sum) {
  float v[4], x2[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) { v[r] = sum[r] * rs; x2[r] = other_half(v[r]); }
  epi_paired_vals<T, EPI>(a, frag, m, M, g, v, x2);
}

// residual: split ks stores its fp32 partial of output features n0 + 4g .. +4 of block row m
__device__ __forceinline__ void epi_residual(const GemmArgs &a, int ks, int m, int n0, int g, const f32x4 &sum) {
  float *dst = a.hpart + ((size_t)ks * a.Mcap + m) * a.N;
  *reinterpret_cast<float4 *>(dst + n0 + 4 * g) =
      float4{sum[0] * a.out_scale, sum[1] * a.out_scale, sum[2] * a.out_scale, sum[3] * a.out_scale};
}

// unembedding: optional logits, and the best (value, id) of block row m over the FN fragments of `group`
// (vocabulary rows nbase[f] ..): ascending ids, so the first maximum stays
template <int FN>
__device__ __forceinline__ void epi_unembed(const GemmArgs &a, int group, int m, bool live, int g, float rs,
                                            const int (&nbase)[FN], const f32x4 (&sum)[FN]) {
  float bv = kNegBig;
  int bi = 0x7fffffff;
#pragma unroll
  for (int f = 0; f < FN; ++f)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = sum[f][r] * rs;
      const int n = nbase[f] + 4 * g + r;
      if (a.logits && live) a.logits[(size_t)m * a.N + n] = v;
      if (v > bv) { bv = v; bi = n; }
    }
#pragma unroll
  for (int off = 16; off < 64; off <<= 1) {
    const float ov = __shfl_xor(bv, off);
    const int oi = __shfl_xor(bi, off);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if (live && g == 0) {
    a.pmax_val[(size_t)group * a.Mcap + m] = bv;
    a.pmax_idx[(size_t)group * a.Mcap + m] = bi;
  }
}

template <typename T, int EPI, int FM, int WN, int WK, int RING, int FN>
__global__ __launch_bounds__(64 * WN * WK) void gemm_skinny_kernel(const GemmArgs a) {
  constexpr int XD = FM > 4 ? 1 : 2;         // X register stages (chunks fetched ahead); one when the tile is 128 rows
  static_assert(WN * WK == 4 || WN * WK == 8, "four or eight waves per workgroup");
  constexpr bool PAIRED = EPI == EPI_QKV || EPI == EPI_GATEUP;   // fragments that hold both halves of 8 output pairs
  static_assert(PAIRED ? WN == 1 : FN == 2, "paired epilogues: one set of FN fragments per workgroup, waves split K");
  constexpr int NT = 64 * WN * WK;           // threads per workgroup
  constexpr int KC = KChunk<T>::value;
  constexpr int SPC = KC / 32;               // steps per chunk
  constexpr int SPW = SPC / WK;              // steps per wave per chunk
  constexpr int PAD = 16 / (int)sizeof(T);
  constexpr int LDX = KC + PAD;              // LDS row stride in elements
  constexpr int ROWS = 16 * FM;
  constexpr int PIECES = ROWS * KC * (int)sizeof(T) / 16 / NT;    // 16-byte pieces per thread per chunk
  constexpr int PPR = KC * (int)sizeof(T) / 16;                   // pieces per row
  constexpr int UC0 = (RING % SPW == 0) ? RING / SPW : 1;
  constexpr int UC = UC0 % 2 == 0 ? UC0 : 2 * UC0;                // chunks per unrolled iteration (even: two X stages)
  static_assert((UC * SPW) % RING == 0, "ring slots must be static after unrolling");
  static_assert(PIECES >= 1, "chunk too small for the workgroup");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *xs = reinterpret_cast<T *>(smem);       // [2][ROWS][LDX]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int li = lane & 15, g = lane >> 4;
  const int wn = wave % WN, wk = wave / WN;
  const int K = a.K, M = a.M;
  // When X holds h * gain, the RMSNorm kernel left the sums of squares of every row's segments
  // (kNormSegs floats per row, unused ones zero); the epilogue turns them into 1 / rms.
  static_assert(kNormSegs == 4, "one float4 per row");
  auto row_ss_load = [&](int m) {                        // (f32x4, not float4: arrays of the HIP struct go to scratch)
    if (!a.row_ss) return f32x4{0.f, 0.f, 0.f, 0.f};
    return *reinterpret_cast<const f32x4 *>(a.row_ss + (size_t)(m < a.Mcap ? m : a.Mcap - 1) * kNormSegs);
  };
  // ... times the factor that undoes the power-of-two scales of the stored operands (1 for fp32 models)
  auto row_scale = [&](const f32x4 &ss) {
    return (a.row_ss ? 1.0f / sqrtf((((ss[0] + ss[1]) + ss[2]) + ss[3]) / (float)K + a.ss_eps) : 1.0f) * a.out_scale;
  };
  const int n_groups = a.n_groups;
  int group = blockIdx.x * WN + wn;
  const bool group_live = group < n_groups;
  if (!group_live) group = n_groups - 1;     // idle waves still help staging X and hit every barrier

  // ---- the 16-row fragments of W this wave owns (W is stored in operand order: see tile_weights) ----
  // Residual and unembedding: group = 2 consecutive fragments.  q/k/v and gate/up: n_groups counts
  // fragments, the workgroup owns FN consecutive ones, and each fragment holds rows 0..7 = the first
  // members and rows 8..15 = the second members of 8 output pairs (rotary pairs (i, i + hd/2) of one
  // head; gate and up of 8 FFN features), so one accumulator has both halves of every pair it needs.
  const int n_steps = K / 32;
  const T *wblk[FN];                         // this lane's slice of the fragment's first 32-step block
  int nbase[FN];                             // first output feature (residual, unembedding) / fragment index (paired)
  bool frag_live[FN];
#pragma unroll
  for (int f = 0; f < FN; ++f) {
    int frag = PAIRED ? blockIdx.x * FN + f : group * FN + f;
    frag_live[f] = PAIRED ? frag < n_groups : group_live;
    if (PAIRED && !frag_live[f]) frag = n_groups - 1;      // the last workgroup repeats a fragment it does not store
    nbase[f] = PAIRED ? frag : frag * 16;
    wblk[f] = tiled_block((const T *)a.W0, frag, n_steps, lane);
  }

  // ---- this workgroup's range of chunks -----------------------------------------------------------
  const int n_chunks = (n_steps + SPC - 1) / SPC;
  const int KS = gridDim.y, ks = blockIdx.y;
  const int c0 = (int)(((long)n_chunks * ks) / KS), c1 = (int)(((long)n_chunks * (ks + 1)) / KS);

  for (int m0 = 0; m0 < M; m0 += ROWS) {
    // X staging: piece p = tid + NT*i covers row p / PPR (= tid / PPR + i * NT / PPR), 16 bytes at column
    // piece p % PPR.
    static_assert(NT % PPR == 0, "row stride of the staging pieces must be constant");
    constexpr int RPI = NT / PPR;                          // rows between a thread's consecutive pieces
    // (rows past the block's last one repeat it: the same cache lines as the threads that stage that row, so they
    // cost no further traffic from L2; what lands in their LDS rows is never stored)
    const T *xsrc0 = (const T *)a.X + (tid % PPR) * PAD;                 // chunk c adds c * Mcap * KC, piece i its row * KC
    const int xrow0 = m0 + tid / PPR, xrow_last = M - 1;
    const int xdst0 = (tid / PPR) * LDX + (tid % PPR) * PAD;
    // X is fetched XD chunks ahead into register stages (an L2 hit takes longer than one chunk of
    // MFMA work), then written to the LDS buffer of its chunk's parity.
    u32x4 stage[XD][PIECES];
    auto stage_load = [&](u32x4 (&st)[PIECES], int c) {
      const int cl = c < n_chunks ? c : n_chunks - 1;      // activation buffers are padded to whole chunks
#pragma unroll
      for (int i = 0; i < PIECES; ++i)
        st[i] = *reinterpret_cast<const u32x4 *>(xsrc0 + ((size_t)cl * a.Mcap + min(xrow0 + i * RPI, xrow_last)) * KC);
    };
    auto stage_store = [&](const u32x4 (&st)[PIECES], int buf) {
#pragma unroll
      for (int i = 0; i < PIECES; ++i) *reinterpret_cast<u32x4 *>(xs + (size_t)buf * ROWS * LDX + xdst0 + i * RPI * LDX) = st[i];
    };

    f32x4 acc[FN][FM];
#pragma unroll
    for (int f = 0; f < FN; ++f)
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) acc[f][fm] = f32x4{0.f, 0.f, 0.f, 0.f};

    // wave-step t is global step (c0 + t/SPW)*SPC + wk + WK*(t % SPW); steps outside the matrix are
    // clamped into it (loaded, never multiplied)
    Frag<T> ring[RING][FN];
    auto load_w = [&](Frag<T> (&slot)[FN], int t) {
      int s = c0 * SPC + (t / SPW) * SPC + wk + WK * (t % SPW);   // t >= 0 here
      s = s < n_steps ? s : n_steps - 1;
#pragma unroll
      for (int f = 0; f < FN; ++f) slot[f] = load_frag_stream(wblk[f] + (size_t)s * 512);
    };

    // The loop has no separate prologue: it starts one unrolled group early (ci = -UC) with the
    // multiplications switched off, so the loads that fill the ring and the X stages are issued by the
    // very instructions that refill them later.  Every trip then enters with the same set of loads
    // outstanding, in the same order, and the compiler's s_waitcnt vmcnt(n) before each use is exact
    // (with a prologue in another order it merged the two states and waited for nearly everything).
    const int n_iter = (c1 - c0 + UC - 1) / UC * UC;       // whole unrolled groups; extra chunks only load
    for (int ci = -UC; ci < n_iter; ci += UC) {
      const bool warm = ci < 0;
#pragma unroll
      for (int cc = 0; cc < UC; ++cc) {
        const int ch = c0 + ci + cc;
        const int buf = cc & 1;                          // UC is even
        if (!warm) stage_store(stage[cc % XD], buf);
        __syncthreads();
        stage_load(stage[cc % XD], max(ch + XD, 0));
        const T *xb = xs + (size_t)buf * ROWS * LDX + li * LDX + g * 8;
        // X fragments are read from LDS one step ahead of the MFMAs that use them (unconditionally:
        // during the warm-up group the buffer holds nothing yet and the values go unused)
        constexpr bool XPRE = FM <= 4;                     // 128-row tiles have no registers to spare
        Frag<T> xf[XPRE ? 2 : 1][FM];
        if constexpr (XPRE) {
#pragma unroll
          for (int fm = 0; fm < FM; ++fm) xf[0][fm] = load_frag(xb + fm * 16 * LDX + wk * 32);
        }
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
          const int slot = (cc * SPW + i) % RING;        // constant after unrolling
          const int ls = wk + WK * i;                    // step inside the chunk
          if constexpr (XPRE) {
            if (i + 1 < SPW) {
#pragma unroll
              for (int fm = 0; fm < FM; ++fm) xf[(i + 1) & 1][fm] = load_frag(xb + fm * 16 * LDX + (ls + WK) * 32);
            }
          } else {
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) xf[0][fm] = load_frag(xb + fm * 16 * LDX + ls * 32);
          }
          if (!warm && ch < c1 && ch * SPC + ls < n_steps) {      // uniform per wave; no global load inside
#pragma unroll
            for (int f = 0; f < FN; ++f)
#pragma unroll
              for (int fm = 0; fm < FM; ++fm) mma(acc[f][fm], ring[slot][f], xf[XPRE ? (i & 1) : 0][fm]);
          }
          load_w(ring[slot], max((ci + cc) * SPW + i + RING, 0));
        }
      }
    }
    __syncthreads();                                     // everyone is done with xs
    // 1 / rms of the pass's block rows, one per thread, left in LDS for the epilogues (fetched only now:
    // the main loop keeps every vector register it can get)
    float *rs_lds = reinterpret_cast<float *>(smem);     // [ROWS]; the hand-over buffers start behind it
    if (tid < ROWS) rs_lds[tid] = row_scale(row_ss_load(m0 + tid));

    // ---- q/k/v and gate/up: every wave hands its partial fragments over through LDS; wave wk then
    //      sums items wk, wk + WK, ... of the FN x FM accumulator fragments (waves in the order 0 .. WK-1)
    //      and runs their epilogue, one item at a time ------------------------------------------------------
    if constexpr (PAIRED) {
      // at most 4 column blocks of every fragment per round, so that the hand-over fits the LDS; the last
      // round of a tile of 5, 6 or 7 column blocks is shorter
      constexpr int FMR = FM < 4 ? FM : 4, ROUNDS = (FM + FMR - 1) / FMR;
      constexpr int IPW = (FN * FMR + WK - 1) / WK;        // items per round and wave, at most
      f32x4 *red = reinterpret_cast<f32x4 *>(smem + ROWS * sizeof(float));   // [WK][FN * cnt][64] lanes x 4 registers
#pragma unroll
      for (int rd = 0; rd < ROUNDS; ++rd) {
      const int cnt = (rd + 1) * FMR <= FM ? FMR : FM - rd * FMR;    // column blocks of this round (constant after unrolling)
      const int items = FN * cnt;                          // item idx = f * cnt + fr covers column block rd * FMR + fr
      if (rd > 0) __syncthreads();                       // the previous round's items were all read
#pragma unroll
      for (int f = 0; f < FN; ++f)
#pragma unroll
        for (int fr = 0; fr < FMR; ++fr)
          if (fr < cnt) red[((size_t)wk * items + f * cnt + fr) * 64 + lane] = acc[f][rd * FMR + (fr < cnt ? fr : 0)];
      __syncthreads();                                   // also: rs_lds is complete
      // unrolled where the items are short (SwiGLU) or few: the q/k/v item (rotary tables, three kinds of
      // stores) times 8 would not fit the registers
      constexpr int UNR = (EPI == EPI_GATEUP || IPW <= 3) ? IPW : 1;
#pragma unroll UNR
      for (int j = 0; j < IPW; ++j) {
        const int idx = wk + WK * j;
        if (idx >= items) break;
        const int f = idx / cnt;
        const int fm = rd * FMR + (idx - f * cnt);
        const int m = m0 + fm * 16 + li;
        const float rs = rs_lds[fm * 16 + li];
        const int frag = blockIdx.x * FN + f;              // fragment index over the whole matrix
        f32x4 sum = red[(size_t)idx * 64 + lane];
#pragma unroll
        for (int o = 1; o < WK; ++o) sum += red[((size_t)o * items + idx) * 64 + lane];
        if (frag < n_groups) epi_paired<T, EPI>(a, frag, m, M, g, rs, sum);   // (uniform per wave)
      }
      }
    }

    // ---- sum the WK waves that share a wn: wave (wn, 0) adds (wn, 1) .. (wn, WK-1) in that order ---
    if constexpr (!PAIRED && WK == 1) __syncthreads();   // rs_lds is complete
    if constexpr (!PAIRED && WK > 1) {
      float *red = reinterpret_cast<float *>(smem) + ROWS;   // [(WK-1)][WN][FN*FM*4][64]
      if (wk > 0) {
        float *dst = red + (size_t)((wk - 1) * WN + wn) * (FN * FM * 4 * 64);
#pragma unroll
        for (int f = 0; f < FN; ++f)
#pragma unroll
          for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[((f * FM + fm) * 4 + r) * 64 + lane] = acc[f][fm][r];
      }
      __syncthreads();
      if (wk == 0) {
        for (int o = 1; o < WK; ++o) {
          const float *src = red + (size_t)((o - 1) * WN + wn) * (FN * FM * 4 * 64);
#pragma unroll
          for (int f = 0; f < FN; ++f)
#pragma unroll
            for (int fm = 0; fm < FM; ++fm)
#pragma unroll
              for (int r = 0; r < 4; ++r) acc[f][fm][r] += src[((f * FM + fm) * 4 + r) * 64 + lane];
        }
      }
    }

    // ---- epilogue, waves (wn, 0): lane holds, per group f and column block fm, column
    //      m = m0 + fm*16 + li and output features nbase[f] + 4g .. +4 -----------------------------------
    if (!PAIRED && wk == 0 && group_live) {
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) {
        const int m = m0 + fm * 16 + li;
        const bool live = m < M;
        if constexpr (EPI == EPI_RESIDUAL) {
          if (live) {
#pragma unroll
            for (int f = 0; f < FN; ++f) epi_residual(a, ks, m, nbase[f], g, acc[f][fm]);
          }
        } else {   // EPI_UNEMBED
          f32x4 sums[FN];
#pragma unroll
          for (int f = 0; f < FN; ++f) sums[f] = acc[f][fm];
          epi_unembed<FN>(a, group, m, live, g, rs_lds[fm * 16 + li], nbase, sums);
        }
      }
    }
    __syncthreads();                                       // LDS is reused by the next column block
  }
}


// ---------------------------------------------------------------------------------------------
// Wide blocks (more than 128 rows; 16-bit types): one pass over W for up to 16*FM = 288 block rows.
// Section 3's cost model has the call leave the memory-bound regime as k*(w+1) grows; with 128-row
// tiles the skinny kernel re-streamed all of W for every further 128 rows, which put that transition
// far below the chip's ops-to-bytes ratio.  Here a workgroup owns 2 FN fragments of W (64 or 128 rows) and
// all row blocks of the tile; its four waves are laid out 2 x 2: a wave takes FN of the fragments and half
// of the row blocks (FN * FM / 2 <= 36 accumulator fragments), so a W fragment is loaded once from HBM and
// meets every block row.  X is staged through LDS in slices of 64 contraction elements (two MFMA steps),
// double buffered; a wave reads only its half of the rows from LDS (with the four waves side by side along
// W every wave read all of X, and the LDS reads cost as much as the MFMAs: 10-20 % slower at 130-290 rows).
// W goes from global memory straight into registers, 4 steps ahead, as in the skinny kernel; the two waves
// that share a fragment both load it (the second request is served by the L2).  No hand-over between waves:
// each wave finishes its own accumulators.  gridDim.y splits the contraction (residual only).
// ---------------------------------------------------------------------------------------------
template <typename T, int EPI, int FM, int FN, bool TILED>
__global__ __launch_bounds__(256) void gemm_wide_kernel(const GemmArgs a, int MT) {
  static_assert(sizeof(T) == 2, "16-bit operands only");
  constexpr bool PAIRED = EPI == EPI_QKV || EPI == EPI_GATEUP;
  static_assert(PAIRED || FN % 2 == 0, "unembedding partials are indexed by pairs of fragments");
  static_assert(FM % 2 == 0, "the waves are laid out 2 x 2 over (row blocks, fragments)");
  constexpr int FMW = FM / 2;                // row blocks per wave
  constexpr int KC = KChunk<T>::value;       // chunk of the activation layout (256)
  constexpr int KW = 64;                     // contraction elements staged per slice: two steps
  constexpr int SPS = KW / 32;               // steps per slice
  constexpr int LDX = KW + 8;                // LDS row stride in elements (16 bytes of padding)
  constexpr int ROWS = 16 * FM;
  constexpr int PPR = KW / 8;                // 16-byte pieces per row
  constexpr int PIECES = (ROWS * PPR + 255) / 256;
  constexpr int RING = 4;                    // W steps in flight per wave (two slices)

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *xs = reinterpret_cast<T *>(smem);       // [2][ROWS][LDX]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int li = lane & 15, g = lane >> 4;
  const int wn = wave & 1, wm = wave >> 1;   // this wave: fragments wn * FN .. of the workgroup's 2 FN, row blocks wm * FMW ..
  const int K = a.K, M = a.M;
  const int n_frags = a.n_groups;            // 16-row fragments of W (the launcher fills it)
  const int n_steps = K / 32;
  const int n_slices = (n_steps + SPS - 1) / SPS;
  const int KS = gridDim.y, ks = blockIdx.y;
  // Workgroup -> (rows of W, row tile).  With several row tiles (TILED: prefill pieces of more than 288 rows) the
  // MT workgroups that share rows of W take consecutive slots of one XCD (workgroup b runs on XCD b % 8), so they
  // run at about the same time on one L2 and the rows come from HBM once; W is then read with ordinary loads
  // (a non-temporal line may be gone before the next workgroup asks for it).
  const int nb = TILED ? (blockIdx.x / 8 / MT) * 8 + blockIdx.x % 8 : blockIdx.x;
  const int m0 = TILED ? (blockIdx.x / 8 % MT) * (16 * FM) : 0;
  if (TILED && nb * 2 * FN >= n_frags) return;               // padding of the last row of 8
  const int c0 = (int)(((long)n_slices * ks) / KS), c1 = (int)(((long)n_slices * (ks + 1)) / KS);

  const T *wblk[FN];
  int fragi[FN];
  bool frag_live[FN];
#pragma unroll
  for (int f = 0; f < FN; ++f) {
    int frag = (nb * 2 + wn) * FN + f;
    frag_live[f] = frag < n_frags;
    if (!frag_live[f]) frag = n_frags - 1;   // repeats a fragment it does not store
    fragi[f] = frag;
    wblk[f] = tiled_block((const T *)a.W0, frag, n_steps, lane);
  }

  static_assert(kNormSegs == 4, "one float4 per row");
  auto row_scale = [&](int m) {
    float r = 1.0f;
    if (a.row_ss) {
      const f32x4 ss = *reinterpret_cast<const f32x4 *>(a.row_ss + (size_t)(m < a.Mcap ? m : a.Mcap - 1) * kNormSegs);
      r = 1.0f / sqrtf((((ss[0] + ss[1]) + ss[2]) + ss[3]) / (float)K + a.ss_eps);
    }
    return r * a.out_scale;
  };

  {
    // X staging: piece p = tid + 256 i is row p / PPR, 16 bytes at column piece p % PPR of the slice; pieces
    // past the tile repeat its last row, rows past the block's last row repeat that row (the same cache lines
    // as the threads that stage it: no further traffic from L2; never stored)
    const T *xsrc[PIECES];
    int xdst[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int p = tid + 256 * i;
      const int row = min(p / PPR, ROWS - 1), col = p % PPR;
      xsrc[i] = (const T *)a.X + (size_t)min(m0 + row, M - 1) * KC + col * 8;
      xdst[i] = row * LDX + col * 8;
    }
    u32x4 stage[2][PIECES];
    auto stage_load = [&](u32x4 (&st)[PIECES], int c) {     // slice c of the matrix (clamped into it)
      const int cl = min(c, n_slices - 1);
      const int k0 = cl * KW;
      const size_t off = (size_t)(k0 / KC) * a.Mcap * KC + k0 % KC;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) st[i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + off);
    };
    auto stage_store = [&](const u32x4 (&st)[PIECES], int buf) {
#pragma unroll
      for (int i = 0; i < PIECES; ++i) *reinterpret_cast<u32x4 *>(xs + (size_t)buf * ROWS * LDX + xdst[i]) = st[i];
    };

    f32x4 acc[FN][FMW];
#pragma unroll
    for (int f = 0; f < FN; ++f)
#pragma unroll
      for (int fm = 0; fm < FMW; ++fm) acc[f][fm] = f32x4{0.f, 0.f, 0.f, 0.f};

    Frag<T> ring[RING][FN];
    auto load_w = [&](Frag<T> (&slot)[FN], int t) {         // wave-step t >= 0 is global step c0 * SPS + t (clamped)
      const int st = min(c0 * SPS + t, n_steps - 1);
#pragma unroll
      for (int f = 0; f < FN; ++f) slot[f] = TILED ? load_frag(wblk[f] + (size_t)st * 512) : load_frag_stream(wblk[f] + (size_t)st * 512);
    };

    // As in the skinny kernel the loop starts one unrolled group (two slices) early with the multiplications
    // off, so that every trip enters with the same loads outstanding in the same order.
    const int n_iter = (c1 - c0 + 1) / 2 * 2;
    for (int ci = -2; ci < n_iter; ci += 2) {
      const bool warm = ci < 0;
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const int sl = c0 + ci + cc;                         // slice of this half trip
        if (!warm) stage_store(stage[cc], cc);
        __syncthreads();
        const T *xb = xs + (size_t)cc * ROWS * LDX + (wm * FMW * 16 + li) * LDX + g * 8;
        // All X fragments of a step are read from LDS in one go: those of the slice's first step right behind
        // the barrier (the global loads of the next slices are issued while they are on their way), those of
        // the second step before the first step's MFMAs.  The scheduling barriers keep that order (left alone,
        // the compiler fetched one fragment at a time and waited for each between the MFMAs).
        const bool live = !warm && sl < c1;                  // uniform per workgroup
        Frag<T> xf[SPS][FMW];
#pragma unroll
        for (int fm = 0; fm < FMW; ++fm) xf[0][fm] = load_frag(xb + fm * 16 * LDX);
        __builtin_amdgcn_sched_barrier(0);
        stage_load(stage[cc], max(sl + 2, c0));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < SPS; ++i) {
          const int slot = cc * SPS + i;
          if (i + 1 < SPS) {
#pragma unroll
            for (int fm = 0; fm < FMW; ++fm) xf[i + 1][fm] = load_frag(xb + fm * 16 * LDX + (i + 1) * 32);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (live && sl * SPS + i < n_steps) {
#pragma unroll
            for (int fm = 0; fm < FMW; ++fm)
#pragma unroll
              for (int f = 0; f < FN; ++f) mma(acc[f][fm], ring[slot][f], xf[i][fm]);
          }
          __builtin_amdgcn_sched_barrier(0);
          load_w(ring[slot], max((ci + cc) * SPS + i + RING, 0));
        }
      }
    }
    __syncthreads();                                         // everyone is done with xs
    float *rs_lds = reinterpret_cast<float *>(smem);         // [ROWS] 1 / rms (times the operand scales) of the tile's rows
    for (int r = tid; r < ROWS; r += 256) rs_lds[r] = row_scale(m0 + r);
    __syncthreads();

    const int row0 = wm * FMW * 16 + li;
    if constexpr (EPI == EPI_QKV) {
      // q/k/v: the accumulators leave the registers through LDS (every wave its own region, behind the row scales)
      // and the rotary epilogue takes them back one item at a time.  Unrolled over the registers, the FN * FM / 2
      // items' table entries and addresses were all live at once and the register allocator answered by storing
      // every accumulator to scratch memory right where the main loop produces it.
      f32x4 *dump = reinterpret_cast<f32x4 *>(smem + (ROWS * sizeof(float) + 15) / 16 * 16) + (size_t)wave * (FN * FMW * 64);
#pragma unroll
      for (int f = 0; f < FN; ++f)
#pragma unroll
        for (int fm = 0; fm < FMW; ++fm) dump[(f * FMW + fm) * 64 + lane] = acc[f][fm];
#pragma unroll 2
      for (int idx = 0; idx < FN * FMW; ++idx) {
        const int f = idx / FMW, fm = idx - f * FMW;
        const int frag = (nb * 2 + wn) * FN + f;
        const int row = row0 + fm * 16;
        if (frag < n_frags) epi_paired<T, EPI>(a, frag, m0 + row, M, g, rs_lds[row], dump[idx * 64 + lane]);   // uniform per wave
      }
    } else {
#pragma unroll
    for (int fm = 0; fm < FMW; ++fm) {
      const int row = row0 + fm * 16;                        // row of the tile
      const int m = m0 + row;
      const bool live = m < M;
      if constexpr (PAIRED) {
        const float rs = rs_lds[row];
#pragma unroll
        for (int f = 0; f < FN; ++f)
          if (frag_live[f]) epi_paired<T, EPI>(a, fragi[f], m, M, g, rs, acc[f][fm]);     // uniform per wave
      } else if constexpr (EPI == EPI_RESIDUAL) {
#pragma unroll
        for (int f = 0; f < FN; ++f)
          if (live && frag_live[f]) epi_residual(a, ks, m, fragi[f] * 16, g, acc[f][fm]);
      } else {
#pragma unroll
        for (int f = 0; f < FN; f += 2)
          if (frag_live[f]) {                                // a pair of fragments is live or not as a whole (N % 32 == 0)
            const int nbase[2] = {fragi[f] * 16, fragi[f + 1] * 16};
            const f32x4 sums[2] = {acc[f][fm], acc[f + 1][fm]};
            epi_unembed<2>(a, fragi[f] / 2, m, live, g, rs_lds[row], nbase, sums);
          }
      }
    }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The wide kernel on the 32x32x16 MFMA, for tiles whose row blocks come in pairs (FM a multiple of 4, an even
// number of fragments).  Same workgroup, staging and ring as above; what changes is the tile one instruction
// covers: 32 rows of W (two neighbouring fragments) times 32 block rows over 16 contraction elements.  An
// operand register then meets twice as many multiply-adds, so the kernel reads half the LDS bytes and issues half
// the W loads per flop, and the instruction itself runs closer to the matrix cores' rate on this part (a loop of
// nothing but MFMAs on all CUs: 2.1-2.2 PFLOP/s with 32x32x16 against 1.45-1.55 with 16x16x32).
// Operand lanes: lane = 32 h + r takes row r of the 32 and contraction elements 8 h .. 8 h + 7 of the 16.  The
// weights stay in their 16 x 32 blocks: for the q-th half of a step, lane (r, h) reads the 16 bytes that lane
// (16 (2 q + h) + r % 16) of fragment r / 16 owns in the block (each load still covers whole 128-byte lines: 512
// contiguous bytes in each of the two blocks).  Accumulator register 4 j + i of lane (r, h) is row
// 8 j + 4 h + i of the 32 W rows at block row r: fragment j / 2, and inside it what the 16x16 layout keeps
// in lane group 2 (j % 2) + h, so the epilogues above are called with that group.  Both halves of an output
// pair now sit in one lane (registers of j and j + 1).  The unembedding stays on gemm_wide_kernel.
// ---------------------------------------------------------------------------------------------
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename T, int EPI, int FM, int FN, bool TILED>
__global__ __launch_bounds__(256) void gemm_wide32_kernel(const GemmArgs a, int MT) {
  static_assert(sizeof(T) == 2, "16-bit operands only");
  constexpr bool PAIRED = EPI == EPI_QKV || EPI == EPI_GATEUP;
  static_assert(FN % 2 == 0 && FM % 4 == 0, "pairs of fragments, pairs of row blocks per wave");
  static_assert(EPI != EPI_UNEMBED, "the unembedding stays on gemm_wide_kernel");
  constexpr int FNP = FN / 2;                // pairs of fragments (32 rows of W) per wave
  constexpr int FMB = FM / 4;                // 32-row blocks of the tile per wave (the waves are laid out 2 x 2)
  constexpr int KC = KChunk<T>::value;       // chunk of the activation layout (256)
  constexpr int KW = 64;                     // contraction elements staged per slice: two steps
  constexpr int SPS = KW / 32;               // steps per slice
  constexpr int LDX = KW + 8;                // LDS row stride in elements (16 bytes of padding)
  constexpr int ROWS = 16 * FM;
  constexpr int PPR = KW / 8;                // 16-byte pieces per row
  constexpr int PIECES = (ROWS * PPR + 255) / 256;
  constexpr int RING = 4;                    // W steps in flight per wave (two slices)

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *xs = reinterpret_cast<T *>(smem);       // [2][ROWS][LDX]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r32 = lane & 31, h = lane >> 5;
  const int wn = wave & 1, wm = wave >> 1;   // this wave: fragments wn * FN .. of the workgroup's 2 FN, 32-row blocks wm * FMB ..
  const int K = a.K, M = a.M;
  const int n_frags = a.n_groups;            // 16-row fragments of W, an even number (the launcher checks)
  const int n_steps = K / 32;
  const int n_slices = (n_steps + SPS - 1) / SPS;
  const int KS = gridDim.y, ks = blockIdx.y;
  // workgroup -> (rows of W, row tile) as in gemm_wide_kernel
  const int nb = TILED ? (blockIdx.x / 8 / MT) * 8 + blockIdx.x % 8 : blockIdx.x;
  const int m0 = TILED ? (blockIdx.x / 8 % MT) * (16 * FM) : 0;
  if (TILED && nb * 2 * FN >= n_frags) return;               // padding of the last row of 8
  const int c0 = (int)(((long)n_slices * ks) / KS), c1 = (int)(((long)n_slices * (ks + 1)) / KS);

  const T *wptr[FNP];                        // this lane's 16 bytes of the pair's first step, first half
  int frag0[FNP];                            // first fragment of the pair
  bool pair_live[FNP];
#pragma unroll
  for (int p = 0; p < FNP; ++p) {
    int f0 = (nb * 2 + wn) * FN + 2 * p;
    pair_live[p] = f0 < n_frags;
    if (!pair_live[p]) f0 = n_frags - 2;     // repeats a pair it does not store
    frag0[p] = f0;
    wptr[p] = tiled_block((const T *)a.W0, f0 + (r32 >> 4), n_steps, 16 * h + (r32 & 15));
  }

  static_assert(kNormSegs == 4, "one float4 per row");
  auto row_scale = [&](int m) {
    float r = 1.0f;
    if (a.row_ss) {
      const f32x4 ss = *reinterpret_cast<const f32x4 *>(a.row_ss + (size_t)(m < a.Mcap ? m : a.Mcap - 1) * kNormSegs);
      r = 1.0f / sqrtf((((ss[0] + ss[1]) + ss[2]) + ss[3]) / (float)K + a.ss_eps);
    }
    return r * a.out_scale;
  };

  // X staging as in gemm_wide_kernel
  const T *xsrc[PIECES];
  int xdst[PIECES];
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const int p = tid + 256 * i;
    const int row = min(p / PPR, ROWS - 1), col = p % PPR;
    xsrc[i] = (const T *)a.X + (size_t)min(m0 + row, M - 1) * KC + col * 8;
    xdst[i] = row * LDX + col * 8;
  }
  u32x4 stage[2][PIECES];
  auto stage_load = [&](u32x4 (&st)[PIECES], int c) {       // slice c of the matrix (clamped into it)
    const int cl = min(c, n_slices - 1);
    const int k0 = cl * KW;
    const size_t off = (size_t)(k0 / KC) * a.Mcap * KC + k0 % KC;
#pragma unroll
    for (int i = 0; i < PIECES; ++i) st[i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + off);
  };
  auto stage_store = [&](const u32x4 (&st)[PIECES], int buf) {
#pragma unroll
    for (int i = 0; i < PIECES; ++i) *reinterpret_cast<u32x4 *>(xs + (size_t)buf * ROWS * LDX + xdst[i]) = st[i];
  };

  f32x16 acc[FNP][FMB];
#pragma unroll
  for (int p = 0; p < FNP; ++p)
#pragma unroll
    for (int b = 0; b < FMB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[p][b][r] = 0.f;
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < PIECES; ++i) stage[c][i] = u32x4{0u, 0u, 0u, 0u};

  Frag<T> ring[RING][FN];                                   // [2 p + q]: pair p, half q of the step
  auto load_w = [&](Frag<T> (&slot)[FN], int t) {           // wave-step t >= 0 is global step c0 * SPS + t (clamped)
    const int st = min(c0 * SPS + t, n_steps - 1);
#pragma unroll
    for (int p = 0; p < FNP; ++p)
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const T *src = wptr[p] + (size_t)st * 512 + q * 256;
        slot[2 * p + q] = TILED ? load_frag(src) : load_frag_stream(src);
      }
  };

  // One slice = two steps = two blocks of MFMAs, and between them the slice's only barrier.  The memory
  // instructions ride in the shadow of the MFMAs (one wave per SIMD: whatever is issued while no MFMA is in
  // flight leaves the matrix core idle; with the phases one after the other it was busy 38 % of the time):
  //   first block (step 0 of slice s):  LDS reads of step 1, global loads of slice s + 2, LDS writes of slice s + 1
  //                                     into the other buffer (its last readers passed the previous barrier)
  //   barrier; LDS reads of step 0 of slice s + 1 (they land under the second block)
  //   second block (step 1 of slice s): the W loads that refill the ring
  // The groups below ask the scheduler for that order.
  constexpr int NM = 2 * FMB * FNP;                         // MFMAs per step
  constexpr int MEM_A = 2 * FMB + 2 * PIECES;               // memory instructions of the first block
  constexpr int PER_A = (MEM_A + NM - 1) / NM;
  const int rowoff = (wm * FMB * 32 + r32) * LDX + h * 8;
  Frag<T> xf[SPS][2 * FMB];                                 // [2 b + q]: 32-row block b, half q of the step
#pragma unroll
  for (int i = 0; i < SPS; ++i)
#pragma unroll
    for (int e = 0; e < 2 * FMB; ++e) xf[i][e].v = half8{0, 0, 0, 0, 0, 0, 0, 0};
  auto half_trip = [&](auto cc_tag, auto live_tag, int sl, int t0) {
    constexpr int cc = decltype(cc_tag)::value;
    constexpr bool live = decltype(live_tag)::value;
    const T *xcur = xs + (size_t)cc * ROWS * LDX + rowoff, *xnxt = xs + (size_t)(cc ^ 1) * ROWS * LDX + rowoff;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 0; b < FMB; ++b)
#pragma unroll
      for (int q = 0; q < 2; ++q) xf[1][2 * b + q] = load_frag(xcur + b * 32 * LDX + 32 + q * 16);
    stage_load(stage[cc], max(sl + 2, c0));
    stage_store(stage[cc ^ 1], cc ^ 1);
    if constexpr (live) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int b = 0; b < FMB; ++b)
#pragma unroll
          for (int p = 0; p < FNP; ++p)
            acc[p][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ring[2 * cc][2 * p + q].v, xf[0][2 * b + q].v, acc[p][b], 0, 0, 0);
#pragma unroll
      for (int k = 0; k < NM; ++k) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x320, PER_A, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
#pragma unroll
    for (int b = 0; b < FMB; ++b)
#pragma unroll
      for (int q = 0; q < 2; ++q) xf[0][2 * b + q] = load_frag(xnxt + b * 32 * LDX + q * 16);
    __builtin_amdgcn_sched_barrier(0);
    load_w(ring[2 * cc], max(t0 + RING, 0));
    if constexpr (live) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int b = 0; b < FMB; ++b)
#pragma unroll
          for (int p = 0; p < FNP; ++p)
            acc[p][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ring[2 * cc + 1][2 * p + q].v, xf[1][2 * b + q].v, acc[p][b], 0, 0, 0);
#pragma unroll
      for (int k = 0; k < NM; ++k) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (k < FN) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    load_w(ring[2 * cc + 1], max(t0 + 1 + RING, 0));
  };

  // two slices without MFMAs fill the pipeline (the same memory instructions in the same order as the loop's, so
  // the loop is entered with the loads outstanding that every later trip finds); the loop itself has no branch
  using Cc0 = std::integral_constant<int, 0>;
  using Cc1 = std::integral_constant<int, 1>;
  half_trip(Cc0{}, std::false_type{}, c0 - 2, -2 * SPS);
  half_trip(Cc1{}, std::false_type{}, c0 - 1, -1 * SPS);
  int sl = c0;
  for (; sl + 1 < c1; sl += 2) {
    half_trip(Cc0{}, std::true_type{}, sl, (sl - c0) * SPS);
    half_trip(Cc1{}, std::true_type{}, sl + 1, (sl + 1 - c0) * SPS);
  }
  if (sl < c1) half_trip(Cc0{}, std::true_type{}, sl, (sl - c0) * SPS);   // an odd number of slices
  __syncthreads();                                           // everyone is done with xs
  float *rs_lds = reinterpret_cast<float *>(smem);           // [ROWS] 1 / rms (times the operand scales) of the tile's rows
  for (int r = tid; r < ROWS; r += 256) rs_lds[r] = row_scale(m0 + r);
  __syncthreads();

  const int row0 = wm * FMB * 32 + r32;                      // this lane's row of the tile in 32-row block 0
  if constexpr (EPI == EPI_QKV) {
    // the accumulators leave the registers through LDS (every wave its own region, behind the row scales) and the
    // rotary epilogue takes them back one fragment at a time, as in gemm_wide_kernel
    f32x4 *dump = reinterpret_cast<f32x4 *>(smem + (ROWS * sizeof(float) + 15) / 16 * 16) + (size_t)wave * (FN * FMB * 2 * 64);
#pragma unroll
    for (int p = 0; p < FNP; ++p)
#pragma unroll
      for (int b = 0; b < FMB; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          dump[((p * FMB + b) * 4 + j) * 64 + lane] = f32x4{acc[p][b][4 * j], acc[p][b][4 * j + 1], acc[p][b][4 * j + 2], acc[p][b][4 * j + 3]};
#pragma unroll 2
    for (int idx = 0; idx < FNP * FMB * 2; ++idx) {          // item: (pair, 32-row block, fragment of the pair)
      const int pb = idx >> 1, t = idx & 1;
      const int p = pb / FMB, b = pb - p * FMB;
      const int frag = (nb * 2 + wn) * FN + 2 * p + t;
      const int row = row0 + b * 32;
      if (frag < n_frags) {                                  // uniform per wave
        const float rs = rs_lds[row];
        const f32x4 lo = dump[(pb * 4 + 2 * t) * 64 + lane], hi = dump[(pb * 4 + 2 * t + 1) * 64 + lane];
        const float v[4] = {lo[0] * rs, lo[1] * rs, lo[2] * rs, lo[3] * rs};
        const float x2[4] = {hi[0] * rs, hi[1] * rs, hi[2] * rs, hi[3] * rs};
        epi_paired_vals<T, EPI>(a, frag, m0 + row, M, h, v, x2);
      }
    }
  } else {
#pragma unroll
    for (int b = 0; b < FMB; ++b) {
      const int row = row0 + b * 32;                         // row of the tile
      const int m = m0 + row;
      const bool live = m < M;
      const float rs = PAIRED ? rs_lds[row] : 1.0f;
#pragma unroll
      for (int p = 0; p < FNP; ++p) {
        if (!pair_live[p]) continue;                         // uniform per wave
        if constexpr (EPI == EPI_GATEUP) {
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            float v[4], x2[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) { v[r] = acc[p][b][8 * t + r] * rs; x2[r] = acc[p][b][8 * t + 4 + r] * rs; }
            epi_paired_vals<T, EPI>(a, frag0[p] + t, m, M, h, v, x2);
          }
        } else {
          if (live) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              epi_residual(a, ks, m, (frag0[p] + (j >> 1)) * 16, 2 * (j & 1) + h,
                           f32x4{acc[p][b][4 * j], acc[p][b][4 * j + 1], acc[p][b][4 * j + 2], acc[p][b][4 * j + 3]});
          }
        }
      }
    }
  }
}

// FN: fragments per wave; a workgroup owns 2 FN.  MT: row tiles of 16 FM rows (1: the tile holds the whole block).
template <typename T, int EPI, int FM, int FN>
static void launch_wide_cfg(const GemmArgs &a, int KS, int MT, hipStream_t s) {
  size_t lds = (size_t)2 * 16 * FM * (64 + 8) * sizeof(T);
  if (EPI == EPI_QKV) lds = std::max(lds, (size_t)(16 * FM * 4 + 15) / 16 * 16 + (size_t)4 * FN * (FM / 2) * 1024);   // accumulator hand-back
  const int blocks = (a.n_groups + 2 * FN - 1) / (2 * FN);
  if (lds > 64 * 1024) {
    static const hipError_t opted = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_wide_kernel<T, EPI, FM, FN, false>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    static const hipError_t opted_t = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_wide_kernel<T, EPI, FM, FN, true>),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)opted; (void)opted_t;
  }
  if (MT == 1) hipLaunchKernelGGL((gemm_wide_kernel<T, EPI, FM, FN, false>), dim3(blocks, KS), dim3(256), lds, s, a, 1);
  else hipLaunchKernelGGL((gemm_wide_kernel<T, EPI, FM, FN, true>), dim3((blocks + 7) / 8 * 8 * MT, KS), dim3(256), lds, s, a, MT);
}

template <typename T, int EPI, int FM, int FN>
static void launch_wide32_cfg(const GemmArgs &a, int KS, int MT, hipStream_t s) {
  size_t lds = (size_t)2 * 16 * FM * (64 + 8) * sizeof(T);
  if (EPI == EPI_QKV) lds = std::max(lds, (size_t)(16 * FM * 4 + 15) / 16 * 16 + (size_t)4 * FN * (FM / 2) * 1024);   // accumulator hand-back
  const int blocks = (a.n_groups + 2 * FN - 1) / (2 * FN);
  if (lds > 64 * 1024) {
    static const hipError_t opted = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_wide32_kernel<T, EPI, FM, FN, false>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    static const hipError_t opted_t = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_wide32_kernel<T, EPI, FM, FN, true>),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)opted; (void)opted_t;
  }
  if (MT == 1) hipLaunchKernelGGL((gemm_wide32_kernel<T, EPI, FM, FN, false>), dim3(blocks, KS), dim3(256), lds, s, a, 1);
  else hipLaunchKernelGGL((gemm_wide32_kernel<T, EPI, FM, FN, true>), dim3((blocks + 7) / 8 * 8 * MT, KS), dim3(256), lds, s, a, MT);
}

template <typename T, int EPI, int FM>
static void launch_wide_fm(const GemmArgs &a_in, int KS, int MT, hipStream_t s) {
  GemmArgs a = a_in;
  a.n_groups = a.N / 16 * ((EPI == EPI_GATEUP) ? 2 : 1);     // fragments: gate/up interleaves 2 * d_ffn rows
  if (EPI == EPI_QKV) a.n_groups = (a.H + 2 * a.Hkv) * (a.hd / 16);
  // 128 rows of W per workgroup (four fragments per wave) where that still gives most CUs a workgroup, 64
  // otherwise (q/k/v of a 4096-wide model has 768 fragments: 96 workgroups against 192): every workgroup reads
  // all of X whatever it owns, so the W rows per workgroup only matter once the chip is full.  q/k/v always
  // takes 64: the unrolled rotary epilogue over more accumulator fragments does not fit the registers.
  bool narrow = false;
  if constexpr (EPI == EPI_QKV || EPI == EPI_GATEUP) narrow = (a.n_groups + 7) / 8 * KS * MT < 160;
  // The 32x32x16 kernel where the tile's row blocks pair up (192 and 256 rows: every prefill piece of 2048 tokens)
  // and it measured faster on MI355X: q/k/v and gate/up always (7B shapes, 161-192 and 225-256 block rows: q/k/v
  // 52 -> 48 and 64 -> 57 us, gate/up 70.5 -> 69 and 82 -> 79 us; prefill pieces: 271 -> 230 and 519 -> 464 us), the
  // residual GEMMs only with several row tiles (prefill: 77 -> 72 and 242 -> 232 us; a single tile streams W from
  // HBM and was 5 % slower: 18.2 -> 19.2 and 41 -> 42 us).
  if constexpr (FM % 4 == 0 && EPI != EPI_UNEMBED) {
    constexpr bool paired = EPI == EPI_QKV || EPI == EPI_GATEUP;
    if (a.n_groups % 2 == 0 && a.K % 64 == 0 && (paired || MT > 1)) {
      if (narrow) launch_wide32_cfg<T, EPI, FM, 2>(a, KS, MT, s);
      else launch_wide32_cfg<T, EPI, FM, 4>(a, KS, MT, s);
      return;
    }
  }
  if (narrow) launch_wide_cfg<T, EPI, FM, 2>(a, KS, MT, s);
  else launch_wide_cfg<T, EPI, FM, 4>(a, KS, MT, s);
}

// Row tiles of the wide kernel: as few as possible (288 rows at most each), then the smallest even
// number of 16-row blocks that holds a tile's share of the rows.
static int gemm_wide_row_tiles(int M) { return (M + 287) / 288; }
int gemm_wide_row_blocks(int M) {
  const int tiles = gemm_wide_row_tiles(M);
  const int rows = (M + tiles - 1) / tiles;
  const int fm = (rows + 15) / 16;
  return (fm + 1) / 2 * 2 < 10 ? 10 : (fm + 1) / 2 * 2;
}

template <typename T, int EPI>
static void launch_wide(const GemmArgs &a, int KS, hipStream_t s) {
  const int MT = gemm_wide_row_tiles(a.M);
  switch (gemm_wide_row_blocks(a.M)) {
    case 10: launch_wide_fm<T, EPI, 10>(a, KS, MT, s); break;
    case 12: launch_wide_fm<T, EPI, 12>(a, KS, MT, s); break;
    case 14: launch_wide_fm<T, EPI, 14>(a, KS, MT, s); break;
    case 16: launch_wide_fm<T, EPI, 16>(a, KS, MT, s); break;
    default: launch_wide_fm<T, EPI, 18>(a, KS, MT, s);
  }
}

template <typename T, int EPI, int FM, int WN, int WK, int RING, int FN = 2>
void launch_gemm_cfg(const GemmArgs &a, int KS, hipStream_t s) {
  constexpr int KC = KChunk<T>::value;
  constexpr int PAD = 16 / (int)sizeof(T);
  constexpr bool PAIRED = EPI == EPI_QKV || EPI == EPI_GATEUP;
  size_t lds = (size_t)2 * 16 * FM * (KC + PAD) * sizeof(T);
  const size_t red = (size_t)(PAIRED ? WK * (FM < 4 ? FM : 4) : (WK - 1) * WN * FM) * FN * 4 * 64 * sizeof(float) +
                     (size_t)16 * FM * sizeof(float);          // + one 1 / rms per block row of the pass
  if (red > lds) lds = red;
  const int blocks = PAIRED ? (a.n_groups + FN - 1) / FN : (a.n_groups + WN - 1) / WN;
  if (lds > 64 * 1024) {                     // more than the default dynamic LDS limit: opt in once
    static const hipError_t opted = hipFuncSetAttribute(
        reinterpret_cast<const void *>(&gemm_skinny_kernel<T, EPI, FM, WN, WK, RING, FN>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)opted;
  }
  hipLaunchKernelGGL((gemm_skinny_kernel<T, EPI, FM, WN, WK, RING, FN>), dim3(blocks, KS), dim3(64 * WN * WK), lds, s, a);
}

// residual, unembedding: pairs of 16-row fragments; q/k/v and gate/up: 16-row fragments of 8 output pairs
int gemm_groups(int epi, const GemmArgs &a) {
  switch (epi) {
    case EPI_QKV: return (a.H + 2 * a.Hkv) * (a.hd / 16);
    case EPI_GATEUP: return a.N / 8;
    default: return a.N / 32;
  }
}

// The row tile holds the block's rows in 16-row column blocks of the MFMA: as many as the block needs, up
// to 8 (128 rows; more rows take another pass over W).  Every extra column block costs activation traffic
// from L2, LDS reads and MFMA work, so a 40-row block runs on 3 of them, not 4.
static int gemm_row_blocks(int M) { return M >= 128 ? 8 : (M + 15) / 16; }

template <typename T, int EPI, int WN, int WK, int RING>
static void launch_fm(const GemmArgs &a, int KS, hipStream_t s) {
  switch (gemm_row_blocks(a.M)) {                            // 16-row column blocks of the tile
    case 1: launch_gemm_cfg<T, EPI, 1, WN, WK, RING>(a, KS, s); break;
    case 2: launch_gemm_cfg<T, EPI, 2, WN, WK, RING>(a, KS, s); break;
    case 3: launch_gemm_cfg<T, EPI, 3, WN, WK, RING>(a, KS, s); break;
    case 4: launch_gemm_cfg<T, EPI, 4, WN, WK, RING>(a, KS, s); break;
    case 5: launch_gemm_cfg<T, EPI, 5, WN, WK, RING>(a, KS, s); break;
    case 6: launch_gemm_cfg<T, EPI, 6, WN, WK, RING>(a, KS, s); break;
    case 7: launch_gemm_cfg<T, EPI, 7, WN, WK, RING>(a, KS, s); break;
    default: launch_gemm_cfg<T, EPI, 8, WN, WK, RING>(a, KS, s);   // 128-row tiles; more rows loop over W again
  }
}

// q/k/v and gate/up: one workgroup = FN fragments, its four waves split the steps of every chunk
// (WN = 1, WK = 4).  FN is chosen so that the fragments spread evenly over the 256 CUs (7B shapes:
// 768 q/k/v fragments = 3 per workgroup, 1792 gate/up fragments = 7 per workgroup, 256 workgroups
// each); wide fragment sets keep a 2-deep ring (FN KB per slot and wave are in flight anyway).
template <typename T, int EPI, int FM>
static void launch_paired_fm(const GemmArgs &a, hipStream_t s) {
  constexpr int FMAX = sizeof(T) == 4 ? 2 : (FM == 8 ? 7 : 8);   // accumulators: FN * FM * 4 registers; fp32 fragments: twice the ring
  int fn = (a.n_groups + 255) / 256;
  fn = fn < 1 ? 1 : (fn > FMAX ? FMAX : fn);
  switch (fn) {
    case 1: launch_gemm_cfg<T, EPI, FM, 1, 4, 4, 1>(a, 1, s); break;
    case 2: launch_gemm_cfg<T, EPI, FM, 1, 4, 4, 2>(a, 1, s); break;
    default:
      if constexpr (FMAX >= 4) {
        switch (fn) {
          case 3: launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 3>(a, 1, s); break;
          case 4: launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 4>(a, 1, s); break;
          default:
            if constexpr (FMAX >= 6) {
              switch (fn) {
                case 5: launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 5>(a, 1, s); break;
                case 6: launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 6>(a, 1, s); break;
                default:
                  if constexpr (FMAX >= 8) {
                    if (fn == 7) launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 7>(a, 1, s);
                    else launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 8>(a, 1, s);
                  } else {
                    launch_gemm_cfg<T, EPI, FM, 1, 4, 2, 7>(a, 1, s);   // 128-row tiles: 8 fragments no longer fit the registers
                  }
              }
            }
        }
      }
  }
}

template <typename T, int EPI>
static void launch_paired(const GemmArgs &a, hipStream_t s) {
  switch (gemm_row_blocks(a.M)) {
    case 1: launch_paired_fm<T, EPI, 1>(a, s); break;
    case 2: launch_paired_fm<T, EPI, 2>(a, s); break;
    case 3: launch_paired_fm<T, EPI, 3>(a, s); break;
    case 4: launch_paired_fm<T, EPI, 4>(a, s); break;
    case 5: launch_paired_fm<T, EPI, 5>(a, s); break;
    case 6: launch_paired_fm<T, EPI, 6>(a, s); break;
    case 7: launch_paired_fm<T, EPI, 7>(a, s); break;
    default: launch_paired_fm<T, EPI, 8>(a, s);
  }
}

// Residual GEMMs: a workgroup takes 64 rows of W (WN = 2, its waves 2 x 2), or 32 rows with all four
// waves splitting the steps (WN = 1) where that measured faster on MI355X: single-token steps, and the
// square output projection (4096 x 4096: 11.0 against 11.7 us at 60 block rows, 8.2 against 9.5 at one;
// down 4096 x 14336: 26.2 against 23.4 at 60 rows, 19.6 against 20.5 at one).  Narrower workgroups need
// half the splits of the contraction, so the RMSNorm that follows adds half the partials.
static bool residual_narrow(int M, int N, int K) { return M <= 16 || K <= N; }

// Split of the contraction across workgroups for the residual GEMMs: about one workgroup per CU, as
// long as each split keeps at least 2 chunks.
int gemm_residual_splits(int dtype, int M, int N, int K) {
  if (dtype == 1 && M > 128) {              // wide kernel: 128 rows of W per workgroup, slices of 64; at least 8 slices per split
    const int blocks = (N / 16 + 7) / 8 * ((M + 287) / 288), n_slices = (K + 63) / 64;   // row tiles count as workgroups
    int ks = (256 + blocks - 1) / blocks;
    ks = ks > kMaxResidualSplits ? kMaxResidualSplits : ks;
    while (ks > 1 && n_slices / ks < 8) --ks;
    return ks < 1 ? 1 : ks;
  }
  const int kc = dtype == 1 ? KChunk<half_t>::value : KChunk<float>::value;
  const int n_chunks = (K + kc - 1) / kc;
  const int blocks = residual_narrow(M, N, K) ? N / 32 : (N / 32 + 1) / 2;
  int ks = (256 + blocks - 1) / blocks;
  ks = ks > kMaxResidualSplits ? kMaxResidualSplits : ks;
  while (ks > 1 && n_chunks / ks < 2) --ks;
  return ks < 1 ? 1 : ks;
}

// Workgroup shapes measured on MI355X at the 7B shapes (M = 60 and M = 1).  Unembedding: wide tiles
// (WN = 4) where there are enough row groups to give every CU a workgroup, otherwise two waves per
// pair of groups; residual GEMMs: WN x WK = 2 x 2 or 1 x 4 (residual_narrow) with the contraction split
// across workgroups.
template <typename T>
static void launch_t(int epi, const GemmArgs &a_in, hipStream_t s) {
  GemmArgs a = a_in;
  if constexpr (sizeof(T) == 2) {
    if (a.M > 128) {
      switch (epi) {
        case EPI_QKV: launch_wide<T, EPI_QKV>(a, 1, s); break;
        case EPI_GATEUP: launch_wide<T, EPI_GATEUP>(a, 1, s); break;
        case EPI_RESIDUAL: launch_wide<T, EPI_RESIDUAL>(a, a.KS, s); break;
        default: launch_wide<T, EPI_UNEMBED>(a, 1, s);
      }
      return;
    }
  }
  a.n_groups = gemm_groups(epi, a);
  const bool wide = a.n_groups >= 4 * 200;
  switch (epi) {
    case EPI_QKV: launch_paired<T, EPI_QKV>(a, s); break;
    case EPI_GATEUP: launch_paired<T, EPI_GATEUP>(a, s); break;
    case EPI_RESIDUAL:
      if (residual_narrow(a.M, a.N, a.K)) launch_fm<T, EPI_RESIDUAL, 1, 4, 4>(a, a.KS, s);
      else launch_fm<T, EPI_RESIDUAL, 2, 2, 4>(a, a.KS, s);
      break;
    default:
      if (wide) launch_fm<T, EPI_UNEMBED, 4, 1, 8>(a, 1, s);
      else launch_fm<T, EPI_UNEMBED, 2, 2, 4>(a, 1, s);
  }
}

void launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t s) {
  if (dtype == 1) launch_t<half_t>(epi, a, s);
  else launch_t<float>(epi, a, s);
}

}  // namespace ngg
