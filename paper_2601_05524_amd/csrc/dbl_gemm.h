// Weight-streaming small-M projection kernels (M = batch * window rows <= 16 per pass).
//
// The verify step reads every weight once and reuses it for M <= 16 rows, so it is
// bound by HBM bandwidth (arithmetic intensity M flop/byte against a ridge of ~300).
// Design:
//   * weights are the MFMA A operand (16 output features x 32 inputs per block) in
//     the tiled layout of dbl_dev.h, so every wave-level load is 1 KiB contiguous;
//   * the activations (the B operand, 32 inputs x 16 rows) of a wave's K slice live
//     in registers for the whole kernel: a wave owns KS k-blocks of every output
//     tile its workgroup visits, so activations are fetched once per wave;
//   * the NW waves of a workgroup own NW consecutive K slices of the same output
//     tile; their partial tiles are summed through LDS in a fixed order
//     (deterministic, no atomics) and wave 0 applies the epilogue;
//   * loads run RING blocks ahead of the MFMAs and the ring runs across output
//     tiles, so the memory pipe never drains inside a kernel;
//   * a workgroup walks output tiles wg/SS, +nwg/SS, ...; if K is too long
//     for 8 waves x KS blocks, SS workgroup "super slices" split K and each writes
//     its own partial result (summed by the consumer kernel).
// The body is a device function so that the same code runs as a stand-alone kernel
// and as a phase of the persistent layer kernel (dbl_layer.h); there (COH = true)
// activations and results cross workgroups inside one launch and are accessed with
// agent-coherent loads / stores, and the first ring of weights can be fetched
// before the phase starts.
#pragma once
#include "dbl_dev.h"

namespace dbl {

enum GemmEpi { EPI_PARTIAL = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

// Per-workgroup, per-row statistics left by the LM-head epilogue.
struct LmStat {
  float best; int best_id;        // arg-max of the raw logits
  float smax, ssum;               // online soft-max of logits/T: running max, sum exp
  float zdraft;                   // logit of the row's draft token if seen, else -inf
  float p1; int p1_id;            // largest Gumbel-perturbed score logits/T + G
  float p2; int p2_id;            // second largest
};

struct LmArgs {
  LmStat* stats;                  // [grid][Mtot]
  const int32_t* window;          // [B][k]
  const uint64_t* commits;        // device counter added to `step`
  int k;                          // window rows per sequence
  float inv_T;                    // 0 => greedy statistics only
  uint64_t seed, step;
};

template <typename T>
struct GemmArgs {
  const T* W;       // tiled weights: NT * NACC tile rows of KBp blocks
  const T* X;       // activations [Mtot][ldx], ldx >= KBp*32, zero beyond K
  int ldx;
  int m0, mrows;    // rows m0 .. m0+mrows-1 (mrows <= 16) are computed by this launch
  int Mtot;
  int NT;           // output tiles (tile pairs for EPI_SWIGLU)
  int N;            // valid output features (per half for EPI_SWIGLU)
  int KBp;          // k-blocks per tile row
  int SS;           // super slices; number of workgroups % SS == 0
  float* out;       // PARTIAL: [SS][Mtot][ldo] ; RESIDUAL: h[Mtot][ldo] (+=) ; LMHEAD: logits[Mtot][ldo]
  int ldo;
  T* act;           // SWIGLU: [Mtot][ldact]
  int ldact;
  LmArgs lm;
};

template <typename T> struct GemmCfg;
template <> struct GemmCfg<bf16_t> { static constexpr int RING = 16; };
template <> struct GemmCfg<float> { static constexpr int RING = 8; };

typedef f32x4 GemmRed[8][2][WAVE];   // one LDS reduction buffer: [wave][accumulator][lane]

template <typename T, int NACC>
__device__ __forceinline__ size_t gemm_blk(const GemmArgs<T>& a, int tile, int sub, int kb) {
  return ((size_t)tile * NACC + sub) * a.KBp + kb;
}

// Issue the first RING weight loads of workgroup `wg` for this projection.  Weights do
// not depend on any activation, so this may run before the producer of X has finished.
template <typename T, int EPI, int KS, int RING = GemmCfg<T>::RING>
__device__ __forceinline__ void gemm_prefetch(const GemmArgs<T>& a, int wg, int nwg, int nw, Frag<T> (&ring)[RING]) {
  constexpr int NACC = (EPI == EPI_SWIGLU) ? 2 : 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ss = wg % a.SS, t = wg / a.SS;
  if (wave >= nw || t >= a.NT) return;
  const int kb0 = (ss * nw + wave) * KS;
#pragma unroll
  for (int j = 0; j < RING; ++j) ring[j] = frag_load_w(a.W, gemm_blk<T, NACC>(a, t, 0, kb0 + j), lane);
}

// BPACK (at most 8 rows): the activation operand has 16 columns but only 8 rows to
// put in them, so one register set holds TWO k-blocks: lanes c < 8 carry block 2i (row
// c), lanes c >= 8 carry block 2i+1 (row c-8).  Block 2i is used as it is (columns
// 8..15 of the product are never read); for block 2i+1 the halves are swapped with a
// DPP rotate by 8 inside each 16-lane row.  This halves the registers the activations
// take (64 instead of 128 for a 32-block slice).
template <typename T, int EPI, int KS, bool COH, bool BPACK = false, int RING = GemmCfg<T>::RING>
__device__ __forceinline__ void gemm_body(const GemmArgs<T>& a, int wg, int nwg, int nw, GemmRed* red,
                                          Frag<T> (&ring)[RING], bool prefetched) {
  constexpr int NACC = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr int NB = BPACK ? KS / 2 : KS;      // activation register sets
  static_assert(!BPACK || KS % 2 == 0, "packed activations pair k-blocks");
  static_assert(KS % RING == 0, "slice must be a whole number of rings");
  static_assert(!(COH && EPI == EPI_LMHEAD), "the LM head runs as its own kernel");

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool active = wave < nw;             // waves beyond nw only keep the barriers company
  const int c = lane & 15, g = lane >> 4;
  const int ss = wg % a.SS;
  const int tstep = nwg / a.SS;
  int t = wg / a.SS;
  const int kb0 = (ss * nw + wave) * KS;

  if (!prefetched) gemm_prefetch<T, EPI, KS, RING>(a, wg, nwg, nw, ring);

  // activations of this wave's K slice -> registers.  Output column j of a tile depends
  // only on activation row j, so lanes of the unused rows (c >= mrows) simply re-read the
  // last valid row: all loads are unconditional and stay in flight together.
  Frag<T> breg[NB];
  {
    const int wv = active ? wave : 0;
    const int row = BPACK ? (c & 7) : c, odd = BPACK ? (c >> 3) : 0;
    const T* xrow = a.X + (size_t)(a.m0 + min(row, a.mrows - 1)) * a.ldx + (size_t)((ss * nw + wv) * KS + odd) * TILE_K + g * 8;
#pragma unroll
    for (int j = 0; j < NB; ++j) breg[j] = frag_load_row<COH>(xrow + (size_t)j * (BPACK ? 2 : 1) * TILE_K);
  }

  // LM-head running statistics (wave 0 only)
  float best = -INFINITY, smax = -INFINITY, ssum = 0.f, zdraft = -INFINITY, p1 = -INFINITY, p2 = -INFINITY;
  int best_id = 0x7fffffff, p1_id = 0x7fffffff, p2_id = 0x7fffffff;
  int draft = -1; uint32_t pb = 0, pj = 0; uint64_t stepv = 0;
  if (EPI == EPI_LMHEAD && wave == 0 && c < a.mrows) {
    const int m = a.m0 + c;
    pb = m / a.lm.k; pj = m % a.lm.k;
    if ((int)pj + 1 < a.lm.k) draft = a.lm.window[m + 1];
    stepv = a.lm.step + *a.lm.commits;
  }

  // Per-lane pointer to block 0 of this wave's slice of tile row 0; a tile row is KBp
  // blocks of BLOCK_ELEMS elements.  All weight addresses below are this plus a
  // tile-row offset plus a compile-time block offset: no branches around the loads, so
  // the compiler can count outstanding loads exactly (s_waitcnt vmcnt(N) with N > 0).
  const T* wlane = a.W + (size_t)kb0 * BLOCK_ELEMS;
  const size_t row_elems = (size_t)a.KBp * BLOCK_ELEMS;
  for (int it = 0; t < a.NT; t += tstep, ++it) {
    // after the last tile the refill loads go on, harmlessly, into tile 0 (an L2 hit)
    const int tn = (t + tstep < a.NT) ? t + tstep : 0;
    f32x4 acc[NACC];
#pragma unroll
    for (int s = 0; s < NACC; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (active) {
      const T* wcur = wlane + (size_t)t * NACC * row_elems;
      const T* wnext = wlane + (size_t)tn * NACC * row_elems;
#pragma unroll
      for (int s = 0; s < NACC; ++s) {
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          if (BPACK) acc[s] = mma(ring[j % RING], (j & 1) ? frag_swap_halves(breg[j / 2]) : breg[j / 2], acc[s]);
          else acc[s] = mma(ring[j % RING], breg[j], acc[s]);
          const int jn = j + RING;
          if (jn < KS) ring[j % RING] = frag_load_w(wcur + s * row_elems, jn, lane);
          else if (s + 1 < NACC) ring[j % RING] = frag_load_w(wcur + (s + 1) * row_elems, jn - KS, lane);
          else ring[j % RING] = frag_load_w(wnext, jn - KS, lane);
        }
      }
    }
    const int buf = it & 1;
    if (active && wave != 0) {
#pragma unroll
      for (int s = 0; s < NACC; ++s) red[buf][wave][s][lane] = acc[s];
    }
    __syncthreads();
    if (wave == 0) {
      for (int w = 1; w < nw; ++w) {
#pragma unroll
        for (int s = 0; s < NACC; ++s) acc[s] += red[buf][w][s][lane];
      }
      if (c < a.mrows) {
        const int m = a.m0 + c;
        const int n = t * TILE_N + 4 * g;   // first of this lane's 4 output features
        if (EPI == EPI_PARTIAL) {
          st_f4<COH>(a.out + ((size_t)ss * a.Mtot + m) * a.ldo + n, acc[0]);
        } else if (EPI == EPI_RESIDUAL) {
          float* p = a.out + (size_t)m * a.ldo + n;
          st_f4<COH>(p, ld_f4<COH>(p) + acc[0]);
        } else if (EPI == EPI_SWIGLU) {
          f32x4 v;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float gt = acc[0][i], up = acc[1][i];
            v[i] = (n + i < a.N) ? gt / (1.f + expf(-gt)) * up : 0.f;
          }
          st_round4<COH>(a.act + (size_t)m * a.ldact + n, v);
        } else {  // EPI_LMHEAD
          *reinterpret_cast<f32x4*>(a.out + (size_t)m * a.ldo + n) = acc[0];
          Philox4 rnd{0, 0, 0, 0};
          const bool sampling = a.lm.inv_T > 0.f;
          if (sampling)
            rnd = philox4x32_10((uint32_t)stepv, pb, pj, 1u + (uint32_t)(n >> 2), (uint32_t)a.lm.seed,
                                (uint32_t)(a.lm.seed >> 32));
          const uint32_t rw[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int v = n + i;
            if (v >= a.N) continue;
            const float z = acc[0][i];
            if (better(z, v, best, best_id)) { best = z; best_id = v; }
            if (v == draft) zdraft = z;
            if (sampling) {
              const float zs = z * a.lm.inv_T;
              if (zs > smax) { ssum = ssum * expf(smax - zs) + 1.f; smax = zs; }
              else ssum += expf(zs - smax);
              const float sc = zs + gumbel(rw[i]);
              if (better(sc, v, p1, p1_id)) { p2 = p1; p2_id = p1_id; p1 = sc; p1_id = v; }
              else if (better(sc, v, p2, p2_id)) { p2 = sc; p2_id = v; }
            }
          }
        }
      }
    }
  }

  if (EPI == EPI_LMHEAD && wave == 0) {
    // merge the four lane groups that share a row
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float ob = __shfl_xor(best, off); const int obi = __shfl_xor(best_id, off);
      if (better(ob, obi, best, best_id)) { best = ob; best_id = obi; }
      const float oz = __shfl_xor(zdraft, off);
      zdraft = fmaxf(zdraft, oz);
      const float om = __shfl_xor(smax, off), os = __shfl_xor(ssum, off);
      const float nm = fmaxf(smax, om);
      if (nm > -INFINITY) ssum = ssum * expf(smax - nm) + os * expf(om - nm);
      smax = nm;
      const float o1 = __shfl_xor(p1, off), o2 = __shfl_xor(p2, off);
      const int o1i = __shfl_xor(p1_id, off), o2i = __shfl_xor(p2_id, off);
      // merge two sorted pairs
      if (better(o1, o1i, p1, p1_id)) {
        if (better(p1, p1_id, o2, o2i)) { p2 = p1; p2_id = p1_id; } else { p2 = o2; p2_id = o2i; }
        p1 = o1; p1_id = o1i;
      } else if (better(o1, o1i, p2, p2_id)) { p2 = o1; p2_id = o1i; }
    }
    if (g == 0 && c < a.mrows) {
      LmStat s;
      s.best = best; s.best_id = best_id; s.smax = smax; s.ssum = ssum; s.zdraft = zdraft;
      s.p1 = p1; s.p1_id = p1_id; s.p2 = p2; s.p2_id = p2_id;
      a.lm.stats[(size_t)wg * a.Mtot + a.m0 + c] = s;
    }
  }
}

template <typename T, int EPI, int KS, bool BPACK>
__global__ void __launch_bounds__(512) gemm_stream_kernel(const GemmArgs<T> a) {
  __shared__ GemmRed red[2];
  Frag<T> ring[GemmCfg<T>::RING];
  gemm_body<T, EPI, KS, false, BPACK>(a, blockIdx.x, gridDim.x, blockDim.x >> 6, red, ring, false);
}

}  // namespace dbl
