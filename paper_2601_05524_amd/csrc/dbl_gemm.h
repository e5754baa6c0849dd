// Weight-streaming projection kernels.
//
// The verify step reads every weight once and reuses it for the M = batch * window rows, so it
// is bound by HBM bandwidth (arithmetic intensity M flop/byte against a ridge of ~300).  Weights
// are the MFMA A operand (16 output features x 32 inputs per block) in the tiled layout of
// dbl_dev.h, so every wave-level load is 1 KiB contiguous and non-temporal; activations (the B
// operand, 32 inputs x 16 rows) live in registers; loads run a ring of blocks ahead of the
// MFMAs and the ring never drains inside a kernel; partial sums of the waves that split K are
// added through LDS in a fixed order (deterministic, no atomics).  Two kernels:
//
// gemm_stream_kernel (at most 8 rows: the q/k/v projection, and output/down at narrow widths):
//   * a wave owns KS k-blocks of every output tile its workgroup visits, so activations are
//     fetched once per wave (once per K chunk in the chunked form), two k-blocks per register
//     set, and RMSNorm is applied while they are loaded;
//   * the NW <= 8 waves of a workgroup own consecutive K slices of the same output tile; wave 0
//     applies the epilogue;
//   * a workgroup starts at output tile wg/SS and steps by nwg/SS;
//   * K longer than NW*KS blocks is covered either by SS workgroup "super slices", each writing
//     its own partial result that the consumer sums (q/k/v projection), or by NCH sequential K
//     chunks inside the workgroup with the accumulator kept in registers (CHUNK form).
//
// gemm_rows_kernel (any number of rows in passes of up to 64; gate/up and the LM head always):
// see its own comment.
//
// RMSNorm is not a kernel of its own.  Whichever kernel wrote the residual stream h last
// (embedding, output projection, down projection) also stores hg = h * gain of the next
// norm, and each of its workgroups leaves one partial sum of squares per row in
// ssq[row][workgroup] (SSQ_PARTS slots per row, unused ones zero).  gemm_stream_kernel adds the
// partials in a fixed order and builds bf16(hg * rsqrt(mean(h^2) + eps)) while loading its
// activation registers; xn_kernel stores that tensor for gemm_rows_kernel.
#pragma once
#include <type_traits>
#include "dbl_dev.h"

namespace dbl {

enum GemmEpi { EPI_PARTIAL = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

constexpr int SSQ_PARTS = 256;    // sum-of-squares partials per row; a producer launches at most this many workgroups

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

// Row statistics of the LM head: empty state, merge of two states (any order of merges
// gives the same arg-max / top-2; the soft-max sums are added in whatever order the caller
// fixes), and the update with four consecutive logits n..n+3 of one row.
__device__ __forceinline__ void lm_init(LmStat& s) {
  s.best = -INFINITY; s.best_id = 0x7fffffff; s.smax = -INFINITY; s.ssum = 0.f; s.zdraft = -INFINITY;
  s.p1 = -INFINITY; s.p1_id = 0x7fffffff; s.p2 = -INFINITY; s.p2_id = 0x7fffffff;
}
__device__ __forceinline__ void lm_merge(LmStat& x, const LmStat& y) {
  if (better(y.best, y.best_id, x.best, x.best_id)) { x.best = y.best; x.best_id = y.best_id; }
  x.zdraft = fmaxf(x.zdraft, y.zdraft);
  const float nm = fmaxf(x.smax, y.smax);
  if (nm > -INFINITY) x.ssum = x.ssum * expf(x.smax - nm) + y.ssum * expf(y.smax - nm);
  x.smax = nm;
  if (better(y.p1, y.p1_id, x.p1, x.p1_id)) {
    if (better(x.p1, x.p1_id, y.p2, y.p2_id)) { x.p2 = x.p1; x.p2_id = x.p1_id; } else { x.p2 = y.p2; x.p2_id = y.p2_id; }
    x.p1 = y.p1; x.p1_id = y.p1_id;
  } else if (better(y.p1, y.p1_id, x.p2, x.p2_id)) { x.p2 = y.p1; x.p2_id = y.p1_id; }
}
__device__ __forceinline__ LmStat lm_shfl_xor(const LmStat& s, int off) {
  LmStat o;
  o.best = __shfl_xor(s.best, off); o.best_id = __shfl_xor(s.best_id, off);
  o.smax = __shfl_xor(s.smax, off); o.ssum = __shfl_xor(s.ssum, off); o.zdraft = __shfl_xor(s.zdraft, off);
  o.p1 = __shfl_xor(s.p1, off); o.p1_id = __shfl_xor(s.p1_id, off);
  o.p2 = __shfl_xor(s.p2, off); o.p2_id = __shfl_xor(s.p2_id, off);
  return o;
}
// (pb, pj) = (sequence, window row) of the logits' row, draft = that row's draft token or -1
__device__ __forceinline__ void lm_update(LmStat& s, const f32x4& z4, int n, int N, int draft, uint32_t pb, uint32_t pj,
                                          uint64_t stepv, const LmArgs& lm) {
  Philox4 rnd{0, 0, 0, 0};
  const bool sampling = lm.inv_T > 0.f;
  if (sampling)
    rnd = philox4x32_10((uint32_t)stepv, pb, pj, 1u + (uint32_t)(n >> 2), (uint32_t)lm.seed, (uint32_t)(lm.seed >> 32));
  const uint32_t rw[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = n + i;
    if (v >= N) continue;
    const float z = z4[i];
    if (better(z, v, s.best, s.best_id)) { s.best = z; s.best_id = v; }
    if (v == draft) s.zdraft = z;
    if (sampling) {
      const float zs = z * lm.inv_T;
      if (zs > s.smax) { s.ssum = s.ssum * expf(s.smax - zs) + 1.f; s.smax = zs; }
      else s.ssum += expf(zs - s.smax);
      const float sc = zs + gumbel(rw[i]);
      if (better(sc, v, s.p1, s.p1_id)) { s.p2 = s.p1; s.p2_id = s.p1_id; s.p1 = sc; s.p1_id = v; }
      else if (better(sc, v, s.p2, s.p2_id)) { s.p2 = sc; s.p2_id = v; }
    }
  }
}

template <typename T>
struct GemmArgs {
  const T* W;          // tiled weights: NT * NACC tile rows of KBp blocks
  // activations, one of:
  const T* X;          //   EPI_RESIDUAL, or more than 8 rows: [Mtot][ldx] elements of type T, ldx >= KBp*32,
                       //   zero beyond K
  const float* HG;     //   other epilogues, at most 8 rows: residual stream times the RMSNorm gain,
                       //   [Mtot][ldx] fp32, zero beyond K; scaled by 1/rms and rounded on load
  int ldx;
  const float* ssq_in; // [Mtot][SSQ_PARTS] partial sums of squares of the residual rows
  float d, eps;        // mean = sum / d
  int m0, mrows;       // rows m0 .. m0+mrows-1 (mrows <= 16) are computed by this launch
  int Mtot;
  int NT;              // output tiles (tile pairs for EPI_SWIGLU)
  int N;               // valid output features (per half for EPI_SWIGLU)
  int KBp;             // k-blocks per tile row = SS * NCH * NW * KS
  int SS;              // super slices; number of workgroups % SS == 0
  int NCH;             // K chunks walked by one workgroup (1 unless the CHUNK form runs)
  float* out;          // PARTIAL: [SS][Mtot][ldo] ; RESIDUAL: h[Mtot][ldo] (+=) ; LMHEAD: logits[Mtot][ldo] or nullptr (statistics only)
  int ldo;
  float* ssq_out;      // RESIDUAL: [Mtot][SSQ_PARTS] partial sums of squares of the updated rows
  float* hg_out;       // RESIDUAL: [Mtot][ldo] updated rows times gain_out (input of the next RMSNorm)
  const float* gain_out;   // RESIDUAL: [>= NT*16] gain of the next RMSNorm
  T* act;              // SWIGLU: [Mtot][ldact]
  int ldact;
  int act_tiled;       // SWIGLU in gemm_rows_kernel: act in the fragment-tiled layout (its reader is gemm_rows_kernel too)
  float* sk_part;      // gemm_rows_kernel, split units: partial sums, two slots per workgroup
  int* sk_cnt;         //   arrivals per unit, zero between launches
  LmArgs lm;
};

// 16 bytes to / from memory that other workgroups of the launch read / wrote: device-scope relaxed
// atomics (two 8-byte ones), which go past the L2 of the XCD
__device__ __forceinline__ void st_device(float* p, const f32x4& v) {
  unsigned long long* q = reinterpret_cast<unsigned long long*>(p);
  const unsigned long long lo = (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32);
  const unsigned long long hi = (unsigned long long)__float_as_uint(v.z) | ((unsigned long long)__float_as_uint(v.w) << 32);
  __hip_atomic_store(q, lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x4 ld_device(const float* p) {
  const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
  const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return f32x4{__uint_as_float((uint32_t)lo), __uint_as_float((uint32_t)(lo >> 32)), __uint_as_float((uint32_t)hi),
               __uint_as_float((uint32_t)(hi >> 32))};
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant in every copy of the body
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

template <typename T> struct GemmCfg;
template <> struct GemmCfg<bf16_t> { static constexpr int RING = 16; };
template <> struct GemmCfg<float> { static constexpr int RING = 8; };

typedef f32x4 GemmRed[8][WAVE];   // one LDS reduction buffer: [wave][lane]

// gemm_rows_kernel: k-blocks per wave and chunk for R row groups (halved for 8 row groups: registers;
// host and kernel share this)
constexpr int rows_ks(bool two_byte, int R) { return (two_byte ? 8 : 4) / (R > 4 ? 2 : 1); }

// 1 / rms of the row a lane of gemm_stream_kernel works on: row (lane & 7), clamped to the
// valid rows.  Eight lanes add the 256 partials of one row (32 each, then a butterfly); the
// result is fetched from that group's first lane.
__device__ __forceinline__ float row_scale(const float* ssq, int m0, int mrows, float d, float eps, int lane) {
  const int rr = min(lane >> 3, mrows - 1);
  const f32x4* p = reinterpret_cast<const f32x4*>(ssq + (size_t)(m0 + rr) * SSQ_PARTS) + (lane & 7) * 8;
  f32x4 v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) v[u] = p[u];
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u) s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
  s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4);
  const float r = rsqrtf(s / d + eps);
  return __shfl(r, (lane & 7) * 8);
}

// Eight activations of one row as an MFMA fragment: T((h * gain) * r), the RMSNorm output
// rounded to the element type (rounding point r1 of the numerics contract).  hg = h * gain
// was stored by the producer of h.
__device__ __forceinline__ Frag<bf16_t> norm_frag(const float* hg, float r, bf16_t) {
  const f32x4 h0 = *reinterpret_cast<const f32x4*>(hg), h1 = *reinterpret_cast<const f32x4*>(hg + 4);
  Frag<bf16_t> f;
  f.v = u32x4{pack_bf16(h0.x * r, h0.y * r), pack_bf16(h0.z * r, h0.w * r),
              pack_bf16(h1.x * r, h1.y * r), pack_bf16(h1.z * r, h1.w * r)};
  return f;
}
__device__ __forceinline__ Frag<float> norm_frag(const float* hg, float r, float) {
  Frag<float> f;
  f.lo = *reinterpret_cast<const f32x4*>(hg) * r;
  f.hi = *reinterpret_cast<const f32x4*>(hg + 4) * r;
  return f;
}

// Activation registers of the KS k-blocks starting at block kblk, for at most 8 rows: the B
// operand has 16 columns but only 8 rows to put in them, so one register set holds TWO
// k-blocks: lanes c < 8 carry block 2i (row c), lanes c >= 8 carry block 2i+1 (row c-8).
// Block 2i is used as it is (columns 8..15 of the product are never read); for block 2i+1
// the halves are swapped with a DPP rotate by 8 inside each 16-lane row.  This halves the
// registers the activations take.  Output column j of a tile depends only on activation row
// j, so lanes of unused rows re-read the last valid row: all loads are unconditional and stay
// in flight together.
// The 16-row form: one register set per k-block, lane (c, g) carries inputs 8g .. 8g+7 of row c (rows beyond the
// valid ones re-read the last one).
template <typename T, bool NORM, int KS>
__device__ __forceinline__ void load_acts16(const GemmArgs<T>& a, int kblk, float r, int lane, Frag<T> (&b)[KS]) {
  const int c = lane & 15, g = lane >> 4;
  const int row = a.m0 + min(c, a.mrows - 1);
  const size_t k0 = (size_t)kblk * TILE_K + g * 8;
  if (NORM) {
    const float* hp = a.HG + (size_t)row * a.ldx + k0;
#pragma unroll
    for (int j = 0; j < KS; ++j) b[j] = norm_frag(hp + j * TILE_K, r, T());
  } else {
    const T* xp = a.X + (size_t)row * a.ldx + k0;
#pragma unroll
    for (int j = 0; j < KS; ++j) b[j] = frag_load_row(xp + j * TILE_K);
  }
}

template <typename T, bool NORM, int KS>
__device__ __forceinline__ void load_acts(const GemmArgs<T>& a, int kblk, float r, int lane, Frag<T> (&b)[KS / 2]) {
  const int c = lane & 15, g = lane >> 4;
  const int row = a.m0 + min(c & 7, a.mrows - 1);
  const size_t k0 = (size_t)(kblk + (c >> 3)) * TILE_K + g * 8;
  if (NORM) {
    const float* hp = a.HG + (size_t)row * a.ldx + k0;
#pragma unroll
    for (int j = 0; j < KS / 2; ++j) b[j] = norm_frag(hp + j * 2 * TILE_K, r, T());
  } else {
    const T* xp = a.X + (size_t)row * a.ldx + k0;
#pragma unroll
    for (int j = 0; j < KS / 2; ++j) b[j] = frag_load_row(xp + j * 2 * TILE_K);
  }
}

// At most 8 rows; EPI_PARTIAL (q/k/v: RMSNorm applied on load, partial store per super slice)
// or EPI_RESIDUAL (output / down projection at widths whose tiles do not fill the chip in
// pairs).  CHUNK: the workgroup walks NCH K chunks per output tile (EPI_RESIDUAL only); the
// activations of the next chunk are fetched while the current one is multiplied.
// ROWS16: up to 16 rows, one activation register set per k-block (EPI_PARTIAL only): the q/k/v projection of 9 .. 16
// rows, which otherwise needs a stored RMSNorm output and gemm_rows_kernel's per-unit activation reads.
template <typename T, int EPI, int KS, bool CHUNK, bool ROWS16 = false>
__global__ void __launch_bounds__(512) gemm_stream_kernel(const GemmArgs<T> a) {
  static_assert(EPI == EPI_PARTIAL || EPI == EPI_RESIDUAL, "the other epilogues live in gemm_rows_kernel");
  static_assert(!ROWS16 || (EPI == EPI_PARTIAL && !CHUNK), "16 rows: the q/k/v projection only");
  constexpr int RING = GemmCfg<T>::RING;
  constexpr int NB = ROWS16 ? KS : KS / 2;     // activation register sets
  constexpr bool NORM = EPI != EPI_RESIDUAL;
  static_assert(KS % 2 == 0, "packed activations pair k-blocks");
  static_assert(KS % RING == 0, "slice must be a whole number of rings");
  static_assert(!CHUNK || EPI == EPI_RESIDUAL, "only the residual projections walk K chunks");

  __shared__ GemmRed red[2];
  const int wg = blockIdx.x, nwg = gridDim.x, nw = blockDim.x >> 6;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int ss = wg % a.SS;
  const int tstep = nwg / a.SS;
  // Tile order: a workgroup starts at tile wg/SS and steps by nwg/SS.
  int t = wg / a.SS;
  int tn = t + tstep;
  const int nch = CHUNK ? a.NCH : 1;
  const int seg = nw * KS;                       // k-blocks per chunk
  const int kb0 = ss * nch * seg + wave * KS;    // this wave's first k-block of chunk 0

  // Per-lane pointer to block 0 of this wave's slice of tile row 0, chunk 0; a tile row is
  // KBp blocks of BLOCK_ELEMS elements.  All weight addresses below are this plus a
  // tile-row offset plus a chunk offset plus a compile-time block offset: no branches
  // around the loads, so the compiler can count outstanding loads exactly.
  const T* wlane = a.W + (size_t)kb0 * BLOCK_ELEMS;
  const size_t row_elems = (size_t)a.KBp * BLOCK_ELEMS;
  const size_t seg_elems = (size_t)seg * BLOCK_ELEMS;

  // weights first: they depend on nothing
  Frag<T> ring[RING];
  {
    const int tf = t < a.NT ? t : 0;
#pragma unroll
    for (int j = 0; j < RING; ++j) ring[j] = frag_load_w(wlane + (size_t)tf * row_elems, j, lane);
  }
  float r = 1.f;
  if constexpr (ROWS16 && NORM) {
    // the workgroup's waves share the 16 rows out (wave w: rows w, w + nw, ...), each adding a row's 256 partials
    // (four per lane, then a butterfly), and pass the scales through LDS
    __shared__ float sc16[16];
    for (int rr = wave; rr < 16; rr += nw) {
      const f32x4 v = *(reinterpret_cast<const f32x4*>(a.ssq_in + (size_t)(a.m0 + min(rr, a.mrows - 1)) * SSQ_PARTS) + lane);
      float sm = (v.x + v.y) + (v.z + v.w);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) sm += __shfl_xor(sm, off);
      if (lane == 0) sc16[rr] = rsqrtf(sm / a.d + a.eps);
    }
    __syncthreads();
    r = sc16[c];
  } else if (NORM) {
    r = row_scale(a.ssq_in, a.m0, a.mrows, a.d, a.eps, lane);
  }
  Frag<T> breg[NB];
  if constexpr (ROWS16) load_acts16<T, NORM, KS>(a, kb0, r, lane, breg);
  else load_acts<T, NORM, KS>(a, kb0, r, lane, breg);
  float sq = 0.f;   // RESIDUAL: this lane's share of the rows' sums of squares

  // Everything requested so far has to be there before the first product anyway (the
  // activations were requested after the ring).  Waiting for all of it here, once, also
  // lets the compiler enter the loop with nothing but the ring in flight, which it needs to
  // keep exact counts inside the loop.
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)

  // One iteration = one K chunk of one output tile (a whole tile unless CHUNK); a single
  // flat loop, so that the loads in flight (weight ring, next chunk's activations) are
  // carried by one loop only and the compiler keeps exact counts of them.
  int ch = 0;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; t < a.NT;) {
    const bool last = !CHUNK || ch + 1 == nch;
    // after the last tile the refill loads go on, harmlessly, into tile 0 (an L2 hit)
    const int tnc = tn < a.NT ? tn : 0;
    const T* wcur = wlane + (size_t)t * row_elems + (size_t)ch * seg_elems;
    const T* wnext = last ? wlane + (size_t)tnc * row_elems : wcur + seg_elems;
    Frag<T> bnext[NB];
    f32x4 hold, gout;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      if constexpr (ROWS16) acc = mma(ring[j % RING], breg[j], acc);
      else acc = mma(ring[j % RING], (j & 1) ? frag_swap_halves(breg[j / 2]) : breg[j / 2], acc);
      const int jn = j + RING;
      if (jn < KS) ring[j % RING] = frag_load_w(wcur, jn, lane);
      else ring[j % RING] = frag_load_w(wnext, jn - KS, lane);
      if (j == 0) {
        // (after the first product, so that the loop starts with the oldest weight load)
        if constexpr (CHUNK) load_acts<T, NORM, KS>(a, kb0 + (last ? 0 : ch + 1) * seg, r, lane, bnext);
        // RESIDUAL: this lane's old h values and gains, fetched ahead of the epilogue (every
        // chunk, unconditionally; only this workgroup writes them, and only after the last chunk)
        if constexpr (EPI == EPI_RESIDUAL) {
          const int n = t * TILE_N + 4 * g;
          hold = *reinterpret_cast<const f32x4*>(a.out + (size_t)(a.m0 + min(c, a.mrows - 1)) * a.ldo + n);
          gout = *reinterpret_cast<const f32x4*>(a.gain_out + n);
        }
      }
      // keep program order: products and loads stay where they are, scalar and vector ALU work may cross
      __builtin_amdgcn_sched_barrier(0x6);
    }
    if constexpr (CHUNK) {
#pragma unroll
      for (int j = 0; j < NB; ++j) breg[j] = bnext[j];
      if (!last) { ++ch; continue; }
    }
    const int buf = it & 1;
    if (wave != 0) red[buf][wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
      for (int w = 1; w < nw; ++w) acc += red[buf][w][lane];
      if (c < a.mrows) {
        const int m = a.m0 + c;
        const int n = t * TILE_N + 4 * g;   // first of this lane's 4 output features
        if (EPI == EPI_PARTIAL) {
          *reinterpret_cast<f32x4*>(a.out + ((size_t)ss * a.Mtot + m) * a.ldo + n) = acc;
        } else {
          const f32x4 hv = hold + acc;
          *reinterpret_cast<f32x4*>(a.out + (size_t)m * a.ldo + n) = hv;
          *reinterpret_cast<f32x4*>(a.hg_out + (size_t)m * a.ldo + n) = hv * gout;
          sq += (hv.x * hv.x + hv.y * hv.y) + (hv.z * hv.z + hv.w * hv.w);
        }
      }
    }
    t = tn;
    tn += tstep;
    ++it; ch = 0;
    acc = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  if (EPI == EPI_RESIDUAL && wave == 0) {
    // this workgroup's partial sum of squares per row; the slots of workgroups that do
    // not exist are zeroed by the ones that do
    sq += __shfl_xor(sq, 16); sq += __shfl_xor(sq, 32);
    if (g == 0 && c < a.mrows) {
      float* dst = a.ssq_out + (size_t)(a.m0 + c) * SSQ_PARTS;
      for (int p = wg; p < SSQ_PARTS; p += nwg) dst[p] = p == wg ? sq : 0.f;
    }
  }
}

// ---------------------------------------------------------------------------
// Any number of rows, in passes of R = 1, 2, 4 or 8 row groups of 16 rows: every weight fragment
// is multiplied with all R groups before the next one is fetched, so the weights are read once
// per 16*R rows.
//   * Four waves per workgroup (one per SIMD, the whole register file each) split the k-blocks
//     of a chunk: KS blocks per wave, 4*KS per chunk.  A wave keeps the activations of its
//     slice for all R groups in registers (R*KS fragments) and fetches the next chunk's while
//     it multiplies the current one.  (Eight waves with half the registers each and no second
//     set were measured 10-15 % slower.)
//   * A workgroup works on a unit of Q tile rows at a time (Q/NACC output tiles): per chunk a
//     wave streams Q*KS weight fragments against R*KS activation fragments, so the activation
//     traffic through L1 (from L2) is R/Q of the weight traffic.  The ring is 2*KS fragments
//     deep and runs across chunks and units.
//   * At the end of a unit the four partial sums of every (tile, row group) pair are added in
//     wave order through LDS; the pairs are shared out over the waves for the epilogue.
//   * A slice whose length is not a multiple of 4*KS ends with waves that have no k-blocks left:
//     they multiply zeros (their loads are redirected to the start of the slice).
// Activations are always stored tensors of type T in the fragment-tiled layout of xt_offset
// (the host runs xn_kernel first for the normalising projections; the attention merge and
// the SwiGLU epilogue below write that layout directly).  Epilogues: partial store, residual
// add + hg + sum-of-squares partial, SwiGLU, LM head (logits + the row statistics of every row
// group, kept per lane and merged over lane groups and waves at the end).
// Work is shared out statically, in one of two ways:
//   * SK = false: whole units, workgroup w takes units w, w + grid, ... (K cut into SS super slices
//     with one partial result each, if the plan has them).  Right when the units fill the chip evenly.
//   * SK = true ("stream-K"): the (unit, chunk) items of the launch form one sequence that is cut
//     into gridDim.x equal ranges, so every workgroup streams the same number of bytes whatever the
//     number of units (320 tile rows over 256 CUs would otherwise cost two rounds for 1.25 rounds
//     of work).  A unit that straddles ranges is finished by whichever of its workgroups arrives
//     last: each stores the sum of its chunks (slot 2*wg + 1 if its part starts the unit, else
//     2*wg) and counts itself in; the one that completes the count adds the parts in workgroup
//     order -- a fixed order, so results do not depend on who came last -- applies the epilogue
//     and clears the counter.  Nobody waits for anybody.  The parts travel as device-scope
//     relaxed atomic stores and loads (they pass the per-XCD L2s), ordered against the counter
//     by a wait for the stores' completion: a device-scope fence would write back and
//     invalidate the whole L2 of the XCD each time, which more than doubled the kernel's time
//     (an acquire-release fetch-add at agent scope on the counter, the memory model's way of saying
//     the same, was timed too: the 32B-shaped step 13.65 -> 16.06 ms).  The fences below are
//     therefore workgroup-scoped: what crosses workgroups does so in sc1 accesses that do not use
//     the non-coherent caches, and vmcnt(0) orders them against the counter on this hardware; under
//     the language's memory model alone this hand-off would be a race.
template <typename T, int EPI, int R, int Q, bool SK>
__global__ void __launch_bounds__(256) gemm_rows_kernel(const GemmArgs<T> a) {
  constexpr int NACC = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr int TT = Q / NACC;                  // output tiles per unit
  constexpr int NWV = 4;                        // waves: one per SIMD, the whole register file each
  constexpr int KS = rows_ks(sizeof(T) == 2, R);   // k-blocks per wave and chunk
  constexpr int NF = Q * KS;                    // weight fragments per wave and chunk
  constexpr int RING = GemmCfg<T>::RING;
  constexpr int P = TT * R;                     // (tile, row group) pairs per unit
  constexpr int PH = P > 8 ? 8 : P;             // pairs per reduction round
  static_assert(Q % NACC == 0 && NF % RING == 0 && P % PH == 0, "unit shape");
  static_assert(R <= 4 || EPI != EPI_LMHEAD, "the LM head's row statistics fit for at most four row groups");
  static_assert(!SK || EPI != EPI_LMHEAD, "the LM head runs whole units");
  constexpr int SLOT = P * NACC * WAVE * 4;     // floats per slot of sk_part
  __shared__ int sk_last;
  __shared__ f32x4 red[NWV][PH][NACC][WAVE];
  __shared__ float wsq[NWV][R][16];
  __shared__ LmStat lmred[EPI == EPI_LMHEAD ? NWV : 1][R][16];
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int ss = SK ? 0 : wg % a.SS, ustep = SK ? 1 : nwg / a.SS;
  const int KBs = SK ? a.KBp : a.KBp / a.SS;    // k-blocks of a super slice
  const int nch = (KBs + NWV * KS - 1) / (NWV * KS);
  const int NU = (a.NT + TT - 1) / TT;
  const size_t row_elems = (size_t)a.KBp * BLOCK_ELEMS;
  const T* wbase = a.W + (size_t)(ss * KBs) * BLOCK_ELEMS;
  // this wave's first k-block of chunk ch inside the slice (0 if it has none), and whether it has one
  auto kofs = [&](int ch) { const int o = (ch * NWV + wave) * KS; return o < KBs ? o : 0; };
  auto kval = [&](int ch) { return (ch * NWV + wave) * KS < KBs; };
  // tile row q of unit u (tiles beyond the last one re-read it; their results are dropped)
  auto wptr = [&](int u, int q, int ch) {
    const int t = min(u * TT + q / NACC, a.NT - 1);
    return wbase + (size_t)(t * NACC + q % NACC) * row_elems + (size_t)kofs(ch) * BLOCK_ELEMS;
  };
  // activations in the fragment-tiled layout (xt_offset): every load is 1 KiB of consecutive memory
  // (building them from the fp32 residual rows on load, as gemm_stream_kernel does for 8 rows,
  // was measured slower than a stored copy at every width: those loads are 16 separate rows)
  auto load_b = [&](Frag<T> (&dst)[R][KS], int ch) {
    const int kb = ss * KBs + kofs(ch), KBx = a.ldx >> 5, glast = (a.mrows - 1) >> 4;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const T* xp = a.X + ((size_t)((a.m0 >> 4) + min(r, glast)) * KBx + kb) * BLOCK_ELEMS + lane * 8;
#pragma unroll
      for (int j = 0; j < KS; ++j) dst[r][j] = frag_load_row(xp + j * BLOCK_ELEMS);
    }
  };
  auto take_b = [&](Frag<T> (&dst)[R][KS], const Frag<T> (&src)[R][KS], bool valid) {
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        dst[r][j] = src[r][j];
        if (!valid) frag_zero(dst[r][j]);
      }
  };

  // SK: items it .. it1-1 of the sequence (unit 0 chunk 0, unit 0 chunk 1, ...) are this workgroup's;
  // ch0 = the chunk at which its part of the current unit starts
  const int IT = NU * nch;
  int u = wg / a.SS, ch = 0, it = 0, it1 = 0, ch0 = 0;
  if constexpr (SK) {
    it = (int)((long)IT * wg / nwg); it1 = (int)((long)IT * (wg + 1) / nwg);
    u = it / nch; ch = it % nch; ch0 = ch;
  }
  auto more = [&]() { return SK ? it < it1 : u < NU; };
  Frag<T> ring[RING];
  {
    const int uf = more() ? u : 0, cf = more() ? ch : 0;
#pragma unroll
    for (int i = 0; i < RING; ++i) ring[i] = frag_load_w(wptr(uf, i / KS, cf), i % KS, lane);
  }
  Frag<T> breg[R][KS], bnext[R][KS];
  load_b(bnext, ch);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): enter the loop with nothing but known loads in flight
  take_b(breg, bnext, kval(ch));

  f32x4 acc[Q][R];
  float sq[R];
  // LM head: running statistics of this lane's row in every row group
  LmStat st[EPI == EPI_LMHEAD ? R : 1];
  int draft[R]; uint32_t pb[R], pj[R]; uint64_t stepv = 0;
  if constexpr (EPI == EPI_LMHEAD) {
    stepv = a.lm.step + *a.lm.commits;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      lm_init(st[r]);
      const int m = a.m0 + min(16 * r + c, a.mrows - 1);
      pb[r] = m / a.lm.k; pj[r] = m % a.lm.k;
      draft[r] = ((int)pj[r] + 1 < a.lm.k) ? a.lm.window[m + 1] : -1;
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    sq[r] = 0.f;
#pragma unroll
    for (int q = 0; q < Q; ++q) acc[q][r] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // epilogue of pair p = (tile tt of unit u, row group r) with the complete sums v
  auto epilogue = [&](int p, const f32x4 (&v)[NACC]) {
    const int tt = p / R, r = p % R;
    const int t = u * TT + tt, mr = 16 * r + c;
    if (t < a.NT && mr < a.mrows) {
      const int m = a.m0 + mr;
      const int n = t * TILE_N + 4 * g;
      if (EPI == EPI_PARTIAL) {
        *reinterpret_cast<f32x4*>(a.out + ((size_t)ss * a.Mtot + m) * a.ldo + n) = v[0];
      } else if (EPI == EPI_RESIDUAL) {
        f32x4* hp = reinterpret_cast<f32x4*>(a.out + (size_t)m * a.ldo + n);
        const f32x4 hv = *hp + v[0];
        *hp = hv;
        *reinterpret_cast<f32x4*>(a.hg_out + (size_t)m * a.ldo + n) = hv * *reinterpret_cast<const f32x4*>(a.gain_out + n);
        const float e = (hv.x * hv.x + hv.y * hv.y) + (hv.z * hv.z + hv.w * hv.w);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) sq[rr] += rr == r ? e : 0.f;
      } else if (EPI == EPI_LMHEAD) {
        // (the logits themselves only if somebody will read them: the caller, or a residual draw under dense q)
        if (a.out) *reinterpret_cast<f32x4*>(a.out + (size_t)m * a.ldo + n) = v[0];
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
          if (rr == r) lm_update(st[EPI == EPI_LMHEAD ? rr : 0], v[0], n, a.N, draft[rr], pb[rr], pj[rr], stepv, a.lm);
      } else {   // EPI_SWIGLU
        f32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float gt = v[0][i], up = v[NACC - 1][i];
          o[i] = (n + i < a.N) ? gt / (1.f + expf(-gt)) * up : 0.f;
        }
        st_round4(a.act_tiled ? a.act + xt_offset(m, n, a.ldact) : a.act + (size_t)m * a.ldact + n, o);
      }
    }
  };
  // SK, residual projections: the finished unit's sums of squares go to slot `unit` of the rows'
  // partials (a unit is finished by whichever workgroup arrives last, so a slot per workgroup
  // would make the order of the consumer's sum, and its last bit, depend on the timing)
  auto flush_sq = [&](int unit) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float v = sq[r];
      v += __shfl_xor(v, 16); v += __shfl_xor(v, 32);
      if (g == 0) wsq[wave][r][c] = v;
      sq[r] = 0.f;
    }
    __syncthreads();
    if (wave == 0) {
      for (int rg = g; rg < R; rg += 4) {
        const int mr = 16 * rg + c;
        if (mr < a.mrows) {
          float v = wsq[0][rg][c];
#pragma unroll
          for (int w = 1; w < NWV; ++w) v += wsq[w][rg][c];
          a.ssq_out[(size_t)(a.m0 + mr) * SSQ_PARTS + unit] = v;
        }
      }
    }
    __syncthreads();
  };
  while (more()) {
    const bool uend = ch + 1 == nch;                            // last chunk of the unit
    const bool last = SK ? (uend || it + 1 == it1) : uend;      // ... of this workgroup's part of it
    int un, chn;
    if constexpr (SK) {
      const bool fin = it + 1 == it1;                           // (the refill loads then go on into unit 0)
      un = fin ? 0 : (uend ? u + 1 : u); chn = (fin || uend) ? 0 : ch + 1;
    } else {
      un = last ? u + ustep : u; chn = last ? 0 : ch + 1;
    }
    const int unc = un < NU ? un : 0;   // after the last unit the refill loads go on, harmlessly, into unit 0
    const T *wc[Q], *wn[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) { wc[q] = wptr(u, q, ch); wn[q] = wptr(unc, q, chn); }
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      const int q = i / KS, j = i % KS;
#pragma unroll
      for (int r = 0; r < R; ++r) acc[q][r] = mma(ring[i % RING], breg[r][j], acc[q][r]);
      const int in = i + RING;
      if (in < NF) ring[i % RING] = frag_load_w(wc[in / KS], in % KS, lane);
      else ring[i % RING] = frag_load_w(wn[(in - NF) / KS], (in - NF) % KS, lane);
      if (i == 0) load_b(bnext, chn);   // (after the first product, so that the loop starts with the oldest weight load)
      __builtin_amdgcn_sched_barrier(0x6);
    }
    take_b(breg, bnext, kval(chn));
    if (!last) { ++ch; if constexpr (SK) ++it; continue; }
    // this workgroup's part of the unit is done: add the four partial sums of every pair, PH pairs
    // per round; a whole unit goes through the epilogue, a part of one into this workgroup's slot
    const bool whole = !SK || (ch0 == 0 && uend);
    float* slot = nullptr;
    if constexpr (SK) slot = a.sk_part + (size_t)(2 * wg + (ch0 == 0 ? 1 : 0)) * SLOT + lane * 4;
#pragma unroll
    for (int h = 0; h < P / PH; ++h) {
#pragma unroll
      for (int pp = 0; pp < PH; ++pp) {
        const int p = h * PH + pp, tt = p / R, r = p % R;
#pragma unroll
        for (int s = 0; s < NACC; ++s) red[wave][pp][s][lane] = acc[tt * NACC + s][r];
      }
      __syncthreads();
      for (int pp = wave; pp < PH; pp += NWV) {
        const int p = h * PH + pp;
        f32x4 v[NACC];
#pragma unroll
        for (int s = 0; s < NACC; ++s) {
          v[s] = red[0][pp][s][lane];
#pragma unroll
          for (int w = 1; w < NWV; ++w) v[s] += red[w][pp][s][lane];
        }
        if (whole) {
          epilogue(p, v);
        } else {
#pragma unroll
          for (int s = 0; s < NACC; ++s) st_device(slot + (p * NACC + s) * (WAVE * 4), v[s]);
        }
      }
      __syncthreads();
    }
    if constexpr (SK && EPI == EPI_RESIDUAL) {
      if (whole) flush_sq(u);
    }
    if constexpr (SK) {
      if (!whole) {
        // first and last workgroup with items of unit u: those whose ranges hold its first and last item
        const int fw = (int)((((long)u * nch + 1) * nwg - 1) / IT), lw = (int)(((long)(u + 1) * nch * nwg - 1) / IT);
        // this workgroup's part is in device memory before it is counted: every wave waits for its stores
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0) {
          const int arrived = atomicAdd(a.sk_cnt + u, 1);
          sk_last = arrived == lw - fw;
          if (arrived == lw - fw) atomicExch(a.sk_cnt + u, 0);   // (for the next launch)
        }
        __syncthreads();
        if (sk_last) {
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
          for (int p = wave; p < P; p += NWV) {
            f32x4 v[NACC];
            for (int w = fw; w <= lw; ++w) {
              // workgroup w's part starts the unit iff its range starts at or before the unit's first item
              const int w0 = (int)((long)IT * w / nwg);
              const float* src = a.sk_part + (size_t)(2 * w + (w0 <= u * nch ? 1 : 0)) * SLOT + lane * 4;
#pragma unroll
              for (int s = 0; s < NACC; ++s) {
                const f32x4 x = ld_device(src + (p * NACC + s) * (WAVE * 4));
                v[s] = w == fw ? x : v[s] + x;
              }
            }
            epilogue(p, v);
          }
          if constexpr (EPI == EPI_RESIDUAL) flush_sq(u);
        }
      }
      ch0 = 0; ++it;
    }
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
      for (int r = 0; r < R; ++r) acc[q][r] = f32x4{0.f, 0.f, 0.f, 0.f};
    u = SK ? (uend ? u + 1 : u) : un; ch = 0;
  }

  if constexpr (EPI == EPI_LMHEAD) {
    // this workgroup's statistics per row: the four lane groups of a row, then the waves in order
#pragma unroll
    for (int r = 0; r < R; ++r) {
      lm_merge(st[r], lm_shfl_xor(st[r], 16));
      lm_merge(st[r], lm_shfl_xor(st[r], 32));
      if (g == 0) lmred[wave][r][c] = st[r];
    }
    __syncthreads();
    if (wave == 0 && g < R) {   // lane group g takes row group g (R <= 4 here)
      const int mr = 16 * g + c;
      if (mr < a.mrows) {
        LmStat s = lmred[0][g][c];
        for (int w = 1; w < NWV; ++w) lm_merge(s, lmred[w][g][c]);
        a.lm.stats[(size_t)wg * a.Mtot + a.m0 + mr] = s;
      }
    }
  }

  if constexpr (SK && EPI == EPI_RESIDUAL) {
    // one slot per unit was filled above; the slots beyond the units are zeroed
    static_assert(R * 16 <= 256, "one thread per row");
    if ((int)threadIdx.x < a.mrows)
      for (int p = NU + wg; p < SSQ_PARTS; p += nwg) a.ssq_out[(size_t)(a.m0 + threadIdx.x) * SSQ_PARTS + p] = 0.f;
  } else if (EPI == EPI_RESIDUAL) {
    // this workgroup's partial sum of squares per row: lane groups, then waves in order
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float v = sq[r];
      v += __shfl_xor(v, 16); v += __shfl_xor(v, 32);
      if (g == 0) wsq[wave][r][c] = v;
    }
    __syncthreads();
    if (wave == 0) {
      for (int rg = g; rg < R; rg += 4) {   // lane group g takes row groups g, g + 4
        const int mr = 16 * rg + c;
        if (mr < a.mrows) {
          float v = wsq[0][rg][c];
#pragma unroll
          for (int w = 1; w < NWV; ++w) v += wsq[w][rg][c];
          float* dst = a.ssq_out + (size_t)(a.m0 + mr) * SSQ_PARTS;
          for (int p = wg; p < SSQ_PARTS; p += nwg) dst[p] = p == wg ? v : 0.f;
        }
      }
    }
  }
}

// Gate/up projection, bf16: every pass of more than 16 rows (R = 2, 4 or 8 row groups) and, at widths whose
// tile rows gemm_rows_kernel cannot share out in full rounds, the smaller ones too (R = 1).  In
// gemm_rows_kernel every wave owns a K slice and therefore its own activations: R*KS fragments
// per Q*KS weight fragments, twice the weight bytes at 128 rows, all of it through the CU's L1.
// Here the four waves of a workgroup own four different units of Q = 4 tile rows (two gate/up
// tile pairs) and walk K together, KC = 4 k-blocks at a time: the R*KC activation fragments of a
// chunk are fetched once per workgroup (a quarter each, one chunk ahead, into registers), staged
// through one of two LDS buffers (one barrier per chunk) and read from there by every wave, so the
// activation bytes through L1 fall to R/16 of the weight bytes.  A wave holds complete sums (no
// reduction between waves); its 16 weight fragments per chunk are exactly one revolution of the
// ring, consumed and re-requested in the same order (k-block major, so that only R activation
// fragments are live at a time).  Workgroup w takes the groups of four units w, w + grid, ...
// Requires KBp % 4 == 0; the activations are the stored RMSNorm output in the fragment-tiled layout.
template <typename T, int R>
__global__ void __launch_bounds__(256) gemm_wide_swiglu_kernel(const GemmArgs<T> a) {
  static_assert(sizeof(T) == 2, "bf16 only");
  constexpr int Q = 4, KC = 4, RING = Q * KC, AF = R * KC / 4;
  static_assert(RING == GemmCfg<T>::RING, "one ring revolution per chunk");
  __shared__ u32x4 xs[2][R * KC][WAVE];
  const int wg = blockIdx.x, nwg = gridDim.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int nch = a.KBp / KC;
  const int NTR = 2 * a.NT;                              // tile rows (gate and up rows of a pair are neighbours)
  const int NSU = (NTR + 4 * Q - 1) / (4 * Q);           // groups of four units
  const size_t row_elems = (size_t)a.KBp * BLOCK_ELEMS;
  const int KBx = a.ldx >> 5, glast = (a.mrows - 1) >> 4;
  // tile row q of this wave's unit in group su (rows beyond the last one re-read it; their results are dropped)
  auto wptr = [&](int su, int q, int ch) {
    return a.W + (size_t)min((su * 4 + wave) * Q + q, NTR - 1) * row_elems + (size_t)ch * KC * BLOCK_ELEMS;
  };
  // this wave's quarter of the activation fragments (row group r, k-block j of chunk ch): fragment f = r * KC + j
  auto fetch_x = [&](u32x4 (&dst)[AF], int ch) {
#pragma unroll
    for (int i = 0; i < AF; ++i) {
      const int f = wave * AF + i, r = f / KC, j = f % KC;
      const T* xp = a.X + ((size_t)((a.m0 >> 4) + min(r, glast)) * KBx + ch * KC + j) * BLOCK_ELEMS + lane * 8;
      dst[i] = *reinterpret_cast<const u32x4*>(xp);
    }
  };

  int su = wg, ch = 0;
  Frag<T> ring[RING];                                    // ring[j * Q + q] = fragment (tile row q, k-block j)
  {
    const int sf = su < NSU ? su : 0;
#pragma unroll
    for (int i = 0; i < RING; ++i) ring[i] = frag_load_w(wptr(sf, i % Q, 0), i / Q, lane);
  }
  u32x4 xpre[AF];
  fetch_x(xpre, 0);
  f32x4 acc[Q][R];
#pragma unroll
  for (int q = 0; q < Q; ++q)
#pragma unroll
    for (int r = 0; r < R; ++r) acc[q][r] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int it = 0; su < NSU; ++it) {
    const bool uend = ch + 1 == nch;
    const int sun = uend ? su + nwg : su, chn = uend ? 0 : ch + 1;
    const int sunc = sun < NSU ? sun : 0;                // after the last group the refill loads go on, harmlessly, into group 0
    const T* wn[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) wn[q] = wptr(sunc, q, chn);
    u32x4 (&buf)[R * KC][WAVE] = xs[it & 1];
#pragma unroll
    for (int i = 0; i < AF; ++i) buf[wave * AF + i][lane] = xpre[i];
    fetch_x(xpre, chn);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KC; ++j) {
      Frag<T> b[R];
#pragma unroll
      for (int r = 0; r < R; ++r) b[r].v = buf[r * KC + j][lane];
#pragma unroll
      for (int q = 0; q < Q; ++q) {
#pragma unroll
        for (int r = 0; r < R; ++r) acc[q][r] = mma(ring[j * Q + q], b[r], acc[q][r]);
        ring[j * Q + q] = frag_load_w(wn[q], j, lane);
        __builtin_amdgcn_sched_barrier(0x6);             // products and loads keep their program order
      }
    }
    if (uend) {
      // SwiGLU epilogue of this wave's two tile pairs x R row groups
#pragma unroll
      for (int tt = 0; tt < Q / 2; ++tt) {
        const int t = (su * 4 + wave) * (Q / 2) + tt;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int mr = 16 * r + c;
          if (t < a.NT && mr < a.mrows) {
            const int m = a.m0 + mr, n = t * TILE_N + 4 * g;
            f32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float gt = acc[2 * tt][r][i], up = acc[2 * tt + 1][r][i];
              o[i] = (n + i < a.N) ? gt / (1.f + expf(-gt)) * up : 0.f;
            }
            st_round4(a.act_tiled ? a.act + xt_offset(m, n, a.ldact) : a.act + (size_t)m * a.ldact + n, o);
          }
          acc[2 * tt][r] = f32x4{0.f, 0.f, 0.f, 0.f};
          acc[2 * tt + 1][r] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
    }
    su = sun; ch = chn;
  }
}

// LM head of passes of more than 32 rows (R = 4 or 8 row groups), bf16: gemm_wide_swiglu_kernel's form -- four
// units of Q = 4 vocabulary tiles per workgroup, one per wave, on one set of activations staged through LDS --
// with gemm_rows_kernel's LM-head epilogue: logits stored once if anybody reads them, and the row statistics
// kept per lane for every row group, merged over lane groups and waves (in that fixed order) at the end into
// stats[workgroup][row].  gemm_rows_kernel holds statistics for at most four row groups and reads its
// activations per wave, so a 128-row window cost it two passes over the matrix; here it is one.
// Requires KBp % 4 == 0; the activations are the stored final RMSNorm output in the fragment-tiled layout.
template <typename T, int R>
__global__ void __launch_bounds__(256) gemm_wide_lmhead_kernel(const GemmArgs<T> a) {
  static_assert(sizeof(T) == 2, "bf16 only");
  constexpr int Q = 4, KC = 4, RING = Q * KC, AF = R * KC / 4, NWV = 4;
  static_assert(RING == GemmCfg<T>::RING, "one ring revolution per chunk");
  __shared__ u32x4 xs[2][R * KC][WAVE];
  // running statistics of every thread's row in every row group: touched only at the end of a unit, so they live
  // in LDS and the registers stay with the accumulators
  __shared__ LmStat lst[R][NWV * WAVE];
  __shared__ LmStat lmred[NWV][R][16];
  const int wg = blockIdx.x, nwg = gridDim.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int nch = a.KBp / KC;
  const int NSU = (a.NT + 4 * Q - 1) / (4 * Q);          // groups of four units
  const size_t row_elems = (size_t)a.KBp * BLOCK_ELEMS;
  const int KBx = a.ldx >> 5, glast = (a.mrows - 1) >> 4;
  // tile q of this wave's unit in group su (tiles beyond the last one re-read it; their results are dropped)
  auto wptr = [&](int su, int q, int ch) {
    return a.W + (size_t)min((su * 4 + wave) * Q + q, a.NT - 1) * row_elems + (size_t)ch * KC * BLOCK_ELEMS;
  };
  auto fetch_x = [&](u32x4 (&dst)[AF], int ch) {
#pragma unroll
    for (int i = 0; i < AF; ++i) {
      const int f = wave * AF + i, r = f / KC, j = f % KC;
      const T* xp = a.X + ((size_t)((a.m0 >> 4) + min(r, glast)) * KBx + ch * KC + j) * BLOCK_ELEMS + lane * 8;
      dst[i] = *reinterpret_cast<const u32x4*>(xp);
    }
  };

  int su = wg, ch = 0;
  Frag<T> ring[RING];                                    // ring[j * Q + q] = fragment (tile q, k-block j)
  {
    const int sf = su < NSU ? su : 0;
#pragma unroll
    for (int i = 0; i < RING; ++i) ring[i] = frag_load_w(wptr(sf, i % Q, 0), i / Q, lane);
  }
  u32x4 xpre[AF];
  fetch_x(xpre, 0);
  f32x4 acc[Q][R];
  const uint64_t stepv = a.lm.step + *a.lm.commits;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    LmStat s0;
    lm_init(s0);
    lst[r][threadIdx.x] = s0;
#pragma unroll
    for (int q = 0; q < Q; ++q) acc[q][r] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  for (int it = 0; su < NSU; ++it) {
    const bool uend = ch + 1 == nch;
    const int sun = uend ? su + nwg : su, chn = uend ? 0 : ch + 1;
    const int sunc = sun < NSU ? sun : 0;                // after the last group the refill loads go on, harmlessly, into group 0
    const T* wn[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) wn[q] = wptr(sunc, q, chn);
    u32x4 (&buf)[R * KC][WAVE] = xs[it & 1];
#pragma unroll
    for (int i = 0; i < AF; ++i) buf[wave * AF + i][lane] = xpre[i];
    fetch_x(xpre, chn);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KC; ++j) {
      Frag<T> b[R];
#pragma unroll
      for (int r = 0; r < R; ++r) b[r].v = buf[r * KC + j][lane];
#pragma unroll
      for (int q = 0; q < Q; ++q) {
#pragma unroll
        for (int r = 0; r < R; ++r) acc[q][r] = mma(ring[j * Q + q], b[r], acc[q][r]);
        ring[j * Q + q] = frag_load_w(wn[q], j, lane);
        __builtin_amdgcn_sched_barrier(0x6);             // products and loads keep their program order
      }
    }
    if (uend) {
      // (compile-time loops: the accumulators must keep constant indices whatever the unroller thinks of the body's size)
      static_for<R>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        const int mr = 16 * r + c;
        if (mr < a.mrows) {
          const int m = a.m0 + mr;
          const uint32_t pb = m / a.lm.k, pj = m % a.lm.k;
          const int draft = ((int)pj + 1 < a.lm.k) ? a.lm.window[m + 1] : -1;
          LmStat s = lst[r][threadIdx.x];
          static_for<Q>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            const int t = (su * 4 + wave) * Q + q, n = t * TILE_N + 4 * g;
            if (t < a.NT) {
              // (the logits themselves only if somebody will read them: the caller, or a residual draw under dense q)
              if (a.out) *reinterpret_cast<f32x4*>(a.out + (size_t)m * a.ldo + n) = acc[q][r];
              lm_update(s, acc[q][r], n, a.N, draft, pb, pj, stepv, a.lm);
            }
          });
          lst[r][threadIdx.x] = s;
        }
        static_for<Q>([&](auto qc) { acc[decltype(qc)::value][r] = f32x4{0.f, 0.f, 0.f, 0.f}; });
      });
    }
    su = sun; ch = chn;
  }

  // this workgroup's statistics per row: the four lane groups of a row, then the waves in order
#pragma unroll
  for (int r = 0; r < R; ++r) {
    LmStat s = lst[r][threadIdx.x];
    lm_merge(s, lm_shfl_xor(s, 16));
    lm_merge(s, lm_shfl_xor(s, 32));
    if (g == 0) lmred[wave][r][c] = s;
  }
  __syncthreads();
  if (wave == 0) {
    for (int rg = g; rg < R; rg += 4) {                  // lane group g takes row groups g, g + 4
      const int mr = 16 * rg + c;
      if (mr < a.mrows) {
        LmStat s = lmred[0][rg][c];
        for (int w = 1; w < NWV; ++w) lm_merge(s, lmred[w][rg][c]);
        a.lm.stats[(size_t)wg * a.Mtot + a.m0 + mr] = s;
      }
    }
  }
}

// Output and down projection of 128-row passes (R = 8) and down projection of 64-row passes (R = 4), bf16:
// gemm_wide_swiglu_kernel's form -- four
// units of 4 tile rows per workgroup on one set of activations staged through LDS -- for matrices
// whose 32 groups of 16 tile rows do not fill the chip: K is cut into gridDim.y slices of whole chunks,
// workgroup (x, y) multiplies group x with slice y and stores its sums as part y of the result,
// part[y][row][feature] (plain stores); resid_reduce_kernel adds the parts in slice order and
// applies the residual epilogue.  Requires KBp % 4 == 0 and no empty slice (the host sees to both).
template <typename T, int R>
__global__ void __launch_bounds__(256) gemm_wide_slice_kernel(const GemmArgs<T> a, float* __restrict__ part) {
  static_assert(sizeof(T) == 2, "bf16 only");
  constexpr int Q = 4, KC = 4, RING = Q * KC, AF = R * KC / 4;
  static_assert(RING == GemmCfg<T>::RING, "one ring revolution per chunk");
  __shared__ u32x4 xs[2][R * KC][WAVE];
  const int gi = blockIdx.x, ss = blockIdx.y, SSW = gridDim.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, c = lane & 15, g = lane >> 4;
  const int nch = a.KBp / KC, cps = (nch + SSW - 1) / SSW;
  const int c0 = ss * cps, c1 = min(nch, c0 + cps);      // this slice's chunks
  const size_t row_elems = (size_t)a.KBp * BLOCK_ELEMS;
  const int KBx = a.ldx >> 5, glast = (a.mrows - 1) >> 4;
  const T* wrow[Q];                                      // tile rows beyond the last one re-read it; their results are dropped
#pragma unroll
  for (int q = 0; q < Q; ++q) wrow[q] = a.W + (size_t)min((gi * 4 + wave) * Q + q, a.NT - 1) * row_elems;
  auto fetch_x = [&](u32x4 (&dst)[AF], int ch) {
#pragma unroll
    for (int i = 0; i < AF; ++i) {
      const int f = wave * AF + i, r = f / KC, j = f % KC;
      const T* xp = a.X + ((size_t)((a.m0 >> 4) + min(r, glast)) * KBx + ch * KC + j) * BLOCK_ELEMS + lane * 8;
      dst[i] = *reinterpret_cast<const u32x4*>(xp);
    }
  };
  Frag<T> ring[RING];                                    // ring[j * Q + q] = fragment (tile row q, k-block j)
#pragma unroll
  for (int i = 0; i < RING; ++i) ring[i] = frag_load_w(wrow[i % Q] + (size_t)c0 * KC * BLOCK_ELEMS, i / Q, lane);
  u32x4 xpre[AF];
  fetch_x(xpre, c0);
  f32x4 acc[Q][R];
#pragma unroll
  for (int q = 0; q < Q; ++q)
#pragma unroll
    for (int r = 0; r < R; ++r) acc[q][r] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int ch = c0; ch < c1; ++ch) {
    const int chn = ch + 1 < c1 ? ch + 1 : c0;           // after the last chunk the refill loads go on, harmlessly, into the first
    u32x4 (&buf)[R * KC][WAVE] = xs[(ch - c0) & 1];
#pragma unroll
    for (int i = 0; i < AF; ++i) buf[wave * AF + i][lane] = xpre[i];
    fetch_x(xpre, chn);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KC; ++j) {
      Frag<T> b[R];
#pragma unroll
      for (int r = 0; r < R; ++r) b[r].v = buf[r * KC + j][lane];
#pragma unroll
      for (int q = 0; q < Q; ++q) {
#pragma unroll
        for (int r = 0; r < R; ++r) acc[q][r] = mma(ring[j * Q + q], b[r], acc[q][r]);
        ring[j * Q + q] = frag_load_w(wrow[q] + (size_t)chn * KC * BLOCK_ELEMS, j, lane);
        __builtin_amdgcn_sched_barrier(0x6);             // products and loads keep their program order
      }
    }
  }
  float* dst = part + (size_t)ss * a.mrows * a.ldo;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int t = (gi * 4 + wave) * Q + q;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int mr = 16 * r + c;
      if (t < a.NT && mr < a.mrows) *reinterpret_cast<f32x4*>(dst + (size_t)mr * a.ldo + t * TILE_N + 4 * g) = acc[q][r];
    }
  }
}

// h[row] += sum of the nparts parts (in order); hg = h * gain of the next norm; one sum-of-squares partial per row
// and workgroup.  Workgroup w owns features 32w .. 32w+31 (ldo / 32 <= SSQ_PARTS workgroups); thread = (row mod 32, four features).
__global__ void __launch_bounds__(256) resid_reduce_kernel(const float* __restrict__ part, int nparts, float* __restrict__ h,
                                                           float* __restrict__ hg, const float* __restrict__ gain,
                                                           float* __restrict__ ssq, int m0, int mrows, int ldo) {
  const int wg = blockIdx.x, nwg = gridDim.x, n = 32 * wg + 4 * (threadIdx.x & 7);
  const f32x4 gn = *reinterpret_cast<const f32x4*>(gain + n);
  // four rows per thread at a time, all their loads requested before the first sum (rows beyond the pass re-read the last one)
  for (int mb = threadIdx.x >> 3; mb < ((mrows + 127) & ~127); mb += 128) {
    f32x4 v[4], hv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int mr = min(mb + 32 * u, mrows - 1);
      v[u] = *reinterpret_cast<const f32x4*>(part + (size_t)mr * ldo + n);
      hv[u] = *reinterpret_cast<const f32x4*>(h + (size_t)(m0 + mr) * ldo + n);
    }
    for (int p = 1; p < nparts; ++p) {
      f32x4 x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = *reinterpret_cast<const f32x4*>(part + ((size_t)p * mrows + min(mb + 32 * u, mrows - 1)) * ldo + n);
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] += x[u];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int mr = mb + 32 * u;
      float sq = 0.f;
      if (mr < mrows) {
        const f32x4 r = hv[u] + v[u];
        *reinterpret_cast<f32x4*>(h + (size_t)(m0 + mr) * ldo + n) = r;
        *reinterpret_cast<f32x4*>(hg + (size_t)(m0 + mr) * ldo + n) = r * gn;
        sq = (r.x * r.x + r.y * r.y) + (r.z * r.z + r.w * r.w);
      }
      sq += __shfl_xor(sq, 1); sq += __shfl_xor(sq, 2); sq += __shfl_xor(sq, 4);
      if ((threadIdx.x & 7) == 0 && mr < mrows) {
        float* dst = ssq + (size_t)(m0 + mr) * SSQ_PARTS;
        for (int p = wg; p < SSQ_PARTS; p += nwg) dst[p] = p == wg ? sq : 0.f;
      }
    }
  }
}

// xn[row][:] = T(hg[row][:] * rsqrt(mean(h[row]^2) + eps)) for rows m0 + blockIdx.x / nsl: the
// RMSNorm output as a stored tensor in the fragment-tiled layout, for gemm_rows_kernel.
// 256 threads; thread p adds slot p of the row's sum-of-squares partials; the nsl workgroups
// of a row (each adds the partials for itself) take every nsl-th group of 1024 columns.
template <typename T>
__global__ void __launch_bounds__(256) xn_kernel(const float* __restrict__ hg, const float* __restrict__ ssq,
                                                 T* __restrict__ xn, int ld, int m0, int nsl, float d, float eps) {
  __shared__ float part[4];
  const int row = m0 + blockIdx.x / nsl, sl = blockIdx.x % nsl;
  float s = ssq[(size_t)row * SSQ_PARTS + threadIdx.x];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  const float r = rsqrtf(((part[0] + part[1]) + (part[2] + part[3])) / d + eps);
  const float* src = hg + (size_t)row * ld;
  for (int i = 4 * (threadIdx.x + 256 * sl); i < ld; i += 4 * 256 * nsl) {
    st_round4(xn + xt_offset(row, i, ld), *reinterpret_cast<const f32x4*>(src + i) * r);
  }
}

}  // namespace dbl
