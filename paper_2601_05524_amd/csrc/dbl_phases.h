// The per-layer steps between the projections: q/k-norm + RoPE + KV append, split-KV
// GQA attention, combine.  Each is a device function over a "task" index (one wave per
// task) with a thin kernel around it.
#pragma once
#include "dbl_dev.h"

namespace dbl {

// ------------------------------------------------------------------ reductions

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// sum over a workgroup (blockDim.x multiple of 64, <= 1024); every thread gets the
// result; scratch must hold 16 floats
__device__ __forceinline__ float block_sum(float v, float* scratch) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < nw; ++w) t += scratch[w];
  return t;
}

// ---------------------------------------------- q/k norm + RoPE + KV append

// One wave per task = (row m, head hh) with hh in [0, H + 2*Hkv): q heads, then k
// heads, then v heads.  Sums the QKV partials, applies the optional per-head RMSNorm
// and the rotary embedding (pairs (i, i+hd/2); cos/sin from the fp32 table at the
// row's position kv_len[b] + j), rounds to T, and writes
//   q  -> qbuf[b][kvh][j*g + hg][hd]
//   k  -> kc[layer][b][kvh] at kc_offset(pos, dim)     (MFMA-tiled, see dbl_dev.h)
//   v  -> vt[layer][b][kvh] at vt_offset(pos, dim)
template <typename T>
struct RopeArgs {
  const float* qkv; int nparts, Mtot, ldq;   // partials [nparts][Mtot][ldq]
  const float *gq, *gk;                      // per-head gains (qk_norm) or nullptr
  const float *cosT, *sinT;                  // [max_ctx][hd/2]
  const int32_t* kv_len;                     // [B]
  T *qbuf, *kc, *vt;                         // kc / vt already offset to the layer
  int k, H, Hkv, hd, max_ctx, max_batch, qrows_pad;
  float eps;
};

template <typename T>
__device__ __forceinline__ void rope_task(const RopeArgs<T>& a, int task) {
  const int lane = threadIdx.x & 63;
  const int heads = a.H + 2 * a.Hkv;
  const int m = task / heads, hh = task % heads;
  const int b = m / a.k, j = m % a.k;
  const int pos = a.kv_len[b] + j;
  if (pos >= a.max_ctx) return;   // capacity guard; the host refuses such calls
  const int hd = a.hd, half = hd >> 1;
  // lane i < half holds the pair (i, i+half); hd = 128 -> 64 lanes, hd = 64 -> 32 lanes
  const bool act = lane < half;
  float x0 = 0.f, x1 = 0.f;
  if (act) {
    for (int p = 0; p < a.nparts; ++p) {
      const float* src = a.qkv + ((size_t)p * a.Mtot + m) * a.ldq + (size_t)hh * hd;
      x0 += *(src + lane); x1 += *(src + lane + half);
    }
  }
  const bool is_q = hh < a.H, is_k = !is_q && hh < a.H + a.Hkv;
  if (!is_q && !is_k) {  // v head: no norm, no rotation
    if (act) {
      const int kvh = hh - a.H - a.Hkv;
      T* dst = a.vt + (size_t)(b * a.Hkv + kvh) * a.max_ctx * hd;
      st_round1(dst + vt_offset(pos, lane, hd), x0);
      st_round1(dst + vt_offset(pos, lane + half, hd), x1);
    }
    return;
  }
  const float* gn = is_q ? a.gq : a.gk;
  if (gn) {
    float ss = wave_sum(act ? x0 * x0 + x1 * x1 : 0.f);
    const float r = rsqrtf(ss / (float)hd + a.eps);
    if (act) { x0 = x0 * r * gn[lane]; x1 = x1 * r * gn[lane + half]; }
  }
  if (act) {
    const float cs = a.cosT[(size_t)pos * half + lane], sn = a.sinT[(size_t)pos * half + lane];
    const float y0 = x0 * cs - x1 * sn, y1 = x0 * sn + x1 * cs;
    if (is_q) {
      const int g = a.H / a.Hkv, kvh = hh / g, hg = hh % g;
      T* dst = a.qbuf + ((size_t)(b * a.Hkv + kvh) * a.qrows_pad + (j * g + hg)) * hd;
      st_round1(dst + lane, y0);
      st_round1(dst + lane + half, y1);
    } else {
      const int kvh = hh - a.H;
      T* dst = a.kc + (size_t)(b * a.Hkv + kvh) * a.max_ctx * hd;
      st_round1(dst + kc_offset(pos, lane, hd), y0);
      st_round1(dst + kc_offset(pos, lane + half, hd), y1);
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256) rope_kv_kernel(const RopeArgs<T> a) {
  const int task = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (task >= a.Mtot * (a.H + 2 * a.Hkv)) return;
  rope_task<T>(a, task);
}

// ------------------------------------------------------------ GQA attention

// Split-KV ("flash-decode") attention for a short query window.  The g query heads
// of one KV head and the k window rows form g*k query rows (row = j*g + hg); one
// wave (task) owns one 16-row query block and one token range of one (b, kv head).
// Per 32-token step:
//   S^T = K Q^T    (K tile is the MFMA A operand: 16 tokens x 32 dims per block)
//   online soft-max per query row (a row lives in the 4 lanes l%16 == row)
//   O^T += V^T P^T (V^T tile from the transposed cache is A, probabilities are B)
// The two 16-token score tiles give each lane tokens {4g..4g+3} and {16+4g..}, which
// is taken as that lane's 8 contraction elements of the second product; the V^T
// fragment gathers the same tokens, so no data moves between lanes.
// Output: unnormalised partial (m, l, O) per split; combine_task merges.
template <typename T>
struct AttnArgs {
  const T *qbuf, *kc, *vt;          // kc / vt offset to the layer
  const int32_t* kv_len;
  float *pm, *pl, *po;              // [B][Hkv][nsplit][qrows_pad] / ...[hd]
  int k, g, Hkv, hd, max_ctx, qrows_pad, nsplit, nqb;   // nqb = query blocks per (b, kv head)
  float scale;                      // log2(e) / sqrt(hd): scores and running maxima are kept in the log2 domain
};

// Probabilities (fp32, in [0,1]) as MFMA B operands.  For bf16 models they are split
// into a bf16 head and a bf16 tail (p = hi + lo up to 2^-17 relative), so the PV
// product sees ~16 significant bits of every probability at the cost of a second,
// HBM-free MFMA per V^T tile.
// heads = bf16 of the four values (two packed words); `a` is replaced by the remainders
__device__ __forceinline__ void split_bf16(f32x4& a, uint32_t& h0, uint32_t& h1) {
  h0 = pack_bf16(a.x, a.y);
  h1 = pack_bf16(a.z, a.w);
  a = a - f32x4{__uint_as_float(h0 << 16), __uint_as_float(h0 & 0xffff0000u), __uint_as_float(h1 << 16),
                __uint_as_float(h1 & 0xffff0000u)};
}
template <int HT>
__device__ __forceinline__ void pv_accumulate(f32x4 (&o)[HT], const Frag<bf16_t> (&vf)[HT], f32x4 a, f32x4 b) {
  Frag<bf16_t> hi, lo;
  uint32_t h0, h1, h2, h3;
  split_bf16(a, h0, h1);
  split_bf16(b, h2, h3);
  hi.v = u32x4{h0, h1, h2, h3};
  lo.v = u32x4{pack_bf16(a.x, a.y), pack_bf16(a.z, a.w), pack_bf16(b.x, b.y), pack_bf16(b.z, b.w)};
#pragma unroll
  for (int h = 0; h < HT; ++h) { o[h] = mma(vf[h], lo, o[h]); o[h] = mma(vf[h], hi, o[h]); }
}
template <int HT>
__device__ __forceinline__ void pv_accumulate(f32x4 (&o)[HT], const Frag<float> (&vf)[HT], f32x4 a, f32x4 b) {
  Frag<float> pf; pf.lo = a; pf.hi = b;
#pragma unroll
  for (int h = 0; h < HT; ++h) o[h] = mma(vf[h], pf, o[h]);
}

template <typename T, int HD>
struct KvFrags { Frag<T> kf[2][HD / 32]; Frag<T> vf[HD / 16]; };

template <typename T, int HD>
__device__ __forceinline__ void load_kv(KvFrags<T, HD>& f, const T* kbase, const T* vbase, int tb, int lane) {
  // tb is a multiple of 32 and tb + 31 < roundup32(len) <= max_ctx.  See kc_offset / vt_offset:
  // K fragments (A operand) of the two 16-token tiles (token = tb + 16*h + lane%16, dims
  // ks*32 + 8*(lane/16) ..), V^T fragments (dim = h*16 + lane%16, tokens tb + 4*(lane/16) + {0..3}
  // and tb + 16 + 4*(lane/16) + {0..3}); each is the lane's 8 consecutive elements of a tile.
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int ks = 0; ks < HD / 32; ++ks)
      f.kf[h][ks] = frag_load_row(kbase + ((size_t)(((tb >> 4) + h) * (HD / 32) + ks) * 64 + lane) * 8);
#pragma unroll
  for (int h = 0; h < HD / 16; ++h)
    f.vf[h] = frag_load_row(vbase + ((size_t)((tb >> 5) * (HD / 16) + h) * 64 + lane) * 8);
}

// task = ((b * Hkv + kvh) * nsplit + sp) * nqb + qb.  The next step's K/V are fetched
// into registers while the current one is computed.
template <typename T, int HD, int PRE>
__device__ __forceinline__ void attn_task(const AttnArgs<T>& a, int task) {
  constexpr int KSTEPS = HD / 32, HT = HD / 16;
  const int lane = threadIdx.x & 63, c = lane & 15, g4 = lane >> 4;
  int id = task;
  const int qb = id % a.nqb; id /= a.nqb;
  const int sp = id % a.nsplit; id /= a.nsplit;
  const int kvh = id % a.Hkv; const int b = id / a.Hkv;
  const int P = a.kv_len[b];
  const int len = min(P + a.k, a.max_ctx);          // slots visible to the last row
  int per = (len + a.nsplit - 1) / a.nsplit;
  per = (per + 31) & ~31;                            // token ranges start on 32-token steps
  const int t0 = sp * per, t1 = min(len, t0 + per);
  const int nq = a.g * a.k;
  const int row = qb * 16 + c;

  // query fragments (B operand): dims ks*32 + 8*g4 ..
  Frag<T> qf[KSTEPS];
  const int jrow = row < nq ? row / a.g : -1;
  {
    const T* qp = a.qbuf + ((size_t)(b * a.Hkv + kvh) * a.qrows_pad + row) * HD + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      if (row < nq) qf[ks] = frag_load_row(qp + ks * 32); else frag_zero(qf[ks]);
    }
  }
  f32x4 o[HT];
#pragma unroll
  for (int h = 0; h < HT; ++h) o[h] = f32x4{0.f, 0.f, 0.f, 0.f};
  float mrun = -INFINITY, lrun = 0.f;
  const T* kbase = a.kc + (size_t)(b * a.Hkv + kvh) * a.max_ctx * HD;
  const T* vbase = a.vt + (size_t)(b * a.Hkv + kvh) * a.max_ctx * HD;
  const int lim = jrow < 0 ? -1 : min(P + jrow, t1 - 1);   // last slot this query row may see

  // One 32-token step: scores, online soft-max, O^T += V^T P^T.
  auto step = [&](const KvFrags<T, HD>& f, int tb) {
    f32x4 s[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) s[h] = mma(f.kf[h][ks], qf[ks], s[h]);
    }
    // lane holds scores of query row c for tokens tb + 16*h + 4*g4 + i
    float mx = -INFINITY;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int tok = tb + 16 * h + 4 * g4 + i;
        const float v = tok <= lim ? s[h][i] * a.scale : -INFINITY;
        s[h][i] = v; mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mnew = fmaxf(mrun, mx);
    float alpha = 1.f, psum = 0.f;
    if (mnew > -INFINITY) {
      alpha = fast_exp2(mrun - mnew);   // 2^(-inf) = 0 on the first visible step
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) { const float p = fast_exp2(s[h][i] - mnew); s[h][i] = p; psum += p; }
    } else {
      s[0] = f32x4{0.f, 0.f, 0.f, 0.f}; s[1] = s[0];
    }
    mrun = mnew;
    lrun = lrun * alpha + psum;       // per-lane share; lane groups are summed at the end
#pragma unroll
    for (int h = 0; h < HT; ++h) o[h] = o[h] * alpha;
    pv_accumulate<HT>(o, f.vf, s[0], s[1]);
  };
  // The K/V of PRE steps are requested together, before any of them is used: a step
  // computes in a fraction of a memory round trip, so fetching only one step ahead costs one
  // round trip per step.  PRE = 4 (128 tokens) needs the CU's registers for one workgroup
  // (256 VGPRs + 114 AGPRs per lane): right when there is at most one workgroup per CU;
  // with more workgroups than CUs PRE = 2 lets two of them share a CU.
  // Steps beyond the range re-read its first step (a valid address) and are skipped.
  for (int tg = t0; tg < t1; tg += 32 * PRE) {
    KvFrags<T, HD> f[PRE];
#pragma unroll
    for (int u = 0; u < PRE; ++u) load_kv<T, HD>(f[u], kbase, vbase, tg + 32 * u < t1 ? tg + 32 * u : t0, lane);
#pragma unroll
    for (int u = 0; u < PRE; ++u)
      if (tg + 32 * u < t1) step(f[u], tg + 32 * u);
  }
  // write the partial
  float l = lrun;
  l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
  const size_t pidx = ((size_t)(b * a.Hkv + kvh) * a.nsplit + sp) * a.qrows_pad + row;
  if (g4 == 0) { a.pm[pidx] = mrun; a.pl[pidx] = l; }
#pragma unroll
  for (int h = 0; h < HT; ++h) *reinterpret_cast<f32x4*>(a.po + pidx * HD + h * 16 + 4 * g4) = o[h];
}

// grid = B * Hkv * nsplit * ceil(nqb / wpg) workgroups of wpg waves; the waves of a
// workgroup own consecutive query blocks of the same K/V range, so those reads are
// shared through the CU's L1.
template <typename T, int HD, int PRE>
__global__ void __launch_bounds__(256) attn_split_kernel(const AttnArgs<T> a) {
  const int wpg = blockDim.x >> 6;
  const int nqg = (a.nqb + wpg - 1) / wpg;
  const int qb = (blockIdx.x % nqg) * wpg + (threadIdx.x >> 6);
  if (qb >= a.nqb) return;
  attn_task<T, HD, PRE>(a, (blockIdx.x / nqg) * a.nqb + qb);
}

// Merge the split partials of one (row m, query head): softmax-weighted sum,
// normalise, round to T, write attn[m][head*hd + :].  One wave per task = (m, head);
// nsplit <= 64: lane s first handles split s's (m, l), then every lane owns HD/64
// consecutive output dims and walks the splits with the weights broadcast by shuffle.
template <typename T>
struct CombineArgs {
  const float *pm, *pl, *po;
  T* attn; int ldat;
  int Mtot, k, H, Hkv, qrows_pad, nsplit;
};

template <typename T, int HD>
__device__ __forceinline__ void combine_task(const CombineArgs<T>& a, int task) {
  constexpr int DPL = HD / 64;   // dims per lane
  const int lane = threadIdx.x & 63;
  const int m = task / a.H, hh = task % a.H;
  const int b = m / a.k, j = m % a.k, g = a.H / a.Hkv, kvh = hh / g, hg = hh % g;
  const int row = j * g + hg;
  const size_t base = (size_t)(b * a.Hkv + kvh) * a.nsplit;
  float ms = -INFINITY, ls = 0.f;
  if (lane < a.nsplit) {
    ms = *(a.pm + (base + lane) * a.qrows_pad + row);
    ls = *(a.pl + (base + lane) * a.qrows_pad + row);
  }
  float M = ms;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  const float w = ms > -INFINITY ? fast_exp2(ms - M) : 0.f;
  const float L = wave_sum(ls * w);
  float acc[DPL];
#pragma unroll
  for (int i = 0; i < DPL; ++i) acc[i] = 0.f;
  const float* o = a.po + (base * a.qrows_pad + row) * HD + lane * DPL;
  const size_t sstride = (size_t)a.qrows_pad * HD;
  auto ldo = [&](int s, float (&v)[DPL]) {
    if (DPL == 2) { const f32x2 t = *reinterpret_cast<const f32x2*>(o + (size_t)s * sstride); v[0] = t.x; v[DPL - 1] = t.y; }
    else v[0] = *(o + (size_t)s * sstride);
  };
  int s = 0;
  for (; s + 4 <= a.nsplit; s += 4) {
    float v[4][DPL];
#pragma unroll
    for (int u = 0; u < 4; ++u) ldo(s + u, v[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wu = __shfl(w, s + u);
#pragma unroll
      for (int i = 0; i < DPL; ++i) acc[i] += v[u][i] * wu;
    }
  }
  for (; s < a.nsplit; ++s) {
    float v[DPL];
    ldo(s, v);
    const float wu = __shfl(w, s);
#pragma unroll
    for (int i = 0; i < DPL; ++i) acc[i] += v[i] * wu;
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  T* dst = a.attn + (size_t)m * a.ldat + (size_t)hh * HD + lane * DPL;
  if (DPL == 2 && sizeof(T) == 2) {
    *reinterpret_cast<uint32_t*>(dst) = (pack_bf16(acc[0] * inv, acc[DPL - 1] * inv));
  } else {
#pragma unroll
    for (int i = 0; i < DPL; ++i) st_round1(dst + i, acc[i] * inv);
  }
}

template <typename T, int HD>
__global__ void __launch_bounds__(256) attn_combine_kernel(const CombineArgs<T> a) {
  const int task = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (task >= a.Mtot * a.H) return;
  combine_task<T, HD>(a, task);
}

}  // namespace dbl
