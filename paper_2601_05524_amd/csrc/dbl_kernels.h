// The small kernels around the projections: embedding gather, residual + RMSNorm,
// q/k-norm + RoPE + KV append, split-KV GQA attention and its combine, acceptance,
// n-gram retrieval, window build, commit, and the seeded weight generator.
#pragma once
#include "dbl_dev.h"
#include "dbl_gemm.h"

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

// ------------------------------------------------------------------ embedding

// h[m][:] = E[window[m]][:]   (grid = rows)
template <typename T>
__global__ void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ window, float* __restrict__ h,
                             int d, int ldh, int vocab) {
  const int m = blockIdx.x;
  int tok = window[m];
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const T* e = E + (size_t)tok * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)m * ldh + i] = Elem<T>::to_f(e[i]);
}

// ------------------------------------------------------- residual + RMSNorm

// h[m] += sum_p part[p][m] (written back when nparts > 0), then
// xn[m][i] = T( h[m][i] * rsqrt(mean(h[m]^2) + eps) * gain[i] ).   grid = rows.
// d % 4 == 0.  A thread owns up to RMS_VPT float4 columns (d <= 4*1024*RMS_VPT); all
// its loads are issued before the first use, so the kernel costs one memory latency,
// one workgroup reduction and one store.
constexpr int RMS_VPT = 4;
constexpr int RMS_MAXP = 8;

__device__ __forceinline__ void store4(float* p, const f32x4& v) { *reinterpret_cast<f32x4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, const f32x4& v) {
  *reinterpret_cast<u32x2*>(p) = u32x2{pack_bf16(v.x, v.y), pack_bf16(v.z, v.w)};
}

template <typename T>
__global__ void __launch_bounds__(1024) rmsnorm_kernel(float* __restrict__ h, int ldh, const float* __restrict__ part,
                                                       int nparts, int Mtot, int ldp, const float* __restrict__ gain,
                                                       T* __restrict__ xn, int ldx, int d, float eps) {
  __shared__ float scratch[16];
  const int m = blockIdx.x;
  float* hr = h + (size_t)m * ldh;
  const int nv = d >> 2;
  f32x4 v[RMS_VPT], gn[RMS_VPT];
#pragma unroll
  for (int u = 0; u < RMS_VPT; ++u) {
    const int i = threadIdx.x + u * blockDim.x;
    v[u] = f32x4{0.f, 0.f, 0.f, 0.f}; gn[u] = v[u];
    if (i < nv) { v[u] = reinterpret_cast<const f32x4*>(hr)[i]; gn[u] = reinterpret_cast<const f32x4*>(gain)[i]; }
  }
  if (nparts > 0) {
#pragma unroll
    for (int p = 0; p < RMS_MAXP; ++p) {
      if (p < nparts) {
        const float* pr = part + ((size_t)p * Mtot + m) * ldp;
#pragma unroll
        for (int u = 0; u < RMS_VPT; ++u) {
          const int i = threadIdx.x + u * blockDim.x;
          if (i < nv) v[u] += reinterpret_cast<const f32x4*>(pr)[i];
        }
      }
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < RMS_VPT; ++u) ss += v[u].x * v[u].x + v[u].y * v[u].y + v[u].z * v[u].z + v[u].w * v[u].w;
  ss = block_sum(ss, scratch);
  const float r = rsqrtf(ss / (float)d + eps);
#pragma unroll
  for (int u = 0; u < RMS_VPT; ++u) {
    const int i = threadIdx.x + u * blockDim.x;
    if (i < nv) {
      if (nparts > 0) reinterpret_cast<f32x4*>(hr)[i] = v[u];
      store4(xn + (size_t)m * ldx + 4 * i, f32x4{v[u].x * r * gn[u].x, v[u].y * r * gn[u].y, v[u].z * r * gn[u].z, v[u].w * r * gn[u].w});
    }
  }
}

// ---------------------------------------------- q/k norm + RoPE + KV append

// One wave per (row m, head hh) with hh in [0, H + 2*Hkv): q heads, then k heads,
// then v heads.  Sums the QKV partials, applies the optional per-head RMSNorm and
// the rotary embedding (pairs (i, i+hd/2); cos/sin from the fp32 table at the
// row's position kv_len[b] + j), rounds to T, and writes
//   q  -> qbuf[b][kvh][j*g + hg][hd]
//   k  -> kc[layer][b][kvh][pos][hd]
//   v  -> vt[layer][b][kvh][pos/64][hd][pos%64]      (transposed, 64-token blocks)
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
__global__ void __launch_bounds__(256) rope_kv_kernel(const RopeArgs<T> a) {
  const int lane = threadIdx.x & 63;
  const int wid = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int heads = a.H + 2 * a.Hkv;
  if (wid >= a.Mtot * heads) return;
  const int m = wid / heads, hh = wid % heads;
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
      x0 += src[lane]; x1 += src[lane + half];
    }
  }
  const bool is_q = hh < a.H, is_k = !is_q && hh < a.H + a.Hkv;
  if (!is_q && !is_k) {  // v head: no norm, no rotation
    if (act) {
      const int kvh = hh - a.H - a.Hkv;
      T* dst = a.vt + ((size_t)(b * a.Hkv + kvh) * (a.max_ctx / VT_BLOCK) + pos / VT_BLOCK) * hd * VT_BLOCK + pos % VT_BLOCK;
      dst[(size_t)lane * VT_BLOCK] = Elem<T>::from_f(x0);
      dst[(size_t)(lane + half) * VT_BLOCK] = Elem<T>::from_f(x1);
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
    T* dst;
    if (is_q) {
      const int g = a.H / a.Hkv, kvh = hh / g, hg = hh % g;
      dst = a.qbuf + ((size_t)(b * a.Hkv + kvh) * a.qrows_pad + (j * g + hg)) * hd;
    } else {
      const int kvh = hh - a.H;
      dst = a.kc + ((size_t)(b * a.Hkv + kvh) * a.max_ctx + pos) * hd;
    }
    dst[lane] = Elem<T>::from_f(y0);
    dst[lane + half] = Elem<T>::from_f(y1);
  }
}

// ------------------------------------------------------------ GQA attention

// Split-KV ("flash-decode") attention for a short query window.  The g query heads
// of one KV head and the k window rows form g*k query rows (row = j*g + hg); one
// wave owns QB 16-row query blocks and one token range of one (b, kv head), so each
// K/V byte is read once per QB blocks.  Per 32-token step:
//   S^T = K Q^T    (K tile is the MFMA A operand: 16 tokens x 32 dims per block)
//   online soft-max per query row (a row lives in the 4 lanes l%16 == row)
//   O^T += V^T P^T (V^T tile from the transposed cache is A, probabilities are B)
// The two 16-token score tiles give each lane tokens {4g..4g+3} and {16+4g..}, which
// is taken as that lane's 8 contraction elements of the second product; the V^T
// fragment gathers the same tokens, so no data moves between lanes.
// Output: unnormalised partial (m, l, O) per split; attn_combine_kernel merges.
template <typename T>
struct AttnArgs {
  const T *qbuf, *kc, *vt;          // kc / vt offset to the layer
  const int32_t* kv_len;
  float *pm, *pl, *po;              // [B][Hkv][nsplit][qrows_pad] / ...[hd]
  int k, g, Hkv, hd, max_ctx, qrows_pad, nsplit, nqg;
  float scale;                      // log2(e) / sqrt(hd): scores and running maxima are kept in the log2 domain
};

template <typename T> __device__ __forceinline__ Frag<T> vt_frag(const T* v0, const T* v1);
template <> __device__ __forceinline__ Frag<bf16_t> vt_frag<bf16_t>(const bf16_t* v0, const bf16_t* v1) {
  Frag<bf16_t> f;
  const u32x2 a = *reinterpret_cast<const u32x2*>(v0), b = *reinterpret_cast<const u32x2*>(v1);
  f.v = u32x4{a.x, a.y, b.x, b.y};
  return f;
}
template <> __device__ __forceinline__ Frag<float> vt_frag<float>(const float* v0, const float* v1) {
  Frag<float> f;
  f.lo = *reinterpret_cast<const f32x4*>(v0);
  f.hi = *reinterpret_cast<const f32x4*>(v1);
  return f;
}
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
__device__ __forceinline__ void load_kv(KvFrags<T, HD>& f, const T* kbase, const T* vbase, int tb, int c, int g4) {
  // K fragments (A operand) of the two 16-token tiles: token = tb + 16*h + c  (< max_ctx:
  // tb + 31 < roundup32(len) <= max_ctx)
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const T* kp = kbase + (size_t)(tb + 16 * h + c) * HD + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < HD / 32; ++ks) f.kf[h][ks] = frag_load_row(kp + ks * 32);
  }
  // V^T fragments: dim row = ht*16 + c; tokens tb + 4*g4 + {0..3} and tb + 16 + 4*g4 + {0..3}
  const T* vp = vbase + (size_t)(tb / VT_BLOCK) * HD * VT_BLOCK + (tb % VT_BLOCK) + 4 * g4;
#pragma unroll
  for (int h = 0; h < HD / 16; ++h) {
    const T* r = vp + (size_t)(h * 16 + c) * VT_BLOCK;
    f.vf[h] = vt_frag<T>(r, r + 16);
  }
}

// grid = B * Hkv * nsplit * nqg workgroups of (query blocks per group) waves; wave w of
// a workgroup owns query block qg*wpg + w; all waves of a workgroup read the same K/V
// range, so those reads are shared through the CU's L1.
template <typename T, int HD>
__global__ void __launch_bounds__(256) attn_split_kernel(const AttnArgs<T> a) {
  constexpr int KSTEPS = HD / 32, HT = HD / 16;
  const int lane = threadIdx.x & 63, c = lane & 15, g4 = lane >> 4;
  const int wpg = blockDim.x >> 6;
  int id = blockIdx.x;
  const int qg = id % a.nqg; id /= a.nqg;
  const int sp = id % a.nsplit; id /= a.nsplit;
  const int kvh = id % a.Hkv; const int b = id / a.Hkv;
  const int qb = qg * wpg + (threadIdx.x >> 6);
  const int P = a.kv_len[b];
  const int len = min(P + a.k, a.max_ctx);          // slots visible to the last row
  int per = (len + a.nsplit - 1) / a.nsplit;
  per = (per + 31) & ~31;                            // token ranges start on 32-token steps
  const int t0 = sp * per, t1 = min(len, t0 + per);
  const int nq = a.g * a.k;
  const int row = qb * 16 + c;
  if (qb * 16 >= a.qrows_pad) return;                // (whole wave) no such query block

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
  const T* vbase = a.vt + (size_t)(b * a.Hkv + kvh) * (a.max_ctx / VT_BLOCK) * HD * VT_BLOCK;
  const int lim = jrow < 0 ? -1 : min(P + jrow, t1 - 1);   // last slot this query row may see

  KvFrags<T, HD> cur, nxt;
  if (t0 < t1) load_kv<T, HD>(cur, kbase, vbase, t0, c, g4);
  for (int tb = t0; tb < t1; tb += 32) {
    if (tb + 32 < t1) load_kv<T, HD>(nxt, kbase, vbase, tb + 32, c, g4);
    f32x4 s[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) s[h] = mma(cur.kf[h][ks], qf[ks], s[h]);
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
    pv_accumulate<HT>(o, cur.vf, s[0], s[1]);
    cur = nxt;
  }
  // write the partial
  float l = lrun;
  l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
  const size_t pidx = ((size_t)(b * a.Hkv + kvh) * a.nsplit + sp) * a.qrows_pad + row;
  if (g4 == 0) { a.pm[pidx] = mrun; a.pl[pidx] = l; }
#pragma unroll
  for (int h = 0; h < HT; ++h)
    *reinterpret_cast<f32x4*>(a.po + pidx * HD + h * 16 + 4 * g4) = o[h];
}

// Merge the split partials of one (row m, query head): softmax-weighted sum,
// normalise, round to T, write attn[m][head*hd + :].  One wave per (m, head);
// nsplit <= 64: lane s first handles split s's (m, l), then every lane owns HD/64
// consecutive output dims and walks the splits with the weights broadcast by shuffle.
template <typename T, int HD>
__global__ void __launch_bounds__(256) attn_combine_kernel(const float* __restrict__ pm, const float* __restrict__ pl,
                                                           const float* __restrict__ po, T* __restrict__ attn, int ldat,
                                                           int Mtot, int k, int H, int Hkv, int qrows_pad, int nsplit) {
  constexpr int DPL = HD / 64;   // dims per lane
  const int lane = threadIdx.x & 63;
  const int wid = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (wid >= Mtot * H) return;
  const int m = wid / H, hh = wid % H;
  const int b = m / k, j = m % k, g = H / Hkv, kvh = hh / g, hg = hh % g;
  const int row = j * g + hg;
  const size_t base = (size_t)(b * Hkv + kvh) * nsplit;
  float ms = -INFINITY, ls = 0.f;
  if (lane < nsplit) { ms = pm[(base + lane) * qrows_pad + row]; ls = pl[(base + lane) * qrows_pad + row]; }
  float M = ms;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  const float w = ms > -INFINITY ? fast_exp2(ms - M) : 0.f;
  const float L = wave_sum(ls * w);
  float acc[DPL];
#pragma unroll
  for (int i = 0; i < DPL; ++i) acc[i] = 0.f;
  const float* o = po + (base * qrows_pad + row) * HD + lane * DPL;
  const size_t sstride = (size_t)qrows_pad * HD;
  int s = 0;
  for (; s + 4 <= nsplit; s += 4) {
    float v[4][DPL];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < DPL; ++i) v[u][i] = o[(size_t)(s + u) * sstride + i];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wu = __shfl(w, s + u);
#pragma unroll
      for (int i = 0; i < DPL; ++i) acc[i] += v[u][i] * wu;
    }
  }
  for (; s < nsplit; ++s) {
    const float wu = __shfl(w, s);
#pragma unroll
    for (int i = 0; i < DPL; ++i) acc[i] += o[(size_t)s * sstride + i] * wu;
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  T* dst = attn + (size_t)m * ldat + (size_t)hh * HD + lane * DPL;
#pragma unroll
  for (int i = 0; i < DPL; ++i) dst[i] = Elem<T>::from_f(acc[i] * inv);
}

// ------------------------------------------------------------------- accept

struct AcceptArgs {
  const LmStat* stats; int nstat, Mtot;      // [nstat][Mtot]
  const float* logits; int ldl;              // [Mtot][ldl]
  const int32_t* window;                     // [B][k]
  const float* q;                            // [B][k-1][V] or nullptr
  const uint64_t* commits;
  int32_t *n_acc, *emit, *guide;             // caller outputs
  int32_t *n_acc_i, *emit_i;                 // context copies for commit
  int k, V, mode;
  float inv_T;
  uint64_t seed, step;
};

// One workgroup per sequence.  Merges the LM-head statistics of its k rows, runs
// the acceptance scan, and (dense q only) makes one pass over the rejected row to
// draw from max(0, p - q).
__global__ void __launch_bounds__(256) accept_kernel(const AcceptArgs a) {
  __shared__ LmStat row[32];
  __shared__ LmStat tmp[4];
  __shared__ int s_n, s_need_resid, s_tok;
  __shared__ float s_lse;
  __shared__ float rbest[4]; __shared__ int rbest_id[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t stepv = a.step + *a.commits;

  for (int j = 0; j < a.k; ++j) {
    const int m = b * a.k + j;
    LmStat s;
    s.best = -INFINITY; s.best_id = 0x7fffffff; s.smax = -INFINITY; s.ssum = 0.f; s.zdraft = -INFINITY;
    s.p1 = -INFINITY; s.p1_id = 0x7fffffff; s.p2 = -INFINITY; s.p2_id = 0x7fffffff;
    auto merge = [](LmStat& x, const LmStat& y) {
      if (better(y.best, y.best_id, x.best, x.best_id)) { x.best = y.best; x.best_id = y.best_id; }
      x.zdraft = fmaxf(x.zdraft, y.zdraft);
      const float nm = fmaxf(x.smax, y.smax);
      if (nm > -INFINITY) x.ssum = x.ssum * expf(x.smax - nm) + y.ssum * expf(y.smax - nm);
      x.smax = nm;
      if (better(y.p1, y.p1_id, x.p1, x.p1_id)) {
        if (better(x.p1, x.p1_id, y.p2, y.p2_id)) { x.p2 = x.p1; x.p2_id = x.p1_id; } else { x.p2 = y.p2; x.p2_id = y.p2_id; }
        x.p1 = y.p1; x.p1_id = y.p1_id;
      } else if (better(y.p1, y.p1_id, x.p2, x.p2_id)) { x.p2 = y.p1; x.p2_id = y.p1_id; }
    };
    for (int i = tid; i < a.nstat; i += blockDim.x) merge(s, a.stats[(size_t)i * a.Mtot + m]);
    // butterfly inside the wave, then across the 4 waves (fixed order)
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      LmStat o;
      o.best = __shfl_xor(s.best, off); o.best_id = __shfl_xor(s.best_id, off);
      o.smax = __shfl_xor(s.smax, off); o.ssum = __shfl_xor(s.ssum, off); o.zdraft = __shfl_xor(s.zdraft, off);
      o.p1 = __shfl_xor(s.p1, off); o.p1_id = __shfl_xor(s.p1_id, off);
      o.p2 = __shfl_xor(s.p2, off); o.p2_id = __shfl_xor(s.p2_id, off);
      merge(s, o);
    }
    if (lane == 0) tmp[wave] = s;
    __syncthreads();
    if (tid == 0) {
      LmStat r = tmp[0];
      for (int w = 1; w < (int)(blockDim.x >> 6); ++w) merge(r, tmp[w]);
      row[j] = r;
    }
    __syncthreads();
  }

  const int32_t* win = a.window + (size_t)b * a.k;
  if (tid == 0) {
    int n = a.k - 1, need = 0, tok = -1;
    if (a.mode == 0) {
      n = 0;
      while (n < a.k - 1 && win[n + 1] == row[n].best_id) ++n;
      tok = row[n].best_id;
      for (int j = 0; j < a.k; ++j) a.guide[(size_t)b * a.k + j] = row[j].best_id;
    } else {
      for (int j = 0; j < a.k - 1; ++j) {
        const int x = win[j + 1];
        const float lse = row[j].smax + logf(row[j].ssum);
        const float px = expf(row[j].zdraft * a.inv_T - lse);
        const Philox4 r = philox4x32_10((uint32_t)stepv, (uint32_t)b, (uint32_t)j, 0u, (uint32_t)a.seed,
                                        (uint32_t)(a.seed >> 32));
        const float u = u01(r.x);
        const float qx = a.q ? a.q[((size_t)b * (a.k - 1) + j) * a.V + x] : 1.f;
        if (!(u * qx < px)) { n = j; break; }
      }
      if (n < a.k - 1) {
        if (a.q) { need = 1; tok = row[n].p1_id; /* fallback if the residual is empty */ }
        else { const int x = win[n + 1]; tok = row[n].p1_id != x ? row[n].p1_id : row[n].p2_id; }
      } else {
        tok = row[n].p1_id;
      }
      for (int j = 0; j < a.k; ++j) a.guide[(size_t)b * a.k + j] = j <= n ? row[j].p1_id : -1;
    }
    s_n = n; s_need_resid = need; s_tok = tok;
    s_lse = a.mode ? row[n].smax + logf(row[n].ssum) : 0.f;
  }
  __syncthreads();
  const int n = s_n;
  if (s_need_resid) {
    // draw from max(0, p_n - q_n): argmax_v log(w_v) + Gumbel_v over w_v > 0
    const int m = b * a.k + n;
    const float* z = a.logits + (size_t)m * a.ldl;
    const float* qn = a.q + ((size_t)b * (a.k - 1) + n) * a.V;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int v4 = tid; v4 * 4 < a.V; v4 += blockDim.x) {
      const Philox4 r = philox4x32_10((uint32_t)stepv, (uint32_t)b, (uint32_t)n, 1u + (uint32_t)v4, (uint32_t)a.seed,
                                      (uint32_t)(a.seed >> 32));
      const uint32_t rw[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = v4 * 4 + i;
        if (v >= a.V) break;
        const float w = expf(z[v] * a.inv_T - s_lse) - qn[v];
        if (w > 0.f) {
          const float sc = logf(w) + gumbel(rw[i]);
          if (better(sc, v, bv, bi)) { bv = sc; bi = v; }
        }
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off); const int oi = __shfl_xor(bi, off);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { rbest[wave] = bv; rbest_id[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
      for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
        if (better(rbest[w], rbest_id[w], rbest[0], rbest_id[0])) { rbest[0] = rbest[w]; rbest_id[0] = rbest_id[w]; }
      if (rbest[0] > -INFINITY) s_tok = rbest_id[0];
    }
    __syncthreads();
  }
  if (tid == 0) {
    a.n_acc[b] = n; a.n_acc_i[b] = n;
    for (int j = 0; j < a.k; ++j) {
      const int e = j < n ? win[j + 1] : (j == n ? s_tok : -1);
      a.emit[(size_t)b * a.k + j] = e;
      a.emit_i[(size_t)b * a.k + j] = e;
    }
  }
}

// ----------------------------------------------------------------- retrieve

// One workgroup per sequence.  Thread-strided over end positions e in [1, len-1]:
// nm(e) = number of tokens before e that equal the history's last tokens read
// backwards (capped at n_max); a candidate needs nm >= n_min; its start is e - nm
// and its continuation the next min(max_cont, len - e) tokens.  The winner
// maximises (nm, continuation length, e) -- one packed 64-bit max.
__global__ void __launch_bounds__(1024) retrieve_kernel(const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_len,
                                                        int max_hist, int n_max, int n_min, int max_cont,
                                                        int32_t* __restrict__ cont, int32_t* __restrict__ cont_len,
                                                        int32_t* __restrict__ match_n, int32_t* __restrict__ match_pos) {
  __shared__ unsigned long long wbest[16];
  __shared__ int32_t suf[32];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* h = hist + (size_t)b * max_hist;
  const int len = min(hist_len[b], max_hist);
  const int nm_cap = min(n_max, len - 1);
  if (tid < 32) suf[tid] = (tid < nm_cap) ? h[len - 1 - tid] : -1;   // suffix read backwards
  __syncthreads();
  unsigned long long best = 0ull;
  for (int e = 1 + tid; e <= len - 1; e += blockDim.x) {
    int nm = 0;
    const int cap = min(nm_cap, e);
    while (nm < cap && h[e - 1 - nm] == suf[nm]) ++nm;
    if (nm >= n_min) {
      const int cl = min(max_cont, len - e);
      const unsigned long long key = ((unsigned long long)nm << 48) | ((unsigned long long)cl << 32) | (unsigned)e;
      best = key > best ? key : best;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(best, off);
    best = o > best ? o : best;
  }
  if (lane == 0) wbest[wave] = best;
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) best = wbest[w] > best ? wbest[w] : best;
    wbest[0] = best;
  }
  __syncthreads();
  best = wbest[0];
  const int nm = (int)(best >> 48), cl = (int)((best >> 32) & 0xffff), e = (int)(best & 0xffffffffu);
  if (tid == 0) {
    cont_len[b] = best ? cl : 0;
    match_n[b] = best ? nm : 0;
    match_pos[b] = best ? e - nm : -1;
  }
  for (int i = tid; i < max_cont; i += blockDim.x)
    cont[(size_t)b * max_cont + i] = (best && i < cl) ? h[e + i] : -1;
}

// window[b][0] = last history token, then the continuation, then padding
__global__ void build_window_kernel(const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_len, int max_hist,
                                    const int32_t* __restrict__ cont, const int32_t* __restrict__ cont_len, int max_cont,
                                    int k, int32_t pad, int32_t* __restrict__ window) {
  const int b = blockIdx.x;
  const int len = min(hist_len[b], max_hist);
  const int cl = min(cont_len[b], max_cont);
  for (int j = threadIdx.x; j < k; j += blockDim.x) {
    int32_t v;
    if (j == 0) v = len > 0 ? hist[(size_t)b * max_hist + len - 1] : pad;
    else v = (j - 1 < cl) ? cont[(size_t)b * max_cont + j - 1] : pad;
    window[(size_t)b * k + j] = v;
  }
}

// ------------------------------------------------------------------- commit

// kv_len[b] += n_keep[b]; optionally hist ⊕= emit[b][0..n_keep[b]).  Capacity
// violations clamp and raise status bit 0 (max_ctx) / bit 1 (max_hist).
__global__ void commit_kernel(int32_t* __restrict__ kv_len, int32_t* __restrict__ hist_len, int32_t* __restrict__ hist,
                              int max_hist, int max_ctx, const int32_t* __restrict__ n_keep_in,
                              const int32_t* __restrict__ n_acc_i, const int32_t* __restrict__ emit_i, int k, int B,
                              int append, uint64_t* __restrict__ commits, int32_t* __restrict__ status) {
  const int b = threadIdx.x;
  if (b < B) {
    int nk = n_keep_in ? n_keep_in[b] : n_acc_i[b] + 1;
    nk = max(0, min(nk, k));
    int kl = kv_len[b];
    if (kl + nk > max_ctx) { nk = max_ctx - kl; atomicOr(status, 1); }
    kv_len[b] = kl + nk;
    if (append) {
      int hl = hist_len[b];
      int na = nk;
      if (hl + na > max_hist) { na = max_hist - hl; atomicOr(status, 2); }
      for (int i = 0; i < na; ++i) hist[(size_t)b * max_hist + hl + i] = emit_i[(size_t)b * k + i];
      hist_len[b] = hl + na;
    }
  }
  if (threadIdx.x == 0) *commits += 1;
}

__global__ void set_counters_kernel(int32_t* kv_len, int32_t* hist_len, int seq, int B) {
  const int b = threadIdx.x;
  if (b < B && (seq < 0 || b == seq)) { kv_len[b] = 0; hist_len[b] = 0; }
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ------------------------------------------------------- weight generator

// Value of element `elem` of tensor (tensor_id, layer): see dbl.h (dbl_create).
__device__ __forceinline__ float weight_value(uint64_t seed, int tensor_id, int layer, uint64_t elem) {
  const Philox4 r = philox4x32_10((uint32_t)elem, (uint32_t)(elem >> 32), (uint32_t)tensor_id, (uint32_t)layer,
                                  (uint32_t)seed, (uint32_t)(seed >> 32));
  const int32_t s = (int32_t)(r.x & 0xffffu) + (int32_t)(r.x >> 16) + (int32_t)(r.y & 0xffffu) + (int32_t)(r.y >> 16) +
                    (int32_t)(r.z & 0xffffu) + (int32_t)(r.z >> 16) + (int32_t)(r.w & 0xffffu) + (int32_t)(r.w >> 16);
  // 0.02 / sqrt(8 * (65536^2 - 1) / 12) rounded to fp32
  return __fmul_rn((float)(s - 262140), 0x1.91530cp-22f);
}

// A tiled container holds up to 3 row segments (e.g. Wq | Wk | Wv); with
// `interleave` the tile rows alternate between segment 0 and 1 (gate / up).
struct FillSeg { int tensor_id, rows; };
struct FillArgs {
  FillSeg seg[3]; int nseg, interleave;
  int K, KBp, ntile_rows, layer;
  uint64_t seed;
};

template <typename T>
__global__ void fill_tiled_kernel(T* __restrict__ W, const FillArgs a) {
  // one thread per (block, lane): 8 elements
  const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t nblk = (size_t)a.ntile_rows * a.KBp;
  if (gid >= nblk * 64) return;
  const int lane = (int)(gid & 63);
  const size_t blkid = gid >> 6;
  const int trow = (int)(blkid / a.KBp), kb = (int)(blkid % a.KBp);
  const int r = lane & 15, g = lane >> 4;
  int seg, row;   // logical segment and row within it
  if (a.interleave) { seg = trow & 1; row = (trow >> 1) * 16 + r; }
  else {
    row = trow * 16 + r; seg = 0;
    while (seg < a.nseg - 1 && row >= a.seg[seg].rows) { row -= a.seg[seg].rows; ++seg; }
  }
  const bool row_ok = row < a.seg[seg].rows;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k = kb * 32 + g * 8 + e;
    float v = 0.f;
    if (row_ok && k < a.K) v = weight_value(a.seed, a.seg[seg].tensor_id, a.layer, (uint64_t)row * a.K + k);
    W[tiled_offset<T>(trow * 16 + r, k, a.KBp)] = Elem<T>::from_f(v);
  }
}

template <typename T>
__global__ void fill_rowmajor_kernel(T* __restrict__ W, size_t n, int tensor_id, int layer, uint64_t seed) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) W[i] = Elem<T>::from_f(weight_value(seed, tensor_id, layer, i));
}

__global__ void fill_f32_kernel(float* p, float v, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace dbl
