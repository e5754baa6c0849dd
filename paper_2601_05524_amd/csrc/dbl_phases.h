// The per-layer steps between the projections: split-KV GQA attention (q/k-norm and RoPE
// applied while it loads its operands) and the merge of its partials, which also appends
// the window rows to the KV cache.  Each is a device function over a "task" index (one
// wave per task) with a thin kernel around it.
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

// ---------------------------------------------- q/k norm + RoPE on load, KV append

// Where the q/k/v projection left its result (nparts partial sums per element; columns: the
// q heads, then the k heads, then the v heads) and what turns it into attention operands.
// There is no kernel for this step: the attention builds its query and window-row operands
// from here, and the kernel that merges the attention partials appends the window rows to
// the KV cache.
struct QkvSrc {
  const float* qkv; int nparts, Mtot, ldq;   // partials [nparts][Mtot][ldq]
  const float *gq, *gk;                      // per-head RMSNorm gains (qk_norm) or nullptr
  const float *cosT, *sinT;                  // [max_ctx][hd/2]
  int H, Hkv;
  float eps;
};

__device__ __forceinline__ Frag<bf16_t> frag_round(const float (&x)[8], bf16_t) {
  Frag<bf16_t> f;
  f.v = u32x4{pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7])};
  return f;
}
__device__ __forceinline__ Frag<float> frag_round(const float (&x)[8], float) {
  Frag<float> f;
  f.lo = f32x4{x[0], x[1], x[2], x[3]}; f.hi = f32x4{x[4], x[5], x[6], x[7]};
  return f;
}

// Sum over the partials of 8 consecutive columns of row m, in partial order.
__device__ __forceinline__ void qkv_sum8(const QkvSrc& s, int m, int col, float (&x)[8]) {
  const size_t pstride = (size_t)s.Mtot * s.ldq;
  const float* src = s.qkv + (size_t)m * s.ldq + col;
  f32x4 a = *reinterpret_cast<const f32x4*>(src), b = *reinterpret_cast<const f32x4*>(src + 4);
  if (s.nparts > 1) {   // the usual case, written out so that both partials are in flight together
    a += *reinterpret_cast<const f32x4*>(src + pstride); b += *reinterpret_cast<const f32x4*>(src + pstride + 4);
  }
  for (int p = 2; p < s.nparts; ++p) {
    a += *reinterpret_cast<const f32x4*>(src + p * pstride); b += *reinterpret_cast<const f32x4*>(src + p * pstride + 4);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
}

// One q or k head vector of row m (columns col0 .. col0+HD-1 of the projection result) as MFMA
// fragments: partial sums added, optional per-head RMSNorm (gain), rotary embedding at
// position pos (pairs (i, i + HD/2), cos/sin from the fp32 table), rounded to T.  Lane group
// g4 gets dims ks*32 + 8*g4 .. +7 in out[ks]; a dim and its rotation partner fall in the same
// lane.  The four lanes l, l^16, l^32, l^48 must work on the same head (they share the
// sum of squares); every user of a head vector goes through here, so the cache and the
// in-flight window rows hold the same bits.
// Two phases, so that a caller can request several heads (and other data) before it waits
// for any: head_load only issues loads (no branch, no arithmetic), head_finish does the rest.
template <int HD>
struct HeadRaw {
  f32x4 p0[HD / 32][2], p1[HD / 32][2];   // partials 0 and 1 (partial 0 again when there is only one)
  f32x4 cs[HD / 64][2], sn[HD / 64][2];
};

template <int HD>
__device__ __forceinline__ void head_load(const QkvSrc& s, int m, int col0, int pos, int g4, HeadRaw<HD>& r) {
  constexpr int KSTEPS = HD / 32, HK = KSTEPS / 2, HALF = HD / 2;
  const float* src = s.qkv + (size_t)m * s.ldq + col0 + 8 * g4;
  const float* src1 = src + (s.nparts > 1 ? (size_t)s.Mtot * s.ldq : 0);
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    r.p0[ks][0] = *reinterpret_cast<const f32x4*>(src + ks * 32); r.p0[ks][1] = *reinterpret_cast<const f32x4*>(src + ks * 32 + 4);
    r.p1[ks][0] = *reinterpret_cast<const f32x4*>(src1 + ks * 32); r.p1[ks][1] = *reinterpret_cast<const f32x4*>(src1 + ks * 32 + 4);
  }
#pragma unroll
  for (int ks = 0; ks < HK; ++ks) {
    const size_t o = (size_t)pos * HALF + ks * 32 + 8 * g4;
    r.cs[ks][0] = *reinterpret_cast<const f32x4*>(s.cosT + o); r.cs[ks][1] = *reinterpret_cast<const f32x4*>(s.cosT + o + 4);
    r.sn[ks][0] = *reinterpret_cast<const f32x4*>(s.sinT + o); r.sn[ks][1] = *reinterpret_cast<const f32x4*>(s.sinT + o + 4);
  }
}

template <typename T, int HD>
__device__ __forceinline__ void head_finish(const QkvSrc& s, const HeadRaw<HD>& r, int m, int col0, const float* gain,
                                            int g4, Frag<T> (&out)[HD / 32]) {
  constexpr int KSTEPS = HD / 32, HK = KSTEPS / 2;
  const float w1 = s.nparts > 1 ? 1.f : 0.f;   // p0 + 1*p1 is p0 + p1 exactly; p0 + 0*p0 is p0
  float x[KSTEPS][8];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
    for (int e = 0; e < 8; ++e) x[ks][e] = r.p0[ks][e >> 2][e & 3] + w1 * r.p1[ks][e >> 2][e & 3];
  for (int p = 2; p < s.nparts; ++p) {         // further partials (unusual shapes), in order
    const float* src = s.qkv + ((size_t)p * s.Mtot + m) * s.ldq + col0 + 8 * g4;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const f32x4 u0 = *reinterpret_cast<const f32x4*>(src + ks * 32), u1 = *reinterpret_cast<const f32x4*>(src + ks * 32 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[ks][e] += u0[e]; x[ks][4 + e] += u1[e]; }
    }
  }
  if (gain) {
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += x[ks][e] * x[ks][e];
    ss += __shfl_xor(ss, 16); ss += __shfl_xor(ss, 32);
    const float rn = rsqrtf(ss / (float)HD + s.eps);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + ks * 32 + 8 * g4);
      const f32x4 g1 = *reinterpret_cast<const f32x4*>(gain + ks * 32 + 8 * g4 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[ks][e] = x[ks][e] * rn * g0[e]; x[ks][4 + e] = x[ks][4 + e] * rn * g1[e]; }
    }
  }
#pragma unroll
  for (int ks = 0; ks < HK; ++ks) {
    float y0[8], y1[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float c = r.cs[ks][e >> 2][e & 3], sv = r.sn[ks][e >> 2][e & 3];
      const float x0 = x[ks][e], x1 = x[ks + HK][e];
      y0[e] = x0 * c - x1 * sv; y1[e] = x0 * sv + x1 * c;
    }
    out[ks] = frag_round(y0, T());
    out[ks + HK] = frag_round(y1, T());
  }
}

template <typename T, int HD>
__device__ __forceinline__ void rope_head(const QkvSrc& s, int m, int col0, const float* gain, int pos, int g4,
                                          Frag<T> (&out)[HD / 32]) {
  HeadRaw<HD> r;
  head_load<HD>(s, m, col0, pos, g4, r);
  head_finish<T, HD>(s, r, m, col0, gain, g4, out);
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
  QkvSrc src;                       // the window rows' q / k / v as the projection left them
  const T* qbuf;                    // throughput form only: the queries, already normed / rotated / rounded
  const T *kc, *vt;                 // KV cache, offset to the layer: the tokens before the window
  const int32_t* kv_len;
  const int32_t* page_table;        // paged cache: [max_batch][pps] page ids (page = KV_PAGE tokens of every kv head)
  int pps;                          //   pages per sequence
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

// The shared form's second product with the probabilities as ONE fp16 operand (11 significant bits, rounded to
// nearest) against V^T fragments converted to fp16 when they were staged: a third fewer matrix instructions and a
// fraction of the conversion work of the head + tail split.  A probability's rounding error (2^-12 relative at
// most) is an eighth of the bf16 step the attention output is rounded to afterwards.
template <int HT>
__device__ __forceinline__ void pv_accumulate_f16(f32x4 (&o)[HT], const u32x4 (&vf)[HT], f32x4 a, f32x4 b) {
  const u32x4 p = {pack_f16(a.x, a.y), pack_f16(a.z, a.w), pack_f16(b.x, b.y), pack_f16(b.z, b.w)};
#pragma unroll
  for (int h = 0; h < HT; ++h)
    o[h] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, vf[h]), __builtin_bit_cast(f16x8, p), o[h], 0, 0, 0);
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

// One wave: NB consecutive 16-row query blocks (from block qb0) of (b, kv head) = bh against split sp.
// The P = kv_len[b] cached tokens are cut into nsplit - 1 ranges; the last split takes the k window
// rows themselves, whose keys and values are not in the cache yet: it builds them from the
// projection result (one 32-token step, row j sees window rows 0..j).  With nsplit = 1 the one
// split does both.
// NB > 1 keeps the K/V fragments of a step in registers for NB query blocks: at long contexts and
// many query rows the kernel is bound by the bytes the four waves of a CU pull through its L1
// (every wave 16 KiB per 32-token step, about 1000 cycles for the four), not by its arithmetic, and
// a second block per wave halves those bytes per query row.
// WIN_ONLY: the caller's splits over cached tokens are handled elsewhere (attn_shared_kernel); only the window split is compiled.
template <typename T, int HD, int PRE, bool PAGED, int NB, bool WIN_ONLY = false>
__device__ __forceinline__ void attn_task(const AttnArgs<T>& a, int bh, int sp, int qb0) {
  constexpr int KSTEPS = HD / 32, HT = HD / 16;
  constexpr bool HALF_REGS = PRE == 2 && sizeof(T) == 2 && NB == 1;   // see attn_split_kernel
  constexpr bool QBUF = HALF_REGS || NB > 1;                          // queries prepared by rope_q_kernel
  const int lane = threadIdx.x & 63, c = lane & 15, g4 = lane >> 4;
  const int kvh = bh % a.Hkv; const int b = bh / a.Hkv;
  const int P = min(a.kv_len[b], a.max_ctx - a.k);   // (the host refuses windows that do not fit)
  const int ncs = a.nsplit - 1;                      // splits over the cached tokens; the last split is the window
  const bool win = sp == ncs;
  int t0 = 0, t1 = P;
  if (ncs > 0) {
    int per = (P + ncs - 1) / ncs;
    per = (per + 31) & ~31;                          // token ranges start on 32-token steps
    t0 = min(P, sp * per); t1 = win ? t0 : min(P, t0 + per);
  }
  const int nq = a.g * a.k;
  int row[NB], jrow[NB];
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    row[n] = (qb0 + n) * 16 + c;
    jrow[n] = row[n] < nq ? row[n] / a.g : -1;
  }
  const T* kbase = a.kc + (size_t)(b * a.Hkv + kvh) * a.max_ctx * HD;
  const T* vbase = a.vt + (size_t)(b * a.Hkv + kvh) * a.max_ctx * HD;

  f32x4 o[NB][HT];
  float mrun[NB], lrun[NB];
  Frag<T> qf[NB][KSTEPS];   // query fragments (B operand): dims ks*32 + 8*g4 .. of query row `row` = (window row, head in group)
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    mrun[n] = -INFINITY; lrun[n] = 0.f;
#pragma unroll
    for (int h = 0; h < HT; ++h) o[n][h] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // One 32-token step: scores, online soft-max, O^T += V^T P^T for every block of the wave.  Token
  // tb + i is visible to this lane's query row of block n iff tb + i <= lim[n]; `open` (the same for
  // the whole wave) says that all 32 tokens are visible to every row, so that nothing is compared
  // (rows beyond the last query row then work on the last row's query: finite values that nobody
  // reads).  The running sums are rescaled only when some lane's maximum grew: for the others the
  // factor is exactly 1.
  auto step = [&](const KvFrags<T, HD>& f, int tb, const int (&lim)[NB], bool open) {
    f32x4 s[NB][2];
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        s[n][h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) s[n][h] = mma(f.kf[h][ks], qf[n][ks], s[n][h]);
      }
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      // lane holds scores of query row c for tokens tb + 16*h + 4*g4 + i
      float mx = -INFINITY;
      if (open) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) { const float v = s[n][h][i] * a.scale; s[n][h][i] = v; mx = fmaxf(mx, v); }
      } else {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int tok = tb + 16 * h + 4 * g4 + i;
            const float v = tok <= lim[n] ? s[n][h][i] * a.scale : -INFINITY;
            s[n][h][i] = v; mx = fmaxf(mx, v);
          }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun[n], mx);
      float psum = 0.f;
      if (mnew > -INFINITY) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) { const float p = fast_exp2(s[n][h][i] - mnew); s[n][h][i] = p; psum += p; }
      } else {
        s[n][0] = f32x4{0.f, 0.f, 0.f, 0.f}; s[n][1] = s[n][0];
      }
      if (__builtin_amdgcn_ballot_w64(mnew > mrun[n]) != 0) {
        const float alpha = mnew > mrun[n] ? fast_exp2(mrun[n] - mnew) : 1.f;   // 2^(-inf) = 0 on the first visible step
        lrun[n] *= alpha;               // per-lane share; lane groups are summed at the end
#pragma unroll
        for (int h = 0; h < HT; ++h) o[n][h] = o[n][h] * alpha;
      }
      mrun[n] = mnew;
      lrun[n] += psum;
      pv_accumulate<HT>(o[n], f.vf, s[n][0], s[n][1]);
    }
  };

  int qr[NB], qj[NB], qm[NB], qcol[NB];
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    qr[n] = min(row[n], nq - 1); qj[n] = qr[n] / a.g; qm[n] = b * a.k + qj[n]; qcol[n] = (kvh * a.g + qr[n] % a.g) * HD;
  }
  // throughput form: a wave handles many steps and a (b, kv head, query block) has many splits,
  // so the queries are prepared once by rope_q_kernel instead of by every wave
  auto load_q = [&]() {
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      const T* qp = a.qbuf + ((size_t)(b * a.Hkv + kvh) * a.qrows_pad + qr[n]) * HD + g4 * 8;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) qf[n][ks] = frag_load_row(qp + ks * 32);
    }
  };
  const int kcol = (a.src.H + kvh) * HD, vcol = (a.src.H + a.src.Hkv + kvh) * HD;
  const size_t pstride = (size_t)a.src.Mtot * a.src.ldq;
  const int w1 = a.src.nparts > 1 ? 1 : 0;

  // The window rows as virtual tokens 0..k-1, sixteen at a time (one round in a decoding
  // window, two in a prefill-sized one), in the operand layouts of load_kv with the second
  // 16-token tile left empty.  Key fragment: token r0 + c, dims of lane group g4.  V^T
  // fragment: lane (dim h*16 + c) needs tokens r0 + 4*g4 + {0..3}.  Loads and arithmetic are
  // separate so that the caller can have everything in flight before it waits.
  struct WinRaw { HeadRaw<HD> k; float v0[HT][4], v1[HT][4]; };
  auto win_load_k = [&](WinRaw& w, int r0) {
    const int v = min(r0 + c, a.k - 1);
    head_load<HD>(a.src, b * a.k + v, kcol, P + v, g4, w.k);
  };
  auto win_load_v = [&](WinRaw& w, int r0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float* q = a.src.qkv + (size_t)(b * a.k + min(r0 + 4 * g4 + e, a.k - 1)) * a.src.ldq + vcol + c;
#pragma unroll
      for (int h = 0; h < HT; ++h) { w.v0[h][e] = *(q + h * 16); w.v1[h][e] = *(q + w1 * pstride + h * 16); }
    }
  };
  auto win_step = [&](WinRaw& w, KvFrags<T, HD>& fw, int r0) {
    head_finish<T, HD>(a.src, w.k, b * a.k + min(r0 + c, a.k - 1), kcol, a.src.gk, g4, fw.kf[0]);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) frag_zero(fw.kf[1][ks]);
    if constexpr (HALF_REGS) win_load_v(w, r0);   // (the registers do not hold both sets of loads at once)
#pragma unroll
    for (int h = 0; h < HT; ++h) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[e] = 0.f + w.v0[h][e] + (float)w1 * w.v1[h][e]; x[4 + e] = 0.f; }
      for (int p = 2; p < a.src.nparts; ++p) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          x[e] += *(a.src.qkv + p * pstride + (size_t)(b * a.k + min(r0 + 4 * g4 + e, a.k - 1)) * a.src.ldq + vcol + c + h * 16);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (r0 + 4 * g4 + e >= a.k) x[e] = 0.f;
      fw.vf[h] = frag_round(x, T());
    }
    int lim[NB];
#pragma unroll
    for (int n = 0; n < NB; ++n) lim[n] = min(jrow[n], r0 + 15);
    step(fw, r0, lim, false);
  };

  if (win && ncs > 0) {
    // the window split proper: query and window rows arrive in one round trip (two in the
    // throughput form, whose registers do not hold all of it at once)
    WinRaw w;
    if constexpr (!QBUF) {
      HeadRaw<HD> qraw;
      head_load<HD>(a.src, qm[0], qcol[0], P + qj[0], g4, qraw);
      win_load_k(w, 0); win_load_v(w, 0);
      head_finish<T, HD>(a.src, qraw, qm[0], qcol[0], a.src.gq, g4, qf[0]);
    } else {
      load_q();
      win_load_k(w, 0);
      if constexpr (!HALF_REGS) win_load_v(w, 0);
    }
    KvFrags<T, HD> fw;
    win_step(w, fw, 0);
    if (a.k > 16) {
      win_load_k(w, 16);
      if constexpr (!HALF_REGS) win_load_v(w, 16);
      win_step(w, fw, 16);
    }
  } else if constexpr (!WIN_ONLY) {
    // The K/V of PRE steps are requested together, before any of them is used: a step
    // computes in a fraction of a memory round trip, so fetching only one step ahead costs one
    // round trip per step.  PRE = 4 (128 tokens) needs the CU's registers for one workgroup:
    // right when there is at most one workgroup per CU; with more workgroups than CUs PRE = 2
    // lets two of them share a CU.  The first group is requested before the query is built, so
    // that both arrive in the same round trip.
    // Steps beyond the range re-read its first step (a valid address) and are skipped.
    KvFrags<T, HD> f[PRE];
    // (paged cache: a 32-token step lies inside one page; the page of every step is looked up)
    auto load_group = [&](KvFrags<T, HD> (&fb)[PRE], int tg, int fallback) {
#pragma unroll
      for (int u = 0; u < PRE; ++u) {
        const int tb = tg + 32 * u < t1 ? tg + 32 * u : fallback;
        if constexpr (PAGED) {
          const size_t po = ((size_t)a.page_table[b * a.pps + tb / KV_PAGE] * a.Hkv + kvh) * KV_PAGE * HD;
          load_kv<T, HD>(fb[u], a.kc + po, a.vt + po, tb % KV_PAGE, lane);
        } else {
          load_kv<T, HD>(fb[u], kbase, vbase, tb, lane);
        }
      }
    };
    int lim_c[NB];                                       // every cached token is visible to every window row
#pragma unroll
    for (int n = 0; n < NB; ++n) lim_c[n] = jrow[n] < 0 ? -1 : t1 - 1;
    auto run_group = [&](const KvFrags<T, HD> (&fb)[PRE], int tg) {
#pragma unroll
      for (int u = 0; u < PRE; ++u)
        if (tg + 32 * u < t1) step(fb[u], tg + 32 * u, lim_c, tg + 32 * u + 32 <= t1);
    };
    if constexpr (!QBUF) {
      // latency form (a group or two per wave): the first group is requested before the query
      load_group(f, t0, t0 < t1 ? t0 : 0);
      rope_head<T, HD>(a.src, qm[0], qcol[0], a.src.gq, P + qj[0], g4, qf[0]);
      for (int tg = t0; tg < t1;) {
        run_group(f, tg);
        tg += 32 * PRE;
        if (tg < t1) load_group(f, tg, t0);
      }
    } else if constexpr (NB > 1) {
      // several blocks per wave, one wave per SIMD, nobody else to hide the loads behind: two sets of
      // fragments, the next group requested (unconditionally: beyond the range it re-reads the
      // range's first step) before the current one is worked on
      KvFrags<T, HD> f2[PRE];
      load_q();
      load_group(f, t0, t0 < t1 ? t0 : 0);
      for (int tg = t0; tg < t1; tg += 64 * PRE) {
        load_group(f2, tg + 32 * PRE, t0 < t1 ? t0 : 0);
        run_group(f, tg);
        load_group(f, tg + 64 * PRE, t0 < t1 ? t0 : 0);
        run_group(f2, tg + 32 * PRE);
      }
    } else {
      // throughput form (many groups per wave, two waves per SIMD): loads unconditional and
      // first in the loop body, so that the steps wait for their own fragments only and step u
      // runs while the fragments of step u+1 are still arriving
      load_q();
      for (int tg = t0; tg < t1; tg += 32 * PRE) {
        load_group(f, tg, t0);
        run_group(f, tg);
      }
    }
    if (win) {   // a single split does everything (empty or very short caches)
      WinRaw w;
      for (int r0 = 0; r0 < a.k; r0 += 16) {
        win_load_k(w, r0);
        if constexpr (!HALF_REGS) win_load_v(w, r0);
        win_step(w, f[0], r0);
      }
    }
  }
  // write the partials (blocks beyond the last one fall inside the padded rows and are never read)
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    float l = lrun[n];
    l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
    const size_t pidx = ((size_t)(b * a.Hkv + kvh) * a.nsplit + sp) * a.qrows_pad + row[n];
    if (row[n] < a.qrows_pad) {
      if (g4 == 0) { a.pm[pidx] = mrun[n]; a.pl[pidx] = l; }
#pragma unroll
      for (int h = 0; h < HT; ++h) *reinterpret_cast<f32x4*>(a.po + pidx * HD + h * 16 + 4 * g4) = o[n][h];
    }
  }
}

// grid = B * Hkv * nsplit * ceil(nqw / wpg) workgroups of wpg waves, nqw = ceil(nqb / NB) waves'
// worth of query blocks; the waves of a workgroup own consecutive query blocks of the same K/V
// range, so those reads are shared through the CU's L1.  The workgroups of the cached ranges come
// first, the (short) window splits last: when the grid is larger than the chip holds at once, the
// ones that wait for a free slot are short.
// (PRE = 2 with one block per wave in bf16 is the form for more workgroups than CUs: held to two waves per SIMD.)
template <typename T, int HD, int PRE, bool PAGED, int NB = 1>
__global__ void __launch_bounds__(256, (PRE == 2 && sizeof(T) == 2 && NB == 1) ? 2 : 1) attn_split_kernel(const AttnArgs<T> a) {
  const int wpg = blockDim.x >> 6;
  const int nqw = (a.nqb + NB - 1) / NB;
  const int nqg = (nqw + wpg - 1) / wpg;
  const int ncs = a.nsplit - 1;
  const int ncache = (int)(gridDim.x / a.nsplit) * ncs;   // gridDim.x = (B * Hkv * nqg) * nsplit
  int blk = blockIdx.x, sp, bh, qg;
  if (blk < ncache) { qg = blk % nqg; sp = (blk / nqg) % ncs; bh = blk / (nqg * ncs); }
  else { blk -= ncache; qg = blk % nqg; sp = ncs; bh = blk / nqg; }
  const int qw = qg * wpg + (threadIdx.x >> 6);
  if (qw >= nqw) return;
  attn_task<T, HD, PRE, PAGED, NB>(a, bh, sp, qw * NB);
}

// Shared form of the split-KV attention (bf16), for many query rows over long cached ranges.  The NW
// waves of a workgroup own NB consecutive 16-row query blocks each and walk the SAME token range in
// step: every 32-token step of K and V^T (FR fragments of 1 KiB, contiguous in the cache's tiled
// order) is fetched from memory once per workgroup, FR / NW fragments per wave, DEPTH steps ahead
// into registers, passed through one of two LDS buffers (one barrier per step: a buffer is written
// again only after the barrier that follows its last readers' next step), and read from there by
// every wave as the MFMA operands of its own blocks.  Against attn_split_kernel's forms, where
// each wave pulls the whole range through the CU's L1 for itself, the bytes through L1 fall by NW,
// a wave needs registers for one step of operands only, so two waves per SIMD fit, and little
// register space buys a deep prefetch.  (Running half of the waves one phase behind the others, so
// that one wave's soft-max arithmetic meets the other's second product, was measured: no gain.)
// Splits and partials are attn_split_kernel's; the window split (last in the grid) runs attn_task's
// window path, one query block per wave.  Queries come from rope_q_kernel.  The host picks this form only with at least
// one split over cached tokens.
// PH: the probabilities enter the second product as fp16 (pv_accumulate_f16) instead of a bf16 head + tail.
template <typename T, int HD, bool PAGED, int NB, int NW, bool PH>
__global__ void __launch_bounds__(64 * NW, 2) attn_shared_kernel(const AttnArgs<T> a) {
  static_assert(sizeof(T) == 2, "bf16 caches only");
  constexpr int KSTEPS = HD / 32, HT = HD / 16, FR = 2 * KSTEPS + HT;
  constexpr int FPW = FR / NW;                          // fragments a wave fetches per step
  constexpr int DEPTH = NW == 2 ? 2 : NW == 4 ? 3 : 4;  // steps in flight per wave (deeper, 3 / 4 / 6, measured the same)
  static_assert(FR % NW == 0, "the fragments of a step are shared out evenly");
  __shared__ u32x4 stage_k[2][2 * KSTEPS][WAVE];
  __shared__ u32x4 stage_v[2][HT][WAVE];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 15, g4 = lane >> 4;
  const int nqw = (a.nqb + NB - 1) / NB, nqg = (nqw + NW - 1) / NW, ncs = a.nsplit - 1;
  // gridDim.x = (B * Hkv * nqg) * (ncs + NB): the workgroups of the cached ranges, then, for the window rows
  // themselves, NB workgroups per group whose waves take one query block each (no barriers on that path)
  const int ncache = (int)(gridDim.x / (ncs + NB)) * ncs;
  int blk = blockIdx.x;
  if (blk >= ncache) {
    blk -= ncache;
    const int qb = (blk % (nqg * NB)) * NW + wave;
    if (qb < a.nqb) attn_task<T, HD, 2, PAGED, 1, true>(a, blk / (nqg * NB), ncs, qb);
    return;
  }
  const int qg = blk % nqg, sp = (blk / nqg) % ncs, bh = blk / (nqg * ncs);
  const int qw = qg * NW + wave;
  // waves beyond the last query block fetch their share of K/V like the others; their results are dropped
  const int kvh = bh % a.Hkv, b = bh / a.Hkv;
  const int P = min(a.kv_len[b], a.max_ctx - a.k);
  int per = (P + ncs - 1) / ncs;
  per = (per + 31) & ~31;
  const int t0 = min(P, sp * per), t1 = min(P, t0 + per);
  const int tfirst = t0 < t1 ? t0 : 0;                  // where fetches beyond the range go: a valid step
  const int nsteps = (t1 - t0 + 31) >> 5;
  const int nq = a.g * a.k, qb0 = qw * NB;
  const T* kbase = a.kc + (size_t)(b * a.Hkv + kvh) * a.max_ctx * HD;
  const T* vbase = a.vt + (size_t)(b * a.Hkv + kvh) * a.max_ctx * HD;

  int row[NB], lim[NB];
  Frag<T> qf[NB][KSTEPS];
  f32x4 o[NB][HT];
  float mrun[NB], lrun[NB];
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    row[n] = (qb0 + n) * 16 + c;
    lim[n] = row[n] < nq ? t1 - 1 : -1;                 // every cached token is visible to every window row
    const T* qp = a.qbuf + ((size_t)(b * a.Hkv + kvh) * a.qrows_pad + min(row[n], nq - 1)) * HD + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) qf[n][ks] = frag_load_row(qp + ks * 32);
    mrun[n] = -INFINITY; lrun[n] = 0.f;
#pragma unroll
    for (int h = 0; h < HT; ++h) o[n][h] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // this wave's fragments wave, wave + NW, ... of the step that starts at token tb (a multiple of 32)
  auto fetch = [&](u32x4 (&dst)[FPW], int tb) {
    const T *kp, *vp;
    if constexpr (PAGED) {
      const size_t po = ((size_t)a.page_table[b * a.pps + tb / KV_PAGE] * a.Hkv + kvh) * KV_PAGE * HD;
      const int tp = tb % KV_PAGE;
      kp = a.kc + po + (size_t)(tp >> 4) * (KSTEPS * 512); vp = a.vt + po + (size_t)(tp >> 5) * (HT * 512);
    } else {
      kp = kbase + (size_t)(tb >> 4) * (KSTEPS * 512); vp = vbase + (size_t)(tb >> 5) * (HT * 512);
    }
#pragma unroll
    for (int i = 0; i < FPW; ++i) {
      const int fi = wave + i * NW;
      const T* src = fi < 2 * KSTEPS ? kp + fi * 512 : vp + (fi - 2 * KSTEPS) * 512;
      dst[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + lane);   // read once: streaming
    }
  };

  // S phase of a step: scores of this lane's query row for tokens tb + 16*h + 4*g4 + i, online soft-max as
  // in attn_task's step (running maximum, sum and the rescaling of O^T); leaves the probabilities in pr.
  // P phase: O^T += V^T P^T with the V^T fragments of the same step.
  f32x4 pr[NB][2];
  auto s_phase = [&](const u32x4 (&bk)[2 * KSTEPS][WAVE], int tb) {
    const bool open = tb + 32 <= t1;
    {
      Frag<T> kf[2][KSTEPS];
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) kf[h][ks].v = bk[h * KSTEPS + ks][lane];
#pragma unroll
      for (int n = 0; n < NB; ++n)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          pr[n][h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KSTEPS; ++ks) pr[n][h] = mma(kf[h][ks], qf[n][ks], pr[n][h]);
        }
    }
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      // the scale (positive) is applied to the row maximum and inside the exponent's fused multiply-add,
      // not to the eight scores one by one
      float mx = -INFINITY;
      if (open) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) mx = fmaxf(mx, pr[n][h][i]);
      } else {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int tok = tb + 16 * h + 4 * g4 + i;
            const float v = tok <= lim[n] ? pr[n][h][i] : -INFINITY;
            pr[n][h][i] = v; mx = fmaxf(mx, v);
          }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun[n], mx * a.scale);
      float psum = 0.f;
      if (mnew > -INFINITY) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) { const float p = fast_exp2(fmaf(pr[n][h][i], a.scale, -mnew)); pr[n][h][i] = p; psum += p; }
      } else {
        pr[n][0] = f32x4{0.f, 0.f, 0.f, 0.f}; pr[n][1] = pr[n][0];
      }
      if (__builtin_amdgcn_ballot_w64(mnew > mrun[n]) != 0) {
        const float alpha = mnew > mrun[n] ? fast_exp2(mrun[n] - mnew) : 1.f;
        lrun[n] *= alpha;
#pragma unroll
        for (int h = 0; h < HT; ++h) o[n][h] = o[n][h] * alpha;
      }
      mrun[n] = mnew;
      lrun[n] += psum;
    }
  };
  auto p_phase = [&](const u32x4 (&bv)[HT][WAVE]) {
    if constexpr (PH) {
      u32x4 vh[HT];
#pragma unroll
      for (int h = 0; h < HT; ++h) vh[h] = bv[h][lane];
#pragma unroll
      for (int n = 0; n < NB; ++n) pv_accumulate_f16<HT>(o[n], vh, pr[n][0], pr[n][1]);
    } else {
      Frag<T> vf[HT];
#pragma unroll
      for (int h = 0; h < HT; ++h) vf[h].v = bv[h][lane];
#pragma unroll
      for (int n = 0; n < NB; ++n) pv_accumulate<HT>(o[n], vf, pr[n][0], pr[n][1]);
    }
  };

  u32x4 pre[DEPTH][FPW];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) fetch(pre[d], d < nsteps ? t0 + 32 * d : tfirst);
  // Every round of the loop stages and fetches DEPTH steps, whether the range still has them or not (steps
  // beyond it re-fetch a valid step and are not computed on): the loads in flight are then the same at the
  // loop's head and end, and every wait inside counts exactly the loads that are younger than the one it needs.
  for (int s0 = 0; s0 < nsteps; s0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int st = s0 + d;
#pragma unroll
      for (int i = 0; i < FPW; ++i) {
        const int fi = wave + i * NW;
        if (fi < 2 * KSTEPS) stage_k[st & 1][fi][lane] = pre[d][i];
        else if constexpr (PH)   // V^T is converted once per workgroup here, not once per reader
          stage_v[st & 1][fi - 2 * KSTEPS][lane] = u32x4{bf16x2_to_f16x2(pre[d][i].x), bf16x2_to_f16x2(pre[d][i].y),
                                                         bf16x2_to_f16x2(pre[d][i].z), bf16x2_to_f16x2(pre[d][i].w)};
        else stage_v[st & 1][fi - 2 * KSTEPS][lane] = pre[d][i];
      }
      fetch(pre[d], st + DEPTH < nsteps ? t0 + 32 * (st + DEPTH) : tfirst);
      __syncthreads();
      if (st < nsteps) {
        s_phase(stage_k[st & 1], t0 + 32 * st);
        p_phase(stage_v[st & 1]);
      }
    }
  }
  // the partials, as attn_task leaves them
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    float l = lrun[n];
    l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
    const size_t pidx = ((size_t)(b * a.Hkv + kvh) * a.nsplit + sp) * a.qrows_pad + row[n];
    if (qb0 + n < a.nqb && row[n] < a.qrows_pad) {
      if (g4 == 0) { a.pm[pidx] = mrun[n]; a.pl[pidx] = l; }
#pragma unroll
      for (int h = 0; h < HT; ++h) *reinterpret_cast<f32x4*>(a.po + pidx * HD + h * 16 + 4 * g4) = o[n][h];
    }
  }
}

// Queries for the throughput form of the attention: wave w handles 16 query rows of the
// (b, kv head, row) list, four lanes (one per dim group) each -> qbuf[b][kvh][row][HD].
template <typename T>
struct RopeQArgs {
  QkvSrc src;
  const int32_t* kv_len;
  T* qbuf;
  int B, k, g, qrows_pad, max_ctx;
};

template <typename T, int HD>
__global__ void __launch_bounds__(256) rope_q_kernel(const RopeQArgs<T> a) {
  constexpr int KSTEPS = HD / 32;
  const int w = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, c = lane & 15, g4 = lane >> 4;
  const int nq = a.g * a.k, nitems = a.B * a.src.Hkv * nq;
  if (w * 16 >= nitems) return;
  const int item = w * 16 + c, it = min(item, nitems - 1);
  const int row = it % nq, kvh = (it / nq) % a.src.Hkv, b = it / (nq * a.src.Hkv);
  const int j = row / a.g, hh = kvh * a.g + row % a.g;
  const int P = min(a.kv_len[b], a.max_ctx - a.k);
  Frag<T> qf[KSTEPS];
  rope_head<T, HD>(a.src, b * a.k + j, hh * HD, a.src.gq, P + j, g4, qf);
  if (item < nitems) {
    T* dst = a.qbuf + ((size_t)(b * a.src.Hkv + kvh) * a.qrows_pad + row) * HD + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) *reinterpret_cast<Frag<T>*>(dst + ks * 32) = qf[ks];
  }
}

// Merge the split partials of one (row m, query head): softmax-weighted sum,
// normalise, round to T, write attn[m][head*hd + :].  One wave per task = (m, head);
// nsplit <= 64: lane s first handles split s's (m, l), then every lane owns HD/64
// consecutive output dims and walks the splits with the weights broadcast by shuffle.
template <typename T>
struct CombineArgs {
  const float *pm, *pl, *po;
  T* attn; int ldat;
  int tiled;                        // attn in the fragment-tiled layout (more than 16 rows) or row-major
  int Mtot, k, H, Hkv, qrows_pad, nsplit;
  // KV append (the same launch, further waves): the window rows' keys and values go to
  // cache positions kv_len[b] + j
  QkvSrc src;
  const int32_t* kv_len;
  T *kc, *vt;                       // offset to the layer
  int max_ctx;
  const int32_t* page_table;        // paged cache (else nullptr): [max_batch][pps]
  int pps;
};

// element offset of (sequence b, kv head, position pos) in a layer's cache, up to the
// position-inside-the-tiles part that kc_offset / vt_offset add (pos_local)
template <typename T>
__device__ __forceinline__ size_t cache_base(const CombineArgs<T>& a, int b, int kvh, int pos, int hd, int& pos_local) {
  if (a.page_table) {
    pos_local = pos % KV_PAGE;
    return ((size_t)a.page_table[b * a.pps + pos / KV_PAGE] * a.Hkv + kvh) * KV_PAGE * hd;
  }
  pos_local = pos;
  return (size_t)(b * a.Hkv + kvh) * a.max_ctx * hd;
}

// Key append: wave w handles 16 (row, kv head) items, four lanes (one per dim group) each:
// item = m * Hkv + kvh -> norm, rotary embedding, one 8-element store per fragment.
// Nobody reads these cache rows before the next kernel starts (the attention of this layer
// took the window rows from the projection result).
template <typename T, int HD>
__device__ __forceinline__ void append_k_task(const CombineArgs<T>& a, int w) {
  constexpr int KSTEPS = HD / 32;
  const int lane = threadIdx.x & 63, c = lane & 15, g4 = lane >> 4;
  const int nitems = a.Mtot * a.Hkv;
  const int item = w * 16 + c, it = min(item, nitems - 1);
  const int m = it / a.Hkv, kvh = it % a.Hkv;
  const int b = m / a.k, j = m % a.k;
  const int pos = a.kv_len[b] + j;
  const bool live = item < nitems && pos < a.max_ctx;   // capacity guard; the host refuses such calls
  Frag<T> kf[KSTEPS];
  rope_head<T, HD>(a.src, m, (a.src.H + kvh) * HD, a.src.gk, min(pos, a.max_ctx - 1), g4, kf);
  if (live) {
    int pl;
    T* dst = a.kc + cache_base(a, b, kvh, pos, HD, pl);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) *reinterpret_cast<Frag<T>*>(dst + kc_offset(pl, ks * 32 + 8 * g4, HD)) = kf[ks];
  }
}

// Value append: one wave per (row m, kv head), lane = dim (and dim + 64): the transposed
// cache takes single elements, so the stores are spread over as many lanes as possible.
template <typename T, int HD>
__device__ __forceinline__ void append_v_task(const CombineArgs<T>& a, int w) {
  const int lane = threadIdx.x & 63;
  const int m = w / a.Hkv, kvh = w % a.Hkv;
  const int b = m / a.k, j = m % a.k;
  const int pos = a.kv_len[b] + j;
  if (pos >= a.max_ctx) return;
  const size_t pstride = (size_t)a.src.Mtot * a.src.ldq;
  const float* src = a.src.qkv + (size_t)m * a.src.ldq + (size_t)(a.src.H + a.src.Hkv + kvh) * HD;
  int pl;
  T* dst = a.vt + cache_base(a, b, kvh, pos, HD, pl);
#pragma unroll
  for (int d = lane; d < HD; d += 64) {
    float x = src[d];
    for (int p = 1; p < a.src.nparts; ++p) x += src[d + p * pstride];
    st_round1(dst + vt_offset(pl, d, HD), x);
  }
}

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
  T* dst = a.tiled ? a.attn + xt_offset(m, hh * HD + lane * DPL, a.ldat)
                   : a.attn + (size_t)m * a.ldat + (size_t)hh * HD + lane * DPL;
  if (DPL == 2 && sizeof(T) == 2) {
    *reinterpret_cast<uint32_t*>(dst) = (pack_bf16(acc[0] * inv, acc[DPL - 1] * inv));
  } else {
#pragma unroll
    for (int i = 0; i < DPL; ++i) st_round1(dst + i, acc[i] * inv);
  }
}

// waves 0 .. Mtot*H-1 merge; then ceil(Mtot*Hkv / 16) key-append waves; then Mtot*Hkv
// value-append waves
template <typename T>
__host__ __device__ inline int combine_waves(int Mtot, int H, int Hkv) { return Mtot * H + (Mtot * Hkv + 15) / 16 + Mtot * Hkv; }

template <typename T, int HD>
__global__ void __launch_bounds__(256) attn_combine_kernel(const CombineArgs<T> a) {
  int task = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int nmerge = a.Mtot * a.H, nk = (a.Mtot * a.Hkv + 15) / 16, nv = a.Mtot * a.Hkv;
  if (task < nmerge) { combine_task<T, HD>(a, task); return; }
  task -= nmerge;
  if (task < nk) { append_k_task<T, HD>(a, task); return; }
  task -= nk;
  if (task < nv) append_v_task<T, HD>(a, task);
}

}  // namespace dbl
