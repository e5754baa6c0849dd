// The kernels outside the layer loop: embedding gather, acceptance, n-gram retrieval,
// window build, commit, and the seeded weight generator.
#pragma once
#include "dbl_dev.h"
#include "dbl_gemm.h"
#include "dbl_phases.h"

namespace dbl {

// ------------------------------------------------------------------ embedding

// h[m][:] = E[window[m]][:], hg = h * gain of the first RMSNorm, and the row's sum of
// squares: ssq[m][0] = sum, ssq[m][1..] = 0   (grid = rows, 256 threads).  The kernel also keeps the window for
// the LM head's draft look-up and for acceptance (the caller's buffer is not retained): win_out[m] = the row's
// token, or -1 ("no token") for rows beyond a sequence's own length when win_len is given (ragged windows);
// such rows, like ids outside the vocabulary, embed a valid token and their results are never used.
template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(const T* __restrict__ E, const int32_t* window, const int32_t* __restrict__ win_len,
                                                    int k, int32_t* win_out, float* __restrict__ h, float* __restrict__ hg,
                                                    const float* __restrict__ gain, float* __restrict__ ssq, int d,
                                                    int ldh, int vocab) {
  __shared__ float scratch[16];
  const int m = blockIdx.x;
  int tok = window[m];
  if (win_len && (m % k) >= win_len[m / k]) tok = -1;
  if (threadIdx.x == 0) win_out[m] = tok;
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const T* e = E + (size_t)tok * d;
  float s = 0.f;
  for (int i = 4 * threadIdx.x; i < d; i += 4 * blockDim.x) {      // d is a multiple of 16
    const f32x4 v = {Elem<T>::to_f(e[i]), Elem<T>::to_f(e[i + 1]), Elem<T>::to_f(e[i + 2]), Elem<T>::to_f(e[i + 3])};
    *reinterpret_cast<f32x4*>(h + (size_t)m * ldh + i) = v;
    *reinterpret_cast<f32x4*>(hg + (size_t)m * ldh + i) = v * *reinterpret_cast<const f32x4*>(gain + i);
    s += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
  }
  s = block_sum(s, scratch);
  for (int p = threadIdx.x; p < SSQ_PARTS; p += blockDim.x) ssq[(size_t)m * SSQ_PARTS + p] = p == 0 ? s : 0.f;
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

// One workgroup per sequence.  Merges the LM-head statistics of its k rows (one wave per
// row), runs the acceptance scan, and (dense q only) makes one pass over the rejected row to
// draw from max(0, p - q).
__global__ void __launch_bounds__(1024) accept_kernel(const AcceptArgs a) {
  __shared__ LmStat row[32];
  __shared__ int s_n, s_need_resid, s_tok;
  __shared__ float s_lse;
  __shared__ int s_keep[32];                 // sampling: whether the draft behind row j survives its test
  __shared__ float rbest[16]; __shared__ int rbest_id[16];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t stepv = a.step + *a.commits;

  // one wave per window row (rows wave, wave + number of waves, ...): each lane merges its share of the
  // per-workgroup statistics, then a butterfly inside the wave; lanes and shares are fixed, so
  // the soft-max sums are always added in the same order
  for (int j = wave; j < a.k; j += (int)(blockDim.x >> 6)) {
    const int m = b * a.k + j;
    LmStat s;
    lm_init(s);
    for (int i = lane; i < a.nstat; i += 64) lm_merge(s, a.stats[(size_t)i * a.Mtot + m]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) lm_merge(s, lm_shfl_xor(s, off));
    if (lane == 0) row[j] = s;
  }
  __syncthreads();

  const int32_t* win = a.window + (size_t)b * a.k;
  // sampling: the test of every draft (Sec. 2.1: keep x with probability min(1, p(x) / q(x))), one thread per row;
  // the scan below stops at the first that fails
  if (a.mode != 0 && tid < a.k - 1) {
    const int j = tid, x = win[j + 1];
    int keep = 0;
    if (x >= 0 && x < a.V && win[0] >= 0) {
      const float lse = row[j].smax + logf(row[j].ssum);
      const float px = expf(row[j].zdraft * a.inv_T - lse);
      const Philox4 r = philox4x32_10((uint32_t)stepv, (uint32_t)b, (uint32_t)j, 0u, (uint32_t)a.seed,
                                      (uint32_t)(a.seed >> 32));
      const float u = u01(r.x);
      const float qx = a.q ? a.q[((size_t)b * (a.k - 1) + j) * a.V + x] : 1.f;
      keep = (u * qx < px) ? 1 : 0;
    }
    s_keep[j] = keep;
  }
  __syncthreads();
  if (tid == 0) {
    // A negative id marks a row beyond the sequence's own window (ragged batches): no draft
    // there, and a sequence whose first row is marked takes no part in the step (n = -1).
    int n = a.k - 1, need = 0, tok = -1;
    if (win[0] < 0) {
      n = -1;
      for (int j = 0; j < a.k; ++j) a.guide[(size_t)b * a.k + j] = -1;
    } else if (a.mode == 0) {
      n = 0;
      while (n < a.k - 1 && win[n + 1] == row[n].best_id) ++n;
      tok = row[n].best_id;
      for (int j = 0; j < a.k; ++j) a.guide[(size_t)b * a.k + j] = row[j].best_id;
    } else {
      for (int j = 0; j < a.k - 1; ++j)
        if (!s_keep[j]) { n = j; break; }   // (a row without a draft, id < 0, never keeps)
      if (n < a.k - 1 && win[n + 1] >= 0) {
        if (a.q) { need = 1; tok = row[n].p1_id; /* fallback if the residual is empty */ }
        else { const int x = win[n + 1]; tok = row[n].p1_id != x ? row[n].p1_id : row[n].p2_id; }
      } else {
        tok = row[n].p1_id;
      }
      for (int j = 0; j < a.k; ++j) a.guide[(size_t)b * a.k + j] = j <= n ? row[j].p1_id : -1;
    }
    s_n = n; s_need_resid = need; s_tok = tok;
    s_lse = (a.mode && n >= 0) ? row[n].smax + logf(row[n].ssum) : 0.f;
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

// Alg. 3's priority search over the prior, the generated text and the rejected chains, with the
// plain search as fallback.  Every thread walks end positions of a buffer.  For an end position
// only its longest match matters (shorter lengths at the same place lose to it), so one packed
// 64-bit maximum decides again:
//   bit 63: found in a tier (beats any fallback hit) | n | 3 - tier | continuation | end.
// Two launches: the scan (workgroup (c, b) takes chunk c of the prior for sequence b; chunk 0
// also the sequence itself and its rejected chains) folds its best key into best[b] with an
// atomic maximum, which does not depend on the order of arrival; the finish kernel decodes
// best[b], copies the continuation and clears best[b] for the next call.
constexpr int TIER_CHUNK = 16384;   // prior tokens per scan workgroup

struct TierArgs {
  const int32_t* prior; int prior_len;
  const int32_t *hist, *hist_len, *prompt_len; int max_hist;
  const int32_t *rej, *rej_len; int rej_cap;
  int n_max, n_min, max_cont;
  unsigned long long* best;      // [B], zero between calls
  int32_t *cont, *cont_len, *match_n, *match_pos, *match_tier;
};

// tokens that follow position e in buf[0..len) up to a separator, at most max_cont
__device__ __forceinline__ int cont_run(const int32_t* buf, int len, int e, int max_cont) {
  int c = 0;
  while (c < max_cont && e + c < len && buf[e + c] >= 0) ++c;
  return c;
}

__global__ void __launch_bounds__(1024) retrieve_tiered_scan_kernel(const TierArgs a) {
  __shared__ unsigned long long wbest[16];
  __shared__ int32_t suf[32];
  const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* h = a.hist + (size_t)b * a.max_hist;
  const int len = min(a.hist_len[b], a.max_hist);
  const int plen = min(a.prompt_len[b], len);
  const int32_t* rj = a.rej + (size_t)b * a.rej_cap;
  const int rlen = min(a.rej_len[b], a.rej_cap);
  const int cap_t = min(a.n_max, len);          // key length in a tier
  if (tid < 32) suf[tid] = (tid < cap_t) ? h[len - 1 - tid] : -2;   // the key read backwards (-2 matches nothing)
  __syncthreads();
  unsigned long long best = 0ull;
  auto offer = [&](int in_tier, int n, int tier, int cl, int e) {
    if (n < a.n_min || cl < 1) return;
    const unsigned long long key = ((unsigned long long)in_tier << 63) | ((unsigned long long)n << 56) |
                                   ((unsigned long long)(3 - tier) << 54) | ((unsigned long long)cl << 32) | (unsigned)e;
    best = key > best ? key : best;
  };
  auto scan = [&](const int32_t* buf, int blen, int e_lo, int e_hi, int tier) {   // end positions e_lo .. e_hi-1
    for (int e = e_lo + tid; e < e_hi; e += blockDim.x) {
      int nm = 0;
      const int cap = min(cap_t, e);
      while (nm < cap && buf[e - 1 - nm] == suf[nm]) ++nm;
      if (nm >= a.n_min) offer(1, nm, tier, cont_run(buf, blen, e, a.max_cont), e);
    }
  };
  scan(a.prior, a.prior_len, max(1, chunk * TIER_CHUNK), min(a.prior_len, (chunk + 1) * TIER_CHUNK), 0);
  if (chunk == 0) {
    scan(rj, rlen, 1, rlen, 2);
    // the sequence itself: tier 1 where the n-gram lies in the generated part, and the fallback
    for (int e = 1 + tid; e <= len - 1; e += blockDim.x) {
      int nm = 0;
      const int cap = min(min(a.n_max, len - 1), e);
      while (nm < cap && h[e - 1 - nm] == suf[nm]) ++nm;
      if (nm >= a.n_min) {
        const int cl = min(a.max_cont, len - e);
        offer(0, nm, 3, cl, e);
        offer(1, min(nm, e - plen), 1, cl, e);
      }
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
    if (best) atomicMax(a.best + b, best);
  }
}

__global__ void __launch_bounds__(64) retrieve_tiered_finish_kernel(const TierArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const unsigned long long best = a.best[b];
  const int n = (int)((best >> 56) & 0x7f), cl = (int)((best >> 32) & 0xffff), e = (int)(best & 0xffffffffu);
  const int tier = best ? ((best >> 63) ? 3 - (int)((best >> 54) & 3) : 3) : -1;
  const int32_t* src = tier == 0 ? a.prior : tier == 2 ? a.rej + (size_t)b * a.rej_cap : a.hist + (size_t)b * a.max_hist;
  for (int i = tid; i < a.max_cont; i += blockDim.x)
    a.cont[(size_t)b * a.max_cont + i] = (best && i < cl) ? src[e + i] : -1;
  __syncthreads();
  if (tid == 0) {
    a.cont_len[b] = best ? cl : 0;
    a.match_n[b] = best ? n : 0;
    a.match_pos[b] = best ? e - n : -1;
    a.match_tier[b] = tier;
    a.best[b] = 0ull;
  }
}

// Rejected tier update (one thread per sequence: a handful of tokens).
__global__ void rejected_update_kernel(int32_t* __restrict__ rej, int32_t* __restrict__ rej_len, int rej_cap,
                                       const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_len, int max_hist,
                                       const int32_t* __restrict__ window, const int32_t* __restrict__ n_acc,
                                       const int32_t* __restrict__ n_draft, int k, int B, int ctx_tokens) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int32_t* h = hist + (size_t)b * max_hist;
  const int32_t* w = window + (size_t)b * k;
  int32_t* r = rej + (size_t)b * rej_cap;
  const int len = min(hist_len[b], max_hist);
  if (w[0] < 0 || n_acc[b] < 0) return;   // the sequence took no part in the step
  const int na = max(0, min(n_acc[b], k - 1));
  int nd = n_draft ? max(0, min(n_draft[b], k - 1)) : k - 1;
  while (nd > na && w[nd] < 0) --nd;      // rows beyond the sequence's own window hold no draft
  const int n_rej = nd - na;
  if (n_rej < 1) return;
  const int avail = len + na;
  const int nctx = min(ctx_tokens, avail);
  int rl = min(rej_len[b], rej_cap);
  if (rl + nctx + n_rej + 1 > rej_cap) return;
  for (int i = 0; i < nctx; ++i) {
    const int p = avail - nctx + i;
    r[rl++] = p < len ? h[p] : w[1 + (p - len)];
  }
  for (int i = 0; i < n_rej; ++i) r[rl++] = w[na + 1 + i];
  r[rl++] = -1;
  rej_len[b] = rl;
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

// ------------------------------------------------- the two-model round (Sec. 4.1, 4.2)

// Target-side window of a Double round: pending token + the unverified drafts U + the target's own retrieved
// guidance Y_p (Sec. 4.2: Y_p = Retrieval(x, d), taken at the end of the text the window covers, i.e. of x + U),
// padded to k rows.  The search is retrieve_kernel's over the virtual sequence history + U (nothing is written
// to the history): longest n first, then the longest continuation (at most min(d, free rows)), then the latest
// occurrence.  One workgroup per sequence.  n_draft[b] = |U| + |Y_p| (the real drafts of the window).
struct GuidedArgs {
  const int32_t *hist, *hist_len; int max_hist;
  const int32_t *ahead, *n_ahead; int max_ahead;      // U: [B][max_ahead], lengths [B] (nullptr: none)
  int n_max, n_min, d, k; int32_t pad;
  int32_t *window, *n_draft;                          // [B][k], [B]
};

__global__ void __launch_bounds__(1024) guided_window_kernel(const GuidedArgs a) {
  __shared__ unsigned long long wbest[16];
  __shared__ int32_t suf[32];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* h = a.hist + (size_t)b * a.max_hist;
  const int32_t* ah = a.ahead ? a.ahead + (size_t)b * a.max_ahead : nullptr;
  const int len = min(a.hist_len[b], a.max_hist);
  const int nu = ah && a.n_ahead ? max(0, min(a.n_ahead[b], min(a.k - 1, a.max_ahead))) : 0;
  const int vlen = len + nu;
  const int mc = min(a.d, a.k - 1 - nu);              // guidance tokens the window has room for
  auto tok = [&](int i) { return i < len ? h[i] : ah[i - len]; };
  const int nm_cap = min(a.n_max, vlen - 1);
  if (tid < 32) suf[tid] = (tid < nm_cap) ? tok(vlen - 1 - tid) : -1;
  __syncthreads();
  unsigned long long best = 0ull;
  if (mc >= 1) {
    for (int e = 1 + tid; e <= vlen - 1; e += blockDim.x) {
      int nm = 0;
      const int cap = min(nm_cap, e);
      while (nm < cap && tok(e - 1 - nm) == suf[nm]) ++nm;
      if (nm >= a.n_min) {
        const int cl = min(mc, vlen - e);
        const unsigned long long key = ((unsigned long long)nm << 48) | ((unsigned long long)cl << 32) | (unsigned)e;
        best = key > best ? key : best;
      }
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
  const int cl = best ? (int)((best >> 32) & 0xffff) : 0, e = (int)(best & 0xffffffffu);
  for (int j = tid; j < a.k; j += blockDim.x) {
    int32_t v;
    if (j == 0) v = len > 0 ? h[len - 1] : a.pad;
    else if (j <= nu) v = ah[j - 1];
    else v = (j - 1 - nu < cl) ? tok(e + j - 1 - nu) : a.pad;
    a.window[(size_t)b * a.k + j] = v;
  }
  if (tid == 0) a.n_draft[b] = nu + cl;
}

// The resolve step of a round (Sec. 4.2 "Forward Guidance", Eq. 6; the branches of Alg. 1 / Alg. 2), one thread per
// sequence.  In: n_u = |U| (the unverified drafts the target's window carried), n_acc and emit of the target's
// acceptance (emit = E: accepted window tokens + the target's own next token), the draft model's new chain X_q
// (it continues x + U) and its length.  The verified text always grows by E.  If a token of U was rejected, or X_q
// disagrees with G = E beyond U (the accepted guidance + the target's token), or X_q does not reach past G, no draft
// survives: U' is empty and the target's tokens stand (Eq. 6: verified draft prefix + target suffix).  Otherwise the
// part of X_q behind G becomes the next round's U' (at most max_u tokens).
// Out: U' and |U'|; text = E + U' (what follows the old verified text now, for the draft's history), its length;
// splice_pos = base_len - n_u (where that text starts in the draft's history, base_len = the draft's history length
// when its chain began); record[b][8] = {n_u, n_acc, |E|, |X_q|, |U'|, tokens of X_q that agree with G,
// length of the draft's text behind the old verified text that stays valid, 0}.
struct MergeArgs {
  int B, k, max_chain, max_u;
  const int32_t *n_u, *n_acc, *emit, *chain, *n_chain, *base_len;
  int32_t *u_out, *n_u_out, *text_out, *n_text_out, *splice_pos, *record;
};

__global__ void merge_kernel(const MergeArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  const int nu = max(0, min(a.n_u[b], a.k - 1));
  const int na = min(a.n_acc[b], a.k - 1);
  const int ne = max(0, na + 1);
  const int nc = max(0, min(a.n_chain[b], a.max_chain));
  const int32_t* E = a.emit + (size_t)b * a.k;
  const int32_t* X = a.chain + (size_t)b * a.max_chain;
  int32_t* U = a.u_out + (size_t)b * a.max_u;
  int32_t* T = a.text_out + (size_t)b * (a.k + a.max_u);
  int kept = 0, agree = 0, valid = max(0, na);        // a rejection inside U: the accepted part of U stays valid
  if (na >= nu) {
    const int g = ne - nu;                            // |G| >= 1
    while (agree < g && agree < nc && X[agree] == E[nu + agree]) ++agree;
    if (agree == g && nc > g) kept = min(nc - g, a.max_u);
    valid = nu + (kept > 0 ? g + kept : agree);
  }
  for (int i = 0; i < ne; ++i) T[i] = E[i];
  for (int i = 0; i < kept; ++i) { U[i] = X[ne - nu + i]; T[ne + i] = U[i]; }
  for (int i = kept; i < a.max_u; ++i) U[i] = -1;
  a.n_u_out[b] = kept;
  a.n_text_out[b] = ne + kept;
  a.splice_pos[b] = a.base_len ? a.base_len[b] - nu : 0;
  int32_t* r = a.record + (size_t)b * 8;
  r[0] = nu; r[1] = na; r[2] = ne; r[3] = nc; r[4] = kept; r[5] = agree; r[6] = valid; r[7] = 0;
}

// hist tokens [from[b], hist_len[b]) -> out[b][0..n), n = min(that many, max_n)
__global__ void history_tail_kernel(const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_len, int max_hist,
                                    const int32_t* __restrict__ from, int max_n, int32_t* __restrict__ out,
                                    int32_t* __restrict__ n_out) {
  const int b = blockIdx.x;
  const int len = min(hist_len[b], max_hist);
  const int f = max(0, min(from[b], len));
  const int n = min(len - f, max_n);
  for (int i = threadIdx.x; i < max_n; i += blockDim.x) out[(size_t)b * max_n + i] = i < n ? hist[(size_t)b * max_hist + f + i] : -1;
  if (threadIdx.x == 0) n_out[b] = n;
}

// The history of sequence b becomes hist[0..pos) + tokens[0..n); the KV rows of the tokens that did not change stay,
// the rest is rolled back (kv_len = min(kv_len, first changed position, new length - 1)).  missing[b] = tokens whose
// KV the model has to compute before the last one is pending again.  One thread per sequence (a few tokens).
__global__ void history_splice_kernel(int32_t* __restrict__ hist, int32_t* __restrict__ hist_len, int32_t* __restrict__ prompt_len,
                                      int32_t* __restrict__ kv_len, int max_hist, int B, const int32_t* __restrict__ pos_in,
                                      const int32_t* __restrict__ tokens, const int32_t* __restrict__ n_in, int max_n,
                                      int32_t* __restrict__ missing, int32_t* __restrict__ status) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int32_t* h = hist + (size_t)b * max_hist;
  const int32_t* t = tokens + (size_t)b * max_n;
  const int old_len = min(hist_len[b], max_hist);
  const int pos = max(0, min(pos_in[b], old_len));
  int n = max(0, min(n_in[b], max_n));
  if (pos + n > max_hist) { n = max_hist - pos; atomicOr(status, 2); }
  int p = 0;
  while (p < n && pos + p < old_len && h[pos + p] == t[p]) ++p;
  for (int i = p; i < n; ++i) h[pos + i] = t[i];
  const int new_len = pos + n;
  hist_len[b] = new_len;
  prompt_len[b] = min(prompt_len[b], new_len);
  const int kl = min(kv_len[b], min(pos + p, max(new_len - 1, 0)));
  kv_len[b] = kl;
  if (missing) missing[b] = max(new_len - 1 - kl, 0);
}

// window[b][j] = hist[kv_len[b] + j] for the tokens between the cache and the pending token (at most k), then padding
__global__ void catchup_window_kernel(const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_len,
                                      const int32_t* __restrict__ kv_len, int max_hist, int k, int32_t pad,
                                      int32_t* __restrict__ window, int32_t* __restrict__ win_len) {
  const int b = blockIdx.x;
  const int len = min(hist_len[b], max_hist), kl = max(0, kv_len[b]);
  const int n = max(0, min(len - 1 - kl, k));
  for (int j = threadIdx.x; j < k; j += blockDim.x) window[(size_t)b * k + j] = j < n ? hist[(size_t)b * max_hist + kl + j] : pad;
  if (threadIdx.x == 0) win_len[b] = n;
}

__global__ void copy_lengths_kernel(const int32_t* kv_len, const int32_t* hist_len, int B, int32_t* kv_out, int32_t* hist_out) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  if (kv_out) kv_out[b] = kv_len[b];
  if (hist_out) hist_out[b] = hist_len[b];
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

// (a flush of every sequence also clears the capacity status word)
__global__ void set_counters_kernel(int32_t* kv_len, int32_t* hist_len, int32_t* prompt_len, int32_t* rej_len, int seq, int B,
                                    int32_t* status) {
  const int b = threadIdx.x;
  if (b < B && (seq < 0 || b == seq)) { kv_len[b] = 0; hist_len[b] = 0; prompt_len[b] = 0; rej_len[b] = 0; }
  if (b == 0 && seq < 0) *status = 0;
}

__global__ void truncate_kernel(int32_t* kv_len, int32_t* hist_len, int32_t* prompt_len, int seq, int new_kv, int new_hist) {
  if (threadIdx.x == 0) {
    if (new_kv >= 0) kv_len[seq] = min(kv_len[seq], new_kv);
    if (new_hist >= 0) { hist_len[seq] = min(hist_len[seq], new_hist); prompt_len[seq] = min(prompt_len[seq], new_hist); }
  }
}

__global__ void fill_u64_kernel(unsigned long long* p, unsigned long long v, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = v;
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

// Seeded stand-in KV rows (measurement aid): elements [0, n) of every (layer, kv head) region
// of one sequence; any bit pattern is a valid entry of the tiled cache layout.
// The value of element i of a (layer, kv head) region is the same in both cache forms.
template <typename T>
__global__ void fill_kv_kernel(T* __restrict__ kc, T* __restrict__ vt, size_t region, size_t layer_stride, int n_regions_per_layer,
                               size_t n, uint64_t seed, const int32_t* __restrict__ pages, size_t page_elems) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int r = blockIdx.y % n_regions_per_layer, l = blockIdx.y / n_regions_per_layer;
  size_t off;
  if (pages) off = (size_t)l * layer_stride + ((size_t)pages[i / page_elems] * n_regions_per_layer + r) * page_elems + i % page_elems;
  else off = (size_t)l * layer_stride + (size_t)r * region + i;
  kc[off] = Elem<T>::from_f(32.f * weight_value(seed, 30, (int)blockIdx.y, i));
  vt[off] = Elem<T>::from_f(32.f * weight_value(seed, 31, (int)blockIdx.y, i));
}

// Copy rows pos0 .. pos0+n-1 of one (layer, sequence) between the tiled cache and a staging buffer in the
// logical order [row][kv head][dim]; to_cache != 0 writes the cache.  kc / vt point at the layer; seq_off is
// the sequence's offset in the contiguous form, pages its page-table row in the paged form.
template <typename T>
__global__ void kv_rows_kernel(T* __restrict__ kc, T* __restrict__ vt, T* __restrict__ stage_k, T* __restrict__ stage_v,
                               size_t seq_off, size_t region, const int32_t* __restrict__ pages, int pos0, int n, int Hkv,
                               int hd, int to_cache) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)n * Hkv * hd) return;
  const int d = (int)(i % hd), h = (int)(i / hd % Hkv), t = pos0 + (int)(i / ((size_t)hd * Hkv));
  size_t base; int tt = t;
  if (pages) { tt = t % KV_PAGE; base = ((size_t)pages[t / KV_PAGE] * Hkv + h) * ((size_t)KV_PAGE * hd); }
  else base = seq_off + (size_t)h * region;
  const size_t ko = base + kc_offset(tt, d, hd), vo = base + vt_offset(tt, d, hd);
  if (to_cache) { kc[ko] = stage_k[i]; vt[vo] = stage_v[i]; }
  else { stage_k[i] = kc[ko]; stage_v[i] = vt[vo]; }
}

__global__ void set_page_kernel(int32_t* table, int idx, int32_t page) { if (threadIdx.x == 0) table[idx] = page; }

__global__ void set_kv_len_kernel(int32_t* kv_len, int seq, int32_t v) { if (threadIdx.x == 0) kv_len[seq] = v; }

__global__ void fill_f32_kernel(float* p, float v, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace dbl
