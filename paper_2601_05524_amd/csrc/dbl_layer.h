// Persistent layer kernel: all decoder layers of one verify step in ONE launch.
//
// Why: a 70B-shaped step is 80 layers x 9 dependent kernels; on MI355X every kernel
// boundary costs ~4.4 us (dispatch + cache write-back / invalidate) and every
// projection another ~6 us to refill the memory pipe -- together ~20% of the step.
// Here one workgroup per CU stays resident (cooperative launch), the nine steps of a
// layer become phases separated by a software grid barrier (~2 us), and the first
// ring of the next projection's weights -- which depend on nothing -- is requested
// before the barrier, so HBM keeps streaming across phase boundaries.
//
// Coherence: each XCD has its own L2, so everything one phase writes and a later
// phase reads (residual stream, normalised activations, split-K partials, q, the new
// K/V rows, attention partials and output, SwiGLU output) moves through the
// agent-coherent accessors of dbl_dev.h (relaxed agent-scope atomics: loads and
// stores are performed at the memory side).  Weights, gains, RoPE tables and the KV
// rows of earlier steps are read-only during the launch and use ordinary loads.
// The barrier itself is a relaxed agent-scope counter; before arriving every thread
// waits for its own memory operations to complete.
//
// Safety: the spin is bounded; a workgroup that waits longer than max_spin polls
// raises the error word, every later barrier returns at once, and all workgroups
// leave the kernel.  The host reports the error after the launch.
#pragma once
#include "dbl_gemm.h"
#include "dbl_phases.h"

namespace dbl {

struct GridBar {
  unsigned count; unsigned pad0[31];   // arrivals since the context was created (never reset; wraps)
  unsigned error; unsigned pad1[31];   // != 0: a barrier timed out (sticky: later launches leave at once)
};

// Every thread of every workgroup calls this the same number of times.  Returns false
// (to all threads of the workgroup) once any barrier of the launch has timed out.
// `base` is the value of the counter when the launch started (the host keeps it: every
// launch adds barriers x workgroups); differences are taken modulo 2^32.
__device__ __forceinline__ bool grid_barrier(GridBar* b, unsigned base, unsigned nwg, unsigned& epoch, unsigned max_spin, int* flag) {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // this thread's loads and stores are done
  __syncthreads();
  if (threadIdx.x == 0) {
    ++epoch;
    const unsigned target = base + epoch * nwg;
    int ok = 1;
    __hip_atomic_fetch_add(&b->count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    while ((int)(__hip_atomic_load(&b->count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
      if (++spins > max_spin || __hip_atomic_load(&b->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
        __hip_atomic_store(&b->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
    *flag = ok;
  }
  __syncthreads();
  return *flag != 0;
}

struct LayerLoopArgs {
  GemmArgs<bf16_t> qkv, o, gu, dn;     // pointers of layer 0
  size_t s_qkv, s_o, s_gu, s_dn;       // per-layer weight strides (elements)
  int nw_qkv, nw_o, nw_gu, nw_dn;      // waves per workgroup each projection uses (<= 8)
  NormArgs<bf16_t> n1, n2;             // gains of layer 0; they advance by d per layer
  RopeArgs<bf16_t> rope;               // q/k gains advance by head_dim, caches by s_kv
  AttnArgs<bf16_t> attn;
  CombineArgs<bf16_t> comb;
  size_t s_kv;
  int n_layers, M, d_parts;
  GridBar* bar;
  unsigned bar_base, max_spin;
  long long* trace;                    // tuning aid: [1 + 9*n_layers] clock values of workgroup 0, or nullptr
};

// KSQ / KSO / KSG / KSD: k-blocks per wave of the q/k/v, output, gate/up and down
// projections (compile-time: the activation registers are indexed statically).
// Requirements checked by the host: bf16, M <= 8 (packed activations), the output projection is not
// K-split (residual epilogue), the down projection goes through partials that the next
// norm folds, head_dim == HD, d_model <= 8192, gridDim.x divisible by every
// projection's SS and >= M.
template <int HD, int KSQ, int KSO, int KSG, int KSD>
__global__ void __launch_bounds__(512) layer_loop_kernel(const LayerLoopArgs a) {
  __shared__ GemmRed red[2];
  __shared__ float scratch[16];
  __shared__ int bar_flag;
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  unsigned epoch = 0;
  Frag<bf16_t> ring[GemmCfg<bf16_t>::RING];

  const int rope_tasks = a.M * (a.rope.H + 2 * a.rope.Hkv);
  const int attn_tasks = (a.M / a.attn.k) * a.attn.Hkv * a.attn.nsplit * a.attn.nqb;
  const int comb_tasks = a.M * a.comb.H;

  int nstamp = 0;
#define DBL_STAMP() do { if (a.trace && wg == 0 && threadIdx.x == 0) a.trace[nstamp++] = wall_clock64(); } while (0)
#define DBL_BARRIER() do { if (!grid_barrier(a.bar, a.bar_base, nwg, epoch, a.max_spin, &bar_flag)) return; DBL_STAMP(); } while (0)
  DBL_STAMP();

  for (int l = 0; l < a.n_layers; ++l) {
    GemmArgs<bf16_t> qkv = a.qkv, o = a.o, gu = a.gu, dn = a.dn;
    qkv.W += (size_t)l * a.s_qkv; o.W += (size_t)l * a.s_o; gu.W += (size_t)l * a.s_gu; dn.W += (size_t)l * a.s_dn;
    // ---- fold the previous down-projection partials, RMSNorm -> xn
    gemm_prefetch<bf16_t, EPI_PARTIAL, KSQ>(qkv, wg, nwg, a.nw_qkv, ring);
    if (wg < a.M) {
      NormArgs<bf16_t> n = a.n1;
      n.gain += (size_t)l * n.d;
      n.nparts = l == 0 ? 0 : a.d_parts;
      rmsnorm_row<bf16_t, true>(n, wg, scratch);
    }
    DBL_BARRIER();
    // ---- q/k/v projection -> partials
    gemm_body<bf16_t, EPI_PARTIAL, KSQ, true, true>(qkv, wg, nwg, a.nw_qkv, red, ring, true);
    DBL_BARRIER();
    // ---- (q/k norm,) RoPE, KV append
    {
      RopeArgs<bf16_t> r = a.rope;
      if (r.gq) { r.gq += (size_t)l * r.hd; r.gk += (size_t)l * r.hd; }
      r.kc += (size_t)l * a.s_kv; r.vt += (size_t)l * a.s_kv;
      for (int t = wg * nwaves + wave; t < rope_tasks; t += nwg * nwaves) rope_task<bf16_t, true>(r, t);
    }
    DBL_BARRIER();
    // ---- split-KV attention -> partials
    {
      AttnArgs<bf16_t> at = a.attn;
      at.kc += (size_t)l * a.s_kv; at.vt += (size_t)l * a.s_kv;
      for (int t = wg * nwaves + wave; t < attn_tasks; t += nwg * nwaves) attn_task<bf16_t, HD, true, false>(at, t);
    }
    gemm_prefetch<bf16_t, EPI_RESIDUAL, KSO>(o, wg, nwg, a.nw_o, ring);
    DBL_BARRIER();
    // ---- combine -> attention output
    for (int t = wg * nwaves + wave; t < comb_tasks; t += nwg * nwaves) combine_task<bf16_t, HD, true>(a.comb, t);
    DBL_BARRIER();
    // ---- output projection + residual
    gemm_body<bf16_t, EPI_RESIDUAL, KSO, true, true>(o, wg, nwg, a.nw_o, red, ring, true);
    gemm_prefetch<bf16_t, EPI_SWIGLU, KSG>(gu, wg, nwg, a.nw_gu, ring);
    DBL_BARRIER();
    // ---- RMSNorm -> xn
    if (wg < a.M) {
      NormArgs<bf16_t> n = a.n2;
      n.gain += (size_t)l * n.d;
      rmsnorm_row<bf16_t, true>(n, wg, scratch);
    }
    DBL_BARRIER();
    // ---- gate/up projection + SwiGLU
    gemm_body<bf16_t, EPI_SWIGLU, KSG, true, true>(gu, wg, nwg, a.nw_gu, red, ring, true);
    gemm_prefetch<bf16_t, EPI_PARTIAL, KSD>(dn, wg, nwg, a.nw_dn, ring);
    DBL_BARRIER();
    // ---- down projection -> partials (folded by the next norm)
    gemm_body<bf16_t, EPI_PARTIAL, KSD, true, true>(dn, wg, nwg, a.nw_dn, red, ring, true);
    DBL_BARRIER();
  }
#undef DBL_BARRIER
#undef DBL_STAMP
}
constexpr int LAYER_LOOP_BARRIERS = 9;   // per layer

}  // namespace dbl
