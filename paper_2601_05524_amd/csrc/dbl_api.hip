// libdbl: context, launch logic and the C ABI declared in include/dbl.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/dbl.h"
#include "../../include/dbl_diag.h"
#include "dbl_kernels.h"

using namespace dbl;

namespace {

constexpr int MAX_ROWS = 128;       // max_batch * max_window
constexpr int MAX_WINDOW = 32;
constexpr int MAX_SPLITS = 64;
constexpr int WIDE_SLICES = 8;   // K slices of gemm_wide_slice_kernel at most

// How one projection is cut: NW waves per workgroup, each owning KS k-blocks of a tile
// per K chunk; K longer than NW*KS blocks is covered by SS workgroup super slices
// (partial results, summed by the consumer) or by NCH sequential chunks inside the
// workgroup (projections that add into the residual stream).
struct GemmPlan {
  int N = 0, K = 0;      // logical sizes (N per half for gate/up)
  int NT = 0;            // output tiles (pairs for gate/up)
  int nacc = 1;          // tile rows per unit (2 for gate/up)
  int KS = 0, NW = 0, SS = 1, NCH = 1, KBp = 0;
  int grid = 0;
  size_t elems() const { return (size_t)NT * nacc * KBp * BLOCK_ELEMS; }
  int ldx() const { return KBp * TILE_K; }
  int ldo() const { return NT * TILE_N; }
};

enum PlanKind { PLAN_SLICED = 0, PLAN_SINGLE = 1, PLAN_CHUNKED = 2 };

// PLAN_SLICED: SS >= 1 super slices (q/k/v).  PLAN_SINGLE: the whole K in one pass of one
// workgroup (gate/up, LM head: their epilogues need complete sums).  PLAN_CHUNKED: NCH >= 1
// chunks per workgroup (output and down projection); the chunked kernel keeps two sets
// of activation registers, so it uses the smaller KS, and at most SSQ_PARTS workgroups
// (one sum-of-squares slot each).
bool make_plan(GemmPlan& p, int N, int K, int nacc, bool is_bf16, PlanKind kind, int n_cu) {
  p.N = N; p.K = K; p.nacc = nacc;
  p.NT = (N + TILE_N - 1) / TILE_N;
  const int KB = (K + TILE_K - 1) / TILE_K;
  const int ks_big = is_bf16 ? 32 : 16, ks_small = is_bf16 ? 16 : 8;
  // candidates (KS, NW, SS | NCH): the least streaming time under a model in which every
  // wave slot of the chip is busy or idle for whole rounds (K padding is streamed too),
  // then fewer slices / chunks, then more waves
  double best_cost = 1e30;
  bool found = false;
  for (int ks : {ks_big, ks_small}) {
    if (ks == ks_big && KB < 2 * ks_big) continue;
    const int nsl = (KB + ks - 1) / ks;
    for (int nw = 8; nw >= 1; --nw) {
      const int parts = (nsl + nw - 1) / nw;     // slices or chunks
      if (kind == PLAN_SINGLE && parts != 1) continue;
      if (kind == PLAN_SLICED && parts > 8) continue;
      if (kind == PLAN_CHUNKED && parts > 1 && ks != ks_small) continue;
      const int ss = kind == PLAN_SLICED ? parts : 1, nch = kind == PLAN_CHUNKED ? parts : 1;
      const int kbp = nw * parts * ks;
      const int per_cu = std::max(1, 8 / nw);
      int g = std::min(p.NT * ss, n_cu * per_cu);
      if (kind == PLAN_CHUNKED) g = std::min(g, SSQ_PARTS);
      g = std::max(ss, g / ss * ss);
      const long units = (long)p.NT * ss;
      const long rounds = (units + g - 1) / g;
      const double streamed = (double)rounds * g * nw * ks * nch / (double)(n_cu * 8);
      const double cost = streamed * (1.0 + 0.02 * (parts - 1)) + 1e-3 * (8 - nw);
      if (cost < best_cost) {
        best_cost = cost; p.KS = ks; p.NW = nw; p.SS = ss; p.NCH = nch; p.KBp = kbp; p.grid = g; found = true;
      }
    }
  }
  return found;
}

}  // namespace

// Scratch of dbl_retrieve_tiered_static: one packed best key per sequence, in device memory that belongs to the
// loaded library itself (every GPU the library runs on holds its own copy until the process ends), so that the
// call needs no allocation of anyone's.  In host code the array's name is only a stand-in: the address a kernel
// can use comes from hipGetSymbolAddress, once per device, and is kept in g_static_scratch[device].
constexpr int STATIC_MAX_BATCH = DBL_STATIC_MAX_BATCH;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned long long dbl_static_scratch[STATIC_MAX_BATCH];
static unsigned long long* g_static_scratch[STATIC_MAX_DEVICES] = {};

// Device address of this device's copy of the scratch array (the device must be current); nullptr + *err on failure.
static unsigned long long* static_scratch_of(int device, hipError_t* err) {
  *err = hipSuccess;
  if (device < 0 || device >= STATIC_MAX_DEVICES) { *err = hipErrorInvalidDevice; return nullptr; }
  if (!g_static_scratch[device]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(dbl_static_scratch));
    if (*err != hipSuccess) return nullptr;
    g_static_scratch[device] = reinterpret_cast<unsigned long long*>(p);
  }
  return g_static_scratch[device];
}

struct dbl_ctx {
  dbl_model_cfg cfg{};
  bool bf16 = true, dry = false;
  int device = 0, n_cu = 256;
  hipStream_t stream = nullptr;
  uint64_t seed = 0;
  std::string err;
  size_t esz = 2;

  GemmPlan p_qkv, p_o, p_gu, p_d, p_lm;
  int n_qkv = 0, hq = 0, hkv = 0;   // (H + 2 Hkv) * hd, H*hd, Hkv*hd

  // device memory (all owned)
  void *w_qkv = nullptr, *w_o = nullptr, *w_gu = nullptr, *w_d = nullptr, *w_lm = nullptr, *emb = nullptr;
  float *g1 = nullptr, *g2 = nullptr, *gq = nullptr, *gk = nullptr, *gf = nullptr;
  float *cosT = nullptr, *sinT = nullptr;
  void *kc = nullptr, *vt = nullptr;
  size_t kv_layer_elems = 0;
  int32_t *kv_len = nullptr, *hist_len = nullptr, *hist = nullptr, *status = nullptr;
  int32_t *prompt_len = nullptr;     // [B] history length at the last dbl_history_set (start of the generated text)
  int32_t *rej = nullptr, *rej_len = nullptr;   // rejected tier [B][max_hist], lengths [B]
  unsigned long long* tier_best = nullptr;   // [B] packed best key of a tiered retrieval, zero between calls
  int32_t *prior = nullptr;          // prior tier (allocated by dbl_prior_set)
  int prior_len = 0;
  uint64_t* commits = nullptr;
  float *h = nullptr, *hg = nullptr, *ssq = nullptr;
  void* xn = nullptr;               // RMSNorm output of the current 16-row pass (windows of more than 8 rows)
  float* wide_part = nullptr;       // gemm_wide_slice_kernel's parts: [WIDE_SLICES][rows of a pass][d_model] (contexts of more than 64 rows)
  float* sk_part = nullptr;         // gemm_rows_kernel's split units: two slots of partial sums per workgroup
  int* sk_cnt = nullptr;            //   arrivals per unit (zero between launches)
  // which kernel forms the launch logic may choose (dbl_set_tuning; the defaults are the library's own choice)
  int attn_lds = 1;                 // attention's shared (LDS-staged) form: 1 where it pays, 0 never, 2 wherever a kv head has two query blocks and a cached split exists, 3 / 4 like 2 / 1 with one query block per wave
  int attn_p16 = 1;                 // shared form: probabilities as one fp16 operand (0: bf16 head + tail)
  int attn_nb = 2;                  // query blocks per wave of the attention where it pays; 1 never, 3 wherever possible
  int attn_split_tokens = 0;        // cached tokens per attention split (0: the library's choice)
  int wide_resid = 1;               // output / down projection of many-row passes through gemm_wide_slice_kernel (0: never)
  int stream16 = 1;                 // q/k/v projection of 9 .. 16 rows through gemm_stream_kernel's 16-row form (0: gemm_rows_kernel after xn_kernel)
  int wide_lm = 1;                  // LM head of passes of more than 32 rows through gemm_wide_lmhead_kernel (0: gemm_rows_kernel, 64 rows per pass)
  int wide_gu = 1;                  // gate/up through gemm_wide_swiglu_kernel where wide_gate_up says so (0: always through gemm_rows_kernel)
  int sk_mode = 0;                  // 0: split units where the model says they pay; 1: wherever possible; -1: never
  float *qkv_part = nullptr, *logits = nullptr;
  void *qbuf = nullptr, *attn = nullptr, *act = nullptr;
  int lm_nstat = 0;                 // workgroups of the last LM-head launch (row-statistics entries per row)
  // paged KV cache (DBL_FLAG_PAGED_KV): pool of pages shared by the sequences, table kept by the host
  bool paged = false;
  int pool_pages = 0, pps = 0;      // pages in the pool; table entries per sequence (max_ctx / KV_PAGE)
  int32_t* page_table = nullptr;    // device [max_batch][pps]
  std::vector<int32_t> free_pages;  // host free list (stack)
  std::vector<std::vector<int32_t>> seq_pages;   // pages each sequence holds, in position order
  int ldh = 0;                      // row stride of h and layer stride of g1 / g2 / gf (>= every consumer's K padding)
  float *pm = nullptr, *pl = nullptr, *po = nullptr;
  LmStat* stats = nullptr;
  int32_t *n_acc_i = nullptr, *emit_i = nullptr, *win_i = nullptr;
  int qrows_pad = 0;

  // host-side state
  std::vector<int> kv_upper, hist_upper;
  bool have_verify = false, have_accept = false, verify_sampling = false;
  int last_B = 0, last_k = 0;
  float last_T = 0.f;
  uint64_t last_seed = 0, last_step = 0;
};

namespace {

int fail(dbl_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}

#define HIPCHK(c, expr)                                                                   \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return fail((c), DBL_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_));      \
  } while (0)

template <typename P>
int dmalloc(dbl_ctx* c, P** p, size_t bytes, bool zero) {
  void* v = nullptr;
  hipError_t e = hipMalloc(&v, bytes ? bytes : 256);
  if (e != hipSuccess) return fail(c, DBL_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  if (zero) {
    e = hipMemsetAsync(v, 0, bytes ? bytes : 256, c->stream);
    if (e != hipSuccess) { (void)hipFree(v); return fail(c, DBL_EHIP, std::string("hipMemsetAsync: ") + hipGetErrorString(e)); }
  }
  *p = reinterpret_cast<P*>(v);
  return DBL_OK;
}

int validate_cfg(const dbl_model_cfg* g, std::string& why) {
  auto bad = [&](const char* m) { why = m; return DBL_EINVAL; };
  if (g->n_layers < 0 || g->n_layers > 1024) return bad("n_layers out of range");
  if (g->d_model < 16 || g->d_model % 16) return bad("d_model must be a positive multiple of 16");
  if (g->head_dim != 64 && g->head_dim != 128) return bad("head_dim must be 64 or 128");
  if (g->n_kv_heads < 1 || g->n_q_heads < 1 || g->n_q_heads % g->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
  if (g->d_ffn < 16) return bad("d_ffn too small");
  if (g->vocab < 2) return bad("vocab too small");
  if (g->dtype != DBL_F32 && g->dtype != DBL_BF16) return bad("dtype must be DBL_F32 or DBL_BF16");
  if (!(g->rms_eps > 0.f) || !(g->rope_base > 1.f)) return bad("rms_eps / rope_base out of range");
  if (g->qk_norm != 0 && g->qk_norm != 1) return bad("qk_norm must be 0 or 1");
  if (g->max_batch < 1 || g->max_window < 1 || g->max_window > MAX_WINDOW) return bad("max_batch / max_window out of range");
  if ((int64_t)g->max_batch * g->max_window > MAX_ROWS) return bad("max_batch * max_window exceeds 128 rows");
  if (g->max_ctx < 64 || g->max_ctx % 64) return bad("max_ctx must be a positive multiple of 64");
  if (g->max_hist < 1) return bad("max_hist must be positive");
  if ((g->flags & DBL_FLAG_PAGED_KV) && g->max_ctx % KV_PAGE) return bad("a paged KV cache needs max_ctx to be a multiple of 256");
  if (!(g->flags & DBL_FLAG_PAGED_KV) && (g->flags >> 8)) return bad("a pool size without DBL_FLAG_PAGED_KV");
  return DBL_OK;
}

int make_plans(dbl_ctx* c) {
  const dbl_model_cfg& g = c->cfg;
  c->hq = g.n_q_heads * g.head_dim; c->hkv = g.n_kv_heads * g.head_dim; c->n_qkv = c->hq + 2 * c->hkv;
  bool ok = make_plan(c->p_qkv, c->n_qkv, g.d_model, 1, c->bf16, PLAN_SLICED, c->n_cu) &&
            make_plan(c->p_o, g.d_model, c->hq, 1, c->bf16, PLAN_CHUNKED, c->n_cu) &&
            make_plan(c->p_gu, g.d_ffn, g.d_model, 2, c->bf16, PLAN_SINGLE, c->n_cu) &&
            make_plan(c->p_d, g.d_model, g.d_ffn, 1, c->bf16, PLAN_CHUNKED, c->n_cu) &&
            make_plan(c->p_lm, g.vocab, g.d_model, 1, c->bf16, PLAN_SINGLE, c->n_cu);
  if (!ok) return fail(c, DBL_EINVAL, "d_model too large for a single K slice (max 8192 bf16 / 4096 fp32)");
  c->ldh = std::max({c->p_o.ldo(), c->p_d.ldo(), c->p_qkv.ldx(), c->p_gu.ldx(), c->p_lm.ldx()});
  return DBL_OK;
}

// ----------------------------------------------------------------- launchers

template <typename T, int EPI, bool CHUNK>
void launch_gemm_t(dbl_ctx* c, const GemmPlan& p, const GemmArgs<T>& a) {
  const dim3 grid(p.grid), block(p.NW * 64);
  constexpr bool is_bf = sizeof(T) == 2;
  constexpr int KS_BIG = is_bf ? 32 : 16, KS_SMALL = is_bf ? 16 : 8;
  if constexpr (EPI == EPI_PARTIAL && !CHUNK) {
    if (a.mrows > 8) {   // 9 .. 16 rows: one activation register set per k-block
      if (p.KS == KS_BIG) hipLaunchKernelGGL((gemm_stream_kernel<T, EPI, KS_BIG, false, true>), grid, block, 0, c->stream, a);
      else hipLaunchKernelGGL((gemm_stream_kernel<T, EPI, KS_SMALL, false, true>), grid, block, 0, c->stream, a);
      return;
    }
  }
  if (p.KS == KS_BIG && !CHUNK) hipLaunchKernelGGL((gemm_stream_kernel<T, EPI, KS_BIG, false>), grid, block, 0, c->stream, a);
  else hipLaunchKernelGGL((gemm_stream_kernel<T, EPI, KS_SMALL, CHUNK>), grid, block, 0, c->stream, a);
}

// gemm_rows_kernel: passes of 16*R rows, in units of Q tile rows.  Larger units re-read the
// activations less often but leave fewer of them to share out: Q is the one with the least
// modelled time (units per workgroup, counted half as whole rounds and half as the exact ratio,
// times tile rows per unit, with the activation traffic, R/Q of the weight traffic, at a quarter
// of its cost; fitted to measured launches).  Whole units per workgroup are kept where they fill
// the chip to at least 90 %; otherwise the (unit, chunk) items are cut into equal ranges
// (the kernel's SK form: every workgroup streams the same number of bytes, units that straddle
// ranges are finished by their last workgroup; it ignores the plan's super slices and leaves one
// result, see qkv_parts).
struct RowsChoice { int q = 0, grid = 0; bool sk = false; };

RowsChoice rows_choice(const dbl_ctx* c, const GemmPlan& p, int epi, int R) {
  const int nacc = epi == EPI_SWIGLU ? 2 : 1;
  const int kchunk = 4 * rows_ks(c->bf16, R);                          // k-blocks per chunk (the kernel's NWV * KS)
  const int nch_slice = (p.KBp / p.SS + kchunk - 1) / kchunk, nch_all = (p.KBp + kchunk - 1) / kchunk;
  RowsChoice best, best_sk; double best_cost = 1e30, best_cost_sk = 1e30;
  for (int q : {4, 2}) {
    if (q < nacc) continue;
    if (epi == EPI_LMHEAD && R == 4 && q == 4) continue;   // (the row statistics of four groups leave no room for 16 accumulators)
    if (R == 8 && q != 4) continue;                         // (eight row groups: half the k-blocks per chunk, so 4 tile rows fill the ring)
    const int nu = (p.NT + q / nacc - 1) / (q / nacc);
    const int units = nu * p.SS;
    int g = std::min(units, std::min(c->n_cu, SSQ_PARTS));
    g = std::max(p.SS, g / p.SS * p.SS);
    // modelled time in chunks of one workgroup, times the cost of a chunk
    const double per_chunk = q * (1.0 + 0.25 * R / q);
    const double cost = (0.5 * ((units + g - 1) / g) + 0.5 * (double)units / g) * nch_slice * per_chunk;
    if (cost < best_cost) { best_cost = cost; best = RowsChoice{q, g, false}; }
    // split units: equal ranges of items, plus what publishing and adding the parts costs.  Only where
    // whole units leave more than a quarter of the chip without work: 160 of 256 CUs already draw 6.4 TB/s,
    // so the gain is small (32B-shaped output + down projection 74 -> 69 us) and at better fill there is none
    const long items = (long)nu * nch_all;
    const bool poor_fill = (double)units / ((double)((units + g - 1) / g) * std::min(c->n_cu, SSQ_PARTS)) < 0.75;
    // (a residual projection leaves one sum-of-squares slot per unit)
    if (epi != EPI_LMHEAD && c->sk_part && c->sk_mode >= 0 && (poor_fill || c->sk_mode == 1) && items * SSQ_PARTS < (1L << 31) &&
        (epi != EPI_RESIDUAL || nu <= SSQ_PARTS)) {
      const int gs = (int)std::min<long>(items, std::min(c->n_cu, SSQ_PARTS));
      const double cost_sk = ((double)((items + gs - 1) / gs) + 1.5) * per_chunk;
      if (cost_sk < best_cost_sk) { best_cost_sk = cost_sk; best_sk = RowsChoice{q, gs, true}; }
    }
  }
  if (best_sk.q && (c->sk_mode == 1 || best_cost_sk < best_cost)) return best_sk;
  return best;
}

template <typename T, int EPI, int R>
int launch_gemm_rows_q(dbl_ctx* c, const GemmPlan& p, GemmArgs<T> a) {
  const RowsChoice ch = rows_choice(c, p, EPI, R);
  const dim3 grid(ch.grid), block(256);
  a.sk_part = c->sk_part; a.sk_cnt = c->sk_cnt;
  if constexpr (EPI != EPI_LMHEAD) {
    if (ch.sk) {
      if constexpr (R == 8) {
        hipLaunchKernelGGL((gemm_rows_kernel<T, EPI, R, 4, true>), grid, block, 0, c->stream, a);
      } else {
        if (ch.q == 4) hipLaunchKernelGGL((gemm_rows_kernel<T, EPI, R, 4, true>), grid, block, 0, c->stream, a);
        else hipLaunchKernelGGL((gemm_rows_kernel<T, EPI, R, 2, true>), grid, block, 0, c->stream, a);
      }
      return ch.grid;
    }
  }
  if constexpr (R == 8) {
    hipLaunchKernelGGL((gemm_rows_kernel<T, EPI, R, 4, false>), grid, block, 0, c->stream, a);
  } else {
    if (ch.q == 4) hipLaunchKernelGGL((gemm_rows_kernel<T, EPI, R, 4, false>), grid, block, 0, c->stream, a);
    else hipLaunchKernelGGL((gemm_rows_kernel<T, EPI, R, 2, false>), grid, block, 0, c->stream, a);
  }
  return ch.grid;
}

template <typename T, int R>
void launch_gemm_rows(dbl_ctx* c, const GemmPlan& p, int epi, const GemmArgs<T>& a) {
  switch (epi) {
    case EPI_PARTIAL: launch_gemm_rows_q<T, EPI_PARTIAL, R>(c, p, a); break;
    case EPI_RESIDUAL: launch_gemm_rows_q<T, EPI_RESIDUAL, R>(c, p, a); break;
    case EPI_SWIGLU: launch_gemm_rows_q<T, EPI_SWIGLU, R>(c, p, a); break;
    default:
      if constexpr (R <= 4) c->lm_nstat = launch_gemm_rows_q<T, EPI_LMHEAD, R>(c, p, a);
      break;
  }
}

// Whether the gate/up projection of a pass of mrows rows runs in gemm_wide_swiglu_kernel (bf16): its groups of 16
// tile rows must fill at least three quarters of the chip's rounds (224 groups at the 70B width, 200 at the 32B
// width; 64 at the 1B width do not).  Above 16 rows it then always wins (activation bytes); at 16 rows or fewer only
// where gemm_rows_kernel's whole units leave part of a round empty (32B width: 1600 units, 6.25 rounds, 85.8 -> 80.0
// us; at the 70B width, 7 full rounds, gemm_rows_kernel is ahead, 136 against 147 us).
static bool wide_gate_up(const dbl_ctx* c, const GemmPlan& p, int mrows) {
  if (!c->bf16 || !c->wide_gu || p.KBp % 4 != 0) return false;
  const int ng = (2 * p.NT + 15) / 16, rounds = (ng + c->n_cu - 1) / c->n_cu;
  if (4 * ng < 3 * rounds * c->n_cu) return false;
  if (mrows > 16) return true;
  const RowsChoice ch = rows_choice(c, p, EPI_SWIGLU, 1);
  if (ch.sk) return false;
  const int nu = (p.NT + ch.q / 2 - 1) / (ch.q / 2), r = (nu + ch.grid - 1) / ch.grid;
  return 20 * nu < 19 * r * ch.grid;
}

// Output / down projection of a pass of more than 32 rows through gemm_wide_slice_kernel + resid_reduce_kernel (bf16):
// 0 if not, else the number of K slices.  The groups of 16 tile rows times the slices should about fill the chip; at
// 64 rows the parts cost the output projection what the shared activations gain, so gemm_rows_kernel keeps it.
static int wide_resid_slices(const dbl_ctx* c, const GemmPlan& p, int mrows) {
  if (!c->bf16 || !c->wide_resid || !c->wide_part || mrows <= 32 || p.KBp % 4 != 0) return 0;
  if (mrows <= 64 && p.KBp < 512) return 0;   // (64 rows: only the long-K down projection gains, 90.5 -> 86 us)
  if (p.ldo() % 32 != 0 || p.ldo() / 32 > SSQ_PARTS || p.ldo() != c->ldh) return 0;
  const int ng = (p.NT + 15) / 16, nch = p.KBp / 4;
  int ssw = std::min({c->n_cu / ng, nch, WIDE_SLICES});
  while (ssw > 1 && (ssw - 1) * ((nch + ssw - 1) / ssw) >= nch) --ssw;   // no empty slice
  return ssw >= 2 && 4 * ng * ssw >= 3 * c->n_cu ? ssw : 0;
}

// Which kernel runs a projection of M rows.  Windows of more than 8 rows: gemm_rows_kernel.
// At 8 rows or fewer, measured inside a running layer at three widths: the gate/up projection
// and the LM head are faster through gemm_rows_kernel everywhere (70B width: 8 us per layer and
// 45 us per step; 1B width: 4 us per layer), output and down projection where their tile pairs
// fill the chip (70B width 3 + 4 us, 32B width 2 + 10 us; at the 1B width, 64 whole units for 256
// CUs, slower by 3 + 5 us) or where the split-unit form is the choice (1B width, down projection:
// 2.3 us per layer faster inside a running step), the q/k/v projection nowhere (it needs a stored
// RMSNorm output of its own: 70B width 35.3 us with whole units, 32.8 us with split units,
// against 30.4 us).
static bool rows_kernel_for(const dbl_ctx* c, const GemmPlan& p, int epi, int M) {
  // The q/k/v projection of 9 .. 16 rows stays with the streaming kernel (its 16-row form) while the fp32
  // activations every workgroup pulls through L2 before its first product, M * K * 4 bytes, stay below 384 KiB:
  // that start-up grows with them (70B width 32.3 / 33.7 / 35.1 us at 9 / 12 / 16 rows, 32B width 21.7 / 22.5 /
  // 23.1) while gemm_rows_kernel behind a stored RMSNorm costs the same at any row count (33.5 and 26.3 us).
  if (epi == EPI_PARTIAL && M <= 16 && c->stream16 && (long)M * p.K <= 12L * 8192) return false;
  if (M > 8 || epi == EPI_SWIGLU || epi == EPI_LMHEAD) return true;
  if (epi == EPI_RESIDUAL) return p.NT >= c->n_cu || rows_choice(c, p, epi, 1).sk;
  return false;
}

// Row groups of a pass of mrows rows.
static int pass_groups(int mrows) { return mrows > 64 ? 8 : mrows > 32 ? 4 : mrows > 16 ? 2 : 1; }

// Partial results the q/k/v projection of an M-row window leaves for its readers to add: one per
// super slice of its plan, except that gemm_rows_kernel's SK form leaves a single, complete one.
static int qkv_parts(const dbl_ctx* c, int M) {
  if (rows_kernel_for(c, c->p_qkv, EPI_PARTIAL, M) && rows_choice(c, c->p_qkv, EPI_PARTIAL, pass_groups(std::min(M, 128))).sk) return 1;
  return c->p_qkv.SS;
}

// Whether the LM head of an M-row window runs in gemm_wide_lmhead_kernel (bf16): from 33 rows on, where
// gemm_rows_kernel's per-wave activations cost it most and, above 64 rows, a second pass over the matrix
// (70B width, 128 rows: 2 x 465 us against one pass).
static bool wide_lm_head(const dbl_ctx* c, const GemmPlan& p, int M) {
  return c->bf16 && c->wide_lm && p.KBp % 4 == 0 && M > 32;
}

// The RMSNorm output of rows m0 .. m0+mrows-1 as a stored tensor (a row's columns over several workgroups
// while the rows alone would leave most of the chip idle).
template <typename T>
T* launch_xn(dbl_ctx* c, const GemmArgs<T>& a) {
  T* xn = reinterpret_cast<T*>(c->xn);
  const int nsl = std::max(1, std::min((c->ldh + 1023) / 1024, 64 / a.mrows));
  hipLaunchKernelGGL((xn_kernel<T>), dim3(a.mrows * nsl), dim3(256), 0, c->stream, a.HG, c->ssq, xn, c->ldh, a.m0, nsl, a.d, a.eps);
  return xn;
}

// LM head + row statistics of M rows.  Every pass of a call takes the same kernel, the same number of row groups
// and therefore the same grid, so that one count of statistics entries per row (lm_nstat) serves all rows.
template <typename T>
void launch_lm_head(dbl_ctx* c, const GemmPlan& p, GemmArgs<T> a, int M) {
  const bool wide = wide_lm_head(c, p, M);
  const int pass = wide ? 128 : 64, R = pass_groups(std::min(M, pass));
  for (int m0 = 0; m0 < M; m0 += pass) {
    a.m0 = m0; a.mrows = std::min(pass, M - m0);
    a.X = launch_xn<T>(c, a);
    if constexpr (sizeof(T) == 2) {
      if (wide) {
        const dim3 grid(std::min((p.NT + 15) / 16, c->n_cu)), block(256);
        if (R == 8) hipLaunchKernelGGL((gemm_wide_lmhead_kernel<T, 8>), grid, block, 0, c->stream, a);
        else hipLaunchKernelGGL((gemm_wide_lmhead_kernel<T, 4>), grid, block, 0, c->stream, a);
        c->lm_nstat = (int)grid.x;
        continue;
      }
    }
    if (R == 4) launch_gemm_rows<T, 4>(c, p, EPI_LMHEAD, a);
    else if (R == 2) launch_gemm_rows<T, 2>(c, p, EPI_LMHEAD, a);
    else launch_gemm_rows<T, 1>(c, p, EPI_LMHEAD, a);
  }
}

template <typename T>
void launch_gemm(dbl_ctx* c, const GemmPlan& p, int epi, GemmArgs<T> a, int M) {
  a.NT = p.NT; a.N = p.N; a.KBp = p.KBp; a.SS = p.SS; a.NCH = p.NCH; a.Mtot = M;
  a.d = (float)c->cfg.d_model; a.eps = c->cfg.rms_eps; a.ssq_in = c->ssq; a.ssq_out = c->ssq;
  static_assert(SSQ_PARTS == 256, "xn_kernel adds one partial per thread");
  if (epi == EPI_LMHEAD) { launch_lm_head<T>(c, p, a, M); return; }
  const bool rows = rows_kernel_for(c, p, epi, M);
  if (rows) {
    a.act_tiled = rows_kernel_for(c, c->p_d, EPI_RESIDUAL, M) ? 1 : 0;
    // rows per pass: 128 (eight row groups; measured at the 70B width against two 64-row passes:
    // q/k/v 66 / 98 us, output 58 / 68, gate/up 222 / 335, down 167 / 189)
    const int pass = 128;
    for (int m0 = 0; m0 < M; m0 += pass) {
      a.m0 = m0; a.mrows = std::min(pass, M - m0);
      if (epi != EPI_RESIDUAL) a.X = launch_xn<T>(c, a);   // the RMSNorm output is stored first and read like any activation
      if constexpr (sizeof(T) == 2) {
        // gate/up: four units per workgroup on one set of activations staged through LDS, where that is the better form
        if (epi == EPI_RESIDUAL) {
          if (const int ssw = wide_resid_slices(c, p, a.mrows)) {
            if (a.mrows > 64) hipLaunchKernelGGL((gemm_wide_slice_kernel<T, 8>), dim3((p.NT + 15) / 16, ssw), dim3(256), 0, c->stream, a, c->wide_part);
            else hipLaunchKernelGGL((gemm_wide_slice_kernel<T, 4>), dim3((p.NT + 15) / 16, ssw), dim3(256), 0, c->stream, a, c->wide_part);
            hipLaunchKernelGGL(resid_reduce_kernel, dim3(a.ldo / 32), dim3(256), 0, c->stream, c->wide_part, ssw, a.out, a.hg_out,
                               a.gain_out, c->ssq, a.m0, a.mrows, a.ldo);
            continue;
          }
        }
        if (epi == EPI_SWIGLU && wide_gate_up(c, p, a.mrows)) {
          const dim3 grid(std::min((2 * p.NT + 15) / 16, c->n_cu)), block(256);
          if (a.mrows > 64) hipLaunchKernelGGL((gemm_wide_swiglu_kernel<T, 8>), grid, block, 0, c->stream, a);
          else if (a.mrows > 32) hipLaunchKernelGGL((gemm_wide_swiglu_kernel<T, 4>), grid, block, 0, c->stream, a);
          else if (a.mrows > 16) hipLaunchKernelGGL((gemm_wide_swiglu_kernel<T, 2>), grid, block, 0, c->stream, a);
          else hipLaunchKernelGGL((gemm_wide_swiglu_kernel<T, 1>), grid, block, 0, c->stream, a);
          continue;
        }
      }
      if (a.mrows > 64) launch_gemm_rows<T, 8>(c, p, epi, a);
      else if (a.mrows > 32) launch_gemm_rows<T, 4>(c, p, epi, a);
      else if (a.mrows > 16) launch_gemm_rows<T, 2>(c, p, epi, a);
      else launch_gemm_rows<T, 1>(c, p, epi, a);
    }
    return;
  }
  // at most 8 rows, q/k/v or a narrow output / down projection
  a.m0 = 0; a.mrows = M;
  if (epi == EPI_PARTIAL) launch_gemm_t<T, EPI_PARTIAL, false>(c, p, a);
  else if (p.NCH > 1) launch_gemm_t<T, EPI_RESIDUAL, true>(c, p, a);
  else launch_gemm_t<T, EPI_RESIDUAL, false>(c, p, a);
}

// Arguments of every per-layer step, for layer `l`, window (B, k).
template <typename T>
struct LayerSteps {
  GemmArgs<T> qkv, o, gu, dn;
  AttnArgs<T> attn;
  CombineArgs<T> comb;
  int wpg, nqg;     // attention: waves per workgroup, workgroups per (b, kv head, split)
  int nb;           //   query blocks per wave
  bool deep;        //   latency form
  bool shared;      //   shared form: the workgroup's waves walk one token range together, K/V staged through LDS
};

template <typename T>
LayerSteps<T> layer_steps(dbl_ctx* c, int l, int B, int k) {
  const dbl_model_cfg& g = c->cfg;
  const int M = B * k, d = g.d_model, hd = g.head_dim, H = g.n_q_heads, Hkv = g.n_kv_heads;
  T* attn = reinterpret_cast<T*>(c->attn);
  T* act = reinterpret_cast<T*>(c->act);
  T* kc = reinterpret_cast<T*>(c->kc) + (size_t)l * c->kv_layer_elems;
  T* vt = reinterpret_cast<T*>(c->vt) + (size_t)l * c->kv_layer_elems;
  LayerSteps<T> s{};
  // q/k/v: RMSNorm (gain g1) on load -> per-slice partials
  s.qkv.W = reinterpret_cast<const T*>(c->w_qkv) + (size_t)l * c->p_qkv.elems();
  s.qkv.HG = c->hg; s.qkv.ldx = c->ldh;
  s.qkv.out = c->qkv_part; s.qkv.ldo = c->p_qkv.ldo();
  QkvSrc src{};
  src.qkv = c->qkv_part; src.nparts = qkv_parts(c, M); src.Mtot = M; src.ldq = c->p_qkv.ldo();
  src.gq = g.qk_norm ? c->gq + (size_t)l * hd : nullptr;
  src.gk = g.qk_norm ? c->gk + (size_t)l * hd : nullptr;
  src.cosT = c->cosT; src.sinT = c->sinT; src.H = H; src.Hkv = Hkv; src.eps = g.rms_eps;
  // attention geometry for this window size
  const int gq = H / Hkv, nq = gq * k, qblocks = (nq + 15) / 16;
  // splits: ncs over the cached tokens (none when every cache is empty) + 1 for the window rows
  int ctx_upper = 0;
  for (int b = 0; b < B; ++b) ctx_upper = std::max(ctx_upper, c->kv_upper[b]);
  int ncs = 0;
  // nb query blocks per wave, workgroups for `slots` workgroups per CU
  auto geometry = [&](int nb, int slots) {
    const int nqw = (qblocks + nb - 1) / nb;
    s.nb = nb;
    s.wpg = std::min(nqw, 4);                // waves per workgroup
    s.nqg = (nqw + s.wpg - 1) / s.wpg;
    ncs = (slots * c->n_cu + B * Hkv * s.nqg - 1) / (B * Hkv * s.nqg);
    // at least 128 tokens per split: the partials (m, l, O) are written and read back, so
    // finer splits cost more in traffic than they gain in parallelism
    ncs = std::min({ncs, MAX_SPLITS - 1, (ctx_upper + 127) / 128});
    if (c->attn_split_tokens > 0) {   // tuning aid
      const int tok = std::max(32, c->attn_split_tokens);
      ncs = std::min(MAX_SPLITS - 1, (ctx_upper + tok - 1) / tok);
    }
  };
  geometry(1, 2);
  // bf16: four steps of K/V in flight per wave and queries built in place when every workgroup
  // gets a CU of its own (latency form); else queries prepared once by a kernel of their own and
  // either two steps in flight and two workgroups per CU (throughput form) or, from 4 query blocks
  // per kv head on, two query blocks per wave on one set of K/V fragments and one wave per SIMD
  s.deep = c->bf16 && B * Hkv * (ncs + 1) * s.nqg <= c->n_cu;
  if (c->bf16 && ((!s.deep && qblocks >= 4 && c->attn_nb > 1) || (c->attn_nb > 2 && qblocks >= 2))) {
    const bool was_deep = s.deep;
    // (one wave per SIMD: workgroups of fewer than four waves share a CU)
    geometry(2, 4 / std::min((qblocks + 1) / 2, 4));
    s.deep = false;
    // (ranges of less than 1024 tokens: two workgroups per CU hide the loads of a range's start better; 32B-shaped
    // step at 8192 tokens and 8 query blocks 14.4 against 14.8 ms)
    if (c->attn_nb < 3 && ncs > 0 && ctx_upper / ncs < 1024) { geometry(1, 2); s.deep = was_deep; }
  }
  // shared form (bf16): 2 or more query blocks per kv head, more workgroups than CUs in the forms above, ranges of
  // at least 384 cached tokens per split (shorter ones are mostly start-up: fewer, longer ranges then, as long as
  // half of the CUs still get a workgroup).  2 / 4 / 8 waves per workgroup, 8 waves per CU; two blocks per wave from 8
  // blocks per kv head on, if that still leaves a workgroup for every slot of the chip (else more waves are worth
  // more than fewer K/V reads: 32B-shaped step, 8 (b, kv head) pairs over 8192 tokens, 14.1 against 14.35 ms).
  s.shared = false;
  const bool lds_forced = c->attn_lds == 2 || c->attn_lds == 3;
  if (c->bf16 && c->attn_lds > 0 && qblocks >= 2 && (lds_forced || !s.deep) && ctx_upper > 0) {
    int nb = c->attn_lds >= 3 ? 1 : c->attn_lds == 2 ? 2 : (qblocks >= 8 ? 2 : 1), nw = 0, nqg = 0, n = 0;
    auto shape = [&]() {
      const int nqw = (qblocks + nb - 1) / nb;
      nw = nqw >= 8 ? 8 : nqw >= 4 ? 4 : 2; nqg = (nqw + nw - 1) / nw;
      n = ((8 / nw) * c->n_cu + B * Hkv * nqg - 1) / (B * Hkv * nqg);
      n = std::min({n, MAX_SPLITS - 1, (ctx_upper + 127) / 128});
      if (!lds_forced) n = std::max(1, std::min(n, ctx_upper / 384));
      if (c->attn_split_tokens > 0) {   // tuning aid
        const int tok = std::max(32, c->attn_split_tokens);
        n = std::min(MAX_SPLITS - 1, (ctx_upper + tok - 1) / tok);
      }
    };
    shape();
    if (c->attn_lds == 1 && nb == 2 && B * Hkv * nqg * n < (8 / nw) * c->n_cu) { nb = 1; shape(); }
    if (n >= 1 && (lds_forced || (ctx_upper / n >= 384 && 2 * B * Hkv * nqg * n >= c->n_cu))) {
      s.shared = true; s.deep = false; s.nb = nb; s.wpg = nw; s.nqg = nqg; ncs = n;
    }
  }
  const int nsplit = ncs + 1;
  AttnArgs<T>& at = s.attn;
  at.page_table = c->page_table; at.pps = c->pps;
  at.src = src; at.qbuf = reinterpret_cast<const T*>(c->qbuf); at.kc = kc; at.vt = vt; at.kv_len = c->kv_len; at.pm = c->pm; at.pl = c->pl; at.po = c->po;
  at.k = k; at.g = gq; at.Hkv = Hkv; at.hd = hd; at.max_ctx = g.max_ctx; at.qrows_pad = c->qrows_pad;
  at.nsplit = nsplit; at.nqb = qblocks; at.scale = (float)(1.4426950408889634 / std::sqrt((double)hd));
  s.comb = CombineArgs<T>{c->pm, c->pl, c->po, attn, c->p_o.ldx(), rows_kernel_for(c, c->p_o, EPI_RESIDUAL, M) ? 1 : 0, M, k, H, Hkv, c->qrows_pad, nsplit,
                          src, c->kv_len, kc, vt, g.max_ctx, c->page_table, c->pps};
  s.o.W = reinterpret_cast<const T*>(c->w_o) + (size_t)l * c->p_o.elems();
  s.o.X = attn; s.o.ldx = c->p_o.ldx(); s.o.out = c->h; s.o.ldo = c->ldh;      // h += attn Wo^T
  s.o.hg_out = c->hg; s.o.gain_out = c->g2 + (size_t)l * c->ldh;
  // gate/up: RMSNorm (gain g2) on load -> silu(gate) * up
  s.gu.W = reinterpret_cast<const T*>(c->w_gu) + (size_t)l * c->p_gu.elems();
  s.gu.HG = c->hg; s.gu.ldx = c->ldh;
  s.gu.act = act; s.gu.ldact = c->p_d.ldx();
  s.dn.W = reinterpret_cast<const T*>(c->w_d) + (size_t)l * c->p_d.elems();
  s.dn.X = act; s.dn.ldx = c->p_d.ldx(); s.dn.out = c->h; s.dn.ldo = c->ldh;   // h += act Wd^T
  s.dn.hg_out = c->hg; s.dn.gain_out = l + 1 < g.n_layers ? c->g1 + (size_t)(l + 1) * c->ldh : c->gf;
  (void)d;
  return s;
}

template <typename T, int HD>
void launch_attn_hd(dbl_ctx* c, const LayerSteps<T>& s, int B, int M, int H) {
  // (shared form: nb workgroups per group for the window split, one query block per wave)
  const int nblocks = B * s.attn.Hkv * (s.attn.nsplit - 1 + (s.shared ? s.nb : 1)) * s.nqg;
  const dim3 grid(nblocks), block(64 * s.wpg);
  if (s.shared) {
    if constexpr (sizeof(T) == 2) {
      RopeQArgs<T> q{s.attn.src, s.attn.kv_len, reinterpret_cast<T*>(c->qbuf), B, s.attn.k, s.attn.g, s.attn.qrows_pad,
                     s.attn.max_ctx};
      const int qwaves = (B * s.attn.Hkv * s.attn.g * s.attn.k + 15) / 16;
      hipLaunchKernelGGL((rope_q_kernel<T, HD>), dim3((qwaves + 3) / 4), dim3(256), 0, c->stream, q);
#define DBL_SHARED(NB_, NW_)                                                                                       \
      if (s.nb == NB_ && s.wpg == NW_) {                                                                           \
        if (c->attn_p16) {                                                                                         \
          if (c->paged) hipLaunchKernelGGL((attn_shared_kernel<T, HD, true, NB_, NW_, true>), grid, block, 0, c->stream, s.attn); \
          else hipLaunchKernelGGL((attn_shared_kernel<T, HD, false, NB_, NW_, true>), grid, block, 0, c->stream, s.attn);  \
        } else {                                                                                                   \
          if (c->paged) hipLaunchKernelGGL((attn_shared_kernel<T, HD, true, NB_, NW_, false>), grid, block, 0, c->stream, s.attn); \
          else hipLaunchKernelGGL((attn_shared_kernel<T, HD, false, NB_, NW_, false>), grid, block, 0, c->stream, s.attn);  \
        }                                                                                                          \
      }
      DBL_SHARED(2, 2) DBL_SHARED(2, 4) DBL_SHARED(2, 8) DBL_SHARED(1, 2) DBL_SHARED(1, 4) DBL_SHARED(1, 8)
#undef DBL_SHARED
    }
  } else if (s.deep) {
    if constexpr (sizeof(T) == 2) {
      if (c->paged) hipLaunchKernelGGL((attn_split_kernel<T, HD, 4, true>), grid, block, 0, c->stream, s.attn);
      else hipLaunchKernelGGL((attn_split_kernel<T, HD, 4, false>), grid, block, 0, c->stream, s.attn);
    }
  } else {
    if constexpr (sizeof(T) == 2) {
      RopeQArgs<T> q{s.attn.src, s.attn.kv_len, reinterpret_cast<T*>(c->qbuf), B, s.attn.k, s.attn.g, s.attn.qrows_pad,
                     s.attn.max_ctx};
      const int qwaves = (B * s.attn.Hkv * s.attn.g * s.attn.k + 15) / 16;
      hipLaunchKernelGGL((rope_q_kernel<T, HD>), dim3((qwaves + 3) / 4), dim3(256), 0, c->stream, q);
      if (s.nb == 2) {
        if (c->paged) hipLaunchKernelGGL((attn_split_kernel<T, HD, 2, true, 2>), grid, block, 0, c->stream, s.attn);
        else hipLaunchKernelGGL((attn_split_kernel<T, HD, 2, false, 2>), grid, block, 0, c->stream, s.attn);
      }
    }
    if (s.nb == 1) {
      if (c->paged) hipLaunchKernelGGL((attn_split_kernel<T, HD, 2, true>), grid, block, 0, c->stream, s.attn);
      else hipLaunchKernelGGL((attn_split_kernel<T, HD, 2, false>), grid, block, 0, c->stream, s.attn);
    }
  }
  const int waves = combine_waves<T>(M, H, s.attn.Hkv);   // merge tasks, then KV-append tasks
  hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3((waves + 3) / 4), dim3(256), 0, c->stream, s.comb);
}

template <typename T>
int verify_impl(dbl_ctx* c, const int32_t* window_in, const int32_t* win_len, int B, int k, float temperature, uint64_t seed, uint64_t step,
                bool store_logits) {
  const dbl_model_cfg& g = c->cfg;
  const int M = B * k, d = g.d_model, hd = g.head_dim, H = g.n_q_heads;
  hipStream_t st = c->stream;
  // (the embedding also keeps the window, with rows beyond a sequence's own length marked, for the LM head and for accept)
  const int32_t* window = c->win_i;

  hipLaunchKernelGGL((embed_kernel<T>), dim3(M), dim3(256), 0, st, reinterpret_cast<const T*>(c->emb), window_in, win_len, k, c->win_i, c->h,
                     c->hg, g.n_layers > 0 ? c->g1 : c->gf, c->ssq, d, c->ldh, g.vocab);
  for (int l = 0; l < g.n_layers; ++l) {
    const LayerSteps<T> s = layer_steps<T>(c, l, B, k);
    launch_gemm<T>(c, c->p_qkv, EPI_PARTIAL, s.qkv, M);
    if (hd == 128) launch_attn_hd<T, 128>(c, s, B, M, H); else launch_attn_hd<T, 64>(c, s, B, M, H);
    launch_gemm<T>(c, c->p_o, EPI_RESIDUAL, s.o, M);
    launch_gemm<T>(c, c->p_gu, EPI_SWIGLU, s.gu, M);
    launch_gemm<T>(c, c->p_d, EPI_RESIDUAL, s.dn, M);
  }
  {
    // final RMSNorm (gain gf) on load -> logits + per-workgroup row statistics
    GemmArgs<T> a{};
    a.W = reinterpret_cast<const T*>(c->w_lm); a.HG = c->hg; a.ldx = c->ldh;
    a.out = store_logits ? c->logits : nullptr; a.ldo = c->p_lm.ldo();
    a.lm.stats = c->stats; a.lm.window = window; a.lm.commits = c->commits; a.lm.k = k;
    a.lm.inv_T = temperature > 0.f ? 1.0f / temperature : 0.f;
    a.lm.seed = seed; a.lm.step = step;
    launch_gemm<T>(c, c->p_lm, EPI_LMHEAD, a, M);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, DBL_EHIP, std::string("verify launch: ") + hipGetErrorString(e));
  return DBL_OK;
}

// ------------------------------------------------------------- weight set-up

template <typename T>
int fill_tiled(dbl_ctx* c, void* base, const GemmPlan& p, int layer, std::initializer_list<FillSeg> segs, bool interleave) {
  FillArgs a{};
  int i = 0;
  for (const FillSeg& s : segs) a.seg[i++] = s;
  a.nseg = i; a.interleave = interleave ? 1 : 0;
  a.K = p.K; a.KBp = p.KBp; a.ntile_rows = p.NT * p.nacc; a.layer = layer; a.seed = c->seed;
  T* W = reinterpret_cast<T*>(base) + (size_t)layer * p.elems();
  const size_t threads = (size_t)a.ntile_rows * p.KBp * 64;
  hipLaunchKernelGGL((fill_tiled_kernel<T>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream, W, a);
  return DBL_OK;
}

template <typename T>
int init_weights(dbl_ctx* c) {
  const dbl_model_cfg& g = c->cfg;
  const size_t ne = (size_t)g.vocab * g.d_model;
  hipLaunchKernelGGL((fill_rowmajor_kernel<T>), dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, c->stream,
                     reinterpret_cast<T*>(c->emb), ne, (int)DBL_T_EMB, 0, c->seed);
  fill_tiled<T>(c, c->w_lm, c->p_lm, 0, {{DBL_T_LM, g.vocab}}, false);
  for (int l = 0; l < g.n_layers; ++l) {
    fill_tiled<T>(c, c->w_qkv, c->p_qkv, l, {{DBL_T_WQ, c->hq}, {DBL_T_WK, c->hkv}, {DBL_T_WV, c->hkv}}, false);
    fill_tiled<T>(c, c->w_o, c->p_o, l, {{DBL_T_WO, g.d_model}}, false);
    fill_tiled<T>(c, c->w_gu, c->p_gu, l, {{DBL_T_WG, g.d_ffn}, {DBL_T_WU, g.d_ffn}}, true);
    fill_tiled<T>(c, c->w_d, c->p_d, l, {{DBL_T_WD, g.d_model}}, false);
  }
  auto ones = [&](float* p, size_t n) {
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, p, 1.0f, n);
  };
  const size_t L = std::max(1, g.n_layers);
  // g1 / g2 / gf rows are ldh long and stay zero beyond d_model
  for (size_t l = 0; l < L; ++l) { ones(c->g1 + l * c->ldh, g.d_model); ones(c->g2 + l * c->ldh, g.d_model); }
  ones(c->gq, L * g.head_dim); ones(c->gk, L * g.head_dim); ones(c->gf, g.d_model);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, DBL_EHIP, std::string("weight init: ") + hipGetErrorString(e));
  return DBL_OK;
}

// where a logical tensor lives: container, plan, row offset / interleave slot
struct TensorLoc {
  void* base = nullptr; const GemmPlan* plan = nullptr;
  int rows = 0, cols = 0, row0 = 0, inter = -1;   // inter: 0 gate, 1 up, -1 none
  bool tiled = false, is_gain = false;
  size_t layer_elems = 0;
};

int locate(dbl_ctx* c, int id, int layer, TensorLoc& t) {
  const dbl_model_cfg& g = c->cfg;
  const bool per_layer = id >= DBL_T_G1;
  if (per_layer && (layer < 0 || layer >= g.n_layers)) return DBL_EINVAL;
  switch (id) {
    case DBL_T_EMB: t.base = c->emb; t.rows = g.vocab; t.cols = g.d_model; break;
    case DBL_T_LM: t.base = c->w_lm; t.plan = &c->p_lm; t.rows = g.vocab; t.cols = g.d_model; t.tiled = true; break;
    case DBL_T_GF: t.base = c->gf; t.rows = 1; t.cols = g.d_model; t.is_gain = true; break;
    case DBL_T_G1: t.base = c->g1 + (size_t)layer * c->ldh; t.rows = 1; t.cols = g.d_model; t.is_gain = true; break;
    case DBL_T_G2: t.base = c->g2 + (size_t)layer * c->ldh; t.rows = 1; t.cols = g.d_model; t.is_gain = true; break;
    case DBL_T_GQ: t.base = c->gq + (size_t)layer * g.head_dim; t.rows = 1; t.cols = g.head_dim; t.is_gain = true; break;
    case DBL_T_GK: t.base = c->gk + (size_t)layer * g.head_dim; t.rows = 1; t.cols = g.head_dim; t.is_gain = true; break;
    case DBL_T_WQ: t.base = c->w_qkv; t.plan = &c->p_qkv; t.rows = c->hq; t.cols = g.d_model; t.row0 = 0; t.tiled = true; break;
    case DBL_T_WK: t.base = c->w_qkv; t.plan = &c->p_qkv; t.rows = c->hkv; t.cols = g.d_model; t.row0 = c->hq; t.tiled = true; break;
    case DBL_T_WV: t.base = c->w_qkv; t.plan = &c->p_qkv; t.rows = c->hkv; t.cols = g.d_model; t.row0 = c->hq + c->hkv; t.tiled = true; break;
    case DBL_T_WO: t.base = c->w_o; t.plan = &c->p_o; t.rows = g.d_model; t.cols = c->hq; t.tiled = true; break;
    case DBL_T_WG: t.base = c->w_gu; t.plan = &c->p_gu; t.rows = g.d_ffn; t.cols = g.d_model; t.inter = 0; t.tiled = true; break;
    case DBL_T_WU: t.base = c->w_gu; t.plan = &c->p_gu; t.rows = g.d_ffn; t.cols = g.d_model; t.inter = 1; t.tiled = true; break;
    case DBL_T_WD: t.base = c->w_d; t.plan = &c->p_d; t.rows = g.d_model; t.cols = g.d_ffn; t.tiled = true; break;
    default: return DBL_EINVAL;
  }
  if (t.tiled) t.layer_elems = t.plan->elems();
  return DBL_OK;
}

// physical tile row of logical row r of a located tensor
inline int phys_row(const TensorLoc& t, int r) {
  if (t.inter >= 0) return ((r >> 4) * 2 + t.inter) * 16 + (r & 15);
  return t.row0 + r;
}

template <typename T>
int copy_tensor(dbl_ctx* c, const TensorLoc& t, int layer, void* host, bool to_device) {
  T* hp = reinterpret_cast<T*>(host);
  if (!t.tiled) {  // embedding: plain row-major
    const size_t bytes = (size_t)t.rows * t.cols * sizeof(T);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (to_device) HIPCHK(c, hipMemcpy(t.base, host, bytes, hipMemcpyHostToDevice));
    else HIPCHK(c, hipMemcpy(host, t.base, bytes, hipMemcpyDeviceToHost));
    return DBL_OK;
  }
  const GemmPlan& p = *t.plan;
  T* dev = reinterpret_cast<T*>(t.base) + (size_t)layer * t.layer_elems;
  const size_t n = p.elems();
  std::vector<T> tmp;
  try { tmp.resize(n); } catch (const std::bad_alloc&) { return fail(c, DBL_ENOMEM, "host staging buffer"); }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(tmp.data(), dev, n * sizeof(T), hipMemcpyDeviceToHost));
  for (int r = 0; r < t.rows; ++r) {
    const int pr = phys_row(t, r);
    for (int k = 0; k < t.cols; ++k) {
      const size_t off = tiled_offset<T>(pr, k, p.KBp);
      if (to_device) tmp[off] = hp[(size_t)r * t.cols + k]; else hp[(size_t)r * t.cols + k] = tmp[off];
    }
  }
  if (to_device) HIPCHK(c, hipMemcpy(dev, tmp.data(), n * sizeof(T), hipMemcpyHostToDevice));
  return DBL_OK;
}

// Paged cache: sequence `seq` gets pages for positions [0, n_tokens) (no-op when it has them).
static int ensure_pages(dbl_ctx* c, int seq, int n_tokens) {
  if (!c->paged) return DBL_OK;
  const int need = (n_tokens + KV_PAGE - 1) / KV_PAGE;
  std::vector<int32_t>& mine = c->seq_pages[seq];
  if ((int)mine.size() >= need) return DBL_OK;
  if (need - (int)mine.size() > (int)c->free_pages.size()) return fail(c, DBL_ENOMEM, "KV page pool exhausted");
  while ((int)mine.size() < need) {
    const int32_t page = c->free_pages.back(); c->free_pages.pop_back();
    hipLaunchKernelGGL(set_page_kernel, dim3(1), dim3(64), 0, c->stream, c->page_table, seq * c->pps + (int)mine.size(), page);
    mine.push_back(page);
  }
  return DBL_OK;
}
// ... and gives back the pages beyond position n_tokens (work already enqueued still sees them;
// whoever gets them next is enqueued later)
static void release_pages(dbl_ctx* c, int seq, int n_tokens) {
  if (!c->paged) return;
  const int keep = (n_tokens + KV_PAGE - 1) / KV_PAGE;
  std::vector<int32_t>& mine = c->seq_pages[seq];
  while ((int)mine.size() > keep) { c->free_pages.push_back(mine.back()); mine.pop_back(); }
}

void free_all(dbl_ctx* c) {
  void* ptrs[] = {c->w_qkv, c->w_o, c->w_gu, c->w_d, c->w_lm, c->emb, c->g1, c->g2, c->gq, c->gk, c->gf, c->cosT,
                  c->sinT, c->kc, c->vt, c->page_table, c->kv_len, c->hist_len, c->hist, c->prompt_len, c->rej, c->rej_len, c->tier_best, c->prior, c->status, c->commits, c->h, c->hg, c->xn, c->wide_part, c->sk_part, c->sk_cnt, c->qkv_part,
                  c->ssq, c->logits, c->qbuf, c->attn, c->act, c->pm, c->pl, c->po, c->stats,
                  c->n_acc_i, c->emit_i, c->win_i};
  for (void* p : ptrs) if (p) (void)hipFree(p);
}

int check_status(dbl_ctx* c) {
  int32_t s = 0;
  HIPCHK(c, hipMemcpy(&s, c->status, sizeof(s), hipMemcpyDeviceToHost));
  if (s) HIPCHK(c, hipMemset(c->status, 0, sizeof(s)));   // reported once: later calls start clean
  if (s) return fail(c, DBL_ESTATE, (s & 1) ? "a commit would exceed max_ctx and was clamped" : "a commit would exceed max_hist and was clamped");
  return DBL_OK;
}

}  // namespace

// ===================================================================== C ABI

extern "C" {

int dbl_create(const dbl_model_cfg* cfg, uint64_t weight_seed, void* hip_stream, dbl_ctx** out) {
  if (!cfg || !out) return DBL_EINVAL;
  *out = nullptr;
  std::string why;
  if (validate_cfg(cfg, why) != DBL_OK) return DBL_EINVAL;
  dbl_ctx* c = new (std::nothrow) dbl_ctx();
  if (!c) return DBL_ENOMEM;
  c->cfg = *cfg; c->bf16 = cfg->dtype == DBL_BF16; c->esz = c->bf16 ? 2 : 4;
  c->dry = (cfg->flags & DBL_FLAG_VALIDATE_ONLY) != 0;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->seed = weight_seed;
  c->kv_upper.assign(cfg->max_batch, 0); c->hist_upper.assign(cfg->max_batch, 0);
  int rc = DBL_OK;
  if (!c->dry) {
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { delete c; return DBL_EHIP; }
    int ncu = 0;
    if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && ncu > 0) c->n_cu = ncu;
    // the library's own scratch on this device (dbl_retrieve_tiered_static): resolved here, once per device
    (void)static_scratch_of(c->device, &e);
    if (e != hipSuccess) { std::fprintf(stderr, "dbl_create: hipGetSymbolAddress: %s\n", hipGetErrorString(e)); delete c; return DBL_EHIP; }
  }
  rc = make_plans(c);
  if (rc != DBL_OK) { delete c; return rc; }
  if (c->dry) { *out = c; return DBL_OK; }

  const dbl_model_cfg& g = c->cfg;
  const size_t L = std::max(1, g.n_layers), esz = c->esz;
  const int Mmax = g.max_batch * g.max_window;
  const int gq = g.n_q_heads / g.n_kv_heads;
  c->qrows_pad = ((gq * g.max_window + 63) / 64) * 64;
  c->kv_layer_elems = (size_t)g.max_batch * g.n_kv_heads * g.max_ctx * g.head_dim;
  c->paged = (g.flags & DBL_FLAG_PAGED_KV) != 0;
  if (c->paged) {
    c->pps = g.max_ctx / KV_PAGE;
    c->pool_pages = (g.flags >> 8) ? (g.flags >> 8) : g.max_batch * c->pps;
    c->kv_layer_elems = (size_t)c->pool_pages * g.n_kv_heads * KV_PAGE * g.head_dim;
    c->seq_pages.assign(g.max_batch, {});
    for (int i = c->pool_pages - 1; i >= 0; --i) c->free_pages.push_back(i);   // page 0 is handed out first
  }
  const size_t part_rows = (size_t)g.max_batch * g.n_kv_heads * MAX_SPLITS * c->qrows_pad;

#define ALLOC(ptr, bytes, zero) if ((rc = dmalloc(c, &c->ptr, (bytes), (zero))) != DBL_OK) break
  do {
    ALLOC(w_qkv, L * c->p_qkv.elems() * esz, false);
    ALLOC(w_o, L * c->p_o.elems() * esz, false);
    ALLOC(w_gu, L * c->p_gu.elems() * esz, false);
    ALLOC(w_d, L * c->p_d.elems() * esz, false);
    ALLOC(w_lm, c->p_lm.elems() * esz, false);
    ALLOC(emb, (size_t)g.vocab * g.d_model * esz, false);
    ALLOC(g1, L * c->ldh * 4, true); ALLOC(g2, L * c->ldh * 4, true);
    ALLOC(gq, L * g.head_dim * 4, false); ALLOC(gk, L * g.head_dim * 4, false);
    ALLOC(gf, (size_t)c->ldh * 4, true);
    ALLOC(cosT, (size_t)g.max_ctx * (g.head_dim / 2) * 4, false);
    ALLOC(sinT, (size_t)g.max_ctx * (g.head_dim / 2) * 4, false);
    ALLOC(kc, L * c->kv_layer_elems * esz, true);
    ALLOC(vt, L * c->kv_layer_elems * esz, true);
    if (c->paged) ALLOC(page_table, (size_t)g.max_batch * c->pps * 4, true);
    ALLOC(kv_len, (size_t)g.max_batch * 4, true); ALLOC(hist_len, (size_t)g.max_batch * 4, true);
    ALLOC(hist, (size_t)g.max_batch * g.max_hist * 4, true);
    ALLOC(prompt_len, (size_t)g.max_batch * 4, true);
    ALLOC(rej, (size_t)g.max_batch * g.max_hist * 4, true); ALLOC(rej_len, (size_t)g.max_batch * 4, true);
    ALLOC(tier_best, (size_t)g.max_batch * 8, true);
    ALLOC(status, 4, true); ALLOC(commits, 8, true);
    ALLOC(h, (size_t)Mmax * c->ldh * 4, true);
    ALLOC(hg, (size_t)Mmax * c->ldh * 4, true);
    const size_t M16 = (size_t)(Mmax + 15) / 16 * 16;   // the fragment-tiled activation layout holds whole groups of 16 rows
    ALLOC(xn, M16 * c->ldh * esz, true);
    ALLOC(ssq, (size_t)Mmax * SSQ_PARTS * 4, true);
    {
      // split units of gemm_rows_kernel: two slots per workgroup of (up to 4 tile rows) x (row groups of
      // the largest pass) x 1 KiB, and one arrival counter per unit
      const size_t rg = Mmax > 64 ? 8 : Mmax > 32 ? 4 : Mmax > 16 ? 2 : 1;
      ALLOC(sk_part, (size_t)2 * SSQ_PARTS * 4 * rg * 1024, false);
      ALLOC(sk_cnt, (size_t)std::max({c->p_qkv.NT, c->p_o.NT, c->p_gu.NT, c->p_d.NT}) * 4, true);
    }
    if (c->bf16 && Mmax > 32) ALLOC(wide_part, (size_t)WIDE_SLICES * Mmax * std::max(c->p_o.ldo(), c->p_d.ldo()) * 4, false);
    ALLOC(qkv_part, (size_t)c->p_qkv.SS * Mmax * c->p_qkv.ldo() * 4, true);
    ALLOC(qbuf, (size_t)g.max_batch * g.n_kv_heads * c->qrows_pad * g.head_dim * esz, true);
    ALLOC(logits, (size_t)Mmax * c->p_lm.ldo() * 4, true);
    ALLOC(attn, M16 * c->p_o.ldx() * esz, true);
    ALLOC(act, M16 * c->p_d.ldx() * esz, true);
    ALLOC(pm, part_rows * 4, true); ALLOC(pl, part_rows * 4, true); ALLOC(po, part_rows * g.head_dim * 4, true);
    ALLOC(stats, (size_t)std::max(c->p_lm.grid, c->n_cu) * Mmax * sizeof(LmStat), true);
    ALLOC(n_acc_i, (size_t)g.max_batch * 4, true); ALLOC(emit_i, (size_t)Mmax * 4, true);
    ALLOC(win_i, (size_t)Mmax * 4, true);
  } while (0);
#undef ALLOC
  if (rc == DBL_OK) {
    // rotary tables: angle = pos * base^(-2i/hd) in fp64, rounded to fp32
    const int half = g.head_dim / 2;
    std::vector<float> cs((size_t)g.max_ctx * half), sn((size_t)g.max_ctx * half);
    for (int i = 0; i < half; ++i) {
      const double theta = std::pow((double)g.rope_base, -2.0 * i / g.head_dim);
      for (int p = 0; p < g.max_ctx; ++p) {
        const double ang = (double)p * theta;
        cs[(size_t)p * half + i] = (float)std::cos(ang);
        sn[(size_t)p * half + i] = (float)std::sin(ang);
      }
    }
    hipError_t e = hipMemcpy(c->cosT, cs.data(), cs.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->sinT, sn.data(), sn.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) rc = fail(c, DBL_EHIP, std::string("rope tables: ") + hipGetErrorString(e));
  }
  if (rc == DBL_OK) rc = c->bf16 ? init_weights<bf16_t>(c) : init_weights<float>(c);
  if (rc == DBL_OK) {
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) rc = fail(c, DBL_EHIP, std::string("create sync: ") + hipGetErrorString(e));
  }
  if (rc != DBL_OK) {
    std::fprintf(stderr, "dbl_create: %s\n", c->err.c_str());
    free_all(c); delete c; return rc;
  }
  *out = c;
  return DBL_OK;
}

int dbl_destroy(dbl_ctx* c) {
  if (!c) return DBL_EINVAL;
  if (!c->dry) { (void)hipStreamSynchronize(c->stream); free_all(c); }
  delete c;
  return DBL_OK;
}

const char* dbl_last_error(const dbl_ctx* c) { return c ? c->err.c_str() : "null context"; }

int dbl_model_bytes(const dbl_ctx* c, uint64_t* weight_bytes, uint64_t* kv_bytes_per_token) {
  if (!c) return DBL_EINVAL;
  const dbl_model_cfg& g = c->cfg;
  if (weight_bytes) {
    // logical (algorithmic) bytes: every layer matrix once + LM head once
    const uint64_t per_layer = (uint64_t)c->n_qkv * g.d_model + (uint64_t)g.d_model * c->hq + 3ull * g.d_ffn * g.d_model;
    *weight_bytes = ((uint64_t)g.n_layers * per_layer + (uint64_t)g.vocab * g.d_model) * c->esz;
  }
  if (kv_bytes_per_token) *kv_bytes_per_token = 2ull * g.n_layers * c->hkv * c->esz;
  return DBL_OK;
}

static int weights_io(dbl_ctx* c, int id, int layer, void* host, size_t bytes, bool to_device) {
  if (!c || !host) return fail(c, DBL_EINVAL, "null argument");
  TensorLoc t;
  if (locate(c, id, layer, t) != DBL_OK) return fail(c, DBL_EINVAL, "unknown tensor id or layer");
  const size_t want = (size_t)t.rows * t.cols * (t.is_gain ? 4 : c->esz);
  if (bytes != want) return fail(c, DBL_EINVAL, "tensor size mismatch");
  if (c->dry) return DBL_ENODEV;
  if (t.is_gain) {
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (to_device) HIPCHK(c, hipMemcpy(t.base, host, bytes, hipMemcpyHostToDevice));
    else HIPCHK(c, hipMemcpy(host, t.base, bytes, hipMemcpyDeviceToHost));
    return DBL_OK;
  }
  return c->bf16 ? copy_tensor<bf16_t>(c, t, layer, host, to_device) : copy_tensor<float>(c, t, layer, host, to_device);
}

int dbl_set_weights(dbl_ctx* c, int id, int layer, const void* host, size_t bytes) {
  return weights_io(c, id, layer, const_cast<void*>(host), bytes, true);
}
int dbl_get_weights(dbl_ctx* c, int id, int layer, void* host, size_t bytes) {
  return weights_io(c, id, layer, host, bytes, false);
}

int dbl_reset(dbl_ctx* c, int seq) {
  if (!c) return DBL_EINVAL;
  if (seq >= c->cfg.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  for (int b = 0; b < c->cfg.max_batch; ++b)
    if (seq < 0 || b == seq) { c->kv_upper[b] = 0; c->hist_upper[b] = 0; }
  c->have_verify = c->have_accept = false;
  if (c->dry) return DBL_ENODEV;
  for (int b = 0; b < c->cfg.max_batch; ++b)
    if (seq < 0 || b == seq) release_pages(c, b, 0);
  hipLaunchKernelGGL(set_counters_kernel, dim3(1), dim3(128), 0, c->stream, c->kv_len, c->hist_len, c->prompt_len, c->rej_len, seq,
                     c->cfg.max_batch, c->status);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_kv_fill(dbl_ctx* c, int seq, int32_t n_tokens, uint64_t seed) {
  if (!c) return DBL_EINVAL;
  const dbl_model_cfg& g = c->cfg;
  if (seq < 0 || seq >= g.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (n_tokens < 0 || n_tokens > g.max_ctx - g.max_window) return fail(c, DBL_EINVAL, "n_tokens out of range");
  c->kv_upper[seq] = n_tokens;
  c->have_verify = c->have_accept = false;
  if (c->dry) return DBL_ENODEV;
  const size_t region = (size_t)g.max_ctx * g.head_dim;                       // one (sequence, kv head)
  const size_t n = (size_t)((n_tokens + 31) / 32 * 32) * g.head_dim;          // whole tiles
  {
    const int rc_pages = ensure_pages(c, seq, n_tokens);
    if (rc_pages != DBL_OK) return rc_pages;
  }
  if (n > 0 && g.n_layers > 0) {
    const dim3 grid((unsigned)((n + 255) / 256), (unsigned)(g.n_layers * g.n_kv_heads));
    const size_t seq_off = c->paged ? 0 : (size_t)seq * g.n_kv_heads * region;
    const int32_t* pages = c->paged ? c->page_table + (size_t)seq * c->pps : nullptr;
    const size_t page_elems = (size_t)KV_PAGE * g.head_dim;
    if (c->bf16)
      hipLaunchKernelGGL((fill_kv_kernel<bf16_t>), grid, dim3(256), 0, c->stream, reinterpret_cast<bf16_t*>(c->kc) + seq_off,
                         reinterpret_cast<bf16_t*>(c->vt) + seq_off, region, c->kv_layer_elems, g.n_kv_heads, n, seed, pages, page_elems);
    else
      hipLaunchKernelGGL((fill_kv_kernel<float>), grid, dim3(256), 0, c->stream, reinterpret_cast<float*>(c->kc) + seq_off,
                         reinterpret_cast<float*>(c->vt) + seq_off, region, c->kv_layer_elems, g.n_kv_heads, n, seed, pages, page_elems);
  }
  hipLaunchKernelGGL(set_kv_len_kernel, dim3(1), dim3(64), 0, c->stream, c->kv_len, seq, n_tokens);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

static int kv_rows_io(dbl_ctx* c, int seq, int layer, int32_t pos0, int32_t n, void* host_k, void* host_v, bool to_cache) {
  if (!c) return DBL_EINVAL;
  const dbl_model_cfg& g = c->cfg;
  if (seq < 0 || seq >= g.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (layer < 0 || layer >= g.n_layers) return fail(c, DBL_EINVAL, "layer out of range");
  if (pos0 < 0 || n < 0 || (int64_t)pos0 + n > g.max_ctx) return fail(c, DBL_EINVAL, "rows out of range");
  if (n > 0 && (!host_k || !host_v)) return fail(c, DBL_EINVAL, "null buffer");
  if (c->dry) return DBL_ENODEV;
  if (n == 0) return DBL_OK;
  if (c->paged) {
    if (to_cache) { const int rc = ensure_pages(c, seq, pos0 + n); if (rc != DBL_OK) return rc; }
    else if ((int)c->seq_pages[seq].size() * KV_PAGE < pos0 + n) return fail(c, DBL_EINVAL, "rows beyond the sequence's pages");
  }
  const size_t elems = (size_t)n * g.n_kv_heads * g.head_dim, bytes = elems * c->esz;
  void *sk = nullptr, *sv = nullptr;
  int rc = dmalloc(c, &sk, bytes, false);
  if (rc == DBL_OK) rc = dmalloc(c, &sv, bytes, false);
  auto done = [&](int code) { if (sk) (void)hipFree(sk); if (sv) (void)hipFree(sv); return code; };
  if (rc != DBL_OK) return done(rc);
  hipError_t e = hipSuccess;
  if (to_cache) {
    e = hipMemcpyAsync(sk, host_k, bytes, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(sv, host_v, bytes, hipMemcpyHostToDevice, c->stream);
  }
  if (e == hipSuccess) {
    const size_t region = (size_t)g.max_ctx * g.head_dim;
    const size_t seq_off = c->paged ? 0 : (size_t)seq * g.n_kv_heads * region;
    const int32_t* pages = c->paged ? c->page_table + (size_t)seq * c->pps : nullptr;
    const dim3 grid((unsigned)((elems + 255) / 256));
    const size_t loff = (size_t)layer * c->kv_layer_elems;
    if (c->bf16)
      hipLaunchKernelGGL((kv_rows_kernel<bf16_t>), grid, dim3(256), 0, c->stream, reinterpret_cast<bf16_t*>(c->kc) + loff,
                         reinterpret_cast<bf16_t*>(c->vt) + loff, reinterpret_cast<bf16_t*>(sk), reinterpret_cast<bf16_t*>(sv),
                         seq_off, region, pages, (int)pos0, (int)n, g.n_kv_heads, g.head_dim, to_cache ? 1 : 0);
    else
      hipLaunchKernelGGL((kv_rows_kernel<float>), grid, dim3(256), 0, c->stream, reinterpret_cast<float*>(c->kc) + loff,
                         reinterpret_cast<float*>(c->vt) + loff, reinterpret_cast<float*>(sk), reinterpret_cast<float*>(sv),
                         seq_off, region, pages, (int)pos0, (int)n, g.n_kv_heads, g.head_dim, to_cache ? 1 : 0);
    e = hipGetLastError();
  }
  if (e == hipSuccess && !to_cache) {
    e = hipMemcpyAsync(host_k, sk, bytes, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(host_v, sv, bytes, hipMemcpyDeviceToHost, c->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return done(fail(c, DBL_EHIP, std::string("kv rows: ") + hipGetErrorString(e)));
  return done(DBL_OK);
}

int dbl_kv_set(dbl_ctx* c, int seq, int layer, int32_t pos0, int32_t n, const void* host_k, const void* host_v) {
  return kv_rows_io(c, seq, layer, pos0, n, const_cast<void*>(host_k), const_cast<void*>(host_v), true);
}
int dbl_kv_get(dbl_ctx* c, int seq, int layer, int32_t pos0, int32_t n, void* host_k, void* host_v) {
  return kv_rows_io(c, seq, layer, pos0, n, host_k, host_v, false);
}

int dbl_truncate(dbl_ctx* c, int seq, int32_t kv_len, int32_t hist_len) {
  if (!c) return DBL_EINVAL;
  if (seq < 0 || seq >= c->cfg.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (kv_len >= 0) c->kv_upper[seq] = std::min(c->kv_upper[seq], (int)kv_len);
  if (hist_len >= 0) c->hist_upper[seq] = std::min(c->hist_upper[seq], (int)hist_len);
  c->have_verify = c->have_accept = false;
  if (c->dry) return DBL_ENODEV;
  if (kv_len >= 0) release_pages(c, seq, c->kv_upper[seq]);
  hipLaunchKernelGGL(truncate_kernel, dim3(1), dim3(64), 0, c->stream, c->kv_len, c->hist_len, c->prompt_len, seq, (int)kv_len,
                     (int)hist_len);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_history_set(dbl_ctx* c, int seq, const int32_t* host_tokens, int n) {
  if (!c) return DBL_EINVAL;
  if (seq < 0 || seq >= c->cfg.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (n < 0 || n > c->cfg.max_hist || (n > 0 && !host_tokens)) return fail(c, DBL_EINVAL, "bad history length");
  c->hist_upper[seq] = n;
  if (c->dry) return DBL_ENODEV;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (n > 0) HIPCHK(c, hipMemcpy(c->hist + (size_t)seq * c->cfg.max_hist, host_tokens, (size_t)n * 4, hipMemcpyHostToDevice));
  const int32_t nn = n;
  HIPCHK(c, hipMemcpy(c->hist_len + seq, &nn, 4, hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(c->prompt_len + seq, &nn, 4, hipMemcpyHostToDevice));
  return DBL_OK;
}

int dbl_history_get(dbl_ctx* c, int seq, int32_t* host_out, int cap, int32_t* n_out) {
  if (!c) return DBL_EINVAL;
  if (seq < 0 || seq >= c->cfg.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (cap < 0 || (cap > 0 && !host_out) || !n_out) return fail(c, DBL_EINVAL, "bad output buffer");
  if (c->dry) return DBL_ENODEV;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int32_t n = 0;
  HIPCHK(c, hipMemcpy(&n, c->hist_len + seq, 4, hipMemcpyDeviceToHost));
  n = std::max(0, std::min(n, c->cfg.max_hist));
  *n_out = n;
  const int m = std::min(n, cap);
  if (m > 0) HIPCHK(c, hipMemcpy(host_out, c->hist + (size_t)seq * c->cfg.max_hist, (size_t)m * 4, hipMemcpyDeviceToHost));
  return DBL_OK;
}

int dbl_retrieve(dbl_ctx* c, int B, int n_max, int n_min, int max_cont, int32_t* cont, int32_t* cont_len,
                 int32_t* match_n, int32_t* match_pos) {
  if (!c) return DBL_EINVAL;
  if (!cont || !cont_len || !match_n || !match_pos) return fail(c, DBL_EINVAL, "null output pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (n_min < 1 || n_max < n_min || n_max > 32) return fail(c, DBL_EINVAL, "need 1 <= n_min <= n_max <= 32");
  if (max_cont < 1 || max_cont > 64) return fail(c, DBL_EINVAL, "need 1 <= max_cont <= 64");
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(retrieve_kernel, dim3(B), dim3(1024), 0, c->stream, c->hist, c->hist_len, c->cfg.max_hist, n_max,
                     n_min, max_cont, cont, cont_len, match_n, match_pos);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

// Both forms of the tiered retrieval; use_static: the best keys live in the library's static scratch
// (cleared by a small kernel first: the array is shared by every call on this GPU and keeps the last one's contents).
static int retrieve_tiered_impl(dbl_ctx* c, bool use_static, int B, int n_max, int n_min, int max_cont, int32_t* cont,
                                int32_t* cont_len, int32_t* match_n, int32_t* match_pos, int32_t* match_tier) {
  if (!c) return DBL_EINVAL;
  if (!cont || !cont_len || !match_n || !match_pos || !match_tier) return fail(c, DBL_EINVAL, "null output pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (use_static && B > STATIC_MAX_BATCH) return fail(c, DBL_EINVAL, "B exceeds the static scratch (DBL_STATIC_MAX_BATCH sequences)");
  if (n_min < 1 || n_max < n_min || n_max > 32) return fail(c, DBL_EINVAL, "need 1 <= n_min <= n_max <= 32");
  if (max_cont < 1 || max_cont > 64) return fail(c, DBL_EINVAL, "need 1 <= max_cont <= 64");
  if (c->dry) return DBL_ENODEV;
  unsigned long long* best = c->tier_best;
  if (use_static) {
    hipError_t e = hipSuccess;
    best = static_scratch_of(c->device, &e);      // resolved by dbl_create; the look-up is a table read here
    if (!best) return fail(c, DBL_EHIP, std::string("hipGetSymbolAddress: ") + hipGetErrorString(e));
    hipLaunchKernelGGL(fill_u64_kernel, dim3(1), dim3(STATIC_MAX_BATCH), 0, c->stream, best, 0ull, B);
  }
  TierArgs a{};
  a.prior = c->prior; a.prior_len = c->prior_len;
  a.hist = c->hist; a.hist_len = c->hist_len; a.prompt_len = c->prompt_len; a.max_hist = c->cfg.max_hist;
  a.rej = c->rej; a.rej_len = c->rej_len; a.rej_cap = c->cfg.max_hist;
  a.n_max = n_max; a.n_min = n_min; a.max_cont = max_cont;
  a.cont = cont; a.cont_len = cont_len; a.match_n = match_n; a.match_pos = match_pos; a.match_tier = match_tier;
  a.best = best;
  const int chunks = std::max(1, (c->prior_len + TIER_CHUNK - 1) / TIER_CHUNK);
  hipLaunchKernelGGL(retrieve_tiered_scan_kernel, dim3(chunks, B), dim3(1024), 0, c->stream, a);
  hipLaunchKernelGGL(retrieve_tiered_finish_kernel, dim3(B), dim3(64), 0, c->stream, a);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_retrieve_tiered(dbl_ctx* c, int B, int n_max, int n_min, int max_cont, int32_t* cont, int32_t* cont_len,
                        int32_t* match_n, int32_t* match_pos, int32_t* match_tier) {
  return retrieve_tiered_impl(c, false, B, n_max, n_min, max_cont, cont, cont_len, match_n, match_pos, match_tier);
}

int dbl_retrieve_tiered_static(dbl_ctx* c, int B, int n_max, int n_min, int max_cont, int32_t* cont, int32_t* cont_len,
                               int32_t* match_n, int32_t* match_pos, int32_t* match_tier) {
  return retrieve_tiered_impl(c, true, B, n_max, n_min, max_cont, cont, cont_len, match_n, match_pos, match_tier);
}

int dbl_session_mark(dbl_ctx* c, int seq, int32_t prompt_len) {
  if (!c) return DBL_EINVAL;
  if (seq < 0 || seq >= c->cfg.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (prompt_len < 0) return fail(c, DBL_EINVAL, "prompt_len must not be negative");
  if (c->dry) return DBL_ENODEV;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int32_t hl = 0;
  HIPCHK(c, hipMemcpy(&hl, c->hist_len + seq, 4, hipMemcpyDeviceToHost));
  const int32_t v = std::min(prompt_len, hl);
  HIPCHK(c, hipMemcpy(c->prompt_len + seq, &v, 4, hipMemcpyHostToDevice));
  return DBL_OK;
}

int dbl_prior_set(dbl_ctx* c, const int32_t* host_tokens, int n) {
  if (!c) return DBL_EINVAL;
  if (n < 0 || (n > 0 && !host_tokens)) return fail(c, DBL_EINVAL, "bad prior length");
  for (int i = 0; i < n; ++i)
    if (host_tokens[i] < -1 || host_tokens[i] >= c->cfg.vocab) return fail(c, DBL_EINVAL, "prior token out of range");
  if (c->dry) { c->prior_len = n; return DBL_ENODEV; }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (c->prior) { (void)hipFree(c->prior); c->prior = nullptr; }
  c->prior_len = 0;
  if (n > 0) {
    int rc = dmalloc(c, &c->prior, (size_t)n * 4, false);
    if (rc != DBL_OK) return rc;
    HIPCHK(c, hipMemcpy(c->prior, host_tokens, (size_t)n * 4, hipMemcpyHostToDevice));
    c->prior_len = n;
  }
  return DBL_OK;
}

int dbl_rejected_update(dbl_ctx* c, const int32_t* n_draft) {
  if (!c) return DBL_EINVAL;
  if (!c->have_verify || !c->have_accept) return fail(c, DBL_ESTATE, "dbl_rejected_update needs dbl_verify_block and dbl_accept first");
  if (c->dry) return DBL_ENODEV;
  const int B = c->last_B, k = c->last_k;
  hipLaunchKernelGGL(rejected_update_kernel, dim3(1), dim3(128), 0, c->stream, c->rej, c->rej_len, c->cfg.max_hist, c->hist,
                     c->hist_len, c->cfg.max_hist, c->win_i, c->n_acc_i, n_draft, k, B, (int)DBL_REJ_CTX);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_rejected_get(dbl_ctx* c, int seq, int32_t* host_out, int cap, int32_t* n_out) {
  if (!c) return DBL_EINVAL;
  if (seq < 0 || seq >= c->cfg.max_batch) return fail(c, DBL_EINVAL, "seq out of range");
  if (!n_out || cap < 0 || (cap > 0 && !host_out)) return fail(c, DBL_EINVAL, "bad output buffer");
  if (c->dry) return DBL_ENODEV;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int32_t n = 0;
  HIPCHK(c, hipMemcpy(&n, c->rej_len + seq, 4, hipMemcpyDeviceToHost));
  n = std::min<int32_t>(n, c->cfg.max_hist);
  *n_out = n;
  const int m = std::min<int>(n, cap);
  if (m > 0) HIPCHK(c, hipMemcpy(host_out, c->rej + (size_t)seq * c->cfg.max_hist, (size_t)m * 4, hipMemcpyDeviceToHost));
  return DBL_OK;
}

int dbl_build_window(dbl_ctx* c, int B, int k, int max_cont, const int32_t* cont, const int32_t* cont_len,
                     int32_t pad_id, int32_t* window) {
  if (!c) return DBL_EINVAL;
  if (!cont || !cont_len || !window) return fail(c, DBL_EINVAL, "null pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (k < 1 || k > c->cfg.max_window) return fail(c, DBL_EINVAL, "k out of range");
  if (max_cont < 1 || max_cont > 64) return fail(c, DBL_EINVAL, "need 1 <= max_cont <= 64");
  if (pad_id < 0 || pad_id >= c->cfg.vocab) return fail(c, DBL_EINVAL, "pad_id out of range");
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(build_window_kernel, dim3(B), dim3(64), 0, c->stream, c->hist, c->hist_len, c->cfg.max_hist, cont,
                     cont_len, max_cont, k, pad_id, window);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_build_guided_window(dbl_ctx* c, int B, int k, const int32_t* ahead, const int32_t* n_ahead, int max_ahead, int n_max,
                            int n_min, int d, int32_t pad_id, int32_t* window, int32_t* n_draft) {
  if (!c) return DBL_EINVAL;
  if (!window || !n_draft) return fail(c, DBL_EINVAL, "null output pointer");
  if ((ahead == nullptr) != (n_ahead == nullptr)) return fail(c, DBL_EINVAL, "ahead and n_ahead go together");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (k < 1 || k > c->cfg.max_window) return fail(c, DBL_EINVAL, "k out of range");
  if (max_ahead < 0 || max_ahead > 64 || (ahead && max_ahead < 1)) return fail(c, DBL_EINVAL, "need 1 <= max_ahead <= 64");
  if (n_min < 1 || n_max < n_min || n_max > 32) return fail(c, DBL_EINVAL, "need 1 <= n_min <= n_max <= 32");
  if (d < 1 || d > 64) return fail(c, DBL_EINVAL, "need 1 <= d <= 64");
  if (pad_id < 0 || pad_id >= c->cfg.vocab) return fail(c, DBL_EINVAL, "pad_id out of range");
  if (c->dry) return DBL_ENODEV;
  GuidedArgs a{c->hist, c->hist_len, c->cfg.max_hist, ahead, n_ahead, max_ahead, n_max, n_min, d, k, pad_id, window, n_draft};
  hipLaunchKernelGGL(guided_window_kernel, dim3(B), dim3(1024), 0, c->stream, a);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_merge(dbl_ctx* c, int B, int k, const int32_t* n_u, const int32_t* n_acc, const int32_t* emit, const int32_t* chain,
              const int32_t* n_chain, int max_chain, int max_u, const int32_t* base_len, int32_t* u_out, int32_t* n_u_out,
              int32_t* text_out, int32_t* n_text_out, int32_t* splice_pos, int32_t* record) {
  if (!c) return DBL_EINVAL;
  if (!n_u || !n_acc || !emit || !chain || !n_chain) return fail(c, DBL_EINVAL, "null input pointer");
  if (!u_out || !n_u_out || !text_out || !n_text_out || !splice_pos || !record) return fail(c, DBL_EINVAL, "null output pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (k < 1 || k > MAX_WINDOW) return fail(c, DBL_EINVAL, "k out of range");
  if (max_chain < 1 || max_chain > 4096) return fail(c, DBL_EINVAL, "need 1 <= max_chain <= 4096");
  if (max_u < 1 || max_u > 64) return fail(c, DBL_EINVAL, "need 1 <= max_u <= 64");
  if (c->dry) return DBL_ENODEV;
  MergeArgs a{B, k, max_chain, max_u, n_u, n_acc, emit, chain, n_chain, base_len, u_out, n_u_out, text_out, n_text_out, splice_pos, record};
  hipLaunchKernelGGL(merge_kernel, dim3(1), dim3(128), 0, c->stream, a);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_history_tail(dbl_ctx* c, int B, const int32_t* from, int max_n, int32_t* tokens_out, int32_t* n_out) {
  if (!c) return DBL_EINVAL;
  if (!from || !tokens_out || !n_out) return fail(c, DBL_EINVAL, "null pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (max_n < 1 || max_n > 4096) return fail(c, DBL_EINVAL, "need 1 <= max_n <= 4096");
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(history_tail_kernel, dim3(B), dim3(256), 0, c->stream, c->hist, c->hist_len, c->cfg.max_hist, from, max_n,
                     tokens_out, n_out);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_history_splice(dbl_ctx* c, int B, const int32_t* pos, const int32_t* tokens, const int32_t* n, int max_n, int32_t* missing_out) {
  if (!c) return DBL_EINVAL;
  if (!pos || !tokens || !n) return fail(c, DBL_EINVAL, "null pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (max_n < 1 || max_n > 128) return fail(c, DBL_EINVAL, "need 1 <= max_n <= 128");
  for (int b = 0; b < B; ++b) c->hist_upper[b] = std::min(c->cfg.max_hist, c->hist_upper[b] + max_n);
  c->have_verify = c->have_accept = false;
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(history_splice_kernel, dim3(1), dim3(128), 0, c->stream, c->hist, c->hist_len, c->prompt_len, c->kv_len,
                     c->cfg.max_hist, B, pos, tokens, n, max_n, missing_out, c->status);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_catchup_window(dbl_ctx* c, int B, int k, int32_t pad_id, int32_t* window, int32_t* win_len) {
  if (!c) return DBL_EINVAL;
  if (!window || !win_len) return fail(c, DBL_EINVAL, "null output pointer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (k < 1 || k > c->cfg.max_window) return fail(c, DBL_EINVAL, "k out of range");
  if (pad_id < 0 || pad_id >= c->cfg.vocab) return fail(c, DBL_EINVAL, "pad_id out of range");
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(catchup_window_kernel, dim3(B), dim3(64), 0, c->stream, c->hist, c->hist_len, c->kv_len, c->cfg.max_hist, k,
                     pad_id, window, win_len);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

int dbl_lengths_dev(dbl_ctx* c, int B, int32_t* kv_len_out, int32_t* hist_len_out) {
  if (!c) return DBL_EINVAL;
  if (!kv_len_out && !hist_len_out) return fail(c, DBL_EINVAL, "null output pointers");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(copy_lengths_kernel, dim3(1), dim3(128), 0, c->stream, c->kv_len, c->hist_len, B, kv_len_out, hist_len_out);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

static int verify_common(dbl_ctx* c, const int32_t* window, const int32_t* win_len, int B, int k, float temperature,
                         uint64_t seed, uint64_t step, float* logits_opt) {
  if (!window) return fail(c, DBL_EINVAL, "null window");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, DBL_EINVAL, "B out of range");
  if (k < 1 || k > c->cfg.max_window) return fail(c, DBL_EINVAL, "k out of range");
  if (!(temperature == temperature)) return fail(c, DBL_EINVAL, "temperature is NaN");
  for (int b = 0; b < B; ++b)
    if (c->kv_upper[b] + k > c->cfg.max_ctx) return fail(c, DBL_EINVAL, "kv_len + k would exceed max_ctx");
  c->have_verify = false; c->have_accept = false;
  if (c->dry) { c->have_verify = true; c->last_B = B; c->last_k = k; c->verify_sampling = temperature > 0.f; return DBL_ENODEV; }
  for (int b = 0; b < B; ++b) {
    const int rc_pages = ensure_pages(c, b, c->kv_upper[b] + k);
    if (rc_pages != DBL_OK) return rc_pages;
  }
  // the fp32 logits are written (once, to scratch) only when somebody reads them: the caller through logits_opt,
  // or dbl_accept's residual draw under dense draft distributions, which needs temperature > 0
  const bool store_logits = logits_opt != nullptr || temperature > 0.f;
  int rc = c->bf16 ? verify_impl<bf16_t>(c, window, win_len, B, k, temperature, seed, step, store_logits)
                   : verify_impl<float>(c, window, win_len, B, k, temperature, seed, step, store_logits);
  if (rc != DBL_OK) return rc;
  if (logits_opt) {
    HIPCHK(c, hipMemcpy2DAsync(logits_opt, (size_t)c->cfg.vocab * 4, c->logits, (size_t)c->p_lm.ldo() * 4,
                               (size_t)c->cfg.vocab * 4, (size_t)B * k, hipMemcpyDeviceToDevice, c->stream));
  }
  c->have_verify = true; c->last_B = B; c->last_k = k; c->verify_sampling = temperature > 0.f;
  c->last_T = temperature; c->last_seed = seed; c->last_step = step;
  return DBL_OK;
}

int dbl_verify_block(dbl_ctx* c, const int32_t* window, int B, int k, float temperature, uint64_t seed, uint64_t step,
                     float* logits_opt) {
  if (!c) return DBL_EINVAL;
  return verify_common(c, window, nullptr, B, k, temperature, seed, step, logits_opt);
}

int dbl_verify_block_ragged(dbl_ctx* c, const int32_t* window, const int32_t* win_len, int B, int k, float temperature,
                            uint64_t seed, uint64_t step, float* logits_opt) {
  if (!c) return DBL_EINVAL;
  if (!win_len) return fail(c, DBL_EINVAL, "null win_len");
  return verify_common(c, window, win_len, B, k, temperature, seed, step, logits_opt);
}

int dbl_accept(dbl_ctx* c, int mode, const float* q_probs, int32_t* n_acc, int32_t* emit, int32_t* guide) {
  if (!c) return DBL_EINVAL;
  if (!n_acc || !emit || !guide) return fail(c, DBL_EINVAL, "null output pointer");
  if (mode != DBL_GREEDY && mode != DBL_SAMPLE) return fail(c, DBL_EINVAL, "bad mode");
  if (!c->have_verify) return fail(c, DBL_ESTATE, "dbl_accept needs a preceding dbl_verify_block");
  if (mode == DBL_SAMPLE && !c->verify_sampling) return fail(c, DBL_ESTATE, "sampling needs temperature > 0 in dbl_verify_block");
  if (mode == DBL_GREEDY && q_probs) return fail(c, DBL_EINVAL, "q_probs given in greedy mode");
  if (c->dry) { c->have_accept = true; return DBL_ENODEV; }
  AcceptArgs a{};
  a.stats = c->stats; a.nstat = c->lm_nstat; a.Mtot = c->last_B * c->last_k;
  a.logits = c->logits; a.ldl = c->p_lm.ldo(); a.window = c->win_i; a.q = q_probs; a.commits = c->commits;
  a.n_acc = n_acc; a.emit = emit; a.guide = guide; a.n_acc_i = c->n_acc_i; a.emit_i = c->emit_i;
  a.k = c->last_k; a.V = c->cfg.vocab; a.mode = mode;
  a.inv_T = c->verify_sampling ? 1.0f / c->last_T : 0.f;
  a.seed = c->last_seed; a.step = c->last_step;
  // a wave per window row, up to 16 at a time (the rows' statistics are merged wave by wave, always in the same order)
  const int accept_waves = std::min(16, std::max(4, c->last_k));
  hipLaunchKernelGGL(accept_kernel, dim3(c->last_B), dim3(64 * accept_waves), 0, c->stream, a);
  HIPCHK(c, hipGetLastError());
  c->have_accept = true;
  return DBL_OK;
}

int dbl_kv_commit(dbl_ctx* c, const int32_t* n_keep) {
  if (!c) return DBL_EINVAL;
  if (!c->have_verify) return fail(c, DBL_ESTATE, "dbl_kv_commit needs a preceding dbl_verify_block");
  if (!n_keep && !c->have_accept) return fail(c, DBL_ESTATE, "dbl_kv_commit(NULL) needs a preceding dbl_accept");
  const int B = c->last_B, k = c->last_k;
  const bool append = n_keep == nullptr;
  for (int b = 0; b < B; ++b) {
    c->kv_upper[b] = std::min(c->cfg.max_ctx, c->kv_upper[b] + k);
    if (append) c->hist_upper[b] = std::min(c->cfg.max_hist, c->hist_upper[b] + k);
  }
  c->have_verify = false; c->have_accept = false;
  if (c->dry) return DBL_ENODEV;
  hipLaunchKernelGGL(commit_kernel, dim3(1), dim3(128), 0, c->stream, c->kv_len, c->hist_len, c->hist, c->cfg.max_hist,
                     c->cfg.max_ctx, n_keep, c->n_acc_i, c->emit_i, k, B, append ? 1 : 0, c->commits, c->status);
  HIPCHK(c, hipGetLastError());
  return DBL_OK;
}

static int read_counters(dbl_ctx* c, int32_t* host_out, bool kv) {
  if (!c) return DBL_EINVAL;
  if (!host_out) return fail(c, DBL_EINVAL, "null output pointer");
  if (c->dry) return DBL_ENODEV;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  const int n = c->cfg.max_batch;
  std::vector<int32_t> a(n), b(n);
  HIPCHK(c, hipMemcpy(a.data(), c->kv_len, (size_t)n * 4, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(b.data(), c->hist_len, (size_t)n * 4, hipMemcpyDeviceToHost));
  for (int i = 0; i < n; ++i) { c->kv_upper[i] = a[i]; c->hist_upper[i] = b[i]; }
  // paged cache: pages handed out against the host's (looser) upper bound go back to the pool,
  // except the ones a window that is verified but not committed yet may still need
  for (int i = 0; i < n; ++i) release_pages(c, i, a[i] + c->cfg.max_window);
  std::memcpy(host_out, kv ? a.data() : b.data(), (size_t)n * 4);
  return check_status(c);
}

}  // extern "C"

template <typename T>
static void bench_launch(dbl_ctx* c, int which, int layer, int M) {
  GemmArgs<T> a{};
  const dbl_model_cfg& g = c->cfg;
  const LayerSteps<T> s = layer_steps<T>(c, layer, 1, M);
  switch (which) {
    case 0: launch_gemm<T>(c, c->p_qkv, EPI_PARTIAL, s.qkv, M); break;
    case 1: launch_gemm<T>(c, c->p_o, EPI_RESIDUAL, s.o, M); break;
    case 2: launch_gemm<T>(c, c->p_gu, EPI_SWIGLU, s.gu, M); break;
    case 3: launch_gemm<T>(c, c->p_d, EPI_RESIDUAL, s.dn, M); break;
    default:
      a.W = reinterpret_cast<const T*>(c->w_lm); a.HG = c->hg; a.ldx = c->ldh;
      a.out = c->logits; a.ldo = c->p_lm.ldo();
      a.lm.stats = c->stats; a.lm.window = c->win_i; a.lm.commits = c->commits; a.lm.k = M; a.lm.inv_T = 0.f;
      launch_gemm<T>(c, c->p_lm, EPI_LMHEAD, a, M); break;
  }
  (void)g;
}

extern "C" {

int dbl_bench_projection(dbl_ctx* c, int which, int M, int iters, float* ms_out, uint64_t* bytes_out) {
  if (!c) return DBL_EINVAL;
  if (!ms_out || !bytes_out) return fail(c, DBL_EINVAL, "null output pointer");
  if (which < 0 || which > 4 || iters < 1 || iters > 100000) return fail(c, DBL_EINVAL, "bad which / iters");
  if (M < 1 || M > c->cfg.max_batch * c->cfg.max_window) return fail(c, DBL_EINVAL, "M out of range");
  if (which < 4 && c->cfg.n_layers < 1) return fail(c, DBL_EINVAL, "model has no layers");
  const dbl_model_cfg& g = c->cfg;
  const uint64_t elems[5] = {(uint64_t)c->n_qkv * g.d_model, (uint64_t)g.d_model * c->hq, 2ull * g.d_ffn * g.d_model,
                             (uint64_t)g.d_model * g.d_ffn, (uint64_t)g.vocab * g.d_model};
  *bytes_out = elems[which] * c->esz;
  if (c->dry) return DBL_ENODEV;
  hipEvent_t e0, e1;
  HIPCHK(c, hipEventCreate(&e0));
  HIPCHK(c, hipEventCreate(&e1));
  const int L = std::max(1, g.n_layers);
  for (int pass = 0; pass < 2; ++pass) {   // pass 0 warms up (2 launches), pass 1 is timed
    const int n = pass == 0 ? 2 : iters;
    if (pass == 1) HIPCHK(c, hipEventRecord(e0, c->stream));
    for (int i = 0; i < n; ++i) {
      if (c->bf16) bench_launch<bf16_t>(c, which, i % L, M); else bench_launch<float>(c, which, i % L, M);
    }
    if (pass == 1) HIPCHK(c, hipEventRecord(e1, c->stream));
  }
  HIPCHK(c, hipEventSynchronize(e1));
  HIPCHK(c, hipGetLastError());
  float ms = 0.f;
  HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  *ms_out = ms / (float)iters;
  return DBL_OK;
}

int dbl_debug_buffer(dbl_ctx* c, int which, void* host, size_t bytes, int32_t* ld_out) {
  if (!c) return DBL_EINVAL;
  if (!host || !ld_out || which < 0 || which > 2) return fail(c, DBL_EINVAL, "bad debug buffer request");
  const size_t rows = (size_t)c->cfg.max_batch * c->cfg.max_window;
  const void* src = which == 0 ? (const void*)c->h : which == 1 ? (const void*)c->attn : (const void*)c->act;
  const int ld = which == 0 ? c->ldh : which == 1 ? c->p_o.ldx() : c->p_d.ldx();
  const size_t need = rows * ld * (which == 0 ? 4 : c->esz);
  if (bytes < need) return fail(c, DBL_EINVAL, "debug buffer too small");
  *ld_out = ld;
  if (c->dry) return DBL_ENODEV;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(host, src, need, hipMemcpyDeviceToHost));
  return DBL_OK;
}

int dbl_tuning_default(dbl_tuning* t) {
  if (!t) return DBL_EINVAL;
  *t = dbl_tuning{0, 1, 1, 1, 1, 1, 2, 1, 0, 0};
  return DBL_OK;
}

int dbl_set_tuning(dbl_ctx* c, const dbl_tuning* t) {
  if (!c) return DBL_EINVAL;
  if (!t) return fail(c, DBL_EINVAL, "null tuning");
  if (t->split_units < -1 || t->split_units > 1 || t->attn_shared < 0 || t->attn_shared > 4 || t->attn_blocks < 1 || t->attn_blocks > 3 ||
      t->attn_split_tokens < 0)
    return fail(c, DBL_EINVAL, "tuning value out of range");
  c->sk_mode = t->split_units; c->wide_gu = t->wide_gate_up != 0; c->wide_resid = t->wide_residual != 0; c->wide_lm = t->wide_lm_head != 0; c->stream16 = t->stream_16_rows != 0;
  c->attn_lds = t->attn_shared; c->attn_nb = t->attn_blocks; c->attn_p16 = t->attn_p16 != 0;
  c->attn_split_tokens = t->attn_split_tokens;
  if (t->verbose) {
    const GemmPlan* ps[5] = {&c->p_qkv, &c->p_o, &c->p_gu, &c->p_d, &c->p_lm};
    const char* nm[5] = {"qkv", "o", "gate_up", "down", "lm_head"};
    for (int i = 0; i < 5; ++i)
      std::fprintf(stderr, "[dbl] plan %-8s N=%d K=%d tiles=%d KS=%d NW=%d SS=%d NCH=%d KBp=%d grid=%d\n", nm[i],
                   ps[i]->N, ps[i]->K, ps[i]->NT, ps[i]->KS, ps[i]->NW, ps[i]->SS, ps[i]->NCH, ps[i]->KBp, ps[i]->grid);
  }
  return DBL_OK;
}

int dbl_projection_plan(dbl_ctx* c, int which, int M, int32_t* out4) {
  if (!c) return DBL_EINVAL;
  if (!out4) return fail(c, DBL_EINVAL, "null output pointer");
  if (which < 0 || which > 4) return fail(c, DBL_EINVAL, "bad which");
  if (M < 1 || M > c->cfg.max_batch * c->cfg.max_window) return fail(c, DBL_EINVAL, "M out of range");
  const GemmPlan* ps[5] = {&c->p_qkv, &c->p_o, &c->p_gu, &c->p_d, &c->p_lm};
  const int epis[5] = {EPI_PARTIAL, EPI_RESIDUAL, EPI_SWIGLU, EPI_RESIDUAL, EPI_LMHEAD};
  const GemmPlan& p = *ps[which];
  const int epi = epis[which], mrows = std::min(M, which == 4 && !wide_lm_head(c, p, M) ? 64 : 128), R = pass_groups(mrows);
  int kernel = 0, q = 0, grid = p.grid, sk = 0;
  if (epi == EPI_LMHEAD && wide_lm_head(c, p, M)) { kernel = 4; q = 4; grid = std::min((p.NT + 15) / 16, c->n_cu); }
  else if (rows_kernel_for(c, p, epi, M)) {
    if (c->bf16 && epi == EPI_RESIDUAL && wide_resid_slices(c, p, mrows)) { kernel = 3; q = wide_resid_slices(c, p, mrows); grid = (p.NT + 15) / 16 * q; }
    else if (c->bf16 && epi == EPI_SWIGLU && wide_gate_up(c, p, mrows)) { kernel = 2; q = 4; grid = std::min((2 * p.NT + 15) / 16, c->n_cu); }
    else { const RowsChoice ch = rows_choice(c, p, epi, R); kernel = 1; q = ch.q; grid = ch.grid; sk = ch.sk ? 1 : 0; }
  }
  out4[0] = kernel; out4[1] = q; out4[2] = grid; out4[3] = sk;
  return DBL_OK;
}

int dbl_attn_plan(dbl_ctx* c, int B, int k, int32_t* out4) {
  if (!c) return DBL_EINVAL;
  if (!out4) return fail(c, DBL_EINVAL, "null output pointer");
  if (B < 1 || B > c->cfg.max_batch || k < 1 || k > c->cfg.max_window) return fail(c, DBL_EINVAL, "B / k out of range");
  if (c->cfg.n_layers < 1) return fail(c, DBL_EINVAL, "model has no layers");
  int form, nb, wpg, nsplit;
  if (c->bf16) { const LayerSteps<bf16_t> s = layer_steps<bf16_t>(c, 0, B, k); form = s.shared ? 2 : s.deep ? 0 : 1; nb = s.nb; wpg = s.wpg; nsplit = s.attn.nsplit; }
  else { const LayerSteps<float> s = layer_steps<float>(c, 0, B, k); form = s.shared ? 2 : s.deep ? 0 : 1; nb = s.nb; wpg = s.wpg; nsplit = s.attn.nsplit; }
  out4[0] = form; out4[1] = nb; out4[2] = wpg; out4[3] = nsplit;
  return DBL_OK;
}

int dbl_kv_len(dbl_ctx* c, int32_t* host_out) { return read_counters(c, host_out, true); }
int dbl_hist_len(dbl_ctx* c, int32_t* host_out) { return read_counters(c, host_out, false); }

}  // extern "C"
