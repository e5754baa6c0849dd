/*
 * dbl_diag.h -- measurement, diagnostics and tuning entry points of libdbl.  None of them is part of a step
 * (include/dbl.h holds those); they exist for the benchmark, the profiles and the tests.  Same conventions as
 * dbl.h: 0 or a negative dbl_status, argument checks before any GPU call, nothing throws.
 */
#ifndef DBL_DIAG_H
#define DBL_DIAG_H

#include "dbl.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Which kernel forms the launch logic may choose.  The defaults are the library's own choice per launch; the other
 * values force or forbid a form so that tests reach it on small models and measurements can compare forms.  Results
 * stay within the same parity bars whatever is set.
 */
typedef struct {
  int32_t split_units;       /* projection kernel's split-unit form: 0 where the cost model says so, 1 wherever a
                                projection can take it, -1 never                                                    */
  int32_t wide_gate_up;      /* 1: gate/up through the kernel that shares activations through LDS where it pays;
                                0: always through the general projection kernel                                     */
  int32_t wide_residual;     /* 1: output / down projection of many-row passes as K slices of that form plus a reduce
                                kernel where it pays; 0: never                                                      */
  int32_t wide_lm_head;      /* 1: LM head of passes of more than 32 rows through that form (one pass for up to 128
                                rows); 0: through the general projection kernel, 64 rows per pass                  */
  int32_t stream_16_rows;    /* 1: the q/k/v projection of 9 .. 16 rows through the streaming kernel (activations in
                                registers for the whole launch, RMSNorm applied while they are loaded); 0: through the
                                general projection kernel after a stored RMSNorm                                    */
  int32_t attn_shared;       /* attention's shared form (one token range per workgroup, K/V staged through LDS):
                                1 where it pays, 0 never, 2 / 3 wherever a kv head has two 16-row query blocks and
                                cached tokens (two / one block per wave), 4 the library's choice of when, one block
                                per wave                                                                            */
  int32_t attn_blocks;       /* register form with two query blocks per wave: 2 where it pays, 1 never, 3 wherever
                                possible                                                                            */
  int32_t attn_p16;          /* shared form: probabilities enter the second product as one fp16 operand (1) or as a
                                bf16 head + tail (0)                                                                */
  int32_t attn_split_tokens; /* cached tokens per attention split; 0 = the library's choice                        */
  int32_t verbose;           /* dbl_set_tuning prints the projection plans to stderr                                */
} dbl_tuning;

int dbl_tuning_default(dbl_tuning* t);                    /* {0, 1, 1, 1, 1, 1, 2, 1, 0, 0} */
/* Takes effect from the next call on; touches no GPU state.  Out-of-range values: DBL_EINVAL. */
int dbl_set_tuning(dbl_ctx* ctx, const dbl_tuning* t);

/* Measurement: launch one projection kernel `iters` times (layer = launch index
 * mod n_layers, so consecutive launches stream different weights, as in a real
 * step) for M <= max_batch*max_window rows on the context's stream between two HIP
 * events, with the launch configuration dbl_verify_block uses for that many rows.  which: 0 = fused q/k/v, 1 = output
 * projection, 2 = fused gate/up + SwiGLU, 3 = down projection, 4 = LM head + row
 * statistics.  *ms_out = mean milliseconds per launch; *bytes_out = logical weight
 * bytes one launch must read.  Activations are whatever the scratch buffers hold;
 * the residual stream and statistics are overwritten.  Synchronises. */
int dbl_bench_projection(dbl_ctx* ctx, int which, int M, int iters, float* ms_out, uint64_t* bytes_out);

/* Which kernel and launch shape a projection of M rows takes (the decision dbl_verify_block makes): out4[0] = 0 the
 * streaming kernel (at most 8 rows; q/k/v up to 16), 1 the row-group kernel, 2 the LDS-shared gate/up kernel, 3 the K-sliced form
 * plus reduce, 4 the LDS-shared LM-head kernel; out4[1] = tile rows per unit (slices for form 3); out4[2] = workgroups; out4[3] = 1 for split units.
 * `which` as in dbl_bench_projection.  Touches no GPU state. */
int dbl_projection_plan(dbl_ctx* ctx, int which, int M, int32_t* out4);

/* Diagnostics: which form the attention of a (B, k) window would take at the sequences' current
 * lengths (the host's upper bounds), as dbl_verify_block decides it: out4[0] = 0 register form with
 * deep prefetch (one workgroup per CU at most), 1 register form, 2 shared form (K/V staged through LDS);
 * out4[1] = 16-row query blocks per wave; out4[2] = waves per workgroup; out4[3] = splits (token ranges
 * over the cache + 1 for the window rows).  Touches no GPU state. */
int dbl_attn_plan(dbl_ctx* ctx, int B, int k, int32_t* out4);

/* Diagnostics: copy one of the context's scratch buffers, as left by the last
 * dbl_verify_block, to the host (synchronises).  which: 0 = residual stream after
 * the last layer [rows][ld] f32; 1 = last layer's attention output [rows][ld] in
 * the model dtype; 2 = last layer's silu(gate)*up [rows][ld] in the model dtype.
 * *ld_out receives the row stride in elements; `bytes` is the capacity of `host`
 * and must cover max_batch*max_window rows.  Buffers 1 and 2 are row-major only
 * after a call with at most 16 rows (B*k <= 16); larger calls keep them in blocks
 * of 16 rows x 32 columns, element (m, c) at
 * ((m/16 * ld/32 + c/32) * 64 + (c%32/8) * 16 + m%16) * 8 + c%8. */
int dbl_debug_buffer(dbl_ctx* ctx, int which, void* host, size_t bytes, int32_t* ld_out);

#ifdef __cplusplus
}
#endif
#endif /* DBL_DIAG_H */
