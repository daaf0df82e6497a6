/*
 * dfa.h - C ABI of the DistFlashAttn per-worker hot path for AMD MI355X (gfx950).
 *
 * The library computes what ONE sequence-parallel worker of DistFlashAttn
 * (arXiv 2310.03294) computes: attention of a query chunk against one key/value
 * chunk at a time, the exact merge of two partial results, the backward pass that
 * reuses the saved output and logsumexp, and the load-balanced schedule that says
 * which chunk pairs a worker handles at which time step.
 *
 * General conventions (all entry points)
 *  - Every tensor pointer is a DEVICE pointer unless the comment says "host".
 *    All buffers are owned by the caller; the library allocates nothing and keeps
 *    no pointer after a call returns.
 *  - Calls enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and return without synchronising.
 *  - The return value is the only error channel: DFA_OK (0) or a negative
 *    dfa_status.  Arguments are validated on the host before anything is launched,
 *    so a failing call has launched nothing.
 *  - Tensors are [heads, sequence, d] with the innermost (d) stride equal to 1;
 *    head and sequence strides are given in ELEMENTS in dfa_shape, so a chunk can be
 *    a slice of a full-sequence tensor.  Base pointers of [heads, sequence, d] tensors must be
 *    16-byte aligned and their strides multiples of 8 elements; lse / delta vectors
 *    need only float alignment and a head stride >= s_q.  Head strides are at most 2^40
 *    elements.  One head's slice of a chunk must
 *    span less than 2 GiB counted in fp32 (rows * sequence stride * 4 < 2^31, DFA_ERR_SHAPE
 *    otherwise): the kernels address it with 32-bit byte offsets.
 *  - Outputs must not overlap inputs (dfa_merge's documented in-place operand aside).
 *  - Grouped-query attention: h_q % h_kv == 0 and query head h reads key/value head
 *    h / (h_q / h_kv)  (Section 4 "model setup": each key/value head is shared by a
 *    group of consecutive query heads).
 */
#ifndef DFA_H_
#define DFA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DFA_OK = 0,
  DFA_ERR_NULL = -1,      /* a required pointer is NULL */
  DFA_ERR_SHAPE = -2,     /* sizes / strides / alignment the kernels cannot take */
  DFA_ERR_DTYPE = -3,     /* unknown or unsupported dtype combination */
  DFA_ERR_ARG = -4,       /* inconsistent arguments (e.g. causal with s_q != s_k) */
  /* -5 is not used: no entry point takes a workspace (every buffer is an input or an output) */
  DFA_ERR_HIP = -6        /* the HIP runtime refused a launch */
} dfa_status;

typedef enum { DFA_BF16 = 0, DFA_F32 = 1 } dfa_dtype;

/* One (query chunk, key/value chunk) problem.  Batch is folded into the head axis. */
typedef struct {
  int32_t h_q, h_kv;   /* query heads, key/value heads */
  int32_t s_q, s_k;    /* rows of the query chunk, rows of the key/value chunk (>= 0) */
  int32_t d;           /* head dimension: 64 or 128 */
  int32_t dtype;       /* dfa_dtype of q, k, v, dO */
  int32_t o_dtype;     /* dfa_dtype of o (partial or final output) */
  int32_t causal;      /* 1: diagonal chunk, key j visible to query i iff j <= i, needs
                          s_q == s_k;  0: every key visible (an earlier chunk) */
  float scale;         /* multiplies q.k before the softmax (Eq. 1: 1/sqrt(d)) */
  int32_t reserved;    /* must be 0 */
  int64_t q_stride_h, q_stride_s;      /* q and dO */
  int64_t kv_stride_h, kv_stride_s;    /* k and v */
  int64_t o_stride_h, o_stride_s;      /* o */
  int64_t lse_stride_h;                /* lse and delta: [h_q, s_q], row stride 1 */
  int64_t dq_stride_h, dq_stride_s;    /* dq (fp32) */
  int64_t dkv_stride_h, dkv_stride_s;  /* dk and dv (fp32) */
} dfa_shape;

/*
 * dfa_chunk_fwd - one attn(q_p, k_r, v_r) call started from the empty state
 * (Algorithms 1-3, Appendix A; Eq. 1 restricted to one key/value chunk).
 * For every query row i:  lse_i = log sum_j exp(scale q_i.k_j)  over the visible keys
 * of THIS chunk, and  o_i = sum_j exp(scale q_i.k_j - lse_i) v_j.
 * The running (o, m, l) state of the printed algorithm is exchanged as the normalised
 * output plus logsumexp L = m + log l, which carries the same information.
 *   q [h_q,s_q,d], k,v [h_kv,s_k,d] : sh->dtype, read only
 *   o [h_q,s_q,d] : sh->o_dtype, written;  lse [h_q,s_q] : fp32, natural log, written
 * s_q == 0 is a no-op; s_k == 0 writes o = 0, lse = -inf (the merge identity) and
 * accepts NULL k, v.
 * bf16 inputs use bf16 MFMA with fp32 accumulation; fp32 inputs use fp32 arithmetic.
 */
int dfa_chunk_fwd(const dfa_shape* sh, const void* q, const void* k, const void* v,
                  void* o, float* lse, void* stream);

/*
 * dfa_chunk_fwd_acc - attn(q_p, k_r, v_r, o, s) as the schedules call it (Algorithms 1-2): the
 * same computation as dfa_chunk_fwd, started from the state the earlier key/value chunks left
 * in (o, lse) instead of the empty state, and written back IN PLACE.  The state is exchanged
 * as the normalised output and its logsumexp, i.e. the running (o, m, l) with m = lse, l = 1;
 * the result equals dfa_chunk_fwd into a fresh buffer followed by dfa_merge (up to rounding),
 * without the partial output's trip through memory.  (o = anything, lse = -inf) is the empty
 * state.  s_k == 0 leaves (o, lse) untouched.  Arguments as dfa_chunk_fwd; o and lse are read
 * and written.
 */
int dfa_chunk_fwd_acc(const dfa_shape* sh, const void* q, const void* k, const void* v,
                      void* o, float* lse, void* stream);

/*
 * dfa_merge - the rescale(o, s, o', s') update of the balanced schedule (Section 3.2,
 * Algorithm 2): exact combination of two partial results for the same query rows,
 *   lse = log(e^lse_a + e^lse_b),  o = e^(lse_a-lse) o_a + e^(lse_b-lse) o_b,
 * written IN PLACE over (o_a, lse_a).  (o = 0, lse = -inf) is the identity and never
 * produces NaN.  Operands are [heads, rows, d] (o) and [heads, rows] (lse); strides in
 * elements, innermost stride 1; o_dtype is the dtype of both o operands.
 */
typedef struct {
  int32_t heads, rows, d, o_dtype;
  int64_t a_stride_h, a_stride_s, lse_a_stride_h;   /* o_a, lse_a (read and written) */
  int64_t b_stride_h, b_stride_s, lse_b_stride_h;   /* o_b, lse_b (read only) */
} dfa_merge_desc;

int dfa_merge(const dfa_merge_desc* md, void* o_a, float* lse_a,
              const void* o_b, const float* lse_b, void* stream);

/*
 * dfa_delta - D_i = sum_c dO_ic * O_ic for every query row, from the FINAL merged
 * output of the query chunk (Section 3.3: the saved attention output serves the
 * backward).  Uses h_q, s_q, d, dtype (of dO), o_dtype (of o) and the q_/o_/lse_
 * strides of `sh`.  delta [h_q,s_q] fp32 written.
 */
int dfa_delta(const dfa_shape* sh, const void* o, const void* dO, float* delta, void* stream);

/*
 * dfa_chunk_bwd - gradient contributions of one (query chunk, key/value chunk) pair
 * without re-running the forward (Section 3.3; Appendix A: of the forward's results the backward
 * uses the saved logsumexp alone).  With P_ij = exp(scale q_i.k_j - lse_i) for
 * visible keys (0 otherwise), dP_ij = dO_i.v_j and dS_ij = P_ij (dP_ij - D_i):
 *   dq_i (+)= scale sum_j dS_ij k_j;  dk_j (+)= scale sum_i dS_ij q_i;  dv_j (+)= sum_i P_ij dO_i
 * where dk, dv also sum over the query heads that share the key/value head.
 *   lse   : the FINAL logsumexp of the query chunk over all its key/value chunks
 *   delta : D from dfa_delta on the FINAL merged output (same for every pair of the chunk)
 *   dq [h_q,s_q,d], dk, dv [h_kv,s_k,d] : fp32.  accumulate == 0 overwrites them,
 *   accumulate != 0 adds this pair's contribution to what they hold.
 *   A NULL output selects what is computed: dq == NULL gives dk, dv only; dk == dv == NULL
 *   gives dq only (so a worker can send one while the other is still being computed); dk
 *   and dv are given together; all three NULL is DFA_ERR_NULL.
 * The bf16 path runs two kernels (dk/dv, then dq) and is deterministic; the fp32 path adds dq
 * with fp32 atomics, so its rounding order (not its value beyond rounding) can differ between runs.
 */
int dfa_chunk_bwd(const dfa_shape* sh, const void* q, const void* k, const void* v,
                  const float* lse, const float* delta, const void* dO,
                  float* dq, float* dk, float* dv, int accumulate, void* stream);

/* Step kinds of the balanced schedule. */
typedef enum { DFA_STEP_IDLE = 0, DFA_STEP_DIAG = 1, DFA_STEP_OWN = 2, DFA_STEP_HELP = 3 } dfa_step_kind;

typedef struct {
  int32_t t;         /* time step, 0 .. floor(P/2) */
  int32_t kind;      /* dfa_step_kind */
  int32_t q_chunk;   /* chunk whose queries are used (-1 when idle) */
  int32_t kv_chunk;  /* chunk whose keys/values are used (-1 when idle) */
  int32_t send_to;   /* HELP: worker that owns q_chunk and receives (o, lse); else -1 */
  int32_t recv_from; /* worker whose partial (o, lse) for my queries arrives this step; else -1 */
} dfa_step;

typedef enum { DFA_SCHED_BALANCED = 0, DFA_SCHED_RING = 1 } dfa_sched_mode;

/*
 * dfa_schedule - step list of worker `worker_id` (0-based) among P workers under the
 * load-balanced schedule (Section 3.2, Algorithm 2): step 0 is the causal diagonal
 * chunk; at step t >= 1 a worker with at least t earlier chunks attends to the chunk t
 * positions earlier (OWN); otherwise it computes, with its own keys/values, the pair at
 * distance P - t for the worker that still has work (HELP), unless 2t == P.
 * Pure host function: `out` is a HOST array of `cap` entries; writes min(n, cap)
 * steps and returns n = 1 + floor(P/2), or a negative dfa_status.
 */
int dfa_schedule(int32_t P, int32_t worker_id, dfa_step* out, int32_t cap);

/* As dfa_schedule with a mode: DFA_SCHED_RING is the vanilla schedule (Algorithm 1),
 * P steps, no helpers. Returns the number of steps. */
int dfa_schedule_mode(int32_t mode, int32_t P, int32_t worker_id, dfa_step* out, int32_t cap);

/* Local sliding window (appendix on sparse patterns): attention restricted to the query's own
 * chunk and the `window_chunks` chunks before it, i.e. the vanilla schedule with the end of its
 * loop moved: step 0 is the diagonal chunk, step t in 1..min(window_chunks, P-1) the OWN pair
 * with the chunk t positions earlier (idle for a worker with fewer earlier chunks); no helpers,
 * the load is near balanced by itself.  window_chunks >= P-1 gives the vanilla schedule.
 * Pure host function, `out` as for dfa_schedule; returns the number of steps
 * 1 + min(window_chunks, P-1), or a negative dfa_status (window_chunks < 0: DFA_ERR_ARG). */
int dfa_schedule_window(int32_t P, int32_t worker_id, int32_t window_chunks, dfa_step* out, int32_t cap);

/* Measurement aid (no part of the method): launches a register-resident stream of bf16
 * 32x32x16 MFMAs on every SIMD of the device (512 workgroups of 256 lanes, 4 * iters MFMAs per
 * wavefront, no memory traffic in the loop) on `stream`.  Timed by the caller, *flop / time is
 * the matrix throughput the device sustains at its clock under load, the on-box ceiling quoted
 * next to the published peak.  `out`: DEVICE buffer of n_out >= 131072 floats, overwritten with
 * values of no meaning; `flop`: HOST pointer receiving the FLOP count of the launch (may be NULL).
 * Errors: DFA_ERR_NULL (out), DFA_ERR_ARG (iters < 1 or n_out too small), DFA_ERR_HIP. */
int dfa_mfma_probe(float* out, int64_t n_out, int32_t iters, double* flop, void* stream);

/* Measurement aid (no part of the method): the same register-resident MFMA stream fed with operand
 * VALUES of the caller's choosing.  Every wavefront loads eight A and eight B operands from
 * `operands` (DEVICE, bf16 values, 16-byte aligned, operand_bytes >= 1 MiB; a power-of-two prefix of
 * it is used) and rotates through them, 8 * iters MFMAs per wavefront.  The device keeps its power
 * limit by lowering the clock, and how much power an MFMA draws depends on how many operand bits
 * toggle: with i.i.d. N(0,1) operands (the workload's values) the sustained rate is what the
 * attention kernels can at best reach, well below what the plain probe's near-constant operands
 * give.  Run it for 100 ms or more (iters ~ 400000) so that the clock has settled.
 * `out`, `flop`, `stream` and errors as for dfa_mfma_probe; DFA_ERR_SHAPE for a misaligned and
 * DFA_ERR_ARG for a too small operand buffer. */
int dfa_mfma_probe_data(const void* operands, int64_t operand_bytes, float* out, int64_t n_out,
                        int32_t iters, double* flop, void* stream);

/* Human-readable name of a dfa_status (static storage, host). */
const char* dfa_status_str(int status);

/* Library version as major*10000 + minor*100 + patch. */
int dfa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DFA_H_ */
