/*
 * speckv.h -- C ABI of the MI355X (gfx950) verify-and-select library for SpecKV.
 *
 * One speculation step over a batch of B sequences, all on one GPU, all on the caller's
 * HIP stream, with no host synchronisation inside:
 *
 *   speckv_signals       draft logits  -> per-position draft entropy and confidence and the
 *                                         four step aggregates            (paper Section 4.2)
 *   speckv_verify        target logits -> accepted prefix, the one extra token,
 *                                         tokens per step, acceptance rate (paper Section 3.1,
 *                                         with the lossless accept test min(1, p/q) of the
 *                                         speculative-sampling works cited in Section 2.1)
 *   speckv_select_gamma  signals       -> next speculation length in {2,4,6,8} from the
 *                                         16-unit MLP controller           (Section 4.3, Eq. 1)
 *   speckv_step          all of the above in one call and two launches, same results bit for bit
 *
 * Beside the step: speckv_verify_greedy (the accept rule as Section 3.1 words it, top-1 match) and
 * speckv_sample_draft (the draft side's token proposal that precedes a step).
 *
 * Notation: q = draft distribution, p = target distribution (Section 4.2 of the paper writes
 * the draft distribution as p_i).  Positions are 0-based: sequence b owns gamma_b draft rows
 * i = 0..gamma_b-1 and gamma_b+1 target rows i = 0..gamma_b (the last one is the bonus row).
 *
 * Memory: every pointer marked DEVICE is GPU memory owned by the caller (for example the
 * data_ptr() of a torch tensor); the library never allocates, frees or keeps it beyond the
 * call that received it, except that the workspace carries per-row softmax statistics from
 * speckv_signals to the speckv_verify of the same step.  Pointers marked HOST are ordinary
 * host memory read during the call.  Base pointers of logits must be 16-byte aligned;
 * individual rows need not be.
 *
 * Errors: argument errors are found on the host before anything is launched, return a
 * non-zero speckv_status and leave all outputs untouched.  A failed launch returns
 * SPECKV_ERR_DEVICE.  Data-dependent anomalies never abort a call: they set bits in
 * row_flags[b] (SPECKV_FLAG_*).  speckv_last_error() describes the most recent failure.
 *
 * Layout of a batch.  Logits are dense row-major rows of V elements (row pitch = V).
 *   uniform batch (gamma == NULL): draft rows  b*g + i,       target rows b*(g+1) + i
 *   ragged batch  (gamma != NULL): draft rows  row_off[b] + i, target rows row_off[b] + b + i
 * with row_off[b] = gamma[0] + ... + gamma[b-1] (speckv_row_offsets computes it on the GPU).
 */
#ifndef SPECKV_H
#define SPECKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPECKV_OK = 0,
    SPECKV_ERR_NULL = 1,      /* a required pointer is NULL */
    SPECKV_ERR_SHAPE = 2,     /* B, V, n_hidden ... out of range */
    SPECKV_ERR_DTYPE = 3,     /* unknown speckv_dtype / speckv_features / speckv_mlp_form value */
    SPECKV_ERR_ALIGN = 4,     /* a base pointer is not aligned as required */
    SPECKV_ERR_WORKSPACE = 5, /* workspace smaller than speckv_workspace_bytes() */
    SPECKV_ERR_GAMMA = 6,     /* gamma_uniform / gamma_max outside [1, SPECKV_GAMMA_LIMIT] */
    SPECKV_ERR_STATE = 7,     /* speckv_verify without the matching speckv_signals */
    SPECKV_ERR_DEVICE = 8     /* HIP reported an error, or the handle has no device */
} speckv_status;

typedef enum { SPECKV_F32 = 0, SPECKV_F16 = 1, SPECKV_BF16 = 2 } speckv_dtype;

/* Which signals feed the controller.
 * POS0: x = [H_0, c_0, onehot3(comp)]                      n_in = 5 (benchmark configurations)
 * AGG4: x = [mean H, mean c, max H, min c, onehot3(comp)]  n_in = 7 (context vector, Section 4.3) */
typedef enum { SPECKV_FEAT_POS0 = 0, SPECKV_FEAT_AGG4 = 1 } speckv_features;

#define SPECKV_GAMMA_LIMIT 16     /* largest supported gamma_max */
#define SPECKV_HIDDEN_LIMIT 64    /* largest supported n_hidden */
#define SPECKV_N_CANDIDATES 4     /* candidate speculation lengths 2, 4, 6, 8 (Section 4.1) */

#define SPECKV_FLAG_NONFINITE 1u  /* a row of the sequence holds NaN or +inf, or no finite logit */
#define SPECKV_FLAG_BAD_TOKEN 2u  /* a drafted token id of the sequence is outside [0, V) */
#define SPECKV_FLAG_FALLBACK 4u   /* residual mass below 1e-6 (p_n and q_n agree to that distance) or not
                                     finite: token drawn from p_n instead */
#define SPECKV_FLAG_BAD_GAMMA 8u  /* gamma[b] outside [1, gamma_max]: the sequence was processed with the
                                     value clamped into that range (its rows are still taken from row_off) */

typedef struct speckv_handle speckv_handle;
typedef void *speckv_stream; /* a hipStream_t; NULL is the default stream */

/* Shape of one step's batch (HOST struct; the two pointers inside are DEVICE pointers). */
typedef struct {
    int32_t B;              /* sequences, >= 1 */
    int32_t V;              /* vocabulary size, >= 1 */
    int32_t gamma_max;      /* upper bound of every gamma_b, 1..SPECKV_GAMMA_LIMIT */
    int32_t gamma_uniform;  /* speculation length of every row when gamma == NULL */
    const int32_t *gamma;   /* DEVICE [B], each in [1, gamma_max] (a value outside is clamped on the
                               device and sets SPECKV_FLAG_BAD_GAMMA); NULL = uniform batch */
    const int64_t *row_off; /* DEVICE [B+1] draft-row offsets; required iff gamma != NULL */
    uint32_t seq_base;      /* global index of sequence 0 (random numbers are keyed by
                               seq_base + b, so results do not depend on how a job is sharded) */
} speckv_batch;

/* How the predictor f of Section 4.3 is evaluated for the four candidates Gamma = (2, 4, 6, 8).
 * VECTOR: one network with four outputs, f_j = output j (the benchmark configurations).
 * SCALAR: f_j = f([x, Gamma_j]), one output, evaluated four times (the form Section 4.3 writes;
 *         with n_hidden = 0 it is the Ridge predictor of Table 3). */
typedef enum { SPECKV_MLP_VECTOR = 0, SPECKV_MLP_SCALAR = 1 } speckv_mlp_form;

/* Controller weights (HOST struct of DEVICE pointers, row-major binary32).
 * n_x = n_in for VECTOR, n_in + 1 for SCALAR (Gamma_j is appended to the context vector as is);
 * n_out = 4 for VECTOR, 1 for SCALAR.
 *   n_hidden >= 1: h = relu(W1 x + b1), f = W2 h + b2
 *   n_hidden == 0: f = W2 x + b2 (no hidden layer; W1 and b1 are ignored and may be NULL) */
typedef struct {
    int32_t n_in;     /* 5 for POS0, 7 for AGG4 */
    int32_t n_hidden; /* 0..SPECKV_HIDDEN_LIMIT; the paper's controller has 16 */
    const float *W1;  /* DEVICE [n_hidden][n_x] */
    const float *b1;  /* DEVICE [n_hidden] */
    const float *W2;  /* DEVICE [n_out][n_hidden], or [n_out][n_x] when n_hidden == 0 */
    const float *b2;  /* DEVICE [n_out] */
    int32_t form;     /* speckv_mlp_form */
} speckv_mlp;

/* Create a handle bound to HIP device `device` (>= 0).  device = -1 creates a handle without a
 * device: every entry point then validates its arguments and returns SPECKV_ERR_DEVICE where
 * it would have launched (used to test argument checking on machines without a GPU). */
speckv_status speckv_create(speckv_handle **out, int device);
speckv_status speckv_destroy(speckv_handle *h);

/* Text of the most recent error on this handle (never NULL; h may be NULL). */
const char *speckv_last_error(const speckv_handle *h);

/* Bytes of DEVICE workspace a step with up to B sequences of up to gamma_max needs.
 * Returns 0 for arguments out of range. */
size_t speckv_workspace_bytes(int32_t B, int32_t gamma_max);

/* row_off[0] = 0, row_off[b+1] = row_off[b] + gamma[b] (DEVICE in, DEVICE out), so that a
 * chain of steps can feed gamma_next of one step into the packing of the next without a
 * host round trip. */
speckv_status speckv_row_offsets(speckv_handle *h, const int32_t *gamma, int32_t B,
                                 int64_t *row_off, speckv_stream stream);

/* Section 4.2.  Reads every draft row once.
 *   H       DEVICE [n_draft_rows]  entropy of q_i in bits, H = -sum_v q log2 q
 *   conf    DEVICE [n_draft_rows]  max_v q_i(v)
 *   argmax  DEVICE [n_draft_rows]  lowest index attaining the maximum, or NULL
 *   agg     DEVICE [B][4]          mean H, mean conf, max H, min conf over the row's positions
 * ws keeps (max, sum-exp, argmax) of every draft row for speckv_verify. */
speckv_status speckv_signals(speckv_handle *h, const speckv_batch *batch,
                             const void *draft_logits /* DEVICE */, speckv_dtype dtype,
                             void *ws /* DEVICE */, size_t ws_bytes, speckv_stream stream,
                             float *H, float *conf, int32_t *argmax, float *agg);

/* Section 3.1 with the lossless test of Section 2.1's references.  Reads every target row
 * once and, per sequence, position n of both sides a second time.  Must follow the
 * speckv_signals call of the same batch, logits and workspace (else SPECKV_ERR_STATE).
 *   position i is accepted iff  u_i * q_i(t_i) < p_i(t_i),  u_i = (w0 >> 8) * 2^-24 with
 *   (w0, w1, ., .) = Philox4x32-10(key = (seed low, seed high), ctr = (seq_base+b, i, step, 0));
 *   n = number of leading accepts.  The extra token is the smallest v with
 *   sum_{w<=v} r(w) > u' * sum_w r(w),  u' = w1 * 2^-32 of block (seq_base+b, n, step, 0),
 *   r = max(0, p_n - q_n) if n < gamma_b, else r = p_gamma (bonus); if the residual's mass is below
 *   1e-6 the token is drawn from p_n instead and SPECKV_FLAG_FALLBACK is set.
 *   n_accepted   DEVICE [B]               n
 *   tokens       DEVICE [B][gamma_max+1]  t_0..t_{n-1}, the extra token, then -1
 *   num_tokens   DEVICE [B]               n + 1
 *   accept_rate  DEVICE [B] or NULL       n / gamma_b
 *   row_flags    DEVICE [B] or NULL       SPECKV_FLAG_* bits */
speckv_status speckv_verify(speckv_handle *h, const speckv_batch *batch,
                            const void *target_logits /* DEVICE */,
                            const void *draft_logits /* DEVICE, as given to speckv_signals */,
                            speckv_dtype dtype, const int32_t *draft_tokens /* DEVICE [n_draft_rows] */,
                            uint64_t seed, uint32_t step, void *ws, size_t ws_bytes,
                            speckv_stream stream, int32_t *n_accepted, int32_t *tokens,
                            int32_t *num_tokens, float *accept_rate, uint32_t *row_flags);

/* Section 3.1, the accept rule exactly as the paper words it (greedy): position i is accepted iff
 * the target's top prediction argmax_v p_i(v) (lowest index on ties) equals the drafted token
 * t_i; at the first mismatch the target's prediction replaces the draft token, and after gamma_b
 * accepts the extra token is the target's top prediction at position gamma_b.  Reads every target
 * row once; needs no draft logits, no random numbers and no preceding speckv_signals, and leaves
 * what speckv_signals stored for speckv_verify untouched.  Outputs as for speckv_verify;
 * SPECKV_FLAG_FALLBACK is never set. */
speckv_status speckv_verify_greedy(speckv_handle *h, const speckv_batch *batch,
                                   const void *target_logits /* DEVICE */, speckv_dtype dtype,
                                   const int32_t *draft_tokens /* DEVICE [n_draft_rows] */, void *ws,
                                   size_t ws_bytes, speckv_stream stream, int32_t *n_accepted,
                                   int32_t *tokens, int32_t *num_tokens, float *accept_rate,
                                   uint32_t *row_flags);

/* Section 4.3.  f_j = predicted acceptance rate of candidate Gamma_j (see speckv_mlp),
 * score_j = f_j * Gamma_j + 1 with Gamma = (2,4,6,8) (Eq. 1); gamma_next = Gamma[argmax_j score_j],
 * lowest j on ties.
 *   H, conf   DEVICE per-draft-row signals (used by POS0: the row at position 0)
 *   agg       DEVICE [B][4]                (used by AGG4)
 *   comp      DEVICE [B] uint8             compression level of the target: 0 FP16, 1 INT8, 2 NF4
 *   gamma_next DEVICE [B];  scores DEVICE [B][4] or NULL
 * batch->V is ignored. */
speckv_status speckv_select_gamma(speckv_handle *h, const speckv_batch *batch,
                                  const speckv_mlp *mlp, speckv_features mode, const float *H,
                                  const float *conf, const float *agg, const uint8_t *comp,
                                  speckv_stream stream, int32_t *gamma_next, float *scores);

/* The step before verification (Section 3.1: the draft model proposes its gamma tokens):
 * one token per draft row, drawn from q_i = softmax(row) as the smallest v with
 * sum_{w<=v} q_i(w) > u, u = w0 * 2^-32 of Philox4x32-10(key = (seed low, seed high),
 * ctr = (seq_base+b, pos0+i, step, 1)) -- the fourth counter word keeps these draws apart from the
 * ones speckv_verify makes.  Rows are laid out as for speckv_signals; a caller that proposes one
 * position at a time passes a batch with gamma_uniform = 1 and the position in pos0.
 *   tokens    DEVICE [n_draft_rows]
 *   prob      DEVICE [n_draft_rows] q_i(t_i), or NULL
 *   row_flags DEVICE [n_draft_rows] SPECKV_FLAG_NONFINITE for a row with NaN, +inf or no finite
 *             logit (its token is then unspecified but inside [0, V)), or NULL
 * Reads every row once from memory; needs no workspace. */
speckv_status speckv_sample_draft(speckv_handle *h, const speckv_batch *batch,
                                  const void *draft_logits /* DEVICE */, speckv_dtype dtype,
                                  uint64_t seed, uint32_t step, uint32_t pos0, speckv_stream stream,
                                  int32_t *tokens, float *prob, uint32_t *row_flags);

/* One whole step in one call, for callers that hold the draft and the target logits together:
 * the same results, bit for bit, as speckv_signals + speckv_verify + speckv_select_gamma
 * (Sections 4.2, 3.1 and 4.3 / Eq. 1), from two launches: the row statistics of both sides in
 * one, then one workgroup per sequence for signals, accept scan, controller and resample.
 * With args->greedy the verification is speckv_verify_greedy's (again the same bits as the three
 * calls, again two launches, and no second read of any logits).
 * Launches kernels only (no allocation, no host synchronisation, no memset), so the call may be
 * captured in a HIP graph.  HOST struct; every pointer inside is a DEVICE pointer with the layout
 * and meaning documented at the three calls above.  Pointers marked "or NULL" may be NULL. */
typedef struct {
    const void *draft_logits;
    const void *target_logits;
    speckv_dtype dtype;
    const int32_t *draft_tokens;
    const uint8_t *comp;
    uint64_t seed;
    uint32_t step;
    speckv_features mode;
    /* outputs */
    float *H, *conf;
    int32_t *argmax; /* or NULL */
    float *agg;
    int32_t *n_accepted, *tokens, *num_tokens;
    float *accept_rate;  /* or NULL */
    uint32_t *row_flags; /* or NULL */
    int32_t *gamma_next;
    float *scores;       /* or NULL */
    /* 0: lossless accept test and resample (speckv_verify); 1: the greedy rule of Section 3.1
     * (speckv_verify_greedy): seed and step are then unused and the step takes no resample pass */
    int32_t greedy;
} speckv_step_args;

/* Errors as for the three calls; nothing is launched and no output is touched when a check
 * fails.  Does not need, and invalidates, the state speckv_signals leaves for speckv_verify. */
speckv_status speckv_step(speckv_handle *h, const speckv_batch *batch, const speckv_mlp *mlp,
                          const speckv_step_args *args, void *ws /* DEVICE */, size_t ws_bytes,
                          speckv_stream stream);

/* speckv_step for callers that cannot allocate device memory or hand over a workspace: code that
 * runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, checks, launches and results as speckv_step, except that the workspace is an array of
 * SPECKV_STATIC_WS_BYTES bytes inside the library (one copy per GPU, held until the process ends;
 * its device address is looked up once per GPU in speckv_create).  The call allocates nothing:
 * no hipMalloc / hipFree, no allocating library routine, no memset; it launches kernels only.
 * Limit: speckv_workspace_bytes(B, gamma_max) <= SPECKV_STATIC_WS_BYTES, else SPECKV_ERR_WORKSPACE
 * and nothing is launched (B = 4096 at gamma_max = 8 fits, B = 8192 does not).
 * All calls on one GPU, from any handle, share that GPU's array: two calls that overlap on one GPU
 * (different streams or threads) race; calls on one stream, or otherwise ordered, do not.  The array
 * keeps whatever the last call left in it; a step reads only what the same step wrote before.
 * Leaves the state speckv_signals keeps for speckv_verify untouched. */
#define SPECKV_STATIC_WS_BYTES (16u << 20)
speckv_status speckv_step_static(speckv_handle *h, const speckv_batch *batch, const speckv_mlp *mlp,
                                 const speckv_step_args *args, speckv_stream stream);

/* ---- measurement and tuning (not part of the method) ------------------------------------ */

/* Integer launch parameters, by name:
 *   "stats_target_wgs"   workgroups the statistics pass of a whole step (draft and target rows
 *                        together) aims for; rows are split into chunks to reach it (default 8192)
 *   "stats_max_split"    most chunks per row (default 16)
 *   "stats_threads"      128, 256 (default) or 512 threads per workgroup
 *   "stats_unroll"       16-byte loads per lane and tile: 2 (default) or 4
 *   "stats_pipeline"     0/1 (default 1): the next tile's loads are in flight while the current
 *                        one is processed
 *   "stats_nontemporal"  0/1 (default 1): nontemporal loads
 *   "stats_wgs_per_cu"   most statistics workgroups resident on one compute unit: 4 (default), 2..16,
 *                        or 0 = as many as the registers allow (fewer concurrent streams are served
 *                        faster by the memory system; the bound is set through LDS that a workgroup
 *                        occupies without using it)
 *   "step_tail"          1 (default) / 0: one workgroup per sequence runs everything after the
 *                        row statistics in one launch (speckv_step: signals, accept scan,
 *                        controller, resample; speckv_verify: accept scan and resample);
 *                        0 = separate launches for the accept scan and the two resample passes
 *   "sample_threads"     threads per workgroup of the proposal kernel: 0 (default) = 1024 below 512 rows and
 *                        512 from there on; or 512 / 1024
 *   "sample_loads"       16-byte loads per lane and group in the proposal kernel: 0 (default) = 4 with 512
 *                        threads and 2 with 1024; or 2 / 4
 *   "tail_threads"       threads per workgroup of the per-sequence tail kernel: 0 (default) = 1024 below 512
 *                        sequences and 512 from there on; or 512 / 1024
 *   "stats_pos0_last"    0 (default) / 1: speckv_step on a uniform batch lets the statistics launch read the
 *                        rows of position 0 last (same results; the tail's second read of position 0
 *                        then finds them in the memory-side cache more often)
 *   "probe_blocks"       workgroups of speckv_probe_read / speckv_probe_copy
 *   "profile_every"      while profiling, stamp only every n-th launch of a kernel class, so that
 *                        a timed region can carry the events at negligible cost
 * Unknown name or value out of range -> SPECKV_ERR_SHAPE. */
speckv_status speckv_set_option(speckv_handle *h, const char *name, int32_t value);
speckv_status speckv_get_option(const speckv_handle *h, const char *name, int32_t *value);

/* Per-kernel timing with HIP events on the caller's stream: while collecting, each kernel is
 * launched through hipExtLaunchKernel with a start and a stop event, which the runtime stamps
 * with that dispatch's own begin and end times (no extra barrier between kernels).
 * speckv_profile(h, 1) collects for the row-statistics kernels only, speckv_profile(h, 2)
 * for every kernel (both clear earlier records); speckv_profile(h, 0) stops.
 * speckv_profile_read synchronises the recorded events and returns, for the kernel
 * class named `kernel` ("row_stats_draft", "row_stats_target", "signals_finalize", "accept",
 * "resample_mass", "resample_pick", "select_gamma", "greedy_accept", "row_stats_pair",
 * "step_epilogue", "step_tail", "verify_tail", "sample_draft"), the number of launches recorded and
 * their summed duration in milliseconds. */
speckv_status speckv_profile(speckv_handle *h, int32_t enable);
speckv_status speckv_profile_read(speckv_handle *h, const char *kernel, int32_t *launches,
                                  double *total_ms);

/* Where the time inside the two launches of speckv_step goes: while a buffer is set, every
 * workgroup stores readings of the GPU's constant-rate clock (hipDeviceAttributeWallClockRate, kHz).
 *   buf[32*b + k]             tail launch, sequence b, thread 0: k = 0 entry, 1 statistics merged and
 *                             token logits gathered, 2 accept scan done, 3 descriptor visible to all
 *                             waves, 4 this wave's share of the residual masses done, 5 all masses
 *                             done, 6 chunk holding the threshold found, 7 that chunk re-read and
 *                             summed, 8 prefix exchanged, 9 token found, 10 token stored; 16 + w: wave w out of chunks in the mass pass
 *   buf[32*B + 2*w + 0..1]    statistics launch, workgroup w (in launch order): entry, exit
 * buf: DEVICE, 8-byte aligned, at least 8 * (32*B + 2 * statistics workgroups) bytes, else speckv_step
 * returns SPECKV_ERR_WORKSPACE; NULL stops the recording.  Measurement only: results are unchanged. */
speckv_status speckv_trace(speckv_handle *h, uint64_t *buf /* DEVICE or NULL */, size_t bytes);

/* Bandwidth probes: a read-only streaming sum over `bytes` of DEVICE memory (sink receives
 * 8 bytes so the loads are not dead) and a plain copy dst <- src.  bytes must be a multiple
 * of 16 and both pointers 16-byte aligned. */
speckv_status speckv_probe_read(speckv_handle *h, const void *src, size_t bytes,
                                void *sink /* DEVICE, >= 8 bytes */, speckv_stream stream);
speckv_status speckv_probe_copy(speckv_handle *h, void *dst, const void *src, size_t bytes,
                                speckv_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECKV_H */
