// Per-row and per-sequence epilogues: signals (Section 4.2), accept scan (Section 3.1 with the
// lossless test of the works cited in Section 2.1), controller (Section 4.3, Eq. 1), row offsets.
// All of this is O(B * gamma) work; every per-row quantity is formed in binary64.
#include "speckv_epilogue.h"

namespace speckv {

constexpr int kFinThreads = 256;

// ---- signals ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kFinThreads) void signals_finalize_kernel(BatchView bv,
                                                                       const RowStat *__restrict__ partials,
                                                                       int split, RowStat *__restrict__ stat_d,
                                                                       float *__restrict__ H,
                                                                       float *__restrict__ conf,
                                                                       int32_t *__restrict__ argmax,
                                                                       float *__restrict__ agg)
{
    const int gid = blockIdx.x * (kFinThreads / kGroup) + threadIdx.x / kGroup;
    const int i = threadIdx.x % kGroup;
    const bool seq_ok = gid < bv.B;
    const int b = seq_ok ? gid : 0;
    const int g = batch_gamma(bv, b);
    const int64_t row0 = batch_draft_row0(bv, b);
    const bool active = seq_ok && i < g;
    double h = 0.0, c = 0.0;
    if (active) {
        const int64_t r = row0 + i;
        const RowStat s = merge_partials(partials + r * split, split);
        stat_d[r] = s;
        row_signals(s, h, c);
        H[r] = (float)h;
        conf[r] = (float)c;
        if (argmax) argmax[r] = s.argmax;
    }
    write_aggregates(active, h, c, g, seq_ok && i == 0, agg + 4 * (int64_t)b);
}

hipError_t launch_signals_finalize(const BatchView &bv, const RowStat *partials, int split,
                                   RowStat *stat_d, float *H, float *conf, int32_t *argmax,
                                   float *agg, hipStream_t stream)
{
    const int per = kFinThreads / kGroup;
    const int blocks = (bv.B + per - 1) / per;
    return launch(signals_finalize_kernel, dim3(blocks), dim3(kFinThreads), stream, bv, partials,
                  split, stat_d, H, conf, argmax, agg);
}

// ---- accept scan ------------------------------------------------------------------------------
__global__ __launch_bounds__(kFinThreads) void accept_kernel(BatchView bv, AcceptArgs aa,
                                                             const RowStat *__restrict__ stat_d,
                                                             const RowStat *__restrict__ partials_t, int split,
                                                             RowStat *__restrict__ stat_t)
{
    const int gid = blockIdx.x * (kFinThreads / kGroup) + threadIdx.x / kGroup;
    const int i = threadIdx.x % kGroup;
    const bool live = gid < bv.B;
    const int b = live ? gid : 0;
    const int g = batch_gamma(bv, b);
    const int64_t drow0 = batch_draft_row0(bv, b);
    const TokenLogits tl = gather_token_logits(bv, aa, live, b, i, g, drow0); // in flight during the merges
    const Philox4 rnd = accept_block(bv, aa, b, i);
    RowStat sp, sq;
    sp.S = 1.0; sp.T = 0.0; sp.ref = 0.0f; sp.vmax = 0.0f; sp.argmax = 0; sp.pad = 0;
    sq = sp;
    if (live && i <= g) {
        const int64_t tr = drow0 + b + i;
        sp = merge_partials(partials_t + tr * split, split);
        stat_t[tr] = sp;
    }
    if (live && i < g) sq = stat_d[drow0 + i];
    accept_sequence(bv, aa, live, b, i, g, drow0, sp, sq, tl, rnd);
}

hipError_t launch_accept(const BatchView &bv, const void *draft, const void *target,
                         speckv_dtype dtype, const int32_t *draft_tokens, uint64_t seed,
                         uint32_t step, const RowStat *stat_d, const RowStat *partials_t, int split,
                         RowStat *stat_t, ResampleDesc *desc, int32_t *n_accepted, int32_t *tokens,
                         float *accept_rate, hipStream_t stream)
{
    const int per = kFinThreads / kGroup;
    const int blocks = (bv.B + per - 1) / per;
    AcceptArgs aa{draft, target, (int)dtype, draft_tokens, (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32),
                  step, desc, n_accepted, tokens, accept_rate};
    return launch(accept_kernel, dim3(blocks), dim3(kFinThreads), stream, bv, aa, stat_d, partials_t, split,
                  stat_t);
}

// ---- greedy verification ----------------------------------------------------------------------
// The accept rule as Section 3.1 words it: position i is accepted iff the target's top prediction
// (argmax of the target row, lowest index on ties) equals the drafted token; the target's
// prediction at the first mismatch -- or at the bonus position -- is the extra token.
__global__ __launch_bounds__(kFinThreads) void greedy_accept_kernel(BatchView bv,
                                                                    const int32_t *__restrict__ draft_tokens,
                                                                    const RowStat *__restrict__ partials_t,
                                                                    int split, RowStat *__restrict__ stat_t,
                                                                    int32_t *__restrict__ n_accepted,
                                                                    int32_t *__restrict__ tokens,
                                                                    int32_t *__restrict__ num_tokens,
                                                                    float *__restrict__ accept_rate,
                                                                    uint32_t *__restrict__ row_flags)
{
    const int gid = blockIdx.x * (kFinThreads / kGroup) + threadIdx.x / kGroup;
    const int i = threadIdx.x % kGroup;
    const bool live = gid < bv.B;
    const int b = live ? gid : 0;
    const int g = batch_gamma(bv, b);
    const int64_t drow0 = batch_draft_row0(bv, b);
    RowStat sp;
    sp.S = 1.0; sp.T = 0.0; sp.ref = 0.0f; sp.vmax = 0.0f; sp.argmax = 0; sp.pad = 0;
    if (live && i <= g) {
        const int64_t tr = drow0 + b + i;
        sp = merge_partials(partials_t + tr * split, split);
        stat_t[tr] = sp;
    }
    greedy_sequence(bv, draft_tokens, live, b, i, g, drow0, sp,
                    GreedyOut{n_accepted, tokens, num_tokens, accept_rate, row_flags});
}

hipError_t launch_greedy_accept(const BatchView &bv, const int32_t *draft_tokens, const RowStat *partials_t,
                                int split, RowStat *stat_t, int32_t *n_accepted, int32_t *tokens,
                                int32_t *num_tokens, float *accept_rate, uint32_t *row_flags, hipStream_t stream)
{
    const int per = kFinThreads / kGroup;
    const int blocks = (bv.B + per - 1) / per;
    return launch(greedy_accept_kernel, dim3(blocks), dim3(kFinThreads), stream, bv, draft_tokens, partials_t,
                  split, stat_t, n_accepted, tokens, num_tokens, accept_rate, row_flags);
}

// ---- controller -------------------------------------------------------------------------------
__global__ __launch_bounds__(kMlpThreads) void select_gamma_kernel(BatchView bv, MlpView m, int mode,
                                                                   const float *__restrict__ H,
                                                                   const float *__restrict__ conf,
                                                                   const float *__restrict__ agg,
                                                                   const uint8_t *__restrict__ comp,
                                                                   int32_t *__restrict__ gamma_next,
                                                                   float *__restrict__ scores)
{
    __shared__ MlpShared sh;
    stage_mlp(sh, m, threadIdx.x, kMlpThreads);
    const int seq = blockIdx.x * (kMlpThreads / kMlpLanes) + threadIdx.x / kMlpLanes;
    const int j = threadIdx.x % kMlpLanes;
    const bool live = seq < bv.B;
    const int b = live ? seq : 0;
    // context vector (every lane of the group holds all of it)
    float h0 = 0.0f, c0 = 0.0f, a[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (mode == SPECKV_FEAT_POS0) {
        const int64_t r0 = batch_draft_row0(bv, b);
        h0 = H[r0];
        c0 = conf[r0];
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) a[k] = agg[4 * b + k];
    }
    double x[7];
    controller_input(mode, h0, c0, a, comp[b], x);
    __syncthreads();
    controller_decide(sh, m, x, j, live, b, gamma_next, scores);
}

hipError_t launch_select_gamma(const BatchView &bv, const speckv_mlp &mlp, int mode, const float *H,
                               const float *conf, const float *agg, const uint8_t *comp,
                               int32_t *gamma_next, float *scores, hipStream_t stream)
{
    const MlpView m = mlp_view(mlp);
    const int per = kMlpThreads / kMlpLanes;
    const int blocks = (bv.B + per - 1) / per;
    return launch(select_gamma_kernel, dim3(blocks), dim3(kMlpThreads), stream, bv, m, mode, H, conf, agg,
                  comp, gamma_next, scores);
}

// ---- whole-step epilogue ----------------------------------------------------------------------
// Everything between the row statistics and the resample pass in one launch, for callers that hand
// over draft and target logits together: signals (Section 4.2), accept scan (Section 3.1) and
// the controller's decision (Section 4.3, Eq. 1), 32 lanes per sequence.  Same arithmetic, in the
// same order, as signals_finalize_kernel, accept_kernel and select_gamma_kernel.  With `greedy` the
// accept scan is the top-1 match of Section 3.1 (as in greedy_accept_kernel) and the step ends here.
__global__ __launch_bounds__(kFinThreads) void step_epilogue_kernel(BatchView bv, AcceptArgs aa,
                                                                    const RowStat *__restrict__ partials_d,
                                                                    int split_d,
                                                                    const RowStat *__restrict__ partials_t,
                                                                    int split_t, RowStat *__restrict__ stat_d,
                                                                    RowStat *__restrict__ stat_t, MlpView m, int mode,
                                                                    const uint8_t *__restrict__ comp, StepOut out,
                                                                    int greedy, GreedyOut go)
{
    __shared__ MlpShared sh;
    stage_mlp(sh, m, threadIdx.x, kFinThreads);
    const int gid = blockIdx.x * (kFinThreads / kGroup) + threadIdx.x / kGroup;
    const int i = threadIdx.x % kGroup;
    const bool live = gid < bv.B;
    const int b = live ? gid : 0;
    const int g = batch_gamma(bv, b);
    const int64_t drow0 = batch_draft_row0(bv, b);
    const int level = comp[b];
    TokenLogits tl;
    tl.tok = -1; tl.xq = 0.0f; tl.xp = 0.0f; tl.bad = false;
    Philox4 rnd = {{0, 0, 0, 0}};
    if (!greedy) {
        tl = gather_token_logits(bv, aa, live, b, i, g, drow0); // in flight during the merges
        rnd = accept_block(bv, aa, b, i);
    }
    RowStat sp, sq;
    sp.S = 1.0; sp.T = 0.0; sp.ref = 0.0f; sp.vmax = 0.0f; sp.argmax = 0; sp.pad = 0;
    sq = sp;
    if (live && i <= g) {
        const int64_t tr = drow0 + b + i;
        sp = merge_partials(partials_t + tr * split_t, split_t);
        stat_t[tr] = sp;
    }
    const bool active = live && i < g;
    double h = 0.0, c = 0.0;
    if (active) {
        const int64_t r = drow0 + i;
        sq = merge_partials(partials_d + r * split_d, split_d);
        stat_d[r] = sq;
        row_signals(sq, h, c);
        out.H[r] = (float)h;
        out.conf[r] = (float)c;
        if (out.argmax) out.argmax[r] = sq.argmax;
    }
    float a[4];
    sequence_aggregates(active, h, c, g, a);
    if (live && i == 0) {
#pragma unroll
        for (int k = 0; k < 4; ++k) out.agg[4 * (int64_t)b + k] = a[k];
    }
    if (greedy)
        greedy_sequence(bv, aa.draft_tokens, live, b, i, g, drow0, sp, go);
    else
        accept_sequence(bv, aa, live, b, i, g, drow0, sp, sq, tl, rnd);
    // controller: the first 16 lanes of the group, from the signals as stored (binary32)
    const float h0 = __shfl((float)h, 0, kGroup), c0 = __shfl((float)c, 0, kGroup);
    double x[7];
    controller_input(mode, h0, c0, a, level, x);
    __syncthreads();
    controller_decide(sh, m, x, i % kMlpLanes, live && i < kMlpLanes, b, out.gamma_next, out.scores);
}

hipError_t launch_step_epilogue(const BatchView &bv, const AcceptArgs &aa, const RowStat *partials_d, int split_d,
                                const RowStat *partials_t, int split_t, RowStat *stat_d, RowStat *stat_t,
                                const speckv_mlp &mlp, int mode, const uint8_t *comp, float *H, float *conf,
                                int32_t *argmax, float *agg, int32_t *gamma_next, float *scores, bool greedy,
                                int32_t *num_tokens, uint32_t *row_flags, hipStream_t stream)
{
    const MlpView m = mlp_view(mlp);
    StepOut out{H, conf, argmax, agg, gamma_next, scores};
    const GreedyOut go{aa.n_accepted, aa.tokens, num_tokens, aa.accept_rate, row_flags};
    const int per = kFinThreads / kGroup;
    const int blocks = (bv.B + per - 1) / per;
    return launch(step_epilogue_kernel, dim3(blocks), dim3(kFinThreads), stream, bv, aa, partials_d, split_d,
                  partials_t, split_t, stat_d, stat_t, m, mode, comp, out, greedy ? 1 : 0, go);
}

// ---- row offsets ------------------------------------------------------------------------------
// Exclusive prefix sum of gamma[B] by one workgroup: each thread sums a contiguous slice, the
// slice totals are scanned through LDS, then each thread writes its slice.
__global__ __launch_bounds__(1024) void row_offsets_kernel(const int32_t *__restrict__ gamma, int B,
                                                           int64_t *__restrict__ row_off)
{
    __shared__ int64_t part[1024];
    const int tid = threadIdx.x;
    const int per = (B + 1023) / 1024;
    const int lo = min(B, tid * per), hi = min(B, lo + per);
    int64_t s = 0;
    for (int k = lo; k < hi; ++k) s += gamma[k];
    part[tid] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) { // Hillis-Steele inclusive scan
        const int64_t add = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int64_t run = tid ? part[tid - 1] : 0;
    for (int k = lo; k < hi; ++k) {
        row_off[k] = run;
        run += gamma[k];
    }
    if (tid == 1023) row_off[B] = part[1023];
}

hipError_t launch_row_offsets(const int32_t *gamma, int B, int64_t *row_off, hipStream_t stream)
{
    return launch(row_offsets_kernel, dim3(1), dim3(1024), stream, gamma, B, row_off);
}

} // namespace speckv
