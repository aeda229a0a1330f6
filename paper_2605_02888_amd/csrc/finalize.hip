// Per-row and per-sequence epilogues: signals (Section 4.2), accept scan (Section 3.1 with the
// lossless test of the works cited in Section 2.1), controller (Section 4.3, Eq. 1), row offsets.
// All of this is O(B * gamma) work; every per-row quantity is formed in binary64.
#include "speckv_device.h"

namespace speckv {

constexpr int kGroup = 32; // lanes per sequence: one per position, gamma_max + 1 <= 17 of them used
constexpr int kFinThreads = 256;

__device__ __forceinline__ float load_logit(const void *base, int dtype, int64_t i)
{
    switch (dtype) {
    case SPECKV_F32: return Elem<SPECKV_F32>::load1(base, i);
    case SPECKV_F16: return Elem<SPECKV_F16>::load1(base, i);
    default: return Elem<SPECKV_BF16>::load1(base, i);
    }
}

__device__ __forceinline__ bool stat_is_bad(const RowStat &s)
{
    return !(s.S > 0.0) || !(s.S < INFINITY) || !(s.vmax < INFINITY) || !(s.vmax > -INFINITY);
}

template <typename T> __device__ __forceinline__ T group_sum(T v)
{
#pragma unroll
    for (int o = kGroup / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kGroup);
    return v;
}
__device__ __forceinline__ double group_max(double v)
{
#pragma unroll
    for (int o = kGroup / 2; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, kGroup));
    return v;
}
__device__ __forceinline__ double group_min(double v)
{
#pragma unroll
    for (int o = kGroup / 2; o > 0; o >>= 1) v = fmin(v, __shfl_xor(v, o, kGroup));
    return v;
}

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
        // entropy in bits: log2 S - T/S; confidence: the largest term of S over S
        h = log2(s.S) - s.T / s.S;
        c = exp2((double)fmaf(s.vmax, L2E_F, -s.ref)) / s.S;
        H[r] = (float)h;
        conf[r] = (float)c;
        if (argmax) argmax[r] = s.argmax;
    }
    const double sumH = group_sum(active ? h : 0.0);
    const double sumC = group_sum(active ? c : 0.0);
    const double maxH = group_max(active ? h : -INFINITY);
    const double minC = group_min(active ? c : INFINITY);
    if (seq_ok && i == 0) {
        agg[4 * b + 0] = (float)(sumH / g);
        agg[4 * b + 1] = (float)(sumC / g);
        agg[4 * b + 2] = (float)maxH;
        agg[4 * b + 3] = (float)minC;
    }
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
// Lane i of a sequence's group handles position i: merges the target row's chunk statistics,
// gathers the two logits at the drafted token, forms q(t) and p(t), draws u and tests
// u*q < p.  A ballot over the group gives the accept mask; the accepted prefix length is the
// number of trailing ones.  Lane n then describes the row(s) the resample pass must read.
__global__ __launch_bounds__(kFinThreads) void accept_kernel(
    BatchView bv, const void *__restrict__ draft, const void *__restrict__ target, int dtype,
    const int32_t *__restrict__ draft_tokens, uint32_t key0, uint32_t key1, uint32_t step,
    const RowStat *__restrict__ stat_d, const RowStat *__restrict__ partials_t, int split,
    RowStat *__restrict__ stat_t, ResampleDesc *__restrict__ desc, int32_t *__restrict__ n_accepted,
    int32_t *__restrict__ tokens, float *__restrict__ accept_rate)
{
    const int gid = blockIdx.x * (kFinThreads / kGroup) + threadIdx.x / kGroup;
    const int i = threadIdx.x % kGroup;
    const bool seq_ok = gid < bv.B;
    const int b = seq_ok ? gid : 0;
    const int g = batch_gamma(bv, b);
    const int64_t drow0 = batch_draft_row0(bv, b);
    const int64_t trow0 = drow0 + b;
    const int V = bv.V;

    RowStat sp, sq;
    sp.S = 1.0; sp.T = 0.0; sp.ref = 0.0f; sp.vmax = 0.0f; sp.argmax = 0; sp.pad = 0;
    sq = sp;
    bool accept = false;
    uint32_t flags = 0;
    int32_t tok = -1;
    Philox4 rnd = {{0, 0, 0, 0}};
    if (seq_ok && i <= g) {
        const int64_t tr = trow0 + i;
        sp = merge_partials(partials_t + tr * split, split);
        stat_t[tr] = sp;
        if (stat_is_bad(sp)) flags |= SPECKV_FLAG_NONFINITE;
        rnd = philox4x32_10(bv.seq_base + (uint32_t)b, (uint32_t)i, step, 0u, key0, key1);
    }
    if (seq_ok && i < g) {
        const int64_t dr = drow0 + i;
        sq = stat_d[dr];
        if (stat_is_bad(sq)) flags |= SPECKV_FLAG_NONFINITE;
        tok = draft_tokens[dr];
        double qt = 0.0, pt = 0.0;
        if (tok >= 0 && tok < V) {
            const float xq = load_logit(draft, dtype, dr * (int64_t)V + tok);
            const float xp = load_logit(target, dtype, (trow0 + i) * (int64_t)V + tok);
            qt = exp2((double)fmaf(xq, L2E_F, -sq.ref)) / sq.S;
            pt = exp2((double)fmaf(xp, L2E_F, -sp.ref)) / sp.S;
        } else {
            flags |= SPECKV_FLAG_BAD_TOKEN; // probability 0 on both sides: rejected here
        }
        const double u = (double)(rnd.w[0] >> 8) * 0x1.0p-24;
        accept = u * qt < pt;
    }
    // accept mask of this sequence's 32-lane group
    const uint64_t ball = __ballot(accept);
    const int shift = (threadIdx.x % kWave) & ~(kGroup - 1);
    const uint32_t mask = (uint32_t)(ball >> shift);
    const int n = __ffs((int)~mask) - 1; // leading accepts; lane g never accepts, so n <= g
    // OR of the flags over the group
#pragma unroll
    for (int o = kGroup / 2; o > 0; o >>= 1) flags |= __shfl_xor(flags, o, kGroup);

    if (!seq_ok) return;
    if (i <= bv.gamma_max) tokens[(int64_t)b * (bv.gamma_max + 1) + i] = (i < n) ? tok : -1;
    if (i == n) {
        ResampleDesc d;
        d.prow = trow0 + n;
        d.qrow = (n < g) ? drow0 + n : -1;
        d.u2 = (double)rnd.w[1] * 0x1.0p-32;
        d.nref_p = -sp.ref;
        d.inv_p = (float)(1.0 / sp.S);
        d.nref_q = -sq.ref;
        d.inv_q = (n < g) ? (float)(1.0 / sq.S) : 0.0f;
        d.n = n;
        d.flags = flags;
        d.pad[0] = d.pad[1] = d.pad[2] = d.pad[3] = 0;
        desc[b] = d;
        n_accepted[b] = n;
        if (accept_rate) accept_rate[b] = (float)n / (float)g;
    }
}

hipError_t launch_accept(const BatchView &bv, const void *draft, const void *target,
                         speckv_dtype dtype, const int32_t *draft_tokens, uint64_t seed,
                         uint32_t step, const RowStat *stat_d, const RowStat *partials_t, int split,
                         RowStat *stat_t, ResampleDesc *desc, int32_t *n_accepted, int32_t *tokens,
                         float *accept_rate, hipStream_t stream)
{
    const int per = kFinThreads / kGroup;
    const int blocks = (bv.B + per - 1) / per;
    return launch(accept_kernel, dim3(blocks), dim3(kFinThreads), stream, bv, draft, target,
                       (int)dtype, draft_tokens, (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32),
                       step, stat_d, partials_t, split, stat_t, desc, n_accepted, tokens, accept_rate);
}

// ---- controller -------------------------------------------------------------------------------
// One thread per sequence, weights staged in LDS, plain binary64 fused multiply-adds: about 300
// flops per decision, far too small for the matrix cores to matter.
struct MlpView {
    int n_in, n_hidden;
    const float *W1, *b1, *W2, *b2;
};

__global__ __launch_bounds__(256) void select_gamma_kernel(BatchView bv, MlpView m, int mode,
                                                           const float *__restrict__ H,
                                                           const float *__restrict__ conf,
                                                           const float *__restrict__ agg,
                                                           const uint8_t *__restrict__ comp,
                                                           int32_t *__restrict__ gamma_next,
                                                           float *__restrict__ scores)
{
    __shared__ float w1[SPECKV_HIDDEN_LIMIT * 7], c1[SPECKV_HIDDEN_LIMIT];
    __shared__ float w2[SPECKV_N_CANDIDATES * SPECKV_HIDDEN_LIMIT], c2[SPECKV_N_CANDIDATES];
    for (int k = threadIdx.x; k < m.n_hidden * m.n_in; k += blockDim.x) w1[k] = m.W1[k];
    for (int k = threadIdx.x; k < m.n_hidden; k += blockDim.x) c1[k] = m.b1[k];
    for (int k = threadIdx.x; k < SPECKV_N_CANDIDATES * m.n_hidden; k += blockDim.x) w2[k] = m.W2[k];
    if (threadIdx.x < SPECKV_N_CANDIDATES) c2[threadIdx.x] = m.b2[threadIdx.x];
    __syncthreads();
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= bv.B) return;
    double x[7];
    int k = 0;
    if (mode == SPECKV_FEAT_POS0) {
        const int64_t r0 = batch_draft_row0(bv, b);
        x[k++] = (double)H[r0];
        x[k++] = (double)conf[r0];
    } else {
        for (int j = 0; j < 4; ++j) x[k++] = (double)agg[4 * b + j];
    }
    const int cl = comp[b];
    for (int c = 0; c < 3; ++c) x[k++] = (cl == c) ? 1.0 : 0.0;
    double o[SPECKV_N_CANDIDATES];
    for (int j = 0; j < SPECKV_N_CANDIDATES; ++j) o[j] = (double)c2[j];
    for (int hdx = 0; hdx < m.n_hidden; ++hdx) {
        double a = (double)c1[hdx];
        for (int i = 0; i < m.n_in; ++i) a = fma((double)w1[hdx * m.n_in + i], x[i], a);
        a = a > 0.0 ? a : 0.0;
        for (int j = 0; j < SPECKV_N_CANDIDATES; ++j) o[j] = fma((double)w2[j * m.n_hidden + hdx], a, o[j]);
    }
    int best = 0;
    double best_score = 0.0;
    for (int j = 0; j < SPECKV_N_CANDIDATES; ++j) {
        const double sc = o[j] * (double)(2 * (j + 1)) + 1.0; // Eq. 1 with Gamma_j = 2, 4, 6, 8
        if (scores) scores[4 * b + j] = (float)sc;
        if (j == 0 || sc > best_score) { // strict: lowest index wins ties
            best = j;
            best_score = sc;
        }
    }
    gamma_next[b] = 2 * (best + 1);
}

hipError_t launch_select_gamma(const BatchView &bv, const speckv_mlp &mlp, int mode, const float *H,
                               const float *conf, const float *agg, const uint8_t *comp,
                               int32_t *gamma_next, float *scores, hipStream_t stream)
{
    MlpView m{mlp.n_in, mlp.n_hidden, mlp.W1, mlp.b1, mlp.W2, mlp.b2};
    const int blocks = (bv.B + 255) / 256;
    return launch(select_gamma_kernel, dim3(blocks), dim3(256), stream, bv, m, mode, H, conf, agg,
                       comp, gamma_next, scores);
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
