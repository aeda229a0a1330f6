// Per-row and per-sequence epilogue arithmetic shared by the stand-alone epilogue kernels and by
// the per-sequence tail kernel: signals of a row (Section 4.2), aggregates of a
// sequence, and the accept scan of a sequence (Section 3.1 with the lossless test of the works
// cited in Section 2.1).  Everything here is O(gamma) work per sequence in binary64.
#pragma once

#include "speckv_device.h"

namespace speckv {

constexpr int kGroup = 32; // lanes per sequence: one per position, gamma_max + 1 <= 17 of them used

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

// Entropy in bits (log2 S - T/S) and max probability (largest term of S over S) of one row.
__device__ __forceinline__ void row_signals(const RowStat &s, double &h, double &c)
{
    h = log2(s.S) - s.T / s.S;
    // the maximum is one of the terms of S, which holds it to one ulp of the hardware exp2: cap at 1
    c = fmin(1.0, exp2((double)fmaf(s.vmax, L2E_F, -s.ref)) / s.S);
}

// Aggregates of one sequence by its 32-lane group: lane i holds (h, c) of position i if active.
// Every lane of the group receives (mean H, mean c, max H, min c) as the binary32 values stored.
__device__ __forceinline__ void sequence_aggregates(bool active, double h, double c, int g, float (&a)[4])
{
    const double sumH = group_sum(active ? h : 0.0);
    const double sumC = group_sum(active ? c : 0.0);
    const double maxH = group_max(active ? h : -INFINITY);
    const double minC = group_min(active ? c : INFINITY);
    a[0] = (float)(sumH / g);
    a[1] = (float)(sumC / g);
    a[2] = (float)maxH;
    a[3] = (float)minC;
}

__device__ __forceinline__ void write_aggregates(bool active, double h, double c, int g, bool writer,
                                                 float *__restrict__ agg4)
{
    float a[4];
    sequence_aggregates(active, h, c, g, a);
    if (writer) {
#pragma unroll
        for (int k = 0; k < 4; ++k) agg4[k] = a[k];
    }
}

// What lane i of a sequence's group reads from the logits for the accept test: the drafted token
// and its logit on both sides.  A separate step so that a caller can issue these dependent loads
// (token, then logits) before it turns to the row statistics.
struct TokenLogits {
    int32_t tok;
    float xq, xp;
    bool bad; // token id outside [0, V)
};
// `tok` is the drafted token of position i (loaded by the caller, who may have other loads in flight
// beside it); ignored where no position is live.
__device__ __forceinline__ TokenLogits gather_token_logits(const BatchView &bv, const AcceptArgs &aa, bool live, int b,
                                                           int i, int g, int64_t drow0, int32_t tok)
{
    TokenLogits t;
    t.tok = -1; t.xq = 0.0f; t.xp = 0.0f; t.bad = false;
    if (live && i < g) {
        const int64_t dr = drow0 + i;
        t.tok = tok;
        if (t.tok >= 0 && t.tok < bv.V) {
            t.xq = load_logit(aa.draft, aa.dtype, dr * (int64_t)bv.V + t.tok);
            t.xp = load_logit(aa.target, aa.dtype, (drow0 + b + i) * (int64_t)bv.V + t.tok);
        } else {
            t.bad = true;
        }
    }
    return t;
}

__device__ __forceinline__ TokenLogits gather_token_logits(const BatchView &bv, const AcceptArgs &aa, bool live, int b,
                                                           int i, int g, int64_t drow0)
{
    const int32_t tok = (live && i < g) ? aa.draft_tokens[drow0 + i] : -1;
    return gather_token_logits(bv, aa, live, b, i, g, drow0, tok);
}

// The random numbers of position i of sequence b: word 0 drives the accept test, word 1 the resample
// draw should the scan stop at i.  They depend on no data, so a caller draws them while its loads
// are in flight.
__device__ __forceinline__ Philox4 accept_block(const BatchView &bv, const AcceptArgs &aa, int b, int i)
{
    return philox4x32_10(bv.seq_base + (uint32_t)b, (uint32_t)i, aa.step, 0u, aa.key0, aa.key1);
}

// The flag bits any lane of a 32-lane group holds, in every lane of the group (`shift` = first lane
// of the group inside the wave): one ballot per flag instead of a butterfly of permutes.
__device__ __forceinline__ uint32_t group_or_flags(uint32_t flags, int shift)
{
    uint32_t all = 0;
#pragma unroll
    for (uint32_t bit = 1; bit <= 8u; bit <<= 1)
        if ((uint32_t)(__ballot((flags & bit) != 0) >> shift)) all |= bit;
    return all;
}

// What an accept scan leaves in memory: the accepted prefix of the token row (lane i stores slot i),
// and, by the lane for which `writer` holds, the resample descriptor `d`, n and n / g.
__device__ __forceinline__ void accept_store(const BatchView &bv, const AcceptArgs &aa, bool live, int b, int i, int g,
                                             int n, int32_t tok, bool writer, const ResampleDesc &d)
{
    if (!live) return;
    if (i <= bv.gamma_max) aa.tokens[(int64_t)b * (bv.gamma_max + 1) + i] = (i < n) ? tok : -1;
    if (writer) {
        aa.desc[b] = d;
        aa.n_accepted[b] = n;
        if (aa.accept_rate) aa.accept_rate[b] = (float)n / (float)g;
    }
}

// Accept scan of sequence b by one 32-lane group (all 64 lanes of the wave must call this; lanes
// outside a live group pass live = false).  Lane i holds sp = statistics of target row i (i <= g),
// sq = statistics of draft row i (i < g) and tl = its drafted token with the two logits.  Lane i
// forms q(t_i), p(t_i), takes u_i from rnd = accept_block(b, i) and tests u*q < p; a ballot gives the accept mask and the
// accepted prefix length n is its number of trailing ones.  Lane n then describes the rows the
// resample pass must read.  With DEFER_STORES nothing is stored to memory here (only *desc_copy is
// written): the caller issues accept_store later, where no barrier waits for the stores.
template <bool DEFER_STORES = false>
__device__ __forceinline__ void accept_sequence(const BatchView &bv, const AcceptArgs &aa, bool live, int b,
                                                int i, int g, int64_t drow0, const RowStat &sp,
                                                const RowStat &sq, const TokenLogits &tl, const Philox4 &rnd,
                                                ResampleDesc *desc_copy = nullptr)
{
    const int64_t trow0 = drow0 + b;
    bool accept = false;
    uint32_t flags = 0;
    const int32_t tok = tl.tok;
    if (live && i <= g) {
        if (stat_is_bad(sp)) flags |= SPECKV_FLAG_NONFINITE;
        if (i == 0 && batch_gamma_clamped(bv, b)) flags |= SPECKV_FLAG_BAD_GAMMA;
    }
    if (live && i < g) {
        if (stat_is_bad(sq)) flags |= SPECKV_FLAG_NONFINITE;
        double qt = 0.0, pt = 0.0;
        if (!tl.bad) {
            qt = exp2((double)fmaf(tl.xq, L2E_F, -sq.ref)) / sq.S;
            pt = exp2((double)fmaf(tl.xp, L2E_F, -sp.ref)) / sp.S;
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
    flags = group_or_flags(flags, shift);

    if (!live) return;
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
        if (desc_copy) *desc_copy = d; // for a caller that goes on to the resample pass itself
        if (!DEFER_STORES) accept_store(bv, aa, live, b, i, g, n, tok, true, d);
    } else if (!DEFER_STORES) {
        accept_store(bv, aa, live, b, i, g, n, tok, false, ResampleDesc{});
    }
}

// Greedy verification of sequence b by one 32-lane group (all 64 lanes of the wave call this; lanes
// outside a live group pass live = false): the accept rule as Section 3.1 words it.  Lane i holds
// sp = statistics of target row i (i <= g) with its argmax; position i is accepted iff that top
// prediction equals the drafted token, and the target's prediction at the first mismatch -- or at
// the bonus position -- is the extra token.
struct GreedyOut {
    int32_t *n_accepted, *tokens, *num_tokens;
    float *accept_rate;
    uint32_t *row_flags;
};
__device__ __forceinline__ void greedy_sequence(const BatchView &bv, const int32_t *__restrict__ draft_tokens,
                                                bool live, int b, int i, int g, int64_t drow0, const RowStat &sp,
                                                const GreedyOut &o)
{
    uint32_t flags = 0;
    int32_t top = -1, tok = -1;
    bool match = false;
    if (live && i <= g) {
        if (stat_is_bad(sp)) flags |= SPECKV_FLAG_NONFINITE;
        if (i == 0 && batch_gamma_clamped(bv, b)) flags |= SPECKV_FLAG_BAD_GAMMA;
        top = sp.argmax;
    }
    if (live && i < g) {
        tok = draft_tokens[drow0 + i];
        if (tok < 0 || tok >= bv.V) flags |= SPECKV_FLAG_BAD_TOKEN;
        match = tok == top;
    }
    const uint64_t ball = __ballot(match);
    const int shift = (threadIdx.x % kWave) & ~(kGroup - 1);
    const uint32_t mask = (uint32_t)(ball >> shift);
    const int n = __ffs((int)~mask) - 1; // leading matches; lane g never matches, so n <= g
    flags = group_or_flags(flags, shift);
    if (!live) return;
    if (i <= bv.gamma_max) o.tokens[(int64_t)b * (bv.gamma_max + 1) + i] = (i < n) ? tok : (i == n ? top : -1);
    if (i == n) {
        o.n_accepted[b] = n;
        o.num_tokens[b] = n + 1;
        if (o.accept_rate) o.accept_rate[b] = (float)n / (float)g;
        if (o.row_flags) o.row_flags[b] = flags;
    }
}

// ---- controller (Section 4.3, Eq. 1) ------------------------------------------------------------
// 16 lanes per sequence, weights staged in LDS, plain binary64 fused multiply-adds: lane j takes
// hidden units j, j+16, ... and their contributions to the four outputs; a 4-step shuffle tree
// adds the lanes.  About 300 flops per decision: far too small for the matrix cores to matter.
struct MlpView {
    int n_in, n_hidden, form;
    const float *W1, *b1, *W2, *b2;
};
__host__ __device__ inline MlpView mlp_view(const speckv_mlp &m)
{
    return MlpView{m.n_in, m.n_hidden, m.form, m.W1, m.b1, m.W2, m.b2};
}

constexpr int kMlpLanes = 16;
constexpr int kMlpThreads = 256;
constexpr int kMlpMaxX = 8; // context vector (<= 7) plus the candidate gamma of the scalar form

struct MlpShared {
    float w1[SPECKV_HIDDEN_LIMIT * kMlpMaxX], c1[SPECKV_HIDDEN_LIMIT];
    float w2[SPECKV_N_CANDIDATES * SPECKV_HIDDEN_LIMIT], c2[SPECKV_N_CANDIDATES];
};

// All threads of the workgroup; a barrier must follow before the weights are used.
__device__ __forceinline__ void stage_mlp(MlpShared &sh, const MlpView &m, int tid, int nthreads)
{
    const int n_x = m.n_in + (m.form == SPECKV_MLP_SCALAR ? 1 : 0);
    const int n_out = m.form == SPECKV_MLP_SCALAR ? 1 : SPECKV_N_CANDIDATES;
    const int n_w2 = n_out * (m.n_hidden > 0 ? m.n_hidden : n_x);
    for (int k = tid; k < m.n_hidden * n_x; k += nthreads) sh.w1[k] = m.W1[k];
    for (int k = tid; k < m.n_hidden; k += nthreads) sh.c1[k] = m.b1[k];
    for (int k = tid; k < n_w2; k += nthreads) sh.w2[k] = m.W2[k];
    if (tid < n_out) sh.c2[tid] = m.b2[tid];
}

// Context vector of Section 4.3 from the stored binary32 signals.
__device__ __forceinline__ void controller_input(int mode, float h0, float c0, const float (&a)[4], int level,
                                                 double (&x)[7])
{
#pragma unroll
    for (int k = 0; k < 7; ++k) x[k] = 0.0;
    if (mode == SPECKV_FEAT_POS0) {
        x[0] = (double)h0;
        x[1] = (double)c0;
#pragma unroll
        for (int c = 0; c < 3; ++c) x[2 + c] = (level == c) ? 1.0 : 0.0;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = (double)a[k];
#pragma unroll
        for (int c = 0; c < 3; ++c) x[4 + c] = (level == c) ? 1.0 : 0.0;
    }
}

// Called by 16 consecutive lanes (j = 0..15) that all hold the same x; lane 0 with `writer` set
// stores the decision of sequence b (Eq. 1: score = predicted rate * Gamma + 1, lowest index on ties).
// Lane j takes hidden units j, j + 16, ...; without a hidden layer lane 0 does the few products.
__device__ __forceinline__ void controller_decide(const MlpShared &sh, const MlpView &m, const double (&x)[7], int j,
                                                  bool writer, int b, int32_t *__restrict__ gamma_next,
                                                  float *__restrict__ scores)
{
    double o[SPECKV_N_CANDIDATES] = {0, 0, 0, 0};
    const bool scalar = m.form == SPECKV_MLP_SCALAR;
    const int n_x = m.n_in + (scalar ? 1 : 0);
    if (m.n_hidden > 0) {
        for (int hdx = j; hdx < m.n_hidden; hdx += kMlpLanes) {
            double a = (double)sh.c1[hdx];
#pragma unroll
            for (int i = 0; i < 7; ++i)
                if (i < m.n_in) a = fma((double)sh.w1[hdx * n_x + i], x[i], a);
            if (!scalar) {
                a = a > 0.0 ? a : 0.0;
#pragma unroll
                for (int k = 0; k < SPECKV_N_CANDIDATES; ++k) o[k] = fma((double)sh.w2[k * m.n_hidden + hdx], a, o[k]);
            } else {
                const double wg = (double)sh.w1[hdx * n_x + m.n_in], w2 = (double)sh.w2[hdx];
#pragma unroll
                for (int k = 0; k < SPECKV_N_CANDIDATES; ++k) {
                    const double u = fma(wg, (double)(2 * (k + 1)), a);
                    o[k] = fma(w2, u > 0.0 ? u : 0.0, o[k]);
                }
            }
        }
    } else if (j == 0) {
#pragma unroll
        for (int k = 0; k < SPECKV_N_CANDIDATES; ++k) {
            const float *w = sh.w2 + (scalar ? 0 : k * n_x);
            double a = 0.0;
#pragma unroll
            for (int i = 0; i < 7; ++i)
                if (i < m.n_in) a = fma((double)w[i], x[i], a);
            if (scalar) a = fma((double)w[m.n_in], (double)(2 * (k + 1)), a);
            o[k] = a;
        }
    }
#pragma unroll
    for (int k = 0; k < SPECKV_N_CANDIDATES; ++k) {
#pragma unroll
        for (int s = kMlpLanes / 2; s > 0; s >>= 1) o[k] += __shfl_xor(o[k], s, kMlpLanes);
    }
    if (!writer || j != 0) return;
    int best = 0;
    double best_score = 0.0;
#pragma unroll
    for (int k = 0; k < SPECKV_N_CANDIDATES; ++k) {
        const double sc = (o[k] + (double)sh.c2[scalar ? 0 : k]) * (double)(2 * (k + 1)) + 1.0; // Eq. 1, Gamma_k = 2, 4, 6, 8
        if (scores) scores[4 * b + k] = (float)sc;
        if (k == 0 || sc > best_score) { // strict: lowest index wins ties
            best = k;
            best_score = sc;
        }
    }
    gamma_next[b] = 2 * (best + 1);
}

// Output pointers of the kernels that run a whole step's epilogue.
struct StepOut {
    float *H, *conf;
    int32_t *argmax;
    float *agg;
    int32_t *gamma_next;
    float *scores;
};

// Sequence that owns packed row `row` (draft rows: extra = 0, target rows: extra = 1).
__device__ __forceinline__ int seq_of_row(const BatchView &bv, int64_t row, int extra)
{
    if (!bv.row_off) return (int)(row / (bv.gamma_uniform + extra));
    int lo = 0, hi = bv.B - 1; // largest b with row_off[b] + extra*b <= row
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (bv.row_off[mid] + (int64_t)extra * mid <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

} // namespace speckv
