// The one extra token of a speculation step (Section 3.1: the target's own token at the first
// rejected position, or one more token after gamma accepts),
// drawn as in the lossless scheme of the works cited in Section 2.1:
//     r(v) = max(0, p_n(v) - q_n(v))  if the draft at position n was rejected,
//     r(v) = p_gamma(v)               if every draft was accepted (bonus),
// token = smallest v with  sum_{w<=v} r(w) > u' * sum_w r(w).
//
// Two phases.  Mass: one wave per (sequence, chunk of the row) sums r over the chunk (coalesced
// 16-byte loads, two register buffers, binary32 per element, binary64 across lanes).  Pick: 256
// threads per sequence scan the chunk masses, find the chunk holding the threshold, re-read only
// that chunk in vocabulary order with a prefix sum over the threads and walk to the token.
// Per-element values are computed by the same expression in both phases, and every kernel below
// forms a chunk mass by the same function, so all of them return identical results:
//   resample_mass_kernel + resample_pick_kernel   two launches, any batch
//   step_tail_kernel                              one workgroup per sequence does the whole tail of
//                                                 a step: signals, accept scan, controller, mass, pick
// The same pick also serves sample_rows_kernel, the draft side's token proposal (further below).
#include "speckv_accum.h"
#include "speckv_epilogue.h"

namespace speckv {

constexpr int kRsThreads = 256;
constexpr double kResidualFloor = 1e-6; // residual mass (total-variation distance of p_n and q_n) below which
                                        // the correction is drawn from p_n

// p(v) (or p(v) - q(v) clipped at 0) from raw logits with the row's reference and 1/S.
__device__ __forceinline__ float resid(float xp, float xq, bool has_q, float nref_p, float inv_p,
                                       float nref_q, float inv_q)
{
    const float p = exp2_hw(fmaf(xp, L2E_F, nref_p)) * inv_p;
    if (!has_q) return p;
    const float q = exp2_hw(fmaf(xq, L2E_F, nref_q)) * inv_q;
    return fmaxf(p - q, 0.0f);
}

typedef unsigned int rs_v4u32 __attribute__((ext_vector_type(4)));
template <bool NT> __device__ __forceinline__ uint4 rs_ld16(const uint4 *p)
{
    if (!NT) return *p;
    const rs_v4u32 v = __builtin_nontemporal_load(reinterpret_cast<const rs_v4u32 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
// 16 bytes from an address that is only 4-byte aligned (the hardware takes dword-aligned vector loads).
typedef unsigned int rs_v4u32_a4 __attribute__((ext_vector_type(4), aligned(4)));
template <bool NT> __device__ __forceinline__ uint4 rs_ld16_a4(const void *p)
{
    const rs_v4u32_a4 *q = static_cast<const rs_v4u32_a4 *>(p);
    const rs_v4u32_a4 v = NT ? __builtin_nontemporal_load(q) : *q;
    return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int kMassLoads = 2; // 16-byte loads per row, lane and iteration, all requested before any is used
                              // (measured at the headline workload: 2 beats 4 by 1 us, 1 and 8 lose 3 us)

// Sum of r over elements [e0, e1) of the row(s) of `d` by one wave; every lane gets the result.
// NT: nontemporal loads (the mass pass streams; the fallback inside the pick pass does not).
// HAS_Q: residual max(0, p - q); otherwise r = p (bonus row, fall-back, token proposal).  A template
// parameter, not a run-time flag: with a flag the compiler put a wait and a branch between the load
// of a target vector and the load of its draft vector, and every group of loads cost three memory
// round trips instead of one.
template <int DT, bool NT, bool HAS_Q>
__device__ __forceinline__ double wave_chunk_mass_of(const void *draft, const void *target, int V,
                                                     const ResampleDesc &d, int e0, int e1, int lane)
{
    using E = Elem<DT>;
    constexpr int NE = E::NE;
    const int n = max(0, e1 - e0);
    const int64_t p0 = d.prow * (int64_t)V + e0;
    const int64_t q0 = (HAS_Q ? d.qrow : 0) * (int64_t)V + e0;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(target) + (uintptr_t)p0 * E::BYTES;
    const uintptr_t qa = reinterpret_cast<uintptr_t>(draft) + (uintptr_t)q0 * E::BYTES;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    // The vectors are aligned for the target row.  The draft row may sit at another 16-byte phase
    // (row pitch not a multiple of 16 bytes), so its vectors are always fetched as 16 bytes from a
    // 4-byte aligned address; rows of 16-bit elements at an odd element offset fall back to element loads.
    const bool vec_ok = !HAS_Q || (((pa ^ qa) & 3) == 0);
    int head = n, nvec = 0;
    if (vec_ok) {
        head = min((int)(((16 - (pa & 15)) & 15) / E::BYTES), n);
        nvec = (n - head) / NE;
    }
    // derived from the kernel arguments so that the loads stay in the global address space
    const uint4 *pv = reinterpret_cast<const uint4 *>(static_cast<const char *>(target) + (p0 + head) * E::BYTES);
    const uint4 *qv = reinterpret_cast<const uint4 *>(static_cast<const char *>(draft) + (q0 + head) * E::BYTES);
    // Two register buffers: the loads of the next group of vectors are in flight while the current
    // group is exponentiated (the vector ALU work of this pass is of the same order as its memory
    // time, so the two must overlap inside a wave, not only across waves).  Groups are consumed in
    // ascending order, so the sums do not depend on the buffering.
    constexpr int kGroupVecs = kMassLoads * kWave;
    const int groups = (nvec + kGroupVecs - 1) / kGroupVecs;
    uint4 ap[kMassLoads], aq[kMassLoads], bp[kMassLoads], bq[kMassLoads];
    auto issue = [&](int gi, uint4 (&wp)[kMassLoads], uint4 (&wq)[kMassLoads]) {
#pragma unroll
        for (int j = 0; j < kMassLoads; ++j) {
            const int i = min(gi * kGroupVecs + lane + j * kWave, nvec - 1); // clamped: a duplicate is loaded but not added
            wp[j] = rs_ld16<NT>(pv + i);
            if (HAS_Q) wq[j] = rs_ld16_a4<NT>(qv + i);
        }
    };
    auto consume = [&](int gi, const uint4 (&wp)[kMassLoads], const uint4 (&wq)[kMassLoads]) {
#pragma unroll
        for (int j = 0; j < kMassLoads; ++j) {
            if (gi * kGroupVecs + lane + j * kWave < nvec) {
                float xp[NE], xq[NE];
                E::unpack(wp[j], xp);
                if (HAS_Q) E::unpack(wq[j], xq);
#pragma unroll
                for (int k = 0; k < NE; ++k)
                    acc[k & 3] += resid(xp[k], HAS_Q ? xq[k] : 0.f, HAS_Q, d.nref_p, d.inv_p, d.nref_q, d.inv_q);
            }
        }
    };
    if (groups > 0) issue(0, ap, aq);
    for (int gi = 0; gi < groups; gi += 2) {
        if (gi + 1 < groups) issue(gi + 1, bp, bq);
        consume(gi, ap, aq);
        if (gi + 2 < groups) issue(gi + 2, ap, aq);
        if (gi + 1 < groups) consume(gi + 1, bp, bq);
    }
    // scalars: the head, and whatever follows the vectors
    const int ntail = n - head - nvec * NE;
    for (int k = lane; k < head + ntail; k += kWave) {
        const int e = k < head ? k : nvec * NE + k;
        const float xp = E::load1(target, p0 + e);
        const float xq = HAS_Q ? E::load1(draft, q0 + e) : 0.f;
        acc[0] += resid(xp, xq, HAS_Q, d.nref_p, d.inv_p, d.nref_q, d.inv_q);
    }
    return wave_sum_dpp(((double)acc[0] + (double)acc[1]) + ((double)acc[2] + (double)acc[3]));
}

template <int DT, bool NT>
__device__ __forceinline__ double wave_chunk_mass(const void *draft, const void *target, int V,
                                                  const ResampleDesc &d, bool has_q, int e0, int e1, int lane)
{
    return has_q ? wave_chunk_mass_of<DT, NT, true>(draft, target, V, d, e0, e1, lane)
                 : wave_chunk_mass_of<DT, NT, false>(draft, target, V, d, e0, e1, lane);
}

constexpr int kRsWaves = kRsThreads / kWave;

template <int DT>
__global__ __launch_bounds__(kRsThreads) void resample_mass_kernel(BatchView bv,
                                                                   const void *__restrict__ draft,
                                                                   const void *__restrict__ target,
                                                                   const ResampleDesc *__restrict__ desc,
                                                                   int n_chunks, int chunk,
                                                                   double *__restrict__ mass)
{
    const int groups = (n_chunks + kRsWaves - 1) / kRsWaves;
    const int b = blockIdx.x / groups;
    const int c = (blockIdx.x - b * groups) * kRsWaves + threadIdx.x / kWave;
    if (c >= n_chunks) return;
    const ResampleDesc d = desc[b];
    const int e0 = c * chunk, e1 = min(bv.V, e0 + chunk);
    const double m = wave_chunk_mass<DT, true>(draft, target, bv.V, d, d.qrow >= 0, e0, e1, threadIdx.x % kWave);
    if (threadIdx.x % kWave == 0) mass[(int64_t)b * kMaxResampleChunks + c] = m;
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ double wave_inclusive_scan(double v, int)
{
    return wave_inclusive_scan_dpp(v);
}

constexpr int kPickRun = 16; // elements a thread keeps in registers in the pick pass

// Pick a token from the chunk masses of one row (pair): the first kRsThreads threads of a
// workgroup, all of them, with sh_mass[0..n_chunks) in LDS.  Returns the token in thread 0.
//   1. every wave scans the <= 64 chunk masses (shuffles): R, tau = u' R, the chunk holding tau
//   2. each thread takes a contiguous run of that chunk in vocabulary order, sums it in binary64;
//      wave scan + one LDS exchange give every thread its exclusive prefix
//   3. the thread whose interval holds tau walks its run (still in registers) to the token
// Barriers inside: any other thread of the workgroup must have exited before.
// chunk_ref (LDS, optional): the masses are in units of 2^row_ref, but the elements of chunk c are
// to be exponentiated relative to chunk_ref[c] (the caller summed them that way); the search
// inside the chunk is then done in the chunk's own units.
template <int DT>
__device__ __forceinline__ int pick_token(int V, const void *__restrict__ draft,
                                          const void *__restrict__ target, const ResampleDesc &d,
                                          double *sh_mass, int n_chunks, int chunk, uint32_t &flags,
                                          const float *chunk_ref = nullptr, float row_ref = 0.0f,
                                          const Trace tr = Trace{nullptr})
{
    using E = Elem<DT>;
    constexpr int WAVES = kRsWaves;
    __shared__ double sh_wave[WAVES];
    __shared__ int sh_tok, sh_lastw[WAVES];
    const int tid = threadIdx.x;
    const int wave = tid / kWave, lane = tid % kWave;
    bool has_q = d.qrow >= 0;
    flags = d.flags;

    if (tid == 0) sh_tok = 0x7fffffff;
    __syncthreads();
    double m = lane < n_chunks ? sh_mass[lane] : 0.0;
    double incl = wave_inclusive_scan(m, lane);
    double R = wave_read_lane(incl, kWave - 1);
    // A residual whose mass is below kResidualFloor means p_n and q_n agree to within that distance:
    // the correction is then drawn from p_n itself (a threshold, so that the decision does not hang on
    // rounding noise in a mass that is zero mathematically).  Without a draft row there is no
    // residual, and only a row without any mass (or with a NaN) falls back.
    if ((has_q ? !(R >= kResidualFloor) : !(R > 0.0)) || !(R < INFINITY)) {
        // draw from p_n instead and say so
        flags |= SPECKV_FLAG_FALLBACK;
        has_q = false;
        __syncthreads(); // every wave has read the old masses
        for (int c = wave; c < n_chunks; c += WAVES) {
            const int e0 = c * chunk, e1 = min(V, e0 + chunk);
            const double mc = wave_chunk_mass<DT, false>(draft, target, V, d, false, e0, e1, lane);
            if (lane == 0) sh_mass[c] = mc;
        }
        __syncthreads();
        m = lane < n_chunks ? sh_mass[lane] : 0.0;
        incl = wave_inclusive_scan(m, lane);
        R = wave_read_lane(incl, kWave - 1);
    }
    const double tau = d.u2 * R;
    // smallest chunk whose inclusive prefix exceeds tau; else (rounding, or R not a number) the last
    // chunk that has mass; else the last chunk
    const uint64_t over = __ballot(lane < n_chunks && incl > tau);
    const uint64_t pos = __ballot(lane < n_chunks && m > 0.0);
    int cs;
    if (over)
        cs = __ffsll((unsigned long long)over) - 1;
    else if (pos)
        cs = 63 - __clzll((unsigned long long)pos);
    else
        cs = n_chunks - 1;
    double base = cs ? wave_read_lane(incl, cs - 1) : 0.0;
    double tau_c = tau; // threshold and prefix in the units the chunk's elements are computed in
    float nref_p = d.nref_p;
    if (chunk_ref) {
        const float rc = chunk_ref[cs];
        nref_p = -rc;
        tau_c = ldexp(tau - base, (int)fminf(fmaxf(row_ref - rc, 0.0f), 4000.0f));
        base = 0.0;
    }
    const int e0 = cs * chunk, e1 = min(V, e0 + chunk);
    const int64_t p0 = d.prow * (int64_t)V;
    const int64_t q0 = (has_q ? d.qrow : 0) * (int64_t)V;
    tr.mark(6, tid == 0);
    // each thread owns a contiguous run of the chunk, in vocabulary order
    const int per = (chunk + kRsThreads - 1) / kRsThreads;
    const int lo = min(e1, e0 + tid * per), hi = min(e1, lo + per);
    double local = 0.0;
    int last_pos = -1;
    float r[kPickRun];
    if (per <= kPickRun) {
        float xp[kPickRun], xq[kPickRun];
        // a full run that starts on a 16-byte boundary in both rows is fetched with vector loads
        const char *pp = static_cast<const char *>(target) + (p0 + lo) * E::BYTES;
        const char *qp = static_cast<const char *>(draft) + (q0 + lo) * E::BYTES;
        // (runs are `per` elements long; elements of a vector beyond the run are loaded but not used)
        const bool vec = per % E::NE == 0 && lo + per <= hi && (reinterpret_cast<uintptr_t>(pp) & 15) == 0 &&
                         (!has_q || (reinterpret_cast<uintptr_t>(qp) & 15) == 0);
        if (vec) {
#pragma unroll
            for (int j = 0; j < kPickRun / E::NE; ++j) {
                if (j * E::NE < per) {
                    E::unpack(*reinterpret_cast<const uint4 *>(pp + 16 * j), xp + j * E::NE);
                    if (has_q) E::unpack(*reinterpret_cast<const uint4 *>(qp + 16 * j), xq + j * E::NE);
                } else {
#pragma unroll
                    for (int k = 0; k < E::NE; ++k) xp[j * E::NE + k] = xq[j * E::NE + k] = 0.f;
                }
            }
            if (!has_q) {
#pragma unroll
                for (int k = 0; k < kPickRun; ++k) xq[k] = 0.f;
            }
        } else {
#pragma unroll
            for (int k = 0; k < kPickRun; ++k) xp[k] = (lo + k < hi) ? E::load1(target, p0 + lo + k) : 0.f;
#pragma unroll
            for (int k = 0; k < kPickRun; ++k) xq[k] = (has_q && lo + k < hi) ? E::load1(draft, q0 + lo + k) : 0.f;
        }
#pragma unroll
        for (int k = 0; k < kPickRun; ++k) {
            r[k] = (lo + k < hi) ? resid(xp[k], xq[k], has_q, nref_p, d.inv_p, d.nref_q, d.inv_q) : 0.f;
            local += (double)r[k];
            if (r[k] > 0.f) last_pos = lo + k;
        }
    } else { // very large vocabularies: runs too long for registers, recomputed when walked
        for (int e = lo; e < hi; ++e) {
            const float xp = E::load1(target, p0 + e);
            const float xq = has_q ? E::load1(draft, q0 + e) : 0.f;
            const float rr = resid(xp, xq, has_q, nref_p, d.inv_p, d.nref_q, d.inv_q);
            local += (double)rr;
            if (rr > 0.f) last_pos = e;
        }
    }
    tr.mark(7, tid == 0);
    // exclusive prefix of the per-thread sums: scan inside the wave, then add the earlier waves
    const double wincl = wave_inclusive_scan(local, lane);
    double wprev = __shfl_up(wincl, 1, kWave); // the left neighbour's inclusive value, bit for bit
    if (lane == 0) wprev = 0.0;
    if (lane == kWave - 1) sh_wave[wave] = wincl;
    // last position of the chunk with mass (for the rounding fall-back): reduced inside the wave first;
    // an atomic per thread on one LDS word would serialise 256 ways
    const int wlast = wave_max_int_dpp(last_pos);
    if (lane == 0) sh_lastw[wave] = wlast;
    __syncthreads();
    tr.mark(8, tid == 0);
    double before = base;
    for (int w = 0; w < wave; ++w) before += sh_wave[w];
    // [prev_incl, t_incl) tile the chunk without gaps: each bound is computed by one expression
    const double t_incl = before + wincl;
    const double prev_incl = before + wprev;
    if (prev_incl <= tau_c && tau_c < t_incl) {
        // the threshold falls inside this thread's run: walk it
        double C = prev_incl;
        int found = -1;
        if (per <= kPickRun) {
#pragma unroll
            for (int k = 0; k < kPickRun; ++k) {
                C += (double)r[k];
                if (found < 0 && lo + k < hi && C > tau_c) found = lo + k;
            }
        } else {
            for (int e = lo; e < hi && found < 0; ++e) {
                const float xp = E::load1(target, p0 + e);
                const float xq = has_q ? E::load1(draft, q0 + e) : 0.f;
                C += (double)resid(xp, xq, has_q, nref_p, d.inv_p, d.nref_q, d.inv_q);
                if (C > tau_c) found = e;
            }
        }
        if (found < 0) found = last_pos;
        atomicMin(&sh_tok, found);
    }
    __syncthreads();
    tr.mark(9, tid == 0);
    int y = sh_tok;
    if (y == 0x7fffffff || y < 0) {
        int sh_last = -1;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sh_last = max(sh_last, sh_lastw[w]);
        y = sh_last >= 0 ? sh_last : min(max(e0, 0), V - 1);
    }
    return y;
}

// The same for the extra token of sequence b in a verification step: stores the token behind the
// accepted prefix, the token count and the sequence's flags.
template <int DT>
__device__ __forceinline__ void pick_sequence(const BatchView &bv, const void *__restrict__ draft,
                                              const void *__restrict__ target, const ResampleDesc &d,
                                              double *sh_mass, int n_chunks, int chunk, int b,
                                              int32_t *__restrict__ tokens, int32_t *__restrict__ num_tokens,
                                              uint32_t *__restrict__ row_flags, const Trace tr = Trace{nullptr})
{
    uint32_t flags;
    const int y = pick_token<DT>(bv.V, draft, target, d, sh_mass, n_chunks, chunk, flags, nullptr, 0.0f, tr);
    if (threadIdx.x == 0) {
        tokens[(int64_t)b * (bv.gamma_max + 1) + d.n] = y;
        num_tokens[b] = d.n + 1;
        if (row_flags) row_flags[b] = flags;
    }
}


template <int DT>
__global__ __launch_bounds__(kRsThreads) void resample_pick_kernel(
    BatchView bv, const void *__restrict__ draft, const void *__restrict__ target,
    const ResampleDesc *__restrict__ desc, const double *__restrict__ mass, int n_chunks, int chunk,
    int32_t *__restrict__ tokens, int32_t *__restrict__ num_tokens, uint32_t *__restrict__ row_flags)
{
    __shared__ double sh_mass[kMaxResampleChunks];
    const int b = blockIdx.x;
    const ResampleDesc d = desc[b];
    if (threadIdx.x < n_chunks) sh_mass[threadIdx.x] = mass[(int64_t)b * kMaxResampleChunks + threadIdx.x];
    __syncthreads();
    pick_sequence<DT>(bv, draft, target, d, sh_mass, n_chunks, chunk, b, tokens, num_tokens, row_flags);
}

// ---- the whole tail of a step, one workgroup per sequence ---------------------------------------
// For callers that hand over a whole step (speckv_step).  Wave 0 runs the accept scan of Section 3.1
// and leaves the resample descriptor in LDS; wave 1 forms the signals of Section 4.2 and the
// controller's decision of Section 4.3; then all waves sum the residual over the chunks of
// position n, each taking the next chunk when it is free; then the first four waves pick the
// token.  Nothing crosses workgroups, so no counters in memory, no coherent accesses and no further
// launch: one launch replaces step_epilogue + resample_mass + resample_pick with identical results.
// With out.H == NULL the kernel does the accept scan and the resample pass only (speckv_verify after
// speckv_signals: partials_d then holds the finished draft-row statistics, split_d = 1).
// A workgroup streams its sequence's two rows alone, so the launch uses the whole chip only when
// the batch has at least as many sequences as the chip has compute units.
// Threads per workgroup: with about one sequence per compute unit, 16 waves stream the sequence's
// rows fastest; with several sequences per compute unit, 8 waves let two workgroups share a unit,
// so that one streams while the other is in its latency-bound accept scan or pick (measured:
// 1024 threads 29 us vs 34 us at B = 256; 512 threads 118 us vs 129 us at B = 1024).
constexpr int kComputeUnits = 256;

template <int DT, int THREADS>
__global__ __launch_bounds__(THREADS) void step_tail_kernel(
    BatchView bv, AcceptArgs aa, const RowStat *__restrict__ partials_d, int split_d,
    const RowStat *__restrict__ partials_t, int split_t, RowStat *__restrict__ stat_d, RowStat *__restrict__ stat_t,
    MlpView m, int mode, const uint8_t *__restrict__ comp, StepOut out, int n_chunks, int chunk,
    int32_t *__restrict__ num_tokens, uint32_t *__restrict__ row_flags, unsigned long long *__restrict__ trace)
{
    // measurement only, usually null: clock readings of thread 0 along the way (see speckv_trace)
    const Trace tr{trace ? trace + kTraceSlots * (size_t)blockIdx.x : nullptr};
    tr.mark(0, threadIdx.x == 0);
    constexpr int kTailWaves = THREADS / kWave;
    __shared__ MlpShared shm;
    __shared__ ResampleDesc sh_desc;
    __shared__ double sh_mass[kMaxResampleChunks];
    __shared__ int sh_next; // next chunk of the mass pass to hand out
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int b = blockIdx.x;
    // Wave 0 runs the accept scan; the resample pass of all waves waits for its descriptor.  Wave 1
    // forms the signals and decides gamma on its own (it stages the controller weights in LDS for
    // itself): after the barrier, beside the mass pass of the other waves -- chunks are handed out on
    // request, so a wave that joins late simply takes fewer of them, and nobody waits at the barrier
    // for it -- except in a batch of one with a short mass pass, where it runs beside the accept scan.
    const bool whole_step = out.H != nullptr; // else: accept scan and resample only (speckv_verify)
    const int i = lane % kGroup;
    const bool live = lane < kGroup;
    // Measured: after the barrier is better from two sequences up whatever the length of the mass pass
    // (V = 32000: 23.1 -> 22.0 us per step at B = 64, 17.7 -> 17.1 at B = 2: wave 1's stores no longer
    // hold the barrier); only a batch of one, whose single workgroup has the chip to itself and a
    // mass pass of a microsecond, is 1.9 us faster with the controller in front.
    const bool controller_late = n_chunks > kTailWaves || gridDim.x > 1;
    auto signals_and_controller = [&]() {
        const int g = batch_gamma(bv, b);
        const int64_t drow0 = batch_draft_row0(bv, b);
        const bool active = live && i < g;
        stage_mlp(shm, m, lane, kWave);
        double h = 0.0, c = 0.0;
        float a[4];
        if (active) {
            const int64_t r = drow0 + i;
            const RowStat sq = merge_partials(partials_d + r * split_d, split_d);
            stat_d[r] = sq;
            row_signals(sq, h, c);
            out.H[r] = (float)h;
            out.conf[r] = (float)c;
            if (out.argmax) out.argmax[r] = sq.argmax;
        }
        sequence_aggregates(active, h, c, g, a);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) out.agg[4 * (int64_t)b + k] = a[k];
        }
        // the weights were written by this wave's own lanes: once its LDS writes have completed
        // (the fence waits for them) every lane of the wave may read them
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
        const float h0 = __shfl((float)h, 0, kGroup), c0 = __shfl((float)c, 0, kGroup);
        double x[7];
        controller_input(mode, h0, c0, a, comp[b], x);
        controller_decide(shm, m, x, lane % kMlpLanes, lane < kMlpLanes, b, out.gamma_next, out.scores);
    };
    if (tid == kWave) sh_next = 0;
    // What wave 0 stores to memory it stores after the barrier, beside the mass pass: a barrier waits
    // until the stores before it are acknowledged, about a microsecond that every wave would spend idle.
    int acc_g = 0;
    int32_t acc_tok = -1;
    int64_t acc_trow = 0;
    bool acc_lt = false;
    RowStat sp;
    sp.S = 1.0; sp.T = 0.0; sp.ref = 0.0f; sp.vmax = 0.0f; sp.argmax = 0; sp.pad = 0;
    if (wave == 0) {
        const int g = batch_gamma(bv, b);
        const int64_t drow0 = batch_draft_row0(bv, b);
        RowStat sq;
        sq = sp;
        TokenLogits tl;
        const int64_t trow = drow0 + b + i;
        if (split_t <= 2 && split_d <= 2) {
            // Everything that depends on no other load goes out first -- the token and the (at most
            // two) chunk statistics of this lane's target row and draft row -- then the two logits
            // that need the token: two memory round trips in all.  Merged as merge_partials merges.
            const bool lt = live && i <= g, ld = live && i < g;
            const int32_t tok = ld ? aa.draft_tokens[drow0 + i] : -1;
            const RowStat *pt = partials_t + trow * split_t, *pd = partials_d + (drow0 + i) * split_d;
            RowStat t0 = sp, t1 = sp, d0 = sp, d1 = sp;
            if (lt) t0 = pt[0];
            if (lt && split_t == 2) t1 = pt[1];
            if (ld) d0 = pd[0];
            if (ld && split_d == 2) d1 = pd[1];
            tl = gather_token_logits(bv, aa, live, b, i, g, drow0, tok);
            if (lt) {
                sp = t0;
                if (split_t == 2) merge_stat(sp, t1);
            }
            if (ld) {
                sq = d0;
                if (split_d == 2) merge_stat(sq, d1);
            }
        } else {
            tl = gather_token_logits(bv, aa, live, b, i, g, drow0); // in flight during the merges
            if (live && i <= g) sp = merge_partials(partials_t + trow * split_t, split_t);
            if (live && i < g) sq = merge_partials(partials_d + (drow0 + i) * split_d, split_d);
        }
        const Philox4 rnd = accept_block(bv, aa, b, i); // needs no data
        tr.mark(1, tid == 0);
        accept_sequence<true>(bv, aa, live, b, i, g, drow0, sp, sq, tl, rnd, &sh_desc);
        tr.mark(2, tid == 0);
        acc_g = g; acc_tok = tl.tok; acc_trow = trow; acc_lt = live && i <= g;
    } else if (wave == 1 && whole_step && !controller_late) {
        signals_and_controller();
    }
    __syncthreads(); // the descriptor is in LDS
    tr.mark(3, tid == 0);
    if (wave == 1 && whole_step && controller_late) signals_and_controller();
    const ResampleDesc d = sh_desc;
    if (wave == 0) {
        accept_store(bv, aa, live, b, i, acc_g, d.n, acc_tok, lane == 0, d);
        if (acc_lt) stat_t[acc_trow] = sp;
    }
    // A wave takes the next chunk whenever it is free (an LDS counter): waves that are served faster
    // by the memory system take more chunks, so that all of them finish together.  Which wave sums a
    // chunk does not change the chunk's mass.  The loop holds no branch that differs between lanes:
    // all 64 lanes of the wave add one to the counter (so it advances by 64 per request, and whatever
    // order the lanes are served in, each reads a value inside the wave's own block of 64) and every
    // lane stores the same mass.  A wave asks at most n_chunks + 1 times: each earlier answer was a
    // chunk of its own.
    for (int asked = 0; asked <= n_chunks; ++asked) {
        const int mine = atomicAdd(&sh_next, 1);
        const int ch = __builtin_amdgcn_readfirstlane(mine) >> 6;
        if (ch >= n_chunks) break;
        const int e0 = ch * chunk, e1 = min(bv.V, e0 + chunk);
        sh_mass[ch] = wave_chunk_mass<DT, true>(aa.draft, aa.target, bv.V, d, d.qrow >= 0, e0, e1, lane);
    }
    tr.mark(16 + wave, lane == 0);
    tr.mark(4, tid == 0);
    __syncthreads();
    tr.mark(5, tid == 0);
    if (tid >= kRsThreads) return;
    pick_sequence<DT>(bv, aa.draft, aa.target, d, sh_mass, n_chunks, chunk, b, aa.tokens, num_tokens, row_flags, tr);
    tr.mark(10, tid == 0);
}

hipError_t launch_step_tail(const BatchView &bv, const AcceptArgs &aa, speckv_dtype dtype, const RowStat *partials_d,
                            int split_d, const RowStat *partials_t, int split_t, RowStat *stat_d, RowStat *stat_t,
                            const speckv_mlp &mlp, int mode, const uint8_t *comp, float *H, float *conf,
                            int32_t *argmax, float *agg, int32_t *gamma_next, float *scores, int32_t *num_tokens,
                            uint32_t *row_flags, unsigned long long *trace, int tail_threads, hipStream_t stream)
{
    const ResampleGeom rg = resample_geom(bv.V);
    const MlpView m = mlp_view(mlp);
    const StepOut out{H, conf, argmax, agg, gamma_next, scores};
    // tail_threads: 0 = by batch size (see above), else 512 or 1024
    const int th = tail_threads ? tail_threads : (bv.B >= 2 * kComputeUnits ? 512 : 1024);
#define SPECKV_TAIL(DTV, TH)                                                                       \
    if (dtype == DTV && th == TH)                                                                  \
        return launch((step_tail_kernel<DTV, TH>), dim3(bv.B), dim3(TH), stream, bv, aa, partials_d, split_d,    \
                      partials_t, split_t, stat_d, stat_t, m, mode, comp, out, rg.n_chunks, rg.chunk, num_tokens,  \
                      row_flags, trace);
#define SPECKV_DT(DTV) SPECKV_TAIL(DTV, 256) SPECKV_TAIL(DTV, 512) SPECKV_TAIL(DTV, 1024)
    SPECKV_DT(SPECKV_F32) SPECKV_DT(SPECKV_F16) SPECKV_DT(SPECKV_BF16)
#undef SPECKV_DT
#undef SPECKV_TAIL
    return hipErrorInvalidValue;
}

// ---- token proposal on the draft side ---------------------------------------------------------------
// One token per row of logits, drawn from softmax(row) by the same inverse-CDF search (the draft
// model's sampling step, which precedes verification in Section 3.1).  One workgroup per row and
// one pass over the row from HBM: a wave per chunk sums 2^(x log2e - ref) with the running
// reference of the statistics kernel; chunk sums are rebased to the row's reference by exact
// power-of-two shifts; the pick then searches inside the chosen chunk in that chunk's units, where
// the elements are recomputed against the chunk's final reference.
// u = w0 * 2^-32 of Philox block (sequence, position, step, 1).
// Workgroup size: 16 waves when there is about one row per compute unit, 8 waves when rows queue up.

template <int DT, int THREADS, int kLoads>
__global__ __launch_bounds__(THREADS) void sample_rows_kernel(BatchView bv, const void *__restrict__ logits,
                                                                     int n_chunks, int chunk, uint32_t key0,
                                                                     uint32_t key1, uint32_t step, uint32_t pos0,
                                                                     int32_t *__restrict__ tokens,
                                                                     float *__restrict__ prob,
                                                                     uint32_t *__restrict__ row_flags)
{
    constexpr int kSampleWaves = THREADS / kWave;
    __shared__ double sh_mass[kMaxResampleChunks];
    __shared__ float sh_ref[kMaxResampleChunks];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int64_t row = blockIdx.x;
    if (bv.row_off && row >= bv.row_off[bv.B]) return; // ragged batch: the launch covers B * gamma_max rows
    const int b = seq_of_row(bv, row, 0);
    const int i = (int)(row - batch_draft_row0(bv, b));
    const int V = bv.V;
    const int64_t row_elem0 = row * (int64_t)V;
    using E = Elem<DT>;
    constexpr int NE = E::NE;
    // One sweep per chunk with the running reference of the statistics kernel (speckv_accum.h): no
    // maximum has to be known beforehand, nothing is held in registers between sweeps, and the
    // kernel's register count leaves room for eight waves per SIMD.  A chunk's sum comes out
    // relative to the reference the wave ended the chunk with, which is what the pick is given.
    // Two 16-byte loads per lane and group, the next group in flight while one is exponentiated.
    constexpr int kGroupVecs = kLoads * kWave;
    for (int c = wave; c < n_chunks; c += kSampleWaves) {
        const int e0 = c * chunk, n = max(0, min(V, e0 + chunk) - e0);
        const uintptr_t addr = reinterpret_cast<uintptr_t>(logits) + (uintptr_t)(row_elem0 + e0) * E::BYTES;
        const int head = min((int)(((16 - (addr & 15)) & 15) / E::BYTES), n);
        const int nvec = (n - head) / NE;
        const uint4 *pv = reinterpret_cast<const uint4 *>(static_cast<const char *>(logits) +
                                                          (row_elem0 + e0 + head) * E::BYTES);
        LaneAcc a;
        lane_init(a);
        const int groups = (nvec + kGroupVecs - 1) / kGroupVecs;
        uint4 wa[kLoads], wb[kLoads];
        auto issue = [&](int gi, uint4 (&w)[kLoads]) {
#pragma unroll
            for (int j = 0; j < kLoads; ++j) // clamped: a duplicate is loaded and then replaced by -inf
                w[j] = rs_ld16<true>(pv + min(gi * kGroupVecs + lane + j * kWave, nvec - 1));
        };
        auto consume = [&](int gi, const uint4 (&w)[kLoads]) {
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                float x[NE];
                E::unpack(w[j], x);
                if (gi * kGroupVecs + lane + j * kWave >= nvec) {
#pragma unroll
                    for (int k = 0; k < NE; ++k) x[k] = -INFINITY;
                }
                accum<NE, false, false>(a, x); // every lane of the wave: the reference is the wave's
            }
        };
        if (groups > 0) issue(0, wa);
        for (int gi = 0; gi < groups; gi += 2) {
            if (gi + 1 < groups) issue(gi + 1, wb);
            consume(gi, wa);
            if (gi + 2 < groups) issue(gi + 2, wa);
            if (gi + 1 < groups) consume(gi + 1, wb);
        }
        // unaligned elements in front of and behind the vectors: fewer than 2 * NE <= 64, one per lane
        const int ends = head + (n - head - nvec * NE);
        if (ends > 0) {
            const float xe[1] = {lane < ends ? E::load1(logits, row_elem0 + e0 + (lane < head ? lane : nvec * NE + lane))
                                             : -INFINITY};
            accum<1, false, false>(a, xe);
        }
        const double S = wave_sum_dpp(((double)a.s[0] + (double)a.s[1]) + ((double)a.s[2] + (double)a.s[3]));
        // every lane holds the same values; a.ref is -inf when the chunk held nothing finite
        sh_ref[c] = a.ref;
        sh_mass[c] = S;
    }
    __syncthreads();
    if (tid >= kRsThreads) return;
    // chunk sums in units of the row's reference (every wave computes the same values)
    const float rc = lane < n_chunks ? sh_ref[lane] : -INFINITY;
    const float row_ref = wave_max(rc);
    const double Sc = lane < n_chunks ? sh_mass[lane] : 0.0;
    // a chunk without a finite value adds nothing, unless it held a NaN (its sum is then NaN)
    const double mine = rc > -INFINITY ? ldexp(Sc, (int)fmaxf(rc - row_ref, -4000.0f)) : (Sc != Sc ? Sc : 0.0);
    __syncthreads(); // all four waves have read the chunk-relative sums
    if (wave == 0 && lane < n_chunks) sh_mass[lane] = mine;
    const Philox4 rnd = philox4x32_10(bv.seq_base + (uint32_t)b, pos0 + (uint32_t)i, step, 1u, key0, key1);
    ResampleDesc d;
    d.prow = row; d.qrow = -1;
    d.u2 = (double)rnd.w[0] * 0x1.0p-32;
    d.nref_p = 0.0f; d.inv_p = 1.0f; d.nref_q = 0.0f; d.inv_q = 0.0f;
    d.n = 0; d.flags = 0;
    d.pad[0] = d.pad[1] = d.pad[2] = d.pad[3] = 0;
    uint32_t pick_flags;
    const int y = pick_token<DT>(V, logits, logits, d, sh_mass, n_chunks, chunk, pick_flags, sh_ref, row_ref);
    if (tid == 0) {
        double S = 0.0;
        for (int c = 0; c < n_chunks; ++c) S += sh_mass[c];
        const bool bad = !(S > 0.0) || !(S < INFINITY) || !(row_ref < INFINITY);
        tokens[row] = y;
        if (prob) {
            const float xt = Elem<DT>::load1(logits, row_elem0 + y);
            prob[row] = (float)(exp2((double)fmaf(xt, L2E_F, -row_ref)) / S);
        }
        if (row_flags) row_flags[row] = bad ? SPECKV_FLAG_NONFINITE : 0u;
    }
}

// Chunks of the proposal kernel: as long as a wave's registers hold (8 KB: 4096 16-bit or 2048
// binary32 elements), at most 64 of them; longer ones (very large vocabularies) are swept from memory.
static ResampleGeom sample_geom(int V, speckv_dtype dtype)
{
    const int cap = dtype == SPECKV_F32 ? 2048 : 4096;
    int n = (V + cap - 1) / cap;
    if (n < 1) n = 1;
    if (n > kMaxResampleChunks) n = kMaxResampleChunks;
    int chunk = (V + n - 1) / n;
    chunk = (chunk + 63) & ~63;
    n = (V + chunk - 1) / chunk;
    return {n, chunk};
}

hipError_t launch_sample_rows(const BatchView &bv, const void *logits, speckv_dtype dtype, int64_t rows_bound,
                              uint64_t seed, uint32_t step, uint32_t pos0, int32_t *tokens, float *prob,
                              uint32_t *row_flags, int threads, int loads, hipStream_t stream)
{
    const ResampleGeom rg = sample_geom(bv.V, dtype);
    if (rows_bound <= 0 || rows_bound > 0x7fffffffLL) return hipErrorInvalidValue;
    // threads: 0 = by the number of rows (see above), else 512 or 1024; loads: 16-byte loads per lane and group
    const int th = threads ? threads : (rows_bound >= 2 * kComputeUnits ? 512 : 1024);
    if (!loads) loads = th == 512 ? 4 : 2; // measured on 2048 rows of 128256 bf16: 512/4 and 1024/2 87 us, 512/2 90, 1024/4 98
#define SPECKV_SMP(DTV, TH, LD)                                                                    \
    if (dtype == DTV && th == TH && loads == LD)                                                   \
        return launch((sample_rows_kernel<DTV, TH, LD>), dim3((unsigned)rows_bound), dim3(TH), stream, bv, logits,  \
                      rg.n_chunks, rg.chunk, (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32), step, pos0,  \
                      tokens, prob, row_flags);
#define SPECKV_DT(DTV) SPECKV_SMP(DTV, 512, 2) SPECKV_SMP(DTV, 1024, 2) SPECKV_SMP(DTV, 512, 4) SPECKV_SMP(DTV, 1024, 4)
    SPECKV_DT(SPECKV_F32) SPECKV_DT(SPECKV_F16) SPECKV_DT(SPECKV_BF16)
#undef SPECKV_DT
#undef SPECKV_SMP
    return hipErrorInvalidValue;
}

hipError_t launch_resample_mass(const BatchView &bv, const void *draft, const void *target,
                                speckv_dtype dtype, const ResampleDesc *desc, double *mass,
                                hipStream_t stream)
{
    const ResampleGeom rg = resample_geom(bv.V);
    const int64_t blocks = (int64_t)bv.B * ((rg.n_chunks + kRsWaves - 1) / kRsWaves);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
#define SPECKV_DT(DTV)                                                                             \
    if (dtype == DTV) {                                                                            \
        return launch((resample_mass_kernel<DTV>), dim3((unsigned)blocks), dim3(kRsThreads), stream, bv,  \
                      draft, target, desc, rg.n_chunks, rg.chunk, mass);                          \
    }
    SPECKV_DT(SPECKV_F32) SPECKV_DT(SPECKV_F16) SPECKV_DT(SPECKV_BF16)
#undef SPECKV_DT
    return hipErrorInvalidValue;
}

hipError_t launch_resample_pick(const BatchView &bv, const void *draft, const void *target,
                                speckv_dtype dtype, const ResampleDesc *desc, const double *mass,
                                int32_t *tokens, int32_t *num_tokens, uint32_t *row_flags,
                                hipStream_t stream)
{
    const ResampleGeom rg = resample_geom(bv.V);
#define SPECKV_DT(DTV)                                                                             \
    if (dtype == DTV) {                                                                            \
        return launch((resample_pick_kernel<DTV>), dim3(bv.B), dim3(kRsThreads), stream, bv,    \
                           draft, target, desc, mass, rg.n_chunks, rg.chunk, tokens, num_tokens,   \
                           row_flags);\
    }
    SPECKV_DT(SPECKV_F32) SPECKV_DT(SPECKV_F16) SPECKV_DT(SPECKV_BF16)
#undef SPECKV_DT
    return hipErrorInvalidValue;
}

} // namespace speckv
