// The one extra token of a speculation step (Section 3.1: "correction or bonus prediction"),
// drawn as in the lossless scheme of the works cited in Section 2.1:
//     r(v) = max(0, p_n(v) - q_n(v))  if the draft at position n was rejected,
//     r(v) = p_gamma(v)               if every draft was accepted (bonus),
// token = smallest v with  sum_{w<=v} r(w) > u' * sum_w r(w).
//
// Two kernels.  resample_mass: one workgroup per (sequence, chunk of the row) sums r over the
// chunk (coalesced 16-byte loads, binary32 per element, binary64 across lanes).  resample_pick:
// one workgroup per sequence scans the chunk masses, finds the chunk holding the threshold,
// re-reads only that chunk in vocabulary order with a block-wide prefix sum in LDS and walks to the
// token.  Per-element values are computed by the same expression in both kernels.
#include "speckv_device.h"

namespace speckv {

constexpr int kRsThreads = 256;

// p(v) (or p(v) - q(v) clipped at 0) from raw logits with the row's reference and 1/S.
__device__ __forceinline__ float resid(float xp, float xq, bool has_q, float nref_p, float inv_p,
                                       float nref_q, float inv_q)
{
    const float p = exp2_hw(fmaf(xp, L2E_F, nref_p)) * inv_p;
    if (!has_q) return p;
    const float q = exp2_hw(fmaf(xq, L2E_F, nref_q)) * inv_q;
    return fmaxf(p - q, 0.0f);
}

template <int DT>
__device__ __forceinline__ double chunk_mass(const void *draft, const void *target, int V,
                                             const ResampleDesc &d, bool has_q, int e0, int e1, int tid)
{
    using E = Elem<DT>;
    constexpr int NE = E::NE;
    const int n = max(0, e1 - e0);
    const int64_t p0 = d.prow * (int64_t)V + e0;
    const int64_t q0 = (has_q ? d.qrow : 0) * (int64_t)V + e0;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(target) + (uintptr_t)p0 * E::BYTES;
    const uintptr_t qa = reinterpret_cast<uintptr_t>(draft) + (uintptr_t)q0 * E::BYTES;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    // vector path only when both rows share the same 16-byte phase; otherwise element loads
    const bool vec_ok = !has_q || ((pa & 15) == (qa & 15));
    int head = n, nvec = 0;
    if (vec_ok) {
        head = min((int)(((16 - (pa & 15)) & 15) / E::BYTES), n);
        nvec = (n - head) / NE;
    }
    // derived from the kernel arguments so that the loads stay in the global address space
    const uint4 *pv = reinterpret_cast<const uint4 *>(static_cast<const char *>(target) + (p0 + head) * E::BYTES);
    const uint4 *qv = reinterpret_cast<const uint4 *>(static_cast<const char *>(draft) + (q0 + head) * E::BYTES);
    for (int i = tid; i < nvec; i += kRsThreads) {
        float xp[NE], xq[NE];
        E::unpack(pv[i], xp);
        if (has_q) {
            E::unpack(qv[i], xq);
        } else {
#pragma unroll
            for (int k = 0; k < NE; ++k) xq[k] = 0.f;
        }
#pragma unroll
        for (int k = 0; k < NE; ++k)
            acc[k & 3] += resid(xp[k], xq[k], has_q, d.nref_p, d.inv_p, d.nref_q, d.inv_q);
    }
    // scalars: the head, and whatever follows the vectors
    const int ntail = n - head - nvec * NE;
    for (int k = tid; k < head + ntail; k += kRsThreads) {
        const int e = k < head ? k : nvec * NE + k;
        const float xp = E::load1(target, p0 + e);
        const float xq = has_q ? E::load1(draft, q0 + e) : 0.f;
        acc[0] += resid(xp, xq, has_q, d.nref_p, d.inv_p, d.nref_q, d.inv_q);
    }
    return ((double)acc[0] + (double)acc[1]) + ((double)acc[2] + (double)acc[3]);
}

// Sum over the workgroup; every thread gets the result.
__device__ __forceinline__ double block_sum(double v, double *sh /* kRsThreads / 64 + 1 */)
{
    v = wave_sum(v);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    __syncthreads(); // protect sh from the previous use
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kRsThreads / kWave; ++w) s += sh[w];
    return s;
}

template <int DT>
__global__ __launch_bounds__(kRsThreads) void resample_mass_kernel(BatchView bv,
                                                                   const void *__restrict__ draft,
                                                                   const void *__restrict__ target,
                                                                   const ResampleDesc *__restrict__ desc,
                                                                   int n_chunks, int chunk,
                                                                   double *__restrict__ mass)
{
    __shared__ double sh[kRsThreads / kWave];
    const int b = blockIdx.x / n_chunks;
    const int c = blockIdx.x - b * n_chunks;
    const ResampleDesc d = desc[b];
    const int e0 = c * chunk, e1 = min(bv.V, e0 + chunk);
    const double m = block_sum(chunk_mass<DT>(draft, target, bv.V, d, d.qrow >= 0, e0, e1, threadIdx.x), sh);
    if (threadIdx.x == 0) mass[(int64_t)b * kMaxResampleChunks + c] = m;
}

template <int DT>
__global__ __launch_bounds__(kRsThreads) void resample_pick_kernel(
    BatchView bv, const void *__restrict__ draft, const void *__restrict__ target,
    const ResampleDesc *__restrict__ desc, const double *__restrict__ mass, int n_chunks, int chunk,
    int32_t *__restrict__ tokens, int32_t *__restrict__ num_tokens, uint32_t *__restrict__ row_flags)
{
    using E = Elem<DT>;
    __shared__ double sh[kRsThreads / kWave];
    __shared__ double sh_mass[kMaxResampleChunks];
    __shared__ double sh_scan[kRsThreads];
    __shared__ int sh_chunk, sh_tok, sh_last;
    __shared__ double sh_base, sh_tau;
    const int b = blockIdx.x, tid = threadIdx.x, V = bv.V;
    ResampleDesc d = desc[b];
    bool has_q = d.qrow >= 0;
    uint32_t flags = d.flags;

    if (tid < n_chunks) sh_mass[tid] = mass[(int64_t)b * kMaxResampleChunks + tid];
    __syncthreads();
    double R = 0.0;
    for (int c = 0; c < n_chunks; ++c) R += sh_mass[c];
    if (!(R > 0.0) || !(R < INFINITY)) {
        // no residual mass (or not a number): draw from p_n instead and say so
        flags |= SPECKV_FLAG_FALLBACK;
        has_q = false;
        for (int c = 0; c < n_chunks; ++c) {
            const int e0 = c * chunk, e1 = min(V, e0 + chunk);
            const double m = block_sum(chunk_mass<DT>(draft, target, V, d, false, e0, e1, tid), sh);
            __syncthreads();
            if (tid == 0) sh_mass[c] = m;
        }
        __syncthreads();
        R = 0.0;
        for (int c = 0; c < n_chunks; ++c) R += sh_mass[c];
    }
    if (tid == 0) {
        const double tau = d.u2 * R;
        double base = 0.0;
        int cs = -1;
        for (int c = 0; c < n_chunks; ++c) {
            if (base + sh_mass[c] > tau) { cs = c; break; }
            base += sh_mass[c];
        }
        if (cs < 0) { // rounding, or R not a number: last chunk with mass, else the last chunk
            cs = n_chunks - 1;
            for (int c = n_chunks - 1; c >= 0; --c)
                if (sh_mass[c] > 0.0) { cs = c; break; }
            base = 0.0;
            for (int c = 0; c < cs; ++c) base += sh_mass[c];
        }
        sh_chunk = cs;
        sh_base = base;
        sh_tau = tau;
        sh_tok = 0x7fffffff;
        sh_last = -1;
    }
    __syncthreads();
    const int cs = sh_chunk;
    const double base = sh_base, tau = sh_tau;
    const int e0 = cs * chunk, e1 = min(V, e0 + chunk);
    // each thread owns a contiguous run of the chunk, in vocabulary order
    const int per = (chunk + kRsThreads - 1) / kRsThreads;
    const int lo = min(e1, e0 + tid * per), hi = min(e1, lo + per);
    const int64_t p0 = d.prow * (int64_t)V;
    const int64_t q0 = (has_q ? d.qrow : 0) * (int64_t)V;
    double local = 0.0;
    int last_pos = -1;
    for (int e = lo; e < hi; ++e) {
        const float xp = E::load1(target, p0 + e);
        const float xq = has_q ? E::load1(draft, q0 + e) : 0.f;
        const float r = resid(xp, xq, has_q, d.nref_p, d.inv_p, d.nref_q, d.inv_q);
        local += (double)r;
        if (r > 0.f) last_pos = e;
    }
    // inclusive scan of the per-thread sums (Hillis-Steele through LDS)
    sh_scan[tid] = local;
    __syncthreads();
    for (int o = 1; o < kRsThreads; o <<= 1) {
        const double add = tid >= o ? sh_scan[tid - o] : 0.0;
        __syncthreads();
        sh_scan[tid] += add;
        __syncthreads();
    }
    const double incl = base + sh_scan[tid];
    const double excl = base + (tid ? sh_scan[tid - 1] : 0.0);
    if (last_pos >= 0) atomicMax(&sh_last, last_pos);
    if (excl <= tau && tau < incl) {
        // the threshold falls inside this thread's run: walk it
        double C = excl;
        int found = -1;
        for (int e = lo; e < hi && found < 0; ++e) {
            const float xp = E::load1(target, p0 + e);
            const float xq = has_q ? E::load1(draft, q0 + e) : 0.f;
            C += (double)resid(xp, xq, has_q, d.nref_p, d.inv_p, d.nref_q, d.inv_q);
            if (C > tau) found = e;
        }
        if (found < 0) found = last_pos; // cannot happen: incl is this same sum
        atomicMin(&sh_tok, found);
    }
    __syncthreads();
    if (tid == 0) {
        int y = sh_tok;
        if (y == 0x7fffffff || y < 0) y = sh_last >= 0 ? sh_last : min(max(e0, 0), V - 1);
        tokens[(int64_t)b * (bv.gamma_max + 1) + d.n] = y;
        num_tokens[b] = d.n + 1;
        if (row_flags) row_flags[b] = flags;
    }
}

hipError_t launch_resample_mass(const BatchView &bv, const void *draft, const void *target,
                                speckv_dtype dtype, const ResampleDesc *desc, double *mass,
                                hipStream_t stream)
{
    const ResampleGeom rg = resample_geom(bv.V);
    const int64_t blocks = (int64_t)bv.B * rg.n_chunks;
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
