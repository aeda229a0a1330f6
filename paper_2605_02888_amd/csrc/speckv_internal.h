// Internal declarations shared by the HIP translation units of libspeckv.so.
// Nothing here is part of the C ABI (see include/speckv.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "speckv.h"

namespace speckv {

// log2(e).  Every vocabulary element is exponentiated as 2^(x * L2E_F - ref) with one binary32
// fused multiply-add feeding the hardware exp2; per-row quantities that must agree with that
// sum (max probability, q(t), p(t)) are formed from the same binary32 product.
constexpr float L2E_F = 1.44269504088896340736f;

// Softmax statistics of one vocabulary row, or of one chunk of a row.
//   S = sum_v 2^(x_v * log2e - ref),  T = sum_v 2^(x_v * log2e - ref) * (x_v * log2e - ref)
// ref is integer valued, so changing it rescales S and T by an exact power of two.
// Entropy in bits = log2 S - T / S; max probability = 2^(vmax * log2e - ref) / S.
struct alignas(16) RowStat {
    double S;
    double T;
    float ref;
    float vmax;     // largest logit of the row (exact, as binary32)
    int32_t argmax; // lowest index attaining vmax
    uint32_t pad;
};
static_assert(sizeof(RowStat) == 32, "RowStat layout");

// What the resample kernels need to know about one sequence (written by the accept kernel).
struct alignas(16) ResampleDesc {
    int64_t prow;  // target row of position n
    int64_t qrow;  // draft row of position n, or -1 for the bonus case (r = p)
    double u2;     // resample uniform in [0,1)
    float nref_p;  // -ref of the target row
    float inv_p;   // 1 / S of the target row
    float nref_q;
    float inv_q;
    int32_t n;     // accepted prefix length
    uint32_t flags;
    uint32_t pad[4];
};
static_assert(sizeof(ResampleDesc) == 64, "ResampleDesc layout");

constexpr int kMaxResampleChunks = 64;  // chunks of a row in the residual-mass pass
constexpr int kMaxStatsTargetWgs = 65536;

// Device-side view of speckv_batch.
struct BatchView {
    int32_t B, V, gamma_max, gamma_uniform;
    const int32_t *gamma;   // may be null
    const int64_t *row_off; // may be null
    uint32_t seq_base;
};

// Speculation length of sequence b.  A per-sequence value outside [1, gamma_max] is data the host
// cannot see: it is clamped here, so that every kernel indexes positions 0..gamma_max only and the
// accepted length stays inside the token row, and the accept scan reports it (SPECKV_FLAG_BAD_GAMMA).
__device__ __forceinline__ int batch_gamma(const BatchView &bv, int b)
{
    return bv.gamma ? min(max(bv.gamma[b], 1), bv.gamma_max) : bv.gamma_uniform;
}
__device__ __forceinline__ bool batch_gamma_clamped(const BatchView &bv, int b)
{
    return bv.gamma && (bv.gamma[b] < 1 || bv.gamma[b] > bv.gamma_max);
}
__device__ __forceinline__ int64_t batch_draft_row0(const BatchView &bv, int b)
{
    return bv.row_off ? bv.row_off[b] : (int64_t)b * bv.gamma_uniform;
}

// Workspace carving (host and device agree through these offsets).
struct WsLayout {
    size_t stat_d, stat_t, partial, partial_d, desc, mass, total;
};
inline WsLayout ws_layout(int64_t B, int64_t gamma_max)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    WsLayout L;
    size_t off = 0;
    L.stat_d = off; off = up(off + sizeof(RowStat) * (size_t)(B * gamma_max));
    L.stat_t = off; off = up(off + sizeof(RowStat) * (size_t)(B * (gamma_max + 1)));
    L.partial = off; off = up(off + sizeof(RowStat) * (size_t)(B * (gamma_max + 1) + kMaxStatsTargetWgs));
    // speckv_step keeps the draft rows' chunk statistics beside the target rows' (one launch)
    L.partial_d = off; off = up(off + sizeof(RowStat) * (size_t)(B * gamma_max + kMaxStatsTargetWgs));
    L.desc = off; off = up(off + sizeof(ResampleDesc) * (size_t)B);
    L.mass = off; off = up(off + sizeof(double) * (size_t)B * kMaxResampleChunks);
    L.total = off;
    return L;
}

// Chunking of a row for the residual-mass pass: n_chunks chunks of `chunk` elements.
struct ResampleGeom {
    int n_chunks;
    int chunk;
};
inline ResampleGeom resample_geom(int V)
{
    // chunks of about 2048 elements (at most 64 of them, so longer for vocabularies beyond 131072); a
    // row too short to give each of 16 waves such a chunk is cut into up to 16 shorter ones (no
    // shorter than 512 elements), so that every wave has work
    int n = (V + 2047) / 2048;
    if (n < 16) n = (V + 511) / 512 < 16 ? (V + 511) / 512 : 16;
    if (n < 1) n = 1;
    if (n > kMaxResampleChunks) n = kMaxResampleChunks;
    int chunk = (V + n - 1) / n;
    chunk = (chunk + 63) & ~63;
    n = (V + chunk - 1) / chunk;
    return {n, chunk};
}

// Launch parameters of the row-statistics kernel.
struct StatsLaunch {
    int threads; // 128 / 256 / 512
    int unroll;  // 16-byte loads in flight per lane: 2 / 4
    int split;   // chunks per row
    int chunk;   // elements per chunk (multiple of 64)
    int pipeline;    // 1: next tile's loads in flight while the current one is processed
    int nontemporal; // 1: nontemporal loads
    int want_argmax; // 1: resolve the lowest index of each chunk's maximum (else argmax = -1)
    int lds_pad;     // bytes of LDS a workgroup occupies beyond its own (bounds the workgroups per compute unit)
};

// Events for the next kernel launch on this thread (set by the ABI layer while profiling).  When
// set, the kernel is launched through hipExtLaunchKernelGGL, which stamps the two events with the
// dispatch's own begin and end times, so the measurement adds no barrier packets to the stream.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local LaunchEvents g_launch_events;

// ---- launchers (defined in the .hip files) -------------------------------------------------
// Everything the accept scan reads and writes besides the row statistics.
struct AcceptArgs {
    const void *draft;
    const void *target;
    int dtype;
    const int32_t *draft_tokens;
    uint32_t key0, key1, step;
    ResampleDesc *desc;
    int32_t *n_accepted;
    int32_t *tokens;
    float *accept_rate;
};

hipError_t launch_row_stats(const void *logits, speckv_dtype dtype, bool with_entropy, int V,
                            int64_t rows_bound, const int64_t *row_off, int B, int rows_extra_per_seq,
                            const StatsLaunch &sl, RowStat *partials, hipStream_t stream);

// Draft and target rows in one launch (default launch shape only: see row_stats_pair_supported).
bool row_stats_pair_supported(const StatsLaunch &sd, const StatsLaunch &st);
hipError_t launch_row_stats_pair(const void *draft, const void *target, speckv_dtype dtype, int V,
                                 int64_t rows_bound_d, int64_t rows_bound_t, const int64_t *row_off, int B,
                                 const StatsLaunch &sd, const StatsLaunch &st, int pos0_last, RowStat *partials_d,
                                 RowStat *partials_t, unsigned long long *trace, hipStream_t stream);

// signals + accept scan + controller of every sequence in one launch.
hipError_t launch_step_epilogue(const BatchView &bv, const AcceptArgs &aa, const RowStat *partials_d, int split_d,
                                const RowStat *partials_t, int split_t, RowStat *stat_d, RowStat *stat_t,
                                const speckv_mlp &mlp, int mode, const uint8_t *comp, float *H, float *conf,
                                int32_t *argmax, float *agg, int32_t *gamma_next, float *scores, bool greedy,
                                int32_t *num_tokens, uint32_t *row_flags, hipStream_t stream);

// The same plus the resample pass, one workgroup per sequence: the whole tail of a step in one launch.
hipError_t launch_step_tail(const BatchView &bv, const AcceptArgs &aa, speckv_dtype dtype, const RowStat *partials_d,
                            int split_d, const RowStat *partials_t, int split_t, RowStat *stat_d, RowStat *stat_t,
                            const speckv_mlp &mlp, int mode, const uint8_t *comp, float *H, float *conf,
                            int32_t *argmax, float *agg, int32_t *gamma_next, float *scores, int32_t *num_tokens,
                            uint32_t *row_flags, unsigned long long *trace, int tail_threads, hipStream_t stream);

hipError_t launch_signals_finalize(const BatchView &bv, const RowStat *partials, int split,
                                   RowStat *stat_d, float *H, float *conf, int32_t *argmax,
                                   float *agg, hipStream_t stream);

hipError_t launch_accept(const BatchView &bv, const void *draft, const void *target,
                         speckv_dtype dtype, const int32_t *draft_tokens, uint64_t seed,
                         uint32_t step, const RowStat *stat_d, const RowStat *partials_t, int split,
                         RowStat *stat_t, ResampleDesc *desc, int32_t *n_accepted, int32_t *tokens,
                         float *accept_rate, hipStream_t stream);

hipError_t launch_greedy_accept(const BatchView &bv, const int32_t *draft_tokens, const RowStat *partials_t,
                                int split, RowStat *stat_t, int32_t *n_accepted, int32_t *tokens,
                                int32_t *num_tokens, float *accept_rate, uint32_t *row_flags, hipStream_t stream);

hipError_t launch_resample_mass(const BatchView &bv, const void *draft, const void *target,
                                speckv_dtype dtype, const ResampleDesc *desc, double *mass,
                                hipStream_t stream);

hipError_t launch_resample_pick(const BatchView &bv, const void *draft, const void *target,
                                speckv_dtype dtype, const ResampleDesc *desc, const double *mass,
                                int32_t *tokens, int32_t *num_tokens, uint32_t *row_flags,
                                hipStream_t stream);

// One token per row of `logits`, drawn from softmax(row); rows laid out like the draft rows of bv.
hipError_t launch_sample_rows(const BatchView &bv, const void *logits, speckv_dtype dtype, int64_t rows_bound,
                              uint64_t seed, uint32_t step, uint32_t pos0, int32_t *tokens, float *prob,
                              uint32_t *row_flags, int threads, int loads, hipStream_t stream);

hipError_t launch_select_gamma(const BatchView &bv, const speckv_mlp &mlp, int mode, const float *H,
                               const float *conf, const float *agg, const uint8_t *comp,
                               int32_t *gamma_next, float *scores, hipStream_t stream);

hipError_t launch_row_offsets(const int32_t *gamma, int B, int64_t *row_off, hipStream_t stream);

hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, int max_blocks, hipStream_t stream);
hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t stream);

} // namespace speckv
