// Row statistics: one pass over logits, no materialised softmax.
//
// For every vocabulary row (or chunk of a row) the kernel produces
//     vmax = max_v x_v, argmax, S = sum_v 2^(x_v*log2e - ref), T = sum_v 2^(.)*(x_v*log2e - ref)
// from which the paper's per-position signals follow (Section 4.2):
//     entropy in bits  H = log2 S - T/S        (= -sum_v q log2 q)
//     confidence       c = 2^(vmax*log2e - ref) / S   (= max_v q(v))
// and, for the accept test, q(t) = 2^(x_t*log2e - ref) / S.
//
// Work decomposition: one workgroup per (row, chunk).  Each lane streams 16-byte vectors with two
// register buffers (the next tile is in flight while the current one is processed).  The 64 lanes
// of a wave share one integer-valued reference exponent `ref`: before a vector is exponentiated its
// maximum is compared with the wave's limit, and only when some lane exceeds it (a uniform branch,
// taken a few times per chunk) the wave raises the reference to ceil(largest value * log2e), which
// rescales every lane's sums by an exact power of two.  The limit sits kRefSlack above the
// reference, so t = x*log2e - ref <= kRefSlack for every term: nothing can overflow, and the
// dominant terms of a peaked row have |t| <= kRefSlack + 1, which keeps their products e*t
// accurate enough for the entropy -- there a small difference of terms of size |t| -- to come out
// right (a reference far below the row maximum would not: the binary32 rounding of a large t alone
// is then larger than the entropy).
// Steady state per element: one convert, half a max3, one fused multiply-add, one hardware exp2,
// one add and (draft rows only) one more fused multiply-add; the kernel issues close to one vector
// instruction per cycle and SIMD, so this count matters as much as the bytes.  A masked logit
// (-inf) makes 0 * (-inf) = NaN in the entropy sum; that is detected after the chunk and the
// workgroup repeats the chunk on a guarded path.  Lane partial sums are binary32 over four
// independent accumulators; everything across lanes, waves and chunks is binary64 and, because
// references are integers, rebasing is an exact power-of-two shift.
#include "speckv_accum.h"
#include "speckv_epilogue.h"

namespace speckv {

// Vector path: the position of the lane maximum is recorded per tile by the caller.
template <int N, bool WITH_T, bool SAFE> __device__ __forceinline__ void accum_fast(LaneAcc &a, const float (&x)[N])
{
    const float mv = accum<N, WITH_T, SAFE>(a, x);
    a.vmax = max3(a.vmax, mv, mv);
}

// Scalar path (elements in front of and behind the aligned vectors), all 64 lanes; a lane without
// an element passes -inf.  Records its own position.  `prefer` makes this group win ties for the
// maximum (elements in front of the body).
template <bool WITH_T, bool TRACK>
__device__ __forceinline__ void accum_scalar(LaneAcc &a, float x0, int code, bool prefer)
{
    const float x[1] = {x0};
    const float tm = accum<1, WITH_T, true>(a, x);
    const bool gt = prefer ? (tm >= a.vmax && tm > -INFINITY) : (tm > a.vmax);
    if (TRACK) a.vcode = gt ? code : a.vcode;
    a.vmax = gt ? tm : a.vmax;
}

typedef unsigned int v4u32 __attribute__((ext_vector_type(4)));

// One 16-byte load, optionally nontemporal.
template <bool NT> __device__ __forceinline__ uint4 ld16(const uint4 *p)
{
    if (!NT) return *p;
    const v4u32 v = __builtin_nontemporal_load(reinterpret_cast<const v4u32 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <int U, bool NT>
__device__ __forceinline__ void load_tile(uint4 (&w)[U], const uint4 *p, int stride)
{
#pragma unroll
    for (int j = 0; j < U; ++j) w[j] = ld16<NT>(p + (int64_t)j * stride);
}

// Geometry of one chunk: head scalars, nvec 16-byte vectors, tail scalars.
struct ChunkGeom {
    int e0, head, nvec, tail;
    const uint4 *vp; // first aligned vector
};

// Launch-time code variants.
//   PIPE: keep the next tile's loads in flight while the current tile is processed (two register
//         buffers, ping-pong, no copies); otherwise load-then-process and rely on occupancy.
//   NT:   nontemporal loads (the data is read once by this kernel).
//   TRACK: remember per lane which tile held the lane's maximum, for the argmax; without it the
//         hot loop is a quarter shorter.
template <int DT, bool WITH_T, int THREADS, int U, bool PIPE, bool NT, bool TRACK> struct Body {
    using E = Elem<DT>;
    static constexpr int NE = E::NE;

    // this lane's U vectors of the ragged last tile (indices clamped: duplicates are real row data)
    static __device__ __forceinline__ void load_ragged(uint4 (&w)[U], const ChunkGeom &g, int rag0)
    {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            w[j] = ld16<NT>(g.vp + min(rag0 + j * THREADS, g.nvec - 1));
        }
    }

    template <bool FAST>
    static __device__ __forceinline__ void tile(LaneAcc &a, const uint4 (&w)[U], int first_vec)
    {
        const float before = a.vmax;
#pragma unroll
        for (int j = 0; j < U; ++j) {
            float x[NE];
            E::unpack(w[j], x);
            accum_fast<NE, WITH_T, !FAST>(a, x);
        }
        if (TRACK) a.vcode = a.vmax > before ? ((first_vec << 2) | 0) : a.vcode;
    }

    // The last, partial tile of the chunk: every lane of the wave takes part (the reference is the
    // wave's), a lane whose vector lies beyond the chunk adds -inf, i.e. nothing.
    static __device__ __forceinline__ void ragged_tile(LaneAcc &a, const uint4 (&w)[U], const ChunkGeom &g, int rag0)
    {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int vi = rag0 + j * THREADS;
            float x[NE];
            E::unpack(w[j], x);
            if (vi >= g.nvec) {
#pragma unroll
                for (int k = 0; k < NE; ++k) x[k] = -INFINITY;
            }
            const float before = a.vmax;
            accum_fast<NE, WITH_T, true>(a, x);
            if (TRACK) a.vcode = a.vmax > before ? ((vi << 2) | 1) : a.vcode;
        }
    }

    // Stream the aligned body of a chunk.  FAST: unguarded entropy term.
    template <bool FAST> static __device__ __forceinline__ void run(LaneAcc &a, const ChunkGeom &g, int tid)
    {
        constexpr int TV = THREADS * U; // vectors per tile
        // both are the same for all lanes of a wave; taken from the first lane so that the loop
        // control below stays in scalar registers and branches
        const int ntiles = __builtin_amdgcn_readfirstlane(g.nvec / TV);
        const int rag0 = ntiles * TV + tid; // this lane's first vector of the ragged last tile
        const bool ragged = __builtin_amdgcn_readfirstlane((int)(rag0 - (tid % kWave) < g.nvec)) != 0;
        const uint4 *p = g.vp + tid;
        if (!PIPE) {
            for (int t = 0; t < ntiles; ++t) {
                uint4 w[U];
                load_tile<U, NT>(w, p + (int64_t)t * TV, THREADS);
                tile<FAST>(a, w, t * TV + tid);
            }
            if (ragged) {
                uint4 w[U];
                load_ragged(w, g, rag0);
                ragged_tile(a, w, g, rag0);
            }
            return;
        }
        // Two register buffers, both in flight: A holds tile t, Bf holds tile t+1, and the request
        // for tile t+2 goes out as soon as tile t has been consumed.
        uint4 A[U], Bf[U];
        if (ntiles > 0)
            load_tile<U, NT>(A, p, THREADS);
        else if (ragged)
            load_ragged(A, g, rag0);
        if (ntiles > 1)
            load_tile<U, NT>(Bf, p + TV, THREADS);
        else if (ntiles == 1 && ragged)
            load_ragged(Bf, g, rag0);
        int t = 0;
        while (t + 1 < ntiles) {
            tile<FAST>(a, A, t * TV + tid);
            if (t + 2 < ntiles)
                load_tile<U, NT>(A, p + (int64_t)(t + 2) * TV, THREADS);
            else if (ragged) // t + 2 == ntiles: the ragged tile follows
                load_ragged(A, g, rag0);
            tile<FAST>(a, Bf, (t + 1) * TV + tid);
            if (t + 3 < ntiles)
                load_tile<U, NT>(Bf, p + (int64_t)(t + 3) * TV, THREADS);
            else if (t + 3 == ntiles && ragged)
                load_ragged(Bf, g, rag0);
            t += 2;
        }
        if (t < ntiles) { // one full tile left in A; the ragged tile, if any, is already in Bf
            tile<FAST>(a, A, t * TV + tid);
            if (ragged) ragged_tile(a, Bf, g, rag0);
        } else if (ragged) {
            ragged_tile(a, A, g, rag0);
        }
    }
};

template <int DT, bool WITH_T, int THREADS, int U, bool PIPE, bool NT, bool TRACK, bool FAST>
__device__ __forceinline__ void stream_chunk(LaneAcc &a, const void *logits, int64_t row_elem0,
                                             const ChunkGeom &g, int tid)
{
    using E = Elem<DT>;
    lane_init(a);
    Body<DT, WITH_T, THREADS, U, PIPE, NT, TRACK>::template run<FAST>(a, g, tid);
    // The few elements in front of and behind the aligned vectors (fewer than 16 each) belong to the
    // first lanes of wave 0; the whole wave goes through the motions, the other lanes add -inf.
    if (tid < kWave && g.head + g.tail > 0) {
        // in front of the body: lower indices than anything seen so far, so they win ties
        const bool hd = tid < g.head;
        const int eh = g.e0 + tid;
        accum_scalar<WITH_T, TRACK>(a, hd ? E::load1(logits, row_elem0 + eh) : -INFINITY, (eh << 2) | 2, true);
        // behind the body: higher indices, strict comparison
        const bool tl = tid >= g.head && tid < g.head + g.tail;
        const int et = g.e0 + g.head + g.nvec * E::NE + (tid - g.head);
        accum_scalar<WITH_T, TRACK>(a, tl ? E::load1(logits, row_elem0 + et) : -INFINITY, (et << 2) | 2, false);
    }
}

template <int DT, bool WITH_T, int THREADS, int U, bool PIPE, bool NT, bool TRACK>
__device__ __forceinline__ void row_stats_item(int64_t item0, const void *__restrict__ logits, int V,
                                               int64_t rows_bound, const int64_t *__restrict__ row_off, int B,
                                               int rows_extra_per_seq, int split, int chunk, int want_argmax,
                                               RowStat *partials)
{
    using E = Elem<DT>;
    constexpr int NE = E::NE;
    constexpr int WAVES = THREADS / kWave;
    const int tid = threadIdx.x;
    const int64_t item = item0;
    const int64_t row = item / split;
    const int c = (int)(item - row * split);
    if (row >= rows_bound) return;
    if (row_off) { // ragged batch: the packed buffer may hold fewer rows than the launch bound
        const int64_t total = row_off[B] + (int64_t)rows_extra_per_seq * B;
        if (row >= total) return;
    }
    const int64_t row_elem0 = row * (int64_t)V;
    ChunkGeom g;
    g.e0 = c * chunk;
    const int n = max(0, min(V, g.e0 + chunk) - g.e0);
    const uintptr_t addr = reinterpret_cast<uintptr_t>(logits) + (uintptr_t)(row_elem0 + g.e0) * E::BYTES;
    g.head = min((int)(((16 - (addr & 15)) & 15) / E::BYTES), n);
    g.nvec = (n - g.head) / NE;
    g.tail = (n - g.head) - g.nvec * NE;
    // derived from the kernel argument so that the loads stay in the global address space
    g.vp = reinterpret_cast<const uint4 *>(static_cast<const char *>(logits) +
                                           (row_elem0 + g.e0 + g.head) * E::BYTES);

    LaneAcc a;
    stream_chunk<DT, WITH_T, THREADS, U, PIPE, NT, TRACK, true>(a, logits, row_elem0, g, tid);
    if (WITH_T) {
        // A -inf logit makes 0 * (-inf) = NaN in the entropy sum.  Rare: stream the chunk again, guarded.
        const float tsum = (a.t[0] + a.t[1]) + (a.t[2] + a.t[3]);
        const float ssum = (a.s[0] + a.s[1]) + (a.s[2] + a.s[3]);
        if (__syncthreads_or(tsum != tsum && ssum == ssum))
            stream_chunk<DT, WITH_T, THREADS, U, PIPE, NT, TRACK, false>(a, logits, row_elem0, g, tid);
    }

    // lanes -> wave in binary64; the lanes of a wave share their reference
    const float Rw = a.ref;
    double S = ((double)a.s[0] + (double)a.s[1]) + ((double)a.s[2] + (double)a.s[3]);
    double T = ((double)a.t[0] + (double)a.t[1]) + ((double)a.t[2] + (double)a.t[3]);
    S = wave_sum(S);
    T = wave_sum(T);
    const float Mw = wave_max(a.vmax);

    __shared__ float sh_ref[WAVES], sh_max[WAVES];
    __shared__ double sh_S[WAVES], sh_T[WAVES];
    __shared__ float sh_gmax;
    __shared__ int sh_arg;
    const int wave = tid / kWave, lane = tid % kWave;
    if (lane == 0) {
        sh_ref[wave] = Rw;
        sh_max[wave] = Mw;
        sh_S[wave] = S;
        sh_T[wave] = T;
    }
    if (tid == 0) sh_arg = 0x7fffffff;
    __syncthreads();
    RowStat out;
    if (tid == 0) {
        out.S = sh_S[0]; out.T = sh_T[0]; out.ref = sh_ref[0]; out.vmax = sh_max[0];
        out.argmax = -1; out.pad = 0;
        for (int w = 1; w < WAVES; ++w) {
            RowStat b;
            b.S = sh_S[w]; b.T = sh_T[w]; b.ref = sh_ref[w]; b.vmax = sh_max[w]; b.argmax = -1; b.pad = 0;
            merge_stat(out, b);
        }
        sh_gmax = out.vmax;
    }
    int arg = -1;
    if (TRACK && want_argmax) { // uniform: costs two more barriers and a dependent load, so only on request
        __syncthreads();
        // only lanes holding the chunk maximum look their group up again
        const float gmax = sh_gmax;
        if (a.vcode >= 0 && a.vmax == gmax) {
            const int kind = a.vcode & 3, idx = a.vcode >> 2;
            int cand = 0x7fffffff;
            if (kind == 2) {
                cand = idx;
            } else {
                const int cnt = kind == 0 ? U : 1;
                for (int j = 0; j < cnt && cand == 0x7fffffff; ++j) {
                    const int vi = idx + j * THREADS;
                    const uint4 w = g.vp[vi];
                    float x[NE];
                    E::unpack(w, x);
#pragma unroll
                    for (int k = NE - 1; k >= 0; --k)
                        if (x[k] == gmax) cand = g.e0 + g.head + vi * NE + k;
                }
            }
            atomicMin(&sh_arg, cand);
        }
        __syncthreads();
        arg = sh_arg == 0x7fffffff ? g.e0 : sh_arg;
    }
    if (tid == 0) {
        out.argmax = arg;
        partials[item] = out;
    }
}

template <int DT, bool WITH_T, int THREADS, int U, bool PIPE, bool NT>
__global__ __launch_bounds__(THREADS) void row_stats_kernel(const void *__restrict__ logits, int V,
                                                            int64_t rows_bound,
                                                            const int64_t *__restrict__ row_off, int B,
                                                            int rows_extra_per_seq, int split, int chunk,
                                                            int want_argmax, RowStat *partials)
{
    row_stats_item<DT, WITH_T, THREADS, U, PIPE, NT, true>(blockIdx.x, logits, V, rows_bound, row_off, B,
                                                     rows_extra_per_seq, split, chunk, want_argmax, partials);
}

// Draft rows and target rows of one step in a single launch.  One launch instead of two saves one
// ramp-up and one drain of the chip per step.
// Order of the workgroups (blockIdx -> item):
//   pos0_last == 0: all draft items (with the entropy sum), then all target items, each in row order.
//   pos0_last  > 0 (uniform batches; the value is the batch's speculation length g): the rows of
//     positions 1.. of both sides first, then, sequence by sequence, the chunks of draft row 0 and of
//     target row 0.  Workgroups start in blockIdx order, so the position-0 rows are the last bytes
//     the launch reads: when the tail kernel reads position n of a sequence a second time -- n = 0
//     for most sequences when drafts are often rejected at once -- those rows are the ones most
//     likely still held by the memory-side cache.  Which item a workgroup takes does not change any
//     sum: the chunking of a row and the order inside a chunk stay the same.
// TRACK = false: neither side's argmax is wanted, and the hot loops carry no position.
template <int DT, int THREADS, int U, bool TRACK>
__global__ __launch_bounds__(THREADS) void row_stats_pair_kernel(const void *__restrict__ draft,
                                                                 const void *__restrict__ target, int V,
                                                                 int64_t rows_bound_d, int64_t rows_bound_t,
                                                                 const int64_t *__restrict__ row_off, int B,
                                                                 int split_d, int chunk_d, int split_t, int chunk_t,
                                                                 int want_argmax_d, int want_argmax_t, int64_t items_d,
                                                                 int pos0_last, RowStat *partials_d, RowStat *partials_t,
                                                                 unsigned long long *__restrict__ trace)
{
    // trace (measurement only, usually null): constant-rate clock at entry and exit of every workgroup
    if (trace && threadIdx.x == 0) trace[2 * (size_t)blockIdx.x] = wall_clock64();
    bool is_draft;
    int64_t item;
    if (pos0_last <= 0) {
        is_draft = (int64_t)blockIdx.x < items_d;
        item = is_draft ? (int64_t)blockIdx.x : (int64_t)blockIdx.x - items_d;
    } else {
        const int g = pos0_last;
        int64_t j = blockIdx.x;
        const int64_t rest_d = (int64_t)B * (g - 1) * split_d, rest_t = (int64_t)B * g * split_t;
        if (j < rest_d) { // draft rows of positions 1..g-1
            const int64_t r = j / split_d;
            const int64_t b = r / (g - 1);
            is_draft = true;
            item = (b * g + 1 + (r - b * (g - 1))) * split_d + (j - r * split_d);
        } else if ((j -= rest_d) < rest_t) { // target rows of positions 1..g
            const int64_t r = j / split_t;
            const int64_t b = r / g;
            is_draft = false;
            item = (b * (g + 1) + 1 + (r - b * g)) * split_t + (j - r * split_t);
        } else { // position 0 of sequence b: its draft chunks, then its target chunks
            j -= rest_t;
            const int per = split_d + split_t;
            const int64_t b = j / per;
            const int k = (int)(j - b * per);
            is_draft = k < split_d;
            item = is_draft ? b * g * split_d + k : b * (g + 1) * split_t + (k - split_d);
        }
    }
    if (is_draft)
        row_stats_item<DT, true, THREADS, U, true, true, TRACK>(item, draft, V, rows_bound_d, row_off, B, 0, split_d,
                                                         chunk_d, want_argmax_d, partials_d);
    else
        row_stats_item<DT, false, THREADS, U, true, true, TRACK>(item, target, V, rows_bound_t, row_off, B, 1, split_t,
                                                          chunk_t, want_argmax_t, partials_t);
    if (trace && threadIdx.x == 0) trace[2 * (size_t)blockIdx.x + 1] = wall_clock64();
}

// ---- host launcher ----------------------------------------------------------------------------
template <int DT, bool WITH_T, int THREADS, int U, bool PIPE, bool NT>
static hipError_t launch_one(const void *logits, int V, int64_t rows_bound, const int64_t *row_off, int B,
                             int extra, const StatsLaunch &sl, RowStat *partials, hipStream_t stream)
{
    const int64_t items = rows_bound * sl.split;
    if (items <= 0 || items > 0x7fffffffLL) return hipErrorInvalidValue;
    return launch_lds((row_stats_kernel<DT, WITH_T, THREADS, U, PIPE, NT>), dim3((unsigned)items), dim3(THREADS),
                  (size_t)sl.lds_pad, stream, logits, V, rows_bound, row_off, B, extra, sl.split, sl.chunk, sl.want_argmax, partials);
}

template <int DT, bool WITH_T, bool PIPE, bool NT>
static hipError_t launch_shape(const void *logits, int V, int64_t rows_bound, const int64_t *row_off, int B,
                               int extra, const StatsLaunch &sl, RowStat *partials, hipStream_t stream)
{
#define SPECKV_CASE(TH, UU)                                                                        \
    if (sl.threads == TH && sl.unroll == UU)                                                       \
        return launch_one<DT, WITH_T, TH, UU, PIPE, NT>(logits, V, rows_bound, row_off, B, extra, sl, partials, stream);
#ifndef SPECKV_FEWER_SHAPES
    SPECKV_CASE(128, 2) SPECKV_CASE(128, 4)
    SPECKV_CASE(512, 2) SPECKV_CASE(512, 4)
#endif
    SPECKV_CASE(256, 2) SPECKV_CASE(256, 4)
#undef SPECKV_CASE
    return hipErrorInvalidValue;
}

template <int DT, bool WITH_T>
static hipError_t launch_variant(const void *logits, int V, int64_t rows_bound, const int64_t *row_off, int B,
                                 int extra, const StatsLaunch &sl, RowStat *partials, hipStream_t stream)
{
    if (sl.pipeline)
        return sl.nontemporal ? launch_shape<DT, WITH_T, true, true>(logits, V, rows_bound, row_off, B, extra, sl, partials, stream)
                              : launch_shape<DT, WITH_T, true, false>(logits, V, rows_bound, row_off, B, extra, sl, partials, stream);
    return sl.nontemporal ? launch_shape<DT, WITH_T, false, true>(logits, V, rows_bound, row_off, B, extra, sl, partials, stream)
                          : launch_shape<DT, WITH_T, false, false>(logits, V, rows_bound, row_off, B, extra, sl, partials, stream);
}

hipError_t launch_row_stats(const void *logits, speckv_dtype dtype, bool with_entropy, int V,
                            int64_t rows_bound, const int64_t *row_off, int B, int rows_extra_per_seq,
                            const StatsLaunch &sl, RowStat *partials, hipStream_t stream)
{
#define SPECKV_DT(DTV)                                                                             \
    if (dtype == DTV)                                                                              \
        return with_entropy ? launch_variant<DTV, true>(logits, V, rows_bound, row_off, B,         \
                                                        rows_extra_per_seq, sl, partials, stream)  \
                            : launch_variant<DTV, false>(logits, V, rows_bound, row_off, B,        \
                                                         rows_extra_per_seq, sl, partials, stream);
    SPECKV_DT(SPECKV_F32) SPECKV_DT(SPECKV_F16) SPECKV_DT(SPECKV_BF16)
#undef SPECKV_DT
    return hipErrorInvalidValue;
}

bool row_stats_pair_supported(const StatsLaunch &sd, const StatsLaunch &st)
{
    auto ok = [](const StatsLaunch &s) {
        return (s.threads == 256 || s.threads == 512) && s.unroll == 2 && s.pipeline == 1 && s.nontemporal == 1;
    };
    return ok(sd) && ok(st) && sd.threads == st.threads;
}

hipError_t launch_row_stats_pair(const void *draft, const void *target, speckv_dtype dtype, int V,
                                 int64_t rows_bound_d, int64_t rows_bound_t, const int64_t *row_off, int B,
                                 const StatsLaunch &sd, const StatsLaunch &st, int pos0_last, RowStat *partials_d,
                                 RowStat *partials_t, unsigned long long *trace, hipStream_t stream)
{
    if (!row_stats_pair_supported(sd, st)) return hipErrorInvalidValue;
    if (row_off) pos0_last = 0; // packed rows: position 0 of a sequence is not at a fixed stride
    const int64_t items_d = rows_bound_d * sd.split, items = items_d + rows_bound_t * st.split;
    if (items <= 0 || items > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool track = sd.want_argmax || st.want_argmax;
#define SPECKV_PAIR_T(DTV, TH, TR)                                                                 \
    return launch_lds((row_stats_pair_kernel<DTV, TH, 2, TR>), dim3((unsigned)items), dim3(TH), (size_t)sd.lds_pad, stream, draft, target, V, \
                  rows_bound_d, rows_bound_t, row_off, B, sd.split, sd.chunk, st.split, st.chunk,  \
                  sd.want_argmax, st.want_argmax, items_d, pos0_last, partials_d, partials_t, trace);
#define SPECKV_PAIR(DTV, TH)                                                                       \
    if (dtype == DTV && sd.threads == TH) {                                                        \
        if (track) { SPECKV_PAIR_T(DTV, TH, true) }                                                \
        SPECKV_PAIR_T(DTV, TH, false)                                                              \
    }
    SPECKV_PAIR(SPECKV_F32, 256) SPECKV_PAIR(SPECKV_F16, 256) SPECKV_PAIR(SPECKV_BF16, 256)
    SPECKV_PAIR(SPECKV_F32, 512) SPECKV_PAIR(SPECKV_F16, 512) SPECKV_PAIR(SPECKV_BF16, 512)
#undef SPECKV_PAIR
#undef SPECKV_PAIR_T
    return hipErrorInvalidValue;
}

} // namespace speckv
