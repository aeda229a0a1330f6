// C ABI of libspeckv.so: argument validation, workspace carving, launch sequencing.
// Every check that can fail runs before the first launch, so a rejected call leaves all outputs
// untouched.  See include/speckv.h for the contract of each entry point.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "speckv_internal.h"

using namespace speckv;

namespace {

enum KernelClass {
    K_STATS_DRAFT = 0,
    K_STATS_TARGET,
    K_STATS_PAIR,
    K_SIGNALS_FIN,
    K_ACCEPT,
    K_RS_MASS,
    K_RS_PICK,
    K_SELECT,
    K_GREEDY,
    K_STEP_EPI,
    K_STEP_TAIL,
    K_VERIFY_TAIL,
    K_SAMPLE,
    K_COUNT
};
const char *const kKernelNames[K_COUNT] = {"row_stats_draft", "row_stats_target", "row_stats_pair",
                                           "signals_finalize", "accept",          "resample_mass",
                                           "resample_pick",   "select_gamma",     "greedy_accept",
                                           "step_epilogue",   "step_tail",        "verify_tail",
                                           "sample_draft"};

struct EventRec {
    int kind;
    hipEvent_t a, b;
};

thread_local std::string g_null_handle_error = "no error";

} // namespace

namespace speckv {
thread_local LaunchEvents g_launch_events;
}

// Workspace of speckv_step_static: one array per GPU, inside the library's code object, so that the
// call itself allocates nothing.  In host code this name is only a handle for hipGetSymbolAddress;
// the device address it stands for on a given GPU is looked up once per device (scratch_of) and
// that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[SPECKV_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on `device`, which must be the current device.
hipError_t scratch_of(int device, void **out)
{
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}
} // namespace

struct speckv_handle {
    int device = -1;
    void *static_ws = nullptr; // this device's address of the library-owned workspace (speckv_step_static)
    std::string err = "no error";
    // launch options
    int stats_target_wgs = 8192;
    int stats_max_split = 16;
    int stats_threads = 256;
    int stats_unroll = 2;
    int stats_pipeline = 1;
    int stats_nontemporal = 1;
    int probe_blocks = 16384; // most workgroups of the read probe (it loops beyond that)
    int step_tail = 1; // speckv_step: one workgroup per sequence runs everything after the row statistics
    int sample_threads = 0, sample_loads = 0; // proposal kernel: threads per workgroup (0 = by row count), loads per group
    int tail_threads = 0; // threads per workgroup of the tail kernel: 0 = by batch size, else 512 or 1024
    int stats_pos0_last = 0; // speckv_step, uniform batches: the statistics launch reads the position-0 rows last
    int stats_wgs_per_cu = 4; // most statistics workgroups resident on a compute unit (0 = as many as fit)
    // measurement: per-workgroup clock readings of the two launches of speckv_step (speckv_trace)
    unsigned long long *trace = nullptr;
    size_t trace_words = 0;
    // what the last speckv_signals left in the workspace
    bool sig_valid = false;
    const void *sig_ws = nullptr;
    const void *sig_draft = nullptr;
    int sig_dtype = -1;
    speckv_batch sig_batch{};
    // profiling
    int prof_level = 0;
    int prof_every = 1;          // stamp every prof_every-th launch of a kernel class
    int prof_seen[16] = {0};
    std::vector<EventRec> recs;
    std::vector<hipEvent_t> pool;
};

namespace {

speckv_status fail(speckv_handle *h, speckv_status st, const std::string &msg)
{
    if (h)
        h->err = msg;
    else
        g_null_handle_error = msg;
    return st;
}

speckv_status hip_fail(speckv_handle *h, hipError_t e, const char *what)
{
    return fail(h, SPECKV_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int dtype_bytes(speckv_dtype d) { return d == SPECKV_F32 ? 4 : 2; }

speckv_status check_batch(speckv_handle *h, const speckv_batch *b, bool need_V)
{
    if (!b) return fail(h, SPECKV_ERR_NULL, "batch is NULL");
    if (b->B < 1 || b->B > (1 << 24)) return fail(h, SPECKV_ERR_SHAPE, "B must be in [1, 2^24]");
    if (need_V && (b->V < 1 || b->V > (1 << 28))) return fail(h, SPECKV_ERR_SHAPE, "V must be in [1, 2^28]");
    if (b->gamma_max < 1 || b->gamma_max > SPECKV_GAMMA_LIMIT)
        return fail(h, SPECKV_ERR_GAMMA, "gamma_max must be in [1, SPECKV_GAMMA_LIMIT]");
    if (b->gamma) {
        if (!b->row_off) return fail(h, SPECKV_ERR_NULL, "ragged batch (gamma != NULL) needs row_off");
    } else {
        if (b->row_off) return fail(h, SPECKV_ERR_NULL, "row_off given without gamma");
        if (b->gamma_uniform < 1 || b->gamma_uniform > b->gamma_max)
            return fail(h, SPECKV_ERR_GAMMA, "gamma_uniform must be in [1, gamma_max]");
    }
    return SPECKV_OK;
}

speckv_status check_mlp(speckv_handle *h, const speckv_mlp *mlp, speckv_features mode)
{
    if (!mlp->W2 || !mlp->b2) return fail(h, SPECKV_ERR_NULL, "an MLP weight pointer is NULL");
    if (mode != SPECKV_FEAT_POS0 && mode != SPECKV_FEAT_AGG4) return fail(h, SPECKV_ERR_DTYPE, "unknown feature mode");
    if (mlp->form != SPECKV_MLP_VECTOR && mlp->form != SPECKV_MLP_SCALAR)
        return fail(h, SPECKV_ERR_DTYPE, "unknown MLP form");
    const int want_in = mode == SPECKV_FEAT_POS0 ? 5 : 7;
    if (mlp->n_in != want_in) return fail(h, SPECKV_ERR_SHAPE, "mlp.n_in must be 5 for POS0 and 7 for AGG4");
    if (mlp->n_hidden < 0 || mlp->n_hidden > SPECKV_HIDDEN_LIMIT)
        return fail(h, SPECKV_ERR_SHAPE, "mlp.n_hidden must be in [0, SPECKV_HIDDEN_LIMIT]");
    if (mlp->n_hidden > 0 && (!mlp->W1 || !mlp->b1)) return fail(h, SPECKV_ERR_NULL, "an MLP weight pointer is NULL");
    return SPECKV_OK;
}

BatchView view_of(const speckv_batch &b)
{
    BatchView v;
    v.B = b.B; v.V = b.V; v.gamma_max = b.gamma_max; v.gamma_uniform = b.gamma_uniform;
    v.gamma = b.gamma; v.row_off = b.row_off; v.seq_base = b.seq_base;
    return v;
}

bool same_batch(const speckv_batch &a, const speckv_batch &b)
{
    return a.B == b.B && a.V == b.V && a.gamma_max == b.gamma_max && a.gamma_uniform == b.gamma_uniform &&
           a.gamma == b.gamma && a.row_off == b.row_off && a.seq_base == b.seq_base;
}

// Chunks per row so that the statistics pass of a whole step (draft rows and target rows, in one
// launch or in two) has about stats_target_wgs workgroups, each chunk a whole number of load
// tiles (threads * unroll 16-byte vectors) so that only a row's last chunk is ragged.  Every entry
// point derives the chunking from the step's total row count, so that the same batch is summed
// in the same order whichever way the step is issued.
int64_t step_rows(const speckv_batch &b)
{
    const int64_t g = b.gamma ? b.gamma_max : b.gamma_uniform;
    return (int64_t)b.B * (2 * g + 1);
}

StatsLaunch choose_stats(const speckv_handle *h, int64_t rows_bound, int V, speckv_dtype dtype)
{
    StatsLaunch sl;
    sl.threads = h->stats_threads;
    sl.unroll = h->stats_unroll;
    sl.pipeline = h->stats_pipeline;
    sl.nontemporal = h->stats_nontemporal;
    sl.want_argmax = 0;
    // Fewer resident workgroups mean fewer streams that the memory system serves at once: measured on
    // the one-launch kernel, 7 per compute unit (what the registers allow) against 4: 165.0 -> 164.0 us
    // on 2048 + 2304 rows of 128256 bf16, 2095 -> 2033 us on 32768 + 36864 rows of 50257 binary32; 3
    // are too few (168 us).  Bounded through LDS that a workgroup occupies without using it: with
    // 160 KB per compute unit, n workgroups fit and n + 1 do not when each holds 160 / (n + 1) + 1 KB.
    sl.lds_pad = h->stats_wgs_per_cu > 0 ? (160 / (h->stats_wgs_per_cu + 1) + 1) << 10 : 0;
    const int ne = 16 / dtype_bytes(dtype);
    const int64_t tile = (int64_t)sl.threads * sl.unroll * ne;
    int64_t want = (h->stats_target_wgs + rows_bound - 1) / rows_bound;
    // A workgroup's fixed cost (prologue, binary64 reductions) is that of streaming a few tens of
    // KB, so a chunk should hold at least 64 KB -- unless there are so few rows that the chunks would
    // not even give every compute unit one workgroup (measured: B = 64 rows of 64 KB, 576 workgroups
    // of a whole row 11.6 us, 4608 of an eighth 16.3 us; B = 1, 144 workgroups 4.3 us, 18 5.0 us)
    const int64_t by_bytes = std::max<int64_t>(1, (int64_t)V * dtype_bytes(dtype) / (64 << 10));
    const int64_t to_fill = (256 + rows_bound - 1) / rows_bound;
    want = std::min(want, std::max(by_bytes, to_fill));
    if (want > h->stats_max_split) want = h->stats_max_split;
    if (want < 1) want = 1;
    int64_t chunk = (V + want - 1) / want;
    chunk = (chunk + tile - 1) / tile * tile;
    sl.chunk = (int)chunk;
    sl.split = (int)((V + chunk - 1) / chunk);
    return sl;
}

// While alive, the next launch on this thread is stamped with a pair of pooled events.
struct ProfScope {
    speckv_handle *h;
    int kind;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(speckv_handle *h_, hipStream_t, int kind_) : h(h_), kind(kind_)
    {
        const bool wanted = h->prof_level >= 2 || (h->prof_level == 1 && kind <= K_STATS_PAIR);
        if (!wanted || h->pool.size() < 2) return;
        if (h->prof_seen[kind]++ % h->prof_every) return;
        a = h->pool.back(); h->pool.pop_back();
        b = h->pool.back(); h->pool.pop_back();
        g_launch_events.start = a;
        g_launch_events.stop = b;
    }
    ~ProfScope()
    {
        if (!a) return;
        g_launch_events = LaunchEvents{};
        h->recs.push_back({kind, a, b});
    }
};

} // namespace
extern "C" {

speckv_status speckv_create(speckv_handle **out, int device)
{
    if (!out) return fail(nullptr, SPECKV_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (device < -1) return fail(nullptr, SPECKV_ERR_SHAPE, "device must be >= -1");
    if (device >= 0) {
        int count = 0;
        hipError_t e = hipGetDeviceCount(&count);
        if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDeviceCount");
        if (device >= count) return fail(nullptr, SPECKV_ERR_DEVICE, "no such HIP device");
        e = hipSetDevice(device);
        if (e != hipSuccess) return hip_fail(nullptr, e, "hipSetDevice");
    }
    void *static_ws = nullptr;
    if (device >= 0) { // with `device` current: each GPU holds its own copy of the array at its own address
        const hipError_t e = scratch_of(device, &static_ws);
        if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetSymbolAddress(scratch)");
    }
    speckv_handle *h = new speckv_handle();
    h->device = device;
    h->static_ws = static_ws;
    *out = h;
    return SPECKV_OK;
}

speckv_status speckv_destroy(speckv_handle *h)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    for (auto &r : h->recs) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    for (auto e : h->pool) (void)hipEventDestroy(e);
    delete h;
    return SPECKV_OK;
}

const char *speckv_last_error(const speckv_handle *h)
{
    return h ? h->err.c_str() : g_null_handle_error.c_str();
}

size_t speckv_workspace_bytes(int32_t B, int32_t gamma_max)
{
    if (B < 1 || B > (1 << 24) || gamma_max < 1 || gamma_max > SPECKV_GAMMA_LIMIT) return 0;
    return ws_layout(B, gamma_max).total;
}

speckv_status speckv_row_offsets(speckv_handle *h, const int32_t *gamma, int32_t B, int64_t *row_off,
                                 speckv_stream stream)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    if (!gamma || !row_off) return fail(h, SPECKV_ERR_NULL, "gamma / row_off is NULL");
    if (B < 1 || B > (1 << 24)) return fail(h, SPECKV_ERR_SHAPE, "B must be in [1, 2^24]");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    hipError_t e = launch_row_offsets(gamma, B, row_off, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "row_offsets launch");
    return SPECKV_OK;
}

speckv_status speckv_signals(speckv_handle *h, const speckv_batch *batch, const void *draft_logits,
                             speckv_dtype dtype, void *ws, size_t ws_bytes, speckv_stream stream,
                             float *H, float *conf, int32_t *argmax, float *agg)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    h->sig_valid = false;
    speckv_status st = check_batch(h, batch, true);
    if (st != SPECKV_OK) return st;
    if (!draft_logits || !ws || !H || !conf || !agg)
        return fail(h, SPECKV_ERR_NULL, "draft_logits / ws / H / conf / agg is NULL");
    if (dtype != SPECKV_F32 && dtype != SPECKV_F16 && dtype != SPECKV_BF16)
        return fail(h, SPECKV_ERR_DTYPE, "unknown dtype");
    if (!aligned16(draft_logits)) return fail(h, SPECKV_ERR_ALIGN, "draft_logits must be 16-byte aligned");
    if (!aligned16(ws)) return fail(h, SPECKV_ERR_ALIGN, "workspace must be 16-byte aligned");
    const WsLayout L = ws_layout(batch->B, batch->gamma_max);
    if (ws_bytes < L.total) return fail(h, SPECKV_ERR_WORKSPACE, "workspace smaller than speckv_workspace_bytes()");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    RowStat *stat_d = reinterpret_cast<RowStat *>(w + L.stat_d);
    RowStat *partial = reinterpret_cast<RowStat *>(w + L.partial);
    const BatchView bv = view_of(*batch);
    const int64_t rows_bound = (int64_t)batch->B * (batch->gamma ? batch->gamma_max : batch->gamma_uniform);
    StatsLaunch sl = choose_stats(h, step_rows(*batch), batch->V, dtype);
    sl.want_argmax = argmax != nullptr;
    hipError_t e;
    {
        ProfScope p(h, s, K_STATS_DRAFT);
        e = launch_row_stats(draft_logits, dtype, true, batch->V, rows_bound, batch->row_off, batch->B, 0, sl,
                             partial, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "row_stats (draft) launch");
    {
        ProfScope p(h, s, K_SIGNALS_FIN);
        e = launch_signals_finalize(bv, partial, sl.split, stat_d, H, conf, argmax, agg, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "signals_finalize launch");
    h->sig_valid = true;
    h->sig_ws = ws;
    h->sig_draft = draft_logits;
    h->sig_dtype = dtype;
    h->sig_batch = *batch;
    return SPECKV_OK;
}

speckv_status speckv_verify(speckv_handle *h, const speckv_batch *batch, const void *target_logits,
                            const void *draft_logits, speckv_dtype dtype, const int32_t *draft_tokens,
                            uint64_t seed, uint32_t step, void *ws, size_t ws_bytes, speckv_stream stream,
                            int32_t *n_accepted, int32_t *tokens, int32_t *num_tokens, float *accept_rate,
                            uint32_t *row_flags)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    speckv_status st = check_batch(h, batch, true);
    if (st != SPECKV_OK) return st;
    if (!target_logits || !draft_logits || !draft_tokens || !ws || !n_accepted || !tokens || !num_tokens)
        return fail(h, SPECKV_ERR_NULL, "a required pointer is NULL");
    if (dtype != SPECKV_F32 && dtype != SPECKV_F16 && dtype != SPECKV_BF16)
        return fail(h, SPECKV_ERR_DTYPE, "unknown dtype");
    if (!aligned16(target_logits) || !aligned16(draft_logits))
        return fail(h, SPECKV_ERR_ALIGN, "logits must be 16-byte aligned");
    if (!aligned16(ws)) return fail(h, SPECKV_ERR_ALIGN, "workspace must be 16-byte aligned");
    const WsLayout L = ws_layout(batch->B, batch->gamma_max);
    if (ws_bytes < L.total) return fail(h, SPECKV_ERR_WORKSPACE, "workspace smaller than speckv_workspace_bytes()");
    if (!h->sig_valid || h->sig_ws != ws || h->sig_draft != draft_logits || h->sig_dtype != (int)dtype ||
        !same_batch(h->sig_batch, *batch))
        return fail(h, SPECKV_ERR_STATE, "speckv_verify must follow speckv_signals of the same batch, "
                                         "draft logits, dtype and workspace");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    RowStat *stat_d = reinterpret_cast<RowStat *>(w + L.stat_d);
    RowStat *stat_t = reinterpret_cast<RowStat *>(w + L.stat_t);
    RowStat *partial = reinterpret_cast<RowStat *>(w + L.partial);
    ResampleDesc *desc = reinterpret_cast<ResampleDesc *>(w + L.desc);
    double *mass = reinterpret_cast<double *>(w + L.mass);
    const BatchView bv = view_of(*batch);
    const int64_t rows_bound =
        (int64_t)batch->B * ((batch->gamma ? batch->gamma_max : batch->gamma_uniform) + 1);
    StatsLaunch sl = choose_stats(h, step_rows(*batch), batch->V, dtype);
    h->sig_valid = false; // the statistics are consumed by this call
    hipError_t e;
    {
        ProfScope p(h, s, K_STATS_TARGET);
        e = launch_row_stats(target_logits, dtype, false, batch->V, rows_bound, batch->row_off, batch->B, 1, sl,
                             partial, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "row_stats (target) launch");
    if (h->step_tail) { // accept scan, residual masses and token pick: one workgroup per sequence, one launch
        ProfScope p(h, s, K_VERIFY_TAIL);
        const AcceptArgs aa{draft_logits, target_logits, (int)dtype, draft_tokens, (uint32_t)(seed & 0xffffffffu),
                            (uint32_t)(seed >> 32), step, desc, n_accepted, tokens, accept_rate};
        const speckv_mlp none{};
        e = launch_step_tail(bv, aa, dtype, stat_d, 1, partial, sl.split, nullptr, stat_t, none, 0, nullptr, nullptr,
                             nullptr, nullptr, nullptr, nullptr, nullptr, num_tokens, row_flags, nullptr, h->tail_threads, s);
        if (e != hipSuccess) return hip_fail(h, e, "verify_tail launch");
        return SPECKV_OK;
    }
    {
        ProfScope p(h, s, K_ACCEPT);
        e = launch_accept(bv, draft_logits, target_logits, dtype, draft_tokens, seed, step, stat_d, partial,
                          sl.split, stat_t, desc, n_accepted, tokens, accept_rate, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "accept launch");
    {
        ProfScope p(h, s, K_RS_MASS);
        e = launch_resample_mass(bv, draft_logits, target_logits, dtype, desc, mass, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "resample_mass launch");
    {
        ProfScope p(h, s, K_RS_PICK);
        e = launch_resample_pick(bv, draft_logits, target_logits, dtype, desc, mass, tokens, num_tokens,
                                 row_flags, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "resample_pick launch");
    return SPECKV_OK;
}

speckv_status speckv_verify_greedy(speckv_handle *h, const speckv_batch *batch, const void *target_logits,
                                   speckv_dtype dtype, const int32_t *draft_tokens, void *ws, size_t ws_bytes,
                                   speckv_stream stream, int32_t *n_accepted, int32_t *tokens,
                                   int32_t *num_tokens, float *accept_rate, uint32_t *row_flags)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    speckv_status st = check_batch(h, batch, true);
    if (st != SPECKV_OK) return st;
    if (!target_logits || !draft_tokens || !ws || !n_accepted || !tokens || !num_tokens)
        return fail(h, SPECKV_ERR_NULL, "a required pointer is NULL");
    if (dtype != SPECKV_F32 && dtype != SPECKV_F16 && dtype != SPECKV_BF16)
        return fail(h, SPECKV_ERR_DTYPE, "unknown dtype");
    if (!aligned16(target_logits)) return fail(h, SPECKV_ERR_ALIGN, "logits must be 16-byte aligned");
    if (!aligned16(ws)) return fail(h, SPECKV_ERR_ALIGN, "workspace must be 16-byte aligned");
    const WsLayout L = ws_layout(batch->B, batch->gamma_max);
    if (ws_bytes < L.total) return fail(h, SPECKV_ERR_WORKSPACE, "workspace smaller than speckv_workspace_bytes()");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    RowStat *stat_t = reinterpret_cast<RowStat *>(w + L.stat_t);
    RowStat *partial = reinterpret_cast<RowStat *>(w + L.partial);
    const int64_t rows_bound =
        (int64_t)batch->B * ((batch->gamma ? batch->gamma_max : batch->gamma_uniform) + 1);
    StatsLaunch sl = choose_stats(h, step_rows(*batch), batch->V, dtype);
    sl.want_argmax = 1;
    hipError_t e;
    {
        ProfScope p(h, s, K_STATS_TARGET);
        e = launch_row_stats(target_logits, dtype, false, batch->V, rows_bound, batch->row_off, batch->B, 1, sl,
                             partial, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "row_stats (target) launch");
    {
        ProfScope p(h, s, K_GREEDY);
        e = launch_greedy_accept(view_of(*batch), draft_tokens, partial, sl.split, stat_t, n_accepted, tokens,
                                 num_tokens, accept_rate, row_flags, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "greedy_accept launch");
    return SPECKV_OK;
}

speckv_status speckv_sample_draft(speckv_handle *h, const speckv_batch *batch, const void *draft_logits,
                                  speckv_dtype dtype, uint64_t seed, uint32_t step, uint32_t pos0,
                                  speckv_stream stream, int32_t *tokens, float *prob, uint32_t *row_flags)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    speckv_status st = check_batch(h, batch, true);
    if (st != SPECKV_OK) return st;
    if (!draft_logits || !tokens) return fail(h, SPECKV_ERR_NULL, "draft_logits / tokens is NULL");
    if (dtype != SPECKV_F32 && dtype != SPECKV_F16 && dtype != SPECKV_BF16)
        return fail(h, SPECKV_ERR_DTYPE, "unknown dtype");
    if (!aligned16(draft_logits)) return fail(h, SPECKV_ERR_ALIGN, "draft_logits must be 16-byte aligned");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t rows_bound = (int64_t)batch->B * (batch->gamma ? batch->gamma_max : batch->gamma_uniform);
    hipError_t e;
    {
        ProfScope p(h, s, K_SAMPLE);
        e = launch_sample_rows(view_of(*batch), draft_logits, dtype, rows_bound, seed, step, pos0, tokens, prob,
                               row_flags, h->sample_threads, h->sample_loads, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "sample_draft launch");
    return SPECKV_OK;
}

speckv_status speckv_select_gamma(speckv_handle *h, const speckv_batch *batch, const speckv_mlp *mlp,
                                  speckv_features mode, const float *H, const float *conf, const float *agg,
                                  const uint8_t *comp, speckv_stream stream, int32_t *gamma_next,
                                  float *scores)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    speckv_status st = check_batch(h, batch, false);
    if (st != SPECKV_OK) return st;
    if (!mlp || !comp || !gamma_next) return fail(h, SPECKV_ERR_NULL, "mlp / comp / gamma_next is NULL");
    st = check_mlp(h, mlp, mode);
    if (st != SPECKV_OK) return st;
    if (mode == SPECKV_FEAT_POS0 && (!H || !conf)) return fail(h, SPECKV_ERR_NULL, "POS0 needs H and conf");
    if (mode == SPECKV_FEAT_AGG4 && !agg) return fail(h, SPECKV_ERR_NULL, "AGG4 needs agg");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    {
        ProfScope p(h, s, K_SELECT);
        e = launch_select_gamma(view_of(*batch), *mlp, (int)mode, H, conf, agg, comp, gamma_next, scores, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "select_gamma launch");
    return SPECKV_OK;
}

// One whole step with the workspace at `ws`.  static_ws: the workspace is the library's own array
// (its size is fixed, so the batch must fit it; the handle without a device has none).
static speckv_status step_impl(speckv_handle *h, const speckv_batch *batch, const speckv_mlp *mlp,
                               const speckv_step_args *a, void *ws, size_t ws_bytes, speckv_stream stream,
                               bool static_ws)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    speckv_status st = check_batch(h, batch, true);
    if (st != SPECKV_OK) return st;
    if (static_ws) {
        if (ws_layout(batch->B, batch->gamma_max).total > ws_bytes)
            return fail(h, SPECKV_ERR_WORKSPACE,
                        "batch too large for speckv_step_static: speckv_workspace_bytes(B, gamma_max) exceeds "
                        "SPECKV_STATIC_WS_BYTES (use speckv_step with a workspace of the caller's)");
    }
    if (!a || !mlp || (!ws && !static_ws)) return fail(h, SPECKV_ERR_NULL, "args / mlp / ws is NULL");
    if (!a->draft_logits || !a->target_logits || !a->draft_tokens || !a->comp || !a->H || !a->conf || !a->agg ||
        !a->n_accepted || !a->tokens || !a->num_tokens || !a->gamma_next)
        return fail(h, SPECKV_ERR_NULL, "a required pointer of the step arguments is NULL");
    if (a->dtype != SPECKV_F32 && a->dtype != SPECKV_F16 && a->dtype != SPECKV_BF16)
        return fail(h, SPECKV_ERR_DTYPE, "unknown dtype");
    if (a->greedy != 0 && a->greedy != 1) return fail(h, SPECKV_ERR_DTYPE, "greedy must be 0 or 1");
    st = check_mlp(h, mlp, a->mode);
    if (st != SPECKV_OK) return st;
    if (!aligned16(a->target_logits) || !aligned16(a->draft_logits))
        return fail(h, SPECKV_ERR_ALIGN, "logits must be 16-byte aligned");
    if (!aligned16(ws)) return fail(h, SPECKV_ERR_ALIGN, "workspace must be 16-byte aligned");
    const WsLayout L = ws_layout(batch->B, batch->gamma_max);
    if (ws_bytes < L.total) return fail(h, SPECKV_ERR_WORKSPACE, "workspace smaller than speckv_workspace_bytes()");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    if (!ws) return fail(h, SPECKV_ERR_DEVICE, "the library's workspace has no address on this device");

    if (!static_ws) h->sig_valid = false; // the caller's workspace may be the one speckv_signals wrote
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    RowStat *stat_d = reinterpret_cast<RowStat *>(w + L.stat_d);
    RowStat *stat_t = reinterpret_cast<RowStat *>(w + L.stat_t);
    RowStat *partial_t = reinterpret_cast<RowStat *>(w + L.partial);
    RowStat *partial_d = reinterpret_cast<RowStat *>(w + L.partial_d);
    ResampleDesc *desc = reinterpret_cast<ResampleDesc *>(w + L.desc);
    double *mass = reinterpret_cast<double *>(w + L.mass);
    const BatchView bv = view_of(*batch);
    const int gb = batch->gamma ? batch->gamma_max : batch->gamma_uniform;
    const int64_t rows_d = (int64_t)batch->B * gb, rows_t = (int64_t)batch->B * (gb + 1);
    StatsLaunch sd = choose_stats(h, step_rows(*batch), batch->V, a->dtype);
    StatsLaunch stt = sd;
    sd.want_argmax = a->argmax != nullptr;
    stt.want_argmax = a->greedy ? 1 : 0; // the greedy rule compares the target's top prediction
    hipError_t e;
    // trace buffer layout: 32 words per sequence (tail launch), then 2 words per statistics workgroup
    unsigned long long *trace_tail = nullptr, *trace_stats = nullptr;
    if (h->trace) {
        const size_t need = 32 * (size_t)batch->B + 2 * (size_t)(rows_d * sd.split + rows_t * stt.split);
        if (h->trace_words < need) return fail(h, SPECKV_ERR_WORKSPACE, "trace buffer too small for this batch");
        trace_tail = h->trace;
        trace_stats = h->trace + 32 * (size_t)batch->B;
    }
    if (row_stats_pair_supported(sd, stt)) {
        ProfScope p(h, s, K_STATS_PAIR);
        const int pos0_last = (h->stats_pos0_last && !batch->gamma) ? batch->gamma_uniform : 0;
        e = launch_row_stats_pair(a->draft_logits, a->target_logits, a->dtype, batch->V, rows_d, rows_t, batch->row_off,
                                  batch->B, sd, stt, pos0_last, partial_d, partial_t, trace_stats, s);
        if (e != hipSuccess) return hip_fail(h, e, "row_stats (pair) launch");
    } else { // launch shapes other than the default: one launch per side
        {
            ProfScope p(h, s, K_STATS_DRAFT);
            e = launch_row_stats(a->draft_logits, a->dtype, true, batch->V, rows_d, batch->row_off, batch->B, 0, sd,
                                 partial_d, s);
        }
        if (e != hipSuccess) return hip_fail(h, e, "row_stats (draft) launch");
        {
            ProfScope p(h, s, K_STATS_TARGET);
            e = launch_row_stats(a->target_logits, a->dtype, false, batch->V, rows_t, batch->row_off, batch->B, 1, stt,
                                 partial_t, s);
        }
        if (e != hipSuccess) return hip_fail(h, e, "row_stats (target) launch");
    }
    const AcceptArgs aa{a->draft_logits, a->target_logits, (int)a->dtype, a->draft_tokens,
                        (uint32_t)(a->seed & 0xffffffffu), (uint32_t)(a->seed >> 32), a->step, desc,
                        a->n_accepted, a->tokens, a->accept_rate};
    if (a->greedy) { // signals + top-1 match + controller: the step ends after this launch
        ProfScope p(h, s, K_STEP_EPI);
        e = launch_step_epilogue(bv, aa, partial_d, sd.split, partial_t, stt.split, stat_d, stat_t, *mlp, (int)a->mode,
                                 a->comp, a->H, a->conf, a->argmax, a->agg, a->gamma_next, a->scores, true,
                                 a->num_tokens, a->row_flags, s);
        if (e != hipSuccess) return hip_fail(h, e, "step_epilogue launch");
        return SPECKV_OK;
    }
    if (h->step_tail) {
        ProfScope p(h, s, K_STEP_TAIL);
        e = launch_step_tail(bv, aa, a->dtype, partial_d, sd.split, partial_t, stt.split, stat_d, stat_t, *mlp,
                             (int)a->mode, a->comp, a->H, a->conf, a->argmax, a->agg, a->gamma_next, a->scores,
                             a->num_tokens, a->row_flags, trace_tail, h->tail_threads, s);
        if (e != hipSuccess) return hip_fail(h, e, "step_tail launch");
        return SPECKV_OK;
    }
    {
        ProfScope p(h, s, K_STEP_EPI);
        e = launch_step_epilogue(bv, aa, partial_d, sd.split, partial_t, stt.split, stat_d, stat_t, *mlp, (int)a->mode,
                                 a->comp, a->H, a->conf, a->argmax, a->agg, a->gamma_next, a->scores, false,
                                 a->num_tokens, a->row_flags, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "step_epilogue launch");
    {
        ProfScope p(h, s, K_RS_MASS);
        e = launch_resample_mass(bv, a->draft_logits, a->target_logits, a->dtype, desc, mass, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "resample_mass launch");
    {
        ProfScope p(h, s, K_RS_PICK);
        e = launch_resample_pick(bv, a->draft_logits, a->target_logits, a->dtype, desc, mass, a->tokens, a->num_tokens,
                                 a->row_flags, s);
    }
    if (e != hipSuccess) return hip_fail(h, e, "resample_pick launch");
    return SPECKV_OK;
}

speckv_status speckv_step(speckv_handle *h, const speckv_batch *batch, const speckv_mlp *mlp,
                          const speckv_step_args *a, void *ws, size_t ws_bytes, speckv_stream stream)
{
    return step_impl(h, batch, mlp, a, ws, ws_bytes, stream, false);
}

// The same step with the library's own per-GPU array as workspace: no allocation of any kind here
// or below (kernel launches only).  Every region of the workspace that a step reads was written
// earlier in the same step (chunk statistics by the statistics launch, row statistics and the
// resample descriptor by the tail), so nothing has to be cleared between calls, whatever the last
// call left behind.
speckv_status speckv_step_static(speckv_handle *h, const speckv_batch *batch, const speckv_mlp *mlp,
                                 const speckv_step_args *a, speckv_stream stream)
{
    return step_impl(h, batch, mlp, a, h ? h->static_ws : nullptr, SPECKV_STATIC_WS_BYTES, stream, true);
}

// ---- options, profiling, probes ---------------------------------------------------------------

speckv_status speckv_set_option(speckv_handle *h, const char *name, int32_t value)
{
    if (!h || !name) return fail(h, SPECKV_ERR_NULL, "handle / name is NULL");
    const std::string n(name);
    if (n == "stats_target_wgs") {
        if (value < 1 || value > kMaxStatsTargetWgs) return fail(h, SPECKV_ERR_SHAPE, "stats_target_wgs out of range");
        h->stats_target_wgs = value;
    } else if (n == "stats_max_split") {
        if (value < 1 || value > 1024) return fail(h, SPECKV_ERR_SHAPE, "stats_max_split out of range");
        h->stats_max_split = value;
    } else if (n == "stats_threads") {
        if (value != 128 && value != 256 && value != 512) return fail(h, SPECKV_ERR_SHAPE, "stats_threads must be 128, 256 or 512");
        h->stats_threads = value;
    } else if (n == "stats_unroll") {
        if (value != 2 && value != 4) return fail(h, SPECKV_ERR_SHAPE, "stats_unroll must be 2 or 4");
        h->stats_unroll = value;
    } else if (n == "probe_blocks") {
        if (value < 1 || value > (1 << 22)) return fail(h, SPECKV_ERR_SHAPE, "probe_blocks out of range");
        h->probe_blocks = value;
    } else if (n == "step_tail") {
        if (value != 0 && value != 1) return fail(h, SPECKV_ERR_SHAPE, "step_tail must be 0 or 1");
        h->step_tail = value;
    } else if (n == "sample_threads") {
        if (value != 0 && value != 512 && value != 1024) return fail(h, SPECKV_ERR_SHAPE, "sample_threads must be 0, 512 or 1024");
        h->sample_threads = value;
    } else if (n == "sample_loads") {
        if (value != 0 && value != 2 && value != 4) return fail(h, SPECKV_ERR_SHAPE, "sample_loads must be 0, 2 or 4");
        h->sample_loads = value;
    } else if (n == "tail_threads") {
        if (value != 0 && value != 256 && value != 512 && value != 1024) return fail(h, SPECKV_ERR_SHAPE, "tail_threads must be 0, 256, 512 or 1024");
        h->tail_threads = value;
    } else if (n == "stats_pos0_last") {
        if (value != 0 && value != 1) return fail(h, SPECKV_ERR_SHAPE, "stats_pos0_last must be 0 or 1");
        h->stats_pos0_last = value;
    } else if (n == "stats_wgs_per_cu") {
        if (value != 0 && (value < 2 || value > 16)) return fail(h, SPECKV_ERR_SHAPE, "stats_wgs_per_cu must be 0 or 2..16");
        h->stats_wgs_per_cu = value;
    } else if (n == "profile_every") {
        if (value < 1 || value > 1 << 20) return fail(h, SPECKV_ERR_SHAPE, "profile_every out of range");
        h->prof_every = value;
    } else if (n == "stats_pipeline") {
        if (value != 0 && value != 1) return fail(h, SPECKV_ERR_SHAPE, "stats_pipeline must be 0 or 1");
        h->stats_pipeline = value;
    } else if (n == "stats_nontemporal") {
        if (value != 0 && value != 1) return fail(h, SPECKV_ERR_SHAPE, "stats_nontemporal must be 0 or 1");
        h->stats_nontemporal = value;
    } else {
        return fail(h, SPECKV_ERR_SHAPE, "unknown option: " + n);
    }
    return SPECKV_OK;
}

speckv_status speckv_get_option(const speckv_handle *h, const char *name, int32_t *value)
{
    if (!h || !name || !value) return SPECKV_ERR_NULL;
    const std::string n(name);
    if (n == "stats_target_wgs") *value = h->stats_target_wgs;
    else if (n == "stats_max_split") *value = h->stats_max_split;
    else if (n == "stats_threads") *value = h->stats_threads;
    else if (n == "stats_unroll") *value = h->stats_unroll;
    else if (n == "step_tail") *value = h->step_tail;
    else if (n == "stats_pos0_last") *value = h->stats_pos0_last;
    else if (n == "stats_wgs_per_cu") *value = h->stats_wgs_per_cu;
    else if (n == "tail_threads") *value = h->tail_threads;
    else if (n == "sample_threads") *value = h->sample_threads;
    else if (n == "sample_loads") *value = h->sample_loads;
    else if (n == "probe_blocks") *value = h->probe_blocks;
    else if (n == "profile_every") *value = h->prof_every;
    else if (n == "stats_pipeline") *value = h->stats_pipeline;
    else if (n == "stats_nontemporal") *value = h->stats_nontemporal;
    else return SPECKV_ERR_SHAPE;
    return SPECKV_OK;
}

speckv_status speckv_profile(speckv_handle *h, int32_t enable)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    if (enable < 0 || enable > 2) return fail(h, SPECKV_ERR_SHAPE, "enable must be 0, 1 or 2");
    if (enable && h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    if (enable) {
        for (auto &r : h->recs) {
            h->pool.push_back(r.a);
            h->pool.push_back(r.b);
        }
        h->recs.clear();
        while (h->pool.size() < 8192) {
            hipEvent_t ev;
            // device-scope release: the stamp needs no system-wide cache flush when the event completes
            hipError_t e = hipEventCreateWithFlags(&ev, hipEventReleaseToDevice);
            if (e != hipSuccess) return hip_fail(h, e, "hipEventCreate");
            h->pool.push_back(ev);
        }
    }
    h->prof_level = enable;
    for (int &c : h->prof_seen) c = 0;
    return SPECKV_OK;
}

speckv_status speckv_trace(speckv_handle *h, uint64_t *buf, size_t bytes)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    if (buf && (reinterpret_cast<uintptr_t>(buf) & 7)) return fail(h, SPECKV_ERR_ALIGN, "trace buffer must be 8-byte aligned");
    h->trace = reinterpret_cast<unsigned long long *>(buf);
    h->trace_words = buf ? bytes / 8 : 0;
    return SPECKV_OK;
}

speckv_status speckv_profile_read(speckv_handle *h, const char *kernel, int32_t *launches, double *total_ms)
{
    if (!h || !kernel || !launches || !total_ms) return fail(h, SPECKV_ERR_NULL, "a pointer is NULL");
    int kind = -1;
    for (int k = 0; k < K_COUNT; ++k)
        if (std::strcmp(kernel, kKernelNames[k]) == 0) kind = k;
    if (kind < 0) return fail(h, SPECKV_ERR_SHAPE, "unknown kernel class");
    int n = 0;
    double ms = 0.0;
    for (auto &r : h->recs) {
        if (r.kind != kind) continue;
        hipError_t e = hipEventSynchronize(r.b);
        if (e != hipSuccess) return hip_fail(h, e, "hipEventSynchronize");
        float t = 0.f;
        e = hipEventElapsedTime(&t, r.a, r.b);
        if (e != hipSuccess) return hip_fail(h, e, "hipEventElapsedTime");
        ms += t;
        ++n;
    }
    *launches = n;
    *total_ms = ms;
    return SPECKV_OK;
}

speckv_status speckv_probe_read(speckv_handle *h, const void *src, size_t bytes, void *sink, speckv_stream stream)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    if (!src || !sink) return fail(h, SPECKV_ERR_NULL, "src / sink is NULL");
    if (bytes == 0 || bytes % 16) return fail(h, SPECKV_ERR_SHAPE, "bytes must be a positive multiple of 16");
    if (!aligned16(src) || (reinterpret_cast<uintptr_t>(sink) & 7)) return fail(h, SPECKV_ERR_ALIGN, "misaligned pointer");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    hipError_t e = launch_probe_read(src, bytes, sink, h->probe_blocks, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "probe_read launch");
    return SPECKV_OK;
}

speckv_status speckv_probe_copy(speckv_handle *h, void *dst, const void *src, size_t bytes, speckv_stream stream)
{
    if (!h) return fail(nullptr, SPECKV_ERR_NULL, "handle is NULL");
    if (!src || !dst) return fail(h, SPECKV_ERR_NULL, "src / dst is NULL");
    if (bytes == 0 || bytes % 16) return fail(h, SPECKV_ERR_SHAPE, "bytes must be a positive multiple of 16");
    if (!aligned16(src) || !aligned16(dst)) return fail(h, SPECKV_ERR_ALIGN, "misaligned pointer");
    if (h->device < 0) return fail(h, SPECKV_ERR_DEVICE, "handle has no device");
    hipError_t e = launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "probe_copy launch");
    return SPECKV_OK;
}

} // extern "C"
