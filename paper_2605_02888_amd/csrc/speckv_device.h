// Device-side helpers: stored-dtype decoding, 16-byte vector unpacking, wave64 reductions,
// Philox4x32-10.  gfx950 only (wave64).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <hip/hip_ext.h>

#include "speckv_internal.h"

namespace speckv {

// Launch `kernel` and return that launch's own status (not whatever error an earlier HIP call of
// the caller may have left behind); timed through the thread's launch events when the ABI layer set
// them.  The arguments are converted to the kernel's parameter types before their addresses are taken.
template <typename T> struct same_as { using type = T; };
// `lds` bytes of dynamic LDS are requested on top of what the kernel declares: a kernel that uses
// none of it still occupies it, which bounds the number of its workgroups per compute unit.
template <typename... KArgs>
inline hipError_t launch_lds(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                             typename same_as<KArgs>::type... args)
{
    void *argv[] = {const_cast<void *>(static_cast<const void *>(&args))...};
    const LaunchEvents ev = g_launch_events;
    if (ev.start && ev.stop)
        return hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, lds, stream, ev.start,
                                  ev.stop, 0);
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, lds, stream);
}
template <typename... KArgs>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream,
                         typename same_as<KArgs>::type... args)
{
    return launch_lds(kernel, grid, block, 0, stream, args...);
}

constexpr int kWave = 64;

// Measurement only: readings of the GPU's constant-rate clock by one thread of a workgroup, stored
// into that workgroup's slots of a trace buffer.  Nothing is stored while the buffer is null (the
// usual case), so the branch is uniform and costs one scalar compare.
constexpr int kTraceSlots = 32;
struct Trace {
    unsigned long long *slots; // this workgroup's kTraceSlots words, or null
    __device__ __forceinline__ void mark(int k, bool writer) const
    {
        if (slots) {
            __builtin_amdgcn_s_waitcnt(0); // what was issued before this point has completed
            __builtin_amdgcn_sched_barrier(0);
            if (writer) slots[k] = wall_clock64();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
};

// ---- element types ---------------------------------------------------------------------------
// DT is a speckv_dtype value.  NE = elements per 16-byte vector.
template <int DT> struct Elem;
template <> struct Elem<SPECKV_F32> {
    using type = float;
    static constexpr int NE = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ float load1(const void *base, int64_t i)
    {
        return static_cast<const float *>(base)[i];
    }
    __device__ static __forceinline__ void unpack(const uint4 &w, float *x)
    {
        x[0] = __uint_as_float(w.x);
        x[1] = __uint_as_float(w.y);
        x[2] = __uint_as_float(w.z);
        x[3] = __uint_as_float(w.w);
    }
};
template <> struct Elem<SPECKV_BF16> {
    using type = uint16_t;
    static constexpr int NE = 8;
    static constexpr int BYTES = 2;
    __device__ static __forceinline__ float load1(const void *base, int64_t i)
    {
        return __uint_as_float((uint32_t) static_cast<const uint16_t *>(base)[i] << 16);
    }
    // bfloat16 is the upper half of a binary32: one shift or one mask per element.
    __device__ static __forceinline__ void unpack(const uint4 &w, float *x)
    {
        x[0] = __uint_as_float(w.x << 16);
        x[1] = __uint_as_float(w.x & 0xffff0000u);
        x[2] = __uint_as_float(w.y << 16);
        x[3] = __uint_as_float(w.y & 0xffff0000u);
        x[4] = __uint_as_float(w.z << 16);
        x[5] = __uint_as_float(w.z & 0xffff0000u);
        x[6] = __uint_as_float(w.w << 16);
        x[7] = __uint_as_float(w.w & 0xffff0000u);
    }
};
template <> struct Elem<SPECKV_F16> {
    using type = uint16_t;
    static constexpr int NE = 8;
    static constexpr int BYTES = 2;
    __device__ static __forceinline__ float load1(const void *base, int64_t i)
    {
        return __half2float(static_cast<const __half *>(base)[i]);
    }
    __device__ static __forceinline__ void unpack(const uint4 &w, float *x)
    {
        const __half2 *h = reinterpret_cast<const __half2 *>(&w);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float2 f = __half22float2(h[k]);
            x[2 * k] = f.x;
            x[2 * k + 1] = f.y;
        }
    }
};

__device__ __forceinline__ float exp2_hw(float t) { return __builtin_amdgcn_exp2f(t); }

// max(a, b, c) in one instruction.  Written out because fmaxf on values that were assembled from
// integer bit patterns makes the compiler insert a quieting instruction per operand.  A NaN
// operand is ignored, like fmaxf.
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// max(m, x[0..N-1])
template <int N> __device__ __forceinline__ float max_into(float m, const float (&x)[N])
{
#pragma unroll
    for (int k = 0; k + 1 < N; k += 2) m = max3(m, x[k], x[k + 1]);
    if (N & 1) m = max3(m, x[N - 1], x[N - 1]);
    return m;
}

// ---- wave64 reductions (every lane ends with the result) ---------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// The same sum by data-parallel-primitive moves instead of LDS permutes: four shifts inside each row
// of 16 lanes, then the row totals are passed on to the rows behind (row_bcast 15 into rows 1 and 3,
// row_bcast 31 into rows 2 and 3), which leaves the wave's total in lane 63.  A third of the
// instructions of wave_sum; used where a wave reduces once per few thousand elements.  (The order of
// the additions differs from wave_sum's, so the two are not interchangeable bit for bit.)
template <int CTRL, int ROW_MASK> __device__ __forceinline__ double dpp_shifted(double v)
{
    // lanes without a source, and rows outside ROW_MASK, receive 0
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xf, true);
    return __hiloint2double(hi, lo);
}
// Inclusive prefix sum over the 64 lanes by the same moves: the four shifts leave every row of 16
// lanes with its own inclusive sums (a lane without a source adds 0), then the rows behind receive
// the totals of the rows in front.
__device__ __forceinline__ double wave_inclusive_scan_dpp(double v)
{
    v += dpp_shifted<0x111, 0xf>(v); // row_shr:1
    v += dpp_shifted<0x112, 0xf>(v); // row_shr:2
    v += dpp_shifted<0x114, 0xf>(v); // row_shr:4
    v += dpp_shifted<0x118, 0xf>(v); // row_shr:8
    v += dpp_shifted<0x142, 0xa>(v); // row_bcast:15: rows 1 and 3 add the total of the row in front
    v += dpp_shifted<0x143, 0xc>(v); // row_bcast:31: rows 2 and 3 add the total of rows 0 and 1
    return v;
}
// The value lane `src` holds, in every lane; `src` must be the same in all lanes.
__device__ __forceinline__ double wave_read_lane(double v, int src)
{
    const int s = __builtin_amdgcn_readfirstlane(src);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), s);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), s);
    return __hiloint2double(hi, lo);
}
// Largest value of the wave, in every lane.
__device__ __forceinline__ int wave_max_int_dpp(int v)
{
    constexpr int lowest = -2147483647 - 1; // what a lane without a source, or a row not addressed, takes part with
    v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x111, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x112, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x114, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x118, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x142, 0xa, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x143, 0xc, 0xf, false));
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ double wave_sum_dpp(double v)
{
    v += dpp_shifted<0x111, 0xf>(v); // row_shr:1
    v += dpp_shifted<0x112, 0xf>(v); // row_shr:2
    v += dpp_shifted<0x114, 0xf>(v); // row_shr:4
    v += dpp_shifted<0x118, 0xf>(v); // row_shr:8: lane 15 of each row holds the row's sum
    v += dpp_shifted<0x142, 0xa>(v); // row_bcast:15 into rows 1 and 3
    v += dpp_shifted<0x143, 0xc>(v); // row_bcast:31 into rows 2 and 3: lane 63 holds the total
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

// ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) ---------------------------------------
struct Philox4 {
    uint32_t w[4];
};
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

// ---- statistics algebra ----------------------------------------------------------------------
// Re-express (S, T) given relative to `ref` relative to `new_ref` >= ref (both integer valued,
// or ref = -inf for an empty state).  Exact up to the rounding of one fused multiply-add.
__device__ __forceinline__ void rebase(double &S, double &T, float ref, float new_ref)
{
    if (!(ref > -INFINITY)) { // nothing finite has been seen: an empty state, unless a NaN went by
        S = S != S ? S : 0.0; // (a NaN among nothing but -inf leaves the reference at -inf: keep it visible)
        T = 0.0;
        return;
    }
    const float d = fmaxf(ref - new_ref, -4000.0f); // <= 0; a huge gap underflows to zero below
    const int sh = (int)d;
    T = ldexp(fma((double)d, S, T), sh);
    S = ldexp(S, sh);
}

// Merge b into a.
__device__ __forceinline__ void merge_stat(RowStat &a, const RowStat &b)
{
    const float R = fmaxf(a.ref, b.ref);
    double Sa = a.S, Ta = a.T, Sb = b.S, Tb = b.T;
    rebase(Sa, Ta, a.ref, R);
    rebase(Sb, Tb, b.ref, R);
    a.S = Sa + Sb;
    a.T = Ta + Tb;
    a.ref = R;
    if (b.vmax > a.vmax) { // strict: chunks are merged in ascending order, lowest index wins
        a.vmax = b.vmax;
        a.argmax = b.argmax;
    }
}

// Merge the `split` chunk statistics of one row, in chunk order.  Loads go out eight at a time so
// that a row costs one or two memory round trips rather than `split` of them.
__device__ __forceinline__ RowStat merge_partials(const RowStat *p, int split)
{
    RowStat a = p[0];
    for (int c0 = 1; c0 < split; c0 += 8) {
        RowStat t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (c0 + k < split) t[k] = p[c0 + k];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (c0 + k < split) merge_stat(a, t[k]);
    }
    return a;
}

} // namespace speckv
