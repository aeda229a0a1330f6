// The streaming accumulator shared by the row-statistics kernel and the token-proposal kernel:
// sums of 2^(x * log2e - ref) (and of the same times its exponent) over a stream of values, with one
// integer-valued reference per wave that follows the data.
//
// The 64 lanes of a wave share the reference `ref`: before a group of values is exponentiated its
// maximum is compared with the wave's limit, and only when some lane exceeds it (a uniform branch,
// taken a few times per chunk) the wave raises the reference to ceil(largest value * log2e), which
// rescales every lane's sums by an exact power of two.  The limit sits kRefSlack above the
// reference, so t = x*log2e - ref <= kRefSlack for every term: nothing can overflow, and the
// dominant terms of a peaked row have |t| <= kRefSlack + 1, which keeps their products e*t accurate
// enough for the entropy -- there a small difference of terms of size |t| -- to come out right.
#pragma once

#include "speckv_device.h"

namespace speckv {

constexpr float kRefSlack = 2.0f; // a term may exceed the reference by this many binary orders

struct LaneAcc {
    // shared by the 64 lanes of a wave (same value in every lane)
    float ref;   // integer valued, -inf before the first finite value
    float nref;  // -ref, or 0 while ref is -inf
    float xlim;  // (ref + kRefSlack) / log2e: a value above it needs a larger reference
    // per lane
    float s[4];
    float t[4];
    float vmax;  // largest value seen by this lane
    int vcode;   // where: (index << 2) | kind, kind 0 = tile of U vectors starting at vector `index`,
                 // 1 = single vector `index`, 2 = scalar element `index` (row-relative); -1 = none
};

__device__ __forceinline__ void lane_init(LaneAcc &a)
{
    a.ref = -INFINITY;
    a.nref = 0.0f;
    a.xlim = -INFINITY;
#pragma unroll
    for (int k = 0; k < 4; ++k) { a.s[k] = 0.0f; a.t[k] = 0.0f; }
    a.vmax = -INFINITY;
    a.vcode = -1;
}

__device__ __forceinline__ float uniform(float v) // the compiler may keep it in a scalar register
{
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(v)));
}

// Raise the wave's reference so that it covers `mv`, the largest value any lane is about to add.
// All 64 lanes.
template <bool WITH_T> __device__ __forceinline__ void wave_rescale(LaneAcc &a, float mv)
{
    const float need = uniform(ceilf(wave_max(mv) * L2E_F)); // +inf for +inf: the sums turn NaN
    const float d = fmaxf(a.ref - need, -512.0f); // -inf (first data) clamps; the sums are 0 then
    const int sh = (int)d;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (WITH_T) a.t[k] = ldexpf(fmaf(d, a.s[k], a.t[k]), sh);
        a.s[k] = ldexpf(a.s[k], sh);
    }
    a.ref = need;
    a.nref = -need;
    a.xlim = (need + kRefSlack) * (1.0f / L2E_F);
}

// One group of N values per lane, all 64 lanes of the wave: raise the reference if some lane's
// maximum asks for it, then exponentiate.  A lane without data passes -inf and SAFE.
// SAFE guards the entropy term against 0 * (-inf).
template <int N, bool WITH_T, bool SAFE> __device__ __forceinline__ float accum(LaneAcc &a, const float (&x)[N])
{
    const float mv = max_into<N>(-INFINITY, x);
    if (__builtin_amdgcn_ballot_w64(mv > a.xlim)) wave_rescale<WITH_T>(a, mv);
    const float nref = a.nref;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float t = fmaf(x[k], L2E_F, nref);
        const float e = exp2_hw(t);
        a.s[k & 3] += e;
        if (WITH_T) {
            if (SAFE)
                a.t[k & 3] = (e > 0.0f) ? fmaf(e, t, a.t[k & 3]) : a.t[k & 3];
            else
                a.t[k & 3] = fmaf(e, t, a.t[k & 3]);
        }
    }
    return mv;
}

} // namespace speckv
