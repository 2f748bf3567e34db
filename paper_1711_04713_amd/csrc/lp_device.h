// Device-side helpers shared by the gfx950 kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lp.h"

namespace lp {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef short v2s __attribute__((ext_vector_type(2)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

// Requantization parameters of the LPAct step (Sec. 2.1): divide by 2^s,
// round to nearest, clip to [lo, hi].
struct ActParams {
    int s;        // f_acc - f_out; > 0 shifts right, <= 0 shifts left
    int relu;     // clamp negatives to zero first
    int even;     // tie rule: 0 away from zero, 1 to even
    int lo, hi;   // code range of the output format
};

__host__ inline ActParams make_act_params(int f_acc, lp_qfmt qy, int relu, lp_round r)
{
    ActParams a;
    a.s = f_acc - qy.f;
    a.relu = relu ? 1 : 0;
    a.even = (r == LP_ROUND_NEAREST_EVEN) ? 1 : 0;
    a.lo = -(1 << (qy.n - 1));
    a.hi = (1 << (qy.n - 1)) - 1;
    return a;
}

// One accumulator -> one output code.  |v| < 2^62.  sat: the rounded value lay outside
// [lo, hi] and was clipped.
__device__ __forceinline__ int act_one(int64_t v, const ActParams &p, bool &sat)
{
    if (p.relu && v < 0) v = 0;
    int64_t r;
    if (p.s > 0) {
        const int64_t half = (int64_t)1 << (p.s - 1);
        if (!p.even) {
            const int64_t mag = v < 0 ? -v : v;
            const int64_t q = (mag + half) >> p.s;
            r = v < 0 ? -q : q;
        } else {
            int64_t q = v >> p.s;                       // floor
            const int64_t rem = v & (((int64_t)1 << p.s) - 1);
            if (rem > half || (rem == half && (q & 1))) q += 1;
            r = q;
        }
    } else {
        // beyond the code range the product stays beyond it: one step outside keeps it in 64 bits
        int64_t c = v;
        if (c > p.hi) c = (int64_t)p.hi + 1;
        if (c < p.lo) c = (int64_t)p.lo - 1;
        r = c * ((int64_t)1 << (-p.s));
    }
    sat = r > p.hi || r < p.lo;
    if (r > p.hi) r = p.hi;
    if (r < p.lo) r = p.lo;
    return (int)r;
}

__device__ __forceinline__ int act_one(int64_t v, const ActParams &p)
{
    bool sat;
    return act_one(v, p, sat);
}

// Number of lanes of the wavefront for which pred holds (ballot + popcount).
__device__ __forceinline__ unsigned wave_count(bool pred)
{
    return (unsigned)__popcll(__ballot(pred));
}

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline bool fmt_ok(lp_qfmt q)
{
    return q.n >= 2 && q.n <= 16 && q.m >= 1 && q.m <= q.n && q.f >= 0 && q.n == q.m + q.f;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Status of the launches this call has made.  clear_stale_error() at the call's entry drops an
// error that an earlier, unrelated HIP call left pending, so that it is not reported as this
// call's.
inline void clear_stale_error() { (void)hipGetLastError(); }
inline lp_status launch_status()
{
    return hipGetLastError() == hipSuccess ? LP_OK : LP_EDEVICE;
}

} // namespace lp
