// HBM-bound kernels of the low-precision forward pass: quantize, dynamic-range
// histogram, standalone LPAct, 2x2 max-pool.  Each thread moves 16-byte vectors;
// counters use the wave ballot (a v_cmp result) + popcount and one atomic per wave.
#include <algorithm>

#include "lp_device.h"

namespace lp {

constexpr int kThreads = 256;

static int grid_for(size_t groups)
{
    // enough blocks to fill 256 CUs several times over, grid-stride beyond that
    size_t blocks = (groups + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 16) blocks = 256 * 16;
    return (int)blocks;
}

// ------------------------------------------------------------------ Philox4x32-10
// Counter-based generator of Salmon, Moraes, Dror, Shaw (SC'11): ten rounds of two
// 32x32->64 multiplies and xors, key bumped by the Weyl constants each round.  One block gives four
// words; element i of a tensor draws word i % 4 of the block with counter (i / 4, 0).
struct PhiloxBlock {
    uint32_t w[4];
};
__device__ __forceinline__ PhiloxBlock philox4x32_10(uint64_t ctr, uint64_t key)
{
    uint32_t c0 = (uint32_t)ctr, c1 = (uint32_t)(ctr >> 32), c2 = 0, c3 = 0;
    uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return PhiloxBlock{{c0, c1, c2, c3}};
}
// the draw of element i by itself (ragged tails)
__device__ __forceinline__ uint32_t philox_draw(uint64_t i, uint64_t key)
{
    const PhiloxBlock b = philox4x32_10(i >> 2, key);
    const unsigned k = (unsigned)i & 3u;
    return k == 0 ? b.w[0] : k == 1 ? b.w[1] : k == 2 ? b.w[2] : b.w[3];
}

// ------------------------------------------------------------------------ quantize

template <int MODE>
__device__ __forceinline__ int quantize_one(float x, float scale, float lo, float hi, uint32_t w, bool &sat)
{
    const float t = x * scale; // exact: scale is a power of two
    float r;
    if (MODE == LP_ROUND_NEAREST_AWAY) {
        r = roundf(t);
    } else if (MODE == LP_ROUND_NEAREST_EVEN) {
        r = rintf(t);
    } else {
        // the fractional part in double: t has 24 significant bits, and for a negative t just
        // below zero t - floor(t) needs more than float holds (-0.25 + 2^-26 -> 0.75 + 2^-26)
        const float fl = floorf(t);
        const double frac = (double)t - (double)fl; // exact
        r = ((double)w < frac * 4294967296.0) ? fl + 1.0f : fl; // w: the element's draw
    }
    if (t != t) r = 0.0f;
    sat = (r < lo) || (r > hi);
    r = fminf(fmaxf(r, lo), hi);
    return (int)r;
}

template <typename OutT, int MODE, bool COUNT>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float *__restrict__ x,
                                                           OutT *__restrict__ y, size_t count,
                                                           float scale, float lo, float hi,
                                                           uint64_t seed,
                                                           unsigned long long *zero_count,
                                                           unsigned long long *sat_count)
{
    const size_t groups = count / 8;
    unsigned zeros = 0, sats = 0; // wave-uniform running totals
    // lane 0 of a wave has the smallest index, so it runs every iteration any lane of its
    // wave runs and its running totals see every ballot
    for (size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x; g < groups;
         g += (size_t)gridDim.x * kThreads) {
        int c[8];
        bool z[8], s[8];
        {
            const v4f a = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(x) + 2 * g);
            const v4f b = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(x) + 2 * g + 1);
            const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            // elements 8g .. 8g+7 draw the words of blocks 2g and 2g+1
            PhiloxBlock d0 = {}, d1 = {};
            if constexpr (MODE == LP_ROUND_STOCHASTIC) {
                d0 = philox4x32_10(2 * g, seed);
                d1 = philox4x32_10(2 * g + 1, seed);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                c[j] = quantize_one<MODE>(v[j], scale, lo, hi, j < 4 ? d0.w[j & 3] : d1.w[j & 3], s[j]);
                z[j] = (c[j] == 0);
            }
            if (sizeof(OutT) == 2) {
                v4i o;
                o.x = (c[0] & 0xffff) | (c[1] << 16);
                o.y = (c[2] & 0xffff) | (c[3] << 16);
                o.z = (c[4] & 0xffff) | (c[5] << 16);
                o.w = (c[6] & 0xffff) | (c[7] << 16);
                reinterpret_cast<v4i *>(y)[g] = o;
            } else {
                v2i o;
                o.x = (c[0] & 0xff) | ((c[1] & 0xff) << 8) | ((c[2] & 0xff) << 16) | (c[3] << 24);
                o.y = (c[4] & 0xff) | ((c[5] & 0xff) << 8) | ((c[6] & 0xff) << 16) | (c[7] << 24);
                reinterpret_cast<v2i *>(y)[g] = o;
            }
        }
        if (COUNT) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                zeros += wave_count(z[j]);
                sats += wave_count(s[j]);
            }
        }
    }
    // ragged tail (fewer than 8 elements): first wave of block 0
    if (blockIdx.x == 0 && threadIdx.x < 64) {
        const size_t i = groups * 8 + threadIdx.x;
        bool z = false, s = false;
        if (threadIdx.x < 8 && i < count) {
            const int c = quantize_one<MODE>(x[i], scale, lo, hi, MODE == LP_ROUND_STOCHASTIC ? philox_draw(i, seed) : 0u, s);
            y[i] = (OutT)c;
            z = (c == 0);
        }
        if (COUNT) {
            zeros += wave_count(z);
            sats += wave_count(s);
        }
    }
    if (COUNT && (threadIdx.x & 63) == 0) {
        if (zero_count && zeros) atomicAdd(zero_count, (unsigned long long)zeros);
        if (sat_count && sats) atomicAdd(sat_count, (unsigned long long)sats);
    }
}

template <typename OutT, int MODE>
static void launch_quantize(const float *x, void *y, size_t count, float scale, float lo, float hi,
                            uint64_t seed, uint64_t *zc, uint64_t *sc, hipStream_t st)
{
    const int grid = grid_for(count / 8);
    if (zc || sc)
        hipLaunchKernelGGL((quantize_kernel<OutT, MODE, true>), dim3(grid), dim3(kThreads), 0, st, x,
                           (OutT *)y, count, scale, lo, hi, seed, (unsigned long long *)zc,
                           (unsigned long long *)sc);
    else
        hipLaunchKernelGGL((quantize_kernel<OutT, MODE, false>), dim3(grid), dim3(kThreads), 0, st, x,
                           (OutT *)y, count, scale, lo, hi, seed, nullptr, nullptr);
}

// --------------------------------------------------------------------------- range
// Bucket b of a value = the smallest m (integer bits incl. sign) for which it is not
// lost, i.e. |v| < 2^(b-1); b in 1..17, 17 collecting everything that needs more than
// 16.  Each thread owns one column of an LDS histogram, so there are no conflicts.

constexpr int kBuckets = 18;

__device__ __forceinline__ int bucket_f32(float v)
{
    const uint32_t bits = __float_as_uint(v) & 0x7fffffffu;
    if (bits > 0x7f800000u) return 1; // NaN: never counted as lost
    const int e = (int)(bits >> 23) - 127;
    if (e < 0) return 1;
    return e + 2 > 17 ? 17 : e + 2;
}

__device__ __forceinline__ int bucket_i64(int64_t a, int f_acc, int relu)
{
    if (relu && a < 0) a = 0;
    const uint64_t mag = (uint64_t)(a < 0 ? -a : a);
    if ((mag >> f_acc) == 0) return 1; // |v| < 1
    const int top = 63 - __clzll((long long)mag); // floor(log2 mag)
    const int b = top - f_acc + 2;
    return b > 17 ? 17 : b;
}

// Column sums of a block's histogram, then one global atomic per non-empty bucket and block
// (the launch keeps the number of blocks small: thousands of atomics on 17 addresses would
// cost more than reading the tensor).
__device__ __forceinline__ void flush_hist(unsigned *h, unsigned long long *hist_out)
{
    __shared__ unsigned long long part_sum[(kBuckets - 1) * 8];
    __syncthreads();
    const int t = threadIdx.x;
    if (t < (kBuckets - 1) * 8) {
        const int b = 1 + t / 8, part = t % 8;
        unsigned long long sum = 0;
        for (int i = 0; i < kThreads / 8; ++i) sum += h[b * kThreads + part * (kThreads / 8) + i];
        part_sum[t] = sum;
    }
    __syncthreads();
    if (t < kBuckets - 1) {
        unsigned long long sum = 0;
        for (int i = 0; i < 8; ++i) sum += part_sum[t * 8 + i];
        if (sum) atomicAdd(&hist_out[1 + t], sum);
    }
}

// one LDS add without return value per element: nothing to wait for
__device__ __forceinline__ void count_in(unsigned *h, int bucket)
{
    __hip_atomic_fetch_add(&h[bucket * kThreads + threadIdx.x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

static int range_grid(size_t groups)
{
    size_t blocks = (groups + kThreads - 1) / kThreads;
    return (int)std::min<size_t>(std::max<size_t>(blocks, 1), 256 * 2); // grid-stride beyond two blocks per CU
}

__global__ __launch_bounds__(kThreads) void range_f32_kernel(const float *__restrict__ x, size_t count,
                                                            unsigned long long *hist_out)
{
    __shared__ unsigned h[kBuckets * kThreads];
    for (int b = 0; b < kBuckets; ++b) h[b * kThreads + threadIdx.x] = 0;
    // columns are private to a thread: no barrier needed before use
    // four 16-byte requests per thread in flight: one per trip leaves the memory system idle most of
    // the time (a trip's work is a handful of instructions)
    const size_t groups = count / 4, stride = (size_t)gridDim.x * kThreads;
    constexpr int U = 4;
    size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;
    for (; g + (U - 1) * stride < groups; g += U * stride) {
        v4f a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(x) + g + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            count_in(h, bucket_f32(a[u].x));
            count_in(h, bucket_f32(a[u].y));
            count_in(h, bucket_f32(a[u].z));
            count_in(h, bucket_f32(a[u].w));
        }
    }
    for (; g < groups; g += stride) {
        const v4f a = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(x) + g);
        count_in(h, bucket_f32(a.x));
        count_in(h, bucket_f32(a.y));
        count_in(h, bucket_f32(a.z));
        count_in(h, bucket_f32(a.w));
    }
    if (blockIdx.x == 0 && threadIdx.x < 4) {
        const size_t i = groups * 4 + threadIdx.x;
        if (i < count) count_in(h, bucket_f32(x[i]));
    }
    flush_hist(h, hist_out);
}

__global__ __launch_bounds__(kThreads) void range_i64_kernel(const int64_t *__restrict__ acc,
                                                            size_t count, int f_acc, int relu,
                                                            unsigned long long *hist_out)
{
    __shared__ unsigned h[kBuckets * kThreads];
    for (int b = 0; b < kBuckets; ++b) h[b * kThreads + threadIdx.x] = 0;
    const size_t groups = count / 2, stride = (size_t)gridDim.x * kThreads;
    constexpr int U = 4; // requests in flight per thread (see range_f32_kernel)
    auto take = [&](const v4i &a) __attribute__((always_inline)) {
        const int64_t a0 = (int64_t)(((uint64_t)(uint32_t)a.y << 32) | (uint32_t)a.x);
        const int64_t a1 = (int64_t)(((uint64_t)(uint32_t)a.w << 32) | (uint32_t)a.z);
        count_in(h, bucket_i64(a0, f_acc, relu));
        count_in(h, bucket_i64(a1, f_acc, relu));
    };
    size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;
    for (; g + (U - 1) * stride < groups; g += U * stride) {
        v4i a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(acc) + g + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) take(a[u]);
    }
    for (; g < groups; g += stride) take(__builtin_nontemporal_load(reinterpret_cast<const v4i *>(acc) + g));
    if (blockIdx.x == 0 && threadIdx.x == 0 && (count & 1)) count_in(h, bucket_i64(acc[count - 1], f_acc, relu));
    flush_hist(h, hist_out);
}

__global__ void clear_words_kernel(unsigned long long *p, int words)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0;
}

// Host side of the rule of Sec. 2.3: smallest m whose lost share is within the threshold.
static void pick_format(const unsigned long long *hist, size_t count, int n, double threshold,
                        lp_qfmt *out, uint64_t *lost_host)
{
    int chosen = n;
    bool found = false;
    for (int m = 1; m <= n; ++m) {
        unsigned long long lost = 0;
        for (int b = m + 1; b < kBuckets; ++b) lost += hist[b];
        if (lost_host) lost_host[m] = lost;
        if (!found && (double)lost <= threshold * (double)count) {
            chosen = m;
            found = true;
        }
    }
    if (lost_host) lost_host[0] = 0;
    out->n = n;
    out->m = chosen;
    out->f = n - chosen;
}

static lp_status finish_range(unsigned long long *hist_dev, size_t count, int n, double threshold,
                              lp_qfmt *out, uint64_t *lost_host, hipStream_t st)
{
    if (hipGetLastError() != hipSuccess) return LP_EDEVICE;
    unsigned long long hist[LP_RANGE_WORKSPACE_WORDS];
    if (hipMemcpyAsync(hist, hist_dev, sizeof(hist), hipMemcpyDeviceToHost, st) != hipSuccess)
        return LP_EDEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return LP_EDEVICE;
    pick_format(hist, count, n, threshold, out, lost_host);
    return LP_OK;
}

// ----------------------------------------------------------------------------- act

// Sec. 2.4 on an accumulator: floor(v / 2^s) + [u < frac], u = 2^-32 * the element's Philox draw
// w32; the comparison u * 2^s < rem is done in integers (rem < 2^s <= 2^62).
__device__ __forceinline__ int act_one_stochastic(int64_t v, const ActParams &p, uint32_t w32, bool &sat)
{
    if (p.relu && v < 0) v = 0;
    int64_t r;
    if (p.s > 0) {
        int64_t q = v >> p.s; // floor
        const uint64_t rem = (uint64_t)v & (((uint64_t)1 << p.s) - 1);
        const uint64_t w = w32;
        const bool up = p.s >= 32 ? (w << (p.s - 32)) < rem : w < (rem << (32 - p.s));
        r = q + (up ? 1 : 0);
    } else {
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

template <typename OutT, bool STOCH>
__global__ __launch_bounds__(kThreads) void act_kernel(const int64_t *__restrict__ acc,
                                                      OutT *__restrict__ y, size_t count,
                                                      ActParams p, uint64_t seed,
                                                      unsigned long long *zero_count,
                                                      unsigned long long *sat_count)
{
    // counts are kept when either counter is wanted; a wave's totals are scalars
    const bool counting = zero_count || sat_count;
    unsigned sats = 0;
    // w: the element's draw (stochastic scheme only)
    auto one = [&](int64_t v, uint32_t w, bool &sat) {
        if constexpr (STOCH) return act_one_stochastic(v, p, w, sat);
        else return act_one(v, p, sat);
    };
    auto draw = [&](size_t index) { return STOCH ? philox_draw(index, seed) : 0u; };
    // A block takes 8 * kThreads consecutive accumulators per trip, as four rows of kThreads
    // 16-byte pairs: a lane's loads are 16 bytes apart from its neighbours' (1 KB contiguous per
    // wave and instruction), and it stores the two codes of each pair (4 or 2 bytes, again
    // contiguous over the wave).
    const size_t groups = count / 8;            // whole groups of 8; the rest is handled below
    const size_t trips = groups / kThreads;     // whole block trips
    unsigned zeros = 0;
    for (size_t t = blockIdx.x; t < trips; t += gridDim.x) {
        const size_t pair0 = t * (4 * kThreads) + threadIdx.x;
        v4i a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            a[j] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(acc) + pair0 + j * kThreads);
        // Elements 2 * pair and 2 * pair + 1 draw two neighbouring words of block pair / 2, which a
        // lane shares with its neighbour (lanes 2k and 2k + 1 hold pairs 2m and 2m + 1 in every
        // row).  The even lane computes the blocks of rows 0 and 2, the odd lane those of rows 1
        // and 3, and each hands the other its half of the words: two blocks per lane, not four.
        const unsigned par = threadIdx.x & 1u; // = pair & 1 in every row (kThreads is even)
        PhiloxBlock blk[2] = {};
        if constexpr (STOCH) {
            blk[0] = philox4x32_10((pair0 + par * kThreads) >> 1, seed);
            blk[1] = philox4x32_10((pair0 + (2 + par) * kThreads) >> 1, seed);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t a0 = (int64_t)(((uint64_t)(uint32_t)a[j].y << 32) | (uint32_t)a[j].x);
            const int64_t a1 = (int64_t)(((uint64_t)(uint32_t)a[j].w << 32) | (uint32_t)a[j].z);
            const size_t pair = pair0 + j * kThreads;
            bool s0, s1;
            uint32_t w0 = 0, w1 = 0;
            if constexpr (STOCH) {
                const unsigned pj = j & 1;         // parity of the lanes that hold this row's block
                const PhiloxBlock &d = blk[j >> 1];
                // what the other lane needs: the odd lane words 2 and 3, the even lane words 0 and 1
                const uint32_t x0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)(pj == 0 ? d.w[2] : d.w[0]), 0xB1, 0xF, 0xF, true);
                const uint32_t x1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)(pj == 0 ? d.w[3] : d.w[1]), 0xB1, 0xF, 0xF, true);
                w0 = par == pj ? (pj == 0 ? d.w[0] : d.w[2]) : x0;
                w1 = par == pj ? (pj == 0 ? d.w[1] : d.w[3]) : x1;
            }
            const int c0 = one(a0, w0, s0), c1 = one(a1, w1, s1);
            if (sizeof(OutT) == 2)
                reinterpret_cast<int *>(y)[pair] = (c0 & 0xffff) | (c1 << 16);
            else
                reinterpret_cast<short *>(y)[pair] = (short)((c0 & 0xff) | (c1 << 8));
            if (counting) {
                zeros += wave_count(c0 == 0) + wave_count(c1 == 0);
                sats += wave_count(s0) + wave_count(s1);
            }
        }
    }
    // the groups that do not fill a block trip: one group of 8 per thread of block 0
    if (blockIdx.x == 0) {
        const size_t g = trips * kThreads + threadIdx.x;
        bool z[8] = {false, false, false, false, false, false, false, false};
        bool st[8] = {false, false, false, false, false, false, false, false};
        if (g < groups) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = one(acc[8 * g + j], draw(8 * g + j), st[j]);
                y[8 * g + j] = (OutT)c;
                z[j] = (c == 0);
            }
        }
        if (counting) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                zeros += wave_count(z[j]);
                sats += wave_count(st[j]);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 64) {
        const size_t i = groups * 8 + threadIdx.x;
        bool z = false, st = false;
        if (threadIdx.x < 8 && i < count) {
            const int c = one(acc[i], draw(i), st);
            y[i] = (OutT)c;
            z = (c == 0);
        }
        if (counting) {
            zeros += wave_count(z);
            sats += wave_count(st);
        }
    }
    if ((threadIdx.x & 63) == 0) {
        if (zero_count && zeros) atomicAdd(zero_count, (unsigned long long)zeros);
        if (sat_count && sats) atomicAdd(sat_count, (unsigned long long)sats);
    }
}

// ------------------------------------------------------------------------- maxpool

// One thread: one output pixel x one 16-byte channel group (8 int16 or 16 int8).
template <typename VecT>
__global__ __launch_bounds__(kThreads) void maxpool_vec_kernel(const VecT *__restrict__ x,
                                                              VecT *__restrict__ y, int Ho, int Wo,
                                                              int Cv, size_t total)
{
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (size_t)gridDim.x * kThreads) {
        const int c = (int)(i % Cv);
        size_t t = i / Cv;
        const int xo = (int)(t % Wo);
        t /= Wo; // t = n*Ho + yo
        const size_t W = (size_t)2 * Wo;
        const size_t base = ((2 * t) * W + 2 * xo) * Cv + c;
        const VecT a = x[base], b = x[base + Cv], d = x[base + W * Cv], e = x[base + W * Cv + Cv];
        y[i] = __builtin_elementwise_max(__builtin_elementwise_max(a, b),
                                         __builtin_elementwise_max(d, e));
    }
    (void)Ho;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool_scalar_kernel(const T *__restrict__ x,
                                                                 T *__restrict__ y, int Wo, int C,
                                                                 size_t total)
{
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (size_t)gridDim.x * kThreads) {
        const int c = (int)(i % C);
        size_t t = i / C;
        const int xo = (int)(t % Wo);
        t /= Wo;
        const size_t W = (size_t)2 * Wo;
        const size_t base = ((2 * t) * W + 2 * xo) * C + c;
        T m = x[base];
        const T b = x[base + C], d = x[base + W * C], e = x[base + W * C + C];
        m = b > m ? b : m;
        m = d > m ? d : m;
        m = e > m ? e : m;
        y[i] = m;
    }
}

} // namespace lp

using namespace lp;

extern "C" const char *lp_status_string(lp_status s)
{
    switch (s) {
    case LP_OK: return "ok";
    case LP_EINVAL: return "invalid argument";
    case LP_EUNSUPPORTED: return "unsupported problem";
    case LP_EWORKSPACE: return "workspace or packed buffer too small";
    case LP_EDEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" lp_status lp_range(const float *x_dev, size_t count, int n, double loss_threshold,
                              lp_qfmt *out_host, uint64_t *lost_host, uint64_t *workspace_dev,
                              void *stream)
{
    if (!out_host || !workspace_dev || n < 2 || n > 16 || !(loss_threshold >= 0.0)) return LP_EINVAL;
    if (count && (!x_dev || !aligned16(x_dev))) return LP_EINVAL;
    hipStream_t st = as_stream(stream);
    clear_stale_error();
    unsigned long long *hist = (unsigned long long *)workspace_dev;
    hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, st, hist, LP_RANGE_WORKSPACE_WORDS);
    if (count)
        hipLaunchKernelGGL(range_f32_kernel, dim3(range_grid(count / 4)), dim3(kThreads), 0, st, x_dev,
                           count, hist);
    return finish_range(hist, count, n, loss_threshold, out_host, lost_host, st);
}

extern "C" lp_status lp_range_acc(const int64_t *acc_dev, size_t count, int f_acc, int relu, int n,
                                  double loss_threshold, lp_qfmt *out_host, uint64_t *lost_host,
                                  uint64_t *workspace_dev, void *stream)
{
    if (!out_host || !workspace_dev || n < 2 || n > 16 || !(loss_threshold >= 0.0) || f_acc < 0 ||
        f_acc > 40)
        return LP_EINVAL;
    if (count && (!acc_dev || !aligned16(acc_dev))) return LP_EINVAL;
    hipStream_t st = as_stream(stream);
    clear_stale_error();
    unsigned long long *hist = (unsigned long long *)workspace_dev;
    hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, st, hist, LP_RANGE_WORKSPACE_WORDS);
    if (count)
        hipLaunchKernelGGL(range_i64_kernel, dim3(range_grid(count / 2)), dim3(kThreads), 0, st,
                           acc_dev, count, f_acc, relu ? 1 : 0, hist);
    return finish_range(hist, count, n, loss_threshold, out_host, lost_host, st);
}

extern "C" lp_status lp_quantize(const float *x_dev, void *codes_dev, size_t count, lp_qfmt q,
                                 lp_round r, uint64_t seed, uint64_t *zero_count_dev,
                                 uint64_t *sat_count_dev, void *stream)
{
    if (!fmt_ok(q) || (int)r < 0 || (int)r > 2) return LP_EINVAL;
    if (count == 0) return LP_OK;
    if (!x_dev || !codes_dev || !aligned16(x_dev) || !aligned16(codes_dev)) return LP_EINVAL;
    hipStream_t st = as_stream(stream);
    clear_stale_error();
    const float scale = (float)(1 << q.f);
    const float lo = -(float)(1 << (q.n - 1)), hi = (float)((1 << (q.n - 1)) - 1);
    const bool wide = q.n > 8;
#define LP_Q(T, M) launch_quantize<T, M>(x_dev, codes_dev, count, scale, lo, hi, seed, zero_count_dev, sat_count_dev, st)
    if (wide) {
        if (r == LP_ROUND_NEAREST_AWAY) LP_Q(int16_t, 0);
        else if (r == LP_ROUND_NEAREST_EVEN) LP_Q(int16_t, 1);
        else LP_Q(int16_t, 2);
    } else {
        if (r == LP_ROUND_NEAREST_AWAY) LP_Q(int8_t, 0);
        else if (r == LP_ROUND_NEAREST_EVEN) LP_Q(int8_t, 1);
        else LP_Q(int8_t, 2);
    }
#undef LP_Q
    return launch_status();
}

static lp_status act_launch(const int64_t *acc_dev, size_t count, int f_acc, lp_qfmt qy, int relu,
                            lp_round r, uint64_t seed, void *y_codes_dev, uint64_t *zero_count_dev,
                            uint64_t *sat_count_dev, void *stream)
{
    if (!fmt_ok(qy) || f_acc < 0) return LP_EINVAL;
    const int s = f_acc - qy.f;
    if (s > 62 || s < -31) return LP_EINVAL;
    if (count == 0) return LP_OK;
    if (!acc_dev || !y_codes_dev || !aligned16(acc_dev) || !aligned16(y_codes_dev)) return LP_EINVAL;
    hipStream_t st = as_stream(stream);
    clear_stale_error();
    const ActParams p = make_act_params(f_acc, qy, relu, r);
    const int grid = grid_for(count / 8); // one trip of the kernel's loop per block, up to the cap
#define LP_A(T, STOCH) \
    hipLaunchKernelGGL((act_kernel<T, STOCH>), dim3(grid), dim3(kThreads), 0, st, acc_dev, \
                       (T *)y_codes_dev, count, p, seed, (unsigned long long *)zero_count_dev, \
                       (unsigned long long *)sat_count_dev)
    if (r == LP_ROUND_STOCHASTIC) {
        if (qy.n > 8) LP_A(int16_t, true);
        else LP_A(int8_t, true);
    } else {
        if (qy.n > 8) LP_A(int16_t, false);
        else LP_A(int8_t, false);
    }
#undef LP_A
    return launch_status();
}

extern "C" lp_status lp_act(const int64_t *acc_dev, size_t count, int f_acc, lp_qfmt qy, int relu,
                            lp_round r, void *y_codes_dev, uint64_t *zero_count_dev,
                            uint64_t *sat_count_dev, void *stream)
{
    if (r != LP_ROUND_NEAREST_AWAY && r != LP_ROUND_NEAREST_EVEN) return LP_EINVAL;
    return act_launch(acc_dev, count, f_acc, qy, relu, r, 0, y_codes_dev, zero_count_dev, sat_count_dev, stream);
}

extern "C" lp_status lp_act_stochastic(const int64_t *acc_dev, size_t count, int f_acc, lp_qfmt qy,
                                       int relu, uint64_t seed, void *y_codes_dev,
                                       uint64_t *zero_count_dev, uint64_t *sat_count_dev, void *stream)
{
    return act_launch(acc_dev, count, f_acc, qy, relu, LP_ROUND_STOCHASTIC, seed, y_codes_dev,
                      zero_count_dev, sat_count_dev, stream);
}

extern "C" lp_status lp_maxpool2x2(const void *x_codes_dev, void *y_codes_dev, int N, int H, int W,
                                   int C, int n_bits, void *stream)
{
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1) || n_bits < 2 || n_bits > 16)
        return LP_EINVAL;
    if (!x_codes_dev || !y_codes_dev || !aligned16(x_codes_dev) || !aligned16(y_codes_dev))
        return LP_EINVAL;
    hipStream_t st = as_stream(stream);
    clear_stale_error();
    const int Ho = H / 2, Wo = W / 2;
    const int per_vec = n_bits > 8 ? 8 : 16;
    typedef short s8v __attribute__((ext_vector_type(8)));
    typedef signed char c16v __attribute__((ext_vector_type(16)));
    if (C % per_vec == 0) {
        const int Cv = C / per_vec;
        const size_t total = (size_t)N * Ho * Wo * Cv;
        if (n_bits > 8)
            hipLaunchKernelGGL(maxpool_vec_kernel<s8v>, dim3(grid_for(total)), dim3(kThreads), 0, st,
                               (const s8v *)x_codes_dev, (s8v *)y_codes_dev, Ho, Wo, Cv, total);
        else
            hipLaunchKernelGGL(maxpool_vec_kernel<c16v>, dim3(grid_for(total)), dim3(kThreads), 0, st,
                               (const c16v *)x_codes_dev, (c16v *)y_codes_dev, Ho, Wo, Cv, total);
    } else {
        const size_t total = (size_t)N * Ho * Wo * C;
        if (n_bits > 8)
            hipLaunchKernelGGL(maxpool_scalar_kernel<int16_t>, dim3(grid_for(total)), dim3(kThreads), 0,
                               st, (const int16_t *)x_codes_dev, (int16_t *)y_codes_dev, Wo, C, total);
        else
            hipLaunchKernelGGL(maxpool_scalar_kernel<int8_t>, dim3(grid_for(total)), dim3(kThreads), 0,
                               st, (const int8_t *)x_codes_dev, (int8_t *)y_codes_dev, Wo, C, total);
    }
    return launch_status();
}
