// Pieces shared by the convolution and inner-product kernels: the kernel argument block, exact
// index division by run-time values, and the tile epilogue (limb combine, corrections, bias, LPAct,
// counters; Sec. 2 and 2.1 of the paper) that follows every int8-MFMA main loop.
#pragma once
#include <type_traits>

#include "lp_device.h"

namespace lp {

constexpr int kCUs = 256;    // compute units of the chip the launch geometry is tuned for
constexpr int kXCDs = 8;     // consecutive workgroup ids go round-robin to this many dies

static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// --------------------------------------------------------------------- kernel arguments

struct ConvArgs {
    const void *x;
    const unsigned char *wp;
    const int64_t *corr;
    const void *bias;
    int bias16, bias_shift;
    int64_t *acc_out;
    void *y;
    int y16;
    unsigned long long *zero_count, *sat_count; // either may be null
    unsigned *zero_partial; // per workgroup (MFMA path): [grid] zero counts, then [grid] counts of clipped
                            // values; summed by a second kernel
    int partial_stride;     // = grid
    int direct_counts;      // no partials: every workgroup adds its counts to zero_count / sat_count itself (small grids)
    int count_sat;          // sat_count is wanted: the epilogue also counts the values it clips
    int N, H, W, Cin, Cout, R, S, stride, pad;
    int Ho, Wo, Hp, FR;
    int RH, TW, PW, NPIXA, NTAB, APLANE, PITCH;
    int tiles_c, tiles_n, CoutP, nchunks, taps, ksteps, Kflat;
    // window-row kernel: K = 32 pieces per window row / in all (a multiple of 4), 16-code units per
    // patch row / per window row / per pixel
    int KHR, KHP, UPR, SU, CU;
    int total_work, per_xcd, full_per_xcd, split;
    unsigned char *partials; // tail tiles' partial accumulators, part_bytes per (tile, part)
    int part_bytes;
    // floor(2^32 / d) for the divisors the kernel's index arithmetic uses (see udivmod)
    unsigned mg_tiles_n, mg_tiles_c, mg_Ho, mg_Hp, mg_PW, mg_TW, mg_taps, mg_S, mg_Cin, mg_SC, mg_rowlen, mg_UPR, mg_CU;
    // Skipping of all-zero input (Sec. 3.1: the sparsity the low-precision layers produce is there
    // to be skipped).  zin: flags written by the layer that produced x, one byte per (pixel tile,
    // channel tile) of ITS output, 1 = the tile holds a nonzero code; its geometry: z_rh x z_tw
    // pixels (rows of the stacked output rows), z_tiles_c tiles per row of tiles, z_tiles_n channel
    // tiles of z_bn channels; z_scale = 2 when x is the 2x2-pooled output.  zout: this layer's own
    // flags [tiles_m][tiles_n].  skipped: += (tile, 64-channel chunk) pairs not multiplied.
    // wsum: [nchunks][CoutP] sums of the weight codes per chunk, for the correction of skipped chunks.
    const unsigned char *zin;
    int z_rh, z_tw, z_tiles_c, z_tiles_n, z_bn, z_scale;
    unsigned char *zout;
    unsigned long long *skipped;
    const int *wsum;
    int fast; // 32-bit requantization is exact for this call (see epilogue)
    int pool; // store the 2x2 maxima of the codes (planner guarantees the tile geometry)
    ActParams act;
};

// x / d and x % d for 0 <= x < 2^31, d >= 1, with m = floor(2^32 / d) from the host: the high half
// of x * m is the quotient or one below it, one compare settles it.  Five cheap operations
// instead of the float-reciprocal sequence a division by a run-time value compiles to (on scalars
// they run on the scalar unit).
__host__ inline unsigned udiv_magic(int d) { return d <= 1 ? 0xffffffffu : (unsigned)((1ull << 32) / (unsigned)d); }
__device__ __forceinline__ void udivmod(int x, int d, unsigned m, int &q, int &r)
{
    unsigned qq = __umulhi((unsigned)x, m);
    unsigned rr = (unsigned)x - qq * (unsigned)d;
    if (rr >= (unsigned)d) {
        ++qq;
        rr -= (unsigned)d;
    }
    q = (int)qq;
    r = (int)rr;
}

__device__ __forceinline__ int64_t bias_term(const ConvArgs &a, int co)
{
    if (!a.bias) return 0;
    const int b = a.bias16 ? (int)((const int16_t *)a.bias)[co] : (int)((const int8_t *)a.bias)[co];
    return (int64_t)b * ((int64_t)1 << a.bias_shift);
}

// One workgroup's count (which: 0 zero codes, 1 clipped values) goes to its slot of the partials, or,
// on small grids, straight to the caller's counter.
__device__ __forceinline__ void publish_count(const ConvArgs &a, int which, unsigned total)
{
    if (a.zero_partial) {
        a.zero_partial[which * a.partial_stride + blockIdx.x] = total;
    } else if (a.direct_counts && total) {
        unsigned long long *c = which ? a.sat_count : a.zero_count;
        if (c) atomicAdd(c, (unsigned long long)total);
    }
}

__device__ __forceinline__ v16i mfma_i8(v4i a, v4i b, v16i c)
{
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

// min(max(q, 0), cmax) for 0 <= cmax as the one instruction the hardware has for it (with cmax in
// a scalar register the compiler emits a max and a min).
__device__ __forceinline__ int clamp_code(int q, int cmax)
{
    int r;
    asm("v_med3_i32 %0, %1, 0, %2" : "=v"(r) : "v"(q), "s"(cmax));
    return r;
}

// Requantization of v = 65536*hi + lo16 (hi = floor(v / 65536), 0 <= lo16 < 65536) to
// floor((v + 2^(s-1)) / 2^s) in 32-bit arithmetic, 1 <= s <= 31; the caller clamps to [0, cmax]
// (negative v give 0: ReLU).  The value returned is exact wherever it lies inside the code range
// and stays on the same side of it wherever it does not.  S16: 0 for s >= 17 (lo16 cannot
// matter), 1 for s == 16, 2 for s <= 15.
template <int S16>
__device__ __forceinline__ int requant_relu32(int hi, int lo16, int s)
{
    int q;
    if (S16 == 0) {
        q = (hi + (1 << (s - 17))) >> (s - 16);
    } else if (S16 == 1) {
        q = hi + (lo16 >> 15);
    } else {
        // beyond 32768 the result saturates anyway, below 0 it is 0 anyway: kept inside, the
        // shifted value cannot leave 32 bits
        const int h = min(max(hi, -1), 32768);
        q = (h << (16 - s)) + ((lo16 + (1 << (s - 1))) >> s);
    }
    return q;
}

// Per-channel constants of a tile (weight correction + bias) into LDS, in the form the epilogue
// wants: three int32 planes (bits 16.., 8..15, 0..7) for the 32-bit epilogue, else int64.
// deadmask: chunks of 64 input channels that were skipped as all-zero; their share of the weight
// correction, 128 * sum(w over the chunk) - 16384 * (positions of the chunk), is taken out again
// (their limb products, which it would have cancelled, were never formed).
template <int BN, int THREADS>
__device__ __forceinline__ void build_colterms(const ConvArgs &a, int ntile, int *ctab, int limbs, unsigned deadmask = 0)
{
    for (int c = threadIdx.x; c < BN; c += THREADS) {
        const int colg = ntile * BN + c;
        int64_t t = colg < a.Cout ? a.corr[colg] + bias_term(a, colg) : 0;
        if (limbs == 2 && deadmask && colg < a.Cout) {
            for (unsigned rem = deadmask; rem; rem &= rem - 1) {
                const int ch = __builtin_ctz(rem);
                const int kc = a.taps * min(64, a.Cin - 64 * ch);
                t -= (int64_t)128 * a.wsum[(size_t)ch * a.CoutP + colg] - (int64_t)16384 * kc;
            }
        }
        if (a.fast) {
            // (shifts 9..16: the epilogue's rounding half 2^(s-1) rides in the constants, as 2^(s-9)
            // at the scale of v / 256; one limb: the top plane arrives clamped and at that scale,
            // the middle plane holds the low 16 bits)
            const bool mid = a.act.s >= 9 && a.act.s <= 16;
            const int half9 = mid ? 1 << (a.act.s - 9) : 0;
            if (mid && limbs == 1) {
                const int64_t top = t >> 16;
                const int topc = (int)(top > (1 << 22) ? (1 << 22) : top < -(1 << 22) ? -(1 << 22) : top);
                ctab[c] = topc * 256 + half9;
                ctab[BN + c] = (int)(t & 65535);
                ctab[2 * BN + c] = 0;
            } else {
                ctab[c] = (int)(t >> 16);
                ctab[BN + c] = (int)((t >> 8) & 255) + (limbs == 2 ? half9 : 0);
                ctab[2 * BN + c] = (int)(t & 255);
            }
        } else {
            ((int64_t *)ctab)[c] = t;
        }
    }
}

// Epilogue of one tile of output pixels x BN channels: combine limbs exactly, add corrections and
// bias, LPAct (or raw accumulators), count zeros.  The MFMAs are issued with the weights as the
// row operand, so in the 32x32 result layout a lane holds one output pixel (tile row row0 + mb*32
// + (lane & 31), row0 being the first tile row of the calling wave) and, in register v, channel
// 8*(v/4) + 4*(lane/32) + v%4 of its 32-channel block (the wave's blocks start at channel col0w
// of the tile): four consecutive channels per group of four registers, which leave as one 8-byte
// (4-byte) store.
// row_sum(m): sum of the codes under tile row m's window (two-limb only); outoff and ctab (see
// build_colterms) are LDS tables, complete and visible.  Returns the wave's counts of zero codes
// and (when a.count_sat) of values clipped at an end of the code range, the same in every lane.
// The accumulators passed in cover MBL of the wave's MB row blocks, starting at block mb0, and GL
// of the four channel groups, starting at group g0 (register 4*gl + e = channel 8*(g0+gl) +
// 4*(lane/32) + e): the main kernel passes everything (MBL = MB, GL = 4, mb0 = g0 = 0), the
// finishing kernel one (row block, channel group) at a time.
struct TileCounts {
    unsigned zeros, sats;
};

template <int LIMBS, int NB, int BN, int MBL, int GL, typename RowSum>
__device__ __forceinline__ TileCounts tile_epilogue(const ConvArgs &a, v16i (&acc)[MBL][NB][LIMBS == 2 ? 3 : 1],
                                                  RowSum row_sum, const int *outoff, const int *pooloff,
                                                  const int *ctab, int ntile, int row0, int col0w, int mb0, int g0)
{
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, kg = lane >> 5;
    unsigned nz = 0, ns = 0; // zero codes written / values clipped by this lane (at most 16 * MB * NB <= 64 each)
    unsigned wz = 0, wsat = 0; // counted for the whole wave (scalars: ballots and popcounts)
    int oo[MBL], po[MBL], rs[MBL];
#pragma unroll
    for (int mb = 0; mb < MBL; ++mb) {
        const int m = row0 + (mb0 + mb) * 32 + l32;
        oo[mb] = outoff[m];
        po[mb] = a.pool ? pooloff[m] : -1; // pooled output pixel, at the window's top-left lane only
        rs[mb] = (LIMBS == 2) ? row_sum(m) : 0;
    }
    if (a.fast) {
        // v = 2^16*A + 2^8*B + C with every piece in int32: the channel constant is split the same
        // way, 128*rowsum = 2^8*(rowsum >> 1) + 128*(rowsum & 1); then carries are pushed upward.
        // Shift class, code width and store mode are compile-time: about ten VALU operations per
        // value.  Stores go through a buffer descriptor that starts at the tile's first output
        // pixel (the smallest address of the tile) with 32-bit offsets from there; a lane with
        // nothing to store (a row outside the image, a padded channel, a lane that is not the
        // top-left of its pooling window) gets an offset past the descriptor and its store is
        // dropped: no branches, no 64-bit address arithmetic.
        const int s = a.act.s, cmax = a.act.hi;
        __builtin_assume(cmax >= 0);
        constexpr unsigned NOWHERE = 0x80000000u; // the descriptor never covers more than 2^31 - 1 bytes
        auto requant_tile = [&](auto s16c, auto y16c, auto modec, auto satc) __attribute__((always_inline)) {
            constexpr int S16 = decltype(s16c)::value;
            constexpr bool Y16 = decltype(y16c)::value;
            constexpr int MODE = decltype(modec)::value; // 0: four codes per store, 1: fused 2x2 max-pool, 2: ragged channels
            constexpr bool SAT = decltype(satc)::value;  // also count the values clipped at cmax (with ReLU the only end)
            constexpr int ESZ = Y16 ? 2 : 1;
            const int first = __builtin_amdgcn_readfirstlane(MODE == 1 ? pooloff[0] : outoff[0]);
            const size_t pixels = MODE == 1 ? (size_t)a.N * (a.Ho >> 1) * (a.Wo >> 1) : (size_t)a.N * a.Ho * a.Wo;
            const size_t left = (pixels - (size_t)first) * a.Cout * ESZ;
            const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(
                (unsigned char *)a.y + (size_t)first * a.Cout * ESZ, 0, (int)(left < 0x7fffffffu ? left : 0x7fffffffu), 0x00020000);
            unsigned rel[MBL]; // byte offset of the lane's output pixel from the tile's first one
            unsigned long long rowmask[MBL]; // lanes whose output pixel exists (zero count)
#pragma unroll
            for (int mb = 0; mb < MBL; ++mb) {
                const int o = MODE == 1 ? po[mb] : oo[mb];
                rel[mb] = o >= 0 ? (unsigned)((o - first) * a.Cout * ESZ) : NOWHERE;
                rowmask[mb] = __builtin_amdgcn_ballot_w64(oo[mb] >= 0);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int gl = 0; gl < GL; ++gl) {
                    // a group of eight channels that lies past Cout altogether has nothing to write
                    // or count (uniform: a scalar branch)
                    if (ntile * BN + col0w + nb * 32 + 8 * (g0 + gl) >= a.Cout) continue;
                    const int cl = col0w + nb * 32 + 8 * (g0 + gl) + 4 * kg; // channel within the tile
                    const int col0 = ntile * BN + cl;
                    const bool col_ok = col0 < a.Cout;
                    const unsigned long long colmask = __builtin_amdgcn_ballot_w64(col_ok); // lanes whose channels exist
                    const v4i cA = *(const v4i *)(ctab + cl);
                    const v4i cB = *(const v4i *)(ctab + BN + cl);
                    const v4i cC = *(const v4i *)(ctab + 2 * BN + cl);
#pragma unroll
                    for (int mb = 0; mb < MBL; ++mb) {
                        int q[4], raw[4]; // codes, and the rounded values before clipping
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int v = 4 * gl + e;
                            int hi, lo16 = 0;
                            if constexpr (LIMBS == 2 && S16 == 3) {
                                // Shifts 9..16 (above, only the top plane matters and the class-0 form is
                                // shorter).  With W = floor(v / 256) the code is (W + 2^(s-9)) >> (s-8):
                                // the dropped low byte of v cannot carry into a multiple of 256.  W =
                                // 256*A + B + (C >> 8) + (rowsum >> 1) in 32 bits: A is clamped to +-2^22
                                // first (beyond that the code saturates for every s <= 22, and |B + ...|
                                // stays below 2^29 for K <= 8192); the half is part of cB.
                                const int C = acc[mb][nb][2][v] + cC[e] + ((rs[mb] & 1) << 7);
                                const int T = acc[mb][nb][1][v] + cB[e] + (C >> 8);
                                const int A = min(max(acc[mb][nb][0][v] + cA[e], -(1 << 22)), 1 << 22);
                                const int W = (A << 8) + T + (rs[mb] >> 1);
                                raw[e] = W >> (s - 8);
                                q[e] = clamp_code(raw[e], cmax);
                                continue;
                            } else if constexpr (S16 == 3) {
                                // one limb, shifts 9..16: the same with v = 65536*cA + (acc + low 16
                                // bits of the constant); cA arrives clamped, times 256, plus the half
                                const int W = ((acc[mb][nb][0][v] + cB[e]) >> 8) + cA[e];
                                raw[e] = W >> (s - 8);
                                q[e] = clamp_code(raw[e], cmax);
                                continue;
                            } else if constexpr (LIMBS == 2) {
                                const int C = acc[mb][nb][2][v] + cC[e] + ((rs[mb] & 1) << 7);
                                const int B = acc[mb][nb][1][v] + cB[e] + (rs[mb] >> 1) + (C >> 8);
                                hi = acc[mb][nb][0][v] + cA[e] + (B >> 8);
                                if constexpr (S16 != 0) lo16 = ((B & 255) << 8) | (C & 255);
                            } else {
                                // one limb: the plane split is 2^16*cA + (2^8*cB + cC)
                                const int C = acc[mb][nb][0][v] + (cB[e] << 8) + cC[e];
                                hi = cA[e] + (C >> 16);
                                lo16 = C & 65535;
                            }
                            raw[e] = requant_relu32<S16 == 3 ? 2 : S16>(hi, lo16, s);
                            q[e] = clamp_code(raw[e], cmax);
                        }
                        const bool counted = oo[mb] >= 0 && col_ok; // the lane's codes exist in the output tensor
                        if constexpr (MODE == 2) { // ragged channel tail: code by code
                            if (counted) {
                                unsigned char *dst = (unsigned char *)a.y + ((size_t)oo[mb] * a.Cout + col0) * ESZ;
                                const int ncodes = min(4, a.Cout - col0);
                                for (int e = 0; e < ncodes; ++e) {
                                    if constexpr (Y16) ((int16_t *)dst)[e] = (int16_t)q[e];
                                    else ((int8_t *)dst)[e] = (int8_t)q[e];
                                    nz += (q[e] == 0);
                                    if constexpr (SAT) ns += (raw[e] > cmax);
                                }
                            }
                        } else if constexpr (Y16) {
                            // codes are in [0, cmax]: packing needs no masks
                            unsigned w0 = (unsigned)q[0] | ((unsigned)q[1] << 16);
                            unsigned w1 = (unsigned)q[2] | ((unsigned)q[3] << 16);
                            // zeros: one compare per code into a lane mask, masks counted by the
                            // scalar unit (codes of lanes whose pixel or channels do not exist are
                            // masked out)
                            const unsigned long long live = rowmask[mb] & colmask;
#pragma unroll
                            for (int e = 0; e < 4; ++e) wz += __builtin_popcountll(__builtin_amdgcn_ballot_w64(q[e] == 0) & live);
                            if constexpr (SAT) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) wsat += __builtin_popcountll(__builtin_amdgcn_ballot_w64(raw[e] > cmax) & live);
                            }
                            if constexpr (MODE == 1) {
                                // 2x2 maximum across lanes: the horizontal neighbour is the next lane,
                                // the vertical one sits TW lanes further in the same 32-row block.
                                // Every lane takes part; only the window's top-left lane stores.
                                auto pkmax = [](unsigned x, unsigned y) __attribute__((always_inline)) {
                                    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(v2s, x),
                                                                                                  __builtin_bit_cast(v2s, y)));
                                };
                                w0 = pkmax(w0, (unsigned)__builtin_amdgcn_mov_dpp((int)w0, 0xB1, 0xF, 0xF, true));
                                w1 = pkmax(w1, (unsigned)__builtin_amdgcn_mov_dpp((int)w1, 0xB1, 0xF, 0xF, true));
                                const int below = ((lane + a.TW) & 63) * 4;
                                w0 = pkmax(w0, (unsigned)__builtin_amdgcn_ds_bpermute(below, (int)w0));
                                w1 = pkmax(w1, (unsigned)__builtin_amdgcn_ds_bpermute(below, (int)w1));
                            }
                            const unsigned at = col_ok ? rel[mb] + (unsigned)col0 * 2u : NOWHERE;
                            __builtin_amdgcn_raw_buffer_store_b64((v2u){w0, w1}, yrsrc, (int)at, 0, 0);
                        } else {
                            const unsigned w0 = (unsigned)q[0] | ((unsigned)q[1] << 8) | ((unsigned)q[2] << 16) | ((unsigned)q[3] << 24);
                            const unsigned long long live = rowmask[mb] & colmask;
#pragma unroll
                            for (int e = 0; e < 4; ++e) wz += __builtin_popcountll(__builtin_amdgcn_ballot_w64(q[e] == 0) & live);
                            if constexpr (SAT) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) wsat += __builtin_popcountll(__builtin_amdgcn_ballot_w64(raw[e] > cmax) & live);
                            }
                            const unsigned at = col_ok ? rel[mb] + (unsigned)col0 : NOWHERE;
                            __builtin_amdgcn_raw_buffer_store_b32(w0, yrsrc, (int)at, 0, 0);
                        }
                    }
                }
        };
        using std::integral_constant;
        auto by_sat = [&](auto s16c, auto y16c, auto modec) __attribute__((always_inline)) {
            if (a.count_sat) requant_tile(s16c, y16c, modec, integral_constant<bool, true>{});
            else requant_tile(s16c, y16c, modec, integral_constant<bool, false>{});
        };
        auto by_mode = [&](auto s16c, auto y16c) __attribute__((always_inline)) {
            if constexpr (decltype(y16c)::value) {
                if (a.pool) return by_sat(s16c, y16c, integral_constant<int, 1>{});
            }
            if ((a.Cout & 3) == 0) by_sat(s16c, y16c, integral_constant<int, 0>{}); // every group of four channels is aligned
            else by_sat(s16c, y16c, integral_constant<int, 2>{});
        };
        // shift classes: 9..16 (the usual ones) -> 3; else >= 17 -> 0, 16 -> 1, <= 15 -> 2
        const bool mid = s >= 9 && s <= 16;
        if (a.y16) {
            if (mid) {
                by_mode(integral_constant<int, 3>{}, integral_constant<bool, true>{});
            } else if (s >= 17) by_mode(integral_constant<int, 0>{}, integral_constant<bool, true>{});
            else if (s == 16) by_mode(integral_constant<int, 1>{}, integral_constant<bool, true>{});
            else by_mode(integral_constant<int, 2>{}, integral_constant<bool, true>{});
        } else {
            if (mid) {
                by_mode(integral_constant<int, 3>{}, integral_constant<bool, false>{});
            } else if (s >= 17) by_mode(integral_constant<int, 0>{}, integral_constant<bool, false>{});
            else if (s == 16) by_mode(integral_constant<int, 1>{}, integral_constant<bool, false>{});
            else by_mode(integral_constant<int, 2>{}, integral_constant<bool, false>{});
        }
    } else {
        const int64_t *ct64 = (const int64_t *)ctab;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int gl = 0; gl < GL; ++gl) {
                const int cl = col0w + nb * 32 + 8 * (g0 + gl) + 4 * kg;
                const int col0 = ntile * BN + cl;
#pragma unroll
                for (int mb = 0; mb < MBL; ++mb) {
                    const int64_t rt = (LIMBS == 2) ? (int64_t)rs[mb] * 128 : 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * gl + e;
                        int64_t val;
                        if constexpr (LIMBS == 2)
                            val = ((int64_t)acc[mb][nb][0][v] << 16) + ((int64_t)acc[mb][nb][1][v] << 8) +
                                  (int64_t)acc[mb][nb][2][v] + rt + ct64[cl + e];
                        else
                            val = (int64_t)acc[mb][nb][0][v] + ct64[cl + e];
                        if (oo[mb] >= 0 && col0 + e < a.Cout) {
                            const size_t idx = (size_t)oo[mb] * a.Cout + col0 + e;
                            if (a.acc_out) a.acc_out[idx] = val;
                            if (a.y) {
                                bool sat;
                                const int c = act_one(val, a.act, sat);
                                if (a.y16) ((int16_t *)a.y)[idx] = (int16_t)c;
                                else ((int8_t *)a.y)[idx] = (int8_t)c;
                                nz += (c == 0);
                                ns += sat;
                            }
                        }
                    }
                }
            }
    }
    // wave total of the per-lane counts, bit plane by bit plane: ballot + popcount
    TileCounts t = {wz, wsat};
#pragma unroll
    for (int b = 0; b < 7; ++b) t.zeros += wave_count((nz >> b) & 1) << b;
    if (a.count_sat) {
#pragma unroll
        for (int b = 0; b < 7; ++b) t.sats += wave_count((ns >> b) & 1) << b;
    }
    return t;
}


// corr[co] = 128 * sum_k w[co][k] - 16384 * K for the two-limb path, 0 otherwise: the weight half of
// the offset correction, computed once when the weights are packed.  One wave per output channel
// (blockIdx.x = co, 64 threads), lanes striding over K.
template <typename WT>
__global__ __launch_bounds__(64) void weight_corr_kernel(const WT *__restrict__ w, int64_t *__restrict__ corr, int Cout,
                                                        int CoutP, int K, int limbs)
{
    const int co = blockIdx.x;
    if (co >= CoutP) return;
    long long s = 0;
    if (limbs == 2 && co < Cout)
        for (int k = threadIdx.x; k < K; k += 64) s += (long long)w[(size_t)co * K + k];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_down(s, off, 64);
    if (threadIdx.x == 0) corr[co] = (limbs == 2 && co < Cout) ? 128 * s - (long long)16384 * K : 0;
}

// Adds n per-workgroup counts (zeros at partials[0..n), clipped values at partials[n..2n)) to the
// caller's counters (either may be null); defined with the convolution kernels.
lp_status launch_sum_partials(const unsigned *partials, int n, unsigned long long *zero_count,
                              unsigned long long *sat_count, hipStream_t st);

// LPInnerProduct through the convolution kernels (a 1x1 convolution over 1x1 images): the route
// for operand widths the inner-product kernel does not take.
lp_status fc_conv_packed_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host);
lp_status fc_conv_pack_weights(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, const void *w_codes_dev,
                               void *packed_dev, size_t packed_bytes, void *stream);
lp_status fc_conv_workspace_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host);
lp_status fc_conv_fwd(int M, int K, int Nout, const void *x_codes_dev, lp_qfmt qx, const void *w_packed_dev,
                      lp_qfmt qw, const void *bias_codes_dev, lp_qfmt qb, int64_t *acc_out_dev,
                      void *y_codes_dev, lp_qfmt qy, int relu, lp_round r, uint64_t *zero_count_dev,
                      uint64_t *sat_count_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

} // namespace lp
