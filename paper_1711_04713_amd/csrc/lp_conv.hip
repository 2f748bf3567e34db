// LPConvolution / LPInnerProduct forward on Qm.f codes for gfx950 (Sec. 2 of the paper),
// exact: int8 MFMA products, int32 limb sums, int64 results, fused LPAct+ReLU tail (Sec. 2.1).
//
// 16-bit codes are split into two int8 limbs, a = 256*ah + al + 128 with ah = a >> 8 and
// al = (a & 255) - 128 in [-128, 127].  Over the K real positions of a dot product
//     sum a*b = 2^16*HH + 2^8*(HL+LH) + LL + 128*sum(a) + 128*sum(b) - 16384*K
// where HH = sum ah*bh etc. are int32 MFMA accumulators.  A tap outside the image is the
// code 0, i.e. limbs (0, -128); channel padding is (0, 0) on both operands and drops out.
// sum(b) - 128*K per output channel is folded into the packed weights; sum(a) per output
// pixel comes from per-pixel channel sums gathered while the input patch is staged.
//
// Kernel shape: one 256-thread workgroup computes 128 output pixels x BN channels.  The
// pixels are RH consecutive rows (of the N*Ho stacked output rows) x TW columns; the
// input patch they need, (rows + R-1) x (TW + S-1) pixels x 64 channels, is staged in LDS
// once per 64-channel chunk and every tap reads it at a shifted offset (implicit GEMM with
// halo reuse).  Weights are packed one (chunk, tap) slab after the other and are read from
// global memory / L2 straight into MFMA operand registers, half a slab ahead of their use.
// Layers with very few input channels (the first VGG16 layer, Cin = 3) run conv_flat_kernel:
// the whole R*S*Cin window is one K <= 64 slab, gathered per output pixel from the raw patch.
#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

#include "lp_tile.h"

namespace lp {

constexpr int BM = 128;      // output pixels per workgroup
constexpr int CK = 64;       // channels (bytes per limb) per staged chunk
constexpr int kFlatRawBytes = 8192; // LDS for the raw input patch of the flat-window kernel
constexpr int PSP = 80;      // LDS bytes per staged patch pixel and limb: 64 of codes and 16 of padding, so that
                             // consecutive pixels start 20 banks apart (see choose_pitch)
constexpr int kConvThreads = 256;

constexpr int kMaxDevices = 64;
constexpr int kDirectCountGrid = 2048; // largest grid whose workgroups add to the zero / saturation counters directly

enum { PATH_DIRECT = 0, PATH_MFMA = 1 };

struct Plan {
    int path;
    int pool;    // the epilogue stores 2x2 maxima instead of the codes
    int limbs;   // 1: int8 x int8, 2: 16-bit x 16-bit
    int flat;    // whole window gathered as one K <= 64 slab (tiny Cin)
    int rows;    // reduction over window rows (16-bit codes, 16 / 32 / 48 input channels): conv_rows_kernel
    int KHR, KHP; // rows: K = 32 pieces per window row, and in all (padded to a multiple of 4)
    int taps, ksteps; // slabs per chunk, K=32 MFMA steps per slab
    int Ho, Wo, Hp, FR;
    int nchunks, CoutP, BN;
    int RH, TW, PW, PRA, NPIXA;
    int PITCH;   // LDS bytes between staged patch rows
    int tiles_r, tiles_c, tiles_m, tiles_n;
    // Launch geometry.  Every die gets per_xcd consecutive tiles.  The first full_per_xcd of
    // them (a whole number of rounds of the die's workgroup slots) are computed by one workgroup
    // each; each of the remaining tail tiles is cut along the reduction into `split` parts, so
    // that the last, partly filled round keeps every CU busy (see the kernel's merge step).
    int per_xcd, full_per_xcd, split, grid;
    size_t part_bytes;   // bytes of one part's accumulators and row sums in the workspace
    size_t lds_bytes;
    size_t packed_bytes, corr_offset;
    size_t wsum_offset;  // per-chunk weight sums [nchunks][CoutP] int32 (two-limb patch path), else 0
};

// Workspace layout: one zero count per workgroup, then the tail tiles' partial accumulators
// [die][tail tile][part].
struct WorkspaceLayout {
    size_t partials, total;
};

static bool desc_ok(const lp_conv_desc *d)
{
    return d && d->N > 0 && d->H > 0 && d->W > 0 && d->Cin > 0 && d->Cout > 0 && d->R > 0 &&
           d->S > 0 && d->stride > 0 && d->pad >= 0 && d->H + 2 * d->pad >= d->R &&
           d->W + 2 * d->pad >= d->S && (d->pool == 0 || d->pool == 1);
}

// Bank conflicts of the fragment reads for a patch whose rows are pitch16 * 16 bytes apart.  A
// 16-byte read is served 16 lanes at a time, the 64 banks covering 256 bytes: the 16 lanes (16
// consecutive tile rows, the same 16-byte slot of their pixels at one tap) must fall into 16
// different 16-byte groups modulo 256 bytes.  A pixel is PSP = 80 bytes, so the group of pixel
// (prow, pcol) is prow * pitch16 + 5 * pcol: along a patch row the groups never collide (5 is odd),
// and the pitch decides how the rows of a narrow tile interleave.
static int pitch_conflicts(int tw, int rh, int R, int S, int pitch16)
{
    int cost = 0;
    const int rows = rh * tw;
    for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s)
            for (int m0 = 0; m0 < rows; m0 += 16) {
                int seen[16] = {0};
                int worst = 0;
                for (int m = m0; m < std::min(m0 + 16, rows); ++m) {
                    const int prow = m / tw + r, pcol = m % tw + s;
                    worst = std::max(worst, ++seen[(prow * pitch16 + 5 * pcol) & 15]);
                }
                cost += worst - 1;
            }
    return cost;
}

// Smallest row pitch (in 16-byte units, at most 15 units of padding) with the fewest conflicts.
static int choose_pitch(int pw, int tw, int rh, int R, int S)
{
    int best = 1 << 30, best_pitch = pw * (PSP / 16);
    for (int p16 = pw * (PSP / 16); p16 < pw * (PSP / 16) + 16; ++p16) {
        const int c = pitch_conflicts(tw, rh, R, S, p16);
        if (c < best) {
            best = c;
            best_pitch = p16;
        }
    }
    return best_pitch;
}

// Window-row kernel: pixels are Cin bytes per limb and dense along a patch row; the 16 lanes served
// together read the same 16-byte slot of 16 consecutive tile rows.  Smallest row pitch (bytes,
// up to 240 of padding) with the fewest conflicts.
static int rows_pitch(int pw, int tw, int rh, int cin)
{
    int best = 1 << 30, best_pitch = pw * cin;
    const int rows = rh * tw;
    for (int pitch = pw * cin; pitch < pw * cin + 256; pitch += 16) {
        int cost = 0;
        for (int m0 = 0; m0 < rows; m0 += 16) {
            int seen[16] = {0};
            int worst = 0;
            for (int m = m0; m < std::min(m0 + 16, rows); ++m)
                worst = std::max(worst, ++seen[(((m / tw) * pitch + (m % tw) * cin) >> 4) & 15]);
            cost += worst - 1;
        }
        if (cost < best) {
            best = cost;
            best_pitch = pitch;
        }
    }
    return best_pitch;
}

// LDS of the window-row kernel: unit sums, four row tables, channel constants, wave counts, two planes
static size_t rows_lds_bytes(int pra, int pw, int cin, int pitch)
{
    const size_t nu = (size_t)pra * pw * (cin / 16);
    return (round_up(nu, 4) + 4 * BM + 3 * 64 + 8) * 4 + 2 * ((size_t)pra * pitch + 32);
}

// 16-byte pieces a thread requests per batch while staging a patch (two batches are in flight).
// Three fit the two-limb kernel's registers as well, but the patches of the VGG16 layers are 6 to
// 7 pieces per thread, which batches of two cover in 8 and batches of three in 12 (measured: 2 %
// slower); four, which would put a whole patch in flight at once, spill.
constexpr int kStageBatch = 2;

// Entries of the per-pixel patch tables.  The staging loops run whole batches of pieces, so they
// overshoot the patch by less than two double batches and the first, deep batch covers 8 * 256
// pieces whatever the patch size; the entries past the patch send those pieces to a source
// offset that reads as zeros and to a parking slot behind the plane.
static int patch_table_len(int limbs, int npixa, int flat)
{
    if (flat) return std::max(npixa, BM);
    const int per_pass = 256 / (limbs == 2 ? 8 : 4); // pixels a pass of all threads covers
    return std::max(npixa + 2 * kStageBatch * per_pass, 8 * per_pass);
}

// LDS: tables (3*ntab + 2*BM ints, 3*bn ints of channel constants, BM pooled offsets), staged patch (one plane per
// limb); the flat-window kernel: its fixed arrays (raw patch, weight operands, tables)
static size_t mfma_lds_bytes(int limbs, int pra, int pw, int pitch_bytes, int bn, int flat)
{
    if (flat) return (size_t)kFlatRawBytes + 8192 + 4096;
    const int ntab = patch_table_len(limbs, pra * pw, flat);
    const size_t plane = (size_t)pra * pitch_bytes + PSP; // + the slot overshoot pieces are parked in
    size_t tables = round_up((size_t)(3 * ntab + 2 * BM) * 4, 16) + (size_t)3 * bn * 4 + (size_t)BM * 4;
    return tables + (size_t)limbs * plane;
}
// LDS budgets tried in turn: three workgroups per CU (160 KB / 3), else two
constexpr size_t kLdsBudgets[2] = {54400, 80000};

// Parts per tail tile.  Durations are estimated in units of one weight slab's MFMA work, with
// constants fitted to measurements on 3x3 layers: a workgroup pays a fixed cost of about 10
// slabs (tables, first patch, epilogue or partial store) on top of its share of the slabs, the
// tail takes as many rounds as its parts need slots, the finishing kernel costs about 6, and
// every part adds traffic (its accumulators are written once and read once).  A split must
// promise a clear gain over the plain launch to be taken.
static int choose_split(int tail_tiles, int slots, int nslabs, size_t part_bytes)
{
    const double fixed = 10.0, finish = 6.0, per_part = 0.03 * (double)part_bytes / 98816.0;
    const double whole = nslabs + fixed;
    int best = 1;
    double best_t = 0.8 * whole;
    for (int s = 2; s <= std::min(nslabs, 8); ++s) {
        const int rounds = (tail_tiles * s + slots - 1) / slots;
        const double t = rounds * ((double)nslabs / s + fixed) + finish + per_part * kXCDs * tail_tiles * s;
        if (t < best_t) {
            best_t = t;
            best = s;
        }
    }
    return best;
}

// virtual row (in the stack of zero-padded images, Hp rows each) of stacked output row fr
static inline int vrow(int fr, int Ho, int Hp) { return (fr / Ho) * Hp + fr % Ho; }

// Plans are pure functions of (descriptor, operand widths); the tile search costs tens of
// microseconds, so results are remembered.
struct PlanKey {
    lp_conv_desc d;
    int x16, w16;
    bool operator==(const PlanKey &o) const
    {
        return d.N == o.d.N && d.H == o.d.H && d.W == o.d.W && d.Cin == o.d.Cin && d.Cout == o.d.Cout &&
               d.R == o.d.R && d.S == o.d.S && d.stride == o.d.stride && d.pad == o.d.pad &&
               d.pool == o.d.pool && x16 == o.x16 && w16 == o.w16;
    }
};
static std::mutex g_plan_mutex;
static std::vector<std::pair<PlanKey, Plan>> g_plan_cache;

static lp_status make_plan_uncached(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, Plan *pl);

// Chooses path and tile geometry.  Returns LP_OK or the reason the problem is refused.
static lp_status make_plan(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, Plan *pl)
{
    if (!desc_ok(d) || !fmt_ok(qx) || !fmt_ok(qw)) return LP_EINVAL;
    const PlanKey key = {*d, qx.n > 8, qw.n > 8};
    {
        std::lock_guard<std::mutex> lock(g_plan_mutex);
        for (const auto &e : g_plan_cache)
            if (e.first == key) {
                *pl = e.second;
                return LP_OK;
            }
    }
    const lp_status st = make_plan_uncached(d, qx, qw, pl);
    if (st == LP_OK) {
        std::lock_guard<std::mutex> lock(g_plan_mutex);
        if (g_plan_cache.size() >= 256) g_plan_cache.clear();
        g_plan_cache.emplace_back(key, *pl);
    }
    return st;
}

static lp_status make_plan_uncached(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, Plan *pl)
{
    Plan p = {};
    p.Ho = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    p.Wo = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    p.Hp = d->H + 2 * d->pad;
    const long long in_elems = (long long)d->N * d->H * d->W * d->Cin;
    const long long out_elems = (long long)d->N * p.Ho * p.Wo * d->Cout;
    const long long w_elems = (long long)d->Cout * d->R * d->S * d->Cin;
    const long long K = (long long)d->R * d->S * d->Cin;
    if (in_elems >= (1LL << 31) || out_elems >= (1LL << 31) || w_elems >= (1LL << 31))
        return LP_EUNSUPPORTED;
    if (K >= 65536 && (qx.n > 8 || qw.n > 8)) return LP_EUNSUPPORTED;
    if (K >= 131072) return LP_EUNSUPPORTED;
    p.FR = d->N * p.Ho;
    const bool x16 = qx.n > 8, w16 = qw.n > 8;
    p.limbs = x16 ? 2 : 1;
    p.path = PATH_DIRECT;
    const int cvec = x16 ? 8 : 16; // codes per 16-byte load
    const bool chunked = d->Cin % cvec == 0 && d->Cin >= 16;
    p.flat = (!chunked && x16 && K <= 64) ? 1 : 0;
    if (d->stride == 1 && (x16 || !w16) && (chunked || p.flat)) {
        // tile search: RH x TW <= 128 output pixels, minimise wasted MFMA rows, then patch size
        // With the pooling fused, a 2x2 window must lie inside one 32-row block of one tile: an
        // even number of tile rows (tiles then start on even stacked rows, and with Ho even a
        // row pair never straddles two images) and a width that divides 16.  Such a geometry is
        // taken only if it costs no more than 3 % over the best unconstrained one.
        const int RS = d->R * d->S;
        double best = 1e300, best_free = 1e300;
        for (int pass = 0; pass < 2 && best == 1e300; ++pass)
        for (int tw = 1; tw <= std::min(p.Wo, BM); ++tw)
            for (int rh = std::min(BM / tw, p.FR); rh >= 1; --rh) {
                const bool poolable = (tw == 2 || tw == 4 || tw == 8 || tw == 16) && rh % 2 == 0;
                const int tiles_c = (p.Wo + tw - 1) / tw, tiles_r = (p.FR + rh - 1) / rh;
                const int pw = tw + d->S - 1;
                // patch rows: the tile's rows, the R-1 halo, and R-1 more per image boundary
                // the tile can straddle (none when tiles divide the image height)
                const int cross = (p.Ho % rh == 0) ? 0 : std::min((rh - 1 + p.Ho - 1) / p.Ho, d->N - 1);
                const int pra = rh + d->R - 1 + cross * (d->R - 1);
                const int npixa = pra * pw;
                const double cost = (double)tiles_c * tiles_r * ((double)BM * RS + 0.5 * npixa);
                if (cost >= best_free && (cost >= best || (d->pool && !poolable))) continue; // improves nothing
                // LDS need: first with the smallest row pitch, then (the pitch search is the
                // expensive part) with the pitch this geometry would get
                const int bn_max = p.limbs == 2 ? 64 : 128;
                if (mfma_lds_bytes(p.limbs, pra, pw, pw * PSP, bn_max, p.flat) > kLdsBudgets[pass]) continue;
                if (!p.flat &&
                    mfma_lds_bytes(p.limbs, pra, pw, 16 * choose_pitch(pw, tw, rh, d->R, d->S), bn_max, 0) > kLdsBudgets[pass])
                    continue;
                if (p.flat && (size_t)npixa * d->Cin * 2 > (size_t)kFlatRawBytes) continue;
                best_free = std::min(best_free, cost);
                if (d->pool && !poolable) continue;
                if (cost < best) {
                    best = cost;
                    p.RH = rh; p.TW = tw; p.PW = pw; p.PRA = pra; p.NPIXA = npixa;
                    p.tiles_r = tiles_r; p.tiles_c = tiles_c;
                }
            }
        if (best < 1e300) p.path = PATH_MFMA;
        if (d->pool && (best == 1e300 || best > 1.03 * best_free)) return LP_EUNSUPPORTED;
        if (best < 1e300 && chunked && x16 && d->Cin % 16 == 0 && d->Cin < CK && in_elems < (1LL << 31) - 64) {
            const int khr = (d->S * d->Cin + 31) / 32;
            const int pitch = rows_pitch(p.PW, p.TW, p.RH, d->Cin);
            if (d->R * khr <= 256 && rows_lds_bytes(p.PRA, p.PW, d->Cin, pitch) <= 40 * 1024) {
                p.rows = 1;
                p.KHR = khr;
                p.KHP = (int)round_up((size_t)d->R * khr, 4);
                p.PITCH = pitch;
            }
        }
    }
    if (d->pool && (p.path != PATH_MFMA || p.Ho % 2 || p.Wo % 2)) return LP_EUNSUPPORTED;
    p.pool = d->pool;
    if (p.path == PATH_MFMA) {
        const bool one_slab = p.flat || p.rows; // nothing to cut along the reduction
        p.nchunks = one_slab ? 1 : (d->Cin + CK - 1) / CK;
        p.taps = one_slab ? 1 : d->R * d->S;
        p.ksteps = p.flat ? (int)((K + 31) / 32) : 2;
        p.CoutP = (int)round_up(d->Cout, 64);
        p.tiles_m = p.tiles_r * p.tiles_c;
        // 128-wide channel tiles halve the patch re-reads, but a grid with fewer workgroups than
        // the chip has slots (256 CUs x 2) is better cut finer
        p.BN = (p.CoutP % 128 == 0 && (long long)p.tiles_m * (p.CoutP / 128) >= 512) ? 128 : 64;
        // the two-limb kernel holds three accumulator sets; at 128 channels they leave too few
        // registers for the prefetch pipeline, so it always runs 64-wide
        if (p.limbs == 2) p.BN = 64;
        p.tiles_n = p.CoutP / p.BN;
        if (!p.rows) p.PITCH = p.flat ? 0 : 16 * choose_pitch(p.PW, p.TW, p.RH, d->R, d->S);
        p.lds_bytes = p.rows ? rows_lds_bytes(p.PRA, p.PW, d->Cin, p.PITCH)
                             : mfma_lds_bytes(p.limbs, p.PRA, p.PW, p.PITCH, p.BN, p.flat);
        {
            // workgroup slots per die: what registers and LDS allow
            const int total = p.tiles_m * p.tiles_n, nslabs = p.nchunks * p.taps;
            // (two-limb kernel: three waves per SIMD by registers; one-limb kernels: four)
            // (window-row kernel: four, or three where it takes two column blocks)
            const int by_regs = p.rows ? (d->Cout <= 32 ? 4 : 3) : p.limbs == 2 ? 3 : 4;
            const int wg_per_cu = (int)std::max<size_t>(1, std::min<size_t>(by_regs, (160 * 1024) / p.lds_bytes));
            const int slots = wg_per_cu * (kCUs / kXCDs);
            p.per_xcd = (total + kXCDs - 1) / kXCDs;
            p.full_per_xcd = p.per_xcd / slots * slots;
            p.part_bytes = (size_t)BM * p.BN * (p.limbs == 2 ? 3 : 1) * 4 + (size_t)BM * 4;
            p.split = 1;
            if (p.per_xcd > p.full_per_xcd && nslabs > 1)
                p.split = choose_split(p.per_xcd - p.full_per_xcd, slots, nslabs, p.part_bytes);
            if (p.split == 1) p.full_per_xcd = p.per_xcd;
            p.grid = kXCDs * (p.full_per_xcd + (p.per_xcd - p.full_per_xcd) * p.split);
        }
        p.corr_offset = p.rows ? round_up((size_t)p.KHP * 2 * p.CoutP * 32, 256)
                               : round_up((size_t)p.taps * p.nchunks * p.limbs * p.CoutP * CK, 256);
        // the kernel addresses the slabs with 32-bit byte offsets
        if (p.corr_offset >= (1ull << 31)) return LP_EUNSUPPORTED;
        p.packed_bytes = p.corr_offset + (size_t)p.CoutP * sizeof(int64_t);
        if (p.limbs == 2 && !p.flat && !p.rows) {
            p.wsum_offset = p.packed_bytes;
            p.packed_bytes += (size_t)p.nchunks * p.CoutP * sizeof(int);
        }
    } else {
        // direct path keeps a plain int16 copy of the weights
        p.corr_offset = 0;
        p.packed_bytes = round_up((size_t)w_elems * sizeof(int16_t), 256);
    }
    *pl = p;
    return LP_OK;
}

// --------------------------------------------------------------------- weight packing

// Byte kk (0..63) of output channel co inside one limb plane of a slab: the two K = 32 halves are
// separate blocks of CoutP x 32 bytes, so that the 16-byte pieces a wave requests for one half (32
// channels x 2 pieces) are 1 KB of consecutive memory, i.e. whole cache lines.
__host__ __device__ inline size_t slab_byte(int co, int kk, int CoutP) { return ((size_t)(kk >> 5) * CoutP + co) * 32 + (kk & 31); }

// MFMA layout: [chunk][tap][limb][K half][CoutP][32] int8, i.e. slabs in the order the kernel streams them.
template <typename WT, int LIMBS>
__global__ void pack_weights_kernel(const WT *__restrict__ w, unsigned char *__restrict__ out, int Cout,
                                    int Cin, int RS, int nchunks, int CoutP, size_t total)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int kk = (int)(i % CK);
        size_t t = i / CK;
        const int co = (int)(t % CoutP);
        t /= CoutP;
        const int chunk = (int)(t % nchunks);
        const int tap = (int)(t / nchunks);
        const int ci = chunk * CK + kk;
        int hi = 0, lo = 0;
        if (co < Cout && ci < Cin) {
            const int code = (int)w[((size_t)co * RS + tap) * Cin + ci];
            if constexpr (LIMBS == 2) {
                hi = code >> 8;
                lo = (code & 255) - 128;
            } else {
                hi = code;
            }
        }
        const size_t base = (((size_t)chunk * RS + tap) * LIMBS) * CoutP * CK;
        out[base + slab_byte(co, kk, CoutP)] = (unsigned char)hi;
        if constexpr (LIMBS == 2) out[base + (size_t)CoutP * CK + slab_byte(co, kk, CoutP)] = (unsigned char)lo;
    }
}

// Flat layout: one slab [limb][K half][CoutP][32], byte k of a row = weight k of the (r, s, ci) window.
template <typename WT>
__global__ void pack_weights_flat_kernel(const WT *__restrict__ w, unsigned char *__restrict__ out,
                                         int Cout, int K, int CoutP)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= CoutP * CK) return;
    const int kk = i % CK, co = i / CK;
    int hi = 0, lo = 0;
    if (co < Cout && kk < K) {
        const int code = (int)w[(size_t)co * K + kk];
        hi = code >> 8;
        lo = (code & 255) - 128;
    }
    out[slab_byte(co, kk, CoutP)] = (unsigned char)hi;
    out[(size_t)CoutP * CK + slab_byte(co, kk, CoutP)] = (unsigned char)lo;
}

// Window-row layout: [piece][limb][CoutP][32]; piece h = (window row h / KHR, 32 positions from
// 32 * (h % KHR) of that row's S * Cin weights); positions past the row, pad pieces and padded
// channels hold the bytes (0, 0).
template <typename WT>
__global__ void pack_weights_rows_kernel(const WT *__restrict__ w, unsigned char *__restrict__ out, int Cout, int R,
                                         int SC, int KHR, int KHP, int CoutP)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= KHP * CoutP * 32) return;
    const int kk = i & 31, co = (i >> 5) % CoutP, h = (i >> 5) / CoutP;
    const int r = h / KHR, pos = (h % KHR) * 32 + kk;
    int hi = 0, lo = 0;
    if (co < Cout && r < R && pos < SC) {
        const int code = (int)w[((size_t)co * R + r) * SC + pos];
        hi = code >> 8;
        lo = (code & 255) - 128;
    }
    const size_t at = ((size_t)h * 2 * CoutP + co) * 32 + kk;
    out[at] = (unsigned char)hi;
    out[at + (size_t)CoutP * 32] = (unsigned char)lo;
}

template <typename WT>
__global__ void widen_weights_kernel(const WT *__restrict__ w, int16_t *__restrict__ out, size_t total)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x)
        out[i] = (int16_t)w[i];
}

// wsum[chunk][co] = sum of the weight codes of output channel co over the chunk's 64 input
// channels and all taps (one wave per (chunk, co)).
template <typename WT>
__global__ __launch_bounds__(64) void chunk_weight_sums_kernel(const WT *__restrict__ w, int *__restrict__ wsum, int Cout,
                                                              int CoutP, int Cin, int RS)
{
    const int co = blockIdx.x, chunk = blockIdx.y;
    int s = 0;
    if (co < Cout) {
        const int nch = min(CK, Cin - chunk * CK);
        for (int i = threadIdx.x; i < RS * nch; i += 64) {
            const int tap = i / nch, c = i - tap * nch;
            s += (int)w[((size_t)co * RS + tap) * Cin + chunk * CK + c];
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_down(s, off, 64);
    if (threadIdx.x == 0) wsum[(size_t)chunk * CoutP + co] = s;
}

// ------------------------------------------------------------------------ direct path
// One thread per output value; any stride / kernel size / operand width.  Correctness
// fallback for shapes the MFMA kernel does not take.
template <typename XT>
__global__ __launch_bounds__(256) void conv_direct_kernel(const ConvArgs a)
{
    const size_t total = (size_t)a.FR * a.Wo * a.Cout;
    const XT *x = (const XT *)a.x;
    const int16_t *w = (const int16_t *)a.wp;
    unsigned zeros = 0, sats = 0;
    for (size_t i0 = (size_t)blockIdx.x * 256; i0 < total; i0 += (size_t)gridDim.x * 256) {
        const size_t i = i0 + threadIdx.x;
        bool z = false, sat = false;
        if (i < total) {
            const int co = (int)(i % a.Cout);
            size_t t = i / a.Cout;
            const int xo = (int)(t % a.Wo);
            t /= a.Wo;
            const int yo = (int)(t % a.Ho);
            const int n = (int)(t / a.Ho);
            int64_t acc = 0;
            for (int r = 0; r < a.R; ++r) {
                const int iy = yo * a.stride + r - a.pad;
                if (iy < 0 || iy >= a.H) continue;
                for (int s = 0; s < a.S; ++s) {
                    const int ix = xo * a.stride + s - a.pad;
                    if (ix < 0 || ix >= a.W) continue;
                    const XT *xp = x + (((size_t)n * a.H + iy) * a.W + ix) * a.Cin;
                    const int16_t *wq = w + (((size_t)co * a.R + r) * a.S + s) * a.Cin;
                    for (int ci = 0; ci < a.Cin; ++ci) acc += (int64_t)((int)xp[ci] * (int)wq[ci]);
                }
            }
            acc += bias_term(a, co);
            if (a.acc_out) a.acc_out[i] = acc;
            if (a.y) {
                const int c = act_one(acc, a.act, sat);
                if (a.y16) ((int16_t *)a.y)[i] = (int16_t)c;
                else ((int8_t *)a.y)[i] = (int8_t)c;
                z = (c == 0);
            }
        }
        zeros += wave_count(z);
        sats += wave_count(sat);
    }
    if (a.y && (threadIdx.x & 63) == 0) {
        if (a.zero_count && zeros) atomicAdd(a.zero_count, (unsigned long long)zeros);
        if (a.sat_count && sats) atomicAdd(a.sat_count, (unsigned long long)sats);
    }
}

// -------------------------------------------------------------------------- MFMA path

// LIMBS: 1 (int8 codes) or 2 (16-bit codes as two int8 limbs).  NB: 32-column blocks per
// wave; the workgroup covers BN = 64*NB output channels with 2x2 waves of 64 x 32*NB each.
template <int LIMBS, int NB, int MB>
__global__ __launch_bounds__(MB == 2 ? 256 : 512)
    __attribute__((amdgpu_waves_per_eu(MB == 2 && LIMBS == 2 ? 3 : 4, MB == 2 && LIMBS == 2 ? 3 : 4))) void conv_mfma_kernel(
        const ConvArgs a)
{
    // MB: 32-row blocks per wave.  MB = 2: 4 waves (2 x 2) of 64 rows, the only form launched.
    // MB = 1 (8 waves of 32 rows, a fourth wave per SIMD) is kept compilable as a tuning knob: with
    // the weights read per wave it doubles their traffic and measured 14 % slower even on the
    // smallest grids.
    constexpr int THREADS = (MB == 2) ? 256 : 512;
    constexpr int WMC = BM / (32 * MB);       // waves along the pixel dimension
    constexpr int WROWS = 32 * MB;            // tile rows per wave
    constexpr int BN = 64 * NB;
    constexpr int NACC = (LIMBS == 2) ? 3 : 1;
    extern __shared__ __align__(16) unsigned char smem[];

    // XCD-aware work order: consecutive workgroup ids land on the 8 XCDs round-robin, so
    // each XCD is handed one contiguous range of (pixel tile, channel tile) work items and
    // the tiles sharing an input patch or a halo meet in the same L2.
    // A die's first full_per_xcd work items are whole tiles; each later one is cut along the
    // reduction into a.split parts (consecutive slots), dispatched after all whole tiles.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int tl = slot, part = 0, nparts = 1;
    if (slot >= a.full_per_xcd) {
        const int u = slot - a.full_per_xcd;
        tl = a.full_per_xcd + u / a.split;
        part = u % a.split;
        nparts = a.split;
    }
    const int wi = xcd * a.per_xcd + tl;
    if (tl >= a.per_xcd || wi >= a.total_work) {
        if (a.zero_partial && threadIdx.x == 0) a.zero_partial[blockIdx.x] = a.zero_partial[a.partial_stride + blockIdx.x] = 0;
        return;
    }
    int mtile, ntile, tile_r, tile_c, img0, yo0;
    udivmod(wi, a.tiles_n, a.mg_tiles_n, mtile, ntile);
    udivmod(mtile, a.tiles_c, a.mg_tiles_c, tile_r, tile_c);
    const int fr0 = tile_r * a.RH, x0 = tile_c * a.TW;
    udivmod(fr0, a.Ho, a.mg_Ho, img0, yo0);
    const int vr0 = img0 * a.Hp + yo0;

    const int NPIXA = a.NPIXA;
    int *tab = (int *)smem;          // staged pixel -> byte offset of its codes in x, all ones outside the image
    int *psum = tab + a.NTAB;        // per staged pixel: sum of its codes
    int *apos = psum + a.NTAB;       // staged pixel -> byte offset inside a limb plane
    int *outoff = apos + a.NTAB;     // tile row -> output pixel index, -1 if not an output
    int *abase_s = outoff + BM;      // tile row -> staged pixel of its (r=0, s=0) tap
    int *ctab = (int *)(smem + (((size_t)(3 * a.NTAB + 2 * BM) * 4 + 15) & ~(size_t)15)); // channel constants
    int *pooloff = ctab + 3 * BN;    // tile row -> pooled output pixel (top-left rows of 2x2 windows), else -1
    unsigned char *Asm = (unsigned char *)(pooloff + BM);
    const int APL = a.APLANE;        // bytes per limb plane of the staged activations
    unsigned char *Bsm = Asm + (size_t)LIMBS * APL;

    const int tid = threadIdx.x;
    // LDS address of the staged planes (patch path: positions and fragment offsets are kept as LDS addresses)
    const int planes_lds = (int)(unsigned long)(__attribute__((address_space(3))) unsigned char *)Asm;
    // Entries past the patch (the staging loops overshoot it by up to a few batches) read as
    // zeros and are parked in the spare slot at the end of a plane.
    const unsigned px_bytes = (unsigned)a.Cin * (LIMBS == 2 ? 2u : 1u);
    for (int p = tid; p < a.NTAB; p += THREADS) {
        int g = -1, pos = APL - PSP;
        if (p < NPIXA) {
            int pr, pc, n, iy;
            udivmod(p, a.PW, a.mg_PW, pr, pc);
            pos = pr * a.PITCH + pc * PSP;
            udivmod(vr0 + pr, a.Hp, a.mg_Hp, n, iy);
            iy -= a.pad;
            const int ix = x0 - a.pad + pc;
            if (n < a.N && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) g = (n * a.H + iy) * a.W + ix;
        }
        tab[p] = g >= 0 ? (int)((unsigned)g * px_bytes) : -1;
        apos[p] = planes_lds + pos; // as an LDS address: parking a piece then costs no base add
        psum[p] = 0;
    }
    unsigned livemask = 0xffffffffu, deadmask = 0; // see "skipping" below
    // The tables of the tile rows and the channel constants are not needed to request the first
    // patch: they are built while those requests are in flight (see the first staging below).
    auto row_tables = [&]() __attribute__((always_inline)) {
        for (int m = tid; m < BM; m += THREADS) {
            int j, t, img, yo;
            udivmod(m, a.TW, a.mg_TW, j, t);
            const int fr = fr0 + j, xo = x0 + t;
            const bool ok = j < a.RH && fr < a.FR && xo < a.Wo;
            udivmod(fr, a.Ho, a.mg_Ho, img, yo);
            outoff[m] = ok ? fr * a.Wo + xo : -1;
            abase_s[m] = ok ? (img * a.Hp + yo - vr0) * a.PW + t : 0;
            pooloff[m] = (a.pool && ok && !(j & 1) && !(t & 1)) ? (img * (a.Ho >> 1) + (yo >> 1)) * (a.Wo >> 1) + (xo >> 1) : -1;
        }
        build_colterms<BN, THREADS>(a, ntile, ctab, LIMBS, deadmask);
    };
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WMC, wn = wave / WMC;
    const int l32 = lane & 31, kg = lane >> 5;

    // Skipping of all-zero input chunks.  The layer that produced x has left one flag per (pixel
    // tile, channel tile) of its output; a 64-channel chunk whose flags are clear in every
    // producer tile that the patch touches holds only the code 0 and is neither staged nor
    // multiplied.  livemask: bit c = chunk c is multiplied (uniform).  Every wave works it out for
    // itself: lane c looks at chunk c.  Tiles whose reduction is shared between workgroups, and
    // layers with more than 32 chunks, multiply everything.
    const bool skipping = a.zin && nparts == 1 && a.nchunks <= 32;
    if (skipping) {
        // input rows (of the N * H stacked rows) and columns the patch really holds
        int n_lo, p_lo, n_hi, p_hi;
        udivmod(vr0, a.Hp, a.mg_Hp, n_lo, p_lo);
        udivmod(vr0 + a.NPIXA / a.PW - 1, a.Hp, a.mg_Hp, n_hi, p_hi);
        int r_lo = p_lo < a.pad ? n_lo * a.H : p_lo >= a.pad + a.H ? (n_lo + 1) * a.H : n_lo * a.H + p_lo - a.pad;
        int r_hi = p_hi < a.pad ? n_hi * a.H - 1 : p_hi >= a.pad + a.H ? (n_hi + 1) * a.H - 1 : n_hi * a.H + p_hi - a.pad;
        r_hi = min(r_hi, a.N * a.H - 1);
        const int c_lo = max(0, x0 - a.pad), c_hi = min(a.W - 1, x0 - a.pad + a.PW - 1);
        unsigned live = (1u << (a.nchunks - 1) << 1) - 1u;
        if (r_lo <= r_hi && c_lo <= c_hi) {
            const int sc = a.z_scale;
            const int tr0 = (r_lo * sc) / a.z_rh, tr1 = (r_hi * sc + sc - 1) / a.z_rh;
            const int tc0 = (c_lo * sc) / a.z_tw, tc1 = min((c_hi * sc + sc - 1) / a.z_tw, a.z_tiles_c - 1);
            if ((tr1 - tr0 + 1) * (tc1 - tc0 + 1) <= 64) {
                bool any = false;
                if (lane < a.nchunks) {
                    const int zn = (lane * CK) / a.z_bn; // the producer's channel tile that holds this chunk
                    for (int tr = tr0; tr <= tr1; ++tr)
                        for (int tc = tc0; tc <= tc1; ++tc) any |= a.zin[(size_t)(tr * a.z_tiles_c + tc) * a.z_tiles_n + zn] != 0;
                }
                live = (unsigned)__builtin_amdgcn_ballot_w64(any);
            }
        }
        if (live == 0) live = 1; // nothing to multiply: chunk 0 (all zeros) is multiplied for form's sake
        livemask = live;
        deadmask = ~live & ((1u << (a.nchunks - 1) << 1) - 1u);
        if (a.skipped && tid == 0 && deadmask) atomicAdd(a.skipped, (unsigned long long)__builtin_popcount(deadmask));
    }
    // the chunk after chunk c in the order of multiplication (c itself past the last one)
    auto next_chunk = [&](int c) __attribute__((always_inline)) {
        if (!skipping) return c + 1;
        const unsigned rem = c >= 31 ? 0u : livemask >> (c + 1);
        return rem ? c + 1 + (int)__builtin_ctz(rem) : c;
    };

    // Weight slabs: slab (chunk, tap) lives at [chunk][tap][limb][K half][CoutP][32], i.e.
    // consecutive in memory in the order they are consumed; they never pass through LDS (see
    // the operand loads below).  t counts the slabs this workgroup multiplies.
    const int nslabs = (skipping ? __builtin_popcount(livemask) : a.nchunks) * a.taps;
    const int s0 = part * nslabs / nparts, s1 = (part + 1) * nslabs / nparts; // this workgroup's slabs
    const int slab_bytes = LIMBS * a.CoutP * CK;
    constexpr bool LATE_ROWS = LIMBS == 2; // (the one-limb kernels' 128 registers leave no room for the overlap)
    if constexpr (!LATE_ROWS) row_tables();
    __syncthreads(); // the patch tables are complete

    int aoff[MB]; // filled once the row tables are visible
    auto lane_constants = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = wm * WROWS + mb * 32 + l32;
            // the row's (r=0, s=0) pixel: the lane's 16-byte slot of the first K half in it
            aoff[mb] = apos[abase_s[row]] + kg * 16;
        }
    };
    if constexpr (!LATE_ROWS) lane_constants();
    v16i acc[MB][NB][NACC]; // zeroed after the first patch is staged: until then its registers are free

    // Activations travel global -> registers -> LDS in batches of APF 16-byte pieces per thread,
    // two batches in flight: while one is unpacked and parked, the next is on its way.  PIECES:
    // 16-byte pieces per staged pixel and chunk (8 x 8 int16 codes, or 4 x 16 int8 codes); since
    // THREADS is a multiple of PIECES, a thread always handles the same piece of its pixels.
    // A chunk's channel sums are collected by the part that holds the chunk's first tap, so that
    // parts which share a chunk do not count it twice.
    bool own_sums = (s0 % a.taps) == 0;
    constexpr int APF = kStageBatch;
    constexpr int PIECES = (LIMBS == 2) ? 8 : 4;
    constexpr int ESZ_X = (LIMBS == 2) ? 2 : 1;
    v4i aregA[APF], aregB[APF];
    int atA[APF], atB[APF];
    const int apiece = tid & (PIECES - 1), apix0 = tid / PIECES;
    // Loads go through a buffer descriptor that covers exactly the input tensor: a piece outside
    // the image or past the last channel is given an offset beyond it and reads as zeros, the
    // code 0, with no branch and no select on the data.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((unsigned)(a.N * a.H * a.W) * (unsigned)a.Cin * ESZ_X), 0x00020000);
    // piece number `first + tid` of chunk cc: request it / unpack it and park it in LDS
    // A staged pixel's table entries carry everything that does not depend on the chunk, so a
    // piece costs one table read and one add on the way in, one table read and one add on the
    // way out: the source offset is the pixel's entry plus the piece's channel offset (a
    // saturating add: either being all ones, the sum is all ones and the piece reads as zeros),
    // the LDS position is the pixel's entry plus the place of the thread's piece in the pixel
    // (16-byte slot, and for limb bytes the 8-byte half of it).
    const int piece_at = LIMBS == 2 ? ((apiece >> 1) << 4) | ((apiece & 1) << 3) : apiece << 4;
    // The LDS position is read together with the source offset, when the piece is requested:
    // read where the piece is parked, it would wait for the LDS writes of the piece before it
    // (LDS operations complete in order), a round trip per piece.
    // chb: byte offset of the thread's piece inside a pixel for the chunk being staged (see
    // channel_offset)
    auto load_piece = [&](unsigned chb, int first, v4i &reg, int &at) __attribute__((always_inline)) {
        const int p = apix0 + first / PIECES;
        const unsigned off = __builtin_elementwise_add_sat((unsigned)tab[p], chb);
        at = apos[p] + piece_at;
        const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)off, 0, 0);
        reg = (v4i){(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
    };
    auto store_piece = [&](int first, const v4i &reg, int at) __attribute__((always_inline)) {
        const int p = apix0 + first / PIECES;
        const v4i v = reg;
        if constexpr (LIMBS == 2) {
            v2i hi, lo;
            hi.x = (int)__builtin_amdgcn_perm((unsigned)v.y, (unsigned)v.x, 0x07050301u);
            hi.y = (int)__builtin_amdgcn_perm((unsigned)v.w, (unsigned)v.z, 0x07050301u);
            lo.x = (int)(__builtin_amdgcn_perm((unsigned)v.y, (unsigned)v.x, 0x06040200u) ^ 0x80808080u);
            lo.y = (int)(__builtin_amdgcn_perm((unsigned)v.w, (unsigned)v.z, 0x06040200u) ^ 0x80808080u);
            // sum of the eight codes: four two-element dot products with (1, 1); each of a
            // pixel's eight pieces adds its share to the pixel's sum
            const v2s ones = {1, 1};
            const int w0 = v.x, w1 = v.y, w2 = v.z, w3 = v.w;
            int sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, w0), ones, 0, false);
            sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, w1), ones, sum, false);
            sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, w2), ones, sum, false);
            sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, w3), ones, sum, false);
            if (own_sums) atomicAdd(&psum[p], sum); // no value returned
            *(__attribute__((address_space(3))) v2i *)(unsigned)at = hi;
            *(__attribute__((address_space(3))) v2i *)(unsigned)(at + APL) = lo;
        } else {
            *(__attribute__((address_space(3))) v4i *)(unsigned)at = v;
        }
    };
    auto channel_offset = [&](int cc) __attribute__((always_inline)) {
        const int ch = cc * CK + apiece * (CK / PIECES);
        unsigned chb = ch < a.Cin ? (unsigned)ch * ESZ_X : 0xffffffffu;
        asm volatile("" : "+v"(chb)); // opaque: one select per staging, not one per piece behind the saturating add
        return chb;
    };
    auto load_act = [&](unsigned chb, int first, v4i *reg, int *at) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < APF; ++j) load_piece(chb, first + j * THREADS, reg[j], at[j]);
    };
    auto store_act = [&](int first, const v4i *reg, const int *at) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < APF; ++j) store_piece(first + j * THREADS, reg[j], at[j]);
    };
    constexpr int DEEP = 8;
    // between(): work that does not depend on the patch, done while the first requests fly
    auto stage_activations = [&](int cc, bool deep, auto between) __attribute__((always_inline)) {
        // two batches of requests in flight; a request past the end of the patch reads as
        // zeros and is parked in the spare slot (see the patch tables)
        const int total = NPIXA * PIECES;
        const unsigned chb = channel_offset(cc);
        int first = 0;
        if (deep) {
            // the accumulators are not live yet: request the first DEEP pieces of every
            // thread at once and pay the memory latency a single time
            v4i d[DEEP];
            int dat[DEEP];
#pragma unroll
            for (int j = 0; j < DEEP; ++j) load_piece(chb, j * THREADS, d[j], dat[j]);
            between();
#pragma unroll
            for (int j = 0; j < DEEP; ++j) store_piece(j * THREADS, d[j], dat[j]);
            first = DEEP * THREADS;
            if (first >= total) {
                __builtin_amdgcn_s_waitcnt(0x0F70);
                return;
            }
        }
        // Two batches of requests are in flight inside the loop; the last two batches are
        // taken out of it, so that no request is left in flight when the staging is over (its
        // destination registers are reused in the multiply loop, and the wait that protects
        // them would sit at the top of every slab, where it would also wait for the weight
        // operands just requested) and the loop has one way out.
        load_act(chb, first, aregA, atA);
        for (; first + 2 * APF * THREADS < total; first += 2 * APF * THREADS) {
            load_act(chb, first + APF * THREADS, aregB, atB);
            store_act(first, aregA, atA);
            load_act(chb, first + 2 * APF * THREADS, aregA, atA);
            store_act(first + APF * THREADS, aregB, atB);
        }
        load_act(chb, first + APF * THREADS, aregB, atB);
        store_act(first, aregA, atA);
        store_act(first + APF * THREADS, aregB, atB);
        // vmcnt(0), stated where every path passes (the waits above sit partly inside branches
        // on lane masks); by now it costs nothing
        __builtin_amdgcn_s_waitcnt(0x0F70);
    };
    // chunk and tap of the current slab, and the tap's patch offset, kept incrementally
    // (when chunks are skipped the workgroup owns its whole tile: s0 = 0 and the first chunk is
    // the first one that is multiplied)
    int cc, tap, tap_r = 0, tap_s = 0;
    udivmod(s0, a.taps, a.mg_taps, cc, tap);
    if (skipping) cc = __builtin_ctz(livemask);
    udivmod(tap, a.S, a.mg_S, tap_r, tap_s);
    int taprow = tap_r * a.PITCH, tapoff = taprow + tap_s * PSP;
    // Weights go straight from global memory / L2 into the MFMA operand registers, NSETS - 1
    // K=32 halves ahead of their use; with no slab to publish, the waves of a workgroup meet only
    // when a new patch is staged.  A lane's B operand for (slab, K half, limb, column block) is the
    // 16 bytes number lane / 32 of row (column block + lane % 32) in the slab's block for that half
    // (see slab_byte): the 64 pieces of one request are consecutive memory.
    // NSETS register sets rotate: the half being multiplied owns one, the requests for the next
    // NSETS - 1 halves are in flight into the others.  Which set a half uses is fixed at compile
    // time, so the loop below is unrolled over a whole rotation (UT slabs).
    constexpr int NSETS = 3, LEAD = NSETS - 1;
    constexpr int UT = (NSETS % 2 == 0) ? NSETS / 2 : NSETS;
    v4i bh[NSETS][NB], bl[NSETS][NB];
    // One descriptor over the packed weights; a lane's byte offset inside a slab never changes,
    // the slab (and the limb plane) is a scalar offset, the K half an immediate: no address
    // arithmetic in vector registers inside the loop.
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(a.wp), 0, (int)((unsigned)(a.nchunks * a.taps) * (unsigned)slab_bytes), 0x00020000);
    const int blane = ((ntile * BN + wn * (NB * 32) + l32) * 32 + kg * 16);
    const int limb_bytes = a.CoutP * CK, half_bytes = a.CoutP * 32;
    // request the operands of K half `half` of the slab at byte offset wslab (past the last slab
    // the last one is read again and never used: every path issues the same number of requests)
    int wcur = (cc * a.taps + tap) * slab_bytes, wnext = wcur; // the slab being multiplied, the one after it
    auto bload = [&](int wslab, int half, v4i *h, v4i *l) __attribute__((always_inline)) {
        const int slab_off = wslab + (half ? half_bytes : 0);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const auto vh = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, blane + nb * 32 * 32, slab_off, 0);
            h[nb] = (v4i){(int)vh[0], (int)vh[1], (int)vh[2], (int)vh[3]};
            if constexpr (LIMBS == 2) {
                const auto vl = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, blane + nb * 32 * 32, slab_off + limb_bytes, 0);
                l[nb] = (v4i){(int)vl[0], (int)vl[1], (int)vl[2], (int)vl[3]};
            }
        }
    };
    // The activation fragments (A operands) of a row block stay in registers from their LDS read
    // to the MFMAs that consume them.  They are read one step ahead: as soon as the MFMAs of row
    // block mb of a K half are issued, the fragments of the same row block for the next K half (of
    // this slab or the next) are requested, so that the LDS latency runs under the other row
    // block's MFMAs.
    v4i ah[MB], al[MB];
    // off / offl are the LDS addresses themselves (high and low plane), so that a read costs no
    // address arithmetic
    typedef __attribute__((address_space(3))) const v4i lds_cv4i;
    auto afetch = [&](int mb, int off, int offl) __attribute__((always_inline)) {
        ah[mb] = *(lds_cv4i *)(unsigned)off;
        if constexpr (LIMBS == 2) al[mb] = *(lds_cv4i *)(unsigned)offl;
    };
    auto mfma_mb = [&](int mb, const v4i *wh, const v4i *wl) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            acc[mb][nb][0] = mfma_i8(wh[nb], ah[mb], acc[mb][nb][0]);
            if constexpr (LIMBS == 2) {
                acc[mb][nb][1] = mfma_i8(wl[nb], ah[mb], acc[mb][nb][1]);
                acc[mb][nb][2] = mfma_i8(wl[nb], al[mb], acc[mb][nb][2]);
            }
        }
        if constexpr (LIMBS == 2) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[mb][nb][1] = mfma_i8(wh[nb], al[mb], acc[mb][nb][1]);
        }
    };
    constexpr int HALF2 = 32;
    auto second_half = [&](int off) __attribute__((always_inline)) { return off + HALF2; };
    using std::integral_constant;
    // One K half of slab t, which is slab number P of the current rotation: request the weights
    // that are LEAD halves ahead, then multiply this half row block by row block.  cur / nxt:
    // fragment offsets of this slab and the next.  The second half always requests the next
    // slab's fragments, also when a new patch comes first (they are then read again after the
    // staging) or nothing follows: the offsets stay inside the patch, and a request that does
    // not depend on the path keeps the fragment registers from being doubled.
    auto half_step = [&](int t, auto P, auto HH, const int *cur, const int *curl, const int *nxt, const int *nxtl) __attribute__((always_inline)) {
        constexpr int hh = decltype(HH)::value;
        constexpr int h = 2 * decltype(P)::value + hh;
        constexpr int use = h % NSETS, fill = (h + LEAD) % NSETS;
        constexpr int ahead = hh + LEAD;
        static_assert((ahead >> 1) == 1, "the prefetch runs one slab ahead");
        bload(wnext, ahead & 1, bh[fill], bl[fill]);
        // the requests leave before this half's MFMAs, not among them
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            mfma_mb(mb, bh[use], bl[use]);
            __builtin_amdgcn_sched_barrier(0);
            if (hh == 0) afetch(mb, second_half(cur[mb]), second_half(curl[mb]));
            else afetch(mb, nxt[mb], nxtl[mb]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // fragment offsets of the slab the tap bookkeeping points at: the lane's slot (kg) of its
    // pixel per row block; the second K=32 half is slot kg+2, 32 bytes further.  A tap moves every
    // lane by the same amount, so a slab costs one add per row block.
    auto fragment_offsets = [&](int *afrag, int *afragl) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            afrag[mb] = aoff[mb] + tapoff;
            afragl[mb] = afrag[mb] + APL;
        }
    };
#pragma unroll
    for (int j = 0; j < LEAD; ++j) {
        static_assert(LEAD == 2, "the first slab's two K halves are requested here");
        bload(wcur, j & 1, bh[j], bl[j]);
    }

    stage_activations(cc, true, [&] {
        if constexpr (LATE_ROWS) row_tables();
    });
    own_sums = true; // every later chunk starts at its first tap
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int q = 0; q < NACC; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][nb][q][v] = 0;
    int cur[MB], curl[MB];
    if constexpr (!LATE_ROWS) fragment_offsets(cur, curl);
    __syncthreads(); // the freshly staged patch and the row tables are visible
    // Inside the multiply loop a wave runs at raised priority: the waves of the other workgroups
    // on the SIMD that are staging a patch or storing a tile mostly wait for memory, and the
    // matrix pipe should not wait for their address arithmetic (measured: 1 % on the VGG16 stack;
    // the opposite choice costs 1 %).
    __builtin_amdgcn_s_setprio(3);
    if constexpr (LATE_ROWS) {
        lane_constants();
        fragment_offsets(cur, curl);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) afetch(mb, cur[mb], curl[mb]);
    auto step = [&](int t, auto P) __attribute__((always_inline)) {
        // move the bookkeeping on to slab t + 1
        if (++tap == a.taps) {
            tap = 0;
            cc = next_chunk(cc);
            tap_s = tap_r = 0;
            tapoff = taprow = 0;
        } else {
            tapoff += PSP;
            if (++tap_s == a.S) {
                tap_s = 0;
                ++tap_r;
                taprow += a.PITCH;
                tapoff = taprow;
            }
        }
        int nxt[MB], nxtl[MB];
        fragment_offsets(nxt, nxtl);
        const bool more = t + 1 < s1;
        const bool restage = more && tap == 0; // slab t + 1 opens a chunk: a new patch
        wnext = more ? (cc * a.taps + tap) * slab_bytes : wcur;
        half_step(t, P, integral_constant<int, 0>{}, cur, curl, nxt, nxtl);
        half_step(t, P, integral_constant<int, 1>{}, cur, curl, nxt, nxtl);
        if (restage) {
            __builtin_amdgcn_s_setprio(0);
            __syncthreads(); // all reads of the previous chunk's activations are done
            stage_activations(cc, false, [] {});
            __syncthreads(); // the freshly staged patch is visible
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) afetch(mb, nxt[mb], nxtl[mb]);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            cur[mb] = nxt[mb];
            curl[mb] = nxtl[mb];
        }
        wcur = wnext;
    };
    // whole rotations inside the loop, the slabs left over after it
    int t = s0;
    for (; t + UT <= s1; t += UT) {
        step(t, integral_constant<int, 0>{});
        if constexpr (UT > 1) step(t + 1, integral_constant<int, 1>{});
        if constexpr (UT > 2) step(t + 2, integral_constant<int, 2>{});
    }
    if constexpr (UT > 1) {
        if (t < s1) {
            step(t, integral_constant<int, 0>{});
            if constexpr (UT > 2) {
                if (t + 1 < s1) step(t + 1, integral_constant<int, 1>{});
            }
        }
    }

    __builtin_amdgcn_s_setprio(0);
    // ---- sum of the codes under a tile row's window (two-limb correction term 128 * sum(a)):
    // the channel sums of its R x S patch pixels, complete since the last chunk was staged
    auto row_sum = [&](int m) __attribute__((always_inline)) {
        const int base = abase_s[m];
        int sum = 0;
        if (a.R == 3 && a.S == 3) { // the common window, unrolled: nine independent LDS reads
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) sum += psum[base + r * a.PW + s];
            return sum;
        }
        for (int r = 0; r < a.R; ++r)
            for (int s = 0; s < a.S; ++s) sum += psum[base + r * a.PW + s];
        return sum;
    };

    // ---- tail tiles: a part stores its accumulators and row sums and is done; the finishing
    // kernel adds the parts up (integer sums: the order cannot matter) and runs the epilogue.
    if (nparts > 1) {
        const int tail_tile = xcd * (a.per_xcd - a.full_per_xcd) + (tl - a.full_per_xcd);
        v4i *mine = (v4i *)(a.partials + ((size_t)tail_tile * nparts + part) * a.part_bytes);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int q = 0; q < NACC; ++q)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const v16i &c = acc[mb][nb][q];
                        mine[(((mb * NB + nb) * NACC + q) * 4 + g) * THREADS + tid] =
                            (v4i){c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
                    }
        if constexpr (LIMBS == 2) {
            int *rs = (int *)(mine + MB * NB * NACC * 4 * THREADS);
            for (int m = tid; m < BM; m += THREADS) rs[m] = row_sum(m);
        }
        if (a.zero_partial && tid == 0) a.zero_partial[blockIdx.x] = a.zero_partial[a.partial_stride + blockIdx.x] = 0;
        if (a.zout && part == 0 && tid == 0) a.zout[wi] = 0; // the finishing kernel sets it if it meets a nonzero code
        return;
    }

    const TileCounts counts = tile_epilogue<LIMBS, NB, BN, MB, 4>(a, acc, row_sum, outoff, pooloff, ctab, ntile, wm * WROWS,
                                                                  wn * (NB * 32), 0, 0);
    // one pair of counts per workgroup; on large grids they go to per-workgroup slots, not to the
    // counters: thousands of same-address atomics would serialise
    if (a.zero_partial || a.zout || a.direct_counts) {
        if (lane == 0) { // tab[] was last read while staging
            tab[wave] = (int)counts.zeros;
            tab[THREADS / 64 + wave] = (int)counts.sats;
        }
        __syncthreads();
        if (tid < 2) {
            unsigned total = 0;
            for (int w = 0; w < THREADS / 64; ++w) total += (unsigned)tab[tid * (THREADS / 64) + w];
            publish_count(a, tid, total);
        }
        if (a.zout && wave == 0) {
            // the tile's flag: it holds a code that is not zero (codes that exist: rows x channels)
            int rows = 0;
            for (int m = lane; m < BM; m += 64) rows += (int)wave_count(outoff[m] >= 0);
            unsigned zeros = 0;
            for (int w = 0; w < THREADS / 64; ++w) zeros += (unsigned)tab[w];
            if (lane == 0) a.zout[wi] = (unsigned)(rows * min(BN, a.Cout - ntile * BN)) != zeros;
        }
    }
}


// Finishes the tail tiles.  A tile's parts are added up and the epilogue run by 4 * MB workgroups,
// one per (32-row block, channel group of the MFMA layout): each thread then needs only NB * NACC
// 16-byte pieces per part, so the pieces of all parts are requested together and the memory
// latency is paid once.  Zero counts go straight to the total (few workgroups); workgroup 0 also
// adds the per-workgroup counts of the main kernel.
template <int LIMBS, int NB, int MB>
__global__ __launch_bounds__(256) void conv_finish_kernel(const ConvArgs a, int main_grid)
{
    constexpr int THREADS = 256;
    constexpr int BN = 64 * NB;
    constexpr int NACC = (LIMBS == 2) ? 3 : 1;
    constexpr int SUB = 4 * MB;       // workgroups per tile
    constexpr int MAXP = 8;           // most parts a tile is cut into (see choose_split)
    __shared__ int outoff[BM];
    __shared__ int rowsum[BM];
    __shared__ int pooloff[BM];
    __shared__ __align__(16) int ctab[3 * BN];
    __shared__ unsigned wave_zeros[2][THREADS / 64]; // [zeros, clipped][wave]
    const int tid = threadIdx.x;
    const int tails = a.per_xcd - a.full_per_xcd;
    const int tile_b = blockIdx.x / SUB, sub = blockIdx.x % SUB;
    const int mb0 = sub >> 2, g0 = sub & 3;
    const int xcd = tile_b / tails, tl = a.full_per_xcd + tile_b % tails;
    const int wi = xcd * a.per_xcd + tl;
    unsigned long long total = 0; // thread 0: zeros, thread 1: clipped values
    if (wi < a.total_work) {
        const int mtile = wi / a.tiles_n, ntile = wi % a.tiles_n;
        const int tile_r = mtile / a.tiles_c, tile_c = mtile % a.tiles_c;
        const int fr0 = tile_r * a.RH, x0 = tile_c * a.TW;
        // every request first: accumulator pieces and row sums of all parts
        const unsigned char *slots = a.partials + (size_t)tile_b * a.split * a.part_bytes;
        v4i piece[MAXP][NB][NACC];
        int rsp[MAXP];
#pragma unroll
        for (int o = 0; o < MAXP; ++o) {
            const unsigned char *theirs = slots + (size_t)min(o, a.split - 1) * a.part_bytes; // clamped: unconditional loads
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int q = 0; q < NACC; ++q)
                    piece[o][nb][q] = ((const v4i *)theirs)[((((mb0 * NB + nb) * NACC + q) * 4 + g0) * THREADS) + tid];
            rsp[o] = (LIMBS == 2 && tid < BM) ? ((const int *)(theirs + (size_t)MB * NB * NACC * 4 * THREADS * 16))[tid] : 0;
        }
        for (int m = tid; m < BM; m += THREADS) {
            const int j = m / a.TW, t = m % a.TW;
            const int fr = fr0 + j, xo = x0 + t;
            const bool ok = j < a.RH && fr < a.FR && xo < a.Wo;
            outoff[m] = ok ? fr * a.Wo + xo : -1;
            pooloff[m] = (a.pool && ok && !(j & 1) && !(t & 1))
                             ? ((fr / a.Ho) * (a.Ho >> 1) + ((fr % a.Ho) >> 1)) * (a.Wo >> 1) + (xo >> 1) : -1;
        }
        build_colterms<BN, THREADS>(a, ntile, ctab, LIMBS);
        v16i acc[1][NB][NACC];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int q = 0; q < NACC; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[0][nb][q][v] = 0;
        int rs = 0;
#pragma unroll
        for (int o = 0; o < MAXP; ++o) {
            if (o < a.split) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int q = 0; q < NACC; ++q) {
                        acc[0][nb][q][0] += piece[o][nb][q].x;
                        acc[0][nb][q][1] += piece[o][nb][q].y;
                        acc[0][nb][q][2] += piece[o][nb][q].z;
                        acc[0][nb][q][3] += piece[o][nb][q].w;
                    }
                rs += rsp[o];
            }
        }
        if (tid < BM) rowsum[tid] = rs;
        __syncthreads();
        // same wave arrangement as the main kernel: BM / (32 * MB) waves along the pixels
        constexpr int WMC = BM / (32 * MB);
        const int wave = tid >> 6;
        const TileCounts counts = tile_epilogue<LIMBS, NB, BN, 1, 1>(
            a, acc, [&](int m) { return rowsum[m]; }, outoff, pooloff, ctab, ntile, (wave % WMC) * (32 * MB),
            (wave / WMC) * (NB * 32), mb0, g0);
        if (a.zout) {
            // codes of this workgroup's part of the tile that exist; a zero count below it = a nonzero code
            const int m = (wave % WMC) * (32 * MB) + mb0 * 32 + (tid & 31);
            const int col0 = ntile * BN + (wave / WMC) * (NB * 32) + 8 * g0 + 4 * ((tid & 63) >> 5);
            unsigned exist = 0;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) exist += outoff[m] >= 0 ? (unsigned)min(max(a.Cout - (col0 + nb * 32), 0), 4) : 0u;
            unsigned wave_exist = 0;
#pragma unroll
            for (int b = 0; b < 5; ++b) wave_exist += wave_count((exist >> b) & 1) << b;
            if ((tid & 63) == 0 && wave_exist != counts.zeros) a.zout[wi] = 1;
        }
        if ((tid & 63) == 0) {
            wave_zeros[0][tid >> 6] = counts.zeros;
            wave_zeros[1][tid >> 6] = counts.sats;
        }
        __syncthreads();
        if (tid < 2)
            for (int w = 0; w < THREADS / 64; ++w) total += wave_zeros[tid][w];
    }
    if (!a.zero_partial) return;
    if (blockIdx.x == 0) {
        unsigned long long sum[2] = {0, 0};
        for (int i = tid; i < main_grid; i += THREADS) {
            sum[0] += a.zero_partial[i];
            sum[1] += a.zero_partial[a.partial_stride + i];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            sum[0] += __shfl_down(sum[0], off, 64);
            sum[1] += __shfl_down(sum[1], off, 64);
        }
        __syncthreads(); // wave_zeros[] has been read
        if ((tid & 63) == 0) { // a launch has fewer than 2^32 outputs
            wave_zeros[0][tid >> 6] = (unsigned)sum[0];
            wave_zeros[1][tid >> 6] = (unsigned)sum[1];
        }
        __syncthreads();
        if (tid < 2)
            for (int w = 0; w < THREADS / 64; ++w) total += wave_zeros[tid][w];
    }
    if (tid == 0 && total && a.zero_count) atomicAdd(a.zero_count, total);
    if (tid == 1 && total && a.sat_count) atomicAdd(a.sat_count, total);
}

// Adds the per-workgroup counts to the caller's counters: blockIdx.y = 0 the zero counts, 1 the
// counts of clipped values (launched only when wanted); a few blocks, eight independent loads per
// thread and pass, one atomic per block.  Either counter may be null.
__global__ __launch_bounds__(256) void sum_partials_kernel(const unsigned *__restrict__ partials, int n,
                                                          unsigned long long *out_zero, unsigned long long *out_sat)
{
    __shared__ unsigned long long part[4];
    const unsigned *partial = partials + (size_t)blockIdx.y * n;
    unsigned long long *out = blockIdx.y ? out_sat : out_zero;
    if (!out) return;
    unsigned long long s = 0;
    for (int i0 = blockIdx.x * 2048 + threadIdx.x; i0 < n; i0 += gridDim.x * 2048) {
        unsigned v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (i0 + j * 256 < n) ? partial[i0 + j * 256] : 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) s += v[j];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_down(s, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long t = part[0] + part[1] + part[2] + part[3];
        if (t) atomicAdd(out, t);
    }
}


// Layers with very few input channels (the first VGG16 layer: Cin = 3, K = 27): the whole R*S*Cin
// window is one K <= 64 slab, the layer is bound by its output (64 codes written per 27 read) and by
// the vector instructions of the epilogue, and everything that the patch kernel does between
// global memory and the MFMA is overhead.  Here a wave owns 32 tile rows x all NCB*32 channels of
// the tile, and lane (row, K quarter) gathers the 16 window codes of its MFMA operand straight
// from the raw input patch in LDS into registers: no staged planes, no fragment reads, one
// barrier.  The sum of a row's codes (offset correction) is the sum over its lanes' gathers.
// NCB: 32-channel blocks per tile (1 for layers with at most 32 output channels); KS: K halves (1: K <= 32).
template <int NCB, int KS>
__global__ __launch_bounds__(256)
    __attribute__((amdgpu_waves_per_eu(NCB * KS == 4 ? 3 : 4, NCB * KS == 4 ? 3 : 4))) void conv_flat_kernel(const ConvArgs a)
{
    constexpr int THREADS = 256, BN = 64;
    __shared__ __align__(16) short raw[kFlatRawBytes / 2]; // the raw input patch, all channels (the planner keeps it within)
    __shared__ v4i wlds[KS * 2 * NCB][64];      // weight operands: [(K half, limb, column block)][lane]
    __shared__ int koff[64];                    // window position k -> byte offset behind the window's first code
    __shared__ int outoff[BM], pooloff[BM], abase[BM];
    __shared__ __align__(16) int ctab[3 * BN];
    __shared__ unsigned wave_counts[2][THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int wi = xcd * a.per_xcd + slot;
    if (slot >= a.per_xcd || wi >= a.total_work) {
        if (a.zero_partial && tid == 0) a.zero_partial[blockIdx.x] = a.zero_partial[a.partial_stride + blockIdx.x] = 0;
        return;
    }
    int mtile, ntile, tile_r, tile_c, img0, yo0;
    udivmod(wi, a.tiles_n, a.mg_tiles_n, mtile, ntile);
    udivmod(mtile, a.tiles_c, a.mg_tiles_c, tile_r, tile_c);
    const int fr0 = tile_r * a.RH, x0 = tile_c * a.TW;
    udivmod(fr0, a.Ho, a.mg_Ho, img0, yo0);
    const int vr0 = img0 * a.Hp + yo0;

    // weights of the tile: a lane's operand for (K half, limb, column block) is 16 bytes of the row
    // it owns (see slab_byte).  The waves share the WPIECES operands of 64 lanes each: requested
    // first, parked in LDS, read back when a column block is multiplied.
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(a.wp), 0, 2 * a.CoutP * CK, 0x00020000);
    constexpr int WPIECES = KS * 2 * NCB, WPT = (WPIECES + 3) / 4; // piece = (h * 2 + limb) * NCB + cb
    v4i wreg[WPT];
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        const int piece = wave + 4 * i;
        const int cb = piece % NCB, hl = piece / NCB, limb = hl & 1, h = hl >> 1;
        const int at = ((h * a.CoutP + ntile * BN + cb * 32 + l32) * 32) + kg * 16 + limb * a.CoutP * CK;
        const auto v = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, piece < WPIECES ? at : (int)0x80000000, 0, 0);
        wreg[i] = (v4i){(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
    }
    // raw patch, row by row: a patch row is PW * Cin consecutive codes of an image row (code e of
    // patch row pr is code (x0 - pad) * Cin + e of that image row); codes outside the image read as 0
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((unsigned)(a.N * a.H * a.W) * (unsigned)a.Cin * 2u), 0x00020000);
    const int nraw = a.NPIXA * a.Cin, rowlen = a.PW * a.Cin, wlen = a.W * a.Cin;
    const int e0 = (x0 - a.pad) * a.Cin;
    constexpr int RU = 3; // requests in flight per thread (a 18 x 10 x 3 patch is 2.1 codes per thread)
    for (int i0 = tid; i0 < nraw; i0 += RU * THREADS) {
        short v[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int i = min(i0 + u * THREADS, nraw - 1);
            int pr, e, n, iy;
            udivmod(i, rowlen, a.mg_rowlen, pr, e);
            udivmod(vr0 + pr, a.Hp, a.mg_Hp, n, iy);
            iy -= a.pad;
            const int c = e0 + e; // position in the image row, in codes
            const bool in = n < a.N && iy >= 0 && iy < a.H && c >= 0 && c < wlen;
            const unsigned off = in ? (unsigned)((n * a.H + iy) * wlen + c) * 2u : 0xffffffffu;
            v[u] = (short)__builtin_amdgcn_raw_buffer_load_b16(xrsrc, (int)off, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < RU; ++u)
            if (i0 + u * THREADS < nraw) raw[i0 + u * THREADS] = v[u];
    }
    // tables: window position -> offset, tile row -> output pixel / window start, channel constants
    const int SC = a.S * a.Cin;
    for (int k = tid; k < 64; k += THREADS) {
        int r, rem;
        udivmod(k, SC, a.mg_SC, r, rem);
        koff[k] = k < a.Kflat ? 2 * (r * a.PW * a.Cin + rem) : 0;
    }
    for (int m = tid; m < BM; m += THREADS) {
        int j, t, img, yo;
        udivmod(m, a.TW, a.mg_TW, j, t);
        const int fr = fr0 + j, xo = x0 + t;
        const bool ok = j < a.RH && fr < a.FR && xo < a.Wo;
        udivmod(fr, a.Ho, a.mg_Ho, img, yo);
        outoff[m] = ok ? fr * a.Wo + xo : -1;
        abase[m] = ok ? ((img * a.Hp + yo - vr0) * a.PW + t) * a.Cin * 2 : 0;
        pooloff[m] = (a.pool && ok && !(j & 1) && !(t & 1)) ? (img * (a.Ho >> 1) + (yo >> 1)) * (a.Wo >> 1) + (xo >> 1) : -1;
    }
    build_colterms<BN, THREADS>(a, ntile, ctab, 2);
#pragma unroll
    for (int i = 0; i < WPT; ++i)
        if (wave + 4 * i < WPIECES) wlds[wave + 4 * i][lane] = wreg[i];
    __syncthreads();

    const unsigned char *rawb = (const unsigned char *)raw;
    const int base = abase[wave * 32 + l32];
    int sum = 0;
    v4i ah[KS], al[KS];
#pragma unroll
    for (int h = 0; h < KS; ++h) {
        // the lane's 16 window codes k0 .. k0 + 15, two per register, then split into limb bytes
        const int k0 = h * 32 + kg * 16;
        const v4i o0 = *(const v4i *)(koff + k0), o1 = *(const v4i *)(koff + k0 + 4);
        const v4i o2 = *(const v4i *)(koff + k0 + 8), o3 = *(const v4i *)(koff + k0 + 12);
        const int o[16] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w, o2.x, o2.y, o2.z, o2.w, o3.x, o3.y, o3.z, o3.w};
        unsigned pr[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const v2s two = {*(const short *)(rawb + base + o[2 * q]), *(const short *)(rawb + base + o[2 * q + 1])};
            pr[q] = __builtin_bit_cast(unsigned, two);
        }
        const int nv = a.Kflat - k0; // codes of this piece that exist (the same for half a wave)
        if (nv < 16) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int m = min(max(nv - 2 * q, 0), 2);
                pr[q] &= m == 2 ? 0xffffffffu : m == 1 ? 0xffffu : 0u;
            }
        }
        unsigned hi[4], lo[4];
        const v2s ones = {1, 1};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            hi[q] = __builtin_amdgcn_perm(pr[2 * q + 1], pr[2 * q], 0x07050301u);
            lo[q] = __builtin_amdgcn_perm(pr[2 * q + 1], pr[2 * q], 0x06040200u) ^ 0x80808080u;
            sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pr[2 * q]), ones, sum, false);
            sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pr[2 * q + 1]), ones, sum, false);
        }
        // (a position past K is the code 0 = limbs (0, -128) here; it meets zero weights)
        ah[h] = v4i{(int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        al[h] = v4i{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3]};
    }
    // the row's code sum: its two lanes hold different window positions
    const int rowsum = sum + __shfl_xor(sum, 32, 64);
    // one 32-channel block at a time: its three accumulators, then its outputs
    TileCounts counts = {0, 0};
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        v16i acc[1][1][3];
#pragma unroll
        for (int q = 0; q < 3; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[0][0][q][v] = 0;
#pragma unroll
        for (int h = 0; h < KS; ++h) {
            const v4i wh = wlds[(h * 2 + 0) * NCB + cb][lane], wl = wlds[(h * 2 + 1) * NCB + cb][lane];
            acc[0][0][0] = mfma_i8(wh, ah[h], acc[0][0][0]);
            acc[0][0][1] = mfma_i8(wl, ah[h], acc[0][0][1]);
            acc[0][0][2] = mfma_i8(wl, al[h], acc[0][0][2]);
            acc[0][0][1] = mfma_i8(wh, al[h], acc[0][0][1]);
        }
        const TileCounts c = tile_epilogue<2, 1, BN, 1, 4>(
            a, acc, [&](int) { return rowsum; }, outoff, pooloff, ctab, ntile, wave * 32, cb * 32, 0, 0);
        counts.zeros += c.zeros;
        counts.sats += c.sats;
    }
    if (a.zero_partial || a.zout || a.direct_counts) {
        if (lane == 0) {
            wave_counts[0][wave] = counts.zeros;
            wave_counts[1][wave] = counts.sats;
        }
        __syncthreads();
        if (tid < 2) {
            unsigned total = 0;
            for (int w = 0; w < THREADS / 64; ++w) total += wave_counts[tid][w];
            publish_count(a, tid, total);
        }
        if (a.zout && wave == 0) {
            int rows = 0;
            for (int m = lane; m < BM; m += 64) rows += (int)wave_count(outoff[m] >= 0);
            unsigned zeros = 0;
            for (int w = 0; w < THREADS / 64; ++w) zeros += wave_counts[0][w];
            if (lane == 0) a.zout[wi] = (unsigned)(rows * min(BN, a.Cout - ntile * BN)) != zeros;
        }
    }
}

// Layers with 16, 32 or 48 input channels (16-bit codes): a 64-channel chunk would be mostly
// padding, so the reduction runs over window rows instead.  The patch is staged densely (Cin bytes
// per pixel and limb), which makes the S * Cin codes under one kernel row of a window consecutive:
// a window row is KHR = ceil(S * Cin / 32) K = 32 pieces at consecutive addresses.  The positions
// past S * Cin in a row's last piece read the neighbouring pixels and meet weight bytes (0, 0),
// which add nothing to any limb product.  A wave owns 32 tile rows and takes the tile's 32-channel
// blocks one after the other; the weights
// ([piece][limb][CoutP][32], pieces padded with zeros to a multiple of four) go from L2 straight
// into one of four rotating operand sets, three pieces ahead of their use.
// The sum of the codes under a window (offset correction) is gathered from per-unit sums (a unit
// = 16 consecutive codes of a pixel) left by the staging.
// NCB: 32-channel blocks a workgroup takes (1 for layers with at most 32 output channels).
template <int NCB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NCB == 1 ? 4 : 3, NCB == 1 ? 4 : 3))) void conv_rows_kernel(
    const ConvArgs a)
{
    constexpr int THREADS = 256, BN = 64, NSETS = 4;
    extern __shared__ __align__(16) unsigned char smem[];
    const int NU = a.NPIXA * a.CU; // units of the patch
    int *usum = (int *)smem;                    // unit -> sum of its 16 codes
    int *outoff = usum + ((NU + 3) & ~3);       // tile row -> output pixel index, -1 if not an output
    int *pooloff = outoff + BM;                 // tile row -> pooled output pixel (top-left rows of 2x2 windows), else -1
    int *abase = pooloff + BM;                  // tile row -> byte offset of its window's first code in a plane
    int *ubase = abase + BM;                    // tile row -> unit of its window's first code
    int *ctab = ubase + BM;                     // channel constants
    unsigned *wave_counts = (unsigned *)(ctab + 3 * BN); // [zeros, clipped][wave]
    unsigned char *Asm = (unsigned char *)(wave_counts + 2 * (THREADS / 64)); // high plane, then low plane
    const int APL = a.APLANE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int wi = xcd * a.per_xcd + slot;
    if (slot >= a.per_xcd || wi >= a.total_work) {
        if (a.zero_partial && tid == 0) a.zero_partial[blockIdx.x] = a.zero_partial[a.partial_stride + blockIdx.x] = 0;
        return;
    }
    int mtile, ntile, tile_r, tile_c, img0, yo0;
    udivmod(wi, a.tiles_n, a.mg_tiles_n, mtile, ntile);
    udivmod(mtile, a.tiles_c, a.mg_tiles_c, tile_r, tile_c);
    const int fr0 = tile_r * a.RH, x0 = tile_c * a.TW;
    udivmod(fr0, a.Ho, a.mg_Ho, img0, yo0);
    const int vr0 = img0 * a.Hp + yo0;

    // weight operands: a lane's 16 bytes of (piece, limb, column block) never move inside a piece;
    // the piece is a scalar offset.  Requests past the last piece read it again and are not used.
    const int piece_bytes = 2 * a.CoutP * 32;
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(a.wp), 0, a.KHP * piece_bytes, 0x00020000);
    int blane = (ntile * BN + l32) * 32 + kg * 16;
    v4i bh[NSETS], bl[NSETS];
    auto bload = [&](int h, v4i &hh, v4i &ll) __attribute__((always_inline)) {
        const int so = min(h, a.KHP - 1) * piece_bytes;
        const auto vh = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, blane, so, 0);
        const auto vl = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, blane, so + a.CoutP * 32, 0);
        hh = (v4i){(int)vh[0], (int)vh[1], (int)vh[2], (int)vh[3]};
        ll = (v4i){(int)vl[0], (int)vl[1], (int)vl[2], (int)vl[3]};
    };
#pragma unroll
    for (int h = 0; h < NSETS - 1; ++h) bload(h, bh[h], bl[h]);

    // patch: unit i = (patch row, 16 codes of it) -> limb bytes into the two planes, code sum into usum;
    // pixels outside the image read as zeros (an offset past the descriptor)
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((unsigned)(a.N * a.H * a.W) * (unsigned)a.Cin * 2u), 0x00020000);
    constexpr int UF = 2; // units in flight per thread
    for (int i0 = tid; i0 < NU; i0 += UF * THREADS) {
        v4i c[UF][2];
        int dst[UF];
#pragma unroll
        for (int u = 0; u < UF; ++u) {
            const int i = min(i0 + u * THREADS, NU - 1);
            int pr, uu, pc, q, n, iy;
            udivmod(i, a.UPR, a.mg_UPR, pr, uu);
            udivmod(uu, a.CU, a.mg_CU, pc, q);
            udivmod(vr0 + pr, a.Hp, a.mg_Hp, n, iy);
            iy -= a.pad;
            const int ix = x0 - a.pad + pc;
            const bool in = n < a.N && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
            const unsigned off = in ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cin + q * 16) * 2u : 0xffffffe0u;
            const auto v0 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)off, 0, 0);
            const auto v1 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)(off + 16u), 0, 0);
            c[u][0] = (v4i){(int)v0[0], (int)v0[1], (int)v0[2], (int)v0[3]};
            c[u][1] = (v4i){(int)v1[0], (int)v1[1], (int)v1[2], (int)v1[3]};
            dst[u] = pr * a.PITCH + uu * 16;
        }
#pragma unroll
        for (int u = 0; u < UF; ++u) {
            if (i0 + u * THREADS >= NU) continue;
            const unsigned pr2[8] = {(unsigned)c[u][0].x, (unsigned)c[u][0].y, (unsigned)c[u][0].z, (unsigned)c[u][0].w,
                                     (unsigned)c[u][1].x, (unsigned)c[u][1].y, (unsigned)c[u][1].z, (unsigned)c[u][1].w};
            unsigned hi[4], lo[4];
            int sum = 0;
            const v2s ones = {1, 1};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                hi[q] = __builtin_amdgcn_perm(pr2[2 * q + 1], pr2[2 * q], 0x07050301u);
                lo[q] = __builtin_amdgcn_perm(pr2[2 * q + 1], pr2[2 * q], 0x06040200u) ^ 0x80808080u;
                sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pr2[2 * q]), ones, sum, false);
                sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pr2[2 * q + 1]), ones, sum, false);
            }
            *(v4i *)(Asm + dst[u]) = v4i{(int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            *(v4i *)(Asm + APL + dst[u]) = v4i{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3]};
            usum[i0 + u * THREADS] = sum;
        }
    }
    for (int m = tid; m < BM; m += THREADS) {
        int j, t, img, yo;
        udivmod(m, a.TW, a.mg_TW, j, t);
        const int fr = fr0 + j, xo = x0 + t;
        const bool ok = j < a.RH && fr < a.FR && xo < a.Wo;
        udivmod(fr, a.Ho, a.mg_Ho, img, yo);
        const int prow = img * a.Hp + yo - vr0;
        outoff[m] = ok ? fr * a.Wo + xo : -1;
        abase[m] = ok ? prow * a.PITCH + t * a.Cin : 0;
        ubase[m] = ok ? prow * a.UPR + t * a.CU : 0;
        pooloff[m] = (a.pool && ok && !(j & 1) && !(t & 1)) ? (img * (a.Ho >> 1) + (yo >> 1)) * (a.Wo >> 1) + (xo >> 1) : -1;
    }
    build_colterms<BN, THREADS>(a, ntile, ctab, 2);
    __syncthreads();

    // the sum of the codes under the row's window: its two lanes take alternate window rows
    int sum = 0;
    {
        const int ub = ubase[wave * 32 + l32];
        for (int r = kg; r < a.R; r += 2)
            for (int u = 0; u < a.SU; ++u) sum += usum[ub + r * a.UPR + u];
    }
    const int rowsum = sum + __shfl_xor(sum, 32, 64);
    // the lane's 16-byte slot of its row's first window code, as an LDS address
    typedef __attribute__((address_space(3))) const v4i lds_cv4i;
    const int a_l = (int)(unsigned long)(__attribute__((address_space(3))) unsigned char *)Asm + abase[wave * 32 + l32] + kg * 16;
    using std::integral_constant;
    TileCounts counts = {0, 0};
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        if (cb) { // (the first block's first pieces were requested at the top)
            blane += 32 * 32;
#pragma unroll
            for (int h = 0; h < NSETS - 1; ++h) bload(h, bh[h], bl[h]);
        }
        v16i acc[1][1][3];
#pragma unroll
        for (int q = 0; q < 3; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[0][0][q][v] = 0;
        int kr = 0, kj = 0; // window row and piece within it of the next piece (pad pieces stay on the last row)
        auto step = [&](int h, auto P) __attribute__((always_inline)) {
            constexpr int use = decltype(P)::value, fill = (use + NSETS - 1) % NSETS;
            bload(h + NSETS - 1, bh[fill], bl[fill]);
            const int at = a_l + min(kr, a.R - 1) * a.PITCH + kj * 32;
            if (++kj == a.KHR) {
                kj = 0;
                ++kr;
            }
            const v4i ah = *(lds_cv4i *)(unsigned)at;
            const v4i al = *(lds_cv4i *)(unsigned)(at + APL);
            acc[0][0][0] = mfma_i8(bh[use], ah, acc[0][0][0]);
            acc[0][0][1] = mfma_i8(bl[use], ah, acc[0][0][1]);
            acc[0][0][2] = mfma_i8(bl[use], al, acc[0][0][2]);
            acc[0][0][1] = mfma_i8(bh[use], al, acc[0][0][1]);
        };
        for (int h = 0; h < a.KHP; h += NSETS) {
            step(h, integral_constant<int, 0>{});
            step(h + 1, integral_constant<int, 1>{});
            step(h + 2, integral_constant<int, 2>{});
            step(h + 3, integral_constant<int, 3>{});
        }
        const TileCounts c = tile_epilogue<2, 1, BN, 1, 4>(
            a, acc, [&](int) { return rowsum; }, outoff, pooloff, ctab, ntile, wave * 32, cb * 32, 0, 0);
        counts.zeros += c.zeros;
        counts.sats += c.sats;
    }
    if (a.zero_partial || a.zout || a.direct_counts) {
        if (lane == 0) {
            wave_counts[wave] = counts.zeros;
            wave_counts[THREADS / 64 + wave] = counts.sats;
        }
        __syncthreads();
        if (tid < 2) {
            unsigned total = 0;
            for (int w = 0; w < THREADS / 64; ++w) total += wave_counts[tid * (THREADS / 64) + w];
            publish_count(a, tid, total);
        }
        if (a.zout && wave == 0) {
            int rows = 0;
            for (int m = lane; m < BM; m += 64) rows += (int)wave_count(outoff[m] >= 0);
            unsigned zeros = 0;
            for (int w = 0; w < THREADS / 64; ++w) zeros += wave_counts[w];
            if (lane == 0) a.zout[wi] = (unsigned)(rows * min(BN, a.Cout - ntile * BN)) != zeros;
        }
    }
}


lp_status launch_sum_partials(const unsigned *partials, int n, unsigned long long *zero_count,
                              unsigned long long *sat_count, hipStream_t st)
{
    hipLaunchKernelGGL(sum_partials_kernel, dim3(std::min((n + 2047) / 2048, 16), sat_count ? 2 : 1), dim3(256), 0, st,
                       partials, n, zero_count, sat_count);
    return launch_status();
}

template <int LIMBS, int NB, int MB>
static lp_status launch_mfma(const ConvArgs &a, const Plan &p, int grid, int tails, hipStream_t st)
{
    // raise the dynamic LDS limit once per kernel instance and device
    static std::atomic<bool> attr_set[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LP_EDEVICE;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void *)conv_mfma_kernel<LIMBS, NB, MB>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return LP_EDEVICE;
        attr_set[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((conv_mfma_kernel<LIMBS, NB, MB>), dim3(grid), dim3(MB == 2 ? 256 : 512),
                       p.lds_bytes, st, a);
    if (tails) // the split tail tiles are merged and written by a second, small kernel
        hipLaunchKernelGGL((conv_finish_kernel<LIMBS, NB, MB>), dim3(tails * 4 * MB), dim3(256), 0, st, a, grid);
    return launch_status();
}

static WorkspaceLayout workspace_layout(const Plan &p)
{
    WorkspaceLayout w = {0, 0};
    if (p.path != PATH_MFMA) return w;
    const size_t tails = (size_t)kXCDs * (p.per_xcd - p.full_per_xcd);
    w.partials = round_up((size_t)2 * p.grid * sizeof(unsigned), 256); // zero counts, counts of clipped values
    w.total = w.partials + tails * p.split * p.part_bytes;
    return w;
}

// The 32-bit epilogue (and with it the fused pool) applies when only codes are wanted, with ReLU,
// round-half-away, a right shift of 1..31 bits, K <= 8192 and a bias shift of at most 24 bits,
// and when the pixels of a tile span less than 2^31 bytes of output.
static bool fast_epilogue_ok(const lp_conv_desc *d, const Plan &p, int f_acc, bool has_bias, lp_qfmt qb, lp_qfmt qy, int relu,
                             lp_round r)
{
    const long long K = (long long)d->R * d->S * d->Cin;
    const int s = f_acc - qy.f;
    const bool span_ok = (unsigned long long)p.RH * p.Wo * d->Cout * (qy.n > 8 ? 2 : 1) < (1ull << 31);
    return relu && r == LP_ROUND_NEAREST_AWAY && s >= 1 && s <= 31 && K <= 8192 && (!has_bias || f_acc - qb.f <= 24) && span_ok;
}

static lp_status conv_forward(const lp_conv_desc *d, const void *x, lp_qfmt qx, const void *wp,
                              lp_qfmt qw, const void *bias, lp_qfmt qb, int64_t *acc_out, void *y,
                              lp_qfmt qy, int relu, lp_round r, uint64_t *zero_count, uint64_t *sat_count,
                              void *workspace, size_t workspace_bytes, void *stream,
                              const lp_zero_map *x_map = nullptr, uint8_t *y_flags = nullptr, uint64_t *skipped = nullptr)
{
    Plan p;
    lp_status st = make_plan(d, qx, qw, &p);
    if (st != LP_OK) return st;
    if (!x || !wp || (!acc_out && !y) || !aligned16(x) || !aligned16(wp)) return LP_EINVAL;
    if ((acc_out && !aligned16(acc_out)) || (y && !aligned16(y))) return LP_EINVAL;
    const int f_acc = qx.f + qw.f;
    if (bias && (!fmt_ok(qb) || qb.f > f_acc || f_acc - qb.f > 40)) return LP_EINVAL;
    if (r != LP_ROUND_NEAREST_AWAY && r != LP_ROUND_NEAREST_EVEN) return LP_EINVAL;
    ConvArgs a = {};
    if (y) {
        if (!fmt_ok(qy)) return LP_EINVAL;
        const int s = f_acc - qy.f;
        if (s > 62 || s < -31) return LP_EINVAL;
        a.act = make_act_params(f_acc, qy, relu, r);
        a.y16 = qy.n > 8;
    }
    a.x = x;
    a.wp = (const unsigned char *)wp;
    a.corr = (const int64_t *)((const unsigned char *)wp + p.corr_offset);
    a.bias = bias;
    a.bias16 = bias ? (qb.n > 8) : 0;
    a.bias_shift = bias ? f_acc - qb.f : 0;
    a.acc_out = acc_out;
    a.y = y;
    a.zero_count = (unsigned long long *)zero_count;
    a.sat_count = (unsigned long long *)sat_count;
    a.count_sat = (sat_count && y) ? 1 : 0;
    if (x_map || y_flags) {
        // zero flags: read by the patch kernels, written by any MFMA-path layer that emits codes
        if (p.path != PATH_MFMA) return LP_EUNSUPPORTED;
        if (y_flags && (!y || !workspace)) return LP_EINVAL;
        if (x_map) {
            if (!x_map->flags_dev || x_map->tile_rows <= 0 || x_map->tile_cols <= 0 || x_map->tiles_c <= 0 ||
                x_map->tiles_n <= 0 || x_map->bn < CK || x_map->bn % CK || (x_map->scale != 1 && x_map->scale != 2))
                return LP_EINVAL;
            // the flags must describe this layer's input: its width and channels
            if (x_map->tiles_c != (d->W * x_map->scale + x_map->tile_cols - 1) / x_map->tile_cols ||
                x_map->tiles_n != (d->Cin + x_map->bn - 1) / x_map->bn)
                return LP_EINVAL;
            a.zin = x_map->flags_dev;
            a.z_rh = x_map->tile_rows; a.z_tw = x_map->tile_cols; a.z_tiles_c = x_map->tiles_c;
            a.z_tiles_n = x_map->tiles_n; a.z_bn = x_map->bn; a.z_scale = x_map->scale;
            a.skipped = (unsigned long long *)skipped;
        }
        a.zout = y_flags;
    }
    a.wsum = p.wsum_offset ? (const int *)((const unsigned char *)wp + p.wsum_offset) : nullptr;
    a.N = d->N; a.H = d->H; a.W = d->W; a.Cin = d->Cin; a.Cout = d->Cout;
    a.R = d->R; a.S = d->S; a.stride = d->stride; a.pad = d->pad;
    a.Ho = p.Ho; a.Wo = p.Wo; a.Hp = p.Hp; a.FR = p.FR;
    hipStream_t hs = as_stream(stream);
    clear_stale_error();
    if (p.path == PATH_DIRECT) {
        const size_t total = (size_t)p.FR * p.Wo * d->Cout;
        const int grid = (int)std::min<size_t>((total + 255) / 256, 256 * 64);
        if (qx.n > 8) hipLaunchKernelGGL(conv_direct_kernel<int16_t>, dim3(grid), dim3(256), 0, hs, a);
        else hipLaunchKernelGGL(conv_direct_kernel<int8_t>, dim3(grid), dim3(256), 0, hs, a);
        return launch_status();
    }
    a.RH = p.RH; a.TW = p.TW; a.PW = p.PW; a.NPIXA = p.NPIXA;
    a.NTAB = patch_table_len(p.limbs, p.NPIXA, p.flat);
    a.PITCH = p.PITCH;
    a.APLANE = p.flat ? 0 : p.rows ? p.PRA * p.PITCH + 32 : p.PRA * p.PITCH + PSP; // the last slot of a plane parks overshoot pieces
    a.KHR = p.KHR; a.KHP = p.KHP;
    a.CU = d->Cin / 16; a.UPR = p.PW * a.CU; a.SU = d->S * a.CU;
    a.mg_UPR = udiv_magic(a.UPR); a.mg_CU = udiv_magic(a.CU);
    a.tiles_c = p.tiles_c; a.tiles_n = p.tiles_n; a.CoutP = p.CoutP; a.nchunks = p.nchunks;
    a.taps = p.taps; a.ksteps = p.ksteps; a.Kflat = d->R * d->S * d->Cin;
    a.mg_tiles_n = udiv_magic(a.tiles_n); a.mg_tiles_c = udiv_magic(a.tiles_c);
    a.mg_Ho = udiv_magic(a.Ho); a.mg_Hp = udiv_magic(a.Hp);
    a.mg_PW = udiv_magic(a.PW); a.mg_TW = udiv_magic(a.TW);
    a.mg_taps = udiv_magic(a.taps); a.mg_S = udiv_magic(d->S);
    a.mg_Cin = udiv_magic(d->Cin); a.mg_SC = udiv_magic(d->S * d->Cin);
    a.mg_rowlen = udiv_magic(p.PW * d->Cin);
    a.total_work = p.tiles_m * p.tiles_n;
    a.per_xcd = p.per_xcd;
    a.full_per_xcd = p.full_per_xcd;
    a.split = p.split;
    int grid = p.grid;
    const bool counting = ((zero_count || sat_count) && y) || y_flags;
    const WorkspaceLayout wl = workspace_layout(p);
    if (workspace) {
        if (workspace_bytes < wl.total || !aligned16(workspace)) return LP_EWORKSPACE;
        if (counting) a.zero_partial = (unsigned *)workspace;
        a.partial_stride = grid;
        a.partials = (unsigned char *)workspace + wl.partials;
        a.part_bytes = (int)p.part_bytes;
    } else {
        if (counting) return LP_EWORKSPACE;
        // nowhere to merge partial sums: every tile is computed by one workgroup
        a.full_per_xcd = p.per_xcd;
        a.split = 1;
        grid = kXCDs * p.per_xcd;
    }
    // The 32-bit epilogue is exact when only codes are wanted, with ReLU, round-half-away,
    // a right shift of 1..31 bits, and sums small enough that no int32 piece can overflow
    // (K <= 8192 keeps |HH|, |HL+LH| and the folded constants below 2^29).
    a.fast = (y && !acc_out && fast_epilogue_ok(d, p, f_acc, bias != nullptr, qb, qy, relu, r)) ? 1 : 0;
    a.pool = p.pool;
    if (p.pool && !(a.fast && a.y16 && d->Cout % 4 == 0)) return LP_EUNSUPPORTED;
    lp_status st2;
    const int tails = a.split > 1 ? kXCDs * (p.per_xcd - p.full_per_xcd) : 0; // finishing workgroups
    // A small grid adds its counts to the counters itself: two atomics per workgroup cost less than
    // the launch of the kernel that sums the per-workgroup slots.
    const bool direct = counting && !tails && grid <= kDirectCountGrid;
    if (direct) {
        a.zero_partial = nullptr;
        a.direct_counts = ((zero_count || sat_count) && y) ? 1 : 0;
    }
    if (p.rows) {
        if (p.tiles_n == 1 && d->Cout <= 32) hipLaunchKernelGGL(conv_rows_kernel<1>, dim3(grid), dim3(256), p.lds_bytes, hs, a);
        else hipLaunchKernelGGL(conv_rows_kernel<2>, dim3(grid), dim3(256), p.lds_bytes, hs, a);
        st2 = launch_status();
    }
    else if (p.flat) {
        // one slab: nothing to split; channel tiles of at most 32 channels need one column block
        const bool narrow = p.tiles_n == 1 && d->Cout <= 32;
        if (p.ksteps == 1) {
            if (narrow) hipLaunchKernelGGL((conv_flat_kernel<1, 1>), dim3(grid), dim3(256), 0, hs, a);
            else hipLaunchKernelGGL((conv_flat_kernel<2, 1>), dim3(grid), dim3(256), 0, hs, a);
        } else {
            if (narrow) hipLaunchKernelGGL((conv_flat_kernel<1, 2>), dim3(grid), dim3(256), 0, hs, a);
            else hipLaunchKernelGGL((conv_flat_kernel<2, 2>), dim3(grid), dim3(256), 0, hs, a);
        }
        st2 = launch_status();
    }
    else if (p.limbs == 2) st2 = launch_mfma<2, 1, 2>(a, p, grid, tails, hs);
    else st2 = p.BN == 128 ? launch_mfma<1, 2, 2>(a, p, grid, tails, hs) : launch_mfma<1, 1, 2>(a, p, grid, tails, hs);
    if (st2 != LP_OK || tails || !counting || direct) return st2;
    return launch_sum_partials(a.zero_partial, grid, (unsigned long long *)zero_count, (unsigned long long *)sat_count, hs);
}

static lp_status pack_weights(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, const void *w,
                              void *packed, size_t packed_bytes, void *stream)
{
    Plan p;
    lp_status st = make_plan(d, qx, qw, &p);
    if (st != LP_OK) return st;
    if (!w || !packed || !aligned16(w) || !aligned16(packed)) return LP_EINVAL;
    if (packed_bytes < p.packed_bytes) return LP_EWORKSPACE;
    hipStream_t hs = as_stream(stream);
    clear_stale_error();
    const bool w16 = qw.n > 8;
    const int RS = d->R * d->S;
    if (p.path == PATH_DIRECT) {
        const size_t total = (size_t)d->Cout * RS * d->Cin;
        const int grid = (int)std::min<size_t>((total + 255) / 256, 65535);
        if (w16) hipLaunchKernelGGL(widen_weights_kernel<int16_t>, dim3(grid), dim3(256), 0, hs,
                                    (const int16_t *)w, (int16_t *)packed, total);
        else hipLaunchKernelGGL(widen_weights_kernel<int8_t>, dim3(grid), dim3(256), 0, hs,
                                (const int8_t *)w, (int16_t *)packed, total);
        return launch_status();
    }
    const size_t total = (size_t)RS * p.nchunks * p.CoutP * CK;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 65535);
    unsigned char *out = (unsigned char *)packed;
    int64_t *corr = (int64_t *)(out + p.corr_offset);
    const int cgrid = p.CoutP; // one wave per output channel
    if (p.rows) {
        const int K = RS * d->Cin, rgrid = (p.KHP * p.CoutP * 32 + 255) / 256;
        if (w16) {
            hipLaunchKernelGGL(pack_weights_rows_kernel<int16_t>, dim3(rgrid), dim3(256), 0, hs, (const int16_t *)w, out,
                               d->Cout, d->R, d->S * d->Cin, p.KHR, p.KHP, p.CoutP);
            hipLaunchKernelGGL(weight_corr_kernel<int16_t>, dim3(cgrid), dim3(64), 0, hs,
                               (const int16_t *)w, corr, d->Cout, p.CoutP, K, 2);
        } else {
            hipLaunchKernelGGL(pack_weights_rows_kernel<int8_t>, dim3(rgrid), dim3(256), 0, hs, (const int8_t *)w, out,
                               d->Cout, d->R, d->S * d->Cin, p.KHR, p.KHP, p.CoutP);
            hipLaunchKernelGGL(weight_corr_kernel<int8_t>, dim3(cgrid), dim3(64), 0, hs,
                               (const int8_t *)w, corr, d->Cout, p.CoutP, K, 2);
        }
        return launch_status();
    }
    if (p.flat) {
        const int K = RS * d->Cin, fgrid = (p.CoutP * CK + 255) / 256;
        if (w16) {
            hipLaunchKernelGGL(pack_weights_flat_kernel<int16_t>, dim3(fgrid), dim3(256), 0, hs,
                               (const int16_t *)w, out, d->Cout, K, p.CoutP);
            hipLaunchKernelGGL(weight_corr_kernel<int16_t>, dim3(cgrid), dim3(64), 0, hs,
                               (const int16_t *)w, corr, d->Cout, p.CoutP, K, 2);
        } else {
            hipLaunchKernelGGL(pack_weights_flat_kernel<int8_t>, dim3(fgrid), dim3(256), 0, hs,
                               (const int8_t *)w, out, d->Cout, K, p.CoutP);
            hipLaunchKernelGGL(weight_corr_kernel<int8_t>, dim3(cgrid), dim3(64), 0, hs,
                               (const int8_t *)w, corr, d->Cout, p.CoutP, K, 2);
        }
        return launch_status();
    }
#define LP_PACK(WT, L)                                                                              \
    hipLaunchKernelGGL((pack_weights_kernel<WT, L>), dim3(grid), dim3(256), 0, hs, (const WT *)w, out, \
                       d->Cout, d->Cin, RS, p.nchunks, p.CoutP, total);                                \
    hipLaunchKernelGGL(weight_corr_kernel<WT>, dim3(cgrid), dim3(64), 0, hs, (const WT *)w, corr,      \
                       d->Cout, p.CoutP, RS * d->Cin, L);                                              \
    if (L == 2)                                                                                        \
    hipLaunchKernelGGL(chunk_weight_sums_kernel<WT>, dim3(p.CoutP, p.nchunks), dim3(64), 0, hs,        \
                       (const WT *)w, (int *)(out + p.wsum_offset), d->Cout, p.CoutP, d->Cin, RS)
    if (p.limbs == 2) {
        if (w16) { LP_PACK(int16_t, 2); } else { LP_PACK(int8_t, 2); }
    } else {
        LP_PACK(int8_t, 1);
    }
#undef LP_PACK
    return launch_status();
}

// Workspace of lp_conv_fwd_static: one array per GPU, part of the loaded code object, for callers
// that cannot allocate.  The name below is only a host-side handle; the array's device address
// on the current GPU comes from hipGetSymbolAddress and is looked up once per device.
static __device__ __align__(256) unsigned char scratch[LP_STATIC_WORKSPACE_BYTES];

static lp_status static_scratch(void **out)
{
    static std::mutex mutex;
    static void *ptr_of_device[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LP_EDEVICE;
    std::lock_guard<std::mutex> lock(mutex);
    if (!ptr_of_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LP_EDEVICE;
        ptr_of_device[dev] = p;
    }
    *out = ptr_of_device[dev];
    return LP_OK;
}

static lp_conv_desc fc_desc(int M, int K, int Nout)
{
    lp_conv_desc d = {M, 1, 1, K, Nout, 1, 1, 1, 0};
    return d;
}

} // namespace lp

using namespace lp;

extern "C" lp_status lp_conv_packed_bytes(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw,
                                          size_t *bytes_host)
{
    if (!bytes_host) return LP_EINVAL;
    Plan p;
    lp_status st = make_plan(d, qx, qw, &p);
    if (st == LP_OK) *bytes_host = p.packed_bytes;
    return st;
}

extern "C" lp_status lp_conv_pack_weights(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw,
                                          const void *w_codes_dev, void *packed_dev,
                                          size_t packed_bytes, void *stream)
{
    return pack_weights(d, qx, qw, w_codes_dev, packed_dev, packed_bytes, stream);
}

extern "C" lp_status lp_conv_plan_info(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw,
                                       lp_plan_info *out_host)
{
    if (!out_host) return LP_EINVAL;
    Plan p;
    lp_status st = make_plan(d, qx, qw, &p);
    if (st != LP_OK) return st;
    lp_plan_info o = {};
    o.path = p.path;
    o.limbs = p.limbs;
    if (p.path == PATH_MFMA) {
        o.bn = p.BN; o.tile_rows = p.RH; o.tile_cols = p.TW; o.patch_rows = p.PRA; o.patch_cols = p.PW;
        o.tiles_m = p.tiles_m; o.tiles_n = p.tiles_n; o.lds_bytes = (int32_t)p.lds_bytes;
        o.patch_pitch = p.PITCH;
        o.patch_pixel = p.flat ? d->Cin * 2 : p.rows ? d->Cin : PSP;
        o.kernel = p.rows ? LP_KERNEL_ROWS : p.flat ? LP_KERNEL_FLAT : LP_KERNEL_PATCH;
        o.workgroups = p.grid;
        o.split = p.split;
        o.items_per_die = p.per_xcd;
        o.whole_items_per_die = p.full_per_xcd;
    }
    *out_host = o;
    return LP_OK;
}

extern "C" lp_status lp_conv_pool_check(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, int has_bias, lp_qfmt qb, lp_qfmt qy,
                                        int relu, lp_round r)
{
    if (!d || !d->pool) return LP_EINVAL;
    Plan p;
    const lp_status st = make_plan(d, qx, qw, &p);
    if (st != LP_OK) return st;
    if (!fmt_ok(qy) || (has_bias && !fmt_ok(qb))) return LP_EINVAL;
    const bool ok = fast_epilogue_ok(d, p, qx.f + qw.f, has_bias != 0, qb, qy, relu, r) && qy.n > 8 && d->Cout % 4 == 0;
    return ok ? LP_OK : LP_EUNSUPPORTED;
}

extern "C" lp_status lp_conv_workspace_bytes(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw,
                                             size_t *bytes_host)
{
    if (!bytes_host) return LP_EINVAL;
    Plan p;
    lp_status st = make_plan(d, qx, qw, &p);
    if (st == LP_OK) *bytes_host = workspace_layout(p).total;
    return st;
}

extern "C" lp_status lp_conv_fwd(const lp_conv_desc *d, const void *x_codes_dev, lp_qfmt qx,
                                 const void *w_packed_dev, lp_qfmt qw, const void *bias_codes_dev,
                                 lp_qfmt qb, int64_t *acc_out_dev, void *y_codes_dev, lp_qfmt qy,
                                 int relu, lp_round r, uint64_t *zero_count_dev, uint64_t *sat_count_dev,
                                 void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return conv_forward(d, x_codes_dev, qx, w_packed_dev, qw, bias_codes_dev, qb, acc_out_dev,
                        y_codes_dev, qy, relu, r, zero_count_dev, sat_count_dev, workspace_dev, workspace_bytes, stream);
}

extern "C" lp_status lp_conv_fwd_zskip(const lp_conv_desc *d, const void *x_codes_dev, lp_qfmt qx,
                                       const lp_zero_map *x_zero_map_host, const void *w_packed_dev, lp_qfmt qw,
                                       const void *bias_codes_dev, lp_qfmt qb, void *y_codes_dev, lp_qfmt qy, int relu,
                                       lp_round r, uint64_t *zero_count_dev, uint64_t *sat_count_dev,
                                       uint8_t *y_tile_flags_dev, uint64_t *skipped_dev, void *workspace_dev,
                                       size_t workspace_bytes, void *stream)
{
    return conv_forward(d, x_codes_dev, qx, w_packed_dev, qw, bias_codes_dev, qb, nullptr, y_codes_dev, qy, relu, r,
                        zero_count_dev, sat_count_dev, workspace_dev, workspace_bytes, stream, x_zero_map_host,
                        y_tile_flags_dev, skipped_dev);
}

extern "C" lp_status lp_conv_fwd_static(const lp_conv_desc *d, const void *x_codes_dev, lp_qfmt qx,
                                        const void *w_packed_dev, lp_qfmt qw, const void *bias_codes_dev,
                                        lp_qfmt qb, int64_t *acc_out_dev, void *y_codes_dev, lp_qfmt qy,
                                        int relu, lp_round r, uint64_t *zero_count_dev,
                                        uint64_t *sat_count_dev, void *stream)
{
    Plan p;
    const lp_status st = make_plan(d, qx, qw, &p);
    if (st != LP_OK) return st;
    if (workspace_layout(p).total > (size_t)LP_STATIC_WORKSPACE_BYTES) return LP_EWORKSPACE;
    void *ws = nullptr;
    const lp_status sp = static_scratch(&ws);
    if (sp != LP_OK) return sp;
    return conv_forward(d, x_codes_dev, qx, w_packed_dev, qw, bias_codes_dev, qb, acc_out_dev,
                        y_codes_dev, qy, relu, r, zero_count_dev, sat_count_dev, ws,
                        (size_t)LP_STATIC_WORKSPACE_BYTES, stream);
}

lp_status lp::fc_conv_packed_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw,
                                        size_t *bytes_host)
{
    const lp_conv_desc d = fc_desc(M, K, Nout);
    return lp_conv_packed_bytes(&d, qx, qw, bytes_host);
}

lp_status lp::fc_conv_pack_weights(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw,
                                        const void *w_codes_dev, void *packed_dev, size_t packed_bytes,
                                        void *stream)
{
    const lp_conv_desc d = fc_desc(M, K, Nout);
    return pack_weights(&d, qx, qw, w_codes_dev, packed_dev, packed_bytes, stream);
}

lp_status lp::fc_conv_workspace_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw,
                                           size_t *bytes_host)
{
    const lp_conv_desc d = fc_desc(M, K, Nout);
    return lp_conv_workspace_bytes(&d, qx, qw, bytes_host);
}

lp_status lp::fc_conv_fwd(int M, int K, int Nout, const void *x_codes_dev, lp_qfmt qx,
                               const void *w_packed_dev, lp_qfmt qw, const void *bias_codes_dev,
                               lp_qfmt qb, int64_t *acc_out_dev, void *y_codes_dev, lp_qfmt qy,
                               int relu, lp_round r, uint64_t *zero_count_dev, uint64_t *sat_count_dev,
                               void *workspace_dev, size_t workspace_bytes, void *stream)
{
    const lp_conv_desc d = fc_desc(M, K, Nout);
    return conv_forward(&d, x_codes_dev, qx, w_packed_dev, qw, bias_codes_dev, qb, acc_out_dev,
                        y_codes_dev, qy, relu, r, zero_count_dev, sat_count_dev, workspace_dev, workspace_bytes, stream);
}
