// LPInnerProduct forward on Qm.f codes for gfx950 (Sec. 2 of the paper), exact, with the fused
// LPAct (+ReLU) tail of Sec. 2.1: a split-K GEMM on the int8 MFMA.
//
//     acc[b][o] = sum_k X[b][k] * W[o][k] (+ bias)
//
// The limb algebra is that of the convolution kernels: a 16-bit code is a = 256*ah + al + 128 with
// two int8 limbs, and sum a*b = 2^16*HH + 2^8*(HL+LH) + LL + 128*sum(a) + 128*sum(b) - 16384*K.
//
// Shape of the work.  An inner product streams a large weight matrix (205 MB for 25088 -> 4096)
// against few input rows, so every weight byte should leave HBM once, and the matrix pipe must
// not wait for the instructions that feed it:
//   - a workgroup (8 waves, two per SIMD) owns FM = 256 input rows x FN = 64 output columns over
//     one part of the reduction; a wave owns 32 rows x 64 columns (two MFMA blocks, three
//     accumulator sets: 96 registers).  A wave's own loads, LDS reads and address arithmetic do not
//     overlap with its own MFMAs (measured: a lone wave per SIMD loses 7 to 36 cycles per such
//     instruction), so a second wave per SIMD is what hides them;
//   - weights are packed per 64-column tile in the order of use, so a workgroup's weights are one
//     linear stream: each wave fetches an eighth of a stage (4 K = 32 halves, 16 KB) into registers
//     three stages ahead (48 KB per CU in flight, enough to cover HBM latency at full rate), parks
//     it in one of three LDS stage buffers, and all eight waves read their fragments from there
//     (one barrier per stage);
//   - input rows are split once per call into limb planes in fragment order (fc_split_x_kernel,
//     which also sums each row's codes for the offset correction), so a wave loads its own rows'
//     fragments straight from L2 into MFMA operand registers, 1 KB of consecutive memory per
//     request, one stage ahead; workgroups that share a K range sit on the same die and walk it
//     in step, so those reads hit that die's L2;
//   - the reduction is cut into ksplit parts so that the grid fills the chip; a part stores its
//     sums combined to one int64 per output, and fc_finish_kernel adds the parts (integer sums:
//     order cannot matter) and runs the same tile epilogue as the convolution.
#include <algorithm>

#include "lp_tile.h"

namespace lp {

constexpr int FM = 256;        // input rows per workgroup tile (8 waves x 32)
constexpr int FN = 64;         // output columns per workgroup tile
constexpr int FSK = 4;         // K = 32 halves per stage
constexpr int FRAG = 1024;     // bytes of one MFMA operand fragment: 64 lanes x 16
constexpr int kFcThreads = 512;
constexpr int FMAXP = 8;       // most parts the reduction is cut into
constexpr int FKC = 32;        // most K chunks the input split works in (one partial row sum each)

struct FcPlan {
    int limbs;
    int KH;                    // K = 32 halves of the whole reduction
    int mblocks;               // 32-row blocks of the input
    int n_tiles, m_tiles, tiles, ksplit, khp; // khp: K halves per part (a multiple of FSK)
    int kc, khc;               // input split: K chunks and K halves per chunk (a multiple of 16)
    int per_xcd, grid;
    size_t wslab;              // packed weight bytes of one 64-column tile
    size_t corr_offset, packed_bytes;
    size_t part_bytes;
    size_t ws_counts, ws_xs, ws_xsum, ws_parts, ws_total; // workspace: [counts][split input][row sums][partial sums]
};

// The inner-product kernel takes 16-bit inputs with 8- or 16-bit weights (two limbs) and 8-bit
// inputs with 8-bit weights (one limb).
static bool fc_kernel_takes(lp_qfmt qx, lp_qfmt qw) { return qx.n > 8 || qw.n <= 8; }

static lp_status make_fc_plan(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, FcPlan *out)
{
    if (M <= 0 || K <= 0 || Nout <= 0 || !fmt_ok(qx) || !fmt_ok(qw)) return LP_EINVAL;
    FcPlan p = {};
    p.limbs = qx.n > 8 ? 2 : 1;
    if ((long long)M * K >= (1LL << 30) || (long long)M * Nout >= (1LL << 31) || (long long)Nout * K >= (1LL << 31))
        return LP_EUNSUPPORTED;
    if (K >= 65536 && p.limbs == 2) return LP_EUNSUPPORTED; // int32 limb sums could overflow
    if (K >= 131072) return LP_EUNSUPPORTED;
    p.KH = (K + 31) / 32;
    p.mblocks = (M + 31) / 32;
    p.n_tiles = (Nout + FN - 1) / FN;
    p.m_tiles = (M + FM - 1) / FM;
    p.tiles = p.n_tiles * p.m_tiles;
    // parts: fill the chip's CUs (one workgroup each), at least two stages per part
    const int stages = (p.KH + FSK - 1) / FSK;
    int ks = std::max(1, kCUs / p.tiles);
    ks = std::min(ks, std::min(FMAXP, std::max(1, stages / 2)));
    p.khp = ((stages + ks - 1) / ks) * FSK;
    p.ksplit = (p.KH + p.khp - 1) / p.khp;
    const int total = p.tiles * p.ksplit;
    p.per_xcd = (total + kXCDs - 1) / kXCDs;
    p.grid = kXCDs * p.per_xcd;
    // input split: about one block (sixteen waves, a K half each per trip) per CU
    const int want = std::max(1, std::min(FKC, kCUs / p.mblocks));
    p.khc = ((((p.KH + 15) / 16) + want - 1) / want) * 16;
    p.kc = (p.KH + p.khc - 1) / p.khc;
    p.wslab = (size_t)p.KH * p.limbs * 2 * FRAG;
    p.corr_offset = round_up((size_t)p.n_tiles * p.wslab, 256);
    p.packed_bytes = p.corr_offset + (size_t)p.n_tiles * FN * sizeof(int64_t);
    if (p.corr_offset >= (1ull << 32)) return LP_EUNSUPPORTED;
    p.part_bytes = (size_t)FM * FN * (p.limbs == 2 ? 8 : 4);
    p.ws_counts = round_up((size_t)2 * p.grid * sizeof(unsigned), 256);
    p.ws_xs = round_up((size_t)p.mblocks * p.KH * p.limbs * FRAG, 256);
    p.ws_xsum = round_up((size_t)p.kc * p.mblocks * 32 * sizeof(int), 256);
    p.ws_parts = p.ksplit > 1 ? (size_t)p.tiles * p.ksplit * p.part_bytes : 0;
    p.ws_total = p.ws_counts + p.ws_xs + p.ws_xsum + p.ws_parts;
    *out = p;
    return LP_OK;
}

// ------------------------------------------------------------------------- packing

// Packed weights: [64-column tile][K half][limb hi, lo][32-column block][lane 0..63][16 bytes]; lane
// l of a fragment holds the 16 reduction positions (l / 32) * 16 .. + 15 of the K half for column
// (l % 32) of the block: what the MFMA's row operand wants, 1 KB per fragment, and a tile's
// fragments consecutive in the order the kernel consumes them.
template <typename WT, int LIMBS>
__global__ __launch_bounds__(256) void fc_pack_weights_kernel(const WT *__restrict__ w, unsigned char *__restrict__ out,
                                                             int Nout, int K, int KH, size_t pieces)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (size_t)gridDim.x * 256) {
        const int lane = (int)(i & 63);
        size_t t = i >> 6;
        const int cb = (int)(t & 1);
        t >>= 1;
        const int kh = (int)(t % KH);
        const int nt = (int)(t / KH);
        const int col = nt * FN + cb * 32 + (lane & 31);
        const int k0 = kh * 32 + (lane >> 5) * 16;
        alignas(16) unsigned char hi[16], lo[16];
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            int code = 0;
            if (col < Nout && k0 + b < K) code = (int)w[(size_t)col * K + k0 + b];
            if constexpr (LIMBS == 2) {
                hi[b] = (unsigned char)(code >> 8);
                lo[b] = (col < Nout && k0 + b < K) ? (unsigned char)((code & 255) - 128) : 0;
            } else {
                hi[b] = (unsigned char)code;
            }
        }
        unsigned char *dst = out + (((size_t)nt * KH + kh) * LIMBS * 2 + cb) * FRAG + lane * 16;
        *(v4i *)dst = *(const v4i *)hi;
        if constexpr (LIMBS == 2) *(v4i *)(dst + 2 * FRAG) = *(const v4i *)lo;
    }
}

// Input rows into limb planes in fragment order: [32-row block][K half][limb][lane][16 bytes], lane l
// holding positions (l / 32) * 16 .. + 15 of the K half for row (l % 32) of the block.  Rows past M
// and positions past K are (0, 0) limbs: they meet zero weights.  blockIdx.x = 32-row block,
// blockIdx.y = K chunk of khc K halves; a block's sixteen waves take sixteen K halves per trip.  Every
// thread also adds up the codes it moves (its row never changes), and the block writes its 32
// partial row sums to xsum[K chunk][row]: the epilogue's offset correction needs the sum of each
// row's codes (two-limb path).
constexpr int kSplitWaves = 16;
template <typename XT, int LIMBS>
__global__ __launch_bounds__(64 * kSplitWaves) void fc_split_x_kernel(const XT *__restrict__ x, unsigned char *__restrict__ xs,
                                                        int *__restrict__ xsum, int M, int K, int KH, int khc)
{
    __shared__ int part[2 * kSplitWaves][32];
    const bool vec = (K % 16) == 0; // rows start on 16-byte boundaries and no piece straddles the end
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int mb = blockIdx.x, row = mb * 32 + (lane & 31);
    const int khe = min(KH, ((int)blockIdx.y + 1) * khc);
    int sum = 0;
    for (int kh = blockIdx.y * khc + wave; kh < khe; kh += kSplitWaves) {
        const int k0 = kh * 32 + (lane >> 5) * 16;
        unsigned char *dst = xs + ((size_t)(mb * KH + kh) * LIMBS) * FRAG + lane * 16;
        if constexpr (LIMBS == 2) {
            unsigned pr[8] = {0, 0, 0, 0, 0, 0, 0, 0}; // two codes per word
            if (row < M && k0 < K) {
                const XT *src = x + (size_t)row * K + k0;
                if (vec) {
                    const v4i a = *(const v4i *)src, b = *(const v4i *)(src + 8);
                    pr[0] = a.x; pr[1] = a.y; pr[2] = a.z; pr[3] = a.w;
                    pr[4] = b.x; pr[5] = b.y; pr[6] = b.z; pr[7] = b.w;
                } else {
#pragma unroll
                    for (int b = 0; b < 16; ++b)
                        if (k0 + b < K) pr[b >> 1] |= ((unsigned)(unsigned short)src[b]) << (16 * (b & 1));
                }
            }
            unsigned h[4], l[4];
            const v2s ones = {1, 1};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                h[q] = __builtin_amdgcn_perm(pr[2 * q + 1], pr[2 * q], 0x07050301u);
                l[q] = __builtin_amdgcn_perm(pr[2 * q + 1], pr[2 * q], 0x06040200u) ^ 0x80808080u;
                sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pr[2 * q]), ones, sum, false);
                sum = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, pr[2 * q + 1]), ones, sum, false);
            }
            if (!(row < M && k0 + 16 <= K)) {
                // positions that do not exist are the limbs (0, 0), not the code 0
#pragma unroll
                for (int b = 0; b < 16; ++b)
                    if (!(row < M && k0 + b < K)) l[b >> 2] &= ~(0xffu << (8 * (b & 3)));
            }
            *(v4i *)dst = (v4i){(int)h[0], (int)h[1], (int)h[2], (int)h[3]};
            *(v4i *)(dst + FRAG) = (v4i){(int)l[0], (int)l[1], (int)l[2], (int)l[3]};
        } else {
            v4i v = {0, 0, 0, 0};
            if (row < M && k0 < K) {
                const XT *src = x + (size_t)row * K + k0;
                if (vec) {
                    v = *(const v4i *)src;
                } else {
                    unsigned wds[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int b = 0; b < 16; ++b)
                        if (k0 + b < K) wds[b >> 2] |= ((unsigned)(unsigned char)src[b]) << (8 * (b & 3));
                    v = (v4i){(int)wds[0], (int)wds[1], (int)wds[2], (int)wds[3]};
                }
            }
            *(v4i *)dst = v;
        }
    }
    if constexpr (LIMBS == 2) {
        part[wave * 2 + (lane >> 5)][lane & 31] = sum;
        __syncthreads();
        if (threadIdx.x < 32) {
            int t = 0;
#pragma unroll
            for (int i = 0; i < 2 * kSplitWaves; ++i) t += part[i][threadIdx.x];
            xsum[((size_t)blockIdx.y * gridDim.x + mb) * 32 + threadIdx.x] = t;
        }
    }
}

// ------------------------------------------------------------------------ main kernel

struct FcArgs {
    ConvArgs c;                // what the shared tile epilogue reads (N = M rows of 1 x 1 pixels)
    const unsigned char *xs;   // split input, see fc_split_x_kernel
    const int *xsum;           // [kc][mblocks * 32] partial sums of each row's codes
    unsigned xs_bytes;
    int M, K, KH, khp, ksplit, n_tiles, tiles, per_xcd, total, kc, mrows;
    unsigned wslab;
};

// the epilogue's LDS tables of a tile: tile row -> output row, the rows' code sums, channel constants
template <int LIMBS>
__device__ __forceinline__ void fc_tile_tables(const FcArgs &f, int mt, int nt, int *outoff, int *rowsum, int *ctab)
{
    for (int m = threadIdx.x; m < FM; m += kFcThreads) {
        const int row = mt * FM + m;
        outoff[m] = row < f.M ? row : -1;
        // the row's partial sums, all requested before any is added (kc is uniform)
        int t = 0;
        if (LIMBS == 2 && row < f.mrows) {
            int v[FKC];
#pragma unroll
            for (int i = 0; i < FKC; ++i) v[i] = i < f.kc ? f.xsum[(size_t)i * f.mrows + row] : 0;
#pragma unroll
            for (int i = 0; i < FKC; ++i) t += v[i];
        }
        rowsum[m] = t;
    }
    build_colterms<FN, kFcThreads>(f.c, nt, ctab, LIMBS);
}

// Sums in the 32-bit pieces the epilogue combines <-> one exact int64 per output.
__device__ __forceinline__ long long fc_combine(int hh, int mid, int ll) { return ((long long)hh << 16) + ((long long)mid << 8) + ll; }

template <int LIMBS>
__global__ __launch_bounds__(kFcThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fc_mfma_kernel(const FcArgs f)
{
    constexpr int NACC = (LIMBS == 2) ? 3 : 1;
    constexpr int WAVES = kFcThreads / 64;
    constexpr int KHB = LIMBS * 2 * FRAG;     // weight bytes of one K half of a tile
    constexpr int STAGE = FSK * KHB;          // 16 KB (8 KB with one limb)
    constexpr int NBL = STAGE / WAVES / FRAG; // 16-byte requests per thread and stage
    constexpr int NBR = 3;                    // stages in flight in registers, and LDS stage buffers
    static_assert(NBL >= 1, "a stage must give every wave a whole fragment to fetch");
    __shared__ __align__(16) unsigned char Bs[NBR][STAGE];
    __shared__ int outoff[FM];
    __shared__ int rowsum[FM];
    __shared__ __align__(16) int ctab[3 * FN];
    __shared__ unsigned wave_counts[2][WAVES];

    // Work order: consecutive workgroup ids go round-robin to the dies, so each die is handed one
    // contiguous range of work items, ordered part-major: the workgroups of a die share a K range
    // (and with it the input fragments they read) and differ in their column tile.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int wi = xcd * f.per_xcd + slot;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (slot >= f.per_xcd || wi >= f.total) {
        if (f.c.zero_partial && tid == 0) f.c.zero_partial[blockIdx.x] = f.c.zero_partial[f.c.partial_stride + blockIdx.x] = 0;
        return;
    }
    const int part = wi / f.tiles, tile = wi - part * f.tiles;
    const int mt = tile / f.n_tiles, nt = tile - mt * f.n_tiles;
    const int kh0 = part * f.khp, kh1 = min(f.KH, kh0 + f.khp);
    const int nst = (kh1 - kh0 + FSK - 1) / FSK;

    // Weights: one descriptor over this tile's fragments up to the end of the part (requests past
    // it read as zeros: the last stage may be partly empty), a wave's share of a stage as a
    // per-lane offset to which the stage's offset is added (in the per-lane offset, not as the
    // instruction's scalar offset: the range check must see it).
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(f.c.wp) + (size_t)nt * f.wslab, 0, kh1 * KHB, 0x00020000);
    const int boff = wave * (STAGE / WAVES) + lane * 16;
    v4i breg[NBR][NBL];
    auto bload = [&](int st, v4i *r) __attribute__((always_inline)) {
        const int at = boff + (kh0 + st * FSK) * KHB;
#pragma unroll
        for (int i = 0; i < NBL; ++i) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, at + i * FRAG, 0, 0);
            r[i] = (v4i){(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
        }
    };
    auto bpark = [&](int buf, const v4i *r) __attribute__((always_inline)) {
        unsigned char *dst = Bs[buf] + boff;
#pragma unroll
        for (int i = 0; i < NBL; ++i) *(v4i *)(dst + i * FRAG) = r[i];
    };
    // Inputs: the wave's 32-row block; fragment (K half, limb) is 1 KB at ((block * KH + kh) *
    // LIMBS + limb) * 1 KB.  A block past the input reads as zeros.
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(f.xs), 0, (int)f.xs_bytes, 0x00020000);
    const long long ao = ((long long)(mt * (FM / 32) + wave) * f.KH) * (LIMBS * FRAG) + lane * 16;
    const int aoff = ao < (long long)f.xs_bytes ? (int)ao : 0x7fffffff;
    v4i areg[FSK][LIMBS];
    auto aload = [&](int kh, v4i (&r)[LIMBS]) __attribute__((always_inline)) {
        const int at = aoff + kh * (LIMBS * FRAG);
#pragma unroll
        for (int l = 0; l < LIMBS; ++l) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, at + l * FRAG, 0, 0);
            r[l] = (v4i){(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
        }
    };

    // prologue: three stages of weights and the first stage of inputs on their way
#pragma unroll
    for (int s = 0; s < NBR; ++s) bload(s, breg[s]);
#pragma unroll
    for (int j = 0; j < FSK; ++j) aload(kh0 + j, areg[j]);

    v16i acc[1][2][NACC];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int q = 0; q < NACC; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[0][cb][q][v] = 0;

    // Three LDS stage buffers: while stage st is multiplied from buffer st % 3, stage st + 1 is
    // complete in the next one (its first fragments are read before stage st ends) and stage
    // st + 2 is being parked in the third, which was last read during stage st - 1.
    bpark(0, breg[0]);
    bpark(1, breg[1]);
    bload(NBR, breg[0]);
    bload(NBR + 1, breg[1]);
    __syncthreads();
    // weight fragments of the K half being multiplied and of the one after it
    v4i wf[2][2][LIMBS];
    auto wfetch = [&](int buf, int j, v4i (&w)[2][LIMBS]) __attribute__((always_inline)) {
        const unsigned char *bs = Bs[buf] + lane * 16 + j * KHB;
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) w[cb][l] = *(const v4i *)(bs + (l * 2 + cb) * FRAG);
    };
    wfetch(0, 0, wf[0]);

    // One stage: after the barrier (every wave has finished stage st - 1 and has parked stage
    // st + 1), park stage st + 2 and refill its registers with stage st + 5; then multiply this
    // stage's FSK K halves.  Each half first requests the next half's weight fragments (of this
    // stage or the next), and requests its own input fragments again for the next stage as soon
    // as they have been used.
    using std::integral_constant;
    auto stage = [&](int st, auto RC) __attribute__((always_inline)) {
        constexpr int R = decltype(RC)::value; // st % NBR
        __syncthreads();
        bpark((R + 2) % NBR, breg[(R + 2) % NBR]);
        bload(st + 2 + NBR, breg[(R + 2) % NBR]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < FSK; ++j) {
            if (j + 1 < FSK) wfetch(R, j + 1, wf[(j + 1) & 1]);
            else wfetch((R + 1) % NBR, 0, wf[0]);
            __builtin_amdgcn_sched_barrier(0);
            v4i (&w)[2][LIMBS] = wf[j & 1];
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                acc[0][cb][0] = mfma_i8(w[cb][0], areg[j][0], acc[0][cb][0]);
                if constexpr (LIMBS == 2) {
                    acc[0][cb][1] = mfma_i8(w[cb][1], areg[j][0], acc[0][cb][1]);
                    acc[0][cb][2] = mfma_i8(w[cb][1], areg[j][1], acc[0][cb][2]);
                    acc[0][cb][1] = mfma_i8(w[cb][0], areg[j][1], acc[0][cb][1]);
                }
            }
            aload(kh0 + (st + 1) * FSK + j, areg[j]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int st = 0;
    for (; st + NBR <= nst; st += NBR) {
        stage(st, integral_constant<int, 0>{});
        stage(st + 1, integral_constant<int, 1>{});
        stage(st + 2, integral_constant<int, 2>{});
    }
    if (st < nst) {
        stage(st, integral_constant<int, 0>{});
        if (st + 1 < nst) stage(st + 1, integral_constant<int, 1>{});
    }

    if (f.ksplit > 1) {
        // A part stores its sums, one exact int64 per output (int32 with one limb), in register
        // order: piece (column block, group of four channels, half) of thread tid.
        v4i *mine = (v4i *)(f.c.partials + ((size_t)tile * f.ksplit + part) * f.c.part_bytes);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if constexpr (LIMBS == 2) {
                    long long v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        v[e] = fc_combine(acc[0][cb][0][4 * g + e], acc[0][cb][1][4 * g + e], acc[0][cb][2][4 * g + e]);
                    mine[((cb * 4 + g) * 2) * kFcThreads + tid] =
                        (v4i){(int)v[0], (int)(v[0] >> 32), (int)v[1], (int)(v[1] >> 32)};
                    mine[((cb * 4 + g) * 2 + 1) * kFcThreads + tid] =
                        (v4i){(int)v[2], (int)(v[2] >> 32), (int)v[3], (int)(v[3] >> 32)};
                } else {
                    const v16i &c = acc[0][cb][0];
                    mine[(cb * 4 + g) * kFcThreads + tid] = (v4i){c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
                }
            }
        if (f.c.zero_partial && tid == 0) f.c.zero_partial[blockIdx.x] = f.c.zero_partial[f.c.partial_stride + blockIdx.x] = 0;
        return;
    }

    fc_tile_tables<LIMBS>(f, mt, nt, outoff, rowsum, ctab);
    __syncthreads();
    const TileCounts counts = tile_epilogue<LIMBS, 2, FN, 1, 4>(
        f.c, acc, [&](int m) { return rowsum[m]; }, outoff, outoff, ctab, nt, wave * 32, 0, 0, 0);
    if (f.c.zero_partial || f.c.direct_counts) {
        if (lane == 0) {
            wave_counts[0][wave] = counts.zeros;
            wave_counts[1][wave] = counts.sats;
        }
        __syncthreads();
        if (tid < 2) {
            unsigned total = 0;
            for (int w = 0; w < WAVES; ++w) total += wave_counts[tid][w];
            publish_count(f.c, tid, total);
        }
    }
}

// Adds up the parts of a tile and runs the epilogue: eight workgroups per tile, one per (column
// block, group of four channels) of the MFMA layout, threads mapped to rows as in the main
// kernel, so that a thread needs two 16-byte pieces (one with one limb) per part.  Counts go
// straight to the caller's counters.
template <int LIMBS>
__global__ __launch_bounds__(kFcThreads) void fc_finish_kernel(const FcArgs f)
{
    constexpr int NACC = (LIMBS == 2) ? 3 : 1;
    constexpr int WAVES = kFcThreads / 64;
    constexpr int PP = LIMBS == 2 ? 2 : 1;    // pieces per part and thread
    __shared__ int outoff[FM];
    __shared__ int rowsum[FM];
    __shared__ __align__(16) int ctab[3 * FN];
    __shared__ unsigned wave_counts[2][WAVES];
    const int tid = threadIdx.x, wave = tid >> 6;
    const int tile = blockIdx.x >> 3, cb = (blockIdx.x >> 2) & 1, g = blockIdx.x & 3;
    const int mt = tile / f.n_tiles, nt = tile - mt * f.n_tiles;
    const v4i *slots = (const v4i *)(f.c.partials + (size_t)tile * f.ksplit * f.c.part_bytes);
    const size_t part_v4 = (size_t)f.c.part_bytes / 16;
    // every part's pieces are requested before any is used (the number of parts is uniform)
    v4i piece[FMAXP][PP];
#pragma unroll
    for (int o = 0; o < FMAXP; ++o)
        if (o < f.ksplit) {
#pragma unroll
            for (int h = 0; h < PP; ++h) piece[o][h] = slots[o * part_v4 + ((cb * 4 + g) * PP + h) * kFcThreads + tid];
        }
    fc_tile_tables<LIMBS>(f, mt, nt, outoff, rowsum, ctab);
    v16i acc[1][1][NACC];
#pragma unroll
    for (int q = 0; q < NACC; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[0][0][q][v] = 0;
    if constexpr (LIMBS == 2) {
        long long v[4] = {0, 0, 0, 0};
#pragma unroll
        for (int o = 0; o < FMAXP; ++o)
            if (o < f.ksplit) {
                v[0] += (long long)(((unsigned long long)(unsigned)piece[o][0].y << 32) | (unsigned)piece[o][0].x);
                v[1] += (long long)(((unsigned long long)(unsigned)piece[o][0].w << 32) | (unsigned)piece[o][0].z);
                v[2] += (long long)(((unsigned long long)(unsigned)piece[o][1].y << 32) | (unsigned)piece[o][1].x);
                v[3] += (long long)(((unsigned long long)(unsigned)piece[o][1].w << 32) | (unsigned)piece[o][1].z);
            }
        // back into pieces the epilogue combines: v = 2^16 * (v >> 16) + 2^8 * 0 + (v & 65535) would
        // do, but its 32-bit form wants a low piece below 2^8 of its own scale: (v >> 16, bits
        // 8..15, bits 0..7); |v| < 2^47, so the top piece fits
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[0][0][0][e] = (int)(v[e] >> 16);
            acc[0][0][1][e] = (int)((v[e] >> 8) & 255);
            acc[0][0][2][e] = (int)(v[e] & 255);
        }
    } else {
#pragma unroll
        for (int o = 0; o < FMAXP; ++o)
            if (o < f.ksplit) {
                acc[0][0][0][0] += piece[o][0].x;
                acc[0][0][0][1] += piece[o][0].y;
                acc[0][0][0][2] += piece[o][0].z;
                acc[0][0][0][3] += piece[o][0].w;
            }
    }
    __syncthreads();
    const TileCounts counts = tile_epilogue<LIMBS, 1, FN, 1, 1>(
        f.c, acc, [&](int m) { return rowsum[m]; }, outoff, outoff, ctab, nt, wave * 32, cb * 32, 0, g);
    if (!f.c.zero_count && !f.c.sat_count) return;
    if ((tid & 63) == 0) {
        wave_counts[0][wave] = counts.zeros;
        wave_counts[1][wave] = counts.sats;
    }
    __syncthreads();
    if (tid < 2) {
        unsigned long long total = 0;
        for (int w = 0; w < WAVES; ++w) total += wave_counts[tid][w];
        unsigned long long *dst = tid ? f.c.sat_count : f.c.zero_count;
        if (total && dst) atomicAdd(dst, total);
    }
}

// ---------------------------------------------------------------------------- host

static lp_status fc_pack(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, const void *w, void *packed, size_t packed_bytes,
                         void *stream)
{
    FcPlan p;
    const lp_status st = make_fc_plan(M, K, Nout, qx, qw, &p);
    if (st != LP_OK) return st;
    if (!w || !packed || !aligned16(w) || !aligned16(packed)) return LP_EINVAL;
    if (packed_bytes < p.packed_bytes) return LP_EWORKSPACE;
    hipStream_t hs = as_stream(stream);
    clear_stale_error();
    const size_t pieces = (size_t)p.n_tiles * p.KH * 2 * 64;
    const int grid = (int)std::min<size_t>((pieces + 255) / 256, 65535);
    unsigned char *out = (unsigned char *)packed;
    int64_t *corr = (int64_t *)(out + p.corr_offset);
    const int CoutP = p.n_tiles * FN;
#define LP_FCPACK(WT, L)                                                                                     \
    hipLaunchKernelGGL((fc_pack_weights_kernel<WT, L>), dim3(grid), dim3(256), 0, hs, (const WT *)w, out, Nout, K, \
                       p.KH, pieces);                                                                        \
    hipLaunchKernelGGL(weight_corr_kernel<WT>, dim3(CoutP), dim3(64), 0, hs, (const WT *)w, corr, Nout, CoutP, K, L)
    if (p.limbs == 2) {
        if (qw.n > 8) { LP_FCPACK(int16_t, 2); } else { LP_FCPACK(int8_t, 2); }
    } else {
        LP_FCPACK(int8_t, 1);
    }
#undef LP_FCPACK
    return launch_status();
}

static lp_status fc_forward(int M, int K, int Nout, const void *x, lp_qfmt qx, const void *wp, lp_qfmt qw,
                            const void *bias, lp_qfmt qb, int64_t *acc_out, void *y, lp_qfmt qy, int relu, lp_round r,
                            uint64_t *zero_count, uint64_t *sat_count, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    FcPlan p;
    const lp_status st = make_fc_plan(M, K, Nout, qx, qw, &p);
    if (st != LP_OK) return st;
    if (!x || !wp || (!acc_out && !y) || !aligned16(x) || !aligned16(wp)) return LP_EINVAL;
    if ((acc_out && !aligned16(acc_out)) || (y && !aligned16(y))) return LP_EINVAL;
    const int f_acc = qx.f + qw.f;
    if (bias && (!fmt_ok(qb) || qb.f > f_acc || f_acc - qb.f > 40)) return LP_EINVAL;
    if (r != LP_ROUND_NEAREST_AWAY && r != LP_ROUND_NEAREST_EVEN) return LP_EINVAL;
    // the split input lives in the workspace: unlike lp_conv_fwd's, this one is always needed
    if (!workspace || workspace_bytes < p.ws_total || !aligned16(workspace)) return LP_EWORKSPACE;
    FcArgs f = {};
    ConvArgs &a = f.c;
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
    a.N = M; a.H = 1; a.W = 1; a.Cin = K; a.Cout = Nout; a.R = 1; a.S = 1; a.stride = 1; a.pad = 0;
    a.Ho = 1; a.Wo = 1; a.Hp = 1; a.FR = M;
    const bool counting = (zero_count || sat_count) && y;
    unsigned char *ws = (unsigned char *)workspace;
    // (a small grid adds its counts to the counters itself, a large one leaves per-workgroup slots)
    const bool direct = counting && p.ksplit == 1 && p.grid <= 2048;
    a.direct_counts = direct ? 1 : 0;
    if (counting && p.ksplit == 1 && !direct) a.zero_partial = (unsigned *)ws;
    a.partial_stride = p.grid;
    a.partials = ws + p.ws_counts + p.ws_xs + p.ws_xsum;
    a.part_bytes = (int)p.part_bytes;
    // The 32-bit epilogue: as for the convolution (codes only, ReLU, round-half-away, a right shift
    // of 1..31 bits, K <= 8192 so that no int32 piece can overflow).
    a.fast = (y && !acc_out && relu && r == LP_ROUND_NEAREST_AWAY && a.act.s >= 1 && a.act.s <= 31 && K <= 8192 &&
              (!bias || a.bias_shift <= 24) && (unsigned long long)FM * Nout * 2 < (1ull << 31)) ? 1 : 0;
    f.xs = ws + p.ws_counts;
    f.xs_bytes = (unsigned)((size_t)p.mblocks * p.KH * p.limbs * FRAG);
    f.xsum = (const int *)(ws + p.ws_counts + p.ws_xs);
    f.kc = p.kc;
    f.mrows = p.mblocks * 32;
    f.M = M; f.K = K; f.KH = p.KH; f.khp = p.khp; f.ksplit = p.ksplit;
    f.n_tiles = p.n_tiles; f.tiles = p.tiles; f.per_xcd = p.per_xcd; f.total = p.tiles * p.ksplit;
    f.wslab = (unsigned)p.wslab;
    hipStream_t hs = as_stream(stream);
    clear_stale_error();
    const dim3 sgrid(p.mblocks, p.kc);
    if (p.limbs == 2) {
        hipLaunchKernelGGL((fc_split_x_kernel<int16_t, 2>), sgrid, dim3(64 * kSplitWaves), 0, hs, (const int16_t *)x,
                           const_cast<unsigned char *>(f.xs), const_cast<int *>(f.xsum), M, K, p.KH, p.khc);
        hipLaunchKernelGGL(fc_mfma_kernel<2>, dim3(p.grid), dim3(kFcThreads), 0, hs, f);
        if (p.ksplit > 1) hipLaunchKernelGGL(fc_finish_kernel<2>, dim3(p.tiles * 8), dim3(kFcThreads), 0, hs, f);
    } else {
        hipLaunchKernelGGL((fc_split_x_kernel<int8_t, 1>), sgrid, dim3(64 * kSplitWaves), 0, hs, (const int8_t *)x,
                           const_cast<unsigned char *>(f.xs), const_cast<int *>(f.xsum), M, K, p.KH, p.khc);
        hipLaunchKernelGGL(fc_mfma_kernel<1>, dim3(p.grid), dim3(kFcThreads), 0, hs, f);
        if (p.ksplit > 1) hipLaunchKernelGGL(fc_finish_kernel<1>, dim3(p.tiles * 8), dim3(kFcThreads), 0, hs, f);
    }
    const lp_status ls = launch_status();
    if (ls != LP_OK || p.ksplit > 1 || !counting || direct) return ls;
    return launch_sum_partials(a.zero_partial, p.grid, a.zero_count, a.sat_count, hs);
}

} // namespace lp

using namespace lp;

extern "C" lp_status lp_fc_packed_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host)
{
    if (!bytes_host) return LP_EINVAL;
    if (!fmt_ok(qx) || !fmt_ok(qw)) return LP_EINVAL;
    if (!fc_kernel_takes(qx, qw)) return fc_conv_packed_bytes(M, K, Nout, qx, qw, bytes_host);
    FcPlan p;
    const lp_status st = make_fc_plan(M, K, Nout, qx, qw, &p);
    if (st == LP_OK) *bytes_host = p.packed_bytes;
    return st;
}

extern "C" lp_status lp_fc_pack_weights(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, const void *w_codes_dev,
                                        void *packed_dev, size_t packed_bytes, void *stream)
{
    if (!fmt_ok(qx) || !fmt_ok(qw)) return LP_EINVAL;
    if (!fc_kernel_takes(qx, qw)) return fc_conv_pack_weights(M, K, Nout, qx, qw, w_codes_dev, packed_dev, packed_bytes, stream);
    return fc_pack(M, K, Nout, qx, qw, w_codes_dev, packed_dev, packed_bytes, stream);
}

extern "C" lp_status lp_fc_workspace_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host)
{
    if (!bytes_host) return LP_EINVAL;
    if (!fmt_ok(qx) || !fmt_ok(qw)) return LP_EINVAL;
    if (!fc_kernel_takes(qx, qw)) return fc_conv_workspace_bytes(M, K, Nout, qx, qw, bytes_host);
    FcPlan p;
    const lp_status st = make_fc_plan(M, K, Nout, qx, qw, &p);
    if (st == LP_OK) *bytes_host = p.ws_total;
    return st;
}

extern "C" lp_status lp_fc_fwd(int M, int K, int Nout, const void *x_codes_dev, lp_qfmt qx, const void *w_packed_dev,
                               lp_qfmt qw, const void *bias_codes_dev, lp_qfmt qb, int64_t *acc_out_dev,
                               void *y_codes_dev, lp_qfmt qy, int relu, lp_round r, uint64_t *zero_count_dev,
                               uint64_t *sat_count_dev, void *workspace_dev, size_t workspace_bytes, void *stream)
{
    if (!fmt_ok(qx) || !fmt_ok(qw)) return LP_EINVAL;
    if (!fc_kernel_takes(qx, qw))
        return fc_conv_fwd(M, K, Nout, x_codes_dev, qx, w_packed_dev, qw, bias_codes_dev, qb, acc_out_dev, y_codes_dev,
                           qy, relu, r, zero_count_dev, sat_count_dev, workspace_dev, workspace_bytes, stream);
    return fc_forward(M, K, Nout, x_codes_dev, qx, w_packed_dev, qw, bias_codes_dev, qb, acc_out_dev, y_codes_dev, qy,
                      relu, r, zero_count_dev, sat_count_dev, workspace_dev, workspace_bytes, stream);
}
