/*
 * lp.h -- C ABI of the MI355X (gfx950) low-precision fixed-point forward library.
 *
 * The library runs the forward pass of the paper's low-precision layers
 * (LPConvolution, LPInnerProduct, LPAct; Sec. 2 "Low-precision add-on for
 * Caffe") on integer Qm.f codes, exactly: int8 MFMA products, int32 partial
 * sums, int64 results.
 *
 * Notation (Sec. 2, footnote on Qm.f and the BD / AD parameters): a format is
 * (n, m, f): n total bits, m integer bits INCLUDING the sign bit (BD), f
 * fraction bits (AD), n = m + f.  A code q in [-2^(n-1), 2^(n-1)-1] stands for
 * the real number q * 2^-f.
 *
 * General rules of this ABI
 *   - Pointers named *_dev are device (HBM) pointers, *_host are host pointers.
 *     The caller owns every buffer; the library allocates no device memory.
 *   - Code storage: int8_t when n <= 8, int16_t when 9 <= n <= 16, sign-extended.
 *   - Activations are NHWC, weights [Cout][R][S][Cin], FC inputs [M][K], FC
 *     weights [Nout][K]: the contraction index is always contiguous.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     only enqueue work and return, except lp_range / lp_range_acc, which wait
 *     for the stream because they return a result on the host.
 *   - Counters (zero_count_dev, sat_count_dev) are uint64 in device memory and
 *     are ADDED to: the caller clears them when a fresh count is wanted.
 *   - Every argument is validated before anything is launched; a call that
 *     returns anything but LP_OK has launched nothing.  Errors are return codes
 *     only.  Device pointers must be aligned to 16 bytes.
 */
#ifndef LP_H
#define LP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct { int32_t n, m, f; } lp_qfmt; /* n == m + f, 1 <= m <= n, 2 <= n <= 16 */

/* rounding_scheme of Sec. 2: deterministic (two tie rules offered, the paper
 * names none) or stochastic (Sec. 2.4). */
typedef enum {
    LP_ROUND_NEAREST_AWAY = 0, /* halfway cases away from zero (default) */
    LP_ROUND_NEAREST_EVEN = 1, /* halfway cases to the even code */
    LP_ROUND_STOCHASTIC = 2    /* lp_quantize and lp_act_stochastic only */
} lp_round;

typedef enum {
    LP_OK = 0,
    LP_EINVAL = 1,       /* bad format, size, null or misaligned pointer */
    LP_EUNSUPPORTED = 2, /* valid request outside what the kernels cover */
    LP_EWORKSPACE = 3,   /* workspace / packed buffer too small */
    LP_EDEVICE = 4       /* the HIP runtime reported an error for a launch of this call (an error
                            that an earlier, unrelated HIP call left pending is dropped at entry) */
} lp_status;

/* stride-s convolution with zero padding `pad` on all four sides;
 * output is N x Ho x Wo x Cout, Ho = (H + 2*pad - R)/stride + 1.
 * pool (0 or 1, may be left out of an initialiser): 1 asks lp_conv_fwd to apply the 2x2 /
 * stride-2 max-pool that follows the layer ("Pooling" column of Table 1) before storing, so
 * that y is N x Ho/2 x Wo/2 x Cout and the unpooled codes never reach memory.  Offered only
 * where the tiling allows it at no loss (else LP_EUNSUPPORTED from every call that takes
 * the descriptor: run the layer with pool = 0 and lp_maxpool2x2 instead). */
typedef struct { int32_t N, H, W, Cin, Cout, R, S, stride, pad, pool; } lp_conv_desc;

const char *lp_status_string(lp_status s);

/* Number of uint64 words of device scratch lp_range / lp_range_acc need. */
#define LP_RANGE_WORKSPACE_WORDS 32

/*
 * lp_range -- layer-wise bit allocation from the dynamic range (Sec. 2.3
 * "Layer-wise quantization").  With n fixed, a value is lost for m integer
 * bits when |v| >= 2^(m-1).  Writes to *out_host the format with the smallest
 * m in [1, n] whose lost share (lost / count) is <= loss_threshold (m = n if
 * none); loss_threshold 0 places the point from max|v|.  NaN is never lost,
 * +-Inf always.  lost_host (nullable) receives n+1 counts, lost_host[m] for
 * m = 1..n (entry 0 unused).  workspace_dev: LP_RANGE_WORKSPACE_WORDS uint64.
 * Synchronises the stream.  count == 0 yields m = 1.
 */
lp_status lp_range(const float *x_dev, size_t count, int n, double loss_threshold,
                   lp_qfmt *out_host, uint64_t *lost_host, uint64_t *workspace_dev, void *stream);

/*
 * lp_range_acc -- the same rule for exact accumulators that stand for
 * acc * 2^-f_acc (as lp_conv_fwd / lp_fc_fwd emit), after ReLU when relu != 0.
 * Used to fix a layer's output format from a calibration batch (Sec. 2.1: the
 * ranges are measured on a sample of inputs, then frozen).
 */
lp_status lp_range_acc(const int64_t *acc_dev, size_t count, int f_acc, int relu, int n,
                       double loss_threshold, lp_qfmt *out_host, uint64_t *lost_host,
                       uint64_t *workspace_dev, void *stream);

/*
 * lp_quantize -- the Qm.f quantizer of the low-precision layers (Sec. 2):
 * code = clip(round(x * 2^f)) to the signed n-bit range (Sec. 2.5: values that
 * do not fit saturate).  NaN gives code 0.  codes_dev: int8 (n <= 8) or int16.
 * LP_ROUND_STOCHASTIC (Sec. 2.4): floor(x*2^f) + [u < frac], where u in [0,1)
 * is 2^-32 * a word of Philox4x32-10 (Salmon et al., SC'11) with key
 * (seed lo, seed hi): element i draws word i % 4 of the block with counter
 * (b lo, b hi, 0, 0), b = i / 4; the other modes ignore `seed`.
 * zero_count_dev / sat_count_dev (nullable): += number of zero codes / clipped values.
 */
lp_status lp_quantize(const float *x_dev, void *codes_dev, size_t count, lp_qfmt q, lp_round r,
                      uint64_t seed, uint64_t *zero_count_dev, uint64_t *sat_count_dev,
                      void *stream);

/*
 * lp_act -- LPAct followed by the activation function (Sec. 2.1: activations
 * are quantized, then passed to ReLU; the two commute, so ReLU is applied to
 * the accumulator first).  acc stands for acc * 2^-f_acc; the output code has
 * qy.f fraction bits: code = clip(round(max(acc,0) / 2^(f_acc - qy.f))).
 * |acc| must be below 2^62; -31 <= f_acc - qy.f <= 62.
 * zero_count_dev (nullable): += number of zero output codes (Sec. 3.1 defines
 * sparsity as zeros over elements).  sat_count_dev (nullable): += number of
 * values whose rounded result lay outside the code range and was clipped, i.e.
 * the activations this format loses (Sec. 2.3 keeps their share under a
 * threshold when it places the point; Sec. 2.5: they saturate).  After ReLU
 * only the upper end can clip.  r: NEAREST_AWAY or NEAREST_EVEN.
 */
lp_status lp_act(const int64_t *acc_dev, size_t count, int f_acc, lp_qfmt qy, int relu, lp_round r,
                 void *y_codes_dev, uint64_t *zero_count_dev, uint64_t *sat_count_dev, void *stream);

/*
 * lp_act_stochastic -- lp_act with the stochastic rounding_scheme (Sec. 2.4):
 * with t = max(acc,0) / 2^(f_acc - qy.f) (ReLU only if relu != 0) the code is
 * clip(floor(t) + [u < t - floor(t)]), u as in lp_quantize: 2^-32 * word i % 4
 * of the Philox4x32-10 block with key (seed lo, seed hi) and counter (i / 4, 0)
 * for element index i.  The comparison is exact (integers).  f_acc <= qy.f
 * needs no rounding and gives lp_act's result.  Other arguments, limits and
 * errors as lp_act.  lp_conv_fwd / lp_fc_fwd do not fuse this scheme: pass
 * their acc_out_dev here.
 */
lp_status lp_act_stochastic(const int64_t *acc_dev, size_t count, int f_acc, lp_qfmt qy, int relu,
                            uint64_t seed, void *y_codes_dev, uint64_t *zero_count_dev,
                            uint64_t *sat_count_dev, void *stream);

/*
 * Weight packing for lp_conv_fwd / lp_fc_fwd.  Done once per layer, outside
 * the timed path (the paper converts weight blobs offline, Sec. 2.1).  The
 * packed buffer is opaque: int8 limb planes in the order the kernel streams
 * them plus per-output-channel correction sums.  qx is needed because the
 * layout depends on whether activations are 8- or 16-bit.
 * lp_conv_packed_bytes writes the buffer size to *bytes_host.
 */
lp_status lp_conv_packed_bytes(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host);
lp_status lp_conv_pack_weights(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, const void *w_codes_dev,
                               void *packed_dev, size_t packed_bytes, void *stream);

/*
 * lp_conv_plan_info -- how lp_conv_fwd will run this problem (host-only query, for
 * reports and tests).  path: 0 = direct one-thread-per-output kernel, 1 = int8-MFMA
 * implicit GEMM.  For path 1: kernel (LP_KERNEL_PATCH: 64-channel chunks of a staged patch, every
 * tap a shifted read; LP_KERNEL_FLAT: fewer than 16 input channels, the whole window as one K <= 64
 * slab; LP_KERNEL_ROWS: 16-bit codes with 16, 32 or 48 input channels, the reduction runs over
 * window rows of a densely staged patch), limbs (1 = int8 codes, 2 = 16-bit codes as two int8
 * limbs), the workgroup tile (128 output pixels = tile_rows consecutive rows of the
 * N*Ho stacked output rows x tile_cols columns, times bn output channels), the staged
 * input patch (patch_rows x patch_cols pixels; a pixel takes patch_pixel bytes per limb -- patch kernel: 64 of
 * codes and the rest padding that spreads consecutive pixels over the LDS banks; rows are
 * patch_pitch bytes apart), tile counts and LDS bytes per workgroup; the launch: workgroups in the grid, and split = parts into which each tile of the
 * last, partly filled round of workgroup slots is cut along the reduction (1 = none; used
 * only when a workspace is passed).  Work item wi = pixel tile * tiles_n + channel tile (pixel
 * tiles row-major over stacked output rows x columns); die j of the chip's eight owns the items
 * j * items_per_die ... (j + 1) * items_per_die - 1, of which the first whole_items_per_die are
 * computed by one workgroup each and the rest are the split ones.
 */
typedef struct {
    int32_t path, limbs, bn, tile_rows, tile_cols, patch_rows, patch_cols, tiles_m, tiles_n;
    int32_t lds_bytes, patch_pitch, patch_pixel, workgroups, split;
    int32_t items_per_die, whole_items_per_die;
    int32_t kernel;
} lp_plan_info;
enum { LP_KERNEL_DIRECT = 0, LP_KERNEL_PATCH = 1, LP_KERNEL_FLAT = 2, LP_KERNEL_ROWS = 3 };
lp_status lp_conv_plan_info(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, lp_plan_info *out_host);

/*
 * lp_conv_pool_check -- whether lp_conv_fwd will take this call with d->pool = 1 (host-only
 * query; the plan-level conditions are those of lp_conv_plan_info).  The fused pool rides on the
 * 32-bit epilogue: 16-bit codes out, ReLU, round-half-away, a right shift qx.f + qw.f - qy.f of
 * 1..31 bits, R*S*Cin <= 8192, a bias (has_bias != 0, format qb) whose shift qx.f + qw.f - qb.f
 * is at most 24 bits, Cout a multiple of 4.  LP_OK, or LP_EUNSUPPORTED: run the layer with
 * pool = 0 and lp_maxpool2x2.
 */
lp_status lp_conv_pool_check(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, int has_bias, lp_qfmt qb, lp_qfmt qy,
                             int relu, lp_round r);

/* Bytes of device workspace lp_conv_fwd uses for this problem (may be 0): per-workgroup
 * partial zero counts, and room for the partial sums of tiles whose reduction is shared
 * between workgroups.  The workspace is required when zero_count_dev or sat_count_dev is given; otherwise it
 * is optional, and without it every tile is reduced by a single workgroup (same results,
 * idle CUs in the last round).  Its contents need no initialisation and carry nothing from
 * call to call; calls that share one workspace must not overlap in time. */
lp_status lp_conv_workspace_bytes(const lp_conv_desc *d, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host);

/*
 * lp_conv_fwd -- LPConvolution forward (Sec. 2) with the LPAct + ReLU step
 * fused (Sec. 2.1):
 *   acc[n,y,x,co] = sum_{r,s,ci} X[n, y*stride+r-pad, x*stride+s-pad, ci] * W[co,r,s,ci]
 *                   (+ bias[co] * 2^(qx.f + qw.f - qb.f)),   zero outside the image,
 * exact in int64, fraction bits f_acc = qx.f + qw.f.
 *   x_codes_dev   NHWC codes in format qx
 *   w_packed_dev  from lp_conv_pack_weights (same d, qx, qw)
 *   bias_codes_dev nullable; Cout codes in format qb (int8/int16 by qb.n), qb.f <= f_acc
 *   acc_out_dev   nullable; receives the raw int64 accumulators, N x Ho x Wo x Cout
 *   y_codes_dev   nullable; receives lp_act(acc) in format qy (see lp_act), same shape
 *                 (d->pool: the 2x2 maxima of those codes, N x Ho/2 x Wo/2 x Cout)
 *   zero_count_dev nullable; += zeros among the y codes (d->pool: among the codes before
 *                 pooling, i.e. the layer's activation sparsity); needs workspace_dev
 *   sat_count_dev nullable; += y codes that were clipped (see lp_act; counted before pooling
 *                 too); needs workspace_dev
 *   workspace_dev nullable unless a counter is given; 16-byte aligned and at least
 *                 lp_conv_workspace_bytes long, else LP_EWORKSPACE
 * At least one of acc_out_dev / y_codes_dev must be given.
 * LP_EUNSUPPORTED: R*S*Cin >= 65536 with 16-bit operands (int32 limb sums
 * could overflow), tensors with 2^31 or more elements, packed weights of 2 GiB or more;
 * d->pool outside its conditions (no acc_out_dev, even Ho and Wo, a tile geometry of even
 * rows and columns as good as the unconstrained one, and those of lp_conv_pool_check).
 * Shapes the int8-MFMA kernels do not take (stride > 1, 8-bit activations with 16-bit
 * weights, Cin neither a multiple of 8 (16 for 8-bit codes) nor small enough for R*S*Cin <= 64)
 * run on a plain one-thread-per-output kernel, correct but some hundred times slower:
 * lp_conv_plan_info reports path = 0 for them.
 */
lp_status lp_conv_fwd(const lp_conv_desc *d, const void *x_codes_dev, lp_qfmt qx,
                      const void *w_packed_dev, lp_qfmt qw, const void *bias_codes_dev, lp_qfmt qb,
                      int64_t *acc_out_dev, void *y_codes_dev, lp_qfmt qy, int relu, lp_round r,
                      uint64_t *zero_count_dev, uint64_t *sat_count_dev, void *workspace_dev,
                      size_t workspace_bytes, void *stream);

/*
 * Skipping multiplications by zero (abstract and Sec. 3.1: the sparsity that low-precision
 * training produces is there so that the target hardware can skip it), at the granularity a
 * matrix unit allows: whole tiles.  A layer run through lp_conv_fwd_zskip leaves one byte per
 * (pixel tile, channel tile) of its output in y_tile_flags_dev (tiles_m * tiles_n bytes, see
 * lp_conv_plan_info), 1 = the tile holds a code that is not zero.  The next layer is handed
 * those flags with the geometry they were written in (lp_zero_map, filled from the PRODUCER's
 * lp_plan_info: tile_rows, tile_cols, tiles_c = ceil(Wo / tile_cols), tiles_n, bn; scale = 2 if
 * the codes went through the 2x2 max-pool, fused or not, before this layer reads them, else 1)
 * and neither stages nor multiplies a 64-channel chunk of a workgroup's input patch when every
 * producer tile the patch touches is flagged all-zero.  Results are those of lp_conv_fwd, bit
 * for bit.  skipped_dev (nullable): += (workgroup tile, chunk) pairs skipped.  Either of
 * x_zero_map_host / y_tile_flags_dev may be null.  Needs the int8-MFMA path (path 1), codes out
 * (no raw accumulators) and, for y_tile_flags_dev, the workspace; else LP_EUNSUPPORTED /
 * LP_EINVAL.  Other arguments and errors as lp_conv_fwd.
 */
typedef struct {
    const uint8_t *flags_dev;
    int32_t tile_rows, tile_cols, tiles_c, tiles_n, bn, scale;
} lp_zero_map;
lp_status lp_conv_fwd_zskip(const lp_conv_desc *d, const void *x_codes_dev, lp_qfmt qx,
                            const lp_zero_map *x_zero_map_host, const void *w_packed_dev, lp_qfmt qw,
                            const void *bias_codes_dev, lp_qfmt qb, void *y_codes_dev, lp_qfmt qy, int relu,
                            lp_round r, uint64_t *zero_count_dev, uint64_t *sat_count_dev,
                            uint8_t *y_tile_flags_dev, uint64_t *skipped_dev, void *workspace_dev,
                            size_t workspace_bytes, void *stream);

/*
 * lp_conv_fwd_static -- lp_conv_fwd for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): the workspace is
 * an array of LP_STATIC_WORKSPACE_BYTES that the library's code object holds on every GPU it is
 * loaded on, until the process ends; the call allocates nothing on host or device through HIP.
 * Arguments, results and errors as lp_conv_fwd (with that workspace passed); problems whose
 * lp_conv_workspace_bytes exceeds LP_STATIC_WORKSPACE_BYTES return LP_EWORKSPACE.  The array
 * used is that of the device current at the call, which must be the stream's device.  All calls
 * on one GPU share the array: calls that overlap in time on one GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.  Nothing is carried from call to call.
 */
#define LP_STATIC_WORKSPACE_BYTES (64u << 20)
lp_status lp_conv_fwd_static(const lp_conv_desc *d, const void *x_codes_dev, lp_qfmt qx,
                             const void *w_packed_dev, lp_qfmt qw, const void *bias_codes_dev, lp_qfmt qb,
                             int64_t *acc_out_dev, void *y_codes_dev, lp_qfmt qy, int relu, lp_round r,
                             uint64_t *zero_count_dev, uint64_t *sat_count_dev, void *stream);

/*
 * lp_fc_fwd -- LPInnerProduct forward (Sec. 2) with the same fused tail:
 *   acc[b,o] = sum_k X[b,k] * W[o,k] (+ bias), x [M][K], w packed from [Nout][K].
 * Packing / workspace: the lp_fc_* functions below.  Other arguments as lp_conv_fwd, except
 * that the workspace is always required (LP_EWORKSPACE without it): the call first splits the
 * input rows into int8 limb planes there, then runs a split-K GEMM whose parts meet there.
 * Its contents need no initialisation and carry nothing from call to call; calls that share
 * one workspace must not overlap in time.
 */
lp_status lp_fc_packed_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host);
lp_status lp_fc_pack_weights(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, const void *w_codes_dev,
                             void *packed_dev, size_t packed_bytes, void *stream);
lp_status lp_fc_workspace_bytes(int M, int K, int Nout, lp_qfmt qx, lp_qfmt qw, size_t *bytes_host);
lp_status lp_fc_fwd(int M, int K, int Nout, const void *x_codes_dev, lp_qfmt qx,
                    const void *w_packed_dev, lp_qfmt qw, const void *bias_codes_dev, lp_qfmt qb,
                    int64_t *acc_out_dev, void *y_codes_dev, lp_qfmt qy, int relu, lp_round r,
                    uint64_t *zero_count_dev, uint64_t *sat_count_dev, void *workspace_dev,
                    size_t workspace_bytes, void *stream);

/*
 * lp_maxpool2x2 -- 2x2 max, stride 2, on NHWC codes (the pooling between VGG16
 * blocks; "Pooling" column of Table 1).  H and W must be even.  n_bits selects
 * int8 (<= 8) or int16 storage.  Output N x H/2 x W/2 x C.
 */
lp_status lp_maxpool2x2(const void *x_codes_dev, void *y_codes_dev, int N, int H, int W, int C,
                        int n_bits, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LP_H */
