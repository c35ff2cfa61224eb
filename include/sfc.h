/*
 * sfc.h -- C ABI of the MI355X (gfx950) library for quantized 3x3 convolution by
 * Symbolic Fourier Convolution, SFC-6(6x6,3x3) and SFC-6(7x7,3x3) (arXiv 2407.02913),
 * with SFC-4(4x4,3x3), the 5x5-filter algorithm SFC-6(6x6,5x5) and the 7x7-filter algorithm
 * SFC-6(4x4,7x7) beside them.
 *
 * The library computes, for int8 activations x[N,Cin,H,W] and int8 filters
 * w[Cout,Cin,R,R] (R = 3, or 5 for the SFC-6(6x6,5x5) and 7 for the SFC-6(4x4,7x7)
 * algorithms; stride 1, zero padding (R-1)/2, cross-correlation),
 *
 *      y = A^T [ (G f G^T) . (B^T x B) ] A        summed over Cin      (Eq. 1)
 *
 * with the addition-only symbolic DFT-6 transforms of Sec. 4.1, the correction
 * terms of Sec. 4.2 and the integrated matrices of Appendix A, on MxM output
 * tiles ((M+2)x(M+2) input tiles), M = 6 or 7 -- or 4, with the four-point transforms
 * of SFC-4(4x4,3x3).  Per tile and (Cin,Cout) pair it spends P = 88 / 132 / 46
 * multiplications (Hermitian form, M = 6 / 7 / 4) or P = 100 / 144 / 49 (nested form),
 * Appendix A.  SFC-6(6x6,5x5) works on 6x6 output tiles (10x10 input tiles) with
 * P = 184 (Hermitian) or 196 (nested) multiplications instead of 900; SFC-6(4x4,7x7) on
 * 4x4 output tiles (the same 10x10 input tiles) with as many instead of 784.
 *
 * Conventions
 *  - "dev" pointers are device (HBM) addresses on the current HIP device, "host"
 *    pointers are ordinary host memory.  Device pointers must be 16-byte aligned.
 *  - The library never allocates or frees device memory and never synchronizes
 *    the stream, except where a call says it blocks.  The caller owns every
 *    device buffer and keeps it alive until the work queued on `stream` is done.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - Every call returns an sfc_status; argument errors are detected before any
 *    launch; nothing is printed and nothing aborts.
 *  - A plan is host memory owned by the library.  After sfc_transform_filter it
 *    is read-only and may serve concurrent sfc_conv2d_nchw calls on different
 *    streams provided each call has its own workspace.
 */
#ifndef SFC_H_
#define SFC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sfc_plan_s sfc_plan_t;

typedef enum {
  SFC_OK = 0,
  SFC_EINVAL = 1,       /* null pointer, non-positive size, misaligned pointer, bad enum */
  SFC_EUNSUPPORTED = 2, /* valid request this build does not implement */
  SFC_ENOMEM = 3,       /* host allocation failed */
  SFC_ENOTREADY = 4,    /* scales or filter not set yet */
  SFC_EHIP = 5,         /* a HIP runtime call or kernel launch failed */
  SFC_EWORKSPACE = 6    /* a caller-owned device buffer is smaller than sfc_plan_sizes says */
} sfc_status;

/* Which 2-D point set realizes the element-wise product of Eq. (1), Appendix A. */
typedef enum {
  /* sfc_plan picks the tile size for 3x3 filters from the layer shape (sfc_plan_choice tells
   * which).  Requantized mode: SFC-4's 4x4 tiles, except 7x7 tiles on 14x14 and 7x7 maps
   * with many (tile, filter) pairs; exact mode: 6x6 tiles; always the Hermitian point set. */
  SFC_ALG_AUTO = -1,
  SFC_ALG_6X6_P88 = 0,  /* SFC-6(6x6,3x3), Hermitian symmetry fully used: 88 multiplications per tile */
  SFC_ALG_6X6_P100 = 1, /* SFC-6(6x6,3x3), nested (Kronecker) form: 100 multiplications */
  SFC_ALG_7X7_P132 = 2, /* SFC-6(7x7,3x3) (Sec. 4.2, Appendix A), Hermitian form: 132 multiplications */
  SFC_ALG_7X7_P144 = 3, /* SFC-6(7x7,3x3), nested form: 144 multiplications */
  /* SFC-4(4x4,3x3) (Appendix A, four-point symbolic DFT, s = j): 46 multiplications per
   * 4x4 tile with Hermitian symmetry fully used, 49 in the nested form.  Every path. */
  SFC_ALG_4X4_P46 = 4,
  SFC_ALG_4X4_P49 = 5,
  /* SFC-6(6x6,5x5) (Appendix A): 5x5 filters w[Cout,Cin,5,5], zero padding 2, 6x6 output
   * tiles; 184 multiplications per tile in the Hermitian form, 196 in the nested form.
   * B^T and G are the printed ones; the printed A (seven columns for six outputs) is
   * replaced by the one matrix that fits them.  Staged and fused paths. */
  SFC_ALG_6X6_5X5_P184 = 6,
  SFC_ALG_6X6_5X5_P196 = 7,
  /* SFC-6(4x4,7x7) (Table 1, last row): 7x7 filters w[Cout,Cin,7,7], zero padding 3, 4x4
   * output tiles from the same 10x10 input tiles and the same input transform as
   * SFC-6(6x6,5x5).  The paper prints no matrices for it; G and A follow from the steps of
   * Sec. 4.1-4.2 that reproduce the printed SFC-6(6x6,5x5) ones (filter DFT
   * G_k = sum_r f_r s^(k r), six correction terms).  184 multiplications per tile in the
   * Hermitian form, 196 nested, of 784 (Table 1's 21.99 % is no whole number of
   * multiplications and is not reproduced).  Staged and fused paths. */
  SFC_ALG_4X4_7X7_P184 = 8,
  SFC_ALG_4X4_7X7_P196 = 9
} sfc_alg;

typedef enum {
  /* Transform domain kept in exact integers (int16 operands, int32 sums): the
   * result equals direct convolution bit for bit (Sec. 5.1 assumes the
   * transforms accurate).  int32 sums are guaranteed for Cin <= 404 (3x3 filters),
   * Cin <= 145 (5x5 filters) and Cin <= 74 (7x7 filters). */
  SFC_MODE_EXACT = 0,
  /* Transform-domain operands rounded to int8 with one scale per point for the
   * activations and one per (point, Cout) for the filters (Sec. 5, the
   * frequency-wise / channel-wise quantization equation). */
  SFC_MODE_REQUANT_I8 = 1
} sfc_mode;

typedef enum {
  SFC_OUT_F32 = 0, /* y float32 [N,Cout,H,W], dequantized */
  SFC_OUT_I32 = 1, /* exact mode only: the raw integer sums, int32 [N,Cout,H,W] */
  /* requantized mode only: the next layer's int8 activations,
   * clamp(round-half-even(max(y, 0) / y_scale), 0, 127), int8 [N,Cout,H,W]; the
   * scale is set with sfc_set_output_scale.  This is the epilogue that chains
   * stride-1 layers of a stack without a float32 round trip. */
  SFC_OUT_I8_RELU = 2
} sfc_out;

typedef enum {
  /* sfc_plan picks the fastest path that covers the layer (sfc_plan_choice tells which) */
  SFC_PATH_AUTO = -1,
  SFC_PATH_STAGED = 0, /* V and M pass through the workspace; taps available */
  SFC_PATH_FUSED = 1,  /* product and output transform in one kernel; M never leaves the chip */
  /* Input transform, products and output transform in one kernel; neither V nor M leaves the
   * chip, the workspace is used by calibration only.  Cin <= 64; with the SFC-4 forms also
   * Cin <= 128, and Cin <= 512 on feature maps of at most 16 tiles (16x16 and smaller). */
  SFC_PATH_SINGLE = 2
} sfc_path;

typedef struct {
  int32_t N, Cin, Cout, H, W; /* stride 1; filter size and zero padding follow from alg */
  int32_t alg;                /* sfc_alg */
  int32_t mode;               /* sfc_mode */
  int32_t out;                /* sfc_out */
  int32_t path;               /* sfc_path */
  int32_t per_channel_wscale; /* 0: one filter scale, 1: Cout filter scales */
  /* Requantized mode: bit width b of the transform-domain operands, 2..8 (0 = 8).  V and U
   * are rounded to integers in [-(2^(b-1) - 1), 2^(b-1) - 1] and still travel as int8, so
   * the low-precision settings the paper evaluates (int8 down to int4 in the transform
   * domain, Sec. 6) run on the same kernels; the abs-max calibration helpers divide by the
   * same bound.  Must be 0 in exact mode. */
  int32_t transform_bits;
  /* SFC_FLAG_* bits, 0 for none */
  int32_t flags;
} sfc_conv_desc;

/* Exact mode keeps every sum in 32 bits.  The sums an output is made of (kDen = 36, or 16 for
 * SFC-4, times the convolution sum) are guaranteed to fit for Cin <= 404 with 3x3 filters and
 * Cin <= 145 with 5x5 and Cin <= 74 with 7x7 filters; sfc_plan refuses more channels (SFC_EUNSUPPORTED) unless this
 * flag is set.  The arithmetic runs modulo 2^32 (unsigned, so wrap-around is defined): with
 * the SFC-6 forms an output is exact whenever its kDen-fold sum lies inside the int32 range,
 * whatever the intermediate sums do (the only division on the way, by 3, is a multiplication
 * by the inverse of 3 modulo 2^32); the SFC-4 forms halve intermediate sums, which must fit
 * as well.  With the flag the caller vouches for that on its data. */
enum { SFC_FLAG_EXACT_WIDE = 1 };

/* Host only.  Validates the description and derives the tile grid
 * (ceil(H/M) x ceil(W/M) tiles per image) and all buffer sizes.  No device work.
 * *out receives a plan to be released with sfc_plan_destroy. */
sfc_status sfc_plan(const sfc_conv_desc* desc, sfc_plan_t** out);
void sfc_plan_destroy(sfc_plan_t* plan);

/* What sfc_plan chose (or was given): the sfc_alg and sfc_path the plan runs.  Either output
 * pointer may be NULL. */
sfc_status sfc_plan_choice(const sfc_plan_t* plan, int32_t* alg, int32_t* path);

/* Sizes the caller must allocate (device bytes) and the derived counts:
 * P = multiplications per tile (88, 100, 132, 144, 46, 49, 184 or 196),
 * tiles = N*ceil(H/M)*ceil(W/M).
 * Any output pointer may be NULL. */
sfc_status sfc_plan_sizes(const sfc_plan_t* plan, size_t* filter_bytes, size_t* workspace_bytes,
                          int32_t* P, int64_t* tiles);

/* Requantized mode: the transform-domain scales of Sec. 5, copied into the plan.
 * sx_host[P]: one activation scale per point (s_Tx).  sw_host[P*Cout], laid out
 * [P][Cout]: one filter scale per point and output channel (s_Tf).  All > 0.
 * Point order, with R = 10 (M = 6), 12 (M = 7), 7 (M = 4) or 14 (5x5 and 7x7 filters) rows in the
 * printed 1-D matrices: nested form, p = R*p1 + p2 (p1 vertical); Hermitian form, first the nested
 * points that are not complex x complex (R*R - 36 of them, R*R - 9 for M = 4), in that
 * same order, then for (k1,k2) = (1,1),(1,2),(2,1),(2,2) (only (1,1) for M = 4) the six
 * points U0,U1,U0+U1,V0,V1,V0+V1 of the two independent 2-D frequencies.
 * Must precede sfc_transform_filter. */
sfc_status sfc_set_point_scales(sfc_plan_t* plan, const float* sx_host, const float* sw_host);

/* SFC_OUT_I8_RELU plans: the activation scale of the output tensor (> 0), host only.
 * Must precede sfc_conv2d_nchw (SFC_ENOTREADY otherwise). */
sfc_status sfc_set_output_scale(sfc_plan_t* plan, float y_scale);

/* Abs-max calibration helpers (the paper tunes scales with AdaQuant on real
 * data; abs-max over a calibration tensor stands in): scale = max|value|/qmax
 * (qmax = 127, or 2^(transform_bits-1) - 1),
 * 1 where the maximum is 0.  Both block until the result is in host memory.
 * workspace_dev holds workspace_bytes bytes, at least the plan's workspace size
 * (SFC_EWORKSPACE otherwise, nothing launched); n_images <= the plan's N. */
sfc_status sfc_calibrate_act_scales(const sfc_plan_t* plan, const int8_t* x_dev, int32_t n_images,
                                    void* workspace_dev, size_t workspace_bytes, void* stream,
                                    float* sx_host_out /*[P]*/);
sfc_status sfc_calibrate_filter_scales(const sfc_plan_t* plan, const int8_t* w_dev,
                                       void* workspace_dev, size_t workspace_bytes, void* stream,
                                       float* sw_host_out /*[P*Cout]*/);

/* Scale granularities of the ablation study (Sec. 6, "Ablation Study on Quantization
 * Granularity"): activations per tensor or per frequency (= per multiplication point),
 * filters per output channel, per frequency, or per channel and frequency (Sec. 5's
 * [T x T] and [OC x T x T] factors are the finest of each). */
typedef enum { SFC_ACT_PER_TENSOR = 0, SFC_ACT_PER_POINT = 1 } sfc_act_granularity;
typedef enum {
  SFC_FILTER_PER_CHANNEL = 0,
  SFC_FILTER_PER_POINT = 1,
  SFC_FILTER_PER_CHANNEL_POINT = 2
} sfc_filter_granularity;

/* Host only, in place.  Coarsens the finest-granularity abs-max scales (as the calibration
 * helpers return them) to the requested grouping: every scale becomes the maximum over its
 * group, which is the abs-max scale of the group because all scales share the divisor qmax.
 * sx_host [P]: per tensor -> all P entries equal.  sw_host [P*Cout] laid out [P][Cout]: per
 * channel -> the maximum over points for each Cout; per point -> the maximum over Cout for
 * each point.  The finest settings leave the arrays as they are.  The result is what
 * sfc_set_point_scales takes, so every granularity runs on the same kernels. */
sfc_status sfc_group_scales(const sfc_plan_t* plan, int32_t act_granularity,
                            int32_t filter_granularity, float* sx_host, float* sw_host);

/* Filter transform U = G f G^T (Appendix A's G, additions only), once per layer.
 * w_dev: int8 [Cout,Cin,R,R].  wscale_host: [1] or [Cout] spatial-domain filter
 * scales.  filter_dev: filter_bytes bytes, at least the plan's filter size
 * (SFC_EWORKSPACE otherwise, nothing launched); receives U (int16 in exact mode, rounded
 * to int8 in requantized mode) and the per-point dequantization table; the plan
 * remembers the pointer.  Asynchronous on `stream` apart from a small pageable
 * host-to-device copy.  Requantized mode needs sfc_set_point_scales first
 * (SFC_ENOTREADY otherwise).  Also raises, on the current device, the dynamic-LDS limit of
 * the kernels this plan launches (SFC_EHIP if the device refuses): sfc_conv2d_nchw runs
 * on the device that was current here. */
sfc_status sfc_transform_filter(sfc_plan_t* plan, const int8_t* w_dev, const float* wscale_host,
                                void* filter_dev, size_t filter_bytes, void* stream);

/* The hot path: input-tile transform V = B^T x B, P products
 * M_p[tiles x Cout] = V_p[tiles x Cin] . U_p[Cin x Cout], output transform with
 * the correction terms, dequantization and the NCHW store.
 * x_dev: int8 [N,Cin,H,W]; x_scale: spatial-domain activation scale.
 * y_dev: float32 (SFC_OUT_F32), int32 (SFC_OUT_I32) or int8 (SFC_OUT_I8_RELU) [N,Cout,H,W].
 * workspace_dev: workspace_bytes bytes, at least the plan's workspace size (SFC_EWORKSPACE
 * otherwise, nothing launched), private to this call until it completes.
 * SFC_ENOTREADY before sfc_transform_filter. */
sfc_status sfc_conv2d_nchw(const sfc_plan_t* plan, const int8_t* x_dev, float x_scale, void* y_dev,
                           void* workspace_dev, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace along (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same work as
 * sfc_conv2d_nchw with the workspace taken from a buffer of SFC_STATIC_WORKSPACE_BYTES that
 * is part of the library's code object, one copy per GPU, held until the process ends.  The
 * call allocates and frees nothing.  Plans whose workspace is larger are refused with
 * SFC_EWORKSPACE before any launch.  Every call on a GPU shares that GPU's buffer: calls that
 * overlap on one GPU (different streams, or threads) race; calls queued on one stream do
 * not.  V (and M) of the previous call are overwritten, nothing needs clearing. */
#define SFC_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
sfc_status sfc_conv2d_nchw_static(const sfc_plan_t* plan, const int8_t* x_dev, float x_scale,
                                  void* y_dev, void* stream);

/* Profiling aid: the same work as sfc_conv2d_nchw restricted to the stages in
 * stage_mask, so that one stage can be timed alone on buffers a full call has
 * filled.  SFC_STAGE_INPUT: V = B^T x B.  SFC_STAGE_PRODUCT: M = V.U (staged path).
 * SFC_STAGE_OUTPUT: y from M (staged path); on the fused path SFC_STAGE_PRODUCT |
 * SFC_STAGE_OUTPUT must be given together and run the one fused kernel; on
 * SFC_PATH_SINGLE only SFC_STAGE_ALL is accepted. */
enum { SFC_STAGE_INPUT = 1, SFC_STAGE_PRODUCT = 2, SFC_STAGE_OUTPUT = 4, SFC_STAGE_ALL = 7 };
sfc_status sfc_conv2d_stages(const sfc_plan_t* plan, const int8_t* x_dev, float x_scale,
                             void* y_dev, void* workspace_dev, size_t workspace_bytes, void* stream,
                             int32_t stage_mask);

/* Where the intermediate tensors of the last call live, for parity checks.
 * which: 0 = V [P][tiles][Cin], 1 = U [P][Cout][Cin], 2 = M [P][tiles][Cout] (int32).
 * ptr receives a device address inside workspace_dev (V, M) or the filter buffer
 * (U); elem_bytes is 1 or 2 for V and U (int8 / int16) and 4 or 3 for M: in requantized
 * mode, when Cin rounded up to 64, times the square of the transform-domain bound
 * 2^(bits-1) - 1, is below 2^23 (int8: up to 512 channels), no sum can reach 2^23 in
 * magnitude and each is kept as a little-endian 24-bit two's complement integer.  The tensor is
 * described as a five-axis strided view (strides in elements): element (p, a, b) of
 * the logical tensor [P][A][B] sits at
 *   p*strides[0] + (a / dims[2])*strides[1] + (a % dims[2])*strides[2]
 *                + (b / dims[4])*strides[3] + (b % dims[4])*strides[4],
 * dims[0] = P, dims[1]*dims[2] >= A and dims[3]*dims[4] >= B (tiles, filters and
 * channels are padded up; entries beyond the true counts are padding).  Plain layouts
 * have dims[2] = dims[4] = 1; in requantized mode M is kept in blocks of 16 tiles x 4
 * filters (the 256 bytes one wave of the output transform reads per point).
 * V exists on SFC_PATH_STAGED and SFC_PATH_FUSED, M only on SFC_PATH_STAGED
 * (SFC_EUNSUPPORTED otherwise). */
sfc_status sfc_tap_info(const sfc_plan_t* plan, const void* workspace_dev, int32_t which,
                        const void** ptr, int32_t* elem_bytes, int64_t dims[5], int64_t strides[5]);

/* Measurement aid: a plain streaming copy of `bytes` (a multiple of 16, both
 * pointers 16-byte aligned) from src_dev to dst_dev on `stream`.  It reads and
 * writes every byte exactly once, so hardware byte counters and achieved-bandwidth
 * figures of the convolution kernels can be calibrated against a kernel of known
 * traffic on the same device. */
sfc_status sfc_stream_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

const char* sfc_status_string(sfc_status s);

#ifdef __cplusplus
}
#endif
#endif /* SFC_H_ */
