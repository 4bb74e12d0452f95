/*
 * escoin.h -- C ABI of the MI355X (gfx950) direct sparse convolution library.
 *
 * The library computes one pruned convolution layer without lowering it to a matrix
 * product: the M x (C*R*S) filter matrix is held in CSR, one row per output channel
 * (Section 2.3), its column indices are "stretched" once into offsets of a zero-padded
 * 1-D input array (Section 3.1), and the output is accumulated nonzero by nonzero as in
 * Algorithm 2.  Shape names follow Table 1: N batch, M filters / ofmap channels, C ifmap
 * channels, H/W ifmap height/width, R/S filter height/width, E/F ofmap height/width.
 *
 * Conventions for every entry point
 *   - All tensors are contiguous fp32 NCHW (filters MCRS); all indices are int32.
 *   - Hp = H + 2*pad, Wp = W + 2*pad, E = (Hp - R)/stride + 1, F = (Wp - S)/stride + 1.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory on
 *     the current device.  The library owns no memory: every buffer is the caller's and
 *     must stay valid until the stream work that uses it has finished.
 *   - Device entry points enqueue on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream), never synchronise and never allocate.
 *   - Every call returns ESCOIN_OK (0) or a negative code; nothing throws or aborts.  On an
 *     error no kernel is launched and no output is written.
 *   - Output buffers are overwritten (no accumulation into their previous contents) and
 *     must not alias any input.
 */
#ifndef ESCOIN_H
#define ESCOIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct escoin_conv_desc {
    int32_t N, C, H, W; /* input  N x C x H x W (unpadded)                     */
    int32_t M, R, S;    /* filter M x C x R x S                                */
    int32_t stride;     /* same stride on both axes, >= 1                      */
    int32_t pad;        /* symmetric zero padding on all four sides, >= 0      */
} escoin_conv_desc;

enum {
    ESCOIN_OK = 0,
    ESCOIN_EINVAL = -1, /* null pointer, non-positive dim, malformed CSR, bad flags   */
    ESCOIN_ERANGE = -2, /* an index would not fit int32 (C*Hp*Wp, M*E*F or nnz)       */
    ESCOIN_EHIP = -3,   /* a HIP call (launch, attribute query) failed                */
    ESCOIN_ESIZE = -4   /* a caller-provided buffer is too small                      */
};

enum {
    ESCOIN_F_BIAS = 1u, /* add bias[m] to every element of output channel m          */
    ESCOIN_F_RELU = 2u  /* clamp the result at zero: x > 0 ? x : 0                    */
};

/* Human-readable text for a return code (static storage, never NULL). */
const char *escoin_strerror(int code);

/* Validates a descriptor: ESCOIN_EINVAL for non-positive dims / stride < 1 / pad < 0 /
 * filter larger than the padded input, ESCOIN_ERANGE when C*Hp*Wp or M*E*F reaches 2^31. */
int escoin_check_desc(const escoin_conv_desc *desc);

/* Output extent E, F (Eq. 1 generalised by padding and stride).  Returns a code. */
int escoin_output_dims(const escoin_conv_desc *desc, int32_t *E, int32_t *F);

/* Element counts of the padded input N*C*Hp*Wp and of the output N*M*E*F; 0 on a bad desc. */
size_t escoin_padded_elems(const escoin_conv_desc *desc);
size_t escoin_output_elems(const escoin_conv_desc *desc);

/*
 * Weight stretching (Section 3.1).  Host, pure, run once per (layer, input size).
 * Each column index j = (c*R + r)*S + s of the M x CRS filter matrix is rewritten to the
 * CHW layout offset f(c, r, s) = (c*Hp + r)*Wp + s of the padded input; `value` and
 * `rowptr` are unchanged and the map is element-wise and order-preserving (entries may be
 * in any order inside a row and may repeat).
 *   rowptr            host, M+1 entries, rowptr[0] == 0, non-decreasing
 *   colidx            host, nnz = rowptr[M] entries, each in [0, C*R*S)
 *   colidx_stretched  host, nnz entries, caller-owned; may alias colidx (in-place)
 * ESCOIN_EINVAL on a malformed CSR (nothing useful is written then).
 */
int escoin_sconv_pack(const escoin_conv_desc *desc, const int32_t *rowptr, const int32_t *colidx,
                      int32_t *colidx_stretched);

/*
 * pad_in (Sections 3.1 and 4.2): the zero-padded 1-D input array
 *   padded[n][c][y + pad][x + pad] = in[n][c][y][x], +0.0f elsewhere.
 *   d_in      device, N*C*H*W floats
 *   d_padded  device, N*C*Hp*Wp floats, fully overwritten
 * With pad == 0 this is a plain copy.
 */
int escoin_pad_in(const escoin_conv_desc *desc, const float *d_in, float *d_padded,
                  void *hip_stream);

/*
 * sconv, Algorithm 2 as stated, for any filter size / stride and any CSR entry order:
 *   out[n][m][h][w] = sum over j in row m of
 *       value[j] * padded[n][ colidx_stretched[j] + h*stride*Wp + w*stride ]
 * optionally followed by the fused epilogue out = relu(out + bias[m]) (flags).
 *   d_rowptr, d_colidx_stretched, d_value   device CSR (stretched by escoin_sconv_pack)
 *   d_padded  device, N*C*Hp*Wp floats (from escoin_pad_in; the input itself when pad==0)
 *   d_out     device, N*M*E*F floats, overwritten
 *   d_bias    device, M floats; may be NULL unless ESCOIN_F_BIAS is set
 * The CSR on the device is trusted (it was validated by escoin_sconv_pack): offsets outside
 * the padded image are the caller's error.
 */
int escoin_sconv_forward(const escoin_conv_desc *desc, const int32_t *d_rowptr,
                         const int32_t *d_colidx_stretched, const float *d_value,
                         const float *d_padded, float *d_out, const float *d_bias,
                         uint32_t flags, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * LDS-tiled sconv: the same result as escoin_sconv_forward, computed from the UNPADDED input
 * (the zero frame of pad_in is produced while the input window is staged on chip, so the
 * padded array of Section 3.1 only ever exists tile by tile in LDS).  It needs a plan: a
 * kernel-specific re-encoding of the stretched CSR (nonzeros regrouped by input-channel chunk
 * and row bin, offsets re-stretched to the on-chip window; Section 3.3's "weights stationary,
 * inputs streamed" with Section 4.3's tiling).  The stretched CSR stays the externally
 * visible, bit-exact packing result; the plan is derived data and opaque.
 * ------------------------------------------------------------------------------------------ */

/* Tiling knobs; a zero field means "choose for me".  Out-of-range combinations make the plan
 * calls return ESCOIN_EINVAL / ESCOIN_ERANGE (e.g. a window that does not fit LDS). */
typedef struct escoin_sconv_tuning {
    int32_t K;  /* output channels accumulated per wave: 1, 2, 4 or 8               */
    int32_t Q;  /* 16-byte position groups per lane, 1 or 2                         */
    int32_t B;  /* nonzeros per record batch, 2 or 4 (not every K/Q/B mix exists)   */
    int32_t WM; /* waves per workgroup along the output-channel axis (WS included)  */
    int32_t CC; /* input channels staged per LDS chunk                              */
    int32_t NB; /* images per workgroup                                             */
    int32_t TH; /* output rows per tile                                             */
    int32_t CS; /* workgroups sharing one output tile, each taking every CS-th      */
                /* channel chunk and adding its partial sums with float atomics     */
    int32_t WS; /* every output channel's nonzeros are split over at least WS waves */
                /* of a workgroup, whose partial sums are added in LDS (rows much   */
                /* longer than a wave's share are split further by the library)     */
    int32_t CC0;/* input channels of the first chunk, <= CC (a short first chunk    */
                /* lets the arithmetic start before the whole window has arrived)   */
} escoin_sconv_tuning;

/* Bytes the plan blob needs.  Host; rowptr / colidx_stretched as returned by
 * escoin_sconv_pack (any order inside a row, duplicates allowed); tuning may be NULL. */
int escoin_sconv_plan_size(const escoin_conv_desc *desc, const int32_t *rowptr,
                           const int32_t *colidx_stretched, const escoin_sconv_tuning *tuning,
                           size_t *plan_bytes);

/* Builds the plan into caller-owned host memory `plan` (plan_bytes from the size query, else
 * ESCOIN_ESIZE).  A plan is valid for every batch size (only C, H, W, M, R, S, stride and pad are
 * checked at launch); desc->N only guides the default tiling.  The caller then copies the blob
 * verbatim to device memory (256-byte aligned) and keeps the host copy for escoin_sconv_forward_tiled.
 * ESCOIN_EINVAL if an offset is not one weight stretching can produce for this desc. */
int escoin_sconv_plan_build(const escoin_conv_desc *desc, const int32_t *rowptr,
                            const int32_t *colidx_stretched, const float *value,
                            const escoin_sconv_tuning *tuning, void *plan, size_t plan_bytes);

/*
 * out[n][m][h][w] = sum_j value[j] * Ipad[n][...]  (Algorithm 2 / Eq. 1 with zero padding and
 * stride), optional fused epilogue as in escoin_sconv_forward.
 *   plan_host  host copy of the blob (only its header is read, synchronously)
 *   d_plan     device copy of the same blob
 *   d_in       device, N*C*H*W floats, UNPADDED
 *   d_out      device, N*M*E*F floats, overwritten
 * ESCOIN_EINVAL if the plan was built for another layer geometry.
 *
 * By default a launch that would leave compute units idle (small batches) splits every output
 * channel's nonzeros over several waves of a workgroup and adds their partial sums on chip: one
 * kernel, and the same bits on every run.
 *
 * A plan with CS > 1 (only on request, through the tuning) splits the input channels of a tile
 * over CS workgroups instead.  The call then enqueues three kernels: a zero fill of d_out, the
 * convolution, whose workgroups add their partial sums with fp32 atomics (the order of those
 * additions, and with it the last bits of the result, may differ from run to run), and, with
 * ESCOIN_F_RELU, the clamp as a pass of its own.
 *
 * d_in and d_plan that are 16-byte aligned let the kernel stage with 16-byte loads (or with
 * global -> LDS copies); any 4-byte aligned pointer is accepted.
 */
int escoin_sconv_forward_tiled(const escoin_conv_desc *desc, const void *plan_host,
                               const void *d_plan, const float *d_in, float *d_out,
                               const float *d_bias, uint32_t flags, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ESCOIN_H */
