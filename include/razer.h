/*
 * razer.h -- C ABI of the MI355X (gfx950) RaZeR library.
 *
 * RaZeR (Redundant Zero Remapping, arxiv 2501.04052) is NVFP4 with the
 * redundant FP4 zero code turned into a per-block "special value":
 *
 *   element   FP4-E2M1 code S|EE|M (Sec. 4.1, FP4 equation): +-{0,.5,1,1.5,2,3,4,6};
 *             code 0x8 (negative zero) is the remapped one (Sec. 4.2).
 *   block     16 consecutive elements along the last (contraction) axis share one
 *             scale byte (Sec. 3; the evaluated configuration of Sec. 5.1: 16 elements, 8-bit scale);
 *             32, 64 and 128 are accepted too (block-size study of Sec. 5.4):
 *               weights      bit7 = special-value sign, bit6 = special-value selector,
 *                            bits5:0 = E3M3 scale EEE|MMM, value 2^(E-3)(1+M/8), E=0: M/32
 *                            (Sec. 4.1 adopts E3M3 for weights; 2 freed bits, Sec. 4.2)
 *               activations  bit7 = special-value sign, bits6:0 = FP8-E4M3 scale
 *                            EEEE|MMM, value 2^(E-7)(1+M/8), E=0: M/512 (Sec. 4.1, FP8
 *                            equation; 1 freed bit, Sec. 4.2); code 0x7F is never written.
 *   tensor    one FP32 scale = absmax / (Qmax_scale * 6)  (Eq. 1).
 *   special   weights: {+sv[0], +sv[1], -sv[0], -sv[1]} indexed by (sign<<1 | selector);
 *             activations: {+sv[0], -sv[0]} (Sec. 4.2, Sec. 4.4 decoder, App. B.2).
 *   value     x^ = tensor_scale * block_scale * (code == 0x8 ? special : FP4[code]).
 *
 * Storage (dense, row-major, all DEVICE memory, caller-owned):
 *   codes  [rows][cols/2]      uint8, element k even in the LOW nibble, k odd in the high
 *   scales [rows][cols/block]  uint8 as above
 *   tensor_scale               one float
 * i.e. 4.5 bits per element plus 4 bytes at block 16, the NVFP4 footprint (Sec. 4.2);
 * 4 + 8 / block bits in general.
 *
 * Every entry point only enqueues kernels on the HIP stream passed in
 * (hipStream_t cast to void*, NULL = default stream); nothing allocates or
 * synchronizes, and no state is kept from one call to the next (the one
 * exception: the first launch of a large-tile kernel on a device raises that
 * kernel's dynamic-LDS limit, once, thread-safely -- make a first call outside
 * stream capture).  Errors are returned as status codes; no exceptions, no
 * aborts.  Non-finite inputs give unspecified values, no faults.
 */
#ifndef RAZER_H
#define RAZER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RAZER_OK = 0,
    RAZER_ERR_NULL = 1,        /* a required pointer is NULL                        */
    RAZER_ERR_SHAPE = 2,       /* negative size, cols % 32 != 0, ld too small       */
    RAZER_ERR_ALIGN = 3,       /* a pointer or leading dimension is not 16-byte aligned */
    RAZER_ERR_CONFIG = 4,      /* bad format id, dtype or special value             */
    RAZER_ERR_WORKSPACE = 5,   /* workspace missing, misaligned or too small        */
    RAZER_ERR_HIP = 6          /* a kernel launch failed                            */
} razer_status;

typedef enum {
    RAZER_FMT_WEIGHT = 0,      /* E3M3 scale + 2 metadata bits, 4 special values    */
    RAZER_FMT_ACT = 1,         /* E4M3 scale + 1 metadata bit, 2 special values     */
    /* The format of the paper's own weight-only kernel (Sec. 4.3): blocks of 128 elements with ONE
     * FP16 scale whose sign bit and most significant exponent bit hold the 2 metadata bits (4 special
     * values, 4.125 bits per weight).  scales is then [rows][cols/128] little-endian 16-bit words:
     * bit 15 = special-value sign, bit 14 = selector, bits 13..0 = the low 14 bits of an IEEE half
     * (exponent below 16: values up to 2 - 2^-10; the tensor scale of Eq. 1 uses that maximum).
     * block must be 0 or 128; cols a multiple of 128.  A weight format: accepted wherever
     * RAZER_FMT_WEIGHT is, except that razer_linear takes bf16 activations only: wavefront dot products
     * up to 4 activation rows; beyond that matrix-core kernels that multiply bare FP4 operands and fold
     * each block's partial sums with the block's scale in fp32 (no workspace is used up to 64 rows; from
     * 65 rows the usual razer_workspace_bytes rule -- K is cut into slices of whole blocks while tiles are
     * few). */
    RAZER_FMT_WEIGHT_F16 = 2
} razer_format;

typedef enum { RAZER_F32 = 0, RAZER_BF16 = 1 } razer_dtype;

/* Special-value configuration.  Each magnitude must be 6 + an offset that the
 * decoder's 4-bit offset register can hold (multiple of 0.5 in [-3.5, 3.5],
 * Sec. 4.4) and must not be an FP4 value: {2.5,3.5,4.5,5,5.5,6.5,...,9.5}.
 * The paper uses sv = {5, 8} for most models' weights ({5,7}, {5,9} for two)
 * and {5} for activations (App. B.2).  sv[1] is ignored for RAZER_FMT_ACT. */
typedef struct {
    int32_t format;            /* razer_format */
    float sv[2];
    int32_t block;             /* elements per scale byte: 16, 32, 64 or 128; 0 means 16.  cols must be
                                  a multiple of max(32, block).                                         */
    int32_t layout;            /* RAZER_LAYOUT_CANONICAL (0: the storage described above) or
                                  RAZER_LAYOUT_INTERLEAVED (a razer_prepack result, see there)          */
} razer_config;

enum { RAZER_LAYOUT_CANONICAL = 0, RAZER_LAYOUT_INTERLEAVED = 1 };

/* A quantized tensor: device pointers + shape + configuration. */
typedef struct {
    const uint8_t *codes;        /* [rows][cols/2]  */
    const uint8_t *scales;       /* [rows][cols/block] bytes (16-bit words for RAZER_FMT_WEIGHT_F16) */
    const float *tensor_scale;   /* device float    */
    int64_t rows, cols;
    razer_config cfg;
} razer_tensor;

enum { RAZER_OP_QUANTIZE = 0, RAZER_OP_DEQUANT = 1, RAZER_OP_LINEAR = 2, RAZER_OP_LINEAR_W4A4 = 3 };

/* razer_quantize flag: *tensor_scale is an input (a calibrated / static scale)
 * instead of being computed from the tensor's absmax by Eq. 1. */
#define RAZER_GIVEN_TENSOR_SCALE 1u

/* Bytes of device workspace the given operation needs for these sizes
 * (rows x cols operand; m = activation rows for RAZER_OP_LINEAR, else 0).
 * Non-zero for RAZER_OP_LINEAR where K is cut into slices whose fp32 partial
 * sums [slices][m][rows] meet in the workspace and are added in slice order
 * (the number of slices depends on the shape: always ask, do not estimate);
 * 0 means the workspace may be NULL.
 * RAZER_OP_LINEAR_W4A4: what lets razer_linear with a RaZeR activation operand (a_q) take its faster
 * form -- the activation tensor decoded once into the workspace as bf16 (m x cols x 2 bytes, rounded
 * up to 256, plus a 256-byte cell for the product of the two tensor scales), then the weight-only
 * path for this m, whose own RAZER_OP_LINEAR figure is included.  With any smaller workspace that
 * satisfies RAZER_OP_LINEAR the same call runs the single fused kernel instead.  Both forms multiply
 * the same exactly decoded bf16 operands and accumulate in fp32; only the order of the sum differs. */
size_t razer_workspace_bytes(int op, int64_t rows, int64_t cols, int64_t m);

/* The same for razer_linear_grouped with `count` weight matrices of rows[i] x cols (rows is a HOST
 * array): a workspace of this size lets the group run as ONE launch wherever the other conditions
 * listed at razer_linear_grouped hold (the K-slices are then chosen for all matrices together,
 * which can take more than the per-matrix sizes added up), and is also enough for the sequence of
 * razer_linear calls it falls back to.  0 for an invalid count or shape.                        */
size_t razer_workspace_bytes_grouped(int32_t count, const int64_t *rows, int64_t cols, int64_t m);

/* Encoder: Eq. 1 (tensor scale), Eq. 2 (block scale, round-to-nearest-even on
 * the format's scale grid, saturating), Eq. 4 (per block, the special value
 * with the smallest squared error in the scaled domain, fp64 sum over the block's
 * elements in index order, ties to the smallest metadata index) and Eq. 5
 * (round-to-nearest on Q_FP4 U {special}; ties between FP4 values go to the
 * even code, an FP4 value beats the special value on a tie, zero is always
 * code 0).  A block whose scale rounds to 0 is written as all-zero codes.
 * For blocks longer than 16 the fp64 error sum of Eq. 4 likewise runs over the block's elements
 * in index order.
 *   x       device, [rows][ld] elements of dtype (fp32 or bf16), cols used per row
 *   codes, scales, tensor_scale   device outputs (tensor_scale input with the flag)
 *   workspace  device, >= razer_workspace_bytes(RAZER_OP_QUANTIZE, ...) bytes, 16-aligned
 * Requirements: cols % 32 == 0, ld >= cols, x/codes/scales 16-byte aligned,
 * ld * sizeof(elt) % 16 == 0.                                               */
razer_status razer_quantize(const razer_config *cfg, const void *x, int32_t dtype,
                            int64_t rows, int64_t cols, int64_t ld,
                            uint8_t *codes, uint8_t *scales, float *tensor_scale,
                            uint32_t flags, void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/* Decoder (Sec. 3 dequantization identity, Sec. 4.4 decoder): out[r][k] =
 * fp32(tensor_scale * (block_scale * element)), the inner product exact, one
 * fp32 rounding; bf16 output is that fp32 rounded to nearest even.
 *   out   device, [rows][ld] elements of dtype.  ld >= cols, 16-byte aligned rows. */
razer_status razer_dequant(const razer_tensor *t, void *out, int32_t dtype, int64_t ld,
                           void *hip_stream);

/* Quantized linear layer Y = A W^T (Sec. 4.3 weight-only kernels; App. D.3
 * weight-activation).  w is [N][K] in a weight format.  Exactly one of
 *   a_bf16  device bf16 [m][K] dense                      (W4A16), or
 *   a_q     RAZER_FMT_ACT tensor [m][K]                   (W4A4)
 * is non-NULL.  Products are accumulated in fp32 (bf16 matrix cores for large
 * m, wavefront dot products for m <= 4, a decode-once MFMA kernel in between), scaled by the
 * tensor scale(s) and rounded to bf16:  y_bf16 device [m][ld_y], ld_y >= N.
 * The first call on a device that reaches one of the large-tile matrix-core kernels raises that kernel's
 * dynamic-LDS limit (hipFuncSetAttribute, once per kernel and device, race-free): a caller that captures
 * a stream into a HIP graph makes one ordinary call of each shape first.
 * workspace: device, 16-byte aligned, >= razer_workspace_bytes(RAZER_OP_LINEAR, N, K, m) bytes
 * (non-zero where K is split over workgroups and the slices meet in fp32: W4A16 with 5 <= m <= 32,
 * and m > 32 with too few output tiles to occupy the GPU -- ask razer_workspace_bytes; else may be
 * NULL); too small -> RAZER_ERR_WORKSPACE. */
razer_status razer_linear(const razer_tensor *w, const void *a_bf16, const razer_tensor *a_q,
                          int64_t m, void *y_bf16, int64_t ld_y,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Private pre-packed weight layout (the paper shuffles its weights offline so that a thread's loads are
 * contiguous, Sec. 4.3).  Here: per row, every run of 2048 elements is stored as its 1024 bytes of codes
 * followed by its 128 scale bytes (a last, shorter run is padded to the same 1152 bytes), so that the
 * scale bytes a wavefront needs travel in the same stream as its codes instead of coming from a second
 * array.  razer_prepack copies a canonical RAZER_FMT_WEIGHT tensor with 16-element blocks into `packed`
 * (device, 16-byte aligned, razer_prepack_bytes(t) bytes = rows * ceil(cols / 2048) * 1152); the result is
 * used as a razer_tensor with codes = packed, scales = NULL, the same tensor_scale, rows, cols and cfg
 * with cfg.layout = RAZER_LAYOUT_INTERLEAVED.  Such a tensor is accepted by razer_linear and
 * razer_linear_grouped (all matrices of a group in the same layout) for the decode regime they are meant
 * for -- bf16 activations, m <= 4, cols <= 32768 -- with results bit-identical to the canonical tensor's;
 * every other use returns RAZER_ERR_CONFIG (keep the canonical tensor for prefill, razer_dequant and W4A4). */
size_t razer_prepack_bytes(const razer_tensor *t);
razer_status razer_prepack(const razer_tensor *t, void *packed, size_t packed_bytes, void *hip_stream);

/* razer_linear for callers that cannot allocate device memory or pass a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the
 * workspace, same kernels, same results; the K-slices meet in a static device array of
 * RAZER_STATIC_WORKSPACE_BYTES that each GPU the library runs on holds until the process ends.
 * Allocates nothing.  Sizes for which razer_workspace_bytes(RAZER_OP_LINEAR, rows, cols, m) exceeds
 * RAZER_STATIC_WORKSPACE_BYTES are refused with RAZER_ERR_WORKSPACE.  All calls on one GPU share that
 * array: calls that overlap in time on one GPU (different streams) race; calls on one stream do not. */
#define RAZER_STATIC_WORKSPACE_BYTES (32u << 20)
razer_status razer_linear_static(const razer_tensor *w, const void *a_bf16, const razer_tensor *a_q,
                                 int64_t m, void *y_bf16, int64_t ld_y, void *hip_stream);

/* The same layer for several weight matrices that consume the SAME activation rows (fused q/k/v,
 * gate/up projections; the paper's stripe partition likewise lets one launch span several N
 * ranges, Sec. 4.3): y_bf16[i] = A w[i]^T for i < count, count <= RAZER_MAX_GROUP.  All w[i] must
 * have the same cols; W4A16 only.  With equal format, block size and special values and no empty
 * matrix this is ONE kernel launch (short kernels are launch-latency-bound, and one launch fills the
 * last round of workgroups of a GEMM better than one per matrix) when
 *   m <= 4 (RAZER_FMT_WEIGHT or RAZER_FMT_WEIGHT_F16);
 *   RAZER_FMT_WEIGHT, 5 <= m <= 32, every rows[i] and ld_y[i] a multiple of 4, y_bf16[i] 8-byte
 *     aligned, and the workspace holds razer_workspace_bytes_grouped(count, rows, cols, m) bytes
 *     (plus one launch that adds the K-slices up); RAZER_FMT_WEIGHT_F16 under the same conditions on
 *     rows, ld_y and y_bf16, without a workspace;
 *   RAZER_FMT_WEIGHT, m >= 33: without a workspace when m > 128 and the matrices together have
 *     >= 512 output tiles of 256 x 128, or 192..256 of them with cols >= 1024; otherwise K is cut into
 *     slices (plus one launch that adds them up) under the conditions of the 5 <= m <= 32 case --
 *     rows, ld_y, alignment of y_bf16, and a workspace of razer_workspace_bytes_grouped bytes.
 * Otherwise it is the sequence of razer_linear calls with the same workspace (which then must
 * satisfy each call).  y_bf16[i] is device [m][ld_y[i]].  The pointer arrays are HOST arrays. */
#define RAZER_MAX_GROUP 4
razer_status razer_linear_grouped(const razer_tensor *const *w, int32_t count, const void *a_bf16,
                                  int64_t m, void *const *y_bf16, const int64_t *ld_y,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

const char *razer_status_string(razer_status s);

#ifdef __cplusplus
}
#endif
#endif /* RAZER_H */
