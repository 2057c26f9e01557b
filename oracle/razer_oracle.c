/*
 * RaZeR reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, scalar CPU implementation of the RaZeR number format
 * (arxiv 2501.04052): the FP4-E2M1 element table, the FP8-E4M3 / E3M3 block
 * scale codecs, the per-tensor FP32 scale, the block encoder with its
 * special-value search, the decoder and the quantized linear layer.  It is
 * what the HIP library is checked against; it shares no code, header, table
 * or helper with that library, and only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * Every function names the passage of the paper it follows.  Where the paper
 * is silent the reading taken is stated next to the code.  Arithmetic is
 * IEEE-754: fp32 where the format itself is fp32 (Eq. 1-3 operate on "FP32"
 * tensors), fp64 for every error sum and for the reference matmul.  Compile
 * with -ffp-contract=off and without -ffast-math.
 *
 * Parity pins (tests/test_oracle_*.py): every function here is pinned to
 * something other than itself -- the value sets the paper prints, the decoder
 * worked example, the two-pass identity of App. D.3, a library FP8 cast, brute
 * force over all 16 decoded values, and the never-worse-than-NVFP4 invariant.
 * The paper's accuracy results (perplexity etc.) are not reproduced anywhere
 * in this build: parity unpinned for those, by construction out of scope.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define RAZER_BLOCK 16           /* elements per block of the evaluated format (Sec. 3, Sec. 5.1) */
#define RAZER_MAX_BLOCK 128      /* largest block of the block-size study (Sec. 5.4, "Impact of Block Size") */

/* Block sizes of the paper's block-size study: 16, 32, 64, 128 (Sec. 5.4). */
static int block_ok(int block) { return block == 16 || block == 32 || block == 64 || block == 128; }
#define REMAP_CODE 0x8           /* the redundant zero: sign=1, E=0, M=0   */

/* FMT_WEIGHT_F16: the format of the paper's own weight-only kernel (Sec. 4.3): blocks of 128 with one
 * FP16 scale whose sign bit and most significant exponent bit hold the 2 metadata bits. */
enum { FMT_WEIGHT = 0, FMT_ACT = 1, FMT_WEIGHT_F16 = 2 };
static int is_weight(int fmt) { return fmt != FMT_ACT; }

/* ------------------------------------------------------------------ */
/* Number formats                                                      */
/* ------------------------------------------------------------------ */

/* FP4-E2M1 value of a 4-bit code S|EE|M  (Sec. 4.1, the FP4 equation):
 *   E != 0: (-1)^S 2^(E-1) (1 + M/2);   E == 0: (-1)^S M/2.               */
double oracle_fp4_value(int code)
{
    int S = (code >> 3) & 1, E = (code >> 1) & 3, M = code & 1;
    double mag = (E != 0) ? ldexp(1.0 + M / 2.0, E - 1) : M / 2.0;
    return S ? -mag : mag;
}

/* FP8-E4M3 magnitude of the 7 bits EEEE|MMM (Sec. 4.1, the FP8 equation; the
 * sign bit is the redundant one and is not part of the code here):
 *   E != 0: 2^(E-7) (1 + M/8);   E == 0: 2^-6 M/8.
 * Code 0x7F is the NaN of the OCP format the paper cites and is never
 * produced, so the largest scale is 448 (code 0x7E).                       */
double oracle_e4m3_value(int code7)
{
    int E = (code7 >> 3) & 15, M = code7 & 7;
    return (E != 0) ? ldexp(1.0 + M / 8.0, E - 7) : ldexp(M / 8.0, -6);
}

/* E3M3 magnitude of the 6 bits EEE|MMM (Sec. 4.1 adopts "E3M3" for weight
 * scales without printing its value formula).  Reading: the same IEEE-like
 * shape as the FP8 equation with bias 3, subnormals, no Inf/NaN:
 *   E != 0: 2^(E-3) (1 + M/8);   E == 0: 2^-2 M/8.      max = 30, min = 1/32 */
double oracle_e3m3_value(int code6)
{
    int E = (code6 >> 3) & 7, M = code6 & 7;
    return (E != 0) ? ldexp(1.0 + M / 8.0, E - 3) : ldexp(M / 8.0, -2);
}

/* FP16 magnitude with its most significant exponent bit given away (Sec. 4.3: "sign bit and the most
 * significant exponent bit ... store the 2-bit metadata"): the 14 bits EEEE|MMMMMMMMMM of an IEEE half
 * whose exponent field is below 16, i.e. bias 15:
 *   E != 0: 2^(E-15) (1 + M/1024);   E == 0: 2^-14 M/1024.      max = 2 - 2^-10, all codes finite   */
double oracle_e4m10_value(int code14)
{
    int E = (code14 >> 10) & 15, M = code14 & 1023;
    return (E != 0) ? ldexp(1.0 + M / 1024.0, E - 15) : ldexp(M / 1024.0, -14);
}

/* Number of usable scale codes and the scale decoder per format. */
static int scale_ncodes(int fmt) { return fmt == FMT_WEIGHT ? 64 : fmt == FMT_ACT ? 127 : 16384; }
double oracle_scale_value(int fmt, int code)
{
    return fmt == FMT_WEIGHT ? oracle_e3m3_value(code) : fmt == FMT_ACT ? oracle_e4m3_value(code)
                                                                          : oracle_e4m10_value(code);
}
/* Q_max^FP8 of Eq. 1: the largest block-scale value. */
double oracle_scale_max(int fmt) { return oracle_scale_value(fmt, scale_ncodes(fmt) - 1); }

/* The rounding function of Eq. 2 for block scales: nearest representable
 * scale; on an exact tie the even code; beyond the grid the largest code. */
int oracle_round_scale(int fmt, float t)
{
    int n = scale_ncodes(fmt), best = 0;
    double bd = fabs((double)t - oracle_scale_value(fmt, 0));
    for (int c = 1; c < n; ++c) {
        double d = fabs((double)t - oracle_scale_value(fmt, c));
        if (d < bd || (d == bd && (c & 1) == 0 && (best & 1) == 1)) { bd = d; best = c; }
    }
    return best;
}

/* Special value reconstructed the way the decoder of Sec. 4.4 does it: a 4-bit
 * offset register (1 sign, 2 integer, 1 fraction bit; sign-magnitude, step
 * 0.5, range +-3.5) is added to 6.0, the largest FP4 value.                 */
double oracle_sv_from_offset_reg(int reg4)
{
    double off = ((reg4 & 7) * 0.5);
    if (reg4 & 8) off = -off;
    return 6.0 + off;
}
/* Inverse: the offset register for a magnitude, or -1 when the magnitude is
 * not 6 + a multiple of 0.5 within +-3.5, or coincides with an FP4 value.   */
int oracle_offset_reg_from_sv(double mag)
{
    for (int reg = 0; reg < 16; ++reg) {
        if (reg == 8) continue;                      /* "-0" offset: same as 0 */
        if (oracle_sv_from_offset_reg(reg) == mag) {
            for (int c = 0; c < 8; ++c) if (oracle_fp4_value(c) == mag) return -1;
            return reg;
        }
    }
    return -1;
}

/* Candidate special values of a format (Sec. 4.2): weights carry 2 metadata
 * bits -> {+sv0, +sv1, -sv0, -sv1} (bit 1 = sign, bit 0 = selector, matching
 * the decoder's "1-bit selector" and "1-bit sign"); activations carry 1 bit
 * -> {+sv0, -sv0}.  nsv == 0 gives plain NVFP4 (no remap) as a comparator.  */
static int candidates(int fmt, const double sv[2], int nsv_override, double cand[4])
{
    int n = is_weight(fmt) ? 4 : 2;
    if (nsv_override >= 0 && nsv_override < n) n = nsv_override;
    if (is_weight(fmt)) { cand[0] = sv[0]; cand[1] = sv[1]; cand[2] = -sv[0]; cand[3] = -sv[1]; }
    else                   { cand[0] = sv[0]; cand[1] = -sv[0]; cand[2] = cand[3] = 0; }
    return n;
}
double oracle_candidate(int fmt, double sv0, double sv1, int meta)
{
    double sv[2] = { sv0, sv1 }, cand[4];
    candidates(fmt, sv, -1, cand);
    return cand[meta & 3];
}

static int meta_shift(int fmt) { return fmt == FMT_WEIGHT ? 6 : fmt == FMT_ACT ? 7 : 14; }
/* Scale storage: one byte per block, or one little-endian 16-bit word for the FP16-scale format. */
static int get_scale_word(int fmt, const uint8_t *scales, int64_t idx)
{
    return fmt == FMT_WEIGHT_F16 ? (scales[2 * idx] | (scales[2 * idx + 1] << 8)) : scales[idx];
}
static void put_scale_word(int fmt, uint8_t *scales, int64_t idx, int word)
{
    if (fmt == FMT_WEIGHT_F16) { scales[2 * idx] = (uint8_t)(word & 255); scales[2 * idx + 1] = (uint8_t)(word >> 8); }
    else scales[idx] = (uint8_t)word;
}

/* Decoded element of a block (Sec. 4.4 step 3): the remapped zero code gives
 * the block's special value, every other code its FP4 value.               */
double oracle_element_value(int fmt, double sv0, double sv1, int code, int meta)
{
    return (code == REMAP_CODE) ? oracle_candidate(fmt, sv0, sv1, meta) : oracle_fp4_value(code);
}

/* ------------------------------------------------------------------ */
/* Rounding of one scaled element to Q^FP4 U {v}  (Eq. 4 / Eq. 5)       */
/* ------------------------------------------------------------------ */

/* Nearest member of the 15 distinct FP4 values, optionally joined by one
 * special value v.  Returns the 4-bit code (REMAP_CODE for v) and the signed
 * error xs - q in *err.  Ties: a base value beats the special value, and of
 * two base values the one with the even code wins; zero is always code 0.   */
static int round_elem(float xs, int have_v, double v, double *err)
{
    int best = 0;
    double be = (double)xs - oracle_fp4_value(0);
    for (int c = 1; c < 16; ++c) {
        if (c == REMAP_CODE) continue;               /* -0 is not a value of its own */
        double e = (double)xs - oracle_fp4_value(c);
        if (fabs(e) < fabs(be) || (fabs(e) == fabs(be) && (c & 1) == 0 && (best & 1) == 1)) {
            be = e; best = c;
        }
    }
    if (have_v) {
        double e = (double)xs - v;
        if (fabs(e) < fabs(be)) { be = e; best = REMAP_CODE; }
    }
    *err = be;
    return best;
}
int oracle_round_fp4(float xs)                       /* plain Eq. 3 rounding */
{
    double e;
    return round_elem(xs, 0, 0.0, &e);
}
int oracle_round_fp4_sv(float xs, double v, double *err)
{
    return round_elem(xs, 1, v, err);
}

static float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4); return f;
}

/* Round a double to bfloat16 (8 significant bits, exponent range of fp32),
 * ties to even, one rounding only.                                         */
uint16_t oracle_f64_to_bf16(double x)
{
    if (x != x) return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    int e; frexp(a, &e);                             /* a = f 2^e, f in [0.5,1) */
    int qexp = e - 8;                                /* quantum for 8 significant bits */
    if (qexp < -133) qexp = -133;                    /* subnormal spacing 2^-133 */
    double r = nearbyint(ldexp(a, -qexp));           /* default mode: to nearest even */
    double y = ldexp(r, qexp);
    if (y >= ldexp(1.0, 128)) return sign | 0x7F80;
    float f = (float)y; uint32_t u; memcpy(&u, &f, 4);
    return sign | (uint16_t)(u >> 16);
}

/* ------------------------------------------------------------------ */
/* Encoder                                                             */
/* ------------------------------------------------------------------ */

/* Eq. 1: tensor-wise scale = absmax / (Qmax^FP8 * Qmax^FP4), one fp32
 * division by the constant; an all-zero tensor gets scale 1.               */
float oracle_tensor_scale(int fmt, const void *x, int x_is_bf16, int64_t n)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float v = x_is_bf16 ? bf16_to_f32(((const uint16_t *)x)[i]) : ((const float *)x)[i];
        float a = fabsf(v);
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) return 1.0f;
    float denom = (float)(oracle_scale_max(fmt) * 6.0);        /* 180 or 2688 */
    return amax / denom;
}

/* One block of `block` elements (16 in the evaluated format; 32, 64, 128 in the
 * block-size study of Sec. 5.4): Eq. 2 (block scale), the scaling that defines
 * X^Scaled, Eq. 4 (special-value search) and Eq. 5 (final rounding).
 *   delta32 : the tensor scale.   nsv: number of candidates searched
 *   (0 = plain NVFP4 under the same scale).
 * Outputs: the codes, the 6/7-bit scale code, the metadata index, and the
 * block's squared error in the scaled domain.  Eq. 4's squared-error norm is
 * the plain sum over the block's elements in index order k = 0 .. block-1, in
 * fp64 (the paper does not give an order; index order is the one the formula
 * is written in).                                                           */
static double sse_in_order(const double *e2, int block)
{
    double total = 0.0;
    for (int k = 0; k < block; ++k) total += e2[k];
    return total;
}

static void encode_block(int fmt, const double cand[4], int nsv, float delta32, int block,
                         const float *xb, uint8_t *codes,
                         int *scale_code, int *meta, double *sse_out)
{
    float bmax = 0.0f;
    for (int k = 0; k < block; ++k) { float a = fabsf(xb[k]); if (a > bmax) bmax = a; }

    /* Eq. 2: t = bmax / (delta32 * Qmax^FP4), rounded to the scale grid. */
    float d = delta32 * 6.0f;
    float t = bmax / d;
    int sc = oracle_round_scale(fmt, t);
    float s = (float)oracle_scale_value(fmt, sc);
    *scale_code = sc;
    *meta = 0;
    if (s == 0.0f) {                                 /* scale underflowed to 0: block decodes to zeros */
        for (int k = 0; k < block; ++k) { codes[k] = 0; }
        *sse_out = 0.0;
        return;
    }
    /* X^Scaled = X / (delta32 * delta8)  (denominator of Eq. 3). */
    float den = delta32 * s;
    float xs[RAZER_MAX_BLOCK];
    double e2[RAZER_MAX_BLOCK];
    for (int k = 0; k < block; ++k) xs[k] = xb[k] / den;

    if (nsv == 0) {                                  /* Eq. 3 alone: NVFP4 */
        for (int k = 0; k < block; ++k) {
            double e; codes[k] = (uint8_t)round_elem(xs[k], 0, 0.0, &e); e2[k] = e * e;
        }
        *sse_out = sse_in_order(e2, block);
        return;
    }
    /* Eq. 4: try every allowed special value, keep the smallest squared
     * error; on equal error the smallest metadata index.                  */
    double best_sse = 0.0; int best_m = -1;
    for (int m = 0; m < nsv; ++m) {
        for (int k = 0; k < block; ++k) {
            double e; (void)round_elem(xs[k], 1, cand[m], &e); e2[k] = e * e;
        }
        double sse = sse_in_order(e2, block);
        if (best_m < 0 || sse < best_sse) { best_sse = sse; best_m = m; }
    }
    /* Eq. 5: quantize the block with the chosen special value. */
    for (int k = 0; k < block; ++k) {
        double e; codes[k] = (uint8_t)round_elem(xs[k], 1, cand[best_m], &e);
    }
    *meta = best_m;
    *sse_out = best_sse;
}

/* Whole-tensor encoder.  x is [rows][cols] dense, fp32 or bf16 (widened
 * exactly); blocks of `block` elements run along cols.  Layout written:
 *   codes  [rows][cols/2]      element k even -> low nibble, odd -> high nibble
 *   scales [rows][cols/block]  weights: meta<<6 | E3M3; activations: meta<<7 | E4M3;
 *                              FP16-scale weights: 16-bit words meta<<14 | E4M10
 *   *tensor_scale              Eq. 1 (taken as input when given_scale != 0)
 *   block_sse (optional)       [rows][cols/block] squared error in the scaled domain
 * nsv_override < 0 searches the format's full candidate set; 0 = NVFP4.
 * Returns 0, or -1 on a bad shape or block size.                           */
int oracle_quantize(int fmt, double sv0, double sv1, int nsv_override,
                    const void *x, int x_is_bf16, int64_t rows, int64_t cols, int block,
                    uint8_t *codes, uint8_t *scales, float *tensor_scale,
                    int given_scale, double *block_sse)
{
    if (!block_ok(block) || rows < 0 || cols < 0 || cols % block) return -1;
    if (fmt == FMT_WEIGHT_F16 && block != 128) return -1;       /* Sec. 4.3: block size 128 */
    double sv[2] = { sv0, sv1 }, cand[4];
    int nsv = candidates(fmt, sv, nsv_override, cand);
    float delta32 = given_scale ? *tensor_scale : oracle_tensor_scale(fmt, x, x_is_bf16, rows * cols);
    if (!given_scale) *tensor_scale = delta32;
    int64_t nb = cols / block;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t b = 0; b < nb; ++b) {
            float xb[RAZER_MAX_BLOCK]; uint8_t cb[RAZER_MAX_BLOCK]; int sc, meta; double sse;
            for (int k = 0; k < block; ++k) {
                int64_t idx = r * cols + b * block + k;
                xb[k] = x_is_bf16 ? bf16_to_f32(((const uint16_t *)x)[idx]) : ((const float *)x)[idx];
            }
            encode_block(fmt, cand, nsv, delta32, block, xb, cb, &sc, &meta, &sse);
            for (int k = 0; k < block; k += 2)
                codes[(r * cols + b * block + k) / 2] = (uint8_t)(cb[k] | (cb[k + 1] << 4));
            put_scale_word(fmt, scales, r * nb + b, (meta << meta_shift(fmt)) | sc);
            if (block_sse) block_sse[r * nb + b] = sse;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Decoder                                                             */
/* ------------------------------------------------------------------ */

/* The un-numbered dequantization identity of Sec. 3:
 *   x^ = delta32 * delta8_i * xbar,   xbar the decoded element (Sec. 4.4).
 * delta8_i * xbar is exact in fp64 (and in fp32); the product with delta32 is
 * rounded once to fp32 (out_f32) and from there to bf16 (out_bf16).  Also
 * returns the unscaled product delta8_i * xbar in out_sq when not NULL.     */
int oracle_dequant(int fmt, double sv0, double sv1,
                   const uint8_t *codes, const uint8_t *scales, float tensor_scale,
                   int64_t rows, int64_t cols, int block,
                   float *out_f32, uint16_t *out_bf16, double *out_sq)
{
    if (!block_ok(block) || rows < 0 || cols < 0 || cols % block) return -1;
    int64_t nb = cols / block;
    int sh = meta_shift(fmt);
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t k = 0; k < cols; ++k) {
            uint8_t byte = codes[(r * cols + k) / 2];
            int code = (k & 1) ? (byte >> 4) : (byte & 15);
            int sb = get_scale_word(fmt, scales, r * nb + k / block);
            int meta = sb >> sh, sc = sb & ((1 << sh) - 1);
            double sq = oracle_scale_value(fmt, sc) * oracle_element_value(fmt, sv0, sv1, code, meta);
            float w = (float)((double)tensor_scale * sq);   /* exact product rounded once */
            if (out_sq) out_sq[r * cols + k] = sq;
            if (out_f32) out_f32[r * cols + k] = w;
            if (out_bf16) out_bf16[r * cols + k] = oracle_f64_to_bf16((double)w);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Linear layer                                                        */
/* ------------------------------------------------------------------ */

/* Y = A W^T with W [n][k] RaZeR-quantized (Sec. 4.3: weight-only kernel;
 * App. D.3: weight-activation).  The plain definition: every product formed
 * exactly in fp64, summed over k ascending in fp64, scaled by the tensor
 * scale(s), then rounded once to bf16.
 *   a_bf16 != NULL : W4A16, activations [m][k] bf16.
 *   a_codes != NULL: W4A4, activations RaZeR-quantized in the activation
 *                    format with special value a_sv0.
 * w_block / a_block: elements per block scale of each operand (16 in the
 * evaluated format; Sec. 5.4 also studies 32, 64, 128).
 * Outputs y_f64 [m][n] (optional) and y_bf16 [m][n] (optional).  When
 * n_cols_sel > 0 only the listed output columns / rows are computed
 * (sampled check of large problems); outputs are then [m_sel][n_sel].      */
int oracle_linear(int w_fmt, double w_sv0, double w_sv1,
                  const uint8_t *w_codes, const uint8_t *w_scales, float w_tensor_scale,
                  int64_t n, int64_t k, int w_block,
                  const uint16_t *a_bf16,
                  double a_sv0, const uint8_t *a_codes, const uint8_t *a_scales, float a_tensor_scale,
                  int a_block, int64_t m,
                  const int64_t *row_sel, int64_t m_sel, const int64_t *col_sel, int64_t n_sel,
                  double *y_f64, uint16_t *y_bf16)
{
    if (!block_ok(w_block) || k % w_block || (!a_bf16 == !a_codes) || !is_weight(w_fmt)) return -1;
    const int wsh = meta_shift(w_fmt);
    if (a_codes && (!block_ok(a_block) || k % a_block)) return -1;
    int64_t nb = k / w_block, nba = a_codes ? k / a_block : 0;
    int64_t mm = row_sel ? m_sel : m, nn = col_sel ? n_sel : n;
    #pragma omp parallel for schedule(static)
    for (int64_t jn = 0; jn < nn; ++jn) {
        int64_t col = col_sel ? col_sel[jn] : jn;
        for (int64_t im = 0; im < mm; ++im) {
            int64_t row = row_sel ? row_sel[im] : im;
            double acc = 0.0;
            for (int64_t kk = 0; kk < k; ++kk) {
                uint8_t wb = w_codes[(col * k + kk) / 2];
                int wc = (kk & 1) ? (wb >> 4) : (wb & 15);
                int ws = get_scale_word(w_fmt, w_scales, col * nb + kk / w_block);
                double wq = oracle_scale_value(w_fmt, ws & ((1 << wsh) - 1)) *
                            oracle_element_value(w_fmt, w_sv0, w_sv1, wc, ws >> wsh);
                double av;
                if (a_bf16) {
                    av = (double)bf16_to_f32(a_bf16[row * k + kk]);
                } else {
                    uint8_t ab = a_codes[(row * k + kk) / 2];
                    int ac = (kk & 1) ? (ab >> 4) : (ab & 15);
                    uint8_t as = a_scales[row * nba + kk / a_block];
                    av = oracle_scale_value(FMT_ACT, as & 127) *
                         oracle_element_value(FMT_ACT, a_sv0, 0.0, ac, as >> 7);
                }
                acc += av * wq;
            }
            double y = (double)w_tensor_scale * acc;
            if (a_codes) y *= (double)a_tensor_scale;
            if (y_f64) y_f64[im * nn + jn] = y;
            if (y_bf16) y_bf16[im * nn + jn] = oracle_f64_to_bf16(y);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Two-pass decomposition of App. D.3 (used only as a pin of the decoder) */
/* ------------------------------------------------------------------ */

/* Splits one RaZeR weight code into two plain FP4 codes (B_main, B_comp) for
 * special values that are a sum of two FP4 values of the same sign:
 * main_mag + comp_mag[selector].  Non-remapped codes stay in B_main and are
 * masked to zero in B_comp.  Returns 0 on success.                         */
int oracle_two_pass_split(int code, int meta, int main_code_mag, const int comp_code_mag[2],
                          int *b_main, int *b_comp)
{
    if (code != REMAP_CODE) { *b_main = code; *b_comp = 0; return 0; }
    int sign = (meta >> 1) & 1, sel = meta & 1;
    *b_main = (sign << 3) | main_code_mag;
    *b_comp = (sign << 3) | comp_code_mag[sel];
    return 0;
}
