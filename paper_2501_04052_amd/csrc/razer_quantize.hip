// RaZeR block encoder for gfx950: Eq. 1 (tensor scale), Eq. 2 (block scale),
// Eq. 4 (special-value search) and Eq. 5 (final rounding) of arxiv 2501.04052.
//
// Bit-exactness contract: every fp32 operation below is a single IEEE operation
// (true division, no reciprocal, no contraction), squared errors are summed in
// fp64 over the block's elements in index order (also for blocks of 32, 64, 128
// -- the block-size study of Sec. 5.4 -- where the lanes that share a block
// hand the running sum from one to the next), and ties are broken as documented
// in razer.h.
// Compile without fast-math.
#include "razer_device.hpp"
#include "razer_kernels.hpp"

namespace razer {

// ---------------------------------------------------------------- absmax (Eq. 1)
// The running maximum lives in kAbsmaxCells cells of the workspace (workgroup b updates cell
// b % kAbsmaxCells): atomics on a single address serialize at roughly 10 ns each, so a thousand
// workgroups on one cell cost more than the pass over a 32 MB tensor itself.
constexpr int kAbsmaxCells = 64;
constexpr int kAbsmaxBlocks = 1024;
__global__ void absmax_init_kernel(uint32_t* ws) { ws[threadIdx.x] = 0u; }

// max over the cells, by every wavefront that needs it (64 lanes, one cell each)
__device__ __forceinline__ float absmax_from_cells(const uint32_t* __restrict__ ws)
{
    uint32_t m = ws[threadIdx.x & 63u];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
    return u2f(m);
}

template <typename T>
__global__ __launch_bounds__(256) void absmax_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                     int64_t ld, uint32_t* __restrict__ ws)
{
    // 16-byte vectors: 4 floats or 8 bf16.  |x| of finite non-negative floats orders like uint32.
    constexpr int VEC = 16 / sizeof(T);
    __shared__ uint32_t wmax[4];
    uint32_t m = 0;
    auto fold = [&](const uint4& v) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (sizeof(T) == 4) {
                m = max(m, w[j] & 0x7FFFFFFFu);
            } else {
                m = max(m, (w[j] << 16) & 0x7FFFFFFFu);
                m = max(m, w[j] & 0x7FFF0000u);
            }
        }
    };
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (ld == cols) {                                   // dense: one flat array of vectors
        const int64_t total = rows * cols / VEC;
        const uint4* p = reinterpret_cast<const uint4*>(x);
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) fold(p[i]);
    } else {                                            // strided rows: workgroups stride over rows
        const int64_t vec_per_row = cols / VEC;
        for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
            const uint4* p = reinterpret_cast<const uint4*>(x + r * ld);
            for (int64_t c = threadIdx.x; c < vec_per_row; c += blockDim.x) fold(p[c]);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(ws + (blockIdx.x % kAbsmaxCells), max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3])));
}

// ---------------------------------------------------------------- scale rounding (Eq. 2)
// Nearest value of the scale grid, ties to the even code, saturating at the top.
template <int FMT>
__device__ __forceinline__ uint32_t round_scale(float t)
{
    if (FMT == 2) {
        // the hardware's round-to-nearest-even cast to half; anything that would land on 2.0 or
        // above saturates at the largest 14-bit code
        const uint32_t h = __builtin_bit_cast(uint16_t, (_Float16)t);
        return (t >= 2.0f || h > 0x3FFFu) ? 0x3FFFu : h;
    }
    constexpr float kMinNormal = (FMT == 0) ? 0.25f : 0.015625f;          // 2^-2 / 2^-6
    constexpr float kSubScale = (FMT == 0) ? 32.0f : 512.0f;              // 1 / subnormal step
    constexpr uint32_t kBiasAdj = (FMT == 0) ? (124u << 3) : (120u << 3);
    constexpr uint32_t kMaxCode = (FMT == 0) ? 63u : 126u;
    uint32_t code;
    if (t < kMinNormal) {
        code = (uint32_t)__builtin_rintf(t * kSubScale);                  // exact product, RNE
    } else {
        uint32_t b = f2u(t);
        b += 0x7FFFFu + ((b >> 20) & 1u);                                 // RNE to 3 mantissa bits
        code = (b >> 20) - kBiasAdj;
    }
    return code > kMaxCode ? kMaxCode : code;
}

// ---------------------------------------------------------------- block encoder
// One thread encodes one run of 16 elements; G = block / 16 consecutive lanes share a block: they
// agree on the block maximum (hence on the scale) by exchanging their run's maximum, and on the
// special value by forming Eq. 4's error sum as ONE chain over the block's elements in index order:
// lane j of the block continues the sum where lane j - 1 ended (G rounds of 16 additions, of which
// each lane keeps the one round that started from its predecessor's total).
template <typename T, int FMT, int G>
__global__ __launch_bounds__(256) void encode_kernel(const T* __restrict__ x, int64_t rows, int64_t cols,
                                                     int64_t ld, SvConfig cfg,
                                                     const uint32_t* __restrict__ absmax_ws,
                                                     float* __restrict__ tensor_scale, int given_scale,
                                                     uint8_t* __restrict__ codes, uint8_t* __restrict__ scales)
{
    constexpr int NC = (FMT == 1) ? 2 : 4;
    const int64_t nb = cols / kBlock;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;

    float delta32;
    if (given_scale) {
        delta32 = *tensor_scale;
    } else {
        float amax = absmax_from_cells(absmax_ws);
        constexpr float kDenom = (FMT == 0) ? 180.0f : (FMT == 1) ? 2688.0f : 11.994140625f;   // Qmax_scale * 6
        delta32 = (amax == 0.0f) ? 1.0f : amax / kDenom;
        if (gid == 0) *tensor_scale = delta32;
    }
    if (gid >= rows * nb) return;
    const int64_t r = gid / nb, b = gid - r * nb;

    float xv[kBlock];
    if (sizeof(T) == 4) {
        const uint4* p = reinterpret_cast<const uint4*>(x + r * ld + b * kBlock);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint4 v = p[j];
            xv[4 * j + 0] = u2f(v.x); xv[4 * j + 1] = u2f(v.y);
            xv[4 * j + 2] = u2f(v.z); xv[4 * j + 3] = u2f(v.w);
        }
    } else {
        const uint4* p = reinterpret_cast<const uint4*>(x + r * ld + b * kBlock);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            uint4 v = p[j];
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xv[8 * j + 2 * i + 0] = u2f(w[i] << 16);
                xv[8 * j + 2 * i + 1] = u2f(w[i] & 0xFFFF0000u);
            }
        }
    }

    float bmax = 0.0f;
#pragma unroll
    for (int k = 0; k < kBlock; ++k) bmax = fmaxf(bmax, fabsf(xv[k]));
#pragma unroll
    for (int off = 1; off < G; off <<= 1) bmax = fmaxf(bmax, __shfl_xor(bmax, off));   // the block's maximum

    // Eq. 2
    const float d = delta32 * 6.0f;
    const float t = bmax / d;
    const uint32_t sc = round_scale<FMT>(t);
    const float s = (FMT == 0) ? e3m3_value(sc) : (FMT == 1) ? e4m3_value(sc) : half14_value(sc);

    uint32_t lo = 0, hi = 0, meta = 0;                                    // 16 nibbles, low dword = k 0..7
    if (s != 0.0f) {
        const float den = delta32 * s;
        double cand[NC];
        if (FMT != 1) { cand[0] = cfg.sv0; cand[1] = cfg.sv1; cand[2] = -cfg.sv0; cand[3] = -cfg.sv1; }
        else { cand[0] = cfg.sv0; cand[1] = -cfg.sv0; }
        double sse[NC];
        double e2[G > 1 ? NC : 1][kBlock];                                // G > 1: the squared errors, summed as a chain below
        uint32_t take[NC];                                                // bit k: element k takes the special value
#pragma unroll
        for (int m = 0; m < NC; ++m) { sse[m] = 0.0; take[m] = 0u; }
#pragma unroll
        for (int k = 0; k < kBlock; k += 2) {
            const float xs0 = xv[k] / den, xs1 = xv[k + 1] / den;         // X^Scaled
            // Nearest FP4 value, ties to the even code, saturating at +-6: the hardware conversion
            // (verified against the threshold form of the same rule on every boundary +- 1 ulp and
            // 10^6 random values).  It writes the two codes into byte k / 2 of the packed dword; a
            // negative value that rounds to zero comes out as code 0x8 and is cleared below.
            uint32_t& word = (k < 8) ? lo : hi;
            word = (k % 8 == 0)   ? __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(word, xs0, xs1, 1.0f, 0)
                   : (k % 8 == 2) ? __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(word, xs0, xs1, 1.0f, 1)
                   : (k % 8 == 4) ? __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(word, xs0, xs1, 1.0f, 2)
                                  : __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(word, xs0, xs1, 1.0f, 3);
            const v2f q = (k % 8 == 0)   ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, 0)
                          : (k % 8 == 2) ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, 1)
                          : (k % 8 == 4) ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, 2)
                                         : __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, 3);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const double xd = (double)(j ? xs1 : xs0);
                const double eb = xd - (double)(j ? q.y : q.x);           // exact (-0 for a negative zero changes nothing)
#pragma unroll
                for (int m = 0; m < NC; ++m) {
                    const double ev = xd - cand[m];
                    const bool sp = fabs(ev) < fabs(eb);
                    const double e = sp ? ev : eb;
                    if (G > 1) e2[m][k + j] = e * e;                      // exact in fp64
                    else sse[m] = __builtin_fma(e, e, sse[m]);            // e*e is exact in fp64: same as sse + e*e
                    take[m] |= (uint32_t)sp << (k + j);
                }
            }
        }
        if (G > 1) {
            // block error = sum over all 16 G elements in index order.  Round p is the one in which lane
            // base + p of the block holds the right starting value (its predecessor's total of round p - 1).
            const int sub = (int)(threadIdx.x & 63u) & (G - 1), base = (int)(threadIdx.x & 63u) & ~(G - 1);
#pragma unroll
            for (int p = 0; p < G; ++p) {
#pragma unroll
                for (int m = 0; m < NC; ++m) {
                    double a = (p == 0) ? 0.0 : __shfl(sse[m], base + p - 1);
#pragma unroll
                    for (int k = 0; k < kBlock; ++k) a += e2[m][k];
                    sse[m] = (sub == p) ? a : sse[m];
                }
            }
#pragma unroll
            for (int m = 0; m < NC; ++m) sse[m] = __shfl(sse[m], base + G - 1);   // every lane of the block: the block's sum
        }
        // Eq. 4: smallest error, ties to the smallest metadata index
        double best = sse[0];
#pragma unroll
        for (int m = 1; m < NC; ++m)
            if (sse[m] < best) { best = sse[m]; meta = m; }
        uint32_t tk = take[0];
#pragma unroll
        for (int m = 1; m < NC; ++m) tk = (meta == (uint32_t)m) ? take[m] : tk;
        // Eq. 5 on the packed nibbles: zero keeps code 0x0 whatever its sign, taken elements get the
        // remapped code 0x8.  spread() moves bit k of a byte-wide mask to bit 4 k.
        auto spread = [](uint32_t b) {
            b = (b | (b << 12)) & 0x000F000Fu;
            b = (b | (b << 6)) & 0x03030303u;
            return (b | (b << 3)) & 0x11111111u;
        };
        auto finish = [&](uint32_t w, uint32_t taken8) {
            const uint32_t mag = w & 0x77777777u;
            const uint32_t nz = (mag | (mag >> 1) | (mag >> 2)) & 0x11111111u;   // 1 per nibble with a non-zero magnitude
            w &= 0x77777777u | (nz << 3);                                     // -0 -> +0
            const uint32_t t1 = spread(taken8);
            return (w & ~(t1 * 15u)) | (t1 << 3);
        };
        lo = finish(lo, tk & 0xFFu);
        hi = finish(hi, (tk >> 8) & 0xFFu);
    }
    *reinterpret_cast<uint2*>(codes + r * (cols / 2) + b * 8) = make_uint2(lo, hi);
    if ((b & (G - 1)) == 0) {
        if (FMT == 2) reinterpret_cast<uint16_t*>(scales)[r * (nb / G) + b / G] = (uint16_t)((meta << 14) | sc);
        else scales[r * (nb / G) + b / G] = (uint8_t)((meta << (FMT == 0 ? 6 : 7)) | sc);
    }
}

// ---------------------------------------------------------------- host launchers
template <typename T, int FMT>
static void launch_encode(int lb, unsigned grid, unsigned threads, hipStream_t st, const T* x, int64_t rows,
                          int64_t cols, int64_t ld, SvConfig cfg, const uint32_t* ws, float* tensor_scale, int given,
                          uint8_t* codes, uint8_t* scales)
{
#define RAZER_ENC(G) launch(encode_kernel<T, FMT, G>, grid, threads, 0, st, x, rows, cols, ld, cfg, ws, tensor_scale, given, codes, scales)
    switch (lb) {
        case 4: RAZER_ENC(1); break;
        case 5: RAZER_ENC(2); break;
        case 6: RAZER_ENC(4); break;
        default: RAZER_ENC(8); break;
    }
#undef RAZER_ENC
}

template <typename T>
static hipError_t launch_quantize_t(int fmt, SvConfig cfg, const T* x, int64_t rows, int64_t cols, int64_t ld,
                                    uint8_t* codes, uint8_t* scales, float* tensor_scale, int given,
                                    uint32_t* ws, hipStream_t st)
{
    if (rows == 0 || cols == 0) {
        if (!given) {                       // an empty tensor gets the all-zero tensor's scale of 1
            launch(absmax_init_kernel, 1, kAbsmaxCells, 0, st, ws);
            if (fmt == 0) launch_encode<T, 0>(4, 1, 64, st, x, 0, 16, 16, cfg, ws, tensor_scale, 0, codes, scales);
            else launch_encode<T, 1>(4, 1, 64, st, x, 0, 16, 16, cfg, ws, tensor_scale, 0, codes, scales);
        }
        return hipGetLastError();
    }
    if (!given) {
        launch(absmax_init_kernel, 1, kAbsmaxCells, 0, st, ws);
        constexpr int VEC = 16 / sizeof(T);
        int64_t total = rows * (cols / VEC);
        int64_t blocks = (total + 255) / 256;
        if (blocks > kAbsmaxBlocks) blocks = kAbsmaxBlocks;
        launch(absmax_kernel<T>, (unsigned)blocks, 256, 0, st, x, rows, cols, ld, ws);
    }
    int64_t nblk = rows * (cols / kBlock);
    unsigned grid = (unsigned)((nblk + 255) / 256);
    if (fmt == 0) launch_encode<T, 0>(cfg.lb, grid, 256, st, x, rows, cols, ld, cfg, ws, tensor_scale, given, codes, scales);
    else if (fmt == 1) launch_encode<T, 1>(cfg.lb, grid, 256, st, x, rows, cols, ld, cfg, ws, tensor_scale, given, codes, scales);
    else launch(encode_kernel<T, 2, 8>, grid, 256, 0, st, x, rows, cols, ld, cfg, ws, tensor_scale, given, codes, scales);
    return hipGetLastError();
}

hipError_t launch_quantize(int fmt, SvConfig cfg, const void* x, int dtype_bf16, int64_t rows, int64_t cols,
                           int64_t ld, uint8_t* codes, uint8_t* scales, float* tensor_scale, int given,
                           void* ws, hipStream_t st)
{
    if (dtype_bf16)
        return launch_quantize_t<uint16_t>(fmt, cfg, (const uint16_t*)x, rows, cols, ld, codes, scales,
                                           tensor_scale, given, (uint32_t*)ws, st);
    return launch_quantize_t<float>(fmt, cfg, (const float*)x, rows, cols, ld, codes, scales, tensor_scale,
                                    given, (uint32_t*)ws, st);
}

}  // namespace razer
