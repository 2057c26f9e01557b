// RaZeR decoder for gfx950: x^ = tensor_scale * (block_scale * element), the
// dequantization identity of Sec. 3 with the remapped-zero decoder of Sec. 4.4
// (arxiv 2501.04052).  HBM-bound: 0.5625 B in, 4 or 2 B out per element.
#include "razer_device.hpp"
#include "razer_kernels.hpp"

namespace razer {

// One thread decodes 16 consecutive elements (8 code bytes) with the scale byte of their block
// (16, 32, 64 or 128 elements: cfg.lb = log2 of the block size).
template <int FMT, bool OUT_BF16>
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* __restrict__ codes,
                                                      const uint8_t* __restrict__ scales,
                                                      const float* __restrict__ tensor_scale, SvConfig cfg,
                                                      int64_t rows, int64_t cols, void* __restrict__ out,
                                                      int64_t ld, const float* __restrict__ prod_a,
                                                      const float* __restrict__ prod_b, float* __restrict__ prod_out)
{
    const int64_t nb = cols / kBlock;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid == 0 && prod_out) *prod_out = (*prod_a) * (*prod_b);
    if (gid >= rows * nb) return;
    const int64_t r = gid / nb, b = gid - r * nb;
    const float ts = tensor_scale ? *tensor_scale : 1.0f;
    const uint2 cw = *reinterpret_cast<const uint2*>(codes + r * (cols / 2) + b * 8);
    float s, sv;
    if (FMT == 2)                                               // one 16-bit scale word per 128 elements
        decode_scale_word(reinterpret_cast<const uint16_t*>(scales)[r * (nb >> 3) + (b >> 3)], cfg.sv0, cfg.sv1, s, sv);
    else
        decode_scale_byte<FMT>(scales[r * (nb >> (cfg.lb - 4)) + (b >> (cfg.lb - 4))], cfg.sv0, cfg.sv1, s, sv);
    const float ssv = s * sv;                                   // exact: <= 9 significant bits (<= 16 with a half scale)
    float w[kBlock];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t x = h ? cw.y : cw.x;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // hardware FP4 -> fp32 conversion of byte i (low nibble first), exact
            v2f p = (i == 0)   ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(x, 1.0f, 0)
                    : (i == 1) ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(x, 1.0f, 1)
                    : (i == 2) ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(x, 1.0f, 2)
                               : __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(x, 1.0f, 3);
            const uint32_t c0 = (x >> (8 * i)) & 15u, c1 = (x >> (8 * i + 4)) & 15u;
            const float sq0 = (c0 == 8u) ? ssv : s * p.x;       // s * element, exact
            const float sq1 = (c1 == 8u) ? ssv : s * p.y;
            w[8 * h + 2 * i + 0] = ts * sq0;                    // the single fp32 rounding
            w[8 * h + 2 * i + 1] = ts * sq1;
        }
    }
    if (OUT_BF16) {
        uint32_t pk[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            pk[i] = (uint32_t)f32_to_bf16_rne(w[2 * i]) | ((uint32_t)f32_to_bf16_rne(w[2 * i + 1]) << 16);
        uint4* o = reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(out) + r * ld + b * kBlock);
        o[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        o[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
    } else {
        float4* o = reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + r * ld + b * kBlock);
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = make_float4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
    }
}

hipError_t launch_dequant(int fmt, SvConfig cfg, const uint8_t* codes, const uint8_t* scales,
                          const float* tensor_scale, int64_t rows, int64_t cols, void* out, int dtype_bf16,
                          int64_t ld, hipStream_t st, const float* prod_a, const float* prod_b, float* prod_out)
{
    const int64_t nblk = rows * (cols / kBlock);
    if (nblk == 0) return hipSuccess;
    const unsigned grid = (unsigned)((nblk + 255) / 256);
#define RAZER_DQ(F, B) launch(dequant_kernel<F, B>, grid, 256, 0, st, codes, scales, tensor_scale, cfg, rows, cols, out, ld, prod_a, prod_b, prod_out)
    if (fmt == 0)      { if (dtype_bf16) RAZER_DQ(0, true); else RAZER_DQ(0, false); }
    else if (fmt == 1) { if (dtype_bf16) RAZER_DQ(1, true); else RAZER_DQ(1, false); }
    else               { if (dtype_bf16) RAZER_DQ(2, true); else RAZER_DQ(2, false); }
#undef RAZER_DQ
    return hipGetLastError();
}

}  // namespace razer
