// RaZeR linear layer on the gfx950 bf16 matrix cores (prefill-shaped problems,
// Sec. 4.3 of arxiv 2501.04052; weight-activation mode of App. D.3 by decoding
// both operands): packed codes are read from HBM, decoded to scaled bf16 in
// registers, staged in LDS and consumed by v_mfma_f32_32x32x16_bf16 with fp32
// accumulation.  block_scale * element needs at most 8 significant bits for the
// paper's special values, so the bf16 tile is exact; the tensor scale(s) multiply
// the fp32 accumulator once at the end.
//
// Tile: BM activation rows x BN weight rows x 64 k per stage, double-buffered.
// LDS rows are 128 B (64 bf16); 16-byte chunks are xor-swizzled with the row so
// that the 128-bit MFMA operand reads of consecutive rows hit distinct banks.
// The weight fragment is the MFMA "A" operand (rows = n) and the activation
// fragment the "B" operand (columns = m), so every lane ends up holding 4
// consecutive n of one output row; two lanes swap halves and store 16 bytes.
//
// Kernels, chosen by gemm_plan() from M and the number of output tiles:
//   gemm_kernel      both operands decoded into LDS, all waves alike (M <= 128: the fused W4A4 kernel and
//                    the FP16-scale format)
//   gemm_pp_kernel   256-row tiles, two wave groups half a step out of phase (decode | MFMA): few-tile
//                    problems above 128 rows, the fused W4A4 kernel, the FP16-scale format
//   gemm_rb_kernel   W4A16, 16-element blocks: weights decoded in registers by the wave that uses them,
//                    global -> LDS copies by the load unit; 256-row activation tiles when there are
//                    many output tiles, 64- / 128-row tiles for 33..128 activation rows; KG = 2 halves
//                    K inside the workgroup when there is about one tile per compute unit; the grouped
//                    form runs up to four matrices (fused q/k/v, gate/up) as one launch
// Problems with too few tiles split K over workgroups (fp32 slices in the caller's workspace).
#include <mutex>
#include <type_traits>

#include "razer_device.hpp"
#include "razer_kernels.hpp"

namespace razer {

constexpr int kBK = 64;

// The large-tile kernels need more dynamic LDS than the default limit; the limit is raised once per
// kernel and device, on first use.  RAZER_RAISE_LDS_LIMIT expands inside a launch helper that is
// instantiated once per kernel configuration, so its flags are per kernel; std::call_once makes the
// first use safe when several host threads launch at once.
constexpr int kMaxDevices = 16;
#define RAZER_RAISE_LDS_LIMIT(kern, smem)                                                                  \
    do {                                                                                                   \
        static std::once_flag once[kMaxDevices];                                                           \
        static hipError_t result[kMaxDevices];                                                             \
        int dev = 0;                                                                                       \
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice; \
        std::call_once(once[dev], [&] {                                                                    \
            result[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                         \
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)(smem));    \
        });                                                                                                \
        if (result[dev] != hipSuccess) return result[dev];                                                 \
    } while (0)

// LUT entry per scale byte: { block scale (fp32 bits), -(special * scale) as a bf16 pair }.
template <int FMT>
__device__ __forceinline__ void fill_scaled_lut(uint2* lut, float sv0, float sv1, int tid, int nthreads)
{
    for (uint32_t sb = tid; sb < 256u; sb += nthreads) {
        float s, sv;
        decode_scale_byte<FMT>(sb, sv0, sv1, s, sv);
        const uint32_t p = (uint32_t)f32_to_bf16_rne(-(sv * s));
        lut[sb] = make_uint2(f2u(s), p | (p << 16));
    }
}

template <int BYTE>
__device__ __forceinline__ uint32_t cvt_scaled_pair(uint32_t xflip, float s, uint32_t patch)
{
    v2f p = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(xflip, 1.0f, BYTE);   // -element, exact
    p.x *= s;                                                              // exact (<= 6 significant bits)
    p.y *= s;
    v2bf b = __builtin_convertvector(p, v2bf);                             // exact
    return patch_zero_halves(__builtin_bit_cast(uint32_t, b), patch);
}
// 8 codes of one block -> 8 scaled, negated bf16 values (one 16-byte LDS chunk).
__device__ __forceinline__ uint4 decode_dword(uint32_t x, uint2 lut_entry)
{
    const uint32_t xf = x ^ kRemapXor;
    const float s = u2f(lut_entry.x);
    return make_uint4(cvt_scaled_pair<0>(xf, s, lut_entry.y), cvt_scaled_pair<1>(xf, s, lut_entry.y),
                      cvt_scaled_pair<2>(xf, s, lut_entry.y), cvt_scaled_pair<3>(xf, s, lut_entry.y));
}

// 8 codes -> 8 bare, negated FP4 values as bf16 (exact), remapped codes patched with `patch` (the negated
// special value as a bf16 pair): the decode of the FP16-scale format, whose scale multiplies partial sums.
template <int BYTE>
__device__ __forceinline__ uint32_t cvt_bare_pair(uint32_t xflip, uint32_t patch)
{
    v2bf p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(xflip, 1.0f, BYTE);
    return patch_zero_halves(__builtin_bit_cast(uint32_t, p), patch);
}
__device__ __forceinline__ uint4 decode_dword_bare(uint32_t x, uint32_t patch)
{
    const uint32_t xf = x ^ kRemapXor;
    return make_uint4(cvt_bare_pair<0>(xf, patch), cvt_bare_pair<1>(xf, patch), cvt_bare_pair<2>(xf, patch),
                      cvt_bare_pair<3>(xf, patch));
}

// gfx950 LDS: 64 banks x 4 B; a 128-bit access is served 16 lanes per clock, so 16 consecutive rows
// (256-byte period = 2 rows) must land on 16 distinct 16-byte slots: swizzle with bits 1..3 of the row.
__device__ __forceinline__ uint32_t lds_off(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

// Epilogue shared by the GEMM kernels: undo the sign flip of the weight decode (in W4A4 the
// flips of the two operands cancel), apply the tensor scale(s), round to bf16 and store.  Lane l
// of a 32x32 accumulator holds output row m = l % 32 and, per group g of 4 registers, the 4
// consecutive columns n = 8 g + 4 (l / 32) + 0..3.  Lanes l and l + 32 exchange halves
// (v_permlane32_swap) so that each lane ends up with 8 consecutive columns -- groups 0 and 2 in the
// lower half-wave, 1 and 3 in the upper -- and writes them as one 16-byte store.
template <int TM, int TN, bool AQ>
__device__ __forceinline__ void store_tile(const v16f (&acc)[TN][TM], const float* w_ts, const float* a_ts,
                                           int64_t wm0, int64_t wn0, int64_t m, int64_t n, uint16_t* y,
                                           int64_t ld_y, int lane)
{
    const float scale = AQ ? (*w_ts) * (*a_ts) : -(*w_ts);
    const int hi = lane >> 5;
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int64_t gm = wm0 + j * 32 + (lane & 31);
#pragma unroll
            for (int gp = 0; gp < 2; ++gp) {                       // groups (2 gp, 2 gp + 1)
                uint32_t pk[2][2];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int v = 4 * (2 * gp + h) + 2 * e;
                        pk[h][e] = (uint32_t)f32_to_bf16_rne(acc[i][j][v] * scale) |
                                   ((uint32_t)f32_to_bf16_rne(acc[i][j][v + 1] * scale) << 16);
                    }
                uint32_t o[4];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    auto r = __builtin_amdgcn_permlane32_swap(pk[0][e], pk[1][e], false, false);
                    o[e] = r[0];                                    // columns +0..3 of this lane's group
                    o[2 + e] = r[1];                                // columns +4..7
                }
                const int64_t gn = wn0 + i * 32 + 8 * (2 * gp + hi);
                if (gm < m && gn < n) {
                    uint16_t* dst = y + gm * ld_y + gn;
                    if (gn + 7 < n && ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0)) {
                        *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (gn + e < n) dst[e] = (uint16_t)(o[e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
        }
}

// Split-K epilogue: the raw fp32 accumulators of one K-slice go to partial[m][n] (dense, ld = n);
// a second kernel adds the slices in order and applies the tensor scale(s).  Same lane layout as
// store_tile: lane l holds row l % 32 and, per group g of 4 registers, columns 8 g + 4 (l / 32) + 0..3.
template <int TM, int TN>
__device__ __forceinline__ void store_tile_partial(const v16f (&acc)[TN][TM], int64_t wm0, int64_t wn0, int64_t m,
                                                   int64_t n, float* __restrict__ partial, int lane)
{
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int64_t gm = wm0 + j * 32 + (lane & 31);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int64_t gn = wn0 + i * 32 + 8 * g + 4 * (lane >> 5);
                if (gm < m && gn < n) {
                    float* dst = partial + gm * n + gn;
                    if (gn + 3 < n && ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0)) {
                        *reinterpret_cast<float4*>(dst) = make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1],
                                                                      acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (gn + e < n) dst[e] = acc[i][j][4 * g + e];
                    }
                }
            }
        }
}

// SF: the FP16-scale weight format (blocks of 128, one scale word; bf16 activations only).  A half scale
// times an FP4 value does not fit a bf16 operand, so the weights go to LDS as bare FP4 values and the
// matrix instructions accumulate one block (two K-tiles) into a second set of accumulators, which the
// block's scale -- per weight row, fp32 in LDS next to the tile -- then folds into the running sums.
template <int BM, int BN, int WGM, int WGN, bool AQ, bool GB, bool SF = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, const float* __restrict__ w_ts,
    SvConfig wcfg, int64_t n, int64_t k, const uint16_t* __restrict__ a, const uint8_t* __restrict__ a_codes,
    const uint8_t* __restrict__ a_scales, const float* __restrict__ a_ts, SvConfig acfg, int64_t m,
    uint16_t* __restrict__ y, int64_t ld_y, int tiles_m, float* __restrict__ partial)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
    constexpr int NU_A = AQ ? (BM * 2 + NT - 1) / NT : (BM * 8) / NT;   // units per thread: 16 B of global data each
    constexpr int NU_B = (BN * 2 + NT - 1) / NT;
    static_assert(AQ || (BM * 8) % NT == 0, "A tile must divide over the threads");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");

    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* As = smem;                              // 2 stages x BM x 128 B
    uint8_t* Bs = smem + 2 * BM * 128;               // 2 stages x BN x 128 B
    uint2* wlut = reinterpret_cast<uint2*>(smem + 2 * (BM + BN) * 128);
    uint2* alut = wlut + 256;
    float* wsc = reinterpret_cast<float*>(wlut);      // SF: 2 stages x BN block scales in place of the tables
    static_assert(!SF || (!AQ && !GB && 2 * BN * 4 <= 2 * 256 * 8), "FP16-scale variant");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    // blockIdx.y = K-slice (split-K for problems with few output tiles): K-tiles [kt0, kt0 + KT)
    // (SF: slices of whole 128-element blocks, i.e. an even number of K-tiles)
    const int kt_all = (int)((k + kBK - 1) / kBK);
    const int kt_even = (kt_all + (int)gridDim.y - 1) / (int)gridDim.y;
    const int kt_per = SF ? ((kt_even + 1) & ~1) : kt_even;
    const int kt0 = (int)blockIdx.y * kt_per;
    const int KT = kt_all - kt0 < kt_per ? kt_all - kt0 : kt_per;

    if (!SF) fill_scaled_lut<0>(wlut, wcfg.sv0, wcfg.sv1, tid, NT);
    if (AQ) fill_scaled_lut<1>(alut, acfg.sv0, acfg.sv1, tid, NT);

    v16f acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    uint4 ra[NU_A];
    uint32_t rsa[NU_A];
    uint4 rb[NU_B];
    uint32_t rsb[NU_B];

    auto load_tiles = [&](int kt) {
        const int64_t kbase = (int64_t)(kt0 + kt) * kBK;
        if (AQ) {
#pragma unroll
            for (int i = 0; i < NU_A; ++i) {
                const int u = tid + i * NT, row = u >> 1, half = u & 1;
                const int64_t gr = m0 + row, kk = kbase + half * 32;
                ra[i] = make_uint4(0, 0, 0, 0);
                rsa[i] = 0;
                if (u < BM * 2 && gr < m && kk < k) {
                    ra[i] = *reinterpret_cast<const uint4*>(a_codes + gr * (k / 2) + kk / 2);
                    rsa[i] = load_scale_pair<GB>(a_scales + gr * (k >> acfg.lb), kk, acfg.lb);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NU_A; ++i) {
                const int u = tid + i * NT, row = u >> 3, chunk = u & 7;
                const int64_t gr = m0 + row, kk = kbase + chunk * 8;
                ra[i] = make_uint4(0, 0, 0, 0);
                if (gr < m && kk < k) ra[i] = *reinterpret_cast<const uint4*>(a + gr * k + kk);
            }
        }
#pragma unroll
        for (int i = 0; i < NU_B; ++i) {
            const int u = tid + i * NT, row = u >> 1, half = u & 1;
            const int64_t gr = n0 + row, kk = kbase + half * 32;
            rb[i] = make_uint4(0, 0, 0, 0);
            rsb[i] = 0;
            if (u < BN * 2 && gr < n && kk < k) {
                rb[i] = *reinterpret_cast<const uint4*>(w_codes + gr * (k / 2) + kk / 2);
                if (SF) rsb[i] = reinterpret_cast<const uint16_t*>(w_scales)[gr * (k >> 7) + (kk >> 7)];
                else rsb[i] = load_scale_pair<GB>(w_scales + gr * (k >> wcfg.lb), kk, wcfg.lb);
            }
        }
    };
    // part q (0..3) of the register-held tiles -> LDS stage st
    auto store_part = [&](int st, int q) {
        uint8_t* as = As + st * BM * 128;
        uint8_t* bs = Bs + st * BN * 128;
        if (AQ) {
#pragma unroll
            for (int i = 0; i < NU_A; ++i) {
                const int u = tid + i * NT, row = u >> 1, half = u & 1;
                if (u < BM * 2) {
                    const uint32_t x = (q == 0) ? ra[i].x : (q == 1) ? ra[i].y : (q == 2) ? ra[i].z : ra[i].w;
                    const uint2 le = alut[(rsa[i] >> (8 * (q >> 1))) & 255u];
                    *reinterpret_cast<uint4*>(as + lds_off(row, half * 4 + q)) = decode_dword(x, le);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NU_A; ++i) {
                if ((i & 3) == q) {
                    const int u = tid + i * NT, row = u >> 3, chunk = u & 7;
                    *reinterpret_cast<uint4*>(as + lds_off(row, chunk)) = ra[i];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NU_B; ++i) {
            const int u = tid + i * NT, row = u >> 1, half = u & 1;
            if (u < BN * 2) {
                const uint32_t x = (q == 0) ? rb[i].x : (q == 1) ? rb[i].y : (q == 2) ? rb[i].z : rb[i].w;
                if (SF) {
                    float sc, sv;
                    decode_scale_word(rsb[i], wcfg.sv0, wcfg.sv1, sc, sv);          // (rows past N: word 0, scale 0)
                    const uint32_t nsv = (uint32_t)f32_to_bf16_rne(-sv);
                    *reinterpret_cast<uint4*>(bs + lds_off(row, half * 4 + q)) = decode_dword_bare(x, nsv | (nsv << 16));
                    if (q == 0 && half == 0) wsc[st * BN + row] = sc;               // the block's scale, for the fold
                } else {
                    const uint2 le = wlut[(rsb[i] >> (8 * (q >> 1))) & 255u];
                    *reinterpret_cast<uint4*>(bs + lds_off(row, half * 4 + q)) = decode_dword(x, le);
                }
            }
        }
    };
    // SF: sums of the current block of 128 elements (two K-tiles), folded into acc with the block scales
    v16f blk[SF ? TN : 1][SF ? TM : 1];

    load_tiles(0);
    __syncthreads();                                   // LUTs ready
#pragma unroll
    for (int q = 0; q < 4; ++q) store_part(0, q);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int st = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) load_tiles(kt + 1);
        const uint8_t* as = As + st * BM * 128;
        const uint8_t* bs = Bs + st * BN * 128;
        // SF: a block starts with every even K-tile of the matrix (K is a multiple of 128 and K-slices hold
        // whole blocks): its first matrix instruction starts from zero instead of from the previous block
        const bool block_start = SF && ((kt0 + kt) & 1) == 0;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            v8bf fw[TN], fa[TM];
            const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TN; ++i)
                fw[i] = *reinterpret_cast<const v8bf*>(bs + lds_off(wn * WTN + i * 32 + (lane & 31), chunk));
#pragma unroll
            for (int j = 0; j < TM; ++j)
                fa[j] = *reinterpret_cast<const v8bf*>(as + lds_off(wm * WTM + j * 32 + (lane & 31), chunk));
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    if (SF) {
                        if (ks == 0 && block_start) {
                            v16f zero;
#pragma unroll
                            for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
                            blk[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], zero, 0, 0, 0);
                        } else {
                            blk[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], blk[i][j], 0, 0, 0);
                        }
                    } else {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
                    }
                }
            if (more) store_part(st ^ 1, ks);
        }
        if (SF && (((kt0 + kt) & 1) == 1 || !more)) {
            // fold the finished block: register v of a 32x32 accumulator belongs to weight row
            // 8 (v / 4) + 4 (lane / 32) + v % 4 of the fragment (the layout store_tile documents)
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                float sc[16];
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const float4 t = *reinterpret_cast<const float4*>(wsc + st * BN + wn * WTN + i * 32 + 8 * g4 + 4 * (lane >> 5));
                    sc[4 * g4] = t.x; sc[4 * g4 + 1] = t.y; sc[4 * g4 + 2] = t.z; sc[4 * g4 + 3] = t.w;
                }
#pragma unroll
                for (int j = 0; j < TM; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = __builtin_fmaf(sc[v], blk[i][j][v], acc[i][j][v]);
            }
        }
        __syncthreads();
    }

    if (partial)
        store_tile_partial<TM, TN>(acc, m0 + wm * WTM, n0 + wn * WTN, m, n, partial + (int64_t)blockIdx.y * m * n, lane);
    else
        store_tile<TM, TN, AQ>(acc, w_ts, a_ts, m0 + wm * WTM, n0 + wn * WTN, m, n, y, ld_y, lane);
}

// ---------------------------------------------------------------------------------------------
// Large tiles: 8 waves in two groups of 4 (one wave of each group per SIMD) that run half a step
// out of phase.  While one group issues the MFMAs of K-tile i from LDS stage i % 2, the other
// decodes its half of K-tile i + 1 into the other stage; then they swap.  Every SIMD therefore
// always has one wave feeding the matrix core and one wave doing the VALU / LDS-write / global-load
// work, instead of all waves decoding and then all waves multiplying.
//
//   slot 2i    : group 0  MFMA(i)                      | group 1  store its half of tile i+1
//   slot 2i+1  : group 0  store its half of tile i+1   | group 1  MFMA(i)
//
// One barrier ends every slot.  Tile i+1 is complete at the end of slot 2i+1 and is first read in
// slot 2i+2; the stage it overwrites was last read in slot 2i-1.  Global loads for a group's half of
// tile i+2 are issued right after it stored tile i+1 and land during its next MFMA slot.
// SF: the FP16-scale weight format, as in gemm_kernel -- bare FP4 weights in LDS, the blocks' scales as fp32
// beside the tile, a second accumulator set per block of 128 elements (two K-tiles) and a fold after every
// second K-tile (256 x 128 tiles only: the second set must fit the registers of two waves per SIMD).
template <int BM, int BN, int WGM, int WGN, bool AQ, bool GB, bool SF = false>
__global__ __launch_bounds__(512) void gemm_pp_kernel(
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, const float* __restrict__ w_ts,
    SvConfig wcfg, int64_t n, int64_t k, const uint16_t* __restrict__ a, const uint8_t* __restrict__ a_codes,
    const uint8_t* __restrict__ a_scales, const float* __restrict__ a_ts, SvConfig acfg, int64_t m,
    uint16_t* __restrict__ y, int64_t ld_y, int tiles_m, float* __restrict__ partial)
{
    static_assert(WGM * WGN == 8, "two groups of four waves");
    constexpr int GT = 256;                                            // threads per group
    constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
    // per-thread work on one K-tile: a group handles half the rows of each operand tile
    constexpr int A_PT = AQ ? (BM / 2 * 4) / GT : (BM / 2 * 8) / GT;   // blocks of 16 codes, or 16-byte bf16 chunks
    // Weight share of a thread: UB consecutive blocks of one row (UB = 2: 16 bytes of codes + 2 scale
    // bytes; UB = 1: 8 + 1), so that all 256 threads of a group have decode work.
    constexpr int UB = (BN / 2 * 4) / GT >= 2 ? 2 : 1;
    constexpr int B_PT = (BN / 2 * 4) / GT / UB;
    constexpr int UPR = 4 / UB;                                        // units per 64-k row tile
    static_assert(A_PT >= 1 && B_PT >= 1, "tile too small for 512 threads");

    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* As = smem;
    uint8_t* Bs = smem + 2 * BM * 128;
    uint2* wlut = reinterpret_cast<uint2*>(smem + 2 * (BM + BN) * 128);
    uint2* alut = wlut + 256;
    float* wsc = reinterpret_cast<float*>(wlut);       // SF: 2 stages x BN block scales in place of the tables
    static_assert(!SF || (!AQ && !GB && TM * TN <= 4 && 2 * BN * 4 <= 2 * 256 * 8), "FP16-scale variant");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = wave >> 2, gt = tid & (GT - 1);
    const int wm = wave % WGM, wn = wave / WGM;
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    // (SF: slices of whole 128-element blocks, i.e. an even number of K-tiles)
    const int kt_all = (int)((k + kBK - 1) / kBK);
    const int kt_even = (kt_all + (int)gridDim.y - 1) / (int)gridDim.y;
    const int kt_per = SF ? ((kt_even + 1) & ~1) : kt_even;
    const int kt0 = (int)blockIdx.y * kt_per;                          // K-slice of this workgroup (split-K)
    const int KT = kt_all - kt0 < kt_per ? kt_all - kt0 : kt_per;

    if (!SF) fill_scaled_lut<0>(wlut, wcfg.sv0, wcfg.sv1, tid, 512);
    if (AQ) fill_scaled_lut<1>(alut, acfg.sv0, acfg.sv1, tid, 512);

    v16f acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Register-held prefetch of this thread's share of one K-tile.  Two sets: tile t uses set t % 2,
    // so a tile's global loads are issued two store-slots before they are consumed.
    struct Prefetch {
        uint4 ra[AQ ? 1 : A_PT];           // bf16 activations: 8 values per unit
        uint2 rqa[AQ ? A_PT : 1];          // quantized activations: 16 codes per unit
        uint32_t rsa[AQ ? A_PT : 1];
        uint4 rb[B_PT];
        uint32_t rsb[B_PT];
    };
    Prefetch pf0, pf1;

    auto gload = [&](Prefetch& pf, int kt) {
        const int64_t kbase = (int64_t)(kt0 + kt) * kBK;
        if (AQ) {
#pragma unroll
            for (int i = 0; i < A_PT; ++i) {
                const int u = gt + i * GT, row = grp * (BM / 2) + (u >> 2), blk = u & 3;
                const int64_t gr = m0 + row, kk = kbase + blk * 16;
                pf.rqa[i] = make_uint2(0, 0);
                pf.rsa[i] = 0;
                if (gr < m && kk < k) {
                    pf.rqa[i] = *reinterpret_cast<const uint2*>(a_codes + gr * (k / 2) + kk / 2);
                    pf.rsa[i] = a_scales[gr * (k >> acfg.lb) + (kk >> acfg.lb)];
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_PT; ++i) {
                const int u = gt + i * GT, row = grp * (BM / 2) + (u >> 3), chunk = u & 7;
                const int64_t gr = m0 + row, kk = kbase + chunk * 8;
                pf.ra[i] = make_uint4(0, 0, 0, 0);
                if (gr < m && kk < k) pf.ra[i] = *reinterpret_cast<const uint4*>(a + gr * k + kk);
            }
        }
#pragma unroll
        for (int i = 0; i < B_PT; ++i) {
            const int u = gt + i * GT, row = grp * (BN / 2) + u / UPR, part = u % UPR;
            const int64_t gr = n0 + row, kk = kbase + part * (16 * UB);
            pf.rb[i] = make_uint4(0, 0, 0, 0);
            pf.rsb[i] = 0;
            if (gr < n && kk < k) {
                if (UB == 2) {
                    pf.rb[i] = *reinterpret_cast<const uint4*>(w_codes + gr * (k / 2) + kk / 2);
                    if (SF) pf.rsb[i] = reinterpret_cast<const uint16_t*>(w_scales)[gr * (k >> 7) + (kk >> 7)];
                    else pf.rsb[i] = load_scale_pair<GB>(w_scales + gr * (k >> wcfg.lb), kk, wcfg.lb);
                } else {
                    const uint2 t2 = *reinterpret_cast<const uint2*>(w_codes + gr * (k / 2) + kk / 2);
                    pf.rb[i].x = t2.x;
                    pf.rb[i].y = t2.y;
                    if (SF) pf.rsb[i] = reinterpret_cast<const uint16_t*>(w_scales)[gr * (k >> 7) + (kk >> 7)];
                    else pf.rsb[i] = w_scales[gr * (k >> wcfg.lb) + (kk >> wcfg.lb)];
                }
            }
        }
    };
    auto store = [&](const Prefetch& pf, int st) {
        uint8_t* as = As + st * BM * 128;
        uint8_t* bs = Bs + st * BN * 128;
        if (AQ) {
#pragma unroll
            for (int i = 0; i < A_PT; ++i) {
                const int u = gt + i * GT, row = grp * (BM / 2) + (u >> 2), blk = u & 3;
                const uint2 le = alut[pf.rsa[i] & 255u];
                *reinterpret_cast<uint4*>(as + lds_off(row, 2 * blk)) = decode_dword(pf.rqa[i].x, le);
                *reinterpret_cast<uint4*>(as + lds_off(row, 2 * blk + 1)) = decode_dword(pf.rqa[i].y, le);
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_PT; ++i) {
                const int u = gt + i * GT, row = grp * (BM / 2) + (u >> 3), chunk = u & 7;
                *reinterpret_cast<uint4*>(as + lds_off(row, chunk)) = pf.ra[i];
            }
        }
#pragma unroll
        for (int i = 0; i < B_PT; ++i) {
            const int u = gt + i * GT, row = grp * (BN / 2) + u / UPR, part = u % UPR;
            if constexpr (SF) {
                float sc, sv;
                decode_scale_word(pf.rsb[i], wcfg.sv0, wcfg.sv1, sc, sv);      // (rows past N, tiles past K: word 0, scale 0)
                const uint32_t nsv = (uint32_t)f32_to_bf16_rne(-sv), patch = nsv | (nsv << 16);
                *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 0)) = decode_dword_bare(pf.rb[i].x, patch);
                *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 1)) = decode_dword_bare(pf.rb[i].y, patch);
                if (UB == 2) {
                    *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 2)) = decode_dword_bare(pf.rb[i].z, patch);
                    *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 3)) = decode_dword_bare(pf.rb[i].w, patch);
                }
                if (part == 0) wsc[st * BN + row] = sc;                        // the block's scale, for the fold
                continue;
            }
            const uint2 le0 = wlut[pf.rsb[i] & 255u];
            *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 0)) = decode_dword(pf.rb[i].x, le0);
            *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 1)) = decode_dword(pf.rb[i].y, le0);
            if (UB == 2) {
                const uint2 le1 = wlut[(pf.rsb[i] >> 8) & 255u];
                *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 2)) = decode_dword(pf.rb[i].z, le1);
                *reinterpret_cast<uint4*>(bs + lds_off(row, 2 * UB * part + 3)) = decode_dword(pf.rb[i].w, le1);
            }
        }
    };
    // SF: sums of the current block of 128 elements (two K-tiles), folded into acc with the block scales
    v16f blk[SF ? TN : 1][SF ? TM : 1];
    auto mfma_tile = [&](int st, int t) {
        const uint8_t* as = As + st * BM * 128;
        const uint8_t* bs = Bs + st * BN * 128;
        // SF: a block starts with every even K-tile of the matrix (K-slices hold whole blocks)
        const bool block_start = SF && ((kt0 + t) & 1) == 0;
        // operand fragments are fetched DEPTH k-steps ahead of the MFMAs that use them
        constexpr int DEPTH = (!SF && TM + TN <= 4) ? 4 : 2;             // (SF: the second accumulator set needs the registers)
        v8bf fw[DEPTH][TN], fa[DEPTH][TM];
        auto frags = [&](int ks, int buf) {
            const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TN; ++i)
                fw[buf][i] = *reinterpret_cast<const v8bf*>(bs + lds_off(wn * WTN + i * 32 + (lane & 31), chunk));
#pragma unroll
            for (int j = 0; j < TM; ++j)
                fa[buf][j] = *reinterpret_cast<const v8bf*>(as + lds_off(wm * WTM + j * 32 + (lane & 31), chunk));
        };
#pragma unroll
        for (int ks = 0; ks < DEPTH - 1; ++ks) frags(ks, ks);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks + DEPTH - 1 < 4) frags(ks + DEPTH - 1, (ks + DEPTH - 1) % DEPTH);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    if constexpr (SF) {
                        if (ks == 0 && block_start) {
                            v16f zero;
#pragma unroll
                            for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
                            blk[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks % DEPTH][i], fa[ks % DEPTH][j], zero, 0, 0, 0);
                        } else {
                            blk[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks % DEPTH][i], fa[ks % DEPTH][j], blk[i][j], 0, 0, 0);
                        }
                    } else {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks % DEPTH][i], fa[ks % DEPTH][j], acc[i][j], 0, 0, 0);
                    }
                }
        }
        if constexpr (SF) {
            if (((kt0 + t) & 1) == 1 || t + 1 >= KT) {
                // fold the finished block: register v of a 32x32 accumulator belongs to weight row
                // 8 (v / 4) + 4 (lane / 32) + v % 4 of the fragment
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    float sc[16];
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const float4 q = *reinterpret_cast<const float4*>(wsc + st * BN + wn * WTN + i * 32 + 8 * g4 + 4 * (lane >> 5));
                        sc[4 * g4] = q.x; sc[4 * g4 + 1] = q.y; sc[4 * g4 + 2] = q.z; sc[4 * g4 + 3] = q.w;
                    }
#pragma unroll
                    for (int j = 0; j < TM; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][j][v] = __builtin_fmaf(sc[v], blk[i][j][v], acc[i][j][v]);
                }
            }
        }
    };

    gload(pf0, 0);
    if (KT > 1) gload(pf1, 1);
    __syncthreads();                                   // LUTs ready
    store(pf0, 0);
    if (KT > 2) gload(pf0, 2);
    __syncthreads();                                   // tile 0 complete

    // store slot for tile t (set t % 2), then refill that set with tile t + 2
    auto store_slot = [&](Prefetch& pf, int t) {
        if (t < KT) {
            store(pf, t & 1);
            if (t + 2 < KT) gload(pf, t + 2);
        }
    };
    auto mfma_slot = [&](int t) {
        if (t < KT) {
            __builtin_amdgcn_s_setprio(1);
            mfma_tile(t & 1, t);
            __builtin_amdgcn_s_setprio(0);
        }
    };
    // two K-tiles per trip so that the prefetch sets are addressed statically
    if (grp == 0) {
        for (int i = 0; i < KT; i += 2) {
            mfma_slot(i);
            __syncthreads();
            store_slot(pf1, i + 1);
            __syncthreads();
            mfma_slot(i + 1);
            __syncthreads();
            store_slot(pf0, i + 2);
            __syncthreads();
        }
    } else {
        for (int i = 0; i < KT; i += 2) {
            store_slot(pf1, i + 1);
            __syncthreads();
            mfma_slot(i);
            __syncthreads();
            store_slot(pf0, i + 2);
            __syncthreads();
            mfma_slot(i + 1);
            __syncthreads();
        }
    }
    if (partial)
        store_tile_partial<TM, TN>(acc, m0 + wm * WTM, n0 + wn * WTN, m, n, partial + (int64_t)blockIdx.y * m * n, lane);
    else
        store_tile<TM, TN, AQ>(acc, w_ts, a_ts, m0 + wm * WTM, n0 + wn * WTN, m, n, y, ld_y, lane);
}

// ---------------------------------------------------------------------------------------------
// Weights straight from registers (bf16 activations only).  Wave w of a workgroup owns the 32
// weight rows n0 + 32 w .. + 31 against ALL 256 activation rows of the tile, so every packed
// weight is decoded by exactly one wave, in registers, into the MFMA "A" operand it is used in;
// only the activation tile is shared through LDS.  An MFMA sums over any 16 k as long as both
// operands agree on them: lane (r, h) takes the 32 codes k = 64 t + 32 h .. + 31 of its row -- 16
// bytes of codes plus two scale bytes per K-tile -- and step j of the tile uses its dword j, i.e.
// k = 64 t + 32 h + 8 j .. + 7, against the activation chunk 4 h + j of the staged row.
// Per step and wave: ~25 VALU ops of decode, 8 LDS fragment reads, 8 MFMAs.
//
// Everything that comes from global memory is copied global -> LDS by the load unit itself
// (global_load_lds: lane l's 16 bytes land at LDS base + 16 l; a 2-byte copy lands zero-extended at base + 4 l), S stages deep: the activation tile
// (256 rows x 64 k bf16, the xor swizzle of the staged rows applied by choosing which global chunk
// each lane fetches) and each wave's own packed codes and scale bytes, which the lane that requested
// them reads back one tile later.  So the K loop holds no register-returning global load, no LDS
// write and no address arithmetic for staging.  Three quarters through iteration t every wave waits
// (vmcnt) until its own copies for tile t + 1 have landed and (lgkmcnt) until its last fragment reads
// of tile t have returned, then meets the others at the iteration's one barrier: past it tile t + 1
// is complete in LDS and tile t's stage is free, so the wave requests tile t + S into that stage and,
// between the last five MFMAs of tile t, prepares tile t + 1 (LUT lookups, decode of step 0, the
// fragment reads of step 0).  The next iteration therefore starts with its operands on the way: with
// the barrier at the end of the iteration instead, all waves of a workgroup started every K-tile
// with an empty LDS queue at the same moment (2-4 % slower).
//
// KG = 2 (for problems with about one 256 x 128 tile per compute unit): eight waves as two K groups of
// four; group g runs the same loop over its half of the K-tiles with its own activation stages, both
// groups meet at the same barriers, and at the end the two partial sums of every output meet through
// LDS -- each wave finishes half of the 256 rows.  The sum of the two halves is rounded once more than
// a single pass over K would be (fp32), which is inside the output tolerance.
//
// LDS reads are inline assembly with hand-placed s_waitcnt lgkmcnt: the compiler cannot tell the
// stages apart, so before any LDS load it knows of it would wait for ALL outstanding copies, which
// would serialise the prefetch.  Each wait is tied to the registers it guards so that their consumers
// cannot be scheduled above it; sched_barrier keeps the hand-laid slices (one MFMA each) in order.
// GB: blocks of 2^lb = 32, 64 or 128 elements -- the lane's 32 codes of a K-tile share ONE scale byte, at
// byte (64 t + 32 h) >> lb = ((64 t) >> lb) + ((32 h) >> lb) of the row; it is copied with a 1-byte
// global -> LDS copy (lands zero-extended at base + 4 lane, measured) and used for both halves.
template <int NW, int S, int KG = 1, int MT = 8, bool GB = false>
__device__ __forceinline__ void gemm_rb_body(
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, const float* __restrict__ w_ts,
    float sv0, float sv1, int64_t n, int64_t k, const uint16_t* __restrict__ a, int64_t m,
    uint16_t* __restrict__ y, int64_t ld_y, int tile_m, int tile_n, float* __restrict__ partial = nullptr,
    int kslice = 0, int kt_per_slice = 0x7FFFFFFF, int lb = 4)
{
    // MT: 32-row activation groups per tile (8, or 4 / 2 for at most 128 / 64 activation rows)
    static_assert(MT == 8 || ((MT == 4 || MT == 2) && KG == 1), "activation tile height");
    constexpr int NWN = NW / KG;                        // waves side by side along N; KG groups of them split K
    constexpr int NT = 64 * NW, BM = 32 * MT, BN = 32 * NWN;
    constexpr int NU_A = BM * 8 / (64 * NWN);           // 1-KiB activation copies per wave and K-tile
    constexpr int D = S - 1;                            // tiles in flight ahead of the one being computed
    constexpr int L = NU_A + 2;                         // copy instructions per wave and K-tile
    constexpr int A_STAGE = BM * 128, B_CODES = NW * 1024, B_STAGE = NW * 1280;
    static_assert((BM * 8) % (64 * NWN) == 0, "activation tile must divide over the threads");
    static_assert(S >= 2 && S <= 4 && (D - 1) * L < 64, "stage count");
    static_assert(KG == 1 || (KG == 2 && S == 2 && NWN == 4), "K groups: two, of four waves, two stages each");

    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* As = smem;                                 // KG x S stages x 256 rows x 128 B
    uint8_t* Bs = smem + KG * S * A_STAGE;              // S stages x (NW KiB of codes + NW x 256 B of scale-byte pairs)
    uint2* wlut = reinterpret_cast<uint2*>(smem + KG * S * A_STAGE + S * B_STAGE);

    // the wave index is uniform: as a scalar it keeps the LDS destinations of the copies (M0) and the
    // base addresses below on the scalar unit
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / NWN, wn = wave % NWN;         // K group, position along N
    const int r = lane & 31, h = lane >> 5;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int KT = (int)((k + kBK - 1) / kBK);
    const int last = KT - 1;
    // This workgroup's K-tiles: slice kslice of the grid (kt_per_slice tiles; all of them without a
    // workspace), of which K group g computes tiles g KTH .. (g + 1) KTH - 1; tiles past the end of the
    // slice contribute zero weights
    const int kt0 = kslice * kt_per_slice;
    const int kend = (KT - kt0 < kt_per_slice) ? KT : kt0 + kt_per_slice;
    const int KTH = (kend - kt0 + KG - 1) / KG, kbase = kt0 + kg * KTH;

    int64_t wrow = n0 + 32 * wn + r;
    wrow = wrow < n ? wrow : n - 1;                     // rows past N re-read the last row, never stored
    const uint8_t* crow = w_codes + wrow * (k / 2) + 16 * h;
    const int64_t scale_ld = GB ? (k >> lb) : (k / 16);
    const uint32_t s_lane = GB ? ((32u * h) >> lb) : 2u * h;          // this lane's byte inside a K-tile's scale bytes
    const uint8_t* srow = w_scales + wrow * scale_ld + s_lane;
    // the same addresses as a uniform base (first row of the wave, advanced per K-tile on the scalar
    // unit) plus a 32-bit lane offset that never changes: a full K-tile's copies need no vector
    // address arithmetic at all
    const int64_t wrow_first = (n0 + 32 * wn < n) ? n0 + 32 * wn : n - 1;
    const uint8_t* cfirst = w_codes + wrow_first * (k / 2);
    const uint8_t* sfirst = w_scales + wrow_first * scale_ld;
    const uint32_t c_off = (uint32_t)(wrow - wrow_first) * (uint32_t)(k / 2) + 16u * h;
    const uint32_t s_off = (uint32_t)(wrow - wrow_first) * (uint32_t)scale_ld + s_lane;

    // Activation copy i of this wave fills LDS rows 8 (wave NU_A + i) .. + 7 of a stage: lane l writes
    // physical chunk l % 8 of row 8 (..) + l / 8, which must hold logical chunk (l % 8) ^ swizzle(row).
    // Rows past M re-read the last row; byte offsets from the tile's first row fit 32 bits.
    const uint8_t* abase = reinterpret_cast<const uint8_t*>(a + m0 * k);
    const uint32_t rows_here = (uint32_t)((m - m0 < BM) ? m - m0 : BM);
    const uint32_t row_bytes = (uint32_t)k * 2u;
    uint32_t a_src[NU_A];                               // byte offset of (row, k = 0) + 16 * logical chunk
    uint32_t a_chunk[NU_A];
#pragma unroll
    for (int i = 0; i < NU_A; ++i) {
        const uint32_t row = 8u * (wn * NU_A + i) + (lane >> 3);
        const uint32_t c = (lane & 7u) ^ ((row >> 1) & 7u);
        a_chunk[i] = c;
        a_src[i] = (row < rows_here ? row : rows_here - 1) * row_bytes + c * 16u;
    }
    // all copies of K-tile kt into stage st (kt already clamped to the last tile by the caller)
    auto issue = [&](int kt, int st) {
        if ((int64_t)(kt + 1) * kBK <= k) {             // a full K-tile (uniform): scalar base + constant lane offsets
            const uint8_t* ab = abase + (size_t)kt * (kBK * 2);
#pragma unroll
            for (int i = 0; i < NU_A; ++i)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(ab + a_src[i]),
                    (__attribute__((address_space(3))) void*)(As + (kg * S + st) * A_STAGE + (wn * NU_A + i) * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(cfirst + (size_t)kt * 32 + c_off),
                                             (__attribute__((address_space(3))) void*)(Bs + st * B_STAGE + wave * 1024),
                                             16, 0, 0);
            if (GB)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(sfirst + (((size_t)kt * kBK) >> lb) + s_off),
                    (__attribute__((address_space(3))) void*)(Bs + st * B_STAGE + B_CODES + wave * 256), 1, 0, 0);
            else
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(sfirst + (size_t)kt * 4 + s_off),
                    (__attribute__((address_space(3))) void*)(Bs + st * B_STAGE + B_CODES + wave * 256), 2, 0, 0);
            return;
        }
#pragma unroll
        for (int i = 0; i < NU_A; ++i) {
            const uint32_t kk = (uint32_t)kt * kBK + a_chunk[i] * 8u;
            const uint32_t off = kk < (uint32_t)k ? a_src[i] + (uint32_t)kt * (kBK * 2u) : a_src[i] - a_chunk[i] * 16u;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(abase + off),           // past K: any finite data
                (__attribute__((address_space(3))) void*)(As + (kg * S + st) * A_STAGE + (wn * NU_A + i) * 1024), 16, 0, 0);
        }
        const int kc = ((int64_t)kt * kBK + 32 * h < k) ? kt : 0;                       // past K: masked where used
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(crow + 32 * kc),
                                         (__attribute__((address_space(3))) void*)(Bs + st * B_STAGE + wave * 1024),
                                         16, 0, 0);
        if (GB)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(srow + (((size_t)kc * kBK) >> lb)),
                (__attribute__((address_space(3))) void*)(Bs + st * B_STAGE + B_CODES + wave * 256), 1, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srow + 4 * kc),
                                             (__attribute__((address_space(3))) void*)(Bs + st * B_STAGE + B_CODES + wave * 256),
                                             2, 0, 0);
    };

    v16f acc[1][MT];
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[0][j][v] = 0.0f;

    const uint32_t a_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)As + kg * S * A_STAGE;
    const uint32_t lut_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)wlut;
    // this lane's own codes / scale bytes inside a B stage
    const uint32_t bc_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)Bs + wave * 1024 + lane * 16;
    const uint32_t bs_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)Bs + B_CODES + wave * 256 + lane * 4;
#define RAZER_LDS_READ128(dst, addr, imm) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm))
#define RAZER_LDS_READ64(dst, addr) asm volatile("ds_read_b64 %0, %1" : "=v"(dst) : "v"(addr))
#define RAZER_LDS_READ32(dst, addr) asm volatile("ds_read_b32 %0, %1" : "=v"(dst) : "v"(addr))
#define RAZER_LDS_WAIT(n, reg) asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+v"(reg))
#define RAZER_LDS_WAIT3(n, r0, r1, r2) asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+v"(r0), "+v"(r1), "+v"(r2))
    // the same with the count as a constant expression
    auto lds_wait = [](auto cnt, v4u& reg) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(reg) : "n"(decltype(cnt)::value)); };
    auto decode_pair = [](int p, uint32_t x, uint2 le) -> uint32_t {
        switch (p) {
            case 0: return cvt_scaled_pair<0>(x, u2f(le.x), le.y);
            case 1: return cvt_scaled_pair<1>(x, u2f(le.x), le.y);
            case 2: return cvt_scaled_pair<2>(x, u2f(le.x), le.y);
            default: return cvt_scaled_pair<3>(x, u2f(le.x), le.y);
        }
    };
    // LDS byte address of this lane's activation chunk in step j (row r of group 0, stage 0; group mi
    // adds 4096 mi, stage st adds st * A_STAGE)
    uint32_t aoff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) aoff[j] = a_lds + lds_off(r, 4 * h + j);
    // s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14, other counters left at max):
    // at most the copies of the D - 1 newest tiles are still in flight
    constexpr int kWaitN = (D - 1) * L;
    constexpr int kWaitImm = (kWaitN & 15) | ((kWaitN >> 4) << 14) | (7 << 4) | (15 << 8);

    // Weights of the tile about to be computed: sign-flipped codes, LUT entries of its two blocks,
    // decoded pairs of step 0.
    uint32_t xw[4], wq0[4];
    uint2 le0, le1;
    auto flip_and_mask = [&](int kt, const v4u& c, uint32_t& sc) {
        // past K: code 0, scale byte 0 -> weight 0
        const uint32_t msk = (kt < kend && (int64_t)kt * kBK + 32 * h < k) ? 0xFFFFFFFFu : 0u;
        xw[0] = (c.x & msk) ^ kRemapXor;
        xw[1] = (c.y & msk) ^ kRemapXor;
        xw[2] = (c.z & msk) ^ kRemapXor;
        xw[3] = (c.w & msk) ^ kRemapXor;
        if (GB) sc = (sc & 255u) * 0x101u;              // one scale byte for both halves
        sc &= msk;
    };

    // One K-tile.  Slices of one MFMA each; between the MFMAs of step j sit the fragment reads and
    // the decode for step j + 1 (4 code pairs spread over the MT slices), and in the last step the
    // preparation of tile kt + 1.  At the MFMA of (step j < 3, group mi) the MT fragment reads issued
    // after its own are the only LDS operations that may still be in flight, so lgkmcnt(MT - 1) is enough.
    v4u af[2][MT];                                      // af[0] enters compute() holding step 0 of its tile (requested, not yet waited for)
    auto compute = [&](int kt, int st, int st_next) {
        const uint32_t sbase = st * A_STAGE;
        uint32_t wq[2][4] = {{wq0[0], wq0[1], wq0[2], wq0[3]}, {0, 0, 0, 0}};
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int cb = j & 1, nb = cb ^ 1;
            const v8bf wf = __builtin_bit_cast(v8bf, make_uint4(wq[cb][0], wq[cb][1], wq[cb][2], wq[cb][3]));
            const uint2 le = (j + 1 < 2) ? le0 : le1;
            const uint32_t an = aoff[j + 1] + sbase;
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                RAZER_LDS_READ128(af[nb][mi], an, 4096 * mi);
                if (MT == 8) {                                           // one code pair per two MFMAs
                    if (mi % 2 == 0) wq[nb][mi / 2] = decode_pair(mi / 2, xw[j + 1], le);
                } else if (MT == 4) {
                    wq[nb][mi] = decode_pair(mi, xw[j + 1], le);
                } else {
                    wq[nb][2 * mi] = decode_pair(2 * mi, xw[j + 1], le);
                    wq[nb][2 * mi + 1] = decode_pair(2 * mi + 1, xw[j + 1], le);
                }
                lds_wait(std::integral_constant<int, MT - 1>{}, af[cb][mi]);
                acc[0][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, __builtin_bit_cast(v8bf, af[cb][mi]),
                                                                     acc[0][mi], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // this wave's copies for tile kt + 1 have landed
        __builtin_amdgcn_s_waitcnt(kWaitImm);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        {
            const v8bf wf = __builtin_bit_cast(v8bf, make_uint4(wq[1][0], wq[1][1], wq[1][2], wq[1][3]));
            const uint32_t bnext = st_next * B_STAGE;
            v4u cn;
            uint32_t sn;
            uint2 l0n, l1n;
#define RAZER_MFMA(mi) \
            acc[0][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, __builtin_bit_cast(v8bf, af[1][mi]), acc[0][mi], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0)
            // slice 0: request the next tile's codes and scale bytes (this lane's own copy); the first
            // MFMAs wait for their fragments only (MT + 2 LDS operations are in flight)
            constexpr int E = (MT == 8) ? 3 : 1;                         // MFMAs ahead of the barrier
            RAZER_LDS_READ128(cn, bc_lds + bnext, 0);
            RAZER_LDS_READ32(sn, bs_lds + bnext);
            lds_wait(std::integral_constant<int, MT + 1>{}, af[1][0]);
            RAZER_MFMA(0);
            if constexpr (MT == 8) {
                RAZER_LDS_WAIT(8, af[1][1]);
                RAZER_MFMA(1);
                RAZER_LDS_WAIT(7, af[1][2]);
                RAZER_MFMA(2);
            }
            // everything issued so far has returned -- this wave is done reading tile kt's stage, and it
            // has seen its own copies of tile kt + 1 land.  Once every wave is here, tile kt + 1 is
            // complete in LDS and tile kt's stage can be overwritten.  A bare barrier: __syncthreads()
            // would add a fence that waits for every outstanding copy, i.e. also for the tiles that are
            // meant to stay in flight.
            RAZER_LDS_WAIT3(0, af[1][E], cn, sn);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue(kt + S < last ? kt + S : last, st);
            flip_and_mask(kt + 1, cn, sn);
            RAZER_LDS_READ64(l0n, lut_lds + (sn & 255u) * 8u);
            RAZER_LDS_READ64(l1n, lut_lds + ((sn >> 8) & 255u) * 8u);
            // request step 0 of tile kt + 1 between the remaining MFMAs, so that the next iteration starts
            // with its fragments on the way instead of with an empty LDS queue
            const uint32_t a0n = aoff[0] + st_next * A_STAGE;
            if constexpr (MT == 8) {
                RAZER_LDS_READ128(af[0][0], a0n, 4096 * 0);
                RAZER_LDS_READ128(af[0][1], a0n, 4096 * 1);
                RAZER_MFMA(3);
                RAZER_LDS_READ128(af[0][2], a0n, 4096 * 2);
                RAZER_LDS_READ128(af[0][3], a0n, 4096 * 3);
                RAZER_LDS_READ128(af[0][4], a0n, 4096 * 4);
                RAZER_MFMA(4);
                RAZER_LDS_READ128(af[0][5], a0n, 4096 * 5);
                RAZER_LDS_READ128(af[0][6], a0n, 4096 * 6);
                RAZER_LDS_READ128(af[0][7], a0n, 4096 * 7);
                RAZER_MFMA(5);
            } else {
#pragma unroll
                for (int mi = 0; mi < MT; ++mi) RAZER_LDS_READ128(af[0][mi], a0n, 4096 * mi);
                if constexpr (MT == 4) { RAZER_MFMA(1); }
            }
            // decode step 0 of the next tile (the two table entries were requested before the MT
            // fragment reads)
            asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(l0n), "+v"(l1n), "+v"(af[1][MT - 1]) : "n"(MT));
            le0 = l0n;
            le1 = l1n;
            wq0[0] = cvt_scaled_pair<0>(xw[0], u2f(le0.x), le0.y);
            wq0[1] = cvt_scaled_pair<1>(xw[0], u2f(le0.x), le0.y);
            if constexpr (MT >= 4) { RAZER_MFMA(MT - 2); }
            wq0[2] = cvt_scaled_pair<2>(xw[0], u2f(le0.x), le0.y);
            wq0[3] = cvt_scaled_pair<3>(xw[0], u2f(le0.x), le0.y);
            RAZER_MFMA(MT - 1);
#undef RAZER_MFMA
        }
    };

    issue(kbase < last ? kbase : last, 0);              // (short K repeats the last tile)
    fill_scaled_lut<0>(wlut, sv0, sv1, tid, NT);
    __syncthreads();                                    // the first tile has landed, LUT ready
#pragma unroll
    for (int d = 1; d < S; ++d) issue(kbase + d < last ? kbase + d : last, d);
    {
        v4u c0;
        uint32_t s0;
        RAZER_LDS_READ128(c0, bc_lds, 0);
        RAZER_LDS_READ32(s0, bs_lds);
        RAZER_LDS_WAIT(0, c0);
        RAZER_LDS_WAIT(0, s0);
        flip_and_mask(kbase, c0, s0);
        RAZER_LDS_READ64(le0, lut_lds + (s0 & 255u) * 8u);
        RAZER_LDS_READ64(le1, lut_lds + ((s0 >> 8) & 255u) * 8u);
        RAZER_LDS_WAIT(0, le0);
        RAZER_LDS_WAIT(0, le1);
        wq0[0] = cvt_scaled_pair<0>(xw[0], u2f(le0.x), le0.y);
        wq0[1] = cvt_scaled_pair<1>(xw[0], u2f(le0.x), le0.y);
        wq0[2] = cvt_scaled_pair<2>(xw[0], u2f(le0.x), le0.y);
        wq0[3] = cvt_scaled_pair<3>(xw[0], u2f(le0.x), le0.y);
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) RAZER_LDS_READ128(af[0][mi], aoff[0], 4096 * mi);
    }
    int st = 0;                                         // stage of tile kt; tile kt + S follows it into the same stage
    for (int kt = kbase; kt < kbase + KTH; ++kt) {
        const int st_next = st == S - 1 ? 0 : st + 1;
        compute(kt, st, st_next);
        st = st_next;
    }
    // copies and fragment reads requested for tiles past the end: let them finish before the registers
    // and the stages they target are used for anything else
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef RAZER_LDS_READ128
#undef RAZER_LDS_READ64
#undef RAZER_LDS_READ32
#undef RAZER_LDS_WAIT
#undef RAZER_LDS_WAIT3
    if constexpr (KG == 1) {
        if (partial)                                    // K-slices of one output meet in the workspace [slice][m][n]
            store_tile_partial<MT, 1>(acc, m0, n0 + 32 * wave, m, n, partial + (int64_t)kslice * m * n, lane);
        else
            store_tile<MT, 1, false>(acc, w_ts, nullptr, m0, n0 + 32 * wave, m, n, y, ld_y, lane);
    } else {
        // The two K groups hold partial sums of the same 256 x 32 outputs.  Once every wave's copies have
        // landed and its fragment reads have returned (the wait above, then this barrier) the activation
        // stages are free: each wave hands the half of its accumulators that its partner (same rows, other
        // K group) will finish -- 16 KiB per wave, [group][4 registers][lane] -- and finishes the other half.
        __syncthreads();
        float4* mine = reinterpret_cast<float4*>(As + wave * 16384);
        const float4* theirs = reinterpret_cast<const float4*>(As + (wave ^ NWN) * 16384);
        v16f keep[1][MT / 2];
        if (kg == 0) {
#pragma unroll
            for (int j = 0; j < MT / 2; ++j) {
                keep[0][j] = acc[0][j];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    mine[(j * 4 + q) * 64 + lane] = make_float4(acc[0][MT / 2 + j][4 * q], acc[0][MT / 2 + j][4 * q + 1],
                                                                acc[0][MT / 2 + j][4 * q + 2], acc[0][MT / 2 + j][4 * q + 3]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < MT / 2; ++j) {
                keep[0][j] = acc[0][MT / 2 + j];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    mine[(j * 4 + q) * 64 + lane] = make_float4(acc[0][j][4 * q], acc[0][j][4 * q + 1],
                                                                acc[0][j][4 * q + 2], acc[0][j][4 * q + 3]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < MT / 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 t = theirs[(j * 4 + q) * 64 + lane];
                keep[0][j][4 * q] += t.x;
                keep[0][j][4 * q + 1] += t.y;
                keep[0][j][4 * q + 2] += t.z;
                keep[0][j][4 * q + 3] += t.w;
            }
        store_tile<MT / 2, 1, false>(keep, w_ts, nullptr, m0 + 128 * kg, n0 + 32 * wn, m, n, y, ld_y, lane);
    }
}

// Resident waves per SIMD the register budget is set for: 2 with the full 256-row tile (the accumulators
// alone are 128 registers), 3 / 4 with 128 / 64 rows.
template <int NW, int KG, int MT>
constexpr int rb_waves_per_simd() { return KG != 1 ? 1 : MT == 8 ? 8 / NW : MT == 4 ? 3 : 4; }

// grid = (output tiles, K-slices).  partial == nullptr: one slice, bf16 results to y; else slice
// blockIdx.y covers kt_per_slice K-tiles and leaves fp32 sums in partial[slice][m][n].
template <int NW, int S, int KG = 1, int MT = 8, bool GB = false>
__global__ __launch_bounds__(64 * NW, (rb_waves_per_simd<NW, KG, MT>())) void gemm_rb_kernel(
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, const float* __restrict__ w_ts,
    float sv0, float sv1, int64_t n, int64_t k, const uint16_t* __restrict__ a, int64_t m,
    uint16_t* __restrict__ y, int64_t ld_y, int tiles_m, float* __restrict__ partial, int kt_per_slice, int lb)
{
    gemm_rb_body<NW, S, KG, MT, GB>(w_codes, w_scales, w_ts, sv0, sv1, n, k, a, m, y, ld_y,
                                    (int)(blockIdx.x % tiles_m), (int)(blockIdx.x / tiles_m), partial,
                                    (int)blockIdx.y, kt_per_slice, lb);
}

// Up to four weight matrices against the same activations in one launch (fused q/k/v, gate/up): the
// column tiles of the matrices are numbered one after another, t1..t3 are the first tile of matrices
// 1..3 (equal to the total for matrices that are absent).  One launch fills the last round of
// workgroups better than one launch per matrix.
template <int NW, int S, int KG = 1, int MT = 8, bool GB = false>
__global__ __launch_bounds__(64 * NW, (rb_waves_per_simd<NW, KG, MT>())) void gemm_rb_grouped_kernel(
    const uint8_t* c0, const uint8_t* c1, const uint8_t* c2, const uint8_t* c3,
    const uint8_t* s0, const uint8_t* s1, const uint8_t* s2, const uint8_t* s3,
    const float* f0, const float* f1, const float* f2, const float* f3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3,
    int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3,
    int t1, int t2, int t3,
    float sv0, float sv1, int64_t k, const uint16_t* __restrict__ a, int64_t m, int tiles_m,
    float* __restrict__ partial, int kt_per_slice, int lb)
{
    const int tile_m = (int)(blockIdx.x % tiles_m), t = (int)(blockIdx.x / tiles_m);
    const uint8_t* codes = c0; const uint8_t* scales = s0; const float* ts = f0; uint16_t* y = y0;
    int64_t n = n0, ld = l0, before = 0;
    int first = 0;
    if (t >= t1) { codes = c1; scales = s1; ts = f1; y = y1; n = n1; ld = l1; first = t1; before = n0; }
    if (t >= t2) { codes = c2; scales = s2; ts = f2; y = y2; n = n2; ld = l2; first = t2; before = n0 + n1; }
    if (t >= t3) { codes = c3; scales = s3; ts = f3; y = y3; n = n3; ld = l3; first = t3; before = n0 + n1 + n2; }
    // with K-slices (partial != nullptr) matrix i keeps its [slices][m][n_i] sums behind those of matrices 0 .. i-1
    gemm_rb_body<NW, S, KG, MT, GB>(codes, scales, ts, sv0, sv1, n, k, a, m, y, ld, tile_m, t - first,
                                    partial ? partial + (int64_t)gridDim.y * m * before : nullptr, (int)blockIdx.y,
                                    kt_per_slice, lb);
}

// split > 1 (KG == 1 only, workspace of slices * m * n floats): K in slices of whole K-tiles, summed by
// launch_slice_reduce.
template <int NW, int S, int KG = 1, int MT = 8, bool GB = false>
static hipError_t launch_rb(const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts, SvConfig wcfg,
                            int64_t n, int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y,
                            hipStream_t st, int split = 1, float* workspace = nullptr)
{
    constexpr int BM = 32 * MT, BN = 32 * NW / KG;
    constexpr size_t smem = S * (KG * BM * 128 + NW * 1280) + 256 * sizeof(uint2);
    auto kern = gemm_rb_kernel<NW, S, KG, MT, GB>;
    RAZER_RAISE_LDS_LIMIT(kern, smem);
    if (KG != 1 || !workspace) split = 1;
    const int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    // every K-slice must hold at least one K-tile: slices = ceil(KT / ceil(KT / split))
    const int kt_all = (int)((k + kBK - 1) / kBK), kt_per = (kt_all + split - 1) / split;
    const int slices = (kt_all + kt_per - 1) / kt_per;
    launch(kern, dim3((unsigned)(tiles_m * tiles_n), (unsigned)slices), dim3(64 * NW), smem, st, w_codes, w_scales, w_ts, wcfg.sv0, wcfg.sv1, n, k, a, m, y, ld_y, tiles_m, slices > 1 ? workspace : nullptr,
        slices > 1 ? kt_per : 0x7FFFFFFF, wcfg.lb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    return launch_slice_reduce(workspace, w_ts, nullptr, m, n, slices, y, ld_y, st);
}

template <int BM, int BN, int WGM, int WGN, bool AQ, bool PP = false, bool GB = false, bool SF = false>
static hipError_t launch_cfg(const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts, SvConfig wcfg,
                             int64_t n, int64_t k, const uint16_t* a, const uint8_t* a_codes,
                             const uint8_t* a_scales, const float* a_ts, SvConfig acfg, int64_t m, uint16_t* y,
                             int64_t ld_y, int split, float* workspace, hipStream_t st)
{
    constexpr size_t smem = 2 * (BM + BN) * 128 + 2 * 256 * sizeof(uint2);
    void (*kern)(const uint8_t*, const uint8_t*, const float*, SvConfig, int64_t, int64_t, const uint16_t*,
                 const uint8_t*, const uint8_t*, const float*, SvConfig, int64_t, uint16_t*, int64_t, int, float*);
    if constexpr (PP) kern = gemm_pp_kernel<BM, BN, WGM, WGN, AQ, GB, SF>;
    else kern = gemm_kernel<BM, BN, WGM, WGN, AQ, GB, SF>;
    RAZER_RAISE_LDS_LIMIT(kern, smem);
    const int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    // every K-slice must hold at least one K-tile: slices = ceil(KT / ceil(KT / split))
    // (SF: an even number of K-tiles per slice; the kernel rounds its own share of the grid's slices the same way)
    const int kt_all = (int)((k + kBK - 1) / kBK), kt_raw = (kt_all + split - 1) / split;
    const int kt_per = SF ? ((kt_raw + 1) & ~1) : kt_raw;
    const int slices = (kt_all + kt_per - 1) / kt_per;
    launch(kern, dim3((unsigned)(tiles_m * tiles_n), (unsigned)slices), dim3(64 * WGM * WGN), smem, st, w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, tiles_m,
        slices > 1 ? workspace : nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    return launch_slice_reduce(workspace, w_ts, AQ ? a_ts : nullptr, m, n, slices, y, ld_y, st);
}

// Which kernel and how many K-slices.  Tiles: 0 = 32x256, 1 = 64x256, 2 = 128x128 (one stage pair, all
// waves alike), 3 = 256x256 and 4 = 256x128 (two wave groups out of phase), 5 / 6 = register-decode
// kernel with 256x256 / 256x128 tiles, 7 = register-decode kernel, 256x128 tiles, K halved inside
// the workgroup, 8 / 9 = register-decode kernel with 64x128 / 128x128 tiles and K-slices (33..64 /
// 65..128 activation rows: measured 1.3-2.1x faster than tiles 1 / 2 on 4096^2, 11008 x 4096 and
// 4096 x 11008).  A K-tile costs about 1 us of latency however small the tile, so
// when the output tiles cannot occupy the 256 compute units K is split until they do (at most 8 ways,
// at least 8 K-tiles per slice); the slices meet in the workspace.
struct GemmPlan {
    int tile;
    int split;
};
// K-slices of the register-decode kernel with small activation tiles: about one and a half workgroups
// per compute unit (best or within 5 % of it at 32, 86 and 172 tiles, K = 4096 and 11008), at least 8
// K-tiles per slice.
static int rb_split(int64_t tiles, int64_t kt_all, int64_t m = 0, int64_t rows = 0, int64_t k = 0)
{
    // the tuner's entry for (m, rows, k), if any: K-slices 1 .. 16, each at least one K-tile
    const TuneShape t = tuned_shape(kTuneGemmSlices, m, rows, k);
    if (t.source && t.p[0] >= 1 && t.p[0] <= 16 && t.p[0] <= kt_all) return t.p[0];
    int64_t split = (384 + tiles / 2) / tiles;
    if (split > 16) split = 16;
    if (split > kt_all / 8) split = kt_all / 8;
    return split >= 2 ? (int)split : 1;
}
static GemmPlan gemm_plan(int64_t m, int64_t n, int64_t k, bool register_decode_ok)
{
    GemmPlan p{0, 1};
    int64_t tiles;
    if (m > 32 && m <= 128 && register_decode_ok)
        return GemmPlan{m <= 64 ? 8 : 9, rb_split((n + 127) / 128, (k + kBK - 1) / kBK, m, n, k)};
    if (m <= 32) { p.tile = 0; tiles = (n + 255) / 256; }
    else if (m <= 64) { p.tile = 1; tiles = (n + 255) / 256; }
    else if (m <= 128) { p.tile = 2; tiles = ((m + 127) / 128) * ((n + 127) / 128); }
    else {
        // 256-row activation tiles so every weight is decoded once per 256 rows
        const int64_t tm = (m + 255) / 256;
        const int64_t t256 = tm * ((n + 255) / 256), t128 = tm * ((n + 127) / 128);
        // enough tiles for two resident waves per SIMD: the kernel that decodes weights in registers
        // (measured 5-28 % faster than the LDS-staged one on the 7B projection shapes from M = 2048)
        // (256-wide weight tiles from four rounds of workgroups up, or when they fill whole rounds: 4 % over
        // the 128-wide ones on 4096 x 8192 x 8192)
        if (register_decode_ok && (t256 >= 1024 || (t256 >= 512 && t256 % 256 == 0))) return GemmPlan{5, 1};
        if (register_decode_ok && t128 >= 512) return GemmPlan{6, 1};
        // one round of 256x128 tiles (one workgroup per compute unit): the register-decode kernel with
        // two K groups of four waves keeps two waves on every SIMD (measured 9-10 % over the LDS-staged
        // kernel on 2048 x 4096 x {4096, 11008}; slower than it when the tiles need a second round)
        if (register_decode_ok && t128 >= 192 && t128 <= 256 && k >= 16 * kBK) return GemmPlan{7, 1};
        // else the weight-tile width that wastes fewer compute units in the last round of workgroups
        auto eff = [](int64_t t) { return (double)t / (double)(((t + 255) / 256) * 256); };
        if (eff(t256) >= eff(t128)) { p.tile = 3; tiles = t256; }
        else { p.tile = 4; tiles = t128; }
    }
    const int64_t kt_all = (k + kBK - 1) / kBK;
    int64_t split = 256 / tiles;
    if (split > 8) split = 8;
    if (split > kt_all / 8) split = kt_all / 8;
    p.split = split >= 2 ? (int)split : 1;
    return p;
}

size_t gemm_workspace_bytes(int64_t n, int64_t k, int64_t m)
{
    if (n == 0 || k == 0) return 0;
    if (m <= kSkinnyMaxM && k <= kSkinnyMaxK) return 0;          // the small-batch kernel's range (W4A4 there runs unsplit)
    // the caller of this query does not say which operand formats it will pass: the larger of the
    // two plans (register-decode kernel allowed or not)
    size_t need = 0;
    for (int rd = 0; rd < 2; ++rd) {
        const GemmPlan p = gemm_plan(m, n, k, rd != 0 && k <= kRbMaxK);
        if (p.split == 1) continue;
        const int64_t kt_all = (k + kBK - 1) / kBK, kt_per = (kt_all + p.split - 1) / p.split;
        const int64_t slices = (kt_all + kt_per - 1) / kt_per;
        const size_t b = (size_t)(slices * m * n) * sizeof(float);
        need = b > need ? b : need;
    }
    return need;
}

template <bool AQ, bool GB>
static hipError_t launch_gemm_t(const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts, SvConfig wcfg,
                                int64_t n, int64_t k, const uint16_t* a, const uint8_t* a_codes,
                                const uint8_t* a_scales, const float* a_ts, SvConfig acfg, int64_t m, uint16_t* y,
                                int64_t ld_y, float* workspace, hipStream_t st)
{
    // (the register-decode kernel takes every weight block size; GB here also covers the activation
    // operand of W4A4, which that kernel does not decode)
    GemmPlan p = gemm_plan(m, n, k, !AQ && k <= kRbMaxK);
    if ((m <= kSkinnyMaxM && k <= kSkinnyMaxK) || !workspace) p.split = 1;   // not sized a workspace
#define RAZER_GEMM(BM, BN, WGM, WGN, PP) \
    launch_cfg<BM, BN, WGM, WGN, AQ, PP, GB>(w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, p.split, workspace, st)
    switch (p.tile) {
        case 0: return RAZER_GEMM(32, 256, 1, 4, false);
        case 1: return RAZER_GEMM(64, 256, 1, 4, false);
        case 2: return RAZER_GEMM(128, 128, 2, 2, false);
        case 3: return RAZER_GEMM(256, 256, 2, 4, true);
        case 4: return RAZER_GEMM(256, 128, 4, 2, true);
        default: break;
    }
#undef RAZER_GEMM
    if constexpr (!AQ) {
        if (p.tile == 8) return launch_rb<4, 2, 1, 2, GB>(w_codes, w_scales, w_ts, wcfg, n, k, a, m, y, ld_y, st, p.split, workspace);
        if (p.tile == 9) return launch_rb<4, 2, 1, 4, GB>(w_codes, w_scales, w_ts, wcfg, n, k, a, m, y, ld_y, st, p.split, workspace);
        if (p.tile == 5) return launch_rb<8, 2, 1, 8, GB>(w_codes, w_scales, w_ts, wcfg, n, k, a, m, y, ld_y, st);
        if (p.tile == 7) return launch_rb<8, 2, 2, 8, GB>(w_codes, w_scales, w_ts, wcfg, n, k, a, m, y, ld_y, st);
        return launch_rb<4, 2, 1, 8, GB>(w_codes, w_scales, w_ts, wcfg, n, k, a, m, y, ld_y, st);
    }
    return hipErrorInvalidValue;
}

// The grouped launch uses the register-decode kernel only.  Above 128 activation rows the matrices
// together must offer the tile counts that kernel is chosen at (see gemm_plan); a weight-tile width that
// does not divide a matrix's rows just leaves its last tile partly empty.  From 33 to 128 rows it is the
// kernel of the single calls too, and the K-slices are chosen for the tiles of all matrices together.
// Returns 256 / 128 (tile width of the plain kernel), 129 (128-wide tiles, two K groups: one round of
// tiles on at least three quarters of the compute units), 2 / 4 / 8 (64 / 128 / 256 activation rows per
// tile, 128-wide, K-slices when the tiles are few) or 0 (no grouped launch).
static int grouped_tile_width(int count, const GemvProblem* p, int64_t m, int64_t k)
{
    if (m <= 32 || k > kRbMaxK) return 0;
    if (m <= 128) return m <= 64 ? 2 : 4;
    const int64_t tm = (m + 255) / 256;
    int64_t t256 = 0, t128 = 0;
    for (int i = 0; i < count; ++i) {
        t256 += tm * ((p[i].n + 255) / 256);
        t128 += tm * ((p[i].n + 127) / 128);
    }
    if (t256 >= 1024 || (t256 >= 512 && t256 % 256 == 0)) return 256;
    if (t128 >= 512) return 128;
    if (t128 >= 192 && t128 <= 256 && k >= 16 * kBK) return 129;
    return 8;                                           // fewer tiles, or between one and two rounds: K-slices
}
static int grouped_split(int count, const GemvProblem* p, int64_t m, int64_t k)
{
    const int w = grouped_tile_width(count, p, m, k);
    if (w != 2 && w != 4 && w != 8) return 1;
    int64_t tiles = 0, rows = 0;
    for (int i = 0; i < count; ++i) { tiles += (p[i].n + 127) / 128; rows += p[i].n; }
    if (m > 128) return rb_split(tiles * ((m + 32 * w - 1) / (32 * w)), (k + kBK - 1) / kBK);   // (not a tuned family)
    return rb_split(tiles * ((m + 32 * w - 1) / (32 * w)), (k + kBK - 1) / kBK, m, rows, k);
}
bool gemm_grouped_fits(int count, const GemvProblem* p, int64_t m, int64_t k)
{
    return count >= 1 && count <= 4 && grouped_tile_width(count, p, m, k) != 0;
}
size_t gemm_grouped_workspace_bytes(int count, const GemvProblem* p, int64_t m, int64_t k)
{
    const int split = grouped_split(count, p, m, k);
    if (split == 1) return 0;
    const int64_t kt_all = (k + kBK - 1) / kBK, kt_per = (kt_all + split - 1) / split;
    const int64_t slices = (kt_all + kt_per - 1) / kt_per;
    int64_t n_all = 0;
    for (int i = 0; i < count; ++i) n_all += p[i].n;
    return (size_t)(slices * m * n_all) * sizeof(float);
}

template <int NW, int S, int KG = 1, int MT = 8, bool GB = false>
static hipError_t launch_rb_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                                    int64_t m, hipStream_t st, int split = 1, float* workspace = nullptr)
{
    constexpr int BM = 32 * MT, BN = 32 * NW / KG;
    constexpr size_t smem = S * (KG * BM * 128 + NW * 1280) + 256 * sizeof(uint2);
    auto kern = gemm_rb_grouped_kernel<NW, S, KG, MT, GB>;
    RAZER_RAISE_LDS_LIMIT(kern, smem);
    if (KG != 1 || !workspace) split = 1;
    const int tiles_m = (int)((m + BM - 1) / BM);
    const int kt_all = (int)((k + kBK - 1) / kBK), kt_per = (kt_all + split - 1) / split;
    const int slices = (kt_all + kt_per - 1) / kt_per;
    GemvProblem q[4];
    int t[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        q[i] = p[i < count ? i : count - 1];
        t[i + 1] = t[i] + (i < count ? (int)((q[i].n + BN - 1) / BN) : 0);
    }
    launch(kern, dim3((unsigned)(tiles_m * t[4]), (unsigned)slices), dim3(64 * NW), smem, st, q[0].codes, q[1].codes, q[2].codes, q[3].codes, q[0].scales, q[1].scales, q[2].scales, q[3].scales, q[0].ts,
        q[1].ts, q[2].ts, q[3].ts, q[0].y, q[1].y, q[2].y, q[3].y, q[0].n, q[1].n, q[2].n, q[3].n, q[0].ld_y,
        q[1].ld_y, q[2].ld_y, q[3].ld_y, t[1], t[2], t[3], cfg.sv0, cfg.sv1, k, a, m, tiles_m,
        slices > 1 ? workspace : nullptr, slices > 1 ? kt_per : 0x7FFFFFFF, cfg.lb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    return launch_slice_reduce_grouped(workspace, count, p, m, slices, st);
}

template <bool GB>
static hipError_t launch_gemm_grouped_t(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                                        int64_t m, float* workspace, hipStream_t st)
{
    const int w = grouped_tile_width(count, p, m, k);
    if (w == 256) return launch_rb_grouped<8, 2, 1, 8, GB>(cfg, count, p, k, a, m, st);
    if (w == 128) return launch_rb_grouped<4, 2, 1, 8, GB>(cfg, count, p, k, a, m, st);
    if (w == 129) return launch_rb_grouped<8, 2, 2, 8, GB>(cfg, count, p, k, a, m, st);
    if (w == 2 || w == 4 || w == 8) {
        const int split = grouped_split(count, p, m, k);
        if (split > 1 && !workspace) return hipErrorInvalidValue;
        if (w == 2) return launch_rb_grouped<4, 2, 1, 2, GB>(cfg, count, p, k, a, m, st, split, workspace);
        if (w == 4) return launch_rb_grouped<4, 2, 1, 4, GB>(cfg, count, p, k, a, m, st, split, workspace);
        return launch_rb_grouped<4, 2, 1, 8, GB>(cfg, count, p, k, a, m, st, split, workspace);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                               int64_t m, float* workspace, hipStream_t st)
{
    if (count < 1 || count > 4 || cfg.f16) return hipErrorInvalidValue;
    return cfg.lb == 4 ? launch_gemm_grouped_t<false>(cfg, count, p, k, a, m, workspace, st)
                       : launch_gemm_grouped_t<true>(cfg, count, p, k, a, m, workspace, st);
}

// The FP16-scale weight format on the tiled kernels (bf16 activations; the host sends up to 64 activation rows
// to the small-batch kernel): bare FP4 operands and per-block folds on the single-group kernel (32-, 64-, 128-row
// tiles) and, above 128 rows, on the two-group kernel (256 x 128 tiles).  With a workspace, K is cut into slices
// of whole blocks while the tiles are fewer than the compute units (the rule of gemm_plan, whose tiles are never
// smaller than these, so gemm_workspace_bytes covers it).
static int f16_split(int64_t m, int64_t n, int64_t k)
{
    const int64_t tiles = m <= 64 ? (n + 255) / 256 : m <= 128 ? (n + 127) / 128 : ((m + 255) / 256) * ((n + 127) / 128);
    const int64_t kt_all = (k + kBK - 1) / kBK;
    int64_t split = 256 / tiles;
    if (split > 8) split = 8;
    if (split > kt_all / 8) split = kt_all / 8;
    return split >= 2 ? (int)split : 1;
}
static hipError_t launch_gemm_f16(SvConfig wcfg, const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts,
                                  int64_t n, int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y,
                                  float* workspace, hipStream_t st)
{
    const SvConfig none{5.0f, 5.0f};
    const int split = workspace ? f16_split(m, n, k) : 1;
#define RAZER_GEMM_F16(BM, BN, WGM, WGN, PP) \
    launch_cfg<BM, BN, WGM, WGN, false, PP, false, true>(w_codes, w_scales, w_ts, wcfg, n, k, a, nullptr, nullptr, nullptr, none, m, y, ld_y, split, workspace, st)
    if (m <= 32) return RAZER_GEMM_F16(32, 256, 1, 4, false);
    if (m <= 64) return RAZER_GEMM_F16(64, 256, 1, 4, false);
    if (m <= 128) return RAZER_GEMM_F16(128, 128, 2, 2, false);
    // above 128 rows: 256 x 128 tiles on the two-group kernel (decode of one K-tile under the matrix instructions
    // of the other)
    return RAZER_GEMM_F16(256, 128, 4, 2, true);
#undef RAZER_GEMM_F16
}

hipError_t launch_gemm(SvConfig wcfg, const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts,
                       int64_t n, int64_t k, const uint16_t* a, SvConfig acfg, const uint8_t* a_codes,
                       const uint8_t* a_scales, const float* a_ts, int64_t m, uint16_t* y, int64_t ld_y,
                       float* workspace, hipStream_t st)
{
    if (n == 0 || m == 0) return hipSuccess;
    if (wcfg.f16) {
        if (a_codes || !a) return hipErrorInvalidValue;
        return launch_gemm_f16(wcfg, w_codes, w_scales, w_ts, n, k, a, m, y, ld_y, workspace, st);
    }
    // blocks of 32, 64, 128 (either operand) take the variants whose scale-byte loads index by block
    const bool generic = wcfg.lb != 4 || (a_codes && acfg.lb != 4);
#define RAZER_GEMM_ARGS w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, workspace, st
    if (a_codes) return generic ? launch_gemm_t<true, true>(RAZER_GEMM_ARGS) : launch_gemm_t<true, false>(RAZER_GEMM_ARGS);
    return generic ? launch_gemm_t<false, true>(RAZER_GEMM_ARGS) : launch_gemm_t<false, false>(RAZER_GEMM_ARGS);
#undef RAZER_GEMM_ARGS
}

}  // namespace razer
