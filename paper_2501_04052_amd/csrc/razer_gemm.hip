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
// consecutive n of one output row and stores them as one 8-byte write.
#include "razer_device.hpp"
#include "razer_kernels.hpp"

namespace razer {

constexpr int kBK = 64;

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

template <int BM, int BN, int WGM, int WGN, bool AQ>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, const float* __restrict__ w_ts,
    SvConfig wcfg, int64_t n, int64_t k, const uint16_t* __restrict__ a, const uint8_t* __restrict__ a_codes,
    const uint8_t* __restrict__ a_scales, const float* __restrict__ a_ts, SvConfig acfg, int64_t m,
    uint16_t* __restrict__ y, int64_t ld_y, int tiles_m)
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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int KT = (int)((k + kBK - 1) / kBK);

    fill_scaled_lut<0>(wlut, wcfg.sv0, wcfg.sv1, tid, NT);
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
        const int64_t kbase = (int64_t)kt * kBK;
        if (AQ) {
#pragma unroll
            for (int i = 0; i < NU_A; ++i) {
                const int u = tid + i * NT, row = u >> 1, half = u & 1;
                const int64_t gr = m0 + row, kk = kbase + half * 32;
                ra[i] = make_uint4(0, 0, 0, 0);
                rsa[i] = 0;
                if (u < BM * 2 && gr < m && kk < k) {
                    ra[i] = *reinterpret_cast<const uint4*>(a_codes + gr * (k / 2) + kk / 2);
                    rsa[i] = *reinterpret_cast<const uint16_t*>(a_scales + gr * (k / 16) + kk / 16);
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
                rsb[i] = *reinterpret_cast<const uint16_t*>(w_scales + gr * (k / 16) + kk / 16);
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
                const uint2 le = wlut[(rsb[i] >> (8 * (q >> 1))) & 255u];
                *reinterpret_cast<uint4*>(bs + lds_off(row, half * 4 + q)) = decode_dword(x, le);
            }
        }
    };

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
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
            if (more) store_part(st ^ 1, ks);
        }
        __syncthreads();
    }

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
template <int BM, int BN, int WGM, int WGN, bool AQ>
__global__ __launch_bounds__(512) void gemm_pp_kernel(
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, const float* __restrict__ w_ts,
    SvConfig wcfg, int64_t n, int64_t k, const uint16_t* __restrict__ a, const uint8_t* __restrict__ a_codes,
    const uint8_t* __restrict__ a_scales, const float* __restrict__ a_ts, SvConfig acfg, int64_t m,
    uint16_t* __restrict__ y, int64_t ld_y, int tiles_m)
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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = wave >> 2, gt = tid & (GT - 1);
    const int wm = wave % WGM, wn = wave / WGM;
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int KT = (int)((k + kBK - 1) / kBK);

    fill_scaled_lut<0>(wlut, wcfg.sv0, wcfg.sv1, tid, 512);
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
        const int64_t kbase = (int64_t)kt * kBK;
        if (AQ) {
#pragma unroll
            for (int i = 0; i < A_PT; ++i) {
                const int u = gt + i * GT, row = grp * (BM / 2) + (u >> 2), blk = u & 3;
                const int64_t gr = m0 + row, kk = kbase + blk * 16;
                pf.rqa[i] = make_uint2(0, 0);
                pf.rsa[i] = 0;
                if (gr < m && kk < k) {
                    pf.rqa[i] = *reinterpret_cast<const uint2*>(a_codes + gr * (k / 2) + kk / 2);
                    pf.rsa[i] = a_scales[gr * (k / 16) + kk / 16];
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
                    pf.rsb[i] = *reinterpret_cast<const uint16_t*>(w_scales + gr * (k / 16) + kk / 16);
                } else {
                    const uint2 t2 = *reinterpret_cast<const uint2*>(w_codes + gr * (k / 2) + kk / 2);
                    pf.rb[i].x = t2.x;
                    pf.rb[i].y = t2.y;
                    pf.rsb[i] = w_scales[gr * (k / 16) + kk / 16];
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
    auto mfma_tile = [&](int st) {
        const uint8_t* as = As + st * BM * 128;
        const uint8_t* bs = Bs + st * BN * 128;
        // operand fragments are fetched DEPTH k-steps ahead of the MFMAs that use them
        constexpr int DEPTH = (TM + TN <= 4) ? 4 : 2;
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
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks % DEPTH][i], fa[ks % DEPTH][j], acc[i][j], 0, 0, 0);
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
            mfma_tile(t & 1);
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
    store_tile<TM, TN, AQ>(acc, w_ts, a_ts, m0 + wm * WTM, n0 + wn * WTN, m, n, y, ld_y, lane);
}

template <int BM, int BN, int WGM, int WGN, bool AQ, bool PP = false>
static hipError_t launch_cfg(const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts, SvConfig wcfg,
                             int64_t n, int64_t k, const uint16_t* a, const uint8_t* a_codes,
                             const uint8_t* a_scales, const float* a_ts, SvConfig acfg, int64_t m, uint16_t* y,
                             int64_t ld_y, hipStream_t st)
{
    constexpr size_t smem = 2 * (BM + BN) * 128 + 2 * 256 * sizeof(uint2);
    void (*kern)(const uint8_t*, const uint8_t*, const float*, SvConfig, int64_t, int64_t, const uint16_t*,
                 const uint8_t*, const uint8_t*, const float*, SvConfig, int64_t, uint16_t*, int64_t, int);
    if constexpr (PP) kern = gemm_pp_kernel<BM, BN, WGM, WGN, AQ>;
    else kern = gemm_kernel<BM, BN, WGM, WGN, AQ>;
    static bool attr_set = false;                      // one GPU per process
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WGM * WGN), smem, st>>>(
        w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, tiles_m);
    return hipGetLastError();
}

template <bool AQ>
static hipError_t launch_gemm_t(const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts, SvConfig wcfg,
                                int64_t n, int64_t k, const uint16_t* a, const uint8_t* a_codes,
                                const uint8_t* a_scales, const float* a_ts, SvConfig acfg, int64_t m, uint16_t* y,
                                int64_t ld_y, hipStream_t st)
{
#define RAZER_GEMM(BM, BN, WGM, WGN) \
    launch_cfg<BM, BN, WGM, WGN, AQ>(w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, st)
    if (m <= 32) return RAZER_GEMM(32, 256, 1, 4);
    if (m <= 64) return RAZER_GEMM(64, 256, 1, 4);
    if (m <= 128) return RAZER_GEMM(128, 128, 2, 2);
    // Large m: 256-row activation tiles so every weight is decoded once per 256 rows.  Pick the
    // weight-tile width that wastes fewer of the 256 compute units in the last round of workgroups.
    const int64_t tm = (m + 255) / 256;
    const int64_t t256 = tm * ((n + 255) / 256), t128 = tm * ((n + 127) / 128);
    auto eff = [](int64_t tiles) { return (double)tiles / (double)(((tiles + 255) / 256) * 256); };
#define RAZER_GEMM_PP(BM, BN, WGM, WGN) \
    launch_cfg<BM, BN, WGM, WGN, AQ, true>(w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, st)
    if (eff(t256) >= eff(t128)) return RAZER_GEMM_PP(256, 256, 2, 4);
    return RAZER_GEMM_PP(256, 128, 4, 2);
#undef RAZER_GEMM_PP
#undef RAZER_GEMM
}

hipError_t launch_gemm(SvConfig wcfg, const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts,
                       int64_t n, int64_t k, const uint16_t* a, SvConfig acfg, const uint8_t* a_codes,
                       const uint8_t* a_scales, const float* a_ts, int64_t m, uint16_t* y, int64_t ld_y,
                       hipStream_t st)
{
    if (n == 0 || m == 0) return hipSuccess;
    if (a_codes)
        return launch_gemm_t<true>(w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, st);
    return launch_gemm_t<false>(w_codes, w_scales, w_ts, wcfg, n, k, a, a_codes, a_scales, a_ts, acfg, m, y, ld_y, st);
}

}  // namespace razer
