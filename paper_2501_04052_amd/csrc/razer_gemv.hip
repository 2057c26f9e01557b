// Weight-only RaZeR linear layer for 1..4 activation rows on gfx950 (the decode
// regime of Sec. 4.3 / App. D.2 of arxiv 2501.04052): fused decode + dot product,
// bound by the HBM read of the packed weights (0.5625 B per weight).
//
// Mapping.  A workgroup owns a few consecutive weight rows; its waves split K into
// slices of 2048 elements.  In a slice lane l owns the 16-byte code chunk
// [32 l, 32 l + 32) of every row -- so a wave reads 1 KiB of consecutive codes
// and 128 B of consecutive scale bytes per row -- and keeps the matching 32
// activations of each activation row in registers across the rows.  Kernels
// this short are latency-bound (about 3 us of every launch is fixed cost on
// MI355X, the rest streams at 5-6 TB/s): loads are issued before anything else
// happens, the whole problem is in flight at once, and nothing in the kernel may
// touch the dispatch packet or scratch.  Rows up to 32768 elements take the
// streaming kernel (groups of 2 rows, next group in flight while one is decoded);
// longer rows take the multi-pass kernel (4 rows per workgroup).
//
// Two to four activation rows (every block size and weight format) take a variant of the streaming kernel
// that multiplies on the 4x4x4 matrix instruction (gemv_quad_kernel, further down): with v_dot2 every activation row
// costs another half operation per weight and the kernel turns VALU-bound.
//
// Decode.  The 8 codes of a dword are sign-flipped with one xor, converted to
// packed bf16 pairs by the hardware FP4 conversion, and the (now all-zero)
// remapped slots are patched with the block's special value by two packed
// 16-bit integer ops.  Pairs go straight into v_dot2_f32_bf16 against the
// activation pairs; the block scale (negated, undoing the sign flip) multiplies
// the 16-element partial sum once per block.
#include "razer_device.hpp"
#include "razer_kernels.hpp"

namespace razer {

constexpr int kSliceK = 2048;          // K elements one wave covers per pass: 64 lanes x 32 codes
constexpr int kMaxWaves = 16;

// Per scale byte: { -block_scale (fp32 bits), negated special value as a bf16 pair }.
__device__ __forceinline__ void fill_weight_lut(uint2* lut, float sv0, float sv1)
{
    for (uint32_t sb = threadIdx.x; sb < 256u; sb += blockDim.x) {
        float s, sv;
        decode_scale_byte<0>(sb, sv0, sv1, s, sv);
        const uint32_t nsv = (uint32_t)f32_to_bf16_rne(-sv);              // exact: multiples of 0.5 below 16
        lut[sb] = make_uint2(f2u(-s), nsv | (nsv << 16));
    }
}

template <int BYTE>
__device__ __forceinline__ uint32_t cvt_pair(uint32_t x)
{
    v2bf p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(x, 1.0f, BYTE);
    return __builtin_bit_cast(uint32_t, p);
}
__device__ __forceinline__ float dot2(uint32_t w, uint32_t a, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, w), __builtin_bit_cast(v2bf, a), acc, false);
}

// Registers one lane holds for one group of R rows: 16 bytes of codes and 2 scale bytes per row.
template <int R>
struct RowGroup {
    uint4 cw[R];
    uint32_t sw[R];
};

// SF = 0: scale bytes, looked up in the LDS table (decoding them in registers instead was measured
// 12-20 % slower for blocks of 16 and no faster for larger blocks: these kernels feel every VALU op).
// SF = 1: the FP16-scale format (one 16-bit word per 128 elements) -- sw holds the word of the block
// that contains this lane's 32 elements; a half converts to fp32 in one instruction, no table.
template <bool GB, int SF>
__device__ __forceinline__ uint32_t load_scale_bits(const uint8_t* __restrict__ scales, int64_t row, int64_t k,
                                                    int64_t k0, int lb)
{
    if (SF == 1) return reinterpret_cast<const uint16_t*>(scales)[row * (k >> 7) + (k0 >> 7)];
    // GB kernels are launched for blocks of 32 and more only: the 32 elements share one scale byte
    // (no run-time choice between two load widths, which would put a branch between the loads)
    if (GB) return scales[row * (k >> lb) + (k0 >> lb)];
    return load_scale_pair<false>(scales + row * (k >> 4), k0, 4);
}

template <int R, bool GB, int SF>
__device__ __forceinline__ void load_group(RowGroup<R>& g, const uint8_t* __restrict__ codes,
                                           const uint8_t* __restrict__ scales, int64_t row0, int64_t n,
                                           int64_t k, int64_t c, int lb)
{
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t row = (row0 + r < n) ? row0 + r : n - 1;           // clamp: tail rows re-read the last row
        g.cw[r] = load_once16(codes + row * (k / 2) + c * 16);
        g.sw[r] = load_scale_bits<GB, SF>(scales, row, k, c * 32, lb);
    }
}

// sum_k a[m][k] * (scale * element) over this lane's 32 k's, for the R rows of a group.
// ONE: the 32 elements share one scale (blocks of 32 and more, the FP16-scale format) -- one table
// lookup or conversion and one multiplication by the scale per row instead of two.
template <int M, int R, int SF = 0, bool ONE = false>
__device__ __forceinline__ void dot_group(const RowGroup<R>& g, const uint4 (&av)[M][4], const uint2* lut,
                                          float (&acc)[R][M], float sv0 = 0.0f, float sv1 = 0.0f)
{
    constexpr int NBLK = ONE ? 1 : 2, NH = ONE ? 4 : 2;                   // scales per lane, dwords of codes per scale
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t xw[4] = {g.cw[r].x, g.cw[r].y, g.cw[r].z, g.cw[r].w};
#pragma unroll
        for (int m = 0; m < M; ++m) acc[r][m] = 0.0f;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            uint2 le;
            if (SF == 1) {
                float s, sv;
                decode_scale_word(g.sw[r], sv0, sv1, s, sv);
                const uint32_t nsv = (uint32_t)f32_to_bf16_rne(-sv);
                le = make_uint2(f2u(-s), nsv | (nsv << 16));
            } else {
                le = lut[(g.sw[r] >> (8 * blk)) & 255u];
            }
            const float ns = u2f(le.x);
            float p[M];
#pragma unroll
            for (int m = 0; m < M; ++m) p[m] = 0.0f;
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const uint32_t x = xw[NH * blk + h] ^ kRemapXor;
                const uint32_t w0 = patch_zero_halves(cvt_pair<0>(x), le.y);
                const uint32_t w1 = patch_zero_halves(cvt_pair<1>(x), le.y);
                const uint32_t w2 = patch_zero_halves(cvt_pair<2>(x), le.y);
                const uint32_t w3 = patch_zero_halves(cvt_pair<3>(x), le.y);
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    const uint4 aq = av[m][NH * blk + h];
                    p[m] = dot2(w0, aq.x, p[m]);
                    p[m] = dot2(w1, aq.y, p[m]);
                    p[m] = dot2(w2, aq.z, p[m]);
                    p[m] = dot2(w3, aq.w, p[m]);
                }
            }
#pragma unroll
            for (int m = 0; m < M; ++m) acc[r][m] = ONE ? ns * p[m] : __builtin_fmaf(ns, p[m], acc[r][m]);
        }
    }
}

// A workgroup owns R consecutive rows; wave w owns K-slice w (and w + waves, ... when K exceeds
// 2048 elements per wave).  All loads of a wave are issued up front, the rows are decoded, reduced
// over the 64 lanes and the slice totals parked in LDS; after one barrier the first threads add
// the slices and write bf16.  The grid is one workgroup per R rows: for the matrices of a decoder
// layer the whole problem is in flight at once, which is what hides the HBM latency.
template <int M, int R, bool GB = false, int SF = 0>
__device__ __forceinline__ void gemv_body(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                          const float* __restrict__ w_ts, float sv0, float sv1, int64_t n,
                                          int64_t k, const uint16_t* __restrict__ a, uint16_t* __restrict__ y,
                                          int64_t ld_y, int64_t row0, int lb = 4)
{
    __shared__ uint2 lut[256];
    __shared__ float part[kMaxWaves][R][M];
    const float ts = *w_ts;                                               // issued early, used last
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int64_t chunks = k / 32;                                        // 16-byte code chunks per row
    const int npass = (int)((chunks + 64 * nwaves - 1) / (64 * nwaves));  // > 1 only when K > 2048 * waves

    // first pass: loads go out before the LUT is built
    int64_t c = (int64_t)wave * 64 + lane;
    bool active = c < chunks;
    int64_t cc = active ? c : 0;                                          // idle lanes read chunk 0, weight 0
    uint4 av[M][4];
    RowGroup<R> grp;
    auto issue_loads = [&]() {
        const uint32_t amask = active ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const uint4* ap = reinterpret_cast<const uint4*>(a + (int64_t)m * k + cc * 32);
#pragma unroll
            for (int j = 0; j < 4; ++j) {                                 // unconditional load, then mask:
                const uint4 t = ap[j];                                    // keeps the code branch-free
                av[m][j] = make_uint4(t.x & amask, t.y & amask, t.z & amask, t.w & amask);
            }
        }
        load_group<R, GB, SF>(grp, codes, scales, row0, n, k, cc, lb);
    };
    issue_loads();
    fill_weight_lut(lut, sv0, sv1);
    __syncthreads();                                                      // LUT ready

    float tot[R][M];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < M; ++m) tot[r][m] = 0.0f;
    for (int pass = 0; pass < npass; ++pass) {
        if (pass) {
            c = ((int64_t)pass * nwaves + wave) * 64 + lane;
            active = c < chunks;
            cc = active ? c : 0;
            issue_loads();
        }
        float acc[R][M];
        dot_group<M, R, SF, GB || SF == 1>(grp, av, lut, acc, sv0, sv1);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int m = 0; m < M; ++m) tot[r][m] += acc[r][m];
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const float t = wave_sum_to_lane63(tot[r][m]);
            if (lane == 63) part[wave][r][m] = t;
        }
    __syncthreads();
    if (threadIdx.x < R * M) {
        const int r = threadIdx.x / M, m = threadIdx.x - r * M;
        if (row0 + r < n) {
            float t = 0.0f;
            for (int w = 0; w < nwaves; ++w) t += part[w][r][m];
            y[(int64_t)m * ld_y + row0 + r] = f32_to_bf16_rne(t * ts);
        }
    }
}

// Streaming variant for rows of at most 16 slices (K <= 32768): a set of waves owns G consecutive
// groups of R rows (a workgroup holds P such sets side by side) and walks them with D register buffers, so that D - 1 groups of packed weights
// are always in flight while one is decoded.  Wave w owns K-slice w of every row; its 32
// activations per lane stay in registers for the whole walk.  Slice totals of all G * R rows meet
// in LDS after ONE barrier.  Row addresses are uniform (scalar) and lane offsets 32-bit.
// IL: the interleaved layout (razer_device.hpp): `codes` is the packed buffer, a wave's 2048-element run is
// 1152 contiguous bytes -- its 1 KiB of codes, then its 128 scale bytes.
template <int M, int R, int G, int D, int P = 1, bool GB = false, int SF = 0, bool IL = false>
__device__ __forceinline__ void gemv_stream_body(const uint8_t* __restrict__ codes,
                                                 const uint8_t* __restrict__ scales,
                                                 const float* __restrict__ w_ts, float sv0, float sv1, int64_t n,
                                                 int64_t k, const uint16_t* __restrict__ a,
                                                 uint16_t* __restrict__ y, int64_t ld_y, int64_t row0, int lb = 4)
{
    static_assert(D >= 2 && D <= 3, "buffer count");
    __shared__ uint2 lut[256];
    __shared__ float part[P * G * R * M][kMaxWaves / P];
    const float ts = *w_ts;
    // P sets of waves work side by side on P consecutive blocks of G * R rows (fewer, larger workgroups).
    // With one set and two groups the wave index is read as a scalar as well (measured 3-7 % faster on the
    // long launches of a 70B-shaped layer, slower with eight groups); with two sets at M = 1 it keeps the
    // row offsets on the scalar unit too (67 -> 60 vector registers, i.e. eight waves per SIMD; 0-1 % faster).
    static_assert(P == 1 || P == 2, "one or two sets of waves");
    const uint32_t lane = threadIdx.x & 63u, nwaves = (blockDim.x >> 6) / P;
    const uint32_t wid = ((P == 1 && G == 2) || (P == 2 && M == 1)) ? __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) : (threadIdx.x >> 6);
    const uint32_t par = (P == 2 && wid >= nwaves) ? 1u : 0u;             // (no division: a reciprocal sits ahead of the first load)
    const uint32_t wave = wid - par * nwaves;
    const uint32_t chunks = (uint32_t)(k >> 5);                           // 16-byte code chunks per row
    const uint32_t c = wave * 64u + lane;
    const bool active = c < chunks;
    // Idle lanes (K not a multiple of 2048) read chunk 0 of everything and get their scale bits
    // cleared: scale code 0 decodes to 0.0, so whatever they accumulate is multiplied by zero.
    const uint32_t cc = active ? c : 0u;
    const uint32_t smask = active ? 0xFFFFFFFFu : 0u;
    static_assert(!IL || (!GB && SF == 0), "interleaved layout: 16-element blocks, scale bytes");
    // Addresses: the workgroup's first row gives a uniform 64-bit base (scalar unit); a row of the workgroup
    // and the lane's place in it are a 32-bit offset from there (at most 15 rows of at most 18 KiB).  Rows
    // past N (last workgroup of a matrix) re-read the last row.
    const uint32_t code_ld = (uint32_t)(IL ? il_row_bytes(k) : (k >> 1));
    const uint32_t scale_ld = IL ? code_ld : (SF == 1) ? (uint32_t)(k >> 7) * 2u : GB ? (uint32_t)(k >> lb) : (uint32_t)(k >> 4);
    const uint32_t last_row = (uint32_t)((n - 1 - row0 < P * R * G - 1) ? n - 1 - row0 : P * R * G - 1);
    const uint8_t* cbase = codes + row0 * (int64_t)code_ld;
    const uint8_t* sbase = (IL ? codes : scales) + row0 * (int64_t)scale_ld;
    // the lane's byte offsets inside a row: its 16 bytes of codes, its scale bits
    const uint32_t c_lane = IL ? (cc >> 6) * kIlRun + (cc & 63u) * 16u : cc * 16u;
    const uint32_t s_lane = IL ? (cc >> 6) * kIlRun + 1024u + (cc & 63u) * 2u
                               : (SF == 1) ? ((cc * 32u) >> 7) * 2u : GB ? ((cc * 32u) >> lb) : cc * 2u;

    uint4 av[M][4];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const uint8_t* ap = reinterpret_cast<const uint8_t*>(a + (int64_t)m * k);
#pragma unroll
        for (int j = 0; j < 4; ++j) av[m][j] = *reinterpret_cast<const uint4*>(ap + (cc * 64u + 16u * j));
    }
    RowGroup<R> buf[D];
    auto load = [&](RowGroup<R>& g, int gi) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t rel = par * (R * G) + gi * R + r;
            const uint32_t row = rel < last_row ? rel : last_row;
            // (24-bit multiply-add: one 32-bit instruction.  The generic 32-bit form compiles to a 64-bit
            // multiply-add whose unused high input half the register allocator overlaps with a load in
            // flight, and the wave then waits for that load before it requests its weights.)
            g.cw[r] = load_once16(cbase + (__umul24(row, code_ld) + c_lane));
            const uint8_t* sp = sbase + (__umul24(row, scale_ld) + s_lane);
            if (GB && SF == 0) g.sw[r] = *sp & smask;                     // blocks of 32 and more: one scale byte
            else g.sw[r] = *reinterpret_cast<const uint16_t*>(sp) & smask;
        }
    };
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
        if (d < G) load(buf[d], d);
    if (SF == 0) {
        fill_weight_lut(lut, sv0, sv1);
        __syncthreads();                                                  // LUT ready
    }

    // Slice totals of a wave: with two wave sets per workgroup (the short launches of 7B-sized layers) they
    // go to scalar registers and lane i stores total i -- one masked LDS write per wave instead of one per
    // total (1.5-6 % on those launches; measured slower on the one-set kernels of longer rows, which keep
    // the write per total).
    constexpr int NV = G * R * M;
    constexpr bool ONE_WRITE = P == 2 && NV <= 8;
    float tot[ONE_WRITE ? NV : 1];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (g + D - 1 < G) load(buf[(g + D - 1) % D], g + D - 1);
        float acc[R][M];
        dot_group<M, R, SF, GB || SF == 1>(buf[g % D], av, lut, acc, sv0, sv1);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const float t = wave_sum_to_lane63(acc[r][m]);
                if (ONE_WRITE)                         // totals to scalar registers, one LDS write for all of them below
                    tot[(g * R + r) * M + m] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t), 63));
                else if (lane == 63)
                    part[((par * G + g) * R + r) * M + m][wave] = t;
            }
    }
    if (ONE_WRITE) {                                   // lane i writes total i: one masked store instead of NV
        float v = tot[0];
#pragma unroll
        for (int i = 1; i < NV; ++i) v = (lane == (uint32_t)i) ? tot[i] : v;
        if (lane < (uint32_t)NV) part[par * NV + lane][wave] = v;
    }
    __syncthreads();
    if (threadIdx.x < P * G * R * M) {
        const int m = threadIdx.x / (P * G * R), rr = threadIdx.x - m * (P * G * R);
        if (row0 + rr < n) {
            float t = 0.0f;
            for (uint32_t w = 0; w < nwaves; ++w) t += part[rr * M + m][w];
            y[(int64_t)m * ld_y + row0 + rr] = f32_to_bf16_rne(t * ts);
        }
    }
}

template <int M, int R, int G, int D, int P = 1, bool GB = false, int SF = 0, bool IL = false>
__global__ __launch_bounds__(64 * kMaxWaves) void gemv_stream_kernel(const uint8_t* __restrict__ codes,
                                                                     const uint8_t* __restrict__ scales,
                                                                     const float* __restrict__ w_ts, float sv0,
                                                                     float sv1, int64_t n, int64_t k,
                                                                     const uint16_t* __restrict__ a,
                                                                     uint16_t* __restrict__ y, int64_t ld_y, int lb)
{
    gemv_stream_body<M, R, G, D, P, GB, SF, IL>(codes, scales, w_ts, sv0, sv1, n, k, a, y, ld_y,
                                                (int64_t)blockIdx.x * (P * R * G), lb);
}

template <int M, int R, bool GB = false, int SF = 0>
__global__ __launch_bounds__(64 * kMaxWaves) void gemv_kernel(const uint8_t* __restrict__ codes,
                                                              const uint8_t* __restrict__ scales,
                                                              const float* __restrict__ w_ts, float sv0, float sv1,
                                                              int64_t n, int64_t k,
                                                              const uint16_t* __restrict__ a,
                                                              uint16_t* __restrict__ y, int64_t ld_y, int lb)
{
    gemv_body<M, R, GB, SF>(codes, scales, w_ts, sv0, sv1, n, k, a, y, ld_y, (int64_t)blockIdx.x * R, lb);
}

// Up to four weight matrices that share K, the activation rows and the special values, in one
// launch (fused q/k/v, gate/up): workgroups [0, g1) serve matrix 0, [g1, g2) matrix 1, ...  Every
// per-matrix argument is a scalar kernel argument picked with uniform compares: no indexed
// argument arrays, which would cost a private copy.
template <int M, int R, bool GB = false, int SF = 0>
__global__ __launch_bounds__(64 * kMaxWaves) void gemv_grouped_kernel(
    const uint8_t* c0, const uint8_t* c1, const uint8_t* c2, const uint8_t* c3,
    const uint8_t* s0, const uint8_t* s1, const uint8_t* s2, const uint8_t* s3,
    const float* t0, const float* t1, const float* t2, const float* t3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3,
    int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3,
    unsigned g1, unsigned g2, unsigned g3,
    float sv0, float sv1, int64_t k, const uint16_t* __restrict__ a, int lb)
{
    const unsigned b = blockIdx.x;
    const uint8_t* codes = c0; const uint8_t* scales = s0; const float* ts = t0; uint16_t* y = y0;
    int64_t n = n0, ld = l0;
    unsigned first = 0;
    if (b >= g1) { codes = c1; scales = s1; ts = t1; y = y1; n = n1; ld = l1; first = g1; }
    if (b >= g2) { codes = c2; scales = s2; ts = t2; y = y2; n = n2; ld = l2; first = g2; }
    if (b >= g3) { codes = c3; scales = s3; ts = t3; y = y3; n = n3; ld = l3; first = g3; }
    gemv_body<M, R, GB, SF>(codes, scales, ts, sv0, sv1, n, k, a, y, ld, (int64_t)(b - first) * R, lb);
}

template <int M, int R, int G, int D, int P = 1, bool GB = false, int SF = 0, bool IL = false>
__global__ __launch_bounds__(64 * kMaxWaves) void gemv_stream_grouped_kernel(
    const uint8_t* c0, const uint8_t* c1, const uint8_t* c2, const uint8_t* c3,
    const uint8_t* s0, const uint8_t* s1, const uint8_t* s2, const uint8_t* s3,
    const float* t0, const float* t1, const float* t2, const float* t3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3,
    int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3,
    unsigned g1, unsigned g2, unsigned g3,
    float sv0, float sv1, int64_t k, const uint16_t* __restrict__ a, int lb)
{
    const unsigned b = blockIdx.x;
    const uint8_t* codes = c0; const uint8_t* scales = s0; const float* ts = t0; uint16_t* y = y0;
    int64_t n = n0, ld = l0;
    unsigned first = 0;
    if (b >= g1) { codes = c1; scales = s1; ts = t1; y = y1; n = n1; ld = l1; first = g1; }
    if (b >= g2) { codes = c2; scales = s2; ts = t2; y = y2; n = n2; ld = l2; first = g2; }
    if (b >= g3) { codes = c3; scales = s3; ts = t3; y = y3; n = n3; ld = l3; first = g3; }
    gemv_stream_body<M, R, G, D, P, GB, SF, IL>(codes, scales, ts, sv0, sv1, n, k, a, y, ld,
                                                (int64_t)(b - first) * (P * R * G), lb);
}

// ---------------------------------------------------------------------------------------------
// Several activation rows on the 4x4x4 matrix instruction.  v_mfma_f32_4x4x4_16B_bf16 multiplies 16
// independent 4x4x4 blocks per wavefront: lane 4b+i supplies row i of block b's left matrix (4 values
// along k), lane 4b+j column j of its right matrix, and lane 4b+j receives column j of the product in
// 4 registers (rows i) -- checked on the GPU.  Here block b is a run of 32 k's; the LEFT matrix holds
// four activation rows (lane 4b+i: activation row i) and the RIGHT one four weight rows (lane 4b+j:
// weight row j), so a lane decodes the 32 codes of ITS weight row into bare FP4 values (1.5 ops per
// weight, as in the dot-product kernels), eight MFMAs per run multiply them with its activation row's
// 32 values, and the four sums a lane receives per 16-element block -- its own weight row against the
// four activation rows -- take the block scale the lane itself looked up: no cross-lane traffic.  (With
// the roles the other way round a lane held one sum per weight row and needed the scales of its three
// quad neighbours by DPP: 15 % more vector instructions, 9-12 % slower.)  Per weight: 1.5 decode +
// 0.25 MFMA + 0.25 FMA per set of four activation rows, against 1.5 + 0.5 per activation row with
// v_dot2 -- the dot-product kernels are VALU-bound from two activation rows up.  Workgroup structure
// as in the streaming kernel: wave w owns K-slice w (C runs of 512 elements), walks G groups of four
// rows with the next group's loads in flight, partial sums of the waves meet in LDS (each wave leaves
// one sum per row of 16 lanes: the cross-row step of the wave reduction is part of the final sum).
// Idle lanes (K tail) are silenced through their scale bits; activation rows past M are never masked,
// their results are simply not stored.
// FMT: 0 = scale bytes, blocks of 16 (two per run of 32); 1 = scale bytes, blocks of 2^lb >= 32 (one per run);
// 2 = FP16-scale format (one 16-bit word per block of 128, decoded without the table).
template <int C, int G, int D, int P, int MS, int PS = 1, bool IL = false, int FMT = 0>
__device__ __forceinline__ void gemv_quad_body(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                               const float* __restrict__ w_ts, float sv0, float sv1, int64_t n,
                                               int64_t k, const uint16_t* __restrict__ a, int64_t m,
                                               uint16_t* __restrict__ y, int64_t ld_y, int64_t row0, int lb = 4)
{
    static_assert(!(IL && FMT != 0), "the interleaved layout holds 16-element blocks");
    constexpr int R = 4;
    static_assert(D == 2, "two register buffers");
    __shared__ uint2 lut[256];
    __shared__ float part[P * G * R * 4 * MS][4 * kMaxWaves / P];       // per wave: one partial sum per row of 16 lanes
    const float ts = *w_ts;
    static_assert(P == 1 || P == 2, "one or two sets of waves");
    const uint32_t lane = threadIdx.x & 63u, nwaves = (blockDim.x >> 6) / P;
    const uint32_t wid = threadIdx.x >> 6;
    const uint32_t par = (P == 2 && wid >= nwaves) ? 1u : 0u;             // (no division ahead of the first load)
    const uint32_t wave = wid - par * nwaves;
    const uint32_t b = lane >> 2, q = lane & 3u;
    // uniform 64-bit bases (first row of the workgroup) + 32-bit offsets of the lane's row, as in the
    // streaming kernel; rows past N re-read the last row
    const uint32_t code_ld = (uint32_t)(IL ? il_row_bytes(k) : (k >> 1));
    const uint32_t scale_ld = IL ? code_ld : FMT == 2 ? (uint32_t)(k >> 7) * 2u : (uint32_t)(k >> (FMT == 1 ? lb : 4));
    const uint32_t last_row = (uint32_t)((n - 1 - row0 < P * R * G - 1) ? n - 1 - row0 : P * R * G - 1);
    const uint8_t* cbase = codes + row0 * (int64_t)code_ld;
    const uint8_t* sbase = (IL ? codes : scales) + row0 * (int64_t)scale_ld;

    struct Quad {
        uint4 cw[C];
        uint32_t sw[C];
    };
    v4f acc[G][MS];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int s = 0; s < MS; ++s) acc[g][s] = v4f{0.f, 0.f, 0.f, 0.f};
    // A wave's K-slice is PS passes of C runs of 512 elements; the activations of one pass are in
    // registers at a time and every pass walks all G groups, adding to their running sums.
#pragma unroll 1                                       // a real loop: unrolled, the second pass's loads get hoisted and spill
    for (int ps = 0; ps < PS; ++ps) {
        uint32_t koff[C], smask[C];                    // element offset of this lane's run c; 0 / all-ones
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint32_t kk = ((wave * PS + ps) * C + c) * 512u + 32u * b;
            const bool in = kk < (uint32_t)k;
            koff[c] = in ? kk : 0u;
            smask[c] = in ? 0xFFFFFFFFu : 0u;
        }
        uint4 av[MS][C][4];                            // activation row 4 s + q, this lane's runs
#pragma unroll
        for (int s = 0; s < MS; ++s) {
            const int64_t mrow = (4 * s + (int)q < m) ? 4 * s + (int)q : 0;      // rows past M re-read row 0
            const uint8_t* ap = reinterpret_cast<const uint8_t*>(a + mrow * k);
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j) av[s][c][j] = *reinterpret_cast<const uint4*>(ap + (koff[c] * 2u + 16u * j));
        }
        Quad buf[D];
        auto load = [&](Quad& g, int gi) {
            const uint32_t rel = par * (R * G) + gi * R + q;
            const uint32_t row = rel < last_row ? rel : last_row;
            const uint32_t crow = __umul24(row, code_ld), srow = __umul24(row, scale_ld);
#pragma unroll
            for (int c = 0; c < C; ++c) {
                g.cw[c] = load_once16(cbase + (crow + (IL ? il_code_off(koff[c]) : (koff[c] >> 1))));
                if (FMT == 2) {
                    g.sw[c] = *reinterpret_cast<const uint16_t*>(sbase + (srow + ((koff[c] >> 7) << 1))) & smask[c];
                } else if (FMT == 1) {
                    g.sw[c] = sbase[srow + (koff[c] >> lb)] & smask[c];
                } else {
                    g.sw[c] = *reinterpret_cast<const uint16_t*>(sbase + (srow + (IL ? il_scale_off(koff[c]) : (koff[c] >> 4)))) & smask[c];
                }
            }
        };
        load(buf[0], 0);
        if (FMT != 2 && ps == 0) {                                        // the first loads are in flight meanwhile
            fill_weight_lut(lut, sv0, sv1);
            __syncthreads();                                              // LUT ready
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (g + 1 < G) load(buf[(g + 1) % D], g + 1);
            const Quad& cur = buf[g % D];
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const uint32_t xw[4] = {cur.cw[c].x, cur.cw[c].y, cur.cw[c].z, cur.cw[c].w};
                uint2 le0, le1;                       // { -block scale, negated special value as a bf16 pair } of the two halves
                if constexpr (FMT == 2) {
                    float bs, sv;
                    decode_scale_word(cur.sw[c], sv0, sv1, bs, sv);      // (past K: word 0, scale 0)
                    const uint32_t nsv = (uint32_t)f32_to_bf16_rne(-sv);
                    le0 = le1 = make_uint2(f2u(-bs), nsv | (nsv << 16));
                } else if constexpr (FMT == 1) {
                    le0 = le1 = lut[cur.sw[c] & 255u];
                } else {
                    le0 = lut[cur.sw[c] & 255u];
                    le1 = lut[(cur.sw[c] >> 8) & 255u];
                }
                // bare FP4 values of the lane's 32 codes: dwords 0, 1 belong to the first block, 2, 3 to the second
                v4bf wa[4], wb[4];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t x = xw[d] ^ kRemapXor;
                    const uint32_t patch = d < 2 ? le0.y : le1.y;
                    const uint32_t w0 = patch_zero_halves(cvt_pair<0>(x), patch);
                    const uint32_t w1 = patch_zero_halves(cvt_pair<1>(x), patch);
                    const uint32_t w2 = patch_zero_halves(cvt_pair<2>(x), patch);
                    const uint32_t w3 = patch_zero_halves(cvt_pair<3>(x), patch);
                    wa[d] = __builtin_bit_cast(v4bf, make_uint2(w0, w1));
                    wb[d] = __builtin_bit_cast(v4bf, make_uint2(w2, w3));
                }
                // The activations are the LEFT operand (lane 4b+i: activation row i), the weights the right one
                // (lane 4b+j: weight row j), so a lane receives the four products of ITS weight row with the four
                // activation rows and folds them with its own row's (negated) block scale -- no cross-lane traffic.
                // The two blocks' chains of four dependent matrix instructions are interleaved.
                const float sc0 = u2f(le0.x), sc1 = u2f(le1.x);
#pragma unroll
                for (int s = 0; s < MS; ++s) {
                    const uint4 a0 = av[s][c][0], a1 = av[s][c][1], a2 = av[s][c][2], a3 = av[s][c][3];
                    const v4f zero = {0.f, 0.f, 0.f, 0.f};
                    v4f t0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a0.x, a0.y)), wa[0], zero, 0, 0, 0);
                    v4f t1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a2.x, a2.y)), wa[2], zero, 0, 0, 0);
                    t0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a0.z, a0.w)), wb[0], t0, 0, 0, 0);
                    t1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a2.z, a2.w)), wb[2], t1, 0, 0, 0);
                    t0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a1.x, a1.y)), wa[1], t0, 0, 0, 0);
                    t1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a3.x, a3.y)), wa[3], t1, 0, 0, 0);
                    t0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a1.z, a1.w)), wb[1], t0, 0, 0, 0);
                    t1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4bf, make_uint2(a3.z, a3.w)), wb[3], t1, 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        acc[g][s][i] = __builtin_fmaf(sc0, t0[i], acc[g][s][i]);
                        acc[g][s][i] = __builtin_fmaf(sc1, t1[i], acc[g][s][i]);
                    }
                }
            }
            if (ps == PS - 1) {
                // sum over the 16 runs of the wavefront: within each row of 16 lanes by DPP; the four rows' sums go to
                // LDS side by side and meet in the final sum over the waves (no cross-row shuffles)
#pragma unroll
                for (int s = 0; s < MS; ++s)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float v = acc[g][s][i];
                        v = dpp_add<0x114>(v);                            // row_shr:4
                        v = dpp_add<0x118>(v);                            // row_shr:8 -> lanes 12..15 of each row
                        if ((lane & 12u) == 12u) part[((par * G + g) * R + q) * (4 * MS) + 4 * s + i][4 * wave + (lane >> 4)] = v;   // weight row q, activation row 4 s + i
                    }
            }
        }
    }
    __syncthreads();
    for (uint32_t t = threadIdx.x; t < (uint32_t)(P * G * R * 4 * MS); t += blockDim.x) {
        const uint32_t pr = t / (4 * MS), mcol = t - pr * (4 * MS);
        if ((int64_t)mcol < m && row0 + pr < n) {
            float acc = 0.0f;
            for (uint32_t w = 0; w < 4 * nwaves; ++w) acc += part[t][w];
            y[(int64_t)mcol * ld_y + row0 + pr] = f32_to_bf16_rne(acc * ts);
        }
    }
}

template <int C, int G, int D, int P, int MS, int PS = 1, bool IL = false, int FMT = 0>
__global__ __launch_bounds__(64 * kMaxWaves) void gemv_quad_kernel(const uint8_t* __restrict__ codes,
                                                                   const uint8_t* __restrict__ scales,
                                                                   const float* __restrict__ w_ts, float sv0, float sv1,
                                                                   int64_t n, int64_t k, const uint16_t* __restrict__ a,
                                                                   int64_t m, uint16_t* __restrict__ y, int64_t ld_y, int lb)
{
    gemv_quad_body<C, G, D, P, MS, PS, IL, FMT>(codes, scales, w_ts, sv0, sv1, n, k, a, m, y, ld_y,
                                                (int64_t)blockIdx.x * (P * 4 * G), lb);
}

template <int C, int G, int D, int P, int MS, int PS = 1, bool IL = false, int FMT = 0>
__global__ __launch_bounds__(64 * kMaxWaves) void gemv_quad_grouped_kernel(
    const uint8_t* c0, const uint8_t* c1, const uint8_t* c2, const uint8_t* c3,
    const uint8_t* s0, const uint8_t* s1, const uint8_t* s2, const uint8_t* s3,
    const float* t0, const float* t1, const float* t2, const float* t3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3,
    int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3,
    unsigned g1, unsigned g2, unsigned g3,
    float sv0, float sv1, int64_t k, const uint16_t* __restrict__ a, int64_t m, int lb)
{
    const unsigned b = blockIdx.x;
    const uint8_t* codes = c0; const uint8_t* scales = s0; const float* ts = t0; uint16_t* y = y0;
    int64_t n = n0, ld = l0;
    unsigned first = 0;
    if (b >= g1) { codes = c1; scales = s1; ts = t1; y = y1; n = n1; ld = l1; first = g1; }
    if (b >= g2) { codes = c2; scales = s2; ts = t2; y = y2; n = n2; ld = l2; first = g2; }
    if (b >= g3) { codes = c3; scales = s3; ts = t3; y = y3; n = n3; ld = l3; first = g3; }
    gemv_quad_body<C, G, D, P, MS, PS, IL, FMT>(codes, scales, ts, sv0, sv1, n, k, a, m, y, ld, (int64_t)(b - first) * (P * 4 * G), lb);
}

// The matrix-instruction kernel serves 2 to 4 activation rows (one row: the dot-product kernel is faster):
// measured 5-11 % faster than it at M = 2 and 15-40 % at M = 4 over the projection shapes of 7B- and 70B-class
// layers.  One
// 512-element run per lane while that needs at most 16 waves (K <= 8192), two up to K = 16384, two
// passes of two up to K = 32768 (four runs at once do not fit the register budget of a 16-wave
// workgroup); longer rows stay with the dot-product kernel.  4 groups of 4 rows per workgroup, 8 when
// the launch has at least 16384 rows.
static inline bool quad_fits(const SvConfig& cfg, int64_t k, int64_t m)
{
    return (m >= 2 && m <= 4) && k <= 32768;
}
static inline int quad_runs(int64_t k) { return (k + 511) / 512 <= kMaxWaves ? 1 : 2; }
static inline int quad_passes(int64_t k) { return k <= 16384 ? 1 : 2; }
static inline int quad_groups(int64_t rows, int64_t k, int64_t m)
{
    const TuneShape t = tuned_shape(kTuneGemvQuad, m, rows, k);          // the tuner's entry, if it names a built shape
    if (t.source && (t.p[0] == 4 || t.p[0] == 8)) return t.p[0];
    return rows >= 16384 ? 8 : 4;
}

static hipError_t launch_gemv_quad(SvConfig cfg, const uint8_t* codes, const uint8_t* scales, const float* ts,
                                   int64_t n, int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y,
                                   hipStream_t st)
{
    const int runs = quad_runs(k), passes = quad_passes(k);
    const int groups = passes == 2 ? 4 : quad_groups(n, k, m);   // two passes keep G running sums: 8 groups would spill
    const int nwaves = (int)((k + 512 * runs * passes - 1) / (512 * runs * passes));
    const unsigned grid = (unsigned)((n + 4 * groups - 1) / (4 * groups));
#define RAZER_QUAD_ARGS grid, 64 * nwaves, 0, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, cfg.lb
#define RAZER_QUAD(C, G, PS)                                                                              \
    do {                                                                                                  \
        if (cfg.il) launch(gemv_quad_kernel<C, G, 2, 1, 1, PS, true, 0>, RAZER_QUAD_ARGS);                \
        else if (cfg.f16) launch(gemv_quad_kernel<C, G, 2, 1, 1, PS, false, 2>, RAZER_QUAD_ARGS);         \
        else if (cfg.lb != 4) launch(gemv_quad_kernel<C, G, 2, 1, 1, PS, false, 1>, RAZER_QUAD_ARGS);     \
        else launch(gemv_quad_kernel<C, G, 2, 1, 1, PS, false, 0>, RAZER_QUAD_ARGS);                      \
    } while (0)
    if (passes == 2)    { RAZER_QUAD(2, 4, 2); }
    else if (runs == 1) { if (groups == 8) RAZER_QUAD(1, 8, 1); else RAZER_QUAD(1, 4, 1); }
    else                { if (groups == 8) RAZER_QUAD(2, 8, 1); else RAZER_QUAD(2, 4, 1); }
#undef RAZER_QUAD
#undef RAZER_QUAD_ARGS
    return hipGetLastError();
}

static hipError_t launch_gemv_quad_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                                           int64_t m, hipStream_t st)
{
    int64_t rows = 0;
    for (int i = 0; i < count; ++i) rows += p[i].n;
    const int runs = quad_runs(k), passes = quad_passes(k);
    const int groups = passes == 2 ? 4 : quad_groups(rows, k, m);
    const int nwaves = (int)((k + 512 * runs * passes - 1) / (512 * runs * passes));
    const int64_t rows_per_wg = 4 * groups;
    GemvProblem q[4];
    unsigned g[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        q[i] = p[i < count ? i : count - 1];
        g[i + 1] = g[i] + (i < count ? (unsigned)((q[i].n + rows_per_wg - 1) / rows_per_wg) : 0u);
    }
#define RAZER_QUADG_ARGS                                                                                             \
    q[0].codes, q[1].codes, q[2].codes, q[3].codes, q[0].scales, q[1].scales, q[2].scales, q[3].scales, q[0].ts,     \
        q[1].ts, q[2].ts, q[3].ts, q[0].y, q[1].y, q[2].y, q[3].y, q[0].n, q[1].n, q[2].n, q[3].n, q[0].ld_y,        \
        q[1].ld_y, q[2].ld_y, q[3].ld_y, g[1], g[2], g[3], cfg.sv0, cfg.sv1, k, a, m, cfg.lb
#define RAZER_QUADG(C, G, PS)                                                                                                         \
    do {                                                                                                                              \
        if (cfg.il) launch(gemv_quad_grouped_kernel<C, G, 2, 1, 1, PS, true, 0>, g[4], 64 * nwaves, 0, st, RAZER_QUADG_ARGS);         \
        else if (cfg.f16) launch(gemv_quad_grouped_kernel<C, G, 2, 1, 1, PS, false, 2>, g[4], 64 * nwaves, 0, st, RAZER_QUADG_ARGS);  \
        else if (cfg.lb != 4) launch(gemv_quad_grouped_kernel<C, G, 2, 1, 1, PS, false, 1>, g[4], 64 * nwaves, 0, st, RAZER_QUADG_ARGS); \
        else launch(gemv_quad_grouped_kernel<C, G, 2, 1, 1, PS, false, 0>, g[4], 64 * nwaves, 0, st, RAZER_QUADG_ARGS);               \
    } while (0)
    if (passes == 2)    { RAZER_QUADG(2, 4, 2); }
    else if (runs == 1) { if (groups == 8) RAZER_QUADG(1, 8, 1); else RAZER_QUADG(1, 4, 1); }
    else                { if (groups == 8) RAZER_QUADG(2, 8, 1); else RAZER_QUADG(2, 4, 1); }
#undef RAZER_QUADG
#undef RAZER_QUADG_ARGS
    return hipGetLastError();
}

// Rows per group / groups per workgroup of the streaming kernel.  Measured on MI355X over the
// projection shapes of 7B- and 70B-class decoder layers: 2 rows x 2 groups is best while a
// workgroup has few waves (K <= 16384); with many waves per workgroup (long K), or 3-4
// activation rows on more than 4 waves, longer-lived workgroups (8 groups) win by 20-40 %.
constexpr int kStreamR = 2;
static inline int stream_groups(int nwaves, int m) { return (nwaves > 8 || (m >= 3 && nwaves > 4)) ? 8 : 2; }
// Two sets of waves per workgroup (half as many, larger workgroups) measured 5-8 % faster for rows of
// 1-3 and 5-8 slices (K = 4096, 11008), slower for 4 slices (K = 8192): dispatching workgroups is part
// of the cost of these short kernels.
static inline int stream_sets(int nwaves, int groups) { return (groups == 2 && nwaves <= 8 && nwaves != 4) ? 2 : 1; }
// (groups, sets) of a launch: the tuner's entry for (m, rows, k) when it names a shape the kernels are
// built for -- (2, 1), (2, 2) with at most 8 waves per set, (4, 1), (8, 1) -- else the rules above.
static inline void stream_shape(int nwaves, int64_t m, int64_t rows, int64_t k, int& groups, int& sets)
{
    const TuneShape t = tuned_shape(kTuneGemv, m, rows, k);
    if (t.source) {
        const int g = t.p[0], s = t.p[1];
        if (((g == 2 || g == 4 || g == 8) && s == 1) || (g == 2 && s == 2 && nwaves <= 8)) {
            groups = g;
            sets = s;
            return;
        }
    }
    groups = stream_groups(nwaves, (int)m);
    sets = stream_sets(nwaves, groups);
}

template <int M, int R>
static hipError_t launch_gemv_mr(SvConfig cfg, const uint8_t* codes, const uint8_t* scales, const float* ts,
                                 int64_t n, int64_t k, const uint16_t* a, uint16_t* y, int64_t ld_y, hipStream_t st)
{
    // One wave per 2048-element K-slice, at most 16; longer rows take several passes.
    const int64_t nslices = (k + kSliceK - 1) / kSliceK;
    const int nwaves = (int)(nslices < kMaxWaves ? nslices : kMaxWaves);
    const unsigned grid = (unsigned)((n + R - 1) / R);
    if (cfg.f16) launch(gemv_kernel<M, R, true, 1>, grid, 64 * nwaves, 0, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, y, ld_y, 7);
    else if (cfg.lb == 4) launch(gemv_kernel<M, R, false>, grid, 64 * nwaves, 0, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, y, ld_y, 4);
    else launch(gemv_kernel<M, R, true>, grid, 64 * nwaves, 0, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, y, ld_y, cfg.lb);
    return hipGetLastError();
}
template <int M>
static hipError_t launch_gemv_m(SvConfig cfg, const uint8_t* codes, const uint8_t* scales, const float* ts,
                                int64_t n, int64_t k, const uint16_t* a, uint16_t* y, int64_t ld_y, hipStream_t st)
{
    const int64_t nslices = (k + kSliceK - 1) / kSliceK;
    if (nslices > kMaxWaves) {                                            // K > 32768: several passes per wave
        if (cfg.il) return hipErrorInvalidValue;                          // (the host admits K <= 32768 only)
        return launch_gemv_mr<M, 4>(cfg, codes, scales, ts, n, k, a, y, ld_y, st);
    }
    constexpr int R = kStreamR;
    const int nwaves = (int)nslices;
    int groups, sets;
    stream_shape(nwaves, M, n, k, groups, sets);
    const unsigned grid = (unsigned)((n + sets * R * groups - 1) / (sets * R * groups));
#define RAZER_GEMV_ARGS codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, y, ld_y, cfg.lb
#define RAZER_GEMV_SHAPES(GB, SF)                                                                              \
    do {                                                                                                       \
        if (groups == 8) launch(gemv_stream_kernel<M, R, 8, 2, 1, GB, SF>, grid, 64 * nwaves, 0, st, RAZER_GEMV_ARGS);  \
        else if (groups == 4) launch(gemv_stream_kernel<M, R, 4, 2, 1, GB, SF>, grid, 64 * nwaves, 0, st, RAZER_GEMV_ARGS); \
        else if (sets == 2) launch(gemv_stream_kernel<M, R, 2, 2, 2, GB, SF>, grid, 128 * nwaves, 0, st, RAZER_GEMV_ARGS); \
        else launch(gemv_stream_kernel<M, R, 2, 2, 1, GB, SF>, grid, 64 * nwaves, 0, st, RAZER_GEMV_ARGS);              \
    } while (0)
    if (cfg.il) {
        if (groups == 8) launch(gemv_stream_kernel<M, R, 8, 2, 1, false, 0, true>, grid, 64 * nwaves, 0, st, RAZER_GEMV_ARGS);
        else if (groups == 4) launch(gemv_stream_kernel<M, R, 4, 2, 1, false, 0, true>, grid, 64 * nwaves, 0, st, RAZER_GEMV_ARGS);
        else if (sets == 2) launch(gemv_stream_kernel<M, R, 2, 2, 2, false, 0, true>, grid, 128 * nwaves, 0, st, RAZER_GEMV_ARGS);
        else launch(gemv_stream_kernel<M, R, 2, 2, 1, false, 0, true>, grid, 64 * nwaves, 0, st, RAZER_GEMV_ARGS);
    }
    else if (cfg.f16) RAZER_GEMV_SHAPES(true, 1);
    else if (cfg.lb != 4) RAZER_GEMV_SHAPES(true, 0);
    else RAZER_GEMV_SHAPES(false, 0);
#undef RAZER_GEMV_SHAPES
#undef RAZER_GEMV_ARGS
    return hipGetLastError();
}

template <int M>
static hipError_t launch_gemv_grouped_m(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                                        hipStream_t st)
{
    const int64_t nslices = (k + kSliceK - 1) / kSliceK;
    const bool stream = nslices <= kMaxWaves;
    const int nwaves = (int)(stream ? nslices : kMaxWaves);
    int groups = 1, sets = 1;
    if (stream) {
        int64_t rows = 0;
        for (int i = 0; i < count; ++i) rows += p[i].n;
        stream_shape(nwaves, M, rows, k, groups, sets);
    }
    const int64_t rows_per_wg = stream ? sets * kStreamR * groups : 4;
    GemvProblem q[4];
    unsigned g[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        q[i] = p[i < count ? i : count - 1];
        g[i + 1] = g[i] + (i < count ? (unsigned)((q[i].n + rows_per_wg - 1) / rows_per_wg) : 0u);
    }
#define RAZER_GROUPED_ARGS                                                                                       \
    q[0].codes, q[1].codes, q[2].codes, q[3].codes, q[0].scales, q[1].scales, q[2].scales, q[3].scales, q[0].ts, \
        q[1].ts, q[2].ts, q[3].ts, q[0].y, q[1].y, q[2].y, q[3].y, q[0].n, q[1].n, q[2].n, q[3].n, q[0].ld_y,    \
        q[1].ld_y, q[2].ld_y, q[3].ld_y, g[1], g[2], g[3], cfg.sv0, cfg.sv1, k, a, cfg.lb
#define RAZER_GROUPED_SHAPES(GB, SF)                                                                                      \
    do {                                                                                                                  \
        if (!stream)                                                                                                      \
            launch(gemv_grouped_kernel<M, 4, GB, SF>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);                          \
        else if (groups == 8)                                                                                             \
            launch(gemv_stream_grouped_kernel<M, kStreamR, 8, 2, 1, GB, SF>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);   \
        else if (groups == 4)                                                                                             \
            launch(gemv_stream_grouped_kernel<M, kStreamR, 4, 2, 1, GB, SF>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);   \
        else if (sets == 2)                                                                                               \
            launch(gemv_stream_grouped_kernel<M, kStreamR, 2, 2, 2, GB, SF>, g[4], 128 * nwaves, 0, st, RAZER_GROUPED_ARGS);  \
        else                                                                                                              \
            launch(gemv_stream_grouped_kernel<M, kStreamR, 2, 2, 1, GB, SF>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);   \
    } while (0)
    if (cfg.il) {
        if (!stream) return hipErrorInvalidValue;                          // (the host admits K <= 32768 only)
        if (groups == 8) launch(gemv_stream_grouped_kernel<M, kStreamR, 8, 2, 1, false, 0, true>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);
        else if (groups == 4) launch(gemv_stream_grouped_kernel<M, kStreamR, 4, 2, 1, false, 0, true>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);
        else if (sets == 2) launch(gemv_stream_grouped_kernel<M, kStreamR, 2, 2, 2, false, 0, true>, g[4], 128 * nwaves, 0, st, RAZER_GROUPED_ARGS);
        else launch(gemv_stream_grouped_kernel<M, kStreamR, 2, 2, 1, false, 0, true>, g[4], 64 * nwaves, 0, st, RAZER_GROUPED_ARGS);
    }
    else if (cfg.f16) RAZER_GROUPED_SHAPES(true, 1);
    else if (cfg.lb != 4) RAZER_GROUPED_SHAPES(true, 0);
    else RAZER_GROUPED_SHAPES(false, 0);
#undef RAZER_GROUPED_SHAPES
#undef RAZER_GROUPED_ARGS
    return hipGetLastError();
}

hipError_t launch_gemv_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                               int64_t m, hipStream_t st)
{
    if (count < 1 || count > 4 || m < 1 || m > 4) return hipErrorInvalidValue;
    if (quad_fits(cfg, k, m)) return launch_gemv_quad_grouped(cfg, count, p, k, a, m, st);
    switch (m) {
        case 1: return launch_gemv_grouped_m<1>(cfg, count, p, k, a, st);
        case 2: return launch_gemv_grouped_m<2>(cfg, count, p, k, a, st);
        case 3: return launch_gemv_grouped_m<3>(cfg, count, p, k, a, st);
        default: return launch_gemv_grouped_m<4>(cfg, count, p, k, a, st);
    }
}

hipError_t launch_gemv(SvConfig wcfg, const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts,
                       int64_t n, int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y,
                       hipStream_t st)
{
    if (n == 0 || m == 0) return hipSuccess;
    // Up to kGemvMaxM activation rows go through in passes of at most 4 rows; passes after the
    // first find the packed weights in the last-level cache for the matrices of a decoder layer.
    for (int64_t m0 = 0; m0 < m; m0 += 4) {
        const int64_t mc = (m - m0 < 4) ? m - m0 : 4;
        const uint16_t* ap = a + m0 * k;
        uint16_t* yp = y + m0 * ld_y;
        hipError_t e;
        if (quad_fits(wcfg, k, mc)) {
            e = launch_gemv_quad(wcfg, w_codes, w_scales, w_ts, n, k, ap, mc, yp, ld_y, st);
            if (e != hipSuccess) return e;
            continue;
        }
        switch (mc) {
            case 1: e = launch_gemv_m<1>(wcfg, w_codes, w_scales, w_ts, n, k, ap, yp, ld_y, st); break;
            case 2: e = launch_gemv_m<2>(wcfg, w_codes, w_scales, w_ts, n, k, ap, yp, ld_y, st); break;
            case 3: e = launch_gemv_m<3>(wcfg, w_codes, w_scales, w_ts, n, k, ap, yp, ld_y, st); break;
            default: e = launch_gemv_m<4>(wcfg, w_codes, w_scales, w_ts, n, k, ap, yp, ld_y, st); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace razer
