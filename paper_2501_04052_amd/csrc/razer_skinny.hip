// Weight-only RaZeR linear layer for 5..32 activation rows on gfx950 (small-batch decode, Sec. 4.3 /
// App. D.2 of arxiv 2501.04052): every packed weight is read from HBM and decoded exactly once, the
// multiply-accumulate goes to v_mfma_f32_16x16x32_bf16 with the activation rows padded to 16 or 32.
//
// A lane's 8 consecutive codes (one dword) decode straight into the 4 registers of an MFMA "A"
// operand (rows = weight rows n, k = this lane's 8 k's), so the weights never pass through LDS.
// MFMA operands are invariant under a permutation of k applied to both operands: lane group g of
// step s, instruction j holds k = 128 s + 32 g + 8 j .. +7, which makes a lane's 4 operands one
// 16-byte load of codes plus one 16-bit load of scale bytes.  Activations (M x KC bf16, shared by
// the 4 waves = 64 weight rows of a workgroup) are staged once in LDS, chunk-swizzled with the row.
//
// Work split: grid = (N / 64 / nrb) x (K / KC): a workgroup stages its K-slice of the activations once
// and walks through nrb consecutive 64-row blocks, loading the next block's weights while it decodes
// and multiplies the current one.  K-slices of one output tile are summed in fixed order by a second
// kernel (slice_reduce_kernel) from an fp32 workspace [slices][M][N] (deterministic, no atomics).
// The kernel is bound by the decode's vector ALU work (about 3 ops per weight), not by HBM.
//
// A second kernel for up to 16 activation rows (mv_kernel) keeps K inside the workgroup instead: the
// structure of the streaming GEMV -- a wave owns a K-slice of every row, its activation fragments stay in
// registers, it walks over groups of 16 rows with the next group's weights in flight, partial sums of the
// waves meet in LDS -- with the dot products on the 16x16x32 matrix instruction.  One launch, no workspace.
// Which of the two serves a shape, and with which launch shape, is the tuner's choice (razer_tune.h).
#include "razer_device.hpp"
#include "razer_kernels.hpp"

namespace razer {

template <int BYTE>
__device__ __forceinline__ uint32_t sk_cvt_scaled_pair(uint32_t xflip, float s, uint32_t patch)
{
    v2f p = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(xflip, 1.0f, BYTE);   // -element, exact
    p.x *= s;
    p.y *= s;
    v2bf b = __builtin_convertvector(p, v2bf);
    return patch_zero_halves(__builtin_bit_cast(uint32_t, b), patch);
}
// 8 codes -> 8 bare, negated FP4 values as bf16, remapped codes patched with `patch` (the negated special
// value as a bf16 pair): the FP16-scale format, whose scale multiplies the block's partial sum instead.
template <int BYTE>
__device__ __forceinline__ uint32_t sk_cvt_bare_pair(uint32_t xflip, uint32_t patch)
{
    v2bf p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(xflip, 1.0f, BYTE);
    return patch_zero_halves(__builtin_bit_cast(uint32_t, p), patch);
}
__device__ __forceinline__ v8bf sk_decode_dword_bare(uint32_t x, uint32_t patch)
{
    const uint32_t xf = x ^ kRemapXor;
    const uint4 r = make_uint4(sk_cvt_bare_pair<0>(xf, patch), sk_cvt_bare_pair<1>(xf, patch), sk_cvt_bare_pair<2>(xf, patch),
                               sk_cvt_bare_pair<3>(xf, patch));
    return __builtin_bit_cast(v8bf, r);
}
__device__ __forceinline__ v8bf sk_decode_dword(uint32_t x, uint2 le)
{
    const uint32_t xf = x ^ kRemapXor;
    const float s = u2f(le.x);
    const uint4 r = make_uint4(sk_cvt_scaled_pair<0>(xf, s, le.y), sk_cvt_scaled_pair<1>(xf, s, le.y),
                               sk_cvt_scaled_pair<2>(xf, s, le.y), sk_cvt_scaled_pair<3>(xf, s, le.y));
    return __builtin_bit_cast(v8bf, r);
}

constexpr int kSkRows = 64;            // weight rows per workgroup (4 waves x 16)

// NB: activation fragments of 16 rows (M <= 16 NB); STEPS: 128-k steps per workgroup (KC = 128 STEPS).
// NRB: consecutive 64-row blocks per workgroup, a template parameter so that the walk is straight-line
// code -- with the prefetch under a run-time branch the compiler has to assume at every use of the
// current block's registers that the prefetch did not happen, and waits for most of it.
template <int NB, int STEPS, bool GB, int NRB>
__device__ __forceinline__ void skinny_body(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                            const float* __restrict__ w_ts, float sv0, float sv1, int64_t n,
                                            int64_t k, const uint16_t* __restrict__ a, int64_t m,
                                            uint16_t* __restrict__ y, int64_t ld_y, float* __restrict__ partial,
                                            int nslices, int lb, unsigned block)
{
    constexpr int nrb = NRB;
    constexpr int KC = 128 * STEPS;
    constexpr int ROWB = KC * 2;                                   // bytes per activation row in LDS
    __shared__ __align__(16) uint8_t atile[NB * 16 * ROWB];
    __shared__ uint2 lut[256];

    // the wave index is uniform: read as a scalar it keeps the row arithmetic off the vector unit
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tid = wave * 64 + lane;
    const int slice = block % nslices;
    const int64_t nfirst = (int64_t)(block / nslices) * nrb * kSkRows;   // nrb consecutive 64-row blocks
    const int64_t k0 = (int64_t)slice * KC;
    const float ts = *w_ts;

    // this lane's weights of the row block at n0: row n0 + 16 wave + (lane % 16),
    // k = k0 + 128 s + 32 (lane / 16) .. +31.  Rows past N re-read the last row (never stored).  Steps past
    // K re-read step 0; where they are used their scale bytes are cleared: scale code 0 is 0.0, so whatever
    // the codes are, the weights (special values included) decode to 0.  Nothing here touches a loaded
    // value: an operation on one would make the wave wait for the load right where it was issued, and the
    // loads for the next row block are meant to stay in flight while the current one is decoded.
    // Addresses: a uniform 64-bit base per row block (scalar unit) plus 32-bit lane offsets -- the host
    // sends rows longer than kSkinnyMaxK elsewhere.
    const uint32_t code_ld = (uint32_t)(k >> 1), scale_ld = (uint32_t)(k >> lb);
    const uint32_t krem = (uint32_t)((k - k0 < KC) ? k - k0 : KC);       // elements of this slice inside K
    const uint32_t kl = 32u * (lane >> 4);
    auto load_weights = [&](int64_t n0, uint4 (&cw)[STEPS], uint32_t (&sw)[STEPS]) {
        int64_t r0 = n0 + 16 * wave;                               // uniform: first row of this wave
        r0 = r0 < n ? r0 : n - 1;
        const uint32_t left = (uint32_t)((n - 1 - r0 < 15) ? n - 1 - r0 : 15);
        const uint32_t dl = ((uint32_t)lane & 15u) < left ? ((uint32_t)lane & 15u) : left;
        const uint8_t* cbase = codes + r0 * (int64_t)code_ld + (k0 >> 1);
        const uint8_t* sbase = scales + r0 * (int64_t)scale_ld + (k0 >> (GB ? lb : 4));   // k0 holds whole blocks
        const uint32_t crow = dl * code_ld, srow = dl * scale_ld;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const uint32_t kin = 128u * s + kl;                    // offset inside the slice
            const bool in = kin < krem;
            const uint32_t kc = in ? kin : 0u;
            cw[s] = *reinterpret_cast<const uint4*>(cbase + (crow + (kc >> 1)));
            uint32_t sc;
            if (GB) {
                const uint32_t b = sbase[srow + (kc >> lb)];
                sc = b | (b << 8);
            } else {
                sc = *reinterpret_cast<const uint16_t*>(sbase + (srow + (kc >> 4)));
            }
            sw[s] = sc;
        }
    };
    uint4 cw[STEPS];
    uint32_t sw[STEPS];
    // activations [NB*16][KC] -> LDS, 16-byte chunks swizzled with the row (shared by all row blocks).
    // Fragment rows past M copy row M - 1: their product columns are never stored.  Chunks past K must be
    // zero -- the weights there are zero, but 0 x Inf would not be.
    constexpr int CH = KC / 8;                                     // 16-byte chunks per row
    constexpr int UNITS = NB * 16 * CH;
    const uint8_t* abase = reinterpret_cast<const uint8_t*>(a + k0);
    const uint32_t a_ld = (uint32_t)k * 2u;
    // (loads in batches of four, from clamped addresses and without a branch around any of them: a load
    // under a branch is waited for before the next one is issued)
    // The first row block's weights are requested right behind the first batch: loads return in order, so
    // the staging (L2 hits) is not held up behind them (HBM), and they are under way while LDS is filled.
    constexpr int NU = UNITS / 256, BATCH = NU < 4 ? NU : 4;
#pragma unroll
    for (int i0 = 0; i0 < NU; i0 += BATCH) {
        uint4 stage[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const uint32_t u = (uint32_t)tid + (i0 + i) * 256u, row = u / CH, c = u % CH;
            const uint32_t src_row = row < (uint32_t)m ? row : (uint32_t)m - 1u;
            const uint32_t src_c = c * 8u < krem ? c : 0u;
            stage[i] = *reinterpret_cast<const uint4*>(abase + (src_row * a_ld + src_c * 16u));
        }
        if (i0 == 0) load_weights(nfirst, cw, sw);
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const uint32_t u = (uint32_t)tid + (i0 + i) * 256u, row = u / CH, c = u % CH;
            const uint32_t keep = c * 8u < krem ? 0xFFFFFFFFu : 0u;
            const uint4 v = make_uint4(stage[i].x & keep, stage[i].y & keep, stage[i].z & keep, stage[i].w & keep);
            *reinterpret_cast<uint4*>(atile + row * ROWB + ((c ^ (row & 15u)) << 4)) = v;
        }
    }
    // LDS address of this lane's activation fragment for instruction j of step 0, fragment 0: row lane % 16,
    // logical chunk 4 (lane / 16) + j, swizzled; step s adds 256 bytes, fragment b adds 16 rows
    uint32_t afrag[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        afrag[j] = ((uint32_t)lane & 15u) * ROWB + (((4u * (lane >> 4) + j) ^ ((uint32_t)lane & 15u)) << 4);
    for (uint32_t sb = tid; sb < 256u; sb += 256) {
        float s, sv;
        decode_scale_byte<0>(sb, sv0, sv1, s, sv);
        const uint32_t p = (uint32_t)f32_to_bf16_rne(-(sv * s));
        lut[sb] = make_uint2(f2u(s), p | (p << 16));
    }
    __syncthreads();

    // two register buffers in turn; the next row block's weights are in flight while this one is decoded
    // and multiplied.  Blocks past N (last workgroup of a matrix) load clamped rows and store nothing.
    uint4 cwn[STEPS];
    uint32_t swn[STEPS];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int64_t n0 = nfirst + (int64_t)rb * kSkRows;
        uint4 (&cwc)[STEPS] = (rb & 1) ? cwn : cw;
        uint32_t (&swc)[STEPS] = (rb & 1) ? swn : sw;
        if (rb + 1 < NRB) {
            if (rb & 1) load_weights(n0 + kSkRows, cw, sw);
            else load_weights(n0 + kSkRows, cwn, swn);
        }
        __builtin_amdgcn_sched_barrier(0);

        v4f acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const uint32_t sws = (128u * s + kl < krem) ? swc[s] : 0u;      // steps past K: scale 0
            const uint2 le0 = lut[sws & 255u], le1 = lut[(sws >> 8) & 255u];
            const uint32_t xw[4] = {cwc[s].x, cwc[s].y, cwc[s].z, cwc[s].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v8bf wf = sk_decode_dword(xw[j], j < 2 ? le0 : le1);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const v8bf af = *reinterpret_cast<const v8bf*>(atile + afrag[j] + (256 * s + 16 * ROWB * b));
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, af, acc[b], 0, 0, 0);
                }
            }
        }
        // lane holds rows n = 4 (lane / 16) + 0..3 (of this wave's 16), column m = 16 b + lane % 16
        const int64_t gn = n0 + 16 * wave + 4 * (lane >> 4);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int64_t gm = 16 * b + (lane & 15);
            if (gm < m && gn < n) {
                if (nslices == 1) {
                    uint16_t* dst = y + gm * ld_y + gn;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (gn + e < n) dst[e] = f32_to_bf16_rne(-ts * acc[b][e]);
                } else {
                    float* dst = partial + ((int64_t)slice * m + gm) * n + gn;
                    if (gn + 3 < n && ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0)) {
                        *reinterpret_cast<float4*>(dst) = make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (gn + e < n) dst[e] = acc[b][e];
                    }
                }
            }
        }
    }
}

template <int NB, int STEPS, bool GB, int NRB>
__global__ __launch_bounds__(256) void skinny_kernel(const uint8_t* __restrict__ codes,
                                                     const uint8_t* __restrict__ scales,
                                                     const float* __restrict__ w_ts, float sv0, float sv1,
                                                     int64_t n, int64_t k, const uint16_t* __restrict__ a, int64_t m,
                                                     uint16_t* __restrict__ y, int64_t ld_y,
                                                     float* __restrict__ partial, int nslices, int lb)
{
    skinny_body<NB, STEPS, GB, NRB>(codes, scales, w_ts, sv0, sv1, n, k, a, m, y, ld_y, partial, nslices, lb, blockIdx.x);
}

// Up to four weight matrices against the same activations in one launch: workgroups are numbered
// through the matrices one after another (g1..g3 = first workgroup of matrices 1..3); matrix i keeps
// its K-slices in the workspace behind those of matrices 0 .. i-1.
template <int NB, int STEPS, int NRB, bool GB = false>
__global__ __launch_bounds__(256) void skinny_grouped_kernel(
    const uint8_t* c0, const uint8_t* c1, const uint8_t* c2, const uint8_t* c3,
    const uint8_t* s0, const uint8_t* s1, const uint8_t* s2, const uint8_t* s3,
    const float* f0, const float* f1, const float* f2, const float* f3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3,
    int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3,
    unsigned g1, unsigned g2, unsigned g3,
    float sv0, float sv1, int64_t k, const uint16_t* __restrict__ a, int64_t m, float* __restrict__ partial,
    int nslices, int lb)
{
    const unsigned b = blockIdx.x;
    const uint8_t* codes = c0; const uint8_t* scales = s0; const float* ts = f0; uint16_t* y = y0;
    int64_t n = n0, ld = l0, before = 0;
    unsigned first = 0;
    if (b >= g1) { codes = c1; scales = s1; ts = f1; y = y1; n = n1; ld = l1; first = g1; before = n0; }
    if (b >= g2) { codes = c2; scales = s2; ts = f2; y = y2; n = n2; ld = l2; first = g2; before = n0 + n1; }
    if (b >= g3) { codes = c3; scales = s3; ts = f3; y = y3; n = n3; ld = l3; first = g3; before = n0 + n1 + n2; }
    skinny_body<NB, STEPS, GB, NRB>(codes, scales, ts, sv0, sv1, n, k, a, m, y, ld,
                                    partial ? partial + (int64_t)nslices * m * before : nullptr, nslices, lb, b - first);
}

// y[m][n] = bf16(scale * sum over slices, in slice order, of partial[slice][m][n]); scale = -ts_w
// (weight-only: the decode carries a global negation) or ts_w * ts_a (both operands decoded).
// VEC = 4: four consecutive columns per thread (n and ld_y multiples of 4).
template <int VEC>
__global__ __launch_bounds__(256) void slice_reduce_kernel(const float* __restrict__ partial,
                                                           const float* __restrict__ w_ts,
                                                           const float* __restrict__ a_ts, int64_t m, int64_t n,
                                                           int nslices, uint16_t* __restrict__ y, int64_t ld_y)
{
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
    if (i >= m * n) return;
    const float scale = a_ts ? (*w_ts) * (*a_ts) : -(*w_ts);
    const int64_t r = i / n, c = i - r * n;
    if (VEC == 4) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s = 0; s < nslices; ++s) {
            const float4 p = *reinterpret_cast<const float4*>(partial + (int64_t)s * m * n + i);
            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
        }
        const uint32_t lo = (uint32_t)f32_to_bf16_rne(scale * t.x) | ((uint32_t)f32_to_bf16_rne(scale * t.y) << 16);
        const uint32_t hi = (uint32_t)f32_to_bf16_rne(scale * t.z) | ((uint32_t)f32_to_bf16_rne(scale * t.w) << 16);
        *reinterpret_cast<uint2*>(y + r * ld_y + c) = make_uint2(lo, hi);
    } else {
        float t = 0.0f;
        for (int s = 0; s < nslices; ++s) t += partial[(int64_t)s * m * n + i];
        y[r * ld_y + c] = f32_to_bf16_rne(scale * t);
    }
}

hipError_t launch_slice_reduce(const float* partial, const float* w_ts, const float* a_ts, int64_t m, int64_t n,
                               int nslices, uint16_t* y, int64_t ld_y, hipStream_t st)
{
    const int64_t total = m * n;
    if (n % 4 == 0 && ld_y % 4 == 0 && (reinterpret_cast<uintptr_t>(y) & 7u) == 0)
        launch(slice_reduce_kernel<4>, (unsigned)((total / 4 + 255) / 256), 256, 0, st, partial, w_ts, a_ts, m, n, nslices, y, ld_y);
    else
        launch(slice_reduce_kernel<1>, (unsigned)((total + 255) / 256), 256, 0, st, partial, w_ts, a_ts, m, n, nslices, y, ld_y);
    return hipGetLastError();
}

// The same reduction for the matrices of a grouped launch: thread index space = the 4-column groups
// of matrix 0, then of matrix 1, ... (e1..e3 = first group of matrices 1..3; every n a multiple of 4).
__global__ __launch_bounds__(256) void slice_reduce_grouped_kernel(
    const float* __restrict__ partial, const float* f0, const float* f1, const float* f2, const float* f3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3, int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3, int64_t e1, int64_t e2, int64_t e3, int64_t e4, int64_t m,
    int nslices)
{
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= e4) return;
    const float* ts = f0; uint16_t* y = y0;
    int64_t n = n0, ld = l0, first = 0, before = 0;
    if (g >= e1) { ts = f1; y = y1; n = n1; ld = l1; first = e1; before = n0; }
    if (g >= e2) { ts = f2; y = y2; n = n2; ld = l2; first = e2; before = n0 + n1; }
    if (g >= e3) { ts = f3; y = y3; n = n3; ld = l3; first = e3; before = n0 + n1 + n2; }
    const int64_t i = (g - first) * 4;
    const int64_t r = i / n, c = i - r * n;
    const float* src = partial + (int64_t)nslices * m * before + i;
    const float scale = -(*ts);
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < nslices; ++s) {
        const float4 p = *reinterpret_cast<const float4*>(src + (int64_t)s * m * n);
        t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
    }
    const uint32_t lo = (uint32_t)f32_to_bf16_rne(scale * t.x) | ((uint32_t)f32_to_bf16_rne(scale * t.y) << 16);
    const uint32_t hi = (uint32_t)f32_to_bf16_rne(scale * t.z) | ((uint32_t)f32_to_bf16_rne(scale * t.w) << 16);
    *reinterpret_cast<uint2*>(y + r * ld + c) = make_uint2(lo, hi);      // y 8-byte aligned, ld a multiple of 4
}

// partial: matrix i's [nslices][m][n_i] fp32 slices behind those of matrices 0 .. i-1.  Every n a
// positive multiple of 4, every y 8-byte aligned, every ld_y a multiple of 4.
hipError_t launch_slice_reduce_grouped(const float* partial, int count, const GemvProblem* p, int64_t m, int nslices,
                                       hipStream_t st)
{
    GemvProblem q[4];
    int64_t e[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        q[i] = p[i < count ? i : count - 1];
        e[i + 1] = e[i] + (i < count ? m * q[i].n / 4 : 0);
    }
    launch(slice_reduce_grouped_kernel, (unsigned)((e[4] + 255) / 256), 256, 0, st, partial, q[0].ts, q[1].ts, q[2].ts, q[3].ts, q[0].y, q[1].y, q[2].y, q[3].y, q[0].n, q[1].n, q[2].n, q[3].n,
        q[0].ld_y, q[1].ld_y, q[2].ld_y, q[3].ld_y, e[1], e[2], e[3], e[4], m, nslices);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// NB: 16-row activation fragments (M <= 16 NB); S: 128-k steps per wave and pass; G: groups of 16 weight
// rows per workgroup.  Wave w of the workgroup owns K-slice w (S steps) of every row, in pass p slice
// p * waves + w; its activation fragments for that slice stay in registers while it walks the G row
// groups, the next group's packed weights in flight.  Partial sums of the waves meet in LDS after ONE
// barrier.
// SF = 1: the FP16-scale weight format (blocks of 128 = one step: one scale word per lane and step).  The
// operands are bare FP4 values; the roles of the two matrix operands are swapped so that a lane's four
// results of a step belong to ITS weight row (lane % 16) and activation rows 4 (lane / 16) + 0..3, and the
// step's sum is folded into the running sums with the lane's own block scale in fp32.
template <int NB, int S, int G, bool GB, int SF = 0>
__device__ __forceinline__ void mv_body(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                        const float* __restrict__ w_ts, float sv0, float sv1, int64_t n, int64_t k,
                                        const uint16_t* __restrict__ a, int64_t m, uint16_t* __restrict__ y,
                                        int64_t ld_y, int lb, int64_t group0, int npass)
{
    __shared__ uint2 lut[256];
    extern __shared__ __align__(16) uint8_t dyn_smem[];
    float4* part = reinterpret_cast<float4*>(dyn_smem);               // [G][waves][NB][64]
    const float ts = *w_ts;
    const uint32_t lane = threadIdx.x & 63u, nwaves = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t r = lane & 15u, g = lane >> 4;
    const uint32_t kk32 = (uint32_t)k;
    const uint32_t code_ld = (uint32_t)(k >> 1), scale_ld = SF ? (uint32_t)(k >> 7) * 2u : (uint32_t)(k >> (GB ? lb : 4));

    struct WBuf {
        uint32_t cw[S][4];
        uint32_t sw[S];
    };
    v4f acc[G][NB];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[gi][b] = v4f{0.f, 0.f, 0.f, 0.f};

#pragma unroll 1
    for (int p = 0; p < npass; ++p) {
        const uint32_t kw = ((uint32_t)p * nwaves + wave) * (128u * S) + 32u * g;   // this lane's first k of step 0
        // element offsets of this lane's S steps (clamped to 0 past K) and the matching scale masks
        uint32_t koff[S], smask[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const uint32_t kk = kw + 128u * s;
            const bool in = kk < kk32;
            koff[s] = in ? kk : 0u;
            smask[s] = in ? 0xFFFFFFFFu : 0u;
        }
        // activation fragments of this K-slice: row 16 b + r (rows past M re-read row M - 1, their product
        // columns are never stored), 64 contiguous bytes per step
        uint32_t af[NB][S][4][4];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const uint32_t mrow = (16u * b + r < (uint32_t)m) ? 16u * b + r : (uint32_t)m - 1u;
            const uint8_t* ap = reinterpret_cast<const uint8_t*>(a + (int64_t)mrow * k);
#pragma unroll
            for (int s = 0; s < S; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint4 t = *reinterpret_cast<const uint4*>(ap + (koff[s] * 2u + 16u * j));
                    af[b][s][j][0] = t.x; af[b][s][j][1] = t.y; af[b][s][j][2] = t.z; af[b][s][j][3] = t.w;
                }
        }
        auto load = [&](WBuf& w, int gi) {
            int64_t row = (group0 + gi) * 16 + r;
            row = row < n ? row : n - 1;                                  // rows past N re-read the last row
            const uint8_t* crow = codes + row * (int64_t)code_ld;
            const uint8_t* srow = scales + row * (int64_t)scale_ld;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const uint4 t = *reinterpret_cast<const uint4*>(crow + (koff[s] >> 1));
                w.cw[s][0] = t.x; w.cw[s][1] = t.y; w.cw[s][2] = t.z; w.cw[s][3] = t.w;
                if (SF) {
                    w.sw[s] = *reinterpret_cast<const uint16_t*>(srow + ((koff[s] >> 7) << 1));
                } else if (GB) {
                    const uint32_t bb = srow[koff[s] >> lb];
                    w.sw[s] = bb | (bb << 8);
                } else {
                    w.sw[s] = *reinterpret_cast<const uint16_t*>(srow + (koff[s] >> 4));
                }
            }
        };
        WBuf w0, w1;
        load(w0, 0);
        if (!SF && p == 0) {
            for (uint32_t sb = threadIdx.x; sb < 256u; sb += blockDim.x) {
                float s, sv;
                decode_scale_byte<0>(sb, sv0, sv1, s, sv);
                const uint32_t pp = (uint32_t)f32_to_bf16_rne(-(sv * s));
                lut[sb] = make_uint2(f2u(s), pp | (pp << 16));
            }
            __syncthreads();
        }
        auto mul = [&](const WBuf& w, int gi) {
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const uint32_t sws = w.sw[s] & smask[s];                  // past K: scale 0
                if constexpr (SF != 0) {
                    float bs, sv;
                    decode_scale_word(sws, sv0, sv1, bs, sv);
                    const uint32_t nsv = (uint32_t)f32_to_bf16_rne(-sv);
                    v4f blk[NB];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const v8bf wf = sk_decode_dword_bare(w.cw[s][j], nsv | (nsv << 16));
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
                            const v8bf av = __builtin_bit_cast(v8bf, make_uint4(af[b][s][j][0], af[b][s][j][1], af[b][s][j][2], af[b][s][j][3]));
                            blk[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, wf, j == 0 ? v4f{0.f, 0.f, 0.f, 0.f} : blk[b], 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int b = 0; b < NB; ++b)
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[gi][b][i] = __builtin_fmaf(bs, blk[b][i], acc[gi][b][i]);
                    continue;
                }
                const uint2 le0 = lut[sws & 255u], le1 = lut[(sws >> 8) & 255u];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const v8bf wf = sk_decode_dword(w.cw[s][j], j < 2 ? le0 : le1);
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const v8bf av = __builtin_bit_cast(v8bf, make_uint4(af[b][s][j][0], af[b][s][j][1], af[b][s][j][2], af[b][s][j][3]));
                        acc[gi][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, av, acc[gi][b], 0, 0, 0);
                    }
                }
            }
        };
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            if (gi + 1 < G) load((gi & 1) ? w0 : w1, gi + 1);
            mul((gi & 1) ? w1 : w0, gi);
        }
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int b = 0; b < NB; ++b)
            part[((gi * nwaves + wave) * NB + b) * 64 + lane] = make_float4(acc[gi][b][0], acc[gi][b][1], acc[gi][b][2], acc[gi][b][3]);
    __syncthreads();
    // entry e = (group gi, fragment b, lane l): rows 16 (group0 + gi) + 4 (l / 16) + 0..3, column 16 b + l % 16
    for (uint32_t e = threadIdx.x; e < (uint32_t)(G * NB * 64); e += blockDim.x) {
        const uint32_t gi = e / (NB * 64), b = (e / 64) % NB, l = e & 63u;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        for (uint32_t w = 0; w < nwaves; ++w) {
            const float4 q = part[((gi * nwaves + w) * NB + b) * 64 + l];
            t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
        }
        if constexpr (SF != 0) {
            // swapped operands: weight row 16 (group0 + gi) + l % 16, activation rows 16 b + 4 (l / 16) + 0..3
            const int64_t wn = (group0 + gi) * 16 + (l & 15u);
            const float v[4] = {t.x, t.y, t.z, t.w};
            if (wn < n) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t am = 16 * b + 4 * (l >> 4) + i;
                    if (am < m) y[am * ld_y + wn] = f32_to_bf16_rne(-ts * v[i]);
                }
            }
            continue;
        }
        const int64_t gn = (group0 + gi) * 16 + 4 * (l >> 4);
        const int64_t gm = 16 * b + (l & 15u);
        if (gm < m && gn < n) {
            uint16_t* dst = y + gm * ld_y + gn;
            const float sc = -ts;
            if (gn + 3 < n && ((reinterpret_cast<uintptr_t>(dst) & 7u) == 0)) {
                const uint32_t lo = (uint32_t)f32_to_bf16_rne(sc * t.x) | ((uint32_t)f32_to_bf16_rne(sc * t.y) << 16);
                const uint32_t hi = (uint32_t)f32_to_bf16_rne(sc * t.z) | ((uint32_t)f32_to_bf16_rne(sc * t.w) << 16);
                *reinterpret_cast<uint2*>(dst) = make_uint2(lo, hi);
            } else {
                const float v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (gn + i < n) dst[i] = f32_to_bf16_rne(sc * v[i]);
            }
        }
    }
}

template <int NB, int S, int G, bool GB, int MAXW, int SF = 0>
__global__ __launch_bounds__(64 * MAXW) void mv_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                       const float* __restrict__ w_ts, float sv0, float sv1, int64_t n,
                                                       int64_t k, const uint16_t* __restrict__ a, int64_t m,
                                                       uint16_t* __restrict__ y, int64_t ld_y, int lb, int npass)
{
    mv_body<NB, S, G, GB, SF>(codes, scales, w_ts, sv0, sv1, n, k, a, m, y, ld_y, lb, (int64_t)blockIdx.x * G, npass);
}

// Grouped form: workgroups [0, g1) serve matrix 0, [g1, g2) matrix 1, ... (scalar arguments picked by
// uniform compares, as in the other grouped kernels).
template <int NB, int S, int G, bool GB, int MAXW, int SF = 0>
__global__ __launch_bounds__(64 * MAXW) void mv_grouped_kernel(
    const uint8_t* c0, const uint8_t* c1, const uint8_t* c2, const uint8_t* c3,
    const uint8_t* s0, const uint8_t* s1, const uint8_t* s2, const uint8_t* s3,
    const float* f0, const float* f1, const float* f2, const float* f3,
    uint16_t* y0, uint16_t* y1, uint16_t* y2, uint16_t* y3,
    int64_t n0, int64_t n1, int64_t n2, int64_t n3,
    int64_t l0, int64_t l1, int64_t l2, int64_t l3,
    unsigned g1, unsigned g2, unsigned g3,
    float sv0, float sv1, int64_t k, const uint16_t* __restrict__ a, int64_t m, int lb, int npass)
{
    const unsigned b = blockIdx.x;
    const uint8_t* codes = c0; const uint8_t* scales = s0; const float* ts = f0; uint16_t* y = y0;
    int64_t n = n0, ld = l0;
    unsigned first = 0;
    if (b >= g1) { codes = c1; scales = s1; ts = f1; y = y1; n = n1; ld = l1; first = g1; }
    if (b >= g2) { codes = c2; scales = s2; ts = f2; y = y2; n = n2; ld = l2; first = g2; }
    if (b >= g3) { codes = c3; scales = s3; ts = f3; y = y3; n = n3; ld = l3; first = g3; }
    mv_body<NB, S, G, GB, SF>(codes, scales, ts, sv0, sv1, n, k, a, m, y, ld, lb, (int64_t)(b - first) * G, npass);
}

// Launch shapes of the K-in-workgroup kernel: (S steps per wave and pass, G row groups per workgroup,
// at most MAXW waves).  The partial sums take G x waves KiB of LDS.
struct MvShape {
    int s, g, maxw;
};
constexpr MvShape kMvShapes[] = {{1, 1, 16}, {1, 2, 16}, {1, 3, 16}, {1, 4, 16}, {2, 1, 16}, {2, 2, 16}, {2, 3, 16}, {2, 4, 16}, {2, 8, 8}};
static bool mv_shape_ok(int s, int g)
{
    for (const MvShape& sh : kMvShapes)
        if (sh.s == s && sh.g == g) return true;
    return false;
}
static int mv_maxw(int s, int g)
{
    for (const MvShape& sh : kMvShapes)
        if (sh.s == s && sh.g == g) return sh.maxw;
    return 16;
}
// (nb 16-row activation fragments: the partial sums take g x waves x nb KiB of LDS, at most 64)
static void mv_geometry(int s, int g, int64_t k, int& nwaves, int& npass, int nb = 1)
{
    const int64_t slices = (k + 128 * s - 1) / (128 * s);
    int maxw = nb == 4 ? 8 : mv_maxw(s, g) / nb;                    // (two / four fragments: kernels built for 8 waves)
    if (maxw > 64 / (g * nb)) maxw = 64 / (g * nb);
    nwaves = (int)(slices < maxw ? slices : maxw);
    npass = (int)((slices + nwaves - 1) / nwaves);
}

// The launch plan of a small-batch problem: the tuner's entry for (m, rows, k) when it names shapes the
// kernels are built for, else the heuristic -- the K-sliced kernel with 512-element slices (1024 for long
// rows at M <= 16, to bound the number of slices) and 2 or 4 consecutive 64-row blocks per workgroup when
// that still leaves 2048 workgroups (up to 16 activation rows) or 1024 (17..32); measured over 4096^2 ..
// 57344 x 8192: 5-12 % faster on the large matrices, slower on small ones.
struct SkinnyPlan {
    bool in_workgroup;      // K inside the workgroup (mv_kernel): no workspace
    int steps, nrb;         // K-sliced kernel
    int s, g;               // K-in-workgroup kernel
};
// Up to 16 activation rows, no table entry: the K-in-workgroup kernel when some G <= 4 puts the whole launch into
// ONE round of workgroups (a workgroup of 16 waves fills a compute unit, so a second round would run on a nearly
// idle GPU) that still covers half of the 256 compute units; 2 steps per wave from 3 groups up.  Long rows with
// more than 8 activation rows keep the K-sliced kernel.  This rule reproduces what the sweep picked on the
// projection shapes of 7B- and 70B-class layers (4096^2: G = 1; 8192^2: 2; 11008 x 4096 and 10240 x 8192: 3;
// {q,k,v} 3 x 4096 x 4096: 4 -- with G = 3 its 3 x 86 workgroups would be two more than the chip has units).
constexpr int64_t kComputeUnits = 256;
static bool mv_one_round_shape(int64_t rows, int count, int& s, int& g)
{
    const int64_t groups = (rows + 15) / 16;
    for (int gg = 1; gg <= 4; ++gg) {
        const int64_t wgs = (groups + gg - 1) / gg + (count - 1);       // (each matrix of a group rounds up on its own)
        if (wgs <= kComputeUnits) {
            if (wgs < kComputeUnits / 2) return false;
            g = gg;
            s = gg >= 3 ? 2 : 1;
            return true;
        }
    }
    return false;
}
static bool mv_one_round(int64_t rows, int count, int64_t k, int64_t m, int& s, int& g)
{
    if (m > 16 || k > 16384 || (k > 8192 && m > 8)) return false;
    return mv_one_round_shape(rows, count, s, g);
}

static SkinnyPlan skinny_plan(int64_t rows, int64_t k, int64_t m, bool f16 = false, int count = 1)
{
    SkinnyPlan p{false, (m <= 16 && k > 8192) ? 8 : 4, 1, 0, 0};
    const int64_t row_blocks = (rows + kSkRows - 1) / kSkRows;
    const TuneShape t = tuned_shape(kTuneSmallBatch, m, rows, k);
    if (f16) {
        // the FP16-scale format has the K-in-workgroup kernel only (up to 32 activation rows): a forced shape,
        // else 1 step per wave and pass and 2 row groups (best of the five shapes on the 7B-class layer at 8,
        // 16 and 32 rows: 64 / 75 / 105 us against 79-80 / 89-91 / 115 with 4 groups)
        p.in_workgroup = true;
        p.s = 1;
        p.g = 2;
        if (t.source == 1 && t.p[0] == 1 && mv_shape_ok(t.p[1], t.p[2])) { p.s = t.p[1]; p.g = t.p[2]; }
        else if (m <= 16) mv_one_round_shape(rows, count, p.s, p.g);   // one round of workgroups where that is possible
        return p;
    }
    if (t.source && t.p[0] == 1 && m <= 16 && mv_shape_ok(t.p[1], t.p[2])) {
        p.in_workgroup = true;
        p.s = t.p[1];
        p.g = t.p[2];
        return p;
    }
    if (t.source && t.p[0] == 0 && (t.p[1] == 4 || (t.p[1] == 8 && m <= 16)) && (t.p[2] == 1 || t.p[2] == 2 || t.p[2] == 4)) {
        p.steps = t.p[1];
        p.nrb = t.p[2];
        return p;
    }
    if (mv_one_round(rows, count, k, m, p.s, p.g)) {
        p.in_workgroup = true;
        return p;
    }
    const int64_t nslices = (k + 128 * p.steps - 1) / (128 * p.steps);
    const int64_t target = m <= 16 ? 2048 : 1024;
    while (p.nrb < 4 && (row_blocks / (2 * p.nrb)) * nslices >= target) p.nrb *= 2;
    return p;
}

size_t skinny_workspace_bytes(int64_t n, int64_t k, int64_t m)
{
    if (m <= kGemvDirectMaxM || m > kSkinnyMaxM || k == 0 || k > kSkinnyMaxK) return 0;
    const SkinnyPlan p = skinny_plan(n, k, m);
    if (p.in_workgroup) return 0;
    const int64_t kc = 128 * p.steps;
    const int64_t nslices = (k + kc - 1) / kc;
    return nslices > 1 ? (size_t)(nslices * m * n) * sizeof(float) : 0;
}

size_t skinny_grouped_workspace_bytes(int count, const GemvProblem* p, int64_t k, int64_t m)
{
    if (m <= kGemvDirectMaxM || m > kSkinnyMaxM || k == 0 || k > kSkinnyMaxK) return 0;
    int64_t rows = 0;
    for (int i = 0; i < count; ++i) rows += p[i].n;
    const SkinnyPlan pl = skinny_plan(rows, k, m, false, count);
    if (pl.in_workgroup) return 0;
    const int64_t kc = 128 * pl.steps;
    const int64_t nslices = (k + kc - 1) / kc;
    return nslices > 1 ? (size_t)(nslices * m * rows) * sizeof(float) : 0;
}

#define RAZER_MV_SHAPES(LAUNCH)                       \
    do {                                              \
        if (pl.s == 1 && pl.g == 1) LAUNCH(1, 1, 16); \
        else if (pl.s == 1 && pl.g == 2) LAUNCH(1, 2, 16); \
        else if (pl.s == 1 && pl.g == 3) LAUNCH(1, 3, 16); \
        else if (pl.s == 1) LAUNCH(1, 4, 16);         \
        else if (pl.g == 1) LAUNCH(2, 1, 16);         \
        else if (pl.g == 2) LAUNCH(2, 2, 16);         \
        else if (pl.g == 3) LAUNCH(2, 3, 16);         \
        else if (pl.g == 4) LAUNCH(2, 4, 16);         \
        else LAUNCH(2, 8, 8);                         \
    } while (0)

hipError_t launch_skinny(SvConfig cfg, const uint8_t* codes, const uint8_t* scales, const float* ts, int64_t n,
                         int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y, float* workspace,
                         hipStream_t st)
{
    const SkinnyPlan pl = skinny_plan(n, k, m, cfg.f16 != 0);
    if (pl.in_workgroup && cfg.f16 && m > 32) {
        // FP16-scale format, 33..64 activation rows: four 16-row fragments, one step per wave and pass, two row groups
        int nwaves, npass;
        mv_geometry(1, 2, k, nwaves, npass, 4);
        launch(mv_kernel<4, 1, 2, false, 8, 1>, (unsigned)(((n + 15) / 16 + 1) / 2), 64 * nwaves, (size_t)2 * nwaves * 4 * 1024, st,
               codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, cfg.lb, npass);
        return hipGetLastError();
    }
    if (pl.in_workgroup) {
        const int nb = m <= 16 ? 1 : 2;
        int nwaves, npass;
        mv_geometry(pl.s, pl.g, k, nwaves, npass, nb);
        const unsigned grid = (unsigned)(((n + 15) / 16 + pl.g - 1) / pl.g);
        const size_t smem = (size_t)pl.g * nwaves * nb * 1024;
#define RAZER_MV(S, G, MW)                                                                                           \
        do {                                                                                                         \
            if (cfg.f16 && nb == 2) launch(mv_kernel<2, S, G, false, MW / 2, 1>, grid, 64 * nwaves, smem, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, cfg.lb, npass); \
            else if (cfg.f16) launch(mv_kernel<1, S, G, false, MW, 1>, grid, 64 * nwaves, smem, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, cfg.lb, npass); \
            else if (cfg.lb == 4) launch(mv_kernel<1, S, G, false, MW>, grid, 64 * nwaves, smem, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, cfg.lb, npass); \
            else launch(mv_kernel<1, S, G, true, MW>, grid, 64 * nwaves, smem, st, codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, cfg.lb, npass);             \
        } while (0)
        RAZER_MV_SHAPES(RAZER_MV);
#undef RAZER_MV
        return hipGetLastError();
    }
    const int steps = pl.steps;
    const int64_t kc = 128 * steps;
    const int nslices = (int)((k + kc - 1) / kc);
    const int64_t row_blocks = (n + kSkRows - 1) / kSkRows;
    const int nrb = pl.nrb;
    const unsigned grid = (unsigned)(((row_blocks + nrb - 1) / nrb) * nslices);
#define RAZER_SK_ARGS codes, scales, ts, cfg.sv0, cfg.sv1, n, k, a, m, y, ld_y, workspace, nslices, cfg.lb
#define RAZER_SK(NB, ST, GB)                                                                  \
    do {                                                                                      \
        if (nrb == 1) launch(skinny_kernel<NB, ST, GB, 1>, grid, 256, 0, st, RAZER_SK_ARGS);      \
        else if (nrb == 2) launch(skinny_kernel<NB, ST, GB, 2>, grid, 256, 0, st, RAZER_SK_ARGS); \
        else launch(skinny_kernel<NB, ST, GB, 4>, grid, 256, 0, st, RAZER_SK_ARGS);               \
    } while (0)
    if (cfg.lb == 4) {
        if (m <= 16) { if (steps == 8) RAZER_SK(1, 8, false); else RAZER_SK(1, 4, false); }
        else RAZER_SK(2, 4, false);
    } else {                                                            // blocks of 32, 64, 128
        if (m <= 16) { if (steps == 8) RAZER_SK(1, 8, true); else RAZER_SK(1, 4, true); }
        else RAZER_SK(2, 4, true);
    }
#undef RAZER_SK
#undef RAZER_SK_ARGS
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nslices == 1) return e;
    return launch_slice_reduce(workspace, ts, nullptr, m, n, nslices, y, ld_y, st);
}

// One launch (plus one reduction launch when K is sliced over workgroups) for up to 4 matrices sharing K,
// the activation rows (5..32), the block size and the special values; every n a positive multiple of 4.
// Workspace: skinny_grouped_workspace_bytes.
hipError_t launch_skinny_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                                 int64_t m, float* workspace, hipStream_t st)
{
    if (count < 1 || count > 4 || m <= kGemvDirectMaxM || m > kSkinnyMaxM || k > kSkinnyMaxK)
        return hipErrorInvalidValue;
    int64_t rows = 0;
    for (int i = 0; i < count; ++i) rows += p[i].n;
    const SkinnyPlan pl = skinny_plan(rows, k, m, cfg.f16 != 0, count);
    GemvProblem q[4];
    unsigned g[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        q[i] = p[i < count ? i : count - 1];
        if (q[i].n % 4 != 0 || q[i].n <= 0) return hipErrorInvalidValue;
    }
#define RAZER_SKG_COMMON                                                                                             \
    q[0].codes, q[1].codes, q[2].codes, q[3].codes, q[0].scales, q[1].scales, q[2].scales, q[3].scales, q[0].ts,     \
        q[1].ts, q[2].ts, q[3].ts, q[0].y, q[1].y, q[2].y, q[3].y, q[0].n, q[1].n, q[2].n, q[3].n, q[0].ld_y,        \
        q[1].ld_y, q[2].ld_y, q[3].ld_y, g[1], g[2], g[3], cfg.sv0, cfg.sv1, k, a, m
    if (pl.in_workgroup) {
        const int nb = m <= 16 ? 1 : 2;
        int nwaves, npass;
        mv_geometry(pl.s, pl.g, k, nwaves, npass, nb);
        for (int i = 0; i < 4; ++i)
            g[i + 1] = g[i] + (i < count ? (unsigned)(((q[i].n + 15) / 16 + pl.g - 1) / pl.g) : 0u);
        const size_t smem = (size_t)pl.g * nwaves * nb * 1024;
#define RAZER_MVG(S, G, MW)                                                                                                   \
        do {                                                                                                                  \
            if (cfg.f16 && nb == 2) launch(mv_grouped_kernel<2, S, G, false, MW / 2, 1>, g[4], 64 * nwaves, smem, st, RAZER_SKG_COMMON, cfg.lb, npass); \
            else if (cfg.f16) launch(mv_grouped_kernel<1, S, G, false, MW, 1>, g[4], 64 * nwaves, smem, st, RAZER_SKG_COMMON, cfg.lb, npass); \
            else if (cfg.lb == 4) launch(mv_grouped_kernel<1, S, G, false, MW>, g[4], 64 * nwaves, smem, st, RAZER_SKG_COMMON, cfg.lb, npass); \
            else launch(mv_grouped_kernel<1, S, G, true, MW>, g[4], 64 * nwaves, smem, st, RAZER_SKG_COMMON, cfg.lb, npass);             \
        } while (0)
        RAZER_MV_SHAPES(RAZER_MVG);
#undef RAZER_MVG
        return hipGetLastError();
    }
    const int steps = pl.steps;
    const int64_t kc = 128 * steps;
    const int nslices = (int)((k + kc - 1) / kc);
    const int nrb = pl.nrb;
    for (int i = 0; i < 4; ++i) {
        const int64_t rbi = (q[i].n + kSkRows - 1) / kSkRows;
        g[i + 1] = g[i] + (i < count ? (unsigned)((rbi + nrb - 1) / nrb) * nslices : 0u);
    }
    float* partial = nslices > 1 ? workspace : nullptr;
#define RAZER_SKG_ARGS RAZER_SKG_COMMON, partial, nslices, cfg.lb
#define RAZER_SKG(NB, ST, GB)                                                                            \
    do {                                                                                                 \
        if (nrb == 1) launch(skinny_grouped_kernel<NB, ST, 1, GB>, g[4], 256, 0, st, RAZER_SKG_ARGS);        \
        else if (nrb == 2) launch(skinny_grouped_kernel<NB, ST, 2, GB>, g[4], 256, 0, st, RAZER_SKG_ARGS);   \
        else launch(skinny_grouped_kernel<NB, ST, 4, GB>, g[4], 256, 0, st, RAZER_SKG_ARGS);                 \
    } while (0)
    if (cfg.lb == 4) {
        if (m <= 16) { if (steps == 8) RAZER_SKG(1, 8, false); else RAZER_SKG(1, 4, false); }
        else RAZER_SKG(2, 4, false);
    } else {                                                            // blocks of 32, 64, 128
        if (m <= 16) { if (steps == 8) RAZER_SKG(1, 8, true); else RAZER_SKG(1, 4, true); }
        else RAZER_SKG(2, 4, true);
    }
#undef RAZER_SKG
#undef RAZER_SKG_ARGS
#undef RAZER_SKG_COMMON
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || nslices == 1) return err;
    return launch_slice_reduce_grouped(partial, count, p, m, nslices, st);
}

}  // namespace razer
