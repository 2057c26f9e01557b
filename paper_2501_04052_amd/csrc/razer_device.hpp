// Device-side helpers shared by the gfx950 RaZeR kernels.
//
// Format facts used here (arxiv 2501.04052): FP4-E2M1 elements with code 0x8
// remapped to a per-block special value (Sec. 4.2), one scale byte per 16
// elements -- weights: sign|selector|E3M3, activations: sign|E4M3 (Sec. 4.1,
// 4.2, 4.4) -- and one FP32 scale per tensor (Eq. 1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace razer {

constexpr int kBlock = 16;
constexpr uint32_t kRemapXor = 0x88888888u;   // flips the sign bit of all 8 nibbles of a dword

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned short v2us __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

struct SvConfig {          // special-value magnitudes and log2(block size), already validated on the host
    float sv0, sv1;
    int lb = 4;
    int f16 = 0;           // 1: one 16-bit scale word per block of 128 (sign | selector | 14 low bits of an IEEE half)
    int il = 0;            // 1: interleaved layout (below); 16-element blocks, scale-byte format only
};

// Interleaved layout of a weight row: runs of 2048 elements, each stored as 1024 bytes of codes followed
// by its 128 scale bytes (1152 bytes per run, also for a shorter last run).  Byte offsets inside a row of
// the code byte / scale byte of element k, and the bytes of a row of `cols` elements.
constexpr uint32_t kIlRun = 1152;
__host__ __device__ __forceinline__ uint32_t il_code_off(uint32_t k) { return (k >> 11) * kIlRun + ((k & 2047u) >> 1); }
__host__ __device__ __forceinline__ uint32_t il_scale_off(uint32_t k) { return (k >> 11) * kIlRun + 1024u + ((k & 2047u) >> 4); }
__host__ __device__ __forceinline__ int64_t il_row_bytes(int64_t cols) { return ((cols + 2047) >> 11) * (int64_t)kIlRun; }

// The two scale bytes (low byte first) that govern the 32 consecutive elements starting at element
// k0 (a multiple of 32) of a row whose scale bytes start at srow.  GB = false: blocks of 16, one
// 16-bit load.  GB = true: blocks of 2^lb elements chosen at run time; from 32 up both runs of 16
// share one byte.
template <bool GB>
__device__ __forceinline__ uint32_t load_scale_pair(const uint8_t* __restrict__ srow, int64_t k0, int lb)
{
    if (!GB || lb == 4) return *reinterpret_cast<const uint16_t*>(srow + (k0 >> 4));
    const uint32_t b = srow[k0 >> lb];
    return b | (b << 8);
}

// 16 bytes of packed weight codes that the launch reads exactly once: a non-temporal load (`nt`), which tells
// the caches not to keep the line.  Measured on MI355X with a load-only kernel over rotated buffers: 264 MB in
// 42.3 us instead of 46.5 us (6.24 against 5.68 TB/s); the GEMV launches gain 3-5 %.  Activations, which every
// workgroup re-reads, keep the default policy.
__device__ __forceinline__ uint4 load_once16(const void* p)
{
    const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Block-scale value of a weight scale byte's low 6 bits (E3M3, bias 3, subnormals).
__device__ __forceinline__ float e3m3_value(uint32_t c6)
{
    uint32_t E = (c6 >> 3) & 7u, M = c6 & 7u;
    // 2^(E-3)(1+M/8) for E != 0;  M/32 = 2^-2(1+M/8) - 2^-2 for E == 0 (exact).
    uint32_t bits = ((E ? E : 1u) + 124u) << 23 | (M << 20);
    return E ? u2f(bits) : u2f(bits) - 0.25f;
}
// Block-scale value of an activation scale byte's low 7 bits (FP8-E4M3 magnitude).
__device__ __forceinline__ float e4m3_value(uint32_t c7)
{
    uint32_t E = (c7 >> 3) & 15u, M = c7 & 7u;
    uint32_t bits = ((E ? E : 1u) + 120u) << 23 | (M << 20);
    return E ? u2f(bits) : u2f(bits) - 0.015625f;
}
// Scale and signed special value selected by a scale byte.
// sv0 / sv1 are passed as scalars on purpose: selecting between two fields of a by-value
// kernel-argument struct makes the compiler index the struct in memory, and the private
// copy it then needs costs every workgroup a read of the dispatch packet.
template <int FMT>
__device__ __forceinline__ void decode_scale_byte(uint32_t sb, float sv0, float sv1, float& s, float& sv)
{
    if (FMT == 0) {
        s = e3m3_value(sb & 63u);
        const uint32_t mag = (sb & 0x40u) ? f2u(sv1) : f2u(sv0);
        sv = u2f(mag | ((sb & 0x80u) << 24));
    } else {
        s = e4m3_value(sb & 127u);
        sv = u2f(f2u(sv0) | ((sb & 0x80u) << 24));
    }
}

// The FP16-scale weight format of the paper's weight-only kernel (Sec. 4.3): the low 14 bits of the
// scale word are an IEEE half with its exponent MSB clear (values below 2), bit 15 the sign of the
// special value, bit 14 its selector.
__device__ __forceinline__ float half14_value(uint32_t w)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0x3FFFu));
}
__device__ __forceinline__ void decode_scale_word(uint32_t w, float sv0, float sv1, float& s, float& sv)
{
    s = half14_value(w);
    const uint32_t mag = (w & 0x4000u) ? f2u(sv1) : f2u(sv0);
    sv = u2f(mag | ((w & 0x8000u) << 16));
}

// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN kept quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = f2u(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return u2f((uint32_t)b << 16); }

// ---- wavefront (64-lane) sum via DPP; every lane of row 3 / lane 63 holds the total ----
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_add(float v)
{
    int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}
// Sum over the 64 lanes; result valid in lane 63.
__device__ __forceinline__ float wave_sum_to_lane63(float v)
{
    v = dpp_add<0xB1>(v);         // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);         // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);        // row_half_mirror
    v = dpp_add<0x140>(v);        // row_mirror -> every lane has its row-of-16 sum
    v = dpp_add<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

// ---- FP4 pair decode in the "flipped" domain --------------------------------------
// x holds 8 FP4 codes.  After xor with kRemapXor every sign is flipped, so the
// hardware FP4 conversion yields -value for ordinary codes, -0 for the true zero
// (code 0) and +0 -- the only all-zero bit pattern -- for the remapped code 0x8.
// A 16-bit lane that is exactly 0 is therefore a special-value slot.  The
// callers undo the global negation in their final scale.

// Replace all-zero 16-bit halves of d by the matching half of patch.
__device__ __forceinline__ uint32_t patch_zero_halves(uint32_t d, uint32_t patch)
{
    v2us dv = __builtin_bit_cast(v2us, d);
    v2us one = {1, 1};
    v2us flag = __builtin_elementwise_sub_sat(one, dv);          // 1 where the half is 0
    v2us pv = __builtin_bit_cast(v2us, patch);
    v2us r = flag * pv + dv;
    return __builtin_bit_cast(uint32_t, r);
}

}  // namespace razer
