// C ABI of the gfx950 RaZeR library: argument validation and kernel dispatch.
// Every entry point enqueues on the caller's stream and returns; nothing here
// allocates, synchronizes or keeps per-call state.
#include <mutex>

#include "../../include/razer.h"
#include "razer_kernels.hpp"

using namespace razer;

// Scratch of razer_linear_static: the K-slice workspace of the linear layer as a static device array,
// for callers that cannot allocate.  In host code the array's name is only a handle: its device address
// is looked up once per device (hipGetSymbolAddress with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)RAZER_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxScratchDevices = 16;
std::once_flag scratch_once[kMaxScratchDevices];
void* scratch_ptr[kMaxScratchDevices];
hipError_t scratch_err[kMaxScratchDevices];

// device address of `scratch` on the current device, or nullptr
void* static_scratch()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return nullptr;
    std::call_once(scratch_once[dev], [dev] {
        void* p = nullptr;
        scratch_err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        scratch_ptr[dev] = scratch_err[dev] == hipSuccess ? p : nullptr;
    });
    return scratch_ptr[dev];
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A special-value magnitude must be what the decoder's offset register can form:
// 6 + (multiple of 0.5 in [-3.5, 3.5]) (Sec. 4.4), and not an FP4 value itself.
bool sv_ok(float v)
{
    if (!(v >= 2.5f && v <= 9.5f)) return false;
    float twice = v * 2.0f;
    if (twice != (float)(int)twice) return false;
    return v != 3.0f && v != 4.0f && v != 6.0f;
}

razer_status check_cfg(const razer_config& c, SvConfig& out)
{
    if (c.format != RAZER_FMT_WEIGHT && c.format != RAZER_FMT_ACT && c.format != RAZER_FMT_WEIGHT_F16)
        return RAZER_ERR_CONFIG;
    if (!sv_ok(c.sv[0])) return RAZER_ERR_CONFIG;
    if (c.format != RAZER_FMT_ACT && !sv_ok(c.sv[1])) return RAZER_ERR_CONFIG;
    out.sv0 = c.sv[0];
    out.sv1 = (c.format != RAZER_FMT_ACT) ? c.sv[1] : c.sv[0];
    out.f16 = 0;
    out.il = 0;
    if (c.layout != RAZER_LAYOUT_CANONICAL && c.layout != RAZER_LAYOUT_INTERLEAVED) return RAZER_ERR_CONFIG;
    if (c.layout == RAZER_LAYOUT_INTERLEAVED) {                 // scale-byte weights with 16-element blocks only
        if (c.format != RAZER_FMT_WEIGHT || (c.block != 0 && c.block != 16)) return RAZER_ERR_CONFIG;
        out.il = 1;
    }
    if (c.format == RAZER_FMT_WEIGHT_F16) {                     // blocks of 128 only, 16-bit scale words
        if (c.block != 0 && c.block != 128) return RAZER_ERR_CONFIG;
        out.lb = 7;
        out.f16 = 1;
        return RAZER_OK;
    }
    switch (c.block) {
        case 0: case 16: out.lb = 4; break;
        case 32: out.lb = 5; break;
        case 64: out.lb = 6; break;
        case 128: out.lb = 7; break;
        default: return RAZER_ERR_CONFIG;
    }
    return RAZER_OK;
}

// cols must hold whole blocks and whole 16-byte code chunks
bool cols_ok(int64_t cols, const SvConfig& c) { return cols >= 0 && cols % 32 == 0 && cols % ((int64_t)1 << c.lb) == 0; }

razer_status check_tensor(const razer_tensor* t, int want_fmt, SvConfig& cfg)
{
    if (!t) return RAZER_ERR_NULL;
    razer_status s = check_cfg(t->cfg, cfg);
    if (s != RAZER_OK) return s;
    if (t->rows < 0 || !cols_ok(t->cols, cfg)) return RAZER_ERR_SHAPE;
    // a weight operand may be in either weight format
    const int fmt_class = (t->cfg.format == RAZER_FMT_WEIGHT_F16) ? RAZER_FMT_WEIGHT : t->cfg.format;
    if (want_fmt >= 0 && fmt_class != want_fmt) return RAZER_ERR_CONFIG;
    if (!t->tensor_scale) return RAZER_ERR_NULL;
    if (t->rows > 0 && t->cols > 0) {
        if (!t->codes || (!cfg.il && !t->scales)) return RAZER_ERR_NULL;      // interleaved: one buffer
        if (!aligned16(t->codes) || (!cfg.il && !aligned16(t->scales))) return RAZER_ERR_ALIGN;
    }
    return RAZER_OK;
}

// one thread per 16 bytes of the packed buffer: code chunks and scale chunks of the interleaved runs
__global__ __launch_bounds__(256) void prepack_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                      int64_t rows, int64_t cols, uint8_t* __restrict__ packed)
{
    const int64_t row_bytes = il_row_bytes(cols), units_per_row = row_bytes / 16;
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= rows * units_per_row) return;
    const int64_t r = u / units_per_row;
    const uint32_t off = (uint32_t)(u - r * units_per_row) * 16u, run = off / kIlRun, in = off - run * kIlRun;
    uint4 v = make_uint4(0, 0, 0, 0);                                         // padding of a short last run
    if (in < 1024u) {
        const int64_t cb = (int64_t)run * 1024 + in;                          // byte of the row's codes
        if (cb < cols / 2) v = *reinterpret_cast<const uint4*>(codes + r * (cols / 2) + cb);
    } else {
        const int64_t sb = (int64_t)run * 128 + (in - 1024u);                 // byte of the row's scales
        if (sb < cols / 16) {
            // (cols % 32 == 0 only guarantees pairs of scale bytes: copy byte-wise at the row's end)
            const uint8_t* src = scales + r * (cols / 16) + sb;
            uint8_t b[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) b[i] = (sb + i < cols / 16) ? src[i] : (uint8_t)0;
            v = *reinterpret_cast<const uint4*>(b);
        }
    }
    *reinterpret_cast<uint4*>(packed + r * row_bytes + off) = v;
}

__global__ void fill_zero_bf16_kernel(uint16_t* y, int64_t m, int64_t n, int64_t ld)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < m * n) y[(i / n) * ld + (i % n)] = 0;
}

// W4A4 in two steps: the decoded activations (bf16 [m][cols], rounded up to 256 bytes), one 256-byte cell for the
// combined tensor scale, then whatever the weight-only path itself needs for these sizes.
size_t w4a4_staged_bytes(int64_t rows, int64_t cols, int64_t m);

}  // namespace

extern "C" {

const char* razer_status_string(razer_status s)
{
    switch (s) {
        case RAZER_OK: return "ok";
        case RAZER_ERR_NULL: return "null pointer";
        case RAZER_ERR_SHAPE: return "bad shape";
        case RAZER_ERR_ALIGN: return "bad alignment";
        case RAZER_ERR_CONFIG: return "bad configuration";
        case RAZER_ERR_WORKSPACE: return "bad workspace";
        case RAZER_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

size_t razer_workspace_bytes(int op, int64_t rows, int64_t cols, int64_t m)
{
    switch (op) {
        case RAZER_OP_QUANTIZE: return 256;    // the 64 running-maximum cells of Eq. 1
        case RAZER_OP_LINEAR: {                // fp32 partial sums of K-slices (small batch; GEMMs with few tiles)
            const size_t a = skinny_workspace_bytes(rows, cols, m), b = gemm_workspace_bytes(rows, cols, m);
            return a > b ? a : b;
        }
        case RAZER_OP_LINEAR_W4A4:             // room for the activations decoded to bf16 ahead of the weight-only path
            return w4a4_staged_bytes(rows, cols, m);
        default: return 0;
    }
}

}  // extern "C"

namespace {
size_t w4a4_staged_bytes(int64_t rows, int64_t cols, int64_t m)
{
    const size_t base = razer_workspace_bytes(RAZER_OP_LINEAR, rows, cols, m);
    if (rows <= 0 || cols <= 0 || m <= 0) return base;
    return (((size_t)m * (size_t)cols * 2u + 255u) & ~(size_t)255u) + 256u + base;
}
}  // namespace

extern "C" {

size_t razer_workspace_bytes_grouped(int32_t count, const int64_t* rows, int64_t cols, int64_t m)
{
    if (!rows || count < 1 || count > RAZER_MAX_GROUP || cols <= 0 || m <= kGemvDirectMaxM) return 0;
    // what the single launch needs (K-slices of all matrices side by side) ...
    size_t one = 0, each = 0;
    GemvProblem p[RAZER_MAX_GROUP];
    for (int i = 0; i < count; ++i) {
        if (rows[i] < 0) return 0;
        p[i] = GemvProblem{nullptr, nullptr, nullptr, rows[i], nullptr, rows[i]};
        // ... and what the sequence of single calls needs, should the group not qualify for one launch
        const size_t b = razer_workspace_bytes(RAZER_OP_LINEAR, rows[i], cols, m);
        each = b > each ? b : each;
    }
    if (m <= kSkinnyMaxM) {
        one = skinny_grouped_workspace_bytes(count, p, cols, m);
    } else if (gemm_grouped_fits(count, p, m, cols)) {
        one = gemm_grouped_workspace_bytes(count, p, m, cols);
    }
    return one > each ? one : each;
}

razer_status razer_quantize(const razer_config* cfg, const void* x, int32_t dtype, int64_t rows, int64_t cols,
                            int64_t ld, uint8_t* codes, uint8_t* scales, float* tensor_scale, uint32_t flags,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!cfg || !tensor_scale) return RAZER_ERR_NULL;
    SvConfig sv;
    razer_status s = check_cfg(*cfg, sv);
    if (s != RAZER_OK) return s;
    if (dtype != RAZER_F32 && dtype != RAZER_BF16) return RAZER_ERR_CONFIG;
    if (flags & ~RAZER_GIVEN_TENSOR_SCALE) return RAZER_ERR_CONFIG;
    if (rows < 0 || !cols_ok(cols, sv) || ld < cols) return RAZER_ERR_SHAPE;
    const size_t esz = (dtype == RAZER_F32) ? 4 : 2;
    if (rows > 0 && cols > 0) {
        if (!x || !codes || !scales) return RAZER_ERR_NULL;
        if (!aligned16(x) || !aligned16(codes) || !aligned16(scales) || ((size_t)ld * esz) % 16 != 0)
            return RAZER_ERR_ALIGN;
    }
    const int given = (flags & RAZER_GIVEN_TENSOR_SCALE) ? 1 : 0;
    if (!given) {
        if (!workspace || workspace_bytes < razer_workspace_bytes(RAZER_OP_QUANTIZE, rows, cols, 0) ||
            !aligned16(workspace))
            return RAZER_ERR_WORKSPACE;
    }
    hipError_t e = launch_quantize(cfg->format, sv, x, dtype == RAZER_BF16, rows, cols, ld, codes, scales,
                                   tensor_scale, given, workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? RAZER_OK : RAZER_ERR_HIP;
}

razer_status razer_dequant(const razer_tensor* t, void* out, int32_t dtype, int64_t ld, void* hip_stream)
{
    SvConfig sv;
    razer_status s = check_tensor(t, -1, sv);
    if (s != RAZER_OK) return s;
    if (dtype != RAZER_F32 && dtype != RAZER_BF16) return RAZER_ERR_CONFIG;
    if (sv.il) return RAZER_ERR_CONFIG;                                  // the decoder takes the canonical layout
    if (ld < t->cols) return RAZER_ERR_SHAPE;
    const size_t esz = (dtype == RAZER_F32) ? 4 : 2;
    if (t->rows > 0 && t->cols > 0) {
        if (!out) return RAZER_ERR_NULL;
        if (!aligned16(out) || ((size_t)ld * esz) % 16 != 0) return RAZER_ERR_ALIGN;
    }
    hipError_t e = launch_dequant(t->cfg.format, sv, t->codes, t->scales, t->tensor_scale, t->rows, t->cols, out,
                                  dtype == RAZER_BF16, ld, (hipStream_t)hip_stream);
    return e == hipSuccess ? RAZER_OK : RAZER_ERR_HIP;
}

razer_status razer_linear(const razer_tensor* w, const void* a_bf16, const razer_tensor* a_q, int64_t m,
                          void* y_bf16, int64_t ld_y, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    SvConfig wsv, asv = {5.0f, 5.0f};
    razer_status s = check_tensor(w, RAZER_FMT_WEIGHT, wsv);
    if (s != RAZER_OK) return s;
    if (m < 0 || ld_y < w->rows) return RAZER_ERR_SHAPE;
    if (m == 0 && !a_q) return RAZER_OK;                                  // nothing to compute, operands may be NULL
    if ((a_bf16 == nullptr) == (a_q == nullptr)) return RAZER_ERR_NULL;   // exactly one activation operand
    const int64_t n = w->rows, k = w->cols;
    // the interleaved layout serves the decode regime only: bf16 activations, m <= 4, rows of at most 32768
    if (wsv.il && (a_q || m > kGemvDirectMaxM || k > 32768)) return RAZER_ERR_CONFIG;
    if (a_q) {
        s = check_tensor(a_q, RAZER_FMT_ACT, asv);
        if (s != RAZER_OK) return s;
        if (a_q->rows != m || a_q->cols != k) return RAZER_ERR_SHAPE;
    } else if (m > 0 && k > 0 && !aligned16(a_bf16)) {
        return RAZER_ERR_ALIGN;
    }
    if (m > 0 && n > 0 && !y_bf16) return RAZER_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (m == 0 || n == 0) return RAZER_OK;
    hipError_t e;
    if (a_q && k > 0 && !wsv.f16 && workspace && aligned16(workspace) && workspace_bytes >= w4a4_staged_bytes(n, k, m)) {
        // W4A4 with room in the workspace: the activation tensor is decoded ONCE to bf16 (block scale x element:
        // the values the fused kernel stages, exact for the paper's special values) and the layer runs on the
        // weight-only path for this m, with the product of the two tensor scales in place of the weights' scale.
        // Same products, fp32 accumulation; only the order of the sum differs from the fused kernel's.
        uint8_t* wsb = (uint8_t*)workspace;
        const size_t a_bytes = ((size_t)m * (size_t)k * 2u + 255u) & ~(size_t)255u;
        float* prod = (float*)(wsb + a_bytes);
        e = launch_dequant(RAZER_FMT_ACT, asv, a_q->codes, a_q->scales, nullptr, m, k, wsb, 1, k, st, w->tensor_scale,
                           a_q->tensor_scale, prod);
        if (e != hipSuccess) return RAZER_ERR_HIP;
        razer_tensor w2 = *w;
        w2.tensor_scale = prod;
        const size_t rest = workspace_bytes - a_bytes - 256u;
        return razer_linear(&w2, wsb, nullptr, m, y_bf16, ld_y, rest ? wsb + a_bytes + 256u : nullptr, rest, hip_stream);
    }
    if (k == 0) {                                                        // empty contraction: Y = 0
        const int64_t total = m * n;
        launch(fill_zero_bf16_kernel, (unsigned)((total + 255) / 256), 256, 0, st, (uint16_t*)y_bf16, m, n, ld_y);
        e = hipGetLastError();
    } else if (wsv.f16) {
        // FP16-scale format: the GEMV kernels up to 4 activation rows, the K-in-workgroup small-batch kernel up
        // to 64, beyond that the tiled matrix-core kernels; all matrix-core kernels multiply bare FP4 operands
        // and fold each block's partial sums with its scale in fp32
        if (a_q) return RAZER_ERR_CONFIG;
        if (m <= kGemvDirectMaxM || (m <= kSkinnyMaxM && k > kSkinnyMaxK))
            e = launch_gemv(wsv, w->codes, w->scales, w->tensor_scale, n, k, (const uint16_t*)a_bf16, m,
                            (uint16_t*)y_bf16, ld_y, st);
        else if (m <= 64 && k <= kSkinnyMaxK)                        // K inside the workgroup: no workspace
            e = launch_skinny(wsv, w->codes, w->scales, w->tensor_scale, n, k, (const uint16_t*)a_bf16, m,
                              (uint16_t*)y_bf16, ld_y, nullptr, st);
        else {
            const size_t need = gemm_workspace_bytes(n, k, m);       // K-slices while the tiles are few
            if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return RAZER_ERR_WORKSPACE;
            e = launch_gemm(wsv, w->codes, w->scales, w->tensor_scale, n, k, (const uint16_t*)a_bf16, asv, nullptr,
                            nullptr, nullptr, m, (uint16_t*)y_bf16, ld_y, need > 0 ? (float*)workspace : nullptr, st);
        }
    } else if (!a_q && m > kGemvDirectMaxM && m <= kSkinnyMaxM && k <= kSkinnyMaxK) {
        const size_t need = skinny_workspace_bytes(n, k, m);
        if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return RAZER_ERR_WORKSPACE;
        e = launch_skinny(wsv, w->codes, w->scales, w->tensor_scale, n, k, (const uint16_t*)a_bf16, m,
                          (uint16_t*)y_bf16, ld_y, (float*)workspace, st);
    } else if (!a_q && m <= kGemvDirectMaxM) {
        e = launch_gemv(wsv, w->codes, w->scales, w->tensor_scale, n, k, (const uint16_t*)a_bf16, m,
                        (uint16_t*)y_bf16, ld_y, st);
    } else {
        const size_t need = gemm_workspace_bytes(n, k, m);
        if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return RAZER_ERR_WORKSPACE;
        e = launch_gemm(wsv, w->codes, w->scales, w->tensor_scale, n, k, (const uint16_t*)a_bf16, asv,
                        a_q ? a_q->codes : nullptr, a_q ? a_q->scales : nullptr,
                        a_q ? a_q->tensor_scale : nullptr, m, (uint16_t*)y_bf16, ld_y,
                        need > 0 ? (float*)workspace : nullptr, st);
    }
    return e == hipSuccess ? RAZER_OK : RAZER_ERR_HIP;
}

size_t razer_prepack_bytes(const razer_tensor* t)
{
    if (!t || t->rows < 0 || t->cols < 0) return 0;
    return (size_t)(t->rows * il_row_bytes(t->cols));
}

razer_status razer_prepack(const razer_tensor* t, void* packed, size_t packed_bytes, void* hip_stream)
{
    SvConfig sv;
    razer_status s = check_tensor(t, RAZER_FMT_WEIGHT, sv);
    if (s != RAZER_OK) return s;
    if (sv.il || sv.f16 || sv.lb != 4) return RAZER_ERR_CONFIG;          // a canonical scale-byte tensor, blocks of 16
    const size_t need = razer_prepack_bytes(t);
    if (need == 0) return RAZER_OK;
    if (!packed) return RAZER_ERR_NULL;
    if (!aligned16(packed)) return RAZER_ERR_ALIGN;
    if (packed_bytes < need) return RAZER_ERR_WORKSPACE;
    const int64_t units = (int64_t)(need / 16);
    launch(prepack_kernel, (unsigned)((units + 255) / 256), 256, 0, (hipStream_t)hip_stream, t->codes, t->scales, t->rows,
           t->cols, (uint8_t*)packed);
    return hipGetLastError() == hipSuccess ? RAZER_OK : RAZER_ERR_HIP;
}

razer_status razer_linear_static(const razer_tensor* w, const void* a_bf16, const razer_tensor* a_q, int64_t m,
                                 void* y_bf16, int64_t ld_y, void* hip_stream)
{
    if (!w) return RAZER_ERR_NULL;
    if (w->rows < 0 || w->cols < 0 || m < 0) return RAZER_ERR_SHAPE;
    // sizes whose K-slices do not fit the static array are refused, never truncated
    if (razer_workspace_bytes(RAZER_OP_LINEAR, w->rows, w->cols, m) > kStaticScratchBytes) return RAZER_ERR_WORKSPACE;
    void* ws = static_scratch();
    if (!ws) return RAZER_ERR_HIP;
    // every K-slice is written by the main kernel before the reduction reads it: nothing to clear
    return razer_linear(w, a_bf16, a_q, m, y_bf16, ld_y, ws, kStaticScratchBytes, hip_stream);
}

razer_status razer_linear_grouped(const razer_tensor* const* w, int32_t count, const void* a_bf16, int64_t m,
                                  void* const* y_bf16, const int64_t* ld_y, void* workspace,
                                  size_t workspace_bytes, void* hip_stream)
{
    if (!w || !y_bf16 || !ld_y) return RAZER_ERR_NULL;
    if (count < 1 || count > RAZER_MAX_GROUP) return RAZER_ERR_SHAPE;
    SvConfig sv0;
    bool one_launch = m >= 1;
    for (int i = 0; i < count; ++i) {
        SvConfig sv;
        razer_status s = check_tensor(w[i], RAZER_FMT_WEIGHT, sv);
        if (s != RAZER_OK) return s;
        if (w[i]->cols != w[0]->cols) return RAZER_ERR_SHAPE;
        if (m < 0 || ld_y[i] < w[i]->rows) return RAZER_ERR_SHAPE;
        if (m > 0 && w[i]->rows > 0 && !y_bf16[i]) return RAZER_ERR_NULL;
        if (i == 0) sv0 = sv;
        else if (sv.sv0 != sv0.sv0 || sv.sv1 != sv0.sv1 || sv.lb != sv0.lb || sv.f16 != sv0.f16) one_launch = false;
        if (sv.il != sv0.il && i > 0) return RAZER_ERR_CONFIG;           // one layout per group
        if (sv.il && (m > kGemvDirectMaxM || w[i]->cols > 32768)) return RAZER_ERR_CONFIG;
        if (w[i]->rows == 0) one_launch = false;
    }
    if (m == 0) return RAZER_OK;
    if (!a_bf16) return RAZER_ERR_NULL;
    const int64_t k = w[0]->cols;
    if (k > 0 && !aligned16(a_bf16)) return RAZER_ERR_ALIGN;
    GemvProblem p[RAZER_MAX_GROUP];
    for (int i = 0; i < count; ++i)
        p[i] = GemvProblem{w[i]->codes, w[i]->scales, w[i]->tensor_scale, w[i]->rows, (uint16_t*)y_bf16[i], ld_y[i]};
    hipStream_t st = (hipStream_t)hip_stream;
    if (k == 0) one_launch = false;
    // which single-launch kernel, if any
    enum { SEQUENCE, GEMV, SKINNY, GEMM } path = SEQUENCE;
    if (one_launch) {
        if (m <= kGemvDirectMaxM) {
            path = GEMV;                                 // every block size and both weight formats
        } else if (sv0.f16 && m > kSkinnyMaxM) {
            path = SEQUENCE;                             // FP16 scale words: no grouped matrix-core launch
        } else if (m <= kSkinnyMaxM && k > kSkinnyMaxK) {
            path = SEQUENCE;
        } else if (m <= kSkinnyMaxM) {
            // the K-slices of all matrices live in the workspace side by side
            const size_t need = sv0.f16 ? 0 : skinny_grouped_workspace_bytes(count, p, k, m);
            bool ok = true;
            for (int i = 0; i < count; ++i) {
                if (p[i].n % 4 != 0 || (reinterpret_cast<uintptr_t>(p[i].y) & 7u) != 0 || p[i].ld_y % 4 != 0) ok = false;
            }
            if (ok && (need == 0 || (workspace && workspace_bytes >= need && aligned16(workspace)))) path = SKINNY;
        } else if (gemm_grouped_fits(count, p, m, k)) {
            // 33..128 rows with few tiles: K-slices of all matrices in the workspace, summed by the grouped
            // reduction (which stores four columns at a time)
            const size_t need = gemm_grouped_workspace_bytes(count, p, m, k);
            bool ok = true;
            if (need > 0) {
                ok = workspace && workspace_bytes >= need && aligned16(workspace);
                for (int i = 0; i < count; ++i)
                    if (p[i].n % 4 != 0 || (reinterpret_cast<uintptr_t>(p[i].y) & 7u) != 0 || p[i].ld_y % 4 != 0) ok = false;
            }
            if (ok) path = GEMM;
        }
    }
    hipError_t e = hipSuccess;
    switch (path) {
        case GEMV: e = launch_gemv_grouped(sv0, count, p, k, (const uint16_t*)a_bf16, m, st); break;
        case SKINNY: e = launch_skinny_grouped(sv0, count, p, k, (const uint16_t*)a_bf16, m, (float*)workspace, st); break;
        case GEMM: e = launch_gemm_grouped(sv0, count, p, k, (const uint16_t*)a_bf16, m, (float*)workspace, st); break;
        case SEQUENCE:
            for (int i = 0; i < count; ++i) {
                razer_status s = razer_linear(w[i], a_bf16, nullptr, m, y_bf16[i], ld_y[i], workspace, workspace_bytes,
                                              hip_stream);
                if (s != RAZER_OK) return s;
            }
            return RAZER_OK;
    }
    return e == hipSuccess ? RAZER_OK : RAZER_ERR_HIP;
}

}  // extern "C"
