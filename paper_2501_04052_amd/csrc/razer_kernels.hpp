// Host-side launchers of the gfx950 RaZeR kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "razer_device.hpp"

namespace razer {

// Every kernel of the library is launched through launch().  Measurement hook: a host thread may
// hand the library a pair of HIP events (razer_probe_dispatch_events); while they are set, each launch
// made by that thread records the begin and end time stamps of its own dispatch into them -- the
// duration a kernel trace reports per dispatch, without a profiler attached.  Both are null otherwise,
// and the launch is then an ordinary one.
struct ProbeEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
ProbeEvents& probe_events();          // this thread's pair (razer_probe.hip)

template <typename... KArgs, typename... Args>
inline void launch(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t smem, hipStream_t st, Args... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "kernel argument count");
    const ProbeEvents& ev = probe_events();
    hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)smem, st, ev.start, ev.stop, 0u, static_cast<KArgs>(args)...);
}

// Launch shape of a problem: this thread's forced shape (source 1), else the entry of the built-in table
// (source 2), else source 0 -- the caller's heuristic applies (razer_tune.hip; families and parameters as in
// include/razer_tune.h).
struct TuneShape {
    int p[4];
    int source;
};
enum { kTuneGemv = 0, kTuneGemvQuad = 1, kTuneSmallBatch = 2, kTuneGemmSlices = 3 };
TuneShape tuned_shape(int family, int64_t m, int64_t n, int64_t k);

// Encoder (absmax pass + block encoder).  ws: >= 16 bytes of device scratch.
hipError_t launch_quantize(int fmt, SvConfig cfg, const void* x, int dtype_bf16, int64_t rows, int64_t cols,
                           int64_t ld, uint8_t* codes, uint8_t* scales, float* tensor_scale, int given,
                           void* ws, hipStream_t st);

// Decoder to fp32 or bf16 (tensor_scale == nullptr: block scale x element only).  prod_out != nullptr: the
// launch also leaves *prod_a x *prod_b there (one fp32 rounding) -- the combined tensor scale of a W4A4 layer.
hipError_t launch_dequant(int fmt, SvConfig cfg, const uint8_t* codes, const uint8_t* scales,
                          const float* tensor_scale, int64_t rows, int64_t cols, void* out, int dtype_bf16,
                          int64_t ld, hipStream_t st, const float* prod_a = nullptr, const float* prod_b = nullptr,
                          float* prod_out = nullptr);

// Y[m][n] = A[m][:] . W[n][:], m <= kGemvMaxM: wavefront dot products, HBM-bound (4 rows per pass).
constexpr int kGemvMaxM = 16;
constexpr int kGemvDirectMaxM = 4;     // rows the GEMV kernel takes in one pass
constexpr int kSkinnyMaxM = 32;        // above this the tiled GEMM takes over
// The small-batch kernel and the register-decode GEMM address inside a row block / tile with 32-bit
// offsets (up to 31 rows x 2 K bytes, resp. 255 rows x 2 K bytes); longer rows take the LDS-staged GEMM.
constexpr int64_t kSkinnyMaxK = (int64_t)1 << 24;
constexpr int64_t kRbMaxK = (int64_t)1 << 22;

// 5 <= m <= kSkinnyMaxM: decode-once MFMA kernel; K-slices meet in an fp32 workspace of
// skinny_workspace_bytes(n, k, m) bytes (0 when a single slice covers K).
size_t skinny_workspace_bytes(int64_t n, int64_t k, int64_t m);
hipError_t launch_skinny(SvConfig cfg, const uint8_t* codes, const uint8_t* scales, const float* ts, int64_t n,
                         int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y, float* workspace,
                         hipStream_t st);
// y = bf16(scale * sum of the K-slices' fp32 partial sums [slices][m][n], in slice order); scale = -ts_w,
// or ts_w * ts_a when a_ts is given.
hipError_t launch_slice_reduce(const float* partial, const float* w_ts, const float* a_ts, int64_t m, int64_t n,
                               int nslices, uint16_t* y, int64_t ld_y, hipStream_t st);
hipError_t launch_gemv(SvConfig wcfg, const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts,
                       int64_t n, int64_t k, const uint16_t* a, int64_t m, uint16_t* y, int64_t ld_y,
                       hipStream_t st);

// Up to 4 weight matrices sharing K, the activation rows and the special values, one launch (m <= 4 here).
struct GemvProblem {
    const uint8_t* codes;
    const uint8_t* scales;
    const float* ts;
    int64_t n;
    uint16_t* y;
    int64_t ld_y;
};
hipError_t launch_gemv_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                               int64_t m, hipStream_t st);
// workspace of a grouped small-batch launch (the launch shape is chosen for the rows of all matrices together)
size_t skinny_grouped_workspace_bytes(int count, const GemvProblem* p, int64_t k, int64_t m);

// Same contraction on bf16 matrix cores with LDS-staged decoded tiles.  Activations are
// bf16 (a != nullptr) or RaZeR activation-format (a_codes != nullptr).
// Problems with few output tiles split K over workgroups; the slices meet in an fp32 workspace of
// gemm_workspace_bytes(n, k, m) bytes (0 when K is not split).
size_t gemm_workspace_bytes(int64_t n, int64_t k, int64_t m);
hipError_t launch_gemm(SvConfig wcfg, const uint8_t* w_codes, const uint8_t* w_scales, const float* w_ts,
                       int64_t n, int64_t k, const uint16_t* a, SvConfig acfg, const uint8_t* a_codes,
                       const uint8_t* a_scales, const float* a_ts, int64_t m, uint16_t* y, int64_t ld_y,
                       float* workspace, hipStream_t st);

// Grouped form of launch_skinny (5 <= m <= 32, any block size, every n a positive multiple of 4);
// workspace = the matrices' skinny_workspace_bytes added up, matrix after matrix.
hipError_t launch_skinny_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                                 int64_t m, float* workspace, hipStream_t st);

// Sum of the K-slices of a grouped launch: partial holds matrix i's [nslices][m][n_i] fp32 slices
// behind those of matrices 0 .. i-1 (every n a positive multiple of 4, y 8-byte aligned, ld_y % 4 == 0).
hipError_t launch_slice_reduce_grouped(const float* partial, int count, const GemvProblem* p, int64_t m, int nslices,
                                       hipStream_t st);

// Up to 4 weight matrices (equal block size and special values, every n > 0, k > 0) against the
// same bf16 activations in one launch of the register-decode GEMM kernel; possible when
// gemm_grouped_fits() says so (m >= 33).  gemm_grouped_workspace_bytes() > 0 (few output tiles: K is
// sliced): the launch needs that many bytes of workspace and the conditions of
// launch_slice_reduce_grouped.
bool gemm_grouped_fits(int count, const GemvProblem* p, int64_t m, int64_t k);
size_t gemm_grouped_workspace_bytes(int count, const GemvProblem* p, int64_t m, int64_t k);
hipError_t launch_gemm_grouped(SvConfig cfg, int count, const GemvProblem* p, int64_t k, const uint16_t* a,
                               int64_t m, float* workspace, hipStream_t st);

}  // namespace razer
