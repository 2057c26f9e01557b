// Measurement utilities of the gfx950 RaZeR library (include/razer_probe.h): nothing here computes any
// part of the method.  Two ceiling kernels -- a pure streaming read and a register-resident bf16 MFMA
// loop -- so that a benchmark can time, in its own run and on its own GPU, what the memory system and
// the matrix cores give a kernel that does nothing else; and the per-thread event pair through which
// launch() reports the duration of single dispatches.
#include "../../include/razer_probe.h"
#include "razer_kernels.hpp"

namespace razer {

ProbeEvents& probe_events()
{
    static thread_local ProbeEvents ev;
    return ev;
}

// Every workgroup walks the buffer grid-stride in 16-byte loads (one 1 KiB wavefront row per load
// instruction, UNROLL loads in flight per lane) and folds what it read with xor; the fold decides a
// store that (almost) never happens, so the loads cannot be dropped and nothing is written.  The loads
// are non-temporal like the GEMV kernels' weight loads (a buffer is read once per launch): with the
// default cache policy the same kernel is up to 9 % slower on a 264 MB buffer.
template <int UNROLL>
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ buf, size_t n16,
                                                          uint32_t* __restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
        uint4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = load_once16(buf + i + u * stride);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        const uint4 v = buf[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) sink[threadIdx.x & 63u] = acc;     // one chance in 2^32 per lane
}

// iters x 8 independent v_mfma_f32_32x32x16_bf16 per wavefront, operands and accumulators in
// registers the whole time: 2 * 32 * 32 * 16 flops per instruction.
__global__ __launch_bounds__(256, 2) void mfma_loop_kernel(int iters, float* __restrict__ sink)
{
    // operands with well-mixed bits (values of magnitude 0.5 .. 2, both signs): the power a matrix
    // instruction draws, and with it the clock the GPU sustains, depends on how many bits toggle
    v8bf a, b;
    uint32_t h = (threadIdx.x + 1u) * 2654435761u + blockIdx.x * 40503u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        h = h * 1664525u + 1013904223u;
        a[i] = __builtin_bit_cast(__bf16, (uint16_t)(0x3F00u | ((h >> 9) & 0x00FFu) | ((h >> 2) & 0x8000u)));
        h = h * 1664525u + 1013904223u;
        b[i] = __builtin_bit_cast(__bf16, (uint16_t)(0x3F00u | ((h >> 9) & 0x00FFu) | ((h >> 2) & 0x8000u)));
    }
    v16f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float t = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) t += acc[j][v];
    if (t == -1.0f) sink[0] = t;                       // never true: keeps the loop alive
}

// The same loop on the block-scaled FP4 matrix instruction (v_mfma_scale_f32_32x32x64_f8f6f4, both operands
// FP4-E2M1, one E8M0 scale per 32 elements and operand, here 2^0): 2 * 32 * 32 * 64 flops per instruction.
// It is what a two-pass FP4 x FP4 realisation of the weight-activation mode would run on.
typedef int v8i32 __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(256, 2) void mfma_fp4_loop_kernel(int iters, float* __restrict__ sink)
{
    v8i32 a, b;
    uint32_t h = (threadIdx.x + 1u) * 2654435761u + blockIdx.x * 40503u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {                      // (only the low four dwords hold FP4 data)
        h = h * 1664525u + 1013904223u;
        a[i] = (int)h;
        h = h * 1664525u + 1013904223u;
        b[i] = (int)h;
    }
    v16f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[j], 4, 4, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
    }
    float t = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) t += acc[j][v];
    if (t == -1.0f) sink[0] = t;                       // never true: keeps the loop alive
}

}  // namespace razer

using namespace razer;

extern "C" {

void razer_probe_dispatch_events(void* start_event, void* stop_event)
{
    ProbeEvents& ev = probe_events();
    ev.start = (hipEvent_t)start_event;
    ev.stop = (hipEvent_t)stop_event;
}

int razer_probe_stream_read(const void* buf, size_t bytes, int workgroups, void* sink, void* hip_stream)
{
    if (!buf || !sink) return 1;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0 || bytes % 16 != 0 || workgroups < 1 || workgroups > (1 << 20)) return 2;
    launch(stream_read_kernel<4>, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream,
           (const uint4*)buf, bytes / 16, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : 6;
}

int razer_probe_mfma_bf16(int iters, int workgroups, void* sink, void* hip_stream, double* flops)
{
    if (!sink) return 1;
    if (iters < 1 || workgroups < 1 || workgroups > (1 << 20)) return 2;
    launch(mfma_loop_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, (float*)sink);
    if (flops) *flops = 2.0 * 32 * 32 * 16 * 8.0 * iters * 4.0 * workgroups;   // 4 wavefronts per workgroup
    return hipGetLastError() == hipSuccess ? 0 : 6;
}

int razer_probe_mfma_fp4(int iters, int workgroups, void* sink, void* hip_stream, double* flops)
{
    if (!sink) return 1;
    if (iters < 1 || workgroups < 1 || workgroups > (1 << 20)) return 2;
    launch(mfma_fp4_loop_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, (float*)sink);
    if (flops) *flops = 2.0 * 32 * 32 * 64 * 8.0 * iters * 4.0 * workgroups;
    return hipGetLastError() == hipSuccess ? 0 : 6;
}

}  // extern "C"
