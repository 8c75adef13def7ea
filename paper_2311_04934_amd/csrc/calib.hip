// Calibration kernels for benchmarks: what this machine sustains on a plain copy and on a loop of
// nothing but matrix instructions.  They give the "achievable" figures that roofline fractions are
// quoted next to; nothing on the request path uses them.
#include "common.h"

namespace pc {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// dst[i] = src[i], 16 bytes per lane, 8 independent loads in flight per lane, grid-stride
__global__ __launch_bounds__(512) void calib_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * 512 * 8;
    for (size_t base = (size_t)blockIdx.x * 512 * 8; base < n_vec; base += stride) {
        u32x4 r[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t i = base + (size_t)u * 512 + threadIdx.x;
            if (i < n_vec) r[u] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t i = base + (size_t)u * 512 + threadIdx.x;
            if (i < n_vec) dst[i] = r[u];
        }
    }
}

// every wave issues `iters` x 16 v_mfma_f32_32x32x16_bf16 on four independent accumulators
__global__ __launch_bounds__(512) void calib_mfma_kernel(float *out, int iters)
{
    f32x16 c[4];
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(threadIdx.x * 1e-3f + i);
        b[i] = (__bf16)(1.f - i);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i & 3], 0, 0, 0);
    }
    float acc = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) acc += c[j][i];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = acc;
}

}  // namespace
}  // namespace pc

extern "C" {

int pc_calib_copy(pc_ctx *ctx, size_t bytes, int repeats, double *gb_per_s)
{
    using namespace pc;
    if (!ctx || bytes < 16 || repeats < 1 || !gb_per_s) return PC_E_BADARG;
    if (hipSetDevice(ctx->device) != hipSuccess) return PC_E_HIP;
    const size_t n_vec = bytes / 16;
    u32x4 *src = nullptr, *dst = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = PC_E_HIP;
    if (hipMalloc(reinterpret_cast<void **>(&src), n_vec * 16) == hipSuccess &&
        hipMalloc(reinterpret_cast<void **>(&dst), n_vec * 16) == hipSuccess &&
        hipMemset(src, 0x3c, n_vec * 16) == hipSuccess && hipEventCreate(&e0) == hipSuccess &&
        hipEventCreate(&e1) == hipSuccess) {
        const int blocks = ctx->n_cu * 8;
        hipLaunchKernelGGL(calib_copy_kernel, dim3(blocks), dim3(512), 0, 0, src, dst, n_vec);   // warm-up
        (void)hipEventRecord(e0, 0);
        for (int r = 0; r < repeats; ++r) hipLaunchKernelGGL(calib_copy_kernel, dim3(blocks), dim3(512), 0, 0, src, dst, n_vec);
        (void)hipEventRecord(e1, 0);
        float ms = 0.f;
        if (hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f) {
            *gb_per_s = 2.0 * (double)(n_vec * 16) * repeats / (ms * 1e-3) / 1e9;   // read + write
            rc = PC_OK;
        }
    }
    (void)hipGetLastError();
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (src) (void)hipFree(src);
    if (dst) (void)hipFree(dst);
    return rc;
}

int pc_calib_mfma(pc_ctx *ctx, int iters, double *tflop_per_s)
{
    using namespace pc;
    if (!ctx || iters < 1 || !tflop_per_s) return PC_E_BADARG;
    if (hipSetDevice(ctx->device) != hipSuccess) return PC_E_HIP;
    const int blocks = ctx->n_cu;   // one workgroup of 8 waves per CU: two waves per SIMD
    float *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = PC_E_HIP;
    if (hipMalloc(reinterpret_cast<void **>(&out), (size_t)blocks * 512 * sizeof(float)) == hipSuccess &&
        hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        hipLaunchKernelGGL(calib_mfma_kernel, dim3(blocks), dim3(512), 0, 0, out, iters);   // warm-up
        (void)hipEventRecord(e0, 0);
        hipLaunchKernelGGL(calib_mfma_kernel, dim3(blocks), dim3(512), 0, 0, out, iters);
        (void)hipEventRecord(e1, 0);
        float ms = 0.f;
        if (hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f) {
            const double flops = (double)blocks * 8 * iters * 16 * 32768.0;   // 2 x 32 x 32 x 16 per instruction
            *tflop_per_s = flops / (ms * 1e-3) / 1e12;
            rc = PC_OK;
        }
    }
    (void)hipGetLastError();
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (out) (void)hipFree(out);
    return rc;
}

}  // extern "C"
