// Measured ceilings of the device the library runs on: a register-resident bf16 MFMA loop (no memory
// traffic at all), a plain streaming copy, and the LDS read rate of the two fragment-load instructions.  The balanced-partition flow takes the "computing power"
// and "memory bandwidth" of each accelerator as hardware constraints (paper Sec. III-A); the benchmark
// reports kernel throughput against these measured figures beside the published ones.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/bapipe_stage.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// four independent 32x32 accumulators per wavefront, operands never leave registers
__global__ __launch_bounds__(256) void k_probe_mfma(float *out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)(threadIdx.x % 3);
        b[i] = (__bf16)1.0f;
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void k_probe_copy(const u32x4 *__restrict__ a, u32x4 *__restrict__ b, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) b[i] = a[i];
}

__global__ __launch_bounds__(256) void k_probe_fill(u32x4 *a, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) a[i] = u32x4{1u, 2u, 3u, 4u};
}

// LDS read rate of one instruction kind with conflict-free addresses (each lane its own consecutive slot):
// KIND 0 = ds_read_b128 (the fragment loads of the forward / input-gradient kernels), 1 = the transposing
// ds_read_b64_tr_b16 (the fragment loads of the weight-gradient kernels).  Every wavefront of a 256-thread
// block reads its own 16 KB window of a 64 KB tile again and again; nothing leaves the compute unit.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
template <int KIND>
__global__ __launch_bounds__(256) void k_probe_lds(float *out, int iters)
{
    __shared__ __align__(16) unsigned char tile[65536];
    for (int i = threadIdx.x; i < 65536 / 16; i += 256) reinterpret_cast<u32x4 *>(tile)[i] = u32x4{(uint32_t)i, 1u, 2u, 3u};
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char *p = tile + wave * 16384 + lane * (KIND == 0 ? 16 : 8);
    uint32_t n = 0;
    for (int i = 0; i < iters; ++i) {
        if (KIND == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {            // 8 x 1 KB per wavefront
                u32x4 v = *reinterpret_cast<const u32x4 *>(p + j * 1024);
                asm volatile("" ::"v"(v));
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) {           // 16 x 512 bytes per wavefront
                s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + j * 512));
                asm volatile("" ::"v"(v));
            }
        }
        asm volatile("" ::: "memory");
        ++n;
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = (float)n;
}

}  // namespace

extern "C" int bapipe_measure_lds(void *hip_stream, double *read_b128_tbs, double *read_b64_tr_tbs)
{
    if (!read_b128_tbs || !read_b64_tr_tbs) return BAPIPE_E_INVALID;
    hipStream_t s = (hipStream_t)hip_stream;
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return BAPIPE_E_DEVICE;
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const int blocks = cus * 2, iters = 20000;
    float *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = BAPIPE_E_DEVICE;
    float ms = 0.f;
    if (hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)) != hipSuccess) return BAPIPE_E_OOM;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
    for (int kind = 0; kind < 2; ++kind) {
        if (kind == 0) hipLaunchKernelGGL(k_probe_lds<0>, dim3(blocks), dim3(256), 0, s, out, 64);      // warm-up
        else hipLaunchKernelGGL(k_probe_lds<1>, dim3(blocks), dim3(256), 0, s, out, 64);
        (void)hipEventRecord(e0, s);
        if (kind == 0) hipLaunchKernelGGL(k_probe_lds<0>, dim3(blocks), dim3(256), 0, s, out, iters);
        else hipLaunchKernelGGL(k_probe_lds<1>, dim3(blocks), dim3(256), 0, s, out, iters);
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) goto done;
        // blocks x 4 wavefronts x iters x 8 KB
        const double tbs = (double)blocks * 4.0 * iters * 8192.0 / (ms * 1e-3) / 1e12;
        *(kind == 0 ? read_b128_tbs : read_b64_tr_tbs) = tbs;
    }
    rc = hipGetLastError() == hipSuccess ? BAPIPE_OK : BAPIPE_E_DEVICE;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(out);
    return rc;
}

extern "C" int bapipe_measure_peaks(void *hip_stream, double *mfma_bf16_tflops, double *copy_gbs)
{
    if (!mfma_bf16_tflops || !copy_gbs) return BAPIPE_E_INVALID;
    hipStream_t s = (hipStream_t)hip_stream;
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return BAPIPE_E_DEVICE;
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const size_t n = (size_t)1 << 24;                      // 16-byte words: 256 MiB read + 256 MiB written per pass
    u32x4 *a = nullptr, *b = nullptr;
    float *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = BAPIPE_E_DEVICE;
    float ms = 0.f;
    const int blocks = cus * 2, iters = 8192, passes = 8;
    if (hipMalloc(&a, n * 16) != hipSuccess || hipMalloc(&b, n * 16) != hipSuccess ||
        hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)) != hipSuccess) { rc = BAPIPE_E_OOM; goto done; }
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_probe_mfma, dim3(blocks), dim3(256), 0, s, out, 64);                 // warm-up
    (void)hipEventRecord(e0, s);
    hipLaunchKernelGGL(k_probe_mfma, dim3(blocks), dim3(256), 0, s, out, iters);
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) goto done;
    // blocks x 4 wavefronts x iters x 4 MFMAs x 2*32*32*16 FLOP
    *mfma_bf16_tflops = (double)blocks * 4.0 * iters * 4.0 * 32768.0 / (ms * 1e-3) / 1e12;
    hipLaunchKernelGGL(k_probe_fill, dim3(cus * 8), dim3(256), 0, s, a, n);
    hipLaunchKernelGGL(k_probe_copy, dim3(cus * 8), dim3(256), 0, s, a, b, n);                 // warm-up
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < passes; ++i) hipLaunchKernelGGL(k_probe_copy, dim3(cus * 8), dim3(256), 0, s, a, b, n);
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) goto done;
    *copy_gbs = (double)passes * 2.0 * n * 16.0 / (ms * 1e-3) / 1e9;                           // bytes read + written
    rc = hipGetLastError() == hipSuccess ? BAPIPE_OK : BAPIPE_E_DEVICE;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(a);
    (void)hipFree(b);
    (void)hipFree(out);
    return rc;
}
