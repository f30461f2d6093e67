// Measurement aid of the benchmark (its own small library, libhkprobe.so; not part of libhybridkv and no
// operation of the paper): the matrix-core rate this GPU sustains on a loop of nothing but
// v_mfma_f32_16x16x32_f16 (the instruction of the projection kernel, on its 8 x 8 grid of accumulator
// blocks), with all-zero or with random operands.  On MI355X the two differ widely (the shader clock
// drops under random fp16 operands), so the second number is the practical ceiling against which the
// projection kernel's fraction of the published peak should be read.  The accumulators are pinned to
// their registers by inline asm: left to the register allocator, a loop over 64 four-register
// accumulators gets shuffled between register files and measures the shuffling.
#include <stddef.h>
#include <stdint.h>
#include <hip/hip_runtime.h>

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void mfma_rate_kernel(float *sink, int iters, int random_operands)
{
    float4_t acc[64];
#pragma unroll
    for (int q = 0; q < 64; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[q][r] = 0.f;
    half8_t a[8], b[8];
    unsigned x = 12345u + threadIdx.x * 7919u + blockIdx.x * 104729u;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            x = x * 1664525u + 1013904223u;
            a[i][e] = random_operands ? (_Float16)(((int)(x >> 8) % 2001 - 1000) * 0.001f) : (_Float16)0.f;
            x = x * 1664525u + 1013904223u;
            b[i][e] = random_operands ? (_Float16)(((int)(x >> 8) % 2001 - 1000) * 0.00002f) : (_Float16)0.f;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 64; ++q)
            asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[q]) : "v"(a[q >> 3]), "v"(b[q & 7]));
    }
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 64; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += acc[q][r];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

// Runs the loop on every compute unit (4 wavefronts each, `iters` x 64 instructions per wavefront) and returns the
// sustained rate in TFLOP/s through tflops_out (host).  `sink` is device scratch of at least (compute units) * 1024
// bytes.  Synchronises the stream.  Returns 0, or a negative number: -1 null pointer, -2 bad iteration count,
// -5 sink too small, -7 a HIP call failed.
extern "C" int hkprobe_mfma_rate(int32_t random_operands, int32_t iters, float *sink, size_t sink_bytes,
                                 float *tflops_out, void *stream)
{
    enum { HK_OK = 0, HK_ERR_NULL = -1, HK_ERR_SHAPE = -2, HK_ERR_WORKSPACE = -5, HK_ERR_LAUNCH = -7 };
    if (!sink || !tflops_out) return HK_ERR_NULL;
    if (iters <= 0 || iters > (1 << 22)) return HK_ERR_SHAPE;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return HK_ERR_LAUNCH;
    if (sink_bytes < (size_t)cus * 256 * sizeof(float)) return HK_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return HK_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return HK_ERR_LAUNCH; }
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(cus), dim3(256), 0, s, sink, iters / 8 + 1, random_operands);   // warm up
    (void)hipEventRecord(e0, s);
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(cus), dim3(256), 0, s, sink, iters, random_operands);
    (void)hipEventRecord(e1, s);
    int rc = HK_OK;
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
        rc = HK_ERR_LAUNCH;
    else
        *tflops_out = (float)((double)cus * 4 * iters * 64 * 16384.0 / (ms * 1e-3) / 1e12);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
