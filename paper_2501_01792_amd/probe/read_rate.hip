// Measurement aid (part of libhkprobe.so, not of libhybridkv and no operation of the paper): the rate at which a
// row-major matrix of 16-bit elements streams from HBM when every wavefront owns 32 rows and keeps a fixed number
// of 16-byte-per-lane loads in flight, for different shapes of one load instruction (8 rows x 128 bytes, which is
// what the MFMA operand staging of the streaming kernels asks for, down to 1 row x 1024 bytes) and for plain and
// non-temporal loads.  It says what the load structure of those kernels can reach before any arithmetic.
// Read-only; every address lies inside the caller's buffer.
#include <stddef.h>
#include <stdint.h>
#include <hip/hip_runtime.h>

namespace {

typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kDepth = 20;                                   // loads in flight per wavefront

template <int RPI, bool NT>
__global__ __launch_bounds__(256) void read_rate_kernel(const unsigned char *base, int64_t ld_bytes, int row_bytes,
                                                        int rows_total, unsigned *out)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int row0 = gw * 32;
    if (row0 + 32 > rows_total) return;                      // whole wavefront; no barrier in this kernel
    constexpr int LPR = 64 / RPI;                            // lanes per row
    constexpr int SEG = 16 * LPR;                            // bytes per row per instruction
    constexpr int G = 32 / RPI;                              // instructions per segment of the 32 rows
    const int rin = lane / LPR, chunk = lane % LPR;
    const int total = (row_bytes / SEG) * G;
    const unsigned char *p0 = base + (int64_t)(row0 + rin) * ld_bytes + chunk * 16;
    auto load = [&](int idx) {
        if (idx >= total) idx = total - 1;                   // past the end: the last piece again
        const int seg = idx / G, rg = idx % G;
        const uint4v *src = reinterpret_cast<const uint4v *>(p0 + (int64_t)rg * RPI * ld_bytes + (int64_t)seg * SEG);
        return NT ? __builtin_nontemporal_load(src) : *src;
    };
    uint4v buf[kDepth];
#pragma unroll
    for (int u = 0; u < kDepth; ++u) buf[u] = load(u);
    uint4v acc = {0, 0, 0, 0};
    for (int i = 0; i < total; i += kDepth) {
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            acc ^= buf[u];
            buf[u] = load(i + kDepth + u);
        }
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345u) out[gw] = 1;   // keeps the loads alive
}

// The same stream (8 rows x 128 bytes per load, 4 loads = one step of 32 rows x 64 elements, kDepth / 4 steps in
// flight) with, one by one, what a streaming MFMA kernel adds around it, so that each addition's cost in read rate
// can be seen: BAR a workgroup barrier per step; L2 three more 16-byte loads per thread and step from a small
// region every workgroup shares (the shared operand's tile, an L2 hit); LDS every piece written to a private
// 4 KiB LDS block and read back in MFMA operand layout; MMA the 12 MFMAs (3 row blocks of the shared operand x 4 k
// pieces) a streaming product issues per step, on the pieces as they are; TILE the shared operand written to a
// double-buffered LDS tile and read from there as 12 more fragments per step.  (With MMA the rate depends on the
// data: operands that toggle lower the clock.)
template <bool BAR, bool L2, bool LDS, bool MMA = false, bool TILE = false>
__global__ __launch_bounds__(256) void stream_parts_kernel(const unsigned char *base, int64_t ld_bytes, int row_bytes,
                                                           int rows_total, const unsigned char *shared_rows, unsigned *out)
{
    __shared__ __align__(16) unsigned char blocks[4 * 4096];
    __shared__ __align__(16) unsigned char tile[TILE ? 2 * 3 * 4096 : 16];     // TILE: the shared operand goes through LDS as well
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gw = blockIdx.x * 4 + wave;
    const int row0 = gw * 32;                                // rows_total is a multiple of 128: every wavefront has rows
    const int rin = lane >> 3, chunk = lane & 7;
    const int steps = row_bytes / 128;
    const unsigned char *p0 = base + (int64_t)(row0 + rin) * ld_bytes + chunk * 16;
    const unsigned char *q0 = shared_rows + (int64_t)(tid >> 3) * ld_bytes + (tid & 7) * 16;   // rows 0 .. 31 (+ 32, + 64)
    unsigned char *my = blocks + wave * 4096;
    int wr_off[4], rd_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + rin;
        wr_off[j] = row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
        rd_off[j] = (lane & 31) * 128 + (((2 * j + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 4);
    }
    constexpr int D = kDepth / 4;                            // steps in flight
    uint4v sv[D][4], tv[D][3];
    auto fetch = [&](int slot, int sc) {
        if (sc >= steps) sc = steps - 1;
        if (L2) {
#pragma unroll
            for (int r = 0; r < 3; ++r) tv[slot][r] = *reinterpret_cast<const uint4v *>(q0 + (int64_t)32 * r * ld_bytes + (int64_t)sc * 128);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) sv[slot][j] = *reinterpret_cast<const uint4v *>(p0 + (int64_t)8 * j * ld_bytes + (int64_t)sc * 128);
    };
#pragma unroll
    for (int u = 0; u < D - 1; ++u) fetch(u, u);
    uint4v acc = {0, 0, 0, 0};
    float16v facc[3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) facc[r][e] = 0.f;
    for (int s = 0; s < steps; s += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            fetch((u + D - 1) % D, s + u + D - 1);
            if (MMA) {                                       // 3 row blocks of the shared operand x 4 k pieces, as a streaming product issues them
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4v *>(my + wr_off[j]) = sv[u][j];
                if (TILE) {                                 // written for the next step, read for this one (the barrier orders them)
                    const int t_row = tid >> 3, t_chunk = tid & 7;
                    const int t_wr = t_row * 128 + ((t_chunk ^ ((t_row >> 1) & 7)) << 4);
#pragma unroll
                    for (int r = 0; r < 3; ++r) *reinterpret_cast<uint4v *>(tile + (((s + u + 1) & 1) * 3 + r) * 4096 + t_wr) = tv[(u + 1) % D][r];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint4v w = *reinterpret_cast<const uint4v *>(my + rd_off[j]);
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        const uint4v a = TILE ? *reinterpret_cast<const uint4v *>(tile + (((s + u) & 1) * 3 + r) * 4096 + rd_off[j]) : tv[u][r];
                        facc[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, w),
                                                                         facc[r], 0, 0, 0);
                    }
                }
                if (BAR) __syncthreads();
                continue;
            }
            if (L2) {
#pragma unroll
                for (int r = 0; r < 3; ++r) acc ^= tv[u][r];
            }
            if (LDS) {
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4v *>(my + wr_off[j]) = sv[u][j];
#pragma unroll
                for (int j = 0; j < 4; ++j) acc ^= *reinterpret_cast<const uint4v *>(my + rd_off[j]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) acc ^= sv[u][j];
            }
            if (BAR) __syncthreads();                        // steps is the same for every wavefront
        }
    }
    if (MMA) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int e = 0; e < 16; ++e) t += facc[r][e];
        if (t == 12345.f) out[gw] = 2;
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345u) out[gw] = 1;
}

template <int RPI, bool NT>
void launch(const unsigned char *buf, int rows, int row_bytes, unsigned *out, hipStream_t s)
{
    hipLaunchKernelGGL((read_rate_kernel<RPI, NT>), dim3(rows / 128), dim3(256), 0, s, buf, (int64_t)row_bytes, row_bytes, rows, out);
}

}  // namespace

// Streams `rows` x `row_bytes` bytes of `buf` (device; rows a multiple of 128, row_bytes a multiple of 1024) `iters`
// times after two warm-up launches and returns the rate in GB/s through gbps_out (host).  rows_per_load: 8, 4, 2 or 1;
// or 100 + flags for stream_parts_kernel (rows must then be at least 96, the shared rows are the buffer's first 96).
// `sink` is device scratch of rows / 32 * 4 bytes.  Synchronises the stream.  Returns 0, or a negative number:
// -1 null pointer, -2 bad shape, -7 a HIP call failed.
extern "C" int hkprobe_read_rate(int32_t rows_per_load, int32_t nontemporal, const void *buf, int32_t rows, int32_t row_bytes,
                                 void *sink, int32_t iters, float *gbps_out, void *stream)
{
    if (!buf || !sink || !gbps_out) return -1;
    if (rows <= 0 || rows % 128 != 0 || row_bytes <= 0 || row_bytes % 1024 != 0 || iters <= 0 || iters > 1000) return -2;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned char *b = static_cast<const unsigned char *>(buf);
    unsigned *o = static_cast<unsigned *>(sink);
    auto parts = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3(rows / 128), dim3(256), 0, s, b, (int64_t)row_bytes, row_bytes, rows, b, o);
        return true;
    };
    auto go = [&]() {
        const bool nt = nontemporal != 0;
        switch (rows_per_load) {
        // 100 + flags: the 8 x 128-byte stream with parts of a streaming MFMA kernel added (1 barrier, 2 shared loads, 4 LDS;
        // on top of all three: 8 MFMAs, 16 shared operand through an LDS tile)
        case 100: return parts(stream_parts_kernel<false, false, false>);
        case 101: return parts(stream_parts_kernel<true, false, false>);
        case 102: return parts(stream_parts_kernel<false, true, false>);
        case 103: return parts(stream_parts_kernel<true, true, false>);
        case 104: return parts(stream_parts_kernel<false, false, true>);
        case 105: return parts(stream_parts_kernel<true, false, true>);
        case 106: return parts(stream_parts_kernel<false, true, true>);
        case 107: return parts(stream_parts_kernel<true, true, true>);
        case 115: return parts(stream_parts_kernel<true, true, true, true>);         // 8: + the MFMAs
        case 123: return parts(stream_parts_kernel<true, true, true, true, true>);   // 16: + the shared operand's LDS tile
        case 8: nt ? launch<8, true>(b, rows, row_bytes, o, s) : launch<8, false>(b, rows, row_bytes, o, s); return true;
        case 4: nt ? launch<4, true>(b, rows, row_bytes, o, s) : launch<4, false>(b, rows, row_bytes, o, s); return true;
        case 2: nt ? launch<2, true>(b, rows, row_bytes, o, s) : launch<2, false>(b, rows, row_bytes, o, s); return true;
        case 1: nt ? launch<1, true>(b, rows, row_bytes, o, s) : launch<1, false>(b, rows, row_bytes, o, s); return true;
        default: return false;
        }
    };
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return -7;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -7; }
    int rc = 0;
    if (!go() || !go()) rc = -2;
    if (rc == 0) {
        (void)hipEventRecord(e0, s);
        for (int i = 0; i < iters; ++i) go();
        (void)hipEventRecord(e1, s);
        float ms = 0.f;
        if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
            ms <= 0.f)
            rc = -7;
        else
            *gbps_out = (float)((double)rows * row_bytes * iters / (ms * 1e-3) / 1e9);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
