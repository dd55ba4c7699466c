// Measured ceilings of the device the library runs on, for the roofline figures of the
// benchmark: what a register-resident MFMA loop and a plain streaming kernel reach on this
// GPU, next to the datasheet peaks the fractions are quoted against.  Nothing of the
// convolution or cheap-layer arithmetic lives here.
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Four independent accumulator tiles per wave, operands in registers: nothing but the matrix pipe.
__global__ void __launch_bounds__(256) mfma_bf16_loop(float *out, int iters)
{
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 7);
        b[i] = (__bf16)(float)(i & 3);
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ void __launch_bounds__(256) mfma_f32_loop(float *out, int iters)
{
    const float a = (float)(threadIdx.x & 7), b = (float)(threadIdx.x & 3);
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Streaming kernels: 16 bytes per lane and step, four steps in flight, consecutive lanes on
// consecutive addresses.  n16 = number of 16-byte items; the grid covers them exactly once.
__global__ void __launch_bounds__(256) stream_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (base + u * 256 < n16) v[u] = src[base + u * 256];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (base + u * 256 < n16) dst[base + u * 256] = v[u];
}

__global__ void __launch_bounds__(256) stream_read(const uint4 *__restrict__ src, uint32_t *__restrict__ sink, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    uint32_t s = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (base + u * 256 < n16) {
            const uint4 v = src[base + u * 256];
            s ^= v.x ^ v.y ^ v.z ^ v.w;
        }
    if (s == 0x9e3779b9u) sink[0] = s;   // keeps the loads alive; practically never taken
}

__global__ void __launch_bounds__(256) stream_write(uint4 *__restrict__ dst, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (base + u * 256 < n16) dst[base + u * 256] = make_uint4(1, 2, 3, 4);
}

// The bf16 MFMA loop with its operands arriving the way the 3x3 tile kernels get them: a wave owns
// 64 channels x 128 pixels (eight accumulator tiles); per filter column (24 MFMAs) it fetches six
// 1 KB filter items from an L2-resident buffer one column ahead and reads six pixel operands from
// LDS; per 16-channel chunk (72 MFMAs) every thread moves 32 bytes from memory into LDS behind one
// barrier, as the patch does.  Addresses are trivial and nothing is transposed or stored: what is
// left is the cost of the operand streams themselves.  src: FED_SRC_BYTES of readable memory.
constexpr unsigned FED_SRC_BYTES = 2u << 20;

union FedOp { uint4 u; bf16x8 v; };

__global__ void __launch_bounds__(256, 2) mfma_bf16_fed_loop(const uint4 *__restrict__ src, float *out, int chunks)
{
    constexpr unsigned MASK = FED_SRC_BYTES / 16 - 1;
    __shared__ uint4 lds[2048];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 2048; i += 256) lds[i] = make_uint4(0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);
    __syncthreads();
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;
    FedOp a[3][6], b[3][6];
    // the two waves of a channel half stream the same items; workgroups start at different places
    unsigned pos = (blockIdx.x * 2 + (wave >> 1)) * 1152u * 7u;
    const int lbase = (wave & 1) * 1024;
    auto fetch = [&](FedOp (&an)[6], FedOp (&bn)[6], int col) {
#pragma unroll
        for (int j = 0; j < 6; ++j) an[j].u = src[(pos + j * 64 + lane) & MASK];
        pos += 6 * 64;
#pragma unroll
        for (int j = 0; j < 6; ++j) bn[j].u = lds[lbase + ((col * 6 + j) * 64 + lane) % 1024];
    };
    auto multiply = [&](FedOp (&ac)[6], FedOp (&bc)[6]) {
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bc[(r + f) % 6].v, ac[r * 2 + i].v, acc[i][f], 0, 0, 0);
    };
    fetch(a[0], b[0], 0);
    for (int c = 0; c < chunks; ++c) {
        fetch(a[1], b[1], 1);
        multiply(a[0], b[0]);
        fetch(a[2], b[2], 2);
        multiply(a[1], b[1]);
        fetch(a[0], b[0], 0);
        multiply(a[2], b[2]);
        const uint4 t0 = src[(pos + 4096 + tid) & MASK], t1 = src[(pos + 8192 + tid) & MASK];
        __syncthreads();
        lds[(c & 1) * 512 + tid] = t0;
        lds[1024 + (c & 1) * 512 + tid] = t1;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][f][v];
    out[blockIdx.x * 256 + tid] = s;
}

__global__ void __launch_bounds__(256) fill_pattern(uint4 *dst, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = make_uint4(0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);   // bf16 2^-7 everywhere
}

}  // namespace
}  // namespace sn

using namespace sn;

extern "C" sn_status sn_measure_ceiling(sn_ceiling_kind kind, void *buf, size_t buf_bytes, int iters,
                                        sn_stream stream, double *value)
{
    if (!value || iters < 1 || kind < SN_CEIL_MFMA_BF16 || kind > SN_CEIL_MFMA_BF16_FED) return SN_ERR_BAD_ARG;
    if (!buf || (reinterpret_cast<uintptr_t>(buf) & 255) != 0) return SN_ERR_BAD_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool fed = kind == SN_CEIL_MFMA_BF16_FED;
    const bool mfma = kind == SN_CEIL_MFMA_BF16 || kind == SN_CEIL_MFMA_F32 || fed;
    const int fed_blocks = 256 * 2, fed_chunks = 600;   // two workgroups per compute unit, as the tile kernels run
    const int blocks = 256 * 8;   // eight workgroups of four waves per compute unit
    const int loop = 4000;        // MFMA steps per launch and accumulator tile
    size_t half = 0, n16 = 0;
    if (mfma) {
        if (buf_bytes < (size_t)blocks * 256 * sizeof(float) + (fed ? FED_SRC_BYTES : 0)) return SN_ERR_WORKSPACE_TOO_SMALL;
    } else {
        half = (kind == SN_CEIL_COPY ? buf_bytes / 2 : buf_bytes) / 4096 * 4096;
        n16 = half / 16;
        if (n16 == 0 || n16 / 1024 + 1 > 0x7fffffffULL) return SN_ERR_WORKSPACE_TOO_SMALL;
    }
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SN_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SN_ERR_LAUNCH; }
    auto launch = [&]() {
        const dim3 grid_s((unsigned)((n16 + 1023) / 1024));
        switch (kind) {
        case SN_CEIL_MFMA_BF16:
            hipLaunchKernelGGL(mfma_bf16_loop, dim3(blocks), dim3(256), 0, st, static_cast<float *>(buf), loop); break;
        case SN_CEIL_MFMA_F32:
            hipLaunchKernelGGL(mfma_f32_loop, dim3(blocks), dim3(256), 0, st, static_cast<float *>(buf), loop); break;
        case SN_CEIL_MFMA_BF16_FED:
            hipLaunchKernelGGL(mfma_bf16_fed_loop, dim3(fed_blocks), dim3(256), 0, st, static_cast<const uint4 *>(buf),
                               reinterpret_cast<float *>(static_cast<char *>(buf) + FED_SRC_BYTES), fed_chunks); break;
        case SN_CEIL_COPY:
            hipLaunchKernelGGL(stream_copy, grid_s, dim3(256), 0, st, static_cast<const uint4 *>(buf),
                               reinterpret_cast<uint4 *>(static_cast<char *>(buf) + half), n16); break;
        case SN_CEIL_READ:
            hipLaunchKernelGGL(stream_read, grid_s, dim3(256), 0, st, static_cast<const uint4 *>(buf),
                               static_cast<uint32_t *>(buf), n16); break;
        default:
            hipLaunchKernelGGL(stream_write, grid_s, dim3(256), 0, st, static_cast<uint4 *>(buf), n16); break;
        }
    };
    sn_status result = SN_OK;
    float best = -1.f;
    if (fed) hipLaunchKernelGGL(fill_pattern, dim3(FED_SRC_BYTES / 16 / 256), dim3(256), 0, st, static_cast<uint4 *>(buf), (size_t)FED_SRC_BYTES / 16);
    launch();   // untimed
    for (int i = 0; i < iters && result == SN_OK; ++i) {
        float ms = 0.f;
        if (hipEventRecord(e0, st) != hipSuccess) { result = SN_ERR_LAUNCH; break; }
        launch();
        if (hipGetLastError() != hipSuccess || hipEventRecord(e1, st) != hipSuccess ||
            hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            result = SN_ERR_LAUNCH;
            break;
        }
        if (best < 0.f || ms < best) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != SN_OK) return result;
    if (fed) {
        *value = (double)fed_blocks * 4 * fed_chunks * 72 * (2.0 * 32 * 32 * 16) / (best * 1e-3) / 1e12;   // TFLOP/s
    } else if (mfma) {
        const double flop_per = kind == SN_CEIL_MFMA_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
        *value = (double)blocks * 4 * loop * 4 * flop_per / (best * 1e-3) / 1e12;   // TFLOP/s
    } else {
        const double bytes = kind == SN_CEIL_COPY ? 2.0 * (double)half : (double)half;
        *value = bytes / (best * 1e-3) / 1e9;   // GB/s
    }
    return SN_OK;
}
