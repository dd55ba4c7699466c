// The cheap layers that cost-aware recomputation replays (Sec. 3.4 of the
// paper): ACT (ReLU), BN (training mode) and POOL (max), forward and backward.
// All of them stream an N*C*H*W tensor once or twice and are bound by HBM
// bandwidth, so the kernels are about 16-byte coalesced accesses, enough
// workgroups for 256 compute units, and fixed-order wavefront reductions for
// the BN statistics.  Storage is fp32 or bf16; arithmetic is fp32.
#include "sn_internal.h"
#include <type_traits>

namespace sn {
namespace {

constexpr int WAVE = 64;

template <typename T> __device__ inline float ld(const T *p);
template <> __device__ inline float ld<float>(const float *p) { return *p; }
template <> __device__ inline float ld<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ inline void st(float *p, float v) { *p = v; }
__device__ inline void st(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// 16-byte vector of T, unpacked to / packed from floats.
template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float *p, float (&f)[4])
    {
        float4 v = *reinterpret_cast<const float4 *>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static void store(float *p, const float (&f)[4])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(f[0], f[1], f[2], f[3]);
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t *p, float (&f)[8])
    {
        uint4 v = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static void store(bf16_t *p, const float (&f)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// ------------------------------------------------------------------ ReLU
// Flat streaming kernels: each thread moves UNROLL 16-byte vectors, a workgroup
// covers one contiguous run; the ragged end (< one vector) is done by scalars.
constexpr int RELU_UNROLL = 4;

template <typename T>
__global__ void __launch_bounds__(256) relu_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, size_t n)
{
    constexpr int V = Vec<T>::N;
    const size_t nvec = n / V;
    const size_t base = (size_t)blockIdx.x * (256 * RELU_UNROLL) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < RELU_UNROLL; ++u) {
        const size_t i = base + (size_t)u * 256;
        if (i < nvec) {
            uint4 v = reinterpret_cast<const uint4 *>(x)[i];
            if (sizeof(T) == 2) {
                // a bf16 is positive iff its sign bit is clear: clear every half whose sign is set
                uint32_t *w = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t neg = (w[k] >> 15) & 0x00010001u;
                    w[k] &= ~(neg * 0xffffu);
                }
            } else {
                float *f = reinterpret_cast<float *>(&v);
#pragma unroll
                for (int k = 0; k < 4; ++k) f[k] = f[k] > 0.f ? f[k] : 0.f;
            }
            reinterpret_cast<uint4 *>(y)[i] = v;
        }
    }
    if (blockIdx.x == 0) {
        const size_t i = nvec * V + threadIdx.x;
        if (threadIdx.x < V && i < n) {
            float f = ld<T>(x + i);
            st(y + i, f > 0.f ? f : 0.f);
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(256)
relu_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy, T *__restrict__ dx, size_t n)
{
    constexpr int V = Vec<T>::N;
    const size_t nvec = n / V;
    const size_t base = (size_t)blockIdx.x * (256 * RELU_UNROLL) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < RELU_UNROLL; ++u) {
        const size_t i = base + (size_t)u * 256;
        if (i < nvec) {
            uint4 xv = reinterpret_cast<const uint4 *>(x)[i];
            uint4 gv = reinterpret_cast<const uint4 *>(dy)[i];
            if (sizeof(T) == 2) {
                const uint32_t *xw = reinterpret_cast<const uint32_t *>(&xv);
                uint32_t *gw = reinterpret_cast<uint32_t *>(&gv);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    // x > 0 iff the 16 bits are in 0x0001 .. 0x7fff
                    uint32_t lo = xw[k] & 0xffffu, hi = xw[k] >> 16;
                    uint32_t keep = ((lo - 1u) < 0x7fffu ? 0x0000ffffu : 0u) | ((hi - 1u) < 0x7fffu ? 0xffff0000u : 0u);
                    gw[k] &= keep;
                }
            } else {
                const float *xf = reinterpret_cast<const float *>(&xv);
                float *gf = reinterpret_cast<float *>(&gv);
#pragma unroll
                for (int k = 0; k < 4; ++k) gf[k] = xf[k] > 0.f ? gf[k] : 0.f;
            }
            reinterpret_cast<uint4 *>(dx)[i] = gv;
        }
    }
    if (blockIdx.x == 0) {
        const size_t i = nvec * V + threadIdx.x;
        if (threadIdx.x < V && i < n) {
            float f = ld<T>(x + i), gr = ld<T>(dy + i);
            st(dx + i, f > 0.f ? gr : 0.f);
        }
    }
}

// ------------------------------------------------------------------ BN
// One channel's data is N planes of HW contiguous elements.  The planes are cut
// into segments of at most SEG elements; a wavefront takes one segment at a
// time and walks it with 16-byte accesses (scalar head and tail when the segment
// does not start or end on a 16-byte boundary -- planes with odd H*W do not).
// Workgroup (c, slice) takes the segments slice*4 + wave, stepping by 4*nslice,
// so which wave adds which element, and in what order, depends on the shape
// only: the statistics are bit-identical from run to run.
constexpr int SEG = 4096;

struct Slices {
    int nseg_plane;  // segments per plane
    int nseg;        // segments per channel = N * nseg_plane
    int nslice;      // workgroups per channel
};

template <typename T, typename FVec, typename FOne>
__device__ inline void walk_segment(const T *p, int len, int lane, FVec fvec, FOne fone)
{
    constexpr int V = Vec<T>::N;
    const int mis = (int)((reinterpret_cast<uintptr_t>(p) & 15u) / sizeof(T));
    int head = (V - mis) % V;
    if (head > len) head = len;
    if (lane < head) fone(lane);
    const int nvec = (len - head) / V;
    for (int i = lane; i < nvec; i += WAVE) fvec(head + i * V);
    const int done = head + nvec * V;
    if (lane < len - done) fone(done + lane);
}

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// Raw vectors of VB bytes of T, unpacked to / packed from floats.
template <int VB> struct RawVec;
template <> struct RawVec<16> { typedef uint4 type; };
template <> struct RawVec<8> { typedef uint2 type; };
template <> struct RawVec<4> { typedef uint32_t type; };
template <> struct RawVec<2> { typedef unsigned short type; };   // one bf16

template <typename T, int VB> __device__ inline void unpack(const typename RawVec<VB>::type &v, float (&f)[VB / sizeof(T)])
{
    if constexpr (VB == 2) {
        f[0] = __uint_as_float((uint32_t)v << 16);
        return;
    }
    const uint32_t *w = reinterpret_cast<const uint32_t *>(&v);
    if (sizeof(T) == 2) {
#pragma unroll
        for (int i = 0; i < VB / 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < VB / 4; ++i) f[i] = __uint_as_float(w[i]);
    }
}

template <typename T, int VB> __device__ inline typename RawVec<VB>::type pack(const float (&f)[VB / sizeof(T)])
{
    if constexpr (VB == 2) return f32_to_bf16(f[0]);
    typename RawVec<VB>::type v;
    uint32_t *w = reinterpret_cast<uint32_t *>(&v);
    if (sizeof(T) == 2) {
#pragma unroll
        for (int i = 0; i < VB / 4; ++i)
            w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
    } else {
#pragma unroll
        for (int i = 0; i < VB / 4; ++i) w[i] = __float_as_uint(f[i]);
    }
    return v;
}

// Where a backward pass takes the gradient dy from: the tensor itself, or -- when a 2x2 / stride-2
// max-pool (no padding) follows the layer -- the pooled gradient g [N*C][H/2][W/2] and the winners'
// positions idx, from which each element's gradient is formed on the fly exactly as the pool
// backward would have stored it: g of its window if the element is the window's winner, else 0.
template <typename T> struct GradSrc {
    const T *dy;            // the gradient itself, or nullptr
    const T *g;             // pooled gradient
    const int32_t *idx;     // position h*W + v of each window's winner inside its input plane
    int W, Q, HW, PQ;
};

// Gradient of element e of plane pl.
template <typename T> __device__ inline float grad_one(const GradSrc<T> &gs, size_t pl, int e)
{
    if (gs.dy) return ld<T>(gs.dy + pl * gs.HW + e);
    const int h = e / gs.W, w = e - h * gs.W;
    const size_t wi = pl * gs.PQ + (size_t)(h >> 1) * gs.Q + (w >> 1);
    return gs.idx[wi] == e ? ld<T>(gs.g + wi) : 0.f;
}

// Gradients of the VB / sizeof(T) elements from element e (a multiple of that count within the
// plane's 16-byte grid, hence even).  Where a vector cannot cross a row (W a multiple of the
// vector length) its windows' entries are one aligned vector of g and one of idx.
template <typename T, int VB>
__device__ inline void grad_vec(const GradSrc<T> &gs, size_t pl, int e, float (&gr)[VB / sizeof(T)])
{
    constexpr int VE = VB / sizeof(T);
    if (gs.dy) {
        unpack<T, VB>(*reinterpret_cast<const typename RawVec<VB>::type *>(gs.dy + pl * gs.HW + e), gr);
        return;
    }
    if constexpr (VE == 1) {   // single elements: planes of odd size, which no 2x2 pool follows
        gr[0] = grad_one<T>(gs, pl, e);
    } else if (gs.W % VE == 0) {
        const int h = e / gs.W, w = e - h * gs.W;
        const size_t wi = pl * gs.PQ + (size_t)(h >> 1) * gs.Q + (w >> 1);
        float gw[VE / 2];
        unpack<T, VB / 2>(*reinterpret_cast<const typename RawVec<VB / 2>::type *>(gs.g + wi), gw);
        const typename RawVec<2 * VE>::type iv = *reinterpret_cast<const typename RawVec<2 * VE>::type *>(gs.idx + wi);
        const int32_t *iw = reinterpret_cast<const int32_t *>(&iv);
#pragma unroll
        for (int k = 0; k < VE; ++k) gr[k] = iw[k >> 1] == e + k ? gw[k >> 1] : 0.f;
    } else {
#pragma unroll
        for (int k = 0; k < VE; k += 2) {
            const int ee = e + k, h = ee / gs.W, w = ee - h * gs.W;
            const size_t wi = pl * gs.PQ + (size_t)(h >> 1) * gs.Q + (w >> 1);
            const int win = gs.idx[wi];
            const float g = ld<T>(gs.g + wi);
            gr[k] = win == ee ? g : 0.f;
            gr[k + 1] = win == ee + 1 ? g : 0.f;
        }
    }
}

// The activation that may follow BN in the same pass: ReLU as in relu_fwd_kernel (0 unless v > 0).
__device__ inline float act(float v, int relu) { return (!relu || v > 0.f) ? v : 0.f; }

// The BN output before the activation.  Forward and backward both go through this one
// expression (a single fused multiply-add), so the backward pass can re-derive from x,
// bit for bit, what the forward pass stored.
__device__ inline float bn_affine(float x, float mu, float a, float b) { return __builtin_fmaf(x - mu, a, b); }

// Whether the stored output of BN + ReLU is > 0 for the BN output v: v > 0, and for bf16
// storage v does not round to zero (every positive float above 0x8000 rounds to a
// nonzero bf16).  This is the gate of the ReLU backward, taken without reading the output.
template <typename T> __device__ inline bool relu_passes(float v)
{
    if (sizeof(T) == 2) return v > 0.f && __float_as_uint(v) > 0x8000u;
    return v > 0.f;
}

// Pass 1 (forward): per (channel, slice) partial sums of (x - shift) and
// (x - shift)^2, shift = the channel's first element, which keeps the variance
// free of cancellation whatever the channel's mean is.
template <typename T>
__global__ void __launch_bounds__(256)
bn_stats_kernel(const T *__restrict__ x, float *__restrict__ part, int N, int C, int HW, Slices sl)
{
    constexpr int V = Vec<T>::N;
    const int c = blockIdx.x, slice = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float shift = ld<T>(x + (size_t)c * HW);
    float s1 = 0.f, s2 = 0.f;
    for (int seg = slice * 4 + wave; seg < sl.nseg; seg += 4 * sl.nslice) {
        const int n = seg / sl.nseg_plane, k = seg - n * sl.nseg_plane;
        const int e0 = k * SEG, len = min(SEG, HW - e0);
        const T *p = x + ((size_t)n * C + c) * HW + e0;
        walk_segment<T>(
            p, len, lane,
            [&](int off) {
                float f[V];
                Vec<T>::load(p + off, f);
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    float d = f[i] - shift;
                    s1 += d;
                    s2 += d * d;
                }
            },
            [&](int off) {
                float d = ld<T>(p + off) - shift;
                s1 += d;
                s2 += d * d;
            });
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    __shared__ float red[2][4];
    if (lane == 0) { red[0][wave] = s1; red[1][wave] = s2; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float *o = part + ((size_t)c * sl.nslice + slice) * 2;
        o[0] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        o[1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

// Pass 2 (forward): one wavefront per channel folds the slices in fixed order.
template <typename T>
__global__ void __launch_bounds__(64)
bn_stats_final_kernel(const T *__restrict__ x, const float *__restrict__ part, float *__restrict__ mean,
                      float *__restrict__ invstd, int N, int HW, int nslice, float eps)
{
    const int c = blockIdx.x, lane = threadIdx.x;
    double s1 = 0.0, s2 = 0.0;
    for (int i = lane; i < nslice; i += WAVE) {
        s1 += part[((size_t)c * nslice + i) * 2];
        s2 += part[((size_t)c * nslice + i) * 2 + 1];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        s1 += __shfl_xor(s1, o, WAVE);
        s2 += __shfl_xor(s2, o, WAVE);
    }
    if (lane == 0) {
        const double M = (double)N * (double)HW;
        const double shift = (double)ld<T>(x + (size_t)c * HW);
        const double d = s1 / M;
        double var = s2 / M - d * d;
        if (var < 0.0) var = 0.0;
        mean[c] = (float)(shift + d);
        invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
    }
}

// Statistics from the partial results the CONV kernels leave per (channel, pixel tile): count,
// mean, and sum of squared deviations from that mean.  Two such triples combine exactly
// (pairwise update).  One workgroup of 1024 threads per channel: a thread folds the tiles
// t, t + 1024, ... in order, the threads of a wave combine in a butterfly, and thread 0 folds
// the sixteen waves' results, all in fp64 and always in the same order.
struct Moments { double n, mu, m2; };

__device__ inline void moments_fold(Moments &a, double nb, double mb, double m2b)
{
    if (!(nb > 0.0)) return;
    const double nt = a.n + nb, d = mb - a.mu, r = nb / nt;
    a.mu += d * r;
    a.m2 += m2b + d * d * (a.n * r);
    a.n = nt;
}

__global__ void __launch_bounds__(1024)
bn_finalize_tiles_kernel(const float *__restrict__ part, int ntiles, float *__restrict__ mean,
                         float *__restrict__ invstd, float eps)
{
    const int c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Moments a = {0.0, 0.0, 0.0};
    for (int t = tid; t < ntiles; t += 1024) {
        const float *e = part + ((size_t)c * ntiles + t) * 3;
        moments_fold(a, (double)e[0], (double)e[1], (double)e[2]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const Moments b = {__shfl_xor(a.n, o, WAVE), __shfl_xor(a.mu, o, WAVE), __shfl_xor(a.m2, o, WAVE)};
        // both partners arrive at the same bits: the higher lane's triple is folded into the lower's
        if (lane & o) {
            const Moments own = a;
            a = b;
            moments_fold(a, own.n, own.mu, own.m2);
        } else {
            moments_fold(a, b.n, b.mu, b.m2);
        }
    }
    __shared__ double red[16][3];
    if (lane == 0) { red[wave][0] = a.n; red[wave][1] = a.mu; red[wave][2] = a.m2; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 16; ++w) moments_fold(a, red[w][0], red[w][1], red[w][2]);
        double var = a.n > 0.0 ? a.m2 / a.n : 0.0;
        if (var < 0.0) var = 0.0;
        mean[c] = (float)a.mu;
        invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
    }
}

// Pass 3 (forward): y = gamma*invstd*(x - mean) + beta.
template <typename T>
__global__ void __launch_bounds__(256)
bn_apply_kernel(const T *__restrict__ x, T *__restrict__ y, const float *__restrict__ gamma,
                const float *__restrict__ beta, const float *__restrict__ mean,
                const float *__restrict__ invstd, int N, int C, int HW, Slices sl, int relu)
{
    constexpr int V = Vec<T>::N;
    // the statistics pass has just read x front to back: walking it back to front finds the
    // part that was read last still in the memory-side cache
    const int c = gridDim.x - 1 - blockIdx.x, slice = gridDim.y - 1 - blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float mu = mean[c], a = gamma[c] * invstd[c], b = beta[c];
    const int seg0 = slice * 4 + wave, step = 4 * sl.nslice;
    for (int seg = seg0 + (seg0 < sl.nseg ? (sl.nseg - 1 - seg0) / step * step : 0); seg >= seg0 && seg < sl.nseg; seg -= step) {
        const int n = seg / sl.nseg_plane, k = seg - n * sl.nseg_plane;
        const int e0 = k * SEG, len = min(SEG, HW - e0);
        const size_t base = ((size_t)n * C + c) * HW + e0;
        const T *p = x + base;
        T *o = y + base;
        walk_segment<T>(
            p, len, lane,
            [&](int off) {
                float f[V];
                Vec<T>::load(p + off, f);
#pragma unroll
                for (int i = 0; i < V; ++i) f[i] = act(bn_affine(f[i], mu, a, b), relu);
                Vec<T>::store(o + off, f);
            },
            [&](int off) { st(o + off, act(bn_affine(ld<T>(p + off), mu, a, b), relu)); });
    }
}

// Backward pass 1: per (channel, slice) partial sums of dy and dy*(x - mean).
template <typename T>
__global__ void __launch_bounds__(256)
bn_bwd_reduce_kernel(const T *__restrict__ x, const GradSrc<T> gs, const float *__restrict__ gamma,
                     const float *__restrict__ beta, const float *__restrict__ mean,
                     const float *__restrict__ invstd, float *__restrict__ part, int N, int C, int HW, Slices sl)
{
    constexpr int V = Vec<T>::N;
    const int c = blockIdx.x, slice = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float mu = mean[c];
    const bool relu = beta != nullptr;
    const float ga = gamma[c] * invstd[c], gb = relu ? beta[c] : 0.f;
    float s1 = 0.f, s2 = 0.f;
    for (int seg = slice * 4 + wave; seg < sl.nseg; seg += 4 * sl.nslice) {
        const int n = seg / sl.nseg_plane, k = seg - n * sl.nseg_plane;
        const int e0 = k * SEG, len = min(SEG, HW - e0);
        const size_t base = ((size_t)n * C + c) * HW + e0;
        const T *p = x + base;
        const size_t pl = (size_t)n * C + c;
        walk_segment<T>(
            p, len, lane,
            [&](int off) {
                float f[V], gr[V];
                Vec<T>::load(p + off, f);
                grad_vec<T, 16>(gs, pl, e0 + off, gr);
                if (relu) {
#pragma unroll
                    for (int i = 0; i < V; ++i) gr[i] = relu_passes<T>(bn_affine(f[i], mu, ga, gb)) ? gr[i] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    s1 += gr[i];
                    s2 += gr[i] * (f[i] - mu);
                }
            },
            [&](int off) {
                const float f = ld<T>(p + off);
                float gr = grad_one<T>(gs, pl, e0 + off);
                if (relu && !relu_passes<T>(bn_affine(f, mu, ga, gb))) gr = 0.f;
                s1 += gr;
                s2 += gr * (f - mu);
            });
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    __shared__ float red[2][4];
    if (lane == 0) { red[0][wave] = s1; red[1][wave] = s2; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float *o = part + ((size_t)c * sl.nslice + slice) * 2;
        o[0] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        o[1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

__global__ void __launch_bounds__(64)
bn_bwd_final_kernel(const float *__restrict__ part, const float *__restrict__ invstd,
                    float *__restrict__ dgamma, float *__restrict__ dbeta, int nslice)
{
    const int c = blockIdx.x, lane = threadIdx.x;
    double s1 = 0.0, s2 = 0.0;
    for (int i = lane; i < nslice; i += WAVE) {
        s1 += part[((size_t)c * nslice + i) * 2];
        s2 += part[((size_t)c * nslice + i) * 2 + 1];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        s1 += __shfl_xor(s1, o, WAVE);
        s2 += __shfl_xor(s2, o, WAVE);
    }
    if (lane == 0) {
        dbeta[c] = (float)s1;
        dgamma[c] = (float)(s2 * (double)invstd[c]);
    }
}

// Backward pass 3: dx = gamma*invstd * (dy - dbeta/M - xhat*dgamma/M).
template <typename T>
__global__ void __launch_bounds__(256)
bn_bwd_apply_kernel(const T *__restrict__ x, const GradSrc<T> gs, const float *__restrict__ beta,
                    T *__restrict__ dx, const float *__restrict__ gamma, const float *__restrict__ mean,
                    const float *__restrict__ invstd, const float *__restrict__ dgamma,
                    const float *__restrict__ dbeta, int N, int C, int HW, Slices sl)
{
    constexpr int V = Vec<T>::N;
    // back to front, as in bn_apply_kernel: the sums pass has just read x and dy front to back
    const int c = gridDim.x - 1 - blockIdx.x, slice = gridDim.y - 1 - blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float invM = 1.f / ((float)N * (float)HW);
    const float mu = mean[c], is = invstd[c], k1 = gamma[c] * is;
    const float kb = dbeta[c] * invM, kg = dgamma[c] * invM * is;  // xhat*dgamma/M = (x-mu)*kg
    const bool relu = beta != nullptr;
    const float gb = relu ? beta[c] : 0.f;
    const int seg0 = slice * 4 + wave, step = 4 * sl.nslice;
    for (int seg = seg0 + (seg0 < sl.nseg ? (sl.nseg - 1 - seg0) / step * step : 0); seg >= seg0 && seg < sl.nseg; seg -= step) {
        const int n = seg / sl.nseg_plane, k = seg - n * sl.nseg_plane;
        const int e0 = k * SEG, len = min(SEG, HW - e0);
        const size_t base = ((size_t)n * C + c) * HW + e0;
        const T *p = x + base;
        const size_t pl = (size_t)n * C + c;
        T *o = dx + base;
        walk_segment<T>(
            p, len, lane,
            [&](int off) {
                float f[V], gr[V];
                Vec<T>::load(p + off, f);
                grad_vec<T, 16>(gs, pl, e0 + off, gr);
                if (relu) {
#pragma unroll
                    for (int i = 0; i < V; ++i) gr[i] = relu_passes<T>(bn_affine(f[i], mu, k1, gb)) ? gr[i] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < V; ++i) f[i] = k1 * (gr[i] - kb - (f[i] - mu) * kg);
                Vec<T>::store(o + off, f);
            },
            [&](int off) {
                const float f = ld<T>(p + off);
                float gr = grad_one<T>(gs, pl, e0 + off);
                if (relu && !relu_passes<T>(bn_affine(f, mu, k1, gb))) gr = 0.f;
                st(o + off, k1 * (gr - kb - (f - mu) * kg));
            });
    }
}

// ---- BN in one pass over HBM, for channels that fit in the registers of one workgroup.
// A workgroup of BT threads (1024, or 256 where that holds the channel: four times the workgroups per
// compute unit, which is what the short channels of small planes need) takes one channel: thread t holds
// vectors t, t + BT, ...
// (16 or 8 bytes each) of the channel's N*HW elements from the load until the store, so x
// (and dy) are read once and y (dx) written once.  The statistics are two-pass sums over
// the registers, reduced in a fixed order (wavefront butterflies, then the 16 wavefront
// sums in index order), so they are the same from run to run.
// BN + ReLU + 2x2 / stride-2 max-pool (no padding) of one unit: VB bytes of input row 2p and the
// same columns of row 2p + 1 give VB / (2 sizeof(T)) windows.  The activations are rounded to
// the storage type before they are compared, so values, winners and ties (first maximum in
// row-major window order) are those of the pool run on the stored BN + ReLU output.
template <typename T, int VB>
__device__ inline void bn_relu_pool2_unit(const T *__restrict__ x, T *__restrict__ pooled, int32_t *__restrict__ idx,
                                          int u, int c, int C, int H, int W, float mu, float a, float b)
{
    constexpr int VE = VB / sizeof(T);
    typedef typename RawVec<VB>::type VT;
    const int vpr = W / VE, P = H >> 1, Q = W >> 1, upp = P * vpr;
    const int n = u / upp, r = u - n * upp, p = r / vpr, qv = r - p * vpr;
    const size_t pl = (size_t)n * C + c;
    const T *r0 = x + (pl * H + 2 * p) * W + qv * VE;
    float fa[VE], fb[VE];
    unpack<T, VB>(*reinterpret_cast<const VT *>(r0), fa);
    unpack<T, VB>(*reinterpret_cast<const VT *>(r0 + W), fb);
#pragma unroll
    for (int k = 0; k < VE; ++k) {
        fa[k] = act(bn_affine(fa[k], mu, a, b), 1);
        fb[k] = act(bn_affine(fb[k], mu, a, b), 1);
    }
    unpack<T, VB>(pack<T, VB>(fa), fa);   // the values as stored
    unpack<T, VB>(pack<T, VB>(fb), fb);
    const int base = 2 * p * W + qv * VE;
    float out[VE / 2];
    typename RawVec<2 * VE>::type oi;
    int32_t *oiw = reinterpret_cast<int32_t *>(&oi);
#pragma unroll
    for (int j = 0; j < VE / 2; ++j) {
        float bv = fa[2 * j];
        int best = base + 2 * j;
        if (fa[2 * j + 1] > bv) { bv = fa[2 * j + 1]; best = base + 2 * j + 1; }
        if (fb[2 * j] > bv) { bv = fb[2 * j]; best = base + W + 2 * j; }
        if (fb[2 * j + 1] > bv) { bv = fb[2 * j + 1]; best = base + W + 2 * j + 1; }
        out[j] = bv;
        oiw[j] = best;
    }
    const size_t o = (pl * P + p) * Q + qv * (VE / 2);
    *reinterpret_cast<typename RawVec<VB / 2>::type *>(pooled + o) = pack<T, VB / 2>(out);   // exact: stored values
    *reinterpret_cast<typename RawVec<2 * VE>::type *>(idx + o) = oi;
}

// Pass 3 of the forward pass when the pool follows: one thread per unit, back to front as in
// bn_apply_kernel; the full-resolution activation is never written.
template <typename T, int VB>
__global__ void __launch_bounds__(256)
bn_relu_pool2_apply_kernel(const T *__restrict__ x, T *__restrict__ pooled, int32_t *__restrict__ idx,
                           const float *__restrict__ gamma, const float *__restrict__ beta,
                           const float *__restrict__ mean, const float *__restrict__ invstd, int C, int H, int W,
                           int units)
{
    const int c = gridDim.x - 1 - blockIdx.x;
    const float mu = mean[c], a = gamma[c] * invstd[c], b = beta[c];
    const int u0 = (gridDim.y - 1 - blockIdx.y) * 256 + threadIdx.x, step = gridDim.y * 256;
    if (u0 >= units) return;
    for (int u = u0 + (units - 1 - u0) / step * step; u >= u0; u -= step)
        bn_relu_pool2_unit<T, VB>(x, pooled, idx, u, c, C, H, W, mu, a, b);
}

// Sum over the BT threads of a workgroup (whole waves), the same value in every thread.
// A vector at any element alignment (the hardware takes unaligned 16-byte accesses; the type tells the compiler).
template <typename VT, typename T> __device__ inline VT load_any(const T *p)
{
    typedef uint32_t u32v __attribute__((ext_vector_type(sizeof(VT) / 4)));
    struct __attribute__((packed, aligned(2))) U { u32v v; };
    const u32v r = reinterpret_cast<const U *>(p)->v;
    VT o;
    __builtin_memcpy(&o, &r, sizeof(VT));
    return o;
}
template <typename VT, typename T> __device__ inline void store_any(T *p, const VT &v)
{
    typedef uint32_t u32v __attribute__((ext_vector_type(sizeof(VT) / 4)));
    struct __attribute__((packed, aligned(2))) U { u32v v; };
    u32v r;
    __builtin_memcpy(&r, &v, sizeof(VT));
    reinterpret_cast<U *>(p)->v = r;
}

template <int BT> __device__ inline float block_sum(float v, float *red)
{
    v = wave_sum(v);
    __syncthreads();   // red may still be read from the previous sum
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) s += red[i];
    return s;
}

// PVB != 0: BN + ReLU + 2x2 max-pool.  The statistics are taken exactly as without the pool (same
// element-to-thread mapping, same order); the last phase then reads the channel a second time in
// units of PVB bytes of a row pair -- the workgroup has just streamed it, so it comes from the
// caches -- and writes the pooled values and indices only (y is not touched; H, W as the pool
// sees them).
// RAG: planes whose size is not a multiple of the vector (7x7, 17x17, 35x35; at least one vector long): a plane
// is ceil(HW / VE) vectors at any alignment, the last one moved back so that it ends with the plane; the elements
// it shares with the one before count once in the sums and are written twice with the same value.
template <typename T, int VB, int NVMAX, int PVB, int BT, bool RAG = false>
__global__ void __launch_bounds__(BT)
bn_fwd_fused_kernel(const T *__restrict__ x, T *__restrict__ y, const float *__restrict__ gamma,
                    const float *__restrict__ beta, float *__restrict__ mean, float *__restrict__ invstd,
                    int N, int C, int HW, float eps, int relu, T *__restrict__ pooled, int32_t *__restrict__ idx,
                    int H, int W)
{
    constexpr int VE = VB / sizeof(T);
    typedef typename RawVec<VB>::type VT;
    __shared__ float red[16];
    const int c = blockIdx.x, tid = threadIdx.x;
    const int vpp = RAG ? (HW + VE - 1) / VE : HW / VE, nvec = N * vpp;
    VT v[NVMAX];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NVMAX; ++j) {
        const int i = tid + j * BT;
        if (i < nvec) {
            const int n = i / vpp, e = i - n * vpp;
            const int eo = RAG ? min(e * VE, HW - VE) : e * VE, kf = e * VE - eo;   // kf: elements the vector before had
            const T *src = x + ((size_t)n * C + c) * HW + (size_t)eo;
            if constexpr (RAG) v[j] = load_any<VT>(src);
            else v[j] = *reinterpret_cast<const VT *>(src);
            float f[VE];
            unpack<T, VB>(v[j], f);
#pragma unroll
            for (int k = 0; k < VE; ++k) s += (!RAG || k >= kf) ? f[k] : 0.f;
        }
    }
    const float M = (float)N * (float)HW;
    const float mu = block_sum<BT>(s, red) / M;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NVMAX; ++j) {
        const int i = tid + j * BT;
        if (i < nvec) {
            const int e = i % vpp, kf = RAG ? e * VE - min(e * VE, HW - VE) : 0;
            float f[VE];
            unpack<T, VB>(v[j], f);
#pragma unroll
            for (int k = 0; k < VE; ++k) q += (!RAG || k >= kf) ? (f[k] - mu) * (f[k] - mu) : 0.f;
        }
    }
    const float var = block_sum<BT>(q, red) / M;
    const float is = 1.f / sqrtf(var + eps);
    if (tid == 0) { mean[c] = mu; invstd[c] = is; }
    const float a = gamma[c] * is, b = beta[c];
    if (PVB != 0) {
        constexpr int PB = PVB ? PVB : 16;
        const int units = N * (H >> 1) * (W / (PB / (int)sizeof(T)));
        for (int u = tid; u < units; u += BT) bn_relu_pool2_unit<T, PB>(x, pooled, idx, u, c, C, H, W, mu, a, b);
        return;
    }
#pragma unroll
    for (int j = 0; j < NVMAX; ++j) {
        const int i = tid + j * BT;
        if (i < nvec) {
            const int n = i / vpp, e = i - n * vpp;
            const int eo = RAG ? min(e * VE, HW - VE) : e * VE;
            float f[VE];
            unpack<T, VB>(v[j], f);
#pragma unroll
            for (int k = 0; k < VE; ++k) f[k] = act(bn_affine(f[k], mu, a, b), relu);
            T *dst = y + ((size_t)n * C + c) * HW + (size_t)eo;
            if constexpr (RAG) store_any<VT>(dst, pack<T, VB>(f));
            else *reinterpret_cast<VT *>(dst) = pack<T, VB>(f);
        }
    }
}

template <typename T, int VB, int NVMAX, int BT, bool RAG = false>
__global__ void __launch_bounds__(BT)
bn_bwd_fused_kernel(const T *__restrict__ x, const GradSrc<T> gs, const float *__restrict__ beta,
                    T *__restrict__ dx, const float *__restrict__ gamma, const float *__restrict__ mean,
                    const float *__restrict__ invstd, float *__restrict__ dgamma, float *__restrict__ dbeta,
                    int N, int C, int HW)
{
    constexpr int VE = VB / sizeof(T);
    typedef typename RawVec<VB>::type VT;
    __shared__ float red[16];
    const int c = blockIdx.x, tid = threadIdx.x;
    const int vpp = RAG ? (HW + VE - 1) / VE : HW / VE, nvec = N * vpp;
    const float mu = mean[c], is = invstd[c];
    const bool relu = beta != nullptr;
    const float ga = gamma[c] * is, gb = relu ? beta[c] : 0.f;
    VT xv[NVMAX], gv[NVMAX];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NVMAX; ++j) {
        const int i = tid + j * BT;
        if (i < nvec) {
            const int n = i / vpp, e = i - n * vpp;
            const int eo = RAG ? min(e * VE, HW - VE) : e * VE, kf = e * VE - eo;   // kf: elements the vector before had
            const size_t off = ((size_t)n * C + c) * HW + (size_t)eo;
            if constexpr (RAG) xv[j] = load_any<VT>(x + off);
            else xv[j] = *reinterpret_cast<const VT *>(x + off);
            float f[VE], gr[VE];
            unpack<T, VB>(xv[j], f);
            if (gs.dy) {
                if constexpr (RAG) gv[j] = load_any<VT>(gs.dy + off);
                else gv[j] = *reinterpret_cast<const VT *>(gs.dy + off);
                unpack<T, VB>(gv[j], gr);
            } else {
                grad_vec<T, VB>(gs, (size_t)n * C + c, e * VE, gr);
            }
            if (relu) {   // the gradient that passes the ReLU is what is kept in registers
#pragma unroll
                for (int k = 0; k < VE; ++k) gr[k] = relu_passes<T>(bn_affine(f[k], mu, ga, gb)) ? gr[k] : 0.f;
            }
            if (relu || !gs.dy) gv[j] = pack<T, VB>(gr);
#pragma unroll
            for (int k = 0; k < VE; ++k) {
                if (RAG && k < kf) continue;
                s1 += gr[k];
                s2 += gr[k] * (f[k] - mu);
            }
        }
    }
    const float db = block_sum<BT>(s1, red);
    const float dg = block_sum<BT>(s2, red) * is;
    if (tid == 0) { dbeta[c] = db; dgamma[c] = dg; }
    const float invM = 1.f / ((float)N * (float)HW);
    const float k1 = ga, kb = db * invM, kg = dg * invM * is;
#pragma unroll
    for (int j = 0; j < NVMAX; ++j) {
        const int i = tid + j * BT;
        if (i < nvec) {
            const int n = i / vpp, e = i - n * vpp;
            const int eo = RAG ? min(e * VE, HW - VE) : e * VE;
            const size_t off = ((size_t)n * C + c) * HW + (size_t)eo;
            float f[VE], gr[VE];
            unpack<T, VB>(xv[j], f);
            unpack<T, VB>(gv[j], gr);
#pragma unroll
            for (int k = 0; k < VE; ++k) f[k] = k1 * (gr[k] - kb - (f[k] - mu) * kg);
            if constexpr (RAG) store_any<VT>(dx + off, pack<T, VB>(f));
            else *reinterpret_cast<VT *>(dx + off) = pack<T, VB>(f);
        }
    }
}

constexpr int BN_FUSED_NV = 13;   // vectors a thread can hold (13 * 1024 * 8 bf16 = 106496 elements per channel)
constexpr int BN_FUSED_NVS = 4;   // the same kernels built for short channels: fewer registers, two workgroups per compute unit
constexpr int BN_FUSED_NV1 = 32;  // single elements a thread can hold: planes of odd size (7x7, 17x17) have no wider access

// A channel of `count` vectors that 256 threads hold with nv vectors each: the 256-thread build.
inline bool bn_fused_small(long long count, int nv) { return count <= 256LL * nv; }

// Vector size in bytes for the one-pass kernels, 0 if they do not apply.
template <typename T> int bn_fused_vb(const void *a, const void *b, const void *c3, int N, int HW, bool ragged_ok = true)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c3);
    for (int vb = 16; vb >= 8; vb /= 2) {
        const int ve = vb / (int)sizeof(T);
        if (HW % ve != 0 || bits % vb != 0) continue;
        const long long nvec = (long long)N * (HW / ve);
        if (nvec <= 1024LL * BN_FUSED_NV) return vb;
    }
    // planes that are no whole number of 8-byte vectors: 16-byte vectors at any alignment, the last one of a plane
    // moved back (bf16, a given gradient tensor; reported as -16)
    if (ragged_ok && sizeof(T) == 2 && HW % 4 != 0 && HW >= 8 && bits % sizeof(T) == 0 &&
        (long long)N * ((HW + 7) / 8) <= 1024LL * BN_FUSED_NVS)   // longer channels: the two-pass kernels are faster (35x35: 2.9 against 2.6 TB/s)
        return -16;
    if ((HW & 1) && bits % sizeof(T) == 0 && (long long)N * HW <= 1024LL * BN_FUSED_NV1) return (int)sizeof(T);
    return 0;
}

// Tensors too small to hold the partial sums (fewer than 8 bytes per channel):
// one thread per channel does the whole layer.
template <typename T>
__global__ void bn_fwd_tiny_kernel(const T *__restrict__ x, T *__restrict__ y, const float *__restrict__ gamma,
                                   const float *__restrict__ beta, float *__restrict__ mean,
                                   float *__restrict__ invstd, int N, int C, int HW, float eps, int relu)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const float M = (float)N * (float)HW;
    float s = 0.f;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) s += ld<T>(x + ((size_t)n * C + c) * HW + i);
    const float mu = s / M;
    float ss = 0.f;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            float d = ld<T>(x + ((size_t)n * C + c) * HW + i) - mu;
            ss += d * d;
        }
    const float is = 1.f / sqrtf(ss / M + eps);
    mean[c] = mu;
    invstd[c] = is;
    const float a = gamma[c] * is, b = beta[c];
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            const size_t j = ((size_t)n * C + c) * HW + i;
            st(y + j, act(bn_affine(ld<T>(x + j), mu, a, b), relu));
        }
}

template <typename T>
__global__ void bn_bwd_tiny_kernel(const T *__restrict__ x, const T *__restrict__ dy, const float *__restrict__ beta,
                                   T *__restrict__ dx,
                                   const float *__restrict__ gamma, const float *__restrict__ mean,
                                   const float *__restrict__ invstd, float *__restrict__ dgamma,
                                   float *__restrict__ dbeta, int N, int C, int HW)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const float invM = 1.f / ((float)N * (float)HW);
    const float mu = mean[c], is = invstd[c];
    const bool relu = beta != nullptr;
    const float ga = gamma[c] * is, gb = relu ? beta[c] : 0.f;
    float db = 0.f, dg = 0.f;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            const size_t j = ((size_t)n * C + c) * HW + i;
            const float f = ld<T>(x + j);
            const float gr = (relu && !relu_passes<T>(bn_affine(f, mu, ga, gb))) ? 0.f : ld<T>(dy + j);
            db += gr;
            dg += gr * (f - mu);
        }
    dg *= is;
    dbeta[c] = db;
    dgamma[c] = dg;
    const float k1 = ga, kb = db * invM, kg = dg * invM * is;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            const size_t j = ((size_t)n * C + c) * HW + i;
            const float f = ld<T>(x + j);
            const float gr = (relu && !relu_passes<T>(bn_affine(f, mu, ga, gb))) ? 0.f : ld<T>(dy + j);
            st(dx + j, k1 * (gr - kb - (f - mu) * kg));
        }
}

Slices make_slices(int N, int C, int HW, size_t scratch_bytes)
{
    Slices s;
    s.nseg_plane = (HW + SEG - 1) / SEG;
    s.nseg = N * s.nseg_plane;
    long long want = (4096 + C - 1) / C;            // about 4096 workgroups in all
    long long most = (s.nseg + 3) / 4;              // at least one segment per wave
    long long fit = (long long)(scratch_bytes / (2 * sizeof(float)) / (size_t)C);
    if (want > most) want = most;
    if (want > fit) want = fit;
    if (want > 65535) want = 65535;
    if (want < 1) want = 1;
    s.nslice = (int)want;
    return s;
}

// ------------------------------------------------------------------ max-pool
// One thread per output.  IX: the type the output number is split in (32 bits where they do).
template <typename T, typename IX>
__global__ void __launch_bounds__(256)
maxpool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int32_t *__restrict__ idx, size_t total,
                   int H, int W, int P, int Q, int kh, int kw, int sh, int sw, int ph, int pw)
{
    const size_t o = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int PQ = P * Q;
    const size_t nc = (size_t)((IX)o / (IX)PQ);
    const int pq = (int)(o - nc * PQ), p = pq / Q, q = pq - p * Q;
    const T *xp = x + nc * (size_t)H * W;
    const int h0 = p * sh - ph, v0 = q * sw - pw;
    const int hb = max(h0, 0), he = min(h0 + kh, H), vb = max(v0, 0), ve = min(v0 + kw, W);
    // row-major scan, a later element wins only if strictly greater
    int best = hb * W + vb;
    T bestraw = xp[best];
    float bv = ld<T>(&bestraw);
    for (int h = hb; h < he; ++h)
        for (int v = vb; v < ve; ++v) {
            T raw = xp[h * W + v];
            float f = ld<T>(&raw);
            if (f > bv) { bv = f; best = h * W + v; bestraw = raw; }
        }
    y[o] = bestraw;
    idx[o] = best;
}

// One thread per input element; a workgroup stays inside one plane (bpp workgroups per plane), so
// the plane number is a scalar.  K > 0: a K x K window with stride 2 (3x3 / stride 2 is the
// overlapping pool of the AlexNet- and Inception-style workloads), whose window bounds need no
// division; K == 0: the window and stride of the arguments.
template <typename T, int K>
__global__ void __launch_bounds__(256)
maxpool_bwd_kernel(const T *__restrict__ dy, const int32_t *__restrict__ idx, T *__restrict__ dx, unsigned bpp,
                   int H, int W, int P, int Q, int kh, int kw, int sh, int sw, int ph, int pw)
{
    const unsigned nc = blockIdx.x / bpp;
    const int hw = (int)((blockIdx.x - nc * bpp) * 256 + threadIdx.x), HW = H * W;
    if (hw >= HW) return;
    const int h = hw / W, v = hw - h * W;
    if (K > 0) { kh = kw = K; sh = sw = 2; }
    // windows p with p*sh - ph <= h < p*sh - ph + kh
    const int pnum = h + ph - kh + 1, qnum = v + pw - kw + 1;
    const int p0 = pnum > 0 ? (pnum + sh - 1) / sh : 0, p1 = min((h + ph) / sh, P - 1);
    const int q0 = qnum > 0 ? (qnum + sw - 1) / sw : 0, q1 = min((v + pw) / sw, Q - 1);
    const T *gp = dy + (size_t)nc * P * Q;
    const int32_t *ip = idx + (size_t)nc * P * Q;
    float acc = 0.f;
    for (int p = p0; p <= p1; ++p)
        for (int q = q0; q <= q1; ++q)
            if (ip[p * Q + q] == hw) acc += ld<T>(gp + p * Q + q);
    st(dx + (size_t)nc * HW + hw, acc);
}

// 2x2 windows, stride 2, no padding (the pool of the VGG-style workloads): windows do not
// overlap, so a thread owns 8 neighbouring windows of one output row and moves whole
// vectors: forward it reads 16 columns of the two input rows, backward it writes 8 columns
// of the two rows under its 4 windows (and the uncovered last row of an odd-height image).
// Threads of a workgroup are (output row, group of windows), the groups padded to a power
// of two, so that no thread needs a 64-bit division.
template <typename T, int NEL> struct __attribute__((packed, aligned(sizeof(T)))) Pack { T e[NEL]; };

template <typename T>
__global__ void __launch_bounds__(256)
maxpool2_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int32_t *__restrict__ idx, unsigned rows, int H,
                    int W, int P, int Q, int lg, const T *__restrict__ xend)
{
    const unsigned row = blockIdx.x * (256u >> lg) + (threadIdx.x >> lg);
    const int g = threadIdx.x & ((1 << lg) - 1);
    if (row >= rows || g * 8 >= Q) return;
    const unsigned nc = row / (unsigned)P;
    const int p = (int)(row - nc * (unsigned)P);
    const T *r0 = x + ((size_t)nc * H + 2 * p) * W + 16 * g, *r1 = r0 + W;
    T *yo = y + (size_t)row * Q + 8 * g;
    int32_t *io = idx + (size_t)row * Q + 8 * g;
    const int base = 2 * p * W + 16 * g;
    const int nout = min(8, Q - 8 * g);
    // the 16 columns may run past the row end; they are read anyway as long as they are inside
    // the tensor, and the windows they would feed are not stored
    Pack<T, 16> a, b;
    if (r1 + 16 <= xend) {
        a = *reinterpret_cast<const Pack<T, 16> *>(r0);
        b = *reinterpret_cast<const Pack<T, 16> *>(r1);
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            a.e[j] = b.e[j] = T(0);
            if (j < 2 * nout) { a.e[j] = r0[j]; b.e[j] = r1[j]; }
        }
    }
    Pack<T, 8> out;
    Pack<int32_t, 8> oi;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // row-major scan of the window, a later element wins only if strictly greater
        T raw = a.e[2 * j];
        float bv = ld<T>(&raw);
        int best = base + 2 * j;
        float f = ld<T>(&a.e[2 * j + 1]);
        if (f > bv) { bv = f; best = base + 2 * j + 1; raw = a.e[2 * j + 1]; }
        f = ld<T>(&b.e[2 * j]);
        if (f > bv) { bv = f; best = base + W + 2 * j; raw = b.e[2 * j]; }
        f = ld<T>(&b.e[2 * j + 1]);
        if (f > bv) { bv = f; best = base + W + 2 * j + 1; raw = b.e[2 * j + 1]; }
        out.e[j] = raw;
        oi.e[j] = best;
    }
    if (nout == 8) {
        *reinterpret_cast<Pack<T, 8> *>(yo) = out;
        *reinterpret_cast<Pack<int32_t, 8> *>(io) = oi;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < nout) { yo[j] = out.e[j]; io[j] = oi.e[j]; }
    }
}

template <typename T>
__global__ void __launch_bounds__(256)
maxpool2_bwd_kernel(const T *__restrict__ dy, const int32_t *__restrict__ idx, T *__restrict__ dx, unsigned rows,
                    int H, int W, int P, int Q, int lg)
{
    const unsigned row = blockIdx.x * (256u >> lg) + (threadIdx.x >> lg);
    const int g = threadIdx.x & ((1 << lg) - 1);
    if (row >= rows || g * 8 >= W) return;
    const unsigned nc = row / (unsigned)P;
    const int p = (int)(row - nc * (unsigned)P);
    const size_t wrow = (size_t)row * Q + 4 * g;
    const int nwin = max(0, min(4, Q - 4 * g));
    Pack<T, 4> d;
    Pack<int32_t, 4> wi;
    if (nwin == 4) {
        d = *reinterpret_cast<const Pack<T, 4> *>(dy + wrow);
        wi = *reinterpret_cast<const Pack<int32_t, 4> *>(idx + wrow);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wi.e[j] = -1;
            d.e[j] = T(0);
            if (j < nwin) { wi.e[j] = idx[wrow + j]; d.e[j] = dy[wrow + j]; }
        }
    }
    const int ncol = min(8, W - 8 * g);
    const int hlast = (p == P - 1) ? H - 1 : 2 * p + 1;   // an odd height leaves one row without a window
    for (int h = 2 * p; h <= hlast; ++h) {
        Pack<T, 8> out;
#pragma unroll
        for (int c = 0; c < 8; ++c) out.e[c] = wi.e[c >> 1] == h * W + 8 * g + c ? d.e[c >> 1] : T(0);
        T *o = dx + ((size_t)nc * H + h) * W + 8 * g;
        if (ncol == 8) {
            *reinterpret_cast<Pack<T, 8> *>(o) = out;
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c)
                if (c < ncol) o[c] = out.e[c];
        }
    }
}

// 3x3 windows, stride 2, forward: a thread owns 4 neighbouring windows of one output row, i.e.
// 9 columns of 3 input rows, which it reads as one 8-element piece and one element per row where the
// piece lies inside the image and the tensor (anything else: element by element).  The scan of a
// window is the generic kernel's: row-major over the positions inside the image, a later element
// wins only if strictly greater.
template <typename T>
__global__ void __launch_bounds__(256)
maxpool3s2_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int32_t *__restrict__ idx, unsigned rows, int H,
                      int W, int P, int Q, int ph, int pw, int lg, const T *__restrict__ xend)
{
    const unsigned row = blockIdx.x * (256u >> lg) + (threadIdx.x >> lg);
    const int g = threadIdx.x & ((1 << lg) - 1);
    if (row >= rows || g * 4 >= Q) return;
    const unsigned nc = row / (unsigned)P;
    const int p = (int)(row - nc * (unsigned)P), q0 = 4 * g;
    const int nout = min(4, Q - q0);
    const int h0 = 2 * p - ph, v0 = 2 * q0 - pw;
    const T *xp = x + (size_t)nc * H * W;
    // the 3 x 9 elements; outside the image: never looked at
    T e[3][9];
    const bool inside = v0 >= 0 && v0 + 9 <= W;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int h = h0 + r;
        if ((unsigned)h >= (unsigned)H) {
#pragma unroll
            for (int c = 0; c < 9; ++c) e[r][c] = T(0);
            continue;
        }
        const T *rp = xp + (size_t)h * W + v0;
        if (inside && rp + 9 <= xend) {
            const Pack<T, 8> v = *reinterpret_cast<const Pack<T, 8> *>(rp);
#pragma unroll
            for (int c = 0; c < 8; ++c) e[r][c] = v.e[c];
            e[r][8] = rp[8];
        } else {
#pragma unroll
            for (int c = 0; c < 9; ++c) e[r][c] = (unsigned)(v0 + c) < (unsigned)W ? rp[c] : T(0);
        }
    }
    Pack<T, 4> out;
    Pack<int32_t, 4> oi;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        bool have = false;
        float bv = 0.f;
        int best = 0;
        T raw = T(0);
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const int h = h0 + r, v = v0 + 2 * j + c;
                if ((unsigned)h >= (unsigned)H || (unsigned)v >= (unsigned)W) continue;
                const T cand = e[r][2 * j + c];
                const float f = ld<T>(&cand);
                if (!have) { have = true; bv = f; best = h * W + v; raw = cand; }
                else if (f > bv) { bv = f; best = h * W + v; raw = cand; }
            }
        out.e[j] = raw;
        oi.e[j] = best;
    }
    T *yo = y + (size_t)row * Q + q0;
    int32_t *io = idx + (size_t)row * Q + q0;
    if (nout == 4) {
        *reinterpret_cast<Pack<T, 4> *>(yo) = out;
        *reinterpret_cast<Pack<int32_t, 4> *>(io) = oi;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nout) { yo[j] = out.e[j]; io[j] = oi.e[j]; }
    }
}

// 3x3 windows, stride 2 (the overlapping pool of the AlexNet- and Inception-style workloads),
// backward: a thread owns 8 neighbouring columns of one input row.  At most 2 window rows and
// 5 window columns cover them; every window's index and gradient are read once per thread and
// added, in ascending (p, q) order -- the order of the one-thread-per-element kernel -- to
// the column the index names, and the row piece leaves in one store.
template <typename T>
__global__ void __launch_bounds__(256)
maxpool3s2_bwd_kernel(const T *__restrict__ dy, const int32_t *__restrict__ idx, T *__restrict__ dx, unsigned rows,
                      int H, int W, int P, int Q, int ph, int pw, int lg)
{
    const unsigned row = blockIdx.x * (256u >> lg) + (threadIdx.x >> lg);
    const int g = threadIdx.x & ((1 << lg) - 1);
    if (row >= rows || g * 8 >= W) return;
    const unsigned nc = row / (unsigned)H;
    const int h = (int)(row - nc * (unsigned)H), v0 = 8 * g;
    const int ncol = min(8, W - v0);
    // windows p with 2p - ph <= h <= 2p - ph + 2, windows q that reach one of the columns
    const int p0 = max(0, (h + ph - 1) >> 1), p1 = min((h + ph) >> 1, P - 1);
    const int q0 = max(0, (v0 + pw - 1) >> 1), q1 = min((v0 + ncol - 1 + pw) >> 1, Q - 1);
    const T *gp = dy + (size_t)nc * P * Q;
    const int32_t *ip = idx + (size_t)nc * P * Q;
    const int first = h * W + v0;
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    for (int p = p0; p <= p1; ++p)
        for (int q = q0; q <= q1; ++q) {
            const int rel = ip[p * Q + q] - first;
            const float d = ld<T>(gp + p * Q + q);
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] += rel == c ? d : 0.f;
        }
    T *o = dx + (size_t)row * W + v0;
    if (ncol == 8) {
        Pack<T, 8> out;
#pragma unroll
        for (int c = 0; c < 8; ++c) st(&out.e[c], acc[c]);
        *reinterpret_cast<Pack<T, 8> *>(o) = out;
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c)
            if (c < ncol) st(o + c, acc[c]);
    }
}

// ------------------------------------------------------------------ LRN
// LRN across channels (definition in sn.h).  A thread owns VEC neighbouring positions of one
// image and walks the channels, which are H*W elements apart, so a wave reads one contiguous run
// per channel; the window of the last 2 HALF + 1 channels lives in registers (a shift per step),
// so x is read once.  s^(-beta) = exp2(-beta log2 s) on the transcendental unit (s >= k > 0).
// Backward needs, for channel c, the terms r_j = dy_j x_j s_j^(-beta-1) of the channels around
// it, each of which needs the window around j: the loop runs HALF channels ahead for s_j and
// another HALF ahead for x, with r, s^(-beta) and dy of the channels in between in registers;
// x and dy are read once, the forward output is not needed.  The channel loops are unrolled so
// that the loads of several channels are in flight at once: nothing else hides their latency.
// RAG: planes that are no whole number of vectors (55x55, 27x27): a plane is ceil(HW / VEC) vectors at the
// element's own alignment, the last one moved back so that it ends with the plane; the positions it shares
// with the vector before are computed and written twice, with the same values.
template <typename T, int VEC, bool RAG = false> struct LrnIo {
    static constexpr int VB = VEC * (int)sizeof(T);
    typedef typename RawVec<VB>::type VT;
    struct __attribute__((packed, aligned(sizeof(T)))) Loose { uint32_t w[VB / 4 > 0 ? VB / 4 : 1]; };
    __device__ static void load(const T *p, float (&f)[VEC])
    {
        if constexpr (VEC == 1) f[0] = ld<T>(p);
        else if constexpr (RAG) {
            const Loose l = *reinterpret_cast<const Loose *>(p);
            VT v;
            __builtin_memcpy(&v, &l, VB);
            unpack<T, VB>(v, f);
        } else unpack<T, VB>(*reinterpret_cast<const VT *>(p), f);
    }
    __device__ static void store(T *p, const float (&f)[VEC])
    {
        if constexpr (VEC == 1) st(p, f[0]);
        else if constexpr (RAG) {
            const VT v = pack<T, VB>(f);
            Loose l;
            __builtin_memcpy(&l, &v, VB);
            *reinterpret_cast<Loose *>(p) = l;
        } else *reinterpret_cast<VT *>(p) = pack<T, VB>(f);
    }
};

__device__ inline float pow_neg(float s, float beta) { return __builtin_amdgcn_exp2f(-beta * __builtin_amdgcn_logf(s)); }

template <typename T, int VEC, int HALF, bool RAG = false, bool RELU = false>
__global__ void __launch_bounds__(256)
lrn_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int C, int HW, int vpp, size_t total, float a_n,
               float beta, float k, int cc)
{
    const int cb = blockIdx.y * cc, ce = min(C, cb + cc);   // this workgroup's channels
    constexpr int SIZE = 2 * HALF + 1;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const size_t n = t / vpp;
    const size_t off = n * (size_t)C * HW + (RAG ? min((int)(t - n * vpp) * VEC, HW - VEC) : (int)(t - n * vpp) * VEC);
    float xr[SIZE][VEC];   // after channel m has been pushed: xr[i] = channel m - (SIZE - 1) + i, zeros outside [0, C)
#pragma unroll
    for (int i = 0; i < SIZE; ++i)
#pragma unroll
        for (int v = 0; v < VEC; ++v) xr[i][v] = 0.f;
#pragma unroll 8
    for (int m = cb - HALF; m < ce + HALF; ++m) {
#pragma unroll
        for (int i = 0; i + 1 < SIZE; ++i)
#pragma unroll
            for (int v = 0; v < VEC; ++v) xr[i][v] = xr[i + 1][v];
        if (m >= 0 && m < C) {
            LrnIo<T, VEC, RAG>::load(x + off + (size_t)m * HW, xr[SIZE - 1]);
            if (RELU) {   // the layer's input is the ReLU of x, which is never stored
#pragma unroll
                for (int v = 0; v < VEC; ++v) xr[SIZE - 1][v] = act(xr[SIZE - 1][v], 1);
            }
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) xr[SIZE - 1][v] = 0.f;
        }
        const int c = m - HALF;
        if (c < cb) continue;
        float out[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < SIZE; ++i) sum = __builtin_fmaf(xr[i][v], xr[i][v], sum);
            out[v] = xr[HALF][v] * pow_neg(__builtin_fmaf(a_n, sum, k), beta);
        }
        LrnIo<T, VEC, RAG>::store(y + off + (size_t)c * HW, out);
    }
}

template <typename T, int VEC, int HALF, bool RAG = false, bool RELU = false>
__global__ void __launch_bounds__(256)
lrn_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy, T *__restrict__ dx, int C, int HW, int vpp,
               size_t total, float a_n, float beta, float k, int cc)
{
    const int cb = blockIdx.y * cc, ce = min(C, cb + cc);   // this workgroup's channels
    constexpr int SIZE = 2 * HALF + 1, H1 = HALF + 1;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const size_t n = t / vpp;
    const size_t off = n * (size_t)C * HW + (RAG ? min((int)(t - n * vpp) * VEC, HW - VEC) : (int)(t - n * vpp) * VEC);
    const float coef = 2.f * a_n * beta;
    float xr[SIZE][VEC], rr[SIZE][VEC];   // x of channels m - 2 HALF .. m; r of channels j - 2 HALF .. j (j = m - HALF)
    float pr[H1][VEC], gr[H1][VEC];       // s^(-beta) and dy of channels j - HALF .. j
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
#pragma unroll
        for (int i = 0; i < SIZE; ++i) xr[i][v] = rr[i][v] = 0.f;
#pragma unroll
        for (int i = 0; i < H1; ++i) pr[i][v] = gr[i][v] = 0.f;
    }
#pragma unroll 8
    for (int m = cb - 2 * HALF; m < ce + 2 * HALF; ++m) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
#pragma unroll
            for (int i = 0; i + 1 < SIZE; ++i) { xr[i][v] = xr[i + 1][v]; rr[i][v] = rr[i + 1][v]; }
#pragma unroll
            for (int i = 0; i + 1 < H1; ++i) { pr[i][v] = pr[i + 1][v]; gr[i][v] = gr[i + 1][v]; }
            xr[SIZE - 1][v] = 0.f;
            rr[SIZE - 1][v] = pr[H1 - 1][v] = gr[H1 - 1][v] = 0.f;
        }
        if (m >= 0 && m < C) {
            LrnIo<T, VEC, RAG>::load(x + off + (size_t)m * HW, xr[SIZE - 1]);
            if (RELU) {   // LRN saw max(x, 0): negative and zero x both count as 0, and their dx is 0 below
#pragma unroll
                for (int v = 0; v < VEC; ++v) xr[SIZE - 1][v] = act(xr[SIZE - 1][v], 1);
            }
        }
        const int j = m - HALF;   // the channel whose window is complete: x_j = xr[HALF]
        if (j < 0) continue;
        if (j < C) {
            LrnIo<T, VEC, RAG>::load(dy + off + (size_t)j * HW, gr[H1 - 1]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < SIZE; ++i) sum = __builtin_fmaf(xr[i][v], xr[i][v], sum);
                const float s = __builtin_fmaf(a_n, sum, k), p = pow_neg(s, beta);
                pr[H1 - 1][v] = p;
                rr[SIZE - 1][v] = gr[H1 - 1][v] * xr[HALF][v] * (p / s);
            }
        }
        const int c = j - HALF;   // every r of its window is known: x_c = xr[0], dy_c = gr[0], s_c^(-beta) = pr[0]
        if (c < cb) continue;
        float out[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < SIZE; ++i) acc += rr[i][v];
            out[v] = gr[0][v] * pr[0][v] - coef * xr[0][v] * acc;
            if (RELU && !(xr[0][v] > 0.f)) out[v] = 0.f;   // the ReLU's gate: x > 0 (xr holds max(x, 0))
        }
        LrnIo<T, VEC, RAG>::store(dx + off + (size_t)c * HW, out);
    }
}

template <typename F> hipError_t by_dtype(int bf16, F f)
{
    if (bf16) f((bf16_t *)nullptr);
    else f((float *)nullptr);
    return hipGetLastError();
}

// The 2x2 / stride 2 / unpadded kernels apply, and their row count and group count fit.
bool pool2_fast(int NC, int P, int kh, int kw, int sh, int sw, int ph, int pw)
{
    return kh == 2 && kw == 2 && sh == 2 && sw == 2 && ph == 0 && pw == 0 && (long long)NC * P < (1LL << 31);
}

// Smallest lg with 2^lg >= groups, or -1 if a row has more than 256 groups.
int log2_groups(int groups)
{
    for (int lg = 0; lg <= 8; ++lg)
        if ((1 << lg) >= groups) return lg;
    return -1;
}

}  // namespace

hipError_t launch_relu_fwd(const void *x, void *y, size_t n, int bf16, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        const size_t nvec = n / Vec<T>::N;
        const size_t per = 256 * RELU_UNROLL;
        dim3 grid((unsigned)((nvec + per - 1) / per + (nvec == 0 ? 1 : 0))), block(256);
        hipLaunchKernelGGL(relu_fwd_kernel<T>, grid, block, 0, s, (const T *)x, (T *)y, n);
    });
}

hipError_t launch_relu_bwd(const void *x, const void *dy, void *dx, size_t n, int bf16, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        const size_t nvec = n / Vec<T>::N;
        const size_t per = 256 * RELU_UNROLL;
        dim3 grid((unsigned)((nvec + per - 1) / per + (nvec == 0 ? 1 : 0))), block(256);
        hipLaunchKernelGGL(relu_bwd_kernel<T>, grid, block, 0, s, (const T *)x, (const T *)dy, (T *)dx, n);
    });
}

hipError_t launch_bn_fwd(const void *x, const float *gamma, const float *beta, void *y, float *mean,
                         float *invstd, int N, int C, int HW, float eps, int bf16, int relu, hipStream_t s)
{
    const size_t esz = bf16 ? 2 : 4;
    if ((size_t)N * HW * esz < 2 * sizeof(float))
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
            hipLaunchKernelGGL(bn_fwd_tiny_kernel<T>, dim3((C + 63) / 64), dim3(64), 0, s, (const T *)x, (T *)y,
                               gamma, beta, mean, invstd, N, C, HW, eps, relu);
        });
    {
        const int vb = bf16 ? bn_fused_vb<bf16_t>(x, y, nullptr, N, HW) : bn_fused_vb<float>(x, y, nullptr, N, HW);
        if (vb)
            return by_dtype(bf16, [&](auto *tag) {
                typedef typename std::remove_pointer<decltype(tag)>::type T;
                // a channel of at most 4 vectors per thread goes to the build with 4 registers' worth of them
                // (the sums run over the same elements in the same order either way)
                const long long cnt = vb < 0 ? (long long)N * ((HW + 7) / 8)
                                             : (long long)N * (HW / (vb / (int)sizeof(T)));   // vectors per channel
                const bool few = (vb >= 8 || vb < 0) && cnt <= 1024LL * BN_FUSED_NVS;
                if (vb < 0) {
                    if (bn_fused_small(cnt, BN_FUSED_NVS))
                        hipLaunchKernelGGL((bn_fwd_fused_kernel<T, 16, BN_FUSED_NVS, 0, 256, true>), dim3(C), dim3(256), 0, s,
                                           (const T *)x, (T *)y, gamma, beta, mean, invstd, N, C, HW, eps, relu,
                                           (T *)nullptr, (int32_t *)nullptr, 0, 0);
                    else
                        hipLaunchKernelGGL((bn_fwd_fused_kernel<T, 16, BN_FUSED_NVS, 0, 1024, true>), dim3(C), dim3(1024), 0, s,
                                           (const T *)x, (T *)y, gamma, beta, mean, invstd, N, C, HW, eps, relu,
                                           (T *)nullptr, (int32_t *)nullptr, 0, 0);
                    return;
                }
#define SN_BN_FWD(VB_, NV_)                                                                                          \
    do {                                                                                                             \
        if (bn_fused_small(cnt, NV_))                                                                                \
            hipLaunchKernelGGL((bn_fwd_fused_kernel<T, VB_, NV_, 0, 256>), dim3(C), dim3(256), 0, s, (const T *)x,   \
                               (T *)y, gamma, beta, mean, invstd, N, C, HW, eps, relu, (T *)nullptr,                 \
                               (int32_t *)nullptr, 0, 0);                                                            \
        else                                                                                                         \
            hipLaunchKernelGGL((bn_fwd_fused_kernel<T, VB_, NV_, 0, 1024>), dim3(C), dim3(1024), 0, s, (const T *)x, \
                               (T *)y, gamma, beta, mean, invstd, N, C, HW, eps, relu, (T *)nullptr,                 \
                               (int32_t *)nullptr, 0, 0);                                                            \
    } while (0)
                if (vb == 16 && few) SN_BN_FWD(16, BN_FUSED_NVS);
                else if (vb == 8 && few) SN_BN_FWD(8, BN_FUSED_NVS);
                else if (vb == 16) SN_BN_FWD(16, BN_FUSED_NV);
                else if (vb == (int)sizeof(T)) SN_BN_FWD(sizeof(T), BN_FUSED_NV1);
                else SN_BN_FWD(8, BN_FUSED_NV);
#undef SN_BN_FWD
            });
    }
    // y is dead until pass 3, so it holds the per-slice partial sums meanwhile
    const Slices sl = make_slices(N, C, HW, (size_t)N * C * HW * esz);
    float *part = reinterpret_cast<float *>(y);
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        dim3 grid(C, sl.nslice), block(256);
        hipLaunchKernelGGL(bn_stats_kernel<T>, grid, block, 0, s, (const T *)x, part, N, C, HW, sl);
        hipLaunchKernelGGL(bn_stats_final_kernel<T>, dim3(C), dim3(64), 0, s, (const T *)x, part, mean, invstd,
                           N, HW, sl.nslice, eps);
        hipLaunchKernelGGL(bn_apply_kernel<T>, grid, block, 0, s, (const T *)x, (T *)y, gamma, beta, mean,
                           invstd, N, C, HW, sl, relu);
    });
}

hipError_t launch_bn_finalize_tiles(const float *part, int C, int ntiles, float *mean, float *invstd, float eps,
                                    hipStream_t s)
{
    hipLaunchKernelGGL(bn_finalize_tiles_kernel, dim3(C), dim3(1024), 0, s, part, ntiles, mean, invstd, eps);
    return hipGetLastError();
}

size_t bn_stats_scratch_bytes(int N, int C, int HW)
{
    const Slices sl = make_slices(N, C, HW, ~(size_t)0);
    return (size_t)C * sl.nslice * 2 * sizeof(float);
}

hipError_t launch_bn_stats(const void *x, float *scratch, float *mean, float *invstd, int N, int C, int HW, float eps,
                           int bf16, hipStream_t s)
{
    const Slices sl = make_slices(N, C, HW, ~(size_t)0);
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        hipLaunchKernelGGL(bn_stats_kernel<T>, dim3(C, sl.nslice), dim3(256), 0, s, (const T *)x, scratch, N, C, HW, sl);
        hipLaunchKernelGGL(bn_stats_final_kernel<T>, dim3(C), dim3(64), 0, s, (const T *)x, scratch, mean, invstd,
                           N, HW, sl.nslice, eps);
    });
}

hipError_t launch_bn_apply(const void *x, const float *gamma, const float *beta, const float *mean,
                           const float *invstd, void *y, int N, int C, int HW, int bf16, int relu, hipStream_t s)
{
    const Slices sl = make_slices(N, C, HW, ~(size_t)0);
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        hipLaunchKernelGGL(bn_apply_kernel<T>, dim3(C, sl.nslice), dim3(256), 0, s, (const T *)x, (T *)y, gamma, beta,
                           mean, invstd, N, C, HW, sl, relu);
    });
}

int bn_relu_pool2_vb(int W, int bf16)
{
    const int esz = bf16 ? 2 : 4;
    return W % (16 / esz) == 0 ? 16 : W % (8 / esz) == 0 ? 8 : 0;
}

hipError_t launch_bn_relu_pool2_apply(const void *x, const float *gamma, const float *beta, const float *mean,
                                      const float *invstd, void *pooled, int32_t *idx, int N, int C, int H, int W,
                                      int bf16, hipStream_t s)
{
    const int esz = bf16 ? 2 : 4, pvb = bn_relu_pool2_vb(W, bf16);
    if (pvb == 0 || (H & 1)) return hipErrorInvalidValue;
    const int units = N * (H / 2) * (W / (pvb / esz));
    long long want = (4096 + C - 1) / C, most = (units + 255) / 256;
    if (want > most) want = most;
    if (want > 65535) want = 65535;
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        dim3 block(256), pgrid(C, (unsigned)want);
        if (pvb == 16)
            hipLaunchKernelGGL((bn_relu_pool2_apply_kernel<T, 16>), pgrid, block, 0, s, (const T *)x, (T *)pooled, idx,
                               gamma, beta, mean, invstd, C, H, W, units);
        else
            hipLaunchKernelGGL((bn_relu_pool2_apply_kernel<T, 8>), pgrid, block, 0, s, (const T *)x, (T *)pooled, idx,
                               gamma, beta, mean, invstd, C, H, W, units);
    });
}

hipError_t launch_bn_relu_pool2_fwd(const void *x, const float *gamma, const float *beta, void *pooled, int32_t *idx,
                                    float *mean, float *invstd, int N, int C, int H, int W, float eps, int bf16,
                                    hipStream_t s)
{
    const size_t esz = bf16 ? 2 : 4;
    const int HW = H * W, pvb = bn_relu_pool2_vb(W, bf16);
    if (pvb == 0 || (H & 1)) return hipErrorInvalidValue;
    // the statistics come from the very kernels launch_bn_fwd picks for this shape
    const int vb = bf16 ? bn_fused_vb<bf16_t>(x, nullptr, nullptr, N, HW, false) : bn_fused_vb<float>(x, nullptr, nullptr, N, HW, false);
    if (vb != 0 && vb != 16) return hipErrorInvalidValue;
    if (vb)
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
#define SN_POOL_FUSED(VB_, NV_, PVB_)                                                                                \
    do {                                                                                                             \
        if (bn_fused_small((long long)N * (HW / (VB_ / (int)sizeof(T))), NV_))                                       \
            hipLaunchKernelGGL((bn_fwd_fused_kernel<T, VB_, NV_, PVB_, 256>), dim3(C), dim3(256), 0, s,             \
                               (const T *)x, (T *)nullptr, gamma, beta, mean, invstd, N, C, HW, eps, 1, (T *)pooled, \
                               idx, H, W);                                                                           \
        else                                                                                                         \
            hipLaunchKernelGGL((bn_fwd_fused_kernel<T, VB_, NV_, PVB_, 1024>), dim3(C), dim3(1024), 0, s,           \
                               (const T *)x, (T *)nullptr, gamma, beta, mean, invstd, N, C, HW, eps, 1, (T *)pooled, \
                               idx, H, W);                                                                           \
    } while (0)
            // H even and W a multiple of half a 16-byte vector make H*W a multiple of the whole one
            const bool few = (long long)N * (HW / (16 / (int)sizeof(T))) <= 1024LL * BN_FUSED_NVS;
            if (pvb == 16 && few) SN_POOL_FUSED(16, BN_FUSED_NVS, 16);
            else if (pvb == 16) SN_POOL_FUSED(16, BN_FUSED_NV, 16);
            else if (few) SN_POOL_FUSED(16, BN_FUSED_NVS, 8);
            else SN_POOL_FUSED(16, BN_FUSED_NV, 8);
#undef SN_POOL_FUSED
        });
    // idx is dead until the last pass, so it holds the per-slice partial sums meanwhile (launch_bn_fwd
    // keeps them in y; the slices are the same)
    const Slices sl = make_slices(N, C, HW, (size_t)N * C * HW * esz);
    if ((size_t)C * sl.nslice * 2 * sizeof(float) > (size_t)N * C * (HW / 4) * sizeof(int32_t)) return hipErrorInvalidValue;
    float *part = reinterpret_cast<float *>(idx);
    hipError_t e = by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        dim3 grid(C, sl.nslice), block(256);
        hipLaunchKernelGGL(bn_stats_kernel<T>, grid, block, 0, s, (const T *)x, part, N, C, HW, sl);
        hipLaunchKernelGGL(bn_stats_final_kernel<T>, dim3(C), dim3(64), 0, s, (const T *)x, part, mean, invstd,
                           N, HW, sl.nslice, eps);
    });
    if (e != hipSuccess) return e;
    return launch_bn_relu_pool2_apply(x, gamma, beta, mean, invstd, pooled, idx, N, C, H, W, bf16, s);
}

hipError_t launch_bn_bwd(const void *x, const void *dy, const float *relu_beta, const float *gamma, const float *mean,
                         const float *invstd, void *dx, float *dgamma, float *dbeta, int N, int C, int HW,
                         int bf16, hipStream_t s, const void *pool_g, const int32_t *pool_idx, int pool_W)
{
    const size_t esz = bf16 ? 2 : 4;
    if (!dy && (!pool_g || !pool_idx || pool_W < 2 || (pool_W & 1) || HW % (2 * pool_W) != 0)) return hipErrorInvalidValue;
    if ((size_t)N * HW * esz < 2 * sizeof(float))
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
            hipLaunchKernelGGL(bn_bwd_tiny_kernel<T>, dim3((C + 63) / 64), dim3(64), 0, s, (const T *)x,
                               (const T *)dy, relu_beta, (T *)dx, gamma, mean, invstd, dgamma, dbeta, N, C, HW);
        });
    {
        int vb = bf16 ? bn_fused_vb<bf16_t>(x, dy, dx, N, HW, dy != nullptr) : bn_fused_vb<float>(x, dy, dx, N, HW, false);
        if (vb)
            return by_dtype(bf16, [&](auto *tag) {
                typedef typename std::remove_pointer<decltype(tag)>::type T;
                const GradSrc<T> gs{(const T *)dy, (const T *)pool_g, pool_idx, pool_W, pool_W / 2, HW, HW / 4};
                const long long cnt = vb < 0 ? (long long)N * ((HW + 7) / 8)
                                             : (long long)N * (HW / (vb / (int)sizeof(T)));   // vectors per channel
                const bool few = (vb >= 8 || vb < 0) && cnt <= 1024LL * BN_FUSED_NVS;
                if (vb < 0) {
                    if (bn_fused_small(cnt, BN_FUSED_NVS))
                        hipLaunchKernelGGL((bn_bwd_fused_kernel<T, 16, BN_FUSED_NVS, 256, true>), dim3(C), dim3(256), 0, s,
                                           (const T *)x, gs, relu_beta, (T *)dx, gamma, mean, invstd, dgamma, dbeta, N, C, HW);
                    else
                        hipLaunchKernelGGL((bn_bwd_fused_kernel<T, 16, BN_FUSED_NVS, 1024, true>), dim3(C), dim3(1024), 0, s,
                                           (const T *)x, gs, relu_beta, (T *)dx, gamma, mean, invstd, dgamma, dbeta, N, C, HW);
                    return;
                }
#define SN_BN_BWD(VB_, NV_)                                                                                           \
    do {                                                                                                              \
        if (bn_fused_small(cnt, NV_))                                                                                 \
            hipLaunchKernelGGL((bn_bwd_fused_kernel<T, VB_, NV_, 256>), dim3(C), dim3(256), 0, s, (const T *)x, gs,   \
                               relu_beta, (T *)dx, gamma, mean, invstd, dgamma, dbeta, N, C, HW);                     \
        else                                                                                                          \
            hipLaunchKernelGGL((bn_bwd_fused_kernel<T, VB_, NV_, 1024>), dim3(C), dim3(1024), 0, s, (const T *)x, gs, \
                               relu_beta, (T *)dx, gamma, mean, invstd, dgamma, dbeta, N, C, HW);                     \
    } while (0)
                if (vb == 16 && few) SN_BN_BWD(16, BN_FUSED_NVS);
                else if (vb == 8 && few) SN_BN_BWD(8, BN_FUSED_NVS);
                else if (vb == 16) SN_BN_BWD(16, BN_FUSED_NV);
                else if (vb == (int)sizeof(T)) SN_BN_BWD(sizeof(T), BN_FUSED_NV1);
                else SN_BN_BWD(8, BN_FUSED_NV);
#undef SN_BN_BWD
            });
    }
    const Slices sl = make_slices(N, C, HW, (size_t)N * C * HW * esz);
    float *part = reinterpret_cast<float *>(dx);  // dx is dead until pass 3
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        dim3 grid(C, sl.nslice), block(256);
        const GradSrc<T> gs{(const T *)dy, (const T *)pool_g, pool_idx, pool_W, pool_W / 2, HW, HW / 4};
        hipLaunchKernelGGL(bn_bwd_reduce_kernel<T>, grid, block, 0, s, (const T *)x, gs, gamma, relu_beta,
                           mean, invstd, part, N, C, HW, sl);
        hipLaunchKernelGGL(bn_bwd_final_kernel, dim3(C), dim3(64), 0, s, part, invstd, dgamma, dbeta,
                           sl.nslice);
        hipLaunchKernelGGL(bn_bwd_apply_kernel<T>, grid, block, 0, s, (const T *)x, gs, relu_beta,
                           (T *)dx, gamma, mean, invstd, dgamma, dbeta, N, C, HW, sl);
    });
}

template <typename T, int VEC, bool RAG = false, bool RELU = false>
hipError_t lrn_launch(bool bwd, const void *x, const void *dy, void *out, int N, int C, int HW, int half, float a_n,
                      float beta, float k, hipStream_t s)
{
    const int vpp = RAG ? (HW + VEC - 1) / VEC : HW / VEC;
    const size_t total = (size_t)N * vpp;
    // A thread walks its channels one after the other: with few positions the channels are split over
    // blockIdx.y (each part re-reads the HALF or 2 HALF channels beside it) until there are enough threads.
    // (measured on 128 x 256 x 27 x 27: 5 parts of 52 channels 3.1 TB/s forward, 1 part 0.9, 6 parts of 43 2.4)
    long long parts = total >= 400000 ? 1 : (450000 + (long long)total - 1) / (long long)total;
    if (parts > (C + 7) / 8) parts = (C + 7) / 8;
    if (parts < 1) parts = 1;
    const int cc = (int)((C + parts - 1) / parts + 3) / 4 * 4, ny = (C + cc - 1) / cc;
    const dim3 grid((unsigned)((total + 255) / 256), (unsigned)ny), block(256);
#define SN_LRN(H_)                                                                                                  \
    case H_:                                                                                                        \
        if (bwd) hipLaunchKernelGGL((lrn_bwd_kernel<T, VEC, H_, RAG, RELU>), grid, block, 0, s, (const T *)x, (const T *)dy,  \
                                    (T *)out, C, HW, vpp, total, a_n, beta, k, cc);                                \
        else hipLaunchKernelGGL((lrn_fwd_kernel<T, VEC, H_, RAG, RELU>), grid, block, 0, s, (const T *)x, (T *)out, C, HW,    \
                                vpp, total, a_n, beta, k, cc);                                                      \
        break;
    switch (half) {
        SN_LRN(0) SN_LRN(1) SN_LRN(2) SN_LRN(3) SN_LRN(4)
    default: return hipErrorInvalidValue;
    }
#undef SN_LRN
    return hipGetLastError();
}

// size: odd, at most 9.  dy == nullptr: forward (out = y); else backward (out = dx).
// relu != 0: the layer's input is max(x, 0) (forward), and dx is also gated by x > 0 (backward).
template <bool RELU>
static hipError_t lrn_dispatch(const void *x, const void *dy, void *out, int N, int C, int HW, int size, float alpha,
                               float beta, float k, int bf16, hipStream_t s)
{
    const bool bwd = dy != nullptr, vec = HW % 4 == 0, rag = !vec && HW >= 4;
    const float a_n = alpha / (float)size;
    if (bf16) return vec ? lrn_launch<bf16_t, 4, false, RELU>(bwd, x, dy, out, N, C, HW, size / 2, a_n, beta, k, s)
                   : rag ? lrn_launch<bf16_t, 4, true, RELU>(bwd, x, dy, out, N, C, HW, size / 2, a_n, beta, k, s)
                         : lrn_launch<bf16_t, 1, false, RELU>(bwd, x, dy, out, N, C, HW, size / 2, a_n, beta, k, s);
    return vec ? lrn_launch<float, 4, false, RELU>(bwd, x, dy, out, N, C, HW, size / 2, a_n, beta, k, s)
         : rag ? lrn_launch<float, 4, true, RELU>(bwd, x, dy, out, N, C, HW, size / 2, a_n, beta, k, s)
               : lrn_launch<float, 1, false, RELU>(bwd, x, dy, out, N, C, HW, size / 2, a_n, beta, k, s);
}

hipError_t launch_lrn(const void *x, const void *dy, void *out, int N, int C, int HW, int size, float alpha,
                      float beta, float k, int bf16, hipStream_t s, int relu)
{
    if (size < 1 || size > 9 || !(size & 1)) return hipErrorInvalidValue;
    return relu ? lrn_dispatch<true>(x, dy, out, N, C, HW, size, alpha, beta, k, bf16, s)
                : lrn_dispatch<false>(x, dy, out, N, C, HW, size, alpha, beta, k, bf16, s);
}

hipError_t launch_maxpool_fwd(const void *x, void *y, int32_t *idx, int NC, int H, int W, int P, int Q, int kh,
                              int kw, int sh, int sw, int ph, int pw, int bf16, hipStream_t s)
{
    const size_t total = (size_t)NC * P * Q;
    if (total == 0) return hipSuccess;
    if (pool2_fast(NC, P, kh, kw, sh, sw, ph, pw) && log2_groups((Q + 7) / 8) >= 0) {
        const int lg = log2_groups((Q + 7) / 8);
        const unsigned rows = (unsigned)NC * P, rpb = 256u >> lg;
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
            hipLaunchKernelGGL(maxpool2_fwd_kernel<T>, dim3((rows + rpb - 1) / rpb), dim3(256), 0, s, (const T *)x,
                               (T *)y, idx, rows, H, W, P, Q, lg, (const T *)x + (size_t)NC * H * W);
        });
    }
    if (kh == 3 && kw == 3 && sh == 2 && sw == 2 && ph >= 0 && ph <= 2 && pw >= 0 && pw <= 2 &&
        (long long)NC * P <= 0x7fffffffLL && (long long)H * W <= 0x7fffffffLL && log2_groups((Q + 3) / 4) >= 0) {
        const int lg = log2_groups((Q + 3) / 4);
        const unsigned rows = (unsigned)NC * P, rpb = 256u >> lg;
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
            hipLaunchKernelGGL(maxpool3s2_fwd_kernel<T>, dim3((rows + rpb - 1) / rpb), dim3(256), 0, s, (const T *)x,
                               (T *)y, idx, rows, H, W, P, Q, ph, pw, lg, (const T *)x + (size_t)NC * H * W);
        });
    }
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        dim3 grid((unsigned)((total + 255) / 256)), block(256);
        if (total <= 0xffffffffull)
            hipLaunchKernelGGL((maxpool_fwd_kernel<T, uint32_t>), grid, block, 0, s, (const T *)x, (T *)y, idx, total, H,
                               W, P, Q, kh, kw, sh, sw, ph, pw);
        else
            hipLaunchKernelGGL((maxpool_fwd_kernel<T, size_t>), grid, block, 0, s, (const T *)x, (T *)y, idx, total, H,
                               W, P, Q, kh, kw, sh, sw, ph, pw);
    });
}

hipError_t launch_maxpool_bwd(const void *dy, const int32_t *idx, void *dx, int NC, int H, int W, int P, int Q,
                              int kh, int kw, int sh, int sw, int ph, int pw, int bf16, hipStream_t s)
{
    const size_t total = (size_t)NC * H * W;
    if (total == 0) return hipSuccess;
    if (pool2_fast(NC, P, kh, kw, sh, sw, ph, pw) && P > 0 && Q > 0 && log2_groups((W + 7) / 8) >= 0) {
        const int lg = log2_groups((W + 7) / 8);
        const unsigned rows = (unsigned)NC * P, rpb = 256u >> lg;
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
            hipLaunchKernelGGL(maxpool2_bwd_kernel<T>, dim3((rows + rpb - 1) / rpb), dim3(256), 0, s, (const T *)dy,
                               idx, (T *)dx, rows, H, W, P, Q, lg);
        });
    }
    if (kh == 3 && kw == 3 && sh == 2 && sw == 2 && ph >= 0 && ph <= 2 && pw >= 0 && pw <= 2 && P > 0 && Q > 0 &&
        (long long)NC * H <= 0x7fffffffLL && log2_groups((W + 7) / 8) >= 0) {
        const int lg = log2_groups((W + 7) / 8);
        const unsigned rows = (unsigned)NC * H, rpb = 256u >> lg;
        return by_dtype(bf16, [&](auto *tag) {
            typedef typename std::remove_pointer<decltype(tag)>::type T;
            hipLaunchKernelGGL(maxpool3s2_bwd_kernel<T>, dim3((rows + rpb - 1) / rpb), dim3(256), 0, s, (const T *)dy,
                               idx, (T *)dx, rows, H, W, P, Q, ph, pw, lg);
        });
    }
    const unsigned bpp = (unsigned)(((long long)H * W + 255) / 256);
    if ((unsigned long long)bpp * (unsigned)NC > 0x7fffffffULL) return hipErrorInvalidValue;
    return by_dtype(bf16, [&](auto *tag) {
        typedef typename std::remove_pointer<decltype(tag)>::type T;
        dim3 grid(bpp * (unsigned)NC), block(256);
        if (kh == 3 && kw == 3 && sh == 2 && sw == 2)
            hipLaunchKernelGGL((maxpool_bwd_kernel<T, 3>), grid, block, 0, s, (const T *)dy, idx, (T *)dx, bpp, H, W, P,
                               Q, kh, kw, sh, sw, ph, pw);
        else
            hipLaunchKernelGGL((maxpool_bwd_kernel<T, 0>), grid, block, 0, s, (const T *)dy, idx, (T *)dx, bpp, H, W, P,
                               Q, kh, kw, sh, sw, ph, pw);
    });
}

}  // namespace sn
