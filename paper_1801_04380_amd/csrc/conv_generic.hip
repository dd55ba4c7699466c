// Fallback implicit-GEMM convolution for gfx950: any filter size, stride and
// padding, fp32 or bf16 inputs, all three directions, no workspace.
//
// Each direction of a CONV step (Sec. 3.5 of the paper; the definitions are in
// sn.h) is one GEMM  D[M x Ncols] = A[M x Kred] * B[Kred x Ncols]  whose operands
// are gathered on the fly from the NCHW / KCRS tensors:
//   forward          M = K, Ncols = N*P*Q,  Kred = C*R*S   A = w,  B = x patches
//   backward-data    M = C, Ncols = N*H*W,  Kred = K*R*S   A = w,  B = dy patches
//   backward-filter  M = K, Ncols = C*R*S,  Kred = N*P*Q   A = dy, B = x patches
// A 256-thread workgroup owns a BM x 128 tile of D.  Per step of BK reduction
// indices it gathers both operand tiles into LDS in [row][k] order (k contiguous,
// which is what an MFMA lane wants: 8 consecutive bf16 k-values per lane for
// v_mfma_f32_32x32x16_bf16, one fp32 per lane for v_mfma_f32_32x32x2_f32), then
// each of the 4 waves runs 32x32 MFMA tiles over it.  Global loads for step i+1
// are issued before the MFMAs of step i.
//
// Two gather mappings keep the global loads coalesced:
//   "row" mapping: a lane owns one tile row and a run of consecutive k -- used
//       when neighbouring rows are neighbours in memory (pixels of x / dy);
//   "k" mapping:   a lane owns one k and several rows -- used when consecutive
//       k are neighbours in memory (w rows in forward; dy and x in backward-filter,
//       where k runs over pixels).
// Backward-filter of filters larger than 1x1 and strided backward-data have kernels of their own
// further down (igemm_bwd_filter_kernel, igemm_bwd_data_classes_kernel) on the same tiles.
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int DIR_FWD = 0, DIR_BWD_DATA = 1, DIR_BWD_FILTER = 2;
constexpr int BN = 128;      // tile columns
constexpr int NTHREADS = 256;

template <typename T> struct TileCfg;
template <> struct TileCfg<bf16_t> { static constexpr int BK = 32, PITCH = 40; };  // 80-byte rows
template <> struct TileCfg<float>  { static constexpr int BK = 16, PITCH = 20; };  // 80-byte rows

struct GemmDims {
    int M, Ncols, Kred;
    int kchunk;  // reduction indices per blockIdx.z slice (multiple of BK)
};

template <typename T> __device__ inline T zero_of() { return (T)0; }

// ---------------------------------------------------------------- gathers
// Row mapping: this thread owns tile row `row` and E consecutive k starting at
// kseg*E.  `Pre` holds what depends on the row only.
struct RowPre {
    long long base;  // element offset of the row's image (or filter row)
    int a, b;        // forward: h0, w0; backward-data: h+ph, v+pw
    bool valid;
};

template <int DIR>
__device__ inline RowPre row_pre_B(const ConvGeom &g, int j, int Ncols)
{
    RowPre r;
    r.valid = j < Ncols;
    int jj = r.valid ? j : 0;
    if (DIR == DIR_FWD) {
        int PQ = g.P * g.Q, n = jj / PQ, pq = jj - n * PQ, p = pq / g.Q, q = pq - p * g.Q;
        r.base = (long long)n * g.C * g.H * g.W;
        r.a = p * g.sh - g.ph;
        r.b = q * g.sw - g.pw;
    } else {  // backward-data: columns are input pixels (n,h,v)
        int HW = g.H * g.W, n = jj / HW, hw = jj - n * HW, h = hw / g.W, v = hw - h * g.W;
        r.base = (long long)n * g.K * g.P * g.Q;
        r.a = h + g.ph;
        r.b = v + g.pw;
    }
    return r;
}

template <typename T, int DIR, int E>
__device__ inline void fetch_row_B(T (&reg)[E], const T *__restrict__ src, const ConvGeom &g,
                                   const RowPre &pre, int kk0)
{
    const int RS = g.R * g.S;
    int c = kk0 / RS, rs = kk0 - c * RS, r = rs / g.S, s = rs - r * g.S;
    const T *b = src + pre.base;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        T val = zero_of<T>();
        if (DIR == DIR_FWD) {
            int h = pre.a + r, v = pre.b + s;
            if (pre.valid && c < g.C && (unsigned)h < (unsigned)g.H && (unsigned)v < (unsigned)g.W)
                val = b[((long long)c * g.H + h) * g.W + v];
        } else {
            // c is the output channel k here; the tap (r,s) maps input pixel
            // (h,v) back to output pixel (p,q) when the stride divides.
            int hp = pre.a - r, vq = pre.b - s;
            if (pre.valid && c < g.K && hp >= 0 && vq >= 0) {
                int p = hp / g.sh, q = vq / g.sw;
                if (p * g.sh == hp && q * g.sw == vq && p < g.P && q < g.Q)
                    val = b[((long long)c * g.P + p) * g.Q + q];
            }
        }
        reg[e] = val;
        if (++s == g.S) { s = 0; if (++r == g.R) { r = 0; ++c; } }
    }
}

// backward-data A operand: row m is the input channel c, k runs over (k,r,s):
// element w[k][m][r][s].
template <typename T, int E>
__device__ inline void fetch_row_A_bwd_data(T (&reg)[E], const T *__restrict__ w, const ConvGeom &g,
                                            int m, int kk0)
{
    const int RS = g.R * g.S;
    int k = kk0 / RS, rs = kk0 - k * RS;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        T val = zero_of<T>();
        if (m < g.C && k < g.K) val = w[((long long)k * g.C + m) * RS + rs];
        reg[e] = val;
        if (++rs == RS) { rs = 0; ++k; }
    }
}

// k mapping: this thread owns reduction index kk and rows rg + i*RG.
template <typename T, int NR, int RG>
__device__ inline void fetch_k_A_fwd(T (&reg)[NR], const T *__restrict__ w, int M, int Kred, int m0,
                                     int rg, int kk)
{
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        int m = m0 + rg + i * RG;
        reg[i] = (kk < Kred && m < M) ? w[(long long)m * Kred + kk] : zero_of<T>();
    }
}

template <typename T, int NR, int RG>
__device__ inline void fetch_k_A_bwd_filter(T (&reg)[NR], const T *__restrict__ dy, const ConvGeom &g,
                                            int m0, int rg, int kk, int kend)
{
    const int PQ = g.P * g.Q;
    bool ok = kk < kend;
    int kc = ok ? kk : 0, n = kc / PQ, pq = kc - n * PQ;
    const T *b = dy + (long long)n * g.K * PQ + pq;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        int m = m0 + rg + i * RG;
        reg[i] = (ok && m < g.K) ? b[(long long)m * PQ] : zero_of<T>();
    }
}

template <typename T, int NR>
__device__ inline void fetch_k_B_bwd_filter(T (&reg)[NR], const T *__restrict__ x, const ConvGeom &g,
                                            const int (&joff)[NR], const int (&jrs)[NR], int kk, int kend)
{
    const int PQ = g.P * g.Q;
    bool ok = kk < kend;
    int kc = ok ? kk : 0, n = kc / PQ, pq = kc - n * PQ, p = pq / g.Q, q = pq - p * g.Q;
    int hb = p * g.sh, vb = q * g.sw;
    const T *b = x + (long long)n * g.C * g.H * g.W + (long long)hb * g.W + vb;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        int dr = jrs[i] >> 16, ds = (int)(short)(jrs[i] & 0xffff);
        int h = hb + dr, v = vb + ds;
        bool in = ok && jrs[i] != 0x7fffffff && (unsigned)h < (unsigned)g.H && (unsigned)v < (unsigned)g.W;
        reg[i] = in ? b[joff[i]] : zero_of<T>();
    }
}

// ---------------------------------------------------------------- LDS stores
template <typename T, int E>
__device__ inline void store_row(T *tile, int row, int kseg, const T (&reg)[E])
{
    constexpr int PITCH = TileCfg<T>::PITCH;
    T *dst = tile + row * PITCH + kseg * E;
    constexpr int VEC = 16 / sizeof(T);
    static_assert(E % VEC == 0, "row segment must be whole 16-byte pieces");
#pragma unroll
    for (int v = 0; v < E / VEC; ++v) {
        union { T t[VEC]; uint4 u; } pack;
#pragma unroll
        for (int e = 0; e < VEC; ++e) pack.t[e] = reg[v * VEC + e];
        *reinterpret_cast<uint4 *>(dst + v * VEC) = pack.u;
    }
}

template <typename T, int NR, int RG>
__device__ inline void store_k(T *tile, int rg, int kl, const T (&reg)[NR])
{
    constexpr int PITCH = TileCfg<T>::PITCH;
#pragma unroll
    for (int i = 0; i < NR; ++i) tile[(rg + i * RG) * PITCH + kl] = reg[i];
}

// ---------------------------------------------------------------- MFMA over one LDS tile pair
template <int TM, int TN>
__device__ inline void mma_tile(const bf16_t *As, const bf16_t *Bs, int arow, int brow, int lane,
                                f32x16 (&acc)[TM][TN])
{
    constexpr int PITCH = TileCfg<bf16_t>::PITCH;
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int step = 0; step < 2; ++step) {
        bf16x8 a[TM], b[TN];
#pragma unroll
        for (int t = 0; t < TM; ++t)
            a[t] = *reinterpret_cast<const bf16x8 *>(As + (arow + t * 32 + r) * PITCH + step * 16 + hi * 8);
#pragma unroll
        for (int t = 0; t < TN; ++t)
            b[t] = *reinterpret_cast<const bf16x8 *>(Bs + (brow + t * 32 + r) * PITCH + step * 16 + hi * 8);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

template <int TM, int TN>
__device__ inline void mma_tile(const float *As, const float *Bs, int arow, int brow, int lane,
                                f32x16 (&acc)[TM][TN])
{
    constexpr int PITCH = TileCfg<float>::PITCH;
    const int r = lane & 31, hi = lane >> 5;
    float a[TM][8], b[TN][8];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const float4 *p = reinterpret_cast<const float4 *>(As + (arow + t * 32 + r) * PITCH + hi * 8);
        float4 lo = p[0], up = p[1];
        a[t][0] = lo.x; a[t][1] = lo.y; a[t][2] = lo.z; a[t][3] = lo.w;
        a[t][4] = up.x; a[t][5] = up.y; a[t][6] = up.z; a[t][7] = up.w;
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const float4 *p = reinterpret_cast<const float4 *>(Bs + (brow + t * 32 + r) * PITCH + hi * 8);
        float4 lo = p[0], up = p[1];
        b[t][0] = lo.x; b[t][1] = lo.y; b[t][2] = lo.z; b[t][3] = lo.w;
        b[t][4] = up.x; b[t][5] = up.y; b[t][6] = up.z; b[t][7] = up.w;
    }
    // MFMA e multiplies k-index {e (lanes 0-31), 8+e (lanes 32-63)} of the tile:
    // any pairing works as long as A and B use the same one.
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], b[j][e], acc[i][j], 0, 0, 0);
}

// ---------------------------------------------------------------- the kernel
template <typename T, int DIR, int BM>
__global__ void __launch_bounds__(NTHREADS)
igemm_generic_kernel(const T *__restrict__ Asrc, const T *__restrict__ Bsrc, void *__restrict__ out,
                     float *__restrict__ partial, ConvGeom g, GemmDims d)
{
    constexpr int BK = TileCfg<T>::BK, PITCH = TileCfg<T>::PITCH;
    constexpr bool A_ROWMAP = (DIR == DIR_BWD_DATA);
    constexpr bool B_ROWMAP = (DIR != DIR_BWD_FILTER);
    // row mapping
    constexpr int A_KSEGS = NTHREADS / BM, A_E = BK / A_KSEGS;
    constexpr int B_KSEGS = NTHREADS / BN, B_E = BK / B_KSEGS;
    // k mapping
    constexpr int RG = NTHREADS / BK, A_NR = BM / RG, B_NR = BN / RG;
    constexpr int A_REGS = A_ROWMAP ? A_E : A_NR, B_REGS = B_ROWMAP ? B_E : B_NR;
    // wave tiling: BM=128 -> 2x2 waves of 64x64; BM=64 -> 1x4 waves of 64x32
    constexpr int TM = 2, TN = (BM == 128) ? 2 : 1;

    __shared__ __attribute__((aligned(16))) T As[BM * PITCH];
    __shared__ __attribute__((aligned(16))) T Bs[BN * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    const int kbeg = blockIdx.z * d.kchunk;
    const int kend = min(d.Kred, kbeg + d.kchunk);

    // per-thread constants of the gathers
    RowPre preB = {};
    int a_row = 0, a_kseg = 0, b_row = 0, b_kseg = 0;
    if (A_ROWMAP) { a_row = tid % BM; a_kseg = tid / BM; }
    if (B_ROWMAP) {
        b_row = tid % BN; b_kseg = tid / BN;
        preB = row_pre_B<DIR>(g, col0 + b_row, d.Ncols);
    }
    const int kl = tid % BK, rg = tid / BK;
    int joff[B_REGS], jrs[B_REGS];
    if (DIR == DIR_BWD_FILTER) {
        const int RS = g.R * g.S;
#pragma unroll
        for (int i = 0; i < B_REGS; ++i) {
            int j = col0 + rg + i * RG;
            if (j < d.Ncols) {
                int c = j / RS, rs = j - c * RS, r = rs / g.S, s = rs - r * g.S;
                joff[i] = (c * g.H + (r - g.ph)) * g.W + (s - g.pw);
                jrs[i] = ((r - g.ph) << 16) | ((s - g.pw) & 0xffff);
            } else {
                joff[i] = 0;
                jrs[i] = 0x7fffffff;
            }
        }
    }

    T ra[A_REGS], rb[B_REGS];
    auto fetch = [&](int k0) {
        if (DIR == DIR_FWD) fetch_k_A_fwd<T, A_REGS, RG>(ra, Asrc, d.M, d.Kred, m0, rg, k0 + kl);
        if (DIR == DIR_BWD_DATA) fetch_row_A_bwd_data<T, A_REGS>(ra, Asrc, g, m0 + a_row, k0 + a_kseg * A_E);
        if (DIR == DIR_BWD_FILTER) fetch_k_A_bwd_filter<T, A_REGS, RG>(ra, Asrc, g, m0, rg, k0 + kl, kend);
        if (DIR == DIR_BWD_FILTER) fetch_k_B_bwd_filter<T, B_REGS>(rb, Bsrc, g, joff, jrs, k0 + kl, kend);
        else fetch_row_B<T, DIR, B_REGS>(rb, Bsrc, g, preB, k0 + b_kseg * B_E);
    };
    auto stage = [&]() {
        if (A_ROWMAP) store_row<T, A_REGS>(As, a_row, a_kseg, ra);
        else store_k<T, A_REGS, RG>(As, rg, kl, ra);
        if (B_ROWMAP) store_row<T, B_REGS>(Bs, b_row, b_kseg, rb);
        else store_k<T, B_REGS, RG>(Bs, rg, kl, rb);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int arow = (BM == 128) ? (wave >> 1) * 64 : 0;
    const int brow = (BM == 128) ? (wave & 1) * 64 : wave * 32;

    if (kbeg < kend) {
        fetch(kbeg);
        stage();
        __syncthreads();
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            const bool more = k0 + BK < kend;
            if (more) fetch(k0 + BK);
            mma_tile<TM, TN>(As, Bs, arow, brow, lane, acc);
            __syncthreads();
            if (more) {
                stage();
                __syncthreads();
            }
        }
    }

    // epilogue: a 32x32 accumulator tile keeps column (lane % 32) and rows
    // 8*(v/4) + 4*(lane/32) + v%4 in register v.
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int col = col0 + brow + tn * 32 + r;
        if (col >= d.Ncols) continue;
        long long cbase;   // offset of (row 0, col)
        long long rstride; // offset step per row
        if (DIR == DIR_FWD) {
            int PQ = g.P * g.Q, n = col / PQ, pq = col - n * PQ;
            cbase = (long long)n * g.K * PQ + pq;
            rstride = PQ;
        } else if (DIR == DIR_BWD_DATA) {
            int HW = g.H * g.W, n = col / HW, hw = col - n * HW;
            cbase = (long long)n * g.C * HW + hw;
            rstride = HW;
        } else {
            cbase = col;
            rstride = d.Ncols;
        }
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + arow + tm * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
                if (row >= d.M) continue;
                const long long off = cbase + (long long)row * rstride;
                const float val = acc[tm][tn][v];
                if (DIR == DIR_BWD_FILTER) {
                    if (partial) partial[(long long)blockIdx.z * d.M * d.Ncols + off] = val;
                    else if (gridDim.z > 1) unsafeAtomicAdd(reinterpret_cast<float *>(out) + off, val);
                    else reinterpret_cast<float *>(out)[off] = val;
                } else if (g.out_bf16) {
                    reinterpret_cast<bf16_t *>(out)[off] = f32_to_bf16(val);
                } else {
                    reinterpret_cast<float *>(out)[off] = val;
                }
            }
    }
}

// Backward-data of a strided convolution, one residue class of input pixels per blockIdx.z.
// Input pixel (h, v) receives tap (r, s) only where sh divides h + ph - r and sw divides
// v + pw - s, so the pixels with h = a (mod sh), v = b (mod sw) all use the same taps:
// r = r0 + sh*t, s = s0 + sw*u with r0 = (a + ph) mod sh, s0 = (b + pw) mod sw, and pixel
// (a + sh*i, b + sw*j) reads dy at (i + (a + ph)/sh - t, j + (b + pw)/sw - u).  A tile's 128
// columns are pixels (n, i, j) of one class, so the reduction runs over that class's taps only
// (R*S / (sh*sw) of them on average instead of R*S with the rest multiplying zeros), a tap at a
// time over the output channels (padded to whole steps: a step never straddles two taps), and
// neighbouring lanes read neighbouring dy elements.  A class without taps (filter shorter than
// the stride) stores zeros.
template <typename T, int BM>
__global__ void __launch_bounds__(NTHREADS)
igemm_bwd_data_classes_kernel(const T *__restrict__ w, const T *__restrict__ dy, void *__restrict__ dx,
                              ConvGeom g, int Kpad)
{
    constexpr int BK = TileCfg<T>::BK, PITCH = TileCfg<T>::PITCH;
    constexpr int A_KSEGS = NTHREADS / BM, A_E = BK / A_KSEGS;
    constexpr int B_KSEGS = NTHREADS / BN, B_E = BK / B_KSEGS;
    constexpr int TM = 2, TN = (BM == 128) ? 2 : 1;

    __shared__ __attribute__((aligned(16))) T As[BM * PITCH];
    __shared__ __attribute__((aligned(16))) T Bs[BN * PITCH];

    const int ca = blockIdx.z / g.sw, cb = blockIdx.z - ca * g.sw;
    const int Ha = ca < g.H ? (g.H - ca + g.sh - 1) / g.sh : 0;
    const int Wb = cb < g.W ? (g.W - cb + g.sw - 1) / g.sw : 0;
    const int ncols = g.N * Ha * Wb;
    const int col0 = blockIdx.x * BN;
    if (col0 >= ncols) return;  // the grid is sized for the largest class
    const int r0 = (ca + g.ph) % g.sh, s0 = (cb + g.pw) % g.sw;
    const int pa = (ca + g.ph) / g.sh, qb = (cb + g.pw) / g.sw;
    const int nt = r0 < g.R ? (g.R - r0 + g.sh - 1) / g.sh : 0;
    const int nu = s0 < g.S ? (g.S - s0 + g.sw - 1) / g.sw : 0;
    const int kend = nt * nu * Kpad;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * BM;
    const int a_row = tid % BM, a_kseg = tid / BM, b_row = tid % BN, b_kseg = tid / BN;
    const int RS = g.R * g.S, PQ = g.P * g.Q;

    // this thread's column of B: pixel (n, i, j) of the class
    const bool bvalid = col0 + b_row < ncols;
    int bp, bq;
    long long bbase;
    {
        const int j = bvalid ? col0 + b_row : 0;
        const int n = j / (Ha * Wb), ij = j - n * (Ha * Wb), i = ij / Wb;
        bp = i + pa;
        bq = ij - i * Wb + qb;
        bbase = (long long)n * g.K * PQ;
    }
    const bool avalid = m0 + a_row < g.C;
    const long long abase = (long long)(avalid ? m0 + a_row : 0) * RS;

    T ra[A_E], rb[B_E];
    auto fetch = [&](int k0) {
        const int tap = k0 / Kpad, kb = k0 - tap * Kpad;
        const int t = tap / nu, u = tap - t * nu;
        const int rs = (r0 + g.sh * t) * g.S + s0 + g.sw * u;
        const int p = bp - t, q = bq - u;
        const bool in = bvalid && (unsigned)p < (unsigned)g.P && (unsigned)q < (unsigned)g.Q;
        const T *bsrc = dy + bbase + (long long)(in ? p * g.Q + q : 0);
#pragma unroll
        for (int e = 0; e < B_E; ++e) {
            const int k = kb + b_kseg * B_E + e;
            rb[e] = (in && k < g.K) ? bsrc[(long long)k * PQ] : zero_of<T>();
        }
        const T *asrc = w + abase + rs;
#pragma unroll
        for (int e = 0; e < A_E; ++e) {
            const int k = kb + a_kseg * A_E + e;
            ra[e] = (avalid && k < g.K) ? asrc[(long long)k * g.C * RS] : zero_of<T>();
        }
    };
    auto stage = [&]() {
        store_row<T, A_E>(As, a_row, a_kseg, ra);
        store_row<T, B_E>(Bs, b_row, b_kseg, rb);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int arow = (BM == 128) ? (wave >> 1) * 64 : 0;
    const int brow = (BM == 128) ? (wave & 1) * 64 : wave * 32;

    if (kend > 0) {
        fetch(0);
        stage();
        __syncthreads();
        for (int k0 = 0; k0 < kend; k0 += BK) {
            const bool more = k0 + BK < kend;
            if (more) fetch(k0 + BK);
            mma_tile<TM, TN>(As, Bs, arow, brow, lane, acc);
            __syncthreads();
            if (more) {
                stage();
                __syncthreads();
            }
        }
    }

    const int r = lane & 31, hi = lane >> 5;
    const long long HW = (long long)g.H * g.W;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int col = col0 + brow + tn * 32 + r;
        if (col >= ncols) continue;
        const int n = col / (Ha * Wb), ij = col - n * (Ha * Wb), i = ij / Wb, j = ij - i * Wb;
        const long long cbase = (long long)n * g.C * HW + (long long)(ca + g.sh * i) * g.W + cb + g.sw * j;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + arow + tm * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
                if (row >= g.C) continue;
                const long long off = cbase + row * HW;
                const float val = acc[tm][tn][v];
                if (g.out_bf16) reinterpret_cast<bf16_t *>(dx)[off] = f32_to_bf16(val);
                else reinterpret_cast<float *>(dx)[off] = val;
            }
    }
}

template <typename T>
hipError_t launch_bwd_data_classes(const void *dy, const void *w, void *dx, const ConvGeom &g, hipStream_t st)
{
    constexpr int BK = TileCfg<T>::BK;
    const int Kpad = (g.K + BK - 1) / BK * BK;
    const long long cols = (long long)g.N * ((g.H + g.sh - 1) / g.sh) * ((g.W + g.sw - 1) / g.sw);
    const unsigned gx = (unsigned)((cols + BN - 1) / BN), gz = (unsigned)(g.sh * g.sw);
    if (g.C <= 64)
        hipLaunchKernelGGL((igemm_bwd_data_classes_kernel<T, 64>), dim3(gx, (g.C + 63) / 64, gz), dim3(NTHREADS), 0, st,
                           (const T *)w, (const T *)dy, dx, g, Kpad);
    else
        hipLaunchKernelGGL((igemm_bwd_data_classes_kernel<T, 128>), dim3(gx, (g.C + 127) / 128, gz), dim3(NTHREADS), 0,
                           st, (const T *)w, (const T *)dy, dx, g, Kpad);
    return hipGetLastError();
}

// Backward-filter with both operands fetched along the pixels.  The reduction index is the output pixel
// (n, p, q): dy has it contiguous, so a thread's share of the A tile is one 16-byte piece of a dy row (at any
// element alignment; element by element only where the piece crosses an image or the slice's end), stored
// to LDS as it is -- the MFMA layout wants consecutive reduction entries together.  The B tile holds, per
// column (c, r, s), x at (p*sh + r - ph, q*sw + s - pw) for the same pixels: a thread gathers the VEC elements
// of a piece one by one (zeros in the padding) and stores them as one 16-byte item.  Against the generic kernel's
// mapping (a thread owns one pixel and 16 rows of each tile: 32 two-byte loads and 32 two-byte LDS stores per
// step) that is 18 loads and 4 stores.
template <typename T, int BM>
__global__ void __launch_bounds__(NTHREADS)
igemm_bwd_filter_kernel(const T *__restrict__ dy, const T *__restrict__ x, float *__restrict__ out,
                        float *__restrict__ partial, ConvGeom g, GemmDims d)
{
    constexpr int BK = TileCfg<T>::BK, PITCH = TileCfg<T>::PITCH;
    constexpr int VEC = 16 / sizeof(T), SEGS = BK / VEC;        // pieces per tile row
    constexpr int ROWS = NTHREADS / SEGS;                        // tile rows one round of the threads covers
    constexpr int A_IT = BM / ROWS, B_IT = BN / ROWS;
    constexpr int TM = 2, TN = (BM == 128) ? 2 : 1;
    typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
    struct __attribute__((packed, aligned(sizeof(T)))) AnyVec { u32x4v v; };

    __shared__ __attribute__((aligned(16))) T As[BM * PITCH];
    __shared__ __attribute__((aligned(16))) T Bs[BN * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    const int kbeg = blockIdx.z * d.kchunk;
    const int kend = min(d.Kred, kbeg + d.kchunk);
    const int seg = tid % SEGS, r0 = tid / SEGS;
    const int PQ = g.P * g.Q, RS = g.R * g.S;

    // the thread's B columns: tap offsets, and the element of the image the tap reads under output pixel (0, 0)
    // (an image has fewer than 2^31 elements; the batch may have more)
    int bconst[B_IT], bdr[B_IT], bds[B_IT];
    bool bok[B_IT];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int j = col0 + r0 + ROWS * i;
        bok[i] = j < d.Ncols;
        const int jj = bok[i] ? j : 0;
        const int c = jj / RS, rs = jj - c * RS, r = rs / g.S;
        bdr[i] = r - g.ph;
        bds[i] = rs - r * g.S - g.pw;
        bconst[i] = (c * g.H + bdr[i]) * g.W + bds[i];
    }
    const long long xplane_img = (long long)g.C * g.H * g.W;
    // the thread's first pixel of the step about to be fetched, kept from step to step (a step is BK pixels on)
    const int step_q = BK % g.Q, step_p = BK / g.Q;
    int fn, fp, fq;
    {
        const int kk = min(kbeg + seg * VEC, d.Kred - 1);
        fn = kk / PQ;
        const int pq = kk - fn * PQ;
        fp = pq / g.Q;
        fq = pq - fp * g.Q;
    }

    u32x4v ra[A_IT], rb[B_IT];
    auto fetch = [&](int k0) {
        const int kk = k0 + seg * VEC;
        int n = fn, p = fp, q = fq;
        const int pq = p * g.Q + q;
        // the same thread's pixel one step on (past the slice's end nothing is loaded)
        fq += step_q;
        fp += step_p;
        if (fq >= g.Q) { fq -= g.Q; ++fp; }
        while (fp >= g.P) { fp -= g.P; ++fn; }
        // A: dy[n][m][pq .. pq + VEC - 1]
        const bool whole = kk + VEC <= kend && pq + VEC <= PQ;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int m = m0 + r0 + ROWS * i;
            union { T t[VEC]; u32x4v u; } pack;
            if (m < g.K && whole) {
                pack.u = reinterpret_cast<const AnyVec *>(dy + ((long long)n * g.K + m) * PQ + pq)->v;
            } else {
                int ne = n, pe = pq;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    pack.t[e] = (m < g.K && kk + e < kend) ? dy[((long long)ne * g.K + m) * PQ + pe] : zero_of<T>();
                    if (++pe == PQ) { pe = 0; ++ne; }
                }
            }
            ra[i] = pack.u;
        }
        // B: x under each of the VEC pixels
        union { T t[VEC]; u32x4v u; } pb[B_IT];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool live = kk + e < kend;
            const T *img = x + n * xplane_img;
            const int hb = p * g.sh, wb = q * g.sw, po = hb * g.W + wb;
#pragma unroll
            for (int i = 0; i < B_IT; ++i) {
                const bool in = live && bok[i] && (unsigned)(hb + bdr[i]) < (unsigned)g.H &&
                                (unsigned)(wb + bds[i]) < (unsigned)g.W;
                pb[i].t[e] = in ? img[bconst[i] + po] : zero_of<T>();
            }
            if (++q == g.Q) { q = 0; if (++p == g.P) { p = 0; ++n; } }
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) rb[i] = pb[i].u;
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            *reinterpret_cast<u32x4v *>(As + (r0 + ROWS * i) * PITCH + seg * VEC) = ra[i];
#pragma unroll
        for (int i = 0; i < B_IT; ++i)
            *reinterpret_cast<u32x4v *>(Bs + (r0 + ROWS * i) * PITCH + seg * VEC) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int arow = (BM == 128) ? (wave >> 1) * 64 : 0;
    const int brow = (BM == 128) ? (wave & 1) * 64 : wave * 32;

    if (kbeg < kend) {
        fetch(kbeg);
        stage();
        __syncthreads();
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            const bool more = k0 + BK < kend;
            if (more) fetch(k0 + BK);
            mma_tile<TM, TN>(As, Bs, arow, brow, lane, acc);
            __syncthreads();
            if (more) {
                stage();
                __syncthreads();
            }
        }
    }

    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int col = col0 + brow + tn * 32 + r;
        if (col >= d.Ncols) continue;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + arow + tm * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
                if (row >= d.M) continue;
                const long long off = col + (long long)row * d.Ncols;
                const float val = acc[tm][tn][v];
                if (partial) partial[(long long)blockIdx.z * d.M * d.Ncols + off] = val;
                else if (gridDim.z > 1) unsafeAtomicAdd(out + off, val);
                else out[off] = val;
            }
    }
}

template <typename T>
hipError_t launch_bwd_filter_px(const void *dy, const void *x, float *dw, float *partial, const ConvGeom &g,
                                const GemmDims &d, int splits, hipStream_t st)
{
    if (d.M <= 64)
        hipLaunchKernelGGL((igemm_bwd_filter_kernel<T, 64>), dim3((d.Ncols + BN - 1) / BN, (d.M + 63) / 64, splits),
                           dim3(NTHREADS), 0, st, (const T *)dy, (const T *)x, dw, partial, g, d);
    else
        hipLaunchKernelGGL((igemm_bwd_filter_kernel<T, 128>), dim3((d.Ncols + BN - 1) / BN, (d.M + 127) / 128, splits),
                           dim3(NTHREADS), 0, st, (const T *)dy, (const T *)x, dw, partial, g, d);
    return hipGetLastError();
}

__global__ void reduce_partials_kernel(const float *__restrict__ partial, float *__restrict__ dw, size_t n,
                                       int splits, bool accumulate)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = accumulate ? dw[i] : 0.f;
    for (int z = 0; z < splits; ++z) s += partial[(size_t)z * n + i];
    dw[i] = s;
}

// The same sum for n a multiple of 4, 16 bytes per load: a workgroup of TX x TY threads (256 in all)
// takes TX consecutive float4; thread (tx, ty) adds slices ty, ty + TY, ... of its element in
// ascending order, and the TY sums are added in the order of ty.  The order is fixed, so the result
// is the same from run to run.  Few slices: TY = 4, so that a thread still has several loads in
// flight and a row of lanes reads 1 KB at a stretch; many slices: TY = 16.
template <int TY>
__global__ void __launch_bounds__(256)
reduce_partials4_kernel(const float4 *__restrict__ partial, float4 *__restrict__ dw, size_t n4, int splits,
                        bool accumulate)
{
    constexpr int TX = 256 / TY;
    __shared__ float4 part[TY][TX];
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    const size_t i = (size_t)blockIdx.x * TX + tx;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n4) {
#pragma unroll 4
        for (int z = ty; z < splits; z += TY) {
            const float4 v = partial[(size_t)z * n4 + i];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    part[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && i < n4) {
        float4 t = accumulate ? dw[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        const int ny = splits < TY ? splits : TY;
        for (int y = 0; y < ny; ++y) {
            const float4 v = part[y][tx];
            t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
        }
        dw[i] = t;
    }
}

__global__ void fill_zero_kernel(float *__restrict__ p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

template <typename T, int DIR>
hipError_t launch_dir(const void *a, const void *b, void *out, float *partial, const ConvGeom &g,
                      const GemmDims &d, int splits, hipStream_t st)
{
    dim3 block(NTHREADS);
    if (d.M <= 64) {
        dim3 grid((d.Ncols + BN - 1) / BN, (d.M + 63) / 64, splits);
        hipLaunchKernelGGL((igemm_generic_kernel<T, DIR, 64>), grid, block, 0, st, (const T *)a, (const T *)b,
                           out, partial, g, d);
    } else {
        dim3 grid((d.Ncols + BN - 1) / BN, (d.M + 127) / 128, splits);
        hipLaunchKernelGGL((igemm_generic_kernel<T, DIR, 128>), grid, block, 0, st, (const T *)a,
                           (const T *)b, out, partial, g, d);
    }
    return hipGetLastError();
}

template <int DIR>
hipError_t launch_any(const void *a, const void *b, void *out, float *partial, const ConvGeom &g,
                      const GemmDims &d, int splits, hipStream_t st)
{
    if (g.in_bf16) return launch_dir<bf16_t, DIR>(a, b, out, partial, g, d, splits, st);
    return launch_dir<float, DIR>(a, b, out, partial, g, d, splits, st);
}

inline int bk_of(const ConvGeom &g) { return g.in_bf16 ? TileCfg<bf16_t>::BK : TileCfg<float>::BK; }

}  // namespace

hipError_t launch_generic_fwd(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    GemmDims d;
    d.M = g.K;
    d.Ncols = g.N * g.P * g.Q;
    d.Kred = g.C * g.R * g.S;
    d.kchunk = (d.Kred + 31) / 32 * 32;
    return launch_any<DIR_FWD>(w, x, y, nullptr, g, d, 1, st);
}

hipError_t launch_generic_bwd_data(const void *dy, const void *w, void *dx, const ConvGeom &g, hipStream_t st)
{
    if (g.sh > 1 || g.sw > 1) {
        if (g.in_bf16) return launch_bwd_data_classes<bf16_t>(dy, w, dx, g, st);
        return launch_bwd_data_classes<float>(dy, w, dx, g, st);
    }
    GemmDims d;
    d.M = g.C;
    d.Ncols = g.N * g.H * g.W;
    d.Kred = g.K * g.R * g.S;
    d.kchunk = (d.Kred + 31) / 32 * 32;
    return launch_any<DIR_BWD_DATA>(w, dy, dx, nullptr, g, d, 1, st);
}

// Slices of the (n,p,q) sum so that a backward-filter launch has enough
// workgroups to fill 256 compute units; each slice keeps at least 8 steps.
int generic_bwd_filter_splits(const ConvGeom &g)
{
    const int M = g.K, Ncols = g.C * g.R * g.S;
    const long long Kred = (long long)g.N * g.P * g.Q;
    const long long tiles = (long long)((M <= 64) ? (M + 63) / 64 : (M + 127) / 128) * ((Ncols + BN - 1) / BN);
    long long want = (1024 + tiles - 1) / tiles;
    long long most = Kred / (8 * bk_of(g));
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 4096) want = 4096;
    return (int)want;
}

hipError_t launch_generic_bwd_filter(const void *x, const void *dy, float *dw, const ConvGeom &g, int splits,
                                     float *partial, bool accumulate, hipStream_t st)
{
    GemmDims d;
    d.M = g.K;
    d.Ncols = g.C * g.R * g.S;
    d.Kred = g.N * g.P * g.Q;
    const int bk = bk_of(g);
    if (splits < 1) splits = 1;
    d.kchunk = ((d.Kred + splits - 1) / splits + bk - 1) / bk * bk;
    splits = (d.Kred + d.kchunk - 1) / d.kchunk;  // drop empty slices
    if (splits > 1 && !partial) {
        hipError_t e = launch_fill_zero(dw, (size_t)d.M * d.Ncols, st);
        if (e != hipSuccess) return e;
    }
    // 1x1 filters: neighbouring columns are different channel planes, and the pixel-per-lane mapping of the
    // general kernel reads them in longer runs (measured 1024 -> 2048 channels, 14x14 / stride 2: 162 against 212 us)
    hipError_t e = g.R * g.S == 1 ? launch_any<DIR_BWD_FILTER>(dy, x, dw, partial, g, d, splits, st)
                   : g.in_bf16    ? launch_bwd_filter_px<bf16_t>(dy, x, dw, partial, g, d, splits, st)
                                  : launch_bwd_filter_px<float>(dy, x, dw, partial, g, d, splits, st);
    if (e != hipSuccess) return e;
    if (partial) return launch_reduce_partials(partial, dw, (size_t)d.M * d.Ncols, splits, accumulate, st);
    return hipSuccess;
}

// A fill kernel rather than a memset node, so the call stays safe to capture
// into a HIP graph.
hipError_t launch_fill_zero(float *p, size_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(fill_zero_kernel, grid, block, 0, st, p, n);
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const float *partial, float *dw, size_t n, int splits, bool accumulate,
                                  hipStream_t st)
{
    if (n % 4 == 0 && reinterpret_cast<uintptr_t>(partial) % 16 == 0 && reinterpret_cast<uintptr_t>(dw) % 16 == 0) {
        const size_t n4 = n / 4;
        const float4 *p4 = reinterpret_cast<const float4 *>(partial);
        float4 *d4 = reinterpret_cast<float4 *>(dw);
        if (splits >= 64)
            hipLaunchKernelGGL(reduce_partials4_kernel<16>, dim3((unsigned)((n4 + 15) / 16)), dim3(256), 0, st, p4, d4,
                               n4, splits, accumulate);
        else
            hipLaunchKernelGGL(reduce_partials4_kernel<4>, dim3((unsigned)((n4 + 63) / 64)), dim3(256), 0, st, p4, d4,
                               n4, splits, accumulate);
        return hipGetLastError();
    }
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(reduce_partials_kernel, grid, block, 0, st, partial, dw, n, splits, accumulate);
    return hipGetLastError();
}

}  // namespace sn
