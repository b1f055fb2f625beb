// gfx950 kernels of libfreqkv.
//
// The whole compression of one span (orthonormal DCT-II, keep Lc coefficients,
// Lc-point inverse, sqrt(Lc/n) rescale: Sec. 3.3 Eq. 2-3 with the Appendix-A
// transforms) is ONE linear map y = M x per channel, with
//     M[m][j] = (1/2n) * ( D(a_m - b_j) + D(a_m + b_j) ),
//     a_m = pi(2m+1)/(2Lc),  b_j = pi(2j+1)/(2n),  D(t) = sin((Lc-1/2)t)/sin(t/2),
// (the two cosine sums collapse to Dirichlet kernels).  M is centro-symmetric,
// M[Lc-1-m][n-1-j] = M[m][j], so for even n and Lc the map splits into two
// half-size maps on the symmetric and antisymmetric parts of x:
//     xe_j = x_j + x_{n-1-j},  xo_j = x_j - x_{n-1-j}           (j < n/2)
//     E = Ge xe,  O = Go xo,   Ge/Go[m][j] = (M[m][j] +/- M[Lc-1-m][j]) / 2   (m < Lc/2)
//     y_m = E_m + O_m,         y_{Lc-1-m} = E_m - O_m
// which halves the multiply-adds.  Ge is, up to a factor, the same operator for the half-size problem
// (the even-indexed coefficients of an n-point DCT are the n/2-point DCT of xe), hence centro-symmetric
// itself: when n/2 is even the even part folds once more,
//     xee_j = xe_j + xe_{n/2-1-j},  xeo_j = xe_j - xe_{n/2-1-j}     (j < n/4)
//     EE = Gee xee,  EO = Geo xeo,  Gee/Geo[m][j] = (Ge[m][j] +/- Ge[Lc/2-1-m][j]) / 2
//     E_m = EE_m + EO_m,  E_{Lc/2-1-m} = EE_m - EO_m                (m < ceil(Lc/4))
// and the multiply-adds drop to 3/8 of the dense count ("two-level" variant: one launch for E into an
// fp16 buffer, one for O that adds and subtracts E on its way into the cache).
// The kernels below build Ge/Go (or M), fold and
// convert the span into an MFMA-ready fp16 workspace, and contract on the matrix
// cores with fp32 accumulation, writing the Lc rows straight into the cache.
#include "freqkv_internal.h"

namespace freqkv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Register
// arrays indexed through it can never fall back to dynamic indexing (and hence to scratch memory).
template <int I> struct IC { static constexpr int value = I; };
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(IC<I>{});
        static_for<N, I + 1>(f);
    }
}

// ------------------------------------------------------------------------------------------
// addressing helpers
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// two floats -> packed bfloat16 pair, round-to-nearest-even (gfx950's v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// ------------------------------------------------------------------------------------------
// basis: fp64 closed form with integer range reduction
// ------------------------------------------------------------------------------------------

// D(theta) for theta = pi*q/(2*n*Lc), i.e. sin(pi*q*(2Lc-1)/Q) / sin(pi*q/Q), Q = 4*n*Lc.
__device__ double dirichlet_q(long long q, long long Q, long long twoLm1)
{
    if (q == 0) return (double)twoLm1;
    long long r = (q % (2 * Q)) * 1;          // |q| < Q already
    long long num = (r * twoLm1) % (2 * Q);   // |r*twoLm1| < 2^63 for spans up to 2^20 rows
    double s_num = sinpi((double)num / (double)Q);
    double s_den = sinpi((double)q / (double)Q);
    return s_num / s_den;
}

// sin(L*theta/2) * cos((L-1)*theta/2 + phi) / sin(theta/2) = sum_{s<L} cos(theta*s + phi), for
// theta = pi*q/(2*n*L) and phi = pi*p2/Q with Q = 4*n*L; |q| < Q, 0 <= p2 < 2Q.
__device__ double shifted_cos_sum(long long q, long long p2, long long Q, long long L)
{
    if (q == 0) return (double)L * cospi((double)p2 / (double)Q);
    long long qq  = ((q % (2 * Q)) + 2 * Q) % (2 * Q);
    long long num = (L * qq) % (2 * Q);
    long long arg = ((L - 1) * qq + p2) % (2 * Q);
    return sinpi((double)num / (double)Q) * cospi((double)arg / (double)Q) / sinpi((double)q / (double)Q);
}

// Entry (t, j) of the orthonormal n-point DCT-II matrix (Appendix A): alpha_t cos(pi t (2j+1) / 2n).
__device__ double dct_entry(long long t, long long j, long long n)
{
    long long q = (t * (2 * j + 1)) % (4 * n);
    double a = t == 0 ? sqrt(1.0 / (double)n) : sqrt(2.0 / (double)n);
    return a * cospi((double)q / (double)(2 * n));
}

// Entry (m, j) of the fused operator.  band 0: the Lc lowest coefficients are kept (Sec. 3.3).
// band 1: the Lc highest are kept and handed, in order, to the Lc-point inverse (the high-frequency
// ablation): M[m][j] = (2/n) * sum_{s<Lc} w_s cos(a_m s) cos(b_j (s + n - Lc)), w_0 = 1/sqrt(2), else 1.
__device__ double operator_entry(int m, int j, long long n, long long Lc, double scale, int band)
{
    long long Q  = 4 * n * Lc;
    long long am = (2LL * m + 1) * n;
    long long bj = (2LL * j + 1) * Lc;
    if (band == 0) {
        double v = dirichlet_q(am - bj, Q, 2 * Lc - 1) + dirichlet_q(am + bj, Q, 2 * Lc - 1);
        return v * scale / (2.0 * (double)n);
    }
    // phi = b_j * (n - Lc) = pi * 2*bj*(n-Lc) / Q, reduced mod 2*pi in integers
    long long p2 = (2 * ((bj % Q) * ((n - Lc) % Q) % Q)) % (2 * Q);
    double v = shifted_cos_sum(bj + am, p2, Q, Lc) + shifted_cos_sum(bj - am, p2, Q, Lc);
    v -= (2.0 - 1.4142135623730951) * cospi((double)p2 / (double)Q);
    return v * scale / (double)n;
}

// G[kg][row][8]: one thread fills one 16-byte group of 8 consecutive k.
__global__ void k_basis_f16(_Float16* __restrict__ G, Geom g, double scale)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)(g.Kpad / 8) * g.Grows;
    if (idx >= total) return;
    int kg  = (int)(idx / g.Grows);
    int row = (int)(idx - (long long)kg * g.Grows);
    int parity = 0, m = row;
    if (g.fold && row >= g.Mpad) { parity = 1; m = row - g.Mpad; }
    half8 out;
    for (int i = 0; i < 8; ++i) {
        int j = kg * 8 + i;
        double v = 0.0;
        if (g.l2 != 0) {
            // two-level fold.  Ge/Go of the full problem (n0 -> Lc0): (M[m][j] +/- M[Lc0-1-m][j]) / 2.
            const int band = g.high;
            auto Ge = [&](int mm, int jj) {
                return 0.5 * (operator_entry(mm, jj, g.n0, g.Lc0, scale, band) +
                              operator_entry(g.Lc0 - 1 - mm, jj, g.n0, g.Lc0, scale, band));
            };
            auto Go = [&](int mm, int jj) {
                return 0.5 * (operator_entry(mm, jj, g.n0, g.Lc0, scale, band) -
                              operator_entry(g.Lc0 - 1 - mm, jj, g.n0, g.Lc0, scale, band));
            };
            const int L2 = g.Lc0 / 2, n2 = g.n0 / 2, n4 = g.n0 / 4;
            if (g.l2 == 1) {            // even part, folded again: rows m < ceil(L2/2), columns j < n/4
                if (m < g.Mh && j < n4) {
                    double a = Ge(m, j), b = Ge(L2 - 1 - m, j);
                    v = parity ? 0.5 * (a - b) : 0.5 * (a + b);
                }
            } else {                    // odd part, plain; columns in the order the span is laid out:
                                        // positions [0, H) hold j, positions [H, 2H) hold n/2-1-j  (j < n/4)
                if (m < L2) {
                    int jo = -1;
                    if (j < g.H) { if (j < n4) jo = j; }
                    else if (j - g.H < n4) jo = n2 - 1 - (j - g.H);
                    if (jo >= 0) v = Go(m, jo);
                }
            }
        } else if (m < g.Mh && j < g.Kh && g.high == 2) {
            // forward transform only (power spectrum): the even-indexed rows act on the symmetric part of
            // the span and the odd-indexed rows on the antisymmetric part, so the fold needs no mixing
            v = dct_entry(g.fold ? 2 * m + parity : m, j, g.n);
        } else if (m < g.Mh && j < g.Kh) {
            double a = operator_entry(m, j, g.n, g.Lc, scale, g.high);
            if (g.fold) {
                double b = operator_entry(g.Lc - 1 - m, j, g.n, g.Lc, scale, g.high);
                v = parity ? 0.5 * (a - b) : 0.5 * (a + b);
            } else {
                v = a;
            }
        }
        out[i] = (_Float16)v;
    }
    *(half8*)(G + idx * 8) = out;
}

__global__ void k_basis_f32(float* __restrict__ Mf, int n, int Lc, double scale, int band)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)n * Lc) return;
    int m = (int)(idx / n), j = (int)(idx - (long long)m * n);
    Mf[idx] = (float)operator_entry(m, j, n, Lc, scale, band);
}

hipError_t launch_basis_f16(_Float16* G, const Geom& g, int rescale, hipStream_t st)
{
    double scale = rescale ? 1.0 : sqrt((double)g.n / (double)g.Lc);
    long long total = (long long)(g.Kpad / 8) * g.Grows;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(k_basis_f16, dim3(blocks), dim3(256), 0, st, G, g, scale);
    return hipGetLastError();
}

hipError_t launch_basis_f32(float* Mf, int n, int Lc, int rescale, int band, hipStream_t st)
{
    double scale = rescale ? 1.0 : sqrt((double)n / (double)Lc);
    long long total = (long long)n * Lc;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(k_basis_f32, dim3(blocks), dim3(256), 0, st, Mf, n, Lc, scale, band);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// prepare (bf16 cache): fold + convert the span into the MFMA-ready workspace
//
// Workspace layout, in 16-byte groups of 8 consecutive k (fp16):
//     ws[coltile][kstage][parity][kgroup 0..3][column 0..127][8]
// so one pipeline stage of one column tile is P*8 KiB of contiguous memory, already in
// the order the contraction's LDS fragments are read.
// ------------------------------------------------------------------------------------------

// Largest magnitude of the span of every head-tensor (range guard of the fp16 operands).  A lane reads 16 bytes
// (8 channels) of a row, 16 lanes a 256-byte stretch of it, so a wave scans 4 rows of a 128-column tile per step;
// bf16 bit patterns without their sign compare like the magnitudes.  hmax must be zero before the launch.
__global__ __launch_bounds__(256) void k_absmax_bf16(SlabTable tab, Geom g, uint32_t* __restrict__ hmax)
{
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    const int ct = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int vcol = ct * kColTile + (lane & 15) * 8;
    if (vcol >= g.ncols) return;
    int ht;
    const char* base = column_base(tab, g, vcol, 2, &ht);
    const long long rowb = g.stride_token * 2;
    u16x2 m = {0, 0};
    for (int j = (blockIdx.y * 4 + wave) * 4 + (lane >> 4); j < g.n0; j += 16 * gridDim.y) {
        const u32x4 w = *(const u32x4*)(base + (long long)(g.S + j) * rowb);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t wi = w[i] & 0x7fff7fffu;
            m = __builtin_elementwise_max(m, __builtin_bit_cast(u16x2, wi));
        }
    }
    uint32_t a = m[0] > m[1] ? m[0] : m[1];
    if (g.d % kColTile == 0) {
        // the 128 columns of the wave belong to one head-tensor
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)a, off);
            a = o > a ? o : a;
        }
        if (lane == 0) atomicMax(hmax + ht, a);
    } else {
        atomicMax(hmax + ht, a);
    }
}

hipError_t launch_absmax_bf16(const SlabTable& tab, const Geom& g, uint32_t* hmax, hipStream_t st)
{
    // g.n0: rows of the span (set by the caller for every variant)
    dim3 grid(g.ncoltiles, 16);
    hipLaunchKernelGGL(k_absmax_bf16, grid, dim3(256), 0, st, tab, g, hmax);
    return hipGetLastError();
}

// F32: the cache holds float32 (the power-spectrum diagnostic of fp32 caches; compression of fp32 caches has
// its own fp32 path), else bfloat16.
template <bool FOLD, bool F32>
__global__ __launch_bounds__(256) void k_prepare_bf16(SlabTable tab, Geom g, _Float16* __restrict__ ws)
{
    constexpr int P = FOLD ? 2 : 1;
    constexpr int EB = F32 ? 4 : 2;               // bytes per cache element
    const int ct   = blockIdx.x;
    const int ks   = blockIdx.y;
    const int kg   = threadIdx.x >> 6;        // one wave per group of 8 k
    const int lane = threadIdx.x & 63;
    const int col  = lane * 2;                // two adjacent channels per lane
    const int vcol = ct * kColTile + col;
    const int j0   = (ks * 4 + kg) * 8;

    float a0v[8], a1v[8], b0v[8], b1v[8];
    const bool colok = vcol < g.ncols;
    int ht = 0;
    const char* base = colok ? column_base(tab, g, vcol, EB, &ht) : nullptr;
    const float sc = (colok && g.hmax) ? pow2f(guard_exponent(g.hmax[ht])) : 1.0f;
    const long long rowb = g.stride_token * EB;   // bytes per token row
    auto load2 = [&](long long row, float* x0, float* x1) {
        if constexpr (F32) {
            const f32x2 v = *(const f32x2*)(base + row * rowb);
            *x0 = v[0]; *x1 = v[1];
        } else {
            const uint32_t w = *(const uint32_t*)(base + row * rowb);
            *x0 = bf16_to_f32(w & 0xffffu); *x1 = bf16_to_f32(w >> 16);
        }
    };
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int j = j0 + i;
        bool ok = colok && j < g.Kh;
        a0v[i] = a1v[i] = b0v[i] = b1v[i] = 0.f;
        if (ok) load2(g.S + j, &a0v[i], &a1v[i]);
        if (FOLD && ok) load2(g.S + g.n - 1 - j, &b0v[i], &b1v[i]);
    }
    half8 e0, e1, o0, o1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float a0 = a0v[i] * sc, a1 = a1v[i] * sc;
        if (FOLD) {
            float b0 = b0v[i] * sc, b1 = b1v[i] * sc;
            e0[i] = (_Float16)(a0 + b0); e1[i] = (_Float16)(a1 + b1);
            o0[i] = (_Float16)(a0 - b0); o1[i] = (_Float16)(a1 - b1);
        } else {
            e0[i] = (_Float16)a0; e1[i] = (_Float16)a1;
        }
    }
    // 16-byte group index of (parity 0, kg, col)
    size_t stage = ((size_t)ct * g.nkstages + ks) * P;
    size_t ge = ((stage + 0) * 4 + kg) * kColTile + col;
    half8* w = (half8*)ws;
    w[ge] = e0; w[ge + 1] = e1;
    if (FOLD) {
        size_t go = ((stage + 1) * 4 + kg) * kColTile + col;
        w[go] = o0; w[go + 1] = o1;
    }
}

// Two-level fold: one thread takes 8 quarter positions j of 2 adjacent channels, reads the four rows
// j, n/2-1-j, n/2+j, n-1-j and writes
//   wsA (folded layout, stage ks): parity 0  xee_j = x_j + x_{n/2-1-j} + x_{n/2+j} + x_{n-1-j}
//                                  parity 1  xeo_j = x_j - x_{n/2-1-j} - x_{n/2+j} + x_{n-1-j}
//   wsB (plain layout): stage ks          xo_j         = x_j - x_{n-1-j}
//                       stage nksA + ks   xo_{n/2-1-j} = x_{n/2-1-j} - x_{n/2+j}
// g: the geometry of the even-part launch (Kh = n/4, nkstages = nksA).
__global__ __launch_bounds__(256) void k_prepare_bf16_l2(SlabTable tab, Geom g, _Float16* __restrict__ wsA,
                                                         _Float16* __restrict__ wsB)
{
    const int ct   = blockIdx.x;
    const int ks   = blockIdx.y;
    const int kg   = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int col  = lane * 2;
    const int vcol = ct * kColTile + col;
    const int j0   = (ks * 4 + kg) * 8;
    const int n = g.n0, n2 = n / 2, n4 = n / 4;

    const bool colok = vcol < g.ncols;
    int ht = 0;
    const char* base = colok ? column_base(tab, g, vcol, 2, &ht) : nullptr;
    const float sc = (colok && g.hmax) ? pow2f(guard_exponent(g.hmax[ht])) : 1.0f;
    const long long rowb = g.stride_token * 2;
    half8 ee0, ee1, eo0, eo1, od0, od1, om0, om1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int j = j0 + i;
        const bool ok = colok && j < n4;
        uint32_t a = 0u, b = 0u, c = 0u, d = 0u;
        if (ok) {
            a = *(const uint32_t*)(base + (long long)(g.S + j) * rowb);
            b = *(const uint32_t*)(base + (long long)(g.S + n2 - 1 - j) * rowb);
            c = *(const uint32_t*)(base + (long long)(g.S + n2 + j) * rowb);
            d = *(const uint32_t*)(base + (long long)(g.S + n - 1 - j) * rowb);
        }
        const float a0 = bf16_to_f32(a & 0xffffu) * sc, a1 = bf16_to_f32(a >> 16) * sc;
        const float b0 = bf16_to_f32(b & 0xffffu) * sc, b1 = bf16_to_f32(b >> 16) * sc;
        const float c0 = bf16_to_f32(c & 0xffffu) * sc, c1 = bf16_to_f32(c >> 16) * sc;
        const float d0 = bf16_to_f32(d & 0xffffu) * sc, d1 = bf16_to_f32(d >> 16) * sc;
        ee0[i] = (_Float16)((a0 + d0) + (b0 + c0)); ee1[i] = (_Float16)((a1 + d1) + (b1 + c1));
        eo0[i] = (_Float16)((a0 + d0) - (b0 + c0)); eo1[i] = (_Float16)((a1 + d1) - (b1 + c1));
        od0[i] = (_Float16)(a0 - d0);               od1[i] = (_Float16)(a1 - d1);
        om0[i] = (_Float16)(b0 - c0);               om1[i] = (_Float16)(b1 - c1);
    }
    half8* wa = (half8*)wsA;
    half8* wb = (half8*)wsB;
    const size_t stA = ((size_t)ct * g.nkstages + ks) * 2;
    const size_t ge = ((stA + 0) * 4 + kg) * kColTile + col;
    const size_t go = ((stA + 1) * 4 + kg) * kColTile + col;
    wa[ge] = ee0; wa[ge + 1] = ee1;
    wa[go] = eo0; wa[go + 1] = eo1;
    const size_t sd = (((size_t)ct * (2 * g.nkstages) + ks) * 4 + kg) * kColTile + col;
    const size_t sm = (((size_t)ct * (2 * g.nkstages) + g.nkstages + ks) * 4 + kg) * kColTile + col;
    wb[sd] = od0; wb[sd + 1] = od1;
    wb[sm] = om0; wb[sm + 1] = om1;
}

hipError_t launch_prepare_bf16_l2(const SlabTable& tab, const Geom& gA, _Float16* wsA, _Float16* wsB, hipStream_t st)
{
    if (gA.l2 != 1 || !gA.fold || gA.n0 % 4) return hipErrorInvalidValue;
    dim3 grid(gA.ncoltiles, gA.nkstages);
    hipLaunchKernelGGL(k_prepare_bf16_l2, grid, dim3(256), 0, st, tab, gA, wsA, wsB);
    return hipGetLastError();
}

hipError_t launch_prepare_bf16(const SlabTable& tab, const Geom& g, _Float16* ws, hipStream_t st, int elem_bytes)
{
    dim3 grid(g.ncoltiles, g.nkstages);
    if (elem_bytes == 4) {
        if (g.fold) hipLaunchKernelGGL((k_prepare_bf16<true, true>),  grid, dim3(256), 0, st, tab, g, ws);
        else        hipLaunchKernelGGL((k_prepare_bf16<false, true>), grid, dim3(256), 0, st, tab, g, ws);
    } else {
        if (g.fold) hipLaunchKernelGGL((k_prepare_bf16<true, false>),  grid, dim3(256), 0, st, tab, g, ws);
        else        hipLaunchKernelGGL((k_prepare_bf16<false, false>), grid, dim3(256), 0, st, tab, g, ws);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// contraction on the matrix cores
//
// Workgroup = 4 waves, each wave owns a 128(row) x 128(column) fp32 accumulator tile
// (4x4 blocks of v_mfma_f32_32x32x16_f16).  Folded: waves are (parity, row half) of a
// 256-row-per-parity tile.  Plain: waves are the four 128-row quarters of a 512-row tile.
//   - operand A (basis) is private to a wave: loaded global -> registers, already in
//     fragment order ([kgroup][row][8]: lane L takes row L%32, k group L/32);
//   - operand B (folded span) is shared by the waves: one contiguous stage of the workspace
//     is copied global -> LDS directly (a ring of four slots) and read back as 16-byte fragments
//     (lane L: column L%32, k group L/32), conflict-free.
// ------------------------------------------------------------------------------------------

// Workgroup barrier that orders LDS traffic only (waits lgkmcnt, not vmcnt): __syncthreads() would
// also drain every outstanding global load and with it the register prefetch of the next stage.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// MODE 0: rows into the cache (and the optional fp32 tap).
// MODE 1 (spectrum): add the squared results, summed over the 8 channels of an item and scaled by
//         g.spec_scale, to the spectrum line of the item's head: tap[(slab, head)][coefficient].
// MODE 2 (even part of the two-level fold): results only into tap, which is then the fp16 buffer
//         E[head-tensor][Lc][d] of this (half-size) problem; the cache is not written.
// MODE 3 (odd part of the two-level fold, plain operator): row m of the result is O_m; with E_m from
//         g.ebuf, cache row m gets E+O and row Lc0-1-m gets E-O (tap likewise, full-size layout).
template <bool FOLD, int NW, int MODE>
__global__ __launch_bounds__(NW * 64, 1) void k_contract_f16(SlabTable tab, Geom g,
                                                         const _Float16* __restrict__ G,
                                                         const _Float16* __restrict__ ws,
                                                         float* __restrict__ tap)
{
    constexpr int P = FOLD ? 2 : 1;
    constexpr int XSTAGE = P * 8192;                       // bytes per pipeline stage
    constexpr int NT = NW * 64;                            // threads
    constexpr int WPP = FOLD ? NW / 2 : NW;                // waves per parity
    constexpr int WROWS = (FOLD ? kRowsFold : kRowsPlain) / WPP;   // rows per wave
    constexpr int MBN = WROWS / 32;                        // 32-row accumulator blocks per wave
    constexpr int LDS_BYTES = NW * 16384;                  // pipeline: 4 slots of XSTAGE; epilogue: NW x 16 KiB
    __shared__ __attribute__((aligned(1024))) char smem[LDS_BYTES];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, lhi = lane >> 5;

    // blockIdx -> (column tile, row tile).  Workgroups are dealt round-robin to the 8 XCDs, so
    // within a group of 8 column tiles the XCD index picks the column tile and consecutive slots
    // on one XCD are the row tiles of the same columns: they share that XCD's L2 for the span.
    int ct, mt;
    {
        const int bid = blockIdx.x;
        const int per_group = 8 * g.nmtiles;
        const int full = g.ncoltiles / 8;
        const int grp = bid / per_group;
        if (grp < full) {
            int local = bid - grp * per_group;
            ct = grp * 8 + (local & 7);
            mt = local >> 3;
        } else {
            int rem = g.ncoltiles - full * 8;
            int local = bid - full * per_group;
            ct = full * 8 + local % rem;
            mt = local / rem;
        }
    }

    const int par  = FOLD ? (wave / WPP) : 0;
    const int rsub = FOLD ? (wave % WPP) : wave;
    // first basis row of this wave in G's row order
    const int grow0 = FOLD ? (par * g.Mpad + mt * kRowsFold + rsub * WROWS)
                           : (mt * kRowsPlain + wave * WROWS);

    f32x16 acc[MBN][4];
#pragma unroll
    for (int i = 0; i < MBN; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nks = g.nkstages;
    const char* xsrc = (const char*)ws + (size_t)ct * nks * XSTAGE;
    const half8* Gv = (const half8*)G;
    // lane's 16-byte group in G for (stage s, substep u, row block mb): ((s*4 + u*2 + lhi) * Grows + grow0 + mb*32 + l32)
    const size_t a_lane = (size_t)lhi * g.Grows + grow0 + l32;
    const size_t a_kstep = (size_t)2 * g.Grows;     // one 16-k substep
    const size_t a_stage = (size_t)4 * g.Grows;

    // Software pipeline over the K stages (32 contraction rows each).  Global traffic runs three stages ahead of
    // the matrix cores so that an L2 miss (the span and the basis stream from HBM / the Infinity Cache) has two
    // stages of MFMA work to arrive:
    //   step s:  issue  span(s+3)  -> LDS slot (s+3)%4       (global -> LDS directly, no registers)
    //            issue  basis(s+3) -> aset[(s+3)%4]          (global -> registers)
    //            read   span(s+1)  LDS slot (s+1)%4 -> xf[(s+1)%2]
    //            MFMA   stage s    (aset[s%4], xf[s%2])
    //            wait until span(s+2) has landed, barrier
    // Register buffers rotate with periods 4 and 2, so the loop body is four steps long.  Nothing in a step is
    // conditional: near the end the stage indices are clamped (the last stage is requested again, into slots
    // and registers nobody reads), so that every step is the same straight-line code and the loads in flight
    // can be counted exactly; with guarded loads the compiler made each group of matrix instructions wait for
    // loads issued in the same step.
    constexpr int XR = XSTAGE / (NT * 16);  // 16-byte pieces per thread per stage
    constexpr int XPIECE = NT * 16;         // bytes the workgroup moves per piece
    static_assert(4 * XSTAGE <= LDS_BYTES, "four span stages in LDS");
    half8 aset[4][2][MBN];                  // basis fragments [buffer][16-k substep][row block]
    half8 xf[2][2][4];                      // span fragments  [buffer][16-k substep][column block]
    const int tid16 = threadIdx.x * 16;

    auto load_a = [&](int st, auto buf) {
        const half8* pa = Gv + a_lane + (size_t)st * a_stage;
        static_for<2>([&](auto u) {
            static_for<MBN>([&](auto mb) { aset[buf.value][u.value][mb.value] = pa[u.value * a_kstep + mb.value * 32]; });
        });
    };
    // Direct global -> LDS copy of one span stage: lane i of a wave delivers its 16 bytes to M0 + 16 i, so a
    // piece of XPIECE bytes arrives in the order it has in the workspace.  Written as assembly because the
    // compiler, which cannot tell the ring slots apart, would wait for a copy issued through its builtin in
    // front of the next LDS read; it does not count these copies, so the waits for them are placed by hand and
    // its own waits for the basis loads are at worst early.  M0 has no other user in this kernel.
    const uint32_t lds_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem +
                              __builtin_amdgcn_readfirstlane(wave) * 1024;
    auto dma_x = [&](int st) {
        const char* src = xsrc + (size_t)st * XSTAGE + tid16;
        const uint32_t dst = lds_wave + (st & 3) * XSTAGE;
        static_for<XR>([&](auto r) {
            lds_dma16(dst + r.value * XPIECE, src + r.value * XPIECE);
        });
    };
    auto read_xf = [&](int st, auto buf) {
        const char* xs = smem + (st & 3) * XSTAGE + par * 8192;
        static_for<2>([&](auto u) {
            static_for<4>([&](auto nb) {
                xf[buf.value][u.value][nb.value] =
                    *(const half8*)(xs + (((u.value * 2 + lhi) * kColTile) + nb.value * 32 + l32) * 16);
            });
        });
    };
    // One step at phase PH = s mod 4.  The 32 MFMAs run as 8 groups of 4 (one basis fragment against the 4
    // column blocks); the step's 8 basis loads and 8 LDS fragment reads are dealt out between the groups, so
    // the vector-memory and LDS queues drain while the matrix cores work instead of blocking the wave in one
    // burst at the top of the step.
    auto step = [&](int st, auto ph) {
        constexpr int PH = decltype(ph)::value;
        constexpr int A0 = PH % 4, A3 = (PH + 3) % 4, X0 = PH % 2, X1 = (PH + 1) % 2;
        const int ahead = min(st + 3, nks - 1);
        dma_x(ahead);
        const half8* pa = Gv + a_lane + (size_t)ahead * a_stage;
        const char* xs = smem + ((st + 1) & 3) * XSTAGE + par * 8192;
        constexpr int NG = 2 * MBN;             // MFMA groups per step: (substep u, row block mb)
        constexpr int RPG = 8 / NG;             // LDS fragment reads per group
        static_for<NG>([&](auto gi) {
            constexpr int G = decltype(gi)::value;
            constexpr int U = G / MBN, MB = G % MBN;
            aset[A3][U][MB] = pa[U * a_kstep + MB * 32];         // basis fragment G of stage s+3
            static_for<RPG>([&](auto ri) {                         // fragments of stage s+1
                constexpr int F = G * RPG + decltype(ri)::value, FU = F / 4, FN = F % 4;
                xf[X1][FU][FN] = *(const half8*)(xs + (((FU * 2 + lhi) * kColTile) + FN * 32 + l32) * 16);
            });
            static_for<4>([&](auto nb) {
                acc[MB][nb.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    aset[A0][U][MB], xf[X0][U][nb.value], acc[MB][nb.value], 0, 0, 0);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        // span(s+2) was requested one step ago; younger than it are that step's NG basis loads and this step's
        // XR copies and NG basis loads
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * NG + XR) : "memory");
        lds_barrier();
    };

    // prologue: span stages 0..2 -> LDS, basis stages 0..2 in flight
    {
        dma_x(0);
        load_a(0, IC<0>{});
        dma_x(min(1, nks - 1) == 1 ? 1 : 0);
        load_a(min(1, nks - 1), IC<1>{});
        if (nks > 2) dma_x(2);
        load_a(min(2, nks - 1), IC<2>{});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        read_xf(0, IC<0>{});
    }

    int st = 0;
    for (; st + 4 <= nks; st += 4) {
        step(st + 0, IC<0>{});
        step(st + 1, IC<1>{});
        step(st + 2, IC<2>{});
        step(st + 3, IC<3>{});
    }
    // tail: at most three steps, same rotation (st is a multiple of 4 here)
    static_for<3>([&](auto i) {
        if (st + i.value < nks) step(st + i.value, i);
    });
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may land in LDS once the epilogue owns it
    __syncthreads();      // every wave is done with the LDS slots before the epilogue reuses them

    // ---- epilogue ------------------------------------------------------------------------
    // Accumulator layout of a 32x32 block: register r of lane L is row 8*(r/4) + 4*(L/32) + r%4,
    // column L%32.  Each wave parks one 32-row block at a time in LDS as fp32 [32][128]; the
    // workgroup then reads it back row-major, 8 channels per lane, so that every cache row is
    // written with 16-byte stores (a full 256-byte row per 16 lanes).  In the folded variant this
    // pass also pairs the even part E (parity-0 wave) with the odd part O (parity-1 wave):
    // row m gets E+O and row Lc-1-m gets E-O.
    float* T = (float*)smem;                       // [NW waves][32 rows][128 cols]
    const long long rowb = g.stride_token * 2;
    constexpr int ITEMS = WPP * 32 * 16;           // (wave pair | wave, row, 8-column group)
    static_assert(NT % 16 == 0 && ITEMS % NT == 0, "a thread keeps one 8-column group for all its items");
    // the thread's 8-column group is the same for all of its items: resolve its head-tensor once
    const int cg = threadIdx.x & 15;
    const int vcol = ct * kColTile + cg * 8;
    const bool col_ok = vcol < g.ncols;
    char* base = nullptr;
    float* tp = nullptr;
    const _Float16* ep = nullptr;   // MODE 3: the even part of this thread's columns (fp16 buffer)
    _Float16* hp = nullptr;         // MODE 2: where this thread's columns of the even part go
    float unsc = 1.0f;              // undoes the power-of-two scale of the span (not for the fp16 even part,
                                    // which stays in the scaled domain until the odd part is combined with it)
    if (col_ok) {
        int ht;
        base = column_base(tab, g, vcol, 2, &ht);
        const int c = vcol - ht * g.d;
        if (g.hmax && MODE != 2) unsc = pow2f(-guard_exponent(g.hmax[ht]));
        if constexpr (MODE == 1) {
            const int slab = ht / g.hts_per_slab;
            const int h = (ht - slab * g.hts_per_slab) % g.n_heads;
            tp = tap + ((g.tap_slab0 + slab) * (long long)g.n_heads + h) * g.Lc;
        } else if constexpr (MODE == 3) {
            if (tap) tp = tap + ((g.tap_slab0 * g.hts_per_slab + ht) * (long long)g.Lc0) * g.d + c;
            ep = g.ebuf + ((long long)ht * g.Lc) * g.d + c;          // the buffer belongs to this pass alone
        } else if constexpr (MODE == 2) {
            hp = (_Float16*)tap + ((long long)ht * g.Lc) * g.d + c;
        } else {
            if (tap) tp = tap + ((g.tap_slab0 * g.hts_per_slab + ht) * (long long)g.Lc) * g.d + c;
        }
    }
    // MODE 3: the even-part rows this thread will need, fetched one round of 32-row blocks ahead so that the
    // global-load latency hides behind the LDS traffic of the round before (the operand registers of the main
    // loop are free by now).
    constexpr int NIT = ITEMS / NT;
    half8 epre[2][MODE == 3 ? NIT : 1];
    auto fetch_even = [&](auto mbf, auto buf) {
        if constexpr (MODE == 3) {
            static_for<NIT>([&](auto itc) {
                const int item = threadIdx.x + itc.value * NT;
                const int row_a = mt * kRowsPlain + (item >> 9) * WROWS + mbf.value * 32 + ((item >> 4) & 31);
                epre[buf.value][itc.value] = (col_ok && row_a < g.Mh) ? *(const half8*)(ep + (long long)row_a * g.d)
                                                                      : half8{};
            });
        }
    };
    fetch_even(IC<0>{}, IC<0>{});
    static_for<MBN>([&](auto mbc) {
        constexpr int MB = decltype(mbc)::value;
        static_for<4>([&](auto nb) {
            static_for<16>([&](auto r) {
                const int row = (r.value >> 2) * 8 + lhi * 4 + (r.value & 3);
                T[(wave * 32 + row) * 128 + nb.value * 32 + l32] = acc[MB][nb.value][r.value];
            });
        });
        if constexpr (MB + 1 < MBN) fetch_even(IC<MB + 1>{}, IC<(MB + 1) & 1>{});
        __syncthreads();
        static_for<NIT>([&](auto itc) {
            constexpr int it = decltype(itc)::value;
            const int item = threadIdx.x + it * NT;
            const int row = (item >> 4) & 31, w = item >> 9;
            if constexpr (MODE == 1) {
                // Power spectrum: squares of the item's 8 channels; E is coefficient 2*rh and O coefficient
                // 2*rh+1 (folded), or the row itself (plain).  No lane leaves early, so the 16 lanes that
                // hold one row can be summed with lane exchanges when they all belong to one head
                // (head_dim a multiple of 128); otherwise every lane adds its own share.
                const int rh = mt * (FOLD ? kRowsFold : kRowsPlain) + w * WROWS + MB * 32 + row;
                const bool ok = col_ok && rh < g.Mh;
                const float* e = T + (((FOLD ? 0 * WPP : 0) + w) * 32 + row) * 128 + cg * 8;
                const float* o = T + ((1 * WPP + w) * 32 + row) * 128 + cg * 8;
                float pe = 0.f, po = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    pe = fmaf(e[i], e[i], pe);
                    if constexpr (FOLD) po = fmaf(o[i], o[i], po);
                }
                pe = ok ? pe * g.spec_scale : 0.f;
                po = ok ? po * g.spec_scale : 0.f;
                bool lead = true;
                if (g.d % 128 == 0) {
                    for (int sft = 1; sft < 16; sft <<= 1) {
                        pe += __shfl_xor(pe, sft);
                        if constexpr (FOLD) po += __shfl_xor(po, sft);
                    }
                    lead = cg == 0;
                }
                if (ok && lead) {
                    if constexpr (FOLD) {
                        atomicAdd(tp + 2 * rh, pe);
                        atomicAdd(tp + 2 * rh + 1, po);
                    } else {
                        atomicAdd(tp + rh, pe);
                    }
                }
                return;
            }
            if (!col_ok) return;
            float va[8], vb[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            int row_a, row_b = -1;
            if constexpr (FOLD) {
                // w = row sub-tile; E from wave (parity 0, w), O from wave (parity 1, w)
                const float* e = T + ((0 * WPP + w) * 32 + row) * 128 + cg * 8;
                const float* o = T + ((1 * WPP + w) * 32 + row) * 128 + cg * 8;
#pragma unroll
                for (int i = 0; i < 8; ++i) { va[i] = e[i] + o[i]; vb[i] = e[i] - o[i]; }
                const int rh = mt * kRowsFold + w * WROWS + MB * 32 + row;
                if (rh >= g.Mh) return;
                row_a = rh;
                row_b = g.Lc - 1 - rh;
            } else {
                const float* e = T + (w * 32 + row) * 128 + cg * 8;
#pragma unroll
                for (int i = 0; i < 8; ++i) va[i] = e[i];
                row_a = mt * kRowsPlain + w * WROWS + MB * 32 + row;
                if (row_a >= g.Mh) return;
            }
            if constexpr (MODE == 2) {
                // even part of the two-level fold: rows of E only, as fp16 (four times finer than the bf16
                // grid of the rows they end up in; halves the round trip through HBM)
                half8 ha, hb;
#pragma unroll
                for (int i = 0; i < 8; ++i) { ha[i] = (_Float16)va[i]; hb[i] = (_Float16)vb[i]; }
                *(half8*)(hp + (long long)row_a * g.d) = ha;
                if constexpr (FOLD) *(half8*)(hp + (long long)row_b * g.d) = hb;
                return;
            }
            if constexpr (MODE == 3) {
                // va = O_m; y_m = E_m + O_m, y_{Lc0-1-m} = E_m - O_m
                row_b = g.Lc0 - 1 - row_a;
                const half8 eh = epre[MB & 1][it];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float e = (float)eh[i];
                    vb[i] = e - va[i];
                    va[i] = e + va[i];
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) { va[i] *= unsc; vb[i] *= unsc; }
            u32x4 pk;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                pk[i] = pack_bf16x2(va[2 * i], va[2 * i + 1]);
            *(u32x4*)(base + (long long)(g.S + row_a) * rowb) = pk;
            if (tp) {
#pragma unroll
                for (int i = 0; i < 8; ++i) tp[(long long)row_a * g.d + i] = va[i];
            }
            if (FOLD || MODE == 3) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    pk[i] = pack_bf16x2(vb[2 * i], vb[2 * i + 1]);
                *(u32x4*)(base + (long long)(g.S + row_b) * rowb) = pk;
                if (tp) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) tp[(long long)row_b * g.d + i] = vb[i];
                }
            }
        });
        __syncthreads();
    });
}

__global__ void k_fill_zero(float* __restrict__ p, size_t count)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

hipError_t launch_fill_zero(float* p, size_t count, hipStream_t st)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, p, count);
    return hipGetLastError();
}

hipError_t launch_contract_f16(const SlabTable& tab, const Geom& g, const _Float16* G,
                               const _Float16* ws, float* tap, int mode, hipStream_t st)
{
    dim3 grid((unsigned)g.ncoltiles * (unsigned)g.nmtiles);
    // Four waves (one per SIMD, 128x128 accumulators each).  Eight waves of 64x128 are correct too but
    // measured 2.99 ms against 2.16 ms on the 8188 -> 4094 trigger: twice the LDS fragment traffic.
    constexpr int NW = 4;
    const dim3 block(NW * 64);
    switch (mode) {
        case 0:
            if (g.fold) hipLaunchKernelGGL((k_contract_f16<true, NW, 0>),  grid, block, 0, st, tab, g, G, ws, tap);
            else        hipLaunchKernelGGL((k_contract_f16<false, NW, 0>), grid, block, 0, st, tab, g, G, ws, tap);
            break;
        case 1:
            if (!tap) return hipErrorInvalidValue;
            if (g.fold) hipLaunchKernelGGL((k_contract_f16<true, NW, 1>),  grid, block, 0, st, tab, g, G, ws, tap);
            else        hipLaunchKernelGGL((k_contract_f16<false, NW, 1>), grid, block, 0, st, tab, g, G, ws, tap);
            break;
        case 2:
            if (!tap || !g.fold) return hipErrorInvalidValue;
            hipLaunchKernelGGL((k_contract_f16<true, NW, 2>), grid, block, 0, st, tab, g, G, ws, tap);
            break;
        case 3:
            if (!g.ebuf || g.fold || (g.d % 8)) return hipErrorInvalidValue;
            hipLaunchKernelGGL((k_contract_f16<false, NW, 3>), grid, block, 0, st, tab, g, G, ws, tap);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// fp32 cache: copy the span out, then a plain LDS-tiled fp32 FMA contraction y = Mf * x
// workspace: xs[n][ncolsf] fp32, ncolsf = ncols rounded up to 64 (pad columns are zero)
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ int f32_cols_padded(const Geom& g) { return (g.ncols + 63) & ~63; }

__global__ __launch_bounds__(256) void k_prepare_f32(SlabTable tab, Geom g, float* __restrict__ ws)
{
    const int ncp = f32_cols_padded(g);
    const int vcol = blockIdx.x * 256 + threadIdx.x;
    if (vcol >= ncp) return;
    const char* base = vcol < g.ncols ? column_base(tab, g, vcol, 4, nullptr) : nullptr;
    for (int j = blockIdx.y; j < g.n; j += gridDim.y) {
        float v = base ? *(const float*)(base + (long long)(g.S + j) * g.stride_token * 4) : 0.f;
        ws[(size_t)j * ncp + vcol] = v;
    }
}

__global__ __launch_bounds__(256) void k_contract_f32(SlabTable tab, Geom g, const float* __restrict__ Mf,
                                                      const float* __restrict__ ws, float* __restrict__ tap)
{
    __shared__ float As[16][65];   // [k][m]
    __shared__ float Bs[16][64];   // [k][col]
    const int ncp = f32_cols_padded(g);
    const int c0 = blockIdx.x * 64, m0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.n; k0 += 16) {
        for (int e = threadIdx.x; e < 64 * 16; e += 256) {
            int mm = e >> 4, kk = e & 15;
            int m = m0 + mm, j = k0 + kk;
            As[kk][mm] = (m < g.Lc && j < g.n) ? Mf[(size_t)m * g.n + j] : 0.f;
        }
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            int kk = e >> 6, cc = e & 63;
            int j = k0 + kk;
            Bs[kk][cc] = (j < g.n) ? ws[(size_t)j * ncp + c0 + cc] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int i = 0; i < 4; ++i) b[i] = Bs[kk][tx * 4 + i];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[i][q] = fmaf(a[i], b[q], acc[i][q]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int vcol = c0 + tx * 4 + q;
        if (vcol >= g.ncols) continue;
        int ht;
        char* base = column_base(tab, g, vcol, 4, &ht);
        int c = vcol - ht * g.d;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int m = m0 + ty * 4 + i;
            if (m >= g.Lc) continue;
            *(float*)(base + (long long)(g.S + m) * g.stride_token * 4) = acc[i][q];
            if (tap) {
                long long ht_global = g.tap_slab0 * g.hts_per_slab + ht;
                tap[(ht_global * g.Lc + m) * g.d + c] = acc[i][q];
            }
        }
    }
}

hipError_t launch_prepare_f32(const SlabTable& tab, const Geom& g, float* ws, hipStream_t st)
{
    int ncp = (g.ncols + 63) & ~63;
    dim3 grid((ncp + 255) / 256, g.n < 65535 ? g.n : 65535);
    hipLaunchKernelGGL(k_prepare_f32, grid, dim3(256), 0, st, tab, g, ws);
    return hipGetLastError();
}

hipError_t launch_contract_f32(const SlabTable& tab, const Geom& g, const float* Mf, const float* ws,
                               float* tap, hipStream_t st)
{
    int ncp = (g.ncols + 63) & ~63;
    dim3 grid(ncp / 64, (g.Lc + 63) / 64);
    hipLaunchKernelGGL(k_contract_f32, grid, dim3(256), 0, st, tab, g, Mf, ws, tap);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// tail move: rows [src, src+rows) -> [dst, dst+rows), 16 bytes per lane; ranges are disjoint
// ------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_move_rows(SlabTable tab, Geom g, int elem_bytes, int src_row,
                                                   int dst_row, int per16)
{
    // per16 = elements per 16-byte group (8 for bf16, 4 for fp32); d is a multiple of 8
    const long long grp = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long ngroups = (long long)g.ncols / per16;
    if (grp >= ngroups) return;
    const int row = blockIdx.y;
    const int vcol = (int)(grp * per16);
    char* base = column_base(tab, g, vcol, elem_bytes, nullptr);
    const long long rowb = g.stride_token * elem_bytes;
    u32x4 v = *(const u32x4*)(base + (long long)(src_row + row) * rowb);
    *(u32x4*)(base + (long long)(dst_row + row) * rowb) = v;
}

hipError_t launch_move_rows(const SlabTable& tab, const Geom& g, int elem_bytes, int src_row, int dst_row,
                            int rows, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    int per16 = 16 / elem_bytes;
    long long ngroups = (long long)g.ncols / per16;
    // gridDim.y is limited to 65535 rows per launch
    for (int r0 = 0; r0 < rows; r0 += 65535) {
        int nr = rows - r0 < 65535 ? rows - r0 : 65535;
        dim3 grid((unsigned)((ngroups + 255) / 256), nr);
        hipLaunchKernelGGL(k_move_rows, grid, dim3(256), 0, st, tab, g, elem_bytes, src_row + r0,
                           dst_row + r0, per16);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------
// calibration kernels: what this device sustains for a plain copy and for a register-only MFMA
// loop on random (power-realistic) operands; rooflines are quoted against both nominal and these
// ------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_calib_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void k_calib_mfma(float* __restrict__ out, int iters)
{
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    half8 a, b;
    for (int i = 0; i < 8; ++i) {
        h = h * 1664525u + 1013904223u; a[i] = (_Float16)((float)((int)((h >> 16) & 1023) - 512) / 512.f);
        h = h * 1664525u + 1013904223u; b[i] = (_Float16)((float)((int)((h >> 16) & 1023) - 512) / 512.f);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = sum;
}

hipError_t launch_calib_copy(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    size_t n16 = bytes / 16;
    hipLaunchKernelGGL(k_calib_copy, dim3(256 * 16), dim3(256), 0, st, (u32x4*)dst, (const u32x4*)src, n16);
    return hipGetLastError();
}

hipError_t launch_calib_mfma(float* out, int blocks, int iters, hipStream_t st)
{
    hipLaunchKernelGGL(k_calib_mfma, dim3(blocks), dim3(256), 0, st, out, iters);
    return hipGetLastError();
}

}  // namespace freqkv
