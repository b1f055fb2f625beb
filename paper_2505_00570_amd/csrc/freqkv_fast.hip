// Factored ("fast") form of the compression operator for spans n = 4pq with p, q odd and coprime and a
// retained length Lc = n/2 (the paper's default ratio 0.5 on its windows: 8188 = 4*23*89, 4092 = 4*11*93).
//
// What is computed is exactly Sec. 3.3 Eq. 2-3 with the transforms of Appendix A -- orthonormal n-point
// DCT-II along tokens, the Lc lowest coefficients, Lc-point inverse, times sqrt(Lc/n) -- but evaluated the
// way Sec. 3.4 and Appendix A point to (an O(N log N) transform instead of the O(N^2) sums):
//
//   forward   C_t = sum_j x_j cos(pi t (2j+1) / 2n) is Re(e^{-i pi t/2n} V_t), V = DFT_n(v), where v is x with
//             its even-indexed samples first and its odd-indexed samples reversed behind them;
//   inverse   y = sum_t c_t cos(pi t (2m+1) / 2Lc) is recovered the same way from an Lc-point inverse DFT of
//             U_k = e^{i pi k/2Lc} (C_k - i C_{Lc-k}) / n  (C_Lc := 0: that coefficient is not kept);
//   both DFTs are prime-factor transforms: n = 4*p*q and Lc = 2*p*q have coprime factors, so with the
//             input index taken as j = j1 (n/4) + j2 (n/p) + j3 (n/q) mod n and the output index by its
//             residues (t mod 4, t mod p, t mod q) the length-n DFT is a 4 x p x q DFT with no twiddle factors
//             between its stages, and likewise 2 x p x q for the inverse.
//
// One workgroup owns 8 channels (16 where LDS holds them: the shorter spans) of one head-tensor for all rows
// (column ownership): it reads its 16 (32) bytes of every span row straight from the cache, keeps every
// intermediate in LDS, and writes its 16 (32) bytes of the Lc result rows back.  No workspace, no second pass over HBM, and no in-place hazard: nobody else touches
// these channels.  The length-p and length-q stages are small dense DFT matrices applied on the matrix cores
// (fp16 operands, fp32 accumulation) to the rows or columns of LDS-resident tiles; the length-4 and length-2
// stages are butterflies folded into the load and the store; the step between the two transforms (twiddles,
// real parts, Hermitian pairing) is a 2x4 real matrix per frequency pair and parity, precomputed in fp64.
//
// Phases (a barrier after each), with g = (array, channel) and all LDS values fp16:
//   load     rows -> X[g][j2][j3], four real p x q arrays per channel: the length-4 butterfly of the samples
//            j1 = 0..3 (sum, alternating sum, real and imaginary part of the odd outputs), scaled by a power
//            of two chosen from the largest magnitude of the slice so that no stage can overflow fp16
//   stage Q  real -> half-complex DFT over j3:  B[g][f][j2], f = Re 0..qh-1 | Im qh..2qh-1   (in place)
//   stage P  complex DFT over j2:               D[g][f][f2]                                    (in place)
//   middle   per (f2, f3): the four arrays' coefficients -> U of the even and of the odd k:  G[(k1,ch)][f][k2]
//   stage P' inverse complex DFT over k2:       E[(k1,m2,ch)][Re 0..47 | Im 48..95]    (other half of LDS)
//   stage Q' half-complex -> real over k3, the length-2 butterfly over k1 on its accumulators, and the store:
//            output index m = m1 (Lc/2) + m2 (Lc/p) + m3 (Lc/q) mod Lc, rows y_{2m} = u_m, y_{2m+1} = u_{Lc-1-m},
//            one rounding to bf16, straight from the registers to the cache
#include "freqkv_internal.h"

#include <cmath>
#include <vector>

namespace freqkv {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <int I> struct IC { static constexpr int value = I; };
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(IC<I>{});
        static_for<N, I + 1>(f);
    }
}

constexpr int kFragBytes = 1024;          // one 32 x 16 operand fragment set: 64 lanes x 8 halfs

// C_: channels of a head-tensor that one workgroup owns (8: 16 bytes of every row; 16: 32 bytes, which halves
// the cache lines touched per byte and is what LDS holds for the shorter spans).
template <int P_, int Q_, int C_ = 8>
struct FastCfg {
    static constexpr int P = P_, Q = Q_, C = C_;
    static constexpr int CV = C / 8;                  // 16-byte pieces of a row per workgroup
    static constexpr int J2 = C == 16 ? (P + 3) / 4 * 4 : (P + 7) / 8 * 8;   // p padded to whole 8- or 16-byte groups
    static constexpr int QH = (Q + 1) / 2;            // half-complex length of the q stage
    static constexpr int N = P * Q, n = 4 * N, Lc = 2 * N;
    static constexpr int NG = 4 * C;                  // (array, channel) groups
    static constexpr int GH = 96 * J2;                // halfs per group
    static constexpr int LDS_HALFS = NG * GH;
    static constexpr int KP = 2 * J2;                 // contraction length of the complex p stage (Re | Im)
    static constexpr int KSP = (KP + 15) / 16;        // its 16-deep steps
    static constexpr int NTP = (KP + 31) / 32;        // its 32-wide output tiles
    static constexpr int UROWS = (J2 % 32 == 0) ? J2 : ((J2 == 24 || J2 == 12) ? 96 : 32);   // lcm(32, J2)
    static constexpr int RT = UROWS / 32;
    static constexpr int NUNITS = NG * J2 / UROWS;
    static constexpr int NPOS = P * Q;
    static constexpr int NPJ = QH * (J2 / 2);         // middle step: jobs of two neighbouring k2 each
    // table offsets (bytes)
    static constexpr int OFF_Q = 0;
    static constexpr int OFF_P = OFF_Q + 3 * 6 * kFragBytes;
    static constexpr int OFF_PI = OFF_P + NTP * KSP * kFragBytes;
    static constexpr int OFF_QI = OFF_PI + NTP * KSP * kFragBytes;
    static constexpr int OFF_JOBS = OFF_QI + 3 * 6 * kFragBytes;
    static constexpr int TABLE_BYTES = OFF_JOBS + NPJ * 64;
    static_assert(Q <= 96 && 2 * QH <= 96 && QH <= 48, "q stage fits 96-wide tiles");
    // does some group g have ((g J2) >> 2) & 3 == s?  (the load stage needs one LDS offset per such class)
    static constexpr bool rot_class_used(int s)
    {
        for (int gq = 0; gq < NG; ++gq)
            if ((((gq * J2) >> 2) & 3) == s) return true;
        return false;
    }
    static_assert(C == 8 || C == 16, "8 or 16 channels per workgroup");
    static_assert(KP <= 64 && J2 % 4 == 0, "p stage fits two 32-wide tiles");
    static_assert(UROWS % J2 == 0 && UROWS % 32 == 0 && (NG * J2) % UROWS == 0, "in-place units hold whole groups");
    static_assert(LDS_HALFS * 2 + 2 * NTP * KSP * kFragBytes <= 160 * 1024 - 256, "LDS");
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// Rows of 96 halfs are kept as 12 chunks of 8 halfs (16 bytes), rotated by a row-dependent number of chunks:
// with rows 192 bytes apart, the 16-byte fragment reads of 16 consecutive rows would otherwise fall on 4 bank
// groups only.  rot2: the X image of the load stage (quads of rows get 0, 2, 1, 3).  rot12: the E image of stage P',
// where rows 8 apart (consecutive m2) are also written together and must spread as well.
__device__ __forceinline__ int rot2(int row) { return ((row >> 1) & 2) | ((row >> 3) & 1); }
__device__ __forceinline__ int rot12(int row) { return ((row >> 3) + 2 * ((row >> 2) & 1)) % 12; }
__device__ __forceinline__ int wrap12(int c) { return c >= 12 ? c - 12 : c; }

// Four accumulator values -> four fp16, round to nearest even, two packed conversions.
__device__ __forceinline__ half4 cvt4(float a, float b, float c, float d)
{
    f32x4 v = {a, b, c, d};
    return __builtin_convertvector(v, half4);
}

// Makes the compiler materialise a value at this point of the program (no instruction is emitted).
__device__ __forceinline__ void pin(half8& v) { asm volatile("" : "+v"(v)); }

// Row of the span that holds sample j of the even-first / odd-reversed ordering of an n-point sequence.
__device__ __forceinline__ int makhoul_row(int j, int n) { return j < n / 2 ? 2 * j : 2 * (n - 1 - j) + 1; }

// Operand fragment of the p stages: the 8 contraction values k .. k+7, k = (part, j2) with `part` the real or
// imaginary rows of column `col` (RS halfs apart) and J2 values per part.  J2 a multiple of 8: one 16-byte read.
// J2 = 12: two 8-byte runs, each inside one part (4 divides 12); runs at or beyond KP = 2 J2 are zero padding.
template <int J2>
__device__ __forceinline__ half8 p_fragment(const _Float16* col, int RS, int k)
{
    if constexpr (J2 % 8 == 0) {
        const int part = k / J2, j = k - part * J2;
        return *(const half8*)(col + part * RS + j);
    } else {
        half4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
        if (k < 2 * J2) { const int part = k / J2, j = k - part * J2; lo = *(const half4*)(col + part * RS + j); }
        if (k + 4 < 2 * J2) { const int part = (k + 4) / J2, j = k + 4 - part * J2; hi = *(const half4*)(col + part * RS + j); }
        return half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    }
}

// dump: diagnostic only.  When not null, workgroup 0 copies its LDS there after phase `stop` (1 load ...
// 5 stage P') and every workgroup returns without writing the cache.
template <class Cfg, int NW, bool DIAG>
__global__ __launch_bounds__(NW * 64, 1) void k_fast(SlabTable tab, Geom g, const char* __restrict__ tables_arg,
                                                 float rest_scale, float* __restrict__ tap,
                                                 _Float16* __restrict__ dump, int stop)
{
    constexpr int P = Cfg::P, Q = Cfg::Q, J2 = Cfg::J2, QH = Cfg::QH, N = Cfg::N, n = Cfg::n, Lc = Cfg::Lc;
    constexpr int GH = Cfg::GH, C = Cfg::C, CV = Cfg::CV;
    constexpr int NT = NW * 64;                        // threads
    __shared__ __attribute__((aligned(1024))) _Float16 lds[Cfg::LDS_HALFS];
    __shared__ uint32_t red[NW];
    // fragments of the two p-stage matrices, copied once per workgroup: register room for the prefetched rows
    __shared__ __attribute__((aligned(16))) half8 ptab[2][Cfg::NTP * Cfg::KSP][64];

    const int tid0 = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);

    // Virtual block index -> task (8 consecutive virtual columns).  Workgroups are dealt round-robin to the 8
    // XCDs; the d/8 tasks of one head-tensor take consecutive slots of ONE XCD, so that the 16-byte pieces they
    // read of the same 256-byte rows, and the pieces they write, meet in that XCD's L2.  The grid is persistent:
    // a workgroup takes the virtual indices blockIdx.x, blockIdx.x + gridDim.x, ... (gridDim.x is a multiple
    // of 8 whenever it is smaller than the number of tasks, so the XCD of a virtual index is the workgroup's).
    const int ntasks = g.ncols / C;
    const long long rowb = g.stride_token * 2;
    const uint32_t rowb32 = (uint32_t)rowb;            // the host checked that a head-tensor's span stays below 4 GiB
    auto map_task = [&](int vb, char** base_out, int* ht_out, int* c0_out) {
        const int tph = g.d / C;                       // tasks per head-tensor
        const int hts = g.ncols / g.d;
        const int full = hts / 8;                      // groups of 8 head-tensors
        const int per_group = 8 * tph;
        int task = vb;
        if (vb < full * per_group) {
            const int grp = vb / per_group, local = vb - grp * per_group;
            const int xcd = local & 7, slot = local >> 3;
            task = (grp * 8 + xcd) * tph + slot;
        }
        int ht;
        char* b = column_base(tab, g, task * C, 2, &ht);
        *base_out = b + (long long)g.S * rowb;
        *ht_out = ht;
        *c0_out = task * C - ht * g.d;
    };

    // diagnostic: stop == 8 runs everything and leaves the shader-clock reading after each phase in dump
    const bool stamp = DIAG && dump && stop >= 8;       // 9: as 8, but with the persistent grid of a real call
    long long ts[DIAG ? 10 : 1];
    auto take_stamp = [&](auto ic) {
        if constexpr (DIAG) ts[decltype(ic)::value] = stamp ? (long long)clock64() : 0;
    };
    take_stamp(IC<0>{});

    // Lane handles positions pos = tid + NT i of the p x q grid: the 4 x NIT row pieces of a task are requested
    // in one go, for the first task here and for every later one in the middle of the task before it.
    constexpr int NIT = (Cfg::NPOS + NT - 1) / NT;
    u32x4 raw[NIT][4][CV];
    // Requests pieces [F0, F1) of the lane's 4 NIT row pieces (piece f = 4 i + j1) of the task at bp into dst.
    auto issue_loads = [&](const char* bp, int tid, u32x4 (&dst)[NIT][4][CV], auto f0, auto f1) {
        constexpr int F0 = decltype(f0)::value, F1 = decltype(f1)::value < 4 * NIT ? decltype(f1)::value : 4 * NIT;
        static_for<(F1 > F0 ? F1 - F0 : 0)>([&](auto fc) {
            constexpr int f = F0 + decltype(fc)::value;
            constexpr int i = f / 4, j1 = f % 4;
            int pos = tid + NT * i;
            if (pos >= Cfg::NPOS) pos = 0;
            const int j2 = pos / Q, j3 = pos - j2 * Q;
            int j = (j2 * (4 * Q) + j3 * (4 * P)) % n + j1 * N;
            if (j >= n) j -= n;
            const char* rp = bp + (uint32_t)makhoul_row(j, n) * rowb32;
            static_for<CV>([&](auto v) { dst[i][j1][v.value] = *(const u32x4*)(rp + 16 * v.value); });
        });
    };
    int vbid = blockIdx.x;
    char* base;
    int ht, c0;
    map_task(vbid, &base, &ht, &c0);
    issue_loads(base, tid0, raw, IC<0>{}, IC<4 * NIT>{});
    {
        const half8* tp = (const half8*)(tables_arg + Cfg::OFF_P);   // the forward and the inverse table are adjacent
        for (int i = tid0; i < 2 * Cfg::NTP * Cfg::KSP * 64; i += NT) (&ptab[0][0][0])[i] = tp[i];
    }

  for (;;) {                                           // one task per iteration
    // Everything a lane derives from its index is recomputed in every iteration: kept alive across the whole
    // loop instead, these per-lane constants would not fit the register file next to the prefetched rows.
    if constexpr (DIAG) if (vbid != (int)blockIdx.x) take_stamp(IC<0>{});
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    // likewise the stage tables: read where they are used, in every iteration, not hoisted out of the loop
    // (an opaque OFFSET, not an opaque pointer: the pointer must stay recognisably global, or its loads become
    // flat loads, which the compiler can only wait for together with everything else in flight)
    unsigned tables_off = 0;
    asm volatile("" : "+s"(tables_off));
    const char* tables = tables_arg + tables_off;
    const int next_vbid = vbid + (int)gridDim.x;
    const bool has_next = (!DIAG || stop == 9) && next_vbid < ntasks;
    char* next_base = base;
    int next_ht = ht, next_c0 = c0;
    if (has_next) map_task(next_vbid, &next_base, &next_ht, &next_c0);
    // Rows of the next task: their 4 NIT pieces go out in 16 slots spread evenly over the whole task, one wave-wide
    // request at a time between pieces of other work (the L1 fill path takes about one such request per 128
    // cycles; requested in bursts they hold up the waves that issue them).  Without a next task the requests go
    // out all the same, to this task's rows again (3 % more requests over a workgroup's 32 tasks): a branch
    // around them would leave the compiler two possible counts of loads in flight, and it would then wait for
    // the table loads of a stage as if nothing had been issued behind them, i.e. for the fresh rows as well.
    u32x4 nraw[NIT][4][CV];
    auto pf = [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        issue_loads(next_base, tid, nraw, IC<(k * 4 * NIT) / 16>{}, IC<((k + 1) * 4 * NIT) / 16>{});
    };
    // ---- clear LDS while the rows are on their way (pad positions must hold finite values: they meet zero matrix entries)
    {
        u32x4 z = {0u, 0u, 0u, 0u};
        u32x4* l4 = (u32x4*)lds;
        for (int i = tid; i < Cfg::LDS_HALFS / 8; i += NT) l4[i] = z;
    }

    // largest magnitude of the slice (bf16 bit patterns compare like their magnitudes)
    uint32_t amax;
    {
        u16x2 m = {0, 0};
        static_for<NIT>([&](auto ic) {
            static_for<4>([&](auto jc) {
                static_for<4 * CV>([&](auto wc) {
                    uint32_t w = raw[decltype(ic)::value][decltype(jc)::value][decltype(wc)::value / 4][decltype(wc)::value % 4] & 0x7fff7fffu;
                    m = __builtin_elementwise_max(m, __builtin_bit_cast(u16x2, w));
                });
            });
        });
        amax = m[0] > m[1] ? m[0] : m[1];
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t o = (uint32_t)__shfl_xor((int)amax, off);
            amax = o > amax ? o : amax;
        }
        if (lane == 0) red[wave] = amax;
    }
    __syncthreads();                                   // LDS cleared, red[] complete
    take_stamp(IC<8>{});
    pf(IC<0>{});
    {
        uint32_t a = red[0];
        static_for<NW - 1>([&](auto w) { a = red[w.value + 1] > a ? red[w.value + 1] : a; });
        amax = (uint32_t)__builtin_amdgcn_readfirstlane((int)a);     // the same in every lane: keep it, and the scale
                                                                     // derived from it, in scalar registers
    }
    // 2^e brings the largest magnitude into [256, 512): the transforms amplify a constant sequence by at most
    // sqrt(pq) / 2 < 64 after the butterfly's 1/2, so every intermediate stays below the fp16 limit, and 2^-e undoes
    // the scale exactly at the end
    int e = 0;
    const bool nonfinite = (amax >> 7) == 255;         // an inf or nan somewhere in the slice: its channels come out nan
    {
        const int E = (int)(amax >> 7);                // exponent field of the largest magnitude
        if (E > 0 && E < 255) e = 135 - E;
        if (e > 120) e = 120;
    }
    const float unsc = rest_scale * __uint_as_float((uint32_t)(127 - e) << 23);

    // (A packed fp16 butterfly on integer-converted operands was measured: no faster, this stage waits for its
    // 2-byte LDS writes, and one more rounding in the error budget.)
    const float sc = 0.5f * __uint_as_float((uint32_t)(e + 127) << 23);
    static_for<NIT>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const int pos = tid + NT * i;
        if (pos < Cfg::NPOS) {
            const int j2 = pos / Q, j3 = pos - j2 * Q;
            // row = g J2 + j2, and g J2 is a multiple of 4: the rotation depends on g only through bits 2, 3 of g J2
            const int c = j3 >> 3;
            int off[4] = {0, 0, 0, 0};
            static_for<4>([&](auto sc4) {
                constexpr int sv = decltype(sc4)::value;
                if constexpr (Cfg::rot_class_used(sv)) off[sv] = j2 * 96 + wrap12(c + rot2(j2 + 4 * sv)) * 8 + (j3 & 7);
            });
            static_for<4 * CV>([&](auto wc) {
                constexpr int v = decltype(wc)::value / 4, w = decltype(wc)::value % 4;
                static_for<2>([&](auto hc) {
                    constexpr int hf = decltype(hc)::value;
                    constexpr int ch = 8 * v + 2 * w + hf;
                    const float a0 = hf ? bf16_hi(raw[i][0][v][w]) : bf16_lo(raw[i][0][v][w]);
                    const float a1 = hf ? bf16_hi(raw[i][1][v][w]) : bf16_lo(raw[i][1][v][w]);
                    const float a2 = hf ? bf16_hi(raw[i][2][v][w]) : bf16_lo(raw[i][2][v][w]);
                    const float a3 = hf ? bf16_hi(raw[i][3][v][w]) : bf16_lo(raw[i][3][v][w]);
                    const float s02 = a0 + a2, d02 = a0 - a2, s13 = a1 + a3, d13 = a3 - a1;
                    const float xv[4] = {(s02 + s13) * sc, (s02 - s13) * sc, d02 * sc, d13 * sc};
                    static_for<4>([&](auto xc) {
                        constexpr int gq = decltype(xc)::value * C + ch;
                        lds[gq * GH + off[((gq * J2) >> 2) & 3]] = (_Float16)xv[xc.value];
                    });
                });
            });
        }
    });
    pf(IC<1>{});
    __syncthreads();
    take_stamp(IC<1>{});
    auto dump_and_stop = [&](int phase) -> bool {
        if (!DIAG || !dump || stop != phase) return false;
        if (blockIdx.x == 0)
            for (int i = tid; i < Cfg::LDS_HALFS; i += NT) dump[i] = lds[i];
        return true;
    };
    if (dump_and_stop(1)) return;

    // ---- phase 2: stage Q.  Rows (g, j2) x contraction j3 (96) -> f (96); a wave owns whole units of UROWS
    // rows, reads all of a unit, then overwrites it with the transposed result [g][f][j2].  The units of a
    // wave run side by side, so that the fragment reads of one overlap the matrix instructions of the other.
    {
        half8 bq[3][6];
        const half8* tq = (const half8*)(tables + Cfg::OFF_Q) + lane;
        static_for<3>([&](auto ct) {
            static_for<6>([&](auto ks) { bq[ct.value][ks.value] = tq[(ct.value * 6 + ks.value) * 64]; });
        });
        constexpr int UU = Cfg::NUNITS / NW;           // units per wave
        static_assert(Cfg::NUNITS % NW == 0 && UU * Cfg::RT * NW <= 24, "units of a wave fit the register file");
        f32x16 acc[UU][Cfg::RT][3];
        static_for<UU>([&](auto uu) {
            static_for<Cfg::RT>([&](auto rt) {
                static_for<3>([&](auto ct) {
                    static_for<16>([&](auto r) { acc[uu.value][rt.value][ct.value][r.value] = 0.f; });
                });
            });
        });
        // every tile of 32 rows starts at a multiple of 32: the rotation of a lane's row is the same in all of them
        const int rot = rot2(l32);
        pf(IC<2>{});
        static_for<6>([&](auto ks) {
            if constexpr (decltype(ks)::value == 2) pf(IC<3>{});
            if constexpr (decltype(ks)::value == 4) pf(IC<4>{});
            const int coff = wrap12(ks.value * 2 + lhi + rot) * 8;
            static_for<UU>([&](auto uu) {
                const _Float16* src = lds + ((wave + NW * uu.value) * Cfg::UROWS + l32) * 96 + coff;
                static_for<Cfg::RT>([&](auto rt) {
                    const half8 a = *(const half8*)(src + rt.value * 32 * 96);
                    static_for<3>([&](auto ct) {
                        acc[uu.value][rt.value][ct.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            a, bq[ct.value][ks.value], acc[uu.value][rt.value][ct.value], 0, 0, 0);
                    });
                });
            });
        });
        static_for<UU>([&](auto uu) {
            const int u = wave + NW * uu.value;
            static_for<Cfg::RT>([&](auto rt) {
                static_for<4>([&](auto r4) {
                    const int row = u * Cfg::UROWS + rt.value * 32 + 8 * r4.value + 4 * lhi;   // first of 4 rows
                    const int grp = row / J2, j2 = row - grp * J2;
                    static_for<3>([&](auto ct) {
                        const int f = ct.value * 32 + l32;
                        const half4 o = cvt4(acc[uu.value][rt.value][ct.value][4 * r4.value], acc[uu.value][rt.value][ct.value][4 * r4.value + 1], acc[uu.value][rt.value][ct.value][4 * r4.value + 2], acc[uu.value][rt.value][ct.value][4 * r4.value + 3]);
                        *(half4*)(lds + grp * GH + f * J2 + j2) = o;
                    });
                });
            });
        });
        pf(IC<5>{});                                    // behind the epilogue: its accumulators are free by now
    }
    __syncthreads();
    take_stamp(IC<2>{});
    if (dump_and_stop(2)) return;

    // ---- phase 3: stage P.  Columns m' = (g, f3) x contraction (part, j2) -> (part', f2); the data are the
    // second operand, so a lane keeps one column and gets 4 consecutive f2: written back in place.  TU tiles of
    // 32 columns are in flight per wave.
    {
        half8 ap[Cfg::NTP][Cfg::KSP];
        static_for<Cfg::NTP>([&](auto nt) {
            static_for<Cfg::KSP>([&](auto ks) { ap[nt.value][ks.value] = ptab[0][nt.value * Cfg::KSP + ks.value][lane]; });
        });
        constexpr int TU = NW == 8 ? 3 : 4;
        constexpr int NTL = (Cfg::NG / 32) * QH;        // NG QH columns in tiles of 32
        constexpr int NIP = (NTL + NW * TU - 1) / (NW * TU);      // iterations of the tile loop
        static_for<NIP>([&](auto itc) {
            constexpr int it = decltype(itc)::value;
            const int t0 = wave + it * NW * TU;
            if constexpr (it == 0) pf(IC<6>{});
            if constexpr (it == NIP - 1) pf(IC<7>{});
            if (t0 >= NTL) return;
            _Float16* col[TU];
            half8 b[TU][Cfg::KSP];
            static_for<TU>([&](auto tu) {
                int t = t0 + NW * tu.value;
                if (t > NTL - 1) t = NTL - 1;          // a tile past the end repeats the last one and is not written
                const int mp = t * 32 + l32;
                const int grp = mp / QH, f3 = mp - grp * QH;
                col[tu.value] = lds + grp * GH + f3 * J2;
                static_for<Cfg::KSP>([&](auto ks) {
                    b[tu.value][ks.value] = p_fragment<J2>(col[tu.value], QH * J2, ks.value * 16 + 8 * lhi);
                });
            });
            f32x16 acc[TU][Cfg::NTP];
            static_for<TU>([&](auto tu) {
                static_for<Cfg::NTP>([&](auto nt) { static_for<16>([&](auto r) { acc[tu.value][nt.value][r.value] = 0.f; }); });
            });
            static_for<Cfg::KSP>([&](auto ks) {
                static_for<TU>([&](auto tu) {
                    static_for<Cfg::NTP>([&](auto nt) {
                        acc[tu.value][nt.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            ap[nt.value][ks.value], b[tu.value][ks.value], acc[tu.value][nt.value], 0, 0, 0);
                    });
                });
            });
            static_for<TU>([&](auto tu) {
                if (t0 + NW * tu.value < NTL) {
                    static_for<Cfg::NTP>([&](auto nt) {
                        static_for<4>([&](auto r4) {
                            const int n0 = nt.value * 32 + 8 * r4.value + 4 * lhi;
                            if (n0 < Cfg::KP) {
                                const int part = n0 / J2, f2 = n0 - part * J2;
                                const half4 o = cvt4(acc[tu.value][nt.value][4 * r4.value], acc[tu.value][nt.value][4 * r4.value + 1], acc[tu.value][nt.value][4 * r4.value + 2], acc[tu.value][nt.value][4 * r4.value + 3]);
                                *(half4*)(col[tu.value] + part * QH * J2 + f2) = o;
                            }
                        });
                    });
                }
            });
        });
    }
    __syncthreads();
    take_stamp(IC<3>{});
    if (dump_and_stop(3)) return;

    // ---- phase 4: middle.  An item is two neighbouring k2 of one k3 (one dword per array and part) and four
    // channels; per channel the four arrays' coefficients there give, through a 2x4 real map each,
    // U of the even k with these residues (from F0, F2) and of the odd k (from Fr, Fi); both land in place
    // of F0 and F2.  Packed fp16 arithmetic: both k2 of the pair at once.
    {
        constexpr int NITEMS = (C / 4) * Cfg::NPJ;      // (pair of k2, k3) x groups of four channels
        constexpr int NR = (NITEMS + NT - 1) / NT;
        uint32_t* lds32 = (uint32_t*)lds;
        static_for<NR>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            const int it_raw = tid + NT * r;
            const int it = it_raw < NITEMS ? it_raw : NITEMS - 1;     // lanes past the end read a valid table entry
            const int quarter = it / Cfg::NPJ;
            const int pj = it - quarter * Cfg::NPJ;
            const int k3 = pj / (J2 / 2), kp = pj - k3 * (J2 / 2);
            const u32x4* T = (const u32x4*)(tables + Cfg::OFF_JOBS) + pj * 4;
            const u32x4 q0 = T[0], q1 = T[1], q2 = T[2], q3 = T[3];
            __builtin_amdgcn_sched_barrier(0);              // the table first, the rows behind it
            if constexpr (r == 0) pf(IC<8>{});
            if constexpr (r == (NR > 1 ? 1 : 0)) pf(IC<9>{});
            if (it_raw >= NITEMS) return;
            half2v t[16];
            static_for<4>([&](auto i) {
                // (a bit cast straight from a vector ELEMENT reads element 0 whatever the index: copy first)
                const uint32_t w0 = q0[i.value], w1 = q1[i.value], w2 = q2[i.value], w3 = q3[i.value];
                t[i.value] = __builtin_bit_cast(half2v, w0);
                t[4 + i.value] = __builtin_bit_cast(half2v, w1);
                t[8 + i.value] = __builtin_bit_cast(half2v, w2);
                t[12 + i.value] = __builtin_bit_cast(half2v, w3);
            });
            uint32_t* re = lds32 + (k3 * J2) / 2 + kp;
            uint32_t* im = re + (QH * J2) / 2;
            static_for<4>([&](auto cc) {
                const int ch = quarter * 4 + cc.value;
                auto ld = [&](uint32_t* p, int xa) { return __builtin_bit_cast(half2v, p[(xa * C + ch) * (GH / 2)]); };
                const half2v ar = ld(re, 0), ai = ld(im, 0), br = ld(re, 1), bi = ld(im, 1);
                const half2v cr = ld(re, 2), ci = ld(im, 2), dr = ld(re, 3), di = ld(im, 3);
                const half2v er = t[0] * ar + t[1] * ai + t[2] * br + t[3] * bi;
                const half2v ei = t[4] * ar + t[5] * ai + t[6] * br + t[7] * bi;
                const half2v orr = t[8] * cr + t[9] * ci + t[10] * dr + t[11] * di;
                const half2v oi = t[12] * cr + t[13] * ci + t[14] * dr + t[15] * di;
                re[(0 * C + ch) * (GH / 2)] = __builtin_bit_cast(uint32_t, er);
                im[(0 * C + ch) * (GH / 2)] = __builtin_bit_cast(uint32_t, ei);
                re[(1 * C + ch) * (GH / 2)] = __builtin_bit_cast(uint32_t, orr);
                im[(1 * C + ch) * (GH / 2)] = __builtin_bit_cast(uint32_t, oi);
            });
        });
    }
    __syncthreads();
    take_stamp(IC<4>{});
    if (dump_and_stop(4)) return;

    // ---- phase 5: stage P'.  Rows m' = (g', k3 padded to 48), g' = (k1, ch) < 16, x contraction (part, k2)
    // -> (part', m2); results go to the other half of LDS as E[(k1, m2, ch)][part' 48 + k3].
    constexpr int Y0 = 2 * C * GH;
    {
        half8 bp[Cfg::NTP][Cfg::KSP];
        static_for<Cfg::NTP>([&](auto ct) {
            static_for<Cfg::KSP>([&](auto ks) { bp[ct.value][ks.value] = ptab[1][ct.value * Cfg::KSP + ks.value][lane]; });
        });
        pf(IC<10>{});
        constexpr int TU = 3;                          // 2 C x 48 rows = 3 C tiles
        for (int t0 = wave; t0 < 3 * C; t0 += NW * TU) {
            half8 a[TU][Cfg::KSP];
            static_for<TU>([&](auto tu) {
                const int mp = (t0 + NW * tu.value) * 32 + l32;
                const int grp = mp / 48;
                int k3 = mp - grp * 48;
                if (k3 > QH - 1) k3 = QH - 1;          // pad rows: any finite data, their results meet zeros
                const _Float16* rowp = lds + grp * GH + k3 * J2;
                static_for<Cfg::KSP>([&](auto ks) {
                    a[tu.value][ks.value] = p_fragment<J2>(rowp, QH * J2, ks.value * 16 + 8 * lhi);
                });
            });
            f32x16 acc[TU][Cfg::NTP];
            static_for<TU>([&](auto tu) {
                static_for<Cfg::NTP>([&](auto ct) { static_for<16>([&](auto r) { acc[tu.value][ct.value][r.value] = 0.f; }); });
            });
            static_for<Cfg::KSP>([&](auto ks) {
                static_for<TU>([&](auto tu) {
                    static_for<Cfg::NTP>([&](auto ct) {
                        acc[tu.value][ct.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            a[tu.value][ks.value], bp[ct.value][ks.value], acc[tu.value][ct.value], 0, 0, 0);
                    });
                });
            });
            static_for<TU>([&](auto tu) {
                const int t = t0 + NW * tu.value;              // wave-uniform
                static_for<Cfg::NTP>([&](auto ct) {
                    const int nn = ct.value * 32 + l32;
                    if (nn < Cfg::KP) {
                        const int part = nn / J2, m2 = nn - part * J2;
                        const int m2r = (m2 * (C / 8)) % 12;
                        static_for<4>([&](auto r4) {
                            // rows m0 .. m0+3 with m0 = 32 t + 8 r4 + 4 lhi: everything but the last term is the
                            // same for the whole wave, and 48 is a multiple of 8, so g' and the chunk of k3 are too
                            const int mu = t * 32 + 8 * r4.value;
                            const int g2 = mu / 48, k3u = mu - g2 * 48;         // wave-uniform
                            const int k1 = g2 / C, ch = g2 - k1 * C;
                            // row = (k1 J2 + m2) C + ch; m2 C is a multiple of 8, so rot12(row) splits into a
                            // wave-uniform part and m2's
                            const int rowq = k1 * J2 * C + ch;
                            const int rotu = ((rowq >> 3) + 2 * ((rowq >> 2) & 1)) % 12;
                            const int rowu = rowq * 96 + (k3u & 7);
                            const int chunk = wrap12(wrap12(m2r + rotu) + part * 6 + (k3u >> 3));
                            const half4 o = cvt4(acc[tu.value][ct.value][4 * r4.value], acc[tu.value][ct.value][4 * r4.value + 1],
                                                 acc[tu.value][ct.value][4 * r4.value + 2], acc[tu.value][ct.value][4 * r4.value + 3]);
                            *(half4*)(lds + Y0 + rowu + m2 * (C * 96) + chunk * 8 + 4 * lhi) = o;
                        });
                    }
                });
            });
        }
    }
    pf(IC<11>{});
    __syncthreads();
    take_stamp(IC<5>{});
    if (dump_and_stop(5)) return;
    take_stamp(IC<6>{});

    // ---- phase 6: stage Q' and the store.  Rows (k1, m2, ch) x contraction (Re | Im of k3, 96) -> m3.  A wave takes
    // a tile of 32 rows with k1 = 0 together with the tile of the same (m2, ch) with k1 = 1, so the length-2
    // butterfly over k1 is done on the fp32 accumulators: y_a = u0 + u1 belongs to output index m_a, y_b = u0 - u1
    // to m_b = m_a + Lc/2.  A lane holds column m3 and, per group of four registers, four channels of one m2; the
    // lane 32 further on holds the next four.  The two exchange what the other needs (the lower lane keeps y_a, the
    // upper y_b), and each writes one 16-byte piece of one result row: no LDS round trip, one rounding (to bf16).
    if (DIAG && dump && !stamp) return;
    {
        half8 bqi[3][6];
        const half8* tq = (const half8*)(tables + Cfg::OFF_QI) + lane;
        static_for<3>([&](auto ct) {
            static_for<6>([&](auto ks) { bqi[ct.value][ks.value] = tq[(ct.value * 6 + ks.value) * 64]; });
        });
        // pin the table: it is requested AND awaited here, ahead of this stage's row requests (the scheduler would
        // otherwise sink its loads towards their first use, behind them; a mere scheduling fence measured slower)
        static_for<3>([&](auto ct) {
            static_for<6>([&](auto ks) { pin(bqi[ct.value][ks.value]); });
        });
        pf(IC<12>{});
        constexpr int NPAIR = J2 * C / 32;             // tiles per k1
        static_assert(NPAIR <= NW, "one tile pair per wave");
        float* tp = nullptr;
        if (tap) tp = tap + ((g.tap_slab0 * g.hts_per_slab + ht) * (long long)Lc) * g.d + c0;
        if (wave < NPAIR) {
            const int t = wave;
            f32x16 acc0[3], acc1[3];
            static_for<3>([&](auto ct) {
                static_for<16>([&](auto r) { acc0[ct.value][r.value] = 0.f; acc1[ct.value][r.value] = 0.f; });
            });
            const int row0 = t * 32 + l32, row1 = (t + NPAIR) * 32 + l32;
            const _Float16* src0 = lds + Y0 + row0 * 96;
            const _Float16* src1 = lds + Y0 + row1 * 96;
            const int rot0 = rot12(row0) + lhi, rot1 = rot12(row1) + lhi;
            static_for<6>([&](auto ks) {
                const half8 a0 = *(const half8*)(src0 + wrap12(wrap12(ks.value * 2 + rot0)) * 8);
                const half8 a1 = *(const half8*)(src1 + wrap12(wrap12(ks.value * 2 + rot1)) * 8);
                static_for<3>([&](auto ct) {
                    acc0[ct.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, bqi[ct.value][ks.value], acc0[ct.value], 0, 0, 0);
                    acc1[ct.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, bqi[ct.value][ks.value], acc1[ct.value], 0, 0, 0);
                });
            });
            pf(IC<13>{});
            static_for<3>([&](auto ct) {
                if constexpr (decltype(ct)::value == 1) pf(IC<14>{});
                if constexpr (decltype(ct)::value == 2) pf(IC<15>{});
                const int m3 = ct.value * 32 + l32;
                static_for<4>([&](auto r4) {
                    // rows 32 t + 8 r4 + 4 lhi + (0..3): (k1 J2 + m2) C + channel; wave-uniform up to the lhi term
                    const int vu = t * 32 + 8 * r4.value;
                    const int m2 = vu / C, cb = vu - m2 * C;            // cb: first channel of this lane pair's 8
                    float ya[4], yb[4];
                    static_for<4>([&](auto i) {
                        const float u0 = acc0[ct.value][4 * r4.value + i.value], u1 = acc1[ct.value][4 * r4.value + i.value];
                        ya[i.value] = nonfinite ? __builtin_nanf("") : (u0 + u1) * unsc;
                        yb[i.value] = nonfinite ? __builtin_nanf("") : (u0 - u1) * unsc;
                    });
                    const uint32_t a_lo = pack_bf16x2(ya[0], ya[1]), a_hi = pack_bf16x2(ya[2], ya[3]);
                    const uint32_t b_lo = pack_bf16x2(yb[0], yb[1]), b_hi = pack_bf16x2(yb[2], yb[3]);
                    // the lower lane keeps y_a and receives the upper lane's y_a (channels +4); the upper lane keeps y_b
                    const uint32_t r_lo = (uint32_t)__shfl_xor((int)(lhi ? a_lo : b_lo), 32);
                    const uint32_t r_hi = (uint32_t)__shfl_xor((int)(lhi ? a_hi : b_hi), 32);
                    int ma = (m2 * (2 * Q) + m3 * (2 * P)) % Lc;
                    int mb = ma + N;
                    if (mb >= Lc) mb -= Lc;
                    const int orow = lhi ? makhoul_row(mb, Lc) : makhoul_row(ma, Lc);
                    const u32x4 piece = lhi ? u32x4{r_lo, r_hi, b_lo, b_hi} : u32x4{a_lo, a_hi, r_lo, r_hi};
                    const bool ok = m3 < Q && m2 < P;
                    if (ok) *(u32x4*)(base + (uint32_t)orow * rowb32 + 2 * cb) = piece;
                    if (tp) {
                        // the fp32 results before the rounding: the same exchange, in fp32
                        float mine[4], theirs[4];
                        static_for<4>([&](auto i) {
                            mine[i.value] = lhi ? yb[i.value] : ya[i.value];
                            theirs[i.value] = __shfl_xor(lhi ? ya[i.value] : yb[i.value], 32);
                        });
                        if (ok) {
                            float* o = tp + (long long)orow * g.d + cb;
                            static_for<4>([&](auto i) {
                                o[(lhi ? 4 : 0) + i.value] = mine[i.value];
                                o[(lhi ? 0 : 4) + i.value] = theirs[i.value];
                            });
                        }
                    }
                });
            });
        } else {
            pf(IC<13>{});
            pf(IC<14>{});
            pf(IC<15>{});
        }
    }
    if constexpr (DIAG) if (stamp) {
        __syncthreads();
        ts[7] = (long long)clock64();
        if (tid == 0) {
            long long* o = (long long*)dump + (long long)vbid * 9;
            for (int i = 0; i < 9; ++i) o[i] = ts[i];
        }
    }
    if (!has_next) break;
    vbid = next_vbid; base = next_base; ht = next_ht; c0 = next_c0;
    static_for<NIT>([&](auto ic) {
        static_for<4>([&](auto jc) {
            static_for<CV>([&](auto v) { raw[ic.value][jc.value][v.value] = nraw[ic.value][jc.value][v.value]; });
        });
    });
    __syncthreads();                                   // every wave is done with this task's LDS image
  }
}

// ------------------------------------------------------------------------------------------
// host: tables in fp64, rounded once
// ------------------------------------------------------------------------------------------

const double kPi = 3.14159265358979323846;

// Fragment order of a matrix M[k][idx] for v_mfma_f32_32x32x16_f16: tile t, step ks, lane l, element i hold
// M[ks*16 + 8*(l/32) + i][t*32 + l%32] (the same order serves as first or as second operand).
template <class F>
void fill_frags(_Float16* out, int tiles, int ksteps, F&& mat)
{
    for (int t = 0; t < tiles; ++t)
        for (int ks = 0; ks < ksteps; ++ks)
            for (int l = 0; l < 64; ++l)
                for (int i = 0; i < 8; ++i)
                    out[(((size_t)t * ksteps + ks) * 64 + l) * 8 + i] =
                        (_Float16)mat(ks * 16 + 8 * (l / 32) + i, t * 32 + l % 32);
}

long long mod_inverse(long long a, long long m)
{
    long long t = 0, nt = 1, r = m, nr = ((a % m) + m) % m;
    while (nr) {
        long long qq = r / nr;
        long long tmp = t - qq * nt; t = nt; nt = tmp;
        tmp = r - qq * nr; r = nr; nr = tmp;
    }
    return ((t % m) + m) % m;
}

template <class Cfg>
void build_tables(char* out)
{
    constexpr int P = Cfg::P, Q = Cfg::Q, J2 = Cfg::J2, QH = Cfg::QH, N = Cfg::N, n = Cfg::n, Lc = Cfg::Lc;
    const double sq = 1.0 / std::sqrt((double)Q), sp = 1.0 / std::sqrt((double)P);
    // stage Q: k = j3, idx = f (Re f3 | Im QH + f3)
    fill_frags((_Float16*)(out + Cfg::OFF_Q), 3, 6, [&](int k, int f) -> double {
        if (k >= Q || f >= 2 * QH) return 0.0;
        const int f3 = f < QH ? f : f - QH;
        const double a = 2.0 * kPi * (double)((long long)k * f3 % Q) / Q;
        return f < QH ? std::cos(a) * sq : -std::sin(a) * sq;
    });
    // stage P (forward, e^{-i}): k = (part, j2), idx = (part', f2)
    auto pmat = [&](int k, int idx, double sign) -> double {
        if (k >= 2 * J2 || idx >= 2 * J2) return 0.0;
        const int pk = k / J2, j2 = k % J2, pi = idx / J2, f2 = idx % J2;
        if (j2 >= P || f2 >= P) return 0.0;
        const double a = 2.0 * kPi * (double)(j2 * f2 % P) / P;
        // (re + i im)(cos - i sign sin): re' = re cos + sign im sin, im' = im cos - sign re sin
        if (pk == 0 && pi == 0) return std::cos(a) * sp;
        if (pk == 1 && pi == 0) return sign * std::sin(a) * sp;
        if (pk == 0 && pi == 1) return -sign * std::sin(a) * sp;
        return std::cos(a) * sp;
    };
    fill_frags((_Float16*)(out + Cfg::OFF_P), Cfg::NTP, Cfg::KSP, [&](int k, int idx) { return pmat(k, idx, 1.0); });
    fill_frags((_Float16*)(out + Cfg::OFF_PI), Cfg::NTP, Cfg::KSP, [&](int k, int idx) { return pmat(k, idx, -1.0); });
    // stage Q' : k = part' 48 + k3, idx = m3;  u = E_0 + 2 Re sum_{k3 >= 1} E_k3 e^{+2 pi i k3 m3 / q}
    fill_frags((_Float16*)(out + Cfg::OFF_QI), 3, 6, [&](int k, int m3) -> double {
        const int part = k / 48, k3 = k % 48;
        if (k3 >= QH || m3 >= Q) return 0.0;
        const double w = k3 == 0 ? 1.0 : 2.0;
        const double a = 2.0 * kPi * (double)((long long)k3 * m3 % Q) / Q;
        return part == 0 ? w * std::cos(a) * sq : -w * std::sin(a) * sq;
    });
    // middle: per (k2, k3) the 2x4 maps (F0, F2) -> U of the even k and (Fr, Fi) -> U of the odd k
    const long long e2 = (long long)Q * mod_inverse(Q, P) % N, e3 = (long long)P * mod_inverse(P, Q) % N;
    _Float16* jobs = (_Float16*)(out + Cfg::OFF_JOBS);     // [k3][k2 / 2][16 coefficients][k2 & 1]
    for (int k3 = 0; k3 < QH; ++k3) {
        for (int k2 = 0; k2 < J2; ++k2) {
            double T[2][2][8];                                             // [parity of k][re|im][input]
            for (int a = 0; a < 2; ++a) for (int b = 0; b < 2; ++b) for (int c = 0; c < 8; ++c) T[a][b][c] = 0.0;
            if (k2 < P) {
                const long long tau = (k2 * e2 + k3 * e3) % N, taup = N - tau;
                const long long kk[4] = {tau, tau + N, taup, taup + N};   // a, b (these residues); c, d (negated)
                for (int in = 0; in < 8; ++in) {
                    double x[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                    x[in] = 1.0;
                    // inputs: F0 (re, im), F2, Fr, Fi at (k2, k3); at the negated residues each is conjugated
                    auto V = [&](long long k, bool neg, double* vr, double* vi) {
                        const double sg = neg ? -1.0 : 1.0;
                        const double ar = x[0], ai = sg * x[1], br = x[2], bi = sg * x[3];
                        const double cr = x[4], ci = sg * x[5], dr = x[6], di = sg * x[7];
                        switch (k % 4) {
                            case 0: *vr = ar; *vi = ai; break;
                            case 1: *vr = cr - di; *vi = ci + dr; break;          // Fr + i Fi
                            case 2: *vr = br; *vi = bi; break;
                            default: *vr = cr + di; *vi = ci - dr; break;         // Fr - i Fi
                        }
                    };
                    double C[4];
                    for (int w = 0; w < 4; ++w) {
                        if (kk[w] >= Lc) { C[w] = 0.0; continue; }                // the coefficient that is not kept
                        double vr, vi;
                        V(kk[w], w >= 2, &vr, &vi);
                        const double th = kPi * (double)kk[w] / (2.0 * n);
                        C[w] = std::cos(th) * vr + std::sin(th) * vi;             // Re(e^{-i th} V)
                    }
                    // U_a = e^{i pi ka / 2Lc} (C_a - i C_d),  U_b = e^{i pi kb / 2Lc} (C_b - i C_c)
                    const double ta = kPi * (double)kk[0] / (2.0 * Lc), tb = kPi * (double)kk[1] / (2.0 * Lc);
                    const double uar = std::cos(ta) * C[0] + std::sin(ta) * C[3], uai = std::sin(ta) * C[0] - std::cos(ta) * C[3];
                    const double ubr = std::cos(tb) * C[1] + std::sin(tb) * C[2], ubi = std::sin(tb) * C[1] - std::cos(tb) * C[2];
                    const int pa = (int)(kk[0] & 1), pb = (int)(kk[1] & 1);
                    T[pa][0][in] = uar; T[pa][1][in] = uai;
                    T[pb][0][in] = ubr; T[pb][1][in] = ubi;
                }
            }
            _Float16* o = jobs + ((size_t)k3 * (J2 / 2) + k2 / 2) * 32 + (k2 & 1);
            for (int r = 0; r < 2; ++r)
                for (int in = 0; in < 4; ++in) {
                    o[(r * 4 + in) * 2] = (_Float16)T[0][r][in];            // even k: from (F0, F2)
                    o[(8 + r * 4 + in) * 2] = (_Float16)T[1][r][4 + in];    // odd k: from (Fr, Fi)
                }
        }
    }
}

template <class Cfg>
hipError_t launch_cfg(const SlabTable& tab, const Geom& g, const void* tables, float rest_scale, float* tap,
                      _Float16* dump, int stop, hipStream_t st)
{
    constexpr int NW = 8;          // two waves per SIMD: one wave's LDS traffic and conversions overlap the other's matrix work
    const unsigned tasks = (unsigned)(g.ncols / Cfg::C);
    // Persistent grid: as many workgroups as the device holds at once (LDS decides), a multiple of 8 so that a
    // workgroup's tasks stay on its XCD.  The diagnostic modes run one task per workgroup.
    unsigned grid = tasks;
    if (!dump || stop == 9) {
        int dev = 0, cus = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        const unsigned per_cu = (unsigned)(160 * 1024 / (Cfg::LDS_HALFS * 2 + 64));
        const unsigned resident = (unsigned)cus * (per_cu < 1 ? 1 : per_cu) / 8 * 8;
        if (resident >= 8 && tasks > resident) grid = resident;
    }
    if (dump)
        hipLaunchKernelGGL((k_fast<Cfg, NW, true>), dim3(grid), dim3(NW * 64), 0, st, tab, g, (const char*)tables,
                           rest_scale, tap, dump, stop);
    else
        hipLaunchKernelGGL((k_fast<Cfg, NW, false>), dim3(grid), dim3(NW * 64), 0, st, tab, g, (const char*)tables,
                           rest_scale, tap, dump, stop);
    return hipGetLastError();
}

// The factorizations with compiled kernels, n = 4 p q with window = n + 4 sinks: the paper's two windows (8192,
// 4096), two shorter ones (2048, 1024) and two small spans for tests (1260, 140).  Spans up to 4092 have two: 16
// channels per workgroup where head_dim allows (the first match in this list is taken), 8 otherwise.
#define FREQKV_FAST_CFGS(X) X(23, 89, 8) X(11, 93, 16) X(11, 93, 8) X(7, 73, 16) X(7, 73, 8) X(3, 85, 16) X(3, 85, 8) X(7, 45, 8) X(5, 7, 8)
#define FREQKV_FAST_MATCH(P_, Q_, C_) (n == FastCfg<P_, Q_, C_>::n && head_dim % C_ == 0)

}  // namespace

bool fast_supported(int n, int Lc, int head_dim, int* p, int* q, int* channels)
{
    if (Lc * 2 != n) return false;
#define X(P_, Q_, C_) if (FREQKV_FAST_MATCH(P_, Q_, C_)) { if (p) *p = P_; if (q) *q = Q_; if (channels) *channels = C_; return true; }
    FREQKV_FAST_CFGS(X)
#undef X
    return false;
}

size_t fast_table_bytes(int n, int head_dim)
{
#define X(P_, Q_, C_) if (FREQKV_FAST_MATCH(P_, Q_, C_)) return FastCfg<P_, Q_, C_>::TABLE_BYTES;
    FREQKV_FAST_CFGS(X)
#undef X
    return 0;
}

size_t fast_lds_halfs(int n, int head_dim)
{
#define X(P_, Q_, C_) if (FREQKV_FAST_MATCH(P_, Q_, C_)) return FastCfg<P_, Q_, C_>::LDS_HALFS;
    FREQKV_FAST_CFGS(X)
#undef X
    return 0;
}

void fast_build_tables_host(int n, int head_dim, char* out)
{
#define X(P_, Q_, C_) if (FREQKV_FAST_MATCH(P_, Q_, C_)) { build_tables<FastCfg<P_, Q_, C_>>(out); return; }
    FREQKV_FAST_CFGS(X)
#undef X
}

hipError_t launch_fast(const SlabTable& tab, const Geom& g, const void* tables, float rest_scale, float* tap,
                       _Float16* dump, int stop, hipStream_t st)
{
    const int n = g.n, head_dim = g.d;
#define X(P_, Q_, C_) if (FREQKV_FAST_MATCH(P_, Q_, C_)) return launch_cfg<FastCfg<P_, Q_, C_>>(tab, g, tables, rest_scale, tap, dump, stop, st);
    FREQKV_FAST_CFGS(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace freqkv
