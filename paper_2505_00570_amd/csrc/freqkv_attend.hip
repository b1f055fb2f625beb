// gfx950 kernels for decode attention over the compacted cache.
//
// One incoming token attends to every cached row [0, cur_len) of its KV head: sinks, compressed rows
// and the tokens appended since, itself included (Sec. 3.3 Eq. 4, Sec. 3.4 Eq. 5).  Keys are cached
// without the rotary embedding; the key of cache row p is rotated by position p, an index inside the
// cache, when it is read, and the query by its own in-cache position (closing paragraph of Sec. 3.4,
// appendix on key states with RoPE).  Rotary pairing is LLaMA's: channel i turns with channel i + d/2
// by the angle pos * base^(-2i/d).
//
// The work is bound by reading K and V once from HBM, so it runs on the vector ALUs, not on the matrix
// cores.  Two kernels:
//   k_attend_partial  one workgroup per (KV head, chunk of rows, group of <= 4 query heads that share
//                     the KV head); every lane owns 4 rotary pairs of a row (8 channels), D/8 lanes
//                     share a row, and each such lane group walks its rows with a running
//                     max / sum / weighted-V state (online softmax).  cos/sin of the row position are
//                     advanced by a fixed rotation per step from seeds computed with an fp64 range
//                     reduction, so no table is read in the loop.
//   k_attend_merge    combines the per-chunk states of a query head and writes the output row.
#include "freqkv_internal.h"

namespace freqkv {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kUnroll = 2;          // rows in flight per lane group per loop step (times two: prefetch)
constexpr float kMinusBig = -1.0e30f;
constexpr int kReseed = 32;          // loop steps between exact recomputations of the row cos/sin
constexpr float kSlack = 8.0f;      // log2 of the largest un-rescaled softmax weight

template <int I> struct IC { static constexpr int value = I; };
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(IC<I>{});
        static_for<N, I + 1>(f);
    }
}

// ---- P consecutive channels (P = 4 or 8), as stored and as floats ---------------------------------
template <typename T, int P> struct Raw;
template <> struct Raw<uint16_t, 4> { u32x2 a; };
template <> struct Raw<float, 4>    { f32x4 a; };

__device__ __forceinline__ void load_raw(const uint16_t* p, Raw<uint16_t, 4>& r) { r.a = *(const u32x2*)p; }
__device__ __forceinline__ void load_raw(const float* p, Raw<float, 4>& r) { r.a = *(const f32x4*)p; }

template <int P> __device__ __forceinline__ void unpack(const Raw<uint16_t, P>& r, float (&f)[P])
{
    static_for<P / 2>([&](auto i) {
        constexpr int I = decltype(i)::value;
        f[2 * I]     = __uint_as_float(r.a[I] << 16);
        f[2 * I + 1] = __uint_as_float(r.a[I] & 0xffff0000u);
    });
}
__device__ __forceinline__ void unpack(const Raw<float, 4>& r, float (&f)[4])
{
    static_for<4>([&](auto i) { f[decltype(i)::value] = r.a[decltype(i)::value]; });
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Lane exchange inside a row of 16 lanes through the data-parallel primitives (no LDS traffic).
template <int CTRL> __device__ __forceinline__ float dpp(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
// Sum over the LPR (4, 8, 16 or 32) adjacent lanes that share a cache row; every lane gets the sum.
template <int LPR> __device__ __forceinline__ float group_sum(float x)
{
    x += dpp<0xB1>(x);                           // quad_perm [1,0,3,2]
    x += dpp<0x4E>(x);                           // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) x += dpp<0x141>(x);  // mirror inside each half row of 8
    if constexpr (LPR >= 16) x += dpp<0x140>(x); // mirror inside the row of 16
    if constexpr (LPR >= 32) x += __shfl_xor(x, 16);
    return x;
}

// cos and sin of pos * theta.  The product, its reduction to [-pi/4, pi/4] plus a quadrant and the two
// short Taylor sums (truncation below 2e-9 on that interval) are all in fp64; the results are rounded once.
struct CosSin { float c, s; };
__device__ __forceinline__ CosSin seed_sincos(double theta, int pos)
{
    double x = (double)pos * theta;
    double k = rint(x * 0.6366197723675814);              // 2/pi
    double r = fma(-k, 1.5707963267948966, x);
    r = fma(-k, 6.123233995736766e-17, r);
    double r2 = r * r;
    // sin r = r (1 - r2/6 + r2^2/120 - r2^3/5040 + r2^4/362880 - r2^5/39916800)
    double ps = -1.0 / 39916800.0;
    ps = fma(ps, r2, 1.0 / 362880.0);
    ps = fma(ps, r2, -1.0 / 5040.0);
    ps = fma(ps, r2, 1.0 / 120.0);
    ps = fma(ps, r2, -1.0 / 6.0);
    ps = fma(ps, r2, 1.0);
    double sr = r * ps;
    // cos r = 1 - r2/2 + r2^2/24 - r2^3/720 + r2^4/40320 - r2^5/3628800 + r2^6/479001600
    double pc = 1.0 / 479001600.0;
    pc = fma(pc, r2, -1.0 / 3628800.0);
    pc = fma(pc, r2, 1.0 / 40320.0);
    pc = fma(pc, r2, -1.0 / 720.0);
    pc = fma(pc, r2, 1.0 / 24.0);
    pc = fma(pc, r2, -0.5);
    double cr = fma(pc, r2, 1.0);
    // add the quadrant back: angle = r + quad * pi/2
    int quad = (int)((long long)k & 3);
    double cs = (quad & 1) ? sr : cr;
    double ss = (quad & 1) ? cr : sr;
    if (quad == 1 || quad == 2) cs = -cs;
    if (quad >= 2) ss = -ss;
    return CosSin{(float)cs, (float)ss};
}

}  // namespace

// theta_j = base^(-2j/d) and the rotation that advances a row position by `step` rows.
__global__ void k_rope_table(RopeEntry* rt, int d, double base, int step)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= d / 2) return;
    double theta = pow(base, -2.0 * (double)j / (double)d);
    double sd, cd;
    sincos((double)step * theta, &sd, &cd);
    RopeEntry e;
    e.theta = theta;
    e.cd = (float)cd;
    e.sd = (float)sd;
    rt[j] = e;
}

// T: storage type of the cache, the query and the output (uint16_t = bfloat16 bits, or float).
// D: head_dim.  GT: query heads handled together (they share the KV head).  P: rotary pairs per lane
// (the lane owns channels P*l .. P*l+P-1 and their partners D/2 + P*l ..), so D/(2P) lanes share a row.
template <typename T, int D, int GT, int P>
__global__ __launch_bounds__(kWaves * 64, attend_min_waves(sizeof(T), GT, P))
void k_attend_partial(const SlabTable tab, const AttGeom g, const T* __restrict__ q,
                      const RopeEntry* __restrict__ rt, float* __restrict__ part_acc,
                      float* __restrict__ part_ml)
{
    constexpr int LPR = D / (2 * P);       // lanes per cache row
    constexpr int RPW = 64 / LPR;          // rows per wave per load
    constexpr int STEP = kWaves * RPW;     // rows between two consecutive rows of one lane group
    constexpr int U = kUnroll;
    constexpr int HSLOTS = kWaves * RPW / 2;
    typedef Raw<T, P> RawT;

    __shared__ float red[HSLOTS * GT * D];
    __shared__ float xm[GT][kWaves];
    __shared__ float xl[GT][kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l = lane % LPR;
    const int slot = lane / LPR;

    const int unit = blockIdx.x / g.n_split;
    const int split = blockIdx.x - unit * g.n_split;
    const int g0 = blockIdx.y * GT;                   // first query head of this workgroup inside the KV group
    const int layer = unit / g.units_per_layer;
    const int rem = unit - layer * g.units_per_layer;
    const int b = rem / g.n_kv;
    const int kvh = rem - b * g.n_kv;
    const long long head_off = (long long)b * g.stride_batch + (long long)kvh * g.stride_head;
    const T* kbase = (const T*)tab.base[2 * layer] + head_off;
    const T* vbase = (const T*)tab.base[2 * layer + 1] + head_off;

    // Cached rows and query position of this sequence: common to the batch, or per sequence (clamped to
    // [1, g.cur_len] so that every address stays inside the cache whatever the device array holds).
    int cur_len = g.cur_len, q_pos = g.q_pos;
    if (g.cur_lens) {
        cur_len = max(1, min(g.cur_lens[b], g.cur_len));
        q_pos = cur_len - 1;
    }
    const int row0 = split * g.chunk;
    const int row_end = min(row0 + g.chunk, cur_len);   // <= row0 for a chunk beyond a short sequence: no rows
    const int p0 = row0 + wave * RPW + slot;           // first row of this lane group

    // ---- rows of this lane group: p0, p0+STEP, p0+2*STEP, ...
    const int nit = row_end > row0 ? (row_end - row0 + STEP * U - 1) / (STEP * U) : 0;
    const int last = cur_len - 1;
    // Rows are addressed by 32-bit byte offsets inside the head's slab (uniform base + per-lane offset; the host
    // checks the range).  Rows past the end re-read the last row: no load is conditional, so the loads in
    // flight can be counted exactly; such rows are masked in the steps that can contain them.
    const char* kb = (const char*)kbase;
    const char* vb = (const char*)vbase;
    const uint32_t row_bytes = (uint32_t)g.stride_token * (uint32_t)sizeof(T);
    const uint32_t lane_off = (uint32_t)(P * l) * (uint32_t)sizeof(T);
    const uint32_t last_off = (uint32_t)last * row_bytes + lane_off;
    uint32_t next_off = (uint32_t)p0 * row_bytes + lane_off;      // first row of the step to be loaded next
    struct Rows { RawT kl[U], kh[U], vl[U], vh[U]; };
    auto issue = [&](Rows& r) {
        static_for<U>([&](auto uu) {
            constexpr int u = decltype(uu)::value;
            const uint32_t o = min(next_off + (uint32_t)(u * STEP) * row_bytes, last_off);
            load_raw((const T*)(kb + o), r.kl[u]);
            load_raw((const T*)(kb + o) + D / 2, r.kh[u]);
            load_raw((const T*)(vb + o), r.vl[u]);
            load_raw((const T*)(vb + o) + D / 2, r.vh[u]);
        });
        next_off += (uint32_t)(U * STEP) * row_bytes;
    };
    // the first rows are requested before anything else: the seeds below need no cache data
    Rows ra, rb;
    issue(ra);

    // ---- rotary state of the P pairs this lane owns: pair j couples channels P*l+j and D/2+P*l+j.
    // (c, s) = cos/sin of (row position * theta_j); each processed row advances them by the fixed rotation
    // (cd, sd) of STEP rows, and every kReseed loop steps they are recomputed exactly.
    float c[P], s[P], cd[P], sd[P];
    auto seed_rows = [&](int pos) {
        static_for<P>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            RopeEntry e = rt[P * l + j];
            CosSin k0 = seed_sincos(g.rope ? e.theta : 0.0, pos);   // no rotary embedding: every angle is zero
            c[j] = k0.c; s[j] = k0.s;
            cd[j] = g.rope ? e.cd : 1.f;
            sd[j] = g.rope ? e.sd : 0.f;
        });
    };
    seed_rows(p0);

    // ---- queries: rotated at the query's position, scaled by log2(e)/sqrt(d) so that exp is exp2
    float ql[GT][P], qh[GT][P];
    {
        float qc[P], qs[P];
        static_for<P>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            CosSin q0 = seed_sincos(g.rope ? rt[P * l + j].theta : 0.0, q_pos);
            qc[j] = q0.c; qs[j] = q0.s;
        });
        static_for<GT>([&](auto gg) {
            constexpr int gi = decltype(gg)::value;
            const T* qp = q + ((long long)unit * g.G + g0 + gi) * D;
            RawT rl, rh;
            load_raw(qp + P * l, rl);
            load_raw(qp + D / 2 + P * l, rh);
            float a[P], bb[P];
            unpack(rl, a);
            unpack(rh, bb);
            static_for<P>([&](auto jj) {
                constexpr int j = decltype(jj)::value;
                ql[gi][j] = (a[j] * qc[j] - bb[j] * qs[j]) * g.qscale;
                qh[gi][j] = (bb[j] * qc[j] + a[j] * qs[j]) * g.qscale;
            });
        });
    }

    float m[GT], lsum[GT], acc[GT][2 * P];
    static_for<GT>([&](auto gg) {
        constexpr int gi = decltype(gg)::value;
        m[gi] = kMinusBig;
        lsum[gi] = 0.f;
        static_for<2 * P>([&](auto cc) { acc[gi][decltype(cc)::value] = 0.f; });
    });

    // ---- main loop over the rows of this lane group: p0, p0+STEP, p0+2*STEP, ...
    // One step: the U rows in r (loaded a step ago) against the GT queries.
    auto consume = [&](const Rows& r, int it) {
        if (it != 0 && (it & (kReseed - 1)) == 0) seed_rows(p0 + it * U * STEP);
        const bool tail = row0 + (it + 1) * U * STEP > row_end;       // same for the whole workgroup

        float sc[U][GT];
        static_for<U>([&](auto uu) {
            constexpr int u = decltype(uu)::value;
            float a[P], bb[P];
            unpack(r.kl[u], a);
            unpack(r.kh[u], bb);
            float part[GT];
            static_for<GT>([&](auto gg) { part[decltype(gg)::value] = 0.f; });
            static_for<P>([&](auto jj) {
                constexpr int j = decltype(jj)::value;
                float rl = a[j] * c[j] - bb[j] * s[j];
                float rh = bb[j] * c[j] + a[j] * s[j];
                static_for<GT>([&](auto gg) {
                    constexpr int gi = decltype(gg)::value;
                    part[gi] = fmaf(ql[gi][j], rl, part[gi]);
                    part[gi] = fmaf(qh[gi][j], rh, part[gi]);
                });
                float cn = c[j] * cd[j] - s[j] * sd[j];        // advance the pair's angle by STEP rows
                s[j] = s[j] * cd[j] + c[j] * sd[j];
                c[j] = cn;
            });
            static_for<GT>([&](auto gg) {
                constexpr int gi = decltype(gg)::value;
                sc[u][gi] = group_sum<LPR>(part[gi]);
            });
            if (tail) {                                        // only the last steps of a chunk can hold rows past its end
                const bool valid = p0 + (it * U + u) * STEP < row_end;
                static_for<GT>([&](auto gg) {
                    constexpr int gi = decltype(gg)::value;
                    sc[u][gi] = valid ? sc[u][gi] : -INFINITY;
                });
            }
        });

        static_for<GT>([&](auto gg) {
            constexpr int gi = decltype(gg)::value;
            // The reference point m of the running softmax only moves when a score exceeds it by more than
            // 2^kSlack; until then weights up to 2^kSlack are accumulated as they are (any reference point
            // gives the same quotient), and the rescaling of the accumulators is skipped for the whole wave.
            float mx = sc[0][gi];
            static_for<U>([&](auto uu) { mx = fmaxf(mx, sc[decltype(uu)::value][gi]); });
            const bool grow = mx > m[gi] + kSlack;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                float mn = grow ? mx : m[gi];
                float f = exp2_fast(m[gi] - mn);
                m[gi] = mn;
                lsum[gi] *= f;
                static_for<2 * P>([&](auto cc) { acc[gi][decltype(cc)::value] *= f; });
            }
            static_for<U>([&](auto uu) {
                constexpr int u = decltype(uu)::value;
                float pw = exp2_fast(sc[u][gi] - m[gi]);
                lsum[gi] += pw;
                float va[P], vb2[P];
                unpack(r.vl[u], va);
                unpack(r.vh[u], vb2);
                static_for<P>([&](auto jj) {
                    constexpr int j = decltype(jj)::value;
                    acc[gi][j] = fmaf(pw, va[j], acc[gi][j]);
                    acc[gi][P + j] = fmaf(pw, vb2[j], acc[gi][P + j]);
                });
            });
        });
    };
    // Two register sets take turns: while one step is consumed the loads of the next are in flight.  The step
    // count is rounded up to even; a surplus step sees only rows past the end (weights exactly zero).
    for (int it = 0; it < nit; it += 2) {
        issue(rb);
        consume(ra, it);
        issue(ra);
        consume(rb, it + 1);
    }

    // ---- combine the lane groups of the workgroup
    // 1. common maximum per query head: over the lane groups of a wave by shuffles, over waves through LDS
    static_for<GT>([&](auto gg) {
        constexpr int gi = decltype(gg)::value;
        float mx = m[gi];
        for (int o = LPR; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        if (lane == 0) xm[gi][wave] = mx;
    });
    __syncthreads();
    static_for<GT>([&](auto gg) {
        constexpr int gi = decltype(gg)::value;
        float M = fmaxf(fmaxf(xm[gi][0], xm[gi][1]), fmaxf(xm[gi][2], xm[gi][3]));
        float f = exp2_fast(m[gi] - M);
        m[gi] = M;
        float ls = lsum[gi] * f;
        for (int o = LPR; o < 64; o <<= 1) ls += __shfl_xor(ls, o);
        if (lane == 0) xl[gi][wave] = ls;
        // rescale, fold the neighbouring lane group in, park the even groups' sums in LDS
        static_for<2 * P>([&](auto cc) {
            constexpr int ci = decltype(cc)::value;
            float v = acc[gi][ci] * f;
            v += __shfl_xor(v, LPR);
            acc[gi][ci] = v;
        });
        if ((slot & 1) == 0) {
            float* dst = red + ((wave * (RPW / 2) + (slot >> 1)) * GT + gi) * D;
            static_for<P / 4>([&](auto qq) {
                constexpr int o = 4 * decltype(qq)::value;
                *(f32x4*)(dst + P * l + o) = f32x4{acc[gi][o], acc[gi][o + 1], acc[gi][o + 2], acc[gi][o + 3]};
                *(f32x4*)(dst + D / 2 + P * l + o) =
                    f32x4{acc[gi][P + o], acc[gi][P + o + 1], acc[gi][P + o + 2], acc[gi][P + o + 3]};
            });
        }
    });
    __syncthreads();

    // 2. sum over the parked lane groups; one (query head, channel) per thread and pass
    const long long pidx = ((long long)unit * g.G + g0) * g.n_split + split;   // + gi * n_split below
    for (int idx = tid; idx < GT * D; idx += kWaves * 64) {
        int gi = idx / D;
        int ch = idx - gi * D;
        float sum = 0.f;
#pragma unroll
        for (int hs = 0; hs < HSLOTS; ++hs) sum += red[(hs * GT + gi) * D + ch];
        part_acc[(pidx + (long long)gi * g.n_split) * D + ch] = sum;
    }
    if (tid < GT) {
        float M = fmaxf(fmaxf(xm[tid][0], xm[tid][1]), fmaxf(xm[tid][2], xm[tid][3]));
        float Lsum = xl[tid][0] + xl[tid][1] + xl[tid][2] + xl[tid][3];
        float* ml = part_ml + (pidx + (long long)tid * g.n_split) * 2;
        ml[0] = M;
        ml[1] = Lsum;
    }
}

// One workgroup of D threads per query head: merge the chunk states, normalise, store.
template <typename T>
__global__ void k_attend_merge(const AttGeom g, const float* __restrict__ part_acc,
                               const float* __restrict__ part_ml, T* __restrict__ out,
                               float* __restrict__ lse)
{
    const long long head = blockIdx.x;                    // (layer, batch, query head), dense
    const int ch = threadIdx.x;
    const float* ml = part_ml + head * g.n_split * 2;
    float M = kMinusBig;
    for (int sp = 0; sp < g.n_split; ++sp) M = fmaxf(M, ml[2 * sp]);
    float o = 0.f, L = 0.f;
    for (int sp = 0; sp < g.n_split; ++sp) {
        float f = exp2_fast(ml[2 * sp] - M);
        L = fmaf(ml[2 * sp + 1], f, L);
        o = fmaf(part_acc[(head * g.n_split + sp) * g.d + ch], f, o);
    }
    float r = o / L;
    if constexpr (sizeof(T) == 2) {
        f32x2 v = {r, 0.f};
        bf16x2 bv = __builtin_convertvector(v, bf16x2);
        out[head * g.d + ch] = (T)(__builtin_bit_cast(uint32_t, bv) & 0xffffu);
    } else {
        out[head * g.d + ch] = r;
    }
    if (lse && ch == 0) lse[head] = 0.6931471805599453f * (M + log2f(L));
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

hipError_t launch_rope_table(RopeEntry* rt, int d, double base, hipStream_t st)
{
    int step = attend_row_step(d);
    hipLaunchKernelGGL(k_rope_table, dim3((d / 2 + 63) / 64), dim3(64), 0, st, rt, d, base, step);
    return hipGetLastError();
}

template <typename T, int D, int P>
static hipError_t launch_partial_p(const SlabTable& tab, const AttGeom& g, const void* q, const RopeEntry* rt,
                                   float* part_acc, float* part_ml, hipStream_t st)
{
    dim3 grid((unsigned)(g.units * g.n_split), (unsigned)(g.G / g.GT));
    dim3 block(kWaves * 64);
    switch (g.GT) {
        case 4: hipLaunchKernelGGL((k_attend_partial<T, D, 4, P>), grid, block, 0, st, tab, g, (const T*)q, rt, part_acc, part_ml); break;
        case 2: hipLaunchKernelGGL((k_attend_partial<T, D, 2, P>), grid, block, 0, st, tab, g, (const T*)q, rt, part_acc, part_ml); break;
        case 1: hipLaunchKernelGGL((k_attend_partial<T, D, 1, P>), grid, block, 0, st, tab, g, (const T*)q, rt, part_acc, part_ml); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_partial_t(const SlabTable& tab, const AttGeom& g, const void* q, const RopeEntry* rt,
                                   float* part_acc, float* part_ml, hipStream_t st)
{
    if (g.P != attend_pairs_per_lane(g.d)) return hipErrorInvalidValue;
    switch (g.d) {
        case 64:  return launch_partial_p<T, 64, attend_pairs_per_lane(64)>(tab, g, q, rt, part_acc, part_ml, st);
        case 128: return launch_partial_p<T, 128, attend_pairs_per_lane(128)>(tab, g, q, rt, part_acc, part_ml, st);
        case 256: return launch_partial_p<T, 256, attend_pairs_per_lane(256)>(tab, g, q, rt, part_acc, part_ml, st);
        default:  return hipErrorInvalidValue;
    }
}

hipError_t launch_attend_partial(const SlabTable& tab, const AttGeom& g, int elem_bytes, const void* q,
                                 const RopeEntry* rt, float* part_acc, float* part_ml, hipStream_t st)
{
    if (g.units < 1 || g.n_split < 1 || g.chunk < 1 || g.cur_len < 1) return hipErrorInvalidValue;
    if ((long long)(g.n_split - 1) * g.chunk >= g.cur_len) return hipErrorInvalidValue;   // no chunk beyond the longest cache
    if ((long long)g.n_split * g.chunk < g.cur_len) return hipErrorInvalidValue;          // chunks cover the cache
    if (g.G % g.GT) return hipErrorInvalidValue;
    if (g.chunk % (kUnroll * attend_row_step(g.d))) return hipErrorInvalidValue;
    return elem_bytes == 2 ? launch_partial_t<uint16_t>(tab, g, q, rt, part_acc, part_ml, st)
                           : launch_partial_t<float>(tab, g, q, rt, part_acc, part_ml, st);
}

hipError_t launch_attend_merge(const AttGeom& g, int elem_bytes, const float* part_acc, const float* part_ml,
                               void* out, float* lse, hipStream_t st)
{
    dim3 grid((unsigned)((long long)g.units * g.G));
    dim3 block(g.d);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(k_attend_merge<uint16_t>, grid, block, 0, st, g, part_acc, part_ml, (uint16_t*)out, lse);
    else
        hipLaunchKernelGGL(k_attend_merge<float>, grid, block, 0, st, g, part_acc, part_ml, (float*)out, lse);
    return hipGetLastError();
}

}  // namespace freqkv
