// gfx950 kernels for chunk-wise (prefill) attention over the compacted cache.
//
// The tokens of an incoming chunk are the last q_len cached rows; query i sits at in-cache position
// p_i = cur_len - q_len + i and attends to rows [0, p_i]: sinks, compressed rows, the earlier tokens of its
// chunk and itself (Sec. 3.4 Eq. 5).  Keys are cached un-rotated and take the rotary embedding of their
// row index when they are read; queries take the one of p_i (closing paragraph of Sec. 3.4).
//
// Unlike the one-token case this is a dense contraction (q_len x cur_len x d per head, twice), so it runs
// on the matrix cores, as a streaming-softmax attention kernel.  Three small passes put the cached operands
// into MFMA fragment order first (all fp16: a bf16 cache value is exact in fp16, and the rotated keys and
// queries keep 11 significant bits instead of 8):
//   k_prefill_cs      cos/sin of (row * theta_j) for every cached row, fp64 angle reduction, fp32 table
//   k_prefill_prep_k  Kr = rotate(K) in tiles of 32 keys, [tile][group of 8 channels][key][8]
//   k_prefill_prep_v  Vt = V transposed in tiles of 32 keys, [tile][channel block][k-step][half][channel][8 keys],
//                     keys permuted so that a softmax tile, as the matrix core leaves it in registers, is
//                     already the second operand of the weighted sum
// and k_attend_prefill first builds, per wave, Qr = rotate(q) * log2(e)/sqrt(d) for its 32 queries in
// registers (once), then computes S^T = Kr Qr^T for 32 keys x 32 queries at a time, the running softmax per
// query (a query is a column, so its sum is an in-lane reduction plus one exchange between the two
// half-waves at the end), and O^T += Vt P^T.
#include "freqkv_internal.h"

namespace freqkv {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
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

constexpr int kD = 128;            // head_dim served by this kernel
constexpr int kKeyTile = 32;       // keys per tile
constexpr int kQPerWave = 32;      // queries per wave
constexpr int kPrefillWaves = 8;   // waves per workgroup of the attention kernel
constexpr int kTileBytes = kKeyTile * kD * 2;   // one Kr or Vt tile, fp16
constexpr float kSlack = 14.0f;    // log2 of the largest un-rescaled softmax weight (an fp16 operand: < 2^16)
constexpr float kWeightLimit = 16384.0f;   // 2^kSlack

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ half2v pack_half2(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_convertvector(v, half2v);          // round to nearest even, one packed conversion
}

// Position of the key that sits at storage index s (0..31) of a Vt tile: the matrix core leaves a
// 32x32 result with register r of a lane in half-wave hw at row 8*(r/4) + 4*hw + r%4; k-step t of the
// weighted sum takes registers 8t .. 8t+7, so storage index s = 16t + 8hw + e holds key
// 16t + 8*(e/4) + 4*hw + e%4.
__device__ __forceinline__ int vt_key(int s)
{
    int t = s >> 4, hw = (s >> 3) & 1, e = s & 7;
    return 16 * t + 8 * (e >> 2) + 4 * hw + (e & 3);
}

}  // namespace

// cs[p][j] = (cos, sin)(p * base^(-2j/d)), p < rows, j < d/2.
__global__ void k_prefill_cs(float2* __restrict__ cs, int rows, int d, double base, int rope)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    int half = d / 2;
    if (idx >= (long long)rows * half) return;
    int p = (int)(idx / half), j = (int)(idx - (long long)p * half);
    float2 o = {1.f, 0.f};
    if (rope) {
        double theta = pow(base, -2.0 * (double)j / (double)d);
        double x = (double)p * theta;
        double k = rint(x * 0.15915494309189535);
        double r = fma(-k, 6.283185307179586, x);
        r = fma(-k, 2.4492935982947064e-16, r);
        double s, c;
        sincos(r, &s, &c);
        o.x = (float)c;
        o.y = (float)s;
    }
    cs[idx] = o;
}

// One thread per (unit, key row, group of 8 rotary pairs): rotate and store in fragment order; the group of
// the lower half and its partner group of the upper half come from the same two 16-byte loads.
// Kr tile layout (fp16): [group of 8 channels g8 = 0..15][key 0..31][8].
__global__ void k_prefill_prep_k(const SlabTable tab, const PrefillGeom g, const float2* __restrict__ cs,
                                 _Float16* __restrict__ Kr)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    constexpr int half = kD / 2;
    constexpr int pgn = half / 8;                             // groups of 8 pairs per row
    long long total = (long long)g.units * g.key_tiles * kKeyTile * pgn;
    if (idx >= total) return;
    int pg = (int)(idx % pgn);
    long long rest = idx / pgn;
    int p = (int)(rest % ((long long)g.key_tiles * kKeyTile));
    int unit = (int)(rest / ((long long)g.key_tiles * kKeyTile));
    half8 lo8 = {}, up8 = {};                                 // rows beyond cur_len are zero
    if (p < g.cur_len) {
        int layer = unit / g.units_per_layer;
        int rem = unit - layer * g.units_per_layer;
        int b = rem / g.n_kv, kvh = rem - b * g.n_kv;
        const uint16_t* row = (const uint16_t*)tab.base[2 * layer] + (long long)b * g.stride_batch +
                              (long long)kvh * g.stride_head + (long long)p * g.stride_token;
        const int j0 = pg * 8;                                // first rotary pair of this group
        const u32x4 lo = *(const u32x4*)(row + j0), up = *(const u32x4*)(row + half + j0);
        const float2* c = cs + (long long)p * half + j0;
        for (int i = 0; i < 4; ++i) {
            float a0 = bf16_lo(lo[i]), a1 = bf16_hi(lo[i]);
            float b0 = bf16_lo(up[i]), b1 = bf16_hi(up[i]);
            float2 c0 = c[2 * i], c1 = c[2 * i + 1];
            // lower half: x_j cos - x_{j+d/2} sin;  upper half: x_{j+d/2} cos + x_j sin
            lo8[2 * i]     = (_Float16)(a0 * c0.x - b0 * c0.y);
            lo8[2 * i + 1] = (_Float16)(a1 * c1.x - b1 * c1.y);
            up8[2 * i]     = (_Float16)(b0 * c0.x + a0 * c0.y);
            up8[2 * i + 1] = (_Float16)(b1 * c1.x + a1 * c1.y);
        }
    }
    int tile = p / kKeyTile, key = p % kKeyTile;
    _Float16* dst = Kr + ((long long)unit * g.key_tiles + tile) * (kKeyTile * kD) + ((long long)pg * kKeyTile + key) * 8;
    *(half8*)dst = lo8;
    *(half8*)(dst + (long long)pgn * kKeyTile * 8) = up8;
}

// One workgroup per (unit, tile of 32 keys): the 32 x 128 bf16 block of V is read row by row with 16-byte
// loads, turned through LDS, and written as the Vt tile.
// Vt tile layout (fp16): [channel block db = 0..3][k-step t = 0..1][half-wave hw = 0..1][channel 0..31][8 keys].
__global__ __launch_bounds__(256) void k_prefill_prep_v(const SlabTable tab, const PrefillGeom g, _Float16* __restrict__ Vt)
{
    __shared__ uint32_t sm[kKeyTile][kD / 2 + 1];             // [key][pair of channels], one word of padding per row
    const int tile = blockIdx.x % g.key_tiles;
    const int unit = blockIdx.x / g.key_tiles;
    const int layer = unit / g.units_per_layer;
    const int rem = unit - layer * g.units_per_layer;
    const int b = rem / g.n_kv, kvh = rem - b * g.n_kv;
    const uint16_t* head = (const uint16_t*)tab.base[2 * layer + 1] + (long long)b * g.stride_batch +
                           (long long)kvh * g.stride_head;
    for (int piece = threadIdx.x; piece < kKeyTile * (kD / 8); piece += 256) {
        const int key = piece / (kD / 8), seg = piece % (kD / 8);
        const int row = tile * kKeyTile + key;
        u32x4 w = {0u, 0u, 0u, 0u};                           // rows beyond cur_len are zero
        if (row < g.cur_len) w = *(const u32x4*)(head + (long long)row * g.stride_token + seg * 8);
        static_for<4>([&](auto i) { sm[key][seg * 4 + i.value] = w[i.value]; });
    }
    __syncthreads();
    // thread = (k-step t, half-wave hw, pair of channels): two adjacent 16-byte groups of the tile
    const int cp = threadIdx.x & 63, hw = (threadIdx.x >> 6) & 1, t = threadIdx.x >> 7;
    half8 lo, hi;
    static_for<8>([&](auto e) {
        const uint32_t w = sm[vt_key(16 * t + 8 * hw + e.value)][cp];
        lo[e.value] = (_Float16)bf16_lo(w);
        hi[e.value] = (_Float16)bf16_hi(w);
    });
    const int ch = 2 * cp, db = ch >> 5, dl = ch & 31;
    _Float16* dst = Vt + ((long long)unit * g.key_tiles + tile) * (kKeyTile * kD) +
                    (long long)(((db * 2 + t) * 2 + hw) * 32 + dl) * 8;
    *(half8*)dst = lo;
    *(half8*)(dst + 8) = hi;
}

// Workgroup = 8 waves = 8 tasks of one KV unit, two waves per SIMD; a task is (query head of the KV group,
// block of 32 queries), heads fastest, so that with 4 query heads per KV head the waves walk the same keys.
// A wave keeps its 32 queries, their 128 x 32 output block and two 32 x 32 score blocks in vector registers
// (under 256 in all, so that two waves share a SIMD and the matrix instructions take all operands from the
// vector registers).
__global__ __launch_bounds__(kPrefillWaves * 64, 2)
void k_attend_prefill(const PrefillGeom g, const _Float16* __restrict__ Kr, const _Float16* __restrict__ Vt,
                      const uint16_t* __restrict__ q, const float2* __restrict__ cs, uint16_t* __restrict__ out,
                      float* __restrict__ lse)
{
    __shared__ __attribute__((aligned(1024))) char ksm[4][kTileBytes];   // Kr tiles t+1, t+2, t+3 of step t (ring)
    __shared__ __attribute__((aligned(1024))) char vsm[4][kTileBytes];   // Vt tiles t .. t+3 (ring)

    static_assert(kTileBytes == kPrefillWaves * 64 * 16, "one 16-byte piece of a tile per thread");
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: the loop bounds below are per wave
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, hw = lane >> 5;
    const int tasks_per_unit = g.G * g.q_blocks;
    const int wgs_per_unit = (tasks_per_unit + kPrefillWaves - 1) / kPrefillWaves;
    // blockIdx -> (KV unit, workgroup of the unit).  Workgroups are dealt round-robin to the 8 XCDs, so inside a
    // group of 8 units the XCD index picks the unit: all workgroups of a unit run on one XCD and share its L2
    // for the unit's K/V tiles (dealt unit by unit, every XCD fetched every unit: 12.7 GB of fabric reads per
    // launch against 2.2 GB of operands).  The units left over after the last full group are dealt plainly.
    int unit, wg_seq;
    {
        const int per_group = 8 * wgs_per_unit;
        const int grp = blockIdx.x / per_group;
        if (grp < g.units / 8) {
            const int local = blockIdx.x - grp * per_group;
            unit = grp * 8 + (local & 7);
            wg_seq = local >> 3;
        } else {
            const int local = blockIdx.x - (g.units / 8) * per_group;
            unit = (g.units / 8) * 8 + local / wgs_per_unit;
            wg_seq = local % wgs_per_unit;
        }
    }
    // later query blocks see more keys: hand them out first so that the long workgroups start early
    const int wg_in_unit = wgs_per_unit - 1 - wg_seq;
    const int task = wg_in_unit * kPrefillWaves + wave;
    const bool active = task < tasks_per_unit;
    const int qb = active ? task / g.G : 0;
    const int gh = active ? task - qb * g.G : 0;
    const long long head = (long long)unit * g.G + gh;             // dense query-head index
    const int q0 = qb * kQPerWave;                                 // first query row of this wave
    const int pos0 = g.cur_len - g.q_len + q0;                     // its in-cache position

    // keys this wave needs: [0, pos0 + 31] cut at cur_len; the workgroup loads up to its largest need
    const int my_last = active ? min(pos0 + kQPerWave - 1, g.cur_len - 1) : -1;
    const int my_tiles = (my_last + kKeyTile) / kKeyTile;
    const int full_tiles = active ? (pos0 + 1) / kKeyTile : 0;     // tiles every query of the wave sees whole
    int wg_tiles;
    {
        const int last_task = min(wg_in_unit * kPrefillWaves + kPrefillWaves - 1, tasks_per_unit - 1);
        const int last_qb = last_task / g.G;
        const int wg_last = min(g.cur_len - g.q_len + last_qb * kQPerWave + kQPerWave - 1, g.cur_len - 1);
        wg_tiles = (wg_last + kKeyTile) / kKeyTile;
    }

    // ---- queries of this wave: second operand of S^T = Kr Qr^T, lane = query column, 8 channels per k-step half.
    // Qr = rotate(q at its in-cache position) * log2(e)/sqrt(d), computed here once per wave: the lane's groups
    // of 8 channels in the lower half (k-steps 0..3) and their rotary partners in the upper half (k-steps 4..7)
    // come from the same two 16-byte loads.  Rows of the block beyond q_len are zero.
    half8 qf[8];
    {
        const bool have = active && q0 + l32 < g.q_len;
        const uint16_t* qrow = q + (head * g.q_len + (have ? q0 + l32 : 0)) * kD;
        const float2* crow = cs + (long long)(have ? pos0 + l32 : 0) * (kD / 2);
        static_for<4>([&](auto sc) {
            constexpr int S = decltype(sc)::value;
            const int j0 = S * 16 + hw * 8;                   // first rotary pair of the group
            half8 lo8 = {}, up8 = {};
            if (have) {
                const u32x4 lo = *(const u32x4*)(qrow + j0), up = *(const u32x4*)(qrow + kD / 2 + j0);
                static_for<4>([&](auto ec) {
                    constexpr int E = decltype(ec)::value;
                    const float a0 = bf16_lo(lo[E]), a1 = bf16_hi(lo[E]);
                    const float b0 = bf16_lo(up[E]), b1 = bf16_hi(up[E]);
                    const float2 c0 = crow[j0 + 2 * E], c1 = crow[j0 + 2 * E + 1];
                    // lower half: x_j cos - x_{j+d/2} sin;  upper half: x_{j+d/2} cos + x_j sin
                    lo8[2 * E]     = (_Float16)((a0 * c0.x - b0 * c0.y) * g.qscale);
                    lo8[2 * E + 1] = (_Float16)((a1 * c1.x - b1 * c1.y) * g.qscale);
                    up8[2 * E]     = (_Float16)((b0 * c0.x + a0 * c0.y) * g.qscale);
                    up8[2 * E + 1] = (_Float16)((b1 * c1.x + a1 * c1.y) * g.qscale);
                });
            }
            qf[S] = lo8;
            qf[S + 4] = up8;
        });
    }

    f32x16 acc[4];              // O^T: [channel block], 32 channels x 32 queries each
    static_for<4>([&](auto db) { static_for<16>([&](auto r) { acc[db.value][r.value] = 0.f; }); });
    float m = 0.f, lsum = 0.f;  // m: reference point of the lane's query (both half-waves agree); lsum: this half-wave's share
    f32x16 negm;                // -m in every register: the accumulator input of the first score instruction of a tile
    static_for<16>([&](auto r) { negm[r.value] = 0.f; });

    const char* ksrc = (const char*)(Kr + (long long)unit * g.key_tiles * (kKeyTile * kD));
    const char* vsrc = (const char*)(Vt + (long long)unit * g.key_tiles * (kKeyTile * kD));
    const int tid16 = threadIdx.x * 16;
    const int frag = (hw * kKeyTile + l32) * 16;       // this lane's 16 bytes inside a k-step of a tile

    // Step t consumes tile t: it computes S(t+1) = Kr(t+1) Qr^T while the softmax of S(t) runs, then
    // O^T += Vt(t) P(t)^T.  Kr(t+3) and Vt(t+3) are requested at the start of step t, straight into their ring
    // slots (whose tiles t-1 were consumed a step ago), and have landed at the barrier that ends it.  Keys are
    // thus two barriers ahead of their use, so that the first fragments of Kr(t+2) can be read before the
    // barrier of step t: the matrix instructions of step t+1 then start right behind it.
    // A tile is copied global -> LDS directly, each wave its 1 KB share (the copy is issued from assembly: the
    // compiler, which cannot tell the ring slots apart, would wait for a copy issued through its builtin in
    // front of the next LDS read; the waits are placed by hand, before each barrier).
    typedef __attribute__((address_space(3))) char* lptr_t;
    const uint32_t k_lds = (uint32_t)(uintptr_t)(lptr_t)ksm[0] + wave * 1024;
    const uint32_t v_lds = (uint32_t)(uintptr_t)(lptr_t)vsm[0] + wave * 1024;
    auto dma_k = [&](int tile, int slot) { lds_dma16(k_lds + (slot & 3) * kTileBytes, ksrc + (long long)tile * kTileBytes + tid16); };
    auto dma_v = [&](int tile, int slot) { lds_dma16(v_lds + (slot & 3) * kTileBytes, vsrc + (long long)tile * kTileBytes + tid16); };
    // Copies past the last tile are not branched around: they repeat the last tile into a slot that nobody
    // reads any more, which keeps the loop free of branches.
    const int last_tile = wg_tiles - 1;
    static_for<3>([&](auto i) {
        dma_k(min(i.value, last_tile), i.value);
        dma_v(min(i.value, last_tile), i.value);
    });
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    half8 kf[8], vf[8];         // fragments of Kr(t+1) and Vt(t), read from LDS a few matrix instructions ahead
    auto read_k = [&](auto s8, const char* kt) { kf[s8.value] = *(const half8*)(kt + s8.value * (2 * kKeyTile * 16)); };

    // cur holds S(t) - m: the accumulators of the scores start at minus the query's reference point, so the
    // exponent needs no subtraction; nxt receives S(t+1) - m during step t; the two swap roles every step.
    f32x16 cur, nxt;
    static_for<16>([&](auto r) { cur[r.value] = 0.f; });
    if (my_tiles > 0) {
        const char* kt = ksm[0] + frag;
        static_for<8>([&](auto s8) {
            read_k(s8, kt);
            cur = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[s8.value], qf[s8.value], cur, 0, 0, 0);
        });
        static_for<2>([&](auto s8) { read_k(s8, ksm[1] + frag); });
    }

    // Causal mask of a tile that reaches past the first query of the wave.
    auto mask_tile = [&](int tile, f32x16& s) {
        const int key_base = tile * kKeyTile;
        const int qpos = pos0 + l32;
        static_for<16>([&](auto r) {
            constexpr int R = decltype(r)::value;
            const int key = key_base + 8 * (R / 4) + 4 * hw + (R % 4);
            if (key > qpos) s[R] = -INFINITY;
        });
    };
    // Moves the reference point m of every query whose largest score in s exceeds it by more than the slack
    // (all of them on the first tile) up to that score: the accumulated sums and the pending scores follow.
    // Returns the lane's shift.  Any reference point gives the same quotient, so the point only has to keep
    // the weights inside the fp16 range.  Rare after the first tiles.
    auto move_refs = [&](f32x16& s, bool all) -> float {
        float v = s[0];
        static_for<16>([&](auto r) { v = fmaxf(v, s[r.value]); });
        const float mx = fmaxf(v, __shfl_xor(v, 32));
        const bool grow = all || mx > kSlack;
        const float delta = grow ? mx : 0.f;
        const float f = exp2_fast(-delta);
        m += delta;
        lsum *= f;
        static_for<4>([&](auto db) { static_for<16>([&](auto r) { acc[db.value][r.value] *= f; }); });
        static_for<16>([&](auto r) { s[r.value] -= delta; });
        static_for<16>([&](auto r) { negm[r.value] = -m; });
        return delta;
    };

    // One step: tile t, whose scores minus m are in s, is consumed while the scores of tile t+1 go to n.
    bool first = true;          // the first tile sets the reference points whatever the scores are
    auto step = [&](int t, f32x16& s, f32x16& n) {
        const bool mine = t < my_tiles;
        if (mine) {
            if (t >= full_tiles) mask_tile(t, s);
            if (first) move_refs(s, true);
            first = false;
        }
        dma_k(min(t + 3, last_tile), t + 3);
        dma_v(min(t + 3, last_tile), t + 3);
        if (mine) {
            const char* kt = ksm[(t + 1) & 3] + frag;     // past the wave's last tile a stale slot: result unused
            const char* vt = vsm[t & 3] + frag;
            auto read_v = [&](auto i) { vf[i.value] = *(const half8*)(vt + i.value * (2 * kKeyTile * 16)); };
            // ---- scores of the next tile on the matrix cores, dealt out between the exponentials of this tile
            // on the vector units: per 16-channel step one matrix instruction and two weights, packed to fp16
            // as they are produced; kf[0], kf[1] were read before the barrier
            float ps = 0.f;
            u32x4 pw[2];        // P^T, the second operand of the weighted sum, per k-step
            static_for<8>([&](auto s8) {
                constexpr int S8 = decltype(s8)::value;
                if constexpr (S8 < 6) {
                    read_k(IC<S8 + 2>{}, kt);
                } else {                                   // first k-step of the weighted sum: vf[2*db]
                    read_v(IC<(S8 - 6) * 4>{});
                    read_v(IC<(S8 - 6) * 4 + 2>{});
                }
                n = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[S8], qf[S8], S8 == 0 ? negm : n, 0, 0, 0);
                constexpr int R = 2 * S8;
                const half2v ph = pack_half2(exp2_fast(s[R]), exp2_fast(s[R + 1]));
                ps = __builtin_amdgcn_fdot2(ph, half2v{(_Float16)1, (_Float16)1}, ps, false);   // sums the rounded weights
                pw[R / 8][(R % 8) / 2] = __builtin_bit_cast(uint32_t, ph);
                __builtin_amdgcn_sched_barrier(0);
            });
            // No weight may exceed 2^kSlack (fp16 operands).  That is checked after the fact, on the sum of the
            // lane's 16 weights, which is there anyway (an overflowed weight makes it infinite): if it is too
            // large for some lane, the reference points move, the scores of the next tile, which started from
            // the old ones, follow, and the weights of this tile are computed again.
            if (__builtin_amdgcn_ballot_w64(!(ps <= kWeightLimit)) != 0) {
                const float delta = move_refs(s, false);
                static_for<16>([&](auto r) { n[r.value] -= delta; });
                ps = 0.f;
                static_for<8>([&](auto s8) {
                    constexpr int R = 2 * decltype(s8)::value;
                    const half2v ph = pack_half2(exp2_fast(s[R]), exp2_fast(s[R + 1]));
                    ps = __builtin_amdgcn_fdot2(ph, half2v{(_Float16)1, (_Float16)1}, ps, false);
                    pw[R / 8][(R % 8) / 2] = __builtin_bit_cast(uint32_t, ph);
                });
            }
            lsum += ps;
            // ---- O^T += Vt P^T : 128 channels x 32 queries, contraction over the 32 keys; k-step outermost so
            // that dependent accumulations are four instructions apart
            static_for<2>([&](auto k2) {
                const half8 pf = __builtin_bit_cast(half8, pw[k2.value]);
                static_for<4>([&](auto db) {
                    if constexpr (decltype(k2)::value == 0) read_v(IC<decltype(db)::value * 2 + 1>{});   // second k-step
                    else if constexpr (decltype(db)::value < 2) read_k(db, ksm[(t + 2) & 3] + frag);   // first fragments of the step after
                    acc[db.value] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[db.value * 2 + k2.value], pf, acc[db.value], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };
    // The queries are consumed above only by waves that have tiles; using them here makes the compiler wait for
    // their loads on every path, instead of in front of the first matrix instruction of each step (where the
    // wait would also cover the tile loads just issued).
    asm volatile("" : "+v"(qf[0]), "+v"(qf[1]), "+v"(qf[2]), "+v"(qf[3]), "+v"(qf[4]), "+v"(qf[5]), "+v"(qf[6]), "+v"(qf[7]));
    for (int t = 0; t < wg_tiles; t += 2) {
        step(t, cur, nxt);
        if (t + 1 < wg_tiles) step(t + 1, nxt, cur);
    }

    // ---- normalise and store: lane = query, registers = channels 8*(r/4) + 4*hw + r%4 of each block
    lsum += __shfl_xor(lsum, 32);
    const int qi = q0 + l32;
    if (active && qi < g.q_len) {
        const float inv = 1.0f / lsum;
        uint16_t* orow = out + (head * g.q_len + qi) * kD;
        static_for<4>([&](auto db) {
            static_for<4>([&](auto r4) {
                constexpr int R = 4 * decltype(r4)::value;
                f32x2 a = {acc[db.value][R] * inv, acc[db.value][R + 1] * inv};
                f32x2 b = {acc[db.value][R + 2] * inv, acc[db.value][R + 3] * inv};
                u32x2 w;
                w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2));
                w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2));
                *(u32x2*)(orow + db.value * 32 + 8 * r4.value + 4 * hw) = w;
            });
        });
        if (lse && hw == 0) lse[head * g.q_len + qi] = 0.6931471805599453f * (m + log2f(lsum));
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

hipError_t launch_prefill_prepare(const SlabTable& tab, const PrefillGeom& g, double rope_base, float2* cs,
                                  _Float16* Kr, _Float16* Vt, hipStream_t st)
{
    if (g.d != kD || g.cur_len < 1 || g.q_len < 1 || g.q_len > g.cur_len) return hipErrorInvalidValue;
    if (g.key_tiles * kKeyTile < g.cur_len || g.q_pad < g.q_len || g.q_pad % kQPerWave) return hipErrorInvalidValue;
    {
        long long total = (long long)g.cur_len * (kD / 2);
        hipLaunchKernelGGL(k_prefill_cs, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, cs, g.cur_len, kD,
                           rope_base, g.rope);
    }
    {
        long long total = (long long)g.units * g.key_tiles * kKeyTile * (kD / 16);
        hipLaunchKernelGGL(k_prefill_prep_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, tab, g, cs, Kr);
        hipLaunchKernelGGL(k_prefill_prep_v, dim3((unsigned)((long long)g.units * g.key_tiles)), dim3(256), 0, st, tab, g, Vt);
    }
    return hipGetLastError();
}

hipError_t launch_attend_prefill(const PrefillGeom& g, const _Float16* Kr, const _Float16* Vt, const void* q, const float2* cs,
                                 void* out, float* lse, hipStream_t st)
{
    if (g.d != kD || g.q_blocks * kQPerWave != g.q_pad) return hipErrorInvalidValue;
    const int wgs_per_unit = (g.G * g.q_blocks + kPrefillWaves - 1) / kPrefillWaves;
    hipLaunchKernelGGL(k_attend_prefill, dim3((unsigned)((long long)g.units * wgs_per_unit)), dim3(kPrefillWaves * 64), 0,
                       st, g, Kr, Vt, (const uint16_t*)q, cs, (uint16_t*)out, lse);
    return hipGetLastError();
}

}  // namespace freqkv
