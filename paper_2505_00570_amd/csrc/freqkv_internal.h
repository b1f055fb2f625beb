// Internal interface between the host side of libfreqkv (argument checks, plans,
// basis cache, launch sequence) and its gfx950 kernels.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace freqkv {

// One wave copies 64 x 16 bytes global -> LDS without passing registers: lane i reads 16 bytes at its own
// address src and the data lands at LDS byte address lds + 16 i (lds is the same for the whole wave).  The copy
// counts as a vector-memory load (vmcnt); the compiler does not know that it writes LDS, so the kernel waits
// for it by hand (s_waitcnt vmcnt) before the barrier that publishes the data.  M0 carries the LDS address:
// kernels that use this have no other user of M0 (the compiler rejects M0 in a clobber list, so the build
// script checks the generated assembly for that instead).
__device__ __forceinline__ void lds_dma16(uint32_t lds, const void* src)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(lds), "v"(src) : "memory");
}

// One launch group addresses at most this many (layer, K|V) slabs; their base
// pointers travel by value in the kernel arguments.
constexpr int kMaxSlabs = 192;

struct SlabTable {
    char* base[kMaxSlabs];
};

// Tile constants of the fp16-MFMA contraction.
constexpr int kColTile   = 128;   // virtual columns per workgroup tile
constexpr int kKStage    = 32;    // contraction rows staged per pipeline step
constexpr int kRowsFold  = 256;   // rows per parity per workgroup tile (folded variant)
constexpr int kRowsPlain = 512;   // rows per workgroup tile (plain variant)

// Geometry of one pass (by-value kernel argument).
struct Geom {
    int n;               // span length
    int Lc;              // retained length
    int S;               // sink rows
    int d;               // head_dim
    int hts_per_slab;    // batch * n_heads
    int n_heads;
    int ncols;           // virtual columns in this pass = slabs * hts_per_slab * d
    int ncoltiles;       // ceil(ncols / kColTile)
    int fold;            // 1: even/odd folded operator, 0: plain
    int high;            // 0: the Lc lowest coefficients are kept, 1: the highest (ablation variant),
                         // 2: forward transform only, all n coefficients (power spectrum)
    float spec_scale;    // power spectrum: 1 / (batch * head_dim)
    // two-level fold (l2 != 0): this Geom describes one of its two launches
    int l2;              // 0: not used, 1: even part (folded again, n = n0/2, Lc = Lc0/2), 2: odd part (plain)
    int n0, Lc0;         // span and retained length of the full problem
    int H;               // n0/4 rounded up to a pipeline stage: half the contraction length of the odd part
    const _Float16* ebuf; // odd part: fp16 even part E[head-tensor][Lc0/2][d] written by the first launch
    const uint32_t* hmax; // per head-tensor of this pass: largest bf16 magnitude (bit pattern) of its span, or null:
                          // the span is scaled by a power of two on its way into the fp16 workspace (range guard)
    int Kh;              // contraction length: n/2 (fold) or n
    int Kpad;            // Kh rounded up to kKStage
    int nkstages;        // Kpad / kKStage
    int Mh;              // output rows per parity: Lc/2 (fold) or Lc
    int Mpad;            // Mh rounded up to the workgroup tile
    int Grows;           // rows of the stored basis: 2*Mpad (fold) or Mpad
    int nmtiles;         // Mpad / tile rows
    long long stride_batch, stride_head, stride_token;   // elements
    long long tap_slab0; // index of this pass's first slab in the caller's [2][n_layers] order
};

// Byte address of (token 0, channel c) of the head-tensor that owns virtual column vcol.
__device__ __forceinline__ char* column_base(const SlabTable& tab, const Geom& g, int vcol,
                                             int elem_bytes, int* ht_out)
{
    int ht   = vcol / g.d;
    int c    = vcol - ht * g.d;
    int slab = ht / g.hts_per_slab;
    int r    = ht - slab * g.hts_per_slab;
    int b    = r / g.n_heads;
    int h    = r - b * g.n_heads;
    if (ht_out) *ht_out = ht;
    long long off = (long long)b * g.stride_batch + (long long)h * g.stride_head + c;
    return tab.base[slab] + off * elem_bytes;
}

enum Variant { kNone = 0, kFoldF16 = 1, kPlainF16 = 2, kF32 = 3, kDrop = 4, kFold2F16 = 5, kFast = 6 };

// ---- basis construction (fp64 closed form, rounded once) -------------------------
// G: [Kpad/8][Grows][8] fp16.  Folded: rows [0,Mpad) even part, rows [Mpad,2Mpad) odd part.
hipError_t launch_basis_f16(_Float16* G, const Geom& g, int rescale, hipStream_t st);
// Mf: [Lc][n] fp32 row-major.
hipError_t launch_basis_f32(float* Mf, int n, int Lc, int rescale, int band, hipStream_t st);

// Power of two that brings a head-tensor whose largest bf16 magnitude has the bit pattern `amax` into
// [2^11, 2^12): sums of four such values stay far below the fp16 limit, and nothing but values 2^-25 of the
// largest falls into fp16's subnormal range.  Returns the exponent e (scale 2^e); 0 for all-zero, inf or nan.
__device__ __forceinline__ int guard_exponent(uint32_t amax)
{
    const int E = (int)(amax >> 7) & 0xff;
    if (E == 0 || E == 255) return 0;
    int e = 138 - E;
    return e > 120 ? 120 : e;
}
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }

// ---- bf16 cache: largest magnitude per head-tensor (zero hmax first), fold/convert the span, contract
hipError_t launch_absmax_bf16(const SlabTable& tab, const Geom& g, uint32_t* hmax, hipStream_t st);

// elem_bytes 4: the cache holds float32 (power spectrum of fp32 caches only)
hipError_t launch_prepare_bf16(const SlabTable& tab, const Geom& g, _Float16* ws, hipStream_t st, int elem_bytes = 2);
// mode 0: rows into the cache; 1: power-spectrum epilogue, tap = spectrum lines [slab][head][n] (atomics);
// 2: even part of the two-level fold, fp16 rows into the buffer passed as tap, nothing else; 3: odd part, combined with g.ebuf into the cache
hipError_t launch_contract_f16(const SlabTable& tab, const Geom& g, const _Float16* G,
                               const _Float16* ws, float* tap, int mode, hipStream_t st);
// two-level fold: gA = geometry of the even-part launch; wsA folded layout (xee | xeo), wsB plain layout (xo)
hipError_t launch_prepare_bf16_l2(const SlabTable& tab, const Geom& gA, _Float16* wsA, _Float16* wsB, hipStream_t st);
hipError_t launch_fill_zero(float* p, size_t count, hipStream_t st);

// ---- fp32 cache ------------------------------------------------------------------------
hipError_t launch_prepare_f32(const SlabTable& tab, const Geom& g, float* ws, hipStream_t st);
hipError_t launch_contract_f32(const SlabTable& tab, const Geom& g, const float* Mf,
                               const float* ws, float* tap, hipStream_t st);

// ---- factored transform (spans n = 4pq, Lc = n/2, bf16 caches): one kernel, no workspace ------------------
// Is there a compiled kernel for this span and head_dim?  (p, q) are the coprime odd factors of n/4, `channels`
// the channels of a head-tensor one workgroup owns (head_dim is a multiple of it).
bool fast_supported(int n, int Lc, int head_dim, int* p, int* q, int* channels);
size_t fast_table_bytes(int n, int head_dim);         // stage matrices in fragment order + the middle step's maps
size_t fast_lds_halfs(int n, int head_dim);           // fp16 values of one workgroup's LDS image (diagnostics)
void fast_build_tables_host(int n, int head_dim, char* out);   // fp64, rounded once; `out` is host memory
// rest_scale: what is left of the operator's 1/n after the scaled stages (1/2; sqrt(n/Lc)/2 without the
// rescale of Eq. 3).  dump/stop: diagnostic, see the kernel; pass nullptr, 0.
hipError_t launch_fast(const SlabTable& tab, const Geom& g, const void* tables, float rest_scale, float* tap,
                       _Float16* dump, int stop, hipStream_t st);

// ---- tail move: rows [src, src+rows) -> [dst, dst+rows) of every head-tensor; ranges must not overlap
hipError_t launch_move_rows(const SlabTable& tab, const Geom& g, int elem_bytes, int src_row,
                            int dst_row, int rows, hipStream_t st);

// ---- calibration: plain 16-byte copy; register-only MFMA loop (16 x 32x32x16 f16 per iteration per wave)
hipError_t launch_calib_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
hipError_t launch_calib_mfma(float* out, int blocks, int iters, hipStream_t st);

// ---- decode attention over the compacted cache ---------------------------------------------------
// Geometry of one attention pass (by-value kernel argument).  A "unit" is one (layer, batch, KV head).
struct AttGeom {
    int d;                 // head_dim: 64, 128 or 256
    int G;                 // query heads per KV head
    int GT;                // query heads one workgroup handles together: 1, 2 or 4, divides G
    int n_kv;              // KV heads
    int units;             // layers in this pass * batch * n_kv
    int units_per_layer;   // batch * n_kv
    int cur_len;           // cached rows, >= 1 (with cur_lens: the longest sequence's, an upper bound)
    int q_pos;             // in-cache position of the query (with cur_lens: each sequence's last row)
    const int* cur_lens;   // optional device array [batch] of per-sequence cached rows, or null
    int P;                 // rotary pairs per lane, attend_pairs_per_lane(d)
    int rope;              // 1: rotate query and keys at read time, 0: plain dot products
    int n_split;           // row chunks per unit
    int chunk;             // rows per chunk, a multiple of 2 * attend_row_step(d)
    long long stride_batch, stride_head, stride_token;   // elements
    float qscale;          // log2(e) / sqrt(d)
};

// One rotary pair: its frequency and the rotation that advances the position by attend_row_step(d) rows.
struct RopeEntry {
    double theta;
    float cd, sd;
};

// Rotary pairs (and twice as many channels) one lane of the attention kernel owns.
constexpr int attend_pairs_per_lane(int d) { return d > 256 ? 8 : 4; }
// Rows between two consecutive rows handled by one lane group: 4 waves x 64 lanes / (lanes per row).
constexpr int attend_row_step(int d) { return 4 * 64 / (d / (2 * attend_pairs_per_lane(d))); }
// Waves per SIMD the compiler must leave room for (bounds the registers of a lane).
constexpr int attend_min_waves(int elem_bytes, int GT, int P) { return elem_bytes == 2 ? (P == 4 ? (GT == 1 ? 4 : 3) : 2) : (P == 4 ? 2 : 1); }

hipError_t launch_rope_table(RopeEntry* rt, int d, double base, hipStream_t st);
// tab.base[2*i] / [2*i+1]: K / V slab of the pass's i-th layer.  part_acc: [units*G][n_split][d] fp32,
// part_ml: [units*G][n_split][2] fp32 (running maximum in the exp2 domain, sum of weights).
hipError_t launch_attend_partial(const SlabTable& tab, const AttGeom& g, int elem_bytes, const void* q,
                                 const RopeEntry* rt, float* part_acc, float* part_ml, hipStream_t st);
hipError_t launch_attend_merge(const AttGeom& g, int elem_bytes, const float* part_acc, const float* part_ml,
                               void* out, float* lse, hipStream_t st);

// ---- chunk-wise (prefill) attention over the compacted cache ------------------------------------------
struct PrefillGeom {
    int d;                 // head_dim (128)
    int G;                 // query heads per KV head
    int n_kv;
    int units;             // layers in this pass * batch * n_kv
    int units_per_layer;   // batch * n_kv
    int cur_len;           // cached rows, the chunk's tokens included
    int q_len;             // tokens of the chunk = queries per head; they are the last q_len cached rows
    int q_pad;             // q_len rounded up to 32
    int q_blocks;          // q_pad / 32
    int key_tiles;         // ceil(cur_len / 32)
    int rope;
    long long stride_batch, stride_head, stride_token;   // elements
    float qscale;          // log2(e) / sqrt(d)
};

// cs: [cur_len][d/2] (cos, sin); Kr, Vt: [units][key_tiles] tiles of 32 keys x d fp16 in fragment order.
// q: dense [units*G][q_len][d] bf16, rotated inside the attention kernel.
hipError_t launch_prefill_prepare(const SlabTable& tab, const PrefillGeom& g, double rope_base, float2* cs,
                                  _Float16* Kr, _Float16* Vt, hipStream_t st);
hipError_t launch_attend_prefill(const PrefillGeom& g, const _Float16* Kr, const _Float16* Vt, const void* q, const float2* cs,
                                 void* out, float* lse, hipStream_t st);

}  // namespace freqkv
