// Host side of libfreqkv: argument checks, the buffer plan, the per-device basis cache and the
// launch sequence of one trigger.  Everything here is plain C ABI on the outside (freqkv.h).
#include "freqkv.h"
#include "freqkv_internal.h"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <vector>

using namespace freqkv;

namespace {

thread_local char g_last_error[256] = "";

void set_error(const char* what, hipError_t e)
{
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t _e = (expr);                         \
        if (_e != hipSuccess) {                         \
            set_error(#expr, _e);                       \
            return FREQKV_E_HIP;                        \
        }                                               \
    } while (0)

inline long long round_up(long long a, long long b) { return (a + b - 1) / b * b; }

// Sec. 3.3: L = gamma * N, floored to an integer, at least one row.
int retained_len(int n, double ratio)
{
    long long lc = (long long)std::floor(ratio * (double)n + 1e-9);
    if (lc < 1) lc = 1;
    if (lc > n) lc = n;
    return (int)lc;
}

struct Shape {
    int n, Lc, S, W, d, n_heads, batch, n_layers, cur_len, tail;
    int variant;
    int high;                 // 1: FREQKV_FLAG_RETAIN_HIGH
    int elem;                 // bytes per cache element
    long long hts_per_slab;   // batch * n_heads
    int nslabs;               // 2 * n_layers
};

// Geometry for a pass over `slabs` slabs (static part depends only on the shape).
Geom make_geom(const Shape& sh, const freqkv_layout_t& L, int slabs, int slab0)
{
    Geom g;
    memset(&g, 0, sizeof(g));
    g.n = sh.n; g.Lc = sh.Lc; g.S = sh.S; g.d = sh.d;
    g.hts_per_slab = (int)sh.hts_per_slab;
    g.n_heads = sh.n_heads;
    g.ncols = (int)((long long)slabs * sh.hts_per_slab * sh.d);
    g.ncoltiles = (g.ncols + kColTile - 1) / kColTile;
    g.fold = sh.variant == kFoldF16;
    g.high = sh.high;
    if (sh.variant == kFoldF16) {
        g.Kh = sh.n / 2; g.Mh = sh.Lc / 2;
        g.Mpad = (int)round_up(g.Mh, kRowsFold);
        g.Grows = 2 * g.Mpad;
        g.nmtiles = g.Mpad / kRowsFold;
    } else {
        g.Kh = sh.n; g.Mh = sh.Lc;
        g.Mpad = (int)round_up(g.Mh, kRowsPlain);
        g.Grows = g.Mpad;
        g.nmtiles = g.Mpad / kRowsPlain;
    }
    g.Kpad = (int)round_up(g.Kh, kKStage);
    g.nkstages = g.Kpad / kKStage;
    g.n0 = sh.n; g.Lc0 = sh.Lc;
    g.stride_batch = L.stride_batch; g.stride_head = L.stride_head; g.stride_token = L.stride_token;
    g.tap_slab0 = slab0;
    return g;
}

// Two-level fold: geometry of the even-part launch (which = 1) or the odd-part launch (which = 2).
Geom make_geom_l2(const Shape& sh, const freqkv_layout_t& L, int slabs, int slab0, int which)
{
    Geom g;
    memset(&g, 0, sizeof(g));
    const int n4 = sh.n / 4, L2 = sh.Lc / 2;
    g.n = sh.n / 2; g.Lc = L2; g.S = sh.S; g.d = sh.d;
    g.hts_per_slab = (int)sh.hts_per_slab;
    g.n_heads = sh.n_heads;
    g.ncols = (int)((long long)slabs * sh.hts_per_slab * sh.d);
    g.ncoltiles = (g.ncols + kColTile - 1) / kColTile;
    g.high = sh.high;
    g.l2 = which; g.n0 = sh.n; g.Lc0 = sh.Lc;
    g.H = (int)round_up(n4, kKStage);
    if (which == 1) {
        g.fold = 1;
        g.Kh = n4; g.Kpad = g.H;
        g.Mh = (L2 + 1) / 2;                       // an odd Lc/2 has a middle row that pairs with itself
        g.Mpad = (int)round_up(g.Mh, kRowsFold);
        g.Grows = 2 * g.Mpad;
        g.nmtiles = g.Mpad / kRowsFold;
    } else {
        g.fold = 0;
        g.Kh = 2 * g.H; g.Kpad = 2 * g.H;
        g.Mh = L2;
        g.Mpad = (int)round_up(g.Mh, kRowsPlain);
        g.Grows = g.Mpad;
        g.nmtiles = g.Mpad / kRowsPlain;
    }
    g.nkstages = g.Kpad / kKStage;
    g.stride_batch = L.stride_batch; g.stride_head = L.stride_head; g.stride_token = L.stride_token;
    g.tap_slab0 = slab0;
    return g;
}

// Workspace slices of the two-level fold for a pass over `slabs` slabs: folded span of the even part,
// plain span of the odd part, fp16 even part.
struct L2Slices { size_t off_b, off_e, total; };
L2Slices l2_slices(const Shape& sh, int slabs)
{
    const long long ncols = (long long)slabs * sh.hts_per_slab * sh.d;
    const long long ncoltiles = (ncols + kColTile - 1) / kColTile;
    const long long nksA = round_up(sh.n / 4, kKStage) / kKStage;
    L2Slices s;
    s.off_b = (size_t)(ncoltiles * nksA * 2 * 8192);
    s.off_e = s.off_b + (size_t)(ncoltiles * (2 * nksA) * 8192);
    s.total = s.off_e + (size_t)round_up((long long)slabs * sh.hts_per_slab * (sh.Lc / 2) * sh.d * 2, 256);
    return s;
}

// Byte offset of the odd-part basis inside the two-level allocation.
size_t l2_basis_offset(const Shape& sh)
{
    const long long H = round_up(sh.n / 4, kKStage);
    const long long MpA = round_up((sh.Lc / 2 + 1) / 2, kRowsFold);
    return (size_t)((H / 8) * (2 * MpA) * 16);
}

size_t basis_bytes(const Shape& sh, const Geom& g)
{
    if (sh.variant == kFold2F16) {
        // even part then odd part, one allocation
        const long long H = round_up(sh.n / 4, kKStage);
        const long long MpA = round_up((sh.Lc / 2 + 1) / 2, kRowsFold), MpB = round_up(sh.Lc / 2, kRowsPlain);
        return (size_t)((H / 8) * (2 * MpA) * 16 + (2 * H / 8) * MpB * 16);
    }
    if (sh.variant == kF32) return (size_t)sh.n * sh.Lc * sizeof(float);
    if (sh.variant == kNone) return 0;
    if (sh.variant == kFast) return fast_table_bytes(sh.n, sh.d);
    return (size_t)(g.Kpad / 8) * g.Grows * 16;
}

// Workspace bytes of a pass over `slabs` slabs without the range guard's table.
size_t pass_workspace_core(const Shape& sh, int slabs)
{
    if (sh.variant == kFast) return 0;
    if (sh.variant == kFold2F16) return l2_slices(sh, slabs).total;
    long long ncols = (long long)slabs * sh.hts_per_slab * sh.d;
    if (sh.variant == kF32) return (size_t)sh.n * (size_t)round_up(ncols, 64) * sizeof(float);
    int P = sh.variant == kFoldF16 ? 2 : 1;
    long long Kh = sh.variant == kFoldF16 ? sh.n / 2 : sh.n;
    long long nks = round_up(Kh, kKStage) / kKStage;
    long long ncoltiles = (ncols + kColTile - 1) / kColTile;
    return (size_t)ncoltiles * nks * P * 8192;
}

// The fp16 forms keep, behind everything else, one 32-bit word per head-tensor of the pass: the largest
// magnitude of its span, from which the power-of-two scale of the range guard is derived.
bool has_range_guard(const Shape& sh) { return sh.variant == kFoldF16 || sh.variant == kPlainF16 || sh.variant == kFold2F16; }

// Workspace bytes for a pass over `slabs` slabs.
size_t pass_workspace(const Shape& sh, int slabs)
{
    size_t core = (size_t)round_up((long long)pass_workspace_core(sh, slabs), 256);
    if (!has_range_guard(sh)) return core;
    return core + (size_t)round_up((long long)slabs * sh.hts_per_slab * 4, 256);
}

// The two-level fold saves a quarter of the multiply-adds but runs two shorter launches and moves the even
// part through a buffer.  Measured per trigger: 1.96 vs 2.35 ms (8188-row span, 512 head-tensors), 2.66 vs 2.89
// (4092 rows, 2048 head-tensors), 22.0 vs 24.3 (4092 rows, 16384 head-tensors), but 0.133 vs 0.114 for a single
// layer of 64 head-tensors, whose even-part launch has only 128 workgroups for 256 compute units.  So it is
// the default when the span has at least kTwoLevelMinSpan rows and the even-part launch at least
// kTwoLevelMinTiles workgroups.
constexpr int kTwoLevelMinSpan = 2048;
constexpr long long kTwoLevelMinTiles = 512;

freqkv_status_t check_shape(const freqkv_layout_t* L, int n_heads, int head_dim, int cur_len, int window,
                            int n_sink, double ratio, Shape* out)
{
    if (!L) return FREQKV_E_INVALID;
    if (L->dtype != FREQKV_BF16 && L->dtype != FREQKV_F32) return FREQKV_E_INVALID;
    if (L->n_layers < 1 || L->batch < 1 || n_heads < 1) return FREQKV_E_INVALID;
    if (head_dim < 8) return FREQKV_E_INVALID;
    if (head_dim % 8 != 0) return FREQKV_E_UNSUPPORTED;
    if (n_sink < 0 || window < n_sink + 2) return FREQKV_E_INVALID;
    if (cur_len < 0 || cur_len > L->token_capacity) return FREQKV_E_INVALID;
    if (!(ratio > 0.0) || !(ratio <= 1.0)) return FREQKV_E_INVALID;      // also rejects NaN
    if (L->pointer_table != 0 && L->pointer_table != 1) return FREQKV_E_INVALID;
    if (L->flags & ~(FREQKV_FLAG_NO_RESCALE | FREQKV_FLAG_DROPPING | FREQKV_FLAG_RETAIN_HIGH | FREQKV_FLAG_SINGLE_FOLD | FREQKV_FLAG_TWO_LEVEL_FOLD | FREQKV_FLAG_DENSE)) return FREQKV_E_INVALID;
    if ((L->flags & FREQKV_FLAG_DROPPING) && (L->flags & FREQKV_FLAG_RETAIN_HIGH)) return FREQKV_E_INVALID;
    if ((L->flags & FREQKV_FLAG_SINGLE_FOLD) && (L->flags & FREQKV_FLAG_TWO_LEVEL_FOLD)) return FREQKV_E_INVALID;
    if (L->stride_token < head_dim) return FREQKV_E_INVALID;
    if (L->stride_token % 8 || L->stride_head % 8 || L->stride_batch % 8) return FREQKV_E_INVALID;
    if (!L->pointer_table && L->stride_layer % 8) return FREQKV_E_INVALID;
    if (L->stride_head < 0 || L->stride_batch < 0) return FREQKV_E_INVALID;
    if (window - n_sink > (1 << 20)) return FREQKV_E_UNSUPPORTED;        // 64-bit angle reduction of the basis
    long long hts = (long long)L->batch * n_heads;
    if (hts * head_dim > (1LL << 30) / 192) return FREQKV_E_UNSUPPORTED; // virtual column index stays in int
    if (L->n_layers > (1 << 20)) return FREQKV_E_UNSUPPORTED;

    Shape sh;
    sh.W = window; sh.S = n_sink; sh.n = window - n_sink;
    sh.Lc = retained_len(sh.n, ratio);
    sh.d = head_dim; sh.n_heads = n_heads; sh.batch = L->batch; sh.n_layers = L->n_layers;
    sh.cur_len = cur_len;
    sh.tail = cur_len >= window ? cur_len - window : 0;
    sh.elem = L->dtype == FREQKV_BF16 ? 2 : 4;
    sh.hts_per_slab = hts;
    sh.nslabs = 2 * L->n_layers;
    sh.high = (L->flags & FREQKV_FLAG_RETAIN_HIGH) ? 1 : 0;
    if (sh.Lc == sh.n) sh.variant = kNone;
    else if (L->flags & FREQKV_FLAG_DROPPING) sh.variant = kDrop;
    else if (L->dtype == FREQKV_F32) sh.variant = kF32;
    else if (!sh.high && !(L->flags & (FREQKV_FLAG_DENSE | FREQKV_FLAG_SINGLE_FOLD | FREQKV_FLAG_TWO_LEVEL_FOLD)) &&
             fast_supported(sh.n, sh.Lc, head_dim, nullptr, nullptr, nullptr) &&
             (long long)window * L->stride_token * 2 < (1LL << 32))       // its rows are addressed by 32-bit byte offsets
        sh.variant = kFast;
    else if (sh.n % 4 == 0 && sh.Lc % 2 == 0 && !(L->flags & FREQKV_FLAG_SINGLE_FOLD)) {
        // workgroups of the even-part launch over all slabs: column tiles x row tiles of 256 rows per parity
        const long long coltiles = ((long long)sh.nslabs * hts * head_dim + kColTile - 1) / kColTile;
        const long long rowtiles = ((sh.Lc / 2 + 1) / 2 + kRowsFold - 1) / kRowsFold;
        const bool pays = sh.n >= kTwoLevelMinSpan && coltiles * rowtiles >= kTwoLevelMinTiles;
        sh.variant = (pays || (L->flags & FREQKV_FLAG_TWO_LEVEL_FOLD)) ? kFold2F16 : kFoldF16;
    }
    else sh.variant = (sh.n % 2 == 0 && sh.Lc % 2 == 0) ? kFoldF16 : kPlainF16;
    *out = sh;
    return FREQKV_OK;
}

// ---------------------------------------------------------------- basis cache
struct BasisKey {
    int device, n, Lc, variant, rescale, high;
    bool operator<(const BasisKey& o) const
    {
        return std::tie(device, n, Lc, variant, rescale, high) <
               std::tie(o.device, o.n, o.Lc, o.variant, o.rescale, o.high);
    }
};
struct BasisEntry {
    void* ptr = nullptr;
    size_t bytes = 0;
    hipEvent_t ready = nullptr;   // recorded after the build kernel; other streams wait on it
    void* host = nullptr;         // pinned staging copy of tables built on the host (kept until shutdown)
};

std::mutex g_mu;
std::map<BasisKey, BasisEntry> g_basis;

freqkv_status_t get_basis(const Shape& sh, const Geom& g, int rescale, hipStream_t st, void** out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    BasisKey key{dev, sh.n, sh.Lc, sh.variant, rescale, sh.high};
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_basis.find(key);
    if (it == g_basis.end()) {
        BasisEntry e;
        e.bytes = basis_bytes(sh, g);
        hipError_t err = hipMalloc(&e.ptr, e.bytes);
        if (err != hipSuccess) {
            set_error("hipMalloc(basis)", err);
            (void)hipGetLastError();
            return FREQKV_E_ALLOC;
        }
        if (sh.variant == kFast) {
            // built on the host in fp64, copied from pinned memory in stream order (no synchronisation)
            err = hipHostMalloc(&e.host, e.bytes, hipHostMallocDefault);
            if (err == hipSuccess) {
                fast_build_tables_host(sh.n, sh.d, (char*)e.host);
                err = hipMemcpyAsync(e.ptr, e.host, e.bytes, hipMemcpyHostToDevice, st);
            }
        } else if (sh.variant == kF32) {
            err = launch_basis_f32((float*)e.ptr, sh.n, sh.Lc, rescale, sh.high, st);
        } else if (sh.variant == kFold2F16) {
            freqkv_layout_t L0;
            memset(&L0, 0, sizeof(L0));
            Geom gA = make_geom_l2(sh, L0, 1, 0, 1), gB = make_geom_l2(sh, L0, 1, 0, 2);
            err = launch_basis_f16((_Float16*)e.ptr, gA, rescale, st);
            if (err == hipSuccess)
                err = launch_basis_f16((_Float16*)((char*)e.ptr + l2_basis_offset(sh)), gB, rescale, st);
        } else {
            err = launch_basis_f16((_Float16*)e.ptr, g, rescale, st);
        }
        if (err == hipSuccess) err = hipEventCreateWithFlags(&e.ready, hipEventDisableTiming);
        if (err == hipSuccess) err = hipEventRecord(e.ready, st);
        if (err != hipSuccess) {
            set_error("basis build", err);
            (void)hipFree(e.ptr);
            if (e.host) (void)hipHostFree(e.host);
            return FREQKV_E_HIP;
        }
        it = g_basis.emplace(key, e).first;
    } else {
        // built on some stream earlier: order this stream after the build
        HIP_TRY(hipStreamWaitEvent(st, it->second.ready, 0));
    }
    *out = it->second.ptr;
    return FREQKV_OK;
}

// ---------------------------------------------------------------- attention: shape, plan, rotary table
constexpr long long kAttendTargetWgs = 768;   // 256 compute units x 3 resident workgroups

struct AttShape {
    int d, n_q, n_kv, G, GT, batch, n_layers, cur_len, elem;
    int n_split, chunk;
    long long units_all;        // n_layers * batch * n_kv
    size_t ml_offset;           // byte offset of the (max, sum) region inside the workspace
    size_t workspace_bytes;
};

freqkv_status_t check_attend(const freqkv_layout_t* L, int n_q, int n_kv, int d, int cur_len, AttShape* out)
{
    if (!L) return FREQKV_E_INVALID;
    if (L->dtype != FREQKV_BF16 && L->dtype != FREQKV_F32) return FREQKV_E_INVALID;
    if (L->n_layers < 1 || L->batch < 1 || n_kv < 1 || n_q < 1 || n_q % n_kv) return FREQKV_E_INVALID;
    if (d < 8) return FREQKV_E_INVALID;
    if (d != 64 && d != 128 && d != 256) return FREQKV_E_UNSUPPORTED;
    if (cur_len < 1 || cur_len > L->token_capacity) return FREQKV_E_INVALID;
    if (L->pointer_table != 0 && L->pointer_table != 1) return FREQKV_E_INVALID;
    if (L->flags & ~(FREQKV_FLAG_NO_RESCALE | FREQKV_FLAG_DROPPING | FREQKV_FLAG_RETAIN_HIGH | FREQKV_FLAG_SINGLE_FOLD | FREQKV_FLAG_TWO_LEVEL_FOLD | FREQKV_FLAG_DENSE)) return FREQKV_E_INVALID;
    if (L->stride_token < d) return FREQKV_E_INVALID;
    if (L->stride_token % 8 || L->stride_head % 8 || L->stride_batch % 8) return FREQKV_E_INVALID;
    if (!L->pointer_table && L->stride_layer % 8) return FREQKV_E_INVALID;
    if (L->stride_head < 0 || L->stride_batch < 0) return FREQKV_E_INVALID;
    if (L->n_layers > (1 << 20)) return FREQKV_E_UNSUPPORTED;
    long long units = (long long)L->n_layers * L->batch * n_kv;
    if (units * (n_q / n_kv) > (1LL << 24)) return FREQKV_E_UNSUPPORTED;    // grid and index ranges
    // the attention kernels address the rows of one head by 32-bit byte offsets (a few steps past cur_len included)
    if (((long long)cur_len + 1024) * L->stride_token * (L->dtype == FREQKV_BF16 ? 2 : 4) >= (1LL << 32)) return FREQKV_E_UNSUPPORTED;

    AttShape a;
    a.d = d; a.n_q = n_q; a.n_kv = n_kv; a.G = n_q / n_kv;
    a.GT = a.G % 4 == 0 ? 4 : (a.G % 2 == 0 ? 2 : 1);
    a.batch = L->batch; a.n_layers = L->n_layers; a.cur_len = cur_len;
    a.elem = L->dtype == FREQKV_BF16 ? 2 : 4;
    a.units_all = units;
    // Row chunks: a chunk is at least eight loop steps long; the number of chunks is chosen so that the
    // workgroups fill the resident slots of the 256 compute units about once (few, long workgroups: the
    // set-up and the final combination of a workgroup cost several microseconds).
    const int step = attend_row_step(d);
    const long long wgs_per_split = units * (a.G / a.GT);
    long long ns = (kAttendTargetWgs + wgs_per_split / 2) / wgs_per_split;
    long long ns_max = cur_len / (16 * step);
    if (ns > ns_max) ns = ns_max;
    if (ns < 1) ns = 1;
    long long chunk = round_up(((long long)cur_len + ns - 1) / ns, 2 * step);
    ns = ((long long)cur_len + chunk - 1) / chunk;
    if (wgs_per_split * ns > (1LL << 30)) return FREQKV_E_UNSUPPORTED;
    a.n_split = (int)ns; a.chunk = (int)chunk;
    size_t acc_bytes = (size_t)units * a.G * ns * d * sizeof(float);
    a.ml_offset = (size_t)round_up((long long)acc_bytes, 256);
    a.workspace_bytes = a.ml_offset + (size_t)units * a.G * ns * 2 * sizeof(float);
    *out = a;
    return FREQKV_OK;
}

struct RopeKey {
    int device, d;
    double base;
    bool operator<(const RopeKey& o) const { return std::tie(device, d, base) < std::tie(o.device, o.d, o.base); }
};
std::map<RopeKey, BasisEntry> g_rope;

freqkv_status_t get_rope_table(int d, double base, hipStream_t st, RopeEntry** out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    RopeKey key{dev, d, base};
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_rope.find(key);
    if (it == g_rope.end()) {
        BasisEntry e;
        e.bytes = (size_t)(d / 2) * sizeof(RopeEntry);
        hipError_t err = hipMalloc(&e.ptr, e.bytes);
        if (err != hipSuccess) {
            set_error("hipMalloc(rotary table)", err);
            (void)hipGetLastError();
            return FREQKV_E_ALLOC;
        }
        err = launch_rope_table((RopeEntry*)e.ptr, d, base, st);
        if (err == hipSuccess) err = hipEventCreateWithFlags(&e.ready, hipEventDisableTiming);
        if (err == hipSuccess) err = hipEventRecord(e.ready, st);
        if (err != hipSuccess) {
            set_error("rotary table build", err);
            (void)hipFree(e.ptr);
            return FREQKV_E_HIP;
        }
        it = g_rope.emplace(key, e).first;
    } else {
        HIP_TRY(hipStreamWaitEvent(st, it->second.ready, 0));
    }
    *out = (RopeEntry*)it->second.ptr;
    return FREQKV_OK;
}

// ---------------------------------------------------------------- static scratch of the entry point that allocates nothing
// freqkv_attend_decode_noalloc keeps the per-chunk softmax states and the rotary table here instead of in a
// caller's workspace and a cached allocation.  Every device the library runs on holds its own copy of the
// array until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device, with that device current, and only that pointer is ever
// handed to a kernel.
constexpr size_t kScratchBytes = (size_t)8 << 20;
constexpr size_t kScratchRopeBytes = 4096;            // rotary table of up to 256 channels (128 entries x 16 B)
constexpr int kScratchMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
void* g_scratch_ptr[kScratchMaxDevices] = {};

freqkv_status_t scratch_for_current_device(void** out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kScratchMaxDevices) return FREQKV_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) {
            snprintf(g_last_error, sizeof(g_last_error), "static scratch: bad device address %p", ptr);
            return FREQKV_E_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FREQKV_OK;
}

// ---------------------------------------------------------------- profiling
struct ProfSpan { hipEvent_t a, b; int kind; };
std::atomic<bool> g_prof_on{false};
std::vector<ProfSpan> g_prof_spans;
freqkv_profile_t g_prof_acc;

hipError_t prof_begin(hipStream_t st, int kind, ProfSpan* sp)
{
    sp->kind = kind; sp->a = sp->b = nullptr;
    if (!g_prof_on) return hipSuccess;
    hipError_t e = hipEventCreate(&sp->a);
    if (e == hipSuccess) e = hipEventCreate(&sp->b);
    if (e == hipSuccess) e = hipEventRecord(sp->a, st);
    if (e != hipSuccess) {                       // nothing half-made is left behind
        if (sp->a) (void)hipEventDestroy(sp->a);
        if (sp->b) (void)hipEventDestroy(sp->b);
        sp->a = sp->b = nullptr;
    }
    return e;
}
hipError_t prof_end(hipStream_t st, ProfSpan* sp)
{
    if (!g_prof_on || !sp->a) return hipSuccess;
    hipError_t e = hipEventRecord(sp->b, st);
    std::lock_guard<std::mutex> lock(g_mu);
    g_prof_spans.push_back(*sp);
    return e;
}

// Two timing events, destroyed on every path out of the calibration calls.
struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t create()
    {
        hipError_t e = hipEventCreate(&a);
        if (e == hipSuccess) e = hipEventCreate(&b);
        return e;
    }
    ~EventPair()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

}  // namespace

// ================================================================== C ABI

extern "C" {

const char* freqkv_status_string(freqkv_status_t s)
{
    switch (s) {
        case FREQKV_OK: return "FREQKV_OK";
        case FREQKV_NOOP: return "FREQKV_NOOP";
        case FREQKV_E_INVALID: return "FREQKV_E_INVALID";
        case FREQKV_E_UNSUPPORTED: return "FREQKV_E_UNSUPPORTED";
        case FREQKV_E_WORKSPACE: return "FREQKV_E_WORKSPACE";
        case FREQKV_E_HIP: return "FREQKV_E_HIP";
        case FREQKV_E_ALLOC: return "FREQKV_E_ALLOC";
    }
    return "FREQKV_E_UNKNOWN";
}

const char* freqkv_last_error(void) { return g_last_error; }

int freqkv_version(void) { return 200; }

freqkv_status_t freqkv_plan(const freqkv_layout_t* layout, int n_heads, int head_dim, int cur_len,
                            int window, int n_sink, double retain_ratio, freqkv_plan_t* out)
{
    if (!out) return FREQKV_E_INVALID;
    Shape sh;
    freqkv_status_t rc = check_shape(layout, n_heads, head_dim, cur_len, window, n_sink, retain_ratio, &sh);
    if (rc < 0) return rc;
    memset(out, 0, sizeof(*out));
    out->span_len = sh.n;
    out->retained_len = sh.Lc;
    out->new_len = sh.S + sh.Lc + sh.tail;
    out->head_tensors = (int)(sh.nslabs * sh.hts_per_slab);
    out->variant = sh.variant;
    double hts = (double)sh.nslabs * (double)sh.hts_per_slab;
    if (sh.variant == kDrop) {
        out->bytes_algorithmic = (2.0 * sh.Lc + 2.0 * sh.tail) * sh.d * sh.elem * hts;
    } else if (sh.variant != kNone) {
        Geom g = make_geom(sh, *layout, sh.nslabs, 0);
        int max_slabs = sh.nslabs < kMaxSlabs ? sh.nslabs : kMaxSlabs;
        out->workspace_bytes = pass_workspace(sh, max_slabs);
        out->workspace_min_bytes = pass_workspace(sh, 1);
        out->basis_bytes = basis_bytes(sh, g);
        out->flops_dense = 2.0 * sh.Lc * (double)sh.n * sh.d * hts;
        out->flops_executed = sh.variant == kFoldF16 ? out->flops_dense * 0.5
                            : sh.variant == kFold2F16 ? out->flops_dense * 0.375 : out->flops_dense;
        if (sh.variant == kFast) {
            // multiply-adds of the four matrix stages and the middle step, per channel, padding not counted
            int p = 0, q = 0;
            fast_supported(sh.n, sh.Lc, sh.d, &p, &q, nullptr);
            const double qh = (q + 1) / 2;
            const double per_channel = 2.0 * (4.0 * p * q * 2 * qh + 4.0 * qh * 4.0 * p * p + 16.0 * p * qh +
                                              2.0 * qh * 4.0 * p * p + 2.0 * p * 2 * qh * q);
            out->flops_executed = per_channel * sh.d * hts;
        }
        out->bytes_algorithmic = ((double)sh.n + sh.Lc + 2.0 * sh.tail) * sh.d * sh.elem * hts;
    }
    return cur_len < window ? FREQKV_NOOP : FREQKV_OK;
}

freqkv_status_t freqkv_prepare(int dtype, uint32_t flags, int window, int n_sink, double retain_ratio,
                               void* stream)
{
    freqkv_layout_t L;
    memset(&L, 0, sizeof(L));
    L.dtype = dtype; L.n_layers = 1; L.batch = 1; L.token_capacity = window;
    L.stride_token = 8; L.flags = flags;
    Shape sh;
    freqkv_status_t rc = check_shape(&L, 1, 8, window, window, n_sink, retain_ratio, &sh);
    if (rc < 0) return rc;
    if (sh.variant == kNone || sh.variant == kDrop) return FREQKV_OK;
    Geom g = make_geom(sh, L, 1, 0);
    void* basis = nullptr;
    int key = !(flags & FREQKV_FLAG_NO_RESCALE);
    if (sh.variant == kFast) fast_supported(sh.n, sh.Lc, sh.d, nullptr, nullptr, &key);   // keyed by channels per workgroup
    return get_basis(sh, g, key, (hipStream_t)stream, &basis);
}

namespace {

// Base pointers of every (K|V, layer) slab in [K|V][layer] order, each moved forward by `batch0` sequences.
freqkv_status_t resolve_bases(void* k, void* v, const freqkv_layout_t& L, const Shape& sh, int batch0,
                              std::vector<char*>* out)
{
    out->assign((size_t)sh.nslabs, nullptr);
    for (int kv = 0; kv < 2; ++kv) {
        void* root = kv ? v : k;
        for (int l = 0; l < sh.n_layers; ++l) {
            char* p = L.pointer_table ? (char*)((void* const*)root)[l]
                                      : (char*)root + (long long)l * L.stride_layer * sh.elem;
            if (!p || ((uintptr_t)p & 15)) return FREQKV_E_INVALID;
            (*out)[(size_t)kv * sh.n_layers + l] = p + (long long)batch0 * L.stride_batch * sh.elem;
        }
    }
    return FREQKV_OK;
}

// One trigger over sh.batch sequences that share cur_len; `bases` already point at the first of them.
freqkv_status_t compress_resolved(const std::vector<char*>& bases, const freqkv_layout_t& L, const Shape& sh,
                                  float* tap, hipStream_t st)
{
    if (sh.cur_len < sh.W) return FREQKV_NOOP;
    if (sh.variant == kNone) return FREQKV_OK;                // retain_ratio == 1: identity

    if (sh.variant == kDrop) {
        // Dropping: rows [W-Lc, W) -> [S, S+Lc), then the tail -> [S+Lc, ...); both in chunks of at most
        // (n - Lc) rows, the distance of the move, so that no chunk overlaps its own source.
        if (g_prof_on) { std::lock_guard<std::mutex> lock(g_mu); g_prof_acc.calls++; }
        const int gap = sh.n - sh.Lc;
        for (int s0 = 0; s0 < sh.nslabs; s0 += kMaxSlabs) {
            int slabs = sh.nslabs - s0 < kMaxSlabs ? sh.nslabs - s0 : kMaxSlabs;
            Geom g = make_geom(sh, L, slabs, s0);
            SlabTable tab;
            memset(&tab, 0, sizeof(tab));
            for (int i = 0; i < slabs; ++i) tab.base[i] = bases[(size_t)s0 + i];
            ProfSpan sp;
            HIP_TRY(prof_begin(st, 2, &sp));
            for (int r0 = 0; r0 < sh.Lc + sh.tail; r0 += gap) {
                int rows = sh.Lc + sh.tail - r0 < gap ? sh.Lc + sh.tail - r0 : gap;
                // rows [W-Lc, cur_len) are contiguous: the retained rows and the tail move by the same distance
                HIP_TRY(launch_move_rows(tab, g, sh.elem, sh.W - sh.Lc + r0, sh.S + r0, rows, st));
            }
            HIP_TRY(prof_end(st, &sp));
        }
        return FREQKV_OK;
    }

    const int rescale = !(L.flags & FREQKV_FLAG_NO_RESCALE);

    if (sh.variant == kFast) {
        // Factored transform: one kernel reads the span from the cache and writes the retained rows in place
        // (a workgroup owns its channels for all rows); the tail moves afterwards, when the span has been read.
        void* tables = nullptr;
        {
            Geom g0 = make_geom(sh, L, 1, 0);
            int channels = 8;
            fast_supported(sh.n, sh.Lc, sh.d, nullptr, nullptr, &channels);
            // the tables do not depend on the rescale; they do on the channels per workgroup (the p stage's
            // padding differs), which takes the key's place
            freqkv_status_t rc = get_basis(sh, g0, channels, st, &tables);
            if (rc < 0) return rc;
        }
        if (g_prof_on) { std::lock_guard<std::mutex> lock(g_mu); g_prof_acc.calls++; }
        const float rest = rescale ? 0.5f : (float)(0.5 * std::sqrt((double)sh.n / (double)sh.Lc));
        for (int s0 = 0; s0 < sh.nslabs; s0 += kMaxSlabs) {
            int slabs = sh.nslabs - s0 < kMaxSlabs ? sh.nslabs - s0 : kMaxSlabs;
            Geom g = make_geom(sh, L, slabs, s0);
            SlabTable tab;
            memset(&tab, 0, sizeof(tab));
            for (int i = 0; i < slabs; ++i) tab.base[i] = bases[(size_t)s0 + i];
            ProfSpan sp;
            HIP_TRY(prof_begin(st, 1, &sp));
            HIP_TRY(launch_fast(tab, g, tables, rest, tap, nullptr, 0, st));
            HIP_TRY(prof_end(st, &sp));
            if (sh.tail > 0) {
                HIP_TRY(prof_begin(st, 2, &sp));
                const int gap = sh.n - sh.Lc;
                for (int r0 = 0; r0 < sh.tail; r0 += gap) {
                    int rows = sh.tail - r0 < gap ? sh.tail - r0 : gap;
                    HIP_TRY(launch_move_rows(tab, g, sh.elem, sh.W + r0, sh.S + sh.Lc + r0, rows, st));
                }
                HIP_TRY(prof_end(st, &sp));
            }
        }
        return FREQKV_OK;
    }

    size_t min_ws = pass_workspace(sh, 1);
    if (!L.workspace || ((uintptr_t)L.workspace & 255) || L.workspace_bytes < min_ws) return FREQKV_E_WORKSPACE;

    // slabs per pass: as many as the workspace and the pointer table hold
    int per_pass = sh.nslabs < kMaxSlabs ? sh.nslabs : kMaxSlabs;
    while (per_pass > 1 && pass_workspace(sh, per_pass) > L.workspace_bytes) --per_pass;

    void* basis = nullptr;
    {
        Geom g0 = make_geom(sh, L, per_pass, 0);
        freqkv_status_t rc = get_basis(sh, g0, rescale, st, &basis);
        if (rc < 0) return rc;
    }
    if (g_prof_on) { std::lock_guard<std::mutex> lock(g_mu); g_prof_acc.calls++; }

    if (sh.variant == kFold2F16) {
        // Two-level fold: span -> (xee | xeo), xo;  E = Gee xee +/- Geo xeo into an fp16 buffer;  O = Go xo,
        // combined with E on its way into the cache.
        for (int s0 = 0; s0 < sh.nslabs; s0 += per_pass) {
            int slabs = sh.nslabs - s0 < per_pass ? sh.nslabs - s0 : per_pass;
            Geom gA = make_geom_l2(sh, L, slabs, s0, 1), gB = make_geom_l2(sh, L, slabs, s0, 2);
            const L2Slices sl = l2_slices(sh, slabs);
            _Float16* wsA = (_Float16*)L.workspace;
            _Float16* wsB = (_Float16*)((char*)L.workspace + sl.off_b);
            _Float16* ebuf = (_Float16*)((char*)L.workspace + sl.off_e);
            // the E buffer is indexed like a tap of this pass alone
            gA.tap_slab0 = 0;
            gB.ebuf = ebuf;
            uint32_t* hmax = (uint32_t*)((char*)L.workspace + round_up((long long)pass_workspace_core(sh, slabs), 256));
            gA.hmax = gB.hmax = hmax;
            SlabTable tab;
            memset(&tab, 0, sizeof(tab));
            for (int i = 0; i < slabs; ++i) tab.base[i] = bases[(size_t)s0 + i];
            ProfSpan sp;
            HIP_TRY(prof_begin(st, 0, &sp));
            HIP_TRY(launch_fill_zero((float*)hmax, (size_t)slabs * sh.hts_per_slab, st));
            HIP_TRY(launch_absmax_bf16(tab, gA, hmax, st));
            HIP_TRY(launch_prepare_bf16_l2(tab, gA, wsA, wsB, st));
            HIP_TRY(prof_end(st, &sp));
            if (sh.tail > 0) {
                HIP_TRY(prof_begin(st, 2, &sp));
                Geom gm = make_geom(sh, L, slabs, s0);
                const int gap = sh.n - sh.Lc;
                for (int r0 = 0; r0 < sh.tail; r0 += gap) {
                    int rows = sh.tail - r0 < gap ? sh.tail - r0 : gap;
                    HIP_TRY(launch_move_rows(tab, gm, sh.elem, sh.W + r0, sh.S + sh.Lc + r0, rows, st));
                }
                HIP_TRY(prof_end(st, &sp));
            }
            HIP_TRY(prof_begin(st, 1, &sp));
            HIP_TRY(launch_contract_f16(tab, gA, (const _Float16*)basis, wsA, (float*)ebuf, 2, st));
            HIP_TRY(launch_contract_f16(tab, gB, (const _Float16*)((const char*)basis + l2_basis_offset(sh)), wsB,
                                        tap, 3, st));
            HIP_TRY(prof_end(st, &sp));
        }
        return FREQKV_OK;
    }

    for (int s0 = 0; s0 < sh.nslabs; s0 += per_pass) {
        int slabs = sh.nslabs - s0 < per_pass ? sh.nslabs - s0 : per_pass;
        Geom g = make_geom(sh, L, slabs, s0);
        SlabTable tab;
        memset(&tab, 0, sizeof(tab));
        for (int i = 0; i < slabs; ++i) tab.base[i] = bases[(size_t)s0 + i];

        ProfSpan sp;
        // 1. span -> workspace (fold + convert, or copy); fp16 forms: first the largest magnitude per head-tensor
        HIP_TRY(prof_begin(st, 0, &sp));
        if (sh.variant == kF32) {
            HIP_TRY(launch_prepare_f32(tab, g, (float*)L.workspace, st));
        } else {
            uint32_t* hmax = (uint32_t*)((char*)L.workspace + round_up((long long)pass_workspace_core(sh, slabs), 256));
            g.hmax = hmax;
            HIP_TRY(launch_fill_zero((float*)hmax, (size_t)slabs * sh.hts_per_slab, st));
            HIP_TRY(launch_absmax_bf16(tab, g, hmax, st));
            HIP_TRY(launch_prepare_bf16(tab, g, (_Float16*)L.workspace, st));
        }
        HIP_TRY(prof_end(st, &sp));

        // 2. recent tail: rows [W, cur_len) -> [S+Lc, ...).  The span has been copied out, so the
        //    destination is free; chunks of at most (n - Lc) rows never overlap their source.
        if (sh.tail > 0) {
            HIP_TRY(prof_begin(st, 2, &sp));
            const int gap = sh.n - sh.Lc;
            for (int r0 = 0; r0 < sh.tail; r0 += gap) {
                int rows = sh.tail - r0 < gap ? sh.tail - r0 : gap;
                HIP_TRY(launch_move_rows(tab, g, sh.elem, sh.W + r0, sh.S + sh.Lc + r0, rows, st));
            }
            HIP_TRY(prof_end(st, &sp));
        }

        // 3. contraction, written straight into rows [S, S+Lc)
        HIP_TRY(prof_begin(st, 1, &sp));
        if (sh.variant == kF32)
            HIP_TRY(launch_contract_f32(tab, g, (const float*)basis, (const float*)L.workspace, tap, st));
        else
            HIP_TRY(launch_contract_f16(tab, g, (const _Float16*)basis, (const _Float16*)L.workspace, tap, 0, st));
        HIP_TRY(prof_end(st, &sp));
    }
    return FREQKV_OK;
}

}  // namespace

freqkv_status_t freqkv_compress(void* k, void* v, const freqkv_layout_t* layout, int n_heads, int head_dim,
                                int cur_len, int window, int n_sink, double retain_ratio, void* stream)
{
    g_last_error[0] = 0;
    Shape sh;
    freqkv_status_t rc = check_shape(layout, n_heads, head_dim, cur_len, window, n_sink, retain_ratio, &sh);
    if (rc < 0) return rc;
    if (!k || !v) return FREQKV_E_INVALID;
    std::vector<char*> bases;
    rc = resolve_bases(k, v, *layout, sh, 0, &bases);
    if (rc < 0) return rc;
    return compress_resolved(bases, *layout, sh, layout->tap_f32, (hipStream_t)stream);
}

freqkv_status_t freqkv_debug_fast_stage(void* k, void* v, const freqkv_layout_t* layout, int n_heads, int head_dim,
                                        int window, int n_sink, int stop, void* dump, size_t dump_bytes,
                                        void* stream)
{
    g_last_error[0] = 0;
    Shape sh;
    freqkv_status_t rc = check_shape(layout, n_heads, head_dim, window, window, n_sink, 0.5, &sh);
    if (rc < 0) return rc;
    if (!k || !v || !dump || stop < 1 || stop > 9 || stop == 6 || stop == 7) return FREQKV_E_INVALID;
    if (sh.variant != kFast) return FREQKV_E_UNSUPPORTED;
    int channels = 8;
    fast_supported(sh.n, sh.Lc, sh.d, nullptr, nullptr, &channels);
    const size_t need = stop >= 8 ? (size_t)sh.hts_per_slab * sh.d / channels * 72 : fast_lds_halfs(sh.n, sh.d) * 2;
    if (dump_bytes < need) return FREQKV_E_WORKSPACE;
    std::vector<char*> bases;
    rc = resolve_bases(k, v, *layout, sh, 0, &bases);
    if (rc < 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    void* tables = nullptr;
    Geom g0 = make_geom(sh, *layout, 1, 0);
    rc = get_basis(sh, g0, channels, st, &tables);
    if (rc < 0) return rc;
    SlabTable tab;
    memset(&tab, 0, sizeof(tab));
    tab.base[0] = bases[0];
    HIP_TRY(launch_fast(tab, g0, tables, 0.5f, nullptr, (_Float16*)dump, stop, st));
    return FREQKV_OK;
}

freqkv_status_t freqkv_compress_ragged(void* k, void* v, const freqkv_layout_t* layout, int n_heads, int head_dim,
                                       const int32_t* cur_lens, int32_t* new_lens, int window, int n_sink,
                                       double retain_ratio, void* stream)
{
    g_last_error[0] = 0;
    if (!layout || !cur_lens || !k || !v) return FREQKV_E_INVALID;
    const int batch = layout->batch;
    if (batch < 1) return FREQKV_E_INVALID;
    // validate every sequence before anything is enqueued
    bool any = false;
    for (int b = 0; b < batch; ++b) {
        Shape sh;
        freqkv_status_t rc = check_shape(layout, n_heads, head_dim, cur_lens[b], window, n_sink, retain_ratio, &sh);
        if (rc < 0) return rc;
        if (cur_lens[b] >= window && sh.variant != kNone) {
            any = true;
            size_t min_ws = sh.variant == kDrop ? 0 : pass_workspace(sh, 1);
            if (min_ws && (!layout->workspace || ((uintptr_t)layout->workspace & 255) || layout->workspace_bytes < min_ws))
                return FREQKV_E_WORKSPACE;
        }
    }
    {   // base pointers must be valid whatever the lengths are
        Shape sh;
        check_shape(layout, n_heads, head_dim, 0, window, n_sink, retain_ratio, &sh);
        std::vector<char*> probe;
        freqkv_status_t rc = resolve_bases(k, v, *layout, sh, 0, &probe);
        if (rc < 0) return rc;
    }
    // maximal runs of neighbouring sequences that share cur_len >= window: one trigger per run
    for (int b0 = 0; b0 < batch;) {
        int b1 = b0 + 1;
        while (b1 < batch && cur_lens[b1] == cur_lens[b0]) ++b1;
        freqkv_layout_t Lrun = *layout;
        Lrun.batch = b1 - b0;
        Shape sh;
        check_shape(&Lrun, n_heads, head_dim, cur_lens[b0], window, n_sink, retain_ratio, &sh);
        if (cur_lens[b0] >= window) {
            std::vector<char*> bases;
            freqkv_status_t rc = resolve_bases(k, v, *layout, sh, b0, &bases);
            if (rc < 0) return rc;
            rc = compress_resolved(bases, Lrun, sh, nullptr, (hipStream_t)stream);
            if (rc < 0) return rc;
        }
        if (new_lens)
            for (int b = b0; b < b1; ++b)
                new_lens[b] = cur_lens[b] >= window ? sh.S + sh.Lc + sh.tail : cur_lens[b];
        b0 = b1;
    }
    return any ? FREQKV_OK : FREQKV_NOOP;
}

freqkv_status_t freqkv_attend_plan(const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads, int head_dim,
                                   int cur_len, freqkv_attend_plan_t* out)
{
    if (!out) return FREQKV_E_INVALID;
    AttShape a;
    freqkv_status_t rc = check_attend(layout, n_q_heads, n_kv_heads, head_dim, cur_len, &a);
    if (rc < 0) return rc;
    memset(out, 0, sizeof(*out));
    out->n_split = a.n_split;
    out->chunk_rows = a.chunk;
    out->heads_together = a.GT;
    out->workspace_bytes = a.workspace_bytes;
    double units = (double)a.units_all;
    out->bytes_algorithmic = units * (2.0 * cur_len * a.d * a.elem + 2.0 * a.G * a.d * a.elem);
    out->flops = units * a.G * 4.0 * cur_len * a.d;
    return FREQKV_OK;
}

namespace {
// use_static: the softmax states and the rotary table live in the library's static device array instead of
// layout->workspace and a cached allocation; nothing is allocated, on the host or on the device.
freqkv_status_t attend_impl(const void* q, const void* k, const void* v, void* out, float* lse,
                            const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads, int head_dim,
                            int cur_len, int q_pos, const int32_t* cur_lens, double rope_base, void* stream,
                            bool use_static = false)
{
    g_last_error[0] = 0;
    AttShape a;
    freqkv_status_t rc = check_attend(layout, n_q_heads, n_kv_heads, head_dim, cur_len, &a);
    if (rc < 0) return rc;
    if (!q || !k || !v || !out) return FREQKV_E_INVALID;
    if (((uintptr_t)q | (uintptr_t)out | (uintptr_t)lse) & 15) return FREQKV_E_INVALID;
    if (q_pos < -1 || q_pos >= (1 << 24)) return FREQKV_E_INVALID;
    if (!(rope_base >= 0.0) || !(rope_base < 1e30)) return FREQKV_E_INVALID;      // also rejects NaN
    if (q_pos < 0) q_pos = cur_len - 1;
    const freqkv_layout_t& L = *layout;

    char* fixed_bases[kMaxSlabs];                              // [layer][K|V]; one pass needs no more
    std::vector<char*> heap_bases;
    char** bases = fixed_bases;
    if (2 * a.n_layers > kMaxSlabs) {
        if (use_static) {
            snprintf(g_last_error, sizeof(g_last_error), "at most %d layers per call without a workspace", kMaxSlabs / 2);
            return FREQKV_E_WORKSPACE;
        }
        heap_bases.resize((size_t)2 * a.n_layers);
        bases = heap_bases.data();
    }
    for (int l = 0; l < a.n_layers; ++l) {
        for (int kv = 0; kv < 2; ++kv) {
            const void* root = kv ? v : k;
            char* p = L.pointer_table ? (char*)((void* const*)root)[l]
                                      : (char*)root + (long long)l * L.stride_layer * a.elem;
            if (!p || ((uintptr_t)p & 15)) return FREQKV_E_INVALID;
            bases[(size_t)2 * l + kv] = p;
        }
    }
    hipStream_t st = (hipStream_t)stream;
    const int rope = rope_base > 0.0;
    RopeEntry* rt = nullptr;
    char* ws = (char*)L.workspace;
    if (use_static) {
        if (kScratchRopeBytes + a.workspace_bytes > kScratchBytes) {
            snprintf(g_last_error, sizeof(g_last_error),
                     "softmax states need %zu bytes, the static scratch holds %zu", a.workspace_bytes,
                     kScratchBytes - kScratchRopeBytes);
            return FREQKV_E_WORKSPACE;
        }
        void* sp = nullptr;
        rc = scratch_for_current_device(&sp);
        if (rc < 0) return rc;
        // the table is rebuilt by every call (a few hundred bytes, one tiny kernel on the caller's stream),
        // so that calls on different streams never depend on each other's table
        rt = (RopeEntry*)sp;
        HIP_TRY(launch_rope_table(rt, a.d, rope ? rope_base : 1.0, st));
        ws = (char*)sp + kScratchRopeBytes;
    } else {
        if (!L.workspace || ((uintptr_t)L.workspace & 255) || L.workspace_bytes < a.workspace_bytes)
            return FREQKV_E_WORKSPACE;
        rc = get_rope_table(a.d, rope ? rope_base : 1.0, st, &rt);
        if (rc < 0) return rc;
    }

    float* part_acc = (float*)ws;
    float* part_ml = (float*)(ws + a.ml_offset);
    const int upl = a.batch * a.n_kv;
    const int layers_per_pass = kMaxSlabs / 2;
    for (int l0 = 0; l0 < a.n_layers; l0 += layers_per_pass) {
        int layers = a.n_layers - l0 < layers_per_pass ? a.n_layers - l0 : layers_per_pass;
        SlabTable tab;
        memset(&tab, 0, sizeof(tab));
        for (int i = 0; i < 2 * layers; ++i) tab.base[i] = bases[(size_t)2 * l0 + i];
        AttGeom g;
        memset(&g, 0, sizeof(g));
        g.d = a.d; g.G = a.G; g.GT = a.GT; g.n_kv = a.n_kv; g.P = attend_pairs_per_lane(a.d);
        g.units = layers * upl; g.units_per_layer = upl;
        g.cur_len = cur_len; g.q_pos = q_pos; g.cur_lens = cur_lens; g.rope = rope;
        g.n_split = a.n_split; g.chunk = a.chunk;
        g.stride_batch = L.stride_batch; g.stride_head = L.stride_head; g.stride_token = L.stride_token;
        g.qscale = (float)(1.4426950408889634 / std::sqrt((double)a.d));
        const long long head0 = (long long)l0 * upl * a.G;                 // first query head of this pass
        const char* qp = (const char*)q + head0 * a.d * a.elem;
        char* op = (char*)out + head0 * a.d * a.elem;
        float* pa = part_acc + head0 * a.n_split * a.d;
        float* pm = part_ml + head0 * a.n_split * 2;
        ProfSpan sp;
        sp.a = sp.b = nullptr;
        if (!use_static) HIP_TRY(prof_begin(st, 3, &sp));       // timing events are created per call: not here
        HIP_TRY(launch_attend_partial(tab, g, a.elem, qp, rt, pa, pm, st));
        if (!use_static) HIP_TRY(prof_end(st, &sp));
        HIP_TRY(launch_attend_merge(g, a.elem, pa, pm, op, lse ? lse + head0 : nullptr, st));
    }
    return FREQKV_OK;
}
}  // namespace

freqkv_status_t freqkv_attend_decode(const void* q, const void* k, const void* v, void* out, float* lse,
                                     const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads, int head_dim,
                                     int cur_len, int q_pos, double rope_base, void* stream)
{
    return attend_impl(q, k, v, out, lse, layout, n_q_heads, n_kv_heads, head_dim, cur_len, q_pos, nullptr,
                       rope_base, stream);
}

freqkv_status_t freqkv_attend_decode_noalloc(const void* q, const void* k, const void* v, void* out, float* lse,
                                             const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads,
                                             int head_dim, int cur_len, int q_pos, double rope_base, void* stream)
{
    return attend_impl(q, k, v, out, lse, layout, n_q_heads, n_kv_heads, head_dim, cur_len, q_pos, nullptr,
                       rope_base, stream, true);
}

size_t freqkv_noalloc_scratch_bytes(void) { return kScratchBytes - kScratchRopeBytes; }

freqkv_status_t freqkv_attend_decode_ragged(const void* q, const void* k, const void* v, void* out, float* lse,
                                            const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads,
                                            int head_dim, const int32_t* cur_lens, int max_cur_len,
                                            double rope_base, void* stream)
{
    if (!cur_lens || ((uintptr_t)cur_lens & 3)) return FREQKV_E_INVALID;
    return attend_impl(q, k, v, out, lse, layout, n_q_heads, n_kv_heads, head_dim, max_cur_len, -1, cur_lens,
                       rope_base, stream);
}

freqkv_status_t freqkv_power_spectrum(const void* k, const void* v, float* out, const freqkv_layout_t* layout,
                                      int n_heads, int head_dim, int row0, int n_rows, void* stream)
{
    g_last_error[0] = 0;
    if (!layout || !k || !v || !out) return FREQKV_E_INVALID;
    if (row0 < 0 || n_rows < 2) return FREQKV_E_INVALID;
    if ((long long)row0 + n_rows > layout->token_capacity) return FREQKV_E_INVALID;
    if ((uintptr_t)out & 15) return FREQKV_E_INVALID;
    // same shape rules as a trigger whose span is rows [row0, row0 + n_rows) and keeps every coefficient
    Shape sh;
    freqkv_status_t rc = check_shape(layout, n_heads, head_dim, row0 + n_rows, row0 + n_rows, row0, 1.0, &sh);
    if (rc < 0) return rc;
    sh.variant = (sh.n % 2 == 0) ? kFoldF16 : kPlainF16;        // fp32 caches too: converted to the fp16 operands
    sh.high = 2;
    const freqkv_layout_t& L = *layout;
    std::vector<char*> bases;
    rc = resolve_bases(const_cast<void*>(k), const_cast<void*>(v), L, sh, 0, &bases);
    if (rc < 0) return rc;
    size_t min_ws = pass_workspace(sh, 1);
    if (!L.workspace || ((uintptr_t)L.workspace & 255) || L.workspace_bytes < min_ws) return FREQKV_E_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    int per_pass = sh.nslabs < kMaxSlabs ? sh.nslabs : kMaxSlabs;
    while (per_pass > 1 && pass_workspace(sh, per_pass) > L.workspace_bytes) --per_pass;
    void* basis = nullptr;
    {
        Geom g0 = make_geom(sh, L, per_pass, 0);
        rc = get_basis(sh, g0, 1, st, &basis);
        if (rc < 0) return rc;
    }
    HIP_TRY(launch_fill_zero(out, (size_t)sh.nslabs * sh.n_heads * sh.n, st));
    for (int s0 = 0; s0 < sh.nslabs; s0 += per_pass) {
        int slabs = sh.nslabs - s0 < per_pass ? sh.nslabs - s0 : per_pass;
        Geom g = make_geom(sh, L, slabs, s0);
        g.spec_scale = (float)(1.0 / ((double)sh.batch * sh.d));
        SlabTable tab;
        memset(&tab, 0, sizeof(tab));
        for (int i = 0; i < slabs; ++i) tab.base[i] = bases[(size_t)s0 + i];
        ProfSpan sp;
        HIP_TRY(prof_begin(st, 0, &sp));
        HIP_TRY(launch_prepare_bf16(tab, g, (_Float16*)L.workspace, st, sh.elem));
        HIP_TRY(prof_end(st, &sp));
        HIP_TRY(prof_begin(st, 1, &sp));
        HIP_TRY(launch_contract_f16(tab, g, (const _Float16*)basis, (const _Float16*)L.workspace, out, 1, st));
        HIP_TRY(prof_end(st, &sp));
    }
    return FREQKV_OK;
}

namespace {
struct PrefillShape {
    AttShape a;
    int q_len, q_pad, key_tiles, layers_per_pass;
    size_t off_kr, off_vt, workspace_bytes;
};

freqkv_status_t check_prefill(const freqkv_layout_t* L, int n_q, int n_kv, int d, int cur_len, int q_len,
                              PrefillShape* out)
{
    PrefillShape p;
    freqkv_status_t rc = check_attend(L, n_q, n_kv, d, cur_len, &p.a);
    if (rc < 0) return rc;
    if (q_len < 1 || q_len > cur_len) return FREQKV_E_INVALID;
    if (d != 128 || L->dtype != FREQKV_BF16) return FREQKV_E_UNSUPPORTED;
    p.q_len = q_len;
    p.q_pad = (int)round_up(q_len, 32);
    p.key_tiles = (cur_len + 31) / 32;
    p.layers_per_pass = p.a.n_layers < kMaxSlabs / 2 ? p.a.n_layers : kMaxSlabs / 2;
    const long long units = (long long)p.layers_per_pass * p.a.batch * n_kv;
    if (units * p.a.G * (p.q_pad / 32) > (1LL << 30)) return FREQKV_E_UNSUPPORTED;
    size_t cs_bytes = (size_t)round_up((long long)cur_len * (d / 2) * 8, 256);
    size_t kv_bytes = (size_t)units * p.key_tiles * 32 * d * 2;
    p.off_kr = cs_bytes;
    p.off_vt = p.off_kr + kv_bytes;
    p.workspace_bytes = p.off_vt + kv_bytes;
    *out = p;
    return FREQKV_OK;
}
}  // namespace

freqkv_status_t freqkv_attend_prefill_plan(const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads,
                                           int head_dim, int cur_len, int q_len, freqkv_prefill_plan_t* out)
{
    if (!out) return FREQKV_E_INVALID;
    PrefillShape p;
    freqkv_status_t rc = check_prefill(layout, n_q_heads, n_kv_heads, head_dim, cur_len, q_len, &p);
    if (rc < 0) return rc;
    memset(out, 0, sizeof(*out));
    out->workspace_bytes = p.workspace_bytes;
    out->key_tiles = p.key_tiles;
    out->query_blocks = p.q_pad / 32;
    // query i sees cur_len - q_len + i + 1 rows; 4 d flops per (query, row): scores and weighted sum
    const double rows_seen = (double)q_len * (cur_len - q_len) + 0.5 * (double)q_len * (q_len + 1);
    const double heads = (double)p.a.units_all * p.a.G;
    out->flops = heads * 4.0 * head_dim * rows_seen;
    out->bytes_algorithmic = (double)p.a.units_all * 2.0 * cur_len * head_dim * 2 + heads * 2.0 * q_len * head_dim * 2;
    return FREQKV_OK;
}

freqkv_status_t freqkv_attend_prefill(const void* q, const void* k, const void* v, void* out, float* lse,
                                      const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads, int head_dim,
                                      int cur_len, int q_len, double rope_base, void* stream)
{
    g_last_error[0] = 0;
    PrefillShape p;
    freqkv_status_t rc = check_prefill(layout, n_q_heads, n_kv_heads, head_dim, cur_len, q_len, &p);
    if (rc < 0) return rc;
    if (!q || !k || !v || !out) return FREQKV_E_INVALID;
    if (((uintptr_t)q | (uintptr_t)out | (uintptr_t)lse) & 15) return FREQKV_E_INVALID;
    if (!(rope_base >= 0.0) || !(rope_base < 1e30)) return FREQKV_E_INVALID;
    const freqkv_layout_t& L = *layout;
    const AttShape& a = p.a;
    std::vector<char*> bases((size_t)2 * a.n_layers);          // [layer][K|V]
    for (int l = 0; l < a.n_layers; ++l) {
        for (int kv = 0; kv < 2; ++kv) {
            const void* root = kv ? v : k;
            char* bp = L.pointer_table ? (char*)((void* const*)root)[l]
                                       : (char*)root + (long long)l * L.stride_layer * a.elem;
            if (!bp || ((uintptr_t)bp & 15)) return FREQKV_E_INVALID;
            bases[(size_t)2 * l + kv] = bp;
        }
    }
    if (!L.workspace || ((uintptr_t)L.workspace & 255) || L.workspace_bytes < p.workspace_bytes)
        return FREQKV_E_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)L.workspace;
    const int upl = a.batch * a.n_kv;
    for (int l0 = 0; l0 < a.n_layers; l0 += p.layers_per_pass) {
        int layers = a.n_layers - l0 < p.layers_per_pass ? a.n_layers - l0 : p.layers_per_pass;
        SlabTable tab;
        memset(&tab, 0, sizeof(tab));
        for (int i = 0; i < 2 * layers; ++i) tab.base[i] = bases[(size_t)2 * l0 + i];
        PrefillGeom g;
        memset(&g, 0, sizeof(g));
        g.d = a.d; g.G = a.G; g.n_kv = a.n_kv;
        g.units = layers * upl; g.units_per_layer = upl;
        g.cur_len = cur_len; g.q_len = q_len; g.q_pad = p.q_pad; g.q_blocks = p.q_pad / 32;
        g.key_tiles = p.key_tiles; g.rope = rope_base > 0.0;
        g.stride_batch = L.stride_batch; g.stride_head = L.stride_head; g.stride_token = L.stride_token;
        g.qscale = (float)(1.4426950408889634 / std::sqrt((double)a.d));
        const long long head0 = (long long)l0 * upl * a.G;
        const char* qp = (const char*)q + head0 * q_len * a.d * a.elem;
        char* op = (char*)out + head0 * q_len * a.d * a.elem;
        ProfSpan sp;
        HIP_TRY(prof_begin(st, 0, &sp));
        HIP_TRY(launch_prefill_prepare(tab, g, rope_base > 0.0 ? rope_base : 1.0, (float2*)ws,
                                       (_Float16*)(ws + p.off_kr), (_Float16*)(ws + p.off_vt), st));
        HIP_TRY(prof_end(st, &sp));
        HIP_TRY(prof_begin(st, 3, &sp));
        HIP_TRY(launch_attend_prefill(g, (const _Float16*)(ws + p.off_kr), (const _Float16*)(ws + p.off_vt), qp,
                                      (const float2*)ws, op, lse ? lse + head0 * q_len : nullptr, st));
        HIP_TRY(prof_end(st, &sp));
    }
    return FREQKV_OK;
}

void freqkv_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    bool have_dev = hipGetDevice(&cur) == hipSuccess;
    for (auto& kv : g_basis) {
        if (hipSetDevice(kv.first.device) != hipSuccess) continue;
        if (kv.second.ready) {
            (void)hipEventSynchronize(kv.second.ready);
            (void)hipEventDestroy(kv.second.ready);
        }
        (void)hipFree(kv.second.ptr);
        if (kv.second.host) (void)hipHostFree(kv.second.host);
    }
    g_basis.clear();
    for (auto& kv : g_rope) {
        if (hipSetDevice(kv.first.device) != hipSuccess) continue;
        if (kv.second.ready) {
            (void)hipEventSynchronize(kv.second.ready);
            (void)hipEventDestroy(kv.second.ready);
        }
        (void)hipFree(kv.second.ptr);
    }
    g_rope.clear();
    for (auto& sp : g_prof_spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    g_prof_spans.clear();
    if (have_dev) (void)hipSetDevice(cur);
    (void)hipGetLastError();
}

freqkv_status_t freqkv_calibrate_copy(void* dst, const void* src, size_t bytes, int repeats, void* stream,
                                      double* gbs_out)
{
    if (!dst || !src || !gbs_out || bytes < 16 || (bytes & 15) || repeats < 1) return FREQKV_E_INVALID;
    if (((uintptr_t)dst | (uintptr_t)src) & 15) return FREQKV_E_INVALID;
    hipStream_t st = (hipStream_t)stream;
    EventPair ev;
    HIP_TRY(ev.create());
    HIP_TRY(launch_calib_copy(dst, src, bytes, st));             // warm-up
    HIP_TRY(hipEventRecord(ev.a, st));
    for (int i = 0; i < repeats; ++i) HIP_TRY(launch_calib_copy(dst, src, bytes, st));
    HIP_TRY(hipEventRecord(ev.b, st));
    HIP_TRY(hipEventSynchronize(ev.b));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
    *gbs_out = 2.0 * (double)bytes * repeats / (ms * 1e-3) / 1e9;     // read + write
    return FREQKV_OK;
}

freqkv_status_t freqkv_calibrate_mfma(int iters, void* stream, double* tflops_out)
{
    if (!tflops_out || iters < 1) return FREQKV_E_INVALID;
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    float* out = nullptr;
    HIP_TRY(hipMalloc(&out, (size_t)cus * 256 * sizeof(float)));
    EventPair ev;
    hipError_t e = ev.create();
    if (e == hipSuccess) e = launch_calib_mfma(out, cus, iters / 10 + 1, st);
    if (e == hipSuccess) e = hipEventRecord(ev.a, st);
    if (e == hipSuccess) e = launch_calib_mfma(out, cus, iters, st);
    if (e == hipSuccess) e = hipEventRecord(ev.b, st);
    if (e == hipSuccess) e = hipEventSynchronize(ev.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
    (void)hipFree(out);
    if (e != hipSuccess) { set_error("calibrate_mfma", e); return FREQKV_E_HIP; }
    // one workgroup per CU, 4 waves, 16 MFMAs of 32*32*16 MACs per iteration
    *tflops_out = (double)cus * 4.0 * iters * 16.0 * 32768.0 / (ms * 1e-3) / 1e12;
    return FREQKV_OK;
}

freqkv_status_t freqkv_profile_enable(int on)
{
    std::lock_guard<std::mutex> lock(g_mu);
    for (auto& sp : g_prof_spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    g_prof_spans.clear();
    memset(&g_prof_acc, 0, sizeof(g_prof_acc));
    g_prof_on = on != 0;
    return FREQKV_OK;
}

freqkv_status_t freqkv_profile_read(freqkv_profile_t* out)
{
    if (!out) return FREQKV_E_INVALID;
    std::lock_guard<std::mutex> lock(g_mu);
    for (auto& sp : g_prof_spans) {
        HIP_TRY(hipEventSynchronize(sp.b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
        if (sp.kind == 0) { g_prof_acc.ms_prepare += ms; g_prof_acc.launches_prepare++; }
        else if (sp.kind == 1) { g_prof_acc.ms_contract += ms; g_prof_acc.launches_contract++; }
        else if (sp.kind == 2) { g_prof_acc.ms_tail += ms; g_prof_acc.launches_tail++; }
        else { g_prof_acc.ms_attend += ms; g_prof_acc.launches_attend++; }
        (void)hipEventDestroy(sp.a);
        (void)hipEventDestroy(sp.b);
    }
    g_prof_spans.clear();
    *out = g_prof_acc;
    return FREQKV_OK;
}

}  // extern "C"
