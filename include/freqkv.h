/*
 * freqkv.h - C ABI of libfreqkv: frequency-domain compression of an LLM KV cache
 * on AMD MI355X (gfx950).
 *
 * The operation (FreqKV, arXiv 2505.00570):
 *   When a cache of `window` tokens is full, the span after the first `n_sink`
 *   tokens (n = window - n_sink rows of every per-head K and V matrix) is taken
 *   through an orthonormal DCT-II along the token axis (Sec. 3.3 Eq. 2,
 *   Appendix A), only the Lc = floor(retain_ratio * n) lowest-frequency
 *   coefficients are kept (Sec. 3.3), an Lc-point inverse DCT brings them back to
 *   Lc time-domain rows, scaled by sqrt(Lc/n) (Sec. 3.3 Eq. 3), and those rows
 *   replace the span in place: [sinks | Lc compressed rows | later tokens]
 *   (Sec. 3.4, Fig. 2b).  Sink rows are never touched (Sec. 3.4).
 *
 * All entry points are plain C, take plain pointers and sizes, never throw and
 * never abort.  Unless a comment says "host", a pointer is a DEVICE pointer.
 * The caller owns every buffer it passes; the library owns only its cached
 * basis tables (freed by freqkv_shutdown).
 */
#ifndef FREQKV_H
#define FREQKV_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define FREQKV_API __attribute__((visibility("default")))
#else
#define FREQKV_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FREQKV_OK            = 0,   /* work was enqueued on the stream                          */
    FREQKV_NOOP          = 1,   /* cur_len < window: cache not full, nothing enqueued       */
    FREQKV_E_INVALID     = -1,  /* an argument violates the documented ranges               */
    FREQKV_E_UNSUPPORTED = -2,  /* valid but not implemented (e.g. odd head_dim)            */
    FREQKV_E_WORKSPACE   = -3,  /* layout.workspace missing, misaligned or too small        */
    FREQKV_E_HIP         = -4,  /* a HIP runtime call failed                                */
    FREQKV_E_ALLOC       = -5   /* the library could not allocate a basis table             */
} freqkv_status_t;

typedef enum {
    FREQKV_BF16 = 0,            /* cache holds bfloat16; fp16 MFMA operands, fp32 accumulate */
    FREQKV_F32  = 1             /* cache holds float32; fp32 FMA throughout                  */
} freqkv_dtype_t;

/* layout.flags */
#define FREQKV_FLAG_NO_RESCALE 0x1u   /* omit the sqrt(Lc/n) factor (rescaling ablation, appendix "Effect of rescaling") */
#define FREQKV_FLAG_DROPPING   0x2u   /* the "Dropping" variant (appendix on the compression overhead): no transform,
                                         the Lc most recent rows of the span, [window-Lc, window), move to [n_sink, n_sink+Lc);
                                         same sinks, same retained size, same tail rule; needs no workspace and no basis */

#define FREQKV_FLAG_RETAIN_HIGH 0x4u  /* the high-frequency variant of the ablation tables (Sec. 3.2 summarisation
                                         table; appendix table on retaining high frequencies): the Lc HIGHEST
                                         coefficients of the n-point DCT are kept and handed, in order, to the
                                         Lc-point inverse; everything else as the default.  Not with DROPPING */

#define FREQKV_FLAG_SINGLE_FOLD 0x8u  /* never use the two-level even/odd fold (default: spans of 2048 rows or more
                                         that are a multiple of 4, with an even retained length, when the cache has
                                         enough head-tensors to fill the device with the shorter launches) */
#define FREQKV_FLAG_TWO_LEVEL_FOLD 0x10u /* use the two-level fold wherever it applies (span a multiple of 4, even
                                         retained length), whatever the sizes.  Not with SINGLE_FOLD */

#define FREQKV_FLAG_DENSE 0x20u      /* never use the factored transform (variant 6); the matrix forms (variants 1, 2, 5)
                                         run instead (SINGLE_FOLD and TWO_LEVEL_FOLD imply it).  Default: spans n = 4pq with a compiled factorization (8188 = 4*23*89,
                                         4092 = 4*11*93, 2044 = 4*7*73, 1020 = 4*3*85, and 1260, 140 for tests) at retain_ratio 0.5 on bf16 caches take the
                                         factored form, which needs no workspace */

/*
 * Memory description of the cache ("layout"): everything the scalar arguments of
 * freqkv_compress do not say.  One head-tensor is the [token][dim] matrix of one
 * (K|V, layer, batch, head); its element (token t, channel c) lives at
 *     base(K|V, layer) + b*stride_batch + h*stride_head + t*stride_token + c      (in elements)
 * where base = k (or v) + layer*stride_layer when pointer_table == 0, and
 *       base = ((void* const*)k)[layer]      when pointer_table == 1 (k and v are then HOST
 *              arrays of n_layers device pointers, read before the call returns).
 * The channel stride is 1.  Head-major caches ([layer][batch][head][token][dim],
 * stride_token == head_dim) are the fast, fully coalesced case; any stride_token >= head_dim works.
 * Every stride must be a multiple of 8 elements and every base pointer 16-byte aligned.
 * The batch shares one cur_len (Sec. 4.1: identical settings for all layers and heads).
 */
typedef struct freqkv_layout {
    int32_t  dtype;             /* freqkv_dtype_t                                               */
    int32_t  n_layers;          /* >= 1                                                         */
    int32_t  batch;             /* >= 1                                                         */
    int32_t  token_capacity;    /* rows allocated per head-tensor, >= cur_len                   */
    int64_t  stride_layer;      /* elements; ignored when pointer_table == 1                    */
    int64_t  stride_batch;      /* elements                                                     */
    int64_t  stride_head;       /* elements                                                     */
    int64_t  stride_token;      /* elements, >= head_dim                                        */
    int32_t  pointer_table;     /* 0 or 1, see above                                            */
    uint32_t flags;             /* FREQKV_FLAG_*                                                */
    void*    workspace;         /* device scratch, 256-byte aligned, see freqkv_plan            */
    size_t   workspace_bytes;
    float*   tap_f32;           /* optional (may be NULL): device array
                                   [2 (K,V)][n_layers][batch][n_heads][Lc][head_dim] that receives
                                   the fp32 results before they are rounded to the cache dtype    */
} freqkv_layout_t;

/* Result of the buffer-plan query (host arithmetic only). */
typedef struct freqkv_plan {
    int32_t span_len;           /* n  = window - n_sink                                          */
    int32_t retained_len;       /* Lc = clamp(floor(retain_ratio*n + 1e-9), 1, n)                */
    int32_t new_len;            /* cache length after the call: n_sink + Lc + (cur_len - window) */
    int32_t head_tensors;       /* 2 * n_layers * batch * n_heads                                */
    int32_t variant;            /* 0 none (no-op or ratio 1), 1 folded fp16-MFMA, 2 plain fp16-MFMA, 3 fp32 FMA,
                                   4 dropping (row moves only), 5 two-level folded fp16-MFMA,
                                   6 factored transform (prime-factor DFT stages on the matrix cores, LDS resident) */
    int32_t reserved;
    size_t  workspace_bytes;    /* scratch for all head-tensors in one pass (fastest)            */
    size_t  workspace_min_bytes;/* smallest scratch accepted (one (layer,K|V) slab per pass)     */
    size_t  basis_bytes;        /* device memory the library itself holds for this (n, Lc)       */
    double  flops_dense;        /* 2*Lc*n*d per head-tensor, summed: the fused operator as one contraction */
    double  flops_executed;     /* what the chosen variant executes (no padding counted)         */
    double  bytes_algorithmic;  /* (n + Lc)*d*e per head-tensor + 2*(cur_len-window)*d*e, summed */
} freqkv_plan_t;

/* Per-kernel GPU time, accumulated by HIP events while profiling is on. */
typedef struct freqkv_profile {
    int64_t calls;              /* freqkv_compress calls that enqueued work                      */
    int64_t launches_prepare;   /* fold/convert (or copy) launches                               */
    int64_t launches_contract;  /* contraction launches                                          */
    int64_t launches_tail;      /* tail-move launches                                            */
    double  ms_prepare;
    double  ms_contract;
    double  ms_tail;
    int64_t launches_attend;    /* freqkv_attend_decode passes: the row-chunk kernel of each (the merge kernel is not timed) */
    double  ms_attend;
} freqkv_profile_t;

/* Result of the attention buffer-plan query (host arithmetic only). */
typedef struct freqkv_attend_plan {
    int32_t n_split;            /* row chunks each KV head's cache is cut into                       */
    int32_t chunk_rows;         /* rows per chunk                                                    */
    int32_t heads_together;     /* query heads of one KV group that one workgroup serves (1, 2 or 4) */
    int32_t reserved;
    size_t  workspace_bytes;    /* scratch for the per-chunk softmax states                          */
    double  bytes_algorithmic;  /* K and V rows [0, cur_len) read once, q read, out written          */
    double  flops;              /* 4 * cur_len * head_dim per query head (scores and weighted sum)   */
} freqkv_attend_plan_t;

/*
 * Buffer-plan query (Sec. 3.3 / Sec. 4.1 arithmetic).  HOST only: needs no GPU, touches no
 * device memory; layout.workspace / tap_f32 are ignored.  `layout` and `out` are host pointers.
 * Returns FREQKV_OK, FREQKV_NOOP (cur_len < window; the plan is still filled for a full cache)
 * or a negative status for invalid arguments.
 *
 * Valid ranges: n_heads >= 1; head_dim >= 8 and a multiple of 8; n_sink >= 0;
 * window >= n_sink + 2; cur_len <= layout.token_capacity; 0 < retain_ratio <= 1.
 */
FREQKV_API freqkv_status_t freqkv_plan(const freqkv_layout_t* layout, int n_heads, int head_dim,
                            int cur_len, int window, int n_sink, double retain_ratio,
                            freqkv_plan_t* out);

/*
 * One compression trigger over every layer's K and V (Sec. 3.3 Eq. 2-3, Sec. 3.4).
 *   k, v     device base pointers of the K and V caches (or host pointer tables, see layout)
 *   layout   host pointer; read before the call returns
 *   cur_len  tokens currently in the cache; the span is rows [n_sink, window); rows
 *            [window, cur_len) are a recent tail that is moved, bit for bit, to start at
 *            n_sink + Lc.  After the call the cache holds freqkv_plan(...).new_len tokens;
 *            rows at and beyond new_len (up to the old cur_len) hold unspecified values.
 *            Nothing outside rows [n_sink, cur_len) of any head-tensor is written.
 *   stream   hipStream_t (NULL = the default stream).  The call only enqueues work: it does not
 *            synchronise the device and never reads results back.  The first call for a new
 *            (device, n, Lc, dtype, flags) builds and caches the basis table (one allocation).
 * retain_ratio == 1 (Lc == n) is the identity and enqueues nothing (FREQKV_OK).
 * Value range (bf16 caches): the matrix cores take fp16 operands, whose range is narrower than bfloat16's.
 * Every head-tensor (every 8- or 16-channel slice of one in the factored form) is therefore scaled by an exact
 * power of two, chosen from the largest magnitude of its span, on its way in and back on its way out, so
 * finite cache values of any magnitude neither overflow nor sink into fp16 subnormals; only values more
 * than 2^24 times smaller than the largest of their head-tensor (slice) lose precision.  An inf or
 * nan in the span makes the results of its channels non-finite (of its whole slice in the factored form).  Basis entries below 6e-5 are fp16 subnormals (absolute error
 * 2^-25, far below the tolerance).
 * On a negative status no device memory has been written.
 */
FREQKV_API freqkv_status_t freqkv_compress(void* k, void* v, const freqkv_layout_t* layout,
                                int n_heads, int head_dim, int cur_len, int window, int n_sink,
                                double retain_ratio, void* stream);

/*
 * The same trigger for a batch whose sequences hold different numbers of tokens (each sequence's cache
 * fills and compacts on its own schedule, Sec. 3.4): sequence b is compressed iff cur_lens[b] >= window,
 * exactly as freqkv_compress would with cur_len = cur_lens[b]; the others are not touched.
 *   cur_lens  HOST array [layout.batch] of int32, each 0 <= cur_lens[b] <= layout.token_capacity
 *   new_lens  optional HOST array [layout.batch] (may be NULL, may alias cur_lens): cache length of every
 *             sequence after the call
 * Neighbouring sequences with equal cur_lens share one launch sequence; layout.tap_f32 is ignored.
 * Returns FREQKV_OK if any sequence was compressed, FREQKV_NOOP if none, or a negative status (checked
 * for every sequence before anything is enqueued: no device memory written).
 */
FREQKV_API freqkv_status_t freqkv_compress_ragged(void* k, void* v, const freqkv_layout_t* layout,
                                       int n_heads, int head_dim, const int32_t* cur_lens /* host */,
                                       int32_t* new_lens /* host */, int window, int n_sink,
                                       double retain_ratio, void* stream);

/*
 * Build and cache the basis table for (window - n_sink, retain_ratio, dtype, flags) on the current
 * device ahead of the first trigger (Appendix A cosine bases fused into one operator).  Optional.
 */
FREQKV_API freqkv_status_t freqkv_prepare(int dtype, uint32_t flags, int window, int n_sink,
                               double retain_ratio, void* stream);

/*
 * Buffer plan of freqkv_attend_decode.  HOST only, like freqkv_plan.  Valid ranges: n_kv_heads >= 1,
 * n_q_heads a multiple of n_kv_heads, 1 <= cur_len <= layout.token_capacity; head_dim 64, 128 or 256
 * (anything else: FREQKV_E_UNSUPPORTED).  The cur_len rows of one head must span less than 4 GiB
 * ((cur_len + 1024) * stride_token * element size < 2^32; FREQKV_E_UNSUPPORTED otherwise): rows are addressed
 * by 32-bit byte offsets.  The same limits hold for the chunk-wise entry points below.
 */
FREQKV_API freqkv_status_t freqkv_attend_plan(const freqkv_layout_t* layout, int n_q_heads, int n_kv_heads,
                                   int head_dim, int cur_len, freqkv_attend_plan_t* out);

/*
 * Decode attention of one incoming token per sequence over the compacted cache, for every layer the
 * layout describes (Sec. 3.3 Eq. 4, Sec. 3.4 Eq. 5): the token attends to all rows [0, cur_len) of its
 * KV head (sinks, compressed rows, tokens appended since, and itself: its own key and value must
 * already be the last cached row).  Keys are cached WITHOUT the rotary embedding; the key in row p is
 * rotated with position p, an index inside the cache, as it is read, and the query with q_pos (closing
 * paragraph of Sec. 3.4, appendix on key states with RoPE).  Rotary pairing: channel i with channel
 * i + head_dim/2, angle pos * rope_base^(-2i/head_dim).  Query head h reads KV head
 * h / (n_q_heads / n_kv_heads).  Scores are scaled by 1/sqrt(head_dim).
 *   q        [n_layers][batch][n_q_heads][head_dim], dense, layout.dtype, un-rotated queries
 *   k, v     the caches, addressed through `layout` exactly as in freqkv_compress (n_heads = n_kv_heads)
 *   out      [n_layers][batch][n_q_heads][head_dim], dense, layout.dtype
 *   lse      optional (may be NULL): [n_layers][batch][n_q_heads] fp32, natural log of the sum of
 *            exp(score); lets a caller merge results over caches sharded by token
 *   q_pos    in-cache position of the query, or -1 for cur_len - 1
 *   rope_base  e.g. 10000 (LLaMA-2) or 500000 (LLaMA-3); 0 applies no rotary embedding
 *   layout.workspace  at least freqkv_attend_plan(...).workspace_bytes, 256-byte aligned
 * q, out and lse must be 16-byte aligned.  The call only enqueues work on `stream`.  The first call
 * for a new (device, head_dim, rope_base) builds a small cached table (one allocation).
 * On a negative status no device memory has been written.
 */
FREQKV_API freqkv_status_t freqkv_attend_decode(const void* q, const void* k, const void* v, void* out,
                                     float* lse, const freqkv_layout_t* layout, int n_q_heads,
                                     int n_kv_heads, int head_dim, int cur_len, int q_pos,
                                     double rope_base, void* stream);

/*
 * freqkv_attend_decode for callers that cannot allocate device memory or pass a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results, but layout.workspace is ignored: the per-chunk softmax states and the
 * small rotary table live in a static device array inside the library (8 MiB per GPU, held until the
 * process ends), and the call allocates nothing, on the host or on the device.
 * Limits: freqkv_attend_plan(...).workspace_bytes <= freqkv_noalloc_scratch_bytes() and n_layers <= 96;
 * beyond either the call returns FREQKV_E_WORKSPACE (freqkv_last_error says which) and writes nothing.
 * The array is shared by every call on a GPU and keeps the last call's contents; every call overwrites
 * all the states it reads, so nothing has to be cleared, but two calls that overlap in time on one GPU
 * (different streams, different threads) race: serialise them.
 */
FREQKV_API freqkv_status_t freqkv_attend_decode_noalloc(const void* q, const void* k, const void* v, void* out,
                                             float* lse, const freqkv_layout_t* layout, int n_q_heads,
                                             int n_kv_heads, int head_dim, int cur_len, int q_pos,
                                             double rope_base, void* stream);
/* Bytes of the static array available to the softmax states of freqkv_attend_decode_noalloc (host). */
FREQKV_API size_t freqkv_noalloc_scratch_bytes(void);

/*
 * The same attention for a batch whose sequences hold different numbers of cached rows (a serving batch:
 * Sec. 3.4's cache of each sequence fills and compacts on its own schedule).
 *   cur_lens     DEVICE array [layout.batch] of int32: cached rows of each sequence, shared by all layers;
 *                each value is clamped to [1, max_cur_len] on the device; the query of sequence b sits at
 *                its last row, cur_lens[b] - 1
 *   max_cur_len  host upper bound of the values in cur_lens, 1 <= max_cur_len <= layout.token_capacity;
 *                sizes the launch (use it with freqkv_attend_plan for the workspace)
 * Everything else as freqkv_attend_decode.  Rows at and beyond a sequence's cur_lens[b] are never read.
 */
FREQKV_API freqkv_status_t freqkv_attend_decode_ragged(const void* q, const void* k, const void* v, void* out,
                                            float* lse, const freqkv_layout_t* layout, int n_q_heads,
                                            int n_kv_heads, int head_dim, const int32_t* cur_lens,
                                            int max_cur_len, double rope_base, void* stream);

/*
 * Average power spectrum of the cached key and value states (Sec. 3.1 and its figure; appendix on the
 * head-wise analysis): rows [row0, row0 + n_rows) of every head-tensor go through the orthonormal
 * n_rows-point DCT-II along the token axis (Appendix A), and the squared coefficients are averaged over
 * the batch ("samples") and the head_dim channels.  A diagnostic: the cache is only read.
 *   out   DEVICE array [2 (K,V)][n_layers][n_heads][n_rows] fp32, 16-byte aligned; overwritten
 *   layout.workspace   as for a trigger with window - n_sink = n_rows (freqkv_plan reports it for
 *                      n_sink = row0, window = row0 + n_rows, any retain_ratio < 1)
 * bf16 and fp32 caches (both converted to fp16 operands); n_rows >= 2.  No range guard here: cache values must
 * stay below 32752 in magnitude (the folded span is an fp16 operand).  fp16 operands put a noise floor of
 * about 2e-7 of the average line under every line.  The sums are accumulated with fp32 atomics, so the
 * last bits can differ from call to call.  The first call for a new (device, n_rows) builds and caches the
 * transform matrix (one allocation of about n_rows^2 bytes).
 */
FREQKV_API freqkv_status_t freqkv_power_spectrum(const void* k, const void* v, float* out,
                                      const freqkv_layout_t* layout, int n_heads, int head_dim,
                                      int row0, int n_rows, void* stream);

/* Result of the chunk-attention buffer-plan query (host arithmetic only). */
typedef struct freqkv_prefill_plan {
    size_t  workspace_bytes;    /* rotary table (fp32), rotated keys and transposed values (fp16)             */
    int32_t key_tiles;          /* ceil(cur_len / 32)                                                         */
    int32_t query_blocks;       /* ceil(q_len / 32)                                                           */
    double  flops;              /* 4 * head_dim per (query, visible row), summed                              */
    double  bytes_algorithmic;  /* K and V rows [0, cur_len) once, q read, out written                        */
} freqkv_prefill_plan_t;

FREQKV_API freqkv_status_t freqkv_attend_prefill_plan(const freqkv_layout_t* layout, int n_q_heads,
                                           int n_kv_heads, int head_dim, int cur_len, int q_len,
                                           freqkv_prefill_plan_t* out);

/*
 * Chunk-wise attention of training and prefilling (Sec. 3.4 Eq. 5): the q_len tokens of the incoming chunk
 * are the LAST q_len cached rows (their keys and values must already be in the cache); query i sits at
 * in-cache position cur_len - q_len + i and attends to rows [0, that position]: sinks, compressed rows,
 * the earlier tokens of its chunk and itself.  Rotary embedding, head grouping and scaling exactly as in
 * freqkv_attend_decode (its last query is this call's last query).
 *   q, out   [n_layers][batch][n_q_heads][q_len][head_dim], dense, bfloat16
 *   lse      optional [n_layers][batch][n_q_heads][q_len] fp32
 *   layout.workspace  at least freqkv_attend_prefill_plan(...).workspace_bytes, 256-byte aligned
 * head_dim 128 and bfloat16 caches only (FREQKV_E_UNSUPPORTED otherwise).  Operands of the matrix cores are
 * fp16 (cache values are exact in fp16; rotated keys and queries keep 11 significant bits), accumulation,
 * softmax and the running sums are fp32.  The call only enqueues work on `stream`.
 */
FREQKV_API freqkv_status_t freqkv_attend_prefill(const void* q, const void* k, const void* v, void* out,
                                      float* lse, const freqkv_layout_t* layout, int n_q_heads,
                                      int n_kv_heads, int head_dim, int cur_len, int q_len,
                                      double rope_base, void* stream);

/*
 * Diagnostic of the factored transform (variant 6), used by the tests to check its stages one by one: runs
 * the kernel on the K cache of layer 0 up to and including stage `stop` (1 load and length-4 butterfly,
 * 2 q-point forward stage, 3 p-point forward stage, 4 step between the transforms, 5 p-point inverse stage;
 * the q-point inverse stage writes straight to the cache and leaves no image), copies the fp16 LDS image of the workgroup that owns channels 0..7 of the first
 * head-tensor to `dump` (device memory, dump_bytes >= what the span needs, at most 160 KiB) and writes
 * nothing to the cache.  stop = 8 (one workgroup per task) or 9 (the persistent grid of a real call) instead
 * runs the whole transform on the K cache of layer 0 (the cache IS
 * written) and leaves, per workgroup, 9 int64 shader-clock readings in dump (start, then after each of the
 * stages above (the sixth repeats the fifth) and after the last stage, then the moment the rows had arrived inside stage 1;
 * dump_bytes >= 72 * batch * n_heads * head_dim / 8).
 * retain_ratio is 0.5.  FREQKV_E_UNSUPPORTED when the span has no factored form.
 */
FREQKV_API freqkv_status_t freqkv_debug_fast_stage(void* k, void* v, const freqkv_layout_t* layout, int n_heads,
                                        int head_dim, int window, int n_sink, int stop, void* dump,
                                        size_t dump_bytes, void* stream);

/* Human-readable name of a status code (static string, host). */
FREQKV_API const char* freqkv_status_string(freqkv_status_t status);

/* Text of the last HIP error seen by the calling thread's most recent failing call ("" if none). */
FREQKV_API const char* freqkv_last_error(void);

/* Free every cached basis table on every device.  Safe to call more than once. */
FREQKV_API void freqkv_shutdown(void);

/* Library version: major*10000 + minor*100 + patch. */
FREQKV_API int freqkv_version(void);

/*
 * Kernel timing with HIP events recorded on the caller's stream around each launch.
 * freqkv_profile_enable(1) starts accumulating (and resets the counters), (0) stops.
 * freqkv_profile_read synchronises on the recorded events and fills *out (host pointer).
 */
FREQKV_API freqkv_status_t freqkv_profile_enable(int on);
FREQKV_API freqkv_status_t freqkv_profile_read(freqkv_profile_t* out);

/*
 * Calibration of the device the library runs on, for quoting rooflines against measured as well as
 * nominal peaks.  Both calls synchronise on their own events (they are measurement tools, not
 * part of the compression path).
 *   freqkv_calibrate_copy: times `repeats` plain 16-byte-per-lane copies of `bytes` (a multiple of
 *       16; dst/src device pointers, 16-byte aligned, not overlapping) and returns read+write GB/s.
 *   freqkv_calibrate_mfma: times a register-only loop of v_mfma_f32_32x32x16_f16 on random operands
 *       (one workgroup per CU, `iters` x 16 instructions per wave) and returns TFLOP/s.
 */
FREQKV_API freqkv_status_t freqkv_calibrate_copy(void* dst, const void* src, size_t bytes, int repeats,
                                      void* stream, double* gbs_out /* host */);
FREQKV_API freqkv_status_t freqkv_calibrate_mfma(int iters, void* stream, double* tflops_out /* host */);

#ifdef __cplusplus
}
#endif
#endif /* FREQKV_H */
