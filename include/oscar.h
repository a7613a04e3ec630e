/*
 * oscar.h -- C ABI of the MI355X (gfx950) OScaR KV-cache library.
 *
 * OScaR ("Omni-Scaled Canalized Rotation") compresses the key/value cache of a
 * decoder-only transformer to 2 or 4 bits:
 *   keys  : Hadamard rotation on the head dimension (Canalized Rotation), then
 *           division by the per-token L2 norm (Omni-Token Scaling, the norm is
 *           kept as metadata), then block-wise per-channel asymmetric uniform
 *           quantization over groups of G_k tokens;
 *   values: per-token asymmetric uniform quantization over groups of G_v
 *           channels (no run-time rotation or scaling);
 *   new tokens wait in a 16-bit residual window of R tokens and are quantized
 *   block-wise once R of them have accumulated;
 *   decode attention rotates the query the same way, dequantizes on the fly,
 *   multiplies the key logits by the stored token norms and runs
 *   softmax(q K^T) V over packed + residual tokens.
 * (Paper: Sec. "Block-Wise Per-Channel Quantization" Eq. 3-4; Sec. "The OScaR
 * Framework"; Sec. "Efficient System Design and CUDA Implementations";
 * App. "Implementation Details of OScaR's CUDA Kernels"; Algorithm
 * "The OScaR algorithm".)
 *
 * Conventions
 *  - Every pointer named "device" is GPU memory owned by the caller; the library
 *    never allocates, frees or retains device memory.  Its only process-wide state is the
 *    cached compute-unit count per device and the oscar_debug_force_generic_decode switch.
 *  - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL =
 *    the default stream). They do not synchronize and never read device memory
 *    on the host (oscar_debug_dump excepted), which is why upper bounds on
 *    sequence lengths are passed as hints.
 *  - Return value: OSCAR_OK (0) or a negative OSCAR_ERR_* code. When an argument
 *    check fails nothing is enqueued. No C++ exception crosses this boundary.
 *  - Calls that touch the same cache on different streams race; order them.
 */
#ifndef OSCAR_H_
#define OSCAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OSCAR_VERSION 100 /* 0.1.0 */

/* element types */
enum { OSCAR_F32 = 0, OSCAR_BF16 = 1, OSCAR_F16 = 2 };
/* zero-point form: integer z = round(-min/Delta) (Eq. 3-4) or float zero = min */
enum { OSCAR_ZP_INT = 0, OSCAR_ZP_MIN = 1 };
/* scope of the token norm: one norm per (token, kv head) (App. "Overall Design": n_k is the
 * norm of the head's vector), or one per token from the squared sums of all kv heads (App.
 * "Fused Hadamard-Norm Kernel"); the cache layout is the same, every head's norm slot of a
 * token then holds the same value */
enum { OSCAR_NORM_PER_HEAD = 0, OSCAR_NORM_ALL_KV_HEADS = 1 };
/* ablation switches (App. "Ablation Study"); 0 everywhere = the method as published */
enum { OSCAR_ROTATION_ON = 0, OSCAR_ROTATION_OFF = 1 }; /* OFF: no Hadamard on K nor on Q */
/* per-token scaling coefficient n: L2 norm; none (n = 1); maximum absolute value over the
 * token's channels; mean absolute value over them */
enum { OSCAR_SCALE_L2 = 0, OSCAR_SCALE_NONE = 1, OSCAR_SCALE_MAX = 2, OSCAR_SCALE_MEAN_ABS = 3 };
/* status codes */
enum {
  OSCAR_OK = 0,
  OSCAR_ERR_INVALID_ARG = -1, /* null pointer, negative size, inconsistent fields */
  OSCAR_ERR_UNSUPPORTED = -2, /* valid in the paper's terms but not built (see oscar_config) */
  OSCAR_ERR_CAPACITY = -3,    /* the hint shows a sequence would outgrow its block table */
  OSCAR_ERR_WORKSPACE = -4,   /* workspace missing or too small */
  OSCAR_ERR_HIP = -5          /* a HIP runtime call or kernel launch failed */
};
/* flags of oscar_quantize_append */
enum {
  OSCAR_APPEND_EAGER = 1u /* prefill rule: quantize every completed block at once */
};

/* Parameters of the method (Algorithm "The OScaR algorithm": G, R, d_h; Eq. 3-4: b).
 * Checked on every call. Built: head_dim 128; bits 2|4; k_group 32|64|128;
 * v_group 32|64|128; page_size 128; io_dtype any; meta_dtype F16|F32;
 * zp_mode OSCAR_ZP_INT|OSCAR_ZP_MIN; norm_scope either; rotation either; scale_mode any;
 * n_q_heads/n_kv_heads <= 8.
 * Anything else returns OSCAR_ERR_UNSUPPORTED. */
typedef struct oscar_config {
  int32_t head_dim;    /* d_h */
  int32_t n_q_heads;   /* query heads; multiple of n_kv_heads; q head h reads kv head h / g */
  int32_t n_kv_heads;
  int32_t bits;        /* b */
  int32_t k_group;     /* G for keys: tokens per per-channel group; divides page_size */
  int32_t v_group;     /* G for values: channels per per-token group; divides head_dim */
  int32_t page_size;   /* R: residual length = flush block = tokens per page */
  int32_t io_dtype;    /* element type of k, v, q and of the value residual */
  int32_t meta_dtype;  /* storage type of Delta, zero-point and token norm */
  int32_t zp_mode;
  int32_t norm_scope;
  int32_t rotation;    /* OSCAR_ROTATION_ON | OSCAR_ROTATION_OFF */
  int32_t scale_mode;  /* OSCAR_SCALE_*; anything but L2 needs OSCAR_NORM_PER_HEAD */
} oscar_config;

/* The paged cache. Plain data; every pointer is DEVICE memory the caller
 * allocated with the sizes oscar_cache_sizes reports (256-byte aligned).
 *
 * Packed part: logical page p of sequence b is physical page block_table[b][p];
 * a physical page holds R tokens of ALL kv heads; pools are indexed
 * [physical page][kv head][bytes]. Inside a page the bytes are ordered for the
 * matrix-core decode kernel (a 64-lane wave loads a 16 x 32-code operand tile as one
 * contiguous block and each lane's codes are already in operand order); use
 * oscar_debug_dump to read a cache in plain [token][channel] form.
 *   k_codes : 8 tiles of 16 tokens; lane (n = t%16, q4) owns the "chunk" of channels
 *             32*q4..32*q4+31 of token 16*tile+n, code of channel 32*q4+u at bit u*bits;
 *             tiles are stored in pairs: chunk (tile, n, q4) starts at byte
 *             ((tile/2)*64 + n*4 + q4) * 8*bits + (tile%2) * 4*bits
 *   v_codes : same structure with 8 tiles of 16 channels; chunk q4 holds the 32 tokens
 *             with t%4 == q4, token 16*e + 4*kk + q4 at code number
 *             slot(kk, e) = 16*(kk/2)+4*(kk%2)+e/2+8*(e%2) (2-bit), 8*kk+e/2+4*(e%2) (4-bit)
 *   k_meta  : Delta[R/k_group][head_dim] then zero[R/k_group][head_dim] (meta_dtype), the
 *             channel axis in operand order: position 32*q4+8*kk+e = channel 32*q4+slot(kk,e)
 *   k_norms : n[R] (meta_dtype), token t at position (t%16)*8 + t/16
 *   v_meta  : Delta[head_dim/v_group][R] then zero[head_dim/v_group][R] (meta_dtype),
 *             token axis as in k_norms
 * Residual part, indexed [sequence][kv head]:
 *   res_k   : [R][head_dim] fp16, rotated and normalized keys K_u (an element that is
 *             exactly zero may be stored as -0)
 *   res_v   : [R][head_dim] io_dtype
 *   res_norm: [R] meta_dtype
 * State: seq_lens[b] = tokens held for sequence b; res_lens[b] of them (0..R,
 * the most recent ones) are in the residual, the rest fill
 * (seq_lens[b]-res_lens[b])/R whole pages. A fresh cache has both arrays zeroed.
 * dev_status (may be NULL): a device int32 the kernels set to OSCAR_ERR_CAPACITY
 * when a sequence would need more than max_pages_per_seq pages; that append is
 * dropped for that sequence.
 * tickets (may be NULL): a device int32[1], zeroed once by the caller. With it the last
 * workgroup of oscar_quantize_append to finish also advances seq_lens / res_lens (one
 * launch) and leaves the ticket zero again; without it, and for appends of 128 tokens or more
 * whose grid exceeds 1024 workgroups (prefills), the length update is a second, tiny launch. */
typedef struct oscar_cache {
  oscar_config cfg;
  int32_t batch;
  int32_t max_pages_per_seq;
  int32_t num_pages;
  int32_t reserved_;
  void *k_codes, *k_meta, *k_norms, *v_codes, *v_meta;
  void *res_k, *res_v, *res_norm;
  int32_t *block_table; /* [batch][max_pages_per_seq], values in [0, num_pages) */
  int32_t *seq_lens;    /* [batch] */
  int32_t *res_lens;    /* [batch] */
  int32_t *dev_status;  /* [1] or NULL */
  int32_t *tickets;     /* [1] zero-initialised, or NULL */
} oscar_cache;

/* Byte sizes of every pool for `batch` sequences and `num_pages` physical pages. */
typedef struct oscar_pool_sizes {
  size_t k_codes, k_meta, k_norms, v_codes, v_meta; /* whole pools */
  size_t res_k, res_v, res_norm;
  size_t block_table, seq_lens, res_lens, tickets;
  size_t page_bytes_per_kv_head;  /* packed bytes of one page of one kv head (all five pools) */
  size_t bytes_per_token_kv_head; /* = page_bytes_per_kv_head / page_size */
} oscar_pool_sizes;

int oscar_version(void);
const char *oscar_status_string(int status);

/* Validates cfg and fills *out. Host only. */
int oscar_cache_sizes(const oscar_config *cfg, int32_t batch, int32_t num_pages,
                      int32_t max_pages_per_seq, oscar_pool_sizes *out);

/* A model keeps one cache per layer (Algorithm "The OScaR algorithm": OScaR-Inference runs in
 * every layer on that layer's K, V, Q); its L layers share ONE block table (a token's page has
 * the same number in every layer) and differ in everything else.  Layout of a multi-layer
 * cache: `all_layers` describes the whole allocation --
 *   k_codes, k_meta, k_norms, v_codes, v_meta, res_k, res_v, res_norm : [n_layers] slices, each
 *       of the size oscar_cache_sizes reports for (batch, num_pages, max_pages_per_seq), so a
 *       pool is indexed [layer][physical page][kv head][bytes]; num_pages = pages PER LAYER
 *   seq_lens, res_lens : [n_layers][batch]  (a decoding step appends to layer 0 and attends in
 *       layer 0 before layer 1 has seen the token, so the lengths are per-layer state)
 *   tickets : [n_layers] (or NULL), dev_status : shared, block_table : shared
 * oscar_cache_layer fills *layer_cache with the view of one layer (pointer arithmetic on the
 * host, nothing else); the view is an ordinary oscar_cache for every other call, and views of
 * different layers may be used on different streams at the same time.
 * Returns OSCAR_ERR_INVALID_ARG for NULL arguments, n_layers < 1 or layer outside
 * [0, n_layers), and whatever oscar_cache_sizes returns for the configuration. */
int oscar_cache_layer(const oscar_cache *all_layers, int32_t n_layers, int32_t layer,
                      oscar_cache *layer_cache);

/* Number of sequence splits oscar_decode_attn uses when num_splits == 0, for the
 * device current at the time of the call. Host only; >= 1. */
int32_t oscar_decode_auto_splits(const oscar_config *cfg, int32_t batch, int32_t max_seq_len);

/* Bytes of split-K scratch oscar_decode_attn needs for `num_splits` splits
 * (fp32 partial outputs and softmax statistics per batch, query head and split). */
size_t oscar_decode_workspace_bytes(const oscar_config *cfg, int32_t batch, int32_t num_splits);

/* KV-cache compression: BufferQuantK / BufferQuantV of the algorithm, with the
 * key transform K_h = H(K)/sqrt(d), n = ||K_h||, K_u = K_h/n fused in front.
 *   k, v     : device, [batch][T][n_kv_heads][head_dim] contiguous, io_dtype,
 *              the T newest tokens of every sequence (keys after RoPE, un-rotated)
 *   new_lens : device int32[batch] or NULL; sequence b appends its first
 *              new_lens[b] (0..T) tokens; NULL = T for all
 *   max_seq_len_hint : upper bound on seq_lens[] BEFORE the call, or < 0 if
 *              unknown; used only for the host-side capacity check
 *   flags    : OSCAR_APPEND_EAGER = prefill rule (every completed block of R
 *              tokens is quantized by this call, the tail < R stays 16-bit).
 *              Default = decode rule: a block completed by this call stays in the
 *              residual through the attention that follows (the algorithm attends
 *              before it flushes) and is quantized by the next append.
 * Updates seq_lens / res_lens on the device. Residual keys are quantized from
 * their stored fp16 values (no second rotation). A sequence that receives no token
 * (T == 0 or new_lens[b] == 0) is left untouched under either rule.
 * One launch (plus the length-update launch without cache->tickets or for a large grid); with
 * OSCAR_NORM_ALL_KV_HEADS a launch in front computes the norms of the new tokens that
 * move into pages and parks them in those pages' norm slots. */
int oscar_quantize_append(const void *k, const void *v, int32_t T, const int32_t *new_lens,
                          oscar_cache *cache, int32_t max_seq_len_hint, uint32_t flags,
                          void *stream);

/* Fused decode attention over the packed + residual cache (kernel (iii) of the
 * paper's system design; OScaR-Inference lines K_all, V_all, Attention):
 *   out[b][h] = softmax_i( scale * n_i * <Q_h, dequant(K_u,i)> ) . dequant(V_i)
 * with Q_h = H(q)/sqrt(d) computed inside (pass the UN-rotated query).
 *   q   : device, [batch][n_q_heads][head_dim], io_dtype
 *   out : device, [batch][n_q_heads][head_dim], out_dtype (OSCAR_F32 or io_dtype)
 *   softmax_scale : <= 0 means 1/sqrt(head_dim)
 *   max_seq_len_hint : upper bound on seq_lens[] (>= 0; negative = OSCAR_ERR_INVALID_ARG);
 *                only used to choose the split count when num_splits == 0 (0 gives one split)
 *   num_splits : split-K factor over the sequence (<= 512), 0 = oscar_decode_auto_splits
 *   workspace  : device scratch of at least oscar_decode_workspace_bytes(...)
 * A sequence with seq_lens[b] == 0 yields zeros.
 * Two launches (split-K partial pass, reduce pass); with a single split the matrix-core kernel
 * writes `out` itself and the reduce launch is left out (same bits: the same sums, divided the
 * same way; the workspace is still required and may then stay untouched).
 * Two kernels sit behind this call: the matrix-core one (fp16 metadata; scale_mode L2 or MAX,
 * i.e. keys scaled into [-1, 1]) and a generic plain-ALU one for every other configuration
 * (fp32 metadata; scale_mode NONE or MEAN_ABS); both are checked against the same
 * oracle.  oscar_debug_force_generic_decode selects the generic kernel for every
 * configuration; it exists for tests and profiling. */
int oscar_decode_attn(const void *q, const oscar_cache *cache, void *out, int32_t out_dtype,
                      float softmax_scale, int32_t max_seq_len_hint, int32_t num_splits,
                      void *workspace, size_t workspace_bytes, void *stream);

/* One decoding step of Algorithm "The OScaR algorithm" (OScaR-Inference, decoding phase) in one
 * call: oscar_quantize_append of ONE new token per sequence under the decode rule, then
 * oscar_decode_attn over the updated cache -- the same launches, one trip through the ABI.
 *   k_new, v_new : device, [batch][1][n_kv_heads][head_dim], io_dtype
 *   q, out, out_dtype, softmax_scale, num_splits, workspace: as in oscar_decode_attn
 *   max_seq_len_hint : upper bound on seq_lens[] AFTER this step's append (>= 1)
 *   partial_timer : NULL, or a timer that receives the duration of the split-K partial kernel
 *                   of this step (measurement aid, see oscar_timer_create)
 * Every argument is checked before anything is enqueued; OSCAR_ERR_CAPACITY as in
 * oscar_quantize_append. */
typedef struct oscar_timer oscar_timer;
int oscar_decode_step(const void *k_new, const void *v_new, const void *q, oscar_cache *cache,
                      void *out, int32_t out_dtype, float softmax_scale, int32_t max_seq_len_hint,
                      int32_t num_splits, void *workspace, size_t workspace_bytes, void *stream,
                      oscar_timer *partial_timer);

/* For callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  oscar_decode_attn with the
 * split-K partials kept in a fixed buffer of OSCAR_NOALLOC_SCRATCH_BYTES inside the library's
 * device image (every GPU the library runs on holds its own copy until the process ends);
 * same kernels, same results.  The call allocates and frees nothing.
 *  - num_splits == 0 picks the split count as oscar_decode_attn does; a configuration whose
 *    partials (oscar_decode_workspace_bytes) exceed the buffer returns OSCAR_ERR_WORKSPACE and
 *    enqueues nothing (pass fewer splits, or use oscar_decode_attn with your own workspace).
 *  - The first call on a device resolves the buffer's address (one runtime query, no
 *    allocation); make that call once before starting a stream capture.
 *  - All calls on one GPU share the one buffer: calls that overlap on different streams of the
 *    same GPU race; serialize them.  Nothing has to be cleared between calls. */
#define OSCAR_NOALLOC_SCRATCH_BYTES (4u << 20)
int oscar_decode_attn_noalloc(const void *q, const oscar_cache *cache, void *out,
                              int32_t out_dtype, float softmax_scale, int32_t max_seq_len_hint,
                              int32_t num_splits, void *stream);

/* Test / profiling switch: on != 0 makes every later decode launch of this process take the
 * generic plain-ALU kernel, 0 restores the automatic choice.  Returns the previous setting.
 * Host only, thread-safe (one atomic flag). */
int oscar_debug_force_generic_decode(int32_t on);

/* The two passes of oscar_decode_attn as separate calls, for callers that want to time
 * or overlap them: oscar_decode_attn(...) == partial(...) followed by reduce(...) on the
 * same stream with the same num_splits (> 0 here) and workspace (these two always go through
 * the workspace, also for a single split).
 * (Split-K partial pass: per (sequence, kv head, split) online-softmax attention over a
 * range of pages, all query heads of the group sharing each packed tile; reduce pass:
 * log-sum-exp merge of the splits.) */
int oscar_decode_attn_partial(const void *q, const oscar_cache *cache, float softmax_scale,
                              int32_t num_splits, void *workspace, size_t workspace_bytes,
                              void *stream);
int oscar_decode_attn_reduce(const oscar_cache *cache, void *out, int32_t out_dtype,
                             int32_t num_splits, const void *workspace, size_t workspace_bytes,
                             void *stream);

/* Stand-alone Canalized Rotation, with or without Omni-Token Scaling (kernel (i) of Sec.
 * "Efficient System Design"; App. "Implementation Details", "Overall Design"), on n_vec
 * vectors of 128 channels, x: device [n_vec][128] of io_dtype.
 *   flags = 0                      : out = H(x)/sqrt(128), device [n_vec][128] fp32 (queries);
 *                                    norms ignored
 *   OSCAR_ROTATE_NORMALIZE         : norms[v] = ||H(x_v)/sqrt(128)||_2 rounded to meta_dtype
 *                                    (F16|F32), out = fp16 [n_vec][128] of the quotient by the
 *                                    stored norm: exactly what oscar_quantize_append keeps in the
 *                                    residual window
 *   ... | OSCAR_ROTATE_FAST_RSQRT  : the norm through the hardware reciprocal square root
 *                                    (the paper's fast variant) instead of sqrt and divide;
 *                                    results agree with the exact mode to about one fp16 ulp
 *                                    and are not bit-reproducible on a CPU
 *   ... | OSCAR_ROTATE_MATRIX_CORE : the rotation as H_8 (x) H_16 with the H_16 factor on matrix
 *                                    cores (App. "Fused Hadamard-Norm Kernel"); 16-bit io_dtype
 *                                    only (OSCAR_ERR_UNSUPPORTED for F32).  Same values up to fp32
 *                                    rounding (another summation order), so not bit-identical
 *                                    to the cache path; combines with the two flags above
 * Returns OSCAR_ERR_INVALID_ARG for NULL pointers, unknown flags, or FAST_RSQRT without
 * NORMALIZE. */
enum { OSCAR_ROTATE_NORMALIZE = 1u, OSCAR_ROTATE_FAST_RSQRT = 2u, OSCAR_ROTATE_MATRIX_CORE = 4u };
int oscar_rotate(const void *x, void *out, void *norms, int64_t n_vec, int32_t io_dtype,
                 int32_t meta_dtype, uint32_t flags, void *stream);

/* Rotation along the row axis of a matrix, for the offline weight preprocessing of Algorithm
 * "The OScaR algorithm" (OScaR-Preprocess: W_V <- W_V H, W_O <- H W_O, one H per head):
 *   w   : device [n_rows][n_cols] of io_dtype, row-major, n_rows a multiple of 128
 *   out : device [n_rows][n_cols] fp32; for every block of 128 rows (one head) and every
 *         column c: out[128 h + i][c] = sum_j H[i][j] w[128 h + j][c] / sqrt(128)
 * With W_O stored [n_q_heads*128][d_model] this call is H W_O; W_V stored
 * [d_model][n_kv_heads*128] takes oscar_rotate (flags 0) on its rows' head segments (H is
 * symmetric: a row times H is H times the row); the transposed storage convention swaps the
 * two calls.  The same butterfly order as everywhere else, so results are bit-identical to
 * oscar_rotate on the transposed matrix.
 * Returns OSCAR_ERR_INVALID_ARG for NULL pointers, negative sizes or n_rows % 128 != 0. */
int oscar_rotate_columns(const void *w, void *out, int64_t n_rows, int64_t n_cols,
                         int32_t io_dtype, void *stream);

/* Measurement aid (not part of the method): a timer owns a pair of HIP events.
 * oscar_decode_attn_partial_timed is oscar_decode_attn_partial with the events attached to
 * the kernel's own dispatch (start/stop events of an extended launch), so that
 * oscar_timer_elapsed_us returns the device time from that dispatch's start marker to its
 * stop marker, with no other kernel in between.  oscar_timer_elapsed_us waits for the kernel; it returns
 * OSCAR_ERR_INVALID_ARG for a timer no launch has used yet.  A timer may be reused by a
 * later launch once its elapsed time has been read.  The caller destroys what it creates. */
int oscar_timer_create(oscar_timer **timer);
int oscar_timer_destroy(oscar_timer *timer);
int oscar_timer_elapsed_us(oscar_timer *timer, float *us);
int oscar_decode_attn_partial_timed(const void *q, const oscar_cache *cache, float softmax_scale,
                                    int32_t num_splits, void *workspace, size_t workspace_bytes,
                                    void *stream, oscar_timer *timer);

/* Measurement aid: reads `bytes` bytes of device memory at `src` (16-byte aligned) once, with
 * `workgroups` workgroups of 256 threads issuing wave-wide 1 KB loads, and nothing else.
 * `bytes` must be a multiple of 32768 * workgroups (OSCAR_ERR_INVALID_ARG otherwise; nothing
 * outside [src, src + bytes) is touched).  `sink` (device, 4 bytes, may be NULL) only keeps
 * the loads alive.  With a timer, oscar_timer_elapsed_us gives the kernel's time: the HBM
 * read bandwidth this timing method reports for a pure stream, next to which the decode
 * kernel's figure can be read. */
int oscar_probe_stream_read(const void *src, size_t bytes, int32_t workgroups, void *sink,
                            void *stream, oscar_timer *timer);

/* 16-bit comparator: the same split-K decode attention on an uncompressed,
 * un-rotated cache (the BF16 FlashDecoding-style baseline of the paper's
 * efficiency section).
 *   q : device [batch][n_q_heads][d];
 *   k, v : device, kv_layout OSCAR_KV_TOKEN_MAJOR: [batch][kv_stride_tokens][n_kv_heads][d],
 *          OSCAR_KV_HEAD_MAJOR: [batch][n_kv_heads][kv_stride_tokens][d] (each kv head's tokens
 *          contiguous, as in a paged 16-bit cache);
 *   all of `dtype` (OSCAR_BF16 or OSCAR_F16); seq_lens: device int32[batch] (<= kv_stride_tokens);
 *   out: device [batch][n_q_heads][d] of out_dtype (OSCAR_F32 or dtype);
 *   workspace as oscar_decode_workspace_bytes for the same head counts. */
enum { OSCAR_KV_TOKEN_MAJOR = 0, OSCAR_KV_HEAD_MAJOR = 1 };
int oscar_bf16_decode_attn(const void *q, const void *k, const void *v, const int32_t *seq_lens,
                           void *out, int32_t dtype, int32_t out_dtype, int32_t batch,
                           int32_t kv_stride_tokens, int32_t kv_layout, int32_t n_q_heads,
                           int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                           int32_t max_seq_len_hint, int32_t num_splits, void *workspace,
                           size_t workspace_bytes, void *stream);

/* Test/debug: copy sequence b, kv head h back to the HOST in a layout-free
 * form (one code per byte). Synchronizes `stream`. Host outputs, each may be
 * NULL; `cap_tokens` is the token capacity of the caller's arrays.
 *   k_codes[cap][d], k_delta/k_zero[cap/k_group][d], k_norm[cap],
 *   v_codes[cap][d], v_delta/v_zero[cap][d/v_group],
 *   res_k[R][d], res_v[R][d] (fp32 widened), res_norm[R];
 *   lens[2] = {seq_len, res_len}. */
int oscar_debug_dump(const oscar_cache *cache, int32_t b, int32_t h, int32_t cap_tokens,
                     uint8_t *k_codes, float *k_delta, float *k_zero, float *k_norm,
                     uint8_t *v_codes, float *v_delta, float *v_zero, float *res_k,
                     float *res_v, float *res_norm, int32_t *lens, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OSCAR_H_ */
