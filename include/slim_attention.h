/*
 * slim_attention.h -- C ABI of the MI355X (gfx950) slim-attention decode library.
 *
 * One multi-head-attention generation step that reads only a K-cache (paper: "K-cache is
 * all you need", eq. 6 and eq. 7 option 2):
 *
 *     p_h   = softmax(q_h K_h^T / sqrt(d_k))              (eq. 2, no causal mask)
 *     out_h = (p_h K) W_KV[:, h-th column block]          (eq. 7, option 2)
 *     W_KV  = W_K^{-1} W_V                                (eq. 6, prepared once, offline)
 *
 * Conventions shared by every entry point
 *   - Row vectors, weights are W[in][out] row-major, head h owns the column block
 *     [h*d_k, (h+1)*d_k) of the projection width e = H*d_k (text below eq. 2).
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory of
 *     the current device.  All buffers are owned by the caller; the library never frees or
 *     retains them beyond the call (device work is asynchronous on `stream`, so the caller
 *     keeps buffers alive until the stream has passed the call).
 *   - Device pointers must be 16-byte aligned; row pitches are dense.
 *   - Every function returns SLIM_OK (0) or a negative SLIM_ERR_* code; nothing throws or
 *     aborts.  Argument errors are detected on the host before anything is launched.
 *   - Waits between workgroups inside the kernels are bounded in real time; if one ever runs out
 *     (the launch's workgroups were not all resident together), the outputs of that call are
 *     written as NaN instead of the kernel hanging, and slim_status reports SLIM_ERR_TIMEOUT.
 *   - q is the already projected, un-scaled query (the library applies 1/sqrt(d_k)); out is
 *     concat(head_1..head_H) before W_O (eq. 5).  Attention runs over exactly the cached
 *     rows handed in (the caller appends the new token's key first if it wants it attended).
 */
#ifndef SLIM_ATTENTION_H
#define SLIM_ATTENTION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------------------- */
#define SLIM_OK              0
#define SLIM_ERR_ARG        -1   /* null pointer, negative size, option the call does not take */
#define SLIM_ERR_SHAPE      -2   /* d % H != 0, d_k not a multiple of the 16-byte vector, T<1 */
#define SLIM_ERR_DTYPE      -3   /* dtype is neither SLIM_F32 nor SLIM_BF16                   */
#define SLIM_ERR_ALIGN      -4   /* a device pointer is not 16-byte aligned                   */
#define SLIM_ERR_WORKSPACE  -5   /* caller workspace smaller than slim_workspace_bytes()      */
#define SLIM_ERR_SINGULAR   -6   /* W_K is singular to working precision (zero pivot)         */
#define SLIM_ERR_ILLCOND    -7   /* result written, but rcond(W_K) < 1e-12: do not trust it   */
#define SLIM_ERR_LAUNCH     -8   /* HIP reported an error at allocation or launch             */
#define SLIM_ERR_SEQLEN     -9   /* a host-side sequence length is < 1 or > T                 */
#define SLIM_ERR_TIMEOUT   -10   /* slim_status: a wait between workgroups ran out (outputs NaN) */
#define SLIM_ERR_LAYOUT    -11   /* opts->k_layout: rows per sequence not a multiple of 32, or a shape or
                                    dtype whose kernels read row-major caches only              */

/* ---- element types of the cache and of packed weights -------------------------------- */
#define SLIM_F32   0
#define SLIM_BF16  1

const char* slim_strerror(int code);

/* ---- offline weight transform (host, fp64, not on the timed path) --------------------- */

/* eq. 6:  W_KV = W_K^{-1} W_V, computed as an LU solve with partial pivoting in fp64
 * (App. A uses fp64 for the inversion; solving W_K W_KV = W_V is the same result with
 * fewer operations than forming the inverse).
 *   Wk, Wv  : host, row-major d x d fp64, read only
 *   Wkv     : host, row-major d x d fp64, written
 *   rcond_out: host, nullable; receives a 1-norm reciprocal condition estimate of W_K
 * Returns SLIM_ERR_SINGULAR (Wkv untouched garbage) on a zero pivot or non-finite input,
 * SLIM_ERR_ILLCOND (Wkv written) when the estimate is below 1e-12. */
int slim_prepare_wkv(const double* Wk, const double* Wv, double* Wkv, int d, double* rcond_out);

/* Non-square projections, option 1 of that section: W_K is d x e with e > d; its right inverse
 * W_K^T (W_K W_K^T)^{-1} gives  W_KV = W_K^T (W_K W_K^T)^{-1} W_V  (e x e), and (X W_K) W_KV = X W_V.
 * The decode step is then slim_decode on the e-wide K-cache with this e x e matrix (its `d` := e).
 *   Wk, Wv : host fp64 row-major [d][e];  Wkv : host fp64 row-major [e][e], written
 *   rcond_out: nullable; reciprocal condition estimate of W_K W_K^T (the square of W_K's)
 * Errors as slim_prepare_wkv; SLIM_ERR_SHAPE when e < d. */
int slim_prepare_wkv_nonsquare(const double* Wk, const double* Wv, double* Wkv, int d, int e,
                               double* rcond_out);

/* Cast a host fp64 row-major rows x cols matrix to the device element type (round to
 * nearest even, via fp32 for bf16), same row-major layout.  This is the form `W_KV`
 * (d x d) and the X-cache weights (d_model x e) are handed to the decode calls; the
 * caller copies `dst_host` (rows*cols*elemsize bytes, host) to the device. */
int slim_pack_weights(const double* W, void* dst_host, int rows, int cols, int dtype);

/* Host copy of a row-major K-cache [B][t_stride][H*d_k] into the banded layout (SLIM_K_BANDED) of the same
 * size; elem_bytes = 2 or 4; t_stride % 32 == 0 (SLIM_ERR_LAYOUT otherwise).  src and dst are host
 * buffers of B * t_stride * H * d_k elements and must not overlap. */
int slim_band_kcache(const void* src_host, void* dst_host, int B, int64_t t_stride, int H, int d_k,
                     int elem_bytes);

/* The look-up table of the RoPE appendix, one table for encoding and decoding:
 *   table[t][j] = { cos(t * theta_j), sin(t * theta_j) },  theta_j = base^(-2j/d_k),
 * for positions t = 0 .. T-1 and the d_k/2 adjacent column pairs (2j, 2j+1) of a head, angles
 * and functions evaluated in fp64, stored as fp32.  The appendix names only "m theta"; the
 * frequencies are those of the RoPE paper it cites (base 10000 there).
 *   table_host: host, T*(d_k/2)*2 floats, written.  d_k even, base > 0. */
int slim_rope_table(float* table_host, int T, int d_k, double base);

/* ---- options -------------------------------------------------------------------------- */
typedef struct slim_opts {
  int            dtype;          /* SLIM_F32 | SLIM_BF16: elements of Kcache/Vcache/X and weights */
  const int32_t* seq_lens;       /* device [B], nullable => every sequence attends T rows;
                                    1 <= seq_lens[b] <= T (ragged batches)                        */
  const int32_t* seq_lens_host;  /* host copy of seq_lens, nullable; only validated (1 <= len <= T,
                                    SLIM_ERR_SEQLEN): the work is partitioned on the device from
                                    seq_lens, a call without the host copy is as fast             */
  int64_t        t_stride;       /* cache rows between consecutive sequences, 0 => T              */
  void*          workspace;      /* device scratch, nullable => library-owned, grown on demand
                                    with hipMalloc and kept per device until process exit.  Calls
                                    that may overlap on one device (different streams or threads)
                                    need a workspace each: the library-owned one is shared, and
                                    growing it frees the old block after waiting for the device.
                                    (The bf16 fast path uses the whole chip per launch; the library
                                    orders such launches of different streams one after the other) */
  size_t         workspace_bytes;
  void*          stream;         /* hipStream_t, null => the null stream                          */
  int            variant;        /* 0 = library's choice; other values select an implementation
                                    (see SLIM_VARIANT_*), for tests and tuning                    */
  float*         stage_ms;       /* host [SLIM_MAX_STAGES], nullable.  Measurement only: when set,
                                    the call brackets each of its kernels with HIP events on
                                    `stream`, waits for the stream, and writes each kernel's
                                    milliseconds in launch order (unused entries = 0)             */
  const float*   rope_table;     /* device fp32 [T][d_k/2][2] from slim_rope_table, nullable => keys
                                    carry no rotary position.  slim_decode only (see there)       */
  int64_t        wait_budget_us; /* bound of every wait between workgroups of the bf16 fast path, in
                                    microseconds of real time: 0 => 20000; negative => no waiting at
                                    all (every wait that is not satisfied at once gives up: for tests
                                    of the failure path, see slim_status)                          */
  int            k_layout;       /* SLIM_K_ROWMAJOR (0) | SLIM_K_BANDED: layout of Kcache in slim_decode,
                                    slim_decode_static and slim_attention_block (see SLIM_K_BANDED)  */
} slim_opts;

/* Layouts of the K-cache of one sequence (sequences are t_stride * d elements apart in both).
 * Which elements a step reads is the method's (the first seq_lens[b] rows, eq. 7); where they sit in
 * memory is the cache's own business, and the kernel that streams them is bound by HBM:
 *   SLIM_K_ROWMAJOR  [t][d]: element (t, h, j) at t*d + h*d_k + j.
 *   SLIM_K_BANDED    [t / 32][H][32][d_k]: bands of 32 rows, head-major inside a band, element
 *                    (t, h, j) at ((t / 32) * H + h) * 32 * d_k + (t % 32) * d_k + j.  A head's 32 x d_k
 *                    block (the unit a wave of the stream kernel loads) is one contiguous run of
 *                    64 * d_k bytes instead of 32 row pieces of 2 * d_k bytes, which for head widths
 *                    that are not a multiple of 64 elements (d_k = 96: 192-byte pieces, one and a half
 *                    cache lines) is the difference between 4.4 and 5.0 TB/s on the long batch.
 *                    t_stride % 32 == 0; bf16 shapes the stream kernel takes (H <= 32, 16 <= d_k <= 128
 *                    on a device where it fits), else SLIM_ERR_LAYOUT.  slim_attention_block appends
 *                    the new row in this layout; slim_band_kcache converts a host copy. */
#define SLIM_K_ROWMAJOR 0
#define SLIM_K_BANDED   1

#define SLIM_MAX_STAGES 8

#define SLIM_VARIANT_AUTO      0
#define SLIM_VARIANT_GENERIC   1   /* plain vector-ALU kernels, any supported shape            */
#define SLIM_VARIANT_FUSED_SPLIT 2 /* as FUSED, but the merge + projection always runs as a launch of
                                      its own; slim_decode_xcache: scores and weighted sum as two
                                      passes over X even where the one-pass kernel applies     */
#define SLIM_VARIANT_FUSED     3   /* bf16, H <= 32, d_k <= 128: single pass over K with the weighted
                                      sum and the projection on MFMA (one launch when B <= 16, else
                                      two); falls back to GENERIC when the shape does not qualify */

/* Per-device set-up for the current device, idempotent and thread-safe: looks up the address of the
 * library's static device array, counts the compute units, checks with one probe launch on the null stream (plus a
 * blocking read-back; no allocation) that consecutive workgroups of a launch are spread round-robin
 * over the XCDs, and creates the event that orders launches of different streams.  The decode calls
 * do this themselves on first use; calling it up front keeps that work (and its synchronisation) out
 * of the first decode call, e.g. before a stream capture starts.  SLIM_ERR_LAUNCH when HIP fails. */
int slim_init(void);

/* Whether the waits between workgroups of the latest bf16 fast-path launch that used this workspace
 * ended normally.  The decode calls are asynchronous and return before their kernels have run, so a
 * wait that runs out inside a kernel (the chip could not keep the launch's workgroups resident
 * together within opts->wait_budget_us, e.g. because other work held compute units) cannot be reported
 * by the call itself: the kernel raises an error word in the workspace and writes NaN outputs.  This
 * query waits for `stream` (hipStream_t, null => the null stream), reads the word back and returns
 * SLIM_ERR_TIMEOUT or SLIM_OK.  The fast path needs the chip free of other kernels while it runs.
 *   workspace: the device scratch the call was given; NULL => the library-owned scratch of the
 *              current device; SLIM_STATIC_SCRATCH => the scratch of slim_decode_static. */
#define SLIM_STATIC_SCRATCH ((const void*)(uintptr_t)1)
int slim_status(const void* workspace, void* stream);

/* The implementation SLIM_VARIANT_AUTO resolves to for a K-cache decode of this shape
 * (one of the SLIM_VARIANT_* values above, never AUTO); 0 on invalid arguments. */
int slim_variant_for(int B, int H, int T, int d, int dtype);

/* Upper bound of the device scratch slim_decode / vanilla_kv_decode need for this shape. */
size_t slim_workspace_bytes(int B, int H, int T, int d, int dtype);
/* The same for slim_decode_xcache (projection width H*d_k, cache width d_model). */
size_t slim_workspace_bytes_xcache(int B, int H, int T, int d_model, int d_k, int dtype);

/* ---- the decode step ------------------------------------------------------------------- */

/* eq. 7 option 2 for B sequences, one new token each.
 *   q      : device fp32 [B][d]           projected, un-scaled queries
 *   Kcache : device dtype [B][t_stride][d] cached keys K = X W_K (eq. 4); only rows
 *            [0, seq_lens[b]) of sequence b are read
 *   W_KV   : device dtype [d][d]          from slim_prepare_wkv + slim_pack_weights
 *   out    : device fp32 [B][d]           concat of heads, written
 *   d = H*d_k.  No V-cache exists anywhere in this call.
 * With opts->rope_table set (RoPE appendix, option 1): the cache holds the raw keys, cached row t
 * of every sequence sits at position t, and each key row is rotated by its position after it is
 * read, for the softmax arguments only -- per head and adjacent pair (x1, x2):
 *   y1 = x1 cos + x2 sin,  y2 = -x1 sin + x2 cos -- while the raw rows enter the weighted sum.
 * q is taken as given (the caller has rotated it to the new token's position).
 * vanilla_kv_decode and slim_decode_xcache return SLIM_ERR_ARG when the table is set: a vanilla
 * cache stores rotated keys and needs no table, and a position-dependent rotation cannot be
 * folded into the X-cache scheme's query. */
int slim_decode(const void* q, const void* Kcache, const void* W_KV, void* out,
                int B, int H, int T, int d, const slim_opts* opts);

/* slim_decode for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * slim_decode, but all scratch lives in one array of SLIM_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (each GPU the library runs on holds it until the process ends), and the call
 * itself makes no hipMalloc / hipFree or other allocating call (after slim_init on this device, or
 * its own first call, nothing but kernel launches and an event record / wait).
 *   - opts->workspace and opts->stage_ms must be null (SLIM_ERR_ARG otherwise).
 *   - Shapes whose scratch plan exceeds the array (slim_workspace_bytes(B, H, T, d, dtype) >
 *     slim_static_scratch_bytes()) are refused with SLIM_ERR_WORKSPACE before anything is launched.
 *   - Every call on a GPU shares that GPU's array: calls that overlap on one GPU (different streams
 *     or threads) race.  Nothing needs clearing between calls: the kernels zero their own counters
 *     and tell fresh exchange words from stale ones by per-launch tags. */
#define SLIM_STATIC_SCRATCH_BYTES (64u << 20)
size_t slim_static_scratch_bytes(void);
int slim_decode_static(const void* q, const void* Kcache, const void* W_KV, void* out,
                       int B, int H, int T, int d, const slim_opts* opts);

/* The same step the vanilla way (eq. 2 with a stored V-cache, Table 2 row "Vanilla"):
 * reads K and V, 2*T*d cache elements per sequence.  The same-GPU comparison kernel. */
int vanilla_kv_decode(const void* q, const void* Kcache, const void* Vcache, void* out,
                      int B, int H, int T, int d, const slim_opts* opts);

/* Non-square projections (e = H*d_k > d_model), option 2 of that section (Fig. 4): the
 * cache holds the layer input X; scores use (q_h W_K,h^T) X^T, the output (p_h X) W_V,h.
 *   q   : device fp32 [B][e]
 *   X   : device dtype [B][t_stride][d_model]
 *   W_K, W_V : device dtype [d_model][e] row-major (slim_pack_weights)
 *   out : device fp32 [B][e] */
int slim_decode_xcache(const void* q, const void* X, const void* W_K, const void* W_V,
                       void* out, int B, int H, int T, int d_model, int d_k,
                       const slim_opts* opts);

/* Measurement only: one plain streaming read of `bytes` bytes of device memory at `buf` (16-byte loads,
 * nothing else), asynchronous on `stream`.  Timed by the benchmark beside the decode step: the read
 * rate this GPU sustains in the same process is the practical ceiling of the K stream (eq. 7 option 2
 * reads the cache once; Table 2 counts those reads). */
int slim_read_probe(const void* buf, size_t bytes, void* stream);

/* ---- the steps either side of the decode step ------------------------------------------- */

/* One generated token per sequence through the whole attention block (Fig. 1; the projection
 * column of Table 2), slim: q = x W_Q and k = x W_K (eq. 3, 4 for one row), k stored as row
 * seq_lens[b]-1 of the K-cache (the generate-phase description under Fig. 2), slim_decode over
 * all seq_lens[b] rows, then the concatenated heads through W_O (eq. 1).  No W_V, no V-cache.
 *   x      : device fp32 [B][d]            input rows of the new tokens
 *   W_Q, W_K, W_KV, W_O : device dtype [d][d] row-major (slim_pack_weights)
 *   Kcache : device dtype [B][t_stride][d], rows [0, seq_lens[b]-1) valid on entry; row
 *            seq_lens[b]-1 is WRITTEN (rounded to dtype) and then read with the others
 *   y      : device fp32 [B][d], written
 *   T and opts->seq_lens count the rows AFTER the append (1 <= seq_lens[b] <= T <= t_stride).
 * With opts->rope_table the new token sits at position seq_lens[b]-1: q is rotated there, the
 * key is stored raw and rotated for the scores as in slim_decode.
 * Scratch: slim_workspace_bytes_block(), else library-owned.  opts->stage_ms, when set, receives
 * three figures: projections + append, decode step, output projection. */
size_t slim_workspace_bytes_block(int B, int H, int T, int d, int dtype);
int slim_attention_block(const void* x, const void* W_Q, const void* W_K, const void* W_KV,
                         const void* W_O, void* Kcache, void* y, int B, int H, int T, int d,
                         const slim_opts* opts);

/* The same block the vanilla way (Table 2 row "Vanilla"): also v = x W_V (eq. 5), k and v stored
 * in both caches (with opts->rope_table the stored key is the rotated one), vanilla_kv_decode,
 * W_O.  The same-GPU comparison for the block. */
int vanilla_attention_block(const void* x, const void* W_Q, const void* W_K, const void* W_V,
                            const void* W_O, void* Kcache, void* Vcache, void* y, int B, int H,
                            int T, int d, const slim_opts* opts);

#ifdef __cplusplus
}
#endif
#endif /* SLIM_ATTENTION_H */
