/*
 * libsparq: SparQ Attention single-token decode step for one MI355X (gfx950).
 *
 * C ABI.  Every buffer named "device" is caller-owned device memory; the library
 * never allocates, frees or synchronises (the one exception, sparq_async_error, says
 * so).  All work is enqueued on the caller's HIP stream (`hip_stream` is a
 * hipStream_t passed as void*; NULL is the default stream) and is complete when the
 * stream reaches that point.  Functions return a sparq_status; nothing throws.
 *
 * Notation follows the paper: B sequences, H query heads, H_kv key/value heads
 * (g = H / H_kv query heads share a KV head), head dimension d_h, S_b cached rows in
 * sequence b, r query components kept in Step 1, k positions kept in Step 2.
 * Equation numbers are the paper's own, counting every displayed equation from its start:
 * (1) attention's share of the data transfers (Section 2); in Section 3 (2) dense attention,
 * (3) M_dense, (4) the exact scores s, (5) top-k sparse values, (6) mean value reallocation,
 * (7) the approximate scores s-hat, (8) attention over the selected positions, (9) the
 * temperature tau, (10) the blend with the mean value vector; (11) M_SparQ (Section 4).
 *
 * Cache layout (Section 6 and Appendix F, "Storing K twice": the key cache is kept in
 * both a d_h-contiguous and an S-contiguous layout so that either axis can be
 * gathered with contiguous reads):
 *   K      [B, H_kv, S_max, d_h]   16-bit, d_h-contiguous   (Step 2 gathers rows)
 *   Kt     [B, H_kv, d_h, S_max]   16-bit, S-contiguous copy of K (Step 1 reads r rows)
 *   V      [B, H_kv, S_max, d_h]   16-bit
 *   v_mean [B, H_kv, d_h]          fp32 running mean of V[b, h, 0:S_b, :]
 *                                  (Section 3, "Mean value reallocation")
 *   seq_lens [B]                   int32, S_b
 * S_max must be a multiple of 64 and every pointer 16-byte aligned.  d_h is 64, 128 or
 * 256.  Rows at positions >= S_b are never read.
 * Kt is maintained by this library only, and 8 positions at a time: its columns below
 * 8 * floor(S_b / 8) equal K transposed; the up to 7 newest keys reach it when the eighth
 * arrives (one aligned 16-byte store per channel row instead of eight scattered 2-byte
 * stores) and until then Step 1 takes them from the rows of K.  Columns from
 * 8 * floor(S_b / 8) on are unspecified.  A caller that fills or edits a cache by itself
 * (instead of through sparq_kv_append / sparq_decode_step) has to write both layouts for all
 * columns below 8 * floor(S_b / 8), K for all rows below S_b, and v_mean; a cache with
 * seq_lens[b] = 0 needs no initialisation of K, Kt, V or v_mean[b] (the first append ignores
 * whatever v_mean holds), only seq_lens must be set.
 */
#ifndef SPARQ_H
#define SPARQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPARQ_OK = 0,
  SPARQ_EINVAL = -1,       /* null / misaligned pointer, inconsistent shape */
  SPARQ_EUNSUPPORTED = -2, /* valid request this build has no kernel for */
  SPARQ_EWORKSPACE = -3,   /* workspace missing or smaller than sparq_workspace_bytes */
  SPARQ_ELAUNCH = -4,      /* the HIP runtime refused the launch */
  SPARQ_ETOOLARGE = -5     /* sparq_decode_noalloc: the shape needs more scratch than the built-in buffer */
} sparq_status;

typedef enum { SPARQ_F16 = 0, SPARQ_BF16 = 1 } sparq_dtype;

enum {
  /* y = y3: skip the blend of Step 3 (Section 4 omits it for grouped-query models) */
  SPARQ_FLAG_NO_REALLOC = 1u << 0,
  /* the paper's grouped-query rule (Section 4, "Grouped query attention"; Appendix B): one
   * channel set per KV head from the group sum of |q|, one position set per KV head from the
   * group sum of the approximate scores s-hat; tau, alpha and the exact attention stay per
   * query head; idx_out / chan_out repeat the shared sets for every head of the group.
   * Built for groups of 2 and 4 query heads (SPARQ_EUNSUPPORTED otherwise).  Without the flag
   * every query head selects independently over its shared KV head. */
  SPARQ_FLAG_GQA_SHARED = 1u << 1,
  /* scheduling hint, no effect on results: the sequence lengths of the batch differ widely;
   * sparq_decode / sparq_decode_step then start the longest sequences first.  Honoured by the
   * one-workgroup-per-head plan for 2 <= B <= 512 and H = H_kv; ignored otherwise */
  SPARQ_FLAG_RAGGED_BATCH = 1u << 2,
  /* the fixed temperatures of the paper's ablation (Section 5.3, "Approximate softmax
   * temperature") in place of Eq. (9): tau = sqrt(d_h), or tau = sqrt(r).  At most one of the two. */
  SPARQ_FLAG_TAU_SQRT_DH = 1u << 3,
  SPARQ_FLAG_TAU_SQRT_R = 1u << 4,
  /* the key cache is stored once, d_h-contiguous only (the "1 x K" variant of Section 6.1): cache.Kt
   * is ignored and may be null, sparq_kv_append writes no second copy, and Step 1 reads the rows of K
   * whole (S d_h elements instead of S r).  Not combined with SPARQ_FLAG_GQA_SHARED. */
  SPARQ_FLAG_SINGLE_K = 1u << 5,
  /* the key cache is stored once in a layout that serves both steps (Section 6.1 closes by asking for
   * alternatives to storing K twice): tiles of 8 positions, channel-major inside a tile.  cache.K is then
   * [B, H_kv, S_max / 8, d_h, 8] (element (position p, channel j) at ((p / 8) d_h + j) 8 + p % 8: the same
   * number of bytes as the row-major K) and cache.Kt is a small buffer [B, H_kv, 8, d_h] holding the rows of
   * the positions 8 floor(S_b / 8) .. S_b - 1, which move into their tile, as one contiguous block, when the
   * eighth arrives.  Step 1 reads 16 bytes per selected channel and group of 8 positions (2 d_h bytes apart),
   * Step 2 collects a key row's components from its tile.  Served by the one-workgroup-per-head kernel
   * (S_max up to about 35 000); dense_decode, SPARQ_FLAG_GQA_SHARED and SPARQ_FLAG_SINGLE_K are not combined
   * with it (SPARQ_EUNSUPPORTED / SPARQ_EINVAL). */
  SPARQ_FLAG_TILED_K = 1u << 6
};

/* bits of the device-side error word (sparq_async_error) */
enum {
  SPARQ_ERR_APPEND_FULL = 1,   /* an append would pass S_max: that sequence was skipped */
  SPARQ_ERR_EMPTY_SEQ = 2,     /* decode of a sequence with S_b = 0: zeros written */
  SPARQ_ERR_IDX_TRUNCATED = 4, /* min(k_b, S_b) exceeded idx_stride: idx_out truncated */
  SPARQ_ERR_BAD_SEQ_LEN = 8,   /* seq_lens[b] outside [0, S_max]: clamped */
  SPARQ_ERR_INTERNAL = 16      /* a consistency check inside a kernel failed (a defect of the library): results invalid */
};

typedef struct {
  int32_t B, H, H_kv, S_max, d_h;
  int32_t r;      /* 1 <= r <= d_h */
  int32_t k;      /* >= 1; clamped per sequence to S_b */
  int32_t dtype;  /* sparq_dtype of K, Kt, V, q and out */
  uint32_t flags;
  /* l >= 0 (the "local window" of the paper's experimental-setup table): the min(l, k_b, S_b) most
   * recent positions are selected unconditionally and the other k_b - l are the best-scoring of the
   * older positions; alpha sums s-hat over the whole set.  0 = the plain top-k rule. */
  int32_t local_window;
  /* 0, or the caller's bound on the lengths for this call: a multiple of 64, <= S_max, with seq_lens[b] <=
   * S_bound for every sequence (for sparq_decode_step: after its append).  K, Kt and V keep the strides of
   * S_max; the kernels, their LDS and the workspace are chosen for S_bound instead, which matters when the
   * buffers are allocated for a far longer context than the batch has reached (one workgroup per head holds a
   * 4-byte key per position up to the bound in LDS: buffers for 32 768 positions used at 8 192 decode 30 % slower
   * when sized by S_max).  The bound is treated exactly as S_max is treated without it: a longer sequence is
   * served over its first S_bound positions and reported (SPARQ_ERR_BAD_SEQ_LEN; its stored length is carried over
   * unchanged), a step whose append would pass the bound leaves that sequence as it is (SPARQ_ERR_APPEND_FULL).  sparq_kv_append ignores the bound.  sparq_workspace_bytes depends on it: size the
   * workspace for every bound that will be used (the calls check). */
  int32_t S_bound;
} sparq_shape;

typedef struct {
  void* K;           /* device */
  void* Kt;          /* device */
  void* V;           /* device */
  float* v_mean;     /* device */
  int32_t* seq_lens; /* device */
} sparq_cache;

/* Bytes of device workspace the calls below need for this shape (>= 64 KiB; depends on every field of
 * the shape, flags included).  The first 64 KiB are a control block (word 0 is the error word) that
 * sparq_workspace_init zeroes; the rest is scratch: the split-sequence partials of dense_decode, and for
 * sparq_decode the keys / candidates / position lists of the multi-launch plans (few heads with long
 * caches, S_max beyond one workgroup's LDS) or the logits of the grouped-query rule.  One workspace
 * serves one stream. */
int sparq_workspace_bytes(const sparq_shape* shape, size_t* out_bytes);

/* Enqueue a clear of the control block.  Call once after allocating the workspace. */
int sparq_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Append rows to the cache and keep Kt and v_mean in step (the "4 d_h" term of the SparQ
 * transfer equation in Section 4: write k and v, read and write the mean value vector;
 * the second, non-contiguous key write is the one Appendix F describes).
 *   k_new, v_new   device [B, H_kv, n_new, d_h], cache dtype
 *   n_new          rows per sequence in k_new / v_new (>= 1)
 *   n_new_per_seq  device [B] or NULL: sequence b appends only its first
 *                  n_new_per_seq[b] rows (0..n_new); NULL appends n_new everywhere
 * For sequence b with n rows: rows land at positions S_b..S_b+n-1 of K and V; Kt is brought up to date
 * to column 8 * floor((S_b+n) / 8) at least (NOT to S_b+n: Kt trails K by up to 7 columns, see the cache
 * layout above; the decode calls take those keys from K); v_mean becomes the mean of the S_b+n value
 * rows (for S_b = 0 the old content of v_mean is ignored); seq_lens[b] += n.  If S_b + n > S_max the sequence is left untouched and SPARQ_ERR_APPEND_FULL is
 * raised in the error word.  The only call that mutates the cache.
 */
int sparq_kv_append(const sparq_shape* shape, const sparq_cache* cache, const void* k_new,
                    const void* v_new, int32_t n_new, const int32_t* n_new_per_seq,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One SparQ decode step for all B x H heads (Section 4, Steps 1-3; Section 3 Eqs. 7-10).
 * Per query head, over the rows 0..S_b-1 of its KV head:
 *   Step 1  i1 = the r largest |q_j| (ties to the lower j);
 *           tau = sqrt(d_h * sum_{j in i1}|q_j| / sum_j |q_j|)  (sqrt(d_h) if q = 0);
 *           z_i = sum_{j in i1} q_j K[i,j] / tau,  s_hat = softmax(z)
 *   Step 2  i2 = the min(k_b, S_b) positions of largest z (ties to the lower i);
 *           y3 = softmax(q K[i2]^T / sqrt(d_h)) V[i2]
 *   Step 3  alpha = sum_{i in i2} s_hat_i;  y = alpha y3 + (1 - alpha) v_mean
 * Arithmetic is fp32 on the 16-bit inputs; `out` is rounded to nearest-even.
 * Sizes: every plan keeps 4 bytes per position (or per candidate) of its unit of work in LDS.  One
 * workgroup per head serves S_max up to about 35 000.  Few (sequence, head) units with long caches (at most 96
 * from S_max = 16 384, at most 64 from 12 288, at most 128 beyond what one workgroup holds) are spread over spans of
 * up to 8192 positions (at most 64 spans: S_max <= 524 288, any k).
 * Larger batches with longer caches are selected in two levels (spans of 8192 positions, at most 64 of
 * them, ceil(S_max / 8192) * min(k, 8192) candidates <= about 36 000: e.g. S_max = 524 288 at k = 512), also
 * under SPARQ_FLAG_GQA_SHARED.  SPARQ_FLAG_SINGLE_K and SPARQ_FLAG_TILED_K stop at about 35 000.
 * Anything else returns SPARQ_EUNSUPPORTED before a launch.  sparq_decode_plan names the kernels of a shape.
 *   q          device [B, H, d_h]
 *   k_per_seq  device [B] or NULL; k_per_seq[b] in 1..shape.k replaces shape.k for sequence b
 *              (shape.k is the maximum that buffers are sized for: values outside are clamped)
 *   out        device [B, H, d_h], cache dtype
 *   alpha_out  device [B, H] fp32 or NULL
 *   idx_out    device [B, H, idx_stride] int32 or NULL: i2 ascending, padded with -1
 *   chan_out   device [B, H, r] int32 or NULL: i1 ascending
 * Reads the cache, writes only the outputs and the error word.
 */
int sparq_decode(const sparq_shape* shape, const sparq_cache* cache, const void* q,
                 const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                 int32_t idx_stride, int32_t* chan_out, void* workspace,
                 size_t workspace_bytes, void* hip_stream);

/*
 * sparq_decode for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels and same results
 * as sparq_decode; the scratch that call takes from `workspace` (partials, keys, candidates and position
 * lists of the multi-launch plans, the logits of the grouped-query rule) comes from a buffer built into the
 * library instead: 32 MiB of device memory per GPU, held from the first call on that GPU until the process
 * ends.  The call allocates nothing and frees nothing (its first call on a device looks up the buffer's
 * address and enqueues one small fill kernel on `hip_stream`).
 *   error_word  device int32 or NULL: the SPARQ_ERR_* bits of this call are OR-ed into it (the caller
 *               clears and reads it); with NULL they are dropped
 * Shapes for which sparq_workspace_bytes exceeds 32 MiB return SPARQ_ETOOLARGE before any launch.
 * All calls on one GPU share the one buffer: two calls that may run at the same time on one GPU (different
 * streams, or graphs replayed concurrently) race on it and must be ordered by the caller.  Nothing in the
 * buffer has to survive between calls.  Other arguments as for sparq_decode.
 */
int sparq_decode_noalloc(const sparq_shape* shape, const sparq_cache* cache, const void* q,
                         const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                         int32_t idx_stride, int32_t* chan_out, int32_t* error_word, void* hip_stream);

/*
 * The whole decode step in one call: exactly sparq_kv_append with n_new = 1 followed by
 * sparq_decode (Section 4: the step writes k and v, updates the mean value vector and attends
 * over the cache including the new token).  One launch where one workgroup serves a head; the
 * three launches of the few-heads-long-cache plan with the append in the last one; for the other
 * plans the append kernel followed by the decode launches.  The small state is not updated in place:
 * the new lengths and means are written to seq_lens_next [B] and v_mean_next [B, H_kv, d_h]
 * (device, must not alias cache->seq_lens / cache->v_mean, which are only read) and the caller
 * swaps the two pairs of buffers between steps.  K and V receive row S_b in place, Kt as in
 * sparq_kv_append.  The new
 * row is taken from k_new / v_new [B, H_kv, d_h] by every head, so no head depends on another
 * one's write.  A sequence with S_b = S_max is decoded without the new row, keeps its length
 * and mean, and raises SPARQ_ERR_APPEND_FULL.  Other arguments as for sparq_decode.
 */
int sparq_decode_step(const sparq_shape* shape, const sparq_cache* cache, const void* k_new,
                      const void* v_new, float* v_mean_next, int32_t* seq_lens_next, const void* q,
                      const int32_t* k_per_seq, void* out, float* alpha_out, int32_t* idx_out,
                      int32_t idx_stride, int32_t* chan_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * Dense single-query attention y = softmax(q K^T / sqrt(d_h)) V over rows 0..S_b-1
 * (Section 3, Eq. 2): the in-library comparison.  Reads K and V once per KV head for
 * all g query heads of the group.  Uses the workspace for split-sequence partials.
 *   q, out  device [B, H, d_h], cache dtype
 */
int dense_decode(const sparq_shape* shape, const sparq_cache* cache, const void* q, void* out,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Copy the device error word to *host_flag, clear it on the device, and WAIT for the
 * stream (this call synchronises). */
int sparq_async_error(void* workspace, int32_t* host_flag, void* hip_stream);

/* Plain device-to-device copy of n_bytes (multiple of 16) by a grid-stride kernel: the
 * known-size copy used to calibrate HBM counters and to measure the attainable rate. */
int sparq_copy_probe(void* dst, const void* src, size_t n_bytes, void* hip_stream);

/* Plain streaming read of n_bytes (multiple of 16) by the same grid; each thread stores one
 * folded word to `sink` (device, at least 2 MiB = 2048 workgroups x 256 threads x 4 bytes). */
int sparq_read_probe(const void* src, size_t n_bytes, void* sink, size_t sink_bytes, void* hip_stream);

/* Which kernels sparq_decode / sparq_decode_step launch for this shape (a static string naming the plan
 * and its launches; "unsupported" where sparq_decode would return SPARQ_EUNSUPPORTED).  Host only. */
const char* sparq_decode_plan(const sparq_shape* shape);

/* Profiling builds only (the library compiled with -DSPARQ_STAGE_CLOCKS; the default build returns
 * SPARQ_EUNSUPPORTED): for shapes served by one workgroup per head, every sparq_decode / sparq_decode_step
 * launch also leaves *stamps_per_workgroup 64-bit time stamps per workgroup (10 ns ticks of the device's
 * constant 100 MHz counter; workgroups in launch order) at workspace + *offset_bytes: start, Step 1 channels
 * selected, the first wave's share of the Step 1 stream done, all approximate scores in LDS, Step 2 threshold
 * found, position list compacted, the first wave's rows attended, all partial results in LDS, end.
 * sparq_workspace_bytes of such a build includes the room.  Host only. */
int sparq_stage_clocks(const sparq_shape* shape, size_t* offset_bytes, int32_t* n_workgroups,
                       int32_t* stamps_per_workgroup);

const char* sparq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPARQ_H */
