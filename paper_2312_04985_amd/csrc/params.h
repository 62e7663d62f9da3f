// Kernel argument blocks and launcher prototypes (internal to libsparq).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sparq {

constexpr int kDecodeThreads = 512;     // threads per workgroup of the fused decode kernel
constexpr int kRadixBins = 2048;        // 11-bit digits: passes of 11, 11 and 10 bits
constexpr int kWorkspaceHeader = 256;   // bytes; word 0 is the error word
constexpr int kControlBytes = 65536;    // control block at the start of the workspace, zeroed by sparq_workspace_init
constexpr int kMaxSplit = 16;           // most workgroups one (sequence, head) is split over
constexpr int kSplitMaxUnits = 128;     // the digit-bucket plan (few units, long caches) serves at most this many (sequence, head) units
constexpr int kProbeBlocks = 256 * 8;   // workgroups (of 256 threads) of the bandwidth probes

struct DecodeArgs {
  void* K; void* Kt; void* V;                  // written only by the fused-append variant
  const float* v_mean; const int32_t* seq_lens;
  const void* q; const int32_t* k_per_seq;
  const void* k_new; const void* v_new;          // non-null: fused append (one-launch decode step)
  float* v_mean_next; int32_t* seq_lens_next;
  void* out; float* alpha_out; int32_t* idx_out; int32_t* chan_out; int32_t* err;
  int32_t B, H, H_kv, S_max, d_h, r, k, idx_stride;   // S_max: the bound on the lengths that LDS and workspace are sized for
  int32_t S_stride;   // positions per head in K and V and per channel row in Kt (the buffers' own S_max, >= S_max)
  uint32_t flags;
  int32_t local_window;
  unsigned long long* clocks = nullptr;   // [workgroups][kStageStamps] time stamps; set only by a SPARQ_STAGE_CLOCKS build
};

// Time stamps per workgroup of the one-workgroup-per-head kernel in a SPARQ_STAGE_CLOCKS build (10 ns ticks of the
// constant 100 MHz counter): start, channels selected, own part of Step 1 done, all keys in LDS, threshold
// found, list compacted, own rows attended, all partials in LDS, end.
constexpr int kStageStamps = 9;

struct AppendArgs {
  void* K; void* Kt; void* V; float* v_mean; int32_t* seq_lens;
  float* v_mean_out; int32_t* seq_lens_out;   // where the new means / lengths go (== v_mean / seq_lens: in place)
  const void* k_new; const void* v_new; const int32_t* n_new_per_seq; int32_t* err;
  int32_t B, H_kv, S_max, d_h, n_new;   // S_max: no length may pass it
  int32_t S_stride;   // positions per head in K and V and per channel row in Kt
  int32_t tiled;   // the tiled single-copy key layout: K holds tiles of 8 positions, Kt the rows of the newest < 8
};

struct DenseArgs {
  const void* K; const void* V; const int32_t* seq_lens; const void* q; void* out;
  float* partials;   // [B*H, n_split, d_h + 2]
  int32_t* err;
  int32_t B, H, H_kv, S_max, d_h, n_split, rows_per_split;
  int32_t S_stride;   // positions per head in K and V
};

// two-level plan: spans of span_len positions (a multiple of 64, at most kLongSpan), at most kMaxSpans per sequence
constexpr int kLongSpan = 8192;
constexpr int kMaxSpans = 64;

struct LongArgs {
  DecodeArgs d;
  int32_t n_span;          // workgroups per (sequence, head) in the scoring launch
  int32_t span_len;        // positions per span
  int32_t cand_cap;        // candidates one span may hand on = min(k, span_len)
  int32_t n_split;         // workgroups per (sequence, head) in the gather launch
  float* tmax_ws;          // [B * H][n_span] largest logit numerator of each span
  float* zsum_ws;          // [B * H][n_span] sum over the span of exp((d - span max) / tau)
  int32_t* cnt_ws;         // [B * H][n_span] candidates of each span
  float* tau_ws;           // [B * H]
  float* alpha_ws;         // [B * H]
  uint32_t* cand_key_ws;   // [B * H][n_span][cand_cap] keys of the candidates, position-ascending
  int32_t* cand_pos_ws;    // [B * H][n_span][cand_cap] their positions
  int32_t* list_ws;        // [B * H][S_max] selected positions, ascending
  float* part_ws;          // [B * H][n_split][d_h + 2] attention partials
};

// grouped-query rule over several workgroups per (sequence, KV head)
struct GsArgs {
  DecodeArgs d;
  int32_t n1, span1;       // logit spans per KV unit and their length (positions)
  int32_t n2, span2;       // selection spans per KV unit and their length
  int32_t cand_cap;        // candidates one selection span may hand on = min(k, span2)
  int32_t n_split;         // gather workgroups per KV unit
  int32_t list_stride;     // entries of one KV unit's position list
  float* z_ws;             // [B * H][S_max] logit numerators
  float* stat_ws;          // [B * H_kv][n1][G][2] span maximum and sum-exp per head
  float* esc_ws;           // [B * H] log2(e) / tau
  float* alpha_ws;         // [B * H]
  int32_t* cnt_ws;         // [B * H_kv][n2]
  uint32_t* cand_key_ws;   // [B * H_kv][n2][cand_cap]
  int32_t* cand_pos_ws;    // [B * H_kv][n2][cand_cap]
  int32_t* list_ws;        // [B * H_kv][list_stride] selected positions, ascending
  float* part_ws;          // [B * H][n_split][d_h + 2] attention partials
};

// the gather and merge launches shared by the multi-launch plans
struct SplitArgs {
  DecodeArgs d;
  int32_t n_split;       // gather workgroups per (sequence, head)
  float* alpha_ws;       // [B * H]
  int32_t* list_ws;      // [B * H][S_max] selected positions, ascending
  float* part_ws;        // [B * H][n_split][d_h + 2] attention partials
};

// digit-bucket plan (few units, long caches): spans of span_len positions, n_span of them per unit
struct BucketArgs {
  DecodeArgs d;
  int32_t n_span, span_len;
  int32_t cand_cap;        // candidates (keys sharing the threshold digit) that bk_select_gather ranks out of LDS
  float* tmax_ws;          // [B * H][n_span] largest logit numerator of each span
  float* zsum_ws;          // [B * H][n_span] sum over the span of exp((d - span max) / tau)
  float* anum_ws;          // [B * H][n_span] the span's share of alpha's numerator (relative to the sequence maximum)
  float* tau_ws;           // [B * H]
  float* zden_ws;          // [B * H] softmax denominator of the approximate scores
  uint16_t* coarse_ws;     // [B * H][n_span][64] A[32 l]
  uint16_t* fine_ws;       // [B * H][n_span][2080] A[d] = keys of the span with first digit >= d
  uint32_t* skey_ws;       // [B * H][n_span][span_len] the span's keys sorted by first digit, descending
  uint32_t* spos_ws;       // [B * H][n_span][span_len] their positions
  float* part_ws;          // [B * H][n_span][d_h + 2] attention partials of the spans
  // the grouped-query rule on this plan (group > 0): one selection per KV head from the group score; the tables
  // and sorted arrays are indexed by KV unit, the logits and per-head statistics come from gs_logits
  int32_t group = 0;       // query heads per KV head, 0 = every head selects for itself
  int32_t n1 = 0;          // logit spans per KV unit of gs_logits
  const float* z_ws = nullptr;      // [B * H][S_max] logit numerators
  const float* stat_ws = nullptr;   // [B * H_kv][n1][group][2] span maximum and sum-exp per head
  const float* esc_ws = nullptr;    // [B * H] log2(e) / tau
};

// LDS bytes the fused decode kernel needs for a cache of S_max rows and head dimension d_h
size_t decode_lds_bytes(int S_max, int d_h);
size_t decode_shared_lds_bytes(int S_max, int d_h, int g);   // 0: no grouped-query kernel for this shape

hipError_t launch_decode(const DecodeArgs& a, int dtype, hipStream_t s);
size_t decode_single_k_lds_bytes(int S_max, int d_h);
hipError_t launch_decode_single_k(const DecodeArgs& a, int dtype, hipStream_t s);
size_t long_scores_lds_bytes(int span_len, int d_h);
size_t long_merge_lds_bytes(int n_span, int cand_cap);
hipError_t launch_decode_long(const LongArgs& a, int dtype, hipStream_t s);
size_t bk_scores_lds_bytes(int span_len, int d_h);
size_t bk_select_lds_bytes(int span_len, int d_h, int n_span, int cand_cap);
int bk_fine_len();
hipError_t launch_decode_bucket(const BucketArgs& a, int dtype, hipStream_t s);
size_t bk_group_scores_lds_bytes(int span_len);
// the grouped-query rule on the digit-bucket plan: after gs_logits (launch_group_logits), uses a.group, n1, z_ws, stat_ws, esc_ws
hipError_t launch_decode_bucket_group(const BucketArgs& a, int dtype, hipStream_t s);
// the first launch of the grouped-query plans alone: logit numerators and per-head span statistics (uses d, n1, span1,
// z_ws, stat_ws, esc_ws of `a`)
hipError_t launch_group_logits(const GsArgs& a, int dtype, hipStream_t s);
// the gather launch and the merge (gather over slices of list_ws, merge): uses d, n_split,
// alpha_ws, list_ws, part_ws of `a`
hipError_t launch_split_gather(const SplitArgs& a, int dtype, hipStream_t s);
// the last launch alone: uses d, n_split, alpha_ws, part_ws
hipError_t launch_split_combine(const SplitArgs& a, int dtype, hipStream_t s);
size_t gs_select_lds_bytes(int span2);
size_t gs_merge_lds_bytes(int n2, int cand_cap);
hipError_t launch_decode_shared_split(const GsArgs& a, int dtype, hipStream_t s);
// z_ws: [B * H][S_max] fp32 scratch for the logit numerators
hipError_t launch_decode_shared(const DecodeArgs& a, float* z_ws, int dtype, hipStream_t s);
hipError_t launch_append(const AppendArgs& a, int dtype, hipStream_t s);
hipError_t launch_dense(const DenseArgs& a, int dtype, hipStream_t s);
hipError_t launch_copy_probe(void* dst, const void* src, size_t n_bytes, hipStream_t s);
hipError_t launch_read_probe(const void* src, size_t n_bytes, void* sink, hipStream_t s);
hipError_t launch_clear(void* workspace, int n_bytes, hipStream_t s);

// A kernel that takes more than 64 KiB of dynamic LDS has to be allowed to, once per kernel and device
// (not per launch: the call costs host time).  `lds` = the bytes the coming launch asks for; `limit` = what the
// kernel is allowed from then on (a kernel with static LDS arrays as well must stay below 160 KiB minus those).
template <auto Kern>
hipError_t allow_lds(size_t lds, int limit = 160 * 1024) {
  if (lds <= 64 * 1024) return hipSuccess;
  static unsigned long long allowed = 0;   // bit d: done on device d (benign race: the call is idempotent)
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64 || !((allowed >> dev) & 1ull)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize, limit);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) allowed |= 1ull << dev;
  }
  return hipSuccess;
}

}  // namespace sparq
