// SparQ decode for few (sequence, head) units with long caches: every launch of the plan runs on
// units x n_span workgroups, so that 32 heads fill 256 compute units, and no workgroup ever selects over
// more than one span's keys.  Step 2's top-k is found exactly without any workgroup seeing the whole
// sequence:
//   bk_scores   (units x n_span) Step 1 on a span of span_len positions: approximate logits as integer
//               keys in LDS, counted by an 11-bit bucket that is monotone in the key; the span's keys go to
//               the workspace sorted by bucket (descending, as (key, position) pairs), together with the table
//               A[d] = number of the span's keys whose bucket is >= d, the span's largest logit and
//               its softmax denominator
//   bk_select_gather  (units x n_span) every workgroup sums the tables of its unit's spans and finds the
//               bucket d0 in which the k-th largest key of the whole sequence lies: all keys of a higher bucket
//               are selected, and of the few keys of bucket d0 (contiguous in every span's sorted array)
//               the best are: they are read by every workgroup of the unit and ranked exactly by
//               (key descending, position ascending) with radix passes over the key bits and,
//               only among identical keys, over the position.  Each workgroup then writes its own span's
//               selected positions, ascending (into idx_out at its place in the unit's list), its share of
//               alpha's numerator, gathers its own span's selected rows of K and V (Step 2b) and leaves one
//               attention partial per span
//   bk_combine  (one workgroup per unit) merges the spans' partials, alpha, blend, store
// Every workgroup attends over the selected rows of its own span: the gather is balanced when the selected
// positions are spread over the sequence, and takes as long as the busiest span when they are not.
// The local window is part of it: its positions count as bucket 2047, above every key's.
// The grouped-query rule runs on the same plan: gs_logits leaves every head's logit numerators and statistics in
// the workspace, bk_group_scores turns the group score into keys and publishes the spans per KV unit, and
// bk_select_gather<GROUP> / bk_combine run per query head on the KV unit's tables (alpha from the head's own logits).
// Inside sparq_decode_step the three launches count the row being appended as position S_b (taken from the
// inputs wherever it is needed) and bk_combine writes it to the cache, after every read of the earlier launches.
#include "group_stages.h"

namespace sparq {

namespace {

constexpr int kFineLen = kRadixBins + 32;   // entries of a span's table A: A[2048..2079] = 0
constexpr int kTopDigit = kRadixBins - 1;   // no finite key has it: float_to_key of the largest float has digit 2043
constexpr uint32_t kPosMask = 0xfffffu;     // positions < 2^20 (S_max <= 64 spans of 8192)

__device__ __forceinline__ void map_span(int U, int n_span, int& u, int& s) {
  const int bid = blockIdx.x;
  if ((U & 7) == 0) {          // the spans of a unit, and the heads of a KV group, share an XCD
    const int x = bid & 7, slot = bid >> 3;
    u = x * (U >> 3) + slot / n_span;
    s = slot % n_span;
  } else {
    u = bid / n_span;
    s = bid % n_span;
  }
}

// The bucket of a key: 11 bits that are monotone in the key (which is all the selection needs of a bucket: ranking
// inside the threshold bucket uses the whole key) and tell the keys around the threshold apart as finely as
// possible; 2047 stays free for the local window.  A key's own first 11 bits (sign, exponent, two mantissa bits)
// leave a few percent of a sequence in one bucket.
//  - Ordinary keys (approximate logit numerators): sign, 5 exponent bits (magnitudes 2^-8 .. 2^23; smaller ones share
//    the bucket next to zero, larger ones the outermost) and 5 mantissa bits: 32 buckets per octave.
//  - Group-score keys are log2 of a sum of probabilities, x <= 2, often down to -1000: the bucket comes from
//    u = 4 - x >= 2: 4 exponent bits and 7 mantissa bits of u (128 buckets per octave of u), counted down so that
//    a larger score has a larger digit.
template <bool GROUP>
__device__ __forceinline__ uint32_t bucket_digit(uint32_t key) {
  if (!GROUP) {
    const bool pos = (key & 0x80000000u) != 0;
    const uint32_t bits = pos ? key & 0x7fffffffu : ~key & 0x7fffffffu;      // magnitude bits of the float
    const int e = (int)(bits >> 23) - 119;
    uint32_t low = e < 0 ? 0u : (e > 31 ? 1023u : ((uint32_t)e << 5) | ((bits >> 18) & 31u));
    low = low > 1022u ? 1022u : low;
    return pos ? 1024u + low : 1023u - low;
  }
  const uint32_t bits = __float_as_uint(4.0f - key_to_float(key));   // u > 0 (or +inf): the bits order like u
  const int e = (int)(bits >> 23) - 128;
  uint32_t low = e < 0 ? 0u : (e > 15 ? 2046u : ((uint32_t)e << 7) | ((bits >> 16) & 127u));
  low = low > 2046u ? 2046u : low;
  return 2046u - low;
}

// The table A[d] = number of the span's keys whose first digit is >= d, from the first-digit counts in `hist`
// (swizzled slots): A as u16 to fine[0..2047] (and 32 zeros behind), A[32 l] to coarse[l], and the write cursors
// of the digit buckets (keys with a larger digit come first) to cur.  One wave: lane l owns digits 32 l .. 32 l + 31.
__device__ __forceinline__ void build_span_table(const uint32_t* hist, uint32_t* cur, uint16_t* fine, uint16_t* coarse, int lane) {
  uint32_t cnt[32], mine = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) { cnt[i] = hist[(i << 6) | lane]; mine += cnt[i]; }
  const uint32_t incl = wave_scan_incl(mine);
  const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
  uint32_t run = total - incl;              // keys with digits owned by higher lanes
  uint32_t packed[16];
#pragma unroll
  for (int i = 31; i >= 0; --i) {
    cur[(i << 6) | lane] = run;             // keys with a digit above 32 l + i
    run += cnt[i];                          // A[32 l + i]
    if (i & 1) packed[i >> 1] = run << 16; else packed[i >> 1] |= run;
  }
  uint4* dst = reinterpret_cast<uint4*>(fine + lane * 32);
#pragma unroll
  for (int i = 0; i < 4; ++i) dst[i] = make_uint4(packed[4 * i], packed[4 * i + 1], packed[4 * i + 2], packed[4 * i + 3]);
  coarse[lane] = (uint16_t)run;             // A[32 l]
  if (lane < 32) fine[kRadixBins + lane] = 0;
}

// Counting sort of a span's keys by first digit into LDS (window positions, relative index >= w0, as the top
// digit; the order inside a bucket is whatever the atomics give: the select only ever uses buckets as sets),
// then one contiguous copy to the workspace.  Called by the whole workgroup after a barrier behind
// build_span_table; contains one barrier.
template <bool GROUP>
__device__ __forceinline__ void sort_span_by_digit(const uint32_t* keys, int len, int w0, int p0, uint32_t* cur, uint32_t* skey,
                                                   uint32_t* spos, uint32_t* gkey, uint32_t* gpos, int tid) {
  for (int i = tid; i < len; i += NT) {
    const uint32_t key = keys[i];
    const uint32_t digit = i >= w0 ? (uint32_t)kTopDigit : bucket_digit<GROUP>(key);
    const uint32_t e = atomicAdd(&cur[hist_slot(digit)], 1u);
    skey[e] = key;
    spos[e] = (uint32_t)(p0 + i);
  }
  __syncthreads();
  // (non-temporal stores: the next launch reads only the head of each array; config 3's step 37.3 -> 36.7 us)
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  for (int i = tid * 4; i < len; i += NT * 4) {     // span_len is a multiple of 64: whole 16-byte pieces
    __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(skey + i), reinterpret_cast<u32x4*>(gkey + i));
    __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(spos + i), reinterpret_cast<u32x4*>(gpos + i));
  }
}

// LDS words of bk_scores besides the three span-sized arrays
template <int DH>
__host__ __device__ constexpr size_t bk_scores_fixed_words() {
  return 2 * (size_t)kRadixBins + NT + 4 * (size_t)DH + 32 + 8;
}

template <class T, int DH>
__global__ __launch_bounds__(NT, 4) void bk_scores(const BucketArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const int P = a.span_len;
  uint32_t* keys = smem;                                        // [P] keys by position
  uint32_t* skey = keys + P;                                    // [P] keys sorted by first digit, descending
  uint32_t* spos = skey + P;                                    // [P] their positions
  uint32_t* hist = spos + P;                                    // [kRadixBins] first-digit counts (swizzled slots)
  uint32_t* cur = hist + kRadixBins;                            // [kRadixBins] write cursors of the digit buckets
  int* rankp = reinterpret_cast<int*>(cur + kRadixBins);        // [NT]
  float* qf = reinterpret_cast<float*>(rankp + NT);             // [DH]
  float* qs = qf + DH;
  int* chan = reinterpret_cast<int*>(qs + DH);
  uint32_t* mag = reinterpret_cast<uint32_t*>(chan + DH);
  float* red = reinterpret_cast<float*>(mag + DH);              // [32]
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int U = d.B * d.H;
  int u, s;
  map_span(U, a.n_span, u, s);
  const int b = u / d.H, h = u - b * d.H;
  const size_t kv_head = (size_t)b * d.H_kv + h / (d.H / d.H_kv);
  const size_t slot = (size_t)u * a.n_span + s;
  uint16_t* fine = a.fine_ws + slot * kFineLen;
  uint16_t* coarse = a.coarse_ws + slot * 64;

  uint16_t qcode = 0;
  if (tid < DH) qcode = reinterpret_cast<const uint16_t*>(d.q)[(size_t)u * DH + tid];
  bool appended, bad, full;
  const int S = visible_length(d, b, appended, bad, full);
  if (tid == 0 && s == 0 && (bad || full)) atomicOr(d.err, (bad ? 8 : 0) | (full ? 1 : 0));
  int32_t* idx_out = d.idx_out ? d.idx_out + (size_t)u * d.idx_stride : nullptr;
  if (S == 0) {   // nothing cached: span 0 writes the defined outputs, the later launches skip the unit
    if (s == 0) {
      if (tid < DH) reinterpret_cast<uint16_t*>(d.out)[(size_t)u * DH + tid] = 0;
      if (tid == 0) { atomicOr(d.err, 2); if (d.alpha_out) d.alpha_out[u] = 0.0f; }
      if (d.chan_out && tid < d.r) d.chan_out[(size_t)u * d.r + tid] = -1;
      if (idx_out) for (int n = tid; n < d.idx_stride; n += NT) idx_out[n] = -1;
    }
    return;
  }
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  const Window win = make_window(d.local_window, S, kq);
  const int p0 = s * P;
  if (p0 >= S) {   // a span beyond the end of this sequence: an empty table
    for (int i = tid; i < kFineLen; i += NT) fine[i] = 0;
    if (tid < 64) coarse[tid] = 0;
    if (tid == 0) { a.tmax_ws[slot] = -INFINITY; a.zsum_ws[slot] = 0.0f; }
    return;
  }
  const int len = S - p0 < P ? S - p0 : P;

  for (int i = tid; i < kRadixBins; i += NT) hist[i] = 0u;
  const QueryLds Q{mag, rankp, qf, qs, chan};
  const float tau = apply_tau_mode(select_channels<T, DH>(Q, qcode, d.r, tid, lane, wave), d.flags, DH, d.r);
  if (s == 0) {
    if (d.chan_out && tid < d.r) d.chan_out[(size_t)u * d.r + tid] = chan[tid];
    if (tid == 0) a.tau_ws[u] = tau;
  }

  // the newest S mod 8 positions are not in Kt (inside a step: up to 8, Kt being up to date for the length before
  // the call): the span that holds them takes them from the rows of K, the row being appended from the inputs
  const int S_fl = (appended ? S - 1 : S) & ~7, r8 = (d.r + 7) & ~7;
  const int n_tail = (S_fl >= p0 && S_fl < p0 + len) ? S - S_fl : 0;
  TailRow tail;
  if (wave < n_tail) {
    const uint16_t* krow = appended && wave == n_tail - 1
                               ? reinterpret_cast<const uint16_t*>(d.k_new) + kv_head * DH
                               : reinterpret_cast<const uint16_t*>(d.K) + (kv_head * d.S_stride + S_fl + wave) * (size_t)DH;
    tail = tail_row_issue(krow, chan, r8, lane);
  }

  const int end = p0 + len < S_fl ? p0 + len : S_fl;     // whole chunks of this span that are in Kt
  const size_t row_bytes = (size_t)d.S_stride * 2;
  const char* Kt_head = reinterpret_cast<const char*>(d.Kt) + kv_head * DH * row_bytes;
  float tmax = -INFINITY;
  const int c_begin = p0 >> 3, c_end = end > p0 ? end >> 3 : p0 >> 3;
  auto finish = [&](int c, const float (&acc)[8]) {
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      tmax = fmaxf(tmax, acc[e]);
      kx[e] = float_to_key(acc[e]);
    }
    uint32_t dg[8];                                        // hist_add_chunk counts by the first 11 bits of what it is given
#pragma unroll
    for (int e = 0; e < 8; ++e) dg[e] = bucket_digit<false>(kx[e]) << 21;
    hist_add_chunk(hist, dg, win.S_old - c * 8);          // the window's positions are counted below
    uint4* dst = reinterpret_cast<uint4*>(keys + (c * 8 - p0));
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  };
  const int nb = r8 >> 3;                                 // batches of 8 channel rows
  if (c_end - c_begin <= NT / 2 && nb >= 2) {
    // At most half as many chunks as threads: the two halves of the workgroup share every chunk, each taking
    // half of the channel rows, so that a thread's loads are all in flight at once (r <= 32) instead of going
    // through the pipeline in two dependent rounds.  The halves' partial sums meet in LDS (the arrays of the
    // sort, which are idle until then), and the first half of the threads finishes the chunks.
    const int half = tid >> 8, t = tid & (NT / 2 - 1);
    const int b0 = half ? (nb + 1) >> 1 : 0, b1 = half ? nb : (nb + 1) >> 1;
    float* pacc = reinterpret_cast<float*>(half ? spos : skey);
    stream_channel_rows<T, NT / 2>(Kt_head, row_bytes, chan + 8 * b0, qs + 8 * b0, 8 * (b1 - b0), c_begin, c_end, t,
                                   [&](int c, const float (&acc)[8]) {
      float4* dst = reinterpret_cast<float4*>(pacc + (c * 8 - p0));
      dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
      dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    });
    __syncthreads();
    if (half == 0 && c_begin + t < c_end) {
      const int c = c_begin + t;
      const float4* x = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(skey) + (c * 8 - p0));
      const float4* y = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(spos) + (c * 8 - p0));
      const float4 x0 = x[0], x1 = x[1], y0 = y[0], y1 = y[1];
      const float acc[8] = {x0.x + y0.x, x0.y + y0.y, x0.z + y0.z, x0.w + y0.w, x1.x + y1.x, x1.y + y1.y, x1.z + y1.z, x1.w + y1.w};
      finish(c, acc);
    }
  } else {
    stream_channel_rows<T>(Kt_head, row_bytes, chan, qs, d.r, c_begin, c_end, tid, finish);
  }
  if (wave < n_tail) {
    const float dot = tail_row_dot<T>(tail, qs, r8, lane);
    tmax = fmaxf(tmax, dot);
    if (lane == 0) {
      const uint32_t key = float_to_key(dot);
      keys[S_fl + wave - p0] = key;
      if (S_fl + wave < win.S_old) atomicAdd(&hist[hist_slot(bucket_digit<false>(key))], 1u);
    }
  }
  // the part of the local window that lies in this span counts as the top digit
  const int w0 = win.S_old > p0 ? win.S_old - p0 : 0;      // first window position, relative to the span
  if (tid == 0 && w0 < len) atomicAdd(&hist[hist_slot(kTopDigit)], (uint32_t)(len - w0));
  tmax = wave_max(tmax);
  if (lane == 0) red[wave] = tmax;
  __syncthreads();
  float dmax = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, red[w]);
  __syncthreads();     // red is reused below

  // the table and the bucket cursors (one wave), and the softmax denominator relative to the span's maximum
  if (wave == 0) {
    build_span_table(hist, cur, fine, coarse, lane);
  } else {
    const float esc = kLog2e / tau;
    float z = 0.0f;
    for (int i = tid - kWave; i < len; i += NT - kWave) z += exp2f((key_to_float(keys[i]) - dmax) * esc);
    z = wave_sum(z);
    if (lane == 0) red[wave] = z;
  }
  __syncthreads();
  if (tid == 0) {
    float z = 0.0f;
#pragma unroll
    for (int w = 1; w < NW; ++w) z += red[w];
    a.tmax_ws[slot] = dmax;
    a.zsum_ws[slot] = z;
  }
  sort_span_by_digit<false>(keys, len, w0, p0, cur, skey, spos, a.skey_ws + slot * P, a.spos_ws + slot * P, tid);
}

// The grouped-query rule's keys for this plan: one workgroup per (KV unit, span) reads the G logit numerators of
// every position of its span (left in the workspace by gs_logits, with every head's span maxima and sums), forms
// the group score sum_h s-hat_h as a key, and publishes the span like bk_scores does (table, sorted arrays),
// indexed by KV unit: the G query heads of the group share one selection.
template <int G>
__global__ __launch_bounds__(NT, 2) void bk_group_scores(const BucketArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const int P = a.span_len;
  uint32_t* keys = smem;
  uint32_t* skey = keys + P;
  uint32_t* spos = skey + P;
  uint32_t* hist = spos + P;
  uint32_t* cur = hist + kRadixBins;
  float* hs = reinterpret_cast<float*>(cur + kRadixBins);        // [G][2] max, 1 / sum-exp
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int ukv, s;
  map_span(d.B * d.H_kv, a.n_span, ukv, s);
  const int b = ukv / d.H_kv, hk = ukv - b * d.H_kv;
  const size_t u0 = (size_t)b * d.H + (size_t)hk * G;
  const size_t slot = (size_t)ukv * a.n_span + s;
  uint16_t* fine = a.fine_ws + slot * kFineLen;
  uint16_t* coarse = a.coarse_ws + slot * 64;
  bool appended, bad, full;
  const int S = visible_length(d, b, appended, bad, full);
  if (S == 0) return;                      // reported, and the outputs written, by gs_logits
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  const Window win = make_window(d.local_window, S, kq);
  const int p0 = s * P;
  if (p0 >= S) {   // a span beyond the end of this sequence: an empty table
    for (int i = tid; i < kFineLen; i += NT) fine[i] = 0;
    if (tid < 64) coarse[tid] = 0;
    return;
  }
  const int len = S - p0 < P ? S - p0 : P;
  for (int i = tid; i < kRadixBins; i += NT) hist[i] = 0u;
  if (wave == 0) combine_span_stats<G>(a.stat_ws + (size_t)ukv * a.n1 * G * 2, a.n1, a.esc_ws + u0, lane, hs);
  __syncthreads();
  float mh[G], inv_z[G], esc[G];
#pragma unroll
  for (int h = 0; h < G; ++h) { mh[h] = hs[h * 2]; inv_z[h] = hs[h * 2 + 1]; esc[h] = a.esc_ws[u0 + h]; }
  const float* z_unit = a.z_ws + u0 * (size_t)d.S_max + p0;
  const int n_chunks = (len + 7) >> 3;
  for (int c = tid; c < n_chunks; c += NT) {
    float4 lo[G], hi[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float4* src = reinterpret_cast<const float4*>(z_unit + (size_t)h * d.S_max + c * 8);
      lo[h] = src[0]; hi[h] = src[1];
    }
    uint32_t kx[8], dg[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float dv[G];
#pragma unroll
      for (int h = 0; h < G; ++h) dv[h] = e < 4 ? (&lo[h].x)[e] : (&hi[h].x)[e - 4];
      kx[e] = c * 8 + e < len ? float_to_key(group_score<G>(dv, mh, esc, inv_z)) : 0u;
      dg[e] = bucket_digit<true>(kx[e]) << 21;      // hist_add_chunk counts by the first 11 bits of what it is given
    }
    hist_add_chunk(hist, dg, (win.S_old < p0 + len ? win.S_old : p0 + len) - (p0 + c * 8));
    uint4* dst = reinterpret_cast<uint4*>(keys + c * 8);
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  }
  // the part of the local window that lies in this span counts as the top digit
  const int w0 = win.S_old > p0 ? win.S_old - p0 : 0;
  if (tid == 0 && w0 < len) atomicAdd(&hist[hist_slot(kTopDigit)], (uint32_t)(len - w0));
  __syncthreads();
  if (wave == 0) build_span_table(hist, cur, fine, coarse, lane);
  __syncthreads();
  sort_span_by_digit<true>(keys, len, w0, p0, cur, skey, spos, a.skey_ws + slot * P, a.spos_ws + slot * P, tid);
}

// LDS words of bk_select_gather: two span-sized arrays and the bitmap, the candidates (keys sharing the
// threshold digit: up to cand_cap of them are ranked out of LDS, more are read again by every pass), a
// histogram, the table window of every span, per-span counters, the attention partials of the waves
__host__ __device__ constexpr size_t bk_tab_words(int n_span) { return n_span * 33 > NT ? (size_t)n_span * 33 : (size_t)NT; }
template <int DH>
__host__ __device__ constexpr size_t bk_select_words(int span_len, int n_span, int cand_cap) {
  return 2 * (size_t)span_len + span_len / 32 + 2 * (size_t)cand_cap + kRadixBins + bk_tab_words(n_span) +
         5 * (kMaxSpans + 8) + NW * (DH + 2) + 32 + 16 + 16;
}

// GROUP = true is the grouped-query rule: the tables and sorted arrays are the KV unit's (one selection for the
// group's query heads, written by bk_group_scores), the statistics and alpha are the head's own, from the logits
// gs_logits left in the workspace.
template <class T, int DH, bool GROUP>
__global__ __launch_bounds__(NT) void bk_select_gather(const BucketArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const int P = a.span_len;
  uint32_t* keyval = smem;                                  // [P] keys of this span's selected positions, by position
  int* list = reinterpret_cast<int*>(keyval + P);           // [P] this span's selected positions, ascending
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(list + P); // [P / 32] selected positions of this span
  uint32_t* ckey = bitmap + P / 32;                         // [cand_cap] candidates: keys with the threshold digit
  uint32_t* cpos = ckey + a.cand_cap;                       // [cand_cap]
  uint32_t* hist = cpos + a.cand_cap;                       // [kRadixBins]
  uint32_t* tabF = hist + kRadixBins;                       // [n_span][33] A_s[32 lc + t] (at least NT words)
  int* a_s = reinterpret_cast<int*>(tabF + bk_tab_words(a.n_span)); // [n_span] entries of span s above the threshold digit
  int* c_s = a_s + kMaxSpans + 8;                           // [n_span] entries of span s with the threshold digit
  int* cpre = c_s + kMaxSpans + 8;                          // [n_span + 1] candidates before span s
  int* csel = cpre + kMaxSpans + 8;                         // [n_span] selected candidates of span s
  int* offs = csel + kMaxSpans + 8;                         // [n_span + 1] list entries before span s
  float* part = reinterpret_cast<float*>(offs + kMaxSpans + 8);   // [NW][DH + 2] attention partials of the waves
  float* red = part + NW * (DH + 2);                        // [32]
  uint32_t* wcnt = reinterpret_cast<uint32_t*>(red + 32);   // [16]
  int* ctl = reinterpret_cast<int*>(wcnt + 16);             // [16]
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int U = d.B * d.H;
  int u, s;
  map_span(U, a.n_span, u, s);
  const int b = u / d.H, h = u - b * d.H;
  const size_t kv_head = (size_t)b * d.H_kv + h / (d.H / d.H_kv);
  const size_t slot = (size_t)u * a.n_span + s;                       // this workgroup's partial and numerator
  const size_t slot0 = (GROUP ? kv_head : (size_t)u) * a.n_span;      // the spans whose tables and sorted arrays it reads
  using G = RowGeometry<DH>;
  const int sub = lane % G::LPR;

  // everything that does not depend on another load is requested at once: the lengths, the query slice of
  // Step 2, the temperature, the spans' statistics, and the coarse tables (wave w takes spans w, w + 8, ...)
  bool appended, bad, full;
  const int S = visible_length(d, b, appended, bad, full);
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  const uint4 qraw = load16(reinterpret_cast<const uint16_t*>(d.q) + (size_t)u * DH + sub * 8);
  const float esc = GROUP ? a.esc_ws[u] : kLog2e / a.tau_ws[u];
  uint32_t v[kMaxSpans / NW];
#pragma unroll
  for (int j = 0; j < kMaxSpans / NW; ++j) {
    const int t = wave + j * NW;
    v[j] = t < a.n_span ? a.coarse_ws[(slot0 + t) * 64 + lane] : 0u;
  }
  float tm = -INFINITY, zs = 0.0f;
  if (GROUP) {         // this head's maximum and sum-exp over each of gs_logits' spans
    const float* st = a.stat_ws + ((kv_head * a.n1 + lane) * a.group + (h % a.group)) * 2;
    if (wave == 1 && lane < a.n1) { tm = st[0]; zs = st[1]; }
  } else if (wave == 1 && lane < a.n_span) {
    tm = a.tmax_ws[slot0 + lane]; zs = a.zsum_ws[slot0 + lane];
  }

  if (S == 0) return;                      // outputs written by bk_scores
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  const int p0 = s * P;
  int32_t* idx_out = d.idx_out ? d.idx_out + (size_t)u * d.idx_stride : nullptr;
  float* my_part = a.part_ws + slot * (DH + 2);
  if (s == 0) {
    if (idx_out) for (int n = kq + tid; n < d.idx_stride; n += NT) idx_out[n] = -1;
    if (tid == 0 && idx_out && kq > d.idx_stride) atomicOr(d.err, 4);
  }
  if (p0 >= S) {                           // nothing of this sequence lies in this span: an empty partial
    if (tid < DH) my_part[tid] = 0.0f;
    if (tid == 0) { my_part[DH] = -INFINITY; my_part[DH + 1] = 0.0f; a.anum_ws[slot] = 0.0f; }
    return;
  }
  const int len = S - p0 < P ? S - p0 : P;

  // ---- the threshold digit d0: the largest d with N(d) = sum over spans of A_s[d] >= kq ----
  for (int i = tid; i < kRadixBins; i += NT) hist[i] = 0u;
  for (int i = tid; i < P / 32; i += NT) bitmap[i] = 0u;
  if (tid < a.n_span) csel[tid] = 0;
  {
    if (wave == 1) {
      // the largest logit of the sequence and the softmax denominator relative to it
      const float gm = wave_max(tm);
      const float z = wave_sum(tm == -INFINITY ? 0.0f : zs * exp2f((tm - gm) * esc));
      if (lane == 0) { red[30] = gm; red[31] = z; }
    }
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < kMaxSpans / NW; ++j) mine += v[j];
    tabF[wave * kWave + lane] = mine;      // tabF is free until the fine tables arrive
  }
  __syncthreads();
  if (wave == 0) {
    uint32_t n32 = 0;                      // N(32 lane)
#pragma unroll
    for (int w = 0; w < NW; ++w) n32 += tabF[w * kWave + lane];
    const uint64_t ok = __ballot(n32 >= (uint32_t)kq);      // lane 0 always: N(0) = S >= kq
    if (lane == 0) ctl[0] = 63 - __builtin_clzll((unsigned long long)ok);
  }
  __syncthreads();
  const int lc = ctl[0];
  const float gmax = red[30];
  if (s == 0 && tid == 0) a.zden_ws[u] = red[31];
  for (int i = tid; i < a.n_span * 33; i += NT) {
    const int t = i / 33, j = i - t * 33;
    tabF[i] = a.fine_ws[(slot0 + t) * kFineLen + lc * 32 + j];
  }
  __syncthreads();
  if (wave == 0) {
    uint32_t nf = 0;                       // lane j <= 32: N(32 lc + j)
    if (lane <= 32)
      for (int t = 0; t < a.n_span; ++t) nf += tabF[t * 33 + lane];
    const uint64_t ok = __ballot(lane < 32 && nf >= (uint32_t)kq);   // bit 0 always: N(32 lc) >= kq
    const int j0 = 63 - __builtin_clzll((unsigned long long)ok);
    const uint32_t n_at = (uint32_t)__shfl((int)nf, j0), above = (uint32_t)__shfl((int)nf, j0 + 1);
    // per span (lane = span): entries above the threshold digit, entries with it
    const bool on = lane < a.n_span;
    const int as = on ? (int)tabF[lane * 33 + j0 + 1] : 0;
    const int cs = on ? (int)tabF[lane * 33 + j0] - as : 0;
    const uint32_t incl = wave_scan_incl((uint32_t)cs);
    if (on) { a_s[lane] = as; c_s[lane] = cs; }
    cpre[lane + 1] = (int)incl;
    if (lane == 0) {
      cpre[0] = 0;
      ctl[1] = lc * 32 + j0;               // d0
      ctl[2] = kq - (int)above;            // candidates still needed
      ctl[3] = (int)(n_at - above);        // candidates
    }
  }
  __syncthreads();
  int need = ctl[2];
  const int C0 = ctl[3];
  const bool resident = C0 <= a.cand_cap;

  // this span's own entries above or in the threshold digit: the first four per thread are requested now,
  // together with the candidates, and looked at after the ranking
  const uint32_t* gkey = a.skey_ws + (slot0 + s) * P;
  const uint32_t* gpos = a.spos_ws + (slot0 + s) * P;
  const int n_above = a_s[s], n_mine = n_above + c_s[s];
  uint32_t okey[4], opos[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = j * NT + tid;
    okey[j] = e < n_mine ? gkey[e] : 0u;
    opos[j] = e < n_mine ? gpos[e] : 0u;
  }

  // candidate number i -> (span, entry of that span's sorted array)
  auto locate = [&](int i, int& t, int& e) {
    int lo = 0, hi = a.n_span - 1;         // the last span t with cpre[t] <= i
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (cpre[mid] <= i) lo = mid; else hi = mid - 1;
    }
    t = lo; e = a_s[lo] + (i - cpre[lo]);
  };
  if (resident) {          // the candidates once into LDS, the span number above the position's 20 bits
    for (int i0 = 0; i0 < C0; i0 += 4 * NT) {       // four candidates per thread in flight
      uint32_t key[4], pos[4];
      int t[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * NT + tid;
        int e = 0;
        t[j] = 0;
        if (i < C0) locate(i, t[j], e);
        key[j] = i < C0 ? a.skey_ws[(slot0 + t[j]) * P + e] : 0u;
        pos[j] = i < C0 ? a.spos_ws[(slot0 + t[j]) * P + e] : 0u;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * NT + tid;
        if (i < C0) { ckey[i] = key[j]; cpos[i] = pos[j] | ((uint32_t)t[j] << 20); }
      }
    }
    __syncthreads();
  }
  // a candidate as one 52-bit number: the key, then the position counted down from the top, so that "larger" is
  // "larger key, or equal key and lower position"; t = its span
  auto candidate = [&](int i, int& t) -> uint64_t {
    uint32_t key, pos;
    if (resident) {
      key = ckey[i]; pos = cpos[i] & kPosMask; t = (int)(cpos[i] >> 20);
    } else {               // more candidates than the LDS holds (many identical keys): every pass reads them again
      int e;
      locate(i, t, e);
      key = a.skey_ws[(slot0 + t) * P + e];
      pos = a.spos_ws[(slot0 + t) * P + e];
    }
    return ((uint64_t)key << 20) | (uint64_t)(kPosMask - pos);
  };

  // ---- exact rank among the candidates: radix passes of 11, 11, 10 (the key) and 10, 10 bits (the position); stop
  // as soon as the remaining bin is taken whole (with distinct keys: after the key bits at the latest).  The keys of
  // an ordinary bucket share their top 14 bits: then the passes take key bits 17..7 and 6..0 (one pass in practice:
  // a few hundred candidates over 2048 bins) ----
  uint64_t mask = 0, thr = 0;
  if (need < C0) {
    int in_bin = C0;
    int first_pass = 0;
    bool shared_top = false;
    if (!GROUP) {
      // An ordinary bucket away from the two ends of the exponent range fixes sign, exponent and five mantissa bits
      // of its keys: take those 14 bits from any candidate instead of looking for them.
      const uint32_t low = (uint32_t)ctl[1] >= 1024u ? (uint32_t)ctl[1] - 1024u : 1023u - (uint32_t)ctl[1];
      if (low >= 1u && low <= 1021u) {
        int t0;
        thr = (candidate(0, t0) >> 38) << 38;
        mask = (uint64_t)0x3fffu << 38;
        first_pass = 1;
        shared_top = true;
      }
    }
    for (int pass = first_pass; pass < 5 && need < in_bin; ++pass) {
      const int shift = pass == 0 ? 41 : (pass == 1 ? (shared_top ? 27 : 30) : 40 - 10 * pass);
      const uint32_t dmask = pass < 2 ? 0x7ffu : (pass == 2 && shared_top ? 0x7fu : 0x3ffu);
      if (pass > first_pass) {
        for (int i = tid; i < kRadixBins; i += NT) hist[i] = 0u;
        __syncthreads();
      }
      for (int i0 = 0; i0 < C0; i0 += NT) {
        const int i = i0 + tid;
        int t = 0;
        const uint64_t c = i < C0 ? candidate(i, t) : 0;
        hist_add_ties(hist, (uint32_t)(c >> shift) & dmask, i < C0 && (c & mask) == thr, lane);
      }
      __syncthreads();
      if (wave == 0) find_threshold_bin(hist, need, lane, ctl + 8);
      __syncthreads();
      thr |= (uint64_t)(uint32_t)ctl[8] << shift;
      mask |= (uint64_t)dmask << shift;
      need = ctl[9];
      in_bin = ctl[10];
      __syncthreads();                     // ctl is rewritten by the next pass
    }
  }
  // selected candidates: (c & mask) >= thr.  Count them per span: the list entries of span t are its a_s
  // entries above the threshold digit plus its selected candidates.
  for (int i = tid; i < C0; i += NT) {
    int t = 0;
    const uint64_t c = candidate(i, t);
    if ((c & mask) >= thr) atomicAdd(&csel[t], 1);
  }
  __syncthreads();
  if (wave == 0) {
    const bool on = lane < a.n_span;
    const uint32_t m = on ? (uint32_t)(a_s[lane] + csel[lane]) : 0u;
    const uint32_t incl = wave_scan_incl(m);
    if (on) offs[lane] = (int)(incl - m);
    // the spans' shares must add up to the k positions asked for
    if (lane == kWave - 1 && incl != (uint32_t)kq) atomicOr(d.err, 16);
  }

  // ---- this span's own selected positions: a bitmap in position order, with their keys ----
  auto mark = [&](int e, uint32_t key, uint32_t pos) {
    bool take = e < n_above;
    if (!take) {
      const uint64_t c = ((uint64_t)key << 20) | (uint64_t)(kPosMask - pos);
      take = (c & mask) >= thr;
    }
    if (take) {
      const uint32_t rel = pos - (uint32_t)p0;
      atomicOr(&bitmap[rel >> 5], 1u << (rel & 31u));
      keyval[rel] = key;
    }
  };
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (j * NT + tid < n_mine) mark(j * NT + tid, okey[j], opos[j]);
  for (int e = 4 * NT + tid; e < n_mine; e += NT) mark(e, gkey[e], gpos[e]);
  __syncthreads();
  // ordered emission: thread t owns bitmap word t (span_len <= 8192: at most 256 words)
  const uint32_t word = tid < (len + 31) / 32 ? bitmap[tid] : 0u;
  uint32_t total;
  uint32_t o = block_scan_excl((uint32_t)__popc(word), wcnt, lane, wave, &total);
  float anum = 0.0f;
  uint32_t w = word;
  while (w) {
    const int bit = __ffs((int)w) - 1;
    w &= w - 1;
    const int rel = tid * 32 + bit;
    list[o] = p0 + rel;
    if (idx_out && offs[s] + (int)o < d.idx_stride) idx_out[offs[s] + o] = p0 + rel;
    if (!GROUP) anum += exp2f((key_to_float(keyval[rel]) - gmax) * esc);
    ++o;
  }
  if (GROUP) {         // this head's own approximate scores of the selected positions, from its stored logits
    __syncthreads();   // the list
    const float* z_head = a.z_ws + (size_t)u * d.S_max;
    for (int n = tid; n < (int)total; n += NT) anum += exp2f((z_head[list[n]] - gmax) * esc);
  }
  anum = wave_sum(anum);
  if (lane == 0) red[wave] = anum;
  __syncthreads();                         // also publishes the list
  if (tid == 0) {
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[i];
    a.anum_ws[slot] = t;
  }

  // ---- Step 2b over this span's selected rows -> one partial (numerator, max, denominator) per span ----
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[8];
  {
    float f[8];
    unpack8<T>(qraw, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) q8[e] = f[e] * qscale;
  }
  const char* K_head = reinterpret_cast<const char*>(d.K) + kv_head * d.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(d.V) + kv_head * d.S_stride * (size_t)(DH * 2) + sub * 16;
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // positions are ascending, so the row being appended (position S - 1, not in the cache yet) can only be the
  // last entry of the last span's list: it is taken from the inputs
  const bool new_selected = appended && total > 0 && list[total - 1] == S - 1;
  attend_rows<T, DH>(K_head, V_head, list, 0, (int)total - (new_selected ? 1 : 0), q8, lane, wave, m_run, l_run, acc);
  if (new_selected)
    attend_row_from_codes<T, DH>(reinterpret_cast<const uint16_t*>(d.k_new) + kv_head * DH,
                                 reinterpret_cast<const uint16_t*>(d.v_new) + kv_head * DH, q8, lane, wave, m_run, l_run, acc);
  store_wave_partial<DH>(m_run, l_run, acc, part, lane, wave);
  __syncthreads();
  if (tid < DH) {
    float m_all, l_all, y;
    combine_partials<DH>(part, NW, tid, m_all, l_all, y);
    my_part[tid] = y;
    if (tid == 0) { my_part[DH] = m_all; my_part[DH + 1] = l_all; }
  }
}

// One workgroup per unit: merge the spans' partials, alpha from the spans' numerators, blend with the mean
// value vector (Eq. 10), round and store.
template <class T, int DH>
__global__ __launch_bounds__(DH) void bk_combine(const BucketArgs a) {
  const DecodeArgs& d = a.d;
  const int u = blockIdx.x, c = threadIdx.x;
  const int b = u / d.H, h = u - b * d.H;
  const size_t kv_head = (size_t)b * d.H_kv + h / (d.H / d.H_kv);
  bool appended, bad, full;
  const int S = visible_length(d, b, appended, bad, full);
  float vm = d.v_mean[kv_head * DH + c];
  // the step's append, after every read of the cache by the earlier launches: the workgroup of the first query
  // head of a KV group writes the rows, the 8 columns of Kt that the row may complete, and the new mean
  // (the same update as sparq_kv_append's; the mean of no rows is ignored); lengths and means go to the *_next
  // buffers.  The inputs are requested here; the stores are issued after the merge (stores ahead of the partials'
  // loads would sit on their critical path: the memory counter retires both in order).
  uint16_t vcode = 0, kc = 0;
  const bool owner = h == (h / (d.H / d.H_kv)) * (d.H / d.H_kv);
  if (d.k_new) {
    vcode = reinterpret_cast<const uint16_t*>(d.v_new)[kv_head * DH + c];
    if (owner && appended) kc = reinterpret_cast<const uint16_t*>(d.k_new)[kv_head * DH + c];
  }
  auto append_stores = [&]() {
    if (owner) {
      d.v_mean_next[kv_head * DH + c] = vm;
      if (appended) {
        uint16_t* K_rows = reinterpret_cast<uint16_t*>(d.K) + kv_head * d.S_stride * (size_t)DH;
        reinterpret_cast<uint16_t*>(d.V)[(kv_head * d.S_stride + (S - 1)) * DH + c] = vcode;
        K_rows[(size_t)(S - 1) * DH + c] = kc;
        if ((S & 7) == 0)
          flush_key_columns(reinterpret_cast<uint16_t*>(d.Kt) + kv_head * DH * (size_t)d.S_stride, K_rows, d.S_stride, DH, S, c, kc);
      }
    }
    if (h == 0 && c == 0) {   // a length beyond the bound of this call that the buffers can hold is carried over as it is
      const int S_in = d.seq_lens[b];
      d.seq_lens_next[b] = (S_in > d.S_max && S_in <= d.S_stride) ? S_in : S;
    }
  };
  if (S <= 0) {                            // outputs written by bk_scores
    if (d.k_new) append_stores();
    return;
  }
  const float* parts = a.part_ws + (size_t)u * a.n_span * (DH + 2);
  const int ln = c & (kWave - 1);
  const float num = wave_sum(ln < a.n_span ? a.anum_ws[(size_t)u * a.n_span + ln] : 0.0f);   // fixed order
  const float zden = a.zden_ws[u];
  float m_all = -INFINITY, l_all = 0.0f, y3 = 0.0f;
  for (int w0 = 0; w0 < a.n_span; w0 += 16) {          // sixteen partials of this channel in flight at a time
    float pm[16], pl[16], py[16];
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const bool on = w0 + w < a.n_span;
      pm[w] = on ? parts[(w0 + w) * (DH + 2) + DH] : -INFINITY;
      pl[w] = on ? parts[(w0 + w) * (DH + 2) + DH + 1] : 0.0f;
      py[w] = on ? parts[(w0 + w) * (DH + 2) + c] : 0.0f;
    }
    float m_new = m_all;
#pragma unroll
    for (int w = 0; w < 16; ++w) m_new = fmaxf(m_new, pm[w]);
    const float sc = weight_exp2(m_all, m_new);
    l_all *= sc; y3 *= sc;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const float sw = weight_exp2(pm[w], m_new);
      l_all += pl[w] * sw;
      y3 += py[w] * sw;
    }
    m_all = m_new;
  }
  y3 /= l_all;
  const float alpha = num / zden;
  if (c == 0 && d.alpha_out) d.alpha_out[u] = alpha;
  if (d.k_new && appended) {               // the mean with the new row: what the blend uses and the owner stores
    if (S == 1) vm = 0.0f;
    vm += (T::widen(vcode) - vm) * (1.0f / (float)S);
  }
  float y = y3;
  if (!(d.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * vm;
  reinterpret_cast<uint16_t*>(d.out)[(size_t)u * DH + c] = T::narrow(y);
  if (d.k_new) append_stores();
}

template <class T, int DH>
hipError_t launch_bucket(const BucketArgs& a, hipStream_t s) {
  const int units = a.d.B * a.d.H;
  const size_t lds1 = bk_scores_lds_bytes(a.span_len, DH), lds2 = bk_select_lds_bytes(a.span_len, DH, a.n_span, a.cand_cap);
  hipError_t e;
  if ((e = allow_lds<bk_scores<T, DH>>(lds1)) != hipSuccess) return e;
  if ((e = allow_lds<bk_select_gather<T, DH, false>>(lds2)) != hipSuccess) return e;
  hipLaunchKernelGGL((bk_scores<T, DH>), dim3(units * a.n_span), dim3(NT), lds1, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((bk_select_gather<T, DH, false>), dim3(units * a.n_span), dim3(NT), lds2, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((bk_combine<T, DH>), dim3(units), dim3(DH), 0, s, a);
  return hipGetLastError();
}

// the grouped-query rule: the keys come from the group's stored logits, the rest is the same two launches
template <class T, int DH>
hipError_t launch_bucket_group(const BucketArgs& a, hipStream_t s) {
  const int units = a.d.B * a.d.H, ukv = a.d.B * a.d.H_kv;
  const size_t lds1 = bk_group_scores_lds_bytes(a.span_len), lds2 = bk_select_lds_bytes(a.span_len, DH, a.n_span, a.cand_cap);
  hipError_t e;
  if ((e = allow_lds<bk_select_gather<T, DH, true>>(lds2)) != hipSuccess) return e;
  switch (a.group) {
    case 2:
      if ((e = allow_lds<bk_group_scores<2>>(lds1)) != hipSuccess) return e;
      hipLaunchKernelGGL(bk_group_scores<2>, dim3(ukv * a.n_span), dim3(NT), lds1, s, a);
      break;
    case 4:
      if ((e = allow_lds<bk_group_scores<4>>(lds1)) != hipSuccess) return e;
      hipLaunchKernelGGL(bk_group_scores<4>, dim3(ukv * a.n_span), dim3(NT), lds1, s, a);
      break;
    default: return hipErrorInvalidValue;
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((bk_select_gather<T, DH, true>), dim3(units * a.n_span), dim3(NT), lds2, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((bk_combine<T, DH>), dim3(units), dim3(DH), 0, s, a);
  return hipGetLastError();
}

}  // namespace

size_t bk_group_scores_lds_bytes(int span_len) { return 4 * (3 * (size_t)span_len + 2 * kRadixBins + 16); }

size_t bk_scores_lds_bytes(int span_len, int d_h) {
  switch (d_h) {
    case 64: return 4 * (3 * (size_t)span_len + bk_scores_fixed_words<64>());
    case 128: return 4 * (3 * (size_t)span_len + bk_scores_fixed_words<128>());
    case 256: return 4 * (3 * (size_t)span_len + bk_scores_fixed_words<256>());
    default: return 0;
  }
}

size_t bk_select_lds_bytes(int span_len, int d_h, int n_span, int cand_cap) {
  switch (d_h) {
    case 64: return 4 * bk_select_words<64>(span_len, n_span, cand_cap);
    case 128: return 4 * bk_select_words<128>(span_len, n_span, cand_cap);
    case 256: return 4 * bk_select_words<256>(span_len, n_span, cand_cap);
    default: return 0;
  }
}

int bk_fine_len() { return kFineLen; }

hipError_t launch_decode_bucket(const BucketArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_bucket<BF16, 64>(a, s) : launch_bucket<F16, 64>(a, s);
    case 128: return bf ? launch_bucket<BF16, 128>(a, s) : launch_bucket<F16, 128>(a, s);
    case 256: return bf ? launch_bucket<BF16, 256>(a, s) : launch_bucket<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

hipError_t launch_decode_bucket_group(const BucketArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_bucket_group<BF16, 64>(a, s) : launch_bucket_group<F16, 64>(a, s);
    case 128: return bf ? launch_bucket_group<BF16, 128>(a, s) : launch_bucket_group<F16, 128>(a, s);
    case 256: return bf ? launch_bucket_group<BF16, 256>(a, s) : launch_bucket_group<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
