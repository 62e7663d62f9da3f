// SparQ decode for many (sequence, head) units with sequences too long for one workgroup's LDS (one 4-byte
// key per cached position does not fit beyond ~35 000 positions; few units with long caches go through the
// digit-bucket plan instead).  The top-k of a sequence is contained in the union of the top-k of
// its parts (a position beaten by fewer than k others overall is beaten by fewer than k in its own part,
// ties to the lower position in both), so the selection of Step 2 is made in two levels:
//   long_scores    (units x n_span workgroups) Step 1 on a span of span_len positions, keys in LDS; the
//                  span's own top-min(k, span) positions go to the workspace as (key, position) candidates,
//                  position-ascending, with the span's largest logit and its softmax denominator
//   long_merge     (one workgroup per unit) the candidates of all spans into LDS (at most n_span x k),
//                  the same radix select and ordered compaction over them, alpha, the position list
//   split_gather / split_combine   exact attention over slices of the list, merge and blend
// The local window is part of both levels: its positions are the last ones of the sequence, every span
// hands on those it holds, and they are the last candidates of the merge.
#include "decode_stages.h"

namespace sparq {

namespace {

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

// LDS words of long_scores besides the span's keys
template <int DH>
__host__ __device__ constexpr size_t scores_fixed_words() {
  return 2 * (size_t)kRadixBins + NT + 4 * (size_t)DH + 32 + 16 + 8;
}

template <class T, int DH>
__global__ __launch_bounds__(NT, 4) void long_scores(const LongArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  uint32_t* keys = smem;                                        // [span_len]
  uint32_t* hist = keys + a.span_len;                           // [2][kRadixBins]
  int* rankp = reinterpret_cast<int*>(hist + 2 * kRadixBins);   // [NT]
  float* qf = reinterpret_cast<float*>(rankp + NT);             // [DH]
  float* qs = qf + DH;
  int* chan = reinterpret_cast<int*>(qs + DH);
  uint32_t* mag = reinterpret_cast<uint32_t*>(chan + DH);
  float* red = reinterpret_cast<float*>(mag + DH);              // [32]
  uint32_t* wcnt = reinterpret_cast<uint32_t*>(red + 32);       // [16]
  int* ctl = reinterpret_cast<int*>(wcnt + 16);                 // [8]
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int U = d.B * d.H;
  int u, s;
  map_span(U, a.n_span, u, s);
  const int b = u / d.H, h = u - b * d.H;
  const size_t kv_head = (size_t)b * d.H_kv + h / (d.H / d.H_kv);

  uint16_t qcode = 0;
  if (tid < DH) qcode = reinterpret_cast<const uint16_t*>(d.q)[(size_t)u * DH + tid];
  int S = d.seq_lens[b];
  if (S < 0 || S > d.S_max) {
    if (tid == 0 && s == 0) atomicOr(d.err, 8);
    S = S < 0 ? 0 : d.S_max;
  }
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
  const size_t slot = (size_t)u * a.n_span + s;
  const int p0 = s * a.span_len;
  if (p0 >= S) {   // a span beyond the end of this sequence
    if (tid == 0) { a.cnt_ws[slot] = 0; a.tmax_ws[slot] = -INFINITY; a.zsum_ws[slot] = 0.0f; }
    return;
  }
  const int len = S - p0 < a.span_len ? S - p0 : a.span_len;

  for (int i = tid; i < 2 * kRadixBins; i += NT) hist[i] = 0u;
  const QueryLds Q{mag, rankp, qf, qs, chan};
  const float tau = apply_tau_mode(select_channels<T, DH>(Q, qcode, d.r, tid, lane, wave), d.flags, DH, d.r);
  if (s == 0) {
    if (d.chan_out && tid < d.r) d.chan_out[(size_t)u * d.r + tid] = chan[tid];
    if (tid == 0) a.tau_ws[u] = tau;
  }

  // the newest S mod 8 positions are not in Kt: the span that holds them takes them from the rows of K
  const int S_fl = S & ~7, r8 = (d.r + 7) & ~7;
  const int n_tail = (S_fl >= p0 && S_fl < p0 + len) ? S - S_fl : 0;
  TailRow tail;
  if (wave < n_tail)
    tail = tail_row_issue(reinterpret_cast<const uint16_t*>(d.K) + (kv_head * d.S_stride + S_fl + wave) * (size_t)DH, chan, r8, lane);

  const int end = p0 + len < S_fl ? p0 + len : S_fl;     // whole chunks of this span that are in Kt
  const size_t row_bytes = (size_t)d.S_stride * 2;
  const char* Kt_head = reinterpret_cast<const char*>(d.Kt) + kv_head * DH * row_bytes;
  float tmax = -INFINITY;
  stream_channel_rows<T>(Kt_head, row_bytes, chan, qs, d.r, p0 >> 3, end > p0 ? end >> 3 : p0 >> 3, tid,
                         [&](int c, const float (&acc)[8]) {
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      tmax = fmaxf(tmax, acc[e]);
      kx[e] = float_to_key(acc[e]);
    }
    hist_add_chunk(hist, kx, win.S_old - c * 8);
    uint4* dst = reinterpret_cast<uint4*>(keys + (c * 8 - p0));
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  });
  if (wave < n_tail) {
    const float dot = tail_row_dot<T>(tail, qs, r8, lane);
    tmax = fmaxf(tmax, dot);
    if (lane == 0) {
      const uint32_t key = float_to_key(dot);
      keys[S_fl + wave - p0] = key;
      if (S_fl + wave < win.S_old) atomicAdd(&hist[hist_slot(key >> 21)], 1u);
    }
  }
  tmax = wave_max(tmax);
  if (lane == 0) red[wave] = tmax;
  __syncthreads();
  float dmax = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, red[w]);
  __syncthreads();     // red is reused by the compaction

  // the span's own selection: its part of the window unconditionally, and as many of its older positions
  // as the whole sequence may take
  int n_old = win.S_old - p0;
  n_old = n_old < 0 ? 0 : (n_old > len ? len : n_old);
  const int k_old = win.k_old < n_old ? win.k_old : n_old;
  const SelectLds sel{hist, wcnt, ctl, red};
  uint32_t pmask, pval;
  int need;
  radix_select(keys, n_old, k_old, sel, tid, lane, wave, pmask, pval, need);
  uint32_t* cand_key = a.cand_key_ws + slot * a.cand_cap;
  uint32_t* cand_pos = reinterpret_cast<uint32_t*>(a.cand_pos_ws) + slot * a.cand_cap;
  float sums[2];
  compact_selected(keys, cand_pos, len, n_old, pmask, pval, need, dmax, kLog2e / tau, nullptr, 0, sel, tid, lane, wave,
                   cand_key, p0, sums);
  if (tid == 0) {
    a.cnt_ws[slot] = k_old + (len - n_old);
    a.tmax_ws[slot] = dmax;
    a.zsum_ws[slot] = sums[0];
  }
}

// One workgroup per unit: merge the candidates of the spans.
__global__ __launch_bounds__(NT) void long_merge(const LongArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const DecodeArgs& d = a.d;
  const int cap_all = a.n_span * a.cand_cap;
  uint32_t* keys = smem;                                          // [round_up(cap_all, 8)]
  uint32_t* hist = keys + ((cap_all + 7) & ~7);                   // [2][kRadixBins]
  float* red = reinterpret_cast<float*>(hist + 2 * kRadixBins);   // [32]
  uint32_t* wcnt = reinterpret_cast<uint32_t*>(red + 32);         // [16]
  int* ctl = reinterpret_cast<int*>(wcnt + 16);                   // [8]
  int* off = ctl + 8;                                             // [kMaxSpans + 1] candidates before each span
  float* stat = reinterpret_cast<float*>(off + kMaxSpans + 8);    // [2]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int u = blockIdx.x, b = u / d.H;
  int S = d.seq_lens[b];
  S = S < 0 ? 0 : (S > d.S_max ? d.S_max : S);
  if (S == 0) return;                      // outputs written by long_scores
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  int32_t* idx_out = d.idx_out ? d.idx_out + (size_t)u * d.idx_stride : nullptr;
  const Window win = make_window(d.local_window, S, kq);
  const float tau = a.tau_ws[u];
  const float esc = kLog2e / tau;

  for (int i = tid; i < 2 * kRadixBins; i += NT) hist[i] = 0u;
  if (wave == 0) {   // kMaxSpans = 64: one lane per span
    const size_t slot = (size_t)u * a.n_span + lane;
    const bool on = lane < a.n_span;
    const int cnt = on ? a.cnt_ws[slot] : 0;
    const float tm = on ? a.tmax_ws[slot] : -INFINITY;
    const float zs = on ? a.zsum_ws[slot] : 0.0f;
    const uint32_t incl = wave_scan_incl((uint32_t)cnt);
    off[lane + 1] = (int)incl;
    if (lane == 0) off[0] = 0;
    const float dmax = wave_max(tm);
    const float z = wave_sum(tm == -INFINITY ? 0.0f : zs * exp2f((tm - dmax) * esc));
    if (lane == 0) { stat[0] = dmax; stat[1] = z; }
  }
  __syncthreads();
  const int n_cand = off[a.n_span];
  const int n_free = n_cand - win.n_local;        // candidates that compete; the window's come last
  const float dmax = stat[0], zsum = stat[1];
  for (int s = 0; s < a.n_span; ++s) {
    const int o = off[s], cnt = off[s + 1] - o;
    const uint32_t* src = a.cand_key_ws + ((size_t)u * a.n_span + s) * a.cand_cap;
    for (int n0 = 0; n0 < cnt; n0 += 4 * NT) {      // four loads in flight per thread
      uint32_t key[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int n = n0 + t * NT + tid;
        key[t] = n < cnt ? src[n] : 0u;
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int n = n0 + t * NT + tid;
        if (n < cnt) {
          keys[o + n] = key[t];
          if (o + n < n_free) atomicAdd(&hist[hist_slot(key[t] >> 21)], 1u);
        }
      }
    }
  }
  __syncthreads();
  const SelectLds sel{hist, wcnt, ctl, red};
  uint32_t pmask, pval;
  int need;
  radix_select(keys, n_free, win.k_old, sel, tid, lane, wave, pmask, pval, need);
  float sums[2];
  compact_selected(keys, keys, n_cand, n_free, pmask, pval, need, dmax, esc, nullptr, 0, sel, tid, lane, wave, nullptr, 0, sums);
  const float alpha = sums[1] / zsum;
  // candidate numbers -> positions
  int32_t* list = a.list_ws + (size_t)u * d.S_max;
  for (int n = tid; n < kq; n += NT) {
    const int ci = (int)keys[n];
    int s = 0;
    while (s + 1 < a.n_span && off[s + 1] <= ci) ++s;
    const int pos = a.cand_pos_ws[((size_t)u * a.n_span + s) * a.cand_cap + (ci - off[s])];
    list[n] = pos;
    if (idx_out && n < d.idx_stride) idx_out[n] = pos;
  }
  if (tid == 0) {
    a.alpha_ws[u] = alpha;
    if (d.alpha_out) d.alpha_out[u] = alpha;
    if (idx_out && kq > d.idx_stride) atomicOr(d.err, 4);
  }
  if (idx_out) for (int n = kq + tid; n < d.idx_stride; n += NT) idx_out[n] = -1;
}

template <class T, int DH>
hipError_t launch_long(const LongArgs& a, int dtype, hipStream_t s) {
  const int units = a.d.B * a.d.H;
  const size_t lds1 = 4 * ((size_t)a.span_len + scores_fixed_words<DH>()), lds2 = long_merge_lds_bytes(a.n_span, a.cand_cap);
  auto k1 = long_scores<T, DH>;
  hipError_t e;
  if ((e = allow_lds<long_scores<T, DH>>(lds1)) != hipSuccess) return e;
  if ((e = allow_lds<long_merge>(lds2)) != hipSuccess) return e;
  hipLaunchKernelGGL(k1, dim3(units * a.n_span), dim3(NT), lds1, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(long_merge, dim3(units), dim3(NT), lds2, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  SplitArgs g;
  g.d = a.d; g.n_split = a.n_split;
  g.alpha_ws = a.alpha_ws;
  g.list_ws = a.list_ws; g.part_ws = a.part_ws;
  return launch_split_gather(g, dtype, s);
}

}  // namespace

size_t long_scores_lds_bytes(int span_len, int d_h) {
  switch (d_h) {
    case 64: return 4 * ((size_t)span_len + scores_fixed_words<64>());
    case 128: return 4 * ((size_t)span_len + scores_fixed_words<128>());
    case 256: return 4 * ((size_t)span_len + scores_fixed_words<256>());
    default: return 0;
  }
}

size_t long_merge_lds_bytes(int n_span, int cand_cap) {
  return 4 * ((((size_t)n_span * cand_cap + 7) & ~(size_t)7) + 2 * kRadixBins + 32 + 16 + 8 + kMaxSpans + 8 + 8);
}

hipError_t launch_decode_long(const LongArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_long<BF16, 64>(a, dtype, s) : launch_long<F16, 64>(a, dtype, s);
    case 128: return bf ? launch_long<BF16, 128>(a, dtype, s) : launch_long<F16, 128>(a, dtype, s);
    case 256: return bf ? launch_long<BF16, 256>(a, dtype, s) : launch_long<F16, 256>(a, dtype, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
