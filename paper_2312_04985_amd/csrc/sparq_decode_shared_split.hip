// The paper's grouped-query rule (Section 4, "Grouped query attention"; Appendix B) over several workgroups
// per (sequence, KV head): for batches whose KV heads are fewer than the compute units, and for sequences
// beyond one workgroup's LDS.  Five launches; data passes between workgroups only across kernel boundaries.
//   gs_logits   (KV units x n1) channel selection from the group sums, Step 1b on a span for the G heads:
//               the logit numerators go to the workspace, each head's span maximum and sum-exp beside them
//   gs_select   (KV units x n2) per-head softmax statistics from the spans' partials, group score
//               sum_h s-hat_h of a span of positions as keys in LDS, the span's own top-min(k, span)
//               as (key, position) candidates (two-level selection, as in sparq_decode_long.hip)
//   gs_merge    (one workgroup per KV unit) select over the candidates, position list, alpha per head from
//               the stored logits of the selected positions
//   gs_gather   (KV units x n_split) each selected K and V row once for the G heads, partials per head
//   split_combine  (one workgroup per query head) merge, blend with the mean value vector (Eq. 10), store
#include "group_stages.h"

namespace sparq {

namespace {

__device__ __forceinline__ void map_kv(int Ukv, int n, int& ukv, int& s) {
  const int bid = blockIdx.x;
  if ((Ukv & 7) == 0) {          // the parts of a KV unit share an XCD (an L2)
    const int x = bid & 7, slot = bid >> 3;
    ukv = x * (Ukv >> 3) + slot / n;
    s = slot % n;
  } else {
    ukv = bid / n;
    s = bid % n;
  }
}

// Thread groups that share the chunks of a gs_logits span (see there): 4 or 2 when the span has at most NT / 4 or
// NT / 2 chunks and there are that many batches of 8 channel rows, else 1.  Host and device agree through this.
__host__ __device__ constexpr int logit_row_groups(int span1, int n_batches) {
  return (span1 <= NT / 4 * 8 && n_batches >= 4) ? 4 : ((span1 <= NT / 2 * 8 && n_batches >= 2) ? 2 : 1);
}

template <class T, int DH, int G>
__global__ __launch_bounds__(NT, 2) void gs_logits(const GsArgs a) {
  __shared__ int rankp[NT];
  __shared__ float qf[G * DH], qs[G * DH];
  __shared__ int chan[DH];
  __shared__ double magd[DH];
  __shared__ float stat[NW * G * 2];
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int ukv, s;
  map_kv(d.B * d.H_kv, a.n1, ukv, s);
  const int b = ukv / d.H_kv, hk = ukv - b * d.H_kv;
  const size_t u0 = (size_t)b * d.H + (size_t)hk * G;
  bool appended, bad, full;      // inside a step of the digit-bucket plan the row being appended counts as position S_b
  const int S = visible_length(d, b, appended, bad, full);
  if (tid == 0 && s == 0 && (bad || full)) atomicOr(d.err, (bad ? 8 : 0) | (full ? 1 : 0));
  if (S == 0) {   // nothing cached: part 0 writes the defined outputs, the later launches skip the unit
    if (s == 0) {
      uint16_t* out = reinterpret_cast<uint16_t*>(d.out) + u0 * DH;
      for (int i = tid; i < G * DH; i += NT) out[i] = 0;
      if (tid < G && d.alpha_out) d.alpha_out[u0 + tid] = 0.0f;
      if (tid == 0) atomicOr(d.err, 2);
      if (d.chan_out) for (int i = tid; i < G * d.r; i += NT) d.chan_out[u0 * d.r + i] = -1;
      if (d.idx_out) for (int i = tid; i < G * d.idx_stride; i += NT) d.idx_out[u0 * d.idx_stride + i] = -1;
    }
    return;
  }
  float* stat_out = a.stat_ws + ((size_t)ukv * a.n1 + s) * G * 2;
  const int p0 = s * a.span1;
  if (p0 >= S) {   // a span beyond the end of this sequence
    if (tid < G) { stat_out[tid * 2] = -INFINITY; stat_out[tid * 2 + 1] = 0.0f; }
    return;
  }
  const int len = S - p0 < a.span1 ? S - p0 : a.span1;

  float esc[G];
  const GroupQueryLds GQ{rankp, qf, qs, chan, magd};
  select_channels_group<T, DH, G>(GQ, reinterpret_cast<const uint16_t*>(d.q) + u0 * DH, d.r, d.flags, tid, lane, wave, esc);
  if (s == 0) {
    if (d.chan_out) for (int i = tid; i < G * d.r; i += NT) d.chan_out[u0 * d.r + i] = chan[i % d.r];
    if (tid == 0) {
#pragma unroll
      for (int h = 0; h < G; ++h) a.esc_ws[u0 + h] = esc[h];
    }
  }

  // the newest S mod 8 positions are not in Kt: the span that holds them takes them from the rows of K
  const size_t kv_head = (size_t)ukv;
  const int S_fl = (appended ? S - 1 : S) & ~7, r8 = (d.r + 7) & ~7;
  const int n_tail = (S_fl >= p0 && S_fl < p0 + len) ? S - S_fl : 0;
  TailRow tail;                  // requested here, used after the stream
  if (wave < n_tail) {
    const uint16_t* krow = appended && wave == n_tail - 1
                               ? reinterpret_cast<const uint16_t*>(d.k_new) + kv_head * DH
                               : reinterpret_cast<const uint16_t*>(d.K) + (kv_head * d.S_stride + S_fl + wave) * (size_t)DH;
    tail = tail_row_issue(krow, chan, r8, lane);
  }

  const int end = p0 + len < S_fl ? p0 + len : S_fl;     // whole chunks of this span that are in Kt
  const size_t row_bytes = (size_t)d.S_stride * 2;
  const char* Kt_head = reinterpret_cast<const char*>(d.Kt) + kv_head * DH * row_bytes;
  float* z_unit = a.z_ws + u0 * (size_t)d.S_max;
  float mt[G], zt[G];
#pragma unroll
  for (int h = 0; h < G; ++h) { mt[h] = -INFINITY; zt[h] = 0.0f; }
  auto finish = [&](int c, const float (&acc)[G][8]) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float4* dst = reinterpret_cast<float4*>(z_unit + (size_t)h * d.S_max + c * 8);
      dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
      dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = acc[h][e];
        if (v > mt[h]) { zt[h] = zt[h] * exp2f((mt[h] - v) * esc[h]) + 1.0f; mt[h] = v; }
        else zt[h] += exp2f((v - mt[h]) * esc[h]);
      }
    }
  };
  const int c_begin = p0 >> 3, c_end = end > p0 ? end >> 3 : p0 >> 3;
  const int nb = r8 >> 3;
  const int F = logit_row_groups(a.span1, nb);
  if (F > 1) {
    // Fewer chunks than threads: F groups of NT / F threads share every chunk, each taking 1 / F of the batches of 8
    // channel rows, so that a thread's loads are in flight together instead of going through the pipeline one
    // batch after the other.  The groups' partial sums meet in LDS and the first group finishes the chunks.
    extern __shared__ __align__(16) float pacc[];                 // [F][G][span1]
    const int P = a.span1;
    if (F == 4) {
      const int part = tid >> 7, t = tid & (NT / 4 - 1);
      const int b0 = part * nb / 4, b1 = (part + 1) * nb / 4;
      stream_channel_rows_group<T, G, NT / 4>(Kt_head, row_bytes, chan + 8 * b0, qs + 8 * b0, DH, 8 * (b1 - b0), c_begin, c_end, t,
                                              [&](int c, const float (&acc)[G][8]) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float4* dst = reinterpret_cast<float4*>(pacc + (size_t)(part * G + h) * P + (c * 8 - p0));
          dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
          dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
        }
      });
    } else {
      const int part = tid >> 8, t = tid & (NT / 2 - 1);
      const int b0 = part * nb / 2, b1 = (part + 1) * nb / 2;
      stream_channel_rows_group<T, G, NT / 2>(Kt_head, row_bytes, chan + 8 * b0, qs + 8 * b0, DH, 8 * (b1 - b0), c_begin, c_end, t,
                                              [&](int c, const float (&acc)[G][8]) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float4* dst = reinterpret_cast<float4*>(pacc + (size_t)(part * G + h) * P + (c * 8 - p0));
          dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
          dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
        }
      });
    }
    __syncthreads();
    for (int c = c_begin + tid; c < c_end; c += NT) {
      float acc[G][8];
#pragma unroll
      for (int h = 0; h < G; ++h) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;
        for (int part = 0; part < F; ++part) {                 // in the order of the channel list
          const float4* src = reinterpret_cast<const float4*>(pacc + (size_t)(part * G + h) * P + (c * 8 - p0));
          const float4 x0 = src[0], x1 = src[1];
          acc[h][0] += x0.x; acc[h][1] += x0.y; acc[h][2] += x0.z; acc[h][3] += x0.w;
          acc[h][4] += x1.x; acc[h][5] += x1.y; acc[h][6] += x1.z; acc[h][7] += x1.w;
        }
      }
      finish(c, acc);
    }
  } else {
    stream_channel_rows_group<T, G>(Kt_head, row_bytes, chan, qs, DH, d.r, c_begin, c_end, tid, finish);
  }
  float tdot[G];
#pragma unroll
  for (int h = 0; h < G; ++h) tdot[h] = wave < n_tail ? tail_row_dot<T>(tail, qs + h * DH, r8, lane) : 0.0f;
  if (wave < n_tail && lane == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float v = tdot[h];
      z_unit[(size_t)h * d.S_max + S_fl + wave] = v;
      if (v > mt[h]) { zt[h] = zt[h] * exp2f((mt[h] - v) * esc[h]) + 1.0f; mt[h] = v; }
      else zt[h] += exp2f((v - mt[h]) * esc[h]);
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float m = mt[h], z = zt[h];
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const float m_o = __shfl_xor(m, o), z_o = __shfl_xor(z, o);
      const float m_new = fmaxf(m, m_o);
      z = (m == -INFINITY ? 0.0f : z * exp2f((m - m_new) * esc[h])) + (m_o == -INFINITY ? 0.0f : z_o * exp2f((m_o - m_new) * esc[h]));
      m = m_new;
    }
    if (lane == 0) { stat[(wave * G + h) * 2] = m; stat[(wave * G + h) * 2 + 1] = z; }
  }
  __syncthreads();
  if (tid < G) {
    const int h = tid;
    float e_h = esc[0];
#pragma unroll
    for (int t = 1; t < G; ++t) if (t == h) e_h = esc[t];
    float m = -INFINITY;
    for (int w = 0; w < NW; ++w) m = fmaxf(m, stat[(w * G + h) * 2]);
    float z = 0.0f;
    for (int w = 0; w < NW; ++w) {
      const float mw = stat[(w * G + h) * 2];
      if (mw != -INFINITY) z += stat[(w * G + h) * 2 + 1] * exp2f((mw - m) * e_h);
    }
    stat_out[h * 2] = m; stat_out[h * 2 + 1] = z;
  }
}

template <int G>
__global__ __launch_bounds__(NT, 2) void gs_select(const GsArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const DecodeArgs& d = a.d;
  uint32_t* keys = smem;                                          // [span2]
  uint32_t* hist = keys + a.span2;                                // [2][kRadixBins]
  float* red = reinterpret_cast<float*>(hist + 2 * kRadixBins);   // [32]
  uint32_t* wcnt = reinterpret_cast<uint32_t*>(red + 32);         // [16]
  int* ctl = reinterpret_cast<int*>(wcnt + 16);                   // [8]
  float* hs = reinterpret_cast<float*>(ctl + 8);                  // [G][2] max, 1 / sum-exp
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int ukv, s;
  map_kv(d.B * d.H_kv, a.n2, ukv, s);
  const int b = ukv / d.H_kv, hk = ukv - b * d.H_kv;
  const size_t u0 = (size_t)b * d.H + (size_t)hk * G;
  int S = d.seq_lens[b];
  S = S < 0 ? 0 : (S > d.S_max ? d.S_max : S);
  if (S == 0) return;
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  const Window win = make_window(d.local_window, S, kq);
  const size_t slot = (size_t)ukv * a.n2 + s;
  const int p0 = s * a.span2;
  if (p0 >= S) {
    if (tid == 0) a.cnt_ws[slot] = 0;
    return;
  }
  const int len = S - p0 < a.span2 ? S - p0 : a.span2;

  for (int i = tid; i < 2 * kRadixBins; i += NT) hist[i] = 0u;
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
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (c * 8 + e < len) {
        float dv[G];
#pragma unroll
        for (int h = 0; h < G; ++h) dv[h] = e < 4 ? (&lo[h].x)[e] : (&hi[h].x)[e - 4];
        kx[e] = float_to_key(group_score<G>(dv, mh, esc, inv_z));
        if (p0 + c * 8 + e < win.S_old) atomicAdd(&hist[hist_slot(kx[e] >> 21)], 1u);
      } else {
        kx[e] = 0u;
      }
    }
    uint4* dst = reinterpret_cast<uint4*>(keys + c * 8);
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  }
  __syncthreads();
  int n_old = win.S_old - p0;
  n_old = n_old < 0 ? 0 : (n_old > len ? len : n_old);
  const int k_old = win.k_old < n_old ? win.k_old : n_old;
  const SelectLds sel{hist, wcnt, ctl, red};
  uint32_t pmask, pval;
  int need;
  radix_select(keys, n_old, k_old, sel, tid, lane, wave, pmask, pval, need);
  compact_selected<false>(keys, reinterpret_cast<uint32_t*>(a.cand_pos_ws) + slot * a.cand_cap, len, n_old, pmask, pval, need,
                          0.0f, 0.0f, nullptr, 0, sel, tid, lane, wave, a.cand_key_ws + slot * a.cand_cap, p0);
  if (tid == 0) a.cnt_ws[slot] = k_old + (len - n_old);
}

template <int G>
__global__ __launch_bounds__(NT) void gs_merge(const GsArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const DecodeArgs& d = a.d;
  const int cap_all = a.n2 * a.cand_cap;
  uint32_t* keys = smem;                                          // [round_up(cap_all, 8)]
  uint32_t* hist = keys + ((cap_all + 7) & ~7);                   // [2][kRadixBins]
  float* red = reinterpret_cast<float*>(hist + 2 * kRadixBins);   // [32]
  uint32_t* wcnt = reinterpret_cast<uint32_t*>(red + 32);         // [16]
  int* ctl = reinterpret_cast<int*>(wcnt + 16);                   // [8]
  int* off = ctl + 8;                                             // [kMaxSpans + 1]
  float* hs = reinterpret_cast<float*>(off + kMaxSpans + 8);      // [G][2]
  float* asum_w = hs + 2 * G;                                     // [NW][G]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ukv = blockIdx.x, b = ukv / d.H_kv, hk = ukv - b * d.H_kv;
  const size_t u0 = (size_t)b * d.H + (size_t)hk * G;
  int S = d.seq_lens[b];
  S = S < 0 ? 0 : (S > d.S_max ? d.S_max : S);
  if (S == 0) return;
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  const Window win = make_window(d.local_window, S, kq);

  for (int i = tid; i < 2 * kRadixBins; i += NT) hist[i] = 0u;
  if (wave == 0) {
    const int cnt = lane < a.n2 ? a.cnt_ws[(size_t)ukv * a.n2 + lane] : 0;
    const uint32_t incl = wave_scan_incl((uint32_t)cnt);
    off[lane + 1] = (int)incl;
    if (lane == 0) off[0] = 0;
    combine_span_stats<G>(a.stat_ws + (size_t)ukv * a.n1 * G * 2, a.n1, a.esc_ws + u0, lane, hs);
  }
  __syncthreads();
  const int n_cand = off[a.n2];
  const int n_free = n_cand - win.n_local;        // candidates that compete; the window's come last
  for (int s = 0; s < a.n2; ++s) {
    const int o = off[s], cnt = off[s + 1] - o;
    const uint32_t* src = a.cand_key_ws + ((size_t)ukv * a.n2 + s) * a.cand_cap;
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
  compact_selected<false>(keys, keys, n_cand, n_free, pmask, pval, need, 0.0f, 0.0f, nullptr, 0, sel, tid, lane, wave);

  // candidate numbers -> positions; alpha_h = sum over the selected positions of s-hat_h from the stored logits
  float mh[G], inv_z[G], esc[G], asum[G];
#pragma unroll
  for (int h = 0; h < G; ++h) { mh[h] = hs[h * 2]; inv_z[h] = hs[h * 2 + 1]; esc[h] = a.esc_ws[u0 + h]; asum[h] = 0.0f; }
  const float* z_unit = a.z_ws + u0 * (size_t)d.S_max;
  int32_t* list = a.list_ws + (size_t)ukv * a.list_stride;
  for (int nb = 0; nb < kq; nb += 4 * NT) {      // four entries per thread at a time: loads of one kind together
    int pos[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int n = nb + t * NT + tid;
      pos[t] = -1;
      if (n < kq) {
        const int ci = (int)keys[n];
        int s = 0;
        while (s + 1 < a.n2 && off[s + 1] <= ci) ++s;
        pos[t] = a.cand_pos_ws[((size_t)ukv * a.n2 + s) * a.cand_cap + (ci - off[s])];
      }
    }
    float zv[4][G];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int h = 0; h < G; ++h) zv[t][h] = pos[t] >= 0 ? z_unit[(size_t)h * d.S_max + pos[t]] : -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int n = nb + t * NT + tid;
      if (pos[t] >= 0) {
        list[n] = pos[t];
        if (d.idx_out && n < d.idx_stride) {
#pragma unroll
          for (int h = 0; h < G; ++h) d.idx_out[(u0 + h) * d.idx_stride + n] = pos[t];
        }
#pragma unroll
        for (int h = 0; h < G; ++h) asum[h] += exp2f((zv[t][h] - mh[h]) * esc[h]);
      }
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float w = wave_sum(asum[h]);
    if (lane == 0) asum_w[wave * G + h] = w;
  }
  __syncthreads();
  if (tid < G) {
    float t = 0.0f;
    for (int w = 0; w < NW; ++w) t += asum_w[w * G + tid];
    const float alpha = t * hs[tid * 2 + 1];
    a.alpha_ws[u0 + tid] = alpha;
    if (d.alpha_out) d.alpha_out[u0 + tid] = alpha;
  }
  if (d.idx_out) {
    if (tid == 0 && kq > d.idx_stride) atomicOr(d.err, 4);
    for (int i = tid; i < G * d.idx_stride; i += NT) {
      const int h = i / d.idx_stride, n = i - h * d.idx_stride;
      if (n >= kq) d.idx_out[(u0 + h) * d.idx_stride + n] = -1;
    }
  }
}

template <class T, int DH, int G>
__global__ __launch_bounds__(NT, 2) void gs_gather(const GsArgs a) {
  __shared__ float part[NW * G * (DH + 2)];
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int ukv, s;
  map_kv(d.B * d.H_kv, a.n_split, ukv, s);
  const int b = ukv / d.H_kv, hk = ukv - b * d.H_kv;
  const size_t u0 = (size_t)b * d.H + (size_t)hk * G;
  const size_t kv_head = (size_t)ukv;
  int S = d.seq_lens[b];
  S = S < 0 ? 0 : (S > d.S_max ? d.S_max : S);
  if (S == 0) return;
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  const int per = (kq + a.n_split - 1) / a.n_split;
  const int n0 = s * per < kq ? s * per : kq;
  const int n1 = n0 + per < kq ? n0 + per : kq;

  using Geo = RowGeometry<DH>;
  constexpr int UNR = 2, GROUP = Geo::RPI * UNR;
  const int sub = lane % Geo::LPR, slot = wave * Geo::RPW + lane / Geo::LPR;
  const int* list = a.list_ws + (size_t)ukv * a.list_stride;
  const char* K_head = reinterpret_cast<const char*>(d.K) + kv_head * d.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(d.V) + kv_head * d.S_stride * (size_t)(DH * 2) + sub * 16;
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[G][8], m_run[G], l_run[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float f[8];
    unpack8<T>(load16(reinterpret_cast<const uint16_t*>(d.q) + (u0 + h) * DH + sub * 8), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) { q8[h][e] = f[e] * qscale; acc[h][e] = 0.0f; }
    m_run[h] = -INFINITY; l_run[h] = 0.0f;
  }
  const int n_groups = (n1 - n0 + GROUP - 1) / GROUP;
  auto issue = [&](uint4 (&kr)[UNR], uint4 (&vr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int n = n0 + g * GROUP + t * Geo::RPI + slot;
      const uint32_t off = (uint32_t)list[n < n1 ? n : n1 - 1] * (uint32_t)(DH * 2);
      kr[t] = load16(K_head + off);
      vr[t] = load16(V_head + off);
    }
  };
  auto consume = [&](const uint4 (&kr)[UNR], const uint4 (&vr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const bool ok = n0 + g * GROUP + t * Geo::RPI + slot < n1;
      float kf[8], vf[8];
      unpack8<T>(kr[t], kf);
      unpack8<T>(vr[t], vf);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf(kf[e], q8[h][e], dot);
        dot = lanes_sum<Geo::LPR>(dot);
        if (ok) {
          const float m_new = fmaxf(m_run[h], dot);
          const float sc = exp2f(m_run[h] - m_new), pr = exp2f(dot - m_new);
          l_run[h] = l_run[h] * sc + pr;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[h][e] = acc[h][e] * sc + pr * vf[e];
          m_run[h] = m_new;
        }
      }
    }
  };
  if (n_groups > 0) {
    uint4 ka[UNR], va[UNR], kb2[UNR], vb2[UNR];
    issue(ka, va, 0);
    int g = 0;
    for (; g + 2 < n_groups; g += 2) {
      issue(kb2, vb2, g + 1);
      consume(ka, va, g);
      issue(ka, va, g + 2);
      consume(kb2, vb2, g + 1);
    }
    if (g + 1 < n_groups) {
      issue(kb2, vb2, g + 1);
      consume(ka, va, g);
      consume(kb2, vb2, g + 1);
    } else {
      consume(ka, va, g);
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h)
    store_wave_partial<DH>(m_run[h], l_run[h], acc[h], part + h * (DH + 2), lane, wave * G);   // part[wave][h]
  __syncthreads();
  for (int i = tid; i < G * DH; i += NT) {
    const int h = i / DH, c = i - h * DH;
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) m_all = fmaxf(m_all, part[(w * G + h) * (DH + 2) + DH]);
    float l_all = 0.0f, y = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float sw = weight_exp2(part[(w * G + h) * (DH + 2) + DH], m_all);
      l_all += part[(w * G + h) * (DH + 2) + DH + 1] * sw;
      y += part[(w * G + h) * (DH + 2) + c] * sw;
    }
    float* mine = a.part_ws + ((u0 + h) * a.n_split + s) * (DH + 2);
    mine[c] = y;
    if (c == 0) { mine[DH] = m_all; mine[DH + 1] = l_all; }
  }
}

// gs_logits with the dynamic LDS its thread groups' partial sums need (on top of ~9 KB of static arrays)
template <class T, int DH, int G>
hipError_t launch_logits(const GsArgs& a, hipStream_t s) {
  const int F = logit_row_groups(a.span1, (a.d.r + 7) >> 3);
  const size_t lds = F > 1 ? (size_t)F * G * a.span1 * sizeof(float) : 0;
  hipError_t e = allow_lds<gs_logits<T, DH, G>>(lds + 16 * 1024, 128 * 1024);   // at most 64 KiB dynamic on top of the static arrays
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gs_logits<T, DH, G>), dim3(a.d.B * a.d.H_kv * a.n1), dim3(NT), lds, s, a);
  return hipGetLastError();
}

template <class T, int DH, int G>
hipError_t launch_gs(const GsArgs& a, int dtype, hipStream_t s) {
  const int Ukv = a.d.B * a.d.H_kv;
  const size_t lds2 = gs_select_lds_bytes(a.span2), lds3 = gs_merge_lds_bytes(a.n2, a.cand_cap);
  hipError_t e;
  if ((e = allow_lds<gs_select<G>>(lds2)) != hipSuccess) return e;
  if ((e = allow_lds<gs_merge<G>>(lds3)) != hipSuccess) return e;
  if ((e = launch_logits<T, DH, G>(a, s)) != hipSuccess) return e;
  hipLaunchKernelGGL(gs_select<G>, dim3(Ukv * a.n2), dim3(NT), lds2, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(gs_merge<G>, dim3(Ukv), dim3(NT), lds3, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((gs_gather<T, DH, G>), dim3(Ukv * a.n_split), dim3(NT), 0, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  SplitArgs c;
  c.d = a.d; c.n_split = a.n_split;
  c.alpha_ws = a.alpha_ws; c.list_ws = nullptr;
  c.part_ws = a.part_ws;
  return launch_split_combine(c, dtype, s);
}

template <class T, int DH>
hipError_t launch_gs_dh(const GsArgs& a, int dtype, hipStream_t s) {
  switch (a.d.H / a.d.H_kv) {
    case 2: return launch_gs<T, DH, 2>(a, dtype, s);
    case 4: return launch_gs<T, DH, 4>(a, dtype, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

size_t gs_select_lds_bytes(int span2) { return 4 * ((size_t)span2 + 2 * kRadixBins + 32 + 16 + 8 + 8); }

size_t gs_merge_lds_bytes(int n2, int cand_cap) {
  return 4 * ((((size_t)n2 * cand_cap + 7) & ~(size_t)7) + 2 * kRadixBins + 32 + 16 + 8 + kMaxSpans + 8 + 8 + NW * 4);
}

namespace {
template <class T, int DH>
hipError_t launch_logits_dh(const GsArgs& a, hipStream_t s) {
  switch (a.d.H / a.d.H_kv) {
    case 2: return launch_logits<T, DH, 2>(a, s);
    case 4: return launch_logits<T, DH, 4>(a, s);
    default: return hipErrorInvalidValue;
  }
}
}  // namespace

hipError_t launch_group_logits(const GsArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_logits_dh<BF16, 64>(a, s) : launch_logits_dh<F16, 64>(a, s);
    case 128: return bf ? launch_logits_dh<BF16, 128>(a, s) : launch_logits_dh<F16, 128>(a, s);
    case 256: return bf ? launch_logits_dh<BF16, 256>(a, s) : launch_logits_dh<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

hipError_t launch_decode_shared_split(const GsArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_gs_dh<BF16, 64>(a, dtype, s) : launch_gs_dh<F16, 64>(a, dtype, s);
    case 128: return bf ? launch_gs_dh<BF16, 128>(a, dtype, s) : launch_gs_dh<F16, 128>(a, dtype, s);
    case 256: return bf ? launch_gs_dh<BF16, 256>(a, dtype, s) : launch_gs_dh<F16, 256>(a, dtype, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
