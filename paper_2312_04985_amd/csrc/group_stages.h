// Stages of the grouped-query rule (Section 4, "Grouped query attention"; Appendix B) that several kernels
// share: the channel selection from the group sum of |q| with the per-head temperatures, and Step 1b for G
// query heads at once.
#pragma once
#include "decode_stages.h"

namespace sparq {

// The group score of a position is sum_h s-hat_h = sum_h exp2((d_h - max_h) esc_h) / Z_h.  Only its order
// matters (alpha is summed from the logits), so the key is formed from log2 of it, as
// max_h x_h + log2(sum_h exp2(x_h - max_h x_h)) with x_h = (d_h - max_h) esc_h - log2 Z_h.  The plain sum
// underflows to 0 for every position far below all heads' maxima: thousands of exactly equal keys, which the
// fp64 definition does not have, and which serialise the histogram atomics of the select (6 us per pass over
// 8192 keys instead of 1).  The logarithm keeps them apart at the same relative accuracy (the rounding of x_h
// dominates either way).  inv_z = 1 / Z_h as the callers hold it.
template <int G>
__device__ __forceinline__ float group_score(const float (&d)[G], const float (&mh)[G], const float (&esc)[G],
                                             const float (&inv_z)[G]) {
  float x[G], mx = -INFINITY;
#pragma unroll
  for (int h = 0; h < G; ++h) { x[h] = (d[h] - mh[h]) * esc[h] + log2f(inv_z[h]); mx = fmaxf(mx, x[h]); }
  float s = 0.0f;
#pragma unroll
  for (int h = 0; h < G; ++h) s += exp2f(x[h] - mx);
  return mx + log2f(s);
}

// Per-head softmax statistics of a whole sequence from the n1 span partials {max, sum-exp relative to it}:
// executed by wave 0 (one lane per span, n1 <= 64); results to out[h] = {max, 1 / sum-exp}.
template <int G>
__device__ __forceinline__ void combine_span_stats(const float* stat_unit, int n1, const float* esc_unit, int lane, float* out) {
  const bool on = lane < n1;
  float m[G], z[G], esc[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {      // all loads first: one round trip
    m[h] = on ? stat_unit[(lane * G + h) * 2] : -INFINITY;
    z[h] = on ? stat_unit[(lane * G + h) * 2 + 1] : 0.0f;
    esc[h] = esc_unit[h];
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float m_all = wave_max(m[h]);
    const float z_all = wave_sum(m[h] == -INFINITY ? 0.0f : z[h] * exp2f((m[h] - m_all) * esc[h]));
    if (lane == 0) { out[h * 2] = m_all; out[h * 2 + 1] = 1.0f / z_all; }
  }
}

struct GroupQueryLds {
  int* rankp;      // [NT] partial ranks
  float* qf;       // [G][DH] the group's queries as fp32
  float* qs;       // [G][DH] per-head components on the shared channel list (padded to a multiple of 8, weight 0)
  int* chan;       // [DH] shared channel list, ascending, same padding
  double* magd;    // [DH] group sums of |q|
};

// Step 1a under the group rule: channel j is ranked by sum_h |q_h,j| (fp64, heads in order, ties to the lower
// channel); esc[h] = log2(e) / tau_h with tau_h from Eq. (9) on the shared channel set (or the fixed
// temperature the flags ask for).  q_group: the G x DH query codes of the group.  Four barriers; the first also
// publishes whatever the caller wrote to LDS before the call.
template <class T, int DH, int G>
__device__ __forceinline__ void select_channels_group(const GroupQueryLds& Q, const uint16_t* q_group, int r, uint32_t flags,
                                                      int tid, int lane, int wave, float (&esc)[G]) {
  for (int i = tid; i < G * DH; i += NT)
    Q.qf[i] = T::widen(q_group[i]);
  __syncthreads();
  if (tid < DH) {
    double m = 0.0;
#pragma unroll
    for (int h = 0; h < G; ++h) m += (double)fabsf(Q.qf[h * DH + tid]);   // head order, as in the definition
    Q.magd[tid] = m;
  }
  __syncthreads();
  {
    constexpr int SL = NT / DH, PER = DH / SL;
    const int j = tid % DH, slice = tid / DH;
    const double mine = Q.magd[j];
    int partial = 0;
#pragma unroll 4
    for (int i = slice * PER; i < (slice + 1) * PER; ++i) {
      const double m = Q.magd[i];
      partial += (m > mine) || (m == mine && i < j);
    }
    Q.rankp[slice * DH + j] = partial;
  }
  __syncthreads();
  {
    constexpr int SL = NT / DH, NG = DH / kWave;
    const int r8 = (r + 7) & ~7;
    int before = 0;
    float l1a[G], l1s[G];
#pragma unroll
    for (int h = 0; h < G; ++h) { l1a[h] = 0.0f; l1s[h] = 0.0f; }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int jj = g * kWave + lane;
      int rank = 0;
#pragma unroll
      for (int s = 0; s < SL; ++s) rank += Q.rankp[s * DH + jj];
      const bool sel = rank < r;
      const uint64_t bal = __ballot(sel);
      if (g == wave) {
        if (sel) {
          const int p = before + __popcll(bal & ((1ull << lane) - 1ull));
          Q.chan[p] = jj;
#pragma unroll
          for (int h = 0; h < G; ++h) Q.qs[h * DH + p] = Q.qf[h * DH + jj];
          if (p == r - 1)
            for (int pp = r; pp < r8; ++pp) {
              Q.chan[pp] = jj;
#pragma unroll
              for (int h = 0; h < G; ++h) Q.qs[h * DH + pp] = 0.0f;
            }
        }
      }
      before += __popcll(bal);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float aq = fabsf(Q.qf[h * DH + jj]);
        l1a[h] += aq; l1s[h] += sel ? aq : 0.0f;
      }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float all = wave_sum(l1a[h]), part = wave_sum(l1s[h]);
      const float tau = part > 0.0f ? sqrtf((float)DH * part / all) : sqrtf((float)DH);   // all logits 0 then
      esc[h] = kLog2e / apply_tau_mode(tau, flags, DH, r);
    }
  }
  __syncthreads();
}

// Step 1b for G heads at once: like stream_channel_rows, every loaded 16-byte chunk feeds G accumulators.
// Thread tid of STRIDE owns chunks chunk_begin + tid + i * STRIDE (STRIDE < NT: the caller divides the channel
// rows of a chunk among NT / STRIDE groups of threads).
template <class T, int G, int STRIDE = NT, class Finish>
__device__ __forceinline__ void stream_channel_rows_group(const char* Kt_head, size_t row_bytes, const int* chan,
                                                          const float* qs, int qs_stride, int r, int chunk_begin,
                                                          int chunk_end, int tid, Finish&& finish) {
  const int n_batches = (r + 7) >> 3;
  const int n_chunks = chunk_end - chunk_begin;
  const int my_chunks = n_chunks > tid ? (n_chunks - tid + STRIDE - 1) / STRIDE : 0;
  const int items = my_chunks * n_batches;
  float acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;
  int ic = 0, ib = 0, cc = 0, cb = 0;
  auto issue_next = [&](uint4 (&v)[8]) {
    const uint32_t voff = (uint32_t)(chunk_begin + tid + ic * STRIDE) * 16u;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int ch = __builtin_amdgcn_readfirstlane(chan[ib * 8 + t]);
      v[t] = load16(Kt_head + (size_t)ch * row_bytes + voff);
    }
    if (++ib == n_batches) { ib = 0; ++ic; }
  };
  auto consume_next = [&](const uint4 (&v)[8]) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float f[8];
      unpack8<T>(v[t], f);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float qv = qs[h * qs_stride + cb * 8 + t];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(f[e], qv, acc[h][e]);
      }
    }
    if (++cb == n_batches) {
      finish(chunk_begin + tid + cc * STRIDE, acc);
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;
      cb = 0; ++cc;
    }
  };
  uint4 va[8], vb[8];
  if (items > 0) {
    issue_next(va);
    int i = 0;
    for (; i + 2 < items; i += 2) {
      issue_next(vb);
      consume_next(va);
      issue_next(va);
      consume_next(vb);
    }
    if (i + 1 < items) {
      issue_next(vb);
      consume_next(va);
      consume_next(vb);
    } else {
      consume_next(va);
    }
  }
}

}  // namespace sparq
