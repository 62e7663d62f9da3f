// SparQ decode for few heads and long sequences: the positions of one (sequence, query head) are
// split over several workgroups, so that a batch with fewer heads than compute units still fills
// the machine.  Four launches; data passes between workgroups only across kernel boundaries.
//   split_scores   (units x n_split workgroups) top-r of |q|, temperature, approximate logits of a
//                  slice of positions -> integer keys in the workspace, the slice's largest logit
//   split_select   (one workgroup per unit) keys into LDS, radix select, ordered position list and
//                  alpha to the workspace
//   split_gather   (units x n_split) exact attention over a slice of the position list -> partial
//                  (numerator, max, denominator)
//   split_combine  (one workgroup per unit) merge, blend with the mean value vector (Eq. 10), store
#include "decode_stages.h"

namespace sparq {

namespace {

// workgroup -> (unit, split): the splits of a unit, and the heads of a KV group, share an XCD (an L2)
__device__ __forceinline__ void map_block(int U, int n_split, int& u, int& s) {
  const int bid = blockIdx.x;
  if ((U & 7) == 0) {
    const int x = bid & 7, slot = bid >> 3;
    u = x * (U >> 3) + slot / n_split;
    s = slot % n_split;
  } else {
    u = bid / n_split;
    s = bid % n_split;
  }
}

template <class T, int DH>
__global__ __launch_bounds__(NT, 4) void split_scores(const SplitArgs a) {
  __shared__ __align__(16) uint32_t mag[DH];
  __shared__ int rankp[NT];
  __shared__ float qf[DH], qs[DH], red[NW];
  __shared__ int chan[DH];
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int U = d.B * d.H;
  int u, s;
  map_block(U, a.n_split, u, s);
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
  if (S == 0) {   // nothing cached: split 0 writes the defined outputs, the later launches skip the unit
    if (s == 0) {
      if (tid < DH) reinterpret_cast<uint16_t*>(d.out)[(size_t)u * DH + tid] = 0;
      if (tid == 0) { atomicOr(d.err, 2); if (d.alpha_out) d.alpha_out[u] = 0.0f; }
      if (d.chan_out && tid < d.r) d.chan_out[(size_t)u * d.r + tid] = -1;
      if (idx_out) for (int n = tid; n < d.idx_stride; n += NT) idx_out[n] = -1;
    }
    return;
  }

  const QueryLds Q{mag, rankp, qf, qs, chan};
  const float tau = apply_tau_mode(select_channels<T, DH>(Q, qcode, d.r, tid, lane, wave), d.flags, DH, d.r);
  if (s == 0) {
    if (d.chan_out && tid < d.r) d.chan_out[(size_t)u * d.r + tid] = chan[tid];
    if (tid == 0) a.tau_ws[u] = tau;
  }

  // the newest S mod 8 positions are not in Kt: the last slice takes them from the rows of K
  const int S_fl = S & ~7, n_tail = s == a.n_split - 1 ? S - S_fl : 0, r8 = (d.r + 7) & ~7;
  TailRow tail;
  if (wave < n_tail)
    tail = tail_row_issue(reinterpret_cast<const uint16_t*>(d.K) + (kv_head * d.S_max + S_fl + wave) * (size_t)DH, chan, r8, lane);

  // this workgroup's slice of the whole 8-position chunks
  const int n_chunks = S >> 3;
  const int per = (n_chunks + a.n_split - 1) / a.n_split;
  const int c0 = s * per < n_chunks ? s * per : n_chunks;
  const int c1 = c0 + per < n_chunks ? c0 + per : n_chunks;
  const size_t row_bytes = (size_t)d.S_max * 2;
  const char* Kt_head = reinterpret_cast<const char*>(d.Kt) + kv_head * DH * row_bytes;
  uint32_t* keys = a.keys_ws + (size_t)u * d.S_max;
  float tmax = -INFINITY;
  stream_channel_rows<T>(Kt_head, row_bytes, chan, qs, d.r, c0, c1, tid, [&](int c, const float (&acc)[8]) {
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      tmax = fmaxf(tmax, acc[e]);
      kx[e] = float_to_key(acc[e]);
    }
    uint4* dst = reinterpret_cast<uint4*>(keys + c * 8);
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  });
  if (wave < n_tail) {
    const float dot = tail_row_dot<T>(tail, qs, r8, lane);
    tmax = fmaxf(tmax, dot);
    if (lane == 0) keys[S_fl + wave] = float_to_key(dot);
  }
  tmax = wave_max(tmax);
  if (lane == 0) red[wave] = tmax;
  __syncthreads();
  if (tid == 0) {
    float m = red[0];
    for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);
    a.tmax_ws[(size_t)u * a.n_split + s] = m;
  }
}

// One workgroup per unit: the keys of all slices into LDS (counting the first digit on the way),
// then the same select and compaction as the one-workgroup kernel; the list goes to the workspace.
__global__ __launch_bounds__(NT) void split_select(const SplitArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const DecodeArgs& d = a.d;
  uint32_t* keys = smem;                                  // [S_max]
  uint32_t* hist = keys + d.S_max;                        // [2][kRadixBins]
  float* red = reinterpret_cast<float*>(hist + 2 * kRadixBins);   // [32]
  uint32_t* wcnt = reinterpret_cast<uint32_t*>(red + 32);         // [16]
  int* ctl = reinterpret_cast<int*>(wcnt + 16);                    // [8]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int u = blockIdx.x, b = u / d.H;
  int S = d.seq_lens[b];
  S = S < 0 ? 0 : (S > d.S_max ? d.S_max : S);
  if (S == 0) return;                      // outputs written by split_scores
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;
  int32_t* idx_out = d.idx_out ? d.idx_out + (size_t)u * d.idx_stride : nullptr;
  const Window win = make_window(d.local_window, S, kq);

  for (int i = tid; i < 2 * kRadixBins; i += NT) hist[i] = 0u;
  float dmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxSplit; ++i)
    if (i < a.n_split) dmax = fmaxf(dmax, a.tmax_ws[(size_t)u * a.n_split + i]);
  const float tau = a.tau_ws[u];
  __syncthreads();
  const uint32_t* src = a.keys_ws + (size_t)u * d.S_max;
  const int n_chunks = (S + 7) >> 3;
  // four chunks (eight 16-byte loads) per thread in flight at a time
  for (int c0 = tid; c0 < n_chunks; c0 += 4 * NT) {
    uint4 lo[4], hi[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int c = c0 + t * NT < n_chunks ? c0 + t * NT : c0;
      lo[t] = reinterpret_cast<const uint4*>(src + c * 8)[0];
      hi[t] = reinterpret_cast<const uint4*>(src + c * 8)[1];
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int c = c0 + t * NT;
      if (c < n_chunks) {
        reinterpret_cast<uint4*>(keys + c * 8)[0] = lo[t];
        reinterpret_cast<uint4*>(keys + c * 8)[1] = hi[t];
        const uint32_t kx[8] = {lo[t].x, lo[t].y, lo[t].z, lo[t].w, hi[t].x, hi[t].y, hi[t].z, hi[t].w};
        hist_add_chunk(hist, kx, win.S_old - c * 8);
      }
    }
  }
  __syncthreads();
  const SelectLds sel{hist, wcnt, ctl, red};
  uint32_t pmask, pval;
  int need;
  radix_select(keys, win.S_old, win.k_old, sel, tid, lane, wave, pmask, pval, need);
  uint32_t* list = reinterpret_cast<uint32_t*>(a.list_ws + (size_t)u * d.S_max);
  const float alpha = compact_selected(keys, list, S, win.S_old, pmask, pval, need, dmax, kLog2e / tau, idx_out, d.idx_stride,
                                       sel, tid, lane, wave);
  if (tid == 0) {
    a.alpha_ws[u] = alpha;
    if (d.alpha_out) d.alpha_out[u] = alpha;
    if (idx_out && kq > d.idx_stride) atomicOr(d.err, 4);
  }
  if (idx_out) for (int n = kq + tid; n < d.idx_stride; n += NT) idx_out[n] = -1;
}

template <class T, int DH>
__global__ __launch_bounds__(NT, 4) void split_gather(const SplitArgs a) {
  __shared__ float part[NW * (DH + 2)];
  const DecodeArgs& d = a.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int U = d.B * d.H;
  int u, s;
  map_block(U, a.n_split, u, s);
  const int b = u / d.H, h = u - b * d.H;
  const size_t kv_head = (size_t)b * d.H_kv + h / (d.H / d.H_kv);
  int S = d.seq_lens[b];
  S = S < 0 ? 0 : (S > d.S_max ? d.S_max : S);
  if (S == 0) return;                      // outputs written by the first launch
  int kb = d.k_per_seq ? d.k_per_seq[b] : d.k;
  kb = kb < 1 ? 1 : (kb > d.k ? d.k : kb);
  const int kq = kb < S ? kb : S;

  using G = RowGeometry<DH>;
  const int sub = lane % G::LPR;
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[8];
  {
    float f[8];
    unpack8<T>(load16(reinterpret_cast<const uint16_t*>(d.q) + (size_t)u * DH + sub * 8), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) q8[e] = f[e] * qscale;
  }
  const int per = (kq + a.n_split - 1) / a.n_split;
  const int n0 = s * per < kq ? s * per : kq;
  const int n1 = n0 + per < kq ? n0 + per : kq;
  const char* K_head = reinterpret_cast<const char*>(d.K) + kv_head * d.S_max * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(d.V) + kv_head * d.S_max * (size_t)(DH * 2) + sub * 16;
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  attend_rows<T, DH>(K_head, V_head, a.list_ws + (size_t)u * d.S_max, n0, n1, q8, lane, wave, m_run, l_run, acc);
  store_wave_partial<DH>(m_run, l_run, acc, part, lane, wave);
  __syncthreads();
  float* mine = a.part_ws + ((size_t)u * a.n_split + s) * (DH + 2);
  if (tid < DH) {
    float m_all, l_all, y;
    combine_partials<DH>(part, NW, tid, m_all, l_all, y);
    mine[tid] = y;
    if (tid == 0) { mine[DH] = m_all; mine[DH + 1] = l_all; }
  }

}

template <class T, int DH>
__global__ __launch_bounds__(DH) void split_combine(const SplitArgs a) {
  const DecodeArgs& d = a.d;
  const int u = blockIdx.x, c = threadIdx.x;
  const int b = u / d.H, h = u - b * d.H;
  const size_t kv_head = (size_t)b * d.H_kv + h / (d.H / d.H_kv);
  const int S = d.seq_lens[b];
  if (S <= 0) return;                      // outputs written by split_scores
  // all partials of this channel in flight at once (n_split <= kMaxSplit)
  const float* parts = a.part_ws + (size_t)u * a.n_split * (DH + 2);
  float pm[kMaxSplit], pl[kMaxSplit], py[kMaxSplit];
#pragma unroll
  for (int w = 0; w < kMaxSplit; ++w) {
    const bool on = w < a.n_split;
    pm[w] = on ? parts[w * (DH + 2) + DH] : -INFINITY;
    pl[w] = on ? parts[w * (DH + 2) + DH + 1] : 0.0f;
    py[w] = on ? parts[w * (DH + 2) + c] : 0.0f;
  }
  const float alpha = a.alpha_ws[u];
  const float vm = d.v_mean[kv_head * DH + c];
  float m_all = -INFINITY;
#pragma unroll
  for (int w = 0; w < kMaxSplit; ++w) m_all = fmaxf(m_all, pm[w]);
  float l_all = 0.0f, y3 = 0.0f;
#pragma unroll
  for (int w = 0; w < kMaxSplit; ++w) {
    const float sw = weight_exp2(pm[w], m_all);
    l_all += pl[w] * sw;
    y3 += py[w] * sw;
  }
  y3 /= l_all;
  float y = y3;
  if (!(d.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * vm;
  reinterpret_cast<uint16_t*>(d.out)[(size_t)u * DH + c] = T::narrow(y);
}

template <class T, int DH>
hipError_t launch_pair(const SplitArgs& a, hipStream_t s) {
  const int units = a.d.B * a.d.H;
  const dim3 grid(units * a.n_split);
  const size_t lds = split_select_lds_bytes(a.d.S_max);
  hipError_t e = allow_lds<split_select>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((split_scores<T, DH>), grid, dim3(NT), 0, s, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(split_select, dim3(units), dim3(NT), lds, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((split_gather<T, DH>), grid, dim3(NT), 0, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((split_combine<T, DH>), dim3(units), dim3(DH), 0, s, a);
  return hipGetLastError();
}

template <class T, int DH>
hipError_t launch_tail(const SplitArgs& a, hipStream_t s) {
  const int units = a.d.B * a.d.H;
  hipLaunchKernelGGL((split_gather<T, DH>), dim3(units * a.n_split), dim3(NT), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((split_combine<T, DH>), dim3(units), dim3(DH), 0, s, a);
  return hipGetLastError();
}

}  // namespace

template <class T, int DH>
hipError_t launch_combine_only(const SplitArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((split_combine<T, DH>), dim3(a.d.B * a.d.H), dim3(DH), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_split_combine(const SplitArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_combine_only<BF16, 64>(a, s) : launch_combine_only<F16, 64>(a, s);
    case 128: return bf ? launch_combine_only<BF16, 128>(a, s) : launch_combine_only<F16, 128>(a, s);
    case 256: return bf ? launch_combine_only<BF16, 256>(a, s) : launch_combine_only<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

hipError_t launch_split_gather(const SplitArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_tail<BF16, 64>(a, s) : launch_tail<F16, 64>(a, s);
    case 128: return bf ? launch_tail<BF16, 128>(a, s) : launch_tail<F16, 128>(a, s);
    case 256: return bf ? launch_tail<BF16, 256>(a, s) : launch_tail<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

size_t split_select_lds_bytes(int S_max) { return 4 * ((size_t)S_max + 2 * kRadixBins + 32 + 16 + 8); }

hipError_t launch_decode_split(const SplitArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d.d_h) {
    case 64:  return bf ? launch_pair<BF16, 64>(a, s) : launch_pair<F16, 64>(a, s);
    case 128: return bf ? launch_pair<BF16, 128>(a, s) : launch_pair<F16, 128>(a, s);
    case 256: return bf ? launch_pair<BF16, 256>(a, s) : launch_pair<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
