// The last two launches of the multi-launch decode plans (two-level selection, grouped-query rule over several
// workgroups): exact attention over slices of a unit's position list, then the merge.
//   split_gather   (units x n_split workgroups) Step 2b over a slice of the position list -> partial
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
  const char* K_head = reinterpret_cast<const char*>(d.K) + kv_head * d.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(d.V) + kv_head * d.S_stride * (size_t)(DH * 2) + sub * 16;
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
  if (S <= 0) return;                      // outputs written by the plan's first launch
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

}  // namespace sparq
