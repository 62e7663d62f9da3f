// Dense single-query attention (Section 3, Eq. 2): the in-library comparison for SparQ.
// Split along the sequence: each workgroup streams a run of K and V rows of one KV head once
// for G query heads of its group (online softmax, fp32), writes (acc, m, l) partials; a second
// kernel merges the partials of each query head.
#include "common.h"
#include "params.h"

namespace sparq {

namespace {

constexpr int DT = 256;            // threads per workgroup
constexpr int DW = DT / kWave;

template <class T, int DH, int G>
__global__ __launch_bounds__(DT) void dense_partial(const DenseArgs a) {
  constexpr int LPR = DH / 8, RPW = kWave / LPR, RPI = DW * RPW, UNR = 4;
  __shared__ float part[DW][G][DH + 2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = a.H / a.H_kv, gpk = g / G;       // query-head bundles per KV head
  int x = blockIdx.x;
  const int split = x % a.n_split; x /= a.n_split;
  const int bundle = x % gpk; x /= gpk;
  const int hk = x % a.H_kv, b = x / a.H_kv;
  const int h0 = hk * g + bundle * G;            // first query head served here
  int S = a.seq_lens[b];
  S = S < 0 ? 0 : (S > a.S_max ? a.S_max : S);
  const int s0 = split * a.rows_per_split;
  const int s1 = (s0 + a.rows_per_split) < S ? (s0 + a.rows_per_split) : S;

  const int sub = lane % LPR, slot = wave * RPW + lane / LPR;
  const size_t kv_head = (size_t)b * a.H_kv + hk;
  const char* K_head = reinterpret_cast<const char*>(a.K) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(a.V) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + ((size_t)b * a.H + h0) * DH + sub * 8;
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[G][8], acc[G][8], m_run[G], l_run[G];
#pragma unroll
  for (int t = 0; t < G; ++t) {
    float f[8];
    unpack8<T>(load16(qp + (size_t)t * DH), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) { q8[t][e] = f[e] * qscale; acc[t][e] = 0.0f; }
    m_run[t] = -INFINITY; l_run[t] = 0.0f;
  }

  for (int n0 = s0; n0 < s1; n0 += RPI * UNR) {
    uint4 kr[UNR], vr[UNR];
    bool ok[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int n = n0 + u * RPI + slot;
      ok[u] = n < s1;
      const size_t off = (size_t)(ok[u] ? n : s0) * (size_t)(DH * 2);
      kr[u] = load16(K_head + off);
      vr[u] = load16(V_head + off);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      float kf[8], vf[8];
      unpack8<T>(kr[u], kf);
      unpack8<T>(vr[u], vf);
#pragma unroll
      for (int t = 0; t < G; ++t) {
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf(kf[e], q8[t][e], dot);
        dot = lanes_sum<LPR>(dot);
        if (ok[u]) {
          const float m_new = fmaxf(m_run[t], dot);
          const float sc = exp2f(m_run[t] - m_new), pr = exp2f(dot - m_new);
          l_run[t] = l_run[t] * sc + pr;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[t][e] = acc[t][e] * sc + pr * vf[e];
          m_run[t] = m_new;
        }
      }
    }
  }
  // merge the row groups of a wave, then the waves, per query head
#pragma unroll
  for (int t = 0; t < G; ++t) {
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) {
      const float m_o = __shfl_xor(m_run[t], o), l_o = __shfl_xor(l_run[t], o);
      const float m_new = fmaxf(m_run[t], m_o);
      const float s1w = weight_exp2(m_run[t], m_new), s2w = weight_exp2(m_o, m_new);
      l_run[t] = l_run[t] * s1w + l_o * s2w;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[t][e] = acc[t][e] * s1w + __shfl_xor(acc[t][e], o) * s2w;
      m_run[t] = m_new;
    }
    if (lane < LPR) {
#pragma unroll
      for (int e = 0; e < 8; ++e) part[wave][t][sub * 8 + e] = acc[t][e];
      if (lane == 0) { part[wave][t][DH] = m_run[t]; part[wave][t][DH + 1] = l_run[t]; }
    }
  }
  __syncthreads();
  for (int i = tid; i < G * DH; i += DT) {
    const int t = i / DH, c = i - t * DH;
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < DW; ++w) m_all = fmaxf(m_all, part[w][t][DH]);
    float l_all = 0.0f, y = 0.0f;
#pragma unroll
    for (int w = 0; w < DW; ++w) {
      const float s = weight_exp2(part[w][t][DH], m_all);
      l_all += part[w][t][DH + 1] * s;
      y += part[w][t][c] * s;
    }
    float* dst = a.partials + (((size_t)b * a.H + h0 + t) * a.n_split + split) * (DH + 2);
    dst[c] = y;
    if (c == 0) { dst[DH] = m_all; dst[DH + 1] = l_all; }
  }
}

// Merge of the n_split partials of one (sequence, query head).  512 threads = 512 / d_h groups of d_h
// channels; group g folds partials g, g + NG, ... online (four loads in flight per thread), the groups
// are merged through LDS.
constexpr int CT = 512;

template <class T, int DH>
__global__ __launch_bounds__(CT) void dense_combine(const DenseArgs a) {
  constexpr int NG = CT / DH;
  __shared__ float sm[NG * (DH + 2)];
  const int u = blockIdx.x, c = threadIdx.x % DH, grp = threadIdx.x / DH;
  const float* src = a.partials + (size_t)u * a.n_split * (DH + 2);
  float m = -INFINITY, l = 0.0f, y = 0.0f;
  for (int s0 = grp; s0 < a.n_split; s0 += NG * 4) {
    float pm[4], pl[4], py[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int s = s0 + t * NG;
      const bool on = s < a.n_split;
      pm[t] = on ? src[s * (DH + 2) + DH] : -INFINITY;
      pl[t] = on ? src[s * (DH + 2) + DH + 1] : 0.0f;
      py[t] = on ? src[s * (DH + 2) + c] : 0.0f;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float m_new = fmaxf(m, pm[t]);
      const float w_old = weight_exp2(m, m_new), w = weight_exp2(pm[t], m_new);
      l = l * w_old + pl[t] * w;
      y = y * w_old + py[t] * w;
      m = m_new;
    }
  }
  sm[grp * (DH + 2) + c] = y;
  if (c == 0) { sm[grp * (DH + 2) + DH] = m; sm[grp * (DH + 2) + DH + 1] = l; }
  __syncthreads();
  if (grp == 0) {
    float m_all = -INFINITY;
#pragma unroll
    for (int g = 0; g < NG; ++g) m_all = fmaxf(m_all, sm[g * (DH + 2) + DH]);
    float l_all = 0.0f, y_all = 0.0f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const float w = weight_exp2(sm[g * (DH + 2) + DH], m_all);
      l_all += sm[g * (DH + 2) + DH + 1] * w;
      y_all += sm[g * (DH + 2) + c] * w;
    }
    uint16_t* out = reinterpret_cast<uint16_t*>(a.out) + (size_t)u * DH;
    out[c] = l_all > 0.0f ? T::narrow(y_all / l_all) : (uint16_t)0;   // empty sequence: zeros
  }
}

template <class T, int DH, int G>
hipError_t launch_g(const DenseArgs& a, hipStream_t s) {
  const int g = a.H / a.H_kv;
  const int blocks = a.B * a.H_kv * (g / G) * a.n_split;
  hipLaunchKernelGGL((dense_partial<T, DH, G>), dim3(blocks), dim3(DT), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((dense_combine<T, DH>), dim3(a.B * a.H), dim3(CT), 0, s, a);
  return hipGetLastError();
}

template <class T, int DH>
hipError_t launch_dh(const DenseArgs& a, hipStream_t s) {
  const int g = a.H / a.H_kv;
  if (g % 8 == 0 && DH <= 128) return launch_g<T, DH, 8>(a, s);
  if (g % 4 == 0) return launch_g<T, DH, 4>(a, s);
  if (g % 2 == 0) return launch_g<T, DH, 2>(a, s);
  return launch_g<T, DH, 1>(a, s);
}

}  // namespace

hipError_t launch_dense(const DenseArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d_h) {
    case 64:  return bf ? launch_dh<BF16, 64>(a, s) : launch_dh<F16, 64>(a, s);
    case 128: return bf ? launch_dh<BF16, 128>(a, s) : launch_dh<F16, 128>(a, s);
    case 256: return bf ? launch_dh<BF16, 256>(a, s) : launch_dh<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
