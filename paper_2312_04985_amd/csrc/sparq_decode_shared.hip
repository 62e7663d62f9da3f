// SparQ decode with the paper's grouped-query rule (Section 4, "Grouped query attention";
// Appendix B): the G query heads that share a KV head select ONE channel set from the group sum of
// |q| and ONE position set from the group sum of their approximate scores s-hat; the temperature,
// alpha and the exact attention stay per query head.  One workgroup per (sequence, KV head).
//   stage 0  group sums of |q| in fp64 (head order, as the definition is written), top-r, per-head tau
//   pass A   stream the r channel rows once for all G heads: the G logit numerators of every position go to
//            the workspace (fp32), per-head max and sum-exp stay in registers
//   pass B   read them back: score_i = sum_h softmax_h(z)_i as integer keys in LDS
//   stage 2  radix select of the k largest scores, ordered position list
//   stage 3  gather each selected K and V row once for the G heads: exact attention per head; per-head
//            alpha from the stored logits of the selected positions
//   blend    y_h = alpha_h y3_h + (1 - alpha_h) v_mean (Eq. 10), round and store
// The group sum of softmaxes is not monotone in any one head's logits, so the logits themselves are needed
// twice (statistics, then scores) and a third time for alpha; G x S floats do not fit in LDS for long
// sequences, so they live in the workspace (16 bytes per position for G = 4, against 2 r bytes for streaming
// the key rows again), written and read by the same workgroup.
#include "group_stages.h"

namespace sparq {

namespace {

template <int DH, int G>
struct SharedLds {
  uint32_t* keys;      // [S_max]
  SelectLds sel;       // hist [2][kRadixBins], wcnt, ctl, red
  float* part;         // [NW][G][DH + 2], aliases hist (+ rankp) after the select
  int* rankp;          // [NT]
  float* qf;           // [G][DH]
  float* qs;           // [G][DH] per-head components on the shared channel list (padded, weight 0)
  int* chan;           // [DH]
  double* magd;        // [DH] group sums of |q|
  float* stat;         // [NW][G][2] and [G][3]
};

template <int DH, int G>
__host__ __device__ constexpr size_t shared_part_words() { return (size_t)NW * G * (DH + 2); }

// words after the key array
template <int DH, int G>
__host__ __device__ constexpr size_t shared_fixed_words() {
  size_t hist_rank = 2 * kRadixBins + NT;
  if (hist_rank < shared_part_words<DH, G>()) hist_rank = shared_part_words<DH, G>();
  return hist_rank + 2 * (size_t)G * DH /* qf, qs */ + DH /* chan */ + 2 * DH /* magd */ + 32 + 16 + 8 + NW * G * 2 + G * 4;
}

template <int DH, int G>
__device__ __forceinline__ SharedLds<DH, G> carve_shared(uint32_t* base, int S_max) {
  SharedLds<DH, G> l;
  l.keys = base; base += S_max;
  size_t hist_rank = 2 * kRadixBins + NT;
  if (hist_rank < shared_part_words<DH, G>()) hist_rank = shared_part_words<DH, G>();
  l.sel.hist = base;
  l.rankp = reinterpret_cast<int*>(base + 2 * kRadixBins);
  l.part = reinterpret_cast<float*>(base);
  base += hist_rank;
  l.magd = reinterpret_cast<double*>(base); base += 2 * DH;      // 8-byte aligned: all sizes before are even
  l.qf = reinterpret_cast<float*>(base); base += G * DH;
  l.qs = reinterpret_cast<float*>(base); base += G * DH;
  l.chan = reinterpret_cast<int*>(base); base += DH;
  l.sel.red = reinterpret_cast<float*>(base); base += 32;
  l.sel.wcnt = base; base += 16;
  l.sel.ctl = reinterpret_cast<int*>(base); base += 8;
  l.stat = reinterpret_cast<float*>(base);
  return l;
}

template <class T, int DH, int G>
__global__ __launch_bounds__(NT, 2) void sparq_decode_shared(const DecodeArgs a, float* __restrict__ z_ws) {
  extern __shared__ __align__(16) uint32_t smem[];
  const SharedLds<DH, G> L = carve_shared<DH, G>(smem, a.S_max);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t kv_head = blockIdx.x;                 // (b, hk)
  const int b = (int)(kv_head / a.H_kv), hk = (int)(kv_head - (size_t)b * a.H_kv);
  const size_t u0 = (size_t)b * a.H + (size_t)hk * G;   // first query head of the group

  int S = a.seq_lens[b];
  if (S < 0 || S > a.S_max) {
    if (tid == 0) atomicOr(a.err, 8);
    S = S < 0 ? 0 : a.S_max;
  }
  int kb = a.k_per_seq ? a.k_per_seq[b] : a.k;
  kb = kb < 1 ? 1 : (kb > a.k ? a.k : kb);
  const int kq = kb < S ? kb : S;
  uint16_t* out = reinterpret_cast<uint16_t*>(a.out) + u0 * DH;
  if (S == 0) {
    for (int i = tid; i < G * DH; i += NT) out[i] = 0;
    if (tid < G) { if (a.alpha_out) a.alpha_out[u0 + tid] = 0.0f; }
    if (tid == 0) atomicOr(a.err, 2);
    if (a.chan_out) for (int i = tid; i < G * a.r; i += NT) a.chan_out[u0 * a.r + i] = -1;
    if (a.idx_out) for (int i = tid; i < G * a.idx_stride; i += NT) a.idx_out[u0 * a.idx_stride + i] = -1;
    return;
  }

  // ---------------- stage 0: shared channel set, per-head temperature ----------------
  for (int i = tid; i < 2 * kRadixBins; i += NT) L.sel.hist[i] = 0u;
  float esc[G];        // log2(e) / tau_h
  const GroupQueryLds GQ{L.rankp, L.qf, L.qs, L.chan, L.magd};
  select_channels_group<T, DH, G>(GQ, reinterpret_cast<const uint16_t*>(a.q) + u0 * DH, a.r, a.flags, tid, lane, wave, esc);
  if (a.chan_out)
    for (int i = tid; i < G * a.r; i += NT) a.chan_out[u0 * a.r + i] = L.chan[i % a.r];

  const Window win = make_window(a.local_window, S, kq);

  // ---------------- pass A: per-head max and sum-exp of the approximate logits ----------------
  const size_t row_bytes = (size_t)a.S_stride * 2;
  const char* Kt_head = reinterpret_cast<const char*>(a.Kt) + kv_head * DH * row_bytes;
  const int n_chunks = S >> 3;   // whole chunks; the newest S mod 8 positions are not in Kt yet
  const int S_fl = S & ~7, n_tail = S - S_fl, r8 = (a.r + 7) & ~7;
  float tdot[G];          // wave w: the logit numerators of position S_fl + w for the G heads, from its K row
#pragma unroll
  for (int h = 0; h < G; ++h) tdot[h] = 0.0f;
  if (wave < n_tail) {
    const TailRow tail = tail_row_issue(reinterpret_cast<const uint16_t*>(a.K) + (kv_head * a.S_stride + S_fl + wave) * (size_t)DH,
                                        L.chan, r8, lane);
#pragma unroll
    for (int h = 0; h < G; ++h) tdot[h] = tail_row_dot<T>(tail, L.qs + h * DH, r8, lane);
  }
  float mt[G], zt[G];   // running max of the logit numerator, sum of exp2((d - max) * esc)
#pragma unroll
  for (int h = 0; h < G; ++h) { mt[h] = -INFINITY; zt[h] = 0.0f; }
  float* z_unit = z_ws + u0 * (size_t)a.S_max;        // [G][S_max] logit numerators of this group
  stream_channel_rows_group<T, G>(Kt_head, row_bytes, L.chan, L.qs, DH, a.r, 0, n_chunks, tid,
                                  [&](int c, const float (&acc)[G][8]) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float4* dst = reinterpret_cast<float4*>(z_unit + (size_t)h * a.S_max + c * 8);
      dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
      dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = acc[h][e];
        if (v > mt[h]) { zt[h] = zt[h] * exp2f((mt[h] - v) * esc[h]) + 1.0f; mt[h] = v; }
        else zt[h] += exp2f((v - mt[h]) * esc[h]);
      }
    }
  });
  if (wave < n_tail && lane == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float v = tdot[h];
      z_unit[(size_t)h * a.S_max + S_fl + wave] = v;
      if (v > mt[h]) { zt[h] = zt[h] * exp2f((mt[h] - v) * esc[h]) + 1.0f; mt[h] = v; }
      else zt[h] += exp2f((v - mt[h]) * esc[h]);
    }
  }
  float mh[G], inv_z[G];
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
    if (lane == 0) { L.stat[(wave * G + h) * 2] = m; L.stat[(wave * G + h) * 2 + 1] = z; }
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) m = fmaxf(m, L.stat[(w * G + h) * 2]);
    float z = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float mw = L.stat[(w * G + h) * 2];
      if (mw != -INFINITY) z += L.stat[(w * G + h) * 2 + 1] * exp2f((mw - m) * esc[h]);
    }
    mh[h] = m; inv_z[h] = 1.0f / z;
  }

  // ---------------- pass B: group score = sum over heads of s-hat, as keys ----------------
  // (the barrier above also orders this workgroup's stores of pass A before these loads)
  for (int c = tid; c < n_chunks; c += NT) {
    float4 lo[G], hi[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float4* src = reinterpret_cast<const float4*>(z_unit + (size_t)h * a.S_max + c * 8);
      lo[h] = src[0]; hi[h] = src[1];
    }
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float dv[G];
#pragma unroll
      for (int h = 0; h < G; ++h) dv[h] = e < 4 ? (&lo[h].x)[e] : (&hi[h].x)[e - 4];
      kx[e] = float_to_key(group_score<G>(dv, mh, esc, inv_z));
      if (c * 8 + e < win.S_old) atomicAdd(&L.sel.hist[hist_slot(kx[e] >> 21)], 1u);
    }
    uint4* dst = reinterpret_cast<uint4*>(L.keys + c * 8);
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  }
  if (wave < n_tail && lane == 0) {
    const uint32_t key = float_to_key(group_score<G>(tdot, mh, esc, inv_z));
    L.keys[S_fl + wave] = key;
    if (S_fl + wave < win.S_old) atomicAdd(&L.sel.hist[hist_slot(key >> 21)], 1u);
  }
  __syncthreads();

  // ---------------- stage 2: the kq positions of largest group score ----------------
  uint32_t pmask, pval;
  int need;
  radix_select(L.keys, win.S_old, win.k_old, L.sel, tid, lane, wave, pmask, pval, need);
  int32_t* idx_out = a.idx_out ? a.idx_out + u0 * a.idx_stride : nullptr;
  compact_selected<false>(L.keys, L.keys, S, win.S_old, pmask, pval, need, 0.0f, 0.0f, idx_out, a.idx_stride, L.sel, tid, lane, wave);
  if (idx_out) {
    if (tid == 0 && kq > a.idx_stride) atomicOr(a.err, 4);
    for (int n = kq + tid; n < a.idx_stride; n += NT) idx_out[n] = -1;
    // the other heads of the group report the same list
    const int shown = kq < a.idx_stride ? kq : a.idx_stride;
    for (int h = 1; h < G; ++h)
      for (int n = tid; n < a.idx_stride; n += NT)
        idx_out[(size_t)h * a.idx_stride + n] = n < shown ? (int)L.keys[n] : -1;
  }

  // alpha_h = sum over the selected positions of s-hat_h, from the stored logits (the same values the
  // normaliser was summed from)
  float asum[G];
#pragma unroll
  for (int h = 0; h < G; ++h) asum[h] = 0.0f;
  for (int n = tid; n < kq; n += NT) {
    const int pos = (int)L.keys[n];
#pragma unroll
    for (int h = 0; h < G; ++h) asum[h] += exp2f((z_unit[(size_t)h * a.S_max + pos] - mh[h]) * esc[h]);
  }

  // ---------------- stage 3: one gather for the G heads ----------------
  using Geo = RowGeometry<DH>;
  constexpr int UNR = 2, GROUP = Geo::RPI * UNR;
  const int sub = lane % Geo::LPR, slot = wave * Geo::RPW + lane / Geo::LPR;
  const int* list = reinterpret_cast<const int*>(L.keys);
  const char* K_head = reinterpret_cast<const char*>(a.K) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(a.V) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[G][8];   // query slices, exp2 domain
  float m_run[G], l_run[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float qv = L.qf[h * DH + sub * 8 + e];
      q8[h][e] = qv * qscale;
      acc[h][e] = 0.0f;
    }
    m_run[h] = -INFINITY; l_run[h] = 0.0f;
  }
  const int n_groups = (kq + GROUP - 1) / GROUP;
  auto issue = [&](uint4 (&kr)[UNR], uint4 (&vr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int n = g * GROUP + t * Geo::RPI + slot;
      const uint32_t off = (uint32_t)list[n < kq ? n : kq - 1] * (uint32_t)(DH * 2);
      kr[t] = load16(K_head + off);
      vr[t] = load16(V_head + off);
    }
  };
  auto consume = [&](const uint4 (&kr)[UNR], const uint4 (&vr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const bool ok = g * GROUP + t * Geo::RPI + slot < kq;
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
  __syncthreads();   // hist and rankp are dead: `part` may overwrite them
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float a_w = wave_sum(asum[h]);
    if (lane == 0) L.stat[(wave * G + h) * 2] = a_w;
    store_wave_partial<DH>(m_run[h], l_run[h], acc[h], L.part + h * (DH + 2), lane, wave * G);   // part[wave][h]
  }
  __syncthreads();
  for (int i = tid; i < G * DH; i += NT) {
    const int h = i / DH, c = i - h * DH;
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) m_all = fmaxf(m_all, L.part[(w * G + h) * (DH + 2) + DH]);
    float l_all = 0.0f, y3 = 0.0f, a_all = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float s = weight_exp2(L.part[(w * G + h) * (DH + 2) + DH], m_all);
      l_all += L.part[(w * G + h) * (DH + 2) + DH + 1] * s;
      y3 += L.part[(w * G + h) * (DH + 2) + c] * s;
      a_all += L.stat[(w * G + h) * 2];
    }
    y3 /= l_all;
    // inv_z of head h: recompute from the broadcast statistics is not needed, every thread holds all G
    float alpha = 0.0f;
#pragma unroll
    for (int hh = 0; hh < G; ++hh) if (hh == h) alpha = a_all * inv_z[hh];
    float y = y3;
    if (!(a.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * a.v_mean[kv_head * DH + c];
    out[(size_t)h * DH + c] = T::narrow(y);
    if (c == 0 && a.alpha_out) a.alpha_out[u0 + h] = alpha;
  }
}

template <class T, int DH, int G>
hipError_t launch_shared_g(const DecodeArgs& a, float* z_ws, hipStream_t s) {
  const size_t lds = 4 * ((size_t)a.S_max + shared_fixed_words<DH, G>());
  auto kern = sparq_decode_shared<T, DH, G>;
  hipError_t e = allow_lds<sparq_decode_shared<T, DH, G>>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(a.B * a.H_kv), dim3(NT), lds, s, a, z_ws);
  return hipGetLastError();
}

template <class T, int DH>
hipError_t launch_shared_dh(const DecodeArgs& a, float* z_ws, hipStream_t s) {
  switch (a.H / a.H_kv) {
    case 2: return launch_shared_g<T, DH, 2>(a, z_ws, s);
    case 4: return launch_shared_g<T, DH, 4>(a, z_ws, s);
    default: return hipErrorInvalidValue;
  }
}

template <int DH>
size_t shared_lds(int S_max, int g) {
  return 4 * ((size_t)S_max + (g == 2 ? shared_fixed_words<DH, 2>() : shared_fixed_words<DH, 4>()));
}

}  // namespace

// LDS bytes of the grouped-query kernel, 0 if the group size or head dimension has no kernel
size_t decode_shared_lds_bytes(int S_max, int d_h, int g) {
  if (g != 2 && g != 4) return 0;
  switch (d_h) {
    case 64: return shared_lds<64>(S_max, g);
    case 128: return shared_lds<128>(S_max, g);
    case 256: return shared_lds<256>(S_max, g);
    default: return 0;
  }
}

hipError_t launch_decode_shared(const DecodeArgs& a, float* z_ws, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d_h) {
    case 64:  return bf ? launch_shared_dh<BF16, 64>(a, z_ws, s) : launch_shared_dh<F16, 64>(a, z_ws, s);
    case 128: return bf ? launch_shared_dh<BF16, 128>(a, z_ws, s) : launch_shared_dh<F16, 128>(a, z_ws, s);
    case 256: return bf ? launch_shared_dh<BF16, 256>(a, z_ws, s) : launch_shared_dh<F16, 256>(a, z_ws, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
