// SparQ decode with the key cache stored once, d_h-contiguous only (Section 6.1, the "1 x K" variant of
// the microbenchmarks; Appendix F "Storing K twice" names the price: Step 1 indexes K along the axis that
// is not contiguous).  One workgroup per (sequence, query head), like the two-copy kernel; only stage 1
// differs: the r selected components of every key are not a contiguous stream, and with r of d_h channels
// spread over the row nearly every 32-byte sector of a row holds one, so stage 1 reads the K rows whole
// (S d_h elements instead of S r) and multiplies by the query with the unselected channels zeroed.
// Stages 0, 2 and 3 are the shared ones.  No key memory beyond K itself, no column scatter on append.
#include "decode_stages.h"

namespace sparq {

namespace {

struct Lds1K {
  uint32_t* keys;   // [S_max]
  SelectLds sel;
  QueryLds qry;
  float* part;      // [NW * (DH + 2)], shares its space with the partial ranks of stage 0
  float* qmask;     // [DH] query with the unselected channels zeroed
};

template <int DH>
__device__ __forceinline__ Lds1K carve_1k(uint32_t* base, int S_max) {
  Lds1K l;
  l.keys = base; base += S_max;
  l.sel.hist = base; base += 2 * kRadixBins;
  l.part = reinterpret_cast<float*>(base);
  l.qry.rankp = reinterpret_cast<int*>(base); base += NW * (DH + 2);
  l.qry.qf = reinterpret_cast<float*>(base); base += DH;
  l.qry.qs = reinterpret_cast<float*>(base); base += DH;
  l.qry.chan = reinterpret_cast<int*>(base); base += DH;
  l.qry.mag = base; base += DH;
  l.qmask = reinterpret_cast<float*>(base); base += DH;
  l.sel.red = reinterpret_cast<float*>(base); base += 32;
  l.sel.wcnt = base; base += 16;
  l.sel.ctl = reinterpret_cast<int*>(base);
  return l;
}

template <int DH>
__host__ __device__ constexpr size_t lds_words_1k() {
  return 2 * (size_t)kRadixBins + (size_t)NW * (DH + 2) + 5 * (size_t)DH + 32 + 16 + 8;
}

// Step 1b from the row-major keys: rows 0..S-1 of one KV head, LPR lanes per row as in the gather of
// Step 2, groups of UNR loads through a two-deep software pipeline.  finish(position, dot) is called by
// the first lane of each row's lane group.  qm8 = the lane's 8 masked query components.
template <class T, int DH, class Finish>
__device__ __forceinline__ void stream_key_rows(const char* K_head_sub, int S, const float (&qm8)[8], int lane, int wave,
                                                Finish&& finish) {
  using G = RowGeometry<DH>;
  constexpr int UNR = 8, GROUP = G::RPI * UNR;
  const int slot = wave * G::RPW + lane / G::LPR;
  const bool first = lane % G::LPR == 0;
  const int n_groups = (S + GROUP - 1) / GROUP;
  auto issue = [&](uint4 (&kr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int n = g * GROUP + t * G::RPI + slot;
      kr[t] = load16(K_head_sub + (size_t)(n < S ? n : S - 1) * (DH * 2));
    }
  };
  auto consume = [&](const uint4 (&kr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int n = g * GROUP + t * G::RPI + slot;
      float f[8];
      unpack8<T>(kr[t], f);
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(f[e], qm8[e], dot);
      dot = lanes_sum<G::LPR>(dot);
      if (first && n < S) finish(n, dot);
    }
  };
  if (n_groups > 0) {
    uint4 ka[UNR], kb[UNR];
    issue(ka, 0);
    int g = 0;
    for (; g + 2 < n_groups; g += 2) {
      issue(kb, g + 1);
      consume(ka, g);
      issue(ka, g + 2);
      consume(kb, g + 1);
    }
    if (g + 1 < n_groups) {
      issue(kb, g + 1);
      consume(ka, g);
      consume(kb, g + 1);
    } else {
      consume(ka, g);
    }
  }
}

template <class T, int DH>
__global__ __launch_bounds__(NT, 4) void sparq_decode_single_k(const DecodeArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const Lds1K L = carve_1k<DH>(smem, a.S_max);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int U = a.B * a.H;
  int u = blockIdx.x;
  if ((U & 7) == 0) u = (u & 7) * (U >> 3) + (u >> 3);   // a contiguous run of units per XCD
  const int b = u / a.H, h = u - b * a.H;
  const size_t kv_head = (size_t)b * a.H_kv + h / (a.H / a.H_kv);

  const uint16_t qcode = tid < DH ? reinterpret_cast<const uint16_t*>(a.q)[(size_t)u * DH + tid] : (uint16_t)0;
  int S = a.seq_lens[b];
  if (S < 0 || S > a.S_max) {
    if (tid == 0) atomicOr(a.err, 8);
    S = S < 0 ? 0 : a.S_max;
  }
  int kb = a.k_per_seq ? a.k_per_seq[b] : a.k;
  kb = kb < 1 ? 1 : (kb > a.k ? a.k : kb);
  const int kq = kb < S ? kb : S;
  uint16_t* out = reinterpret_cast<uint16_t*>(a.out) + (size_t)u * DH;
  int32_t* idx_out = a.idx_out ? a.idx_out + (size_t)u * a.idx_stride : nullptr;
  if (S == 0) {
    if (tid < DH) out[tid] = 0;
    if (tid == 0) { atomicOr(a.err, 2); if (a.alpha_out) a.alpha_out[u] = 0.0f; }
    if (a.chan_out && tid < a.r) a.chan_out[(size_t)u * a.r + tid] = -1;
    if (idx_out) for (int n = tid; n < a.idx_stride; n += NT) idx_out[n] = -1;
    return;
  }

  // ---------------- stage 0 ----------------
  for (int i = tid; i < 2 * kRadixBins; i += NT) L.sel.hist[i] = 0u;
  if (tid < DH) L.qmask[tid] = 0.0f;
  const float tau = apply_tau_mode(select_channels<T, DH>(L.qry, qcode, a.r, tid, lane, wave), a.flags, DH, a.r);
  const Window win = make_window(a.local_window, S, kq);
  if (tid < a.r) {
    const int ch = L.qry.chan[tid];
    L.qmask[ch] = L.qry.qs[tid];
    if (a.chan_out) a.chan_out[(size_t)u * a.r + tid] = ch;
  }
  __syncthreads();

  // ---------------- stage 1: whole key rows, masked query ----------------
  using G = RowGeometry<DH>;
  const int sub = lane % G::LPR;
  const char* K_head = reinterpret_cast<const char*>(a.K) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(a.V) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  float qm8[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) qm8[e] = L.qmask[sub * 8 + e];
  float tmax = -INFINITY;
  stream_key_rows<T, DH>(K_head, S, qm8, lane, wave, [&](int n, float dot) {
    tmax = fmaxf(tmax, dot);
    const uint32_t key = float_to_key(dot);
    L.keys[n] = key;
    if (n < win.S_old) atomicAdd(&L.sel.hist[hist_slot(key >> 21)], 1u);
  });
  // the select reads whole 8-position chunks: clear the tail of the last one
  if (tid < 8 && (S & ~7) + tid >= S && (S & ~7) + tid < a.S_max) L.keys[(S & ~7) + tid] = 0u;
  tmax = wave_max(tmax);
  if (lane == 0) L.sel.red[wave] = tmax;
  __syncthreads();
  float dmax = L.sel.red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, L.sel.red[w]);

  // ---------------- stage 2 ----------------
  uint32_t pmask, pval;
  int need;
  radix_select(L.keys, win.S_old, win.k_old, L.sel, tid, lane, wave, pmask, pval, need);
  const float alpha = compact_selected(L.keys, L.keys, S, win.S_old, pmask, pval, need, dmax, kLog2e / tau, idx_out,
                                       a.idx_stride, L.sel, tid, lane, wave);
  if (tid == 0) {
    if (a.alpha_out) a.alpha_out[u] = alpha;
    if (idx_out && kq > a.idx_stride) atomicOr(a.err, 4);
  }
  if (idx_out) for (int n = kq + tid; n < a.idx_stride; n += NT) idx_out[n] = -1;

  // ---------------- stage 3 ----------------
  const int* list = reinterpret_cast<const int*>(L.keys);
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q8[e] = L.qry.qf[sub * 8 + e] * qscale;
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  attend_rows<T, DH>(K_head, V_head, list, 0, kq, q8, lane, wave, m_run, l_run, acc);
  store_wave_partial<DH>(m_run, l_run, acc, L.part, lane, wave);
  __syncthreads();
  if (tid < DH) {
    float m_all, l_all, y3;
    combine_partials<DH>(L.part, NW, tid, m_all, l_all, y3);
    y3 /= l_all;
    float y = y3;
    if (!(a.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * a.v_mean[kv_head * DH + tid];
    out[tid] = T::narrow(y);
  }
}

template <class T, int DH>
hipError_t launch_1k(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = 4 * ((size_t)a.S_max + lds_words_1k<DH>());
  auto kern = sparq_decode_single_k<T, DH>;
  hipError_t e = allow_lds<sparq_decode_single_k<T, DH>>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(a.B * a.H), dim3(NT), lds, s, a);
  return hipGetLastError();
}

}  // namespace

size_t decode_single_k_lds_bytes(int S_max, int d_h) {
  switch (d_h) {
    case 64: return 4 * ((size_t)S_max + lds_words_1k<64>());
    case 128: return 4 * ((size_t)S_max + lds_words_1k<128>());
    case 256: return 4 * ((size_t)S_max + lds_words_1k<256>());
    default: return 0;
  }
}

hipError_t launch_decode_single_k(const DecodeArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d_h) {
    case 64:  return bf ? launch_1k<BF16, 64>(a, s) : launch_1k<F16, 64>(a, s);
    case 128: return bf ? launch_1k<BF16, 128>(a, s) : launch_1k<F16, 128>(a, s);
    case 256: return bf ? launch_1k<BF16, 256>(a, s) : launch_1k<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
