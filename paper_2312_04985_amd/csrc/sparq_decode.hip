// Fused SparQ decode kernel: one workgroup per (sequence, query head).
//
// Section 4, Steps 1-3, in one launch with no intermediate HBM traffic:
//   stage 0  top-r of |q| (rank by comparison on the 16-bit magnitudes), temperature (Eq. 7)
//   stage 1  stream the r selected rows of the S-contiguous key copy, fp32 approximate logits
//            for every cached position into LDS as order-preserving integer keys
//   stage 2  radix select (11/11/10-bit digits, LDS histograms) of the k-th largest key,
//            ordered compaction of the selected positions (ties to the lower position),
//            alpha = selected share of the softmax mass of the approximate logits
//   stage 3  gather the selected K and V rows, online-softmax exact attention, blend with
//            the mean value vector (Eq. 8), round and store
#include "common.h"
#include "params.h"

namespace sparq {

namespace {

constexpr int NT = kDecodeThreads;
constexpr int NW = NT / kWave;   // waves per workgroup

struct Lds {
  uint32_t* keys;   // [S_max]   stage 1-2: keys; after compaction: selected positions
  uint32_t* hist;   // [kRadixBins]
  float* part;      // [NW * (DH + 2)]
  float* qf;        // [DH] query as fp32
  float* qs;        // [DH] selected query components, channel-ascending
  int* chan;        // [DH] selected channels, ascending
  uint32_t* mag;    // [DH] 15-bit magnitudes
  float* red;       // [32]
  uint32_t* wcnt;   // [16]
  int* ctl;         // [8]
};

template <int DH>
__device__ __forceinline__ Lds carve(uint32_t* base, int S_max) {
  Lds l;
  l.keys = base; base += S_max;
  l.hist = base; base += kRadixBins;
  l.part = reinterpret_cast<float*>(base); base += NW * (DH + 2);
  l.qf = reinterpret_cast<float*>(base); base += DH;
  l.qs = reinterpret_cast<float*>(base); base += DH;
  l.chan = reinterpret_cast<int*>(base); base += DH;
  l.mag = base; base += DH;
  l.red = reinterpret_cast<float*>(base); base += 32;
  l.wcnt = base; base += 16;
  l.ctl = reinterpret_cast<int*>(base);
  return l;
}

// Exclusive prefix sum of v over the workgroup in thread order; *total gets the sum.
// Two barriers; wsum must hold NW words.
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t* wsum, int lane, int wave,
                                                    uint32_t* total) {
  uint32_t incl = wave_scan_incl(v, lane);
  if (lane == kWave - 1) wsum[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    uint32_t t = wsum[w];
    if (w < wave) before += t;
    all += t;
  }
  __syncthreads();
  *total = all;
  return before + incl - v;
}

template <class T, int DH>
__global__ __launch_bounds__(NT) void sparq_decode_fused(const DecodeArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const Lds L = carve<DH>(smem, a.S_max);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of units so
  // that the query heads of one KV group share an L2.
  const int U = a.B * a.H;
  int u = blockIdx.x;
  if ((U & 7) == 0) u = (u & 7) * (U >> 3) + (u >> 3);
  const int b = u / a.H, h = u - b * a.H;
  const int hk = h / (a.H / a.H_kv);
  const size_t kv_head = (size_t)b * a.H_kv + hk;

  int S = a.seq_lens[b];
  if (S < 0 || S > a.S_max) {
    if (tid == 0) atomicOr(a.err, 8);
    S = S < 0 ? 0 : a.S_max;
  }
  int kb = a.k_per_seq ? a.k_per_seq[b] : a.k;
  if (kb < 1) kb = 1;
  const int kq = kb < S ? kb : S;

  uint16_t* out = reinterpret_cast<uint16_t*>(a.out) + (size_t)u * DH;
  if (S == 0) {   // nothing cached: defined output, raise the flag
    if (tid < DH) out[tid] = 0;
    if (tid == 0) { atomicOr(a.err, 2); if (a.alpha_out) a.alpha_out[u] = 0.0f; }
    if (a.chan_out && tid < a.r) a.chan_out[(size_t)u * a.r + tid] = -1;
    if (a.idx_out) for (int n = tid; n < a.idx_stride; n += NT) a.idx_out[(size_t)u * a.idx_stride + n] = -1;
    return;
  }

  // ---------------- stage 0: top-r components of |q|, temperature ----------------
  if (tid < DH) {
    uint16_t c = reinterpret_cast<const uint16_t*>(a.q)[(size_t)u * DH + tid];
    L.mag[tid] = c & 0x7fffu;
    L.qf[tid] = T::widen(c);
  }
  __syncthreads();
  bool sel = false;
  float aq = 0.0f;
  if (tid < DH) {
    const uint32_t mine = L.mag[tid];
    int rank = 0;
    for (int i = 0; i < DH; ++i) {
      const uint32_t m = L.mag[i];
      rank += (m > mine) || (m == mine && i < tid);
    }
    sel = rank < a.r;
    aq = fabsf(L.qf[tid]);
  }
  {
    const uint64_t bal = __ballot(sel);
    const int within = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) L.wcnt[wave] = (uint32_t)__popcll(bal);
    const float l1a = wave_sum(aq), l1s = wave_sum(sel ? aq : 0.0f);
    if (lane == 0) { L.red[wave] = l1a; L.red[NW + wave] = l1s; }
    __syncthreads();
    int off = 0;
    for (int w = 0; w < wave; ++w) off += (int)L.wcnt[w];
    if (sel) { L.chan[off + within] = tid; L.qs[off + within] = L.qf[tid]; }
  }
  float l1_all = 0.0f, l1_sel = 0.0f;
#pragma unroll
  for (int w = 0; w < NW; ++w) { l1_all += L.red[w]; l1_sel += L.red[NW + w]; }
  const float tau = l1_all > 0.0f ? sqrtf((float)DH * l1_sel / l1_all) : sqrtf((float)DH);
  __syncthreads();
  if (a.chan_out && tid < a.r) a.chan_out[(size_t)u * a.r + tid] = L.chan[tid];

  // ---------------- stage 1: approximate logits over the r selected channel rows ----------------
  const int r = a.r;
  const size_t row_bytes = (size_t)a.S_max * 2;
  const char* Kt_head = reinterpret_cast<const char*>(a.Kt) + kv_head * DH * row_bytes;
  const int n_chunks = (S + 7) >> 3;   // 8 positions (16 bytes) per thread per channel row
  float tmax = -INFINITY;
  for (int c = tid; c < n_chunks; c += NT) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const char* base = Kt_head + (size_t)c * 16;
    for (int j0 = 0; j0 < r; j0 += 8) {
      uint4 v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int j = (j0 + t < r) ? j0 + t : r - 1;
        v[t] = load16(base + (size_t)L.chan[j] * row_bytes);
      }
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        if (j0 + t < r) {
          const float qv = L.qs[j0 + t];
          float f[8];
          unpack8<T>(v[t], f);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = fmaf(f[e], qv, acc[e]);
        }
      }
    }
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (c * 8 + e < S) { tmax = fmaxf(tmax, acc[e]); kx[e] = float_to_key(acc[e]); }
      else kx[e] = 0u;
    }
    uint4* dst = reinterpret_cast<uint4*>(L.keys + c * 8);
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  }
  tmax = wave_max(tmax);
  if (lane == 0) L.red[wave] = tmax;
  __syncthreads();
  float dmax = L.red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, L.red[w]);

  // ---------------- stage 2a: radix select of the kq-th largest key ----------------
  uint32_t pmask = 0u, pval = 0u;   // decided high bits of the threshold key
  int need = kq;                    // how many keys equal to the threshold on the decided bits are taken
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const uint32_t dmask = pass == 2 ? 0x3ffu : 0x7ffu;
    for (int i = tid; i < kRadixBins; i += NT) L.hist[i] = 0u;
    __syncthreads();
    for (int i = tid; i < S; i += NT) {
      const uint32_t key = L.keys[i];
      if ((key & pmask) == pval) atomicAdd(&L.hist[(key >> shift) & dmask], 1u);
    }
    __syncthreads();
    // thread t owns bins 4t..4t+3; find the bin where the count from the top reaches `need`
    const uint4 own = reinterpret_cast<const uint4*>(L.hist)[tid];
    const uint32_t mine = own.x + own.y + own.z + own.w;
    uint32_t total;
    const uint32_t below = block_scan_excl(mine, L.wcnt, lane, wave, &total);
    const uint32_t above = total - below - mine;   // keys in bins beyond this thread's
    if (above < (uint32_t)need && (uint32_t)need <= above + mine) {
      const uint32_t cnt[4] = {own.x, own.y, own.z, own.w};
      uint32_t run = above;
      for (int d = 3; d >= 0; --d) {
        if (run + cnt[d] >= (uint32_t)need) {
          L.ctl[0] = tid * 4 + d; L.ctl[1] = need - (int)run; L.ctl[2] = (int)cnt[d];
          break;
        }
        run += cnt[d];
      }
    }
    __syncthreads();
    pval |= (uint32_t)L.ctl[0] << shift;
    pmask |= dmask << shift;
    need = L.ctl[1];
    const int in_bin = L.ctl[2];
    __syncthreads();
    if (need == in_bin) break;   // every key matching the decided bits is taken: no ties to split
  }

  // ---------------- stage 2b: ordered compaction, alpha ----------------
  // Taken: keys above the threshold on the decided bits, plus the first `need` (by position)
  // keys equal to it.  The position list overwrites the key array from the front; a thread
  // never writes past the end of its own chunk and all reads of a sweep precede its writes.
  const float esc = kLog2e / tau;
  float zsum = 0.0f, asum = 0.0f;
  uint32_t run_gt = 0, run_eq = 0;
  int32_t* idx_out = a.idx_out ? a.idx_out + (size_t)u * a.idx_stride : nullptr;
  for (int c0 = 0; c0 < n_chunks; c0 += NT) {
    const int c = c0 + tid;
    uint32_t kx[8];
    if (c < n_chunks) {
      const uint4* src = reinterpret_cast<const uint4*>(L.keys + c * 8);
      const uint4 lo = src[0], hi = src[1];
      kx[0] = lo.x; kx[1] = lo.y; kx[2] = lo.z; kx[3] = lo.w;
      kx[4] = hi.x; kx[5] = hi.y; kx[6] = hi.z; kx[7] = hi.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) kx[e] = 0u;
    }
    uint32_t n_gt = 0, n_eq = 0;
    uint32_t gt_bits = 0, eq_bits = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const bool valid = (c * 8 + e) < S && c < n_chunks;
      const uint32_t hi_bits = kx[e] & pmask;
      const bool g = valid && hi_bits > pval, q = valid && hi_bits == pval;
      gt_bits |= (uint32_t)g << e; eq_bits |= (uint32_t)q << e;
      n_gt += g; n_eq += q;
    }
    uint32_t total;
    const uint32_t ex = block_scan_excl(n_gt | (n_eq << 16), L.wcnt, lane, wave, &total);
    const uint32_t gt_before = run_gt + (ex & 0xffffu);
    uint32_t eq_before = run_eq + (ex >> 16);
    uint32_t o = gt_before + (eq_before < (uint32_t)need ? eq_before : (uint32_t)need);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const bool valid = (c * 8 + e) < S && c < n_chunks;
      if (valid) {
        const float w = exp2f((key_to_float(kx[e]) - dmax) * esc);
        zsum += w;
        bool take = (gt_bits >> e) & 1u;
        if ((eq_bits >> e) & 1u) { take = eq_before < (uint32_t)need; ++eq_before; }
        if (take) {
          asum += w;
          L.keys[o] = (uint32_t)(c * 8 + e);
          if (idx_out && (int)o < a.idx_stride) idx_out[o] = c * 8 + e;
          ++o;
        }
      }
    }
    run_gt += total & 0xffffu;
    run_eq += total >> 16;
  }
  zsum = wave_sum(zsum); asum = wave_sum(asum);
  if (lane == 0) { L.red[wave] = zsum; L.red[NW + wave] = asum; }
  __syncthreads();   // also publishes the position list
  float zt = 0.0f, at = 0.0f;
#pragma unroll
  for (int w = 0; w < NW; ++w) { zt += L.red[w]; at += L.red[NW + w]; }
  const float alpha = at / zt;
  if (tid == 0) {
    if (a.alpha_out) a.alpha_out[u] = alpha;
    if (idx_out && kq > a.idx_stride) atomicOr(a.err, 4);
  }
  if (idx_out) for (int n = kq + tid; n < a.idx_stride; n += NT) idx_out[n] = -1;

  // ---------------- stage 3: exact attention over the gathered rows, blend ----------------
  constexpr int LPR = DH / 8;          // lanes per row (16 bytes each)
  constexpr int RPW = kWave / LPR;     // rows per wave per load
  constexpr int RPI = NW * RPW;        // rows per workgroup per load
  constexpr int UNR = 4;
  const int sub = lane % LPR, slot = wave * RPW + lane / LPR;
  const int* pos = reinterpret_cast<const int*>(L.keys);
  const char* K_head = reinterpret_cast<const char*>(a.K) + kv_head * a.S_max * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(a.V) + kv_head * a.S_max * (size_t)(DH * 2) + sub * 16;
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q8[e] = L.qf[sub * 8 + e] * qscale;
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int n0 = 0; n0 < kq; n0 += RPI * UNR) {
    uint4 kr[UNR], vr[UNR];
    bool ok[UNR];
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int n = n0 + t * RPI + slot;
      ok[t] = n < kq;
      const size_t off = (size_t)pos[ok[t] ? n : 0] * (size_t)(DH * 2);
      kr[t] = load16(K_head + off);
      vr[t] = load16(V_head + off);
    }
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      float f[8];
      unpack8<T>(kr[t], f);
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(f[e], q8[e], dot);
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) dot += __shfl_xor(dot, o);
      if (ok[t]) {
        const float m_new = fmaxf(m_run, dot);
        const float sc = exp2f(m_run - m_new), pr = exp2f(dot - m_new);
        unpack8<T>(vr[t], f);
        l_run = l_run * sc + pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * sc + pr * f[e];
        m_run = m_new;
      }
    }
  }
  // merge the row groups of a wave, then the waves
#pragma unroll
  for (int o = LPR; o < kWave; o <<= 1) {
    const float m_o = __shfl_xor(m_run, o), l_o = __shfl_xor(l_run, o);
    const float m_new = fmaxf(m_run, m_o);
    const float s1 = weight_exp2(m_run, m_new), s2 = weight_exp2(m_o, m_new);
    l_run = l_run * s1 + l_o * s2;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = acc[e] * s1 + __shfl_xor(acc[e], o) * s2;
    m_run = m_new;
  }
  float* part = L.part + wave * (DH + 2);
  if (lane < LPR) {
#pragma unroll
    for (int e = 0; e < 8; ++e) part[sub * 8 + e] = acc[e];
    if (lane == 0) { part[DH] = m_run; part[DH + 1] = l_run; }
  }
  __syncthreads();
  if (tid < DH) {
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) m_all = fmaxf(m_all, L.part[w * (DH + 2) + DH]);
    float l_all = 0.0f, y3 = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float s = weight_exp2(L.part[w * (DH + 2) + DH], m_all);
      l_all += L.part[w * (DH + 2) + DH + 1] * s;
      y3 += L.part[w * (DH + 2) + tid] * s;
    }
    y3 /= l_all;
    float y = y3;
    if (!(a.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * a.v_mean[kv_head * DH + tid];
    out[tid] = T::narrow(y);
  }
}

template <class T, int DH>
hipError_t launch_one(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = decode_lds_bytes(a.S_max, DH);
  auto kern = sparq_decode_fused<T, DH>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(a.B * a.H), dim3(NT), lds, s, a);
  return hipGetLastError();
}

}  // namespace

size_t decode_lds_bytes(int S_max, int d_h) {
  return 4 * ((size_t)S_max + kRadixBins + (size_t)NW * (d_h + 2) + 4 * (size_t)d_h + 32 + 16 + 8);
}

hipError_t launch_decode(const DecodeArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d_h) {
    case 64:  return bf ? launch_one<BF16, 64>(a, s) : launch_one<F16, 64>(a, s);
    case 128: return bf ? launch_one<BF16, 128>(a, s) : launch_one<F16, 128>(a, s);
    case 256: return bf ? launch_one<BF16, 256>(a, s) : launch_one<F16, 256>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace sparq
