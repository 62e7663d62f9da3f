// Fused SparQ decode kernel: one workgroup per (sequence, query head).
//
// Section 4, Steps 1-3, in one launch with no intermediate HBM traffic:
//   stage 0  top-r of |q| (rank by comparison on the 16-bit magnitudes), temperature (Eq. 7)
//   stage 1  stream the r selected rows of the S-contiguous key copy, fp32 approximate logits
//            for every cached position into LDS as order-preserving integer keys
//   stage 2  radix select (11/11/10-bit digits, LDS histograms; the first digit is counted while
//            stage 1 produces the keys) of the k-th largest key,
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
  uint32_t* hist;   // [2][kRadixBins] double-buffered digit histograms
  float* part;      // [NW * (DH + 2)] stage-3 partials; stage 0: partial ranks (NT words)
  float* qf;        // [DH] query as fp32
  float* qs;        // [DH] selected query components, channel-ascending
  int* chan;        // [DH] selected channels, ascending
  uint32_t* mag;    // [DH] 15-bit magnitudes
  float* red;       // [32]
  uint32_t* wcnt;   // [2][NW] double-buffered wave totals of the workgroup scan
  int* ctl;         // [8]
  uint16_t* knew;   // [DH] codes of the key row being appended (fused append only)
  uint16_t* vnew;   // [DH]
};

template <int DH>
__device__ __forceinline__ Lds carve(uint32_t* base, int S_max) {
  Lds l;
  l.keys = base; base += S_max;
  l.hist = base; base += 2 * kRadixBins;
  l.part = reinterpret_cast<float*>(base); base += NW * (DH + 2);
  l.qf = reinterpret_cast<float*>(base); base += DH;
  l.qs = reinterpret_cast<float*>(base); base += DH;
  l.chan = reinterpret_cast<int*>(base); base += DH;
  l.mag = base; base += DH;
  l.red = reinterpret_cast<float*>(base); base += 32;
  l.wcnt = base; base += 16;
  l.ctl = reinterpret_cast<int*>(base); base += 8;
  l.knew = reinterpret_cast<uint16_t*>(base); base += DH / 2;
  l.vnew = reinterpret_cast<uint16_t*>(base);
  return l;
}

// Exclusive prefix sum of v over the workgroup in thread order; *total gets the sum.
// One barrier; callers alternate `wsum` between two NW-word buffers on consecutive calls.
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t* wsum, int lane, int wave,
                                                    uint32_t* total) {
  const uint32_t incl = wave_scan_incl(v);
  if (lane == kWave - 1) wsum[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t t = wsum[w];
    if (w < wave) before += t;
    all += t;
  }
  *total = all;
  return before + incl - v;
}

// Histogram bins are stored swizzled so that the 32 consecutive digits a lane sums in
// find_threshold_bin sit in 32 different rows of 64 words: lane-consecutive, conflict-free reads.
__device__ __forceinline__ uint32_t hist_slot(uint32_t digit) { return ((digit & 31u) << 6) | (digit >> 5); }

// One wave locates the digit at which the count taken from the top digit downwards reaches `need`;
// writes {digit, how many keys of that digit are needed, keys with that digit} to ctl[0..2].
// Two levels: lane l sums digits 32l..32l+31 and a wave scan finds the lane, then the 32 digits of
// that lane are scanned across lanes.  Requires 1 <= need <= total count.
__device__ __forceinline__ void find_threshold_bin(const uint32_t* hist, int need, int lane, int* ctl) {
  uint32_t mine = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) mine += hist[(i << 6) | lane];
  const uint32_t incl = wave_scan_incl(mine);
  const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
  const uint32_t above = total - incl;      // keys with digits owned by higher lanes
  const uint64_t hit = __ballot(above < (uint32_t)need && (uint32_t)need <= above + mine);
  const int ls = hit ? __ffsll((unsigned long long)hit) - 1 : 0;
  const uint32_t need2 = (uint32_t)need - (uint32_t)__shfl((int)above, ls);
  // lane t < 32 takes digit 32*ls + 31 - t, so that the scan runs from the top digit down
  const uint32_t c = lane < 32 ? hist[((31 - lane) << 6) | ls] : 0u;
  const uint32_t inc2 = wave_scan_incl(c);
  if (lane < 32 && (inc2 - c) < need2 && need2 <= inc2) {
    ctl[0] = ls * 32 + 31 - lane; ctl[1] = (int)(need2 - (inc2 - c)); ctl[2] = (int)c;
  }
}

#ifdef SPARQ_TIMELINE
#ifndef SPARQ_TL_MASK
#define SPARQ_TL_MASK 0xffffffffu
#endif
#define TL_MARK(slot) do { if (((SPARQ_TL_MASK >> (slot)) & 1u) && tid == 0 && a.idx_out) a.idx_out[(size_t)blockIdx.x * a.idx_stride + (slot)] = (int)wall_clock64(); } while (0)
#else
#define TL_MARK(slot) do {} while (0)
#endif

// APPEND = true is the one-launch decode step: the new key/value row of every KV head (k_new, v_new)
// counts as position S_b of its sequence without being read back from the cache.  Every workgroup
// takes that row from the inputs; the workgroup of the first query head of a KV group also writes
// it into K, V and Kt and stores the updated mean; lengths and means go to the *_next buffers, so
// no workgroup can observe another one's update of the state it reads.
template <class T, int DH, bool APPEND>
__global__ __launch_bounds__(NT, 4) void sparq_decode_fused(const DecodeArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const Lds L = carve<DH>(smem, a.S_max);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  TL_MARK(0);
#ifdef SPARQ_TIMELINE
  if (tid == 0 && a.idx_out) {
    a.idx_out[(size_t)blockIdx.x * a.idx_stride + 8] = __builtin_amdgcn_s_getreg(63492);   // HW_ID
    a.idx_out[(size_t)blockIdx.x * a.idx_stride + 9] = __builtin_amdgcn_s_getreg(63508);   // XCC_ID
  }
#endif

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of units so
  // that the query heads of one KV group share an L2.
  const int U = a.B * a.H;
  int u = blockIdx.x;
  if ((U & 7) == 0) u = (u & 7) * (U >> 3) + (u >> 3);
  const int b = u / a.H, h = u - b * a.H;
  const int hk = h / (a.H / a.H_kv);
  const size_t kv_head = (size_t)b * a.H_kv + hk;

  uint16_t qcode = 0, kcode = 0, vcode = 0;
  if (tid < DH) {
    qcode = reinterpret_cast<const uint16_t*>(a.q)[(size_t)u * DH + tid];
    if (APPEND) {
      kcode = reinterpret_cast<const uint16_t*>(a.k_new)[kv_head * DH + tid];
      vcode = reinterpret_cast<const uint16_t*>(a.v_new)[kv_head * DH + tid];
    }
  }
  int S = a.seq_lens[b];
  TL_MARK(15);
  if (S < 0 || S > a.S_max) {
    if (tid == 0) atomicOr(a.err, 8);
    S = S < 0 ? 0 : a.S_max;
  }
  bool appended = false;                          // this sequence takes the new row (uniform)
  const bool owner = APPEND && h == hk * (a.H / a.H_kv);   // writes the row and the new mean
  if (APPEND) {
    if (S + 1 <= a.S_max) { appended = true; S += 1; }
    else if (tid == 0) atomicOr(a.err, 1);
    if (h == 0 && tid == 0) a.seq_lens_next[b] = S;
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
    if (owner && tid < DH) a.v_mean_next[kv_head * DH + tid] = a.v_mean[kv_head * DH + tid];
    return;
  }

  // ---------------- stage 0: top-r components of |q|, temperature ----------------
  // Channel j gets the sort key (|q_j| as its 15-bit code) << 9 | (511 - j): keys are distinct and
  // "larger key" is exactly "larger magnitude, or equal magnitude and lower channel".
  for (int i = tid; i < 2 * kRadixBins; i += NT) L.hist[i] = 0u;
  if (tid < DH) {
    L.mag[tid] = ((uint32_t)(qcode & 0x7fffu) << 9) | (uint32_t)(511 - tid);
    L.qf[tid] = T::widen(qcode);
    if (APPEND) { L.knew[tid] = kcode; L.vnew[tid] = vcode; }
  }
  __syncthreads();
  TL_MARK(13);
  int* rankp = reinterpret_cast<int*>(L.part);   // [NT / DH][DH] partial ranks
  {
    // rank of channel j = number of larger keys; the NT threads split the DH x DH comparisons
    constexpr int SL = NT / DH, PER = DH / SL;
    const int j = tid % DH, slice = tid / DH;
    const uint32_t mine = L.mag[j];
    int partial = 0;
#pragma unroll
    for (int i4 = 0; i4 < PER; i4 += 4) {
      const uint4 m = *reinterpret_cast<const uint4*>(L.mag + slice * PER + i4);
      partial += (m.x > mine) + (m.y > mine) + (m.z > mine) + (m.w > mine);
    }
    rankp[slice * DH + j] = partial;
  }
  __syncthreads();
  TL_MARK(14);
  float tau;
  {
    // Every wave finishes the selection for all channels by itself (no further exchange): ranks,
    // ballots and the L1 sums are recomputed per wave; wave g writes the list entries of channels
    // 64g..64g+63.  The list is padded to a multiple of 8 with the last channel at weight 0, so
    // stage 1 works on whole batches of 8 rows (the extra loads repeat a line just read).
    constexpr int SL = NT / DH, NG = DH / kWave;
    const int r8 = (a.r + 7) & ~7;
    int before = 0;
    float l1a = 0.0f, l1s = 0.0f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int jj = g * kWave + lane;
      int rank = 0;
#pragma unroll
      for (int s = 0; s < SL; ++s) rank += rankp[s * DH + jj];
      const bool sel = rank < a.r;
      const float qv = L.qf[jj], aq = fabsf(qv);
      const uint64_t bal = __ballot(sel);
      if (g == wave && sel) {
        const int p = before + __popcll(bal & ((1ull << lane) - 1ull));
        L.chan[p] = jj; L.qs[p] = qv;
        if (p == a.r - 1)
          for (int pp = a.r; pp < r8; ++pp) { L.chan[pp] = jj; L.qs[pp] = 0.0f; }
      }
      before += __popcll(bal);
      l1a += aq; l1s += sel ? aq : 0.0f;
    }
    const float l1_all = wave_sum(l1a), l1_sel = wave_sum(l1s);
    tau = l1_all > 0.0f ? sqrtf((float)DH * l1_sel / l1_all) : sqrtf((float)DH);
  }
  __syncthreads();
  if (a.chan_out && tid < a.r) a.chan_out[(size_t)u * a.r + tid] = L.chan[tid];
  float dot_new = 0.0f;   // approximate logit numerator of the appended row (every wave computes it)
  if (APPEND && appended) {
    float part_new = 0.0f;
    for (int jj = lane; jj < ((a.r + 7) & ~7); jj += kWave)
      part_new = fmaf(T::widen(L.knew[L.chan[jj]]), L.qs[jj], part_new);
    dot_new = wave_sum(part_new);
  }
  TL_MARK(1);

  // ---------------- stage 1: approximate logits over the r selected channel rows ----------------
  // A thread owns chunks of 8 consecutive positions (16 bytes of every channel row); the loads of
  // the next 8 channels are in flight while the current 8 are accumulated.  Each finished key is
  // also counted into the first digit histogram, so the first select pass costs no extra sweep.
  const int r = a.r;
  const size_t row_bytes = (size_t)a.S_max * 2;
  const char* Kt_head = reinterpret_cast<const char*>(a.Kt) + kv_head * DH * row_bytes;
  const int n_chunks = (S + 7) >> 3;
  float tmax = -INFINITY;
  const int n_batches = (r + 7) >> 3;   // batches of 8 channel rows (list padded in stage 0)
  auto issue = [&](uint4 (&v)[8], uint32_t voff, int batch) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int ch = __builtin_amdgcn_readfirstlane(L.chan[batch * 8 + t]);   // uniform: scalar row base
      v[t] = load16(Kt_head + (size_t)ch * row_bytes + voff);
    }
  };
  auto consume = [&](const uint4 (&v)[8], float (&acc)[8], int batch) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float qv = L.qs[batch * 8 + t];
      float f[8];
      unpack8<T>(v[t], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(f[e], qv, acc[e]);
    }
  };
  // The (chunk, batch) pairs a thread owns form one flat sequence that runs through a two-deep
  // software pipeline: a batch of 8 loads is always in flight behind the one being accumulated,
  // also across chunk boundaries, so a short last sweep costs no extra memory round trip.
  {
    const int my_chunks = n_chunks > tid ? (n_chunks - tid + NT - 1) / NT : 0;
    const int items = my_chunks * n_batches;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int ic = 0, ib = 0, cc = 0, cb = 0;   // issue and consume cursors: (own chunk number, batch)
    auto issue_next = [&](uint4 (&v)[8]) {
      issue(v, (uint32_t)(tid + ic * NT) * 16u, ib);
      if (++ib == n_batches) { ib = 0; ++ic; }
    };
    auto consume_next = [&](const uint4 (&v)[8]) {
      consume(v, acc, cb);
      if (++cb == n_batches) {          // chunk finished: keys to LDS and into the first histogram
        const int c = tid + cc * NT;
        uint32_t kx[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (c * 8 + e < S) {
            const float val = (APPEND && appended && c * 8 + e == S - 1) ? dot_new : acc[e];
            tmax = fmaxf(tmax, val);
            kx[e] = float_to_key(val);
            atomicAdd(&L.hist[hist_slot(kx[e] >> 21)], 1u);
          } else {
            kx[e] = 0u;
          }
          acc[e] = 0.0f;
        }
        uint4* dst = reinterpret_cast<uint4*>(L.keys + c * 8);
        dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
        dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
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
  tmax = wave_max(tmax);
  if (lane == 0) L.red[wave] = tmax;
  __syncthreads();
  float dmax = L.red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, L.red[w]);

  TL_MARK(2);
#if defined(SPARQ_STOP_AFTER) && SPARQ_STOP_AFTER == 1
  if (tid < DH) out[tid] = (uint16_t)(L.keys[tid] + __float_as_uint(dmax));
  return;
#endif
  // ---------------- stage 2a: radix select of the kq-th largest key ----------------
  // Digits of 11, 11 and 10 bits from the top.  Pass p counts into hist[p & 1]; the other buffer
  // is cleared meanwhile.  One wave finds the threshold bin, everyone picks it up after a barrier.
  uint32_t pmask = 0u, pval = 0u;   // decided high bits of the threshold key
  int need = kq;                    // how many keys equal to the threshold on the decided bits are taken
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const uint32_t dmask = pass == 2 ? 0x3ffu : 0x7ffu;
    uint32_t* hist = L.hist + (pass & 1) * kRadixBins;
    if (pass > 0) {
      uint32_t* other = L.hist + ((pass + 1) & 1) * kRadixBins;   // free since the last barrier
      for (int i = tid; i < kRadixBins; i += NT) other[i] = 0u;
      for (int c = tid; c < n_chunks; c += NT) {
        const uint4* src = reinterpret_cast<const uint4*>(L.keys + c * 8);
        const uint4 lo = src[0], hi = src[1];
        const uint32_t kx[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (c * 8 + e < S && (kx[e] & pmask) == pval) atomicAdd(&hist[hist_slot((kx[e] >> shift) & dmask)], 1u);
      }
      __syncthreads();
    }
    if (wave == 0) find_threshold_bin(hist, need, lane, L.ctl);
    __syncthreads();
    pval |= (uint32_t)L.ctl[0] << shift;
    pmask |= dmask << shift;
    need = L.ctl[1];
    const int in_bin = L.ctl[2];
    TL_MARK(10 + pass);
    if (need == in_bin) break;   // every key matching the decided bits is taken: no ties to split
  }

  TL_MARK(3);
  // ---------------- stage 2b: ordered compaction, alpha ----------------
  // Taken: keys above the threshold on the decided bits, plus the first `need` (by position)
  // keys equal to it.  The position list overwrites the key array from the front; a thread
  // never writes past the end of its own chunk and all reads of a sweep precede its writes.
  const float esc = kLog2e / tau;
  float zsum = 0.0f, asum = 0.0f;
  uint32_t run_gt = 0, run_eq = 0;
#ifdef SPARQ_TIMELINE
  int32_t* idx_out = nullptr;
#else
  int32_t* idx_out = a.idx_out ? a.idx_out + (size_t)u * a.idx_stride : nullptr;
#endif
  int sweep = 0;
  for (int c0 = 0; c0 < n_chunks; c0 += NT, ++sweep) {
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
    const uint32_t ex = block_scan_excl(n_gt | (n_eq << 16), L.wcnt + (sweep & 1) * NW, lane, wave, &total);
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

  TL_MARK(4);
#if defined(SPARQ_STOP_AFTER) && SPARQ_STOP_AFTER == 2
  if (tid < DH) out[tid] = (uint16_t)(L.keys[tid] + __float_as_uint(alpha));
  return;
#endif
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
  constexpr int GROUP = RPI * UNR;          // rows the workgroup covers per group of loads
  const int n_groups = (kq + GROUP - 1) / GROUP;
  // positions are ascending, so the appended row (position S - 1) can only be the last entry
  const bool new_selected = APPEND && appended && pos[kq - 1] == S - 1;
  auto issue3 = [&](uint4 (&kr)[UNR], uint4 (&vr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int n = g * GROUP + t * RPI + slot;
      const uint32_t off = (uint32_t)pos[n < kq ? n : kq - 1] * (uint32_t)(DH * 2);   // < S_max * 512 bytes
      kr[t] = load16(K_head + off);
      vr[t] = load16(V_head + off);
    }
  };
  auto consume3 = [&](const uint4 (&kr)[UNR], const uint4 (&vr)[UNR], int g) {
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      float f[8];
      const bool from_inputs = APPEND && new_selected && (g * GROUP + t * RPI + slot == kq - 1);
      const uint4 kt = from_inputs ? *reinterpret_cast<const uint4*>(L.knew + sub * 8) : kr[t];
      const uint4 vt = from_inputs ? *reinterpret_cast<const uint4*>(L.vnew + sub * 8) : vr[t];
      unpack8<T>(kt, f);
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(f[e], q8[e], dot);
      dot = lanes_sum<LPR>(dot);
      if (g * GROUP + t * RPI + slot < kq) {
        const float m_new = fmaxf(m_run, dot);
        const float sc = exp2f(m_run - m_new), pr = exp2f(dot - m_new);
        unpack8<T>(vt, f);
        l_run = l_run * sc + pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * sc + pr * f[e];
        m_run = m_new;
      }
    }
  };
  {
    uint4 ka[UNR], va3[UNR], kb3[UNR], vb3[UNR];
    issue3(ka, va3, 0);
    int g = 0;
    for (; g + 2 < n_groups; g += 2) {
      issue3(kb3, vb3, g + 1);
      consume3(ka, va3, g);
      issue3(ka, va3, g + 2);
      consume3(kb3, vb3, g + 1);
    }
    if (g + 1 < n_groups) {
      issue3(kb3, vb3, g + 1);
      consume3(ka, va3, g);
      consume3(kb3, vb3, g + 1);
    } else {
      consume3(ka, va3, g);
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
    float vm = a.v_mean[kv_head * DH + tid];
    if (APPEND) {
      if (appended) vm += (T::widen(L.vnew[tid]) - vm) * (1.0f / (float)S);   // same update as append_one_row
      if (owner) a.v_mean_next[kv_head * DH + tid] = vm;
    }
    float y = y3;
    if (!(a.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * vm;
    out[tid] = T::narrow(y);
  }
  if (APPEND && owner && appended) {
    // the row into both key layouts and the value cache
    uint16_t* Krow = reinterpret_cast<uint16_t*>(a.K) + (kv_head * a.S_max + (S - 1)) * DH;
    uint16_t* Vrow = reinterpret_cast<uint16_t*>(a.V) + (kv_head * a.S_max + (S - 1)) * DH;
    if (tid < DH / 8) {
      reinterpret_cast<uint4*>(Krow)[tid] = reinterpret_cast<const uint4*>(L.knew)[tid];
      reinterpret_cast<uint4*>(Vrow)[tid] = reinterpret_cast<const uint4*>(L.vnew)[tid];
    }
    if (tid < DH) reinterpret_cast<uint16_t*>(a.Kt)[(kv_head * DH + tid) * a.S_max + (S - 1)] = L.knew[tid];
  }
  TL_MARK(5);
}

template <class T, int DH, bool APPEND>
hipError_t launch_one(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = decode_lds_bytes(a.S_max, DH);
  auto kern = sparq_decode_fused<T, DH, APPEND>;
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
  return 4 * ((size_t)S_max + 2 * kRadixBins + (size_t)NW * (d_h + 2) + 5 * (size_t)d_h + 32 + 16 + 8);
}

template <bool APPEND>
hipError_t launch_any(const DecodeArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d_h) {
    case 64:  return bf ? launch_one<BF16, 64, APPEND>(a, s) : launch_one<F16, 64, APPEND>(a, s);
    case 128: return bf ? launch_one<BF16, 128, APPEND>(a, s) : launch_one<F16, 128, APPEND>(a, s);
    case 256: return bf ? launch_one<BF16, 256, APPEND>(a, s) : launch_one<F16, 256, APPEND>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

hipError_t launch_decode(const DecodeArgs& a, int dtype, hipStream_t s) {
  return a.k_new ? launch_any<true>(a, dtype, s) : launch_any<false>(a, dtype, s);
}

}  // namespace sparq
