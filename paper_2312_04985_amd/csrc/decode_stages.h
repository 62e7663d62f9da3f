// The stages of the SparQ decode step (Section 4, Steps 1-3) as workgroup-level device functions.
// Every decode plan is a different distribution of these stages over workgroups: one workgroup per
// (sequence, head) (sparq_decode.hip), digit buckets over spans (sparq_decode_bucket.hip), two-level selection
// (sparq_decode_long.hip), the grouped-query rule (sparq_decode_shared.hip), the single-copy key cache
// (sparq_decode_single_k.hip); sparq_decode_split.hip holds the gather and merge launches that the
// multi-launch plans share; the append kernels use the column flush.
// Unless noted, functions are called by all kDecodeThreads threads of a workgroup (they contain barriers).
#pragma once
#include "common.h"
#include "params.h"

namespace sparq {

constexpr int NT = kDecodeThreads;
constexpr int NW = NT / kWave;   // waves per workgroup
constexpr int kTieHeavy = 2048;  // a radix bin with more keys than this is counted tie-robustly in the next pass

// ------------------------------------------------------------------------------------------------
// small workgroup primitives

// Histogram bins are stored swizzled so that the 32 consecutive digits a lane sums in
// find_threshold_bin sit in 32 different rows of 64 words: lane-consecutive, conflict-free reads.
__device__ __forceinline__ uint32_t hist_slot(uint32_t digit) { return ((digit & 31u) << 6) | (digit >> 5); }

// First-digit counts of the 8 keys of one chunk: runs of equal digits among neighbours (duplicated keys) are
// added with one atomic.  n_valid = how many of the 8 keys count (the leading ones).
__device__ __forceinline__ void hist_add_chunk(uint32_t* hist, const uint32_t (&kx)[8], int n_valid) {
  uint32_t run_d = kx[0] >> 21, run_n = n_valid > 0 ? 1u : 0u;
#pragma unroll
  for (int e = 1; e < 8; ++e) {
    const uint32_t d = kx[e] >> 21;
    const uint32_t v = e < n_valid ? 1u : 0u;
    if (d != run_d) {
      if (run_n) atomicAdd(&hist[hist_slot(run_d)], run_n);
      run_d = d; run_n = 0u;
    }
    run_n += v;
  }
  if (run_n) atomicAdd(&hist[hist_slot(run_d)], run_n);
}

// Count one key per lane into a histogram when many lanes may hold the same digit (exact ties: 64 LDS
// atomics on one address are serialised).  Up to four rounds: the first pending lane's digit is broadcast and
// all lanes holding it are counted with one atomic; what is left goes through plain atomics.  Called by all
// lanes of a wave together; lanes with valid = false contribute nothing.
__device__ __forceinline__ void hist_add_ties(uint32_t* hist, uint32_t digit, bool valid, int lane) {
  uint64_t todo = __ballot(valid);
#pragma unroll 1
  for (int it = 0; it < 4 && todo; ++it) {
    const int leader = __ffsll((unsigned long long)todo) - 1;
    const uint32_t dsel = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
    const uint64_t same = __ballot(valid && digit == dsel) & todo;
    if (lane == leader) atomicAdd(&hist[hist_slot(dsel)], (uint32_t)__popcll(same));
    todo &= ~same;
  }
  if ((todo >> lane) & 1ull) atomicAdd(&hist[hist_slot(digit)], 1u);
}

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

// The length a launch of a multi-launch plan works on.  Inside sparq_decode_step (d.k_new set) the row being appended counts as position
// S_b although it reaches the cache only in the plan's last launch: every launch adds it the same way.
__device__ __forceinline__ int visible_length(const DecodeArgs& d, int b, bool& appended, bool& bad, bool& full) {
  int S = d.seq_lens[b];
  bad = S < 0 || S > d.S_max;
  if (bad) S = S < 0 ? 0 : d.S_max;
  appended = false; full = false;
  if (d.k_new) {
    if (S + 1 <= d.S_max) { appended = true; S += 1; } else full = true;
  }
  return S;
}

// ------------------------------------------------------------------------------------------------
// Step 1a: the r largest components of |q| (ties to the lower channel) and the temperature (Eq. 9)

struct QueryLds {
  uint32_t* mag;   // [DH] sort keys
  int* rankp;      // [NT] partial ranks
  float* qf;       // [DH] query as fp32
  float* qs;       // [DH] selected query components, channel-ascending, padded to a multiple of 8
  int* chan;       // [DH] selected channels, ascending, same padding
};

// Channel j gets the sort key (|q_j| as its 15-bit code) << 9 | (511 - j): keys are distinct and
// "larger key" is exactly "larger magnitude, or equal magnitude and lower channel"; the rank of a
// channel is the number of larger keys and the NT threads split the DH x DH comparisons.  Every
// wave then finishes the selection for all channels by itself (ranks, ballots, L1 sums), wave g
// writing the list entries of channels 64g..64g+63.  The list is padded to a multiple of 8 with the
// last channel at weight 0, so that Step 1b works on whole batches of 8 rows.
// `qcode` is the 16-bit code of q[tid] for tid < DH.  Three barriers; the first also publishes
// whatever the caller wrote to LDS before the call.  Returns tau.
template <class T, int DH>
__device__ __forceinline__ float select_channels(const QueryLds& Q, uint16_t qcode, int r, int tid, int lane, int wave) {
  if (tid < DH) {
    Q.mag[tid] = ((uint32_t)(qcode & 0x7fffu) << 9) | (uint32_t)(511 - tid);
    Q.qf[tid] = T::widen(qcode);
  }
  __syncthreads();
  {
    constexpr int SL = NT / DH, PER = DH / SL;
    const int j = tid % DH, slice = tid / DH;
    const uint32_t mine = Q.mag[j];
    int partial = 0;
#pragma unroll
    for (int i4 = 0; i4 < PER; i4 += 4) {
      const uint4 m = *reinterpret_cast<const uint4*>(Q.mag + slice * PER + i4);
      partial += (m.x > mine) + (m.y > mine) + (m.z > mine) + (m.w > mine);
    }
    Q.rankp[slice * DH + j] = partial;
  }
  __syncthreads();
  float tau;
  {
    constexpr int SL = NT / DH, NG = DH / kWave;
    const int r8 = (r + 7) & ~7;
    int before = 0;
    float l1a = 0.0f, l1s = 0.0f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int jj = g * kWave + lane;
      int rank = 0;
#pragma unroll
      for (int s = 0; s < SL; ++s) rank += Q.rankp[s * DH + jj];
      const bool sel = rank < r;
      const float qv = Q.qf[jj], aq = fabsf(qv);
      const uint64_t bal = __ballot(sel);
      if (g == wave && sel) {
        const int p = before + __popcll(bal & ((1ull << lane) - 1ull));
        Q.chan[p] = jj; Q.qs[p] = qv;
        if (p == r - 1)
          for (int pp = r; pp < r8; ++pp) { Q.chan[pp] = jj; Q.qs[pp] = 0.0f; }
      }
      before += __popcll(bal);
      l1a += aq; l1s += sel ? aq : 0.0f;
    }
    const float l1_all = wave_sum(l1a), l1_sel = wave_sum(l1s);
    tau = l1_all > 0.0f ? sqrtf((float)DH * l1_sel / l1_all) : sqrtf((float)DH);
  }
  __syncthreads();
  return tau;
}

// The temperature actually used: Eq. (9), or one of the two fixed values of the ablation in Section 5.3
// (flag bits 3 and 4).
__device__ __forceinline__ float apply_tau_mode(float tau_l1, uint32_t flags, int d_h, int r) {
  if (flags & 8u) return sqrtf((float)d_h);
  if (flags & 16u) return sqrtf((float)r);
  return tau_l1;
}

// Local window: the last n_local = min(l, kq) positions are selected unconditionally; the select then
// runs over the S - n_local older positions for kq - n_local of them.
struct Window {
  int n_local, S_old, k_old;
};
__device__ __forceinline__ Window make_window(int local_window, int S, int kq) {
  Window w;
  w.n_local = local_window < kq ? local_window : kq;
  w.S_old = S - w.n_local;
  w.k_old = kq - w.n_local;
  return w;
}

// ------------------------------------------------------------------------------------------------
// Step 1b: approximate logit numerators over the r selected rows of the S-contiguous key copy

// Chunks (8 consecutive positions = 16 bytes of every channel row) chunk_begin + tid + i * STRIDE belong to
// thread tid of STRIDE (all NT threads of the workgroup unless the caller divides the rows of a chunk among
// groups of threads).  The (chunk, batch-of-8-rows) pairs a thread owns form one flat sequence that runs through
// a two-deep software pipeline: a batch of 8 loads is always in flight behind the one being accumulated,
// also across chunk boundaries.  fp32 FMA in ascending channel order.  finish(c, acc) is called with the
// 8 sums of chunk c.  No barrier.
// Addressing: chunk c of channel row j lies at Kt_head + j * row_bytes + c * chunk_bytes.  The S-contiguous
// key copy has row_bytes = 2 S_max and chunk_bytes = 16; the tiled single-copy layout (tiles of 8 positions,
// channel-major inside a tile) has row_bytes = 16 and chunk_bytes = 16 d_h.
template <class T, int STRIDE = NT, class Finish>
__device__ __forceinline__ void stream_channel_rows(const char* Kt_head, size_t row_bytes, const int* chan,
                                                    const float* qs, int r, int chunk_begin, int chunk_end,
                                                    int tid, Finish&& finish, uint32_t chunk_bytes = 16u) {
  const int n_batches = (r + 7) >> 3;
  const int n_chunks = chunk_end - chunk_begin;
  const int my_chunks = n_chunks > tid ? (n_chunks - tid + STRIDE - 1) / STRIDE : 0;
  const int items = my_chunks * n_batches;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int ic = 0, ib = 0, cc = 0, cb = 0;   // issue and consume cursors: (own chunk number, batch)
  auto issue_next = [&](uint4 (&v)[8]) {
    const uint32_t voff = (uint32_t)(chunk_begin + tid + ic * STRIDE) * chunk_bytes;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int ch = __builtin_amdgcn_readfirstlane(chan[ib * 8 + t]);   // uniform: scalar row base
      v[t] = load16(Kt_head + (size_t)ch * row_bytes + voff);
    }
    if (++ib == n_batches) { ib = 0; ++ic; }
  };
  auto consume_next = [&](const uint4 (&v)[8]) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float qv = qs[cb * 8 + t];
      float f[8];
      unpack8<T>(v[t], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(f[e], qv, acc[e]);
    }
    if (++cb == n_batches) {
      finish(chunk_begin + tid + cc * STRIDE, acc);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
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

// ------------------------------------------------------------------------------------------------
// The newest S mod 8 keys of a sequence.  The S-contiguous copy Kt is brought up to date 8 positions at
// a time (one aligned 16-byte store per channel row every 8th append, instead of a 2-byte store per
// channel on every append: those cost a 32-byte memory transaction each).  Positions 8 floor(S/8) .. S-1
// therefore are not in Kt yet; there are at most 7 of them and their approximate logit numerators come
// from the rows of K: wave w takes position 8 floor(S/8) + w, lane l the channels l, l + 64, ... of the
// padded list.  The loads are issued before Step 1b streams Kt and used after it.
struct TailRow {
  uint16_t raw[4];   // up to 256 list entries over 64 lanes
};

__device__ __forceinline__ TailRow tail_row_issue(const uint16_t* krow, const int* chan, int r8, int lane) {
  TailRow t;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int jj = lane + i * kWave;
    t.raw[i] = jj < r8 ? krow[chan[jj]] : (uint16_t)0;
  }
  return t;
}

template <class T>
__device__ __forceinline__ float tail_row_dot(const TailRow& t, const float* qs, int r8, int lane) {
  float part = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int jj = lane + i * kWave;
    if (jj < r8) part = fmaf(T::widen(t.raw[i]), qs[jj], part);
  }
  return wave_sum(part);
}

// Positions S-8 .. S-1 of channel j of one KV head, S a multiple of 8, as 16 bytes: rows S-8 .. S-2 of
// K_head (cached by earlier calls) and `newest`, the code of the row being appended.
__device__ __forceinline__ uint4 gather_key_columns(const uint16_t* K_head, int d_h, int S, int j, uint16_t newest) {
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const uint32_t lo = K_head[(size_t)(S - 8 + e) * d_h + j];
    const uint32_t hi = e + 1 < 7 ? K_head[(size_t)(S - 8 + e + 1) * d_h + j] : (uint32_t)newest;
    w[e >> 1] = lo | (hi << 16);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}
// ... written as columns S-8 .. S-1 of Kt: one 16-byte store
__device__ __forceinline__ void flush_key_columns(uint16_t* Kt_head, const uint16_t* K_head, int S_stride, int d_h,
                                                  int S, int j, uint16_t newest) {
  // (a non-temporal store: each of these 16 bytes is a line of its own that nothing reads for the next 8 steps; with
  // 2048 KV heads the step is 1-2 % faster, with 512 it is 0.5 % slower)
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const uint4 c = gather_key_columns(K_head, d_h, S, j, newest);
  u32x4 v;
  v.x = c.x; v.y = c.y; v.z = c.z; v.w = c.w;
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(Kt_head + (size_t)j * S_stride + (S - 8)));
}

// ------------------------------------------------------------------------------------------------
// Step 2a: the kq positions with the largest keys (ties to the lower position)

struct SelectLds {
  uint32_t* hist;   // [2][kRadixBins] double-buffered digit histograms (swizzled slots)
  uint32_t* wcnt;   // [2][NW] wave totals of the compaction scan, double-buffered
  int* ctl;         // [8]
  float* red;       // [2 * NW]
};

// Radix select with digits of 11, 11 and 10 bits from the top.  On entry hist[0] holds the counts of
// the first digit of keys[0..S) and hist[1] is zero.  Pass p counts into hist[p & 1] while the other
// buffer is cleared; one wave finds the threshold digit, everyone picks it up after a barrier; the loop
// ends as soon as the remaining bin is taken whole.  On return the selected keys are those with
// (key & pmask) > pval plus the first `need` keys (by position) with (key & pmask) == pval.
// kq = 0 (everything comes from the local window) selects nothing: returns a predicate no key meets.
__device__ __forceinline__ void radix_select(const uint32_t* keys, int S, int kq, const SelectLds& sl,
                                             int tid, int lane, int wave, uint32_t& pmask, uint32_t& pval, int& need) {
  const int n_chunks = (S + 7) >> 3;
  if (kq == 0) { pmask = 0xffffffffu; pval = 0xffffffffu; need = 0; return; }
  pmask = 0u; pval = 0u; need = kq;
  int in_bin = 0;          // keys in the bin decided by the previous pass
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const uint32_t dmask = pass == 2 ? 0x3ffu : 0x7ffu;
    uint32_t* hist = sl.hist + (pass & 1) * kRadixBins;
    if (pass > 0) {
      uint32_t* other = sl.hist + ((pass + 1) & 1) * kRadixBins;   // free since the last barrier
      for (int i = tid; i < kRadixBins; i += NT) other[i] = 0u;
      if (in_bin <= kTieHeavy) {
        for (int c = tid; c < n_chunks; c += NT) {
          const uint4* src = reinterpret_cast<const uint4*>(keys + c * 8);
          const uint4 lo = src[0], hi = src[1];
          const uint32_t kx[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (c * 8 + e < S && (kx[e] & pmask) == pval) atomicAdd(&hist[hist_slot((kx[e] >> shift) & dmask)], 1u);
        }
      } else {
        // thousands of keys share the decided bits (duplicated keys, underflowed scores): they may share the next
        // digit too, and plain atomics on one address would take microseconds; count per wave first
        for (int c0 = 0; c0 < n_chunks; c0 += NT) {
          const int c = c0 + tid;
          const bool on = c < n_chunks;
          const uint4* src = reinterpret_cast<const uint4*>(keys + (on ? c : 0) * 8);
          const uint4 lo = src[0], hi = src[1];
          const uint32_t kx[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            hist_add_ties(hist, (kx[e] >> shift) & dmask, on && c * 8 + e < S && (kx[e] & pmask) == pval, lane);
        }
      }
      __syncthreads();
    }
    if (wave == 0) find_threshold_bin(hist, need, lane, sl.ctl);
    __syncthreads();
    pval |= (uint32_t)sl.ctl[0] << shift;
    pmask |= dmask << shift;
    need = sl.ctl[1];
    in_bin = sl.ctl[2];
    if (need == in_bin) break;   // every key matching the decided bits is taken: no ties to split
  }
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

// Ordered compaction of the selected positions into list[0..kq) (ascending) and
// alpha = (sum over the selected of exp((d - dmax)/tau)) / (sum over all): Step 3's weight.
// A lane owns up to 4 consecutive chunks per sweep (the chunks of a sweep are dealt out evenly), so lane order is
// position order and one workgroup scan of the packed (above-threshold, equal-to-threshold) counts orders a whole
// sweep of up to 32 NT positions: one barrier for lengths up to 16 384, whatever the length is a multiple of.  (Sweeps of NT chunks,
// one per lane, needed ceil(S / 4096) scans, and a last sweep of a few chunks still cost 0.5 us of one wave's
// dependent arithmetic: 3-4 us per launch at a length just above a multiple of 4096 with 2048 heads.)
// Before the scan a lane reads its keys and sums the softmax weights: of all keys, of the keys above the
// threshold (taken for sure), and of the keys equal to it on the decided bits; after it only the positions are
// written, from two bit masks.  Which of the equal keys are taken (the first `need` by position) does not matter
// for the sums: either all of them are (the select stopped early because the whole bin is taken), or all 32 bits
// are decided and they share one weight.
// `list` may be the key array itself: the list overwrites it from the front; a write never lands beyond the
// position it records and all reads of a sweep precede its writes (the scan's barrier).  With key_out the keys
// are read again after the scan: list must then be another array.
// Ends with a barrier that also publishes the list.  esc = log2(e) / tau.  With WITH_ALPHA = false only
// the list is produced (the grouped-query kernel gets alpha per query head elsewhere) and 0 is returned.
// Positions >= forced_from (the local window) are taken whatever their keys; the predicate applies to
// the positions before them.  Optional: key_out[n] receives the key of the n-th selected entry, the
// entries written to list / idx_out are offset by pos_base, sums_out[0..1] receive the denominator and the
// numerator of alpha.
template <bool WITH_ALPHA = true>
__device__ __forceinline__ float compact_selected(const uint32_t* keys, uint32_t* list, int S, int forced_from,
                                                  uint32_t pmask, uint32_t pval, int need, float dmax, float esc,
                                                  int32_t* idx_out, int idx_stride, const SelectLds& sl, int tid,
                                                  int lane, int wave, uint32_t* key_out = nullptr, int pos_base = 0,
                                                  float* sums_out = nullptr) {
  const int n_chunks = (S + 7) >> 3;
  float zsum = 0.0f, asum = 0.0f, esum = 0.0f;
  uint32_t run_gt = 0, run_eq = 0;
  int sweep = 0;
  for (int c0 = 0; c0 < n_chunks; c0 += 4 * NT, ++sweep) {
    // the chunks of this sweep dealt out evenly, in order: the first `rem` lanes take one more than the others
    const int n_here = n_chunks - c0 < 4 * NT ? n_chunks - c0 : 4 * NT;
    const int per = n_here / NT, rem = n_here - per * NT;
    const int cb = c0 + tid * per + (tid < rem ? tid : rem);   // the lane's first chunk of this sweep
    const int mine = per + (tid < rem ? 1 : 0);
    uint32_t gt_bits = 0, eq_bits = 0;           // bit 8 i + e: key e of the lane's i-th chunk
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = cb + i;
      if (i < mine) {
        const uint4* src = reinterpret_cast<const uint4*>(keys + c * 8);
        const uint4 lo = src[0], hi = src[1];
        const uint32_t kx[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const bool valid = (c * 8 + e) < S;
          const bool old = (c * 8 + e) < forced_from;
          const uint32_t hi_bits = kx[e] & pmask;
          const bool g = valid && (hi_bits > pval || !old), q = valid && old && hi_bits == pval;
          gt_bits |= (uint32_t)g << (8 * i + e); eq_bits |= (uint32_t)q << (8 * i + e);
          if (WITH_ALPHA) {
            const float w = exp2_weight((key_to_float(kx[e]) - dmax) * esc);
            zsum += valid ? w : 0.0f;
            asum += g ? w : 0.0f;
            esum += q ? w : 0.0f;
          }
        }
      }
    }
    uint32_t total;
    const uint32_t ex = block_scan_excl((uint32_t)__popc(gt_bits) | ((uint32_t)__popc(eq_bits) << 16),
                                        sl.wcnt + (sweep & 1) * NW, lane, wave, &total);
    const uint32_t gt_before = run_gt + (ex & 0xffffu);
    const uint32_t eq_before = run_eq + (ex >> 16);
    uint32_t o = gt_before + (eq_before < (uint32_t)need ? eq_before : (uint32_t)need);
    // the taken keys of this lane: everything above the threshold and the first equal keys while they are needed
    uint32_t take_bits = gt_bits;
    if (eq_bits) {
      uint32_t eb = eq_bits;
      for (int room = need - (int)eq_before; eb && room > 0; --room) {
        const uint32_t low = eb & (0u - eb);
        take_bits |= low; eb ^= low;
      }
    }
    for (uint32_t tb = take_bits; tb; tb &= tb - 1) {
      const int at = cb * 8 + (__ffs(tb) - 1);
      list[o] = (uint32_t)(pos_base + at);
      if (key_out) key_out[o] = keys[at];
      if (idx_out && (int)o < idx_stride) idx_out[o] = pos_base + at;
      ++o;
    }
    run_gt += total & 0xffffu;
    run_eq += total >> 16;
  }
  if (!WITH_ALPHA) {
    __syncthreads();
    return 0.0f;
  }
  // run_eq is now the number of equal keys in the whole array, the same in every thread
  const bool all_equal_taken = (uint32_t)need >= run_eq;
  if (all_equal_taken) asum += esum;
  zsum = wave_sum(zsum); asum = wave_sum(asum);
  if (lane == 0) { sl.red[wave] = zsum; sl.red[NW + wave] = asum; }
  __syncthreads();
  float zt = 0.0f, at = 0.0f;
#pragma unroll
  for (int w = 0; w < NW; ++w) { zt += sl.red[w]; at += sl.red[NW + w]; }
  if (!all_equal_taken) at += (float)need * exp2_weight((key_to_float(pval) - dmax) * esc);
  if (sums_out) { sums_out[0] = zt; sums_out[1] = at; }
  return at / zt;
}

// ------------------------------------------------------------------------------------------------
// Step 2b: exact softmax attention over gathered rows (Eq. 8), online softmax in the exp2 domain

template <int DH>
struct RowGeometry {
  static constexpr int LPR = DH / 8;          // lanes per row (16 bytes each)
  static constexpr int RPW = kWave / LPR;     // rows per wave per load
  static constexpr int RPI = NW * RPW;        // rows per workgroup per load
  static constexpr int UNR = 4;
  static constexpr int GROUP = RPI * UNR;     // rows the workgroup covers per group of loads
};

// Rows list[n_begin..n_end) of K and V (K_head / V_head already offset by the lane's 16-byte column
// slice `sub`).  LPR lanes share a row, K and V rows are issued together, groups of UNR loads run
// through a two-deep software pipeline.  q8 = the lane's 8 query components times log2(e)/sqrt(d_h).
// Accumulates into (m_run, l_run, acc).  No barrier.
// TILED: the keys come from the tiled single-copy layout instead: K_head is the head's first tile (tiles of
// 8 positions, channel-major inside a tile: element (position p, channel j) at ((p / 8) d_h + j) 8 + p % 8),
// so a lane's 8 channels of one position are eight 2-byte loads 16 bytes apart; positions from tiled_below on
// (the up to 7 newest, not yet in a tile) are rows of K_stage (row p - tiled_below, already offset by `sub`).
template <class T, int DH, bool TILED = false>
__device__ __forceinline__ void attend_rows(const char* K_head, const char* V_head, const int* list, int n_begin,
                                            int n_end, const float (&q8)[8], int lane, int wave, float& m_run,
                                            float& l_run, float (&acc)[8], const char* K_stage = nullptr,
                                            int tiled_below = 0) {
  using G = RowGeometry<DH>;
  const int slot = wave * G::RPW + lane / G::LPR;
  const int n_groups = (n_end - n_begin + G::GROUP - 1) / G::GROUP;
  auto issue = [&](uint4 (&kr)[G::UNR], uint4 (&vr)[G::UNR], int g) {
#pragma unroll
    for (int t = 0; t < G::UNR; ++t) {
      const int n = n_begin + g * G::GROUP + t * G::RPI + slot;
      const int p = list[n < n_end ? n : n_end - 1];
      const uint32_t off = (uint32_t)p * (uint32_t)(DH * 2);   // < S_max * 512 bytes
      if (!TILED) {
        kr[t] = load16(K_head + off);
      } else if (p >= tiled_below) {
        kr[t] = load16(K_stage + (uint32_t)(p - tiled_below) * (uint32_t)(DH * 2));
      } else {
        const uint16_t* tp = reinterpret_cast<const uint16_t*>(K_head) +
                             ((size_t)(p >> 3) * DH + (lane % G::LPR) * 8) * 8 + (p & 7);
        const uint32_t c0 = tp[0], c1 = tp[8], c2 = tp[16], c3 = tp[24], c4 = tp[32], c5 = tp[40], c6 = tp[48], c7 = tp[56];
        kr[t] = make_uint4(c0 | (c1 << 16), c2 | (c3 << 16), c4 | (c5 << 16), c6 | (c7 << 16));
      }
      vr[t] = load16(V_head + off);
    }
  };
  auto consume = [&](const uint4 (&kr)[G::UNR], const uint4 (&vr)[G::UNR], int g) {
#pragma unroll
    for (int t = 0; t < G::UNR; ++t) {
      const int n = n_begin + g * G::GROUP + t * G::RPI + slot;
      float f[8];
      unpack8<T>(kr[t], f);
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(f[e], q8[e], dot);
      dot = lanes_sum<G::LPR>(dot);
      if (n < n_end) {
        const float m_new = fmaxf(m_run, dot);
        const float sc = exp2_weight(m_run - m_new), pr = exp2_weight(dot - m_new);
        unpack8<T>(vr[t], f);
        l_run = l_run * sc + pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * sc + pr * f[e];
        m_run = m_new;
      }
    }
  };
  if (n_groups > 0) {
    uint4 ka[G::UNR], va[G::UNR], kb[G::UNR], vb[G::UNR];
    issue(ka, va, 0);
    int g = 0;
    for (; g + 2 < n_groups; g += 2) {
      issue(kb, vb, g + 1);
      consume(ka, va, g);
      issue(ka, va, g + 2);
      consume(kb, vb, g + 1);
    }
    if (g + 1 < n_groups) {
      issue(kb, vb, g + 1);
      consume(ka, va, g);
      consume(kb, vb, g + 1);
    } else {
      consume(ka, va, g);
    }
  }
}

// One more row, given as 16-bit codes in LDS (the row a decode step appends), folded into the state of
// the lane group with slot 0.  Executed by all lanes; no barrier.
template <class T, int DH>
__device__ __forceinline__ void attend_row_from_codes(const uint16_t* krow, const uint16_t* vrow, const float (&q8)[8],
                                                      int lane, int wave, float& m_run, float& l_run, float (&acc)[8]) {
  using G = RowGeometry<DH>;
  const int sub = lane % G::LPR;
  float f[8];
  unpack8<T>(*reinterpret_cast<const uint4*>(krow + sub * 8), f);
  float dot = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; ++e) dot = fmaf(f[e], q8[e], dot);
  dot = lanes_sum<G::LPR>(dot);
  if (wave == 0 && lane < G::LPR) {
    const float m_new = fmaxf(m_run, dot);
    const float sc = exp2_weight(m_run - m_new), pr = exp2_weight(dot - m_new);
    unpack8<T>(*reinterpret_cast<const uint4*>(vrow + sub * 8), f);
    l_run = l_run * sc + pr;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = acc[e] * sc + pr * f[e];
    m_run = m_new;
  }
}

// Merge the lane groups of a wave (butterfly over the group index) and store the wave's partial
// (acc[DH], m, l) to part[wave][DH + 2].  The caller puts a barrier after it.
template <int DH>
__device__ __forceinline__ void store_wave_partial(float m_run, float l_run, float (&acc)[8], float* part, int lane, int wave) {
  using G = RowGeometry<DH>;
#pragma unroll
  for (int o = G::LPR; o < kWave; o <<= 1) {
    const float m_o = __shfl_xor(m_run, o), l_o = __shfl_xor(l_run, o);
    const float m_new = fmaxf(m_run, m_o);
    const float s1 = weight_exp2(m_run, m_new), s2 = weight_exp2(m_o, m_new);
    l_run = l_run * s1 + l_o * s2;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = acc[e] * s1 + __shfl_xor(acc[e], o) * s2;
    m_run = m_new;
  }
  float* mine = part + wave * (DH + 2);
  if (lane < G::LPR) {
#pragma unroll
    for (int e = 0; e < 8; ++e) mine[lane * 8 + e] = acc[e];
    if (lane == 0) { mine[DH] = m_run; mine[DH + 1] = l_run; }
  }
}

// Channel c of the merge of n_parts partials laid out [n_parts][DH + 2]: running max, denominator and
// un-normalised numerator (each partial's numerator and denominator are relative to its own max).
template <int DH>
__device__ __forceinline__ void combine_partials(const float* parts, int n_parts, int c, float& m_all, float& l_all, float& y) {
  m_all = -INFINITY;
  for (int w = 0; w < n_parts; ++w) m_all = fmaxf(m_all, parts[w * (DH + 2) + DH]);
  l_all = 0.0f; y = 0.0f;
  for (int w = 0; w < n_parts; ++w) {
    const float s = weight_exp2(parts[w * (DH + 2) + DH], m_all);
    l_all += parts[w * (DH + 2) + DH + 1] * s;
    y += parts[w * (DH + 2) + c] * s;
  }
}

}  // namespace sparq
