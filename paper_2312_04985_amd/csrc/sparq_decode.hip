// SparQ decode, one workgroup per (sequence, query head): Section 4, Steps 1-3, in one launch with
// no intermediate HBM traffic.
//   stage 0  top-r of |q| and the temperature (Eq. 9)
//   stage 1  stream the r selected rows of the S-contiguous key copy; the fp32 approximate logit
//            numerators of all cached positions stay in LDS as order-preserving integer keys and are
//            counted into the first radix histogram as they are produced
//   stage 2  radix select of the k-th largest key, ordered compaction of the selected positions
//            (ties to the lower position), alpha = selected share of the approximate softmax mass
//   stage 3  gather the selected K and V rows, online-softmax exact attention, blend with the
//            mean value vector (Eq. 10), round and store
#include "decode_stages.h"

namespace sparq {

namespace {

// A SPARQ_STAGE_CLOCKS build (a second library for profiling, never the default one) keeps nine time stamps per
// workgroup in scalar registers and stores them when the workgroup ends; otherwise the macro is empty.
#ifdef SPARQ_STAGE_CLOCKS
#define SPARQ_STAMP(i) stamp[i] = wall_clock64()
#else
#define SPARQ_STAMP(i) do {} while (0)
#endif


struct Lds {
  uint32_t* keys;   // [S_max]   stage 1-2: keys; after compaction: selected positions
  SelectLds sel;
  QueryLds qry;
  float* part;      // [NW * (DH + 2)] stage-3 partials; stage 0: partial ranks (NT words)
  uint16_t* knew;   // [DH] codes of the key row being appended (one-launch step only)
  uint16_t* vnew;   // [DH]
};

template <int DH>
__device__ __forceinline__ Lds carve(uint32_t* base, int S_max) {
  Lds l;
  l.keys = base; base += S_max;
  l.sel.hist = base; base += 2 * kRadixBins;
  l.part = reinterpret_cast<float*>(base);
  l.qry.rankp = reinterpret_cast<int*>(base); base += NW * (DH + 2);
  l.qry.qf = reinterpret_cast<float*>(base); base += DH;
  l.qry.qs = reinterpret_cast<float*>(base); base += DH;
  l.qry.chan = reinterpret_cast<int*>(base); base += DH;
  l.qry.mag = base; base += DH;
  l.sel.red = reinterpret_cast<float*>(base); base += 32;
  l.sel.wcnt = base; base += 16;
  l.sel.ctl = reinterpret_cast<int*>(base); base += 8;
  l.knew = reinterpret_cast<uint16_t*>(base); base += DH / 2;
  l.vnew = reinterpret_cast<uint16_t*>(base);
  return l;
}

// APPEND = true is the one-launch decode step: the new key/value row of every KV head (k_new, v_new)
// counts as position S_b of its sequence without being read back from the cache.  Every workgroup
// takes that row from the inputs; the workgroup of the first query head of a KV group also writes
// it into K, V and Kt and stores the updated mean; lengths and means go to the *_next buffers, so no
// workgroup can observe another one's update of the state it reads.
// TILED = true reads the single-copy tiled key layout (flag bit 6): a.K holds tiles of 8 positions, channel-major
// inside a tile, a.Kt the up to 7 newest rows of every KV head (8 rows of d_h each) that do not fill a tile yet.
// Step 1b then strides through the tiles (16 bytes per position chunk and channel), Step 2b collects a row's
// components from its tile, and the append writes a row of the small buffer, or a whole tile with the eighth row.
template <class T, int DH, bool APPEND, bool TILED>
__global__ __launch_bounds__(NT, 4) void sparq_decode_fused(const DecodeArgs a) {
  extern __shared__ __align__(16) uint32_t smem[];
  const Lds L = carve<DH>(smem, a.S_max);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

#ifdef SPARQ_STAGE_CLOCKS
  unsigned long long stamp[kStageStamps];
#endif
  SPARQ_STAMP(0);
  // Workgroup -> unit.  Workgroups are dealt round-robin to the 8 XCDs and started in index order.
  // Default: every XCD gets a contiguous run of units, so the query heads of a KV group share an L2.
  // With the ragged-batch hint (and no grouped heads): workgroup i serves the sequence with the
  // (i / H)-th largest length, so the longest sequences start first and the short ones fill in behind.
  const int U = a.B * a.H;
  int u = blockIdx.x;
  if ((a.flags & 4u) && a.H == a.H_kv && a.B > 1 && a.B <= NT) {
    int* lens = reinterpret_cast<int*>(L.keys);   // free until stage 1
    if (tid < a.B) lens[tid] = a.seq_lens[tid];
    __syncthreads();
    if (tid < a.B) {
      const int mine = lens[tid];
      int rank = 0;
      for (int j = 0; j < a.B; ++j) rank += (lens[j] > mine) || (lens[j] == mine && j < tid);
      if (rank == u / a.H) L.sel.ctl[7] = tid;
    }
    __syncthreads();
    u = L.sel.ctl[7] * a.H + u % a.H;
  } else if ((U & 7) == 0) {
    u = (u & 7) * (U >> 3) + (u >> 3);
  }
  u = __builtin_amdgcn_readfirstlane(u);   // the same in every lane (also where it came through LDS): keep what follows scalar
  const int b = u / a.H, h = u - b * a.H;
  const int hk = h / (a.H / a.H_kv);
  const size_t kv_head = (size_t)b * a.H_kv + hk;

  // everything the unit reads from small tensors is requested here, in one round trip; the mean value
  // vector is only needed for the blend at the very end
  uint16_t qcode = 0, kcode = 0, vcode = 0;
  float vm = 0.0f;
  if (tid < DH) {
    qcode = reinterpret_cast<const uint16_t*>(a.q)[(size_t)u * DH + tid];
    vm = a.v_mean[kv_head * DH + tid];
    if (APPEND) {
      kcode = reinterpret_cast<const uint16_t*>(a.k_new)[kv_head * DH + tid];
      vcode = reinterpret_cast<const uint16_t*>(a.v_new)[kv_head * DH + tid];
    }
  }
  int S = a.seq_lens[b];
  // a length beyond the bound of this call that the buffers can hold is carried over as it is (clamped only here)
  const int S_kept = (S > a.S_max && S <= a.S_stride) ? S : -1;
  if (S < 0 || S > a.S_max) {
    if (tid == 0) atomicOr(a.err, 8);
    S = S < 0 ? 0 : a.S_max;
  }
  bool appended = false;                                    // this sequence takes the new row (uniform)
  const bool owner = APPEND && h == hk * (a.H / a.H_kv);   // writes the row and the new mean
  if (APPEND) {
    if (S + 1 <= a.S_max) { appended = true; S += 1; }
    else if (tid == 0) atomicOr(a.err, 1);
    if (h == 0 && tid == 0) a.seq_lens_next[b] = S_kept >= 0 ? S_kept : S;
  }
  int kb = a.k_per_seq ? a.k_per_seq[b] : a.k;
  kb = kb < 1 ? 1 : (kb > a.k ? a.k : kb);
  const int kq = kb < S ? kb : S;

  uint16_t* out = reinterpret_cast<uint16_t*>(a.out) + (size_t)u * DH;
  int32_t* idx_out = a.idx_out ? a.idx_out + (size_t)u * a.idx_stride : nullptr;
  if (S == 0) {   // nothing cached: defined output, raise the flag
    if (tid < DH) out[tid] = 0;
    if (tid == 0) { atomicOr(a.err, 2); if (a.alpha_out) a.alpha_out[u] = 0.0f; }
    if (a.chan_out && tid < a.r) a.chan_out[(size_t)u * a.r + tid] = -1;
    if (idx_out) for (int n = tid; n < a.idx_stride; n += NT) idx_out[n] = -1;
    if (owner && tid < DH) a.v_mean_next[kv_head * DH + tid] = vm;
    return;
  }
  if (APPEND && appended && tid < DH) {   // same update as append_one_row; the mean of no rows is ignored
    if (S == 1) vm = 0.0f;
    vm += (T::widen(vcode) - vm) * (1.0f / (float)S);
  }

  // ---------------- stage 0 ----------------
  for (int i = tid; i < 2 * kRadixBins; i += NT) L.sel.hist[i] = 0u;
  if (APPEND && tid < DH) { L.knew[tid] = kcode; L.vnew[tid] = vcode; }
  const float tau = apply_tau_mode(select_channels<T, DH>(L.qry, qcode, a.r, tid, lane, wave), a.flags, DH, a.r);
  const Window win = make_window(a.local_window, S, kq);
  if (tid < DH) L.qry.mag[tid] = __float_as_uint(vm);   // parked in LDS until the blend (the ranking keys are dead)
  if (a.chan_out && tid < a.r) a.chan_out[(size_t)u * a.r + tid] = L.qry.chan[tid];
  // the newest S mod 8 positions are not in Kt: wave w gets position S_fl + w from its K row (from the
  // inputs if it is the row being appended); loads issued here, used after stage 1
  // (in the one-launch step Kt is up to date for the length before this call: the group of 8 that the new
  // row may complete is written during this launch, so up to 8 positions come from rows)
  const int S_fl = ((APPEND && appended) ? S - 1 : S) & ~7, n_tail = S - S_fl, r8 = (a.r + 7) & ~7;
  // rows of K by position (two-copy layout), or the rows of the newest positions S_fl .. (tiled layout)
  const uint16_t* K_rows = TILED ? reinterpret_cast<const uint16_t*>(a.Kt) + kv_head * (size_t)(8 * DH) - (size_t)S_fl * DH
                                 : reinterpret_cast<const uint16_t*>(a.K) + kv_head * a.S_stride * (size_t)DH;
  TailRow tail;
  const bool tail_is_new = APPEND && appended && wave == n_tail - 1;
  if (wave < n_tail) {
    if (tail_is_new) tail = tail_row_issue(L.knew, L.qry.chan, r8, lane);
    else tail = tail_row_issue(K_rows + (size_t)(S_fl + wave) * DH, L.qry.chan, r8, lane);
  }

  SPARQ_STAMP(1);
  // ---------------- stage 1 ----------------
  const size_t row_bytes = TILED ? 16 : (size_t)a.S_stride * 2;
  const char* Kt_head = TILED ? reinterpret_cast<const char*>(a.K) + kv_head * a.S_stride * (size_t)(DH * 2)
                              : reinterpret_cast<const char*>(a.Kt) + kv_head * DH * row_bytes;
  float tmax = -INFINITY;
  auto finish = [&](int c, const float (&acc)[8]) {
    uint32_t kx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      tmax = fmaxf(tmax, acc[e]);
      kx[e] = float_to_key(acc[e]);
    }
    hist_add_chunk(L.sel.hist, kx, win.S_old - c * 8);
    uint4* dst = reinterpret_cast<uint4*>(L.keys + c * 8);
    dst[0] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
    dst[1] = make_uint4(kx[4], kx[5], kx[6], kx[7]);
  };
  stream_channel_rows<T>(Kt_head, row_bytes, L.qry.chan, L.qry.qs, a.r, 0, S_fl >> 3, tid, finish, TILED ? DH * 16u : 16u);
  if (wave < n_tail) {
    const float dot = tail_row_dot<T>(tail, L.qry.qs, r8, lane);
    tmax = fmaxf(tmax, dot);
    if (lane == 0) {
      const uint32_t key = float_to_key(dot);
      L.keys[S_fl + wave] = key;
      if (S_fl + wave < win.S_old) atomicAdd(&L.sel.hist[hist_slot(key >> 21)], 1u);
    }
  }
  SPARQ_STAMP(2);
  tmax = wave_max(tmax);
  if (lane == 0) L.sel.red[wave] = tmax;
  __syncthreads();
  SPARQ_STAMP(3);
  float dmax = L.sel.red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, L.sel.red[w]);

  // ---------------- stage 2 ----------------
  uint32_t pmask, pval;
  int need;
  radix_select(L.keys, win.S_old, win.k_old, L.sel, tid, lane, wave, pmask, pval, need);
  SPARQ_STAMP(4);
  const float alpha = compact_selected(L.keys, L.keys, S, win.S_old, pmask, pval, need, dmax, kLog2e / tau, idx_out, a.idx_stride,
                                       L.sel, tid, lane, wave);
  SPARQ_STAMP(5);
  if (tid == 0) {
    if (a.alpha_out) a.alpha_out[u] = alpha;
    if (idx_out && kq > a.idx_stride) atomicOr(a.err, 4);
  }
  if (idx_out) for (int n = kq + tid; n < a.idx_stride; n += NT) idx_out[n] = -1;

  // ---------------- stage 3 ----------------
  using G = RowGeometry<DH>;
  const int sub = lane % G::LPR;
  const int* list = reinterpret_cast<const int*>(L.keys);
  const char* K_head = reinterpret_cast<const char*>(a.K) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const char* V_head = reinterpret_cast<const char*>(a.V) + kv_head * a.S_stride * (size_t)(DH * 2) + sub * 16;
  const float qscale = kLog2e / sqrtf((float)DH);
  float q8[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q8[e] = L.qry.qf[sub * 8 + e] * qscale;
  // positions are ascending, so the appended row (position S - 1) can only be the last entry; it is
  // not read back from the cache but taken from the inputs
  const bool new_selected = APPEND && appended && list[kq - 1] == S - 1;
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (TILED)
    attend_rows<T, DH, true>(Kt_head, V_head, list, 0, new_selected ? kq - 1 : kq, q8, lane, wave, m_run, l_run, acc,
                             reinterpret_cast<const char*>(K_rows + (size_t)S_fl * DH) + sub * 16, S_fl);
  else
    attend_rows<T, DH>(K_head, V_head, list, 0, new_selected ? kq - 1 : kq, q8, lane, wave, m_run, l_run, acc);
  if (APPEND && new_selected) attend_row_from_codes<T, DH>(L.knew, L.vnew, q8, lane, wave, m_run, l_run, acc);
  SPARQ_STAMP(6);
  store_wave_partial<DH>(m_run, l_run, acc, L.part, lane, wave);
  __syncthreads();
  SPARQ_STAMP(7);
  if (tid < DH) {
    float m_all, l_all, y3;
    combine_partials<DH>(L.part, NW, tid, m_all, l_all, y3);
    y3 /= l_all;
    float y = y3;
    if (!(a.flags & 1u)) y = alpha * y3 + (1.0f - alpha) * __uint_as_float(L.qry.mag[tid]);
    out[tid] = T::narrow(y);
  }
  if (APPEND && owner && tid < DH) {
    // The append's stores come last.  (Measured at five places of the kernel: in front of stage 0 they sit
    // on the critical path of every wait that follows, because a wait for a load also waits for the stores
    // issued before it; after Step 1b, after the select, after the compaction and here cost the same within
    // noise when workgroups come in several rounds, and here is best when they all run at once.)  Nobody
    // reads row S - 1 of K or V in this launch (every head takes it from k_new / v_new), the new mean goes to
    // the *_next buffer, and the columns written to Kt lie above S_fl for every head of the group.
    a.v_mean_next[kv_head * DH + tid] = __uint_as_float(L.qry.mag[tid]);
    if (appended) {
      const uint16_t kc = L.knew[tid];
      reinterpret_cast<uint16_t*>(a.V)[(kv_head * a.S_stride + (S - 1)) * DH + tid] = L.vnew[tid];
      if (!TILED) {
        reinterpret_cast<uint16_t*>(a.K)[(kv_head * a.S_stride + (S - 1)) * DH + tid] = kc;
        // a step that completes a group of 8 positions copies it to Kt (one 16-byte store per channel row)
        if ((S & 7) == 0)
          flush_key_columns(reinterpret_cast<uint16_t*>(a.Kt) + kv_head * DH * (size_t)a.S_stride, K_rows, a.S_stride, DH, S, tid, kc);
      } else if ((S & 7) != 0) {
        const_cast<uint16_t*>(K_rows)[(size_t)(S - 1) * DH + tid] = kc;        // row (S - 1) mod 8 of the small buffer
      } else {
        // the eighth row completes a tile: channel tid's 8 positions are 16 contiguous bytes of it
        const uint4 cols = gather_key_columns(K_rows, DH, S, tid, kc);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.K) + (kv_head * a.S_stride + (size_t)(S - 8)) * DH + (size_t)tid * 8) = cols;
      }
    }
  }
#ifdef SPARQ_STAGE_CLOCKS
  SPARQ_STAMP(8);
  if (a.clocks && tid == 0)
    for (int i = 0; i < kStageStamps; ++i) a.clocks[(size_t)blockIdx.x * kStageStamps + i] = stamp[i];
#endif
}

template <class T, int DH, bool APPEND, bool TILED>
hipError_t launch_one(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = decode_lds_bytes(a.S_max, DH);
  auto kern = sparq_decode_fused<T, DH, APPEND, TILED>;
  hipError_t e = allow_lds<sparq_decode_fused<T, DH, APPEND, TILED>>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(a.B * a.H), dim3(NT), lds, s, a);
  return hipGetLastError();
}

template <bool APPEND, bool TILED>
hipError_t launch_any(const DecodeArgs& a, int dtype, hipStream_t s) {
  const bool bf = dtype == 1;
  switch (a.d_h) {
    case 64:  return bf ? launch_one<BF16, 64, APPEND, TILED>(a, s) : launch_one<F16, 64, APPEND, TILED>(a, s);
    case 128: return bf ? launch_one<BF16, 128, APPEND, TILED>(a, s) : launch_one<F16, 128, APPEND, TILED>(a, s);
    case 256: return bf ? launch_one<BF16, 256, APPEND, TILED>(a, s) : launch_one<F16, 256, APPEND, TILED>(a, s);
    default:  return hipErrorInvalidValue;
  }
}

}  // namespace

size_t decode_lds_bytes(int S_max, int d_h) {
  return 4 * ((size_t)S_max + 2 * kRadixBins + (size_t)NW * (d_h + 2) + 5 * (size_t)d_h + 32 + 16 + 8);
}

hipError_t launch_decode(const DecodeArgs& a, int dtype, hipStream_t s) {
  if (a.flags & 64u) return a.k_new ? launch_any<true, true>(a, dtype, s) : launch_any<false, true>(a, dtype, s);
  return a.k_new ? launch_any<true, false>(a, dtype, s) : launch_any<false, false>(a, dtype, s);
}

}  // namespace sparq
