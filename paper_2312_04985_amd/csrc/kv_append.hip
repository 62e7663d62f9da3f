// Cache maintenance: append key/value rows, keep the S-contiguous key copy and the running
// mean value vector in step (Section 3 "Mean value reallocation"; Appendix F "Storing K twice").
#include "decode_stages.h"

namespace sparq {

namespace {

// ---- one row per sequence: the per-token path of the decode loop ----
// One workgroup per sequence so that seq_lens[b] is read by everyone before it is bumped.
// A thread moves one 16-byte chunk (8 channels) of one KV head at a time.
template <class T>
__global__ __launch_bounds__(512) void append_one_row(const AppendArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int S = a.seq_lens[b];
  int n = a.n_new_per_seq ? a.n_new_per_seq[b] : 1;
  n = n < 0 ? 0 : (n > 1 ? 1 : n);
  const bool in_place = a.v_mean_out == a.v_mean;
  const bool full = S < 0 || S + 1 > a.S_max;
  if (n == 0 || full) {      // nothing appended: the state is carried over unchanged
    if (full && n != 0 && tid == 0) atomicOr(a.err, 1);
    if (!in_place) {
      for (int i = tid; i < a.H_kv * a.d_h; i += 512) {
        const size_t e = (size_t)b * a.H_kv * a.d_h + i;
        a.v_mean_out[e] = a.v_mean[e];
      }
      if (tid == 0) a.seq_lens_out[b] = S;
    }
    return;
  }
  const int cpr = a.d_h / 8;                  // 16-byte chunks per row
  const int n_chunks = a.H_kv * cpr;
  const float inv = 1.0f / (float)(S + 1);
  for (int c = tid; c < n_chunks; c += 512) {
    const int hk = c / cpr, j0 = (c - hk * cpr) * 8;
    const size_t head = (size_t)b * a.H_kv + hk;
    const uint4 kc = load16(reinterpret_cast<const uint16_t*>(a.k_new) + head * a.d_h + j0);
    const uint4 vc = load16(reinterpret_cast<const uint16_t*>(a.v_new) + head * a.d_h + j0);
    uint16_t* Krow = reinterpret_cast<uint16_t*>(a.K) + (head * a.S_stride + S) * a.d_h + j0;
    uint16_t* Vrow = reinterpret_cast<uint16_t*>(a.V) + (head * a.S_stride + S) * a.d_h + j0;
    *reinterpret_cast<uint4*>(Krow) = kc;
    *reinterpret_cast<uint4*>(Vrow) = vc;
    // the same 8 key elements go down column S of the S-contiguous copy (2-byte stores)
    // the S-contiguous copy advances 8 positions at a time: when this row completes a group of 8, the
    // thread writes columns S-7 .. S of its 8 channels (rows S-7 .. S-1 come back from K)
    if (a.Kt && ((S + 1) & 7) == 0) {   // null: the cache keeps K once
      const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        flush_key_columns(reinterpret_cast<uint16_t*>(a.Kt) + head * a.d_h * (size_t)a.S_stride,
                          reinterpret_cast<const uint16_t*>(a.K) + head * a.S_stride * (size_t)a.d_h, a.S_stride, a.d_h, S + 1,
                          j0 + e, (uint16_t)((e & 1) ? (kw[e >> 1] >> 16) : (kw[e >> 1] & 0xffffu)));
    }
    // running mean: v_mean += (v - v_mean) / (S + 1)
    const float* vm = a.v_mean + head * a.d_h + j0;
    float* vo = a.v_mean_out + head * a.d_h + j0;
    float4 m0 = *reinterpret_cast<const float4*>(vm), m1 = *reinterpret_cast<const float4*>(vm + 4);
    if (S == 0) m0 = m1 = make_float4(0.f, 0.f, 0.f, 0.f);   // the mean of no rows: whatever the buffer held is ignored
    float f[8];
    unpack8<T>(vc, f);
    m0.x += (f[0] - m0.x) * inv; m0.y += (f[1] - m0.y) * inv; m0.z += (f[2] - m0.z) * inv; m0.w += (f[3] - m0.w) * inv;
    m1.x += (f[4] - m1.x) * inv; m1.y += (f[5] - m1.y) * inv; m1.z += (f[6] - m1.z) * inv; m1.w += (f[7] - m1.w) * inv;
    *reinterpret_cast<float4*>(vo) = m0;
    *reinterpret_cast<float4*>(vo + 4) = m1;
  }
  __syncthreads();
  if (tid == 0) a.seq_lens_out[b] = S + 1;
}

// ---- many rows per sequence (prefill / cache construction) ----
// One workgroup per (sequence, KV head); tiles of 64 positions go through LDS to be written
// transposed; value columns are summed in fp64 and folded into the mean once.
constexpr int BT = 256;       // threads
constexpr int TILE = 64;      // positions per tile

template <class T, int DH>
__global__ __launch_bounds__(BT) void append_rows(const AppendArgs a) {
  constexpr int CPR = DH / 8;            // 16-byte chunks per row
  constexpr int RPP = BT / CPR;          // rows per pass
  constexpr int LD = DH + 2;             // padded LDS row (elements): conflict-free column reads
  __shared__ uint16_t tile[TILE * LD];
  __shared__ double colsum[RPP][DH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t head = blockIdx.x;
  const int b = (int)(head / a.H_kv);
  const int S = a.seq_lens[b];
  int n = a.n_new_per_seq ? a.n_new_per_seq[b] : a.n_new;
  n = n < 0 ? 0 : (n > a.n_new ? a.n_new : n);
  if (n == 0) return;
  if (S < 0 || S + n > a.S_max) {
    if (tid == 0) atomicOr(a.err, 1);
    return;
  }
  const int sub = tid % CPR, prow = tid / CPR;
  const uint16_t* ksrc = reinterpret_cast<const uint16_t*>(a.k_new) + head * a.n_new * DH;
  const uint16_t* vsrc = reinterpret_cast<const uint16_t*>(a.v_new) + head * a.n_new * DH;
  uint16_t* Kdst = reinterpret_cast<uint16_t*>(a.K) + (head * a.S_stride + S) * DH;
  uint16_t* Vdst = reinterpret_cast<uint16_t*>(a.V) + (head * a.S_stride + S) * DH;
  uint16_t* Ktdst = reinterpret_cast<uint16_t*>(a.Kt) + head * DH * (size_t)a.S_stride + S;
  double sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int n0 = 0; n0 < n; n0 += TILE) {
    const int rows = (n - n0) < TILE ? (n - n0) : TILE;
    for (int rr = prow; rr < rows; rr += RPP) {
      const size_t off = (size_t)(n0 + rr) * DH + sub * 8;
      const uint4 kc = load16(ksrc + off), vc = load16(vsrc + off);
      *reinterpret_cast<uint4*>(Kdst + off) = kc;
      *reinterpret_cast<uint4*>(Vdst + off) = vc;
      uint32_t* t32 = reinterpret_cast<uint32_t*>(tile + rr * LD + sub * 8);   // LD even: 4-byte aligned
      t32[0] = kc.x; t32[1] = kc.y; t32[2] = kc.z; t32[3] = kc.w;
      float f[8];
      unpack8<T>(vc, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum[e] += (double)f[e];
    }
    __syncthreads();
    if (a.Kt)
      for (int j = wave; j < DH; j += BT / 64)
        if (lane < rows) Ktdst[(size_t)j * a.S_stride + n0 + lane] = tile[lane * LD + j];
    __syncthreads();
  }
  // the up to 7 rows that were cached before this call and not yet in the S-contiguous copy
  if (a.Kt) {
    const int S_fl = S & ~7;
    const uint16_t* Khead = reinterpret_cast<const uint16_t*>(a.K) + head * a.S_stride * (size_t)DH;
    uint16_t* Kthead = reinterpret_cast<uint16_t*>(a.Kt) + head * DH * (size_t)a.S_stride;
    for (int i = tid; i < (S - S_fl) * DH; i += BT) {
      const int e = i / DH, j = i - e * DH;
      Kthead[(size_t)j * a.S_stride + S_fl + e] = Khead[(size_t)(S_fl + e) * DH + j];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) colsum[prow][sub * 8 + e] = sum[e];
  __syncthreads();
  if (tid < DH) {
    double tot = 0.0;
    for (int p = 0; p < RPP; ++p) tot += colsum[p][tid];
    float* vm = a.v_mean + head * DH + tid;
    const double before = S > 0 ? (double)S * (double)*vm : 0.0;   // S = 0: whatever the buffer held is ignored
    *vm = (float)((before + tot) / (double)(S + n));
  }
}

// ---- the tiled single-copy key layout: tiles of 8 positions, channel-major inside a tile ----
// K element (position p, channel j) of a KV head lies at ((p / 8) d_h + j) 8 + p % 8; the rows of the
// positions 8 floor(S / 8) .. S - 1, which do not fill a tile yet, wait in a buffer of 8 rows per KV head
// (AppendArgs::Kt) and move into their tile, as one contiguous block, when the eighth arrives.

// transpose 8 rows x 8 channels of 16-bit codes (rows[e] = the 16 bytes of row e) and store the 8 channels'
// position runs: 128 contiguous bytes at `dst`
__device__ __forceinline__ void store_tile_piece(uint16_t* dst, const uint4 (&rows)[8]) {
  uint32_t w[8][4];
#pragma unroll
  for (int e = 0; e < 8; ++e) { w[e][0] = rows[e].x; w[e][1] = rows[e].y; w[e][2] = rows[e].z; w[e][3] = rows[e].w; }
#pragma unroll
  for (int c = 0; c < 8; ++c) {            // channel c of the piece: positions 0..7
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const uint32_t lo = (c & 1) ? (w[e][c >> 1] >> 16) : (w[e][c >> 1] & 0xffffu);
      const uint32_t hi = (c & 1) ? (w[e + 1][c >> 1] >> 16) : (w[e + 1][c >> 1] & 0xffffu);
      o[e >> 1] = lo | (hi << 16);
    }
    reinterpret_cast<uint4*>(dst)[c] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// one row per sequence: one workgroup per sequence, a thread moves one 16-byte chunk (8 channels) of one KV head
template <class T>
__global__ __launch_bounds__(512) void append_one_row_tiled(const AppendArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int S = a.seq_lens[b];
  int n = a.n_new_per_seq ? a.n_new_per_seq[b] : 1;
  n = n < 0 ? 0 : (n > 1 ? 1 : n);
  const bool in_place = a.v_mean_out == a.v_mean;
  const bool full = S < 0 || S + 1 > a.S_max;
  if (n == 0 || full) {      // nothing appended: the state is carried over unchanged
    if (full && n != 0 && tid == 0) atomicOr(a.err, 1);
    if (!in_place) {
      for (int i = tid; i < a.H_kv * a.d_h; i += 512) {
        const size_t e = (size_t)b * a.H_kv * a.d_h + i;
        a.v_mean_out[e] = a.v_mean[e];
      }
      if (tid == 0) a.seq_lens_out[b] = S;
    }
    return;
  }
  const int cpr = a.d_h / 8;
  const int n_chunks = a.H_kv * cpr;
  const float inv = 1.0f / (float)(S + 1);
  const int slot = S & 7;
  for (int c = tid; c < n_chunks; c += 512) {
    const int hk = c / cpr, j0 = (c - hk * cpr) * 8;
    const size_t head = (size_t)b * a.H_kv + hk;
    const uint4 kc = load16(reinterpret_cast<const uint16_t*>(a.k_new) + head * a.d_h + j0);
    const uint4 vc = load16(reinterpret_cast<const uint16_t*>(a.v_new) + head * a.d_h + j0);
    uint16_t* stage = reinterpret_cast<uint16_t*>(a.Kt) + head * (size_t)(8 * a.d_h);
    *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.V) + (head * a.S_stride + S) * a.d_h + j0) = vc;
    if (slot != 7) {
      *reinterpret_cast<uint4*>(stage + slot * a.d_h + j0) = kc;
    } else {               // the eighth row: this thread's 8 channels of the finished tile
      uint4 rows[8];
#pragma unroll
      for (int e = 0; e < 7; ++e) rows[e] = load16(stage + e * a.d_h + j0);
      rows[7] = kc;
      store_tile_piece(reinterpret_cast<uint16_t*>(a.K) + (head * a.S_stride + (size_t)(S - 7)) * a.d_h + (size_t)j0 * 8, rows);
    }
    const float* vm = a.v_mean + head * a.d_h + j0;
    float* vo = a.v_mean_out + head * a.d_h + j0;
    float4 m0 = *reinterpret_cast<const float4*>(vm), m1 = *reinterpret_cast<const float4*>(vm + 4);
    if (S == 0) m0 = m1 = make_float4(0.f, 0.f, 0.f, 0.f);
    float f[8];
    unpack8<T>(vc, f);
    m0.x += (f[0] - m0.x) * inv; m0.y += (f[1] - m0.y) * inv; m0.z += (f[2] - m0.z) * inv; m0.w += (f[3] - m0.w) * inv;
    m1.x += (f[4] - m1.x) * inv; m1.y += (f[5] - m1.y) * inv; m1.z += (f[6] - m1.z) * inv; m1.w += (f[7] - m1.w) * inv;
    *reinterpret_cast<float4*>(vo) = m0;
    *reinterpret_cast<float4*>(vo + 4) = m1;
  }
  __syncthreads();
  if (tid == 0) a.seq_lens_out[b] = S + 1;
}

// many rows per sequence: one workgroup per (sequence, KV head); the positions go tile by tile: thread (row e,
// chunk sub) of a tile brings its 16 bytes (from the buffer of waiting rows for positions cached before this
// call, else from k_new) into LDS, and the threads of the first row write the tile's 128-byte pieces; the rows
// of an unfinished last tile go (back) into the buffer.  V rows and the mean as in append_rows.
template <class T, int DH>
__global__ __launch_bounds__(BT) void append_rows_tiled(const AppendArgs a) {
  constexpr int CPR = DH / 8;            // 16-byte chunks per row
  constexpr int TPP = BT / (8 * CPR);    // tiles per pass (BT = 256: 4, 2 or 1)
  constexpr int RPP = BT / CPR;          // value rows per pass
  __shared__ __align__(16) uint16_t tile[TPP * 8 * DH];
  __shared__ double colsum[RPP][DH];
  const int tid = threadIdx.x;
  const size_t head = blockIdx.x;
  const int b = (int)(head / a.H_kv);
  const int S = a.seq_lens[b];
  int n = a.n_new_per_seq ? a.n_new_per_seq[b] : a.n_new;
  n = n < 0 ? 0 : (n > a.n_new ? a.n_new : n);
  if (n == 0) return;
  if (S < 0 || S + n > a.S_max) {
    if (tid == 0) atomicOr(a.err, 1);
    return;
  }
  const uint16_t* ksrc = reinterpret_cast<const uint16_t*>(a.k_new) + head * a.n_new * DH;
  const uint16_t* vsrc = reinterpret_cast<const uint16_t*>(a.v_new) + head * a.n_new * DH;
  uint16_t* Kdst = reinterpret_cast<uint16_t*>(a.K) + head * a.S_stride * (size_t)DH;
  uint16_t* stage = reinterpret_cast<uint16_t*>(a.Kt) + head * (size_t)(8 * DH);
  uint16_t* Vdst = reinterpret_cast<uint16_t*>(a.V) + (head * a.S_stride + S) * DH;
  // keys, tile by tile
  const int sub = tid % CPR, e = (tid / CPR) & 7, tl = tid / (8 * CPR);
  const int g_first = S >> 3, g_last = (S + n - 1) >> 3;
  for (int g0 = g_first; g0 <= g_last; g0 += TPP) {
    const int g = g0 + tl, p = g * 8 + e;                 // this thread's tile and position
    const bool have = g <= g_last && p < S + n;
    uint4 kc = make_uint4(0u, 0u, 0u, 0u);
    if (have) kc = p < S ? load16(stage + e * DH + sub * 8) : load16(ksrc + (size_t)(p - S) * DH + sub * 8);
    *reinterpret_cast<uint4*>(tile + (tl * 8 + e) * DH + sub * 8) = kc;
    __syncthreads();
    if (g <= g_last) {
      if (g * 8 + 8 <= S + n) {                           // a finished tile
        if (e == 0) {
          uint4 rows[8];
#pragma unroll
          for (int r = 0; r < 8; ++r) rows[r] = *reinterpret_cast<const uint4*>(tile + (tl * 8 + r) * DH + sub * 8);
          store_tile_piece(Kdst + ((size_t)g * DH + sub * 8) * 8, rows);
        }
      } else if (have && p >= S) {                        // a new row that waits for its tile
        *reinterpret_cast<uint4*>(stage + e * DH + sub * 8) = kc;
      }
    }
    __syncthreads();
  }
  // values and their column sums
  const int prow = tid / CPR;
  double sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int rr = prow; rr < n; rr += RPP) {
    const size_t off = (size_t)rr * DH + sub * 8;
    const uint4 vc = load16(vsrc + off);
    *reinterpret_cast<uint4*>(Vdst + off) = vc;
    float f[8];
    unpack8<T>(vc, f);
#pragma unroll
    for (int c = 0; c < 8; ++c) sum[c] += (double)f[c];
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) colsum[prow][sub * 8 + c] = sum[c];
  __syncthreads();
  if (tid < DH) {
    double tot = 0.0;
    for (int p = 0; p < RPP; ++p) tot += colsum[p][tid];
    float* vm = a.v_mean + head * DH + tid;
    const double before = S > 0 ? (double)S * (double)*vm : 0.0;
    *vm = (float)((before + tot) / (double)(S + n));
  }
}

__global__ void bump_seq_lens(const AppendArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  const int S = a.seq_lens[b];
  int n = a.n_new_per_seq ? a.n_new_per_seq[b] : a.n_new;
  n = n < 0 ? 0 : (n > a.n_new ? a.n_new : n);
  if (S >= 0 && S + n <= a.S_max) a.seq_lens[b] = S + n;
}

// Both probes: every workgroup streams one contiguous slab of the buffer (a grid-strided walk, where the 8
// loads of a thread are megabytes apart, reaches only ~5.0 TB/s here; contiguous slabs reach 6.2-6.4), 8
// independent 16-byte accesses per thread in flight, the read probe two batches deep.
__device__ __forceinline__ void probe_slab(size_t n16, size_t& begin, size_t& end) {
  const size_t chunk = (size_t)blockDim.x * 8;
  size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  per = (per + chunk - 1) / chunk * chunk;
  begin = (size_t)blockIdx.x * per;
  end = begin + per < n16 ? begin + per : n16;
  if (begin > n16) begin = n16;
}

__global__ __launch_bounds__(256) void copy_probe(uint4* dst, const uint4* src, size_t n16) {
  size_t begin, end;
  probe_slab(n16, begin, end);
  const size_t T = blockDim.x;
  size_t i = begin + threadIdx.x;
  for (; i + 7 * T < end; i += 8 * T) {
    uint4 v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = load16(src + i + t * T);
#pragma unroll
    for (int t = 0; t < 8; ++t) dst[i + t * T] = v[t];
  }
  for (; i < end; i += T) dst[i] = src[i];
}

// streaming read: every thread folds its 16-byte words into one and stores it, so nothing is elided
__global__ __launch_bounds__(256) void read_probe(const uint4* src, size_t n16, uint32_t* sink) {
  size_t begin, end;
  probe_slab(n16, begin, end);
  const size_t T = blockDim.x;
  uint32_t acc = 0;
  size_t i = begin + threadIdx.x;
  auto fold = [&](const uint4 (&v)[8]) {
#pragma unroll
    for (int t = 0; t < 8; ++t) acc ^= v[t].x ^ v[t].y ^ v[t].z ^ v[t].w;
  };
  if (i + 7 * T < end) {
    uint4 va[8], vb[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) va[t] = load16(src + i + t * T);
    i += 8 * T;
    for (; i + 15 * T < end; i += 16 * T) {
#pragma unroll
      for (int t = 0; t < 8; ++t) vb[t] = load16(src + i + t * T);
      fold(va);
#pragma unroll
      for (int t = 0; t < 8; ++t) va[t] = load16(src + i + (8 + t) * T);
      fold(vb);
    }
    fold(va);
  }
  for (; i < end; i += T) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

__global__ void clear_words(int32_t* w, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) w[i] = 0;
}

template <class T>
hipError_t launch_rows(const AppendArgs& a, hipStream_t s) {
  const dim3 grid(a.B * a.H_kv);
  switch (a.d_h) {
    case 64:  if (a.tiled) hipLaunchKernelGGL((append_rows_tiled<T, 64>), grid, dim3(BT), 0, s, a);
              else hipLaunchKernelGGL((append_rows<T, 64>), grid, dim3(BT), 0, s, a); break;
    case 128: if (a.tiled) hipLaunchKernelGGL((append_rows_tiled<T, 128>), grid, dim3(BT), 0, s, a);
              else hipLaunchKernelGGL((append_rows<T, 128>), grid, dim3(BT), 0, s, a); break;
    case 256: if (a.tiled) hipLaunchKernelGGL((append_rows_tiled<T, 256>), grid, dim3(BT), 0, s, a);
              else hipLaunchKernelGGL((append_rows<T, 256>), grid, dim3(BT), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bump_seq_lens, dim3((a.B + 255) / 256), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_append(const AppendArgs& a, int dtype, hipStream_t s) {
  if (a.n_new == 1) {
    if (a.tiled) {
      if (dtype == 1) hipLaunchKernelGGL(append_one_row_tiled<BF16>, dim3(a.B), dim3(512), 0, s, a);
      else hipLaunchKernelGGL(append_one_row_tiled<F16>, dim3(a.B), dim3(512), 0, s, a);
    } else if (dtype == 1) hipLaunchKernelGGL(append_one_row<BF16>, dim3(a.B), dim3(512), 0, s, a);
    else hipLaunchKernelGGL(append_one_row<F16>, dim3(a.B), dim3(512), 0, s, a);
    return hipGetLastError();
  }
  return dtype == 1 ? launch_rows<BF16>(a, s) : launch_rows<F16>(a, s);
}

hipError_t launch_copy_probe(void* dst, const void* src, size_t n_bytes, hipStream_t s) {
  hipLaunchKernelGGL(copy_probe, dim3(kProbeBlocks), dim3(256), 0, s, reinterpret_cast<uint4*>(dst),
                     reinterpret_cast<const uint4*>(src), n_bytes / 16);
  return hipGetLastError();
}

hipError_t launch_read_probe(const void* src, size_t n_bytes, void* sink, hipStream_t s) {
  hipLaunchKernelGGL(read_probe, dim3(kProbeBlocks), dim3(256), 0, s, reinterpret_cast<const uint4*>(src),
                     n_bytes / 16, reinterpret_cast<uint32_t*>(sink));
  return hipGetLastError();
}

hipError_t launch_clear(void* workspace, int n_bytes, hipStream_t s) {
  hipLaunchKernelGGL(clear_words, dim3(1), dim3(256), 0, s, reinterpret_cast<int32_t*>(workspace), n_bytes / 4);
  return hipGetLastError();
}

}  // namespace sparq
