// Key quantizer kernels (Alg. 3, MixQuant): per-channel range over all tokens,
// top-n_a channel selection, and per 32-token group the 2-bit uniform code
// (Eq. 4) of the selected channels and the sign bits of a 32-point real DFT
// (Eq. 5) of the others.
#include "vidkv_common.h"

namespace vidkv {

// ---------------------------------------------------------------------------
// Pass 1: partial per-channel min / max over RANGE_CHUNK tokens of one head.
// grid (range_chunks, nheads), block 256.  Thread (row = tid/16, col = tid%16)
// streams 16-byte pieces (8 channels) of rows row, row+16, ...; fp16 min/max
// are exact, so no precision is involved.
// ws layout: fp16 [nheads][chunks][2][128]  (min then max).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_range_kernel(const u32x4* __restrict__ K, int T,
                                                      int chunks, _Float16* __restrict__ ws) {
  const int chunk = blockIdx.x;
  const long long hd = blockIdx.y;
  const int tid = threadIdx.x;
  const int col = tid & 15, row = tid >> 4;
  const int t0 = chunk * RANGE_CHUNK;
  const int t1 = min(T, t0 + RANGE_CHUNK);
  const u32x4* base = K + (hd * T) * 16 + col;   // 16 u32x4 per token row

  const _Float16 big = (_Float16)65504.0f;
  h2 mn[4], mx[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { mn[i] = h2{big, big}; mx[i] = h2{-big, -big}; }

  int t = t0 + row;
  // 4 independent 16-byte loads in flight per thread
  for (; t + 48 < t1; t += 64) {
    U4H a, b, c, d;
    a.u = __builtin_nontemporal_load(base + (long long)t * 16);
    b.u = __builtin_nontemporal_load(base + (long long)(t + 16) * 16);
    c.u = __builtin_nontemporal_load(base + (long long)(t + 32) * 16);
    d.u = __builtin_nontemporal_load(base + (long long)(t + 48) * 16);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mn[i] = __builtin_elementwise_min(__builtin_elementwise_min(mn[i], a.h[i]),
                                        __builtin_elementwise_min(b.h[i], c.h[i]));
      mn[i] = __builtin_elementwise_min(mn[i], d.h[i]);
      mx[i] = __builtin_elementwise_max(__builtin_elementwise_max(mx[i], a.h[i]),
                                        __builtin_elementwise_max(b.h[i], c.h[i]));
      mx[i] = __builtin_elementwise_max(mx[i], d.h[i]);
    }
  }
  for (; t < t1; t += 16) {
    U4H a;
    a.u = __builtin_nontemporal_load(base + (long long)t * 16);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mn[i] = __builtin_elementwise_min(mn[i], a.h[i]);
      mx[i] = __builtin_elementwise_max(mx[i], a.h[i]);
    }
  }

  __shared__ h2 smn[16][16][4];
  __shared__ h2 smx[16][16][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { smn[row][col][i] = mn[i]; smx[row][col][i] = mx[i]; }
  __syncthreads();
  if (tid < 128) {
    const int c8 = tid >> 3, e = tid & 7;
    _Float16 lo = big, hi = -big;
    for (int r = 0; r < 16; ++r) {
      const _Float16 a = smn[r][c8][e >> 1][e & 1];
      const _Float16 b = smx[r][c8][e >> 1][e & 1];
      lo = a < lo ? a : lo;
      hi = b > hi ? b : hi;
    }
    _Float16* o = ws + ((hd * chunks + chunk) * 2) * D;
    o[tid] = lo;
    o[D + tid] = hi;
  }
}

// ---------------------------------------------------------------------------
// Channel selection: R_c = float(max) - float(min); the n_a largest (ties to
// the lower channel) are anomalous.  perm = anomalous ascending, then normal
// ascending.  grid nheads, block 1024: 64 slices of the chunk list, 8 channels per thread.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_select_kernel(const _Float16* __restrict__ ws,
                                                        int chunks, int n_a,
                                                        uint8_t* __restrict__ perm) {
  const long long hd = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // gather: thread (slice = tid / 16, col = tid % 16) folds 8 channels of the
  // chunks slice, slice + 64, ... with 16-byte loads, 8 chunks in flight
  const int col = tid & 15, slice = tid >> 4;
  const u32x4* p4 = reinterpret_cast<const u32x4*>(ws + hd * chunks * 2 * D) + col;
  const _Float16 big = (_Float16)65504.0f;
  h2 mn[4], mx[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { mn[i] = h2{big, big}; mx[i] = h2{-big, -big}; }
  for (int k0 = slice; k0 < chunks; k0 += 512) {
    U4H a[8], b[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int k = k0 + 64 * u;
      const int kk = k < chunks ? k : k0;             // a repeated chunk changes nothing
      a[u].u = p4[(kk * 2) * 16];
      b[u].u = p4[(kk * 2 + 1) * 16];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        mn[i] = __builtin_elementwise_min(mn[i], a[u].h[i]);
        mx[i] = __builtin_elementwise_max(mx[i], b[u].h[i]);
      }
  }
  // the 4 slices of a wave (lanes 16 apart), then the 16 waves through LDS
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int d = 16; d <= 32; d <<= 1) {
      mn[i] = __builtin_elementwise_min(mn[i], __builtin_bit_cast(h2, __shfl_xor(__builtin_bit_cast(int, mn[i]), d, 64)));
      mx[i] = __builtin_elementwise_max(mx[i], __builtin_bit_cast(h2, __shfl_xor(__builtin_bit_cast(int, mx[i]), d, 64)));
    }
  }
  __shared__ h2 smn[16][16][4];
  __shared__ h2 smx[16][16][4];
  __shared__ float R[D];
  __shared__ int cnt0;
  if (lane < 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { smn[wave][col][i] = mn[i]; smx[wave][col][i] = mx[i]; }
  }
  __syncthreads();
  // from here on threads 0..127 (waves 0 and 1) own one channel each; the other
  // waves only keep the barriers company
  const int c = tid & (D - 1);
  const bool own = tid < D;
  float r = 0.0f;
  if (own) {
    const int c8 = c >> 3, e = c & 7;
    _Float16 lo = big, hi = -big;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const _Float16 a = smn[s][c8][e >> 1][e & 1];
      const _Float16 b = smx[s][c8][e >> 1][e & 1];
      lo = a < lo ? a : lo;
      hi = b > hi ? b : hi;
    }
    r = (float)hi - (float)lo;
    R[c] = r;
  }
  __syncthreads();
  int an = 0, below = 0;
  if (own) {
    int rank = 0;
#pragma unroll 16
    for (int j = 0; j < D; ++j) {
      const float rj = R[j];
      rank += (rj > r || (rj == r && j < c)) ? 1 : 0;
    }
    an = rank < n_a ? 1 : 0;
  }
  // anomalous channels below mine: inside my wave by ballot, wave 0's total through LDS
  const unsigned long long bal = __ballot(an);
  below = __popcll(bal & ((1ull << lane) - 1ull));
  if (tid == 0) cnt0 = __popcll(bal);
  __syncthreads();
  if (own) {
    if (wave == 1) below += cnt0;
    const int pos = an ? below : n_a + (c - below);
    perm[hd * D + pos] = (uint8_t)c;
  }
}

// ---------------------------------------------------------------------------
// The two other channel metrics of Sec. 3.2 (1), both in float64 so that the
// ranking does not depend on the summation order beyond the last bits:
//   variance   sigma^2 = mean(x^2) - mean(x)^2 over all tokens of the channel
//   outliers   N = #{ t : |x_t| > M * mean|x| },  M = 3
// k_metric_kernel<MODE> writes per (head, chunk) partials double [2][128]:
//   MODE 0: sum x, sum x^2      MODE 1: sum |x|, 0      MODE 2: count(|x| > thr), 0
// grid (range_chunks, nheads), block 256: thread (row = tid / 16, col = tid % 16)
// takes 8 channels of rows row, row + 16, ... of its chunk.
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void k_metric_kernel(const u32x4* __restrict__ K, int T,
                                                       int chunks, const double* __restrict__ thr,
                                                       double* __restrict__ part) {
  const int chunk = blockIdx.x;
  const long long hd = blockIdx.y;
  const int tid = threadIdx.x, col = tid & 15, row = tid >> 4;
  const int t1 = min(T, (chunk + 1) * RANGE_CHUNK);
  const u32x4* base = K + (hd * T) * 16 + col;
  double a[8], b[8], th[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = 0.0; b[e] = 0.0;
    th[e] = MODE == 2 ? thr[hd * D + 8 * col + e] : 0.0;
  }
  for (int t = chunk * RANGE_CHUNK + row; t < t1; t += 16) {
    U4H x;
    x.u = base[(long long)t * 16];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const double v = (double)(float)x.e[e];
      if (MODE == 0) { a[e] += v; b[e] = fma(v, v, b[e]); }
      if (MODE == 1) a[e] += fabs(v);
      if (MODE == 2) a[e] += fabs(v) > th[e] ? 1.0 : 0.0;
    }
  }
  __shared__ double sa[16][D], sb[16][D];
#pragma unroll
  for (int e = 0; e < 8; ++e) { sa[row][8 * col + e] = a[e]; sb[row][8 * col + e] = b[e]; }
  __syncthreads();
  if (tid < D) {
    double x = 0.0, y = 0.0;
    for (int r = 0; r < 16; ++r) { x += sa[r][tid]; y += sb[r][tid]; }
    double* o = part + ((hd * chunks + chunk) * 2) * D;
    o[tid] = x;
    o[D + tid] = y;
  }
}

// Folds the partials of one head (chunks in ascending order).  MODE 1: writes the
// outlier threshold M * mean|x| per channel.  MODE 0 / 2: ranks the channels by
// variance / outlier count (ties to the lower channel) and writes PERM like
// k_select_kernel.  grid nheads, block 128: thread = channel.
template <int MODE>
__global__ __launch_bounds__(128) void k_metric_select_kernel(const double* __restrict__ part,
                                                              int chunks, int T, int n_a,
                                                              double* __restrict__ thr,
                                                              uint8_t* __restrict__ perm) {
  const long long hd = blockIdx.x;
  const int c = threadIdx.x;
  double x = 0.0, y = 0.0;
  for (int k = 0; k < chunks; ++k) {
    x += part[((hd * chunks + k) * 2) * D + c];
    y += part[((hd * chunks + k) * 2 + 1) * D + c];
  }
  if (MODE == 1) {
    thr[hd * D + c] = 3.0 * (x / (double)T);
    return;
  }
  const double mean = x / (double)T;
  const double r = MODE == 0 ? y / (double)T - mean * mean : x;
  __shared__ double R[D];
  __shared__ int flag[D];
  R[c] = r;
  __syncthreads();
  int rank = 0;
  for (int j = 0; j < D; ++j) {
    const double rj = R[j];
    rank += (rj > r || (rj == r && j < c)) ? 1 : 0;
  }
  const int an = rank < n_a ? 1 : 0;
  flag[c] = an;
  __syncthreads();
  int below = 0;
  for (int j = 0; j < c; ++j) below += flag[j];
  perm[hd * D + (an ? below : n_a + (c - below))] = (uint8_t)c;
}

// The per-group coding pass (Eq. 4 and Eq. 5) lives in quant_keys_mfma.hip.
void launch_k_encode(const Geom& g, const EncodeSpan& sp, const void* K, uint8_t* packed,
                     bool use_fft, hipStream_t st);

// ---------------------------------------------------------------------------
// stages: bit 0 range pass, bit 1 channel selection, bit 2 coding pass
hipError_t launch_quantize_keys(const Geom& g, const void* K, uint8_t* packed, void* ws,
                                unsigned stages, hipStream_t st) {
  if (g.T == 0) return hipSuccess;
  _Float16* w = reinterpret_cast<_Float16*>(ws);
  dim3 gr1(g.range_chunks, (unsigned)g.nheads);
  const u32x4* k4 = reinterpret_cast<const u32x4*>(K);
  if (g.metric != 0) {
    // variance / outlier count (the paper's ablation; Range is what it adopts): float64
    // partials [nheads][chunks][2][128], then the thresholds [nheads][128]
    double* part = reinterpret_cast<double*>(ws);
    double* thr = part + (size_t)g.nheads * g.range_chunks * 2 * D;
    dim3 gh((unsigned)g.nheads);
    if (g.metric == 1) {
      if (stages & 1u)
        hipLaunchKernelGGL(k_metric_kernel<0>, gr1, dim3(256), 0, st, k4, g.T, g.range_chunks, thr, part);
      if (stages & 2u)
        hipLaunchKernelGGL(k_metric_select_kernel<0>, gh, dim3(128), 0, st, part, g.range_chunks, g.T,
                           g.n_a, thr, packed + g.k_perm);
    } else {
      if (stages & 1u) {
        hipLaunchKernelGGL(k_metric_kernel<1>, gr1, dim3(256), 0, st, k4, g.T, g.range_chunks, thr, part);
        hipLaunchKernelGGL(k_metric_select_kernel<1>, gh, dim3(128), 0, st, part, g.range_chunks, g.T,
                           g.n_a, thr, packed + g.k_perm);
        hipLaunchKernelGGL(k_metric_kernel<2>, gr1, dim3(256), 0, st, k4, g.T, g.range_chunks, thr, part);
      }
      if (stages & 2u)
        hipLaunchKernelGGL(k_metric_select_kernel<2>, gh, dim3(128), 0, st, part, g.range_chunks, g.T,
                           g.n_a, thr, packed + g.k_perm);
    }
    if (stages & 4u)
      launch_k_encode(g, EncodeSpan{g.T, g.ng, 0, g.nheads, 0}, K, packed, g.use_fft, st);
    return hipGetLastError();
  }
  if (stages & 1u)
    hipLaunchKernelGGL(k_range_kernel, gr1, dim3(256), 0, st, k4, g.T, g.range_chunks, w);
  if (stages & 2u)
    hipLaunchKernelGGL(k_select_kernel, dim3((unsigned)g.nheads), dim3(1024), 0, st, w,
                       g.range_chunks, g.n_a, packed + g.k_perm);
  if (stages & 4u)
    launch_k_encode(g, EncodeSpan{g.T, g.ng, 0, g.nheads, 0}, K, packed, g.use_fft, st);
  return hipGetLastError();
}

}  // namespace vidkv
