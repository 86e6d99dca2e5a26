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
// ascending.  grid nheads, block 1024: 8 slices of the chunk list per channel.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_select_kernel(const _Float16* __restrict__ ws,
                                                        int chunks, int n_a,
                                                        uint8_t* __restrict__ perm) {
  const long long hd = blockIdx.x;
  const int c = threadIdx.x & 127, part = threadIdx.x >> 7;
  const _Float16* p = ws + hd * chunks * 2 * D;
  _Float16 lo = (_Float16)65504.0f, hi = (_Float16)-65504.0f;
  for (int k = part; k < chunks; k += 8) {
    const _Float16 a = p[(k * 2) * D + c], b = p[(k * 2 + 1) * D + c];
    lo = a < lo ? a : lo;
    hi = b > hi ? b : hi;
  }
  __shared__ _Float16 slo[8][D], shi[8][D];
  __shared__ float R[D];
  __shared__ int flag[D];
  slo[part][c] = lo;
  shi[part][c] = hi;
  __syncthreads();
  float r = 0.0f;
  if (part == 0) {
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      const _Float16 a = slo[i][c], b = shi[i][c];
      lo = a < lo ? a : lo;
      hi = b > hi ? b : hi;
    }
    r = (float)hi - (float)lo;
    R[c] = r;
  }
  __syncthreads();
  int an = 0;
  if (part == 0) {
    int rank = 0;
    for (int j = 0; j < D; ++j) {
      const float rj = R[j];
      rank += (rj > r || (rj == r && j < c)) ? 1 : 0;
    }
    an = rank < n_a ? 1 : 0;
    flag[c] = an;
  }
  __syncthreads();
  if (part == 0) {
    int below = 0;
    for (int j = 0; j < c; ++j) below += flag[j];
    const int pos = an ? below : n_a + (c - below);
    perm[hd * D + pos] = (uint8_t)c;
  }
}

// ---------------------------------------------------------------------------
// 32-point DFT of a real sequence held in registers, via a 16-point complex
// FFT of z[n] = x[2n] + i x[2n+1] (decimation in frequency, constant-folded
// twiddles) and the even/odd split.  Forward convention X[k] = sum x[t]
// exp(-2 pi i k t / 32), unnormalised.  re[0..16], im[0..16] (im[0]=im[16]=0).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void rdft32(const float* x, float* re, float* im) {
  float zr[16], zi[16];
#pragma unroll
  for (int n = 0; n < 16; ++n) { zr[n] = x[2 * n]; zi[n] = x[2 * n + 1]; }
#pragma unroll
  for (int s = 8; s >= 1; s >>= 1) {
#pragma unroll
    for (int b = 0; b < 16; b += 2 * s) {
#pragma unroll
      for (int j = 0; j < s; ++j) {
        const float wr = cos32(j * (16 / s)), wi = -sin32(j * (16 / s));
        const float ar = zr[b + j], ai = zi[b + j];
        const float cr = zr[b + j + s], ci = zi[b + j + s];
        zr[b + j] = ar + cr;
        zi[b + j] = ai + ci;
        const float dr = ar - cr, di = ai - ci;
        zr[b + j + s] = dr * wr - di * wi;
        zi[b + j + s] = dr * wi + di * wr;
      }
    }
  }
  // Z[k] sits at index bitrev4(k)
#define VIDKV_BR4(k) ((((k) & 1) << 3) | (((k) & 2) << 1) | (((k) & 4) >> 1) | (((k) & 8) >> 3))
#pragma unroll
  for (int k = 0; k <= 8; ++k) {
    const int k2 = (16 - k) & 15;
    const float ar = zr[VIDKV_BR4(k)], ai = zi[VIDKV_BR4(k)];
    const float br = zr[VIDKV_BR4(k2)], bi = zi[VIDKV_BR4(k2)];
    // E = (Z[k] + conj Z[16-k]) / 2 ; O = (Z[k] - conj Z[16-k]) / (2 i)
    const float er = 0.5f * (ar + br), ei = 0.5f * (ai - bi);
    const float orr = 0.5f * (ai + bi), oi = -0.5f * (ar - br);
    {
      const float wr = cos32(k), wi = -sin32(k);
      re[k] = er + (orr * wr - oi * wi);
      im[k] = ei + (orr * wi + oi * wr);
    }
    if (k >= 1 && k <= 7) {
      // X[16-k]: E[16-k] = conj E[k], O[16-k] = conj O[k]
      const float wr = cos32(16 - k), wi = -sin32(16 - k);
      re[16 - k] = er + (orr * wr + oi * wi);
      im[16 - k] = -ei + (orr * wi - oi * wr);
    }
    if (k == 0) {
      re[16] = er - orr;
      im[16] = 0.0f;
      im[0] = 0.0f;
    }
  }
#undef VIDKV_BR4
}

// ---------------------------------------------------------------------------
// Pass 2: code one 32-token group of one head.  grid (ng, nheads), block 128;
// thread i owns channel perm[i]: i < n_a -> Eq. 4 at 2 bits, else Eq. 5.
// The 32 x 128 fp16 tile is staged in LDS with 16-byte loads; the record is
// assembled in LDS and written out with 16-byte stores.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(128) void k_encode_kernel(const u32x4* __restrict__ K,
                                                       const uint8_t* __restrict__ perm, int T,
                                                       int ng, int n_a, int krec,
                                                       uint8_t* __restrict__ rec_out) {
  const int g = blockIdx.x;
  const long long hd = blockIdx.y;
  const int tid = threadIdx.x;
  __shared__ u32x4 tile4[32 * 16];                 // [32 tokens][128 ch] fp16
  __shared__ uint32_t rec[1536 / 4];
  const int n_n = D - n_a;

  const u32x4* src = K + ((hd * T) + (long long)g * G) * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) tile4[tid + 128 * i] = __builtin_nontemporal_load(src + tid + 128 * i);
  for (int i = tid; i < krec / 4; i += 128) rec[i] = 0;
  const int ch = perm[hd * D + tid];
  __syncthreads();

  const _Float16* tile = reinterpret_cast<const _Float16*>(tile4);
  float x[32];
#pragma unroll
  for (int t = 0; t < 32; ++t) x[t] = (float)tile[t * D + ch];

  _Float16* rec16 = reinterpret_cast<_Float16*>(rec);
  if (tid < n_a) {
    const int j = tid;
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int t = 1; t < 32; ++t) { mn = fminf(mn, x[t]); mx = fmaxf(mx, x[t]); }
    const float rng = mx - mn;
    const float s = rng / 3.0f;
    const int nq = n_a >> 2;
#pragma unroll
    for (int t = 0; t < 32; ++t) {
      float u = (rng > 0.0f) ? (3.0f * (x[t] - mn)) / rng : 0.0f;
      u = fminf(fmaxf(rintf(u), 0.0f), 3.0f);
      const uint32_t code = (uint32_t)u;
      const int byte = t * nq + (j >> 2);
      atomicOr(&rec[byte >> 2], code << (8 * (byte & 3) + 2 * (j & 3)));
    }
    rec16[4 * n_a + j] = (_Float16)s;       // byte offset 8 n_a
    rec16[5 * n_a + j] = (_Float16)mn;      // byte offset 10 n_a
  } else {
    const int i = tid - n_a;
    const int blk = i >> 3, e = i & 7;
    float re[17], im[17];
    rdft32(x, re, im);
    float sre = fabsf(re[0]) + fabsf(re[16]);
    float sim = 0.0f;
#pragma unroll
    for (int k = 1; k < 16; ++k) { sre += 2.0f * fabsf(re[k]); sim += 2.0f * fabsf(im[k]); }
    sre *= (1.0f / 32.0f);
    sim *= (1.0f / 32.0f);
    uint32_t* words = rec + 3 * n_a;                       // byte offset 12 n_a
#pragma unroll
    for (int k = 0; k < 16; k += 2) {
      const uint32_t lo0 = !(re[k] < 0.0f) ? 1u : 0u;
      const uint32_t hi0 = (k == 0) ? (!(re[16] < 0.0f) ? 1u : 0u) : (!(im[k] < 0.0f) ? 1u : 0u);
      const uint32_t lo1 = !(re[k + 1] < 0.0f) ? 1u : 0u;
      const uint32_t hi1 = !(im[k + 1] < 0.0f) ? 1u : 0u;
      const uint32_t w = ((lo0 << e) | (hi0 << (8 + e))) | (((lo1 << e) | (hi1 << (8 + e))) << 16);
      atomicOr(&words[(blk * 16 + k) >> 1], w);
    }
    _Float16* meta = rec16 + 6 * n_a + 2 * n_n;            // byte offset 12 n_a + 4 n_n
    meta[(blk * 2 + 0) * 8 + e] = (_Float16)sre;
    meta[(blk * 2 + 1) * 8 + e] = (_Float16)sim;
  }
  __syncthreads();
  u32x4* dst = reinterpret_cast<u32x4*>(rec_out + ((hd * ng) + g) * (long long)krec);
  const u32x4* rec4 = reinterpret_cast<const u32x4*>(rec);
  for (int i = tid; i < krec / 16; i += 128) dst[i] = rec4[i];
}

// ---------------------------------------------------------------------------
// stages: bit 0 range pass, bit 1 channel selection, bit 2 coding pass
hipError_t launch_quantize_keys(const Geom& g, const void* K, uint8_t* packed, void* ws,
                                unsigned stages, hipStream_t st) {
  if (g.T == 0) return hipSuccess;
  _Float16* w = reinterpret_cast<_Float16*>(ws);
  dim3 gr1(g.range_chunks, (unsigned)g.nheads);
  if (stages & 1u)
    hipLaunchKernelGGL(k_range_kernel, gr1, dim3(256), 0, st, reinterpret_cast<const u32x4*>(K),
                       g.T, g.range_chunks, w);
  if (stages & 2u)
    hipLaunchKernelGGL(k_select_kernel, dim3((unsigned)g.nheads), dim3(1024), 0, st, w,
                       g.range_chunks, g.n_a, packed + g.k_perm);
  dim3 gr3(g.ng, (unsigned)g.nheads);
  if (stages & 4u)
    hipLaunchKernelGGL(k_encode_kernel, gr3, dim3(128), 0, st, reinterpret_cast<const u32x4*>(K),
                       packed + g.k_perm, g.T, g.ng, g.n_a, g.krec, packed + g.k_rec);
  return hipGetLastError();
}

}  // namespace vidkv
