// Cross-modal saliency scores of Sec. 3.3 (2), Eq. 7: I(i, j) = X_v(i) . X_t(j),
// aggregated over the text tokens j by summation, so
//   score(i) = sum_j X_v(i) . X_t(j) = X_v(i) . (sum_j X_t(j)):
// one pass over the text rows, then a matrix-vector product that streams the
// visual hidden states once.  HBM-bound: 2 bytes per element of X_v.
#include "vidkv_common.h"

namespace vidkv {

constexpr int SAL_ROWS = 64;         // visual tokens per workgroup (16 per wave)

// tsum[b][c] = sum_j X_t[b][j][c], fp32, j ascending.  grid (ceil(d/256), B).
__global__ __launch_bounds__(256) void sal_text_sum_kernel(const _Float16* __restrict__ Xt, int Nt,
                                                           int d, float* __restrict__ tsum) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int b = blockIdx.y;
  if (c >= d) return;
  const _Float16* p = Xt + (size_t)b * Nt * d + c;
  float acc = 0.0f;
  for (int j = 0; j < Nt; ++j) acc += (float)p[(size_t)j * d];
  tsum[(size_t)b * d + c] = acc;
}

// scores[b][i] = X_v[b][i][:] . tsum[b][:].  One wave takes two token rows at a
// time: lane l takes the 8 channels 512 k + 8 l .. of every 512-channel chunk
// (one 16-byte load each), multiplies by the text sum held in LDS, fp32 FMA
// chain per lane (channels ascending), butterfly sum over the wave.  grid (ceil(Tv / SAL_ROWS), B).
__global__ __launch_bounds__(256) void sal_scores_kernel(const u32x4* __restrict__ Xv,
                                                         const float* __restrict__ tsum, int Tv,
                                                         int d, float* __restrict__ scores) {
  extern __shared__ float ts[];                       // d floats
  const int b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int c = tid; c < d; c += 256) ts[c] = tsum[(size_t)b * d + c];
  __syncthreads();
  const int d8 = d >> 3;                              // 16-byte pieces per row
  const int row0 = blockIdx.x * SAL_ROWS;
  const int row1 = min(Tv, row0 + SAL_ROWS);
  const u32x4* Xb = Xv + (size_t)b * Tv * d8;
  // two rows at a time, 8 pieces of each in flight per lane (a 3584-wide row is 7)
  for (int i = row0 + 2 * wave; i < row1; i += 8) {
    const bool two = i + 1 < row1;
    const u32x4* ra = Xb + (size_t)i * d8;
    const u32x4* rb = Xb + (size_t)(two ? i + 1 : i) * d8;
    float acc_a = 0.0f, acc_b = 0.0f;
    for (int k0 = 0; k0 < d8; k0 += 512) {
      U4H xa[8], xb[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = k0 + 64 * u + lane;
        const bool ok = k < d8;
        xa[u].u = ok ? __builtin_nontemporal_load(ra + k) : u32x4{0u, 0u, 0u, 0u};
        xb[u].u = ok ? __builtin_nontemporal_load(rb + k) : u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = k0 + 64 * u + lane;
        if (k < d8) {
          const float4 t0 = *reinterpret_cast<const float4*>(&ts[8 * k]);
          const float4 t1 = *reinterpret_cast<const float4*>(&ts[8 * k + 4]);
          const float t[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            acc_a = fmaf((float)xa[u].e[e], t[e], acc_a);
            acc_b = fmaf((float)xb[u].e[e], t[e], acc_b);
          }
        }
      }
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
      acc_a += __shfl_xor(acc_a, s, 64);
      acc_b += __shfl_xor(acc_b, s, 64);
    }
    if (lane == 0) {
      scores[(size_t)b * Tv + i] = acc_a;
      if (two) scores[(size_t)b * Tv + i + 1] = acc_b;
    }
  }
}

hipError_t launch_saliency(const void* Xv, const void* Xt, int B, int Tv, int Nt, int d,
                           float* scores, float* tsum, hipStream_t st) {
  hipLaunchKernelGGL(sal_text_sum_kernel, dim3((d + 255) / 256, B), dim3(256), 0, st,
                     reinterpret_cast<const _Float16*>(Xt), Nt, d, tsum);
  if (Tv > 0)
    hipLaunchKernelGGL(sal_scores_kernel, dim3((Tv + SAL_ROWS - 1) / SAL_ROWS, B), dim3(256),
                       (size_t)d * sizeof(float), st, reinterpret_cast<const u32x4*>(Xv), tsum, Tv, d,
                       scores);
  return hipGetLastError();
}

}  // namespace vidkv
