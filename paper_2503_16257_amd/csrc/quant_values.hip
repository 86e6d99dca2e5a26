// Value quantizer kernels (Alg. 2): protected-token selection (top-n saliency
// scores, Sec. 3.3 (2)) and the per-channel ternary code of Eq. 6 over
// 32-token groups, with protected rows copied verbatim in fp16.
#include "vidkv_common.h"

namespace vidkv {

// Order-preserving map float -> uint32 (ascending).
__device__ __forceinline__ uint32_t fkey(float f) {
  const uint32_t b = __float_as_uint(f + 0.0f);   // -0 and +0 are the same score
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exclusive scan of one int per thread over a 1024-thread block; also returns
// the block total.  `sw` is LDS scratch of 16 ints.
__device__ __forceinline__ int block_exscan_1024(int v, int* sw, int* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d, 64);
    if (lane >= d) inc += o;
  }
  __syncthreads();                 // sw may still be read from a previous call
  if (lane == 63) sw[wv] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int s = sw[i];
    base += (i < wv) ? s : 0;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

// ---------------------------------------------------------------------------
// One workgroup of 1024 threads per sequence.  Produces, in the value buffer,
// MASK (bit per token), RANK (protected tokens before each group) and IDX
// (ascending list).  With scores: the n_s largest by (score desc, index asc),
// found by a 4 x 8-bit radix select on the ordered keys; with a given index
// list: the list itself.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void v_select_kernel(const float* __restrict__ scores,
                                                        const int32_t* __restrict__ idx_in,
                                                        int T, int ng, int n_s,
                                                        int32_t* __restrict__ idx_out,
                                                        uint32_t* __restrict__ mask,
                                                        uint32_t* __restrict__ rank) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  __shared__ int hist[256];
  __shared__ int sw[16];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining;
  uint32_t* mk = mask + (size_t)b * ng;
  uint32_t* rk = rank + (size_t)b * ng;
  int32_t* io = idx_out + (size_t)b * n_s;
  const int gpt = (ng + 1023) / 1024;            // groups per thread (contiguous segment)
  const int g0 = min(ng, tid * gpt), g1 = min(ng, g0 + gpt);

  if (scores) {
    const float* sc = scores + (size_t)b * T;
    if (tid == 0) { s_prefix = 0; s_remaining = n_s; }
    uint32_t pmask = 0;
    for (int pass = 3; pass >= 0; --pass) {
      for (int i = tid; i < 256; i += 1024) hist[i] = 0;
      __syncthreads();
      const uint32_t prefix = s_prefix;
      for (int t = tid; t < T; t += 1024) {
        const uint32_t k = fkey(sc[t]);
        if ((k & pmask) == prefix) atomicAdd(&hist[(k >> (8 * pass)) & 255], 1);
      }
      __syncthreads();
      if (tid == 0) {
        int rem = s_remaining, bin = 255;
        for (; bin > 0; --bin) {
          if (hist[bin] >= rem) break;
          rem -= hist[bin];
        }
        s_prefix = prefix | ((uint32_t)bin << (8 * pass));
        s_remaining = rem;
      }
      pmask |= 0xFFu << (8 * pass);
      __syncthreads();
    }
    const uint32_t kth = s_prefix;
    const int take_eq = s_remaining;             // equal-to-kth elements to take, lowest index first
    int neq = 0;
    for (int t = g0 * G; t < g1 * G; ++t) neq += (fkey(sc[t]) == kth) ? 1 : 0;
    int tot;
    int eq_before = block_exscan_1024(neq, sw, &tot);
    for (int g = g0; g < g1; ++g) {
      uint32_t w = 0;
      for (int j = 0; j < G; ++j) {
        const uint32_t k = fkey(sc[g * G + j]);
        bool sel = k > kth;
        if (k == kth) { sel = eq_before < take_eq; ++eq_before; }
        w |= sel ? (1u << j) : 0u;
      }
      mk[g] = w;
    }
  } else {
    for (int g = tid; g < ng; g += 1024) mk[g] = 0;
    __syncthreads();
    for (int i = tid; i < n_s; i += 1024) {
      const int t = idx_in[(size_t)b * n_s + i];
      atomicOr(&mk[t >> 5], 1u << (t & 31));
    }
  }
  __syncthreads();
  int cnt = 0;
  // device-scope loads: the words may have been set by other waves' atomics
  for (int g = g0; g < g1; ++g)
    cnt += __popc(__hip_atomic_load(&mk[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  int tot;
  int before = block_exscan_1024(cnt, sw, &tot);
  for (int g = g0; g < g1; ++g) {
    uint32_t w = __hip_atomic_load(&mk[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    rk[g] = (uint32_t)before;
    while (w) {
      const int j = __ffs(w) - 1;
      w &= w - 1;
      if (before < n_s) io[before] = g * G + j;
      ++before;
    }
  }
}

// ---------------------------------------------------------------------------
// Ternary coding of one 32-token group of one head.  grid (ng, nheads), block
// 128; thread c owns channel c.  s = mean |v| over unprotected tokens,
// alpha = gamma * s, code = sign(v) [|v| > alpha]; protected tokens code 0 and
// their rows go to ROWS at position RANK[g] + (order inside the group).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(128) void v_encode_kernel(const u32x4* __restrict__ V, int T, int ng,
                                                       int B, int H, int n_s, float gamma,
                                                       const uint32_t* __restrict__ mask,
                                                       const uint32_t* __restrict__ rank,
                                                       uint8_t* __restrict__ rec_out,
                                                       u32x4* __restrict__ rows_out) {
  const int g = blockIdx.x;
  const long long hd = blockIdx.y;
  const int tid = threadIdx.x;
  __shared__ u32x4 tile4[32 * 16];
  __shared__ u32x4 rec4[VREC / 16];
  const u32x4* src = V + ((hd * T) + (long long)g * G) * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) tile4[tid + 128 * i] = __builtin_nontemporal_load(src + tid + 128 * i);
  uint32_t m = 0, r0 = 0;
  if (n_s > 0) {
    const int b = (int)((hd / H) % B);
    m = mask[(size_t)b * ng + g];
    r0 = rank[(size_t)b * ng + g];
  }
  __syncthreads();
  const _Float16* tile = reinterpret_cast<const _Float16*>(tile4);
  float x[32];
  float sum = 0.0f;
#pragma unroll
  for (int t = 0; t < 32; ++t) {
    x[t] = (float)tile[t * D + tid];
    sum += ((m >> t) & 1u) ? 0.0f : fabsf(x[t]);
  }
  const int n = 32 - __popc(m);
  const float s = n > 0 ? sum / (float)n : 0.0f;
  const float alpha = gamma * s;
  uint16_t* rec16 = reinterpret_cast<uint16_t*>(rec4);
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    uint32_t w = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int t = (j < 4) ? 4 * kb + j : 16 + 4 * kb + (j - 4);
      const bool keep = !((m >> t) & 1u);
      const uint32_t nz = (keep && (x[t] > alpha || x[t] < -alpha)) ? 1u : 0u;
      const uint32_t ng_ = (keep && x[t] < -alpha) ? 1u : 0u;
      w |= (nz | (ng_ << 1)) << (8 * (j & 1) + 2 * (j >> 1));
    }
    rec16[(kb * 16 + (tid & 15)) * 8 + (tid >> 4)] = (uint16_t)w;
  }
  reinterpret_cast<_Float16*>(rec4)[512 + tid] = (_Float16)s;
  __syncthreads();
  u32x4* dst = reinterpret_cast<u32x4*>(rec_out + ((hd * ng) + g) * (long long)VREC);
  if (tid < VREC / 16) dst[tid] = rec4[tid];
  uint32_t w = m;
  uint32_t r = r0;
  while (w) {
    const int t = __ffs(w) - 1;
    w &= w - 1;
    if (tid < 16) rows_out[(hd * n_s + r) * 16 + tid] = tile4[t * 16 + tid];
    ++r;
  }
}

hipError_t launch_quantize_values(const Geom& g, float gamma, const void* V, const float* scores,
                                  const int32_t* idx, uint8_t* packed, unsigned stages,
                                  hipStream_t st) {
  if (g.T == 0) return hipSuccess;
  uint32_t* mask = reinterpret_cast<uint32_t*>(packed + g.v_mask);
  uint32_t* rank = reinterpret_cast<uint32_t*>(packed + g.v_rank);
  // stages: bit 0 protected-token selection, bit 1 coding pass
  if (g.n_s > 0 && (stages & 1u)) {
    hipLaunchKernelGGL(v_select_kernel, dim3(g.B), dim3(1024), 0, st, scores, idx, g.T, g.ng,
                       g.n_s, reinterpret_cast<int32_t*>(packed + g.v_idx), mask, rank);
  }
  dim3 gr(g.ng, (unsigned)g.nheads);
  if (stages & 2u)
    hipLaunchKernelGGL(v_encode_kernel, gr, dim3(128), 0, st, reinterpret_cast<const u32x4*>(V),
                       g.T, g.ng, g.B, g.H, g.n_s, gamma, mask, rank, packed + g.v_rec,
                       reinterpret_cast<u32x4*>(packed + g.v_rows));
  return hipGetLastError();
}

}  // namespace vidkv
