// Value coding pass (Alg. 2, 1.58Quant with token protection): per channel and
// 32-token group s = mean |v| over the unprotected tokens, alpha = gamma * s,
// code = sign(v) [|v| > alpha] (Eq. 6); protected tokens code 0 and their rows
// are copied verbatim.
//
// One wave codes one group at a time (4 groups per wave, next tile prefetched).
// The [32 tokens x 128 channels] fp16 tile goes through LDS so that each lane
// reads its channel (16 m + x16) at its 8 token slots as 4 packed fp16 pairs -
// the same (lane group kb, slot) token order as the trit words of the record,
// so a lane assembles its 16 bytes of the record in registers and stores them
// straight to global memory (streaming stores: the record is not read again here).  Work is done on packed halves:
//   sum |v|      : v_dot2_f32_f16(|v| pair, keep pair, acc)  (exact products, fp32 sum)
//   |v| > alpha  : fp16 bit patterns of non-negative values order like integers,
//                  so with thr = alpha rounded toward zero to fp16,
//                  |v| > alpha  <=>  bits(|v|) > bits(thr): bit 15 of thr - |v| (16-bit)
//   v < -alpha   : that flag AND the sign bit of v
#include "mfma_util.h"

namespace vidkv {

constexpr int VENC_ROW = 272;        // LDS bytes per token row (256 + 16 of padding)

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, a) - __builtin_bit_cast(u16x2, b));
}

__global__ __launch_bounds__(256) void v_encode_wave_kernel(const u32x4* __restrict__ V, int T,
                                                            int ng, int B, int H, int n_s,
                                                            float gamma, int gpb, int ngc, int g_out0,
                                                            const uint32_t* __restrict__ mask,
                                                            const uint32_t* __restrict__ rank,
                                                            uint8_t* __restrict__ rec_out,
                                                            u32x4* __restrict__ rows_out) {
  const long long hd = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int x16 = lane & 15, kb = lane >> 4;
  const int b = (int)((hd / H) % B);

  __shared__ u32x4 tile4[4][32 * VENC_ROW / 16];   // per wave: the group's tile
  // my 8 token slots start at row 4*kb (slots 0-3) and 16 + 4*kb (slots 4-7); my channel
  // of tile m is 16 m + x16
  const uint8_t* tcol = reinterpret_cast<const uint8_t*>(&tile4[wave][0]) + 4 * kb * VENC_ROW + 2 * x16;

  const int g_begin = blockIdx.x * gpb;
  const int g_end = min(ng, g_begin + gpb);
  const u32x4* head = V + hd * (long long)T * 16;

  u32x4 pre[8];
  auto prefetch = [&](int g) {
    const u32x4* src = head + (long long)g * G * 16 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) pre[i] = __builtin_nontemporal_load(src + 64 * i);
  };
  int g = g_begin + wave;
  if (g < g_end) prefetch(g);

  for (; g < g_end; g += 4) {
    {
      uint8_t* wdst = reinterpret_cast<uint8_t*>(&tile4[wave][0]) + kb * VENC_ROW + x16 * 16;
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(wdst + 4 * i * VENC_ROW) = pre[i];
    }
    if (g + 4 < g_end) prefetch(g + 4);

    uint32_t m = 0, r0 = 0;
    if (n_s > 0) {
      m = __builtin_amdgcn_readfirstlane(mask[(size_t)b * ngc + g]);
      r0 = __builtin_amdgcn_readfirstlane(rank[(size_t)b * ngc + g]);
    }
    // per slot pair: 1.0 / 0.0 halves for the sum, 0x8000 / 0 halves for the codes
    uint32_t keepf[4], keepm[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t k0 = ((m >> slot_token(kb, 2 * r)) & 1u) ^ 1u;
      const uint32_t k1 = ((m >> slot_token(kb, 2 * r + 1)) & 1u) ^ 1u;
      keepf[r] = (k0 ? 0x3C00u : 0u) | (k1 ? 0x3C000000u : 0u);
      keepm[r] = (k0 << 15) | (k1 << 31);
    }
    const int n = 32 - __popc(m);
    const float rn = n > 0 ? 1.0f / (float)n : 0.0f;

    uint32_t words[4];
    uint32_t sc16[4];                          // 8 fp16 scales: tile m in half (m & 1) of sc16[m >> 1]
#pragma unroll
    for (int mp = 0; mp < 4; ++mp) {
      Op X[2];
      float part[2];
#pragma unroll
      for (int mh = 0; mh < 2; ++mh) {
        const uint8_t* cp = tcol + 32 * (2 * mp + mh);      // 16 channels = 32 bytes per tile
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int row = (i < 4) ? i : 12 + i;             // relative to row 4*kb
          X[mh].v[i] = *reinterpret_cast<const _Float16*>(cp + row * VENC_ROW);
        }
        float acc = 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          acc = __builtin_amdgcn_fdot2(bits_h2(X[mh].u[r] & 0x7FFF7FFFu), bits_h2(keepf[r]), acc, false);
        part[mh] = acc;
      }
      // sums over the 4 lane groups; afterwards every lane has both totals
      float tot[2];
      {
        auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(part[0]), __float_as_uint(part[1]), false, false);
        const float t = __uint_as_float(r[0]) + __uint_as_float(r[1]);
        auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
        const float u = __uint_as_float(q[0]) + __uint_as_float(q[1]);
        auto w = __builtin_amdgcn_permlane32_swap(__float_as_uint(u), __float_as_uint(u), false, false);
        tot[0] = __uint_as_float(w[0]);
        tot[1] = __uint_as_float(w[1]);
      }
      uint32_t word = 0;
      _Float16 s16[2];
#pragma unroll
      for (int mh = 0; mh < 2; ++mh) {
        const float s = tot[mh] * rn;
        const float alpha = gamma * s;
        s16[mh] = (_Float16)s;
        const uint32_t thr = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(alpha, alpha));
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t ax = X[mh].u[r] & 0x7FFF7FFFu;
          const uint32_t nz = pk_sub_u16(thr, ax) & keepm[r];   // bit 15 / 31: |v| > alpha and kept
          const uint32_t ng_ = nz & X[mh].u[r];                 // ... and v negative
          const uint32_t c = (nz >> 1) | ng_;                   // (nonzero, negative) at bits 14,15 / 30,31
          const int sh = 14 - 2 * r - 8 * mh;                   // field of slot 2r at 8 mh + 2 r, of 2r+1 16 above
          word |= c >> sh;
        }
      }
      words[mp] = word;
      sc16[mp] = h2_bits(h2{s16[0], s16[1]});
    }
    uint8_t* rec = rec_out + (hd * ngc + g_out0 + g) * (long long)VREC;
    u32x4 wv;
    wv[0] = words[0]; wv[1] = words[1]; wv[2] = words[2]; wv[3] = words[3];
    __builtin_nontemporal_store(wv, reinterpret_cast<u32x4*>(rec) + lane);                 // word (kb, x16, mp) at byte 16 lane + 4 mp
    if (kb == 0) {
      u32x4 sv;
      sv[0] = sc16[0]; sv[1] = sc16[1]; sv[2] = sc16[2]; sv[3] = sc16[3];
      __builtin_nontemporal_store(sv, reinterpret_cast<u32x4*>(rec + 1024) + x16);         // fp16 [r = x16][m]
    }
    // protected rows, verbatim, to ROWS[rank + order inside the group] (not when they are
    // kept at 2 bits: a pass of its own codes them)
    uint32_t w = rows_out ? m : 0u, r = r0;
    while (w) {
      const int t = __ffs(w) - 1;
      w &= w - 1;
      if (lane < 16)
        __builtin_nontemporal_store(
            *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(&tile4[wave][0]) + t * VENC_ROW + lane * 16),
            rows_out + (hd * n_s + r) * 16 + lane);
      ++r;
    }
  }
}

// n_s = 0 codes every token (a flushed residual block has no protected tokens).
void launch_v_encode(const Geom& g, const EncodeSpan& sp, int n_s, float gamma, const void* V,
                     uint8_t* packed, hipStream_t st) {
  // one group per wave: many short-lived workgroups balance the memory system best here
  const int gpb = 4;
  dim3 grid((sp.ng + gpb - 1) / gpb, (unsigned)sp.heads);
  hipLaunchKernelGGL(v_encode_wave_kernel, grid, dim3(256), 0, st, reinterpret_cast<const u32x4*>(V),
                     sp.in_tokens, sp.ng, g.B, g.H, n_s, gamma, gpb, g.ngc, sp.g_out0,
                     reinterpret_cast<const uint32_t*>(packed + g.v_mask),
                     reinterpret_cast<const uint32_t*>(packed + g.v_rank),
                     packed + g.v_rec + (size_t)sp.head0 * g.ngc * VREC,
                     g.sal_bits == 16 ? reinterpret_cast<u32x4*>(packed + g.v_rows) : nullptr);
}

}  // namespace vidkv
