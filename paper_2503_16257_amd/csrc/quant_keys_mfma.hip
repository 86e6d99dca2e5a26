// Key coding pass (Alg. 3): per 32-token group the 2-bit uniform code (Eq. 4)
// of the anomalous channels and the FFT-based 1-bit code (Eq. 5) of the others.
//
// The 32-point DFT along the tokens is a dense contraction, so it runs on
// v_mfma_f32_16x16x32_f16.  One wave codes one group at a time:
//  1. The [32 tokens x 128 channels] fp16 tile goes global -> registers -> LDS
//     with 16-byte accesses (rows padded to 272 bytes).
//  2. Each lane reads, for a tile of 16 channels taken from the head's channel
//     permutation, its channel at its 8 token slots with 16-bit LDS loads that
//     fill register halves directly: the MFMA operand of a contraction over
//     tokens, gathered and transposed for free.
//  3. Normal channels: the DFT matrix, split in three fp16 parts (exact products,
//     fp32 accumulation), times X (32 tokens x 16 channels), as [slot][channel]:
//     each lane gets 8 coefficients of one channel, so the mean-|.| scales need
//     only a 4-lane sum, and a wave-wide ballot of "coefficient >= 0" per
//     accumulator register holds, byte by byte, the record's sign words (8
//     channels of one slot per byte).  One orientation serves both: the key
//     coding pass is limited by what the SIMDs can sustain, not by HBM alone, and
//     a second orientation for the sign bits cost 40 % more MFMA work.
//  4. Anomalous channels: min / max over the 32 tokens, codes, 4 channels per
//     byte assembled inside lane quads.
// The record is assembled in LDS and written with 16-byte stores.
#include "mfma_util.h"

namespace vidkv {

constexpr int ENC_MAXT = 9;          // channel tiles of 16: at most 1 + 8
constexpr int ENC_ROW = 272;         // LDS bytes per token row (256 + 16 of padding)

// DFT operand table.  Slot x of tile tt (tt = 0: Re X[0..15]; tt = 1: Re X[16],
// Im X[1..15]) against token t: 64 * (w/2) * {cos, -sin}(2 pi k t / 32), with
// w = 1 for the two real-only bins and 2 otherwise, so that the sum of |D| over
// a channel's slots is 1024 * Mean|.| of Eq. 5; positive row scaling does not
// change a sign.  Each fp32 entry is split into three fp16 parts that add up to
// it exactly.  Indexed [tt][part][lane][4 words]: the 8 halves of a lane's
// MFMA operand (slot x = lane & 15, tokens slot_token(lane >> 4, 0..7)).
struct DftTab { uint32_t w[2][3][64][4]; };

constexpr uint32_t half_bits(_Float16 h) { return __builtin_bit_cast(uint16_t, h); }

constexpr DftTab make_dft_tab() {
  DftTab tab{};
  for (int tt = 0; tt < 2; ++tt)
    for (int lane = 0; lane < 64; ++lane)
      for (int i = 0; i < 8; ++i) {
        const int kb = lane >> 4, k = lane & 15;
        const int t = (i < 4) ? 4 * kb + i : 16 + 4 * kb + (i - 4);
        float w = 0.0f;
        if (tt == 0) w = cos32(k * t) * (k == 0 ? 32.0f : 64.0f);
        else         w = (k == 0) ? ((t & 1) ? -32.0f : 32.0f) : -cos32(k * t + 24) * 64.0f;
        if (w == 0.0f) w = 0.0f;                       // no negative zero
        const _Float16 a = (_Float16)w;
        const float r1 = w - (float)a;
        const _Float16 b = (_Float16)r1;
        const _Float16 c = (_Float16)(r1 - (float)b);
        const int sh = 16 * (i & 1);
        tab.w[tt][0][lane][i >> 1] |= half_bits(a) << sh;
        tab.w[tt][1][lane][i >> 1] |= half_bits(b) << sh;
        tab.w[tt][2][lane][i >> 1] |= half_bits(c) << sh;
      }
  return tab;
}

static __device__ const DftTab kDftTab = make_dft_tab();

// NA8T >= 0 fixes n_a = 8 * NA8T at compile time (tile loop fully unrolled);
// NA8T < 0 takes n_a at run time.  FFT = false codes the normal channels with
// Eq. 4 at 1 bit on the tokens themselves (the non-FFT 1-bit path of Alg. 3):
// the record keeps its shape, bit (blk, k) e / 8 + e holds the code of channel
// 8 blk + e at token k / 16 + k, and the two scale slots hold s = max - min and
// z = min.
template <int NA8T, bool FFT>
__global__ __launch_bounds__(256) void k_encode_mfma_kernel(const u32x4* __restrict__ K,
                                                            const uint8_t* __restrict__ perm_g,
                                                            int T, int ng, int n_a_rt, int krec, int gpb,
                                                            int ngc, int g_out0,
                                                            uint8_t* __restrict__ rec_out) {
  const int n_a = NA8T >= 0 ? 8 * NA8T : n_a_rt;
  const long long hd = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int x16 = lane & 15, kb = lane >> 4;
  const int n_n = D - n_a;
  const int NTa = (n_a + 15) >> 4, NTn = (n_n + 15) >> 4, NT = NTa + NTn;
  const int nq = n_a >> 2;

  __shared__ u32x4 tile4[4][32 * ENC_ROW / 16];   // per wave: the group's tile
  // per wave: the record being assembled (12 n_a + 8 n_n bytes; 1536 at most).  With n_a known
  // the workgroup stays below a quarter of the LDS and four of them share a compute unit.
  constexpr int RECB = NA8T >= 0 ? 12 * 8 * NA8T + 8 * (D - 8 * NA8T) : 1536;
  __shared__ u32x4 recbuf[4][RECB / 16];

  // the first tile is requested before anything else so that its latency
  // overlaps the set-up below
  const int g_begin = blockIdx.x * gpb;
  const int g_end = min(ng, g_begin + gpb);
  const u32x4* head = K + hd * (long long)T * 16;

  // coalesced tile load: lane reads 16 bytes of row (lane >> 4) + 4 i, i = 0..7
  u32x4 pre[8];
  auto prefetch = [&](int g) {
    const u32x4* src = head + (long long)g * G * 16 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) pre[i] = __builtin_nontemporal_load(src + 64 * i);
  };
  int g = g_begin + wave;
  if (g < g_end) prefetch(g);

  // Channel tile j: anomalous tiles first (16 anomalous channels each, in PERM
  // order), then normal tiles.  My column's channel in every tile, as a byte
  // offset inside a token row (an absent column reads channel 0 and is ignored).
  int chofs[ENC_MAXT];
#pragma unroll
  for (int j = 0; j < ENC_MAXT; ++j) {
    const bool an = j < NTa;
    const int off = an ? 16 * j + x16 : 16 * (j - NTa) + x16;
    const bool valid = j < NT && (an ? off < n_a : off < n_n);
    chofs[j] = valid ? 2 * (int)perm_g[hd * D + (an ? off : n_a + off)] : 0;
  }

  // DFT operand from the precomputed table: slot x16 of tile tt, k-slots = tokens
  Op F[2][3];
  if (FFT) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int part = 0; part < 3; ++part)
        F[tt][part].q = *reinterpret_cast<const u32x4*>(&kDftTab.w[tt][part][lane][0]);
  }

  uint8_t* rec8 = reinterpret_cast<uint8_t*>(&recbuf[wave][0]);
  uint16_t* rec16 = reinterpret_cast<uint16_t*>(rec8);
  const int bits_h = 6 * n_a;                        // half-word offsets inside the record
  const int meta_h = 6 * n_a + 2 * n_n;
  const int nblk = n_n >> 3;
  // my 8 token slots start at row 4*kb (slots 0-3) and 16 + 4*kb (slots 4-7)
  const uint8_t* tcol = reinterpret_cast<const uint8_t*>(&tile4[wave][0]) + 4 * kb * ENC_ROW;

  for (; g < g_end; g += 4) {
    {
      uint8_t* wdst = reinterpret_cast<uint8_t*>(&tile4[wave][0]) + kb * ENC_ROW + x16 * 16;
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(wdst + 4 * i * ENC_ROW) = pre[i];
    }
    if (g + 4 < g_end) prefetch(g + 4);

#pragma unroll
    for (int j = 0; j < ENC_MAXT; ++j) {
      if (j >= NT) break;
      // my column's channel at my 8 token slots: 16-bit LDS loads into register halves
      Op X;
      const uint8_t* cp = tcol + chofs[j];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = (i < 4) ? i : 12 + i;          // relative to row 4*kb
        X.v[i] = *reinterpret_cast<const _Float16*>(cp + row * ENC_ROW);
      }

      if (j < NTa) {
        // ---------------- Eq. 4, 2 bits: z = min, s = (max - min) / 3 over the 32 tokens
        h2 mn2 = __builtin_elementwise_min(__builtin_elementwise_min(X.p[0], X.p[1]),
                                           __builtin_elementwise_min(X.p[2], X.p[3]));
        h2 mx2 = __builtin_elementwise_max(__builtin_elementwise_max(X.p[0], X.p[1]),
                                           __builtin_elementwise_max(X.p[2], X.p[3]));
        // min and -max over the 4 lane groups: both are "min" reductions, so one
        // swap pair serves the two values; a last swap hands both to every lane
        float lo_f = fminf((float)mn2[0], (float)mn2[1]);
        float nh_f = -fmaxf((float)mx2[0], (float)mx2[1]);
        {
          auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo_f), __float_as_uint(nh_f), false, false);
          const float t = fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
          auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
          const float u = fminf(__uint_as_float(q[0]), __uint_as_float(q[1]));   // rows 0,1: min; rows 2,3: -max
          auto w = __builtin_amdgcn_permlane32_swap(__float_as_uint(u), __float_as_uint(u), false, false);
          lo_f = __uint_as_float(w[0]);
          nh_f = __uint_as_float(w[1]);
        }
        const float mnf = lo_f, rng = -nh_f - lo_f;
        const float inv = rng > 0.0f ? 3.0f / rng : 0.0f;
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float u = ((float)X.v[i] - mnf) * inv;
          u = fminf(fmaxf(rintf(u), 0.0f), 3.0f);
          const uint32_t c = (uint32_t)u;
          if (i < 4) w0 |= c << (8 * i); else w1 |= c << (8 * (i - 4));
        }
        // 4 channels of a quad (adjacent lanes) share a byte: channel r in bits 2r, 2r+1
        w0 <<= 2 * (x16 & 3);
        w1 <<= 2 * (x16 & 3);
        const int ja = 16 * j + x16;                 // anomalous index of my column
        if (ja >= n_a) { w0 = 0; w1 = 0; }
        w0 |= __shfl_xor(w0, 1, 64);  w1 |= __shfl_xor(w1, 1, 64);
        w0 |= __shfl_xor(w0, 2, 64);  w1 |= __shfl_xor(w1, 2, 64);
        if (ja < n_a) {
          const int quad = ja >> 2;
          if ((x16 & 3) == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              rec8[(4 * kb + i) * nq + quad] = (uint8_t)(w0 >> (8 * i));
              rec8[(16 + 4 * kb + i) * nq + quad] = (uint8_t)(w1 >> (8 * i));
            }
          }
          if (kb == 0) {
            reinterpret_cast<_Float16*>(rec16)[4 * n_a + ja] = (_Float16)(rng / 3.0f);
            reinterpret_cast<_Float16*>(rec16)[5 * n_a + ja] = (_Float16)lo_f;
          }
        }
      } else if (!FFT) {
        // ---------------- Eq. 4, 1 bit: z = min, s = max - min over the 32 tokens
        const int jn = j - NTa;
        h2 mn2 = __builtin_elementwise_min(__builtin_elementwise_min(X.p[0], X.p[1]),
                                           __builtin_elementwise_min(X.p[2], X.p[3]));
        h2 mx2 = __builtin_elementwise_max(__builtin_elementwise_max(X.p[0], X.p[1]),
                                           __builtin_elementwise_max(X.p[2], X.p[3]));
        float lo_f = fminf((float)mn2[0], (float)mn2[1]);
        float nh_f = -fmaxf((float)mx2[0], (float)mx2[1]);
        {
          auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo_f), __float_as_uint(nh_f), false, false);
          const float t = fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
          auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
          const float u = fminf(__uint_as_float(q[0]), __uint_as_float(q[1]));   // rows 0,1: min; rows 2,3: -max
          auto w = __builtin_amdgcn_permlane32_swap(__float_as_uint(u), __float_as_uint(u), false, false);
          lo_f = __uint_as_float(w[0]);
          nh_f = __uint_as_float(w[1]);
        }
        const float rng = -nh_f - lo_f;
        // code = round-half-even((x - z) / s) in {0, 1} = [x above the midpoint]; a tie codes 0
        const float mid = 0.5f * (lo_f - nh_f);
        const int nidx = 16 * jn + x16;              // normal index of my column
        // ballot i: bit 16 kb + 8 h + e = code of channel 8 (2 jn + h) + e at token slot (kb, i)
        unsigned long long bal[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) bal[i] = __ballot(nidx < n_n && (float)X.v[i] > mid);
        // lane (h = lane / 16, k = lane % 16) < 32 assembles word (blk 2 jn + h, k): low byte =
        // token k = slot (k / 4, k % 4), high byte = token 16 + k = slot (k / 4, 4 + k % 4)
        {
          const int k = x16, h = kb & 1, ii = k & 3;
          unsigned long long lo8 = ii == 0 ? bal[0] : ii == 1 ? bal[1] : ii == 2 ? bal[2] : bal[3];
          unsigned long long hi8 = ii == 0 ? bal[4] : ii == 1 ? bal[5] : ii == 2 ? bal[6] : bal[7];
          const int sh = 8 * (2 * (k >> 2) + h);
          const uint32_t w16 = (uint32_t)((lo8 >> sh) & 0xFFull) | ((uint32_t)((hi8 >> sh) & 0xFFull) << 8);
          const int blk = 2 * jn + h;
          if (kb < 2 && blk < nblk) rec16[bits_h + blk * 16 + k] = (uint16_t)w16;
        }
        if ((kb & 1) == 0 && nidx < n_n) {
          const int b8 = nidx >> 3, e = nidx & 7;
          reinterpret_cast<_Float16*>(rec16)[meta_h + (b8 * 2 + (kb >> 1)) * 8 + e] =
              (kb >> 1) ? (_Float16)lo_f : (_Float16)rng;
        }
      } else {
        // ---------------- Eq. 5: 32-point DFT along tokens, sign bits and mean-|.| scales
        const int jn = j - NTa;
        const f4 zero = f4{0.f, 0.f, 0.f, 0.f};
        // [slot][channel]: my column = channel x16, my rows = slots 4kb + i of the two slot
        // tiles (Re X[0..15]; Re X[16], Im X[1..15]); three exact partial products each
        f4 aRe = mma(F[0][0], X, zero), aIm = mma(F[1][0], X, zero);
        aRe = mma(F[0][1], X, aRe);  aIm = mma(F[1][1], X, aIm);
        aRe = mma(F[0][2], X, aRe);  aIm = mma(F[1][2], X, aIm);
        const int nidx = 16 * jn + x16;              // normal index of my column
        // sign bits (bit = coefficient >= 0): ballot i, bit 16 kb + 8 h + e = channel
        // 8 (2 jn + h) + e at slot 4 kb + i
        unsigned long long bre[4], bim[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          bre[i] = __ballot(nidx < n_n && aRe[i] >= 0.0f);
          bim[i] = __ballot(nidx < n_n && aIm[i] >= 0.0f);
        }
        // lane (h = lane / 16, k = lane % 16) < 32 assembles word (blk 2 jn + h, k): low byte
        // = first slot tile at slot k = (k / 4, k % 4), high byte = second slot tile
        {
          const int k = x16, h = kb & 1, ii = k & 3;
          const unsigned long long lo8 = ii == 0 ? bre[0] : ii == 1 ? bre[1] : ii == 2 ? bre[2] : bre[3];
          const unsigned long long hi8 = ii == 0 ? bim[0] : ii == 1 ? bim[1] : ii == 2 ? bim[2] : bim[3];
          const int sh = 8 * (2 * (k >> 2) + h);
          const uint32_t w16 = (uint32_t)((lo8 >> sh) & 0xFFull) | ((uint32_t)((hi8 >> sh) & 0xFFull) << 8);
          const int blk = 2 * jn + h;
          if (kb < 2 && blk < nblk) rec16[bits_h + blk * 16 + k] = (uint16_t)w16;
        }
        // scales: Re X[16] sits in row 0 of the second tile and counts for the real view
        float sr = fabsf(aRe[0]) + fabsf(aRe[1]) + fabsf(aRe[2]) + fabsf(aRe[3]);
        float si = fabsf(aIm[0]) + fabsf(aIm[1]) + fabsf(aIm[2]) + fabsf(aIm[3]);
        if (kb == 0) { sr += fabsf(aIm[0]); si -= fabsf(aIm[0]); }
        // sum over the 4 lane groups: afterwards rows 0,1 hold the Re total, rows 2,3 the Im total
        auto r32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(sr), __float_as_uint(si), false, false);
        const float t2 = __uint_as_float(r32[0]) + __uint_as_float(r32[1]);
        auto r16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(t2), __float_as_uint(t2), false, false);
        const float tot = (__uint_as_float(r16[0]) + __uint_as_float(r16[1])) * (1.0f / 1024.0f);
        if ((kb & 1) == 0 && nidx < n_n) {
          const int b8 = nidx >> 3, e = nidx & 7;
          reinterpret_cast<_Float16*>(rec16)[meta_h + (b8 * 2 + (kb >> 1)) * 8 + e] = (_Float16)tot;
        }
      }
    }
    // ---- the finished record: LDS -> global, 16 bytes per lane
    u32x4* dst = reinterpret_cast<u32x4*>(rec_out + (hd * ngc + g_out0 + g) * (long long)krec);
    const int nch = krec >> 4;
    if (lane < nch) __builtin_nontemporal_store(recbuf[wave][lane], dst + lane);
    if (lane + 64 < nch) __builtin_nontemporal_store(recbuf[wave][lane + 64], dst + lane + 64);
  }
}

void launch_k_encode(const Geom& g, const EncodeSpan& sp, const void* K, uint8_t* packed,
                     bool use_fft, hipStream_t st) {
  // two groups per wave: short-lived workgroups keep the memory system evenly loaded,
  // and the second group's load overlaps the first group's arithmetic
  const int gpb = 8;
  dim3 grid((sp.ng + gpb - 1) / gpb, (unsigned)sp.heads);
  const u32x4* k4 = reinterpret_cast<const u32x4*>(K);
  const uint8_t* perm = packed + g.k_perm + sp.head0 * D;
  uint8_t* rec = packed + g.k_rec + (size_t)sp.head0 * g.ngc * g.krec;
#define VIDKV_ENC(N)                                                                          \
  do {                                                                                        \
    if (use_fft)                                                                              \
      hipLaunchKernelGGL((k_encode_mfma_kernel<N, true>), grid, dim3(256), 0, st, k4, perm,   \
                         sp.in_tokens, sp.ng, g.n_a, g.krec, gpb, g.ngc, sp.g_out0, rec);     \
    else                                                                                      \
      hipLaunchKernelGGL((k_encode_mfma_kernel<N, false>), grid, dim3(256), 0, st, k4, perm,  \
                         sp.in_tokens, sp.ng, g.n_a, g.krec, gpb, g.ngc, sp.g_out0, rec);     \
  } while (0)
  switch (g.n_a) {
    case 8:  VIDKV_ENC(1); break;
    case 16: VIDKV_ENC(2); break;
    case 32: VIDKV_ENC(4); break;
    case 64: VIDKV_ENC(8); break;
    default: VIDKV_ENC(-1); break;
  }
#undef VIDKV_ENC
}

}  // namespace vidkv
