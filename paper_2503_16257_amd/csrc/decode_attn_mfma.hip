// MFMA decode attention over the packed cache (Eq. 3; Alg. 1, Decoding).
//
// One wave walks PAIRS of 32-token groups.  All contractions run on
// v_mfma_f32_16x16x32_f16 with operands that are exact in fp16 and fp32
// accumulation:
//   * normal key channels (Eq. 5): rows = DFT coefficient slot, K = channels,
//     operand value -(+-s) built from one sign bit and the stored fp16 scale;
//     columns = (group parity, query head) with -q/16 as the other operand.
//     The result is already laid out as the B operand of the next product,
//   * a 32-point inverse real DFT as a product with a constant matrix (split
//     into fp16 hi + lo parts, as is Y) giving scores[token][head],
//   * anomalous key channels (Eq. 4): code*s + z = (z + 1.5 s) + s0 (s/2) + s1 s
//     with s0, s1 = +-1 taken from the two code bits, rows = tokens,
//   * P V: rows = channels, K = tokens, operand +-s/2 * 2 or 0 from the trits.
// Softmax is online in the exp2 domain with a lazily raised running maximum
// shared by the two parities of a head.  Protected (fp16) value rows are added
// on the VALU from the probabilities staged in LDS.
//
// MFMA register layout used throughout (lane = 16*kb + x, x = lane & 15):
//   A operand: row x,    k = 8*kb .. 8*kb+7       B operand: column x, same k
//   C/D      : column x, rows 4*kb .. 4*kb+3
#include "decode_attn.h"

namespace vidkv {

// packed fp16 multiply of a by the low / high half of s broadcast to both lanes
__device__ __forceinline__ uint32_t pk_mul_bcast_lo(uint32_t a, uint32_t s) {
  uint32_t d;
  asm("v_pk_mul_f16 %0, %1, %2 op_sel_hi:[1,0]" : "=v"(d) : "v"(a), "v"(s));
  return d;
}
__device__ __forceinline__ uint32_t pk_mul_bcast_hi(uint32_t a, uint32_t s) {
  uint32_t d;
  asm("v_pk_mul_f16 %0, %1, %2 op_sel:[0,1] op_sel_hi:[1,1]" : "=v"(d) : "v"(a), "v"(s));
  return d;
}

constexpr int KCH_MAX = 1536 / 16;     // 16-byte chunks of the largest key record

template <int NA8>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(AttnArgs a) {
  constexpr int NA = 8 * NA8, NN = D - NA;
  constexpr int NB = NN / 8;                 // normal 8-channel blocks
  constexpr int U = (NB + 3) / 4;            // K-steps over normal channels
  constexpr int NQ = NA / 4;                 // anomalous 4-channel quads
  constexpr int UA = (NQ + 3) / 4;           // K-steps over anomalous channels
  constexpr int KREC = 12 * NA + 8 * NN;
  constexpr int KCH = KREC / 16;
  constexpr int OFF_AS = 8 * NA, OFF_AZ = 10 * NA, OFF_BITS = 12 * NA, OFF_META = 12 * NA + 4 * NN;

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform
  const int x16 = lane & 15, kb = lane >> 4;
  const int hcol = x16 & 7, par = x16 >> 3;          // column role: (parity, head)
  const int R = a.rep;
  const long long hd = ((long long)a.layer * a.B + b) * a.H + kvh;

  __shared__ u32x4 kl4[4][2][KCH_MAX];       // per wave: key records of the two groups
  __shared__ float pl[4][32][16];            // per wave: probabilities [token][column]
  __shared__ float al8[4][8];                // per wave: rescale factors per head
  __shared__ float ow[4][8][D];              // per wave partial outputs
  __shared__ float mw[4][8], lw[4][8];

  // ---------------- constant operands (q and the channel permutation via LDS)
  __shared__ _Float16 qs[8][D];
  __shared__ uint8_t perm_s[D];
  {
    const uint32_t* qsrc = reinterpret_cast<const uint32_t*>(a.q + ((long long)b * a.Hq + kvh * R) * D);
    for (int i = tid; i < R * (D / 2); i += 256) reinterpret_cast<uint32_t*>(&qs[0][0])[i] = qsrc[i];
    if (tid < D / 4)
      reinterpret_cast<uint32_t*>(perm_s)[tid] = reinterpret_cast<const uint32_t*>(a.kperm + hd * D)[tid];
  }
  __syncthreads();
  const bool hv = hcol < R;
  const _Float16* qrow = &qs[hv ? hcol : 0][0];
  const uint8_t* perm = perm_s;
  Op Bn[U > 0 ? U : 1];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int blk = 4 * u + kb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = 0.0f;
      if (hv && blk < NB) v = -(float)qrow[perm[NA + 8 * blk + e]] * 0.0625f;
      Bn[u].v[e] = (_Float16)v;
    }
  }
  Op Ba[UA > 0 ? UA : 1];
#pragma unroll
  for (int ua = 0; ua < UA; ++ua) {
    const int quad = 4 * ua + kb;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float v = 0.0f;
      if (hv && quad < NQ) v = -(float)qrow[perm[4 * quad + r]];
      Ba[ua].p[r] = h2{(_Float16)v, (_Float16)v};
    }
  }
  // 16 * (inverse real DFT matrix): row t, k-slot (kb, i): i < 4 -> Re X[4kb+i],
  // i >= 4 -> Im X[4kb+i-4] (Re X[16] when that index is 0)
  Op Wh[2], Wl[2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int t = 16 * mt + x16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = 4 * kb + (i & 3);
      float w;
      if (i < 4) w = (k == 0) ? 0.5f : kCosT[(k * t) & 31];
      else       w = (k == 0) ? ((t & 1) ? -0.5f : 0.5f) : -kCosT[(k * t + 24) & 31];
      const _Float16 hi = (_Float16)w;
      Wh[mt].v[i] = hi;
      Wl[mt].v[i] = (_Float16)(w - (float)hi);
    }
  }

  // ---------------- running state
  f4 o[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) o[m] = f4{0.f, 0.f, 0.f, 0.f};
  float osal[8][2];
#pragma unroll
  for (int h = 0; h < 8; ++h) { osal[h][0] = 0.f; osal[h][1] = 0.f; }
  float m_run = -INFINITY, l_run = 0.0f;

  const int npairs = (a.ng + 1) >> 1;
  const int p_begin = split * a.gps;
  const int p_end = min(npairs, p_begin + a.gps);

  const uint8_t* krec_base = a.krec + hd * a.ng * (long long)KREC;
  const uint8_t* vrec_base = a.vrec + hd * a.ng * (long long)VREC;

  // prefetch registers: key record chunks, value words and scales of both groups
  u32x4 kpre[2][2], vwpre[2], vspre[2];
  auto prefetch = [&](int p) {
#pragma unroll
    for (int grp = 0; grp < 2; ++grp) {
      const int g = min(2 * p + grp, a.ng - 1);
      const u32x4* ks = reinterpret_cast<const u32x4*>(krec_base + (long long)g * KREC);
      kpre[grp][0] = ks[lane < KCH ? lane : 0];
      kpre[grp][1] = ks[lane + 64 < KCH ? lane + 64 : 0];
      const u32x4* vs = reinterpret_cast<const u32x4*>(vrec_base + (long long)g * VREC);
      vwpre[grp] = vs[lane];
      vspre[grp] = vs[64 + x16];
    }
  };
  // Protected rows are fetched one pair ahead, their masks two pairs ahead.
  // The rows of one pair are consecutive in ROWS (rank grows with the token).
  constexpr int NROW = 8;
  uint32_t rowcur[NROW], rownext[NROW];
  uint32_t sm0c = 0, sm1c = 0, rkc = 0, sm0n = 0, sm1n = 0, rkn = 0;
  const bool has_sal = a.n_s > 0;
  auto load_masks = [&](int pp, uint32_t& s0, uint32_t& s1, uint32_t& rk) {
    s0 = s1 = rk = 0;
    if (has_sal && pp < p_end) {
      const size_t gi = (size_t)b * a.ng + 2 * pp;
      s0 = a.vmask[gi];
      rk = a.vrank[gi];
      if (2 * pp + 1 < a.ng) s1 = a.vmask[gi + 1];
    }
  };
  auto issue_rows = [&](uint32_t s0, uint32_t s1, uint32_t rk, uint32_t* rows) {
    const int cnt = __popc(s0) + __popc(s1);
    const uint32_t* base = reinterpret_cast<const uint32_t*>(a.vrows + (hd * a.n_s + rk) * D) + lane;
#pragma unroll
    for (int j = 0; j < NROW; ++j)
      if (j < cnt) rows[j] = base[j * (D / 2)];
  };
  int p = p_begin + wave;
  if (p < p_end) prefetch(p);
  if (has_sal) {
    load_masks(p, sm0c, sm1c, rkc);
    load_masks(p + 4, sm0n, sm1n, rkn);
    if (sm0c | sm1c) issue_rows(sm0c, sm1c, rkc, rowcur);
  }

  for (; p < p_end; p += 4) {
    const bool v1ok = (2 * p + 1) < a.ng;
    // ---- commit the prefetched data, start the next prefetch
    u32x4 vw[2], vs[2];
#pragma unroll
    for (int grp = 0; grp < 2; ++grp) {
      if (lane < KCH) kl4[wave][grp][lane] = kpre[grp][0];
      if (lane + 64 < KCH) kl4[wave][grp][lane + 64] = kpre[grp][1];
      vw[grp] = vwpre[grp];
      vs[grp] = vspre[grp];
    }
    if (p + 4 < p_end) prefetch(p + 4);
    uint32_t sm0f = 0, sm1f = 0, rkf = 0;        // masks of the pair after the next one
    if (has_sal) {
      if (sm0n | sm1n) issue_rows(sm0n, sm1n, rkn, rownext);
      load_masks(p + 8, sm0f, sm1f, rkf);
    }

    // ---- normal channels: Y[slot][col] per group, K = channels
    f4 accRe[2], accIm[2];
    if (U > 0) {
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint8_t* rec = reinterpret_cast<const uint8_t*>(&kl4[wave][grp][0]);
        accRe[grp] = f4{0.f, 0.f, 0.f, 0.f};
        accIm[grp] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int blk = min(4 * u + kb, NB - 1);
          const uint32_t w = *reinterpret_cast<const uint16_t*>(rec + OFF_BITS + (blk * 16 + x16) * 2);
          const uint32_t xx = w | (w << 15);
          Op sre, sim, A;
          sre.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2) * 16);
          sim.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2 + (x16 ? 1 : 0)) * 16);
#pragma unroll
          for (int r = 0; r < 4; ++r) A.u[r] = ((xx << (15 - 2 * r)) & 0x80008000u) | sre.u[r];
          accRe[grp] = mma(A, Bn[u], accRe[grp]);
#pragma unroll
          for (int r = 0; r < 4; ++r) A.u[r] = ((xx << (7 - 2 * r)) & 0x80008000u) | sim.u[r];
          accIm[grp] = mma(A, Bn[u], accIm[grp]);
        }
      }
    }
    f4 S[2] = {f4{0.f, 0.f, 0.f, 0.f}, f4{0.f, 0.f, 0.f, 0.f}};
    if (U > 0) {
      // my column belongs to group `par`; split Y/16 into fp16 hi + lo
      Op Yh, Yl;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float yr = par ? accRe[1][i] : accRe[0][i];
        const float yi = par ? accIm[1][i] : accIm[0][i];
        const _Float16 hr = (_Float16)yr, hi = (_Float16)yi;
        Yh.v[i] = hr;
        Yh.v[4 + i] = hi;
        Yl.v[i] = (_Float16)(yr - (float)hr);
        Yl.v[4 + i] = (_Float16)(yi - (float)hi);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        S[mt] = mma(Wh[mt], Yh, S[mt]);
        S[mt] = mma(Wl[mt], Yh, S[mt]);
        S[mt] = mma(Wh[mt], Yl, S[mt]);
      }
    }
    // ---- anomalous channels: rows = tokens, K = (channel, bit plane)
    float cst = 0.0f;
    if (UA > 0) {
      f4 accA[2][2], accC[2];
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint8_t* rec = reinterpret_cast<const uint8_t*>(&kl4[wave][grp][0]);
        accA[grp][0] = accA[grp][1] = accC[grp] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ua = 0; ua < UA; ++ua) {
          const int quad = min(4 * ua + kb, NQ - 1);
          union { uint2 u; _Float16 e[4]; } s4, z4;
          s4.u = *reinterpret_cast<const uint2*>(rec + OFF_AS + quad * 8);
          z4.u = *reinterpret_cast<const uint2*>(rec + OFF_AZ + quad * 8);
          uint32_t sp[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) sp[r] = h2_bits(h2{s4.e[r] * (_Float16)0.5f, s4.e[r]});
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) {
            const uint32_t w = rec[(16 * mt + x16) * NQ + quad];
            const uint32_t xx = w | (w << 15);
            Op A;
#pragma unroll
            for (int r = 0; r < 4; ++r) A.u[r] = ((xx << (15 - 2 * r)) & 0x80008000u) | sp[r];
            accA[grp][mt] = mma(A, Ba[ua], accA[grp][mt]);
          }
          // constant part z + 1.5 s = z + s + s/2, same for every row
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            Op Ac, Bc;
            Ac.p[0] = h2{z4.e[2 * hf], s4.e[2 * hf]};
            Ac.u[1] = sp[2 * hf] & 0xFFFFu;
            Ac.p[2] = h2{z4.e[2 * hf + 1], s4.e[2 * hf + 1]};
            Ac.u[3] = sp[2 * hf + 1] & 0xFFFFu;
            Bc.u[0] = Ba[ua].u[2 * hf];
            Bc.u[1] = Ba[ua].u[2 * hf];
            Bc.u[2] = Ba[ua].u[2 * hf + 1];
            Bc.u[3] = Ba[ua].u[2 * hf + 1];
            accC[grp] = mma(Ac, Bc, accC[grp]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        S[0][i] += par ? accA[1][0][i] : accA[0][0][i];
        S[1][i] += par ? accA[1][1][i] : accA[0][1][i];
      }
      cst = par ? accC[1][0] : accC[0][0];      // = -(sum q (z + 1.5 s))
    }
    // ---- scores of my column: token slot i (i < 4: token 4kb+i, else 16+4kb+i-4)
    float sc[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sc[i] = (S[0][i] - cst) * a.scale2;
      sc[4 + i] = (S[1][i] - cst) * a.scale2;
    }
    if (par && !v1ok) {
#pragma unroll
      for (int i = 0; i < 8; ++i) sc[i] = -INFINITY;
    }
    // ---- online softmax.  The running maximum m_run is shared by the 4 k-blocks
    // and the 2 parities of a head and is raised lazily: only when some score
    // exceeds it by more than 8 (p stays below 2^8), which needs no cross-lane
    // traffic in the common case.
    float mx = sc[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sc[i]);
    if (__any(mx > m_run + 8.0f)) {
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 8, 64));
      const float m_new = fmaxf(m_run, mx);
      const float al = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
      for (int m = 0; m < 8; ++m) o[m] *= al;
      l_run *= al;
      m_run = m_new;
      if (has_sal) {
        if (lane < 8) al8[wave][lane] = al;
        float ah[8];
#pragma unroll
        for (int h = 0; h < 8; ++h) ah[h] = al8[wave][h];
#pragma unroll
        for (int h = 0; h < 8; ++h) { osal[h][0] *= ah[h]; osal[h][1] *= ah[h]; }
      }
    }
    float pr[8];
    Op Pp;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pr[i] = __builtin_amdgcn_exp2f(sc[i] - m_run);
      l_run += pr[i];
      Pp.v[i] = (_Float16)pr[i];
    }
    Op Bp[2];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      Bp[0].u[r] = par ? 0u : Pp.u[r];
      Bp[1].u[r] = par ? Pp.u[r] : 0u;
    }
    // ---- P V: rows = channels 16 m + x16, K = token slots
#pragma unroll
    for (int grp = 0; grp < 2; ++grp) {
      Op hs;
#pragma unroll
      for (int r = 0; r < 4; ++r) hs.p[r] = bits_h2(vs[grp][r]) * h2{(_Float16)0.5f, (_Float16)0.5f};
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const uint32_t w = vw[grp][m >> 1];
        Op A;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t t2 = (w << ((m & 1) ? (6 - 2 * r) : (14 - 2 * r))) & 0xC000C000u;   // +-2 or 0
          A.u[r] = (m & 1) ? pk_mul_bcast_hi(t2, hs.u[m >> 1]) : pk_mul_bcast_lo(t2, hs.u[m >> 1]);
        }
        o[m] = mma(A, Bp[grp], o[m]);
      }
    }
    // ---- protected tokens: fp16 rows (prefetched) weighted by the probabilities
    if (has_sal) {
      if (sm0c | sm1c) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int t = (i < 4) ? 4 * kb + i : 16 + 4 * kb + (i - 4);
          pl[wave][t][x16] = pr[i];
        }
        unsigned long long sm = (unsigned long long)sm0c | ((unsigned long long)sm1c << 32);
        auto add_row = [&](uint32_t bits) {
          const int t64 = __ffsll((long long)sm) - 1;      // bit t of parity t64 >> 5
          sm &= sm - 1;
          const h2 v = bits_h2(bits);
          const float v0 = (float)v[0], v1 = (float)v[1];
          const float* pp = &pl[wave][t64 & 31][8 * (t64 >> 5)];
#pragma unroll
          for (int h = 0; h < 8; ++h) {
            const float ph = pp[h];
            osal[h][0] += ph * v0;
            osal[h][1] += ph * v1;
          }
        };
#pragma unroll
        for (int j = 0; j < NROW; ++j)
          if (sm) add_row(rowcur[j]);
        uint32_t rk = rkc + NROW;                           // more than NROW rows: fetch on demand
        while (sm) {
          add_row(*(reinterpret_cast<const uint32_t*>(a.vrows + (hd * a.n_s + rk) * D) + lane));
          ++rk;
        }
      }
      sm0c = sm0n; sm1c = sm1n; rkc = rkn;
      sm0n = sm0f; sm1n = sm1f; rkn = rkf;
#pragma unroll
      for (int j = 0; j < NROW; ++j) rowcur[j] = rownext[j];
    }
  }

  // ---------------- per-wave reduction: 4 k-blocks and 2 parities of each head
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  l_run += __shfl_xor(l_run, 8, 64);
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int i = 0; i < 4; ++i) o[m][i] += __shfl_xor(o[m][i], 8, 64);
  if (par == 0) {
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
      for (int i = 0; i < 4; ++i) ow[wave][hcol][16 * m + 4 * kb + i] = o[m][i];
    if (kb == 0) { mw[wave][hcol] = m_run; lw[wave][hcol] = l_run; }
  }
  if (a.n_s > 0) {
    // same wave, LDS operations complete in order: add the fp16-row part
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      ow[wave][h][2 * lane] += osal[h][0];
      ow[wave][h][2 * lane + 1] += osal[h][1];
    }
  }
  __syncthreads();
  // ---------------- workgroup merge of the 4 waves, then the split partial
  {
    const int c = tid & 127, hh = tid >> 7;
    for (int h = hh; h < R; h += 2) {
      float M = fmaxf(fmaxf(mw[0][h], mw[1][h]), fmaxf(mw[2][h], mw[3][h]));
      float acc = 0.0f, L = 0.0f;
      if (M != -INFINITY) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float mi = mw[w][h];
          if (mi == -INFINITY) continue;
          const float f = exp2f(mi - M);
          acc += f * ow[w][h][c];
          L += f * lw[w][h];
        }
      }
      float* dst = a.part + (((long long)split * a.B + b) * a.Hq + kvh * R + h) * PART_STRIDE;
      dst[c] = acc;
      if (c == 0) { dst[D] = M; dst[D + 1] = L; }
    }
  }
}

bool attn_mfma_supported(int n_a) {
  switch (n_a) {
    case 0: case 8: case 16: case 32: case 64: case 128: return true;
    default: return false;
  }
}

void launch_attn_mfma(const AttnArgs& a, dim3 grid, hipStream_t st) {
  switch (a.n_a) {
    case 0:   hipLaunchKernelGGL(attn_mfma_kernel<0>,  grid, dim3(256), 0, st, a); break;
    case 8:   hipLaunchKernelGGL(attn_mfma_kernel<1>,  grid, dim3(256), 0, st, a); break;
    case 16:  hipLaunchKernelGGL(attn_mfma_kernel<2>,  grid, dim3(256), 0, st, a); break;
    case 32:  hipLaunchKernelGGL(attn_mfma_kernel<4>,  grid, dim3(256), 0, st, a); break;
    case 64:  hipLaunchKernelGGL(attn_mfma_kernel<8>,  grid, dim3(256), 0, st, a); break;
    case 128: hipLaunchKernelGGL(attn_mfma_kernel<16>, grid, dim3(256), 0, st, a); break;
    default: break;
  }
}

}  // namespace vidkv
