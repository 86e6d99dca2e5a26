// MFMA decode attention over the packed cache (Eq. 3; Alg. 1, Decoding).
//
// One wave walks PAIRS of 32-token groups; the 16 "columns" of the score tiles
// are (group parity, query head <= 8).  All contractions run on
// v_mfma_f32_16x16x32_f16 with operands that are exact in fp16 and fp32
// accumulation:
//   * normal key channels (Eq. 5): rows = DFT coefficient slot, K = channels,
//     operand value -(+-s) built from one sign bit and the stored fp16 scale;
//     columns carry -q/16.  The result tile is already laid out as the B operand
//     of the next product,
//   * a 32-point inverse real DFT as a product with a constant matrix (split
//     into fp16 hi + lo parts, as is Y) giving scores[token][column],
//   * anomalous key channels (Eq. 4): code*s + z = (z + 1.5 s) + s0 (s/2) + s1 s
//     with s0, s1 = +-1 taken from the two code bits, rows = tokens; the column
//     operand is masked by parity so both groups add into the same score tile,
//   * P V: rows = columns of the score tile (probabilities are reused in place
//     as the A operand), K = tokens, columns = channels with operand +-2 / 0 from
//     the trits; the per-channel scale of Eq. 6 multiplies the fp32 result.
// Softmax is online in the exp2 domain with a lazily raised running maximum
// shared by the two parities of a head.  Protected (fp16) value rows are added
// on the VALU from the probabilities staged in LDS.
#include "decode_attn.h"

namespace vidkv {

constexpr int KCH_MAX = 1536 / 16;     // 16-byte chunks of the largest key record

__device__ __forceinline__ uint32_t pkrtz(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
__device__ __forceinline__ float swap_sum32(float v) {       // v(lane) + v(lane ^ 32)
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float swap_sum16(float v) {       // v(lane) + v(lane ^ 16)
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float swap_max32(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float swap_max16(float v) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// SAL: 0 no protected tokens, 1 protected rows in fp16, 2 protected rows as 2-bit records.
// FFT: normal key channels coded by Eq. 5 (true) or by Eq. 4 at 1 bit on the tokens (false);
// in the latter case slot = token and code * s + z = (z + s/2) + sigma * s/2, sigma = +-1,
// so the same sign-type operand serves, without the inverse DFT and with a constant term.
template <int NA8, int SAL, bool FFT>
__global__ __launch_bounds__(256, (SAL == 0 && NA8 <= 4) ? 3 : 2) void attn_mfma_kernel(AttnArgs a) {
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
  const f4 zero = f4{0.f, 0.f, 0.f, 0.f};

  constexpr bool KDMA = (SAL == 0);          // key records by direct loads into LDS (see prefetch)
  __shared__ u32x4 kl4[KDMA ? 2 : 1][4][2][KCH_MAX];   // per wave: key records of the two groups
  __shared__ float pl[4][32][16];            // per wave: probabilities [token][column]
  __shared__ float al16[4][16];              // per wave: rescale factors per column
  __shared__ float ow[4][8][D];              // per wave partial outputs
  __shared__ float mw[4][8], lw[4][8];
  __shared__ _Float16 qs[8][D];
  __shared__ __align__(16) uint8_t perm_s[D];

  // ---------------- prefetch machinery (the first request is placed in the set-up below)
  const int npairs = (a.ng + 1) >> 1;
  const int p_begin = split * a.gps;
  const int p_end = min(npairs, p_begin + a.gps);

  const uint8_t* krec_base = a.krec + hd * a.ngc * (long long)KREC;
  const uint8_t* vrec_base = a.vrec + hd * a.ngc * (long long)VREC;

  // Prefetch, one pair ahead.  Without protected tokens the key records go from memory
  // straight into the other LDS buffer (lane l of a wave-wide global_load_lds_dwordx4 lands
  // at M0 + 16 l, i.e. the record keeps its byte order): 16 registers fewer, which is what
  // lets that variant run 3 waves per SIMD.  The compiler is not told about these LDS writes,
  // so the wait that precedes the first read of a buffer is written out below - a wait for
  // every outstanding load, which is why the variants with protected rows (whose row loads
  // are issued late and needed late) keep the key records in registers instead.  The value
  // words of both groups and the value scales of the group whose rows this lane owns in the
  // PV tile (parity kb >> 1) go to registers.
  // (M0, the LDS base of the transfer, is written inside the asm statement; it is a reserved
  // register that the compiler sets itself right before each of its own uses.)
  const uint32_t kl_lds = (uint32_t)reinterpret_cast<uintptr_t>(&kl4[0][0][0][0]);
  auto dma16 = [&](const u32x4* g, uint32_t lds_byte) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                 :: "s"(lds_byte), "v"(g) : "memory");
  };
  u32x4 kpre[2][2], vwpre[2], vspre;
  auto prefetch = [&](int p, int buf) {
#pragma unroll
    for (int grp = 0; grp < 2; ++grp) {
      const int g = min(2 * p + grp, a.ng - 1);
      const u32x4* ks = reinterpret_cast<const u32x4*>(krec_base + (long long)g * KREC);
      if (KDMA) {
        const uint32_t la = kl_lds + (uint32_t)((((buf * 4 + wave) * 2 + grp) * KCH_MAX) * 16);
        dma16(ks + lane, la);
        if (KCH > 64 && lane + 64 < KCH) dma16(ks + lane + 64, la + 1024u);
      } else {
        kpre[grp][0] = __builtin_nontemporal_load(ks + lane);
        kpre[grp][1] = __builtin_nontemporal_load(ks + (lane + 64 < KCH ? lane + 64 : 0));
      }
      const u32x4* vs = reinterpret_cast<const u32x4*>(vrec_base + (long long)g * VREC);
      vwpre[grp] = __builtin_nontemporal_load(vs + lane);
    }
    const int gs = min(2 * p + (kb >> 1), a.ng - 1);
    vspre = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vrec_base + (long long)gs * VREC) + 64 + x16);
  };
  // Protected rows are fetched one pair ahead, their masks two pairs ahead.
  // The rows of one pair are consecutive in ROWS (rank grows with the token).
  constexpr int NROW = 8;
  uint32_t rowcur[NROW], rownext[NROW];
  uint32_t sm0c = 0, sm1c = 0, rkc = 0, sm0n = 0, sm1n = 0, rkn = 0;
  auto load_masks = [&](int pp, uint32_t& s0, uint32_t& s1, uint32_t& rk) {
    s0 = s1 = rk = 0;
    if ((SAL != 0) && pp < p_end) {
      const size_t gi = (size_t)b * a.ngc + 2 * pp;
      s0 = a.vmask[gi];
      rk = a.vrank[gi];
      if (2 * pp + 1 < a.ng) s1 = a.vmask[gi + 1];
    }
  };
  // what a lane keeps of protected row r: its two channels 2 lane, 2 lane + 1 as an fp16
  // pair, or (2-bit records) the byte that holds their codes
  auto row_word = [&](uint32_t r) -> uint32_t {
    if (SAL == 2) {
      const uint8_t* rec = reinterpret_cast<const uint8_t*>(a.vrows) + (hd * a.npg + (r >> 5)) * (long long)PREC;
      return rec[(r & 31) * 32 + (lane >> 1)];
    }
    return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(a.vrows + (hd * a.n_s + r) * D) + lane);
  };
  auto issue_rows = [&](uint32_t s0, uint32_t s1, uint32_t rk, uint32_t* rows) {
    const int cnt = __popc(s0) + __popc(s1);
#pragma unroll
    for (int j = 0; j < NROW; ++j)
      if (j < cnt) rows[j] = row_word(rk + j);
  };
  // scale and zero point (Eq. 4) of my two channels in the current group of protected rows
  int sal_pg = -1;
  float sal_s0 = 0.f, sal_s1 = 0.f, sal_z0 = 0.f, sal_z1 = 0.f;
  int p = p_begin + wave;
  int buf = 0;
  // q and the permutation (to registers, then LDS) and the masks of the first two pairs
  {
    const uint32_t* qsrc = reinterpret_cast<const uint32_t*>(a.q + ((long long)b * a.Hq + kvh * R) * D);
    const int nq = R * (D / 2);                // at most 512 dwords
    const uint32_t q0 = tid < nq ? qsrc[tid] : 0u;
    const uint32_t q1 = tid + 256 < nq ? qsrc[tid + 256] : 0u;
    const uint32_t pw = tid < D / 4 ? reinterpret_cast<const uint32_t*>(a.kperm + hd * D)[tid] : 0u;
    if ((SAL != 0)) {
      load_masks(p, sm0c, sm1c, rkc);
      load_masks(p + 4, sm0n, sm1n, rkn);
    }
    // ---------------- constant operands (q and the channel permutation via LDS)
    if (tid < nq) reinterpret_cast<uint32_t*>(&qs[0][0])[tid] = q0;
    if (tid + 256 < nq) reinterpret_cast<uint32_t*>(&qs[0][0])[tid + 256] = q1;
    if (tid < D / 4) reinterpret_cast<uint32_t*>(perm_s)[tid] = pw;
  }
  __syncthreads();
  // The first pair's records are requested only now.  All workgroups start together, and
  // their first requests are a burst of many MB; q, asked for behind that burst, would
  // arrive after it.  This way q is in first and the burst runs under the operand set-up.
  if (p < p_end) prefetch(p, 0);
  if ((SAL != 0) && (sm0c | sm1c)) issue_rows(sm0c, sm1c, rkc, rowcur);
  const bool hv = hcol < R;
  const _Float16* qrow = &qs[hv ? hcol : 0][0];
  // The permutation bytes of my channel blocks and quads come in one LDS read each, then
  // every q element in one batch of independent reads (no branch around a read: absent
  // blocks read a valid block and are zeroed afterwards).
  Op Bn[U > 0 ? U : 1];                      // normal channels: -q/16 (FFT) or -q/2 at channels 8 (4u+kb) + e
  Op Ba[2][UA > 0 ? UA : 1];                 // anomalous: (-q, -q) per channel, only in my parity
  {
    uint2 pb[U > 0 ? U : 1];
    uint32_t pq[UA > 0 ? UA : 1];
#pragma unroll
    for (int u = 0; u < U; ++u)
      pb[u] = *reinterpret_cast<const uint2*>(&perm_s[NA + 8 * min(4 * u + kb, NB - 1)]);
#pragma unroll
    for (int ua = 0; ua < UA; ++ua)
      pq[ua] = *reinterpret_cast<const uint32_t*>(&perm_s[4 * min(4 * ua + kb, NQ - 1)]);
    _Float16 qn[U > 0 ? U : 1][8], qa[UA > 0 ? UA : 1][4];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) qn[u][e] = qrow[((e < 4 ? pb[u].x : pb[u].y) >> (8 * (e & 3))) & 0xFFu];
#pragma unroll
    for (int ua = 0; ua < UA; ++ua)
#pragma unroll
      for (int r = 0; r < 4; ++r) qa[ua][r] = qrow[(pq[ua] >> (8 * r)) & 0xFFu];
    const _Float16 cn = (_Float16)(FFT ? -0.0625f : -0.5f);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = hv && (4 * u + kb) < NB;
#pragma unroll
      for (int e = 0; e < 8; ++e) Bn[u].v[e] = ok ? (_Float16)(qn[u][e] * cn) : (_Float16)0.0f;
    }
#pragma unroll
    for (int ua = 0; ua < UA; ++ua) {
      const bool ok = hv && (4 * ua + kb) < NQ;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const _Float16 v = ok ? (_Float16)(-qa[ua][r]) : (_Float16)0.0f;
        const uint32_t pr = h2_bits(h2{v, v});
        Ba[0][ua].u[r] = par ? 0u : pr;
        Ba[1][ua].u[r] = par ? pr : 0u;
      }
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
  // o[m][i]: row 4kb+i = (parity, head) column of the score tile, channel 16 m + x16;
  // holds 2 * sum p * code * s of the quantized tokens (halved at the end).
  f4 o[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) o[m] = zero;
  float osal[8][2];                          // protected rows: head h, channels 2 lane, 2 lane + 1
#pragma unroll
  for (int h = 0; h < 8; ++h) { osal[h][0] = 0.f; osal[h][1] = 0.f; }
  float m_run = -INFINITY, l_run = 0.0f;     // of my column (shared by both parities of a head)

  for (; p < p_end; p += 4) {
    const bool v1ok = (2 * p + 1) < a.ng;
    // ---- commit the prefetched data, start the next prefetch
    u32x4 vw[2];
    Op sv;
    if (KDMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this pair's key records are in kl4[buf]
#pragma unroll
    for (int grp = 0; grp < 2; ++grp) {
      if (!KDMA) {
        kl4[0][wave][grp][lane] = kpre[grp][0];
        if (lane + 64 < KCH) kl4[0][wave][grp][lane + 64] = kpre[grp][1];
      }
      vw[grp] = vwpre[grp];
    }
    sv.q = vspre;
    if (p + 4 < p_end) prefetch(p + 4, buf ^ 1);
    uint32_t sm0f = 0, sm1f = 0, rkf = 0;        // masks of the pair after the next one
    if ((SAL != 0)) {
      if (sm0n | sm1n) issue_rows(sm0n, sm1n, rkn, rownext);
      load_masks(p + 8, sm0f, sm1f, rkf);
    }

    f4 S[2] = {zero, zero};                      // scores[token][column]
    // ---- normal channels: Y[slot][col] per group, K = channels
    float cst_n = 0.0f;                          // non-FFT: sum over normal channels of q (z + s/2)
    if (U > 0) {
      f4 accRe[2], accIm[2];
      f4 accCn[2] = {zero, zero};
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint8_t* rec = reinterpret_cast<const uint8_t*>(&kl4[buf][wave][grp][0]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int blk = min(4 * u + kb, NB - 1);
          const uint32_t w = *reinterpret_cast<const uint16_t*>(rec + OFF_BITS + (blk * 16 + x16) * 2);
          const uint32_t xx = w | (w << 15);
          Op sre, sim, A;
          sre.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2) * 16);
          sim.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2 + ((FFT && x16) ? 1 : 0)) * 16);
#pragma unroll
          for (int r = 0; r < 4; ++r) A.u[r] = ((xx << (15 - 2 * r)) & 0x80008000u) | sre.u[r];
          accRe[grp] = mma(A, Bn[u], u == 0 ? zero : accRe[grp]);
#pragma unroll
          for (int r = 0; r < 4; ++r) A.u[r] = ((xx << (7 - 2 * r)) & 0x80008000u) | sim.u[r];
          accIm[grp] = mma(A, Bn[u], u == 0 ? zero : accIm[grp]);
          if (!FFT) {
            // constant term, rows all equal: (-z)(-q/2) + (-s/2)(-q/2) = q (z + s/2) / 2
            Op zq, Az, As;
            zq.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2 + 1) * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              Az.u[r] = zq.u[r] ^ 0x80008000u;
              As.u[r] = h2_bits(sre.p[r] * h2{(_Float16)0.5f, (_Float16)0.5f}) ^ 0x80008000u;
            }
            accCn[grp] = mma(Az, Bn[u], accCn[grp]);
            accCn[grp] = mma(As, Bn[u], accCn[grp]);
          }
        }
      }
      if (!FFT) {
        // slot = token: the products are the scores' normal-channel part for my group
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          S[0][i] = par ? accRe[1][i] : accRe[0][i];
          S[1][i] = par ? accIm[1][i] : accIm[0][i];
        }
        cst_n = 2.0f * (par ? accCn[1][0] : accCn[0][0]);
      }
      // my column belongs to group `par`; split Y/16 into fp16 hi + lo
      Op Yh, Yl;
      if (FFT) {
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        const float r0 = par ? accRe[1][i] : accRe[0][i], r1 = par ? accRe[1][i + 1] : accRe[0][i + 1];
        const float i0 = par ? accIm[1][i] : accIm[0][i], i1 = par ? accIm[1][i + 1] : accIm[0][i + 1];
        Yh.u[i / 2] = pkrtz(r0, r1);
        Yh.u[2 + i / 2] = pkrtz(i0, i1);
        Yl.u[i / 2] = pkrtz(r0 - (float)Yh.v[i], r1 - (float)Yh.v[i + 1]);
        Yl.u[2 + i / 2] = pkrtz(i0 - (float)Yh.v[4 + i], i1 - (float)Yh.v[4 + i + 1]);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        S[mt] = mma(Wh[mt], Yh, zero);
        S[mt] = mma(Wl[mt], Yh, S[mt]);
        S[mt] = mma(Wh[mt], Yl, S[mt]);
      }
      }
    }
    // ---- anomalous channels: rows = tokens, K = (channel, bit plane); the column
    // operand is zero outside my parity, so both groups add into S directly
    float cst = 0.0f;
    if (UA > 0) {
      f4 accC = zero;
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint8_t* rec = reinterpret_cast<const uint8_t*>(&kl4[buf][wave][grp][0]);
#pragma unroll
        for (int ua = 0; ua < UA; ++ua) {
          const int quad = min(4 * ua + kb, NQ - 1);
          Op s4, z4;                                             // 4 halves each (low 8 bytes used)
          *reinterpret_cast<uint2*>(&s4) = *reinterpret_cast<const uint2*>(rec + OFF_AS + quad * 8);
          *reinterpret_cast<uint2*>(&z4) = *reinterpret_cast<const uint2*>(rec + OFF_AZ + quad * 8);
          uint32_t sp[4];                                        // (s/2, s) of channel r
          Op Ac1, Ac2;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            sp[r] = h2_bits(h2{s4.v[r] * (_Float16)0.5f, s4.v[r]});
            Ac1.p[r] = h2{z4.v[r], s4.v[r]};                     // z + s
            Ac2.u[r] = sp[r] & 0xFFFFu;                          // + s/2
          }
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) {
            const uint32_t w = rec[(16 * mt + x16) * NQ + quad];
            const uint32_t xx = w | (w << 15);
            Op A;
#pragma unroll
            for (int r = 0; r < 4; ++r) A.u[r] = ((xx << (15 - 2 * r)) & 0x80008000u) | sp[r];
            S[mt] = mma(A, Ba[grp][ua], S[mt]);
          }
          accC = mma(Ac1, Ba[grp][ua], accC);                    // rows all equal
          accC = mma(Ac2, Ba[grp][ua], accC);
        }
      }
      cst = accC[0];                                             // = -(sum q (z + 1.5 s))
    }
    if (!FFT) cst -= cst_n;
    // ---- t = score - running maximum, in the exp2 domain, for my column at token
    // slot i (i < 4: token 4kb+i, else 16+4kb+i-4)
    float c1 = -cst * a.scale2 - m_run;
    float t[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      t[i] = fmaf(S[0][i], a.scale2, c1);
      t[4 + i] = fmaf(S[1][i], a.scale2, c1);
    }
    if (par && !v1ok) {
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = -INFINITY;
    }
    // ---- online softmax.  The running maximum is raised lazily: only when some
    // score exceeds it by more than 8 (p stays below 2^8), which needs no
    // cross-lane traffic in the common case.
    float mx = t[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = fmaxf(mx, t[i]);
    if (__any(mx > 8.0f)) {
      // true scores again; maximum over the 4 k-blocks and the 2 parities of the head
      float smax = (m_run == -INFINITY) ? -INFINITY : mx + m_run;
      if (m_run == -INFINITY) {
        const float c0 = -cst * a.scale2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          t[i] = fmaf(S[0][i], a.scale2, c0);
          t[4 + i] = fmaf(S[1][i], a.scale2, c0);
        }
        if (par && !v1ok) {
#pragma unroll
          for (int i = 0; i < 8; ++i) t[i] = -INFINITY;
        }
        smax = t[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) smax = fmaxf(smax, t[i]);
      }
      smax = swap_max32(smax);
      smax = swap_max16(smax);
      smax = fmaxf(smax, __shfl_xor(smax, 8, 64));
      const float m_new = fmaxf(m_run, smax);
      const float al = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m_run - m_new);
      const float shift = (m_run == -INFINITY) ? -m_new : m_run - m_new;
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] += shift;
      l_run *= al;
      m_run = m_new;
      // the PV accumulators are laid out by score-tile column as ROW 4kb + i
      if (kb == 0) al16[wave][x16] = al;
      float ar[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) ar[i] = al16[wave][4 * kb + i];
#pragma unroll
      for (int m = 0; m < 8; ++m)
#pragma unroll
        for (int i = 0; i < 4; ++i) o[m][i] *= ar[i];
      if ((SAL != 0)) {
#pragma unroll
        for (int h = 0; h < 8; ++h) {
          const float ah = al16[wave][h];
          osal[h][0] *= ah;
          osal[h][1] *= ah;
        }
      }
    }
    float pr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pr[i] = __builtin_amdgcn_exp2f(t[i]);
      l_run += pr[i];
    }
    // probabilities as the A operand of P V (row = my column), zero outside the group
    Op Ap[2];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t pp = pkrtz(pr[2 * r], pr[2 * r + 1]);
      Ap[0].u[r] = par ? 0u : pp;
      Ap[1].u[r] = par ? pp : 0u;
    }
    // ---- P V: C[column][channel 16 m + x16] = sum_t p * (2 code), then o += s * C
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      f4 C = zero;
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint32_t w = vw[grp][m >> 1];
        Op Bv;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          Bv.u[r] = (w << ((m & 1) ? (6 - 2 * r) : (14 - 2 * r))) & 0xC000C000u;   // +-2 or 0
        C = mma(Ap[grp], Bv, C);
      }
      const float sc = (float)sv.v[m];           // Eq. 6 scale of channel 16 m + x16, my rows' group
#pragma unroll
      for (int i = 0; i < 4; ++i) o[m][i] = fmaf(sc, C[i], o[m][i]);
    }
    // ---- protected tokens: fp16 rows (prefetched) weighted by the probabilities
    if ((SAL != 0)) {
      if (sm0c | sm1c) {
#pragma unroll
        for (int i = 0; i < 8; ++i) pl[wave][slot_token(kb, i)][x16] = pr[i];
        unsigned long long sm = (unsigned long long)sm0c | ((unsigned long long)sm1c << 32);
        auto add_row = [&](uint32_t bits, uint32_t r) {
          const int t64 = __ffsll((long long)sm) - 1;      // bit t of parity t64 >> 5
          sm &= sm - 1;
          float v0, v1;
          if (SAL == 2) {
            if ((int)(r >> 5) != sal_pg) {
              sal_pg = (int)(r >> 5);
              const uint8_t* rec = reinterpret_cast<const uint8_t*>(a.vrows) + (hd * a.npg + sal_pg) * (long long)PREC;
              const h2 s2 = bits_h2(reinterpret_cast<const uint32_t*>(rec + 1024)[lane]);
              const h2 z2 = bits_h2(reinterpret_cast<const uint32_t*>(rec + 1280)[lane]);
              sal_s0 = (float)s2[0]; sal_s1 = (float)s2[1];
              sal_z0 = (float)z2[0]; sal_z1 = (float)z2[1];
            }
            const uint32_t nib = bits >> (4 * (lane & 1));
            v0 = fmaf((float)(nib & 3u), sal_s0, sal_z0);
            v1 = fmaf((float)((nib >> 2) & 3u), sal_s1, sal_z1);
          } else {
            const h2 v = bits_h2(bits);
            v0 = (float)v[0]; v1 = (float)v[1];
          }
          const float* pp = &pl[wave][t64 & 31][8 * (t64 >> 5)];
#pragma unroll
          for (int h = 0; h < 8; ++h) {
            const float ph = pp[h];
            osal[h][0] += ph * v0;
            osal[h][1] += ph * v1;
          }
        };
        // fp16 rows go two at a time: (row A, row B) of one channel as a packed pair against
        // the pair of their probabilities (rounded to nearest fp16: these rows carry the largest
        // values, so a one-sided rounding would show in the output),
        // one v_dot2_f32_f16 per (head, channel)
        auto add_rows2 = [&](uint32_t bitsA, uint32_t bitsB) {
          const int tA = __ffsll((long long)sm) - 1;
          sm &= sm - 1;
          const bool hasB = sm != 0;
          const int tB = hasB ? __ffsll((long long)sm) - 1 : tA;
          if (hasB) sm &= sm - 1; else bitsB = 0u;
          const h2 c0 = bits_h2(__builtin_amdgcn_perm(bitsB, bitsA, 0x05040100u));   // channel 2 lane
          const h2 c1 = bits_h2(__builtin_amdgcn_perm(bitsB, bitsA, 0x07060302u));   // channel 2 lane + 1
          const float* pa = &pl[wave][tA & 31][8 * (tA >> 5)];
          const float* pb = &pl[wave][tB & 31][8 * (tB >> 5)];
#pragma unroll
          for (int h = 0; h < 8; ++h) {
            const h2 w = __builtin_convertvector(f2{pa[h], pb[h]}, h2);   // round to nearest
            osal[h][0] = __builtin_amdgcn_fdot2(c0, w, osal[h][0], false);
            osal[h][1] = __builtin_amdgcn_fdot2(c1, w, osal[h][1], false);
          }
        };
        if (SAL == 1) {
#pragma unroll
          for (int j = 0; j < NROW; j += 2)
            if (sm) add_rows2(rowcur[j], rowcur[j + 1]);
          uint32_t rk = rkc + NROW;                         // more than NROW rows: fetch on demand
          while (sm) {
            const uint32_t ra = row_word(rk);
            const uint32_t rb = (sm & (sm - 1)) ? row_word(rk + 1) : 0u;
            add_rows2(ra, rb);
            rk += 2;
          }
        } else {
#pragma unroll
          for (int j = 0; j < NROW; ++j)
            if (sm) add_row(rowcur[j], rkc + j);
          uint32_t rk = rkc + NROW;                         // more than NROW rows: fetch on demand
          while (sm) {
            add_row(row_word(rk), rk);
            ++rk;
          }
        }
      }
      sm0c = sm0n; sm1c = sm1n; rkc = rkn;
      sm0n = sm0f; sm1n = sm1f; rkn = rkf;
#pragma unroll
      for (int j = 0; j < NROW; ++j) rowcur[j] = rownext[j];
    }
    if (KDMA) buf ^= 1;
  }

  // ---------------- per-wave reduction
  // l: 4 k-blocks and 2 parities of each head
  l_run = swap_sum32(l_run);
  l_run = swap_sum16(l_run);
  l_run += __shfl_xor(l_run, 8, 64);
  // o: rows 4kb+i; parity 1 rows live 32 lanes away from their parity 0 partners
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int i = 0; i < 4; ++i) o[m][i] = swap_sum32(o[m][i]);
  if (kb < 2) {
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
      for (int i = 0; i < 4; ++i) ow[wave][4 * kb + i][16 * m + x16] = 0.5f * o[m][i];
  }
  if (kb == 0 && par == 0) { mw[wave][hcol] = m_run; lw[wave][hcol] = l_run; }
  if ((SAL != 0)) {
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

template <int NA8>
static void launch_one(const AttnArgs& a, dim3 grid, hipStream_t st) {
  const int sal = a.n_s > 0 ? (a.sal_bits == 2 ? 2 : 1) : 0;
#define VIDKV_ATTN(S, F) hipLaunchKernelGGL((attn_mfma_kernel<NA8, S, F>), grid, dim3(256), 0, st, a)
  if (a.use_fft) {
    if (sal == 2) VIDKV_ATTN(2, true); else if (sal == 1) VIDKV_ATTN(1, true); else VIDKV_ATTN(0, true);
  } else {
    if (sal == 2) VIDKV_ATTN(2, false); else if (sal == 1) VIDKV_ATTN(1, false); else VIDKV_ATTN(0, false);
  }
#undef VIDKV_ATTN
}

void launch_attn_mfma(const AttnArgs& a, dim3 grid, hipStream_t st) {
  switch (a.n_a) {
    case 0:   launch_one<0>(a, grid, st); break;
    case 8:   launch_one<1>(a, grid, st); break;
    case 16:  launch_one<2>(a, grid, st); break;
    case 32:  launch_one<4>(a, grid, st); break;
    case 64:  launch_one<8>(a, grid, st); break;
    case 128: launch_one<16>(a, grid, st); break;
    default: break;
  }
}

}  // namespace vidkv
