// MFMA decode attention over the packed cache (Eq. 3; Alg. 1, Decoding).
//
// One wave walks PAIRS of 32-token groups; the 16 "columns" of the score tiles
// are (group parity, query head <= 8).  All contractions run on
// v_mfma_f32_16x16x32_f16 with operands that are exact in fp16 and fp32
// accumulation:
//   * normal key channels (Eq. 5): rows = DFT coefficient slot, K = channels,
//     operand value -(+-s) = sign pattern | stored fp16 scale; columns carry
//     -q/16.  The result tile is already laid out as the B operand of the next
//     product,
//   * a 32-point inverse real DFT as a product with a constant matrix (split
//     into fp16 hi + lo parts, as is Y) giving scores[token][column],
//   * anomalous key channels (Eq. 4): code*s + z = (z + 1.5 s) + s0 (s/2) + s1 s
//     with s0, s1 = +-1 taken from the two code bits, rows = tokens; the column
//     operand is masked by parity so both groups add into the same score tile,
//   * P V: rows = columns of the score tile (probabilities are reused in place
//     as the A operand), K = tokens, columns = channels with operand +-1 / 0 from
//     the trits; the per-channel scale of Eq. 6 multiplies the fp32 result.
//
// Expanding one stored bit (or trit) into an fp16 operand element is what this
// kernel spends its time on, and two units can do it: the vector ALU (shift +
// mask pairs; a 64-bit shift serves two registers at once) and LDS (a byte of
// four trits indexes a 256-entry table of four fp16 values: one 8-byte read and
// nothing else).  Either alone saturates - LDS is shared by the four SIMDs of a
// compute unit - so the work is split: the key operands, which also carry their
// scale, are expanded on the ALU, the value operands through the table.
//
// Key and value records - and protected fp16 rows, four per instruction - go
// from memory straight into a per-wave LDS ring, one pair ahead
// (global_load_lds_dwordx4; lane l of a wave-wide transfer lands at M0 + 16 l,
// i.e. a record keeps its byte order; the two records of a pair are neighbours
// in memory and in the ring, so one run of 1 KB transfers covers both).
//
// Two-stage software pipeline per wave: while the keys of pair p are scored,
// the values of pair p - 4 (the wave's previous pair) are multiplied by the
// probabilities that the previous step left in registers, as one interleaved
// instruction stream; the ring holds two key stages and two value stages.
//
// What orders the hand-offs through LDS.  Every ring, row and probability
// buffer is private to one wave, so no barrier is involved after the set-up
// (whose two __syncthreads order the shared tables, q and the permutation).
//   * transfer -> read: the compiler is not told that the transfer
//     instructions write LDS.  Each step begins with a written-out
//     "s_waitcnt vmcnt(0)" carrying a memory clobber: every transfer the wave
//     has issued - they were all issued in the previous step - has landed, and
//     no LDS read of the step can be moved above it.
//   * read -> overwrite: a stage is refilled by transfers issued only after
//     the step that read it has consumed the data in registers (the loads'
//     results are used, so their lgkmcnt waits have passed), and the transfer
//     statements carry a memory clobber, so the compiler keeps program order.
//   * probabilities and rescale factors staged with ordinary LDS stores are
//     read back by the same wave through ordinary loads: the compiler sees
//     both and inserts the lgkmcnt waits itself; LDS executes a wave's
//     operations in order.
// M0 is written inside the transfer statement and named in its clobber list;
// the kernel has no other user of M0.
//
// Softmax is online in the exp2 domain with a lazily raised running maximum
// shared by the two parities of a head.  Protected (fp16) value rows are added
// on the VALU from the probabilities staged in LDS.
#include <type_traits>

#include "decode_attn.h"

namespace vidkv {

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
// two floats -> packed fp16 pair, round to nearest even
__device__ __forceinline__ uint32_t pk_rne(float a, float b) {
  return h2_bits(__builtin_convertvector(f2{a, b}, h2));
}
__device__ __forceinline__ uint32_t pkrtz(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}

// v << K as one 64-bit vector shift.  The empty asm makes all 64 result bits count as used,
// so the compiler cannot split the shift into two 32-bit ones.  (The shift itself must not
// be written as inline asm: the compiler does not insert the wait states that a vector
// write needs behind an MFMA still reading the same register when the write sits in an asm
// statement, and results came out wrong.)
template <int K>
__device__ __forceinline__ uint64_t shl64(uint64_t v) {
  uint64_t r = v << K;
  asm("" : "+v"(r));
  return r;
}
// byte B of w, times 8 (one instruction with a sub-dword source select)
template <int B>
__device__ __forceinline__ uint32_t byte_x8(uint32_t w) {
  return ((w >> (8 * B)) & 0xFFu) << 3;
}

// SAL: 0 no protected tokens, 1 protected rows in fp16, 2 protected rows as 2-bit records.
// FFT: normal key channels coded by Eq. 5 (true) or by Eq. 4 at 1 bit on the tokens (false);
// in the latter case slot = token and code * s + z = (z + s/2) + sigma * s/2, sigma = +-1,
// so the same sign-type operand serves, without the inverse DFT and with a constant term.
template <int NA8, int SAL, bool FFT>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(AttnArgs a) {
  constexpr int NA = 8 * NA8, NN = D - NA;
  constexpr int NB = NN / 8;                 // normal 8-channel blocks
  constexpr int U = (NB + 3) / 4;            // K-steps over normal channels
  constexpr int NQ = NA / 4;                 // anomalous 4-channel quads
  constexpr int UA = (NQ + 3) / 4;           // K-steps over anomalous channels
  constexpr int KREC = 12 * NA + 8 * NN;
  constexpr int KCH = KREC / 16;             // 16-byte chunks of a key record (64 < KCH <= 96, or 64)
  constexpr int OFF_AS = 8 * NA, OFF_AZ = 10 * NA, OFF_BITS = 12 * NA, OFF_META = 12 * NA + 4 * NN;
  constexpr int RING = 4 * KREC + 4 * VREC;  // a wave's ring: two stages of a pair's key records, two of its value records
  constexpr int NROW = 8;                    // protected rows fetched ahead per pair (2-bit records: to registers)
  constexpr int NROWL = 12;                  // ... fp16 rows: to LDS, four rows per transfer instruction

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform
  const int x16 = lane & 15, kb = lane >> 4;
  const int hcol = x16 & 7, par = x16 >> 3;          // column role: (parity, head)
  const int R = a.rep;
  const long long hd = ((long long)a.layer * a.B + b) * a.H + kvh;
  const f4 zero = f4{0.f, 0.f, 0.f, 0.f};

  __shared__ __align__(16) uint8_t ring[4][RING];   // per wave: 2 key stages, 2 value stages; reused for the wave's partial output
  __shared__ uint2 t_trit[256];              // byte -> 4 halves, half i = +1 / -1 / 0 from bits 2i (nonzero), 2i+1 (negative)
  __shared__ u32x4 w_tab[4][64];             // per lane: inverse-DFT operands Wh[0], Wh[1], Wl[0], Wl[1]
  // q and the channel permutation are needed only until the constant operands are built;
  // the staged probabilities of the protected rows take their place afterwards
  constexpr int PL_BYTES = (SAL != 0) ? 4 * 64 * 8 * 2 : 0;
  constexpr int PRE_BYTES = 8 * D * 2 + D;
  __shared__ __align__(16) uint8_t pre_s[PRE_BYTES > PL_BYTES ? PRE_BYTES : PL_BYTES];
  _Float16 (*qs)[D] = reinterpret_cast<_Float16 (*)[D]>(pre_s);
  uint8_t* perm_s = pre_s + 8 * D * 2;
  _Float16 (*pl)[64][8] = reinterpret_cast<_Float16 (*)[64][8]>(pre_s);   // per wave: probabilities [token of the pair][head]
  __shared__ __align__(16) uint8_t rowring[(SAL == 1) ? 4 : 1][2][(SAL == 1) ? NROWL * 2 * D : 16];   // per wave, two stages of fp16 rows
  __shared__ float al16[4][16];              // per wave: rescale factors per column
  __shared__ float mw[4][8], lw[4][8];
  static_assert(sizeof(float) * 8 * D <= RING, "a wave's partial output must fit its ring");

  // ---------------- the expansion table of the value operands, the inverse-DFT operands
  {
    uint32_t h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t f = ((uint32_t)tid >> (2 * i)) & 3u;
      h[i] = (f & 1u) ? ((f & 2u) ? 0xBC00u : 0x3C00u) : 0u;
    }
    t_trit[tid] = uint2{h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
    // 16 * (inverse real DFT matrix) as fp16 hi + lo parts: row t = 16 mt + x, k-slot (kb, i):
    // i < 4 -> Re X[4kb+i], i >= 4 -> Im X[4kb+i-4] (Re X[16] when that index is 0)
    const int wl = tid & 63, wmt = (tid >> 6) & 1, wlo = tid >> 7;
    const int wt = 16 * wmt + (wl & 15), wkb = wl >> 4;
    // cos(2 pi j / 32) from the first-octant constants by the symmetries (no memory access:
    // this runs before anything has arrived, and a load would only put its latency in front
    // of the first transfers)
    auto cos_rt = [](int j) -> float {
      j &= 31;
      if (j > 16) j = 32 - j;
      const bool neg = j > 8;
      const int i = neg ? 16 - j : j;
      float v = cos32(0);
      v = i == 1 ? cos32(1) : v; v = i == 2 ? cos32(2) : v; v = i == 3 ? cos32(3) : v;
      v = i == 4 ? cos32(4) : v; v = i == 5 ? cos32(5) : v; v = i == 6 ? cos32(6) : v;
      v = i == 7 ? cos32(7) : v; v = i == 8 ? 0.0f : v;
      return neg ? -v : v;
    };
    Op W;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = 4 * wkb + (i & 3);
      float w;
      if (i < 4) w = (k == 0) ? 0.5f : cos_rt(k * wt);
      else       w = (k == 0) ? ((wt & 1) ? -0.5f : 0.5f) : -cos_rt(k * wt + 24);
      const _Float16 hi = (_Float16)w;
      W.v[i] = wlo ? (_Float16)(w - (float)hi) : hi;
    }
    w_tab[2 * wlo + wmt][wl] = W.q;
  }

  // ---------------- transfers
  const int npairs = (a.ng + 1) >> 1;
  const int p_begin = split * a.gps;
  const int p_end = min(npairs, p_begin + a.gps);

  const uint8_t* krec_base = a.krec + hd * a.ngc * (long long)KREC;
  const uint8_t* vrec_base = a.vrec + hd * a.ngc * (long long)VREC;

  // M0 is the LDS base of a transfer.  It is written inside the asm statement and named in
  // its clobber list; this kernel has no other user of M0 (no indirect register indexing,
  // no compiler-generated LDS transfers).
  auto dma16 = [&](const uint8_t* g, uint32_t lds_byte) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                 :: "s"(lds_byte), "v"(g) : "memory", "m0");
  };
  // ring of a wave: key stages 0, 1, then value stages 0, 1 (a stage = the two groups of a pair)
  const uint32_t ring_lds = (uint32_t)reinterpret_cast<uintptr_t>(&ring[0][0]) + (uint32_t)(wave * RING);
  const uint8_t* ring_w = &ring[wave][0];
  // The two records of a pair are neighbours in memory and in the stage: one run of 1 KB
  // instructions covers both.  (A last pair with one group fetches that group twice, so that
  // the unused half of the stage holds finite numbers.)
  constexpr int NDMA_K = (2 * KREC + 1023) / 1024;       // fewest instructions of one key transfer
  constexpr int NDMA_V = (2 * VREC + 1023) / 1024;
  auto fetch_run = [&](const uint8_t* src, uint32_t dst, auto nbytes_c) {
    constexpr int NBYTES = decltype(nbytes_c)::value;
#pragma unroll
    for (int j = 0; j < (NBYTES + 1023) / 1024; ++j)
      if ((j + 1) * 1024 <= NBYTES || j * 1024 + lane * 16 < NBYTES) dma16(src + j * 1024 + lane * 16, dst + j * 1024u);
  };
  auto fetch_keys = [&](int pp, int st) {
    const uint32_t dst = ring_lds + st * 2 * KREC;
    if (2 * pp + 1 < a.ng) {
      fetch_run(krec_base + (long long)(2 * pp) * KREC, dst, std::integral_constant<int, 2 * KREC>{});
    } else {
      const uint8_t* ks = krec_base + (long long)(a.ng - 1) * KREC;
      fetch_run(ks, dst, std::integral_constant<int, KREC>{});
      fetch_run(ks, dst + KREC, std::integral_constant<int, KREC>{});
    }
  };
  auto fetch_values = [&](int pp, int st) {
    const uint32_t dst = ring_lds + 4 * KREC + st * 2 * VREC;
    if (2 * pp + 1 < a.ng) {
      fetch_run(vrec_base + (long long)(2 * pp) * VREC, dst, std::integral_constant<int, 2 * VREC>{});
    } else {
      const uint8_t* vs = vrec_base + (long long)(a.ng - 1) * VREC;
      fetch_run(vs, dst, std::integral_constant<int, VREC>{});
      fetch_run(vs, dst + VREC, std::integral_constant<int, VREC>{});
    }
  };
  // Protected rows of a pair are consecutive in ROWS (rank grows with the token).  Masks:
  // of the pair whose values are being added (v), whose keys are being scored (c), the next (n).
  uint32_t rows0[NROW], rows1[NROW];         // 2-bit records only
  uint32_t sm0v = 0, sm1v = 0, rkv = 0, sm0c = 0, sm1c = 0, rkc = 0, sm0n = 0, sm1n = 0, rkn = 0;
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
  auto issue_rows = [&](uint32_t s0, uint32_t s1, uint32_t rk, uint32_t* rows, int st) {
    const int cnt = __popc(s0) + __popc(s1);
    if (SAL == 2) {
#pragma unroll
      for (int j = 0; j < NROW; ++j)
        if (j < cnt) rows[j] = row_word(rk + j);
    } else {
      // consecutive fp16 rows straight into LDS, four rows (1 KB) per instruction: lane l
      // brings bytes 16 (l & 15) .. of row 4 j + (l >> 4)
      const uint8_t* base = reinterpret_cast<const uint8_t*>(a.vrows + (hd * a.n_s + rk) * D) + lane * 16;
      const uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>(&rowring[wave][st][0]);
      const int n = min(cnt, NROWL);
#pragma unroll
      for (int j = 0; j < NROWL / 4; ++j)
        if (4 * j < n && 4 * j + (lane >> 4) < n) dma16(base + j * 1024, dst + j * 1024u);
    }
  };
  // scale and zero point (Eq. 4) of my two channels in the current group of protected rows
  int sal_pg = -1;
  float sal_s0 = 0.f, sal_s1 = 0.f, sal_z0 = 0.f, sal_z1 = 0.f;
  int p = p_begin + wave;

  // ---------------- set-up: q and the channel permutation go straight to LDS (wave 0 asks for
  // them), the first pair's key records are requested right behind them, and only the
  // former are waited for: the operands are built while the records are on their way
  if (wave == 0) {
    const uint8_t* qsrc = reinterpret_cast<const uint8_t*>(a.q + ((long long)b * a.Hq + kvh * R) * D);
    const uint32_t q_lds = (uint32_t)reinterpret_cast<uintptr_t>(pre_s);
    const int qbytes = R * D * 2;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(q_lds), "v"(qsrc + (lane * 16 < qbytes ? lane * 16 : 0)) : "memory", "m0");
    if (1024 + lane * 16 < qbytes)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                   :: "s"(q_lds + 1024u), "v"(qsrc + 1024 + lane * 16) : "memory", "m0");
    if (lane < D / 16)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                   :: "s"(q_lds + 8u * D * 2u), "v"(a.kperm + hd * D + lane * 16) : "memory", "m0");
  }
  if (p < p_end) fetch_keys(p, 0);
  if ((SAL != 0)) {
    load_masks(p, sm0c, sm1c, rkc);
    load_masks(p + 4, sm0n, sm1n, rkn);
  }
  if (wave == 0) {
    if (p < p_end) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NDMA_K) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  const bool hv = hcol < R;
  const _Float16* qrow = &qs[hv ? hcol : 0][0];
  // The permutation bytes of my channel blocks and quads come in one LDS read each, then
  // every q element in one batch of independent reads (no branch around a read: absent
  // blocks read a valid block and are zeroed afterwards).
  Op Bn[2][U > 0 ? U : 1];                   // normal channels: -q/16 (FFT) or -q/2 at channels 8 (4u+kb) + e, only in my parity
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
      for (int e = 0; e < 8; ++e) {
        const _Float16 v = ok ? (_Float16)(qn[u][e] * cn) : (_Float16)0.0f;
        Bn[0][u].v[e] = par ? (_Float16)0.0f : v;
        Bn[1][u].v[e] = par ? v : (_Float16)0.0f;
      }
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
  __syncthreads();                           // every wave is done with q and the permutation
  const uint32_t keep0 = par ? 0u : ~0u, keep1 = ~keep0;    // which group's P V product my column feeds
  const uint8_t* ttrit_b = reinterpret_cast<const uint8_t*>(&t_trit[0]);

  // ---------------- running state
  // o[m][i]: row 4kb+i = (parity, head) column of the score tile, channel 16 m + x16;
  // holds sum p * code * s of the quantized tokens.
  f4 o[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) o[m] = zero;
  float osal[8][2];                          // protected rows: head h, channels 2 lane, 2 lane + 1
#pragma unroll
  for (int h = 0; h < 8; ++h) { osal[h][0] = 0.f; osal[h][1] = 0.f; }
  float m_run = -INFINITY, l_run = 0.0f;     // of my column (shared by both parities of a head)
  uint32_t pp[4] = {0u, 0u, 0u, 0u};         // probabilities of the pair whose values come next

  // ---------------- the pieces of one step.  Stage numbers are compile-time constants (the
  // loop alternates two instances of the step) so that every LDS address of the records is a
  // register plus an immediate.

  // What a lane reads first of a step, in one batch ahead of everything else (and ahead of
  // the transfer requests of the step: LDS reads issued behind those were seen to wait for
  // them): every sign word and code byte that it expands, the anomalous channels' scale and
  // zero point, the value words and scales.
  constexpr bool HOP_SZ = UA <= 2;           // scale and zero point in the batch too (registers allow it)
  struct FirstHop {
    uint32_t wn[2][U > 0 ? U : 1], wi[2][U > 0 ? U : 1], wa[2][UA > 0 ? UA : 1][2];
    uint2 as[2][HOP_SZ && UA > 0 ? UA : 1], az[2][HOP_SZ && UA > 0 ? UA : 1];
    u32x4 vw[2], sv;
  };
  auto first_hop = [&](auto ks_c, auto dok_c, auto dov_c, FirstHop& hop) {
    constexpr int KS = decltype(ks_c)::value;
    constexpr bool DO_K = decltype(dok_c)::value, DO_V = decltype(dov_c)::value;
    const uint8_t* stage = ring_w + KS * 2 * KREC;
    const uint8_t* vst = ring_w + 4 * KREC + (KS ^ 1) * 2 * VREC;
    if (DO_K) {
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint8_t* rec = stage + grp * KREC;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint8_t* wp = rec + OFF_BITS + (min(4 * u + kb, NB - 1) * 16 + x16) * 2;
          hop.wn[grp][u] = *reinterpret_cast<const uint16_t*>(wp);   // both tiles' bits (the upper 8 never reach a sign position)
          hop.wi[grp][u] = wp[1];                                     // the second tile's alone
        }
#pragma unroll
        for (int ua = 0; ua < UA; ++ua) {
          const int quad = min(4 * ua + kb, NQ - 1);
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) hop.wa[grp][ua][mt] = rec[(16 * mt + x16) * NQ + quad];
          if (HOP_SZ) {
            hop.as[grp][ua] = *reinterpret_cast<const uint2*>(rec + OFF_AS + quad * 8);
            hop.az[grp][ua] = *reinterpret_cast<const uint2*>(rec + OFF_AZ + quad * 8);
          }
        }
      }
    }
    if (DO_V) {
      hop.vw[0] = *reinterpret_cast<const u32x4*>(vst + lane * 16);
      hop.vw[1] = *reinterpret_cast<const u32x4*>(vst + VREC + lane * 16);
      hop.sv = *reinterpret_cast<const u32x4*>(vst + (kb >> 1) * VREC + 1024 + x16 * 16);
    }
  };

  // Scores of one pair from its key records (DO_K; key stage KS) and P V of the pair before
  // it from its value records and the packed probabilities pp (DO_V; value stage KS ^ 1),
  // as ONE instruction stream: the work items of the two - a K-step of channels, a channel
  // tile of values - alternate, each with the LDS reads of its successor in front, and the
  // scheduler is kept from pulling the two chains apart again.  Leaves S[token tile][4]
  // (per column) and the additive constant of the anomalous (and non-FFT) part.
  auto scores_and_values = [&](auto ks_c, auto dok_c, auto dov_c, const FirstHop& hop, f4 (&S)[2], float& cst) {
    constexpr int KS = decltype(ks_c)::value;
    constexpr bool DO_K = decltype(dok_c)::value, DO_V = decltype(dov_c)::value;
    constexpr int NKA = DO_K ? 2 * UA : 0, NKN = DO_K ? 2 * U : 0, NK = NKA + NKN;
    const uint8_t* stage = ring_w + KS * 2 * KREC;
    const uint32_t (&wn)[2][U > 0 ? U : 1] = hop.wn;
    const uint32_t (&wi)[2][U > 0 ? U : 1] = hop.wi;
    const uint32_t (&wa)[2][UA > 0 ? UA : 1][2] = hop.wa;
    u32x4 vw[2];
    Op sv, Ap[2];                                // sv: Eq. 6 scales of channels 16 m + x16, my rows' group
    if (DO_V) {
      vw[0] = hop.vw[0];
      vw[1] = hop.vw[1];
      sv.q = hop.sv;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        Ap[0].u[r] = pp[r] & keep0;
        Ap[1].u[r] = pp[r] & keep1;
      }
    }
    S[0] = zero; S[1] = zero;
    f4 accRe = zero, accIm = zero, accCn = zero, accC = zero;   // my column's group only: the operands are masked

    // ---- the work items
    // scales of the normal K-step n = (group, u)
    auto load_meta = [&](int n, Op& sre, Op& sim) {
      const int grp = n / (U > 0 ? U : 1), u = n % (U > 0 ? U : 1);
      const uint8_t* rec = stage + grp * KREC;
      const int blk = min(4 * u + kb, NB - 1);
      sre.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2) * 16);
      sim.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2 + ((FFT && x16) ? 1 : 0)) * 16);
    };
    // normal channels: Y[slot][col] per group, K = channels
    auto normal_item = [&](int n, const Op& sre, const Op& sim) {
      const int grp = n / (U > 0 ? U : 1), u = n % (U > 0 ? U : 1);
      const uint32_t w = wn[grp][u], w2 = wi[grp][u];
      Op Are, Aim;
      // bit e of a byte: channel e.  In x | x << 15 a channel pair (2r, 2r+1) sits 15 - 2r
      // below bits (15, 31); with the first tile's word in the lower and the second tile's in
      // the upper half, one 64-bit shift positions both (what it carries into the upper word
      // stays below bit 15)
      const uint64_t x2 = ((uint64_t)(w2 | (w2 << 15)) << 32) | (w | (w << 15));
      const uint64_t s0 = shl64<15>(x2), s1 = shl64<13>(x2), s2 = shl64<11>(x2), s3 = shl64<9>(x2);
      Are.u[0] = ((uint32_t)s0 & 0x80008000u) | sre.u[0]; Aim.u[0] = ((uint32_t)(s0 >> 32) & 0x80008000u) | sim.u[0];
      Are.u[1] = ((uint32_t)s1 & 0x80008000u) | sre.u[1]; Aim.u[1] = ((uint32_t)(s1 >> 32) & 0x80008000u) | sim.u[1];
      Are.u[2] = ((uint32_t)s2 & 0x80008000u) | sre.u[2]; Aim.u[2] = ((uint32_t)(s2 >> 32) & 0x80008000u) | sim.u[2];
      Are.u[3] = ((uint32_t)s3 & 0x80008000u) | sre.u[3]; Aim.u[3] = ((uint32_t)(s3 >> 32) & 0x80008000u) | sim.u[3];
      accRe = mma(Are, Bn[grp][u], accRe);
      accIm = mma(Aim, Bn[grp][u], accIm);
      if (!FFT) {
        // constant term, rows all equal: (-z)(-q/2) + (-s/2)(-q/2) = q (z + s/2) / 2
        const uint8_t* rec = stage + grp * KREC;
        const int blk = min(4 * u + kb, NB - 1);
        Op zq, Az, As;
        zq.q = *reinterpret_cast<const u32x4*>(rec + OFF_META + (blk * 2 + 1) * 16);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          Az.u[r] = zq.u[r] ^ 0x80008000u;
          As.u[r] = h2_bits(sre.p[r] * h2{(_Float16)0.5f, (_Float16)0.5f}) ^ 0x80008000u;
        }
        accCn = mma(Az, Bn[grp][u], accCn);
        accCn = mma(As, Bn[grp][u], accCn);
      }
    };
    // anomalous channels: rows = tokens, K = (channel, bit plane); the column operand is
    // zero outside my parity, so both groups add into S directly
    auto anomalous_item = [&](int n) {
      const int grp = n / (UA > 0 ? UA : 1), ua = n % (UA > 0 ? UA : 1);
      Op s4, z4;                                             // 4 halves each (low 8 bytes used)
      if (HOP_SZ) {
        *reinterpret_cast<uint2*>(&s4) = hop.as[grp][ua];
        *reinterpret_cast<uint2*>(&z4) = hop.az[grp][ua];
      } else {
        const uint8_t* rec = stage + grp * KREC;
        const int quad = min(4 * ua + kb, NQ - 1);
        *reinterpret_cast<uint2*>(&s4) = *reinterpret_cast<const uint2*>(rec + OFF_AS + quad * 8);
        *reinterpret_cast<uint2*>(&z4) = *reinterpret_cast<const uint2*>(rec + OFF_AZ + quad * 8);
      }
      uint32_t sp[4];                                        // (s/2, s) of channel r
      Op Ac1, Ac2;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        sp[r] = h2_bits(h2{s4.v[r], s4.v[r]} * h2{(_Float16)0.5f, (_Float16)1.0f});
        Ac1.p[r] = h2{z4.v[r], s4.v[r]};                     // z + s
        Ac2.u[r] = sp[r] & 0xFFFFu;                          // + s/2
      }
      // code bytes of my two tokens (tiles mt = 0, 1): bits (2r, 2r+1) of a byte are the
      // code of channel r, expanded like the sign words
      const uint32_t w0 = wa[grp][ua][0], w1 = wa[grp][ua][1];
      const uint64_t x2 = ((uint64_t)(w1 | (w1 << 15)) << 32) | (w0 | (w0 << 15));
      Op A0, A1;
      const uint64_t s0 = shl64<15>(x2), s1 = shl64<13>(x2), s2 = shl64<11>(x2), s3 = shl64<9>(x2);
      A0.u[0] = ((uint32_t)s0 & 0x80008000u) | sp[0]; A1.u[0] = ((uint32_t)(s0 >> 32) & 0x80008000u) | sp[0];
      A0.u[1] = ((uint32_t)s1 & 0x80008000u) | sp[1]; A1.u[1] = ((uint32_t)(s1 >> 32) & 0x80008000u) | sp[1];
      A0.u[2] = ((uint32_t)s2 & 0x80008000u) | sp[2]; A1.u[2] = ((uint32_t)(s2 >> 32) & 0x80008000u) | sp[2];
      A0.u[3] = ((uint32_t)s3 & 0x80008000u) | sp[3]; A1.u[3] = ((uint32_t)(s3 >> 32) & 0x80008000u) | sp[3];
      S[0] = mma(A0, Ba[grp][ua], S[0]);
      S[1] = mma(A1, Ba[grp][ua], S[1]);
      accC = mma(Ac1, Ba[grp][ua], accC);                    // rows all equal
      accC = mma(Ac2, Ba[grp][ua], accC);
    };
    // table entries of value tile m, both groups: byte (m & 1) of word m >> 1 holds the even
    // token slots 0, 2, 4, 6, byte 2 + (m & 1) the odd slots 1, 3, 5, 7
    auto lookup = [&](int m, uint2 (&E)[2], uint2 (&O)[2]) {
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        const uint32_t w = vw[grp][m >> 1];
        const uint32_t ae = (m & 1) ? byte_x8<1>(w) : byte_x8<0>(w);
        const uint32_t ao = (m & 1) ? byte_x8<3>(w) : byte_x8<2>(w);
        E[grp] = *reinterpret_cast<const uint2*>(ttrit_b + ae);
        O[grp] = *reinterpret_cast<const uint2*>(ttrit_b + ao);
      }
    };
    // P V of tile m: C[column][channel 16 m + x16] = sum_t p * code, then o += s * C
    auto value_tile = [&](int m, const uint2 (&E)[2], const uint2 (&O)[2]) {
      f4 C = zero;
#pragma unroll
      for (int grp = 0; grp < 2; ++grp) {
        Op Bv;
        Bv.u[0] = E[grp].x; Bv.u[1] = E[grp].y; Bv.u[2] = O[grp].x; Bv.u[3] = O[grp].y;
        C = mma(Ap[grp], Bv, C);
      }
      const float sc = (float)sv.v[m];
#pragma unroll
      for (int i = 0; i < 4; ++i) o[m][i] = fmaf(sc, C[i], o[m][i]);
    };

    // ---- the interleaved stream: anomalous items, then normal items; value tile j rides
    // with key item j NK / 8 (all eight at once when there are no key items)
    Op mre[2], mim[2];
    uint2 E[2][2], O[2][2];
    if (NKN > 0) load_meta(0, mre[0], mim[0]);
    if (DO_V) lookup(0, E[0], O[0]);
    __builtin_amdgcn_sched_barrier(0);
    constexpr int NSTEP = NK > 0 ? NK : 1;
#pragma unroll
    for (int k = 0; k < NSTEP; ++k) {
      if (k < NKA) {
        anomalous_item(k);
      } else if (k < NK) {
        const int n = k - NKA;
        if (n + 1 < NKN) load_meta(n + 1, mre[(n + 1) & 1], mim[(n + 1) & 1]);
        normal_item(n, mre[n & 1], mim[n & 1]);
      }
      if (DO_V) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if ((NK > 0 ? (j * NK) / 8 : 0) == k) {
            if (j + 1 < 8) lookup(j + 1, E[(j + 1) & 1], O[(j + 1) & 1]);
            value_tile(j, E[j & 1], O[j & 1]);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    cst = 0.0f;
    if (DO_K) {
      float cst_n = 0.0f;                        // non-FFT: sum over normal channels of q (z + s/2)
      if (U > 0 && !FFT) {
        // slot = token: the products are the scores' normal-channel part for my group
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          S[0][i] += accRe[i];
          S[1][i] += accIm[i];
        }
        cst_n = 2.0f * accCn[0];
      }
      if (U > 0 && FFT) {
        // split Y/16 into fp16 hi + lo, then the inverse DFT
        Op Yh, Yl, Wh[2], Wl[2];
        Wh[0].q = w_tab[0][lane]; Wh[1].q = w_tab[1][lane];
        Wl[0].q = w_tab[2][lane]; Wl[1].q = w_tab[3][lane];
#pragma unroll
        for (int i = 0; i < 4; i += 2) {
          const float r0 = accRe[i], r1 = accRe[i + 1];
          const float i0 = accIm[i], i1 = accIm[i + 1];
          Yh.u[i / 2] = pkrtz(r0, r1);
          Yh.u[2 + i / 2] = pkrtz(i0, i1);
          Yl.u[i / 2] = pkrtz(r0 - (float)Yh.v[i], r1 - (float)Yh.v[i + 1]);
          Yl.u[2 + i / 2] = pkrtz(i0 - (float)Yh.v[4 + i], i1 - (float)Yh.v[4 + i + 1]);
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          S[mt] = mma(Wh[mt], Yh, S[mt]);
          S[mt] = mma(Wl[mt], Yh, S[mt]);
          S[mt] = mma(Wh[mt], Yl, S[mt]);
        }
      }
      if (UA > 0) cst = accC[0];                 // = -(sum q (z + 1.5 s))
      if (!FFT) cst -= cst_n;
    }
  };

  // protected rows of the pair with masks (s0, s1), first rank rk0: fp16 rows (fetched ahead
  // into `rows`) weighted by the probabilities staged in pl
  auto add_protected = [&](uint32_t s0, uint32_t s1, uint32_t rk0, const uint32_t* rows, int st) {
    unsigned long long sm = (unsigned long long)s0 | ((unsigned long long)s1 << 32);
    auto add_row = [&](uint32_t bits, uint32_t r) {
      const int t64 = __ffsll((long long)sm) - 1;      // token of the pair
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
      Op ph;
      ph.q = *reinterpret_cast<const u32x4*>(&pl[wave][t64][0]);
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        const float f = (float)ph.v[h];
        osal[h][0] += f * v0;
        osal[h][1] += f * v1;
      }
    };
    // fp16 rows go two at a time: (row A, row B) of one channel as a packed pair against
    // the pair of their probabilities, one v_dot2_f32_f16 per (head, channel)
    auto add_rows2 = [&](uint32_t bitsA, uint32_t bitsB) {
      const int tA = __ffsll((long long)sm) - 1;
      sm &= sm - 1;
      const bool hasB = sm != 0;
      const int tB = hasB ? __ffsll((long long)sm) - 1 : tA;
      if (hasB) sm &= sm - 1; else bitsB = 0u;
      const h2 c0 = bits_h2(__builtin_amdgcn_perm(bitsB, bitsA, 0x05040100u));   // channel 2 lane
      const h2 c1 = bits_h2(__builtin_amdgcn_perm(bitsB, bitsA, 0x07060302u));   // channel 2 lane + 1
      Op pa, pb;
      pa.q = *reinterpret_cast<const u32x4*>(&pl[wave][tA][0]);
      pb.q = *reinterpret_cast<const u32x4*>(&pl[wave][tB][0]);
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        const h2 w = bits_h2(__builtin_amdgcn_perm(pb.u[h >> 1], pa.u[h >> 1],
                                                   (h & 1) ? 0x07060302u : 0x05040100u));
        osal[h][0] = __builtin_amdgcn_fdot2(c0, w, osal[h][0], false);
        osal[h][1] = __builtin_amdgcn_fdot2(c1, w, osal[h][1], false);
      }
    };
    if (SAL == 1) {
      // my two channels of row j: one dword of the staged row
      const uint32_t* rl = reinterpret_cast<const uint32_t*>(&rowring[wave][st][0]) + lane;
#pragma unroll
      for (int j = 0; j < NROWL; j += 2)
        if (sm) add_rows2(rl[j * (D / 2)], rl[(j + 1) * (D / 2)]);
      uint32_t rk = rk0 + NROWL;                        // more than NROWL rows: fetch on demand
      while (sm) {
        const uint32_t ra = row_word(rk);
        const uint32_t rb = (sm & (sm - 1)) ? row_word(rk + 1) : 0u;
        add_rows2(ra, rb);
        rk += 2;
      }
    } else {
#pragma unroll
      for (int j = 0; j < NROW; ++j)
        if (sm) add_row(rows[j], rk0 + j);
      uint32_t rk = rk0 + NROW;                         // more than NROW rows: fetch on demand
      while (sm) {
        add_row(row_word(rk), rk);
        ++rk;
      }
    }
  };

  // online softmax of the pair's scores: updates m_run, l_run (and rescales the running
  // sums when the maximum is raised), leaves the packed probabilities in pp and, when the
  // pair has protected tokens, stages them in pl as [token][head]
  auto softmax = [&](const f4 (&S)[2], float cst, bool v1ok, bool stage_pl) {
    // t = score - running maximum, in the exp2 domain, for my column at token slot i
    // (i < 4: token 4kb+i, else 16+4kb+i-4); a column without a group gets -inf
    const bool dead = par && !v1ok;
    const float c0 = dead ? -INFINITY : -cst * a.scale2;
    float c1 = c0 - m_run;
    float t[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      t[i] = fmaf(S[0][i], a.scale2, c1);
      t[4 + i] = fmaf(S[1][i], a.scale2, c1);
    }
    // The running maximum is raised lazily: only when some score exceeds it by more than 8
    // (p stays below 2^8), which needs no cross-lane traffic in the common case.
    float mx = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
    if (__any(mx > 8.0f || m_run == -INFINITY)) {
      // true scores again; maximum over the 4 k-blocks and the 2 parities of the head
      float smax;
      if (m_run == -INFINITY) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          t[i] = fmaf(S[0][i], a.scale2, c0);
          t[4 + i] = fmaf(S[1][i], a.scale2, c0);
        }
        smax = t[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) smax = fmaxf(smax, t[i]);
      } else {
        smax = mx + m_run;
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
    // probabilities as the A operand of P V (row = my column).  The k-slots of that product
    // are ordered (0,2), (4,6), (1,3), (5,7) in token-slot numbers: the order in which two
    // trit bytes expand (even slots, then odd slots).
    pp[0] = pk_rne(pr[0], pr[2]);
    pp[1] = pk_rne(pr[4], pr[6]);
    pp[2] = pk_rne(pr[1], pr[3]);
    pp[3] = pk_rne(pr[5], pr[7]);
    if ((SAL != 0) && stage_pl) {
      _Float16* pw = &pl[wave][32 * par][hcol];
      const h2 a0 = bits_h2(pp[0]), a1 = bits_h2(pp[1]), a2 = bits_h2(pp[2]), a3 = bits_h2(pp[3]);
      pw[8 * slot_token(kb, 0)] = a0[0];
      pw[8 * slot_token(kb, 2)] = a0[1];
      pw[8 * slot_token(kb, 4)] = a1[0];
      pw[8 * slot_token(kb, 6)] = a1[1];
      pw[8 * slot_token(kb, 1)] = a2[0];
      pw[8 * slot_token(kb, 3)] = a2[1];
      pw[8 * slot_token(kb, 5)] = a3[0];
      pw[8 * slot_token(kb, 7)] = a3[1];
    }
  };

  // ---------------- the loop, software-pipelined over two pairs: while the keys of pair p
  // are scored, the values (and protected rows) of the pair before it are added - two
  // independent chains of LDS reads, MFMAs and ALU work in one instruction stream.  A
  // pair's value records are therefore requested one step after its key records.
  // Step with key stage KS: keys of pair p in key stage KS; its values are requested into
  // value stage KS and its protected rows into rows<KS>; the previous pair's are in KS ^ 1.
  auto step = [&](auto ks_c, auto first_c) {
    constexpr int KS = decltype(ks_c)::value;
    constexpr bool FIRST = decltype(first_c)::value;
    const bool v1ok = (2 * p + 1) < a.ng;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // keys of p, values and rows of the pair before
    FirstHop hop;
    first_hop(ks_c, std::true_type{}, std::integral_constant<bool, !FIRST>{}, hop);
    __builtin_amdgcn_sched_barrier(0);
    if (p + 4 < p_end) fetch_keys(p + 4, KS ^ 1);
    fetch_values(p, KS);
    if ((SAL != 0)) {
      if (sm0c | sm1c) issue_rows(sm0c, sm1c, rkc, KS ? rows1 : rows0, KS);
      if (!FIRST && (sm0v | sm1v)) add_protected(sm0v, sm1v, rkv, KS ? rows0 : rows1, KS ^ 1);
    }
    f4 S[2];
    float cst;
    scores_and_values(ks_c, std::true_type{}, std::integral_constant<bool, !FIRST>{}, hop, S, cst);
    softmax(S, cst, v1ok, (sm0c | sm1c) != 0);
    if ((SAL != 0)) {
      sm0v = sm0c; sm1v = sm1c; rkv = rkc;
      sm0c = sm0n; sm1c = sm1n; rkc = rkn;
      load_masks(p + 8, sm0n, sm1n, rkn);
    }
  };
  int last_ks = -1;
  if (p < p_end) {
    step(std::integral_constant<int, 0>{}, std::true_type{});
    last_ks = 0;
    p += 4;
    while (p < p_end) {
      step(std::integral_constant<int, 1>{}, std::false_type{});
      last_ks = 1;
      p += 4;
      if (p >= p_end) break;
      step(std::integral_constant<int, 0>{}, std::false_type{});
      last_ks = 0;
      p += 4;
    }
  }
  // the last pair's values
  if (last_ks >= 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (last_ks == 0) {
      if ((SAL != 0) && (sm0v | sm1v)) add_protected(sm0v, sm1v, rkv, rows0, 0);
      f4 S[2]; float cst;
      FirstHop hop;
      first_hop(std::integral_constant<int, 1>{}, std::false_type{}, std::true_type{}, hop);
      scores_and_values(std::integral_constant<int, 1>{}, std::false_type{}, std::true_type{}, hop, S, cst);
    } else {
      if ((SAL != 0) && (sm0v | sm1v)) add_protected(sm0v, sm1v, rkv, rows1, 1);
      f4 S[2]; float cst;
      FirstHop hop;
      first_hop(std::integral_constant<int, 0>{}, std::false_type{}, std::true_type{}, hop);
      scores_and_values(std::integral_constant<int, 0>{}, std::false_type{}, std::true_type{}, hop, S, cst);
    }
  }

  // ---------------- per-wave reduction
  // l: 4 k-blocks and 2 parities of each head
  l_run = swap_sum32(l_run);
  l_run = swap_sum16(l_run);
  l_run += __shfl_xor(l_run, 8, 64);
  // o: rows 4kb+i; the parity 1 rows of a head live 32 lanes away from its parity 0 rows.
  // One lane-half swap of the register pair (tile m, tile m + 4) and one addition leave the
  // sums of tile m in lanes 0..31 and those of tile m + 4 in lanes 32..63.
  float* ow = reinterpret_cast<float*>(&ring[wave][0]);        // [8 heads][128 channels]
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // no transfer into the ring is left
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(o[m][i]), __float_as_uint(o[m + 4][i]), false, false);
      const float s = __uint_as_float(r[0]) + __uint_as_float(r[1]);
      ow[(4 * (kb & 1) + i) * D + 16 * (m + 4 * (kb >> 1)) + x16] = s;
    }
  if (kb == 0 && par == 0) { mw[wave][hcol] = m_run; lw[wave][hcol] = l_run; }
  if ((SAL != 0)) {
    // same wave, LDS operations complete in order: add the fp16-row part
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      ow[h * D + 2 * lane] += osal[h][0];
      ow[h * D + 2 * lane + 1] += osal[h][1];
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
          acc += f * reinterpret_cast<const float*>(&ring[w][0])[h * D + c];
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
