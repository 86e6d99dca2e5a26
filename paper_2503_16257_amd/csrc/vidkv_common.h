// Shared host/device definitions of the VidKV HIP library: cache geometry,
// packed-buffer section offsets, launch helpers.
//
// Packed key buffer   : [PERM uint8 LBH x 128][REC LBH x Tq/32 records]
//   record (12*n_a + 8*n_n bytes):
//     +0            uint8  [32 tok][n_a/4]  2-bit codes, channel 4q+j in bits 2j,2j+1
//     +8 n_a        fp16   [n_a]  s          (Eq. 4)
//     +10 n_a       fp16   [n_a]  z
//     +12 n_a       uint16 [n_n/8][16]      bit e: sign(Re X[k]) of channel 8 blk+e,
//                                            bit 8+e: sign(Im X[k]) (k>=1) / sign(Re X[16]) (k=0)
//     +12 n_a+4 n_n fp16   [n_n/8][2][8]    s_re, s_im      (Eq. 5)
// Packed value buffer : [REC LBH x Tq/32 x 1280][IDX][MASK][RANK][ROWS]
//   record: uint32 [4 kb][16 r][4 mp]: word (kb, r, mp) holds 8 token slots of the
//           channels 16 m + r, m = 2 mp + mh (slot j: token 4 kb + j for j<4,
//           16 + 4 kb + j-4 otherwise); field of (mh, j) at bit 8 mh + 16 (j&1) +
//           2 (j>>1): nonzero flag, then negative flag;
//           then fp16 [16 r][8 m] s (Eq. 6) of channel 16 m + r.
// Every section starts on a 256-byte boundary.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/vidkv.h"

namespace vidkv {

constexpr int D = 128;
constexpr int G = 32;
constexpr int VREC = 1280;         // bytes of one value record
constexpr int PREC = 1536;         // bytes of one record of 32 protected rows at 2 bits (Eq. 4)
constexpr int RANGE_CHUNK = 512;   // tokens per workgroup in the key range pass
constexpr int MAX_REP = 8;         // query heads per KV head
constexpr int ATTN_TAIL_SPLITS = 8; // most workgroups that share one head's residual tokens in attention

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes viewed as 8 fp16 values
union U4H {
  u32x4 u;
  h2 h[4];
  _Float16 e[8];
};

struct Geom {
  int L, B, H, Hq, rep, T, ng, n_a, n_n, n_s;
  int Tcap, ngc;                   // capacity in tokens / groups: every per-head stride uses ngc
  int metric;                      // channel ranking: 0 range, 1 variance, 2 outlier count
  bool use_fft;                    // normal key channels: Eq. 5 (true) or Eq. 4 at 1 bit (false)
  int sal_bits, npg;               // protected rows: 16 = fp16, 2 = Eq. 4 records; groups of 32 rows
  long long nheads;                // L*B*H
  int krec;                        // bytes of one key record
  // key buffer
  size_t k_perm, k_rec, k_total;
  // value buffer
  size_t v_rec, v_idx, v_mask, v_rank, v_rows, v_total;
  int range_chunks;                // workgroups per head in the range pass
};

// Which heads and groups a coding launch covers: the whole tensor at prefill,
// or one layer's residual block appended behind the groups already packed.
struct EncodeSpan {
  int in_tokens;      // tokens per head of the input tensor (its head stride)
  int ng;             // groups to code, from input token 0 on
  int g_out0;         // output group of input group 0
  long long heads;    // heads covered by the launch
  long long head0;    // first of them inside the packed buffer
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline bool make_geom(const vidkv_params* p, Geom* g) {
  if (!p) return false;
  if (p->n_layers < 1 || p->batch < 1 || p->n_kv_heads < 1) return false;
  if (p->n_q_heads < p->n_kv_heads || p->n_q_heads % p->n_kv_heads) return false;
  if (p->n_q_heads / p->n_kv_heads > MAX_REP) return false;
  if (p->head_dim != D || p->group != G) return false;
  if (p->t_quant < 0 || p->t_quant % G) return false;
  if (p->n_anom < 0 || p->n_anom > D || p->n_anom % 8) return false;
  if (p->use_fft != 0 && p->use_fft != 1) return false;
  if (p->n_salient < 0 || p->n_salient > p->t_quant) return false;
  if (p->t_capacity != 0 && (p->t_capacity < p->t_quant || p->t_capacity % G)) return false;
  if (p->salient_bits != 0 && p->salient_bits != 16 && p->salient_bits != 2) return false;
  if (p->channel_metric < 0 || p->channel_metric > 2) return false;
  g->L = p->n_layers; g->B = p->batch; g->H = p->n_kv_heads; g->Hq = p->n_q_heads;
  g->rep = g->Hq / g->H;
  g->T = p->t_quant; g->ng = g->T / G;
  g->Tcap = p->t_capacity ? p->t_capacity : p->t_quant; g->ngc = g->Tcap / G;
  g->n_a = p->n_anom; g->n_n = D - g->n_a; g->n_s = p->n_salient;
  g->use_fft = p->use_fft == 1;
  g->metric = p->channel_metric;
  g->sal_bits = p->salient_bits == 2 ? 2 : 16;
  g->npg = (g->n_s + G - 1) / G;
  g->nheads = (long long)g->L * g->B * g->H;
  g->krec = 12 * g->n_a + 8 * g->n_n;
  g->k_perm = 0;
  g->k_rec = align256((size_t)g->nheads * D);
  g->k_total = align256(g->k_rec + (size_t)g->nheads * g->ngc * g->krec);
  g->v_rec = 0;
  size_t off = align256((size_t)g->nheads * g->ngc * VREC);
  g->v_idx = g->v_mask = g->v_rank = g->v_rows = off;
  if (g->n_s > 0) {
    g->v_idx = off;  off = align256(off + 4ull * g->B * g->n_s);
    g->v_mask = off; off = align256(off + 4ull * g->B * g->ngc);
    g->v_rank = off; off = align256(off + 4ull * g->B * g->ngc);
    g->v_rows = off;
    off = align256(off + (g->sal_bits == 2 ? (size_t)g->nheads * g->npg * PREC
                                           : 2ull * g->nheads * g->n_s * D));
  }
  g->v_total = off;
  g->range_chunks = (g->T + RANGE_CHUNK - 1) / RANGE_CHUNK;
  return true;
}

// cos / sin of 2 pi j / 32 from one first-octant table (values rounded to
// fp32), with the symmetries applied exactly so that quarter-turn values are
// exactly 0 and +-1.  All uses pass compile-time j.
__host__ __device__ constexpr float cos32(int j) {
  constexpr float C[9] = {1.0f, 0.980785251f, 0.923879504f, 0.831469595f, 0.707106769f,
                          0.555570245f, 0.382683426f, 0.195090324f, 0.0f};
  j = ((j % 32) + 32) % 32;
  if (j > 16) j = 32 - j;
  return j > 8 ? -C[16 - j] : C[j];
}
__host__ __device__ constexpr float sin32(int j) { return cos32(j - 8); }

}  // namespace vidkv
