// Shared declarations of the decode-attention kernels.
#pragma once
#include "mfma_util.h"

namespace vidkv {

struct AttnArgs {
  const _Float16* q;         // [B, Hq, 128]
  const uint8_t* kperm;      // key PERM section (whole buffer)
  const uint8_t* krec;       // key REC section (whole buffer)
  const uint8_t* vrec;       // value REC section (whole buffer)
  const uint32_t* vmask;     // [B, ngc] or unused
  const uint32_t* vrank;     // [B, ngc]
  const _Float16* vrows;     // protected rows: [L, B, H, n_s, 128] fp16, or 2-bit records
                             // [L, B, H, npg] of PREC bytes when sal_bits == 2
  const _Float16* ktail;     // [B, H, cap, 128]
  const _Float16* vtail;
  const int32_t* tail_len;   // [B] or NULL
  float* part;               // [nsplit + tail splits, B, Hq, 130]
  int layer, B, H, Hq, rep, ng, n_a, n_n, n_s, krec_bytes, cap, nsplit, gps;
  int ngc;                   // groups of capacity: stride of the per-head record arrays
  int use_fft;               // normal key channels coded by Eq. 5 (1) or by Eq. 4 at 1 bit (0)
  int sal_bits, npg;         // protected rows kept as fp16 (16) or Eq. 4 codes (2); groups of 32 rows
  int split0;                // added to blockIdx.x (tail-only launches start at nsplit)
  int tail_per;              // 32-token steps of the residual buffer per tail split
  float scale2;              // softmax scale * log2(e): scores live in the exp2 domain
};

// One split partial per (split, sequence, query head): o[128], m, l with
// p = 2^(score2 - m), l = sum p, o = sum p v.
constexpr int PART_STRIDE = D + 2;

// Channel c of protected row r of head hd when the rows are kept at 2 bits (Eq. 4):
// code * s + z with the record's fp16 s, z.
__device__ __forceinline__ float protected2_value(const AttnArgs& a, long long hd, uint32_t r, int c) {
  const uint8_t* rec = reinterpret_cast<const uint8_t*>(a.vrows) + (hd * a.npg + (r >> 5)) * (long long)PREC;
  const uint32_t code = (rec[(r & 31) * 32 + (c >> 2)] >> (2 * (c & 3))) & 3u;
  const float s = (float)reinterpret_cast<const _Float16*>(rec + 1024)[c];
  const float z = (float)reinterpret_cast<const _Float16*>(rec + 1280)[c];
  return fmaf((float)code, s, z);
}

// true if the MFMA kernel has an instantiation for this anomalous-channel count
bool attn_mfma_supported(int n_a);
void launch_attn_mfma(const AttnArgs& a, dim3 grid, hipStream_t st);

}  // namespace vidkv
