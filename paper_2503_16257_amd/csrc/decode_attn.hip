// Decode attention over the packed cache (Eq. 3; Alg. 1, Decoding):
// split-T partial softmax-attention with the dequantization fused in, then a
// log-sum-exp merge.  The dequantized K', V' never exist in memory.
//
// Normal key channels are scored in the frequency domain: by linearity
//   sum_c q_c IDFT(Xhat_c)[t] = IDFT(sum_c q_c Xhat_c)[t],
// so per 32-token group the +-s coefficients are contracted over channels first
// (Y[h][slot]) and a single 32-point inverse real DFT per query head follows.
//
// This file holds the plain-VALU kernel (any anomalous-channel count, and the
// fp16 residual tokens), the merge kernel and the launcher; the MFMA kernel
// that handles the common channel counts is in decode_attn_mfma.hip.
#include "decode_attn.h"
#include <atomic>

namespace vidkv {

// One workgroup = one (split, KV head, sequence); 256 threads.  Split index
// nsplit is the block that handles the fp16 residual tokens.
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
  const int split = blockIdx.x + a.split0, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int R = a.rep;
  const long long hd = ((long long)a.layer * a.B + b) * a.H + kvh;

  __shared__ float qp[MAX_REP][D];          // q in PERM order (anomalous first)
  __shared__ float qu[MAX_REP][D];          // q in channel order
  __shared__ u32x4 krec4[1536 / 16];
  __shared__ u32x4 vrec4[VREC / 16];
  __shared__ float Y[MAX_REP][32];
  __shared__ float P[MAX_REP][32];
  __shared__ float Alpha[MAX_REP];
  __shared__ float cs[32], sn[32];

  if (tid < 32) { cs[tid] = kCosT[tid]; sn[tid] = kCosT[(tid + 24) & 31]; }   // sin x = cos(x - pi/2)
  for (int i = tid; i < R * D; i += 256) {
    const int h = i >> 7, c = i & 127;
    const _Float16* qrow = a.q + ((long long)b * a.Hq + kvh * R + h) * D;
    qu[h][c] = (float)qrow[c];
    qp[h][c] = a.ng > 0 ? (float)qrow[a.kperm[hd * D + c]] : 0.0f;
  }
  __syncthreads();

  // roles
  const int t_s = tid & 31, h_s = tid >> 5;          // score / softmax role: (token, head)
  const int c_o = tid & 127, half_o = tid >> 7;      // output role: channel, heads half_o + 2 i
  float m_run = -INFINITY, l_run = 0.0f;             // valid in threads with h_s < R
  float acc[4] = {0.f, 0.f, 0.f, 0.f};

  // splits nsplit .. nsplit + ntail - 1 share the residual tokens, 32 * tail_per at a time
  const bool is_tail = (split >= a.nsplit);
  int n_iter, g_begin = 0, tl = 0, it0 = 0;
  if (!is_tail) {
    g_begin = split * a.gps;
    const int g_end = min(a.ng, g_begin + a.gps);
    n_iter = max(0, g_end - g_begin);
  } else {
    tl = a.tail_len ? a.tail_len[b] : 0;
    tl = min(max(tl, 0), a.cap);
    it0 = (split - a.nsplit) * a.tail_per;
    n_iter = max(0, min((tl + 31) / 32, it0 + a.tail_per) - it0);
  }

  const uint16_t* kbits = reinterpret_cast<const uint16_t*>(krec4) + 6 * a.n_a;
  const _Float16* krec16 = reinterpret_cast<const _Float16*>(krec4);
  const uint8_t* kcodes = reinterpret_cast<const uint8_t*>(krec4);
  const uint32_t* vwords = reinterpret_cast<const uint32_t*>(vrec4);
  const _Float16* vscale = reinterpret_cast<const _Float16*>(vrec4) + 512;

  for (int it = 0; it < n_iter; ++it) {
    float score = -INFINITY;
    uint32_t smask = 0, srank = 0;
    const int g = g_begin + it;
    if (!is_tail) {
      // ---- stage the two records
      const u32x4* ks = reinterpret_cast<const u32x4*>(a.krec + (hd * a.ngc + g) * (long long)a.krec_bytes);
      const u32x4* vs = reinterpret_cast<const u32x4*>(a.vrec + (hd * a.ngc + g) * (long long)VREC);
      if (tid < a.krec_bytes / 16) krec4[tid] = ks[tid];
      if (tid >= 128 && tid - 128 < VREC / 16) vrec4[tid - 128] = vs[tid - 128];
      if (a.n_s > 0) {
        smask = a.vmask[(size_t)b * a.ngc + g];
        srank = a.vrank[(size_t)b * a.ngc + g];
      }
      __syncthreads();
      // ---- Y[h][slot] = sum over normal channels of q * (+-s)
      if (h_s < R) {
        const int slot = t_s, k = slot & 15, hi = slot >> 4;
        const int use_im = (hi && k) ? 1 : 0;
        float y = 0.0f;
        for (int i = 0; i < a.n_n; ++i) {
          const int blk = i >> 3, e = i & 7;
          const uint32_t w = kbits[blk * 16 + k];
          const uint32_t bit = (w >> (8 * hi + e)) & 1u;
          const _Float16* meta = krec16 + 6 * a.n_a + 2 * a.n_n + blk * 16;
          float val;
          if (a.use_fft) {
            val = bit ? (float)meta[use_im * 8 + e] : -(float)meta[use_im * 8 + e];
          } else {
            val = fmaf((float)bit, (float)meta[e], (float)meta[8 + e]);
          }
          y += qp[h_s][a.n_a + i] * val;
        }
        Y[h_s][slot] = y;
      }
      __syncthreads();
      // ---- score[h][t]: inverse real DFT of Y plus the 2-bit channels
      if (h_s < R) {
        const int t = t_s;
        float v;
        if (a.use_fft) {
          v = Y[h_s][0] + ((t & 1) ? -Y[h_s][16] : Y[h_s][16]);
          float w2 = 0.0f;
#pragma unroll
          for (int k = 1; k < 16; ++k) {
            const int ph = (k * t) & 31;
            w2 += Y[h_s][k] * cs[ph] - Y[h_s][16 + k] * sn[ph];
          }
          v = (v + 2.0f * w2) * (1.0f / 32.0f);
        } else {
          v = Y[h_s][t];                     // Eq. 4 at 1 bit: slot = token, value = code * s + z
        }
        const int nq = a.n_a >> 2;
        for (int j = 0; j < a.n_a; ++j) {
          const uint32_t code = (kcodes[t * nq + (j >> 2)] >> (2 * (j & 3))) & 3u;
          const float s = (float)krec16[4 * a.n_a + j], z = (float)krec16[5 * a.n_a + j];
          v += qp[h_s][j] * ((float)code * s + z);
        }
        score = v * a.scale2;
      }
    } else {
      // ---- residual tokens: plain fp16 rows
      const int tok = (it0 + it) * 32 + t_s;
      if (h_s < R && tok < tl) {
        const u32x4* row = reinterpret_cast<const u32x4*>(
            a.ktail + (((long long)b * a.H + kvh) * a.cap + tok) * D);
        float v = 0.0f;
        for (int i = 0; i < 16; ++i) {
          U4H u;
          u.u = row[i];
#pragma unroll
          for (int e = 0; e < 8; ++e) v += qu[h_s][i * 8 + e] * (float)u.e[e];
        }
        score = v * a.scale2;
      }
    }
    // ---- online softmax over the 32 tokens of this step, per head (exp2 domain)
    if (h_s < R) {
      float mx = score;
#pragma unroll
      for (int d = 16; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 32));
      const float m_new = fmaxf(m_run, mx);
      const float p = (score == -INFINITY) ? 0.0f : exp2f(score - m_new);
      const float al = (m_run == -INFINITY) ? 0.0f : exp2f(m_run - m_new);
      float ps = p;
#pragma unroll
      for (int d = 16; d >= 1; d >>= 1) ps += __shfl_xor(ps, d, 32);
      l_run = l_run * al + ps;
      m_run = m_new;
      P[h_s][t_s] = p;
      if (t_s == 0) Alpha[h_s] = al;
    }
    __syncthreads();
    // ---- output accumulation
    if (!is_tail) {
      uint32_t w[4];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) w[kb] = vwords[(kb * 16 + (c_o & 15)) * 4 + (c_o >> 5)];
      const float s = (float)vscale[(c_o & 15) * 8 + (c_o >> 4)];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int h = half_o + 2 * i;
        if (h < R) {
          float dot = 0.0f;
#pragma unroll
          for (int t = 0; t < 32; ++t) {
            const int kb = (t & 15) >> 2, j = (t & 3) + ((t >= 16) ? 4 : 0);
            const uint32_t f = (w[kb] >> (8 * ((c_o >> 4) & 1) + 16 * (j & 1) + 2 * (j >> 1))) & 3u;
            const float val = (f & 1u) ? ((f & 2u) ? -1.0f : 1.0f) : 0.0f;
            dot += P[h][t] * val;
          }
          acc[i] = acc[i] * Alpha[h] + s * dot;
        }
      }
      uint32_t sm = smask;
      uint32_t r = srank;
      while (sm) {
        const int t = __ffs(sm) - 1;
        sm &= sm - 1;
        const float v = a.sal_bits == 2 ? protected2_value(a, hd, r, c_o)
                                        : (float)a.vrows[(hd * a.n_s + r) * D + c_o];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int h = half_o + 2 * i;
          if (h < R) acc[i] += P[h][t] * v;
        }
        ++r;
      }
    } else {
      const int nt = min(32, tl - (it0 + it) * 32);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int h = half_o + 2 * i;
        if (h < R) acc[i] *= Alpha[h];
      }
      // 8 rows in flight per thread (a row past the end repeats the last one and is not used)
      const _Float16* vcol = a.vtail + (((long long)b * a.H + kvh) * a.cap + (it0 + it) * 32) * D + c_o;
      for (int t0 = 0; t0 < nt; t0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (float)vcol[(long long)min(t0 + u, nt - 1) * D];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (t0 + u < nt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int h = half_o + 2 * i;
              if (h < R) acc[i] += P[h][t0 + u] * v[u];
            }
          }
        }
      }
    }
    __syncthreads();
  }

  // ---- write the partial (o, m, l) of every head of this KV head
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int h = half_o + 2 * i;
    if (h < R) {
      float* o = a.part + (((long long)split * a.B + b) * a.Hq + kvh * R + h) * PART_STRIDE;
      o[c_o] = acc[i];
    }
  }
  if (h_s < R && t_s == 0) {
    float* o = a.part + (((long long)split * a.B + b) * a.Hq + kvh * R + h_s) * PART_STRIDE;
    o[D] = m_run;
    o[D + 1] = l_run;
  }
}

// The fp16 residual tokens (Alg. 1's X_Kr, X_Vr): one workgroup = one (tail split, KV head,
// sequence); split ts takes the 32-token steps ts * tail_per .. of the buffer and writes its
// partial (o, m, l) as split index nsplit + ts.  Thread roles: scores (token = tid % 32,
// head = tid / 32), output (channel = tid % 128, heads tid / 128 + 2 i).
__global__ __launch_bounds__(256) void attn_tail_kernel(AttnArgs a) {
  const int ts = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int split = a.nsplit + ts;
  const int tid = threadIdx.x;
  const int R = a.rep;
  __shared__ float t_q[MAX_REP][D];
  __shared__ float t_P[MAX_REP][32];
  __shared__ float t_alpha[MAX_REP];
  for (int i = tid; i < R * D; i += 256)
    t_q[i >> 7][i & 127] = (float)a.q[((long long)b * a.Hq + kvh * R + (i >> 7)) * D + (i & 127)];
  const int t_s = tid & 31, h_s = tid >> 5;
  const int c_o = tid & 127, half_o = tid >> 7;
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  int tl = a.tail_len ? a.tail_len[b] : 0;
  tl = min(max(tl, 0), a.cap);
  const int it0 = ts * a.tail_per;
  const int n_iter = max(0, min((tl + 31) / 32, it0 + a.tail_per) - it0);
  const long long head_row0 = ((long long)b * a.H + kvh) * a.cap;
  for (int it = 0; it < n_iter; ++it) {
    const int tok0 = (it0 + it) * 32;
    const int nt = min(32, tl - tok0);
    // everything this step reads is requested up front: my key row (16 pieces) and my
    // channel of the 32 value rows (a row past the end repeats the last one and is not used)
    const bool scorer = h_s < R && t_s < nt;
    U4H kr[16];
    if (scorer) {
      const u32x4* row = reinterpret_cast<const u32x4*>(a.ktail + (head_row0 + tok0 + t_s) * D);
#pragma unroll
      for (int i = 0; i < 16; ++i) kr[i].u = row[i];
    }
    const _Float16* vcol = a.vtail + (head_row0 + tok0) * D + c_o;
    _Float16 vv[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) vv[u] = vcol[(long long)min(u, nt - 1) * D];
    if (it == 0) __syncthreads();                    // q is in LDS (its loads overlapped the above)
    float score = -INFINITY;
    if (scorer) {
      float v = 0.0f;
#pragma unroll
      for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) v += t_q[h_s][i * 8 + e] * (float)kr[i].e[e];
      score = v * a.scale2;
    }
    if (h_s < R) {                                   // online softmax of this step (exp2 domain)
      float mx = score;
#pragma unroll
      for (int d = 16; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 32));
      const float m_new = fmaxf(m_run, mx);
      const float p = (score == -INFINITY) ? 0.0f : exp2f(score - m_new);
      const float al = (m_run == -INFINITY) ? 0.0f : exp2f(m_run - m_new);
      float ps = p;
#pragma unroll
      for (int d = 16; d >= 1; d >>= 1) ps += __shfl_xor(ps, d, 32);
      l_run = l_run * al + ps;
      m_run = m_new;
      t_P[h_s][t_s] = p;
      if (t_s == 0) t_alpha[h_s] = al;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int h = half_o + 2 * i;
      if (h < R) {
        float s_acc = acc[i] * t_alpha[h];
#pragma unroll
        for (int u = 0; u < 32; ++u) s_acc += t_P[h][u] * (float)vv[u];   // t_P is 0 past the end
        acc[i] = s_acc;
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int h = half_o + 2 * i;
    if (h < R) a.part[(((long long)split * a.B + b) * a.Hq + kvh * R + h) * PART_STRIDE + c_o] = acc[i];
  }
  if (h_s < R && t_s == 0) {
    float* o = a.part + (((long long)split * a.B + b) * a.Hq + kvh * R + h_s) * PART_STRIDE;
    o[D] = m_run;
    o[D + 1] = l_run;
  }
}

// Merge of the split partials: out = sum_i o_i 2^{m_i - M} / sum_i l_i 2^{m_i - M}.
// grid (Hq, B), block 1024 = 128 channels x 8 slices of the split list.
__global__ __launch_bounds__(1024) void attn_merge_kernel(const float* __restrict__ part,
                                                          int nparts, int B, int Hq,
                                                          _Float16* __restrict__ out) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int c = threadIdx.x & 127, sl = threadIdx.x >> 7;
  __shared__ float so[8][D];
  __shared__ float sl_[8];
  // running maximum over all parts: one part per thread, then wave and block maxima
  __shared__ float sW[16];
  float M = -INFINITY;
  for (int i = threadIdx.x; i < nparts; i += 1024)
    M = fmaxf(M, part[(((long long)i * B + b) * Hq + h) * PART_STRIDE + D]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d, 64));
  if ((threadIdx.x & 63) == 0) sW[threadIdx.x >> 6] = M;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) M = fmaxf(M, sW[i]);
  // weighted sums, 4 parts in flight per thread
  float o = 0.0f, l = 0.0f;
  for (int i0 = sl; i0 < nparts; i0 += 32) {
    float mi[4], oi[4], li[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 8 * u;
      const bool ok = i < nparts;
      const float* p = part + (((long long)(ok ? i : 0) * B + b) * Hq + h) * PART_STRIDE;
      mi[u] = ok ? p[D] : -INFINITY;
      oi[u] = ok ? p[c] : 0.0f;
      li[u] = ok ? p[D + 1] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = mi[u] == -INFINITY ? 0.0f : exp2f(mi[u] - M);
      if (w != 0.0f) {                     // an empty part's sums are never looked at
        o += w * oi[u];
        l += w * li[u];
      }
    }
  }
  so[sl][c] = o;
  if (c == 0) sl_[sl] = l;
  __syncthreads();
  if (sl == 0) {
#pragma unroll
    for (int i = 1; i < 8; ++i) { o += so[i][c]; l += sl_[i]; }
    out[((long long)b * Hq + h) * D + c] = (_Float16)(l > 0.0f ? o / l : 0.0f);
  }
}

// The same merge for at most 8 * MAXU parts: every load of a thread is issued before the
// first use (one round trip to memory instead of one per 32 parts and one for the maximum).
// Thread (slice sl, channel c) owns parts sl, sl + 8, ...
template <int MAXU>
__global__ __launch_bounds__(1024) void attn_merge_small_kernel(const float* __restrict__ part,
                                                                int nparts, int B, int Hq,
                                                                _Float16* __restrict__ out) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int c = threadIdx.x & 127, sl = threadIdx.x >> 7;
  __shared__ float so[8][D];
  __shared__ float sl_[8];
  __shared__ float sM[8];
  float mi[MAXU], oi[MAXU], li[MAXU];
#pragma unroll
  for (int u = 0; u < MAXU; ++u) {
    const int i = sl + 8 * u;
    const bool ok = i < nparts;
    const float* p = part + (((long long)(ok ? i : 0) * B + b) * Hq + h) * PART_STRIDE;
    mi[u] = ok ? p[D] : -INFINITY;
    oi[u] = ok ? p[c] : 0.0f;
    li[u] = ok ? p[D + 1] : 0.0f;
  }
  float M = mi[0];
#pragma unroll
  for (int u = 1; u < MAXU; ++u) M = fmaxf(M, mi[u]);
  if (c == 0) sM[sl] = M;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) M = fmaxf(M, sM[i]);
  float o = 0.0f, l = 0.0f;
#pragma unroll
  for (int u = 0; u < MAXU; ++u) {
    const float w = mi[u] == -INFINITY ? 0.0f : exp2f(mi[u] - M);
    if (w != 0.0f) {                       // an empty part's sums are never looked at
      o += w * oi[u];
      l += w * li[u];
    }
  }
  so[sl][c] = o;
  if (c == 0) sl_[sl] = l;
  __syncthreads();
  if (sl == 0) {
#pragma unroll
    for (int i = 1; i < 8; ++i) { o += so[i][c]; l += sl_[i]; }
    out[((long long)b * Hq + h) * D + c] = (_Float16)(l > 0.0f ? o / l : 0.0f);
  }
}

// At most MAXP parts (large batches): one thread per channel holds every part, no LDS.
template <int MAXP>
__global__ __launch_bounds__(128) void attn_merge_tiny_kernel(const float* __restrict__ part,
                                                              int nparts, int B, int Hq,
                                                              _Float16* __restrict__ out) {
  const int h = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  float mi[MAXP], oi[MAXP], li[MAXP];
#pragma unroll
  for (int u = 0; u < MAXP; ++u) {
    const bool ok = u < nparts;
    const float* p = part + (((long long)(ok ? u : 0) * B + b) * Hq + h) * PART_STRIDE;
    mi[u] = ok ? p[D] : -INFINITY;
    oi[u] = ok ? p[c] : 0.0f;
    li[u] = ok ? p[D + 1] : 0.0f;
  }
  float M = mi[0];
#pragma unroll
  for (int u = 1; u < MAXP; ++u) M = fmaxf(M, mi[u]);
  float o = 0.0f, l = 0.0f;
#pragma unroll
  for (int u = 0; u < MAXP; ++u) {
    const float w = mi[u] == -INFINITY ? 0.0f : exp2f(mi[u] - M);
    if (w != 0.0f) {                       // an empty part's sums are never looked at
      o += w * oi[u];
      l += w * li[u];
    }
  }
  out[((long long)b * Hq + h) * D + c] = (_Float16)(l > 0.0f ? o / l : 0.0f);
}

// Compute units of the current device, asked once per device. A process with no usable
// device (a size query on a build host) gets the MI355X figure, 256.
static int device_cu_count() {
  constexpr int MAXDEV = 64;
  static std::atomic<int> cached[MAXDEV];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAXDEV) {
    (void)hipGetLastError();
    return 256;
  }
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
    (void)hipGetLastError();
    n = 256;
  }
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Number of split-T workgroups per (sequence, KV head).
int attn_num_splits(const Geom& g) {
  if (g.ng == 0) return 0;
  const long long bh = (long long)g.B * g.H;
  const bool mfma = attn_mfma_supported(g.n_a);
  // MFMA kernel: 4 waves per workgroup, each wave walks pairs of groups; two workgroups
  // are resident per compute unit, so aim at one full round of them, and at no less than
  // 8 pairs per workgroup. The scalar kernel runs four workgroups per compute unit.
  const long long cus = device_cu_count();
  const long long target = mfma ? 2 * cus : 4 * cus;
  long long n = (target + bh - 1) / bh;
  const long long units = mfma ? ((g.ng + 1) / 2 + 7) / 8 : g.ng;
  if (n > units) n = units;
  if (n < 1) n = 1;
  return (int)n;
}

// A large block of residual tokens is worth a stream of its own: its kernel is short of
// memory parallelism, not of arithmetic, and runs well beside the MFMA kernel.
bool attn_tail_beside(const Geom& g, int cap) {
  if (cap <= 0 || g.ng == 0 || !attn_mfma_supported(g.n_a)) return false;
  const int iters = (cap + 31) / 32;
  const long long wgs = (long long)(iters < ATTN_TAIL_SPLITS ? iters : ATTN_TAIL_SPLITS) * g.B * g.H;
  return wgs >= 4LL * device_cu_count();
}

// side / fork / join: when side is not null (and there are residual tokens for the MFMA
// path) the residual-token kernel is forked onto that stream and joined before the merge.
hipError_t launch_decode_attention(const Geom& g, int layer, float scale, const void* q,
                                   const uint8_t* pk, const uint8_t* pv, const void* ktail,
                                   const void* vtail, int cap, const int32_t* tail_len, void* out,
                                   void* ws, unsigned stages, hipStream_t st, hipStream_t side,
                                   hipEvent_t fork, hipEvent_t join) {
  AttnArgs a;
  a.q = reinterpret_cast<const _Float16*>(q);
  a.kperm = pk + g.k_perm;
  a.krec = pk + g.k_rec;
  a.vrec = pv + g.v_rec;
  a.vmask = reinterpret_cast<const uint32_t*>(pv + g.v_mask);
  a.vrank = reinterpret_cast<const uint32_t*>(pv + g.v_rank);
  a.vrows = reinterpret_cast<const _Float16*>(pv + g.v_rows);
  a.ktail = reinterpret_cast<const _Float16*>(ktail);
  a.vtail = reinterpret_cast<const _Float16*>(vtail);
  const bool has_tail = cap > 0 && ktail && vtail && tail_len;
  a.tail_len = has_tail ? tail_len : nullptr;
  a.part = reinterpret_cast<float*>(ws);
  a.layer = layer; a.B = g.B; a.H = g.H; a.Hq = g.Hq; a.rep = g.rep; a.ng = g.ng; a.ngc = g.ngc;
  a.n_a = g.n_a; a.n_n = g.n_n; a.n_s = g.n_s; a.krec_bytes = g.krec; a.cap = cap;
  a.sal_bits = g.sal_bits; a.npg = g.npg; a.use_fft = g.use_fft ? 1 : 0;
  a.nsplit = attn_num_splits(g);
  a.scale2 = scale * 1.4426950408889634f;
  a.split0 = 0;
  // stages: bit 0 split-T partial kernel(s), bit 1 merge
  const bool mfma = a.nsplit > 0 && attn_mfma_supported(g.n_a);
  // with the MFMA kernel the residual-token block is a launch of its own and is
  // skipped when there is no residual buffer
  // residual tokens: up to ATTN_TAIL_SPLITS workgroups per (sequence, KV head)
  const int tail_iters = has_tail ? (cap + 31) / 32 : 0;
  const int ntail = has_tail ? (tail_iters < ATTN_TAIL_SPLITS ? tail_iters : ATTN_TAIL_SPLITS) : (mfma ? 0 : 1);
  a.tail_per = ntail > 0 && tail_iters > 0 ? (tail_iters + ntail - 1) / ntail : 0;
  const int nparts = a.nsplit + ntail;
  if (stages & 1u) {
    if (mfma) {
      const int npairs = (g.ng + 1) / 2;
      a.gps = (npairs + a.nsplit - 1) / a.nsplit;          // pairs per split
      if (has_tail && side) {
        if (hipEventRecord(fork, st) != hipSuccess) return hipErrorUnknown;
        if (hipStreamWaitEvent(side, fork, 0) != hipSuccess) return hipErrorUnknown;
        // the side stream now depends on `st`: it is joined back whatever fails below
        hipLaunchKernelGGL(attn_tail_kernel, dim3(ntail, g.H, g.B), dim3(256), 0, side, a);
        const bool rec = hipEventRecord(join, side) == hipSuccess;
        launch_attn_mfma(a, dim3(a.nsplit, g.H, g.B), st);
        const bool joined = hipStreamWaitEvent(st, join, 0) == hipSuccess;
        if (!rec || !joined) return hipErrorUnknown;
      } else {
        launch_attn_mfma(a, dim3(a.nsplit, g.H, g.B), st);
        if (has_tail)
          hipLaunchKernelGGL(attn_tail_kernel, dim3(ntail, g.H, g.B), dim3(256), 0, st, a);
      }
    } else {
      a.gps = a.nsplit ? (g.ng + a.nsplit - 1) / a.nsplit : 0;
      hipLaunchKernelGGL(attn_partial_kernel, dim3(a.nsplit + ntail, g.H, g.B), dim3(256), 0, st, a);
    }
  }
  if (stages & 2u) {
    _Float16* o16 = reinterpret_cast<_Float16*>(out);
    if (nparts <= 16)
      hipLaunchKernelGGL(attn_merge_tiny_kernel<16>, dim3(g.Hq, g.B), dim3(128), 0, st, a.part,
                         nparts, g.B, g.Hq, o16);
    else if (nparts <= 32)
      hipLaunchKernelGGL(attn_merge_tiny_kernel<32>, dim3(g.Hq, g.B), dim3(128), 0, st, a.part,
                         nparts, g.B, g.Hq, o16);
    else if (nparts <= 136)
      hipLaunchKernelGGL(attn_merge_small_kernel<17>, dim3(g.Hq, g.B), dim3(1024), 0, st, a.part,
                         nparts, g.B, g.Hq, o16);
    else
      hipLaunchKernelGGL(attn_merge_kernel, dim3(g.Hq, g.B), dim3(1024), 0, st, a.part, nparts,
                         g.B, g.Hq, o16);
  }
  return hipGetLastError();
}

}  // namespace vidkv
