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

// Exclusive scan of one int per thread over a 256-thread block; `sw` is LDS
// scratch of 4 ints.  Returns the exclusive prefix, *total the block sum.
__device__ __forceinline__ int block_exscan_256(int v, int* sw, int* total) {
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
  for (int i = 0; i < 4; ++i) {
    const int s = sw[i];
    base += (i < wv) ? s : 0;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

// ---------------------------------------------------------------------------
// Protected-token selection, several workgroups per sequence.
//
// From scores: the n_s largest by (score desc, index asc) via a 3-level radix
// select on the ordered 32-bit keys (11 + 11 + 10 bits).  Each level is one
// launch: every workgroup histograms its slice of LV_SLICE tokens in LDS and
// adds it to that level's global histogram.  Nobody waits inside a launch: the
// scan of a level's histogram (which bin holds the remaining-th largest key) is
// done by every workgroup of the NEXT launch at its start, redundantly, while
// its score loads are in flight; the first workgroup also records the narrowed
// (prefix, remaining) pair for the launch after.  Then a counting launch
// (selected / tied elements per slice of SEL_SLICE tokens) and a marking launch
// that sums the counts of the slices before its own and writes MASK, RANK and
// IDX.  From an index list: MASK is zeroed and set by atomics, then the same
// counting and marking launches run on the mask.
//
// Workspace (ints): per sequence b
//   st[b][3][2]                (prefix, remaining) after the scan of level 0, 1, 2
//   hist[b][3][2048]
//   cnt[b][nslice][2]          selected, tied          (per slice)
// ---------------------------------------------------------------------------
constexpr int SEL_SLICE = 8192;                  // tokens per workgroup = 256 groups
constexpr int SEL_BINS = 2048;
constexpr int LV_SLICE = 2048;                   // tokens per workgroup of a radix level

struct SelWs {
  int* st; int* hist; int* cnt;
  int nslice;
};

__host__ __device__ inline size_t sel_ws_ints(int B, int nslice) {
  return (size_t)B * (8 + 3 * SEL_BINS + 2 * (size_t)nslice);
}

__device__ __host__ inline SelWs sel_ws(void* ws, int B, int nslice) {
  SelWs w;
  int* p = reinterpret_cast<int*>(ws);
  w.hist = p;  p += (size_t)B * 3 * SEL_BINS;       // zeroed by the init launch
  w.st = p;    p += (size_t)B * 8;
  w.cnt = p;
  w.nslice = nslice;
  return w;
}

// zeroes the histograms (and, for the index-list path, MASK)
__global__ __launch_bounds__(256) void v_sel_init_kernel(int* __restrict__ hist, size_t n_ints,
                                                         uint32_t* __restrict__ mask, size_t n_mask) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_ints) hist[i] = 0;
  if (mask && i < n_mask) mask[i] = 0;
}

// Which bin of a finished histogram holds the rem-th largest key, and which
// rank it has inside that bin.  All 256 threads of the block call this; thread
// t owns the PER bins of group 255 - t, so an exclusive scan over threads gives
// the count of keys in all higher bins.  sres[0] = bin, sres[1] = new remaining.
template <int NB>
__device__ __forceinline__ void find_bin(const int* __restrict__ gh, int rem, int* sw, int* sres) {
  constexpr int PER = NB / 256;
  const int grp = 255 - (int)threadIdx.x;
  int c[PER];
  int mine = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) { c[i] = gh[grp * PER + i]; mine += c[i]; }
  int tot;
  const int above = block_exscan_256(mine, sw, &tot);
  if (above < rem && rem <= above + mine) {          // exactly one thread
    int r = rem - above, i = PER - 1;
#pragma unroll
    for (int k = PER - 1; k > 0; --k)
      if (i == k && c[k] < r) { r -= c[k]; i = k - 1; }
    sres[0] = grp * PER + i;
    sres[1] = r;
  }
  __syncthreads();
}

template <int LEVEL>
__global__ __launch_bounds__(256) void v_sel_level_kernel(const float* __restrict__ scores, int T,
                                                          int n_s, SelWs w) {
  constexpr int SHIFT = LEVEL == 0 ? 21 : (LEVEL == 1 ? 10 : 0);
  constexpr int NB = LEVEL == 2 ? 1024 : 2048;
  constexpr uint32_t PMASK = LEVEL == 0 ? 0u : (LEVEL == 1 ? 0xFFE00000u : 0xFFFFFC00u);
  const int b = blockIdx.y, slice = blockIdx.x, tid = threadIdx.x;
  __shared__ int h[SEL_BINS];
  __shared__ int sw[4];
  __shared__ int sres[2];
  for (int i = tid; i < NB; i += 256) h[i] = 0;
  // T is a multiple of 32 and the scores are 16-byte aligned: whole float4 pieces,
  // all requested before anything else
  const float4* sc4 = reinterpret_cast<const float4*>(scores + (size_t)b * T);
  const int p0 = slice * (LV_SLICE / 4), np = T >> 2;
  float4 v[LV_SLICE / 1024];
#pragma unroll
  for (int q = 0; q < LV_SLICE / 1024; ++q) {
    const int p = p0 + q * 256 + tid;
    v[q] = p < np ? sc4[p] : float4{0.f, 0.f, 0.f, 0.f};
  }
  // the previous level's result: scan its histogram (every workgroup, redundantly)
  uint32_t prefix = 0;
  if (LEVEL == 1) {
    find_bin<2048>(w.hist + ((size_t)b * 3 + 0) * SEL_BINS, n_s, sw, sres);
    prefix = (uint32_t)sres[0] << 21;
    if (slice == 0 && tid == 0) { w.st[b * 8 + 0] = (int)prefix; w.st[b * 8 + 1] = sres[1]; }
  } else if (LEVEL == 2) {
    const uint32_t p1 = (uint32_t)w.st[b * 8 + 0];
    find_bin<2048>(w.hist + ((size_t)b * 3 + 1) * SEL_BINS, w.st[b * 8 + 1], sw, sres);
    prefix = p1 | ((uint32_t)sres[0] << 10);
    if (slice == 0 && tid == 0) { w.st[b * 8 + 2] = (int)prefix; w.st[b * 8 + 3] = sres[1]; }
  } else {
    __syncthreads();
  }
#pragma unroll
  for (int q = 0; q < LV_SLICE / 1024; ++q) {
    if (p0 + q * 256 + tid < np) {
      const float x[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t k = fkey(x[j]);
        if ((k & PMASK) == prefix) atomicAdd(&h[(k >> SHIFT) & (NB - 1)], 1);
      }
    }
  }
  __syncthreads();
  int* gh = w.hist + ((size_t)b * 3 + LEVEL) * SEL_BINS;
  for (int i = tid; i < NB; i += 256)
    if (h[i]) atomicAdd(&gh[i], h[i]);
}

// Flags of one 32-token group: bit j set = token selected-or-tied information.
// FROM_MASK = false: sel = key > kth, tie = key == kth.  true: sel = mask bits.
template <bool FROM_MASK>
__device__ __forceinline__ void group_flags(const float* sc, const uint32_t* mk, int g,
                                            uint32_t kth, uint32_t* sel, uint32_t* tie) {
  if (FROM_MASK) {
    *sel = mk[g];
    *tie = 0;
  } else {
    uint32_t s = 0, e = 0;
    const float4* p = reinterpret_cast<const float4*>(sc + (size_t)g * G);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float4 v = p[q];
      const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t k = fkey(x[j]);
        s |= (k > kth) ? (1u << (4 * q + j)) : 0u;
        e |= (k == kth) ? (1u << (4 * q + j)) : 0u;
      }
    }
    *sel = s;
    *tie = e;
  }
}

template <bool FROM_MASK>
__global__ __launch_bounds__(256) void v_sel_count_kernel(const float* __restrict__ scores,
                                                          const uint32_t* __restrict__ mask, int T,
                                                          int ng, int ngc, SelWs w) {
  const int b = blockIdx.y, slice = blockIdx.x, tid = threadIdx.x;
  __shared__ int sw[4];
  __shared__ int sres[2];
  uint32_t kth = 0;
  if (!FROM_MASK) {
    // the last radix level's result: the n_s-th largest key and how many of its ties to take
    const uint32_t p2 = (uint32_t)w.st[b * 8 + 2];
    find_bin<1024>(w.hist + ((size_t)b * 3 + 2) * SEL_BINS, w.st[b * 8 + 3], sw, sres);
    kth = p2 | (uint32_t)sres[0];
    if (slice == 0 && tid == 0) { w.st[b * 8 + 4] = (int)kth; w.st[b * 8 + 5] = sres[1]; }
  }
  const int g = slice * (SEL_SLICE / G) + tid;
  uint32_t sel = 0, tie = 0;
  if (g < ng) group_flags<FROM_MASK>(scores + (size_t)b * T, mask + (size_t)b * ngc, g, kth, &sel, &tie);
  int tot_s, tot_e;
  block_exscan_256(__popc(sel), sw, &tot_s);
  block_exscan_256(__popc(tie), sw, &tot_e);
  if (tid == 0) {
    w.cnt[((size_t)b * w.nslice + slice) * 2 + 0] = tot_s;
    w.cnt[((size_t)b * w.nslice + slice) * 2 + 1] = tot_e;
  }
}

template <bool FROM_MASK>
__global__ __launch_bounds__(256) void v_sel_mark_kernel(const float* __restrict__ scores, int T,
                                                         int ng, int ngc, int n_s, SelWs w,
                                                         int32_t* __restrict__ idx_out,
                                                         uint32_t* __restrict__ mask,
                                                         uint32_t* __restrict__ rank) {
  const int b = blockIdx.y, slice = blockIdx.x, tid = threadIdx.x;
  __shared__ int sw[4];
  const int g = slice * (SEL_SLICE / G) + tid;
  uint32_t sel = 0, tie = 0;
  const uint32_t kth = FROM_MASK ? 0u : (uint32_t)w.st[b * 8 + 4];
  const int take_eq = FROM_MASK ? 0 : w.st[b * 8 + 5];   // tied elements to take, lowest index first
  // selected / tied elements in the slices before mine
  int pre_s = 0, pre_e = 0;
  for (int i0 = 0; i0 < slice; i0 += 256) {
    const int i = i0 + tid;
    const int cs = i < slice ? w.cnt[((size_t)b * w.nslice + i) * 2 + 0] : 0;
    const int ce = i < slice ? w.cnt[((size_t)b * w.nslice + i) * 2 + 1] : 0;
    int ts, te;
    block_exscan_256(cs, sw, &ts);
    block_exscan_256(ce, sw, &te);
    pre_s += ts;
    pre_e += te;
  }
  uint32_t* mk = mask + (size_t)b * ngc;
  if (g < ng) group_flags<FROM_MASK>(scores + (size_t)b * T, mk, g, kth, &sel, &tie);
  int tot;
  // ties: take those whose (global, index-ordered) tie number is below take_eq
  int tie_before = pre_e + block_exscan_256(__popc(tie), sw, &tot);
  uint32_t e = tie;
  while (e) {
    const int j = __ffs(e) - 1;
    e &= e - 1;
    if (tie_before < take_eq) sel |= 1u << j;
    ++tie_before;
  }
  // number of protected tokens before this group: selected-above-kth before
  // the slice + ties taken before the slice + the same inside the slice
  const int ties_before_slice = min(pre_e, take_eq);
  int before = pre_s + (FROM_MASK ? 0 : ties_before_slice) +
               block_exscan_256(__popc(sel), sw, &tot);
  if (g < ng) {
    if (!FROM_MASK) mk[g] = sel;
    rank[(size_t)b * ngc + g] = (uint32_t)before;
    int32_t* io = idx_out + (size_t)b * n_s;
    uint32_t s = sel;
    while (s) {
      const int j = __ffs(s) - 1;
      s &= s - 1;
      if (before < n_s) io[before] = g * G + j;
      ++before;
    }
  }
}

__global__ __launch_bounds__(256) void v_sel_scatter_kernel(const int32_t* __restrict__ idx_in,
                                                            int n_s, int ng, int ngc,
                                                            uint32_t* __restrict__ mask) {
  const int b = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_s) {
    const int t = idx_in[(size_t)b * n_s + i];
    if (t >= 0 && t < ng * G)                       // an index outside the cache is ignored
      atomicOr(&mask[(size_t)b * ngc + (t >> 5)], 1u << (t & 31));
  }
}

// The ternary coding pass (Eq. 6) lives in quant_values_enc.hip.
void launch_v_encode(const Geom& g, const EncodeSpan& sp, int n_s, float gamma, const void* V,
                     uint8_t* packed, hipStream_t st);

// Alg. 2, STPQuant, protected branch: the protected rows of one head, gathered
// in token order, coded with Eq. 4 at 2 bits per channel over groups of 32
// protected tokens (the last group may hold fewer).  grid (npg, nheads), block
// 128: thread = channel.  Record: codes [32 rows][32 bytes] (channel 4 j + r of
// a row in bits 2r.. of byte j), fp16 s[128], fp16 z[128].
__global__ __launch_bounds__(128) void v_protect2_kernel(const _Float16* __restrict__ V, int T,
                                                         int B, int H, int n_s, int npg,
                                                         const int32_t* __restrict__ idx,
                                                         uint8_t* __restrict__ out) {
  const int pg = blockIdx.x, c = threadIdx.x;
  const long long hd = blockIdx.y;
  const int b = (int)((hd / H) % B);
  const int cnt = min(G, n_s - pg * G);
  __shared__ int tok[G];
  __shared__ uint8_t code_s[G][D];
  // rows beyond the last one repeat it: every load is valid and changes neither min nor max
  // (an index list with repeated or out-of-range entries leaves the end of IDX unwritten:
  // whatever is there is clamped into the tensor, such rows are never read back)
  if (c < G) tok[c] = min(max(idx[(size_t)b * n_s + pg * G + min(c, cnt - 1)], 0), T - 1);
  __syncthreads();
  const _Float16* head = V + hd * (long long)T * D;
  _Float16 xh[G];
#pragma unroll
  for (int r = 0; r < G; ++r) xh[r] = head[(size_t)tok[r] * D + c];
  float x[G];
  float lo = 65504.0f, hi = -65504.0f;
#pragma unroll
  for (int r = 0; r < G; ++r) {
    x[r] = (float)xh[r];
    lo = fminf(lo, x[r]);
    hi = fmaxf(hi, x[r]);
  }
  const float rng = hi - lo;
  const float inv = rng > 0.0f ? 3.0f / rng : 0.0f;
#pragma unroll
  for (int r = 0; r < G; ++r) {
    float u = (x[r] - lo) * inv;
    u = fminf(fmaxf(rintf(u), 0.0f), 3.0f);
    code_s[r][c] = r < cnt ? (uint8_t)u : (uint8_t)0;
  }
  uint8_t* rec = out + (hd * npg + pg) * (long long)PREC;
  reinterpret_cast<_Float16*>(rec + 1024)[c] = (_Float16)(rng / 3.0f);
  reinterpret_cast<_Float16*>(rec + 1280)[c] = (_Float16)lo;
  __syncthreads();
  // 256 dwords of codes: dword w = row w / 8, channels 16 (w % 8) ..
  for (int w = c; w < 256; w += 128) {
    const int r = w >> 3, c0 = 16 * (w & 7);
    uint32_t v = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) v |= (uint32_t)code_s[r][c0 + k] << (2 * k);
    reinterpret_cast<uint32_t*>(rec)[w] = v;
  }
}

// MASK and RANK of groups appended behind the prefill tokens: none of their
// tokens is protected, all n_s protected tokens lie before them.
__global__ __launch_bounds__(256) void v_flush_marks_kernel(uint32_t* __restrict__ mask,
                                                            uint32_t* __restrict__ rank, int B,
                                                            int ngc, int g0, int n, uint32_t n_s) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < B * n) {
    const size_t at = (size_t)(i / n) * ngc + g0 + (i % n);
    mask[at] = 0;
    rank[at] = n_s;
  }
}

void launch_flush_marks(const Geom& g, int n_groups, uint8_t* packed, hipStream_t st) {
  if (g.n_s == 0) return;
  const int n = g.B * n_groups;
  hipLaunchKernelGGL(v_flush_marks_kernel, dim3((n + 255) / 256), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(packed + g.v_mask),
                     reinterpret_cast<uint32_t*>(packed + g.v_rank), g.B, g.ngc, g.ng, n_groups,
                     (uint32_t)g.n_s);
}

size_t values_ws_bytes(const Geom& g) {
  const int nslice = (g.T + SEL_SLICE - 1) / SEL_SLICE;
  return align256(sel_ws_ints(g.B, nslice > 0 ? nslice : 1) * sizeof(int)) + 256;
}

hipError_t launch_quantize_values(const Geom& g, float gamma, const void* V, const float* scores,
                                  const int32_t* idx, uint8_t* packed, void* ws,
                                  unsigned stages, hipStream_t st) {
  if (g.T == 0) return hipSuccess;
  uint32_t* mask = reinterpret_cast<uint32_t*>(packed + g.v_mask);
  uint32_t* rank = reinterpret_cast<uint32_t*>(packed + g.v_rank);
  // stages: bit 0 protected-token selection, bit 1 coding pass
  if (g.n_s > 0 && (stages & 1u)) {
    const int nslice = (g.T + SEL_SLICE - 1) / SEL_SLICE;
    SelWs w = sel_ws(ws, g.B, nslice);
    const size_t n_hist = (size_t)g.B * 3 * SEL_BINS;
    const size_t n_mask = (size_t)g.B * g.ngc;
    const size_t n_init = scores ? n_hist : n_mask;
    int32_t* idx_out = reinterpret_cast<int32_t*>(packed + g.v_idx);
    dim3 gs(nslice, g.B);
    hipLaunchKernelGGL(v_sel_init_kernel, dim3((unsigned)((n_init + 255) / 256)), dim3(256), 0, st,
                       w.hist, scores ? n_hist : 0, scores ? nullptr : mask, n_mask);
    if (scores) {
      dim3 gl((g.T + LV_SLICE - 1) / LV_SLICE, g.B);
      hipLaunchKernelGGL(v_sel_level_kernel<0>, gl, dim3(256), 0, st, scores, g.T, g.n_s, w);
      hipLaunchKernelGGL(v_sel_level_kernel<1>, gl, dim3(256), 0, st, scores, g.T, g.n_s, w);
      hipLaunchKernelGGL(v_sel_level_kernel<2>, gl, dim3(256), 0, st, scores, g.T, g.n_s, w);
      hipLaunchKernelGGL(v_sel_count_kernel<false>, gs, dim3(256), 0, st, scores, mask, g.T, g.ng, g.ngc, w);
      hipLaunchKernelGGL(v_sel_mark_kernel<false>, gs, dim3(256), 0, st, scores, g.T, g.ng, g.ngc, g.n_s,
                         w, idx_out, mask, rank);
    } else {
      hipLaunchKernelGGL(v_sel_scatter_kernel, dim3((g.n_s + 255) / 256, g.B), dim3(256), 0, st,
                         idx, g.n_s, g.ng, g.ngc, mask);
      hipLaunchKernelGGL(v_sel_count_kernel<true>, gs, dim3(256), 0, st, scores, mask, g.T, g.ng, g.ngc, w);
      hipLaunchKernelGGL(v_sel_mark_kernel<true>, gs, dim3(256), 0, st, scores, g.T, g.ng, g.ngc, g.n_s, w,
                         idx_out, mask, rank);
    }
  }
  if (stages & 2u) {
    launch_v_encode(g, EncodeSpan{g.T, g.ng, 0, g.nheads, 0}, g.n_s, gamma, V, packed, st);
    if (g.n_s > 0 && g.sal_bits == 2)
      hipLaunchKernelGGL(v_protect2_kernel, dim3(g.npg, (unsigned)g.nheads), dim3(128), 0, st,
                         reinterpret_cast<const _Float16*>(V), g.T, g.B, g.H, g.n_s, g.npg,
                         reinterpret_cast<const int32_t*>(packed + g.v_idx), packed + g.v_rows);
  }
  return hipGetLastError();
}

}  // namespace vidkv
