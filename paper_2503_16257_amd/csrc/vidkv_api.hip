// C ABI of the VidKV library: argument validation on the host, then kernel
// launches on the caller's stream (and, for two calls, on a second stream that the
// caller hands in).  Nothing here allocates, synchronizes, or creates streams or events.
#include <mutex>

#include "vidkv_common.h"

namespace vidkv {
hipError_t launch_quantize_keys(const Geom& g, const void* K, uint8_t* packed, void* ws,
                                unsigned stages, hipStream_t st);
hipError_t launch_quantize_values(const Geom& g, float gamma, const void* V, const float* scores,
                                  const int32_t* idx, uint8_t* packed, void* ws,
                                  unsigned stages, hipStream_t st);
size_t values_ws_bytes(const Geom& g);
hipError_t launch_decode_attention(const Geom& g, int layer, float scale, const void* q,
                                   const uint8_t* pk, const uint8_t* pv, const void* ktail,
                                   const void* vtail, int cap, const int32_t* tail_len, void* out,
                                   void* ws, unsigned stages, hipStream_t st, hipStream_t side,
                                   hipEvent_t fork, hipEvent_t join);
bool attn_tail_beside(const Geom& g, int cap);
int attn_num_splits(const Geom& g);
void launch_k_encode(const Geom& g, const EncodeSpan& sp, const void* K, uint8_t* packed,
                     bool use_fft, hipStream_t st);
void launch_v_encode(const Geom& g, const EncodeSpan& sp, int n_s, float gamma, const void* V,
                     uint8_t* packed, hipStream_t st);
void launch_flush_marks(const Geom& g, int n_groups, uint8_t* packed, hipStream_t st);
hipError_t launch_saliency(const void* Xv, const void* Xt, int B, int Tv, int Nt, int d,
                           float* scores, float* tsum, hipStream_t st);

static size_t ws_keys(const Geom& g) {
  if (g.metric != 0)     // float64 partials and thresholds of the variance / outlier metrics
    return align256(((size_t)g.nheads * g.range_chunks * 2 + (size_t)g.nheads) * D * sizeof(double)) + 256;
  return align256((size_t)g.nheads * g.range_chunks * 2 * D * sizeof(_Float16)) + 256;
}
static size_t ws_values(const Geom& g) { return values_ws_bytes(g); }
static size_t ws_attn(const Geom& g) {
  // sized for the capacity, so that a workspace allocated once stays large enough
  // while residual flushes make the packed cache longer
  Geom c = g;
  c.T = g.Tcap;
  c.ng = g.ngc;
  const int ns = attn_num_splits(c) > attn_num_splits(g) ? attn_num_splits(c) : attn_num_splits(g);
  return align256((size_t)(ns + ATTN_TAIL_SPLITS) * g.B * g.Hq * (D + 2) * sizeof(float)) + 256;
}
static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

__global__ __launch_bounds__(256) void calib_copy_kernel(const u32x4* __restrict__ src,
                                                         u32x4* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k, i += 256)
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
}  // namespace vidkv

using namespace vidkv;

namespace {
constexpr int MAX_DEVICES = 64;

// The caller's side stream and events, or nothing.  All three handles must be there.
struct Side {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  bool ok = false;
};
Side take_side(const vidkv_side_stream* s) {
  Side r;
  if (s && s->hip_stream && s->fork_event && s->join_event) {
    r.stream = static_cast<hipStream_t>(s->hip_stream);
    r.fork = static_cast<hipEvent_t>(s->fork_event);
    r.join = static_cast<hipEvent_t>(s->join_event);
    r.ok = true;
  }
  return r;
}
bool side_malformed(const vidkv_side_stream* s) {
  return s && !(s->hip_stream && s->fork_event && s->join_event);
}

// A stream of another device than the current one cannot take this call's launches.
// (The NULL stream belongs to the current device.  If the runtime cannot tell, go on.)
bool stream_on_current_device(hipStream_t st) {
  if (!st) return true;
  int cur = 0, dev = 0;
  if (hipGetDevice(&cur) != hipSuccess || hipStreamGetDevice(st, &dev) != hipSuccess) {
    (void)hipGetLastError();
    return true;
  }
  return cur == dev;
}
}  // namespace

extern "C" {

size_t vidkv_packed_keys_bytes(const vidkv_params* p) {
  Geom g;
  return make_geom(p, &g) ? g.k_total : 0;
}

size_t vidkv_packed_values_bytes(const vidkv_params* p) {
  Geom g;
  return make_geom(p, &g) ? g.v_total : 0;
}

size_t vidkv_workspace_bytes(const vidkv_params* p, int which) {
  Geom g;
  if (!make_geom(p, &g)) return 0;
  switch (which) {
    case 0: return ws_keys(g);
    case 1: return ws_values(g);
    case 2: return ws_attn(g);
    case 3: return ws_keys(g) + ws_values(g);
    default: return 0;
  }
}

vidkv_status vidkv_quantize_keys_stages(const vidkv_params* p, const void* K, void* packed,
                                        size_t packed_bytes, void* ws, size_t ws_bytes,
                                        uint32_t stages, void* stream) {
  Geom g;
  if (!p || !packed || !ws) return VIDKV_EINVAL;
  if (!make_geom(p, &g)) return VIDKV_ESHAPE;
  if (g.T > 0 && !K) return VIDKV_EINVAL;
  if (g.nheads > 65535) return VIDKV_ESHAPE;
  if (!aligned(K, 16) || !aligned(packed, 256) || !aligned(ws, 256)) return VIDKV_EINVAL;
  if (packed_bytes < g.k_total || ws_bytes < ws_keys(g)) return VIDKV_ENOSPACE;
  const hipError_t e = launch_quantize_keys(g, K, static_cast<uint8_t*>(packed), ws, stages,
                                            static_cast<hipStream_t>(stream));
  return e == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

vidkv_status vidkv_quantize_keys(const vidkv_params* p, const void* K, void* packed,
                                 size_t packed_bytes, void* ws, size_t ws_bytes, void* stream) {
  return vidkv_quantize_keys_stages(p, K, packed, packed_bytes, ws, ws_bytes, ~0u, stream);
}

vidkv_status vidkv_quantize_values_stages(const vidkv_params* p, const void* V,
                                          const float* saliency, const int32_t* salient_idx,
                                          void* packed, size_t packed_bytes, void* ws,
                                          size_t ws_bytes, uint32_t stages, void* stream) {
  Geom g;
  if (!p || !packed || !ws) return VIDKV_EINVAL;
  if (!make_geom(p, &g)) return VIDKV_ESHAPE;
  if (g.T > 0 && !V) return VIDKV_EINVAL;
  if (g.nheads > 65535) return VIDKV_ESHAPE;
  if (g.n_s > 0 && ((saliency != nullptr) == (salient_idx != nullptr))) return VIDKV_EINVAL;
  if (!(p->gamma >= 0.0f) || !(p->gamma < 1e30f)) return VIDKV_EINVAL;
  if (!aligned(V, 16) || !aligned(packed, 256) || !aligned(ws, 256) || !aligned(saliency, 16) ||
      !aligned(salient_idx, 4))
    return VIDKV_EINVAL;
  if (packed_bytes < g.v_total || ws_bytes < ws_values(g)) return VIDKV_ENOSPACE;
  const hipError_t e =
      launch_quantize_values(g, p->gamma, V, g.n_s > 0 ? saliency : nullptr,
                             g.n_s > 0 ? salient_idx : nullptr, static_cast<uint8_t*>(packed), ws,
                             stages, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

vidkv_status vidkv_quantize_values(const vidkv_params* p, const void* V, const float* saliency,
                                   const int32_t* salient_idx, void* packed, size_t packed_bytes,
                                   void* ws, size_t ws_bytes, void* stream) {
  return vidkv_quantize_values_stages(p, V, saliency, salient_idx, packed, packed_bytes, ws,
                                      ws_bytes, ~0u, stream);
}

vidkv_status vidkv_quantize_kv(const vidkv_params* p, const void* K, const void* V,
                               const float* saliency, const int32_t* salient_idx, void* packed_K,
                               size_t packed_K_bytes, void* packed_V, size_t packed_V_bytes,
                               void* ws, size_t ws_bytes, void* stream,
                               const vidkv_side_stream* side) {
  Geom g;
  if (!p || !packed_K || !packed_V || !ws || side_malformed(side)) return VIDKV_EINVAL;
  if (!make_geom(p, &g)) return VIDKV_ESHAPE;
  if (g.T > 0 && (!K || !V)) return VIDKV_EINVAL;
  if (g.nheads > 65535) return VIDKV_ESHAPE;
  if (g.n_s > 0 && ((saliency != nullptr) == (salient_idx != nullptr))) return VIDKV_EINVAL;
  if (!(p->gamma >= 0.0f) || !(p->gamma < 1e30f)) return VIDKV_EINVAL;
  if (!aligned(K, 16) || !aligned(V, 16) || !aligned(packed_K, 256) || !aligned(packed_V, 256) ||
      !aligned(ws, 256) || !aligned(saliency, 16) || !aligned(salient_idx, 4))
    return VIDKV_EINVAL;
  if (packed_K_bytes < g.k_total || packed_V_bytes < g.v_total) return VIDKV_ENOSPACE;
  if (ws_bytes < ws_keys(g) + ws_values(g)) return VIDKV_ENOSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* pk = static_cast<uint8_t*>(packed_K);
  uint8_t* pv = static_cast<uint8_t*>(packed_V);
  void* ws_k = ws;
  void* ws_v = static_cast<uint8_t*>(ws) + ws_keys(g);
  const float* sc = g.n_s > 0 ? saliency : nullptr;
  const int32_t* ix = g.n_s > 0 ? salient_idx : nullptr;
  if (!stream_on_current_device(st)) return VIDKV_EINVAL;
  // The chain of short dependent launches that selects the protected tokens runs on the side
  // stream beside the bandwidth-bound key passes.  The fork and join cost about as much as
  // three short launches, so this pays only when the key passes are long enough to hide the
  // chain behind them.  (Moving the channel selection over as well, beside the value coding
  // pass, was measured and lost: its four large workgroups wait for free compute units until
  // the coding pass has been dispatched, and the second fork and join come on top.)
  const Side sd = take_side(side);
  const bool fork = sd.ok && (size_t)g.nheads * g.T * D * 2 >= ((size_t)32 << 20);
  if (g.n_s > 0 && g.T > 0 && fork) {
    if (!stream_on_current_device(sd.stream)) return VIDKV_EINVAL;
    if (hipEventRecord(sd.fork, st) != hipSuccess) return VIDKV_EHIP;
    if (hipStreamWaitEvent(sd.stream, sd.fork, 0) != hipSuccess) return VIDKV_EHIP;
    // from here on the side stream depends on `st`: whatever fails, it is joined back, so
    // that a stream capture on `st` can still be ended
    bool good = launch_quantize_values(g, p->gamma, V, sc, ix, pv, ws_v, 1u, sd.stream) == hipSuccess;
    good = (hipEventRecord(sd.join, sd.stream) == hipSuccess) && good;
    good = good && launch_quantize_keys(g, K, pk, ws_k, ~0u, st) == hipSuccess;
    good = (hipStreamWaitEvent(st, sd.join, 0) == hipSuccess) && good;
    if (!good) return VIDKV_EHIP;
    return launch_quantize_values(g, p->gamma, V, sc, ix, pv, ws_v, 2u, st) == hipSuccess
               ? VIDKV_OK : VIDKV_EHIP;
  }
  if (launch_quantize_keys(g, K, pk, ws_k, ~0u, st) != hipSuccess) return VIDKV_EHIP;
  return launch_quantize_values(g, p->gamma, V, sc, ix, pv, ws_v, ~0u, st) == hipSuccess
             ? VIDKV_OK : VIDKV_EHIP;
}

// Argument checks of a decode step, shared by the entry points below.
static vidkv_status check_decode(const vidkv_params* p, Geom* g, int32_t layer, const void* q,
                                 const void* packed_K, const void* packed_V, const void* K_tail,
                                 const void* V_tail, int32_t tail_capacity,
                                 const int32_t* tail_len, const void* out) {
  if (!p || !q || !out) return VIDKV_EINVAL;
  if (!make_geom(p, g)) return VIDKV_ESHAPE;
  if (layer < 0 || layer >= g->L) return VIDKV_EINVAL;
  if (g->T > 0 && (!packed_K || !packed_V)) return VIDKV_EINVAL;
  if (tail_capacity < 0) return VIDKV_EINVAL;
  if (tail_capacity > 0 && tail_len && (!K_tail || !V_tail)) return VIDKV_EINVAL;
  if (g->B > 65535 || g->H > 65535) return VIDKV_ESHAPE;
  if (!(p->softmax_scale > 0.0f) || !(p->softmax_scale < 1e30f)) return VIDKV_EINVAL;
  if (!aligned(q, 16) || !aligned(out, 16) || !aligned(packed_K, 256) || !aligned(packed_V, 256) ||
      !aligned(K_tail, 16) || !aligned(V_tail, 16) || !aligned(tail_len, 4))
    return VIDKV_EINVAL;
  return VIDKV_OK;
}

vidkv_status vidkv_decode_attention_stages(const vidkv_params* p, int32_t layer, const void* q,
                                           const void* packed_K, const void* packed_V,
                                           const void* K_tail, const void* V_tail,
                                           int32_t tail_capacity, const int32_t* tail_len,
                                           void* out, void* ws, size_t ws_bytes, uint32_t stages,
                                           void* stream, const vidkv_side_stream* side) {
  Geom g;
  if (!ws || side_malformed(side)) return VIDKV_EINVAL;
  const vidkv_status chk = check_decode(p, &g, layer, q, packed_K, packed_V, K_tail, V_tail,
                                        tail_capacity, tail_len, out);
  if (chk != VIDKV_OK) return chk;
  if (!aligned(ws, 256)) return VIDKV_EINVAL;
  if (ws_bytes < ws_attn(g)) return VIDKV_ENOSPACE;
  const uint8_t* pk = static_cast<const uint8_t*>(packed_K);
  const uint8_t* pv = static_cast<const uint8_t*>(packed_V);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!stream_on_current_device(st)) return VIDKV_EINVAL;
  const Side sd = take_side(side);
  if (sd.ok && K_tail && V_tail && tail_len && (stages & 1u) && attn_tail_beside(g, tail_capacity)) {
    if (!stream_on_current_device(sd.stream)) return VIDKV_EINVAL;
    return launch_decode_attention(g, layer, p->softmax_scale, q, pk, pv, K_tail, V_tail,
                                   tail_capacity, tail_len, out, ws, stages, st, sd.stream,
                                   sd.fork, sd.join) == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
  }
  const hipError_t e = launch_decode_attention(g, layer, p->softmax_scale, q, pk, pv, K_tail, V_tail,
                                               tail_capacity, tail_len, out, ws, stages, st,
                                               nullptr, nullptr, nullptr);
  return e == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

vidkv_status vidkv_decode_attention(const vidkv_params* p, int32_t layer, const void* q,
                                    const void* packed_K, const void* packed_V, const void* K_tail,
                                    const void* V_tail, int32_t tail_capacity,
                                    const int32_t* tail_len, void* out, void* ws, size_t ws_bytes,
                                    void* stream, const vidkv_side_stream* side) {
  return vidkv_decode_attention_stages(p, layer, q, packed_K, packed_V, K_tail, V_tail,
                                       tail_capacity, tail_len, out, ws, ws_bytes, ~0u, stream, side);
}

}  // extern "C"

// ---- decode step for callers that cannot allocate -------------------------------------------
// The split partials of a decode step (o, m, l per split, sequence and query head) are the one
// scratch buffer of the decode path.  Here they live in a device array that is part of the
// library's image: every GPU that runs the library holds its own copy, at its own address,
// until the process ends.  The array's name is only a handle on the host; its device address
// is looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[VIDKV_NOALLOC_SCRATCH_BYTES];

namespace {
void* g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

// device address of `scratch` on the current device; nullptr on failure
void* scratch_on_current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

vidkv_status vidkv_decode_attention_noalloc(const vidkv_params* p, int32_t layer, const void* q,
                                            const void* packed_K, const void* packed_V,
                                            const void* K_tail, const void* V_tail,
                                            int32_t tail_capacity, const int32_t* tail_len,
                                            void* out, void* stream) {
  Geom g;
  const vidkv_status chk = check_decode(p, &g, layer, q, packed_K, packed_V, K_tail, V_tail,
                                        tail_capacity, tail_len, out);
  if (chk != VIDKV_OK) return chk;
  if (ws_attn(g) > (size_t)VIDKV_NOALLOC_SCRATCH_BYTES) return VIDKV_ENOSPACE;
  void* ws = scratch_on_current_device();
  if (!ws) return VIDKV_EHIP;
  if (!stream_on_current_device(static_cast<hipStream_t>(stream))) return VIDKV_EINVAL;
  // Everything runs in line on the caller's stream.  Nothing in the array has to start at zero: the merge reads
  // only the parts that this call's kernels wrote before it.
  const hipError_t e = launch_decode_attention(
      g, layer, p->softmax_scale, q, static_cast<const uint8_t*>(packed_K),
      static_cast<const uint8_t*>(packed_V), K_tail, V_tail, tail_capacity, tail_len, out, ws, ~0u,
      static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr);
  return e == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

vidkv_status vidkv_flush_residual(const vidkv_params* p, int32_t layer, const void* K_tail,
                                  const void* V_tail, int32_t tail_capacity, int32_t n_flush,
                                  void* packed_K, size_t packed_K_bytes, void* packed_V,
                                  size_t packed_V_bytes, void* stream) {
  Geom g;
  if (!p || !K_tail || !V_tail || !packed_K || !packed_V) return VIDKV_EINVAL;
  if (!make_geom(p, &g)) return VIDKV_ESHAPE;
  if (layer < 0 || layer >= g.L) return VIDKV_EINVAL;
  if (n_flush <= 0 || n_flush % G || tail_capacity < n_flush) return VIDKV_EINVAL;
  if (g.T == 0) return VIDKV_EINVAL;               // no channel selection to code the keys with
  if (!(p->gamma >= 0.0f) || !(p->gamma < 1e30f)) return VIDKV_EINVAL;
  if ((long long)g.B * g.H > 65535) return VIDKV_ESHAPE;
  if (!aligned(K_tail, 16) || !aligned(V_tail, 16) || !aligned(packed_K, 256) ||
      !aligned(packed_V, 256))
    return VIDKV_EINVAL;
  if (g.T + n_flush > g.Tcap) return VIDKV_ENOSPACE;
  if (packed_K_bytes < g.k_total || packed_V_bytes < g.v_total) return VIDKV_ENOSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long long bh = (long long)g.B * g.H;
  const EncodeSpan sp{tail_capacity, n_flush / G, g.ng, bh, layer * bh};
  launch_k_encode(g, sp, K_tail, static_cast<uint8_t*>(packed_K), g.use_fft, st);
  launch_v_encode(g, sp, 0, p->gamma, V_tail, static_cast<uint8_t*>(packed_V), st);
  launch_flush_marks(g, sp.ng, static_cast<uint8_t*>(packed_V), st);
  return hipGetLastError() == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

size_t vidkv_saliency_workspace_bytes(int32_t batch, int32_t hidden_dim) {
  if (batch < 1 || hidden_dim < 8) return 0;
  return align256((size_t)batch * hidden_dim * sizeof(float));
}

vidkv_status vidkv_saliency_scores(const void* X_v, const void* X_t, int32_t batch,
                                   int32_t n_visual, int32_t n_text, int32_t hidden_dim,
                                   float* scores, void* ws, size_t ws_bytes, void* stream) {
  if (!X_t || !ws) return VIDKV_EINVAL;
  if (batch < 1 || n_visual < 0 || n_text < 1) return VIDKV_EINVAL;
  if (n_visual > 0 && (!X_v || !scores)) return VIDKV_EINVAL;
  if (hidden_dim < 8 || hidden_dim % 8 || hidden_dim > 16384 || batch > 65535) return VIDKV_ESHAPE;
  if (!aligned(X_v, 16) || !aligned(X_t, 2) || !aligned(scores, 4) || !aligned(ws, 256))
    return VIDKV_EINVAL;
  if (ws_bytes < vidkv_saliency_workspace_bytes(batch, hidden_dim)) return VIDKV_ENOSPACE;
  const hipError_t e = launch_saliency(X_v, X_t, batch, n_visual, n_text, hidden_dim, scores,
                                       static_cast<float*>(ws), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

vidkv_status vidkv_calib_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return VIDKV_EINVAL;
  if (bytes % 16 || !aligned(dst, 16) || !aligned(src, 16)) return VIDKV_EINVAL;
  if (bytes == 0) return VIDKV_OK;
  const size_t n = bytes / 16;
  const size_t blocks = (n + 1023) / 1024;
  if (blocks > 0x7fffffffull) return VIDKV_ESHAPE;
  hipLaunchKernelGGL(calib_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst), n);
  return hipGetLastError() == hipSuccess ? VIDKV_OK : VIDKV_EHIP;
}

const char* vidkv_status_string(vidkv_status s) {
  switch (s) {
    case VIDKV_OK: return "ok";
    case VIDKV_EINVAL: return "invalid argument";
    case VIDKV_ESHAPE: return "unsupported shape";
    case VIDKV_ENOSPACE: return "buffer too small";
    case VIDKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int vidkv_abi_version(void) { return VIDKV_ABI_VERSION; }

}  // extern "C"
