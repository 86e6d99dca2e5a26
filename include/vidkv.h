/*
 * vidkv.h - C ABI of the MI355X (gfx950) VidKV hot path:
 *   sub-2-bit KV-cache codec + single-query GQA decode attention over the
 *   packed cache.
 *
 * Method (arXiv 2503.16257): keys are quantized per channel with mixed
 * precision - the n_anom channels of largest range get the 2-bit uniform
 * group quantizer (Eq. 4), the rest get the FFT-based 1-bit quantizer (Eq. 5;
 * Alg. 3); values get the per-channel ternary quantizer (Eq. 6; Alg. 2) with
 * the most salient visual tokens (Sec. 3.3 (2)) preserved, here in fp16; one
 * decode step computes Softmax(q K^T / sqrt(D)) V over the dequantized cache
 * followed by the fp16 residual tokens (Eq. 3; Alg. 1, Decoding).
 *
 * General rules
 *  - Every pointer named *_dev is DEVICE memory on the current HIP device;
 *    `params` is HOST memory.  The caller owns every buffer; the library
 *    allocates no memory, keeps no pointer after a call returns and never
 *    synchronizes: all work is enqueued on `hip_stream` (a hipStream_t passed
 *    as void*, NULL = the default stream), which must belong to the current
 *    device (else VIDKV_EINVAL).  The library creates no stream and no event
 *    and keeps no state between calls (the one exception is the device array
 *    of vidkv_decode_attention_noalloc).  vidkv_quantize_kv and
 *    vidkv_decode_attention can run part of a large call beside the rest on a
 *    second stream that the caller hands in (vidkv_side_stream below); without
 *    one, everything runs in line on `hip_stream`.
 *  - All arguments are checked on the host before anything is launched; a
 *    failed check returns a status and launches nothing.  A launch failure
 *    returns VIDKV_EHIP.  Nothing aborts or throws across this boundary.
 *  - Tensors are dense, row-major, fp16 (IEEE binary16) unless stated.
 *    Inputs must be finite; non-finite inputs give unspecified codes.  All
 *    stored scales are fp16: a 32-token group of keys whose mean spectral
 *    magnitude (Eq. 5) exceeds 65504 - values of order 10^4 with a common
 *    sign - overflows its scale, with unspecified results for that group.
 *  - Shapes: L = n_layers, B = batch, Hkv = n_kv_heads, Hq = n_q_heads
 *    (Hq % Hkv == 0, Hq / Hkv <= 8; query head h reads KV head h / (Hq/Hkv)),
 *    D = head_dim = 128, G = group = 32, Tq = t_quant (multiple of 32).
 *    One quantize call covers at most 65535 (layer, sequence, KV head)
 *    triples, one decode or flush call at most 65535 sequences (and
 *    sequences x KV heads for a flush); larger shapes return VIDKV_ESHAPE
 *    and are to be split by the caller, e.g. one set of packed buffers (and
 *    one params with n_layers = 1) per layer.
 *  - The byte sizes of the packed buffers come from the vidkv_packed_*_bytes
 *    functions; their layout - every section, record, bit and byte order - is
 *    written down in LAYOUT.md beside this header, and is part of the ABI
 *    version.  Packed buffers and workspaces must
 *    be 256-byte aligned; fp16 tensors and the saliency scores 16-byte
 *    aligned; int32 arrays 4-byte aligned (else VIDKV_EINVAL).
 *  - A workspace is scratch: undefined contents on entry and exit, not to be
 *    shared by calls that may run at the same time.
 */
#ifndef VIDKV_H
#define VIDKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VIDKV_ABI_VERSION 3

typedef enum {
  VIDKV_OK = 0,
  VIDKV_EINVAL = 1,   /* NULL pointer, bad enum, inconsistent arguments        */
  VIDKV_ESHAPE = 2,   /* a dimension this build does not support               */
  VIDKV_ENOSPACE = 3, /* an output or workspace buffer is too small            */
  VIDKV_EHIP = 4      /* the HIP runtime reported an error at launch           */
} vidkv_status;

/* Hyper-parameters of Alg. 1-3 (G, k, p, gamma) and the cache geometry.
 * Plain data, passed by pointer from host memory, never retained. */
typedef struct vidkv_params {
  int32_t n_layers;      /* L  >= 1                                             */
  int32_t batch;         /* B  >= 1                                             */
  int32_t n_kv_heads;    /* Hkv >= 1                                            */
  int32_t n_q_heads;     /* Hq, multiple of Hkv, Hq/Hkv <= 8                    */
  int32_t head_dim;      /* must be 128                                         */
  int32_t group;         /* G, must be 32 (Sec. 4.1)                            */
  int32_t t_quant;       /* Tq >= 0, multiple of 32: tokens held in packed form */
  int32_t n_anom;        /* 2-bit key channels per head: 0..128, multiple of 8
                            (k * D of Sec. 3.2 (1))                             */
  int32_t use_fft;       /* normal key channels: 1 = FFT-based 1-bit quantizer
                            (Eq. 5), 0 = Eq. 4 at 1 bit on the tokens themselves
                            (the paper's "standard" 1-bit, Sec. 4.1)            */
  int32_t n_salient;     /* protected value tokens per sequence, 0..Tq
                            (n = p * l_v of Sec. 3.3 (2))                       */
  float gamma;           /* ternary threshold factor of Eq. 6 (paper: 0.7)      */
  float softmax_scale;   /* multiplies q.k before the softmax (1/sqrt(128))     */
  int32_t t_capacity;    /* 0: same as t_quant.  Otherwise >= t_quant, multiple
                            of 32: the packed buffers are laid out (and sized)
                            for this many tokens so that vidkv_flush_residual
                            can append blocks in place; every call on the same
                            buffers must pass the same t_capacity              */
  int32_t salient_bits;  /* how the protected value tokens are kept.  0 or 16:
                            verbatim fp16 rows.  2: Alg. 2's STPQuant - the
                            protected rows of a head, gathered in token order,
                            are coded with Eq. 4 at 2 bits per channel over
                            groups of 32 protected tokens (the last group may
                            be shorter)                                        */
  int32_t channel_metric; /* how Alg. 3 ranks the key channels (Sec. 3.2 (1)):
                            0 Range max - min (what the paper adopts), 1
                            Variance, 2 number of Outliers |x| > 3 mean|x|;
                            1 and 2 are the paper's ablation, in float64       */
} vidkv_params;

/* A second stream for the calls that can use one, with the two events that
 * fork it from and join it back into `hip_stream`.  All three are created and
 * owned by the caller, on the device of `hip_stream`, at the default stream
 * priority; the events may have timing disabled.  The call records fork_event
 * on `hip_stream`, lets the side stream wait for it, enqueues part of its work
 * there, records join_event on the side stream and lets `hip_stream` wait for
 * it before anything that depends on that work: to the caller everything
 * stays ordered on `hip_stream`, also under stream capture (the side stream
 * joins the capture and leaves it again within the call).  Once the fork has
 * been recorded the join is enqueued even if a later launch fails.  One such
 * triple serves any number of calls that are enqueued one after another;
 * calls that may be enqueued at the same time from different host threads need
 * one each.  Passing NULL (or using an entry point without the argument)
 * keeps all work in line on `hip_stream`. */
typedef struct vidkv_side_stream {
  void *hip_stream; /* hipStream_t, not the stream the call is enqueued on */
  void *fork_event; /* hipEvent_t */
  void *join_event; /* hipEvent_t */
} vidkv_side_stream;

/* Size queries: pure host functions, usable without a GPU.  Return 0 when
 * `params` is NULL or invalid.  `which`: 0 = quantize_keys, 1 = quantize_values,
 * 2 = decode_attention, 3 = quantize_kv. */
size_t vidkv_packed_keys_bytes(const vidkv_params *params);
size_t vidkv_packed_values_bytes(const vidkv_params *params);
size_t vidkv_workspace_bytes(const vidkv_params *params, int which);

/* Alg. 3 (MixQuant): per (layer, sequence, KV head) rank the 128 channels by
 * range max-min over all Tq tokens (ties: lower channel first), code the top
 * n_anom channels with Eq. 4 at 2 bits (z = min, s = (max-min)/3 per channel
 * and 32-token group, round-half-even) and the others with Eq. 5: a 32-point
 * DFT along the tokens of each group, one sign bit for each of the 17 real and
 * 15 imaginary independent coefficients, and the mean |Re|, mean |Im| over the
 * 32 bins as fp16 scales.  `channel_metric` and `use_fft` in the parameters
 * select the paper's other ranking metrics and its non-FFT 1-bit code.
 *   K_dev        in : [L, B, Hkv, Tq, 128] fp16
 *   packed_K_dev out: >= vidkv_packed_keys_bytes(params) bytes
 *   workspace_dev   : >= vidkv_workspace_bytes(params, 0) bytes, scratch     */
vidkv_status vidkv_quantize_keys(const vidkv_params *params, const void *K_dev,
                                 void *packed_K_dev, size_t packed_bytes,
                                 void *workspace_dev, size_t workspace_bytes,
                                 void *hip_stream);

/* Alg. 2 (1.58Quant with token protection): per channel and 32-token group
 * s = mean |V| over the unprotected tokens, code = +1 / -1 / 0 against
 * +-gamma*s (Eq. 6); protected tokens are coded 0 and their rows copied
 * verbatim.  The protected set is shared by all layers and heads of a
 * sequence and is given either as scores (top n_salient, ties: lower index
 * first; Eq. 7 scores are computed by the caller) or as an index list.
 *   V_dev           in : [L, B, Hkv, Tq, 128] fp16
 *   saliency_dev    in : [B, Tq] float32, or NULL
 *   salient_idx_dev in : [B, n_salient] int32, strictly ascending per
 *                        sequence, or NULL.  With n_salient > 0 exactly one of
 *                        the two is non-NULL; with n_salient == 0 both are
 *                        ignored.  Entries outside 0..Tq-1 and repeated
 *                        entries are not an error: they are dropped, fewer
 *                        tokens are protected (with salient_bits == 2 the
 *                        statistics of the last group of protected rows are
 *                        then unspecified).
 *   packed_V_dev    out: >= vidkv_packed_values_bytes(params) bytes
 *   workspace_dev      : >= vidkv_workspace_bytes(params, 1) bytes           */
vidkv_status vidkv_quantize_values(const vidkv_params *params, const void *V_dev,
                                   const float *saliency_dev,
                                   const int32_t *salient_idx_dev,
                                   void *packed_V_dev, size_t packed_bytes,
                                   void *workspace_dev, size_t workspace_bytes,
                                   void *hip_stream);

/* Alg. 3 and Alg. 2 on the K and V tensors of the same tokens in one call (the
 * compression step at the end of Alg. 1, Prefill): the packed buffers come out
 * byte-identical to vidkv_quantize_keys followed by vidkv_quantize_values.
 * With a side stream the protected-token selection - a chain of short
 * dependent launches - is enqueued there so that it runs beside the key
 * passes (only when the key tensor is 32 MiB or more; smaller inputs run in
 * line); it is joined back before the value coding pass.
 * Arguments as for the two separate calls;
 *   workspace_dev : >= vidkv_workspace_bytes(params, 3) bytes
 *   side          : NULL, or the caller's side stream and events (all three
 *                   handles non-NULL, else VIDKV_EINVAL)                      */
vidkv_status vidkv_quantize_kv(const vidkv_params *params, const void *K_dev,
                               const void *V_dev, const float *saliency_dev,
                               const int32_t *salient_idx_dev, void *packed_K_dev,
                               size_t packed_K_bytes, void *packed_V_dev,
                               size_t packed_V_bytes, void *workspace_dev,
                               size_t workspace_bytes, void *hip_stream,
                               const vidkv_side_stream *side);

/* Alg. 1, Decoding, for one layer: out = Softmax(scale * q [K'; K_r]^T) [V'; V_r]
 * (Eq. 3) where K', V' are the dequantized packed tokens (never materialised
 * in memory) and K_r, V_r the first tail_len[b] rows of the fp16 residual
 * buffers.  Appending the new token to the residual buffers and advancing
 * tail_len is the caller's job.
 *   layer           : 0..L-1, selects the layer inside the packed buffers
 *   q_dev        in : [B, Hq, 128] fp16
 *   packed_K_dev, packed_V_dev in : as written by the two quantize calls with
 *                     the same params
 *   K_tail_dev, V_tail_dev in : [B, Hkv, tail_capacity, 128] fp16 of this
 *                     layer; may be NULL when tail_capacity == 0
 *   tail_len_dev in : [B] int32, each 0..tail_capacity; NULL means all zero
 *   out_dev     out : [B, Hq, 128] fp16 (fp32 accumulation, RNE at the end)
 *   workspace_dev   : >= vidkv_workspace_bytes(params, 2) bytes (the size
 *                     depends on t_capacity, not on t_quant)
 * With Tq == 0 this is plain attention over the residual tokens; a sequence
 * with no token at all gets zeros.
 * With a side stream, a large residual block (32-token blocks over all
 * sequences and KV heads, at most 8 counted per head, numbering four times
 * the device's compute units or more) is read by a kernel that is forked onto
 * it and joined before the split partials are merged.
 *   side            : NULL, or the caller's side stream and events           */
vidkv_status vidkv_decode_attention(const vidkv_params *params, int32_t layer,
                                    const void *q_dev, const void *packed_K_dev,
                                    const void *packed_V_dev, const void *K_tail_dev,
                                    const void *V_tail_dev, int32_t tail_capacity,
                                    const int32_t *tail_len_dev, void *out_dev,
                                    void *workspace_dev, size_t workspace_bytes,
                                    void *hip_stream, const vidkv_side_stream *side);

/* vidkv_decode_attention for callers that cannot allocate device memory or
 * carry a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, checks and result as
 * vidkv_decode_attention, without the workspace: the split partials go to a
 * device array inside the library's image, VIDKV_NOALLOC_SCRATCH_BYTES large,
 * which every GPU that runs the library holds until the process ends.  The
 * call allocates nothing and takes no side stream: all of its kernels, the
 * one for a large residual block included, run in line on `hip_stream`.
 * A shape whose partials (what vidkv_workspace_bytes(params, 2) reports) do
 * not fit the array returns VIDKV_ENOSPACE and launches nothing.  The device
 * address of the array is looked up at the first call on each device (make
 * that call outside a stream capture).  All calls on one GPU share the one
 * array: two such calls that may run at the same time - on different streams
 * of that GPU, or from different host threads - race and give wrong results;
 * calls ordered on one stream are fine.                                        */
#define VIDKV_NOALLOC_SCRATCH_BYTES (16u << 20)
vidkv_status vidkv_decode_attention_noalloc(const vidkv_params *params, int32_t layer,
                                            const void *q_dev, const void *packed_K_dev,
                                            const void *packed_V_dev, const void *K_tail_dev,
                                            const void *V_tail_dev, int32_t tail_capacity,
                                            const int32_t *tail_len_dev, void *out_dev,
                                            void *hip_stream);

/* Alg. 1, Decoding, the step taken when the residual buffers are full (R
 * tokens): the first n_flush residual tokens of every sequence of one layer
 * are coded and appended to the packed buffers as tokens t_quant ..
 * t_quant + n_flush - 1.  Values: Alg. 2's 1.58Quant without protected tokens
 * (Eq. 6).  Keys: the group coding of Alg. 3 (Eq. 4 / Eq. 5) with the channel
 * split chosen when the cache was first quantized - the ranking by range is
 * not repeated, and the groups already packed are not touched (re-coding their
 * dequantized values with the same split would reproduce them).
 *   params          : t_quant = tokens packed so far (> 0), t_capacity >=
 *                     t_quant + n_flush
 *   layer           : 0..L-1
 *   K_tail_dev, V_tail_dev in : [B, Hkv, tail_capacity, 128] fp16 of this layer;
 *                     rows 0..n_flush-1 of every head must be valid tokens
 *   n_flush         : multiple of 32, 0 < n_flush <= tail_capacity
 *   packed_K_dev, packed_V_dev in/out : as written by the quantize calls with
 *                     the same t_capacity
 * Afterwards the caller raises t_quant by n_flush - once every layer has been
 * flushed - and moves any remaining residual rows to the front.  No workspace. */
vidkv_status vidkv_flush_residual(const vidkv_params *params, int32_t layer,
                                  const void *K_tail_dev, const void *V_tail_dev,
                                  int32_t tail_capacity, int32_t n_flush,
                                  void *packed_K_dev, size_t packed_K_bytes,
                                  void *packed_V_dev, size_t packed_V_bytes,
                                  void *hip_stream);

/* Sec. 3.3 (2), Eq. 7: the cross-modal score I(i, j) = X_v(i) . X_t(j) between
 * visual token i and text token j, summed over the text tokens of the
 * sequence: scores[b][i] = sum_j X_v[b][i] . X_t[b][j] (fp32 accumulation).
 * The result is what vidkv_quantize_values takes as saliency_dev.  Which
 * hidden states to pass (the paper does not say which layer) is the caller's
 * choice.
 *   X_v_dev   in : [B, n_visual, hidden_dim] fp16, 16-byte aligned
 *   X_t_dev   in : [B, n_text, hidden_dim] fp16, n_text >= 1
 *   hidden_dim   : multiple of 8, 8..16384
 *   scores_dev out: [B, n_visual] float32
 *   workspace_dev: >= vidkv_saliency_workspace_bytes(B, hidden_dim) bytes      */
size_t vidkv_saliency_workspace_bytes(int32_t batch, int32_t hidden_dim);
vidkv_status vidkv_saliency_scores(const void *X_v_dev, const void *X_t_dev, int32_t batch,
                                   int32_t n_visual, int32_t n_text, int32_t hidden_dim,
                                   float *scores_dev, void *workspace_dev,
                                   size_t workspace_bytes, void *hip_stream);

/* Measurement aids, not part of the method.  Each takes the arguments of the
 * entry point it is named after, checks them the same way, and launches only
 * the kernels selected by `stages`, so that a benchmark can bracket a single
 * kernel with events.  The buffers must already hold what the skipped kernels
 * would have written (run the full entry point once first).
 *   quantize_keys   : bit 0 per-channel min/max over all tokens (Alg. 3, range)
 *                     bit 1 top-n_anom channel selection
 *                     bit 2 per-group coding pass (Eq. 4 and Eq. 5)
 *   quantize_values : bit 0 protected-token selection, bit 1 ternary coding pass
 *   decode_attention: bit 0 split-T partial attention, bit 1 merge              */
vidkv_status vidkv_quantize_keys_stages(const vidkv_params *params, const void *K_dev,
                                        void *packed_K_dev, size_t packed_bytes,
                                        void *workspace_dev, size_t workspace_bytes,
                                        uint32_t stages, void *hip_stream);
vidkv_status vidkv_quantize_values_stages(const vidkv_params *params, const void *V_dev,
                                          const float *saliency_dev,
                                          const int32_t *salient_idx_dev, void *packed_V_dev,
                                          size_t packed_bytes, void *workspace_dev,
                                          size_t workspace_bytes, uint32_t stages,
                                          void *hip_stream);
vidkv_status vidkv_decode_attention_stages(const vidkv_params *params, int32_t layer,
                                           const void *q_dev, const void *packed_K_dev,
                                           const void *packed_V_dev, const void *K_tail_dev,
                                           const void *V_tail_dev, int32_t tail_capacity,
                                           const int32_t *tail_len_dev, void *out_dev,
                                           void *workspace_dev, size_t workspace_bytes,
                                           uint32_t stages, void *hip_stream,
                                           const vidkv_side_stream *side);

/* Measurement aid, not part of the method: dst[i] = src[i] for `bytes` bytes
 * (multiple of 16, both 16-byte aligned) with the library's streaming access
 * pattern; used to calibrate hardware byte counters and the achievable HBM
 * rate. */
vidkv_status vidkv_calib_copy(void *dst_dev, const void *src_dev, size_t bytes,
                              void *hip_stream);

const char *vidkv_status_string(vidkv_status status);
int vidkv_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VIDKV_H */
