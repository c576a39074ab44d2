/*
 * odmoe.h -- C ABI of libodmoe.so: the cacheless Mixture-of-Experts decode layer
 * of OD-MoE (arXiv 2512.03927) on one AMD MI355X (gfx950).
 *
 * What the calls compute.  Per token and per MoE layer (paper Section 3.1: the gating
 * network is the usual one of MoE models, top-2 policy; Section 4.1: Mixtral-8x7B experts):
 *
 *   logit[e] = b[e] + sum_h Wg[e,h] x[h]                  (float64 sum, rounded once to fp32)
 *   idx      = k largest logits, order (logit desc, index asc)       -- ties: lowest index wins
 *   g_i      = exp(l_i - l_0) / sum_j exp(l_j - l_0)      over the k kept experts  (sum g = 1)
 *   FFN_e(x) = W2_e ( silu(W1_e x) * (W3_e x) ),  silu(a) = a / (1 + exp(-a))
 *   y        = sum_{i<k} g_i FFN_{idx_i}(x)               (fp32, i ascending, one final rounding)
 *
 * and, between stacked layers when config.glue = 1 (stand-in for the main node's non-expert
 * work M_l of Section 3.1, which is outside this library):  x <- rmsnorm(x + y), eps 1e-6.
 *
 * Cacheless operation (paper Sections 1-3.1: experts live in CPU DRAM, an expert is loaded
 * to the GPU on demand -- task EL_l -- used once -- task EC_l -- and evicted right after): with
 * config.n_slots > 0 the experts' weights stay in pinned host memory and only n_slots
 * expert-sized slots exist in HBM.  Every activation is a host->HBM copy; nothing is cached.
 *
 * Experts read in place.  With config.n_slots = 0 the kernels read each expert where its
 * pointer says.  Normally that is HBM.  Pinned host memory that is mapped for the device
 * (hipHostMalloc, odmoe_pinned_alloc) also qualifies: then nothing is copied and nothing is
 * held in HBM at all, the GEMV kernels pull the activated experts' weights across the host
 * link while they compute (launch shapes made for the link: about a hundred waves, each streaming
 * one long run), no host synchronisation happens per layer, no prediction is needed, and results
 * are bit for bit those of the other modes.  odmoe_stats counts no loads and no copied bytes in
 * this form.  Batches work too, but the grouped GEMMs fetch an expert's weights once per chunk of
 * 320 of its tokens, and host memory is not kept in the GPU's L2: for long prompts a second handle
 * with a slot pool over the same pinned buffers is the faster way.
 *
 * Conventions.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *   - All matrices are row-major and dense.  dtype applies to x, y, router and expert weights;
 *     bf16 is the upper 16 bits of an fp32 (round-to-nearest-even).
 *   - One expert is ONE contiguous buffer:  W1[F,H] | W3[F,H] | W2[H,F]   (3*H*F elements).
 *   - hidden and ffn must be multiples of 8; 1 <= top_k <= min(n_experts, 8); n_experts <= 1024.
 *   - Experts may instead be int8 codes with a scale per weight row, packed 4-bit codes with a
 *     scale per group of 64, or (fp32 layers) binary16 weights (odmoe_config.expert_quant): the
 *     quantised shadow model of Sections 1 and 3.2, which reads fewer bytes per token.
 *   - The caller owns every buffer it passes in; weight buffers must outlive the handle.
 *     Streams are borrowed (never destroyed here).  The library owns its slot pool, scratch
 *     buffers, events and, if no copy stream was given, its copy streams.
 *   - Every call returns an odmoe_status.  Argument errors are detected before anything is
 *     enqueued.  HIP errors are reported as ODMOE_EHIP by the call that observes them.
 *     odmoe_last_error() gives a thread-local message for the last failing call.
 *   - No call blocks the host except odmoe_decode_step (cacheless mode: once per layer, to
 *     learn which experts to copy, and once at its end), odmoe_expert_ffn in cacheless mode
 *     without idx_host, and odmoe_layer_destroy.
 *   - A handle is not thread-safe: one host thread drives one handle.
 *   - After a failing call a cacheless handle stays usable: odmoe_decode_step waits for the work
 *     in flight and frees every slot (experts loaded earlier through odmoe_expert_load_async
 *     included); odmoe_expert_ffn gives back the slots that the call itself took.
 *
 * Environment (read by odmoe_layer_init; not needed):
 *   ODMOE_COPY_STREAMS=1..8   number of library-owned copy streams (changes timing only)
 *
 * Measurement aids (a streaming probe, per-kernel timings, a copy-only replay) are declared in
 * odmoe_measure.h; they are not part of the method.
 */
#ifndef ODMOE_H
#define ODMOE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct odmoe_layer odmoe_layer_t; /* opaque: one stack of n_layers MoE layers */

typedef enum {
  ODMOE_OK = 0,
  ODMOE_EINVAL = -1, /* bad argument (null pointer, out-of-range index, unsupported shape) */
  ODMOE_ENOMEM = -2, /* device or host allocation failed */
  ODMOE_EHIP = -3,   /* a HIP runtime call failed; see odmoe_last_error() */
  ODMOE_ESTATE = -4, /* an expert that is needed is neither resident nor being loaded */
  ODMOE_EBUSY = -5   /* no free slot for a load */
} odmoe_status;

typedef enum { ODMOE_F32 = 0, ODMOE_BF16 = 1 } odmoe_dtype;

/* Weight formats of the shadow model (Sections 1, 3.2; the paper names FP16 / INT8 / NF4 and
 * prints no scheme: the integer ones are the plain symmetric absmax schemes, round half to even).
 *   INT8_ROW  per weight row:  s = max|w| / 127,  q = clip(rne(w / s), -127, 127)
 *   INT4_G64  per group of 64 consecutive weights of a row:  s = max|w| / 7,  q in -7..7
 *   F16       every weight rounded to IEEE binary16 (nearest, ties to even, |w| clipped to 65504)
 * Integer codes are stored offset-binary in one byte each: q + 128, resp. q + 8.  An all-zero row
 * or group has scale 0 and codes of 0. */
typedef enum { ODMOE_Q_NONE = 0, ODMOE_Q_INT8_ROW = 1, ODMOE_Q_INT4_G64 = 2, ODMOE_Q_F16 = 3 } odmoe_quant;

#define ODMOE_MAX_TOPK 8
#define ODMOE_MAX_EXPERTS 1024

typedef struct {
  int32_t hidden;    /* H */
  int32_t ffn;       /* F */
  int32_t n_experts; /* E */
  int32_t top_k;     /* k */
  int32_t n_layers;  /* L */
  int32_t n_slots;   /* S; 0 = resident: expert_w are DEVICE pointers and nothing is ever loaded
                        (any address the GPU can read will do, see "Experts read in place") */
  int32_t dtype;     /* odmoe_dtype */
  int32_t glue;      /* 0: x_{l+1} = y_l ; 1: x_{l+1} = rmsnorm(x_l + y_l) between stacked layers */
  int32_t expert_quant; /* odmoe_quant of the expert buffers (a shadow model's experts; x, y and the
                        router stay in dtype, the GEMVs dequantise in registers and accumulate in
                        fp32, batches run token by token: no grouped GEMM).
                        ODMOE_Q_NONE: weights in dtype.
                        ODMOE_Q_INT8_ROW: codes W1[F,H] | W3[F,H] | W2[H,F] (one byte each), then
                          fp32 scales s1[F] | s3[F] | s2[H].  hidden and ffn multiples of 16,
                          hidden <= 8192.
                        ODMOE_Q_INT4_G64: codes packed two per byte (element 2j in the low nibble of
                          byte j) W1[F][H/2] | W3[F][H/2] | W2[H][F/2], then fp32 scales, one per
                          group of 64 weights of a row, s1[F][H/64] | s3[F][H/64] | s2[H][F/64].
                          hidden and ffn multiples of 64, hidden <= 8192.
                        ODMOE_Q_F16: binary16 weights W1[F,H] | W3[F,H] | W2[H,F]; dtype must be
                          ODMOE_F32 (the 16-bit shadow of a full-precision model: half its bytes);
                          hidden <= 8192, ffn <= 32768.
                        All as odmoe_quantize_expert writes them. */
} odmoe_config;

typedef struct {
  /* kernel / copy times are HIP-event times summed over the layers of one call; they are 0
     unless timing was asked for (see odmoe_decode_step) */
  float t_route_ms;    /* router GEMV + top-k gate kernel; between stacked layers it starts with the
                          previous layer's glue (one kernel), whose time is therefore counted here */
  float t_load_ms;     /* host->HBM expert copies: time during which at least one copy was in
                          flight (copies on different copy streams overlap) */
  float t_ffn_up_ms;   /* w1/w3 GEMV + SiLU gate kernel */
  float t_ffn_down_ms; /* w2 GEMV + weighted combine kernel */
  float t_glue_ms;     /* stand-alone glue kernel: after the last layer, and between layers only
                          when the hidden vector does not fit the router kernel's LDS (32 KB) */
  float t_step_ms;     /* wall time of the call, host clock */
  uint64_t h2d_bytes; /* bytes copied host->HBM by this call */
  uint64_t loads;     /* expert loads issued by this call (cacheless: n_layers*top_k + reloads) */
  uint64_t reloads;   /* loads caused by wrong predictions (Section 3.1: misprediction fallback) */
  uint64_t hint_hits; /* predicted experts that the router confirmed */
} odmoe_stats;

/*
 * Create a stack of L MoE layers (Section 3.1: gating network + experts; worker memory holds
 * only the scheduled experts).
 *   cfg         host pointer.
 *   router_w    host array of L DEVICE pointers, each Wg[E,H] in cfg->dtype.
 *   router_b    NULL, or host array of L DEVICE pointers (entries may be NULL), each b[E] fp32.
 *   expert_w    host array of L*E pointers (index layer*E + expert), each one expert buffer.
 *               n_slots == 0: DEVICE pointers.  n_slots > 0: HOST pointers to PINNED memory
 *               (hipHostMalloc / torch pin_memory; odmoe_pinned_alloc provides it too).
 *   compute_stream  hipStream_t as void*; NULL = the null stream.
 *   copy_stream     hipStream_t for host->HBM copies; NULL = the library creates four and
 *                   rotates the copies over them, over three of them for copies issued ahead
 *                   of time from hints (back-to-back copies on one stream leave gaps that cost
 *                   about 4 % of the link rate for 17 MB experts; with four streams the copies
 *                   of consecutive layers no longer finish in issue order).
 *   out         receives the handle.
 * Allocates S*expert_bytes of HBM for the slot pool plus small scratch.  n_slots > 0 needs
 * n_slots >= top_k.  Expert buffers the HIP runtime knows to be ordinary (unpinned) host memory, or
 * device memory where n_slots > 0 wants pinned host memory, are refused with EINVAL.  Returns
 * EINVAL / ENOMEM / EHIP; on failure *out is NULL.
 */
int odmoe_layer_init(const odmoe_config* cfg, const void* const* router_w,
                     const void* const* router_b, const void* const* expert_w,
                     void* compute_stream, void* copy_stream, odmoe_layer_t** out);

/* Waits for the compute and copy streams, frees everything the library owns.  NULL is allowed. */
int odmoe_layer_destroy(odmoe_layer_t* h);

/*
 * Router GEMV + top-k softmax gate (Section 3.1, gating network of layer `layer`) for
 * n_tokens rows of x_dev[T,H].  Writes idx_dev[T,k] (int32) and gate_dev[T,k] (fp32).
 * Asynchronous on the compute stream.  NaN logits give an unspecified selection.
 */
int odmoe_route_topk(odmoe_layer_t* h, int32_t layer, const void* x_dev, int32_t n_tokens,
                     int32_t* idx_dev, float* gate_dev);

/*
 * On-demand expert loading EL_l (Sections 1, 3.1): enqueue the copy of expert (layer, expert)
 * from pinned host memory into a free HBM slot on a copy stream.  The copy waits (stream
 * side) for the kernels that last read that slot and for an earlier copy into it.  If the
 * expert is already loading or ready, its slot is returned and nothing is copied.  *slot_out
 * (may be NULL) gets the slot.
 * EBUSY when every slot is occupied; EINVAL in resident mode or for a bad index.
 */
int odmoe_expert_load_async(odmoe_layer_t* h, int32_t layer, int32_t expert, int32_t* slot_out);

/* Drop expert (layer, expert) from its slot without using it (a wrongly predicted expert).
 * ESTATE if it holds no slot. */
int odmoe_expert_evict(odmoe_layer_t* h, int32_t layer, int32_t expert);

/*
 * Expert computation EC_l (Section 3.1) with the weighted combine, for n_tokens tokens:
 *   y[t] = sum_i gate[t,i] * FFN_{idx[t,i]}(x[t]).
 *   idx_dev[T,k], gate_dev[T,k], x_dev[T,H], y_dev[T,H] are device pointers.  An idx entry
 *   outside [0, n_experts) selects no expert: that rank is left out of the sum (the kernels test
 *   it; the library cannot see device memory without blocking).  In cacheless mode such an entry
 *   in the host copy of one token's ids is EINVAL.
 *   idx_host   optional host copy of idx (cacheless mode needs to know the experts on the
 *              host; when NULL there, the library reads idx_dev back and blocks for it).
 *   n_tokens   resident mode: token by token (one fused w1/w3+SiLU GEMV and one w2+combine GEMV
 *              per token) while the token-slots do not outnumber the experts
 *              (n_tokens * top_k <= n_experts and n_tokens < 16); larger batches (hidden and
 *              ffn multiples of 64) take the prefill path of Section 3.3 -- tokens are grouped by
 *              expert and each expert runs a grouped GEMM on the matrix cores, reading its
 *              weights once; in bf16 layers the SwiGLU intermediate is rounded to bf16 there (the
 *              matrix cores take bf16 operands), fp32 layers (the paper's full precision) use the
 *              fp32 matrix instructions and round nothing.  Other shapes stay on the per-token
 *              path.
 *   evict_after  cacheless mode: nonzero releases the experts' slots after the kernels that
 *              read them (the paper's prompt eviction).  Ignored in resident mode.
 * Cacheless mode: n_tokens == 1 needs every chosen expert loading or ready (ESTATE otherwise);
 * the compute stream waits (stream side) for each copy.  n_tokens >= 2 (hidden and ffn
 * multiples of 64; EINVAL otherwise) is the prefill of Section 3.3 from host memory: the call
 * itself streams every expert that received tokens into a slot exactly once (experts already
 * loading or ready are used as they are), runs that expert's grouped GEMMs when its copy has
 * landed, and with evict_after releases the slot for the next expert, so that copies overlap
 * GEMMs.
 */
int odmoe_expert_ffn(odmoe_layer_t* h, int32_t layer, const int32_t* idx_dev,
                     const float* gate_dev, const int32_t* idx_host, const void* x_dev,
                     int32_t n_tokens, void* y_dev, int32_t evict_after);

/*
 * One decode token through all L layers (Section 3.1 pipeline on one GPU):
 * per layer  route -> learn ids on the host -> load the k experts -> FFN + combine -> evict
 * -> glue.  x_dev[H] in, y_dev[H] out.  With glue = 0 the result is the last layer's y
 * (and x_{l+1} = y_l in between); with glue = 1 it is the state after the last layer's glue,
 * x_L = rmsnorm(x_{L-1} + y_{L-1}), each layer's y being rounded to dtype before the glue.
 *   predicted_idx_host  NULL, or int32[L,k] predicted experts per layer (the role of the
 *              shadow node's prediction): loads for coming layers are issued ahead as slots
 *              allow; the router's result is authoritative; wrong predictions are evicted
 *              and the right expert reloaded (misprediction fallback).  Predictions change
 *              timing only, never y.
 *   idx_out_host  NULL, or int32[L,k] receiving the experts actually used.
 *   stats      NULL, or receives counters; kernel/copy times are measured only when
 *              stats->t_step_ms is set to a negative value on entry (adds event overhead).
 * Blocks until y is complete, except in resident mode with idx_out_host == NULL and
 * stats == NULL, where the call only enqueues kernels on the compute stream (no host
 * synchronisation per layer, no allocation, no fill or copy by the runtime): in that form a
 * call can be recorded into a HIP graph captured on the compute stream and replayed.
 */
int odmoe_decode_step(odmoe_layer_t* h, const void* x_dev, void* y_dev,
                      const int32_t* predicted_idx_host, int32_t* idx_out_host,
                      odmoe_stats* stats);

/*
 * For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): odmoe_expert_ffn for experts resident in GPU-readable memory, token by
 * token, without a handle and without any allocation by the library or the runtime:
 *   y[t] = sum_i gate[t,i] * FFN_{idx[t,i]}(x[t]),  t = 0 .. n_tokens-1.
 *   cfg              hidden, ffn, n_experts, top_k, dtype as for odmoe_layer_init; n_slots must be
 *                    0; n_layers and glue are ignored.
 *   expert_table_dev DEVICE array of n_experts pointers, each one expert buffer W1|W3|W2 in
 *                    memory the GPU can read.
 *   idx_dev[T,k], gate_dev[T,k], x_dev[T,H], y_dev[T,H]  device pointers, as for odmoe_expert_ffn
 *                    (an idx entry outside [0, n_experts) selects nothing).
 *   stream           hipStream_t the kernels are enqueued on (NULL = the null stream).
 * The fp32 intermediate h[k, F] lives in a 1 MiB array that is part of the library's code object
 * (each GPU the library runs on holds its own copy until the process ends), so
 * top_k * ffn * 4 bytes must not exceed 1 MiB: larger shapes are refused with EINVAL and a
 * message.  Output bits equal those of odmoe_expert_ffn's per-token path.  Asynchronous.  All
 * calls on one GPU share that array: calls that may overlap (different streams, different host
 * threads) race; calls on one stream are ordered and safe.  Nothing in it needs clearing between
 * calls (every element a token reads was written for that token first).
 */
int odmoe_expert_ffn_static(const odmoe_config* cfg, const void* const* expert_table_dev,
                            const int32_t* idx_dev, const float* gate_dev, const void* x_dev,
                            int32_t n_tokens, void* y_dev, void* stream);

/* Bytes of one expert buffer as a handle made from cfg expects it: 3*H*F elements of dtype, or for
 * ODMOE_Q_INT8_ROW 3*H*F code bytes + 4*(2*F + H) bytes of scales, for ODMOE_Q_INT4_G64 3*H*F/2
 * code bytes + 4*(3*H*F/64) bytes of scales, for ODMOE_Q_F16 3*H*F*2.  0 for a NULL or invalid cfg. */
uint64_t odmoe_expert_bytes(const odmoe_config* cfg);

/*
 * The shadow model's weights (Sections 1, 3.2): quantise w_dev[rows, cols] (row-major, dtype) on
 * the device.  kind: ODMOE_Q_INT8_ROW, ODMOE_Q_INT4_G64 (cols a multiple of 64) or ODMOE_Q_F16.
 * Outputs, each optional (NULL = not wanted), all device pointers:
 *   code_dev     uint8 [rows, cols], offset-binary codes; F16: rows*cols binary16 values (two
 *                bytes each, 2-byte aligned)
 *   scale_dev    fp32 [rows] (INT8_ROW) or [rows, cols/64] (INT4_G64): the float64 scale rounded
 *                once; F16 has none (must be NULL)
 *   dequant_dev  [rows, cols] in dtype: q * scale (float64) rounded once to dtype -- the weights a
 *                shadow copy held in the storage dtype uses
 * The scale, the division and the rounding are done in float64, so every code equals the one a
 * float64 CPU computation of the formulas above gives.  Asynchronous on `stream`.
 */
int odmoe_quantize(const void* w_dev, int32_t dtype, int64_t rows, int64_t cols, int32_t kind,
                   uint8_t* code_dev, float* scale_dev, void* dequant_dev, void* stream);

/* One stored expert W1[F,H] | W3[F,H] | W2[H,F] (cfg->dtype, device) into the expert buffer of
 * format `kind` (ODMOE_Q_INT8_ROW, ODMOE_Q_INT4_G64 or ODMOE_Q_F16) described at odmoe_config; dst_dev: device,
 * odmoe_expert_bytes of the config with expert_quant = kind.  The codes and scales are those of
 * odmoe_quantize on the three matrices.  cfg->expert_quant is ignored.  Asynchronous on `stream`. */
int odmoe_quantize_expert(const odmoe_config* cfg, int32_t kind, const void* expert_dev, void* dst_dev,
                          void* stream);

/*
 * Scaled emulative prediction, emulated on one GPU (Sections 1, 3.2): `shadow` (a stack of the
 * same shape as `main`, normally with quantised weights, resident) decodes each token first, its
 * expert selection is handed to `main` as the prediction, `main` decodes the same token, and the
 * fraction of main's activated experts that were predicted is the token's recall (Section 3.2).
 * There is no attention or KV cache in this library, so an autoregressive iteration is emulated by
 * feeding main's output back as its next input.  aligned != 0: the shadow starts every iteration
 * from main's input (the token / KV alignment of Section 3.2, every iteration); aligned == 0: it
 * follows its own outputs after the first iteration.
 *   x0_dev [H] first input; recall_out host float[n_iter]; x_final_dev [H] or NULL receives main's
 *   last output; shadow_ms / main_ms (host, may be NULL) receive the wall time spent in each
 *   stack's decode steps.  Predictions change main's timing only, never its output.  Blocks;
 *   allocates and frees small device buffers.
 */
int odmoe_sep_emulate(odmoe_layer_t* main_stack, odmoe_layer_t* shadow, const void* x0_dev,
                      int32_t n_iter, int32_t aligned, float* recall_out, void* x_final_dev,
                      float* shadow_ms, float* main_ms);

/* Pinned host memory for the expert store (the workers' DRAM of Section 1). */
int odmoe_pinned_alloc(uint64_t bytes, void** out_host);
int odmoe_pinned_free(void* host);

/*
 * Longest expert-loading time that causes no compute stall (Section 3.1, load-window
 * equation, with its G read as the number of groups so that it reproduces the worked example
 * 4 t^M + 3 t^W of the four-group testbed):  n_groups * t_main + (n_groups - 1) * t_worker.
 * Host-only arithmetic; n_groups < 1 gives 0.
 */
double odmoe_load_window_ms(int32_t n_groups, double t_main_ms, double t_worker_ms);

/* Number of slot groups of the handle, floor(n_slots / top_k): the one-GPU counterpart of the
 * paper's N_W / G worker groups (Section 3.1); 0 in resident mode. */
int32_t odmoe_slot_groups(const odmoe_layer_t* h);

/* Bytes of HBM the handle's slot pool occupies (S * expert bytes); 0 in resident mode. */
uint64_t odmoe_slot_pool_bytes(const odmoe_layer_t* h);

/* Thread-local message of the last failing call on this thread ("" if none). */
const char* odmoe_last_error(void);

/* Library version string. */
const char* odmoe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ODMOE_H */
