/*
 * odmoe_measure.h -- measurement aids of libodmoe.so.  None of them is part of the method of
 * OD-MoE (arXiv 2512.03927) or needed to use the library (that is odmoe.h); the benchmark uses
 * them to time single kernels with HIP events on the stream they run on, to measure the HBM and
 * host-link ceilings the kernels are compared with, and to give a profiler's byte counters a
 * kernel of known traffic to be scaled by.
 */
#ifndef ODMOE_MEASURE_H
#define ODMOE_MEASURE_H

#include "odmoe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A plain streaming kernel over `bytes`
 * (multiple of 16) of device memory, enqueued on `stream`.  mode 0 copies src_dev to dst_dev
 * (both `bytes` long); mode 1 only reads src_dev (dst_dev: at least 4 bytes of scratch).  It
 * gives the measured HBM ceiling the expert GEMVs are compared with, and a kernel of known
 * traffic to scale a profiler's byte counters by.
 */
int odmoe_probe_hbm(void* dst_dev, const void* src_dev, uint64_t bytes, int32_t mode, void* stream);

/*
 * Average duration, in microseconds, of each decode kernel of layer `layer`
 * (resident mode) over the n_tokens rows of x_dev[T,H], taken with HIP events on the compute
 * stream around `reps` passes in which the same kernel is launched back to back for every token
 * (token t uses the experts the router picks for it, as in odmoe_decode_step).  Blocks.
 * Allocates and frees small temporaries.
 */
int odmoe_time_decode_kernels(odmoe_layer_t* h, int32_t layer, const void* x_dev, int32_t n_tokens,
                              int32_t reps, float* route_us, float* ffn_up_us, float* ffn_down_us);

/*
 * The host->HBM copies of `n_tokens` decode tokens (n_layers * top_k expert
 * copies each, layer l taking experts (l*top_k + i) mod n_experts) issued exactly as
 * odmoe_decode_step issues them (same copy streams, slots taken round-robin) but with no kernels
 * in between: *ms_per_token gets the wall-clock time per token.  This is the "load" leg of
 * max(compute, load) a cacheless step is compared with.  Cacheless mode only; ESTATE while an
 * expert holds a slot.  Blocks.
 */
int odmoe_time_expert_loads(odmoe_layer_t* h, int32_t n_tokens, float* ms_per_token);

#ifdef __cplusplus
}
#endif
#endif /* ODMOE_MEASURE_H */
