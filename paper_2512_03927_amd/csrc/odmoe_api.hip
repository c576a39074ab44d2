// C-ABI of libodmoe.so (declared in include/odmoe.h): handle, slot pool + copy engine,
// and the per-token decode loop.  All arithmetic lives in the kernels; this file only
// validates, schedules and enqueues.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <utility>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/odmoe_measure.h"
#include "kernels.h"
#include "sched.hpp"

using namespace odmoe;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) noexcept {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

// No C++ exception crosses the C boundary: host-side allocations (vectors, the scheduler) can throw.
template <class F>
int guarded(F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return fail(ODMOE_ENOMEM, "out of host memory");
  } catch (...) {
    return fail(ODMOE_ESTATE, "unexpected C++ exception");
  }
}

#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t e__ = (expr);                                                               \
    if (e__ != hipSuccess)                                                                 \
      return fail(ODMOE_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__),      \
                  __FILE__, __LINE__);                                                     \
  } while (0)

size_t dtype_size(int32_t dt) { return dt == ODMOE_F32 ? 4 : 2; }

size_t expert_bytes_of(const odmoe_config& c) {
  const size_t hf = (size_t)c.hidden * c.ffn;
  if (c.expert_quant == ODMOE_Q_INT8_ROW) return 3 * hf + sizeof(float) * (2 * (size_t)c.ffn + c.hidden);
  if (c.expert_quant == ODMOE_Q_INT4_G64) return 3 * hf / 2 + sizeof(float) * (3 * hf / 64);
  if (c.expert_quant == ODMOE_Q_F16) return 3 * hf * 2;
  return 3 * hf * dtype_size(c.dtype);
}

}  // namespace

struct odmoe_layer {
  odmoe_config cfg{};
  Shape sh{};
  size_t esize = 0;         // bytes per element
  size_t expert_bytes = 0;  // 3*H*F*esize
  hipStream_t compute = nullptr, copy = nullptr;
  bool own_copy = false;

  std::vector<const void*> router_w, router_b, expert_w;  // host copies of the pointer arrays
  const void** table_dev = nullptr;                        // resident: device table [L*E]

  // cacheless state
  char* pool_mem = nullptr;
  SlotPool* pool = nullptr;
  DecodeScheduler* sched = nullptr;
  std::vector<hipEvent_t> ready_ev, done_ev;  // per slot
  std::vector<char> done_pending;             // done_ev[slot] recorded since the slot's last copy
  std::vector<char> copied_once;              // ready_ev[slot] has been recorded at least once
  // Copies rotate over these streams (copy and, when the library owns it, three more): back-to-back
  // copies on one stream leave a gap of about 10 us between them, which matters for small experts.
  std::vector<hipStream_t> copy_ring;
  uint32_t next_copy = 0;
  uint32_t ring_active = 0;   // streams the rotation uses (0 = all)
  bool ring_fixed = false;    // the environment fixed the number of copy streams

  // scratch
  float* hbuf = nullptr;      // [k*F] fp32
  void* xbuf[2] = {nullptr, nullptr};
  void* ybuf = nullptr;       // [H]
  int32_t* idx_dev = nullptr;   // [L*k]
  float* gate_dev = nullptr;    // [L*k]
  int32_t* idx_pin = nullptr;   // pinned host [L*k], written by the router kernel
  int32_t* idx_pin_dev = nullptr;
  const void** eptr_dev = nullptr;  // resident: [L*k] expert pointers resolved by the router kernel
  hipEvent_t route_ev = nullptr;
  RouteScratch route_scratch{nullptr, nullptr, 0};  // lets few-token router launches use many CUs
  void* prefill_ws = nullptr;
  size_t prefill_ws_bytes = 0;

  // optional timing events (created on first timed decode_step): [L] pairs
  std::vector<hipEvent_t> tev;  // 5 per layer: route begin, up begin, down begin, glue begin, end
  std::vector<hipEvent_t> lev;  // 2 per load (begin/end on the copy stream), room for 2*L*k loads
};

namespace {

int validate_cfg(const odmoe_config* c) {
  if (!c) return fail(ODMOE_EINVAL, "cfg is NULL");
  if (c->hidden <= 0 || c->ffn <= 0 || c->hidden % 8 || c->ffn % 8)
    return fail(ODMOE_EINVAL, "hidden (%d) and ffn (%d) must be positive multiples of 8", c->hidden, c->ffn);
  if (c->n_experts < 1 || c->n_experts > ODMOE_MAX_EXPERTS)
    return fail(ODMOE_EINVAL, "n_experts %d out of range [1, %d]", c->n_experts, ODMOE_MAX_EXPERTS);
  if (c->top_k < 1 || c->top_k > ODMOE_MAX_TOPK || c->top_k > c->n_experts)
    return fail(ODMOE_EINVAL, "top_k %d out of range [1, min(E, %d)]", c->top_k, ODMOE_MAX_TOPK);
  if (c->n_layers < 1) return fail(ODMOE_EINVAL, "n_layers %d < 1", c->n_layers);
  if (c->n_slots < 0 || (c->n_slots > 0 && c->n_slots < c->top_k))
    return fail(ODMOE_EINVAL, "n_slots %d must be 0 (resident) or >= top_k", c->n_slots);
  if (c->dtype != ODMOE_F32 && c->dtype != ODMOE_BF16) return fail(ODMOE_EINVAL, "bad dtype %d", c->dtype);
  if (c->glue != 0 && c->glue != 1) return fail(ODMOE_EINVAL, "bad glue %d", c->glue);
  if (c->expert_quant < ODMOE_Q_NONE || c->expert_quant > ODMOE_Q_F16)
    return fail(ODMOE_EINVAL,
                "expert_quant %d: experts are stored in dtype (0), as int8 rows (1), 4-bit groups (2) or binary16 (3)",
                c->expert_quant);
  if (c->expert_quant == ODMOE_Q_F16) {
    Shape sh{c->hidden, c->ffn, c->n_experts, c->top_k, c->dtype};
    if (!f16_supported(sh))
      return fail(ODMOE_EINVAL, "binary16 experts need dtype fp32, hidden (%d) <= 8192 and ffn (%d) <= 32768",
                  c->hidden, c->ffn);
  }
  if (c->expert_quant == ODMOE_Q_INT4_G64 && (c->hidden % 64 || c->ffn % 64 || c->hidden > 8192))
    return fail(ODMOE_EINVAL, "4-bit experts need hidden (%d) and ffn (%d) to be multiples of 64 and hidden <= 8192",
                c->hidden, c->ffn);
  if (c->expert_quant == ODMOE_Q_INT8_ROW && (c->hidden % 16 || c->ffn % 16 || c->hidden > 8192))
    return fail(ODMOE_EINVAL, "int8 experts need hidden (%d) and ffn (%d) to be multiples of 16 and hidden <= 8192",
                c->hidden, c->ffn);
  // the GEMV kernels keep one fp32 input vector in LDS (160 KB per workgroup on gfx950)
  const long max_vec = 160 * 1024 / 4;
  const long chunk = c->dtype == ODMOE_F32 ? 256 : 512;
  if (((c->hidden + chunk - 1) / chunk) * chunk > max_vec || ((c->ffn + chunk - 1) / chunk) * chunk > max_vec)
    return fail(ODMOE_EINVAL, "hidden/ffn above %ld elements do not fit the LDS-staged GEMV", max_vec);
  return ODMOE_OK;
}

void free_all(odmoe_layer* h) {
  if (!h) return;
  for (auto e : h->ready_ev) if (e) (void)hipEventDestroy(e);
  for (auto e : h->done_ev) if (e) (void)hipEventDestroy(e);
  for (auto e : h->tev) if (e) (void)hipEventDestroy(e);
  for (auto e : h->lev) if (e) (void)hipEventDestroy(e);
  if (h->route_ev) (void)hipEventDestroy(h->route_ev);
  if (h->pool_mem) (void)hipFree(h->pool_mem);
  if (h->table_dev) (void)hipFree((void*)h->table_dev);
  if (h->hbuf) (void)hipFree(h->hbuf);
  if (h->xbuf[0]) (void)hipFree(h->xbuf[0]);
  if (h->xbuf[1]) (void)hipFree(h->xbuf[1]);
  if (h->ybuf) (void)hipFree(h->ybuf);
  if (h->idx_dev) (void)hipFree(h->idx_dev);
  if (h->gate_dev) (void)hipFree(h->gate_dev);
  if (h->eptr_dev) (void)hipFree((void*)h->eptr_dev);
  if (h->route_scratch.logits) (void)hipFree(h->route_scratch.logits);
  if (h->route_scratch.counters) (void)hipFree(h->route_scratch.counters);
  if (h->idx_pin) (void)hipHostFree(h->idx_pin);
  if (h->prefill_ws) (void)hipFree(h->prefill_ws);
  if (h->own_copy)
    for (hipStream_t cs : h->copy_ring) if (cs) (void)hipStreamDestroy(cs);
  delete h->sched;
  delete h->pool;
  delete h;
}

int check_layer(const odmoe_layer* h, int32_t layer) {
  if (!h) return fail(ODMOE_EINVAL, "handle is NULL");
  if (layer < 0 || layer >= h->cfg.n_layers)
    return fail(ODMOE_EINVAL, "layer %d out of range [0, %d)", layer, h->cfg.n_layers);
  return ODMOE_OK;
}

// Enqueue the copy of (layer, expert) into `slot` on the copy stream.
int enqueue_load(odmoe_layer* h, int32_t layer, int32_t expert, int32_t slot, hipEvent_t t0 = nullptr,
                 hipEvent_t t1 = nullptr) {
  const size_t n_ring = (h->ring_active && h->ring_active < h->copy_ring.size()) ? h->ring_active : h->copy_ring.size();
  hipStream_t cs = h->copy_ring[h->next_copy++ % n_ring];
  // The copy must come after the kernels that last read the slot and after an earlier copy into
  // it (possibly on another stream, possibly never read).  Both are usually long done by now (the
  // slot was used two layers ago): a wait is put on the stream only for an event that is still
  // pending, because every wait costs the copy queue about 5 us even when it is already satisfied.
  auto wait_if_pending = [&](hipEvent_t ev) -> hipError_t {
    const hipError_t q = hipEventQuery(ev);
    if (q == hipSuccess) return hipSuccess;
    if (q != hipErrorNotReady) return q;
    (void)hipGetLastError();  // "not ready" is an answer, not a failure
    return hipStreamWaitEvent(cs, ev, 0);
  };
  if (h->done_pending[slot]) {
    HIP_TRY(wait_if_pending(h->done_ev[slot]));
    h->done_pending[slot] = 0;
  }
  if (h->copied_once[slot] && h->copy_ring.size() > 1) HIP_TRY(wait_if_pending(h->ready_ev[slot]));
  const void* src = h->expert_w[(size_t)layer * h->cfg.n_experts + expert];
  if (t0) HIP_TRY(hipEventRecord(t0, cs));
  HIP_TRY(hipMemcpyAsync(h->pool_mem + (size_t)slot * h->expert_bytes, src, h->expert_bytes,
                         hipMemcpyHostToDevice, cs));
  if (t1) HIP_TRY(hipEventRecord(t1, cs));
  HIP_TRY(hipEventRecord(h->ready_ev[slot], cs));
  h->copied_once[slot] = 1;
  return ODMOE_OK;
}

// The kernels that read `slot` have been enqueued on the compute stream: the slot may be
// overwritten once they are done.
int mark_used(odmoe_layer* h, int32_t slot) {
  HIP_TRY(hipEventRecord(h->done_ev[slot], h->compute));
  h->done_pending[slot] = 1;
  return ODMOE_OK;
}

int ensure_prefill_ws(odmoe_layer* h, int32_t n_tokens) {
  const size_t need = prefill_workspace_bytes(h->sh, n_tokens);
  if (need > h->prefill_ws_bytes) {
    if (h->prefill_ws) HIP_TRY(hipFree(h->prefill_ws));  // hipFree waits for the device
    h->prefill_ws = nullptr;
    h->prefill_ws_bytes = 0;
    hipError_t e = hipMalloc(&h->prefill_ws, need);
    if (e != hipSuccess)
      return fail(ODMOE_ENOMEM, "prefill workspace of %zu bytes: %s", need, hipGetErrorString(e));
    h->prefill_ws_bytes = need;
  }
  return ODMOE_OK;
}

int run_ffn_one_token(odmoe_layer* h, const ExpertSrc& src, const int32_t* idx_dev,
                      const float* gate_dev, const void* x, void* y, hipEvent_t between = nullptr) {
  HIP_TRY(launch_ffn_up(h->compute, h->sh, src, idx_dev, x, h->hbuf));
  if (between) HIP_TRY(hipEventRecord(between, h->compute));
  HIP_TRY(launch_ffn_down(h->compute, h->sh, src, idx_dev, gate_dev, h->hbuf, y));
  return ODMOE_OK;
}

// A cacheless call failed after it had taken slots.  Everything in flight is waited for (the
// kernels that may still read a slot, the copies that may still write one) and every slot is
// freed, so the handle can be used again.  Errors of the waits are not reported: the call
// already has one.
void abandon_slots(odmoe_layer* h) {
  if (!h || !h->pool) return;
  (void)hipStreamSynchronize(h->compute);
  for (hipStream_t cs : h->copy_ring) (void)hipStreamSynchronize(cs);
  (void)hipGetLastError();
  h->pool->release_all();
  std::fill(h->done_pending.begin(), h->done_pending.end(), 0);
}

// ---------------------------------------------------------------------------------------------
// Device memory of the entry point that allocates nothing (odmoe_expert_ffn_static): the fp32
// SwiGLU intermediate h[k, F] of one token.  Every GPU holds its own copy of the array for as long
// as the process lives; host code never uses the array's name as an address, only the per-device
// pointer hipGetSymbolAddress gives.
// ---------------------------------------------------------------------------------------------
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)1 << 20;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
void* g_scratch_ptr[STATIC_MAX_DEVICES];   // address of `scratch` on each device, once known

}  // namespace

extern "C" {

const char* odmoe_last_error(void) { return g_err; }
const char* odmoe_version(void) { return "odmoe 0.1 (gfx950)"; }

uint64_t odmoe_expert_bytes(const odmoe_config* cfg) {
  if (!cfg || validate_cfg(cfg) != ODMOE_OK) return 0;
  return expert_bytes_of(*cfg);
}

int odmoe_quantize(const void* w_dev, int32_t dtype, int64_t rows, int64_t cols, int32_t kind,
                   uint8_t* code_dev, float* scale_dev, void* dequant_dev, void* stream) {
  if (!w_dev) return fail(ODMOE_EINVAL, "w is NULL");
  if (dtype != ODMOE_F32 && dtype != ODMOE_BF16) return fail(ODMOE_EINVAL, "bad dtype %d", dtype);
  if (rows < 0 || cols < 0) return fail(ODMOE_EINVAL, "rows / cols negative");
  if (kind != ODMOE_Q_INT8_ROW && kind != ODMOE_Q_INT4_G64 && kind != ODMOE_Q_F16)
    return fail(ODMOE_EINVAL, "bad quantisation kind %d", kind);
  if (kind == ODMOE_Q_INT4_G64 && cols % 64) return fail(ODMOE_EINVAL, "cols (%lld) must be a multiple of 64", (long long)cols);
  if (rows > 0x7fffffffLL) return fail(ODMOE_EINVAL, "too many rows");
  if (kind == ODMOE_Q_F16) {
    if (scale_dev) return fail(ODMOE_EINVAL, "binary16 weights have no scales: scale_dev must be NULL");
    if (reinterpret_cast<uintptr_t>(code_dev) & 1u) return fail(ODMOE_EINVAL, "code_dev must be 2-byte aligned");
    HIP_TRY(launch_round_f16(static_cast<hipStream_t>(stream), w_dev, dtype, (size_t)rows * (size_t)cols,
                             reinterpret_cast<uint16_t*>(code_dev), dequant_dev));
    return ODMOE_OK;
  }
  HIP_TRY(launch_quantize(static_cast<hipStream_t>(stream), w_dev, dtype, rows, cols, kind, code_dev, scale_dev,
                          dequant_dev));
  return ODMOE_OK;
}

int odmoe_quantize_expert(const odmoe_config* cfg, int32_t kind, const void* expert_dev, void* dst_dev,
                          void* stream) {
  if (!cfg) return fail(ODMOE_EINVAL, "cfg is NULL");
  if (kind != ODMOE_Q_INT8_ROW && kind != ODMOE_Q_INT4_G64 && kind != ODMOE_Q_F16)
    return fail(ODMOE_EINVAL, "bad quantisation kind %d", kind);
  odmoe_config qc = *cfg;
  qc.expert_quant = kind;
  int rc = validate_cfg(&qc);
  if (rc) return rc;
  if (!expert_dev || !dst_dev) return fail(ODMOE_EINVAL, "expert / dst is NULL");
  const size_t H = cfg->hidden, F = cfg->ffn, hf = H * F, es = dtype_size(cfg->dtype);
  const char* src = static_cast<const char*>(expert_dev);
  uint8_t* code = static_cast<uint8_t*>(dst_dev);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int dt = cfg->dtype;
  if (kind == ODMOE_Q_INT8_ROW) {
    float* scale = reinterpret_cast<float*>(code + 3 * hf);
    HIP_TRY(launch_quantize(s, src, dt, F, H, kind, code, scale, nullptr));                             // W1
    HIP_TRY(launch_quantize(s, src + hf * es, dt, F, H, kind, code + hf, scale + F, nullptr));          // W3
    HIP_TRY(launch_quantize(s, src + 2 * hf * es, dt, H, F, kind, code + 2 * hf, scale + 2 * F, nullptr));  // W2
  } else if (kind == ODMOE_Q_F16) {
    HIP_TRY(launch_round_f16(s, src, dt, 3 * hf, reinterpret_cast<uint16_t*>(dst_dev), nullptr));
  } else {
    float* scale = reinterpret_cast<float*>(code + 3 * hf / 2);
    const size_t ng = hf / 64;   // groups (= scales) per matrix
    HIP_TRY(launch_quantize_pack4(s, src, dt, F, H, code, scale));                                       // W1
    HIP_TRY(launch_quantize_pack4(s, src + hf * es, dt, F, H, code + hf / 2, scale + ng));               // W3
    HIP_TRY(launch_quantize_pack4(s, src + 2 * hf * es, dt, H, F, code + hf, scale + 2 * ng));           // W2
  }
  return ODMOE_OK;
}

int odmoe_pinned_alloc(uint64_t bytes, void** out_host) {
  if (!out_host || bytes == 0) return fail(ODMOE_EINVAL, "bad arguments");
  *out_host = nullptr;
  hipError_t e = hipHostMalloc(out_host, bytes, hipHostMallocDefault);
  if (e != hipSuccess) {
    *out_host = nullptr;
    return fail(ODMOE_ENOMEM, "hipHostMalloc(%llu) failed: %s", (unsigned long long)bytes, hipGetErrorString(e));
  }
  return ODMOE_OK;
}

int odmoe_pinned_free(void* host) {
  if (!host) return ODMOE_OK;
  HIP_TRY(hipHostFree(host));
  return ODMOE_OK;
}

int odmoe_probe_hbm(void* dst_dev, const void* src_dev, uint64_t bytes, int32_t mode, void* stream) {
  if (!dst_dev || !src_dev) return fail(ODMOE_EINVAL, "dst/src is NULL");
  if (bytes % 16) return fail(ODMOE_EINVAL, "bytes must be a multiple of 16");
  if (mode != 0 && mode != 1) return fail(ODMOE_EINVAL, "mode must be 0 (copy) or 1 (read)");
  HIP_TRY(launch_probe(static_cast<hipStream_t>(stream), dst_dev, src_dev, bytes, mode));
  return ODMOE_OK;
}

int odmoe_time_decode_kernels(odmoe_layer_t* h, int32_t layer, const void* x_dev, int32_t n_tokens,
                              int32_t reps, float* route_us, float* ffn_up_us, float* ffn_down_us) {
  int rc = check_layer(h, layer);
  if (rc) return rc;
  if (h->pool) return fail(ODMOE_EINVAL, "resident mode only");
  if (!x_dev || n_tokens < 1 || reps < 1 || !route_us || !ffn_up_us || !ffn_down_us)
    return fail(ODMOE_EINVAL, "bad arguments");
  const int k = h->cfg.top_k;
  const size_t row = (size_t)h->cfg.hidden * h->esize;
  int32_t* idx = nullptr;
  float* gate = nullptr;
  void* y = nullptr;
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  auto cleanup = [&]() {
    if (idx) (void)hipFree(idx);
    if (gate) (void)hipFree(gate);
    if (y) (void)hipFree(y);
    for (auto e : ev) if (e) (void)hipEventDestroy(e);
  };
#define T_TRY(expr)                                                                              \
  do {                                                                                           \
    hipError_t e__ = (expr);                                                                     \
    if (e__ != hipSuccess) {                                                                     \
      cleanup();                                                                                 \
      return fail(ODMOE_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
    }                                                                                            \
  } while (0)
  T_TRY(hipMalloc(&idx, (size_t)n_tokens * k * sizeof(int32_t)));
  T_TRY(hipMalloc(&gate, (size_t)n_tokens * k * sizeof(float)));
  T_TRY(hipMalloc(&y, row));
  for (auto& e : ev) T_TRY(hipEventCreate(&e));
  ExpertSrc src{};
  src.table = h->table_dev;
  src.table_off = layer * h->cfg.n_experts;
  src.n_experts = h->cfg.n_experts;
  const float* bias = static_cast<const float*>(h->router_b[layer]);
  // warm-up + the routing every later launch uses
  T_TRY(launch_route_topk(h->compute, h->sh, h->router_w[layer], bias, x_dev, n_tokens, idx, gate, nullptr,
                          nullptr, 0, nullptr, &h->route_scratch));
  T_TRY(hipEventRecord(ev[0], h->compute));
  for (int r = 0; r < reps; ++r)
    for (int t = 0; t < n_tokens; ++t)
      T_TRY(launch_route_topk(h->compute, h->sh, h->router_w[layer], bias,
                              static_cast<const char*>(x_dev) + t * row, 1, idx + (size_t)t * k,
                              gate + (size_t)t * k, nullptr, nullptr, 0, nullptr, &h->route_scratch));
  T_TRY(hipEventRecord(ev[1], h->compute));
  for (int r = 0; r < reps; ++r)
    for (int t = 0; t < n_tokens; ++t)
      T_TRY(launch_ffn_up(h->compute, h->sh, src, idx + (size_t)t * k,
                          static_cast<const char*>(x_dev) + t * row, h->hbuf));
  T_TRY(hipEventRecord(ev[2], h->compute));
  for (int r = 0; r < reps; ++r)
    for (int t = 0; t < n_tokens; ++t)
      T_TRY(launch_ffn_down(h->compute, h->sh, src, idx + (size_t)t * k, gate + (size_t)t * k, h->hbuf, y));
  T_TRY(hipEventRecord(ev[3], h->compute));
  T_TRY(hipEventSynchronize(ev[3]));
  float ms[3];
  for (int i = 0; i < 3; ++i) T_TRY(hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]));
#undef T_TRY
  const float n = (float)reps * (float)n_tokens;
  *route_us = ms[0] * 1e3f / n;
  *ffn_up_us = ms[1] * 1e3f / n;
  *ffn_down_us = ms[2] * 1e3f / n;
  cleanup();
  return ODMOE_OK;
}

int odmoe_time_expert_loads(odmoe_layer_t* h, int32_t n_tokens, float* ms_per_token) {
  if (!h || !ms_per_token) return fail(ODMOE_EINVAL, "NULL argument");
  if (!h->pool) return fail(ODMOE_EINVAL, "resident mode has no expert loads");
  if (n_tokens <= 0) return fail(ODMOE_EINVAL, "n_tokens = %d", n_tokens);
  const int S = h->cfg.n_slots, L = h->cfg.n_layers, k = h->cfg.top_k, E = h->cfg.n_experts;
  if (h->pool->n_free() != S) return fail(ODMOE_ESTATE, "an expert holds a slot");
  HIP_TRY(hipStreamSynchronize(h->compute));
  for (hipStream_t cs : h->copy_ring) HIP_TRY(hipStreamSynchronize(cs));
  const auto t0 = std::chrono::steady_clock::now();
  int slot = 0;
  for (int t = 0; t < n_tokens; ++t)
    for (int l = 0; l < L; ++l)
      for (int i = 0; i < k; ++i) {
        const int rc = enqueue_load(h, l, (l * k + i) % E, slot);
        if (rc) return rc;
        slot = slot + 1 == S ? 0 : slot + 1;
      }
  for (hipStream_t cs : h->copy_ring) HIP_TRY(hipStreamSynchronize(cs));
  *ms_per_token =
      std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count() / n_tokens;
  return ODMOE_OK;
}

double odmoe_load_window_ms(int32_t n_groups, double t_main_ms, double t_worker_ms) {
  if (n_groups < 1) return 0.0;
  return n_groups * t_main_ms + (n_groups - 1) * t_worker_ms;
}

int32_t odmoe_slot_groups(const odmoe_layer_t* h) {
  return h && h->pool ? h->cfg.n_slots / h->cfg.top_k : 0;
}

uint64_t odmoe_slot_pool_bytes(const odmoe_layer_t* h) {
  return h && h->pool ? (uint64_t)h->cfg.n_slots * h->expert_bytes : 0;
}

// `*made` receives the handle as soon as it exists, so that the caller can free it on any failure.
static int layer_init_impl(const odmoe_config* cfg, const void* const* router_w, const void* const* router_b,
                           const void* const* expert_w, void* compute_stream, void* copy_stream,
                           odmoe_layer** made) {
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  if (!router_w || !expert_w) return fail(ODMOE_EINVAL, "router_w / expert_w is NULL");
  const int L = cfg->n_layers, E = cfg->n_experts, k = cfg->top_k, S = cfg->n_slots;
  for (int l = 0; l < L; ++l)
    if (!router_w[l]) return fail(ODMOE_EINVAL, "router_w[%d] is NULL", l);
  for (long i = 0; i < (long)L * E; ++i)
    if (!expert_w[i]) return fail(ODMOE_EINVAL, "expert_w[%ld] is NULL", i);

  odmoe_layer* h = new (std::nothrow) odmoe_layer();
  if (!h) return fail(ODMOE_ENOMEM, "out of host memory");
  *made = h;
  h->cfg = *cfg;
  h->sh = Shape{cfg->hidden, cfg->ffn, E, k, cfg->dtype};
  h->sh.quant = cfg->expert_quant;
  h->esize = dtype_size(cfg->dtype);
  h->expert_bytes = expert_bytes_of(*cfg);
  h->compute = static_cast<hipStream_t>(compute_stream);
  h->router_w.assign(router_w, router_w + L);
  h->router_b.assign(L, nullptr);
  if (router_b) h->router_b.assign(router_b, router_b + L);
  h->expert_w.assign(expert_w, expert_w + (size_t)L * E);

#define INIT_TRY(expr, code)                                                                    \
  do {                                                                                          \
    hipError_t e__ = (expr);                                                                    \
    if (e__ != hipSuccess)                                                                      \
      return fail(code, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
  } while (0)

  INIT_TRY(kernels_init(), ODMOE_EHIP);
  // Where the expert buffers live.  The runtime knows every device allocation and every pinned host
  // allocation; memory it has never seen (plain malloc) cannot be read by a kernel and makes a
  // copy synchronous, so it is refused here instead of faulting later.  A failing query says
  // nothing and is ignored.
  for (size_t i = 0; i < h->expert_w.size(); ++i) {
    hipPointerAttribute_t attr{};
    if (hipPointerGetAttributes(&attr, h->expert_w[i]) != hipSuccess) {
      (void)hipGetLastError();
      continue;
    }
    if (attr.type == hipMemoryTypeUnregistered)
      return fail(ODMOE_EINVAL, "expert_w[%zu] is neither device memory nor pinned host memory", i);
    if (S > 0 && attr.type != hipMemoryTypeHost)
      return fail(ODMOE_EINVAL, "expert_w[%zu]: with n_slots > 0 the experts live in pinned host memory", i);
    if (S == 0 && attr.type == hipMemoryTypeHost) h->sh.host_link = 1;   // read in place over the host link
  }
  for (int l = 0; l < L; ++l)
    for (const void* p : {h->router_w[l], h->router_b[l]}) {
      hipPointerAttribute_t attr{};
      if (!p) continue;
      if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        continue;
      }
      if (attr.type == hipMemoryTypeUnregistered)
        return fail(ODMOE_EINVAL, "router weights / bias of layer %d are not in memory the GPU can read", l);
    }
  const size_t H = cfg->hidden, F = cfg->ffn;
  INIT_TRY(hipMalloc(&h->hbuf, (size_t)k * F * sizeof(float)), ODMOE_ENOMEM);
  INIT_TRY(hipMalloc(&h->xbuf[0], H * h->esize), ODMOE_ENOMEM);
  INIT_TRY(hipMalloc(&h->xbuf[1], H * h->esize), ODMOE_ENOMEM);
  INIT_TRY(hipMalloc(&h->ybuf, H * h->esize), ODMOE_ENOMEM);
  INIT_TRY(hipMalloc(&h->idx_dev, (size_t)L * k * sizeof(int32_t)), ODMOE_ENOMEM);
  if (h->cfg.n_experts > 8) {
    INIT_TRY(hipMalloc(&h->route_scratch.logits,
                       (size_t)ROUTE_SPLIT_MAX_TOKENS * h->cfg.n_experts * sizeof(float)), ODMOE_ENOMEM);
    INIT_TRY(hipMalloc(&h->route_scratch.counters, ROUTE_SPLIT_MAX_TOKENS * sizeof(int32_t)), ODMOE_ENOMEM);
    INIT_TRY(hipMemset(h->route_scratch.counters, 0, ROUTE_SPLIT_MAX_TOKENS * sizeof(int32_t)), ODMOE_EHIP);
    INIT_TRY(hipDeviceSynchronize(), ODMOE_EHIP);  // the fill is done before any stream uses the counters
    h->route_scratch.max_tokens = ROUTE_SPLIT_MAX_TOKENS;
  }
  INIT_TRY(hipMalloc(&h->gate_dev, (size_t)L * k * sizeof(float)), ODMOE_ENOMEM);
  INIT_TRY(hipHostMalloc((void**)&h->idx_pin, (size_t)L * k * sizeof(int32_t), hipHostMallocMapped | hipHostMallocCoherent),
           ODMOE_ENOMEM);
  INIT_TRY(hipHostGetDevicePointer((void**)&h->idx_pin_dev, h->idx_pin, 0), ODMOE_EHIP);
  INIT_TRY(hipEventCreateWithFlags(&h->route_ev, hipEventDisableTiming), ODMOE_EHIP);

  if (S == 0) {
    INIT_TRY(hipMalloc((void**)&h->eptr_dev, (size_t)L * k * sizeof(void*)), ODMOE_ENOMEM);
    INIT_TRY(hipMalloc((void**)&h->table_dev, (size_t)L * E * sizeof(void*)), ODMOE_ENOMEM);
    INIT_TRY(hipMemcpy((void*)h->table_dev, h->expert_w.data(), (size_t)L * E * sizeof(void*),
                       hipMemcpyHostToDevice),
             ODMOE_EHIP);
  } else {
    INIT_TRY(hipMalloc((void**)&h->pool_mem, (size_t)S * h->expert_bytes), ODMOE_ENOMEM);
    h->pool = new SlotPool(S);
    h->sched = new DecodeScheduler(L, E, k, h->pool);
    h->ready_ev.assign(S, nullptr);
    h->done_ev.assign(S, nullptr);
    h->done_pending.assign(S, 0);
    for (int s = 0; s < S; ++s) {
      INIT_TRY(hipEventCreateWithFlags(&h->ready_ev[s], hipEventDisableTiming), ODMOE_EHIP);
      INIT_TRY(hipEventCreateWithFlags(&h->done_ev[s], hipEventDisableTiming), ODMOE_EHIP);
    }
    h->copied_once.assign(S, 0);
    if (copy_stream) {
      h->copy = static_cast<hipStream_t>(copy_stream);
      h->copy_ring.push_back(h->copy);
    } else {
      h->own_copy = true;
      // Four streams, of which copies issued ahead of time (with hints) rotate over three: enough
      // concurrent copies to close the gaps between them, few enough that they still complete
      // roughly in issue order (with four, the experts of two consecutive top-2 layers load side
      // by side and finish together, after which both layers compute while the link idles).
      // ODMOE_COPY_STREAMS=1..8 fixes the number for every case.
      int n_copy_streams = 4;
      if (const char* v = getenv("ODMOE_COPY_STREAMS")) {
        const int n = atoi(v);
        if (n >= 1 && n <= 8) {
          n_copy_streams = n;
          h->ring_fixed = true;
        }
      }
      for (int i = 0; i < n_copy_streams; ++i) {
        hipStream_t cs = nullptr;
        INIT_TRY(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking), ODMOE_EHIP);
        h->copy_ring.push_back(cs);
      }
      h->copy = h->copy_ring[0];
    }
  }
#undef INIT_TRY
  return ODMOE_OK;
}

int odmoe_layer_init(const odmoe_config* cfg, const void* const* router_w, const void* const* router_b,
                     const void* const* expert_w, void* compute_stream, void* copy_stream,
                     odmoe_layer_t** out) {
  if (!out) return fail(ODMOE_EINVAL, "out is NULL");
  *out = nullptr;
  odmoe_layer* h = nullptr;
  const int rc = guarded(
      [&] { return layer_init_impl(cfg, router_w, router_b, expert_w, compute_stream, copy_stream, &h); });
  if (rc != ODMOE_OK) {
    free_all(h);
    return rc;
  }
  *out = h;
  return ODMOE_OK;
}

int odmoe_layer_destroy(odmoe_layer_t* h) {
  if (!h) return ODMOE_OK;
  hipError_t e1 = hipStreamSynchronize(h->compute);
  hipError_t e2 = hipSuccess;
  for (hipStream_t cs : h->copy_ring) {
    const hipError_t ec = hipStreamSynchronize(cs);
    if (ec != hipSuccess) e2 = ec;
  }
  free_all(h);
  if (e1 != hipSuccess) return fail(ODMOE_EHIP, "compute stream: %s", hipGetErrorString(e1));
  if (e2 != hipSuccess) return fail(ODMOE_EHIP, "copy stream: %s", hipGetErrorString(e2));
  return ODMOE_OK;
}

int odmoe_route_topk(odmoe_layer_t* h, int32_t layer, const void* x_dev, int32_t n_tokens,
                     int32_t* idx_dev, float* gate_dev) {
  int rc = check_layer(h, layer);
  if (rc) return rc;
  if (n_tokens < 0) return fail(ODMOE_EINVAL, "n_tokens %d < 0", n_tokens);
  if (n_tokens == 0) return ODMOE_OK;
  if (!x_dev || !idx_dev || !gate_dev) return fail(ODMOE_EINVAL, "x/idx/gate is NULL");
  HIP_TRY(launch_route_topk(h->compute, h->sh, h->router_w[layer],
                            static_cast<const float*>(h->router_b[layer]), x_dev, n_tokens, idx_dev,
                            gate_dev, nullptr, nullptr, 0, nullptr, &h->route_scratch));
  return ODMOE_OK;
}

int odmoe_expert_load_async(odmoe_layer_t* h, int32_t layer, int32_t expert, int32_t* slot_out) {
  int rc = check_layer(h, layer);
  if (rc) return rc;
  if (!h->pool) return fail(ODMOE_EINVAL, "resident mode: nothing to load");
  if (expert < 0 || expert >= h->cfg.n_experts)
    return fail(ODMOE_EINVAL, "expert %d out of range [0, %d)", expert, h->cfg.n_experts);
  int s = h->pool->find(layer, expert);
  if (s < 0) {
    s = h->pool->acquire(layer, expert);
    if (s < 0) return fail(ODMOE_EBUSY, "all %d slots are occupied", h->cfg.n_slots);
    rc = enqueue_load(h, layer, expert, s);
    if (rc) {
      h->pool->release(s);
      return rc;
    }
  }
  if (slot_out) *slot_out = s;
  return ODMOE_OK;
}

int odmoe_expert_evict(odmoe_layer_t* h, int32_t layer, int32_t expert) {
  int rc = check_layer(h, layer);
  if (rc) return rc;
  if (!h->pool) return fail(ODMOE_EINVAL, "resident mode: nothing to evict");
  int s = h->pool->find(layer, expert);
  if (s < 0) return fail(ODMOE_ESTATE, "expert (%d, %d) holds no slot", layer, expert);
  h->pool->release(s);
  return ODMOE_OK;
}

static int expert_ffn_impl(odmoe_layer_t* h, int32_t layer, const int32_t* idx_dev, const float* gate_dev,
                           const int32_t* idx_host, const void* x_dev, int32_t n_tokens, void* y_dev,
                           int32_t evict_after) {
  int rc = check_layer(h, layer);
  if (rc) return rc;
  if (n_tokens < 0) return fail(ODMOE_EINVAL, "n_tokens %d < 0", n_tokens);
  if (n_tokens == 0) return ODMOE_OK;
  if (!idx_dev || !gate_dev || !x_dev || !y_dev) return fail(ODMOE_EINVAL, "idx/gate/x/y is NULL");
  const int k = h->cfg.top_k, E = h->cfg.n_experts;
  const size_t row = (size_t)h->cfg.hidden * h->esize;

  if (!h->pool) {  // resident
    ExpertSrc src{};
    src.table = h->table_dev;
    src.table_off = layer * E;
    src.n_experts = E;
    // Tokens grouped by expert read each expert once; token by token reads k experts per token:
    // grouping pays as soon as the token-slots outnumber the experts (and always from 16 tokens).
    if ((n_tokens >= 16 || (int64_t)n_tokens * k > E) && prefill_supported(h->sh) && !h->sh.quant) {
      if ((rc = ensure_prefill_ws(h, n_tokens))) return rc;
      HIP_TRY(launch_prefill(h->compute, h->sh, h->table_dev, layer * E, idx_dev, gate_dev, x_dev,
                             n_tokens, y_dev, h->prefill_ws, h->prefill_ws_bytes));
      return ODMOE_OK;
    }
    for (int t = 0; t < n_tokens; ++t) {
      rc = run_ffn_one_token(h, src, idx_dev + (size_t)t * k, gate_dev + (size_t)t * k,
                             static_cast<const char*>(x_dev) + t * row, static_cast<char*>(y_dev) + t * row);
      if (rc) return rc;
    }
    return ODMOE_OK;
  }

  // cacheless prefill (paper Section 3.3 on one GPU): every expert that received tokens is
  // streamed from host memory into a slot exactly once, its grouped GEMMs run as soon as its
  // copy has landed, and the slot is handed to the next expert: with S >= 2 slots the copy of
  // the next expert overlaps the GEMMs of the current one.
  if (n_tokens >= 2) {
    if (!prefill_supported(h->sh) || h->sh.quant)
      return fail(ODMOE_EINVAL, "cacheless batches need hidden and ffn to be multiples of 64 and experts stored in dtype");
    if ((rc = ensure_prefill_ws(h, n_tokens))) return rc;
    const size_t n = (size_t)n_tokens * k;
    std::vector<int32_t> ids_all(n);
    if (idx_host) {
      memcpy(ids_all.data(), idx_host, n * sizeof(int32_t));
    } else {
      HIP_TRY(hipMemcpyAsync(ids_all.data(), idx_dev, n * sizeof(int32_t), hipMemcpyDeviceToHost, h->compute));
      HIP_TRY(hipStreamSynchronize(h->compute));
    }
    std::vector<int32_t> count(E, 0);
    for (size_t i = 0; i < n; ++i)
      if (ids_all[i] >= 0 && ids_all[i] < E) ++count[ids_all[i]];
    HIP_TRY(prefill_sort(h->compute, h->sh, idx_dev, n_tokens, h->prefill_ws, h->prefill_ws_bytes));
    std::vector<int32_t> order(E);
    prefill_expert_order(count.data(), E, order.data());   // the order of the device's chunk list
    // Slots this call took and still holds: a failure part-way gives them back (the kernels
    // that read them are waited for first), so that the handle stays usable.
    std::vector<int> taken;
    auto stream_experts = [&]() -> int {
      int tile_first = 0;
      for (int p = 0; p < E; ++p) {
        const int e = order[p];
        const int tiles_e = prefill_chunks_of(count[e]);
        if (tiles_e == 0) continue;
        int s = h->pool->find(layer, e);
        if (s < 0) {
          s = h->pool->acquire(layer, e);
          if (s < 0) return fail(ODMOE_EBUSY, "all %d slots are occupied", h->cfg.n_slots);
          taken.push_back(s);
          if ((rc = enqueue_load(h, layer, e, s))) return rc;
        }
        HIP_TRY(hipStreamWaitEvent(h->compute, h->ready_ev[s], 0));
        HIP_TRY(prefill_gemms(h->compute, h->sh, nullptr, 0, h->pool_mem + (size_t)s * h->expert_bytes,
                              tile_first, tiles_e, x_dev, n_tokens, h->prefill_ws));
        if ((rc = mark_used(h, s))) return rc;
        if (evict_after && h->pool->release(s)) taken.erase(std::remove(taken.begin(), taken.end(), s), taken.end());
        tile_first += tiles_e;
      }
      HIP_TRY(prefill_combine(h->compute, h->sh, gate_dev, n_tokens, y_dev, h->prefill_ws));
      return ODMOE_OK;
    };
    rc = stream_experts();
    if (rc != ODMOE_OK) {
      (void)hipStreamSynchronize(h->compute);
      for (hipStream_t cs : h->copy_ring) (void)hipStreamSynchronize(cs);
      (void)hipGetLastError();
      for (int s : taken) h->pool->release(s);
    }
    return rc;
  }

  // cacheless decode (n_tokens == 1)
  int32_t ids[ODMOE_MAX_TOPK];
  if (idx_host) {
    memcpy(ids, idx_host, k * sizeof(int32_t));
  } else {
    HIP_TRY(hipMemcpyAsync(h->idx_pin, idx_dev, k * sizeof(int32_t), hipMemcpyDeviceToHost, h->compute));
    HIP_TRY(hipStreamSynchronize(h->compute));
    memcpy(ids, h->idx_pin, k * sizeof(int32_t));
  }
  ExpertSrc src{};
  int32_t slots[ODMOE_MAX_TOPK];
  for (int i = 0; i < k; ++i) {
    if (ids[i] < 0 || ids[i] >= E) return fail(ODMOE_EINVAL, "idx[%d] = %d out of range", i, ids[i]);
    slots[i] = h->pool->find(layer, ids[i]);
    if (slots[i] < 0)
      return fail(ODMOE_ESTATE, "expert (%d, %d) is neither loading nor ready", layer, ids[i]);
    src.slot[i] = h->pool_mem + (size_t)slots[i] * h->expert_bytes;
  }
  for (int i = 0; i < k; ++i) HIP_TRY(hipStreamWaitEvent(h->compute, h->ready_ev[slots[i]], 0));
  rc = run_ffn_one_token(h, src, idx_dev, gate_dev, x_dev, y_dev);
  if (rc) return rc;
  for (int i = 0; i < k; ++i) {
    rc = mark_used(h, slots[i]);
    if (rc) return rc;
    if (evict_after) h->pool->release(slots[i]);
  }
  return ODMOE_OK;
}

int odmoe_expert_ffn(odmoe_layer_t* h, int32_t layer, const int32_t* idx_dev, const float* gate_dev,
                     const int32_t* idx_host, const void* x_dev, int32_t n_tokens, void* y_dev,
                     int32_t evict_after) {
  return guarded(
      [&] { return expert_ffn_impl(h, layer, idx_dev, gate_dev, idx_host, x_dev, n_tokens, y_dev, evict_after); });
}

static int decode_step_impl(odmoe_layer_t* h, const void* x_dev, void* y_dev,
                            const int32_t* predicted_idx_host, int32_t* idx_out_host, odmoe_stats* stats) {
  if (!h) return fail(ODMOE_EINVAL, "handle is NULL");
  if (!x_dev || !y_dev) return fail(ODMOE_EINVAL, "x/y is NULL");
  const int L = h->cfg.n_layers, k = h->cfg.top_k, E = h->cfg.n_experts;
  const bool timed = stats && stats->t_step_ms < 0.f;
  const auto wall0 = std::chrono::steady_clock::now();
  if (timed && h->tev.empty()) {
    // all or nothing: a failure part-way leaves no half-made set behind for the next call
    std::vector<hipEvent_t> made((size_t)5 * L + (h->pool ? (size_t)4 * L * k : 0), nullptr);
    for (auto& e : made) {
      const hipError_t rc_ev = hipEventCreate(&e);
      if (rc_ev != hipSuccess) {
        for (auto m : made) if (m) (void)hipEventDestroy(m);
        return fail(ODMOE_EHIP, "hipEventCreate failed: %s", hipGetErrorString(rc_ev));
      }
    }
    h->tev.assign(made.begin(), made.begin() + (size_t)5 * L);
    h->lev.assign(made.begin() + (size_t)5 * L, made.end());
  }
  auto TE = [&](int l, int which) -> hipEvent_t { return timed ? h->tev[(size_t)l * 5 + which] : nullptr; };
  size_t n_lev = 0;  // load events used

  uint64_t n_loads = 0, n_reloads = 0, n_hits = 0;
  if (h->sched) h->sched->begin_token(predicted_idx_host);
  if (!h->ring_fixed) h->ring_active = predicted_idx_host ? 3 : 0;
  std::vector<Action> acts;
  int rc;

  auto run_actions = [&]() -> int {
    for (const Action& a : acts) {
      if (a.kind == Action::LOAD) {
        hipEvent_t t0 = nullptr, t1 = nullptr;
        if (timed && n_lev + 2 <= h->lev.size()) {
          t0 = h->lev[n_lev];
          t1 = h->lev[n_lev + 1];
          n_lev += 2;
        }
        int r = enqueue_load(h, a.layer, a.expert, a.slot, t0, t1);
        if (r) return r;
      }
      // DROP: the slot was never read by a kernel; the next copy into it is ordered behind
      // this one on the copy stream.  RELEASE is handled by the caller (needs the event).
    }
    acts.clear();
    return ODMOE_OK;
  };

  // Between stacked layers the glue x_{l+1} = rmsnorm(x_l + y_l) runs at the head of layer l+1's
  // router kernel (one launch fewer per layer; the same bits as the stand-alone glue kernel, which
  // still closes the last layer and serves hidden sizes too long for the router's LDS).
  const bool fuse_glue = h->cfg.glue && route_glue_fusable(h->sh);
  const void* cur = x_dev;          // x_l: the input of layer l
  const void* pend_x = nullptr;     // glue still to be done before layer l: x_{l-1} ...
  const void* pend_y = nullptr;     // ... and y_{l-1}
  for (int l = 0; l < L; ++l) {
    const bool last = (l == L - 1);
    int32_t* idx_l = h->idx_dev + (size_t)l * k;
    float* gate_l = h->gate_dev + (size_t)l * k;
    if (h->sched) {
      h->sched->before_route(l, acts);
      if ((rc = run_actions())) return rc;
    }
    if (timed) HIP_TRY(hipEventRecord(TE(l, 0), h->compute));
    void* x_made = pend_x ? h->xbuf[(l - 1) & 1] : nullptr;   // where the pending glue puts x_l
    HIP_TRY(launch_route_topk(h->compute, h->sh, h->router_w[l], static_cast<const float*>(h->router_b[l]),
                              cur, 1, idx_l, gate_l, h->idx_pin_dev + (size_t)l * k, h->table_dev, l * E,
                              h->sched ? nullptr : h->eptr_dev + (size_t)l * k, &h->route_scratch, pend_x, pend_y,
                              x_made));
    if (pend_x) cur = x_made;
    pend_x = pend_y = nullptr;

    ExpertSrc src{};
    int32_t slots[ODMOE_MAX_TOPK];
    const int32_t* ids = h->idx_pin + (size_t)l * k;
    if (h->sched) {
      // the host has to learn which experts to copy: the one per-layer synchronisation
      HIP_TRY(hipEventRecord(h->route_ev, h->compute));
      HIP_TRY(hipEventSynchronize(h->route_ev));
      for (int i = 0; i < k; ++i)
        if (ids[i] < 0 || ids[i] >= E) return fail(ODMOE_EHIP, "router produced expert %d", ids[i]);
      if (!h->sched->after_route(l, ids, acts, slots)) return fail(ODMOE_EBUSY, "no slot for layer %d", l);
      if ((rc = run_actions())) return rc;
      for (int i = 0; i < k; ++i) {
        src.slot[i] = h->pool_mem + (size_t)slots[i] * h->expert_bytes;
        HIP_TRY(hipStreamWaitEvent(h->compute, h->ready_ev[slots[i]], 0));
      }
    } else {
      src.table = h->table_dev;
      src.table_off = l * E;
      src.n_experts = E;
      src.resolved = h->eptr_dev + (size_t)l * k;
    }

    void* y_l = (h->cfg.glue == 0) ? (last ? y_dev : h->xbuf[l & 1]) : h->ybuf;
    if (timed) HIP_TRY(hipEventRecord(TE(l, 1), h->compute));
    if ((rc = run_ffn_one_token(h, src, idx_l, gate_l, cur, y_l, TE(l, 2)))) return rc;
    if (timed) HIP_TRY(hipEventRecord(TE(l, 3), h->compute));

    if (h->sched) {
      h->sched->after_compute(l, ids, acts);
      for (const Action& a : acts)
        if (a.kind == Action::RELEASE && (rc = mark_used(h, a.slot))) return rc;
      acts.clear();
    }
    if (h->cfg.glue) {
      if (fuse_glue && !last) {
        pend_x = cur;      // done by the next layer's router kernel
        pend_y = y_l;
      } else {
        void* x_next = last ? y_dev : h->xbuf[l & 1];
        HIP_TRY(launch_glue(h->compute, h->sh, cur, y_l, x_next));
        cur = x_next;
      }
    } else {
      cur = y_l;
    }
    if (timed) HIP_TRY(hipEventRecord(TE(l, 4), h->compute));
  }
  // resident mode with nothing to report stays asynchronous on the compute stream
  if (h->sched || idx_out_host || stats) HIP_TRY(hipStreamSynchronize(h->compute));
  if (h->sched) {
    n_loads = h->sched->loads;
    n_reloads = h->sched->reloads;
    n_hits = h->sched->hint_hits;
  }
  if (idx_out_host) memcpy(idx_out_host, h->idx_pin, (size_t)L * k * sizeof(int32_t));
  if (stats) {
    stats->t_route_ms = stats->t_load_ms = stats->t_ffn_up_ms = stats->t_ffn_down_ms = stats->t_glue_ms = 0.f;
    if (timed) {
      for (hipStream_t cs : h->copy_ring) HIP_TRY(hipStreamSynchronize(cs));
      for (int l = 0; l < L; ++l) {
        float ms = 0.f;
        // route includes, in cacheless mode, the wait for this layer's expert copies
        HIP_TRY(hipEventElapsedTime(&ms, TE(l, 0), TE(l, 1)));
        stats->t_route_ms += ms;
        HIP_TRY(hipEventElapsedTime(&ms, TE(l, 1), TE(l, 2)));
        stats->t_ffn_up_ms += ms;
        HIP_TRY(hipEventElapsedTime(&ms, TE(l, 2), TE(l, 3)));
        stats->t_ffn_down_ms += ms;
        HIP_TRY(hipEventElapsedTime(&ms, TE(l, 3), TE(l, 4)));
        stats->t_glue_ms += ms;
      }
      // time during which at least one expert copy was in flight: union of the copies'
      // [begin, end] intervals (they overlap when they run on different copy streams)
      std::vector<std::pair<float, float>> iv;
      for (size_t i = 0; i + 1 < n_lev; i += 2) {
        float b = 0.f, e = 0.f;
        if (i) HIP_TRY(hipEventElapsedTime(&b, h->lev[0], h->lev[i]));
        HIP_TRY(hipEventElapsedTime(&e, h->lev[0], h->lev[i + 1]));
        iv.emplace_back(b, e);
      }
      std::sort(iv.begin(), iv.end());
      float cur_b = 0.f, cur_e = 0.f;
      bool open = false;
      for (const auto& p : iv) {
        if (!open) { cur_b = p.first; cur_e = p.second; open = true; continue; }
        if (p.first > cur_e) { stats->t_load_ms += cur_e - cur_b; cur_b = p.first; cur_e = p.second; }
        else if (p.second > cur_e) cur_e = p.second;
      }
      if (open) stats->t_load_ms += cur_e - cur_b;
    }
    stats->h2d_bytes = n_loads * h->expert_bytes;
    stats->loads = n_loads;
    stats->reloads = n_reloads;
    stats->hint_hits = n_hits;
    stats->t_step_ms =
        std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - wall0).count();
  }
  return ODMOE_OK;
}

int odmoe_decode_step(odmoe_layer_t* h, const void* x_dev, void* y_dev,
                      const int32_t* predicted_idx_host, int32_t* idx_out_host, odmoe_stats* stats) {
  const int rc =
      guarded([&] { return decode_step_impl(h, x_dev, y_dev, predicted_idx_host, idx_out_host, stats); });
  // a token that failed part-way leaves hinted and loaded experts in their slots: give them back
  if (rc != ODMOE_OK && rc != ODMOE_EINVAL) abandon_slots(h);
  return rc;
}

int odmoe_expert_ffn_static(const odmoe_config* cfg, const void* const* expert_table_dev,
                            const int32_t* idx_dev, const float* gate_dev, const void* x_dev,
                            int32_t n_tokens, void* y_dev, void* stream) {
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  if (cfg->n_slots != 0) return fail(ODMOE_EINVAL, "n_slots must be 0: the experts are read where the table points");
  if (n_tokens < 0) return fail(ODMOE_EINVAL, "n_tokens %d < 0", n_tokens);
  const size_t need = (size_t)cfg->top_k * cfg->ffn * sizeof(float);
  if (need > STATIC_SCRATCH_BYTES)
    return fail(ODMOE_EINVAL, "top_k * ffn = %d * %d floats (%zu bytes) exceed the %zu bytes of static scratch",
                cfg->top_k, cfg->ffn, need, STATIC_SCRATCH_BYTES);
  if (n_tokens == 0) return ODMOE_OK;
  if (!expert_table_dev || !idx_dev || !gate_dev || !x_dev || !y_dev)
    return fail(ODMOE_EINVAL, "table/idx/gate/x/y is NULL");
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(ODMOE_EINVAL, "device %d out of range", dev);
  void* hb = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!hb) {
    // first call on this device (it is the current one): where its copy of the array lives.  Two
    // threads racing here get the same answer.
    HIP_TRY(kernels_init());
    HIP_TRY(hipGetSymbolAddress(&hb, HIP_SYMBOL(scratch)));
    if (!hb) return fail(ODMOE_EHIP, "hipGetSymbolAddress gave no address");
    __atomic_store_n(&g_scratch_ptr[dev], hb, __ATOMIC_RELEASE);
  }
  Shape sh{cfg->hidden, cfg->ffn, cfg->n_experts, cfg->top_k, cfg->dtype};
  sh.quant = cfg->expert_quant;
  ExpertSrc src{};
  src.table = expert_table_dev;
  src.table_off = 0;
  src.n_experts = cfg->n_experts;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int k = cfg->top_k;
  const size_t row = (size_t)cfg->hidden * dtype_size(cfg->dtype);
  for (int t = 0; t < n_tokens; ++t) {
    HIP_TRY(launch_ffn_up(s, sh, src, idx_dev + (size_t)t * k, static_cast<const char*>(x_dev) + t * row,
                          static_cast<float*>(hb)));
    HIP_TRY(launch_ffn_down(s, sh, src, idx_dev + (size_t)t * k, gate_dev + (size_t)t * k,
                            static_cast<const float*>(hb), static_cast<char*>(y_dev) + t * row));
  }
  return ODMOE_OK;
}

static int sep_emulate_impl(odmoe_layer_t* main_stack, odmoe_layer_t* shadow, const void* x0_dev, int32_t n_iter,
                            int32_t aligned, float* recall_out, void* x_final_dev, float* shadow_ms,
                            float* main_ms) {
  if (!main_stack || !shadow) return fail(ODMOE_EINVAL, "handle is NULL");
  if (!x0_dev || !recall_out || n_iter < 0) return fail(ODMOE_EINVAL, "bad arguments");
  const odmoe_config &m = main_stack->cfg, &q = shadow->cfg;
  if (m.hidden != q.hidden || m.n_layers != q.n_layers || m.top_k != q.top_k || m.n_experts != q.n_experts ||
      m.dtype != q.dtype)
    return fail(ODMOE_EINVAL, "the shadow stack must have the main stack's hidden size, layers, experts, top_k and dtype");
  if (shadow->pool) return fail(ODMOE_EINVAL, "the shadow stack must be resident (n_slots = 0)");
  const int L = m.n_layers, k = m.top_k;
  const size_t row = (size_t)m.hidden * main_stack->esize;
  char* buf = nullptr;   // four state vectors: main in / out, shadow in / out
  if (hipMalloc((void**)&buf, 4 * row) != hipSuccess) {
    (void)hipGetLastError();
    return fail(ODMOE_ENOMEM, "no device memory for %zu bytes of state", 4 * row);
  }
  std::vector<int32_t> pred((size_t)L * k), used((size_t)L * k);
  using clk = std::chrono::steady_clock;
  double t_shadow = 0.0, t_main = 0.0;
  int rc = ODMOE_OK;
  auto body = [&]() -> int {
    char *xm = buf, *ym = buf + row, *xs = buf + 2 * row, *ys = buf + 3 * row;
    HIP_TRY(hipMemcpyAsync(xm, x0_dev, row, hipMemcpyDeviceToDevice, main_stack->compute));
    HIP_TRY(hipStreamSynchronize(main_stack->compute));
    for (int it = 0; it < n_iter; ++it) {
      const bool from_main = aligned || it == 0;
      auto t0 = clk::now();
      if ((rc = odmoe_decode_step(shadow, from_main ? xm : xs, ys, nullptr, pred.data(), nullptr))) return rc;
      auto t1 = clk::now();
      odmoe_stats st{};
      if ((rc = odmoe_decode_step(main_stack, xm, ym, pred.data(), used.data(), &st))) return rc;
      auto t2 = clk::now();
      t_shadow += std::chrono::duration<double, std::milli>(t1 - t0).count();
      t_main += std::chrono::duration<double, std::milli>(t2 - t1).count();
      // recall of this token (Section 3.2): predicted experts among the activated ones, per layer
      uint64_t hits = 0;
      for (int l = 0; l < L; ++l)
        for (int i = 0; i < k; ++i) {
          bool found = false;
          for (int j = 0; j < k; ++j) found |= pred[(size_t)l * k + j] == used[(size_t)l * k + i];
          hits += found;
        }
      if (main_stack->sched && st.hint_hits != hits)
        return fail(ODMOE_ESTATE, "the scheduler confirmed %llu hints, the index lists say %llu",
                    (unsigned long long)st.hint_hits, (unsigned long long)hits);
      recall_out[it] = (float)hits / (float)(L * k);
      std::swap(xm, ym);   // main's output is its next input
      std::swap(xs, ys);   // and the shadow's own output is what it follows when not aligned
    }
    if (x_final_dev) {
      HIP_TRY(hipMemcpyAsync(x_final_dev, xm, row, hipMemcpyDeviceToDevice, main_stack->compute));
      HIP_TRY(hipStreamSynchronize(main_stack->compute));
    }
    return ODMOE_OK;
  };
  rc = body();
  (void)hipStreamSynchronize(main_stack->compute);
  (void)hipStreamSynchronize(shadow->compute);
  (void)hipFree(buf);
  if (shadow_ms) *shadow_ms = (float)t_shadow;
  if (main_ms) *main_ms = (float)t_main;
  return rc;
}

int odmoe_sep_emulate(odmoe_layer_t* main_stack, odmoe_layer_t* shadow, const void* x0_dev, int32_t n_iter,
                      int32_t aligned, float* recall_out, void* x_final_dev, float* shadow_ms, float* main_ms) {
  return guarded([&] {
    return sep_emulate_impl(main_stack, shadow, x0_dev, n_iter, aligned, recall_out, x_final_dev, shadow_ms, main_ms);
  });
}

}  // extern "C"
