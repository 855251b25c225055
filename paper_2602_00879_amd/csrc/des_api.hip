// C ABI of the DES library: argument validation on the host, then kernel
// launches on the caller's stream.  Declarations and contracts: include/des.h.
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include <math.h>

#include "des_common.h"

namespace des {

static thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char* what) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
  return DES_ERR_HIP;
}

// ---- optional per-kernel timing (a measurement aid, never on by default) ----
bool g_timing_on = false;
namespace {
struct TimedLaunch { int id; hipEvent_t start, stop; };
std::vector<TimedLaunch> g_timed;
double g_ms[kKCount];
long long g_launches[kKCount];
}  // namespace

bool timing_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop) {
  TimedLaunch t;
  t.id = kernel_id;
  if (hipEventCreate(&t.start) != hipSuccess) return false;
  if (hipEventCreate(&t.stop) != hipSuccess) {
    (void)hipEventDestroy(t.start);
    return false;
  }
  g_timed.push_back(t);
  *start = t.start;
  *stop = t.stop;
  return true;
}

static void timing_collect() {
  for (TimedLaunch& t : g_timed) {
    float ms = 0.f;
    if (hipEventSynchronize(t.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
      g_ms[t.id] += ms;
      g_launches[t.id] += 1;
    }
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  g_timed.clear();
}

// Epoch of the routing launch's flags: never zero, never repeated in a process.
static std::atomic<unsigned long long> g_epoch{0x5eed000000000001ull};
static unsigned long long next_epoch() { return g_epoch.fetch_add(1, std::memory_order_relaxed); }

// Shape checks shared by all entry points.  `need_ffn` adds the checks that
// only the expert FFN needs (alignment of F, Fs).
static int check_shape(const des_shape_t* s, bool need_ffn) {
  if (!s) return DES_ERR_NULL;
  if (s->mode != DES_VANILLA && s->mode != DES_SEQ && s->mode != DES_VOTE) return DES_ERR_MODE;
  if (s->dtype != DES_F32 && s->dtype != DES_BF16) return DES_ERR_DTYPE;
  if (s->weight_layout != DES_LAYOUT_ROWMAJOR && s->weight_layout != DES_LAYOUT_PACKED)
    return DES_ERR_DTYPE;
  if (s->weight_layout == DES_LAYOUT_PACKED && s->dtype != DES_BF16) return DES_ERR_DTYPE;
  if (s->n_seqs < 1 || s->n_tokens < 1 || s->hidden < 1 || s->n_experts < 1 || s->top_k < 1)
    return DES_ERR_SHAPE;
  if (s->top_k > s->n_experts || s->top_k > 32 || s->n_experts > 512) return DES_ERR_SHAPE;
  const long long T = static_cast<long long>(s->n_seqs) * s->n_tokens;
  if (T > 4096) return DES_ERR_SHAPE;
  if (static_cast<long long>(s->n_experts) * ((T + 63) / 64) > 4096) return DES_ERR_SHAPE;
  if (s->mode != DES_VANILLA && s->coreset < 1) return DES_ERR_SHAPE;
  if (s->k_seq < 0 || s->k_seq > s->top_k) return DES_ERR_SHAPE;
  if (s->mode == DES_SEQ && s->k_seq > 0) {
    long long u = static_cast<long long>(s->n_tokens) * s->k_seq;
    if (u > s->n_experts) u = s->n_experts;
    if (s->coreset < u) return DES_ERR_SHAPE;
  }
  if (s->residual != 0 && s->residual != 1) return DES_ERR_SHAPE;
  if (s->k_route < 0 || s->k_route > s->top_k) return DES_ERR_SHAPE;
  if (!(s->skip_beta >= 0.0f && s->skip_beta < 1.0f)) return DES_ERR_SHAPE;  // also rejects NaN
  if (s->router_act != DES_ROUTER_SOFTMAX && s->router_act != DES_ROUTER_SIGMOID) return DES_ERR_MODE;
  if (s->vote_renorm != 0 && s->vote_renorm != 1) return DES_ERR_SHAPE;
  if (s->vote_atomic != 0 && s->vote_atomic != 1) return DES_ERR_SHAPE;
  if (s->n_group < 0) return DES_ERR_SHAPE;
  if (s->n_group > 1) {
    if (s->n_experts % s->n_group) return DES_ERR_SHAPE;
    const int gs = s->n_experts / s->n_group;
    if (gs % 8) return DES_ERR_SHAPE;  // a selector lane owns 8 experts of one group
    if (s->topk_group < 1 || s->topk_group > s->n_group) return DES_ERR_SHAPE;
    if (static_cast<long long>(s->topk_group) * gs < s->top_k) return DES_ERR_SHAPE;
    if (s->group_score != DES_GROUP_MAX && s->group_score != DES_GROUP_TOP2SUM) return DES_ERR_MODE;
  }
  const int align = s->dtype == DES_BF16 ? 32 : 4;
  if (s->hidden % align) return DES_ERR_SHAPE;
  if (need_ffn) {
    if (s->ffn < 1 || s->ffn_shared < 0) return DES_ERR_SHAPE;
    if (s->ffn % align || s->ffn_shared % align) return DES_ERR_SHAPE;
  }
  return DES_OK;
}

}  // namespace des

// ---- scratch built into the library (des_moe_forward_builtin_ws) ----
// One copy per GPU the library runs on, held until the process ends.  In host
// code the array's name is only a stand-in for the symbol: the address a kernel
// can use comes from hipGetSymbolAddress(), per device.
static __device__ __align__(256) unsigned char scratch[DES_BUILTIN_WORKSPACE_BYTES];

namespace des {
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device
static std::mutex g_scratch_mutex;

// Device address of the built-in scratch on the current device (looked up once
// per device); DES_ERR_HIP if the runtime refuses.
static int builtin_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "device ordinal");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DES_OK;
}
}  // namespace des

using namespace des;

extern "C" {

int32_t des_coreset_capacity(const des_shape_t* s) {
  if (!s) return 0;
  if (s->mode == DES_VANILLA) return s->n_experts;
  return s->coreset < s->n_experts ? s->coreset : s->n_experts;
}

size_t des_workspace_bytes(const des_shape_t* s) {
  if (check_shape(s, true) != DES_OK) return 0;
  return ws_layout(*s).total;
}

int des_route(const des_shape_t* s, const void* x, const void* w_router, const float* router_bias,
              float* logits, float* probs, void* hip_stream) {
  int rc = check_shape(s, false);
  if (rc != DES_OK) return rc;
  if (!x || !w_router || !logits) return DES_ERR_NULL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  rc = launch_router(*s, x, w_router, router_bias, logits, st);
  if (rc != DES_OK) return rc;
  if (probs) rc = launch_softmax(*s, logits, probs, st);
  return rc;
}

int des_select_coreset(const des_shape_t* s, const float* logits, int32_t* coreset_idx,
                       int32_t* coreset_size, float* votes, int32_t* k_seq_used,
                       void* hip_stream) {
  int rc = check_shape(s, false);
  if (rc != DES_OK) return rc;
  if (!logits || !coreset_idx || !coreset_size) return DES_ERR_NULL;
  return launch_select(*s, logits, coreset_idx, coreset_size, votes, k_seq_used,
                       static_cast<hipStream_t>(hip_stream));
}

int des_moe_forward(const des_shape_t* s, const void* x, const void* w_router,
                    const float* router_bias, const void* w_gate, const void* w_up,
                    const void* w_down, const void* ws_gate, const void* ws_up,
                    const void* ws_down, void* y, float* logits, int32_t* topk_idx, float* topk_w,
                    int32_t* expert_counts, int32_t* n_unique, int32_t* coreset_idx,
                    int32_t* coreset_size, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  int rc = check_shape(s, true);
  if (rc != DES_OK) return rc;
  if (!x || !w_router || !w_gate || !w_up || !w_down || !y || !logits || !topk_idx || !topk_w ||
      !expert_counts || !n_unique || !coreset_idx || !coreset_size || !workspace)
    return DES_ERR_NULL;
  if (s->ffn_shared > 0 && (!ws_gate || !ws_up || !ws_down)) return DES_ERR_NULL;
  if (x == y) return DES_ERR_SHAPE;
  if (workspace_bytes < ws_layout(*s).total) return DES_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return DES_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  const unsigned long long epoch = next_epoch();
  rc = launch_routing(*s, x, w_router, router_bias, logits, coreset_idx, coreset_size, topk_idx,
                      topk_w, expert_counts, n_unique, nullptr, ws, epoch, st);
  if (rc != DES_OK) return rc;
  return launch_ffn(*s, x, w_gate, w_up, w_down, ws_gate, ws_up, ws_down, logits, topk_idx, topk_w,
                    expert_counts, n_unique, y, ws, epoch, st);
}

int des_moe_forward_builtin_ws(const des_shape_t* s, const void* x, const void* w_router,
                               const float* router_bias, const void* w_gate, const void* w_up,
                               const void* w_down, const void* ws_gate, const void* ws_up,
                               const void* ws_down, void* y, float* logits, int32_t* topk_idx,
                               float* topk_w, int32_t* expert_counts, int32_t* n_unique,
                               int32_t* coreset_idx, int32_t* coreset_size, void* hip_stream) {
  const int rc = check_shape(s, true);
  if (rc != DES_OK) return rc;
  if (ws_layout(*s).total > DES_BUILTIN_WORKSPACE_BYTES) return DES_ERR_WORKSPACE;
  void* ws = nullptr;
  const int rs = builtin_scratch(&ws);
  if (rs != DES_OK) return rs;
  return des_moe_forward(s, x, w_router, router_bias, w_gate, w_up, w_down, ws_gate, ws_up, ws_down,
                         y, logits, topk_idx, topk_w, expert_counts, n_unique, coreset_idx,
                         coreset_size, ws, DES_BUILTIN_WORKSPACE_BYTES, hip_stream);
}

// Stack scratch: two activation ping-pong buffers, per-layer routing outputs
// that the stack does not return, then one layer's workspace.
struct StackLayout {
  size_t xa, xb, logits, topk_idx, topk_w, core_idx, core_size, layer_ws, total;
};
static StackLayout stack_layout(const des_shape_t& s) {
  const size_t T = static_cast<size_t>(s.n_seqs) * s.n_tokens;
  const size_t el = s.dtype == DES_BF16 ? 2 : 4;
  StackLayout l;
  size_t p = 0;
  l.xa = p; p = align256(p + T * s.hidden * el);
  l.xb = p; p = align256(p + T * s.hidden * el);
  l.logits = p; p = align256(p + 4 * T * s.n_experts);
  l.topk_idx = p; p = align256(p + 4 * T * s.top_k);
  l.topk_w = p; p = align256(p + 4 * T * s.top_k);
  l.core_idx = p; p = align256(p + 4 * static_cast<size_t>(s.n_seqs) * des_coreset_capacity(&s));
  l.core_size = p; p = align256(p + 4 * static_cast<size_t>(s.n_seqs));
  l.layer_ws = p; p = p + ws_layout(s).total;
  l.total = p;
  return l;
}

size_t des_stack_workspace_bytes(const des_shape_t* s) {
  if (check_shape(s, true) != DES_OK) return 0;
  return stack_layout(*s).total;
}

int des_moe_stack_forward(const des_shape_t* s_in, int32_t n_layers, const void* x,
                          const void* w_router, const float* router_bias, const void* w_gate,
                          const void* w_up, const void* w_down, const void* ws_gate,
                          const void* ws_up, const void* ws_down, void* y, int32_t* expert_counts,
                          int32_t* n_unique, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  int rc = check_shape(s_in, true);
  if (rc != DES_OK) return rc;
  if (n_layers < 1) return DES_ERR_SHAPE;
  if (!x || !w_router || !w_gate || !w_up || !w_down || !y || !expert_counts || !n_unique ||
      !workspace)
    return DES_ERR_NULL;
  if (x == y) return DES_ERR_SHAPE;
  des_shape_t s = *s_in;
  s.residual = 1;
  if (s.ffn_shared > 0 && (!ws_gate || !ws_up || !ws_down)) return DES_ERR_NULL;
  const StackLayout l = stack_layout(s);
  if (workspace_bytes < l.total) return DES_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return DES_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  const size_t el = s.dtype == DES_BF16 ? 2 : 4;
  const size_t M = s.n_experts, D = s.hidden, F = s.ffn, Fs = s.ffn_shared;
  const char* cur = static_cast<const char*>(x);
  for (int layer = 0; layer < n_layers; ++layer) {
    // the last layer writes y; the others alternate between the two buffers
    char* out = layer == n_layers - 1 ? static_cast<char*>(y)
                                      : ws + ((layer & 1) ? l.xb : l.xa);
    const size_t li = static_cast<size_t>(layer);
    const char* wr = static_cast<const char*>(w_router) + li * M * D * el;
    const float* rb = router_bias ? router_bias + li * M : nullptr;
    const char* wg = static_cast<const char*>(w_gate) + li * M * F * D * el;
    const char* wu = static_cast<const char*>(w_up) + li * M * F * D * el;
    const char* wd = static_cast<const char*>(w_down) + li * M * F * D * el;
    const char* sg = ws_gate ? static_cast<const char*>(ws_gate) + li * Fs * D * el : nullptr;
    const char* su = ws_up ? static_cast<const char*>(ws_up) + li * Fs * D * el : nullptr;
    const char* sd = ws_down ? static_cast<const char*>(ws_down) + li * Fs * D * el : nullptr;
    float* logits = reinterpret_cast<float*>(ws + l.logits);
    int32_t* tidx = reinterpret_cast<int32_t*>(ws + l.topk_idx);
    float* tw = reinterpret_cast<float*>(ws + l.topk_w);
    char* lws = ws + l.layer_ws;
    const unsigned long long epoch = next_epoch();
    rc = launch_routing(s, cur, wr, rb, logits, reinterpret_cast<int32_t*>(ws + l.core_idx),
                        reinterpret_cast<int32_t*>(ws + l.core_size), tidx, tw,
                        expert_counts + li * M, n_unique + li,
                        layer > 0 ? n_unique + li - 1 : nullptr, lws, epoch, st);
    if (rc != DES_OK) return rc;
    rc = launch_ffn(s, cur, wg, wu, wd, sg, su, sd, logits, tidx, tw, expert_counts + li * M,
                    n_unique + li, out, lws, epoch, st);
    if (rc != DES_OK) return rc;
    cur = out;
  }
  return DES_OK;
}

// ---- attention sub-layer and decoder stack ----
static int check_attn(const des_shape_t* s, const des_attn_shape_t* t) {
  if (!s || !t) return DES_ERR_NULL;
  if (s->dtype != DES_BF16) return DES_ERR_DTYPE;
  if (s->n_seqs < 1 || s->n_tokens < 1 || s->hidden < 128 || s->hidden % 128) return DES_ERR_SHAPE;
  if (static_cast<long long>(s->n_seqs) * s->n_tokens > 4096) return DES_ERR_SHAPE;
  if (s->residual != 0 && s->residual != 1) return DES_ERR_SHAPE;
  if (t->n_heads < 1 || t->n_kv_heads < 1 || t->head_dim < 8 || t->head_dim % 8 || t->head_dim > 128)
    return DES_ERR_SHAPE;
  if (t->n_heads % t->n_kv_heads) return DES_ERR_SHAPE;
  if (t->n_prefix < 0 || t->n_suffix < 0 || t->n_prefix + t->n_suffix > 4096) return DES_ERR_SHAPE;
  const long long hd = static_cast<long long>(t->n_heads) * t->head_dim;
  const long long kd = static_cast<long long>(t->n_kv_heads) * t->head_dim;
  if (hd % 128 || kd % 32 || hd > 16384) return DES_ERR_SHAPE;
  if (attn_core_lds(*s, *t) > 160 * 1024) return DES_ERR_SHAPE;
  return DES_OK;
}

size_t des_attention_workspace_bytes(const des_shape_t* s, const des_attn_shape_t* t) {
  if (check_attn(s, t) != DES_OK) return 0;
  return attn_layout(*s, *t).total;
}

int des_block_attention(const des_shape_t* s, const des_attn_shape_t* t, const void* x, const void* wq,
                        const void* wk, const void* wv, const void* wo, const void* k_cache,
                        const void* v_cache, void* y, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  const int rc = check_attn(s, t);
  if (rc != DES_OK) return rc;
  if (!x || !wq || !wk || !wv || !wo || !y || !workspace) return DES_ERR_NULL;
  if (attn_cached(*t) > 0 && (!k_cache || !v_cache)) return DES_ERR_NULL;
  if (x == y) return DES_ERR_SHAPE;
  if (workspace_bytes < attn_layout(*s, *t).total) return DES_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return DES_ERR_WORKSPACE;
  return launch_attention(*s, *t, x, wq, wk, wv, wo, k_cache, v_cache, y, static_cast<char*>(workspace),
                          next_epoch(), static_cast<hipStream_t>(hip_stream));
}

size_t des_decoder_workspace_bytes(const des_shape_t* s, const des_attn_shape_t* t) {
  if (check_shape(s, true) != DES_OK || check_attn(s, t) != DES_OK) return 0;
  return align256(stack_layout(*s).total) + attn_layout(*s, *t).total;
}

int des_decoder_stack_forward(const des_shape_t* s_in, const des_attn_shape_t* t, int32_t n_layers,
                              const void* x, const void* wq, const void* wk, const void* wv,
                              const void* wo, const void* k_cache, const void* v_cache,
                              const void* w_router, const float* router_bias, const void* w_gate,
                              const void* w_up, const void* w_down, const void* ws_gate,
                              const void* ws_up, const void* ws_down, void* y, int32_t* expert_counts,
                              int32_t* n_unique, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  int rc = check_shape(s_in, true);
  if (rc != DES_OK) return rc;
  rc = check_attn(s_in, t);
  if (rc != DES_OK) return rc;
  if (n_layers < 1) return DES_ERR_SHAPE;
  if (!x || !wq || !wk || !wv || !wo || !w_router || !w_gate || !w_up || !w_down || !y ||
      !expert_counts || !n_unique || !workspace)
    return DES_ERR_NULL;
  if (attn_cached(*t) > 0 && (!k_cache || !v_cache)) return DES_ERR_NULL;
  if (x == y) return DES_ERR_SHAPE;
  des_shape_t s = *s_in;
  s.residual = 1;
  if (s.ffn_shared > 0 && (!ws_gate || !ws_up || !ws_down)) return DES_ERR_NULL;
  const StackLayout l = stack_layout(s);
  const size_t attn_ws = align256(l.total);
  if (workspace_bytes < attn_ws + attn_layout(s, *t).total) return DES_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return DES_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  const size_t el = 2;
  const size_t M = s.n_experts, D = s.hidden, F = s.ffn, Fs = s.ffn_shared;
  const size_t HD = static_cast<size_t>(t->n_heads) * t->head_dim;
  const size_t KD = static_cast<size_t>(t->n_kv_heads) * t->head_dim;
  const size_t cache = static_cast<size_t>(s.n_seqs) * t->n_kv_heads * attn_cached(*t) * t->head_dim;
  const char* cur = static_cast<const char*>(x);
  for (int layer = 0; layer < n_layers; ++layer) {
    const size_t li = static_cast<size_t>(layer);
    // a = cur + Attn(cur) -> xa;  out = a + MoE(a) -> xb (the last layer: y)
    char* a = ws + l.xa;
    char* out = layer == n_layers - 1 ? static_cast<char*>(y) : ws + l.xb;
    rc = launch_attention(s, *t, cur, static_cast<const char*>(wq) + li * HD * D * el,
                          static_cast<const char*>(wk) + li * KD * D * el,
                          static_cast<const char*>(wv) + li * KD * D * el,
                          static_cast<const char*>(wo) + li * D * HD * el,
                          k_cache ? static_cast<const char*>(k_cache) + li * cache * el : nullptr,
                          v_cache ? static_cast<const char*>(v_cache) + li * cache * el : nullptr, a,
                          ws + attn_ws, next_epoch(), st);
    if (rc != DES_OK) return rc;
    const char* wr = static_cast<const char*>(w_router) + li * M * D * el;
    const float* rb = router_bias ? router_bias + li * M : nullptr;
    const char* wg = static_cast<const char*>(w_gate) + li * M * F * D * el;
    const char* wu = static_cast<const char*>(w_up) + li * M * F * D * el;
    const char* wd = static_cast<const char*>(w_down) + li * M * F * D * el;
    const char* sg = ws_gate ? static_cast<const char*>(ws_gate) + li * Fs * D * el : nullptr;
    const char* su = ws_up ? static_cast<const char*>(ws_up) + li * Fs * D * el : nullptr;
    const char* sd = ws_down ? static_cast<const char*>(ws_down) + li * Fs * D * el : nullptr;
    float* logits = reinterpret_cast<float*>(ws + l.logits);
    int32_t* tidx = reinterpret_cast<int32_t*>(ws + l.topk_idx);
    float* tw = reinterpret_cast<float*>(ws + l.topk_w);
    char* lws = ws + l.layer_ws;
    const unsigned long long epoch = next_epoch();
    rc = launch_routing(s, a, wr, rb, logits, reinterpret_cast<int32_t*>(ws + l.core_idx),
                        reinterpret_cast<int32_t*>(ws + l.core_size), tidx, tw, expert_counts + li * M,
                        n_unique + li, layer > 0 ? n_unique + li - 1 : nullptr, lws, epoch, st);
    if (rc != DES_OK) return rc;
    rc = launch_ffn(s, a, wg, wu, wd, sg, su, sd, logits, tidx, tw, expert_counts + li * M,
                    n_unique + li, out, lws, epoch, st);
    if (rc != DES_OK) return rc;
    cur = out;
  }
  return DES_OK;
}

int des_pack_expert_weights(const void* src, void* dst, int64_t n_mats, int32_t rows, int32_t cols,
                            void* hip_stream) {
  if (!src || !dst) return DES_ERR_NULL;
  if (src == dst) return DES_ERR_SHAPE;
  if (n_mats < 1 || rows < 16 || cols < 32 || rows % 16 || cols % 32) return DES_ERR_SHAPE;
  if (n_mats * rows * static_cast<long long>(cols) / 8 / 256 > 0x7FFFFFFFLL) return DES_ERR_SHAPE;
  return launch_pack(src, dst, n_mats, rows, cols, static_cast<hipStream_t>(hip_stream));
}

int des_hbm_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink) return DES_ERR_NULL;
  if (bytes < 65536 || bytes % 65536 || bytes / 65536 > 0x7FFFFFFFull) return DES_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(sink)) & 15) return DES_ERR_SHAPE;
  return launch_read_probe(src, bytes, sink, static_cast<hipStream_t>(hip_stream));
}

int32_t des_coreset_from_beta(double beta, int32_t n_experts) {
  if (!(beta > 0.0 && beta <= 1.0) || n_experts < 1) return 0;
  // the small addend keeps decimal fractions whose product is an integer (0.3 * 10)
  // from falling just below it in binary
  const int32_t c = static_cast<int32_t>(floor(beta * n_experts + 1e-9));
  return c < 1 ? 1 : c;
}

int des_test_hooks(int skip_router, int max_wait_iters) {
  if (max_wait_iters < 0) return DES_ERR_SHAPE;
  g_test_skip_router = skip_router < 0 ? 0 : (skip_router > 2 ? 1 : skip_router);
  g_test_max_wait = max_wait_iters;
  return DES_OK;
}

const char* des_strerror(int code) {
  switch (code) {
    case DES_OK: return "ok";
    case DES_ERR_NULL: return "a required pointer is NULL";
    case DES_ERR_SHAPE: return "shape out of range or not supported";
    case DES_ERR_MODE: return "unknown mode";
    case DES_ERR_DTYPE: return "unsupported dtype or weight layout";
    case DES_ERR_WORKSPACE:
      return "workspace too small or not 256-byte aligned, or the shape needs more scratch than "
             "the library's built-in buffer holds";
    case DES_ERR_HIP: return "a HIP call failed (see des_last_hip_error)";
    default: return "unknown error code";
  }
}

const char* des_last_hip_error(void) { return g_hip_error; }

int des_kernel_timing_enable(int enable) {
  timing_collect();
  for (int i = 0; i < kKCount; ++i) { g_ms[i] = 0.0; g_launches[i] = 0; }
  g_timing_on = enable != 0;
  return DES_OK;
}

int des_kernel_timing_count(void) { return kKCount; }

const char* des_kernel_timing_name(int kernel_id) {
  static const char* names[kKCount] = {"router", "softmax", "select", "permute", "gateup",
                                       "down", "combine", "pack", "routing", "ffn", "read_probe",
                                       "attn_proj", "attn_core", "attn_out"};
  return (kernel_id >= 0 && kernel_id < kKCount) ? names[kernel_id] : "";
}

int des_kernel_timing_read(int kernel_id, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return DES_ERR_NULL;
  if (kernel_id < 0 || kernel_id >= kKCount) return DES_ERR_SHAPE;
  timing_collect();
  *total_ms = g_ms[kernel_id];
  *launches = g_launches[kernel_id];
  return DES_OK;
}

}  // extern "C"
