// Internal helpers shared by the HIP translation units of the DES library.
// gfx950 (CDNA4) only: 64-wide wavefronts, DPP row broadcasts, bf16 MFMA.
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/des.h"

namespace des {

constexpr int kWave = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- bf16 <-> f32
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round to nearest even (inputs are finite)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// ------------------------------------------------------- wavefront reductions
// DPP controls (GFX9): quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E,
// row_shr:n = 0x110+n, row_bcast:15 = 0x142, row_bcast:31 = 0x143.
// Lanes without a source keep `old`, which is the identity of the operation,
// so after the six steps lane 63 holds the reduction over all 64 lanes.  The
// combination order is fixed by the lane layout, hence bit-reproducible.
template <int kCtrl>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
      static_cast<int>(identity), static_cast<int>(v), kCtrl, 0xF, 0xF, false));
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, dpp_u32<0xB1>(0u, v));
  v = max(v, dpp_u32<0x4E>(0u, v));
  v = max(v, dpp_u32<0x114>(0u, v));
  v = max(v, dpp_u32<0x118>(0u, v));
  v = max(v, dpp_u32<0x142>(0u, v));
  v = max(v, dpp_u32<0x143>(0u, v));
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}

__device__ __forceinline__ float wave_sum_f32(float x) {
  uint32_t v = __float_as_uint(x);
#define DES_STEP(ctrl) v = __float_as_uint(__uint_as_float(v) + __uint_as_float(dpp_u32<ctrl>(0u, v)))
  DES_STEP(0xB1);
  DES_STEP(0x4E);
  DES_STEP(0x114);
  DES_STEP(0x118);
  DES_STEP(0x142);
  DES_STEP(0x143);
#undef DES_STEP
  return __uint_as_float(
      static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), 63)));
}

__device__ __forceinline__ float readlane_f32(float x, int lane_uniform) {
  return __uint_as_float(static_cast<uint32_t>(
      __builtin_amdgcn_readlane(static_cast<int>(__float_as_uint(x)), lane_uniform)));
}

// Order-preserving map float -> uint32 for finite values; +0 and -0 coincide.
// 0 is below every finite key and marks "not a candidate".
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x + 0.0f);  // -0 + +0 = +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ------------------------------------------------------------ workspace layout
// Worst-case number of live experts the FFN launches must cover.
inline int max_live_experts(const des_shape_t& s) {
  const long long TK = static_cast<long long>(s.n_seqs) * s.n_tokens * s.top_k;
  long long m = s.n_experts;
  if (s.mode != DES_VANILLA) {
    long long c = s.coreset < s.n_experts ? s.coreset : s.n_experts;
    long long u = c * s.n_seqs;
    if (u < m) m = u;
  }
  if (TK < m) m = TK;
  return static_cast<int>(m);
}

// The fused routing launch is used only when all of its workgroups (router
// tiles + one per sequence + one) can be resident at once: one per compute
// unit, and never more than this.
constexpr int kMaxFusedRoutingBlocks = 256;

constexpr int kSlotToks = 32;  // tokens per slot kept in the slot-major token table
int device_compute_units();          // of the current device (cached)

// Blocks of more than 32 tokens: an expert's pairs are handed to the FFN
// workgroups in units of this many token rows (what one workgroup pass holds),
// at most kMaxSplits units per expert (an expert with more rows has each unit
// take several passes).  The permutation lists the live units, longest expert
// first; the FFN launches index that list, so no workgroup is spent on units
// that do not exist and neighbouring workgroups have neighbouring units.
inline int lds_rows_pass(int T) { return T <= 64 ? 64 : 128; }
constexpr int kMaxSplits = 8;
inline int max_units(const des_shape_t& s) {
  const long long TK = static_cast<long long>(s.n_seqs) * s.n_tokens * s.top_k;
  const int rows = lds_rows_pass(s.n_seqs * s.n_tokens);
  return max_live_experts(s) + static_cast<int>((TK + rows - 1) / rows);
}

// The selector workgroup (1024 threads) gives a token max(4, next power of two of
// ceil(M/8)) lanes, so it handles this many tokens at once; longer sequences are
// spread over up to kMaxSelGroups selector workgroups (all sequences together),
// which exchange their election partials through the workspace.
constexpr int kMaxSelGroups = 64;
constexpr int kSelPartStride = 512;  // 32-bit words per partial array (M <= 512)
inline int selector_tokens_per_pass(int n_experts) {
  int lanes = (n_experts + 7) / 8, lpt = 4;
  while (lpt < lanes) lpt *= 2;
  return 1024 / lpt;
}

// Short single-sequence blocks under DES ("dense" handling).  Once the coreset is elected
// the FFN's weight addresses are known; which token goes to which coreset expert is not
// needed to start streaming.  So for one sequence of at most 32 tokens the routing launch
// ends with the election, gate/up computes every coreset expert for ALL tokens of the
// block (two token tiles at most: matrix-core work that is free beside the weight
// stream), stage 2 (re-routing and gates, Alg. 1) runs in spare wavefronts of the gate/up
// launch, the down projection keeps only the routed (token, expert) pairs, and the
// permutation disappears.  Not for vanilla routing (its live experts ARE the per-token
// choices), nor where a coreset expert may end up unused (fewer experts per token than
// the election used, skipping, group limits): there the general path streams fewer bytes.
inline bool dense_shape(const des_shape_t& s) {
  return s.dtype == DES_BF16 && s.n_seqs == 1 && s.n_tokens <= 32 && s.mode != DES_VANILLA &&
         (s.k_route == 0 || s.k_route == s.top_k) && !(s.skip_beta > 0.0f) &&
         !(s.n_group > 1 && s.topk_group < s.n_group);
}
bool dense_block(const des_shape_t& s);  // dense_shape and the routing fits one launch

struct DenseArgs {
  int on;                  // 0: general path
  int lpt;                 // selector lanes per token (a power of two, 8 experts per lane)
  int sigmoid;             // router weights are sigmoid(logit)
  const float* logits;     // [N][M]
  int32_t* topk_idx;       // [N][K] S_n, written by stage 2
  float* topk_w;           // [N][K] g_n
  const int32_t* slot_of;  // [M] slot of a coreset expert, -1 otherwise
  uint32_t* tokmask;       // [n_slots] tokens routed to the slot's expert (bit n = token n)
  uint8_t* choice;         // [n_slots][32] which of token n's K choices the slot's expert is
  int32_t* pos;            // [N*K] output row of pair n*K+j (itself), -1 = unused
  int32_t* expert_counts;  // [M] written by the combine launch
  int32_t* n_unique;       // [1]
};

// All offsets in bytes from the (256-byte aligned) workspace base.
struct WsLayout {
  size_t flags;     // u64   [router tiles + 2 * max(B, kMaxSelGroups)]  epoch flags of the routing launch
  size_t sel_part;  // u32   [kMaxSelGroups][3][kSelPartStride]  selectors' election partials
  size_t slot_of;   // int32 [M]       slot of each live expert
  size_t slot_tok;  // u16   [n_slots][kSlotToks]  tokens of each slot's first pairs
  size_t offsets;   // int32 [M + 1]   exclusive scan of expert_counts
  size_t slots;     // int4  [n_slots] {expert, first sorted pair, pairs, token bitmap if T <= 32};
                    //       expert -1 = unused
  size_t meta;      // int32 [64]      [0] live experts, [1] routed pairs, [2] live units
  size_t pair_tok;  // int32 [T*K]     token of each pair, pairs sorted by (expert, token)
  size_t pos;       // int32 [T*K]     sorted position of pair t*K+j; -1 for unused slots
  size_t units;     // int32 [max_units]  slot | split << 16 | splits of that slot << 24
  size_t tokmask;   // u32   [n_slots]      dense short blocks: tokens routed to each slot's expert
  size_t choice;    // u8    [n_slots][32]  ... and which of the token's K choices it is
  size_t h_rows;    // routed rows of H: T*K, or n_slots * T for a dense short block
  size_t h;         // act   [(h_rows + Ts) * max(F, Fs)]   SwiGLU activations
  size_t o;         // f32   [(T*K + Ts) * D]            per-pair expert outputs
  size_t total;
};

inline size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

inline WsLayout ws_layout(const des_shape_t& s) {
  const size_t T = static_cast<size_t>(s.n_seqs) * s.n_tokens;
  const size_t TK = T * s.top_k;
  const size_t Ts = s.ffn_shared > 0 ? T : 0;
  const size_t act = s.dtype == DES_BF16 ? 2 : 4;
  const size_t Fm = s.ffn > s.ffn_shared ? s.ffn : s.ffn_shared;
  const size_t tiles = static_cast<size_t>((s.n_experts + 15) / 16) * ((T + 15) / 16);
  WsLayout w;
  size_t p = 0;
  const size_t nsel = static_cast<size_t>(s.n_seqs) > kMaxSelGroups ? s.n_seqs : kMaxSelGroups;
  w.flags = p;    p = align256(p + 8 * (tiles + 2 * nsel));
  w.sel_part = p; p = align256(p + 4 * static_cast<size_t>(kMaxSelGroups) * 3 * kSelPartStride);
  w.slot_of = p;  p = align256(p + 4 * static_cast<size_t>(s.n_experts));
  w.slot_tok = p; p = align256(p + 2 * static_cast<size_t>(max_live_experts(s)) * kSlotToks);
  w.offsets = p;  p = align256(p + 4 * (static_cast<size_t>(s.n_experts) + 1));
  w.slots = p;    p = align256(p + 16 * static_cast<size_t>(max_live_experts(s)));
  w.meta = p;     p = align256(p + 4 * 64);
  w.pair_tok = p; p = align256(p + 4 * TK);
  w.pos = p;      p = align256(p + 4 * TK);
  w.units = p;    p = align256(p + 4 * static_cast<size_t>(max_units(s)));
  w.tokmask = p;  p = align256(p + 4 * static_cast<size_t>(max_live_experts(s)));
  w.choice = p;   p = align256(p + 32 * static_cast<size_t>(max_live_experts(s)));
  const size_t dense_rows = dense_shape(s) ? static_cast<size_t>(max_live_experts(s)) * T : 0;
  w.h_rows = dense_rows > TK ? dense_rows : TK;
  w.h = p;        p = align256(p + act * (w.h_rows + Ts) * Fm);
  w.o = p;        p = align256(p + 4 * (TK + Ts) * static_cast<size_t>(s.hidden));
  w.total = p;
  return w;
}

// Launchers implemented in the .hip files (host functions).
int launch_router(const des_shape_t& s, const void* x, const void* w_router, const float* bias,
                  float* logits, hipStream_t st);
int launch_softmax(const des_shape_t& s, const float* logits, float* probs, hipStream_t st);
int launch_select(const des_shape_t& s, const float* logits, int32_t* coreset_idx,
                  int32_t* coreset_size, float* votes, int32_t* k_seq_used, hipStream_t st);
// router + election + re-routing + permutation (one launch when it fits)
int launch_routing(const des_shape_t& s, const void* x, const void* w_router, const float* bias,
                   float* logits, int32_t* coreset_idx, int32_t* coreset_size, int32_t* topk_idx,
                   float* topk_w, int32_t* expert_counts, int32_t* n_unique,
                   const int32_t* prev_n_unique, char* ws, unsigned long long epoch,
                   hipStream_t st);
// Test hooks of the routing launch (des_test_hooks).
extern int g_test_max_wait, g_test_skip_router;
int launch_ffn(const des_shape_t& s, const void* x, const void* w_gate, const void* w_up,
               const void* w_down, const void* ws_gate, const void* ws_up, const void* ws_down,
               const float* logits, int32_t* topk_idx, float* topk_w, int32_t* expert_counts,
               int32_t* n_unique, void* y, char* ws, unsigned long long epoch, hipStream_t st);
// Attention sub-layer (des_attention.hip): scratch layout, LDS need of the per-head
// kernel, and the three launches.
struct AttnLayout { size_t q, k, v, o, partial, flags, total; };
inline int attn_cached(const des_attn_shape_t& t) { return t.n_prefix + t.n_suffix; }
AttnLayout attn_layout(const des_shape_t& s, const des_attn_shape_t& t);
size_t attn_core_lds(const des_shape_t& s, const des_attn_shape_t& t);
int launch_attention(const des_shape_t& s, const des_attn_shape_t& t, const void* x, const void* wq,
                     const void* wk, const void* wv, const void* wo, const void* k_cache,
                     const void* v_cache, void* y, char* ws, unsigned long long epoch, hipStream_t st);
int launch_pack(const void* src, void* dst, int64_t n_mats, int rows, int cols, hipStream_t st);
int launch_read_probe(const void* src, size_t bytes, void* sink, hipStream_t st);

int hip_fail(hipError_t e, const char* what);  // records text, returns DES_ERR_HIP

// Kernel ids for the optional per-kernel event timing (des_kernel_timing_*).
enum KernelId { kKRouter = 0, kKSoftmax, kKSelect, kKPermute, kKGateUp, kKDown, kKCombine, kKPack,
                kKRouting, kKFfn, kKProbe, kKAttnProj, kKAttnCore, kKAttnOut, kKCount };
extern bool g_timing_on;
// Creates the event pair of one timed launch and remembers it under kernel_id.
bool timing_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop);

// Every kernel of the library is launched through here.  With timing enabled
// the launch carries its own start/stop events (hipExtLaunchKernelGGL), which
// take the dispatch's begin and end timestamps - the kernel's execution time,
// not the time between two stream markers.
template <typename Kern, typename... Args>
inline void launch(int kernel_id, Kern kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st,
                   Args... args) {
  hipEvent_t ev0, ev1;
  if (g_timing_on && timing_events(kernel_id, &ev0, &ev1)) {
    hipExtLaunchKernelGGL(kernel, grid, block, lds, st, ev0, ev1, 0, args...);
  } else {
    hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
  }
}

}  // namespace des
