// Selection primitives shared by the routing kernel and by the wavefronts that re-route
// the tokens of a short block beside the gate/up projection (Alg. 1 stage 2): a "row" of
// LPT adjacent lanes owns one token, each lane 8 consecutive experts, sorted once.
#pragma once
#include "des_common.h"

namespace des {

// ------------------------------------------------------- row primitives
// A "row" is the group of LPT adjacent lanes that owns one token; each lane
// owns 8 consecutive experts.  All-reduce inside every row: quad swaps, the
// half-row and row mirrors (DPP), then lane exchanges across 16-lane rows.
template <int LPT>
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v) {
  if (LPT >= 2) v = max(v, dpp_u32<0xB1>(0u, v));   // quad_perm [1,0,3,2]
  if (LPT >= 4) v = max(v, dpp_u32<0x4E>(0u, v));   // quad_perm [2,3,0,1]
  if (LPT >= 8) v = max(v, dpp_u32<0x141>(0u, v));  // row_half_mirror
  if (LPT >= 16) v = max(v, dpp_u32<0x140>(0u, v)); // row_mirror
  if (LPT >= 32) v = max(v, static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 16)));
  if (LPT >= 64) v = max(v, static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 32)));
  return v;
}
template <int LPT>
__device__ __forceinline__ float row_sum_f32(float x) {
  uint32_t v = __float_as_uint(x);
#define DES_STEP(ctrl) v = __float_as_uint(__uint_as_float(v) + __uint_as_float(dpp_u32<ctrl>(0u, v)))
  if (LPT >= 2) DES_STEP(0xB1);
  if (LPT >= 4) DES_STEP(0x4E);
  if (LPT >= 8) DES_STEP(0x141);
  if (LPT >= 16) DES_STEP(0x140);
#undef DES_STEP
  float r = __uint_as_float(v);
  if (LPT >= 32) r += __shfl_xor(r, 16);
  if (LPT >= 64) r += __shfl_xor(r, 32);
  return r;
}
// exp(x) for x <= 0 through the hardware exp2: the product x*log2(e) is split
// into a rounded part and its residual, so the result is good to ~2 ulp
// (a plain exp2(x*log2e) loses |x| ulp).  Underflows to 0 below about -87.
__device__ __forceinline__ float exp_neg(float x) {
  const float kL2eHi = 1.44269502162933349609375f, kL2eLo = 1.925963033500011e-8f;
  const float t = x * kL2eHi;
  float r = fmaf(x, kL2eHi, -t);
  r = fmaf(x, kL2eLo, r);
  return __builtin_amdgcn_exp2f(t) * fmaf(r, 0.693147180559945f, 1.0f);
}
// logistic sigmoid, the same accuracy for both signs
__device__ __forceinline__ float sigmoid_f(float x) {
  const float t = exp_neg(-fabsf(x));
  return (x >= 0.f ? 1.0f : t) / (1.0f + t);
}
__device__ __forceinline__ float key_to_f32(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

constexpr int kEpl = 8;  // experts per lane

// A lane's 8 (key, slot) pairs sorted once, best first; every later "best
// remaining candidate" is then a head pointer, not a rescan.  The pair is one
// 64-bit word, key << 3 | (7 - slot), so that equal keys order by ascending
// slot (= ascending expert index) and a plain 19-comparator network does the
// job.  `idx` packs the original slot of sorted position s in bits [3s, 3s+3).
__device__ __forceinline__ void sort8_desc(uint32_t (&k)[kEpl], uint32_t& idx) {
  unsigned long long c[kEpl];
#pragma unroll
  for (int j = 0; j < kEpl; ++j)
    c[j] = (static_cast<unsigned long long>(k[j]) << 3) | static_cast<unsigned>(7 - j);
#define DES_CE(i, j)                              \
  do {                                            \
    const bool sw = c[i] < c[j];                  \
    const unsigned long long hi = sw ? c[j] : c[i]; \
    const unsigned long long lo = sw ? c[i] : c[j]; \
    c[i] = hi;                                    \
    c[j] = lo;                                    \
  } while (0)
  DES_CE(0, 1); DES_CE(2, 3); DES_CE(4, 5); DES_CE(6, 7);
  DES_CE(0, 2); DES_CE(1, 3); DES_CE(4, 6); DES_CE(5, 7);
  DES_CE(1, 2); DES_CE(5, 6); DES_CE(0, 4); DES_CE(3, 7);
  DES_CE(1, 5); DES_CE(2, 6);
  DES_CE(1, 4); DES_CE(3, 6);
  DES_CE(2, 4); DES_CE(3, 5);
  DES_CE(3, 4);
#undef DES_CE
  idx = 0;
#pragma unroll
  for (int j = 0; j < kEpl; ++j) {
    k[j] = static_cast<uint32_t>(c[j] >> 3);
    idx |= (7u - (static_cast<uint32_t>(c[j]) & 7u)) << (3 * j);
  }
}

// Per-token state of one lane while candidates are drawn best-first.
struct Head {
  uint32_t mask;  // sorted positions still in play
  uint32_t key;   // key at the head (0 = none)
  int h;          // head position
};
__device__ __forceinline__ void head_set(Head& hd, uint32_t mask, const uint32_t* my_sorted) {
  hd.mask = mask;
  hd.h = mask ? __builtin_ctz(mask) : 0;
  hd.key = mask ? my_sorted[hd.h * 64] : 0u;
}

// One draw: the best head of every row.  Returns the row's best key (0 = the
// row has no candidate); `mine` is set in the one lane that owns it.
template <int LPT>
__device__ __forceinline__ uint32_t row_draw(const Head& hd, bool& mine) {
  const uint32_t m = row_max_u32<LPT>(hd.key);
  const unsigned long long hit = __ballot(hd.key == m && m != 0u);
  const int lane = threadIdx.x & 63;
  const unsigned long long rowbits =
      LPT == 64 ? hit : ((hit >> (lane & (64 - LPT))) & ((1ull << (LPT & 63)) - 1ull));
  // lowest lane with the best key = lowest expert index among equals
  mine = rowbits != 0ull && (lane & (LPT - 1)) == __builtin_ctzll(rowbits);
  return m;
}

// ---------------------------------------------- stage 2 for a short block, per wavefront
// Alg. 1 stage 2 for the 64 / LPT tokens of one wavefront, given the elected coreset as
// the expert -> slot table: each token draws its K best coreset experts best-first
// (ties to the lowest index), gates = softmax over the drawn logits (or the sigmoid
// scores divided by their sum).  Rows are independent of each other, so this needs no
// workgroup: it runs in spare wavefronts of the gate/up launch, off the critical path.
// Besides S_n and g_n it records, per slot, the bitmap of the tokens routed to the
// slot's expert and which of a token's K choices the expert is (the down projection
// stores a pair's output at row n*K + choice), and the pair positions for the combine.
// Integer atomics only (bit sets): the result does not depend on arrival order.
template <int LPT>
__device__ __forceinline__ void stage2_wave(const DenseArgs& d, int N, int M, int K, int n_core,
                                            int wave_idx, uint32_t* s_sorted) {
  constexpr int RPW = 64 / LPT;
  constexpr int NW = (32 + LPT - 1) / LPT;  // gate slots a lane keeps (K <= 32)
  const int lane = threadIdx.x & 63, row = lane / LPT, rl = lane % LPT;
  const int n = wave_idx * RPW + row;
  const bool live = n < N;
  uint32_t* my_sorted = s_sorted + lane;  // [s * 64]
  const float* rowp = d.logits + static_cast<size_t>(live ? n : 0) * M;
  uint32_t key[kEpl], sidx = 0, nvalid = 0;
#pragma unroll
  for (int j = 0; j < kEpl; ++j) {
    const int idx = rl * kEpl + j;
    const bool ok = live && idx < M;
    key[j] = ok ? order_key(rowp[idx]) : 0u;
    nvalid += ok ? 1u : 0u;
  }
  sort8_desc(key, sidx);
#pragma unroll
  for (int j = 0; j < kEpl; ++j) my_sorted[j * 64] = key[j];
  // candidates: sorted positions whose expert sits in the coreset
  uint32_t cmask = 0;
  int slot_at[kEpl];
#pragma unroll
  for (int sp = 0; sp < kEpl; ++sp) {
    const int e = rl * kEpl + static_cast<int>((sidx >> (3 * sp)) & 7u);
    slot_at[sp] = (static_cast<uint32_t>(sp) < nvalid) ? d.slot_of[e] : -1;
    cmask |= slot_at[sp] >= 0 ? (1u << sp) : 0u;
  }
  Head hd;
  head_set(hd, cmask, my_sorted);
  const int keff = min(K, n_core);
  const size_t o = static_cast<size_t>(live ? n : 0) * K;
  uint32_t mkey[NW], m0 = 0u;  // keys drawn at iterations rl, rl + LPT, ...; the first key
#pragma unroll
  for (int q = 0; q < NW; ++q) mkey[q] = 0u;
  int have = keff;
  for (int it = 0; it < keff; ++it) {
    bool mine;
    const uint32_t m = row_draw<LPT>(hd, mine);  // every lane of the row sees the drawn key
    if (it == 0) m0 = m;
    if (m == 0u) have = min(have, it);
#pragma unroll
    for (int q = 0; q < NW; ++q)
      if (it == q * LPT + rl) mkey[q] = m;
    if (mine) {
      if (live) {
        int sl = 0;
#pragma unroll
        for (int sp = 0; sp < kEpl; ++sp)
          if (sp == hd.h) sl = slot_at[sp];
        d.topk_idx[o + it] = rl * kEpl + static_cast<int>((sidx >> (3 * hd.h)) & 7u);
        atomicOr(d.tokmask + sl, 1u << n);
        d.choice[sl * 32 + n] = static_cast<uint8_t>(it);
      }
      head_set(hd, hd.mask & (hd.mask - 1u), my_sorted);
    }
  }
  // gate numerators of this lane's slots, then the row's sum in a fixed order
  const float mx = key_to_f32(m0);
  float mye[NW], part = 0.f;
#pragma unroll
  for (int q = 0; q < NW; ++q) {
    mye[q] = !mkey[q] ? 0.f
             : d.sigmoid ? sigmoid_f(key_to_f32(mkey[q]))
                         : exp_neg(key_to_f32(mkey[q]) - mx);
    part += mye[q];
  }
  const float den = row_sum_f32<LPT>(part);
  if (live) {
#pragma unroll
    for (int q = 0; q < NW; ++q) {
      const int it = q * LPT + rl;
      if (it < K) {
        d.topk_w[o + it] = it < have ? mye[q] / den : 0.f;
        if (it >= have) d.topk_idx[o + it] = -1;
        d.pos[o + it] = it < have ? static_cast<int>(o) + it : -1;
      }
    }
  }
}

}  // namespace des
