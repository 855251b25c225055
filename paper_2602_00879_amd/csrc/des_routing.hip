// Routing half of the DES layer for gfx950, in ONE launch:
//   router scores G(x)                      (Background, definition of G)
//   coreset election  Phi                   (Alg. 1 stage 1; Eq. 5 / Alg. 2, Eq. 6 / Alg. 3)
//   constrained re-routing + gates          (Alg. 1 stage 2)
//   token permutation by expert, cnt_i      (Eq. 2)
//
// The paper fuses its selection into two kernels that add votes into a global
// vector with float atomics (Sec. 4.3).  Here the whole routing step is one
// kernel whose workgroups take one of three roles, chained through per-producer
// flags in device memory instead of kernel boundaries:
//   role R (one per 16x16 logits tile)  router GEMM tile, then flag[tile] = epoch
//   role S (one per sequence, or one    waits for the R flags, elects the coreset,
//           per group of its tokens)    re-routes, then flag[seq] = epoch
//   role P (one, merged into S if B==1) waits for the S flags, builds counts,
//                                       offsets, the slot table and the permutation
// A flag is a 64-bit word that a producer sets to the call's epoch (a host
// counter that never repeats), so the workspace needs no clearing, stale
// contents can never satisfy a wait, and no two workgroups ever write the same
// word (no atomic read-modify-write at all).  Waiting is safe because the launch
// is only used in this fused form when every workgroup fits on the chip at once
// (one 1024-thread workgroup per compute unit), so a producer can always run;
// every wait is also bounded and gives up, reporting n_unique = -1.
// Larger problems run the same three roles as three launches.
//
// Votes are accumulated without floating-point atomics: a 16-lane row of a
// wavefront owns one token, each lane owns a contiguous slice of the experts,
// votes stay in the owning lane's registers, and rows / waves are combined in a
// fixed order.  Every ranking compares order-preserving integer keys of the
// fp32 logits with ties to the lowest expert index.
#include "des_common.h"
#include "des_select.h"

namespace des {

constexpr int kRtWaves = 16;
constexpr int kRtThreads = kRtWaves * kWave;  // 1024
constexpr int kMaxWaitIters = 1 << 22;        // bounded waits (~ seconds), then give up
int g_test_max_wait = 0;     // test hooks (des_test_hooks): a tiny wait bound, and a fused
int g_test_skip_router = 0;  // routing launch without its router tiles, so that a wait expires

#ifdef DES_ROUTING_TIMESTAMPS  // development aid: 100 MHz timestamps into meta[16..]
#define DES_STAMP(a, i) do { if (threadIdx.x == 0 && (a).meta != nullptr) reinterpret_cast<long long*>((a).meta + 16)[i] = wall_clock64(); } while (0)
#else
#define DES_STAMP(a, i) do { } while (0)
#endif

struct RoutingArgs {
  // router
  const void* x;
  const void* w_router;
  const float* bias;
  float* logits;          // [B][N][M]
  // selection
  int32_t* coreset_idx;   // [B][cap]
  int32_t* coreset_size;  // [B]
  float* votes;           // [B][M] or null
  int32_t* k_seq_used;    // [B] or null
  int32_t* topk_idx;      // [B][N][K] or null (then stage 2 and permutation are skipped)
  float* topk_w;
  // permutation
  int32_t* expert_counts; // [M]
  int32_t* n_unique;      // [1]
  int32_t* offsets;       // [M+1]
  int4* slots;            // [n_slots] {expert, first sorted pair, pairs, 0}; expert -1 = unused
  int32_t* meta;          // [8]: [0] live experts, [1] routed pairs, [2] live units
  int32_t* units;         // [max units] slot | split << 16 | splits of the slot << 24
  int rows_shift;         // log2 of the token rows per unit (blocks of more than 32 tokens)
  int32_t* pair_tok;      // [T*K] token of each sorted pair
  int32_t* pos;           // [T*K] sorted position of pair (t*K+j), -1 = unused slot
  unsigned long long* flags;  // [n_tiles + 2*B*groups] epoch flags: router tiles, selector
                              // partials published, selectors done
  uint32_t* sel_part;         // [B*groups][3][kSelPartStride] per-group election partials
  unsigned long long epoch;
  int32_t* slot_of;       // [M] slot of each live expert, -1 otherwise
  uint16_t* slot_tok;     // [n_slots][kSlotToks] tokens of each slot's first pairs
  int B, N, M, K, C, k_seq, mode, cap, D, n_slots;
  int groups;             // selector workgroups per sequence (each takes every groups-th pass)
  int k_route;            // experts per token in stage 2 (<= K)
  float skip_beta;        // > 0: cumulative-probability skipping of a token's weakest experts
  int sigmoid;            // router weights are sigmoid(logit) instead of softmax over M
  int vote_renorm;        // a token's K votes are divided by their sum
  int n_group;            // > 1: group-limited router over this many groups of experts
  int group_lanes;        // selector lanes per group (group size / 8)
  int topk_group;         // groups a token keeps
  int group_top2;         // group score: sum of the two best router weights (else the best logit)
  int vote_atomic;        // votes meet in floating-point LDS atomics (arrival order) instead of
                          // the fixed-order reduction
  int tiles_m, tiles_t;   // router tiles along experts / tokens
  int max_wait;           // polls before a wait gives up
  const int32_t* prev_n_unique;  // the previous layer's n_unique (a stack), or null: a negative
                                 // value there is carried into this layer's n_unique
  int do_router, do_select, do_permute, use_flags, bf16;
  int skip_router_tiles;  // test hook: the fused launch runs without its router tiles
  int small_perm;         // one selector workgroup, at most 32 tokens, no skipping: the permutation
                          // is built from per-expert token bitmaps recorded during stage 2
  int dense;              // dense short block (dense_block()): the launch ends with the election
                          // and the slot table of the coreset; stage 2 runs beside the gate/up
                          // projection, there is no permutation
  uint32_t* tokmask;      // [n_slots] cleared here for that stage 2
};

// ------------------------------------------------------------------ flags
// Two hand-off styles.  `fenced`: the data was written with ordinary stores, so
// a device-scope fence (an L2 write-back on this chip, ~1 us) precedes the flag
// and the waiter ends with one too.  Unfenced: the data itself is written and
// read with device-scope accesses (the logits), which reach the level all
// compute units share on their own, so the flag only has to follow them.
// A workgroup barrier does not wait for outstanding stores: every thread that
// stored data the flag stands for must have waited for its own stores
// (stores_done()) BEFORE the barrier that precedes the publishing thread's call.
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void flag_publish(unsigned long long* f, unsigned long long epoch,
                                             bool fenced) {
  if (fenced) __threadfence();
  __hip_atomic_store(f, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Every thread polls a subset of the flags; returns false if a wait ran out.
__device__ __forceinline__ bool flags_wait(const unsigned long long* f, int n,
                                           unsigned long long epoch, bool fenced, int max_wait) {
  bool ok = true;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    int it = 0;
    // relaxed polls; the fence after the barrier below is the acquire
    while (__hip_atomic_load(f + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
      __builtin_amdgcn_s_sleep(4);
      if (++it > max_wait) { ok = false; break; }
    }
  }
  const int all = __syncthreads_and(ok ? 1 : 0);
  if (fenced) __threadfence();
  return all != 0;
}

// ------------------------------------------------------------ role R: router
// experts [i0, i0+16) x tokens [t0, t0+16); wave w takes k-steps w, w+16, ...
// MFMA 16x16x32: lane l supplies row (l%16), reduction elements 8*(l/16)..+7;
// the accumulator of lane l holds column (l%16), rows 4*(l/16)..+3.
__device__ __forceinline__ void router_tile_bf16(const RoutingArgs& a, int tile_m, int tile_t,
                                                 float* part /* [16][256] LDS */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int T = a.B * a.N, D = a.D, M = a.M;
  const int i0 = tile_m * 16, t0 = tile_t * 16;
  const int r = lane & 15, kq = (lane >> 4) * 8;
  const int ei = min(i0 + r, M - 1);  // clamped rows are computed and dropped
  const int ti = min(t0 + r, T - 1);
  const uint16_t* ap = static_cast<const uint16_t*>(a.w_router) + static_cast<size_t>(ei) * D + kq;
  const uint16_t* bp = static_cast<const uint16_t*>(a.x) + static_cast<size_t>(ti) * D + kq;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const int nks = D / 32;
  // the bias of the expert this thread will finish (below), fetched now so that its
  // latency is not added after the reduction
  const int er_fin = threadIdx.x & 15;
  const float bias_fin = (threadIdx.x < 256 && a.bias && i0 + er_fin < M) ? a.bias[i0 + er_fin] : 0.f;
  // four k-steps per trip, all eight loads in flight before the first MFMA
  for (int ks = wave; ks < nks; ks += 4 * kRtWaves) {
    bf16x8 av[4], bv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int k = min(ks + u * kRtWaves, nks - 1);  // clamped steps are skipped below
      av[u] = *reinterpret_cast<const bf16x8*>(ap + k * 32);
      bv[u] = *reinterpret_cast<const bf16x8*>(bp + k * 32);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (ks + u * kRtWaves < nks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u], bv[u], acc, 0, 0, 0);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) part[wave * 256 + (4 * (lane >> 4) + q) * 16 + r] = acc[q];
  __syncthreads();
  if (threadIdx.x < 256) {
    const int er = er_fin, tc = threadIdx.x >> 4;
    float s = 0.f;
    const float bias_e = bias_fin;
#pragma unroll
    for (int w = 0; w < kRtWaves; ++w) s += part[w * 256 + er * 16 + tc];  // fixed order
    const int e = i0 + er, t = t0 + tc;
    if (e < M && t < T)  // device-scope store: the selector reads it without a fence
      __hip_atomic_store(a.logits + static_cast<size_t>(t) * M + e, s + bias_e, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  }
}

// fp32 inputs: each wavefront takes (expert, token) dot products of the tile in
// turn, lanes stride the reduction dimension with 16-byte loads.
__device__ __forceinline__ void router_tile_f32(const RoutingArgs& a, int tile_m, int tile_t) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int T = a.B * a.N, D = a.D, M = a.M;
  const float* x = static_cast<const float*>(a.x);
  const float* wr = static_cast<const float*>(a.w_router);
  for (int p = wave; p < 256; p += kRtWaves) {
    const int e = tile_m * 16 + (p & 15), t = tile_t * 16 + (p >> 4);
    if (e >= M || t >= T) continue;  // uniform per wave
    const float4* xp = reinterpret_cast<const float4*>(x + static_cast<size_t>(t) * D);
    const float4* wp = reinterpret_cast<const float4*>(wr + static_cast<size_t>(e) * D);
    float s = 0.f;
    for (int v = lane; v < D / 4; v += 64) {
      const float4 p4 = xp[v], q4 = wp[v];
      s = fmaf(p4.x, q4.x, s);
      s = fmaf(p4.y, q4.y, s);
      s = fmaf(p4.z, q4.z, s);
      s = fmaf(p4.w, q4.w, s);
    }
    s = wave_sum_f32(s);
    if (lane == 0)
      __hip_atomic_store(a.logits + static_cast<size_t>(t) * M + e, s + (a.bias ? a.bias[e] : 0.f),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// LDS carve-up of the selection (bytes).  MP = padded expert count = 8 * LPT.
template <int LPT>
struct SelLds {
  static constexpr int MP = kEpl * LPT;
  static constexpr int sorted = 0;                               // u32 [16 waves][8][64 lanes]
  static constexpr int vpart = sorted + 4 * kRtWaves * kEpl * 64; // float [16 waves][MP]
  static constexpr int level = vpart + 4 * kRtWaves * MP;        // int [MP]
  static constexpr int cnt1 = level + 4 * MP;                    // int [MP]
  static constexpr int key = cnt1 + 4 * MP;                      // u32 [MP]
  static constexpr int rank = key + 4 * MP;                      // int [MP]
  static constexpr int core = rank + 4 * MP;                     // int [MP]
  static constexpr int hist = core + 4 * MP;                     // int [36]
  static constexpr int mask = hist + 4 * 36;                     // u32 [MP] tokens routed to an expert (T <= 32)
  static constexpr int vsum = mask + 4 * MP;                     // float [MP] the votes, all waves added
  static constexpr int off = vsum + 4 * MP;                      // int [MP + 1] first pair of an expert
  static constexpr int liv = off + 4 * (MP + 1);                 // int [MP + 1] live experts before it
  static constexpr int total = liv + 4 * (MP + 1);
};

// ------------------------------------------------------- role S: selection
// `dry` runs the same instructions on whatever the logits buffer holds and
// stores nothing to global memory: the selector workgroup uses it to pull its
// code into the instruction cache while it waits for the router tiles (every
// index below derives from lane and slot numbers, never from the data read).
// EXT = the variants few callers use (group-limited router, votes added with
// floating-point atomics) are compiled in; the plain instantiation leaves them
// out, so the common path pays nothing for them.
template <int LPT, bool EXT>
__device__ bool select_sequence(const RoutingArgs& a, int b, int g, char* smem, bool dry,
                                bool wait_router) {
  using L = SelLds<LPT>;
  constexpr int MP = L::MP;
  constexpr int RPW = 64 / LPT;          // rows (tokens) per wave
  constexpr int TPP = kRtWaves * RPW;    // tokens per pass
  constexpr int NW = (32 + LPT - 1) / LPT;  // gate slots a lane keeps (K <= 32)
  uint32_t* s_sorted = reinterpret_cast<uint32_t*>(smem + L::sorted);
  float* s_vpart = reinterpret_cast<float*>(smem + L::vpart);
  int* s_level = reinterpret_cast<int*>(smem + L::level);
  int* s_cnt1 = reinterpret_cast<int*>(smem + L::cnt1);
  uint32_t* s_key = reinterpret_cast<uint32_t*>(smem + L::key);
  int* s_rank = reinterpret_cast<int*>(smem + L::rank);
  int* s_core = reinterpret_cast<int*>(smem + L::core);
  int* s_hist = reinterpret_cast<int*>(smem + L::hist);  // [0..32] histogram, [33] k used, [34] size
  uint32_t* s_mask = reinterpret_cast<uint32_t*>(smem + L::mask);
  float* s_vsum = reinterpret_cast<float*>(smem + L::vsum);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane / LPT, rl = lane % LPT;
  const int slot = wave * RPW + row;  // fill a wave's rows first: idle waves issue nothing
  const int N = a.N, M = a.M, K = a.K;
  const float* Lg = a.logits + static_cast<size_t>(b) * N * M;
  uint32_t* my_sorted = s_sorted + wave * (kEpl * 64) + lane;  // [s * 64]
  const int G = a.groups;
  const bool single_pass = N <= G * TPP;  // this workgroup sees each of its tokens once

  for (int e = threadIdx.x; e < MP; e += kRtThreads) {
    s_level[e] = K;
    s_cnt1[e] = 0;
    s_rank[e] = 0;
    s_key[e] = 0u;
    s_core[e] = (a.mode == DES_VANILLA && e < M) ? 1 : 0;
    s_vpart[e] = 0.f;  // the accumulator of the atomic vote variant
    s_mask[e] = 0u;
  }
  if (threadIdx.x < 36) s_hist[threadIdx.x] = 0;
  // the LDS set-up above does not need the logits: only now wait for the router
  // tiles (the wait ends with a barrier of its own)
  if (wait_router) {
    if (!flags_wait(a.flags, a.tiles_m * a.tiles_t, a.epoch, false, a.max_wait)) return false;
  } else {
    __syncthreads();
  }
  DES_STAMP(a, 14);

  uint32_t sidx = 0;     // packed original slots of the sorted positions
  uint32_t nvalid = 0;   // sorted positions [0, nvalid) hold real experts

  // Loads token n's logits, sorts this lane's 8 keys into LDS, returns the
  // unsorted values (for the softmax).
  auto load_sort = [&](int n, float (&val)[kEpl], uint32_t (&key)[kEpl]) {
    const bool live = n < N;
    const float* rowp = Lg + static_cast<size_t>(live ? n : 0) * M;
    nvalid = 0;
#pragma unroll
    for (int j = 0; j < kEpl; ++j) {
      const int idx = rl * kEpl + j;
      const bool ok = live && idx < M;
      val[j] = ok ? __hip_atomic_load(rowp + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
      key[j] = ok ? order_key(val[j]) : 0u;
      nvalid += ok ? 1u : 0u;
    }
    uint32_t sk[kEpl];
#pragma unroll
    for (int j = 0; j < kEpl; ++j) sk[j] = key[j];
    sort8_desc(sk, sidx);
#pragma unroll
    for (int j = 0; j < kEpl; ++j) my_sorted[j * 64] = sk[j];
    if (EXT && a.n_group > 1) {
      // Group-limited router (a sigma of Sec. 4.1): a group is GL adjacent lanes
      // of the row.  Its two best keys are merged from the lanes' sorted heads,
      // its score is ranked against the other groups' (ties to the lowest group),
      // and the lanes of a group that is not kept offer no candidate from here on.
      const int GL = a.group_lanes, rowbase = lane - rl;
      const int gidx = rl / GL, gsrc = min(gidx, a.n_group - 1);  // padding lanes read a real group
      uint32_t b1 = 0u, b2 = 0u;
      for (int i = 0; i < GL; ++i) {
        const int src = rowbase + gsrc * GL + i;
        const uint32_t k0 = static_cast<uint32_t>(__shfl(static_cast<int>(sk[0]), src));
        const uint32_t k1 = static_cast<uint32_t>(__shfl(static_cast<int>(sk[1]), src));
        if (k0 > b1) { b2 = max(b1, k1); b1 = k0; } else { b2 = max(b2, k0); }
      }
      uint32_t gs = b1;  // "max": the best logit's key, an exact integer comparison
      if (a.group_top2) {
        // sum of the two best router weights, fp32; positive floats order like their
        // bit patterns.  The softmax denominator is the same for every group of a
        // token, so the numerators suffice.
        const float mx = a.sigmoid ? 0.f : key_to_f32(row_max_u32<LPT>(sk[0]));
        const float s1 = !b1 ? 0.f : a.sigmoid ? sigmoid_f(key_to_f32(b1)) : exp_neg(key_to_f32(b1) - mx);
        const float s2 = !b2 ? 0.f : a.sigmoid ? sigmoid_f(key_to_f32(b2)) : exp_neg(key_to_f32(b2) - mx);
        gs = __float_as_uint(s1 + s2);
      }
      int grank = 0;
      for (int j = 0; j < a.n_group; ++j) {
        const uint32_t o = static_cast<uint32_t>(__shfl(static_cast<int>(gs), rowbase + j * GL));
        grank += (o > gs || (o == gs && j < gidx)) ? 1 : 0;
      }
      if (gidx >= a.n_group || grank >= a.topk_group) nvalid = 0;
    }
  };

  // ---------------------------------------------------------- stage 1: Phi
  if (a.mode != DES_VANILLA) {
    const bool vote = a.mode == DES_VOTE;
    const int kk = (!vote && a.k_seq > 0) ? a.k_seq : K;
    float vacc[kEpl];
#pragma unroll
    for (int j = 0; j < kEpl; ++j) vacc[j] = 0.f;

    for (int n0 = g * TPP; n0 + wave * RPW < N; n0 += G * TPP) {  // fixed token order per row
      float val[kEpl], p[kEpl];
      uint32_t key[kEpl];
      load_sort(n0 + slot, val, key);
      DES_STAMP(a, 15);
      if (vote && a.sigmoid) {  // router weights of a sigmoid router
#pragma unroll
        for (int j = 0; j < kEpl; ++j) p[j] = key[j] ? sigmoid_f(val[j]) : 0.f;
      } else if (vote) {  // softmax over all M experts (Sec. 4.3), fp32
        const float mx = key_to_f32(row_max_u32<LPT>(my_sorted[0]));
        float se = 0.f;
#pragma unroll
        for (int j = 0; j < kEpl; ++j) {
          p[j] = key[j] ? exp_neg(val[j] - mx) : 0.f;
          se += p[j];
        }
        const float den = row_sum_f32<LPT>(se);
        const float inv = den > 0.f ? 1.0f / den : 0.f;
#pragma unroll
        for (int j = 0; j < kEpl; ++j) p[j] *= inv;
      }
      DES_STAMP(a, 16);
      Head hd;
      head_set(hd, (1u << nvalid) - 1u, my_sorted);
      uint32_t taken = 0;  // original slots this token nominated
      for (int it = 0; it < kk; ++it) {  // Mask(I, K): the token's own top-K
        bool mine;
        row_draw<LPT>(hd, mine);
        if (mine) {
          const uint32_t j = (sidx >> (3 * hd.h)) & 7u;
          taken |= 1u << j;
          const int e = rl * kEpl + static_cast<int>(j);
          if (vote) {
            s_level[e] = 0;  // "nominated": only < K matters for votes
          } else {
            atomicMin(&s_level[e], it);
            if (it == 0) atomicAdd(&s_cnt1[e], 1);
          }
          head_set(hd, hd.mask & (hd.mask - 1u), my_sorted);
        }
      }
      if (vote) {
        float scale = 1.0f;
        if (a.vote_renorm) {  // the token's K weights sum to one
          float mine_sum = 0.f;
#pragma unroll
          for (int j = 0; j < kEpl; ++j) mine_sum += ((taken >> j) & 1u) ? p[j] : 0.f;
          const float tot = row_sum_f32<LPT>(mine_sum);
          scale = tot > 0.f ? 1.0f / tot : 0.f;
        }
        if (EXT && a.vote_atomic) {
          // the variant Sec. 4.3 describes: every vote is an atomic add into the
          // shared vector, in whatever order the lanes arrive
#pragma unroll
          for (int j = 0; j < kEpl; ++j)
            if ((taken >> j) & 1u) atomicAdd(&s_vpart[rl * kEpl + j], p[j] * scale);
        } else {
#pragma unroll
          for (int j = 0; j < kEpl; ++j) vacc[j] += ((taken >> j) & 1u) ? p[j] * scale : 0.f;  // Eq. 6
        }
      }
    }
    DES_STAMP(a, 2);
    if (vote && !(EXT && a.vote_atomic)) {
      // rows of a wave in a fixed pairwise order, then waves in order
#pragma unroll
      for (int j = 0; j < kEpl; ++j) {
        float v = vacc[j];
        if (RPW >= 2) v += __shfl_xor(v, LPT);
        if (RPW >= 4) v += __shfl_xor(v, 2 * LPT);
        if (RPW >= 8) v += __shfl_xor(v, 4 * LPT);
        if (RPW >= 16) v += __shfl_xor(v, 8 * LPT);
        if (row == 0) s_vpart[wave * MP + rl * kEpl + j] = v;
      }
    }
    __syncthreads();
    DES_STAMP(a, 11);

    // this workgroup's votes: waves in order (into an array of their own, so that no
    // barrier is needed between reading the partials and writing the sums)
    for (int e = threadIdx.x; e < MP; e += kRtThreads) {
      float v = 0.f;
      if (vote && !(EXT && a.vote_atomic)) {
#pragma unroll
        for (int w = 0; w < kRtWaves; ++w) v += s_vpart[w * MP + e];
      } else if (vote) {
        v = s_vpart[e];
      }
      s_vsum[e] = v;
    }
    if (G > 1) __syncthreads();
    if (G > 1) {
      // The sequence's tokens are spread over G workgroups: each publishes what
      // its tokens contributed (votes, best nomination rank, top-1 nominations),
      // waits for the others and combines all G records in group order, so every
      // workgroup of the sequence elects the same coreset from the same numbers.
      // The records travel with device-scope accesses, like the logits.
      uint32_t* mine = a.sel_part + static_cast<size_t>(b * G + g) * 3 * kSelPartStride;
      for (int e = threadIdx.x; e < MP; e += kRtThreads) {
        __hip_atomic_store(mine + e, __float_as_uint(vote ? s_vsum[e] : 0.f), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + kSelPartStride + e, static_cast<uint32_t>(s_level[e]),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + 2 * kSelPartStride + e, static_cast<uint32_t>(s_cnt1[e]),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      stores_done();
      __syncthreads();
      unsigned long long* pf = a.flags + a.tiles_m * a.tiles_t + b * G;
      if (threadIdx.x == 0) flag_publish(pf + g, a.epoch, false);
      if (!flags_wait(pf, G, a.epoch, false, a.max_wait)) return false;
      for (int e = threadIdx.x; e < MP; e += kRtThreads) {
        float v = 0.f;
        int lvl = K, c1 = 0;
        for (int gg = 0; gg < G; ++gg) {
          const uint32_t* rec = a.sel_part + static_cast<size_t>(b * G + gg) * 3 * kSelPartStride;
          v += __uint_as_float(__hip_atomic_load(rec + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          lvl = min(lvl, static_cast<int>(__hip_atomic_load(rec + kSelPartStride + e, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT)));
          c1 += static_cast<int>(__hip_atomic_load(rec + 2 * kSelPartStride + e, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT));
        }
        s_vsum[e] = v;
        s_level[e] = lvl;
        s_cnt1[e] = c1;
      }
      __syncthreads();
    }

    // (without an exchange every thread reads back only the s_vsum entry it wrote itself)
    if (vote) {
      for (int e = threadIdx.x; e < MP; e += kRtThreads) {
        const float v = s_vsum[e];
        const bool nominated = e < M && s_level[e] < K;
        s_key[e] = nominated ? order_key(v) : 0u;
        if (a.votes && e < M && !dry && g == 0) a.votes[static_cast<size_t>(b) * M + e] = v;
      }
      if (threadIdx.x == 0) s_hist[33] = 0;
    } else if (a.k_seq > 0) {  // Eq. 5 with the caller's k
      for (int e = threadIdx.x; e < MP; e += kRtThreads) s_core[e] = s_level[e] < a.k_seq;
      if (threadIdx.x == 0) s_hist[33] = a.k_seq;
    } else {  // largest k' whose union fits in C
      for (int e = threadIdx.x; e < M; e += kRtThreads)
        if (s_level[e] < K) atomicAdd(&s_hist[s_level[e]], 1);
      __syncthreads();
      if (threadIdx.x == 0) {
        int size = 0, ku = 0;
        for (int k1 = 1; k1 <= K; ++k1) {
          size += s_hist[k1 - 1];
          if (size <= a.C) ku = k1; else break;
        }
        s_hist[33] = ku;
      }
      __syncthreads();
      const int ku = s_hist[33];
      for (int e = threadIdx.x; e < MP; e += kRtThreads) {
        if (ku > 0) s_core[e] = s_level[e] < ku;
        else s_key[e] = (s_level[e] == 0) ? static_cast<uint32_t>(s_cnt1[e]) : 0u;
      }
    }
    __syncthreads();
    DES_STAMP(a, 12);

    if (vote || s_hist[33] == 0) {  // top-C by key, ties to the lowest index
      // rank[e] = #{j : key[j] beats key[e]}; the j range is split over the
      // threads that share an expert, partial counts meet in an integer LDS add
      constexpr int P = kRtThreads / MP;
      constexpr int CH = MP / P;  // keys per thread: a compile-time count (padding keys are 0
                                  // and never beat a candidate), so the reads batch up
      for (int t = threadIdx.x; t < MP * P; t += kRtThreads) {
        const int e = t % MP, part = t / MP;
        const uint32_t ke = s_key[e];
        if (ke == 0u) continue;
        const int j0 = part * CH;
        // key j beats key e if it is larger, or equal with j < e: kj >= ke for j < e,
        // kj >= ke + 1 for j >= e (a candidate's key is never the largest integer).
        // A chunk that lies wholly on one side of e needs one threshold.
        const int d = e - j0;
        int rank = 0;
        if (d <= 0 || d >= CH) {
          const uint32_t thr = ke + (d <= 0 ? 1u : 0u);
#pragma unroll
          for (int jj = 0; jj < CH; ++jj) rank += s_key[j0 + jj] >= thr ? 1 : 0;
        } else {
#pragma unroll
          for (int jj = 0; jj < CH; ++jj) rank += s_key[j0 + jj] >= ke + (jj >= d ? 1u : 0u) ? 1 : 0;
        }
        if (rank) atomicAdd(&s_rank[e], rank);
      }
    }
    __syncthreads();
  }

  DES_STAMP(a, 3);
  // ------------------------------------- coreset as an ascending index list
  // (where the election ranked keys, membership = "rank below C": the first wavefront
  // derives it here and records it for stage 2, which saves a pass and a barrier)
  const bool from_rank = a.mode != DES_VANILLA && (a.mode == DES_VOTE || s_hist[33] == 0);
  if (wave == 0) {
    int base = 0;
    int32_t* out = a.coreset_idx + static_cast<size_t>(b) * a.cap;
    for (int c = 0; c < MP; c += 64) {
      const int e = c + lane;
      const bool f = e < MP && (from_rank ? (s_key[e] != 0u && s_rank[e] < a.C) : (s_core[e] != 0));
      if (from_rank && e < MP) s_core[e] = f ? 1 : 0;
      const unsigned long long bal = __ballot(f);
      const int pre = __popcll(bal & ((1ull << lane) - 1ull));
      if (a.dense && e < MP) s_level[e] = f ? base + pre : -1;  // the expert's slot (stage 1 is done with s_level)
      if (f && base + pre < a.cap && !dry && g == 0) out[base + pre] = e;
      base += __popcll(bal);
    }
    if (!dry && g == 0)
      for (int i = base + lane; i < a.cap; i += 64) out[i] = -1;
    if (lane == 0) {
      s_hist[34] = base;
      if (!dry && g == 0) {
        a.coreset_size[b] = base;
        if (a.k_seq_used) a.k_seq_used[b] = (a.mode == DES_SEQ) ? s_hist[33] : 0;
      }
    }
  }
  __syncthreads();
  if (a.topk_idx == nullptr) return true;
  if (a.dense) {
    // The slot table of the coreset in ascending expert order, every token of the block
    // listed for every slot; stage 2 fills in who is routed where.
    if (!dry) {
      const int size = s_hist[34];
      for (int e = threadIdx.x; e < M; e += kRtThreads) {
        const int sl = s_level[e] < a.n_slots ? s_level[e] : -1;
        a.slot_of[e] = sl;
        if (sl >= 0) {
          a.slots[sl] = make_int4(e, sl * N, N, 0);
          a.tokmask[sl] = 0u;
        }
      }
      for (int sl = size + threadIdx.x; sl < a.n_slots; sl += kRtThreads) a.slots[sl] = make_int4(-1, 0, 0, 0);
      if (threadIdx.x == 0) {
        a.meta[0] = size;
        a.meta[1] = 0;
        a.meta[2] = 0;
        // provisional: the combine launch counts the experts that received a token
        a.n_unique[0] = (a.prev_n_unique != nullptr && a.prev_n_unique[0] < 0) ? -1 : size;
      }
    }
    return true;
  }

  DES_STAMP(a, 4);
  // ------------------------------ stage 2: constrained local routing + gates
  // With several selector workgroups the permutation runs in a workgroup of its own
  // and reads S_n from memory: the indices then travel with device-scope stores
  // and loads, like the logits, so the hand-off needs no fence.
  const bool idx_dev = a.use_flags && a.B * a.groups > 1;
  auto put_idx = [&](int32_t* p, int v) {
    if (idx_dev) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
  };
  const int keff = min(a.k_route, s_hist[34]);  // experts per token: Alg. 1 stage 2 with k <= K
  const bool reuse_sort = single_pass && a.mode != DES_VANILLA;  // stage 1 sorted this token

  for (int n0 = g * TPP; n0 + wave * RPW < N; n0 += G * TPP) {
    const int n = n0 + slot;
    const bool live = n < N && !dry;
    if (!reuse_sort) {
      float val[kEpl];
      uint32_t key[kEpl];
      load_sort(n, val, key);
    }
    // candidates: sorted positions whose expert sits in the coreset
    uint32_t cmask = 0;
#pragma unroll
    for (int sp = 0; sp < kEpl; ++sp) {
      const int e = rl * kEpl + static_cast<int>((sidx >> (3 * sp)) & 7u);
      cmask |= (static_cast<uint32_t>(sp) < nvalid && s_core[e] != 0) ? (1u << sp) : 0u;
    }
    Head hd;
    head_set(hd, cmask, my_sorted);
    const size_t o = (static_cast<size_t>(b) * N + (live ? n : 0)) * K;
    uint32_t mkey[NW], m0 = 0u;  // keys drawn at iterations rl, rl + LPT, ...; the first key
#pragma unroll
    for (int q = 0; q < NW; ++q) mkey[q] = 0u;
    int have = keff;  // experts this token found (fewer only under a group limit)
    for (int it = 0; it < keff; ++it) {  // S_n = TopK(I_n restricted to C, K), best first
      bool mine;
      const uint32_t m = row_draw<LPT>(hd, mine);  // every lane of the row sees the drawn key
      if (it == 0) m0 = m;
      if (m == 0u) have = min(have, it);
#pragma unroll
      for (int q = 0; q < NW; ++q)
        if (it == q * LPT + rl) mkey[q] = m;
      if (mine) {
        const int e = rl * kEpl + static_cast<int>((sidx >> (3 * hd.h)) & 7u);
        if (live) {
          put_idx(a.topk_idx + o + it, e);
          // (a block of at most 32 tokens in one workgroup: the expert's token bitmap is
          // all the permutation needs; integer LDS atomics, independent of arrival order)
          if (a.small_perm) atomicOr(&s_mask[e], 1u << n);
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
               : a.sigmoid ? sigmoid_f(key_to_f32(mkey[q]))
                           : exp_neg(key_to_f32(mkey[q]) - mx);
      part += mye[q];
    }
    float den = row_sum_f32<LPT>(part);
    DES_STAMP(a, 17);
    int keep = have;
    if (a.skip_beta > 0.f && keff > 1) {
      // Sec. 5.1 (Baselines), adapted NAEE rule: drop experts i..k when their
      // gates sum to less than beta of the total.  Tail sums from the weakest
      // expert upwards, fp32, rank order; numerators suffice (the ratio to the
      // total does not depend on the normalisation).
      const float thr = a.skip_beta * den;
      float suf = 0.f;
      for (int it = keff - 1; it >= 1; --it) {  // keff is the same for every row
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < NW; ++q) {
          const float c = __shfl(mye[q], (lane & ~(LPT - 1)) + (it % LPT));
          if (it / LPT == q) v = c;
        }
        suf += v;
        if (it < have && suf < thr) keep = it;
      }
      part = 0.f;
#pragma unroll
      for (int q = 0; q < NW; ++q) part += (q * LPT + rl < keep) ? mye[q] : 0.f;
      den = row_sum_f32<LPT>(part);  // gates re-normalised over the survivors
    }
    // g_n = softmax of the selected logits (Alg. 1 stage 2); unused slots -1 / 0
    if (live) {
#pragma unroll
      for (int q = 0; q < NW; ++q) {
        const int it = q * LPT + rl;
        if (it < K) {
          a.topk_w[o + it] = it < keep ? mye[q] / den : 0.f;
          if (it >= keep) put_idx(a.topk_idx + o + it, -1);
        }
      }
    }
  }
  return true;
}

// ----------------------------------------------------- role P: permutation
// Because a token names an expert at most once, the pairs of expert e ordered
// by (token, slot) are ordered by token alone, so a per-expert bitmap over the
// tokens gives every pair's sorted position with popcounts: no sort, no float,
// integer LDS atomics only (their result does not depend on arrival order).
// idx_dev: S_n was written by other workgroups of this launch with device-scope
// stores (read it the same way).
// MP = the kernel's padded expert count (M <= MP): the counters are kept for MP
// experts (zero past M) so that the ranking below has compile-time trip counts.
template <int MP>
__device__ void permute_all(const RoutingArgs& a, char* smem, bool idx_dev) {
  const int T = a.B * a.N, K = a.K, M = a.M;
  const int words = (T + 31) / 32;
  uint32_t* member = reinterpret_cast<uint32_t*>(smem);           // [M][words]
  int* s_cnt = reinterpret_cast<int*>(member + static_cast<size_t>(M) * words);  // [MP]
  int* s_off = s_cnt + MP;                                         // [M+1]
  int* s_liv = s_off + M + 1;                                      // [M+1]
  int* s_slot = s_liv + M + 1;                                     // [MP] slot of a live expert
  int* s_uoff = s_slot + MP;                                       // [MP] its first unit
  const int tid = threadIdx.x;
  const int TK = T * K;

  auto get_idx = [&](int p) {
    return idx_dev ? __hip_atomic_load(a.topk_idx + p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                   : a.topk_idx[p];
  };
  constexpr int kKeep = 2;  // a thread's first pairs stay in registers for the second pass
  int kept[kKeep];
  for (int i = tid; i < M * words; i += kRtThreads) member[i] = 0u;
#pragma unroll
  for (int i = 0; i < kKeep; ++i) kept[i] = tid + i * kRtThreads < TK ? get_idx(tid + i * kRtThreads) : -1;
  __syncthreads();
  auto mark = [&](int p, int e) {
    if (e >= 0) {
      const int t = p / K;
      atomicOr(&member[static_cast<size_t>(e) * words + (t >> 5)], 1u << (t & 31));
    }
  };
#pragma unroll
  for (int i = 0; i < kKeep; ++i)
    if (tid + i * kRtThreads < TK) mark(tid + i * kRtThreads, kept[i]);
  for (int p = tid + kKeep * kRtThreads; p < TK; p += kRtThreads) mark(p, get_idx(p));
  __syncthreads();
  for (int e = tid; e < MP; e += kRtThreads) {
    int c = 0;
    if (e < M)
      for (int w = 0; w < words; ++w) c += __popc(member[static_cast<size_t>(e) * words + w]);
    s_cnt[e] = c;
    s_slot[e] = 0;
    s_uoff[e] = 0;
    if (e < M) a.expert_counts[e] = c;
  }
  __syncthreads();
  // Slot order.  Up to 32 tokens every FFN task is on the chip at once and the
  // order does not matter: live experts by index.  Longer blocks: most pairs
  // first (ties to the lowest expert index), because the FFN launches hand out
  // their workgroups in slot order and, when not all of them fit on the chip at
  // once, the long ones must not be the ones that start last.  Rank by counting,
  // the comparison range split over the threads that share an expert; the
  // partial ranks meet in an integer LDS add.  The same pass counts the units
  // (groups of 2^rows_shift pairs, at most kMaxSplits per expert) of the experts
  // ahead: the expert's place in the unit list.
  const bool by_count = T > 32;
  const int rsh = a.rows_shift;
  auto units_of = [&](int c) { return min((c + (1 << rsh) - 1) >> rsh, kMaxSplits); };
  if (by_count) {
    constexpr int P = kRtThreads / MP, CH = MP / P;  // MP * P threads: each one expert, CH rivals
    const int e = tid % MP, j0 = (tid / MP) * CH;
    const int ce = s_cnt[e];
    if (ce > 0) {
      int r = 0, uo = 0;
#pragma unroll
      for (int jj = 0; jj < CH; ++jj) {  // counts past M are zero: never ahead of a live expert
        const int cj = s_cnt[j0 + jj];
        const bool ahead = cj > ce || (cj == ce && j0 + jj < e);
        r += ahead ? 1 : 0;
        uo += ahead ? units_of(cj) : 0;
      }
      if (r) {
        atomicAdd(&s_slot[e], r);
        atomicAdd(&s_uoff[e], uo);
      }
    }
  }
  if (tid < 64) {  // exclusive scans of counts and of (count > 0), 64 experts at a time
    int base_c = 0, base_l = 0;
    for (int c0 = 0; c0 < M; c0 += 64) {
      const int e = c0 + tid;
      const int c = e < M ? s_cnt[e] : 0;
      int inc = c;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d);
        if (tid >= d) inc += o;
      }
      const unsigned long long bal = __ballot(c > 0);
      const int lpre = __popcll(bal & ((1ull << tid) - 1ull));
      if (e < M) {
        s_off[e] = base_c + inc - c;
        s_liv[e] = base_l + lpre;
      }
      base_c += __shfl(inc, 63);
      base_l += __popcll(bal);
    }
    if (tid == 0) {
      s_off[M] = base_c;
      s_liv[M] = base_l;
      a.meta[0] = base_l;
      a.meta[1] = base_c;
      a.meta[2] = 0;  // live units: set after the barrier by the last slot's expert, if any
      a.n_unique[0] = (a.prev_n_unique != nullptr && a.prev_n_unique[0] < 0) ? -1 : base_l;
    }
  }
  __syncthreads();
  const int n_live = s_liv[M];
  for (int e = tid; e <= M; e += kRtThreads) a.offsets[e] = s_off[e];
  for (int e = tid; e < M; e += kRtThreads) {
    const int sl = by_count ? s_slot[e] : s_liv[e];
    const bool live = s_cnt[e] > 0 && sl < a.n_slots;
    // (up to 32 tokens the expert's bitmap row is one word: the tokens routed to it)
    if (live) a.slots[sl] = make_int4(e, s_off[e], s_cnt[e], words == 1 ? static_cast<int>(member[e]) : 0);
    a.slot_of[e] = live ? sl : -1;
    if (live && by_count) {
      const int nu = units_of(s_cnt[e]);
      for (int k = 0; k < nu; ++k) a.units[s_uoff[e] + k] = sl | (k << 16) | (nu << 24);
      if (sl == n_live - 1) a.meta[2] = s_uoff[e] + nu;  // the last slot closes the list
    }
  }
  for (int s = n_live + tid; s < a.n_slots; s += kRtThreads) a.slots[s] = make_int4(-1, 0, 0, 0);
  // entries of the slot-major token table past a slot's count must still name a
  // valid token: clear the table, then (after the barrier) fill it
  // (up to 32 tokens the FFN kernels take an expert's tokens from the bitmap in its record)
  if (T > 32)
    for (int i = tid; i < a.n_slots * kSlotToks; i += kRtThreads) a.slot_tok[i] = 0;
  __syncthreads();
  auto place = [&](int p, int e) {
    if (e < 0) { a.pos[p] = -1; return; }
    const int t = p / K;
    const uint32_t* mrow = member + static_cast<size_t>(e) * words;
    int r = s_off[e];
    for (int w = 0; w < (t >> 5); ++w) r += __popc(mrow[w]);
    r += __popc(mrow[t >> 5] & ((1u << (t & 31)) - 1u));
    a.pair_tok[r] = t;
    a.pos[p] = r;
    const int within = r - s_off[e];
    const int sl = by_count ? s_slot[e] : s_liv[e];
    if (T > 32 && within < kSlotToks && sl < a.n_slots)
      a.slot_tok[sl * kSlotToks + within] = static_cast<uint16_t>(t);
  };
#pragma unroll
  for (int i = 0; i < kKeep; ++i)
    if (tid + i * kRtThreads < TK) place(tid + i * kRtThreads, kept[i]);
  for (int p = tid + kKeep * kRtThreads; p < TK; p += kRtThreads) place(p, get_idx(p));
}

// A bounded wait ran out (a fault of the device, or another kernel keeps this
// launch's producers off the chip): leave an EMPTY work list, so that the FFN
// launches that follow find no expert, index nothing and the combine adds no
// routed row - y is then the shared expert's output (+ x under `residual`), and
// n_unique = -1 says so.  Every workgroup that gives up writes the same values.
__device__ void publish_empty(const RoutingArgs& a, int n_flags) {
  const int tid = threadIdx.x;
  if (a.slots != nullptr) {
    for (int s = tid; s < a.n_slots; s += kRtThreads) a.slots[s] = make_int4(-1, 0, 0, 0);
    for (int i = tid; i < a.B * a.N * a.K; i += kRtThreads) a.pos[i] = -1;
    for (int e = tid; e <= a.M; e += kRtThreads) a.offsets[e] = 0;
    for (int e = tid; e < a.M; e += kRtThreads) {
      a.slot_of[e] = -1;
      a.expert_counts[e] = 0;
    }
    if (tid < 3) a.meta[tid] = 0;
  }
  // the flags of this call are abandoned: clear them, so that a replay of a
  // captured launch (same epoch) starts from flags that no producer has set
  if (a.use_flags)
    for (int i = tid; i < n_flags; i += kRtThreads) a.flags[i] = 0ull;
  if (tid == 0 && a.n_unique) a.n_unique[0] = -1;
}

// The same outputs as permute_all for a block of at most 32 tokens whose selection
// ran in this workgroup: stage 2 has left, per expert, the bitmap of the tokens routed
// to it (s_mask), so counts are popcounts, an expert's pairs in token order are its set
// bits in order, and a pair's sorted position is a popcount below its token's bit.  No
// second pass over the indices to build bitmaps, no token table (the FFN kernels take
// the bitmap from the slot record).
template <int LPT>
__device__ void permute_small(const RoutingArgs& a, char* smem) {
  using L = SelLds<LPT>;
  const uint32_t* s_mask = reinterpret_cast<const uint32_t*>(smem + L::mask);
  int* s_off = reinterpret_cast<int*>(smem + L::off);
  int* s_liv = reinterpret_cast<int*>(smem + L::liv);
  const int tid = threadIdx.x, M = a.M, K = a.K, TK = a.B * a.N * a.K;
  if (tid < 64) {  // exclusive scans of counts and of (count > 0), 64 experts at a time
    int base_c = 0, base_l = 0;
    for (int c0 = 0; c0 < M; c0 += 64) {
      const int e = c0 + tid;
      const int c = e < M ? __popc(s_mask[e]) : 0;
      int inc = c;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d);
        if (tid >= d) inc += o;
      }
      const unsigned long long bal = __ballot(c > 0);
      const int lpre = __popcll(bal & ((1ull << tid) - 1ull));
      if (e < M) {
        s_off[e] = base_c + inc - c;
        s_liv[e] = base_l + lpre;
      }
      base_c += __shfl(inc, 63);
      base_l += __popcll(bal);
    }
    if (tid == 0) {
      s_off[M] = base_c;
      s_liv[M] = base_l;
      a.meta[0] = base_l;
      a.meta[1] = base_c;
      a.meta[2] = 0;
      a.n_unique[0] = (a.prev_n_unique != nullptr && a.prev_n_unique[0] < 0) ? -1 : base_l;
    }
  }
  __syncthreads();
  const int n_live = s_liv[M];
  for (int e = tid; e <= M; e += kRtThreads) a.offsets[e] = s_off[e];
  for (int e = tid; e < M; e += kRtThreads) {
    const uint32_t m = s_mask[e];
    const int c = __popc(m), sl = s_liv[e];
    const bool live = c > 0 && sl < a.n_slots;
    a.expert_counts[e] = c;
    if (live) a.slots[sl] = make_int4(e, s_off[e], c, static_cast<int>(m));
    a.slot_of[e] = live ? sl : -1;
  }
  for (int s = n_live + tid; s < a.n_slots; s += kRtThreads) a.slots[s] = make_int4(-1, 0, 0, 0);
  for (int p = tid; p < TK; p += kRtThreads) {
    const int e = a.topk_idx[p];  // (stored by this workgroup before the barrier above)
    if (e < 0) {
      a.pos[p] = -1;
      continue;
    }
    const int t = p / K;
    const int r = s_off[e] + __popc(s_mask[e] & ((1u << t) - 1u));
    a.pair_tok[r] = t;
    a.pos[p] = r;
  }
}

// ---------------------------------------------------------------- the kernel
// LDS of the routing kernel: the selection's carve-up, but at least what the
// router tile (16 KB) and the permutation (bitmap of at most 8192 words plus
// at most 5 * 512 + 2 counters, under 44 KB for every shape the library accepts) need.
constexpr int kMinRoutingLds = 44 * 1024;

template <int LPT, bool EXT>
__global__ __launch_bounds__(kRtThreads) void routing_kernel(RoutingArgs a) {
  constexpr int kLds = SelLds<LPT>::total > kMinRoutingLds ? SelLds<LPT>::total : kMinRoutingLds;
  __shared__ __align__(16) char smem[kLds];
  const int n_tiles = (a.do_router && !a.skip_router_tiles) ? a.tiles_m * a.tiles_t : 0;
  int blk = blockIdx.x;
  if (blk < n_tiles) {  // ---- role R
    if (blk == 0) DES_STAMP(a, 8);
    if (a.bf16) router_tile_bf16(a, blk % a.tiles_m, blk / a.tiles_m, reinterpret_cast<float*>(smem));
    else router_tile_f32(a, blk % a.tiles_m, blk / a.tiles_m);
    if (blk == 0) DES_STAMP(a, 9);
    if (a.use_flags) {
      stores_done();  // this thread's logits have reached the level all compute units share
      __syncthreads();
      if (threadIdx.x == 0) flag_publish(a.flags + blk, a.epoch, false);
    }
    if (blk == 0) DES_STAMP(a, 10);
    return;
  }
  blk -= n_tiles;
  const int n_sel = a.do_select ? a.B * a.groups : 0;
  const int all_tiles = a.tiles_m * a.tiles_t;
  const int n_flags = all_tiles + 2 * a.B * a.groups;
  if (blk < n_sel) {  // ---- role S
    DES_STAMP(a, 0);
    if (!select_sequence<LPT, EXT>(a, blk / a.groups, blk % a.groups, smem, false,
                              a.use_flags && a.do_router)) {
      publish_empty(a, n_flags);  // a bounded wait expired
      return;
    }
    DES_STAMP(a, 5);
    if (a.topk_idx == nullptr) return;
    if (a.dense) {  // no stage 2, no permutation here; the flags of this call are consumed
      if (a.use_flags)
        for (int i = threadIdx.x; i < n_flags; i += kRtThreads) a.flags[i] = 0ull;
      return;
    }
    if (n_sel == 1 && a.do_permute) {  // a single selector: permute right here
      // same workgroup, same compute unit: the barrier orders the topk_idx
      // stores before the loads below, no device-scope fence needed
      __syncthreads();
      DES_STAMP(a, 6);
      if (a.small_perm) permute_small<LPT>(a, smem);
      else permute_all<SelLds<LPT>::MP>(a, smem, false);
      DES_STAMP(a, 7);
      // every flag of this call has been consumed: clear them, so that a replay
      // of a captured launch (same epoch) cannot be satisfied by stale flags
      if (a.use_flags)
        for (int i = threadIdx.x; i < n_flags; i += kRtThreads) a.flags[i] = 0ull;
      return;
    }
    if (a.use_flags) {
      stores_done();
      __syncthreads();
      if (threadIdx.x == 0) flag_publish(a.flags + all_tiles + n_sel + blk, a.epoch, false);
    }
    return;
  }
  blk -= n_sel;
  if (blk == 0 && a.do_permute && a.B * a.groups > 1) {  // ---- role P
    if (a.use_flags && a.do_select &&
        !flags_wait(a.flags + all_tiles + a.B * a.groups, a.B * a.groups, a.epoch, false,
                    a.max_wait)) {
      publish_empty(a, n_flags);  // a bounded wait expired
      return;
    }
    permute_all<SelLds<LPT>::MP>(a, smem, a.use_flags && a.do_select);
    if (a.use_flags)  // all selectors have consumed the other flags and published theirs
      for (int i = threadIdx.x; i < n_flags; i += kRtThreads) a.flags[i] = 0ull;
  }
}

// probs[t][:] = router weights of token t (softmax of its logits, or their
// sigmoids); one wavefront per token (des_route only).
__global__ __launch_bounds__(64) void softmax_kernel(const float* __restrict__ logits,
                                                     float* __restrict__ probs, int M, int sigmoid) {
  const int lane = threadIdx.x;
  const float* row = logits + static_cast<size_t>(blockIdx.x) * M;
  float* out = probs + static_cast<size_t>(blockIdx.x) * M;
  if (sigmoid) {
    for (int i = lane; i < M; i += 64) out[i] = sigmoid_f(row[i]);
    return;
  }
  uint32_t mk = 0;
  for (int i = lane; i < M; i += 64) mk = max(mk, order_key(row[i]));
  const float mx = key_to_f32(wave_max_u32(mk));
  float s = 0.f;
  for (int i = lane; i < M; i += 64) s += expf(row[i] - mx);
  s = wave_sum_f32(s);
  const float inv = 1.0f / s;
  for (int i = lane; i < M; i += 64) out[i] = expf(row[i] - mx) * inv;
}

// ------------------------------------------------------------------ launchers
static int launch_routing_grid(const RoutingArgs& a, int grid, int kernel_id, hipStream_t st) {
  const int lanes = (a.M + kEpl - 1) / kEpl;  // lanes a token's experts need, 8 experts each
  const dim3 g(grid), b(kRtThreads);
#define DES_LAUNCH_ROUTING(EXT)                                                     \
  do {                                                                             \
    if (lanes <= 4) launch(kernel_id, routing_kernel<4, EXT>, g, b, 0, st, a);       \
    else if (lanes <= 8) launch(kernel_id, routing_kernel<8, EXT>, g, b, 0, st, a);  \
    else if (lanes <= 16) launch(kernel_id, routing_kernel<16, EXT>, g, b, 0, st, a); \
    else if (lanes <= 32) launch(kernel_id, routing_kernel<32, EXT>, g, b, 0, st, a); \
    else launch(kernel_id, routing_kernel<64, EXT>, g, b, 0, st, a);                 \
  } while (0)
  if (a.n_group > 1 || a.vote_atomic) DES_LAUNCH_ROUTING(true);
  else DES_LAUNCH_ROUTING(false);
#undef DES_LAUNCH_ROUTING
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "routing launch");
}

// Compute units of the current device (cached).  A routing workgroup fills a
// whole compute unit (16 wavefronts at up to 128 registers), so the fused
// launch may use at most this many workgroups if all are to be resident.
int device_compute_units() {
  static int cached_dev = -1, cached_cus = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (dev != cached_dev) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    cached_dev = dev;
    cached_cus = n;
  }
  return cached_cus;
}

static void fill_common(RoutingArgs& a, const des_shape_t& s) {
  a = RoutingArgs{};
  a.B = s.n_seqs; a.N = s.n_tokens; a.M = s.n_experts; a.K = s.top_k; a.C = s.coreset;
  a.k_seq = s.k_seq; a.mode = s.mode; a.cap = des_coreset_capacity(&s); a.D = s.hidden;
  a.n_slots = max_live_experts(s);
  a.tiles_m = (s.n_experts + 15) / 16;
  a.tiles_t = (s.n_seqs * s.n_tokens + 15) / 16;
  a.bf16 = s.dtype == DES_BF16;
  a.groups = 1;
  a.max_wait = g_test_max_wait > 0 ? g_test_max_wait : kMaxWaitIters;
  a.k_route = s.k_route > 0 ? s.k_route : s.top_k;
  a.skip_beta = s.skip_beta;
  a.sigmoid = s.router_act == DES_ROUTER_SIGMOID;
  a.vote_renorm = s.vote_renorm;
  a.vote_atomic = s.vote_atomic;
  if (s.n_group > 1 && s.topk_group < s.n_group) {  // keeping every group is no limit
    a.n_group = s.n_group;
    a.group_lanes = s.n_experts / s.n_group / kEpl;
    a.topk_group = s.topk_group;
    a.group_top2 = s.group_score == DES_GROUP_TOP2SUM;
  }
}

// The conditions of launch_routing's single launch with one selector workgroup, for a
// shape that qualifies (dense_shape): the FFN launches must take the same decision.
bool dense_block(const des_shape_t& s) {
  if (!dense_shape(s)) return false;
  int fused_limit = device_compute_units();
  if (fused_limit > kMaxFusedRoutingBlocks) fused_limit = kMaxFusedRoutingBlocks;
  const int n_tiles = ((s.n_experts + 15) / 16) * ((s.n_tokens + 15) / 16);
  return s.n_tokens <= selector_tokens_per_pass(s.n_experts) && n_tiles + 1 <= fused_limit;
}

int launch_router(const des_shape_t& s, const void* x, const void* w_router, const float* bias,
                  float* logits, hipStream_t st) {
  RoutingArgs a;
  fill_common(a, s);
  a.x = x; a.w_router = w_router; a.bias = bias; a.logits = logits;
  a.do_router = 1;
  return launch_routing_grid(a, a.tiles_m * a.tiles_t, kKRouter, st);
}

int launch_softmax(const des_shape_t& s, const float* logits, float* probs, hipStream_t st) {
  const int T = s.n_seqs * s.n_tokens;
  launch(kKSoftmax, softmax_kernel, dim3(T), dim3(64), 0, st, logits, probs, s.n_experts,
         static_cast<int>(s.router_act == DES_ROUTER_SIGMOID));
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "softmax launch");
}

int launch_select(const des_shape_t& s, const float* logits, int32_t* coreset_idx,
                  int32_t* coreset_size, float* votes, int32_t* k_seq_used, hipStream_t st) {
  RoutingArgs a;
  fill_common(a, s);
  a.logits = const_cast<float*>(logits);
  a.coreset_idx = coreset_idx; a.coreset_size = coreset_size; a.votes = votes;
  a.k_seq_used = k_seq_used;
  a.do_select = 1;
  return launch_routing_grid(a, a.B, kKSelect, st);
}

int launch_routing(const des_shape_t& s, const void* x, const void* w_router, const float* bias,
                   float* logits, int32_t* coreset_idx, int32_t* coreset_size, int32_t* topk_idx,
                   float* topk_w, int32_t* expert_counts, int32_t* n_unique,
                   const int32_t* prev_n_unique, char* ws, unsigned long long epoch,
                   hipStream_t st) {
  const WsLayout w = ws_layout(s);
  RoutingArgs a;
  fill_common(a, s);
  a.prev_n_unique = prev_n_unique;
  a.x = x; a.w_router = w_router; a.bias = bias; a.logits = logits;
  a.coreset_idx = coreset_idx; a.coreset_size = coreset_size;
  a.topk_idx = topk_idx; a.topk_w = topk_w;
  a.expert_counts = expert_counts; a.n_unique = n_unique;
  a.offsets = reinterpret_cast<int32_t*>(ws + w.offsets);
  a.slots = reinterpret_cast<int4*>(ws + w.slots);
  a.meta = reinterpret_cast<int32_t*>(ws + w.meta);
  a.pair_tok = reinterpret_cast<int32_t*>(ws + w.pair_tok);
  a.pos = reinterpret_cast<int32_t*>(ws + w.pos);
  a.flags = reinterpret_cast<unsigned long long*>(ws + w.flags);
  a.epoch = epoch;
  a.slot_of = reinterpret_cast<int32_t*>(ws + w.slot_of);
  a.units = reinterpret_cast<int32_t*>(ws + w.units);
  a.rows_shift = lds_rows_pass(s.n_seqs * s.n_tokens) == 64 ? 6 : 7;
  a.slot_tok = reinterpret_cast<uint16_t*>(ws + w.slot_tok);
  a.sel_part = reinterpret_cast<uint32_t*>(ws + w.sel_part);
  const int n_tiles = a.tiles_m * a.tiles_t;
  int fused_limit = device_compute_units();
  if (fused_limit > kMaxFusedRoutingBlocks) fused_limit = kMaxFusedRoutingBlocks;
  // A selector workgroup handles selector_tokens_per_pass() tokens at once; a
  // longer sequence is spread over several selector workgroups when they all fit.
  const int tpp = selector_tokens_per_pass(s.n_experts);
  int groups = (s.n_tokens + tpp - 1) / tpp;
  if (groups > kMaxSelGroups / a.B) groups = kMaxSelGroups / a.B > 0 ? kMaxSelGroups / a.B : 1;
  if (n_tiles + a.B * groups + 1 > fused_limit) groups = 1;
  const int roles = n_tiles + a.B * groups + (a.B * groups > 1 ? 1 : 0);
  // One selector workgroup and at most 32 tokens: the short permutation.  (Skipping
  // drops a token's experts after they were drawn, so the bitmaps of stage 2 would name
  // pairs that no longer exist: it keeps the general permutation.)
  const bool small = a.B == 1 && groups == 1 && s.n_tokens <= 32 && !(s.skip_beta > 0.0f);
  if (roles <= fused_limit) {  // all workgroups resident at once: one launch
    a.groups = groups;
    a.small_perm = small;
    a.dense = dense_block(s) ? 1 : 0;
    a.tokmask = reinterpret_cast<uint32_t*>(ws + w.tokmask);
    a.do_router = a.do_select = a.do_permute = 1;
    a.use_flags = 1;
    if (g_test_skip_router) {  // test hook: nobody computes the logits, the selectors' wait expires
      a.skip_router_tiles = 1;
      if (g_test_skip_router == 2) g_test_skip_router = g_test_max_wait = 0;  // one launch only
      return launch_routing_grid(a, roles - n_tiles, kKRouting, st);
    }
    return launch_routing_grid(a, roles, kKRouting, st);
  }
  // too large to wait inside one launch: the same roles as three launches
  RoutingArgs r = a;
  r.do_router = 1;
  int rc = launch_routing_grid(r, n_tiles, kKRouter, st);
  if (rc != DES_OK) return rc;
  RoutingArgs sel = a;
  sel.do_select = 1;
  sel.do_permute = a.B == 1 ? 1 : 0;
  sel.small_perm = a.B == 1 && s.n_tokens <= 32 && !(s.skip_beta > 0.0f);
  rc = launch_routing_grid(sel, a.B, kKSelect, st);
  if (rc != DES_OK || a.B == 1) return rc;
  RoutingArgs p = a;
  p.do_permute = 1;
  return launch_routing_grid(p, 1, kKPermute, st);
}

}  // namespace des
