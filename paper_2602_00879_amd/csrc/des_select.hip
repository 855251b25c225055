// Coreset election (Alg. 1 stage 1: Eq. 5 / Alg. 2 DES-Seq, Eq. 6 / Alg. 3
// DES-Vote), constrained re-routing with gate re-normalisation (Alg. 1 stage 2)
// and the token permutation by expert (cnt_i of Eq. 2), for gfx950.
//
// The paper's selection kernels add votes into a global vector with float
// atomics (Sec. 4.3).  Here one workgroup owns one sequence: each wavefront
// walks a fixed subset of the tokens, keeps the vote of every expert in the
// registers of the lane that owns the expert, and the per-wave partial votes
// are added through LDS in wave order.  No floating-point atomic is used, so
// the vote vector - and with it the coreset - is bit-reproducible.
//
// Every ranking is a comparison of order-preserving integer keys of the fp32
// values with ties to the lowest expert index: lane l owns the contiguous
// experts l*EPL .. l*EPL+EPL-1, so "lowest lane, lowest slot" is "lowest index".
#include "des_common.h"

namespace des {

constexpr int kSelWaves = 16;
constexpr int kSelThreads = kSelWaves * kWave;

struct SelectArgs {
  const float* logits;  // [B][N][M]
  int32_t* coreset_idx; // [B][cap]
  int32_t* coreset_size;
  float* votes;         // [B][M] or null
  int32_t* k_seq_used;  // [B] or null
  int32_t* topk_idx;    // [B][N][K] or null (then stage 2 is skipped)
  float* topk_w;
  int N, M, K, C, k_seq, mode, cap;
};

__device__ __forceinline__ float key_to_f32(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Best remaining candidate of the wavefront: returns its key (0 = none), the
// owning lane and, in that lane only, the slot `lj`.
template <int EPL>
__device__ __forceinline__ uint32_t wave_argmax(const uint32_t (&key)[EPL], int& lj,
                                                int& winner) {
  uint32_t lk = key[0];
  lj = 0;
#pragma unroll
  for (int j = 1; j < EPL; ++j)
    if (key[j] > lk) { lk = key[j]; lj = j; }
  const uint32_t m = wave_max_u32(lk);
  const unsigned long long hit = __ballot(lk == m);
  winner = __builtin_amdgcn_readfirstlane(static_cast<int>(__builtin_ctzll(hit)));
  return m;
}

template <int EPL>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a) {
  constexpr int MP = EPL * kWave;             // padded expert count
  __shared__ float s_vpart[kSelWaves][MP];    // per-wave partial votes
  __shared__ int s_level[MP];                 // best rank position at which any token names e
  __shared__ int s_cnt1[MP];                  // top-1 nominations
  __shared__ uint32_t s_key[MP];              // ranking key for the top-C pass (0 = not eligible)
  __shared__ int s_core[MP];                  // 1 = in the coreset
  __shared__ int s_hist[33];
  __shared__ int s_kused, s_csize;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int b = blockIdx.x;
  const int N = a.N, M = a.M, K = a.K;
  const float* L = a.logits + static_cast<size_t>(b) * N * M;

  for (int e = threadIdx.x; e < MP; e += kSelThreads) {
    s_level[e] = K;
    s_cnt1[e] = 0;
    s_core[e] = (a.mode == DES_VANILLA && e < M) ? 1 : 0;
  }
  if (threadIdx.x < 33) s_hist[threadIdx.x] = 0;
  __syncthreads();

  // ---------------------------------------------------------- stage 1: Phi
  if (a.mode != DES_VANILLA) {
    const bool vote = a.mode == DES_VOTE;
    const int kk = (!vote && a.k_seq > 0) ? a.k_seq : K;
    float vacc[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) vacc[j] = 0.f;

    for (int n = wave; n < N; n += kSelWaves) {  // fixed token order per wave
      const float* row = L + static_cast<size_t>(n) * M;
      float val[EPL], p[EPL];
      uint32_t key[EPL];
#pragma unroll
      for (int j = 0; j < EPL; ++j) {
        const int idx = lane * EPL + j;
        const bool ok = idx < M;
        val[j] = ok ? row[idx] : 0.f;
        key[j] = ok ? order_key(val[j]) : 0u;
        p[j] = 0.f;
      }
      if (vote) {  // softmax over all M experts (Sec. 4.3), fp32
        uint32_t lk = key[0];
#pragma unroll
        for (int j = 1; j < EPL; ++j) lk = max(lk, key[j]);
        const float mx = key_to_f32(wave_max_u32(lk));
        float se = 0.f;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
          p[j] = key[j] ? expf(val[j] - mx) : 0.f;
          se += p[j];
        }
        const float inv = 1.0f / wave_sum_f32(se);
#pragma unroll
        for (int j = 0; j < EPL; ++j) p[j] *= inv;
      }
      for (int it = 0; it < kk; ++it) {  // Mask(I, K): the token's own top-K
        int lj, winner;
        if (wave_argmax<EPL>(key, lj, winner) == 0u) break;
        if (lane == winner) {
#pragma unroll
          for (int j = 0; j < EPL; ++j)
            if (j == lj) {
              key[j] = 0u;
              vacc[j] += p[j];  // V_i += masked weight (Eq. 6)
              atomicMin(&s_level[lane * EPL + j], it);
              if (it == 0) atomicAdd(&s_cnt1[lane * EPL + j], 1);
            }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < EPL; ++j) s_vpart[wave][lane * EPL + j] = vacc[j];
    __syncthreads();

    if (vote) {
      for (int e = threadIdx.x; e < MP; e += kSelThreads) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) v += s_vpart[w][e];  // wave order: fixed
        const bool nominated = e < M && s_level[e] < K;
        s_key[e] = nominated ? order_key(v) : 0u;
        if (a.votes && e < M) a.votes[static_cast<size_t>(b) * M + e] = v;
      }
      if (threadIdx.x == 0) s_kused = 0;
    } else if (a.k_seq > 0) {  // Eq. 5 with the caller's k
      for (int e = threadIdx.x; e < MP; e += kSelThreads) s_core[e] = s_level[e] < a.k_seq;
      if (threadIdx.x == 0) s_kused = a.k_seq;
    } else {  // largest k' whose union fits in C
      for (int e = threadIdx.x; e < M; e += kSelThreads)
        if (s_level[e] < K) atomicAdd(&s_hist[s_level[e]], 1);
      __syncthreads();
      if (threadIdx.x == 0) {
        int size = 0, ku = 0;
        for (int k1 = 1; k1 <= K; ++k1) {
          size += s_hist[k1 - 1];
          if (size <= a.C) ku = k1; else break;
        }
        s_kused = ku;
      }
      __syncthreads();
      const int ku = s_kused;
      for (int e = threadIdx.x; e < MP; e += kSelThreads) {
        if (ku > 0) s_core[e] = s_level[e] < ku;
        else s_key[e] = (s_level[e] == 0) ? static_cast<uint32_t>(s_cnt1[e]) : 0u;
      }
    }
    __syncthreads();

    if (vote || s_kused == 0) {  // top-C by key, ties to the lowest index
      for (int e = threadIdx.x; e < MP; e += kSelThreads) {
        const uint32_t ke = s_key[e];
        int rank = 0;
        for (int j = 0; j < M; ++j) {
          const uint32_t kj = s_key[j];
          rank += (kj > ke || (kj == ke && j < e)) ? 1 : 0;
        }
        s_core[e] = (ke != 0u && rank < a.C) ? 1 : 0;
      }
    }
    __syncthreads();
  }

  // ------------------------------------- coreset as an ascending index list
  if (wave == 0) {
    int base = 0;
    int32_t* out = a.coreset_idx + static_cast<size_t>(b) * a.cap;
#pragma unroll 1
    for (int c = 0; c < EPL; ++c) {
      const int e = c * 64 + lane;
      const bool f = s_core[e] != 0;
      const unsigned long long bal = __ballot(f);
      const int pre = __popcll(bal & ((1ull << lane) - 1ull));
      if (f && base + pre < a.cap) out[base + pre] = e;
      base += __popcll(bal);
    }
    for (int i = base + lane; i < a.cap; i += 64) out[i] = -1;
    if (lane == 0) {
      a.coreset_size[b] = base;
      s_csize = base;
      if (a.k_seq_used) a.k_seq_used[b] = (a.mode == DES_SEQ) ? s_kused : 0;
    }
  }
  __syncthreads();
  if (a.topk_idx == nullptr) return;

  // ------------------------------ stage 2: constrained local routing + gates
  const int keff = min(K, s_csize);
  bool cm[EPL];
#pragma unroll
  for (int j = 0; j < EPL; ++j) cm[j] = (lane * EPL + j < M) && s_core[lane * EPL + j] != 0;

  for (int n = wave; n < N; n += kSelWaves) {
    const float* row = L + static_cast<size_t>(n) * M;
    float val[EPL];
    uint32_t key[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      val[j] = cm[j] ? row[lane * EPL + j] : 0.f;
      key[j] = cm[j] ? order_key(val[j]) : 0u;
    }
    int sel_idx = -1;
    float sel_val = 0.f;
    for (int it = 0; it < keff; ++it) {  // S_n = TopK(I_n restricted to C, K)
      int lj, winner;
      wave_argmax<EPL>(key, lj, winner);
      float lv = val[0];
#pragma unroll
      for (int j = 1; j < EPL; ++j)
        if (j == lj) lv = val[j];
      const int widx = __builtin_amdgcn_readlane(lane * EPL + lj, winner);
      const float wval = readlane_f32(lv, winner);
      if (lane == it) { sel_idx = widx; sel_val = wval; }
      if (lane == winner) {
#pragma unroll
        for (int j = 0; j < EPL; ++j)
          if (j == lj) key[j] = 0u;
      }
    }
    // g_n = softmax of the selected logits; slot 0 holds the largest
    const float mx = readlane_f32(sel_val, 0);
    const float ex = lane < keff ? expf(sel_val - mx) : 0.f;
    const float den = wave_sum_f32(ex);
    if (lane < K) {
      const size_t o = (static_cast<size_t>(b) * N + n) * K + lane;
      a.topk_idx[o] = lane < keff ? sel_idx : -1;
      a.topk_w[o] = lane < keff ? ex / den : 0.f;
    }
  }
}

// ----------------------------------------------------------------------------
// Token permutation by expert.  One workgroup.  Because a token names an
// expert at most once, the pairs of expert e ordered by (token, slot) are
// ordered by token alone, so a per-expert bitmap over tokens gives every
// pair's position with two popcounts: no sort, no float, integer LDS atomics
// only (their result does not depend on arrival order).
// ----------------------------------------------------------------------------
constexpr int kPermThreads = 1024;

__global__ __launch_bounds__(kPermThreads) void permute_kernel(
    const int32_t* __restrict__ topk_idx, int32_t* __restrict__ expert_counts,
    int32_t* __restrict__ n_unique, int32_t* __restrict__ offsets, int32_t* __restrict__ live,
    int32_t* __restrict__ meta, int32_t* __restrict__ perm, int32_t* __restrict__ pos, int T,
    int K, int M, int words /* ceil(T/32) */) {
  extern __shared__ uint32_t s_mem[];
  uint32_t* member = s_mem;                                    // [M][words]
  int* s_cnt = reinterpret_cast<int*>(s_mem + static_cast<size_t>(M) * words);  // [M] counts
  int* s_off = s_cnt + M;                                      // [M+1] exclusive offsets
  int* s_liv = s_off + M + 1;                                  // [M+1] exclusive live flags
  const int tid = threadIdx.x;
  const int TK = T * K;

  for (int i = tid; i < M * words; i += kPermThreads) member[i] = 0u;
  __syncthreads();
  for (int p = tid; p < TK; p += kPermThreads) {
    const int e = topk_idx[p];
    if (e >= 0) {
      const int t = p / K;
      atomicOr(&member[static_cast<size_t>(e) * words + (t >> 5)], 1u << (t & 31));
    }
  }
  __syncthreads();
  for (int e = tid; e < M; e += kPermThreads) {
    int c = 0;
    for (int w = 0; w < words; ++w) c += __popc(member[static_cast<size_t>(e) * words + w]);
    s_cnt[e] = c;
    expert_counts[e] = c;
  }
  __syncthreads();
  // exclusive scans of counts and of (count > 0); M <= 512 so one wave walks
  // 64-wide chunks with a running base
  if (tid < 64) {
    int base_c = 0, base_l = 0;
    for (int c0 = 0; c0 < M; c0 += 64) {
      const int e = c0 + tid;
      const int c = e < M ? s_cnt[e] : 0;
      int inc = c;  // inclusive scan across the wave
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
      meta[0] = base_l;
      meta[1] = base_c;
      n_unique[0] = base_l;
    }
  }
  __syncthreads();
  for (int e = tid; e <= M; e += kPermThreads) offsets[e] = s_off[e];
  for (int e = tid; e < M; e += kPermThreads)
    if (s_cnt[e] > 0) live[s_liv[e]] = e;
  for (int p = tid; p < TK; p += kPermThreads) {
    const int e = topk_idx[p];
    if (e < 0) { pos[p] = -1; continue; }
    const int t = p / K;
    const uint32_t* mrow = member + static_cast<size_t>(e) * words;
    int r = s_off[e];
    for (int w = 0; w < (t >> 5); ++w) r += __popc(mrow[w]);
    r += __popc(mrow[t >> 5] & ((1u << (t & 31)) - 1u));
    perm[r] = p;
    pos[p] = r;
  }
}

static int select_dispatch(const SelectArgs& a, int B, hipStream_t st) {
  const int epl = (a.M + 63) / 64;
  if (epl <= 1) hipLaunchKernelGGL(select_kernel<1>, dim3(B), dim3(kSelThreads), 0, st, a);
  else if (epl <= 2) hipLaunchKernelGGL(select_kernel<2>, dim3(B), dim3(kSelThreads), 0, st, a);
  else if (epl <= 4) hipLaunchKernelGGL(select_kernel<4>, dim3(B), dim3(kSelThreads), 0, st, a);
  else hipLaunchKernelGGL(select_kernel<8>, dim3(B), dim3(kSelThreads), 0, st, a);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "select launch");
}

int launch_select(const des_shape_t& s, const float* logits, int32_t* coreset_idx,
                  int32_t* coreset_size, float* votes, int32_t* k_seq_used, int32_t* topk_idx,
                  float* topk_w, hipStream_t st) {
  SelectArgs a;
  a.logits = logits;
  a.coreset_idx = coreset_idx;
  a.coreset_size = coreset_size;
  a.votes = votes;
  a.k_seq_used = k_seq_used;
  a.topk_idx = topk_idx;
  a.topk_w = topk_w;
  a.N = s.n_tokens;
  a.M = s.n_experts;
  a.K = s.top_k;
  a.C = s.coreset;
  a.k_seq = s.k_seq;
  a.mode = s.mode;
  a.cap = des_coreset_capacity(&s);
  return select_dispatch(a, s.n_seqs, st);
}

int launch_permute(const des_shape_t& s, const int32_t* topk_idx, int32_t* expert_counts,
                   int32_t* n_unique, char* ws, hipStream_t st) {
  const WsLayout w = ws_layout(s);
  const int T = s.n_seqs * s.n_tokens;
  const int words = (T + 31) / 32;
  const size_t lds = 4 * (static_cast<size_t>(s.n_experts) * words + 3 * s.n_experts + 2);
  hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(kPermThreads), lds, st, topk_idx,
                     expert_counts, n_unique, reinterpret_cast<int32_t*>(ws + w.offsets),
                     reinterpret_cast<int32_t*>(ws + w.live),
                     reinterpret_cast<int32_t*>(ws + w.meta),
                     reinterpret_cast<int32_t*>(ws + w.perm),
                     reinterpret_cast<int32_t*>(ws + w.pos), T, s.top_k, s.n_experts, words);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "permute launch");
}

}  // namespace des
