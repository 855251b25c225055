// The attention sub-layer of a block-parallel decoding step, for gfx950: every token of
// the block attends to the cached prefix / suffix positions and to the whole block
// (Sec. 5.1 fixes that window; Fig. 2 left and Sec. 5.2 count attention among the fixed,
// non-MoE costs of a step).  The paper does not define the sub-layer; this is plain
// multi-head scaled-dot-product attention without mask, positional encoding or bias.
//
// Three launches per sub-layer:
//   1. q, k, v = x Wq^T, x Wk^T, x Wv^T     one dense-projection launch over the three
//                                            weight matrices (bf16 MFMA, fp32 accumulate)
//   2. softmax(q K^T / sqrt(dh)) V           one workgroup per (sequence, head), bf16 MFMA
//   3. y = heads Wo^T (+ x)                  the same projection kernel, residual fused
// The projections are weight scans like the expert FFN (a 2048 x 2048 matrix is 8 MB for
// at most a few hundred token rows), so they reuse its streaming building block: weights
// from HBM straight into MFMA operands, token rows staged through LDS.
#include "des_common.h"
#include "des_stream_gemm.h"

namespace des {

struct LinearArgs {
  const uint16_t* in;    // [T][Din] bf16 token rows
  const uint16_t* w[3];  // up to three weight matrices [fout[i]][Din], rows along the reduction
  uint16_t* out[3];      // [T][fout[i]] bf16
  const uint16_t* res;   // [T][fout[0]] bf16 added to out[0] before rounding, or null
  int fout[3];
  int n_mats, T, Din;
  // short blocks, reduction dimension split over two workgroups (ksplit = 2):
  int ksplit;
  float* partial;             // [workgroups][tiles of a workgroup][64 lanes][4] fp32 partial tiles
  unsigned long long* flags;  // [workgroup pairs] set to `epoch` by the half that finishes first
  unsigned long long epoch;   // of this call: never zero, never repeated (stale words cannot match)
};

// Arrival count of the workgroups that share an output tile (reduction dimension split
// over several workgroups).  The word holds (call's epoch << 8 | arrivals); whatever it
// held before this call - garbage, an earlier call's count - is not this epoch and reads
// as zero arrivals, so nothing has to be cleared beforehand.  Returns this workgroup's
// arrival number, 1-based.  Device-scope compare-and-swap; nobody ever waits for anybody.
__device__ __forceinline__ int arrive(unsigned long long* word, unsigned long long epoch) {
  const unsigned long long tag = (epoch & 0x00ffffffffffffffull) << 8;
  unsigned long long cur = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (;;) {
    const unsigned long long base = (cur & ~0xffull) == tag ? cur : tag;
    const unsigned long long want = base + 1ull;
    if (__hip_atomic_compare_exchange_strong(word, &cur, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT))
      return static_cast<int>(want & 0xffull);
  }
}

// out[m][t][f] = sum_d in[t][d] * w[m][f][d].  A workgroup of LW wavefronts owns LW pairs
// of 16-row weight tiles of one matrix and up to ROWS (64 or 128) token rows (blockIdx.y
// names which; the weights are streamed once per ROWS rows).  KD = the reduction length of a workgroup if
// it is one of the unrolled ones (1024, 2048, 4096), else 0.  With ksplit > 1 the reduction
// dimension is split over that many workgroups (blockIdx.z): each writes its fp32 partial
// tiles with device-scope stores and counts itself in; the last to arrive adds all the
// partials in order of their part of the reduction dimension, whoever finished when.
template <int LW, int KD, int ROWS>
__global__ __launch_bounds__(LW* kWave, 2) void linear_lds_kernel(LinearArgs a) {
  constexpr int kRows = ROWS;
  __shared__ __align__(16) uint16_t lds[lds_elems(KD)];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int part = blockIdx.z, kd = a.Din / a.ksplit, k0 = part * kd;
  int bx = blockIdx.x, m = 0;
  for (; m < a.n_mats; ++m) {  // which matrix this workgroup belongs to
    const int per = (a.fout[m] / 32 + LW - 1) / LW;
    if (bx < per) break;
    bx -= per;
  }
  if (m >= a.n_mats) return;
  const int fout = a.fout[m], Din = a.Din;
  const int pair = bx * LW + wave;          // pair of row tiles this wavefront owns
  const bool active = pair * 2 < fout / 16;
  const uint16_t* w = uniform_ptr(a.w[m]);
  const uint16_t* p0 = tile_base<false>(w, active ? pair * 2 : 0, Din) + k0;
  const uint16_t* p1 = tile_base<false>(w, active ? pair * 2 + 1 : 0, Din) + k0;
  const uint32_t wlo = tile_lane_off<false>(Din, lane);
  const uint16_t* in = uniform_ptr(a.in) + k0;
  // this output tile's place among the launch's (x, y) workgroups: its partials and counter
  const size_t tile_id = static_cast<size_t>(blockIdx.y) * gridDim.x + blockIdx.x;
  uint16_t* out = a.out[m];
  const uint16_t* res = m == 0 ? a.res : nullptr;
  {  // one pass of up to 128 token rows per workgroup (blockIdx.y)
    const int g0 = blockIdx.y * kRows;
    const int rows = min(kRows, a.T - g0);
    const int nt = (rows + 15) / 16;
    auto row_off = [&](int r) { return (g0 + r) * Din; };
    auto run = [&](auto ntc) {
      constexpr int NT = decltype(ntc)::value;
      f32x4 acc0[NT], acc1[NT];
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        acc0[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      constexpr int KC = NT <= 4 ? 128 : 64;
      dma_stream_gemm<NT, kLdsBufElems / KC, false, LW, KC, KD>(p0, p1, wlo, wave, kd, rows, in, row_off, lds,
                                                                 acc0, acc1);
      if (a.ksplit > 1) {
        // partial tiles of this wavefront: [tile][part][wave][2][8 token tiles][64 lanes][4]
        constexpr size_t kPerWave = 2 * 8 * 256;
        float* base = a.partial + (tile_id * a.ksplit * LW) * kPerWave;
        float* mine = base + (static_cast<size_t>(part) * LW + wave) * kPerWave;
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            __hip_atomic_store(mine + (i * 64 + lane) * 4 + q, acc0[i][q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(mine + ((8 + i) * 64 + lane) * 4 + q, acc1[i][q], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
          }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's partials have left the compute unit
        __shared__ int s_last;
        __syncthreads();
        if (tid == 0) {
          s_last = arrive(a.flags + tile_id, a.epoch) == a.ksplit ? 1 : 0;
          // everybody has arrived: clear the count, so that a replay of a captured launch
          // (same epoch) counts from zero again
          if (s_last) __hip_atomic_store(a.flags + tile_id, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!s_last) return;
#pragma unroll
        for (int i = 0; i < NT; ++i) {
          acc0[i] = f32x4{0.f, 0.f, 0.f, 0.f};
          acc1[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (int h = 0; h < a.ksplit; ++h) {  // parts in order, not in order of arrival
          const float* src = base + (static_cast<size_t>(h) * LW + wave) * kPerWave;
#pragma unroll
          for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              acc0[i][q] += __hip_atomic_load(src + (i * 64 + lane) * 4 + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              acc1[i][q] += __hip_atomic_load(src + ((8 + i) * 64 + lane) * 4 + q, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
            }
        }
      }
      if (!active) return;
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const int pi = g0 + i * 16 + (lane & 15);
        if (pi < a.T) {
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const f32x4 v = half ? acc1[i] : acc0[i];
            const size_t o = static_cast<size_t>(pi) * fout + (pair * 2 + half) * 16 + 4 * (lane >> 4);
            f32x4 r = v;
            if (res != nullptr) {
              const u16x4 rv = *reinterpret_cast<const u16x4*>(res + o);
#pragma unroll
              for (int q = 0; q < 4; ++q) r[q] += bf16_bits_to_f32(rv[q]);
            }
            u16x4 ob;
#pragma unroll
            for (int q = 0; q < 4; ++q) ob[q] = f32_to_bf16_bits(r[q]);
            *reinterpret_cast<u16x4*>(out + o) = ob;
          }
        }
      }
    };
    if (nt <= 1) run(std::integral_constant<int, 1>{});
    else if (nt <= 2) run(std::integral_constant<int, 2>{});
    else if (kRows <= 64 || nt <= 4) run(std::integral_constant<int, 4>{});
    else if (nt <= 6) run(std::integral_constant<int, kRows <= 64 ? 4 : 6>{});
    else run(std::integral_constant<int, kRows <= 64 ? 4 : 8>{});
  }
}

// The same projection for blocks of at most 32 token rows, where the weights are a pure
// stream and what matters is how many wavefronts pull on it at once: a workgroup owns RT
// 16-row weight tiles, its wavefronts split the reduction dimension (each streams a
// contiguous run of every row straight into MFMA A operands, two stages of U k-steps
// in flight; the token rows come from L2 as the B operand, each fragment used for the RT
// tiles), and the partial tiles are added through LDS in wavefront order, so the result
// does not depend on timing.
template <int RT, int NT>
__global__ __launch_bounds__(512) void linear_splitk_kernel(LinearArgs a) {
  constexpr int U = RT >= 4 ? 2 : 4;
  __shared__ __align__(16) float part[8 * RT * NT * 256];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_waves = blockDim.x >> 6;
  const int half = blockIdx.x % a.ksplit, pair_id = blockIdx.x / a.ksplit;
  int grp_i = pair_id, m = 0;
  for (; m < a.n_mats; ++m) {  // which matrix this workgroup belongs to
    const int per = (a.fout[m] / 16 + RT - 1) / RT;
    if (grp_i < per) break;
    grp_i -= per;
  }
  if (m >= a.n_mats) return;
  const int fout = a.fout[m], Din = a.Din;
  const int n_tiles = fout / 16;
  const int kwg = Din / a.ksplit;                   // reduction elements of this workgroup
  const int kper = kwg / n_waves, nks = kper / 32;  // the host makes kper a multiple of 32
  const int k0 = half * kwg + wave * kper;
  const int col = lane & 15, grp = lane >> 4;
  const uint16_t* wp[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r)  // a tile past the matrix repeats the last one, dropped at the store
    wp[r] = a.w[m] + (static_cast<size_t>(min(grp_i * RT + r, n_tiles - 1)) * 16 + col) * Din + k0 + grp * 8;
  const uint16_t* xp[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i)  // rows past the block repeat the last token, dropped at the store
    xp[i] = a.in + static_cast<size_t>(min(i * 16 + col, a.T - 1)) * Din + k0 + grp * 8;
  f32x4 acc[RT][NT];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[r][i] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 aw[2][U][RT], bx[2][U][NT];
  auto load = [&](int ks, auto stage) {
    constexpr int st = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = ks + u < nks;
      bf16x8 z;
#pragma unroll
      for (int q = 0; q < 8; ++q) z[q] = static_cast<__bf16>(0.0f);
#pragma unroll
      for (int r = 0; r < RT; ++r)
        aw[st][u][r] = in ? __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(wp[r] + (ks + u) * 32)) : z;
#pragma unroll
      for (int i = 0; i < NT; ++i)
        bx[st][u][i] = in ? *reinterpret_cast<const bf16x8*>(xp[i] + (ks + u) * 32) : z;
    }
  };
  auto compute = [&](auto stage) {
    constexpr int st = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int i = 0; i < NT; ++i)
          acc[r][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw[st][u][r], bx[st][u][i], acc[r][i], 0, 0, 0);
  };
  load(0, S0{});
  for (int ks = 0; ks < nks; ks += 2 * U) {
    load(ks + U, S1{});
    compute(S0{});
    load(ks + 2 * U, S0{});
    compute(S1{});
  }
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int i = 0; i < NT; ++i)
      *reinterpret_cast<f32x4*>(part + (((wave * RT + r) * NT + i) * 64 + lane) * 4) = acc[r][i];
  __syncthreads();
  // wavefront w finishes the tiles w, w + n_waves, ... of the workgroup's RT x NT
  uint16_t* out = a.out[m];
  const uint16_t* res = m == 0 ? a.res : nullptr;
  if (a.ksplit == 2) {
    // Two workgroups share these rows, each with half of the reduction dimension.  Both
    // write their partial tiles with device-scope stores, wait for them, and swap the
    // call's epoch into the pair's flag: the one that gets the epoch back is the second to
    // arrive, and it alone goes on - with both partials read back and added as
    // (first half) + (second half), whoever finished first.  No spinning: nobody waits.
    float* mine = a.partial + static_cast<size_t>(blockIdx.x) * (RT * NT * 256);
    for (int t = wave; t < RT * NT; t += n_waves) {
      const int r = t / NT, i = t % NT;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < n_waves; ++w) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(part + (((w * RT + r) * NT + i) * 64 + lane) * 4);
#pragma unroll
        for (int q = 0; q < 4; ++q) sum[q] += v[q];
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        __hip_atomic_store(mine + (t * 64 + lane) * 4 + q, sum[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's partials have left the compute unit
    __shared__ int s_second;
    __syncthreads();
    if (tid == 0) {
      const unsigned long long old =
          __hip_atomic_exchange(a.flags + pair_id, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_second = old == a.epoch ? 1 : 0;
      // the pair is complete: clear the flag, so that a replay of a captured launch (same
      // epoch) starts from a flag nobody has set
      if (old == a.epoch) __hip_atomic_store(a.flags + pair_id, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_second) return;
  }
  const float* p0 = a.partial + static_cast<size_t>(pair_id) * 2 * (RT * NT * 256);
  for (int t = wave; t < RT * NT; t += n_waves) {
    const int r = t / NT, i = t % NT;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    if (a.ksplit == 2) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float lo = __hip_atomic_load(p0 + (t * 64 + lane) * 4 + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float hi = __hip_atomic_load(p0 + RT * NT * 256 + (t * 64 + lane) * 4 + q, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
        sum[q] = lo + hi;
      }
    } else {
      for (int w = 0; w < n_waves; ++w) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(part + (((w * RT + r) * NT + i) * 64 + lane) * 4);
#pragma unroll
        for (int q = 0; q < 4; ++q) sum[q] += v[q];
      }
    }
    const int tok = i * 16 + col, tile = grp_i * RT + r;
    if (tok < a.T && tile < n_tiles) {
      const size_t o = static_cast<size_t>(tok) * fout + tile * 16 + 4 * grp;
      if (res != nullptr) {
        const u16x4 rv = *reinterpret_cast<const u16x4*>(res + o);
#pragma unroll
        for (int q = 0; q < 4; ++q) sum[q] += bf16_bits_to_f32(rv[q]);
      }
      u16x4 ob;
#pragma unroll
      for (int q = 0; q < 4; ++q) ob[q] = f32_to_bf16_bits(sum[q]);
      *reinterpret_cast<u16x4*>(out + o) = ob;
    }
  }
}

struct AttnArgs {
  const uint16_t *q, *k, *v;           // [T][H*dh], [T][Hkv*dh], [T][Hkv*dh] of the block's own tokens
  const uint16_t *k_cache, *v_cache;   // [B][Hkv][P][dh] cached positions (prefix, then suffix)
  uint16_t* o;                         // [T][H*dh] per-head outputs
  int B, N, H, Hkv, dh, P;
  float scale;                         // 1 / sqrt(dh)
};

// One workgroup (four wavefronts) per (sequence, query head); each wavefront takes tiles
// of 16 queries.  Scores and the weighted sum of values are bf16 MFMA contractions with
// fp32 accumulation, laid out so that no operand needs a transpose between them:
//   S^T = K Q^T    A = keys (16 per tile, straight from global memory), B = the 16 queries
//                  -> lane l holds query l % 16, keys 4 (l / 16) .. + 3 of the tile
//   O^T = V^T P^T  B = the weights of two score tiles as they sit in those registers (the
//                  contraction only needs A and B to agree on which key a slot means),
//                  A = values transposed in LDS, read with that same key order
//                  -> lane l holds query l % 16, coordinates 4 (l / 16) .. + 3 of the tile
// The softmax is two passes over the keys (maximum first, then weights and sums; the
// scores are recomputed - a handful of MFMAs - when the window exceeds 64 positions)
// instead of a running rescale; weights are
// rounded to bf16 for the second contraction, their sum is kept in fp32.  Sums run in a
// fixed order, so results are reproducible.
__global__ __launch_bounds__(256) void attention_core_kernel(AttnArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* vt = reinterpret_cast<uint16_t*>(smem_raw);  // [ndt * 16][ldv]: values, transposed
  const int N = a.N, dh = a.dh, P = a.P, nk = a.P + a.N;
  const int nkp = (nk + 31) & ~31, ldv = nkp + 4;
  const int ndt = (dh + 15) / 16, nks = (dh + 31) / 32, nkt = (nk + 15) / 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const int g = h / (a.H / a.Hkv);
  const size_t cbase = (static_cast<size_t>(b) * a.Hkv + g) * P * dh;
  const uint16_t* kc = a.k_cache + cbase;  // cached keys / values of this head (unused if P == 0)
  const uint16_t* vc = a.v_cache + cbase;
  const size_t brow = static_cast<size_t>(b) * N * a.Hkv * dh + static_cast<size_t>(g) * dh;
  const uint16_t* kb = a.k + brow;         // the block's own keys / values, row stride Hkv * dh
  const uint16_t* vb = a.v + brow;
  const int bstride = a.Hkv * dh;
  const int col = lane & 15, grp = lane >> 4;
  const float neg_inf = -__builtin_inff();
  auto key_row = [&](int j) -> const uint16_t* {
    return j < P ? kc + static_cast<size_t>(j) * dh : kb + static_cast<size_t>(j - P) * bstride;
  };
  auto load8 = [&](const uint16_t* row, int s) -> bf16x8 {  // elements 32 s + 8 grp .. + 7, zeros past dh
    const int e = 32 * s + 8 * grp;
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (e < dh) raw = *reinterpret_cast<const uint4*>(row + e);
    return __builtin_bit_cast(bf16x8, raw);
  };
  // values -> LDS, transposed; key slots beyond the window hold zeros (their weights are
  // zero too, but 0 x garbage could be NaN).  A thread's first four pieces are requested
  // here and written after the first pass over the keys, which does not need them: the
  // three kinds of loads (values, queries, keys) then share one round trip.
  const int vec = dh / 8, n_piece = nkp * vec;
  auto value_piece = [&](int i) -> uint4 {
    const int j = i / vec, c = (i % vec) * 8;
    if (i >= n_piece || j >= nk) return make_uint4(0u, 0u, 0u, 0u);
    const uint16_t* src = j < P ? vc + static_cast<size_t>(j) * dh : vb + static_cast<size_t>(j - P) * bstride;
    return *reinterpret_cast<const uint4*>(src + c);
  };
  auto store_piece = [&](int i, const uint4& raw) {
    if (i >= n_piece) return;
    const int j = i / vec, c = (i % vec) * 8;
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      vt[(c + 2 * q) * ldv + j] = static_cast<uint16_t>(w[q] & 0xffffu);
      vt[(c + 2 * q + 1) * ldv + j] = static_cast<uint16_t>(w[q] >> 16);
    }
  };
  uint4 vraw[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) vraw[q] = value_piece(tid + 256 * q);

  bf16x8 qf[4];
  f32x4 sc[4];
  int n = 0;
  float mx = neg_inf;
  auto load_queries = [&](int qt) {
    n = min(qt * 16 + col, N - 1);  // rows past the block repeat the last query, not stored
    const uint16_t* qrow = a.q + (static_cast<size_t>(b) * N + n) * (a.H * dh) + static_cast<size_t>(h) * dh;
#pragma unroll
    for (int s = 0; s < 4; ++s) qf[s] = s < nks ? load8(qrow, s) : bf16x8{};
  };
  // scores of four key tiles at once, every key fragment requested before the first is
  // used (one round trip to L2 instead of sixteen); lane: keys 16 t + 4 grp + r of its query
  auto score_batch = [&](int t0) {
    bf16x8 kf[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint16_t* krow = key_row(min(16 * (t0 + i) + col, nk - 1));
#pragma unroll
      for (int s = 0; s < 4; ++s) kf[i][s] = (s < nks && t0 + i < nkt) ? load8(krow, s) : bf16x8{};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (s < nks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[i][s], qf[s], acc, 0, 0, 0);
      sc[i] = acc;
    }
  };
  auto first_pass = [&](int qt) {  // the largest score of each query
    load_queries(qt);
    mx = neg_inf;
    for (int t0 = 0; t0 < nkt; t0 += 4) {
      score_batch(t0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (16 * (t0 + i) + 4 * grp + r < nk) mx = fmaxf(mx, sc[i][r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
  };
  auto second_pass = [&](int qt) {  // weights, their sum, the weighted values; store
    f32x4 oacc[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f;
    for (int t0 = 0; t0 < nkt; t0 += 4) {
      if (nkt > 4) score_batch(t0);  // a window of at most 64 positions still has them
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const int c = t0 / 2 + cc;  // 32 keys: tiles 2 c and 2 c + 1
        if (c * 32 < nkp) {
          u16x4 pw[2];
#pragma unroll
          for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float pr =
                  16 * (2 * c + half) + 4 * grp + r < nk ? expf((sc[2 * cc + half][r] - mx) * a.scale) : 0.f;
              lsum += pr;
              pw[half][r] = f32_to_bf16_bits(pr);
            }
          }
          struct { u16x4 lo, hi; } pp = {pw[0], pw[1]};
          const bf16x8 pb = __builtin_bit_cast(bf16x8, pp);
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) {
            if (dt < ndt) {
              const uint16_t* vrow = vt + (16 * dt + col) * ldv + 32 * c + 4 * grp;
              struct { u16x4 lo, hi; } vv = {*reinterpret_cast<const u16x4*>(vrow),
                                             *reinterpret_cast<const u16x4*>(vrow + 16)};
              oacc[dt] =
                  __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv), pb, oacc[dt], 0, 0, 0);
            }
          }
        }
      }
    }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    const float inv = 1.0f / lsum;
    if (qt * 16 + col < N) {
      uint16_t* orow = a.o + (static_cast<size_t>(b) * N + n) * (a.H * dh) + static_cast<size_t>(h) * dh;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const int d0 = 16 * dt + 4 * grp;
        if (d0 < dh) {
          u16x4 ob;
#pragma unroll
          for (int r = 0; r < 4; ++r) ob[r] = f32_to_bf16_bits(oacc[dt][r] * inv);
          *reinterpret_cast<u16x4*>(orow + d0) = ob;
        }
      }
    }
  };

  const bool has_tile = wave * 16 < N;
  if (has_tile) first_pass(wave);
#pragma unroll
  for (int q = 0; q < 4; ++q) store_piece(tid + 256 * q, vraw[q]);
  for (int i = tid + 1024; i < n_piece; i += 256) store_piece(i, value_piece(i));
  __syncthreads();
  for (int qt = wave; qt * 16 < N; qt += 4) {
    if (qt != wave) first_pass(qt);
    second_pass(qt);
  }
}

// Long blocks (more than 32 token rows), LW = 2: workgroups of the projection and over how
// many of them the reduction dimension is split.  Few workgroups (the output projection of
// a 2048-wide layer has 32 per 128 token rows) leave most compute units without a stream.
struct LdsLinearPlan { int blocks, rows, passes, ksplit; };
static LdsLinearPlan lds_linear_plan(int T, const int* fout, int n_mats, int Din) {
  constexpr int LW = 2;
  LdsLinearPlan p{0, 128, 1, 1};
  for (int m = 0; m < n_mats; ++m) p.blocks += (fout[m] / 32 + LW - 1) / LW;
  // few workgroups: passes of 64 token rows (chunks of 128 reduction elements, half the
  // steps of a pass of 128 rows, and twice the workgroups)
  if (p.blocks * ((T + 127) / 128) < 100) p.rows = 64;
  p.passes = (T + p.rows - 1) / p.rows;
  // still few: the reduction dimension over two workgroups as well.  Measured on the
  // output projection of the 2048-wide layer at 256 token rows: 41.3 us as one pass of 128
  // rows per workgroup, 30.4 us with passes of 64, 25.8 us with the split on top (four-way:
  // no better); the q/k/v launch, 160 workgroups, is best left alone (21.7 us; split 38.7 us,
  // passes of 64 29.2 us).
  if (p.blocks * p.passes < 150 && Din % 512 == 0) p.ksplit = 2;
  return p;
}
constexpr size_t kLdsPartialBytes = 2 * 2 * 8 * 256 * 4;  // of one workgroup: LW x 2 tiles x 8 token tiles x 1 KB

// Scratch of one attention sub-layer (bytes from a 256-byte aligned base): q, k, v and the
// per-head outputs of the block's tokens, bf16.
AttnLayout attn_layout(const des_shape_t& s, const des_attn_shape_t& t) {
  const size_t T = static_cast<size_t>(s.n_seqs) * s.n_tokens;
  AttnLayout l;
  size_t p = 0;
  l.q = p; p = align256(p + 2 * T * t.n_heads * t.head_dim);
  l.k = p; p = align256(p + 2 * T * t.n_kv_heads * t.head_dim);
  l.v = p; p = align256(p + 2 * T * t.n_kv_heads * t.head_dim);
  l.o = p; p = align256(p + 2 * T * t.n_heads * t.head_dim);
  // short blocks, reduction split over two workgroups: fp32 partial tiles (two halves x two
  // token tiles x 1 KB per 16-row weight tile) and one flag per 16 rows, for the larger of
  // the two projection launches (they run one after the other)
  const size_t tiles_qkv = static_cast<size_t>(t.n_heads + 2 * t.n_kv_heads) * t.head_dim / 16;
  const size_t tiles_out = static_cast<size_t>(s.hidden) / 16;
  const size_t tiles = tiles_qkv > tiles_out ? tiles_qkv : tiles_out;
  size_t part_bytes = tiles * 4096, n_flags = tiles;
  if (T > 32) {  // long blocks: one 32 KB partial per workgroup, one counter per output tile
    const int f_qkv[3] = {t.n_heads * t.head_dim, t.n_kv_heads * t.head_dim, t.n_kv_heads * t.head_dim};
    const int f_out[1] = {s.hidden};
    const LdsLinearPlan a = lds_linear_plan(static_cast<int>(T), f_qkv, 3, s.hidden);
    const LdsLinearPlan b = lds_linear_plan(static_cast<int>(T), f_out, 1, t.n_heads * t.head_dim);
    const size_t wa = static_cast<size_t>(a.blocks) * a.passes, wb = static_cast<size_t>(b.blocks) * b.passes;
    const size_t pa = a.ksplit > 1 ? wa * a.ksplit * kLdsPartialBytes : 0;
    const size_t pb = b.ksplit > 1 ? wb * b.ksplit * kLdsPartialBytes : 0;
    part_bytes = pa > pb ? pa : pb;
    n_flags = wa > wb ? wa : wb;
  }
  l.partial = p; p = align256(p + part_bytes);
  l.flags = p; p = align256(p + n_flags * 8);
  l.total = p;
  return l;
}

size_t attn_core_lds(const des_shape_t& s, const des_attn_shape_t& t) {
  // the head's values, transposed: (dh rounded up to 16) rows of (window rounded up to 32) + 4 bf16
  const size_t nk = static_cast<size_t>(attn_cached(t)) + s.n_tokens;
  const size_t nkp = (nk + 31) / 32 * 32;
  return static_cast<size_t>((t.head_dim + 15) / 16 * 16) * (nkp + 4) * 2;
}

template <int LW>
static void launch_linear(const LinearArgs& a, int kernel_id, hipStream_t st) {
  if (a.T <= 32) {
    // Row tiles per workgroup: two halve the token-row traffic from L2, which costs as much
    // as the weight stream here (measured on the 2048-wide layer: q/k/v 13.6 us against
    // 17.2 us with one), but only while the workgroups still cover most compute units
    // (output projection, 128 tiles: 16 us with one tile per workgroup, 21 us with two).
    // Fewer than 150 workgroups: the reduction dimension is split over two workgroups as
    // well (output projection 15.9 -> 13.3 us; with 160 workgroups, q/k/v, the exchange of
    // partial tiles costs more than the better spread gains: 18.4 against 14.1 us).
    // Wavefronts per workgroup (k-slices): a whole number of 32-element steps each, at
    // least 256 reduction elements per row, at most 8.
    int tiles = 0;
    for (int m = 0; m < a.n_mats; ++m) tiles += a.fout[m] / 16;
    const bool two = tiles >= 2 * 150;
    int groups = 0;
    for (int m = 0; m < a.n_mats; ++m) groups += two ? (a.fout[m] / 16 + 1) / 2 : a.fout[m] / 16;
    LinearArgs b = a;
    b.ksplit = (groups < 150 && a.Din % 64 == 0 && a.Din >= 1024 && b.partial != nullptr) ? 2 : 1;
    const int kwg = a.Din / b.ksplit;
    int nw = 8;
    while (nw > 1 && (kwg % (32 * nw) != 0 || kwg / nw < 256)) nw >>= 1;
    const dim3 g(groups * b.ksplit), blk(nw * kWave);
    if (two) {
      if (a.T <= 16) launch(kernel_id, linear_splitk_kernel<2, 1>, g, blk, 0, st, b);
      else launch(kernel_id, linear_splitk_kernel<2, 2>, g, blk, 0, st, b);
    } else {
      if (a.T <= 16) launch(kernel_id, linear_splitk_kernel<1, 1>, g, blk, 0, st, b);
      else launch(kernel_id, linear_splitk_kernel<1, 2>, g, blk, 0, st, b);
    }
    return;
  }
  static_assert(LW == 2, "lds_linear_plan and the partial tiles assume two wavefronts");
  const LdsLinearPlan pl = lds_linear_plan(a.T, a.fout, a.n_mats, a.Din);
  LinearArgs c = a;
  c.ksplit = c.partial != nullptr ? pl.ksplit : 1;
  const dim3 g(pl.blocks, pl.passes, c.ksplit), b(LW * kWave);
  const int kd = a.Din / c.ksplit;
#define DES_LAUNCH_LIN(KDV)                                                                   \
  do {                                                                                        \
    if (pl.rows == 64) launch(kernel_id, linear_lds_kernel<LW, KDV, 64>, g, b, 0, st, c);     \
    else launch(kernel_id, linear_lds_kernel<LW, KDV, 128>, g, b, 0, st, c);                  \
  } while (0)
  if (kd == 2048) DES_LAUNCH_LIN(2048);
  else if (kd == 4096) DES_LAUNCH_LIN(4096);
  else DES_LAUNCH_LIN(0);
#undef DES_LAUNCH_LIN
}

int launch_attention(const des_shape_t& s, const des_attn_shape_t& t, const void* x, const void* wq,
                     const void* wk, const void* wv, const void* wo, const void* k_cache,
                     const void* v_cache, void* y, char* ws, unsigned long long epoch, hipStream_t st) {
  const AttnLayout l = attn_layout(s, t);
  const int T = s.n_seqs * s.n_tokens;
  const int HD = t.n_heads * t.head_dim, KD_ = t.n_kv_heads * t.head_dim;
  LinearArgs p{};
  p.in = static_cast<const uint16_t*>(x);
  p.w[0] = static_cast<const uint16_t*>(wq);
  p.w[1] = static_cast<const uint16_t*>(wk);
  p.w[2] = static_cast<const uint16_t*>(wv);
  p.out[0] = reinterpret_cast<uint16_t*>(ws + l.q);
  p.out[1] = reinterpret_cast<uint16_t*>(ws + l.k);
  p.out[2] = reinterpret_cast<uint16_t*>(ws + l.v);
  p.fout[0] = HD; p.fout[1] = KD_; p.fout[2] = KD_;
  p.n_mats = 3; p.T = T; p.Din = s.hidden; p.res = nullptr;
  p.ksplit = 1;
  p.partial = reinterpret_cast<float*>(ws + l.partial);
  p.flags = reinterpret_cast<unsigned long long*>(ws + l.flags);
  p.epoch = epoch;
  launch_linear<2>(p, kKAttnProj, st);

  AttnArgs c{};
  c.q = p.out[0]; c.k = p.out[1]; c.v = p.out[2];
  c.k_cache = static_cast<const uint16_t*>(k_cache);
  c.v_cache = static_cast<const uint16_t*>(v_cache);
  c.o = reinterpret_cast<uint16_t*>(ws + l.o);
  c.B = s.n_seqs; c.N = s.n_tokens; c.H = t.n_heads; c.Hkv = t.n_kv_heads; c.dh = t.head_dim;
  c.P = attn_cached(t);
  c.scale = 1.0f / sqrtf(static_cast<float>(t.head_dim));
  const size_t lds = attn_core_lds(s, t);
  if (lds > 48 * 1024) {  // (a property of the function on the current device; cheap to repeat)
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_core_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return hip_fail(e, "attention LDS size");
  }
  launch(kKAttnCore, attention_core_kernel, dim3(s.n_seqs * t.n_heads), dim3(256), lds, st, c);

  LinearArgs o{};
  o.in = c.o;
  o.w[0] = static_cast<const uint16_t*>(wo);
  o.out[0] = static_cast<uint16_t*>(y);
  o.fout[0] = s.hidden;
  o.n_mats = 1; o.T = T; o.Din = HD;
  o.ksplit = 1;
  o.partial = p.partial;
  o.flags = p.flags;
  o.epoch = epoch;
  o.res = s.residual ? static_cast<const uint16_t*>(x) : nullptr;
  launch_linear<2>(o, kKAttnOut, st);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "attention launch");
}

}  // namespace des
