// Grouped SwiGLU expert FFN and weighted combine (Alg. 1 stage 2, last line:
// y_n = sum_{i in S_n} g_{n,i} E_i(x_n)), for gfx950.
//
// The layer is bound by the one-time read of the live experts' weights
// (Eq. 2: the b * |union S_n| term), so the kernels are organised around the
// weight stream, not around the tokens:
//   * a wavefront owns 16 weight rows (gate and up rows of the same
//     intermediate units, or 4 x 16 down rows) and walks the whole reduction
//     dimension, loading each weight fragment straight into the matrix-core A
//     operand with 16-byte loads - every weight byte is read by exactly one
//     wavefront, exactly once;
//   * the expert's tokens are the matrix-core B operand (16 tokens per tile,
//     up to 16 tiles held in accumulators), so a partly empty token tile
//     wastes matrix-core cycles, which are free here, and no bandwidth;
//   * the grid is sized for the worst case and every wavefront looks its
//     expert up in the device-resident live list, so the host never waits for
//     the routing result.
// Nothing is accumulated with floating-point atomics: gate/up writes the
// SwiGLU activations H, down writes one fp32 row per (token, expert) pair, and
// the combine adds a token's K rows in slot order.
#include <type_traits>

#include "des_common.h"
#include "des_select.h"
#include "des_stream_gemm.h"

namespace des {


struct FfnArgs {
  const void* x;
  const void *wg, *wu, *wd;     // routed experts
  const void *sg, *su, *sd;     // shared expert (or null)
  const int32_t* topk_idx;      // [T][K]
  const float* topk_w;          // [T][K]
  const int4* slots;            // [n_slots] {expert, first sorted pair, pairs, 0}
  const int32_t *meta, *pair_tok, *pos;
  const uint16_t* slot_tok;     // [n_slots][kSlotToks] tokens of each slot's first pairs
  void* h;                      // [(TK) x F] then [T x Fs]
  float* o;                     // [(TK + T) x D]
  void* y;                      // [T][D]
  int T, D, M, F, Fs, K, n_slots, residual;
  int splits;                   // units the shared expert's rows are spread over (LDS kernels)
  const int32_t* units;         // live units of the routed experts, longest expert first:
                                // slot | split << 16 | splits of that slot << 24; meta[2] of them
  size_t h_rows;                // routed rows of H (the shared expert's rows follow them)
  DenseArgs dn;                 // dense short block: stage 2 beside gate/up, see des_common.h
};

#ifdef DES_FFN_STAMPS  // development aid (build with DES_FFN_STAMPS=1): per-task 100 MHz
                       // timestamps of the gate/up kernels, [start, task found, end, hardware id
                       // or pairs], read back with des_debug_ffn_stamps()
__device__ long long g_ffn_stamps[8192 * 4];
#define DES_FSTAMP(task, i) do { if ((threadIdx.x & 63) == 0 && (task) < 8192) g_ffn_stamps[(task) * 4 + (i)] = wall_clock64(); } while (0)
#else
#define DES_FSTAMP(task, i) do { } while (0)
#endif

// Work item of one wavefront: which expert's rows, which pairs.
struct Task {
  const uint16_t *w0, *w1;  // weight matrices of the expert (gate, up) or (down, -)
  int slot;                 // slot of the expert (-1 for the shared expert)
  int pre_tok[2];           // this lane's token in the slot's first two token tiles
  int count;                // pairs of this expert
  int pair0;                // first sorted position (routed) or 0 (shared)
  bool shared;
  uint32_t dmask;           // dense short block, down projection: the slot's routed tokens
  size_t row_base;          // first H / O row of these pairs
  int fdim;                 // F of this expert (F or Fs)
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + expf(-z)); }

// ------------------------------------------------------------------ bf16 path
// MFMA 16x16x32 bf16: lane l supplies row (l%16), reduction elements
// 8*(l/16)..+7 of both operands; the accumulator of lane l holds token column
// (l%16) and weight rows 4*(l/16)..+3.
//
// Weight fragment address for (row tile rt, k-step ks):
//   row-major [rows][kd]:  base + (rt*16 + l%16)*kd + ks*32 + 8*(l/16)
//   packed tiles          :  base + ((rt*(kd/32) + ks)*64 + l)*8
template <bool PACKED>
__device__ __forceinline__ const uint16_t* frag_ptr(const uint16_t* base, int rt, int kd, int lane) {
  if (PACKED) return base + (static_cast<size_t>(rt) * (kd / 32) * 64 + lane) * 8;
  return base + (static_cast<size_t>(rt) * 16 + (lane & 15)) * kd + (lane >> 4) * 8;
}

__device__ __forceinline__ bf16x8 ld8(const uint16_t* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}
// Weights are read once and never again: a non-temporal load keeps them from
// displacing the activations in L2 / the last-level cache.
__device__ __forceinline__ bf16x8 ld8_stream(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p));
}
__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = static_cast<__bf16>(0.0f);
  return z;
}

// gate/up for pairs [g0, g0 + 16*NT) of the task, intermediate rows
// (ft0 .. ft0+FT-1)*16..+15.  The FT row tiles share every token fragment.
template <int FT, int NT, int U, bool PACKED>
__device__ __forceinline__ void gateup_group(const FfnArgs& a, const Task& t, int ft0, int g0,
                                             int lane) {
  const int D = a.D;
  const int nks = D / 32;
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  const uint16_t* gp[FT];
  const uint16_t* up[FT];
#pragma unroll
  for (int f = 0; f < FT; ++f) {
    gp[f] = frag_ptr<PACKED>(t.w0, ft0 + f, D, lane);
    up[f] = frag_ptr<PACKED>(t.w1, ft0 + f, D, lane);
  }
  const uint16_t* xp[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    int pi = min(g0 + i * 16 + (lane & 15), t.count - 1);  // clamped rows are dropped at the store
    // the first two token tiles come from the slot-major table, fetched together
    // with the slot record (entries past the slot's count name token 0)
    const int tok = t.shared ? pi
                    : ((g0 == 0 && i < 2) ? t.pre_tok[i < 2 ? i : 0] : a.pair_tok[t.pair0 + pi]);
    xp[i] = x + static_cast<size_t>(tok) * D + (lane >> 4) * 8;
  }
  f32x4 accg[FT][NT], accu[FT][NT];
#pragma unroll
  for (int f = 0; f < FT; ++f)
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      accg[f][i] = f32x4{0.f, 0.f, 0.f, 0.f};
      accu[f][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  bf16x8 ag[2][U][FT], au[2][U][FT], bx[2][U][NT];

  auto load = [&](int ks, auto stage) {
    constexpr int s = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ks + u < nks) {
#pragma unroll
        for (int f = 0; f < FT; ++f) {
          ag[s][u][f] = ld8_stream(gp[f] + static_cast<size_t>(ks + u) * frag_step<PACKED>());
          au[s][u][f] = ld8_stream(up[f] + static_cast<size_t>(ks + u) * frag_step<PACKED>());
        }
#pragma unroll
        for (int i = 0; i < NT; ++i) bx[s][u][i] = ld8(xp[i] + (ks + u) * 32);
      } else {
#pragma unroll
        for (int f = 0; f < FT; ++f) {
          ag[s][u][f] = zero8();
          au[s][u][f] = zero8();
        }
#pragma unroll
        for (int i = 0; i < NT; ++i) bx[s][u][i] = zero8();
      }
    }
  };
  auto compute = [&](auto stage) {
    constexpr int s = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int f = 0; f < FT; ++f)
#pragma unroll
        for (int i = 0; i < NT; ++i) {
          accg[f][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag[s][u][f], bx[s][u][i], accg[f][i], 0, 0, 0);
          accu[f][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(au[s][u][f], bx[s][u][i], accu[f][i], 0, 0, 0);
        }
  };
  load(0, S0{});
  for (int ks = 0; ks < nks; ks += 2 * U) {
    load(ks + U, S1{});
    compute(S0{});
    load(ks + 2 * U, S0{});
    compute(S1{});
  }
  uint16_t* h = static_cast<uint16_t*>(a.h);
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int pi = g0 + i * 16 + (lane & 15);
    if (pi < t.count) {
#pragma unroll
      for (int f = 0; f < FT; ++f) {
        u16x4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = f32_to_bf16_bits(silu_f(accg[f][i][q]) * accu[f][i][q]);
        uint16_t* dst = h + (t.row_base + pi) * t.fdim + (ft0 + f) * 16 + 4 * (lane >> 4);
        *reinterpret_cast<u16x4*>(dst) = v;
      }
    }
  }
}

__device__ __forceinline__ bool make_task(const FfnArgs& a, int slot_or_shared, bool shared,
                                          bool down, Task& t, int lane) {
  const size_t TK = static_cast<size_t>(a.T) * a.K;
  t.dmask = 0u;  // (every path: the down projection tests it)
  if (!shared) {
    // the slot record and (for gate/up) this lane's tokens are fetched together:
    // both addresses depend on the slot number only
    const int4 sl = a.slots[slot_or_shared];
    if (!down && a.T > 32) {
      const uint16_t* st = a.slot_tok + slot_or_shared * kSlotToks + (lane & 15);
      t.pre_tok[0] = st[0];
      t.pre_tok[1] = st[16];
    }
    // an unused slot; also refuses a record that does not fit the problem (the
    // workspace is the caller's memory: never index weights or pairs with it blindly)
    if (sl.x < 0 || sl.x >= a.M || sl.y < 0 || sl.z < 1 ||
        static_cast<long long>(sl.y) + sl.z > static_cast<long long>(a.h_rows))
      return false;
    const int e = sl.x;
    const int off = sl.y;
    if (a.dn.on) {
      // every token of the block, in order: H row = first row of the slot + token
      t.pre_tok[0] = min(lane & 15, a.T - 1);
      t.pre_tok[1] = min(16 + (lane & 15), a.T - 1);
      if (down) {
        // the expert's pairs are the set bits of its bitmap, in order (positions past
        // the count repeat the last one; their results are dropped)
        t.dmask = a.dn.tokmask[slot_or_shared] & (a.T >= 32 ? 0xffffffffu : ((1u << a.T) - 1u));
        if (t.dmask == 0u) return false;  // nobody was routed to this expert
        const int cnt = __popc(t.dmask);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int want = min(i * 16 + (lane & 15), cnt - 1);
          uint32_t mm = t.dmask;
          for (int k = 0; k < want; ++k) mm &= mm - 1u;
          t.pre_tok[i] = __builtin_ctz(mm);
        }
      }
    } else if (!down && a.T <= 32) {
      // at most 32 tokens: the record carries the bitmap of the expert's tokens; its pairs
      // in order are the set bits in order (positions past the count repeat the last one)
      const uint32_t m = static_cast<uint32_t>(sl.w);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int want = min(i * 16 + (lane & 15), sl.z - 1);
        uint32_t mm = m;
        for (int k = 0; k < want; ++k) mm &= mm - 1u;
        t.pre_tok[i] = mm ? min(__builtin_ctz(mm), a.T - 1) : 0;
      }
    }
    t.slot = slot_or_shared;
    // (dense, down: only the routed tokens count, so a slot with at most 16 of them takes
    // the one-tile path)
    t.count = t.dmask ? __popc(t.dmask) : sl.z;
    t.pair0 = off;
    t.shared = false;
    t.row_base = static_cast<size_t>(off);
    t.fdim = a.F;
    const size_t mat = static_cast<size_t>(a.F) * a.D;
    if (down) {
      t.w0 = static_cast<const uint16_t*>(a.wd) + e * mat;
      t.w1 = nullptr;
    } else {
      t.w0 = static_cast<const uint16_t*>(a.wg) + e * mat;
      t.w1 = static_cast<const uint16_t*>(a.wu) + e * mat;
    }
  } else {
    t.slot = -1;
    t.count = a.T;
    t.pair0 = 0;
    t.shared = true;
    t.row_base = TK;  // H: row index in units of its own stride, see h_base below
    t.fdim = a.Fs;
    t.w0 = static_cast<const uint16_t*>(down ? a.sd : a.sg);
    t.w1 = static_cast<const uint16_t*>(down ? nullptr : a.su);
  }
  return true;
}

// H rows of the shared expert start after the TK routed rows of width F; they
// have width Fs.  Express that start as a row offset in Fs-wide rows by
// shifting the base pointer instead (keeps one indexing formula).
__device__ __forceinline__ FfnArgs shared_view(const FfnArgs& a, Task& t, size_t elem_size) {
  FfnArgs v = a;
  v.h = static_cast<char*>(a.h) + a.h_rows * a.F * elem_size;
  t.row_base = 0;
  return v;
}

#ifndef DES_FFN_WAVES
#define DES_FFN_WAVES 1
#endif
constexpr int kFfnWaves = DES_FFN_WAVES;  // wavefronts per workgroup; each is an independent task
constexpr int kGuTiles = 2;   // gate/up row tiles per task (F % 32 == 0, so F/16 is even)

// MAXNT bounds the token tiles a task can have (the host knows T >= any expert's
// count), so that small blocks get a kernel with few registers.  U1 / U2 are
// the k-steps per prefetch stage of the one- and two-token-tile paths; two
// stages of two k-steps measured best on the 128-expert layer (34.3 us against
// 36.2 us for four and 34.5 us for one).
// One gate/up task (see the kernel comment): returns false if the slot is unused.
template <int MAXNT, bool PACKED, int U1 = 2, int U2 = 2, int GT = kGuTiles>
__device__ __forceinline__ bool gateup_task(const FfnArgs& a, int task, int lane) {
  const int tiles_r = a.F / (16 * GT);
  const int routed = a.n_slots * tiles_r;
  Task t;
  int ft;
  FfnArgs v = a;
  DES_FSTAMP(task, 0);
  if (task < routed) {
    if (!make_task(a, task / tiles_r, false, false, t, lane)) return false;
    DES_FSTAMP(task, 1);
    ft = (task % tiles_r) * GT;
  } else {
    make_task(a, 0, true, false, t, lane);
    v = shared_view(a, t, 2);
    ft = (task - routed) * GT;
  }
  const int nt = (t.count + 15) / 16;
  bool done = false;
  if (MAXNT == 1 || nt <= 1) {
    gateup_group<GT, 1, U1, PACKED>(v, t, ft, 0, lane);
    done = true;
  }
  if constexpr (MAXNT >= 2) {
    if (!done && (MAXNT == 2 || nt <= 2)) {
      gateup_group<GT, 2, U2, PACKED>(v, t, ft, 0, lane);
      done = true;
    }
  }
  if constexpr (MAXNT >= 4) {
    if (!done && (MAXNT == 4 || nt <= 4)) {
      gateup_group<GT, 4, 2, PACKED>(v, t, ft, 0, lane);
      done = true;
    }
  }
  if constexpr (MAXNT >= 8) {
    if (!done && (MAXNT == 8 || nt <= 8)) {
      gateup_group<GT, 8, 1, PACKED>(v, t, ft, 0, lane);
      done = true;
    }
  }
  if constexpr (MAXNT >= 16) {
    if (!done)
      for (int g0 = 0; g0 < t.count; g0 += 256)
        for (int f = 0; f < GT; ++f) gateup_group<1, 16, 1, PACKED>(v, t, ft + f, g0, lane);
  }
  DES_FSTAMP(task, 2);
#ifdef DES_FFN_STAMPS
  if ((threadIdx.x & 63) == 0 && task < 8192)
    g_ffn_stamps[task * 4 + 3] = (static_cast<long long>(__builtin_amdgcn_s_getreg(20 | (31 << 11))) << 32) |
                                 static_cast<unsigned>(__builtin_amdgcn_s_getreg(4 | (31 << 11)));
#endif
  return true;
}

// MAXNT bounds the token tiles a task can have (the host knows T >= any expert's
// count), so that small blocks get a kernel with few registers.  U1 / U2 are
// the k-steps per prefetch stage of the one- and two-token-tile paths; two
// stages of two k-steps measured best on the 128-expert layer (34.3 us against
// 36.2 us for four and 34.5 us for one).
// GT = row tiles per task: 2 normally, 1 when the launch would otherwise have
// too few wavefronts to keep enough bytes in flight (small coresets).
template <int MAXNT, bool PACKED, int U1 = 2, int U2 = 2, int GT = kGuTiles>
__global__ __launch_bounds__(kFfnWaves* kWave) void gateup_bf16_kernel(FfnArgs a) {
  const int lane = threadIdx.x & 63;
  int task = blockIdx.x * kFfnWaves + (threadIdx.x >> 6);
  if constexpr (MAXNT <= 2) {
    if (a.dn.on) {
      // dense short block: the first wavefronts of the grid re-route the block's tokens
      // (Alg. 1 stage 2) while the others stream the coreset's weights
      const int n_s2 = (a.T * a.dn.lpt + 63) / 64;
      if (task < n_s2) {
        __shared__ uint32_t s_sorted[kFfnWaves * kEpl * 64];
        uint32_t* srt = s_sorted + (threadIdx.x >> 6) * (kEpl * 64);
        const int n_core = a.meta[0];
        if (n_core <= 0) return;  // the routing launch gave up: nothing was elected
        switch (a.dn.lpt) {
          case 4: stage2_wave<4>(a.dn, a.T, a.M, a.K, n_core, task, srt); break;
          case 8: stage2_wave<8>(a.dn, a.T, a.M, a.K, n_core, task, srt); break;
          case 16: stage2_wave<16>(a.dn, a.T, a.M, a.K, n_core, task, srt); break;
          case 32: stage2_wave<32>(a.dn, a.T, a.M, a.K, n_core, task, srt); break;
          default: stage2_wave<64>(a.dn, a.T, a.M, a.K, n_core, task, srt); break;
        }
        return;
      }
      task -= n_s2;
    }
  }
  const int tasks = a.n_slots * (a.F / (16 * GT)) + a.Fs / (16 * GT);
  if (task < tasks) gateup_task<MAXNT, PACKED, U1, U2, GT>(a, task, lane);
}

// down for pairs [g0, g0+16*NT), output rows (dt0 .. dt0+RT-1)*16
template <int RT, int NT, int U, bool PACKED>
__device__ __forceinline__ void down_group(const FfnArgs& a, const Task& t, int dt0, int g0,
                                           int lane) {
  const int F = t.fdim;
  const int nks = F / 32;
  const uint16_t* h = static_cast<const uint16_t*>(a.h);
  const uint16_t* ap[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) ap[r] = frag_ptr<PACKED>(t.w0, dt0 + r, F, lane);
  const uint16_t* hp[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int pi = min(g0 + i * 16 + (lane & 15), t.count - 1);
    // (dense short block: H holds every token of the block for this slot; the routed
    // ones, in order, are this expert's pairs)
    const int hrow = t.dmask ? t.pre_tok[i < 2 ? i : 0] : pi;
    hp[i] = h + (t.row_base + hrow) * F + (lane >> 4) * 8;
  }
  f32x4 acc[RT][NT];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[r][i] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 aw[2][U][RT], bh[2][U][NT];
  auto load_w = [&](int ks, auto stage) {
    constexpr int s = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r)
        aw[s][u][r] = (ks + u < nks)
                          ? ld8_stream(ap[r] + static_cast<size_t>(ks + u) * frag_step<PACKED>())
                          : zero8();
    }
  };
  auto load_h = [&](int ks, auto stage) {
    constexpr int s = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < NT; ++i)
        bh[s][u][i] = (ks + u < nks) ? ld8(hp[i] + (ks + u) * 32)
                                     : zero8();
    }
  };
  auto load = [&](int ks, auto stage) {
    load_w(ks, stage);
    load_h(ks, stage);
  };
  auto compute = [&](auto stage) {
    constexpr int s = decltype(stage)::value;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int i = 0; i < NT; ++i)
          acc[r][i] =
              __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw[s][u][r], bh[s][u][i], acc[r][i], 0, 0, 0);
  };
  load(0, S0{});
  for (int ks = 0; ks < nks; ks += 2 * U) {
    load(ks + U, S1{});
    compute(S0{});
    load(ks + 2 * U, S0{});
    compute(S1{});
  }
  const size_t orow0 = t.shared ? static_cast<size_t>(a.T) * a.K : static_cast<size_t>(t.pair0);
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int pi = g0 + i * 16 + (lane & 15);
    if (pi < t.count) {
      size_t orow = orow0 + pi;
      if (t.dmask) {
        // dense short block: the pair's row is token * K + (which of the token's
        // choices this expert is)
        const int tok = t.pre_tok[i < 2 ? i : 0];
        orow = static_cast<size_t>(tok) * a.K + a.dn.choice[t.slot * 32 + tok];
      }
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        float* dst = a.o + orow * a.D + (dt0 + r) * 16 + 4 * (lane >> 4);
        *reinterpret_cast<f32x4*>(dst) = acc[r][i];
      }
    }
  }
}

// One down task: 64 output rows of one expert for all of its pairs.
template <int MAXNT, bool PACKED, int U1 = 2, int U2 = 2, int RTG = 4>
__device__ __forceinline__ bool down_task(const FfnArgs& a, int task, int lane) {
  const int dtiles = a.D / 16;
  const int groups = (dtiles + RTG - 1) / RTG;  // 16 * RTG output rows per task
  const int routed = a.n_slots * groups;
  Task t;
  int dg;
  FfnArgs v = a;
  if (task < routed) {
    const int slot = task / groups;
    if (!make_task(a, slot, false, true, t, lane)) return false;
    dg = task % groups;
  } else {
    make_task(a, 0, true, true, t, lane);
    v = shared_view(a, t, 2);
    dg = task - routed;
  }
  const int dt_begin = dg * RTG;
  const int dt_end = min(dt_begin + RTG, dtiles);
  const int nt = (t.count + 15) / 16;
  bool done = false;
  if (dt_end - dt_begin == RTG) {
    if (MAXNT == 1 || nt <= 1) {
      down_group<RTG, 1, U1, PACKED>(v, t, dt_begin, 0, lane);
      done = true;
    }
    if constexpr (MAXNT >= 2) {
      if (!done && (MAXNT == 2 || nt <= 2)) {
        down_group<RTG, 2, U2, PACKED>(v, t, dt_begin, 0, lane);
        done = true;
      }
    }
    if constexpr (MAXNT >= 4) {
      if (!done && (MAXNT == 4 || nt <= 4)) {
        down_group<RTG, 4, 1, PACKED>(v, t, dt_begin, 0, lane);
        done = true;
      }
    }
    if constexpr (MAXNT >= 8) {
      if (!done && (MAXNT == 8 || nt <= 8)) {
        for (int r2 = 0; r2 < RTG; r2 += 2)
          down_group<2, 8, 1, PACKED>(v, t, dt_begin + r2, 0, lane);
        done = true;
      }
    }
  }
  if (!done) {  // ragged row group, or more than 128 pairs: one row tile at a time
    for (int dt = dt_begin; dt < dt_end; ++dt) {
      if constexpr (MAXNT <= 4) {
        down_group<1, MAXNT, 2, PACKED>(v, t, dt, 0, lane);
      } else {
        for (int g0 = 0; g0 < t.count; g0 += 16 * MAXNT)
          down_group<1, MAXNT, 1, PACKED>(v, t, dt, g0, lane);
      }
    }
  }
  return true;
}

template <int MAXNT, bool PACKED, int U1 = 2, int U2 = 2, int RTG = 4>
__global__ __launch_bounds__(kFfnWaves* kWave) void down_bf16_kernel(FfnArgs a) {
  const int lane = threadIdx.x & 63;
  const int task = blockIdx.x * kFfnWaves + (threadIdx.x >> 6);
  const int groups = (a.D / 16 + RTG - 1) / RTG;
  const int tasks = a.n_slots * groups + (a.Fs > 0 ? groups : 0);
  if (task < tasks) down_task<MAXNT, PACKED, U1, U2, RTG>(a, task, lane);
}

// ------------------------------------------ larger blocks: activations via LDS
// (the streaming building block dma_stream_gemm lives in des_stream_gemm.h)
// Which expert, which of its row groups and which pairs a workgroup works on,
// shared by the two kernels.  The grid is one-dimensional and read in hand-out
// order: the shared expert first (every token: the longest workgroups), then
// the live units of the routed experts as the permutation lists them - longest
// expert first, an expert's units next to each other (they read the same
// weights).  So when the workgroups do not all fit on the chip at once the long
// ones start first, consecutive workgroups (which the hardware deals out to the
// XCDs in turn) carry similar work, and the grid's tail beyond the live units
// exits on one scalar load.  `split` of `nsplit`: this workgroup takes every
// nsplit-th group of rows of the expert, starting with group `split`.
template <bool DOWN>
__device__ __forceinline__ bool lds_task(const FfnArgs& a, int per_expert, int per_shared, int& group,
                                         int& split, int& nsplit, Task& t, FfnArgs& v, int lane) {
  int bx = blockIdx.x;
  v = a;
  if (bx < per_shared * a.splits) {
    make_task(a, 0, true, DOWN, t, lane);
    v = shared_view(a, t, 2);
    split = bx / per_shared;
    nsplit = a.splits;
    group = bx % per_shared;
    return true;
  }
  bx -= per_shared * a.splits;
  const int u = bx / per_expert;
  if (u >= a.meta[2]) return false;
  const int rec = a.units[u];
  if ((rec & 0xffff) >= a.n_slots || (rec >> 24) < 1 || (rec >> 24) > kMaxSplits) return false;
  split = (rec >> 16) & 0xff;
  nsplit = rec >> 24;
  group = bx % per_expert;
  return make_task(a, rec & 0xffff, false, DOWN, t, lane);
}

// MAXNT = token tiles per workgroup pass (the LDS buffer holds 16*MAXNT rows);
// LW = wavefronts per workgroup; KD = the reduction length when the host knows
// it to be one of the unrolled cases, else 0.  A split takes every splits-th group of
// 16*MAXNT pairs of the expert: an expert with more pairs than one pass holds
// is spread over several workgroups (its weights are then read once per pass).
template <bool PACKED, int MAXNT, int LW, int KD>
__global__ __launch_bounds__(LW* kWave, ((KD > 0 || MAXNT <= 4) ? 2 : 1)) void gateup_lds_kernel(FfnArgs a) {
  constexpr int kRows = 16 * MAXNT;
  __shared__ __align__(16) uint16_t lds[lds_elems(KD)];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  Task t;
  FfnArgs v;
  int group, split, splits;
  const int per_r = (a.F / 16 + LW - 1) / LW;
  const int per_s = (a.Fs / 16 + LW - 1) / LW;
  DES_FSTAMP(blockIdx.x, 0);
  if (!lds_task<false>(a, per_r, per_s, group, split, splits, t, v, lane)) return;  // uniform per workgroup
  const int tile = group * LW + wave;
  const bool active = tile < t.fdim / 16;
  const uint16_t* w0 = uniform_ptr(t.w0);
  const uint16_t* gp = tile_base<PACKED>(w0, active ? tile : 0, a.D);
  const uint16_t* up = tile_base<PACKED>(uniform_ptr(t.w1), active ? tile : 0, a.D);
  const uint32_t wlo = tile_lane_off<PACKED>(a.D, lane);
  const uint16_t* x = uniform_ptr(static_cast<const uint16_t*>(a.x));
  uint16_t* h = static_cast<uint16_t*>(v.h);
  for (int g0 = split * kRows; g0 < t.count; g0 += splits * kRows) {
    const int rows = min(kRows, t.count - g0);
    const int nt = (rows + 15) / 16;
    auto row_off = [&](int r) {
      const int tok = t.shared ? g0 + r : a.pair_tok[t.pair0 + g0 + r];
      return tok * a.D;
    };
    auto run = [&](auto ntc) {
      constexpr int NT = decltype(ntc)::value;
      f32x4 accg[NT], accu[NT];
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        accg[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        accu[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      constexpr int KC = NT <= 4 ? 128 : 64;  // rows * KC = one 16 KB buffer
      dma_stream_gemm<NT, kLdsBufElems / KC, PACKED, LW, KC, KD>(gp, up, wlo, wave, a.D, rows, x,
                                                                 row_off, lds, accg, accu);
      if (!active) return;
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const int pi = g0 + i * 16 + (lane & 15);
        if (pi < t.count) {
          u16x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = f32_to_bf16_bits(silu_f(accg[i][q]) * accu[i][q]);
          *reinterpret_cast<u16x4*>(h + (t.row_base + pi) * t.fdim + tile * 16 + 4 * (lane >> 4)) = o;
        }
      }
    };
    if (nt <= 1) run(std::integral_constant<int, 1>{});
    else if (nt <= 2) run(std::integral_constant<int, 2>{});
    else if (MAXNT <= 4 || nt <= 4) run(std::integral_constant<int, 4>{});
    else if (nt <= 6) run(std::integral_constant<int, MAXNT >= 8 ? 6 : 4>{});
    else run(std::integral_constant<int, MAXNT >= 8 ? 8 : 4>{});
  }
#ifdef DES_FFN_STAMPS
  DES_FSTAMP(blockIdx.x, 2);
  if (threadIdx.x == 0 && blockIdx.x < 8192) {  // pairs this workgroup worked on, where it ran
    g_ffn_stamps[blockIdx.x * 4 + 3] = max(0, min(static_cast<int>(t.count) - split * kRows, kRows));
    g_ffn_stamps[blockIdx.x * 4 + 1] =
        (static_cast<long long>(__builtin_amdgcn_s_getreg(20 | (31 << 11))) << 32) |
        static_cast<unsigned>(__builtin_amdgcn_s_getreg(4 | (31 << 11)));
  }
#endif
}

template <bool PACKED, int MAXNT, int LW, int KD>
__global__ __launch_bounds__(LW* kWave, ((KD > 0 || MAXNT <= 4) ? 2 : 1)) void down_lds_kernel(FfnArgs a) {
  constexpr int kRows = 16 * MAXNT;
  __shared__ __align__(16) uint16_t lds[lds_elems(KD)];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  Task t;
  FfnArgs v;
  int group, split, splits;
  const int dtiles = a.D / 16;                       // even: D is a multiple of 32
  const int per = (dtiles / 2 + LW - 1) / LW;        // a wavefront owns two row tiles
  if (!lds_task<true>(a, per, a.Fs > 0 ? per : 0, group, split, splits, t, v, lane)) return;
  const int dt0 = (group * LW + wave) * 2;
  const bool active = dt0 < dtiles;
  const int F = t.fdim;
  const uint16_t* w0 = uniform_ptr(t.w0);
  const uint16_t* p0 = tile_base<PACKED>(w0, active ? dt0 : 0, F);
  const uint16_t* p1 = tile_base<PACKED>(w0, active ? dt0 + 1 : 0, F);
  const uint32_t wlo = tile_lane_off<PACKED>(F, lane);
  const uint16_t* h = uniform_ptr(static_cast<const uint16_t*>(v.h));
  const size_t orow0 = t.shared ? static_cast<size_t>(a.T) * a.K : static_cast<size_t>(t.pair0);
  for (int g0 = split * kRows; g0 < t.count; g0 += splits * kRows) {
    const int rows = min(kRows, t.count - g0);
    const int nt = (rows + 15) / 16;
    const int hrow0 = static_cast<int>(t.row_base) + g0;
    auto row_off = [&](int r) { return (hrow0 + r) * F; };
    auto run = [&](auto ntc) {
      constexpr int NT = decltype(ntc)::value;
      f32x4 acc0[NT], acc1[NT];
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        acc0[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      constexpr int KC = NT <= 4 ? 128 : 64;
      dma_stream_gemm<NT, kLdsBufElems / KC, PACKED, LW, KC, KD>(p0, p1, wlo, wave, F, rows, h,
                                                                 row_off, lds, acc0, acc1);
      if (!active) return;
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const int pi = g0 + i * 16 + (lane & 15);
        if (pi < t.count) {
          float* dst = a.o + (orow0 + pi) * a.D + dt0 * 16 + 4 * (lane >> 4);
          *reinterpret_cast<f32x4*>(dst) = acc0[i];
          *reinterpret_cast<f32x4*>(dst + 16) = acc1[i];
        }
      }
    };
    if (nt <= 1) run(std::integral_constant<int, 1>{});
    else if (nt <= 2) run(std::integral_constant<int, 2>{});
    else if (MAXNT <= 4 || nt <= 4) run(std::integral_constant<int, 4>{});
    else if (nt <= 6) run(std::integral_constant<int, MAXNT >= 8 ? 6 : 4>{});
    else run(std::integral_constant<int, MAXNT >= 8 ? 8 : 4>{});
  }
}

// ------------------------------------------------------------------ fp32 path
// Plain fused-multiply-add kernels for the small fp32 configuration: one
// wavefront per output element row-chunk, lanes stride the reduction
// dimension with 16-byte loads, fixed-order wave reduction.
__device__ __forceinline__ float dot_f32(const float* a, const float* b, int n, int lane) {
  const float4* pa = reinterpret_cast<const float4*>(a);
  const float4* pb = reinterpret_cast<const float4*>(b);
  float s = 0.f;
  for (int v = lane; v < n / 4; v += 64) {
    const float4 p = pa[v], q = pb[v];
    s = fmaf(p.x, q.x, s);
    s = fmaf(p.y, q.y, s);
    s = fmaf(p.z, q.z, s);
    s = fmaf(p.w, q.w, s);
  }
  return wave_sum_f32(s);
}

// grid.x = sorted pair row r in [0, TK + Ts); grid.y tiles the F (or D) rows.
__device__ __forceinline__ bool f32_row(const FfnArgs& a, int r, int& e, int& tok, bool& shared) {
  const int TK = a.T * a.K;
  if (r < TK) {
    if (r >= a.meta[1]) return false;  // fewer routed pairs than slots (k_eff < K)
    tok = a.pair_tok[r];
    e = -1;
    for (int j = 0; j < a.K; ++j)  // the slot of this token that sits at sorted position r
      if (a.pos[tok * a.K + j] == r) e = a.topk_idx[tok * a.K + j];
    shared = false;
    return true;
  }
  e = 0;
  tok = r - TK;
  shared = true;
  return a.Fs > 0;
}

__global__ __launch_bounds__(256) void gateup_f32_kernel(FfnArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x;
  int e, tok;
  bool sh;
  if (!f32_row(a, r, e, tok, sh)) return;
  const int F = sh ? a.Fs : a.F;
  const size_t TK = static_cast<size_t>(a.T) * a.K;
  const float* xg = static_cast<const float*>(a.x) + static_cast<size_t>(tok) * a.D;
  const float* wg = sh ? static_cast<const float*>(a.sg)
                       : static_cast<const float*>(a.wg) + static_cast<size_t>(e) * a.F * a.D;
  const float* wu = sh ? static_cast<const float*>(a.su)
                       : static_cast<const float*>(a.wu) + static_cast<size_t>(e) * a.F * a.D;
  float* h = static_cast<float*>(a.h) +
             (sh ? TK * a.F + static_cast<size_t>(tok) * a.Fs : static_cast<size_t>(r) * a.F);
  for (int f = blockIdx.y * 4 + wave; f < F; f += gridDim.y * 4) {
    const float g = dot_f32(xg, wg + static_cast<size_t>(f) * a.D, a.D, lane);
    const float u = dot_f32(xg, wu + static_cast<size_t>(f) * a.D, a.D, lane);
    if (lane == 0) h[f] = silu_f(g) * u;
  }
}

__global__ __launch_bounds__(256) void down_f32_kernel(FfnArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x;
  int e, tok;
  bool sh;
  if (!f32_row(a, r, e, tok, sh)) return;
  const int F = sh ? a.Fs : a.F;
  const size_t TK = static_cast<size_t>(a.T) * a.K;
  const float* h = static_cast<const float*>(a.h) +
                   (sh ? TK * a.F + static_cast<size_t>(tok) * a.Fs : static_cast<size_t>(r) * a.F);
  const float* wd = sh ? static_cast<const float*>(a.sd)
                       : static_cast<const float*>(a.wd) + static_cast<size_t>(e) * a.F * a.D;
  float* o = a.o + static_cast<size_t>(r) * a.D;
  for (int d = blockIdx.y * 4 + wave; d < a.D; d += gridDim.y * 4) {
    const float s = dot_f32(h, wd + static_cast<size_t>(d) * F, F, lane);
    if (lane == 0) o[d] = s;
  }
}

// ---------------------------------------------------------------- combine
// y[t][d] = sum_j topk_w[t][j] * O[pos[t*K+j]][d]  (slot order j = 0..K-1)
//           (+ O[TK + t][d] shared) (+ x[t][d] residual); 4 columns per thread.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(FfnArgs a) {
  const int t = blockIdx.x;
  const int d = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (a.dn.on && blockIdx.x == 0 && blockIdx.y == 0) {
    // dense short block: cnt_i and the number of experts that received a token, from
    // the bitmaps stage 2 left (integer work, the same whatever the order)
    __shared__ int s_live;
    if (threadIdx.x == 0) s_live = 0;
    __syncthreads();
    int live = 0;
    for (int e = threadIdx.x; e < a.M; e += 256) {
      const int sl = a.dn.slot_of[e];
      const int c = (sl >= 0 && sl < a.n_slots) ? __popc(a.dn.tokmask[sl]) : 0;
      a.dn.expert_counts[e] = c;
      live += c > 0 ? 1 : 0;
    }
    if (live) atomicAdd(&s_live, live);
    __syncthreads();
    // (a negative value was put there by a routing launch that gave up, or carried over
    // from an earlier layer of a stack: it stays)
    if (threadIdx.x == 0 && a.dn.n_unique[0] >= 0) a.dn.n_unique[0] = s_live;
  }
  if (d >= a.D) return;
  const int K = a.K;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  // eight slots at a time: their position, gate and output-row loads are all in
  // flight together; the sum still runs in slot order
  for (int j0 = 0; j0 < K; j0 += 8) {
    int r[8];
    float w[8];
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool in = j0 + u < K;
      r[u] = in ? a.pos[t * K + j0 + u] : -1;
      w[u] = in ? a.topk_w[t * K + j0 + u] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = r[u] >= 0 ? *reinterpret_cast<const float4*>(a.o + static_cast<size_t>(r[u]) * a.D + d)
                       : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (r[u] < 0) continue;
      acc.x = fmaf(w[u], v[u].x, acc.x);
      acc.y = fmaf(w[u], v[u].y, acc.y);
      acc.z = fmaf(w[u], v[u].z, acc.z);
      acc.w = fmaf(w[u], v[u].w, acc.w);
    }
  }
  if (a.Fs > 0) {
    const size_t r = static_cast<size_t>(a.T) * K + t;
    const float4 v = *reinterpret_cast<const float4*>(a.o + r * a.D + d);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  const size_t xo = static_cast<size_t>(t) * a.D + d;
  if (BF16) {
    if (a.residual) {
      const u16x4 xv = *reinterpret_cast<const u16x4*>(static_cast<const uint16_t*>(a.x) + xo);
      acc.x += bf16_bits_to_f32(xv[0]); acc.y += bf16_bits_to_f32(xv[1]);
      acc.z += bf16_bits_to_f32(xv[2]); acc.w += bf16_bits_to_f32(xv[3]);
    }
    u16x4 out;
    out[0] = f32_to_bf16_bits(acc.x); out[1] = f32_to_bf16_bits(acc.y);
    out[2] = f32_to_bf16_bits(acc.z); out[3] = f32_to_bf16_bits(acc.w);
    *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(a.y) + xo) = out;
  } else {
    if (a.residual) {
      const float4 xv = *reinterpret_cast<const float4*>(static_cast<const float*>(a.x) + xo);
      acc.x += xv.x; acc.y += xv.y; acc.z += xv.z; acc.w += xv.w;
    }
    *reinterpret_cast<float4*>(static_cast<float*>(a.y) + xo) = acc;
  }
}

// ------------------------------------------------------------------ packing
// dst tile layout documented in des.h (des_pack_expert_weights).
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t* __restrict__ src,
                                                   uint16_t* __restrict__ dst, int rows, int cols,
                                                   long long groups_total) {
  // one thread per group of 8 values
  const long long g = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (g >= groups_total) return;
  const long long per_mat = static_cast<long long>(rows) * cols / 8;
  const long long m = g / per_mat;
  long long q = g % per_mat;
  const int l = static_cast<int>(q % 64);
  q /= 64;
  const int ct = static_cast<int>(q % (cols / 32));
  const int rt = static_cast<int>(q / (cols / 32));
  const uint16_t* s = src + m * rows * cols + static_cast<long long>(rt * 16 + (l & 15)) * cols +
                      ct * 32 + 8 * (l >> 4);
  *reinterpret_cast<uint4*>(dst + g * 8) = *reinterpret_cast<const uint4*>(s);
}

int launch_pack(const void* src, void* dst, int64_t n_mats, int rows, int cols, hipStream_t st) {
  const long long groups = n_mats * rows * static_cast<long long>(cols) / 8;
  const long long blocks = (groups + 255) / 256;
  launch(kKPack, pack_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st,
         static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), rows, cols, groups);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "pack launch");
}

// ------------------------------------------------------------- read ceiling
// Bare streaming read: every wavefront pulls one contiguous 64 KB chunk with
// sixteen 16-byte loads per lane in flight and does nothing else.  What this
// reaches is the machine's practical ceiling for a weight scan, the figure
// the FFN kernels are quoted against beside the 8 TB/s data-sheet peak.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbeChunk = 65536;

__global__ __launch_bounds__(kWave) void read_probe_kernel(const u32x4* __restrict__ src,
                                                           u32x4* __restrict__ sink) {
  constexpr int kVecs = kProbeChunk / 16, kU = 16;
  const u32x4* p = src + static_cast<size_t>(blockIdx.x) * kVecs + threadIdx.x;
  u32x4 acc = {0, 0, 0, 0};
  for (int i = 0; i < kVecs; i += kWave * kU) {
    u32x4 v[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) v[u] = __builtin_nontemporal_load(p + i + u * kWave);
#pragma unroll
    for (int u = 0; u < kU; ++u) acc ^= v[u];
  }
  // keeps the loads alive; the pattern does not occur in real data
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u) sink[0] = acc;
}

int launch_read_probe(const void* src, size_t bytes, void* sink, hipStream_t st) {
  launch(kKProbe, read_probe_kernel, dim3(static_cast<unsigned>(bytes / kProbeChunk)), dim3(kWave), 0,
         st, static_cast<const u32x4*>(src), static_cast<u32x4*>(sink));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "read probe launch");
}

// ------------------------------------------------------------------ launcher
int launch_ffn(const des_shape_t& s, const void* x, const void* w_gate, const void* w_up,
               const void* w_down, const void* ws_gate, const void* ws_up, const void* ws_down,
               const float* logits, int32_t* topk_idx, float* topk_w, int32_t* expert_counts,
               int32_t* n_unique, void* y, char* ws, unsigned long long epoch, hipStream_t st) {
  const WsLayout w = ws_layout(s);
  FfnArgs a;
  a.x = x;
  a.wg = w_gate; a.wu = w_up; a.wd = w_down;
  a.sg = ws_gate; a.su = ws_up; a.sd = ws_down;
  a.topk_idx = topk_idx;
  a.topk_w = topk_w;
  a.slots = reinterpret_cast<const int4*>(ws + w.slots);
  a.meta = reinterpret_cast<const int32_t*>(ws + w.meta);
  a.pair_tok = reinterpret_cast<const int32_t*>(ws + w.pair_tok);
  a.slot_tok = reinterpret_cast<const uint16_t*>(ws + w.slot_tok);
  a.units = reinterpret_cast<const int32_t*>(ws + w.units);
  a.pos = reinterpret_cast<const int32_t*>(ws + w.pos);
  a.h = ws + w.h;
  a.o = reinterpret_cast<float*>(ws + w.o);
  a.y = y;
  a.T = s.n_seqs * s.n_tokens;
  a.D = s.hidden; a.M = s.n_experts; a.F = s.ffn; a.Fs = s.ffn_shared; a.K = s.top_k;
  a.n_slots = max_live_experts(s);
  a.residual = s.residual;
  a.splits = 1;
  a.h_rows = w.h_rows;
  a.dn = DenseArgs{};
  int n_s2 = 0;  // wavefronts of the gate/up launch that run stage 2 (dense short block)
  if (dense_block(s)) {
    a.dn.on = 1;
    a.dn.lpt = 1024 / selector_tokens_per_pass(s.n_experts);
    a.dn.sigmoid = s.router_act == DES_ROUTER_SIGMOID;
    a.dn.logits = logits;
    a.dn.topk_idx = topk_idx;
    a.dn.topk_w = topk_w;
    a.dn.slot_of = reinterpret_cast<const int32_t*>(ws + w.slot_of);
    a.dn.tokmask = reinterpret_cast<uint32_t*>(ws + w.tokmask);
    a.dn.choice = reinterpret_cast<uint8_t*>(ws + w.choice);
    a.dn.pos = reinterpret_cast<int32_t*>(ws + w.pos);
    a.dn.expert_counts = expert_counts;
    a.dn.n_unique = n_unique;
    n_s2 = (a.T * a.dn.lpt + 63) / 64;
  }
  const int TK = a.T * a.K;

  if (s.dtype == DES_BF16) {
    const bool packed = s.weight_layout == DES_LAYOUT_PACKED;
    const int gu_tasks = a.n_slots * (a.F / (16 * kGuTiles)) + a.Fs / (16 * kGuTiles);
    const int gu_blocks = (gu_tasks + n_s2 + kFfnWaves - 1) / kFfnWaves;
    const int groups = (a.D / 16 + 3) / 4;
    const int dn_tasks = a.n_slots * groups + (a.Fs > 0 ? groups : 0);
    const int dn_blocks = (dn_tasks + kFfnWaves - 1) / kFfnWaves;
    // an expert serves a token at most once, so no task has more than T pairs
    const int maxnt = (a.T + 15) / 16;
    const dim3 blk(kFfnWaves * kWave);
    // Few experts (small coreset): halve the task size so that enough wavefronts
    // keep bytes in flight.  Measured: gate/up gains below ~512 tasks (18.4 vs
    // 20.5 us at 272) and loses above (36.4 vs 34.4 us at 768); the down projection
    // gains up to 1024 tasks while a halved task still streams >= 48 KB (F >= 768).
    const bool gu_fine = gu_tasks < 512;
    const bool dn_fine = dn_tasks <= 1024 && a.F >= 768;
    const int gu_fine_tasks = a.n_slots * (a.F / 16) + a.Fs / 16;
    const int dn_fine_groups = (a.D / 16 + 1) / 2;
    const int dn_fine_tasks = a.n_slots * dn_fine_groups + (a.Fs > 0 ? dn_fine_groups : 0);
#define DES_LAUNCH_FFN(NTV, PK)                                                             \
  do {                                                                                      \
    if (gu_fine && NTV <= 2)                                                                \
      launch(kKGateUp, gateup_bf16_kernel<NTV, PK, 4, 4, 1>, dim3(gu_fine_tasks + n_s2), blk, 0, st, a); \
    else                                                                                    \
      launch(kKGateUp, gateup_bf16_kernel<NTV, PK>, dim3(gu_blocks), blk, 0, st, a);        \
    if (dn_fine && NTV <= 2)                                                                \
      launch(kKDown, down_bf16_kernel<NTV, PK, 4, 4, 2>, dim3(dn_fine_tasks), blk, 0, st, a); \
    else                                                                                    \
      launch(kKDown, down_bf16_kernel<NTV, PK>, dim3(dn_blocks), blk, 0, st, a);            \
  } while (0)
#define DES_LAUNCH_BY_NT(PK)                                                                \
  do {                                                                                      \
    if (maxnt <= 1) DES_LAUNCH_FFN(1, PK);                                                  \
    else if (maxnt <= 2) DES_LAUNCH_FFN(2, PK);                                             \
    else if (maxnt <= 4) DES_LAUNCH_FFN(4, PK);                                             \
    else if (maxnt <= 8) DES_LAUNCH_FFN(8, PK);                                             \
    else DES_LAUNCH_FFN(16, PK);                                                            \
  } while (0)
    const bool chunked = a.D % kKC == 0 && a.F % kKC == 0 && a.Fs % kKC == 0;
    if (a.T > 32 && chunked) {
      // Larger blocks: activations staged through LDS.  Token rows per workgroup
      // pass: 64 while no expert can have more, else 128; an expert with more
      // pairs is spread over up to kMaxSplits workgroups (the unit list).  Wavefronts per workgroup:
      // two give the finest spread of the weight bytes over the compute units;
      // four share the staged activations among more weight rows, which
      // measured better once experts have many tokens (48-layer stack: 7.7 ms
      // against 8.0 ms; down projection at T = 128: 23 us against 27 us).
      const int rows_pass = lds_rows_pass(a.T);
      const bool small = rows_pass == 64;
      int splits = (a.T + rows_pass - 1) / rows_pass;  // of the shared expert (all T rows)
      if (splits > kMaxSplits) splits = kMaxSplits;
      const int n_units = max_units(s);
      const int gu_lw = a.T <= 128 ? 2 : 4;
      const int dn_lw = a.T <= 64 ? 2 : 4;
      const int gu_lds = n_units * ((a.F / 16 + gu_lw - 1) / gu_lw) + splits * ((a.Fs / 16 + gu_lw - 1) / gu_lw);
      const int per_dn = (a.D / 32 + dn_lw - 1) / dn_lw;
      const int dn_lds = n_units * per_dn + (a.Fs > 0 ? splits * per_dn : 0);
      const dim3 gg(gu_lds), dg(dn_lds);
      a.splits = splits;
      // unrolled reduction lengths (the shared expert shares the down launch)
      const int gu_kd = a.D == 2048 ? 2048 : 0;
      const int dn_kd = (a.Fs != 0 && a.Fs != a.F) ? 0 : (a.F == 768 || a.F == 512) ? a.F : 0;
#define DES_LAUNCH_GU(PK, MNT, LWV)                                                         \
  do {                                                                                      \
    const dim3 lb(LWV* kWave);                                                              \
    if (gu_kd == 2048) launch(kKGateUp, gateup_lds_kernel<PK, MNT, LWV, 2048>, gg, lb, 0, st, a); \
    else launch(kKGateUp, gateup_lds_kernel<PK, MNT, LWV, 0>, gg, lb, 0, st, a);            \
  } while (0)
#define DES_LAUNCH_DN(PK, MNT, LWV)                                                         \
  do {                                                                                      \
    const dim3 lb(LWV* kWave);                                                              \
    if (dn_kd == 768) launch(kKDown, down_lds_kernel<PK, MNT, LWV, 768>, dg, lb, 0, st, a); \
    else if (dn_kd == 512) launch(kKDown, down_lds_kernel<PK, MNT, LWV, 512>, dg, lb, 0, st, a); \
    else launch(kKDown, down_lds_kernel<PK, MNT, LWV, 0>, dg, lb, 0, st, a);                \
  } while (0)
#define DES_LAUNCH_LDS(PK)                                                        \
  do {                                                                            \
    if (small) DES_LAUNCH_GU(PK, 4, 2);                                           \
    else if (gu_lw == 2) DES_LAUNCH_GU(PK, 8, 2);                                 \
    else DES_LAUNCH_GU(PK, 8, 4);                                                 \
    if (small) DES_LAUNCH_DN(PK, 4, 2);                                           \
    else DES_LAUNCH_DN(PK, 8, 4);                                                 \
  } while (0)
      if (packed) DES_LAUNCH_LDS(true);
      else DES_LAUNCH_LDS(false);
#undef DES_LAUNCH_GU
#undef DES_LAUNCH_DN
#undef DES_LAUNCH_LDS
    } else if (packed) {
      DES_LAUNCH_BY_NT(true);
    } else {
      DES_LAUNCH_BY_NT(false);
    }
#undef DES_LAUNCH_BY_NT
#undef DES_LAUNCH_FFN
    dim3 cg(a.T, (a.D / 4 + 255) / 256);
    launch(kKCombine, combine_kernel<true>, cg, dim3(256), 0, st, a);
  } else {
    const int rows = TK + (a.Fs > 0 ? a.T : 0);
    const int Fm = a.F > a.Fs ? a.F : a.Fs;
    launch(kKGateUp, gateup_f32_kernel, dim3(rows, (Fm + 3) / 4 > 64 ? 64 : (Fm + 3) / 4),
           dim3(256), 0, st, a);
    launch(kKDown, down_f32_kernel, dim3(rows, (a.D + 3) / 4 > 64 ? 64 : (a.D + 3) / 4),
           dim3(256), 0, st, a);
    dim3 cg(a.T, (a.D / 4 + 255) / 256);
    launch(kKCombine, combine_kernel<false>, cg, dim3(256), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "ffn launch");
}

}  // namespace des

#ifdef DES_FFN_STAMPS
extern "C" int des_debug_ffn_stamps(long long* host, int n) {
  return hipMemcpyFromSymbol(host, HIP_SYMBOL(des::g_ffn_stamps), sizeof(long long) * n) == hipSuccess
             ? 0 : -6;
}
#endif
