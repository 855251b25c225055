// Streaming GEMM building block shared by the kernels that stage token rows through
// LDS (the expert FFN for blocks of more than 32 tokens, the dense projections of the
// attention sub-layer): weights from HBM straight into MFMA operands, token rows from
// L2 into LDS by direct loads, explicit wait counts.  gfx950 only.
#pragma once

#include <type_traits>
#include <utility>

#include "des_common.h"

namespace des {

typedef std::integral_constant<int, 0> S0;
typedef std::integral_constant<int, 1> S1;

// elements between consecutive k-steps of a 16-row weight tile
template <bool PACKED>
__device__ __forceinline__ constexpr int frag_step() { return PACKED ? 512 : 32; }

// ------------------------------------------ token rows via LDS, weights via registers
// With more than two token tiles per expert the direct scheme above runs out
// of registers for its prefetch (every token fragment is double-buffered in
// registers).  For T > 32 the expert's activation rows go through LDS instead:
//   * a workgroup of LW wavefronts works on LW weight-row groups of one expert;
//     each wavefront streams its own two weight tiles from HBM straight into
//     MFMA operands, three chunks of 128 reduction elements deep, so that two
//     chunks (16 KB per wavefront) stay in flight across every barrier;
//   * the expert's token rows of the next chunk are gathered from L2 into LDS
//     by direct global-to-LDS loads (no staging registers), double-buffered;
//   * LDS rows are 256 B with the 16-byte pieces of row r stored at piece
//     index p ^ (r & 15): a direct load writes lane l at base + 16*l, so the
//     swizzle is applied on the global side (which piece a lane fetches), and
//     the 16 token rows an MFMA operand reads fall into 16 different banks.
// The compiler cannot tell which LDS reads depend on which direct load and
// would wait for all of them before every read; the token fragments are
// therefore read with inline ds_read_b128 (each group followed by its own
// lgkmcnt wait) and the direct loads are waited for by explicit vmcnt counts.
// None of these asm statements claims to touch memory (a "memory" clobber makes
// the compiler wait for every pending direct load first); they are volatile,
// which keeps them in program order with each other, the barriers and the
// direct loads.
constexpr int kKC = 128;            // reduction lengths must be multiples of this
#define DES_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N));
}

// b[i] = 16 bytes at LDS address addr + BASE + i*TILE (token tile i of a buffer;
// TILE = bytes of 16 token rows).
template <int NT, int BASE, int TILE>
__device__ __forceinline__ void lds_frags(bf16x8 (&b)[NT], uint32_t addr) {
  static_assert(NT >= 1 && NT <= 4, "token tiles fetched at a time");
  if constexpr (NT == 1) {
    asm volatile("ds_read_b128 %0, %1 offset:%2\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(b[0])
                 : "v"(addr), "n"(BASE + 0 * TILE)
                 :);
  }
  if constexpr (NT == 2) {
    asm volatile("ds_read_b128 %0, %2 offset:%3\n\t"
                 "ds_read_b128 %1, %2 offset:%4\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(b[0]), "=&v"(b[1])
                 : "v"(addr), "n"(BASE + 0 * TILE), "n"(BASE + 1 * TILE)
                 :);
  }
  if constexpr (NT == 3) {
    asm volatile("ds_read_b128 %0, %3 offset:%4\n\t"
                 "ds_read_b128 %1, %3 offset:%5\n\t"
                 "ds_read_b128 %2, %3 offset:%6\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2])
                 : "v"(addr), "n"(BASE + 0 * TILE), "n"(BASE + 1 * TILE), "n"(BASE + 2 * TILE)
                 :);
  }
  if constexpr (NT == 4) {
    asm volatile("ds_read_b128 %0, %4 offset:%5\n\t"
                 "ds_read_b128 %1, %4 offset:%6\n\t"
                 "ds_read_b128 %2, %4 offset:%7\n\t"
                 "ds_read_b128 %3, %4 offset:%8\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]), "=&v"(b[3])
                 : "v"(addr), "n"(BASE + 0 * TILE), "n"(BASE + 1 * TILE), "n"(BASE + 2 * TILE), "n"(BASE + 3 * TILE)
                 :);
  }
}

// One 16-byte weight fragment, asynchronously: the register is valid only after
// a wait_weights() that names it.  (The compiler's own vmcnt bookkeeping gives
// up across the rotating stages and early exits of the chunk loop and waits for
// everything at every use, which would drain the prefetch; so these loads and
// their waits are explicit.)
template <int OFF>
__device__ __forceinline__ void ld8_async(bf16x8& v, const uint16_t* ubase, uint32_t lane_off) {
  // s_nop 4: the base may have just been written by a vector instruction (a
  // scalar register restored from a spill lane); a vector-memory instruction
  // needs five wait states after that, and the compiler adds none inside asm.
  asm volatile("s_nop 4\n\tglobal_load_dwordx4 %0, %1, %2 offset:%3 nt"
               : "=v"(v)
               : "v"(lane_off), "s"(ubase), "n"(OFF));
}
// A pointer the compiler may keep in scalar registers (the value is the same in all lanes).
template <typename T>
__device__ __forceinline__ T* uniform_ptr(T* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
  return reinterpret_cast<T*>((static_cast<unsigned long long>(hi) << 32) | lo);
}
// Weight tile rt of a [rows][kd] matrix as uniform base + per-lane byte offset.
template <bool PACKED>
__device__ __forceinline__ const uint16_t* tile_base(const uint16_t* base, int rt, int kd) {
  return base + static_cast<size_t>(rt) * 16 * kd;  // 16 rows of kd values in either layout
}
template <bool PACKED>
__device__ __forceinline__ uint32_t tile_lane_off(int kd, int lane) {
  return PACKED ? lane * 16u : ((lane & 15) * static_cast<uint32_t>(kd) + (lane >> 4) * 8u) * 2u;
}
// Waits until at most N vector-memory operations are outstanding and makes the
// fragments of a stage depend on that wait.
template <int N>
__device__ __forceinline__ void wait_weights(bf16x8 (&a)[4], bf16x8 (&b)[4]) {
  asm volatile("s_waitcnt vmcnt(%8)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]),
                 "+v"(b[3])
               : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_weights(bf16x8 (&a)[2], bf16x8 (&b)[2]) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0]), "+v"(b[1]) : "n"(N));
}

template <int... I, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}

// acc0/acc1 += A0/A1 (this wavefront's two 16-row weight tiles, reduction
// length kd) x token rows.  KC = reduction elements per chunk (128 or 64), KD =
// the reduction length if known at compile time (then kd == KD), else 0; kd is a
// multiple of KC.  Row r of the pass (r < 16*NT) is `base + row_off(min(r,
// rows_valid-1))`.  `lds` is the workgroup's buffer of NB * ROWS * 2*KC bytes
// (ROWS >= 16*NT), NB = 3 if KD > 0, else 2.  All LW wavefronts of the workgroup call it together;
// a0, a1, base and `wave` are wavefront-uniform; w_lane_off is the lane's byte
// offset inside a weight fragment.
//
// LDS rows hold one chunk of a token row (2*KC bytes) with the 16-byte piece p
// of row r stored at piece index p ^ swz(r), swz(r) = r & 15 for 256-byte rows,
// (r >> 1) & 7 for 128-byte rows: the 16 token rows an MFMA operand reads fall
// into 16 different bank groups.  A direct load writes lane l at base + 16*l,
// so the swizzle is applied on the global side (which piece a lane fetches).
//
// A wavefront without a tile of its own (row tiles not a multiple of LW) runs
// on tile 0 and drops its result.
template <int NT, int ROWS, bool PACKED, int LW, int KC, int KD, typename RowOff>
__device__ __forceinline__ void dma_stream_gemm(const uint16_t* a0, const uint16_t* a1,
                                                uint32_t w_lane_off, int wave, int kd,
                                                int rows_valid, const uint16_t* base,
                                                RowOff row_off, uint16_t* lds,
                                                f32x4 (&acc0)[NT], f32x4 (&acc1)[NT]) {
  static_assert(KC == 128 || KC == 64, "chunk of 4 or 2 k-steps");
  static_assert(KD % KC == 0, "reduction length must be whole chunks");
  const int lane = threadIdx.x & 63;
  const int nchunks = kd / KC;
  constexpr int NCH = KD / KC;
  constexpr int KS = KC / 32;        // k-steps per chunk
  constexpr int RB = KC * 2;         // bytes of a token row in LDS
  constexpr int PP = KC / 8;         // 16-byte pieces per row
  constexpr int RPI = 64 / PP;       // rows one direct load (64 lanes x 16 B) covers
  constexpr int NG = 16 * NT / RPI;  // direct loads per chunk (RPI rows each)
  constexpr int ND = (NG + LW - 1) / LW;  // ... per wavefront: every wavefront issues as many,
                                     // so that the wait counts below hold for all of them; one
                                     // without a group of its own repeats the last group
                                     // (same bytes to the same place)
  constexpr int NW = 2 * KS;         // weight loads per wavefront and chunk
  constexpr int kBufBytes = ROWS * RB;
  constexpr int kTile = 16 * RB;     // bytes of one token tile in a buffer
  constexpr int kFragBytes = frag_step<PACKED>() * 2;  // between k-steps of a weight tile
  auto swz = [](int r) { return KC == 128 ? (r & 15) : ((r >> 1) & 7); };
  // All addresses are a uniform base, advanced per chunk in scalar registers,
  // plus a per-lane byte offset that never changes.
  uint32_t off[ND];                  // byte offset of this lane's piece of its rows, chunk 0
#pragma unroll
  for (int i = 0; i < ND; ++i) {
    const int row = min(i * LW + wave, NG - 1) * RPI + lane / PP;
    off[i] = (static_cast<uint32_t>(row_off(min(row, rows_valid - 1))) +
              (((lane % PP) ^ swz(row)) << 3)) * 2u;
  }
  // (asm, not the builtin: after the builtin the compiler waits for all
  // outstanding loads as soon as an address register is reused)
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<size_t>(DES_LDS_PTR(lds)));
  auto dma = [&](int chunk, auto bufc) {
    constexpr int bs = decltype(bufc)::value;
    const uint16_t* g = base + chunk * KC;  // uniform
#pragma unroll
    for (int i = 0; i < ND; ++i) {
      const uint32_t dst = lds0 + bs * kBufBytes + min(i * LW + wave, NG - 1) * 1024;  // uniform
      const uint32_t o = off[i];
      // Wait states the compiler would insert for its own instructions but does
      // not for asm: one between the write of M0 and the load, five between a
      // vector instruction that wrote the base registers (a scalar register
      // restored from a spill lane) and the load.
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1"
                   ::"v"(o), "s"(g), "s"(dst)
                   : "m0");
    }
  };
  bf16x8 aw0[KD > 0 ? 3 : 2][KS], aw1[KD > 0 ? 3 : 2][KS];
  auto loadw = [&](int chunk, auto stage) {
    constexpr int s = decltype(stage)::value;
    const uint16_t* q0 = a0 + static_cast<size_t>(chunk) * KS * frag_step<PACKED>();
    const uint16_t* q1 = a1 + static_cast<size_t>(chunk) * KS * frag_step<PACKED>();
    ld8_async<0 * kFragBytes>(aw0[s][0], q0, w_lane_off);
    ld8_async<0 * kFragBytes>(aw1[s][0], q1, w_lane_off);
    ld8_async<1 * kFragBytes>(aw0[s][1], q0, w_lane_off);
    ld8_async<1 * kFragBytes>(aw1[s][1], q1, w_lane_off);
    if constexpr (KS == 4) {
      ld8_async<2 * kFragBytes>(aw0[s][2], q0, w_lane_off);
      ld8_async<2 * kFragBytes>(aw1[s][2], q1, w_lane_off);
      ld8_async<3 * kFragBytes>(aw0[s][3], q0, w_lane_off);
      ld8_async<3 * kFragBytes>(aw1[s][3], q1, w_lane_off);
    }
  };
  // LDS byte address of this lane's fragment of token tile 0, k-step u of a chunk
  uint32_t fa[KS];
#pragma unroll
  for (int u = 0; u < KS; ++u)
    fa[u] = lds0 + (lane & 15) * RB + (((u * 4 + (lane >> 4)) ^ swz(lane & 15)) << 4);
  auto compute = [&](auto bufc, auto stage) {
    constexpr int bs = decltype(bufc)::value;
    constexpr int s = decltype(stage)::value;
    constexpr int G = NT > 4 ? NT / 2 : NT;  // token tiles fetched from LDS at a time
#pragma unroll
    for (int u = 0; u < KS; ++u) {
#pragma unroll
      for (int g = 0; g < NT; g += G) {
        bf16x8 b[G];
        if (g == 0) lds_frags<G, bs * kBufBytes, kTile>(b, fa[u]);
        else lds_frags<G, bs * kBufBytes + G * kTile, kTile>(b, fa[u]);
#pragma unroll
        for (int i = 0; i < G; ++i) {
          acc0[g + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw0[s][u], b[i], acc0[g + i], 0, 0, 0);
          acc1[g + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw1[s][u], b[i], acc1[g + i], 0, 0, 0);
        }
      }
    }
  };
  if constexpr (KD > 0) {
    // Reduction length known at compile time, three LDS buffers: straight-line
    // code, activations and weights both two chunks ahead.  Issue order of
    // vector-memory operations (A = this wavefront's ND activation loads of a
    // chunk, W = its NW weight loads):
    //   A(0) W(0) A(1) W(1) | step 0: A(2) W(2) | step 1: A(3) W(3) | ...
    // They complete in order, so "at most ND + NW outstanding" at the top of
    // step c means A(c) and W(c) have landed while chunk c+1 is still in flight.
    // A(c+2) overwrites the buffer chunk c-1 was read from; the barrier of step
    // c comes after everybody's reads of it.
    static_assert(ND + NW <= 63, "wait count must fit the counter");
    dma(0, S0{});
    loadw(0, S0{});
    if constexpr (NCH > 1) {
      dma(1, S1{});
      loadw(1, S1{});
    }
    static_for(std::make_integer_sequence<int, NCH>{}, [&](auto cc) {
      constexpr int c = decltype(cc)::value;
      typedef std::integral_constant<int, c % 3> Cur;
      typedef std::integral_constant<int, (c + 2) % 3> Nxt;
      if constexpr (c + 1 < NCH) wait_weights<ND + NW>(aw0[c % 3], aw1[c % 3]);
      else wait_weights<0>(aw0[c % 3], aw1[c % 3]);
      __builtin_amdgcn_s_barrier();
      if constexpr (c + 2 < NCH) {
        dma(c + 2, Nxt{});
        loadw(c + 2, Nxt{});
      }
      compute(Cur{}, Cur{});
    });
  } else {
    // Any reduction length: two stages.  Step c: everything this wavefront asked
    // for (its share of the activations of chunk c, its weights of chunk c) has
    // landed; the barrier then says the same of the other wavefronts' shares, and
    // that everybody is done reading the other buffer, which the loads of chunk
    // c+1 overwrite while chunk c is multiplied.
    auto step = [&](int c, auto bufc, auto nextbuf) {
      constexpr int s = decltype(bufc)::value;
      wait_weights<0>(aw0[s], aw1[s]);
      __builtin_amdgcn_s_barrier();
      if (c + 1 < nchunks) {
        dma(c + 1, nextbuf);
        loadw(c + 1, nextbuf);
      }
      compute(bufc, bufc);
    };
    dma(0, S0{});
    loadw(0, S0{});
    for (int c = 0; c < nchunks; c += 2) {
      step(c, S0{}, S1{});
      if (c + 1 >= nchunks) break;
      step(c + 1, S1{}, S0{});
    }
  }
  __builtin_amdgcn_s_barrier();  // nobody still reads a buffer the next pass refills
}

// Every pass works in buffers of 16 KB: up to 64 token rows with chunks of 128
// reduction elements, or up to 128 rows with chunks of 64.  Three buffers when
// the reduction length is a compile-time constant (48 KB: three workgroups per
// compute unit), else two.
constexpr int kLdsBufElems = 8192;
__host__ __device__ constexpr int lds_elems(int kd) { return (kd > 0 ? 3 : 2) * kLdsBufElems; }

}  // namespace des
