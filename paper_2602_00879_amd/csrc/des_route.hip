// Router scores G(x) (Background, definition of the routing function) and the
// per-token softmax of Sec. 4.3, for gfx950.
//
//   logits[t][i] = sum_d x[t][d] * w_router[i][d] (+ bias[i])
//
// The block is tiny (T = B*N tokens, M experts) but the router matrix is
// 0.5-1 MB, too much for one compute unit to pull quickly, so the bf16 kernel
// splits the product over (expert tile, token tile) workgroups and, inside a
// workgroup, over the reduction dimension across 16 wavefronts whose 16x16
// partial tiles are summed through LDS in a fixed order.
#include "des_common.h"

namespace des {

constexpr int kRouterWaves = 16;

// One workgroup: experts [i0, i0+16) x tokens [t0, t0+16).  Wave w takes the
// k-steps w, w+16, ... (32 reduction elements each).
// MFMA 16x16x32 operand layout: lane l supplies row (l % 16), reduction
// elements 8*(l/16) .. +7; the accumulator of lane l holds column (l % 16),
// rows 4*(l/16) .. +3.  A = router rows (experts), B = tokens.
__global__ __launch_bounds__(kRouterWaves* kWave) void router_bf16_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wr,
    const float* __restrict__ bias, float* __restrict__ logits, int T, int D, int M) {
  __shared__ float part[kRouterWaves][16 * 16];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int i0 = blockIdx.x * 16;
  const int t0 = blockIdx.y * 16;
  const int r = lane & 15;
  const int kq = (lane >> 4) * 8;
  const int ei = min(i0 + r, M - 1);  // clamped rows are computed and dropped
  const int ti = min(t0 + r, T - 1);
  const uint16_t* ap = wr + static_cast<size_t>(ei) * D + kq;
  const uint16_t* bp = x + static_cast<size_t>(ti) * D + kq;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const int nks = D / 32;
  for (int ks = wave; ks < nks; ks += kRouterWaves) {
    bf16x8 a = *reinterpret_cast<const bf16x8*>(ap + ks * 32);
    bf16x8 b = *reinterpret_cast<const bf16x8*>(bp + ks * 32);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  }
  // element (expert row 4*(lane/16)+q, token column lane%16)
#pragma unroll
  for (int q = 0; q < 4; ++q) part[wave][(4 * (lane >> 4) + q) * 16 + r] = acc[q];
  __syncthreads();
  if (threadIdx.x < 256) {
    const int er = threadIdx.x & 15;   // expert within tile (fastest: coalesced store)
    const int tc = threadIdx.x >> 4;   // token within tile
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kRouterWaves; ++w) s += part[w][er * 16 + tc];
    const int e = i0 + er, t = t0 + tc;
    if (e < M && t < T) {
      if (bias) s += bias[e];
      logits[static_cast<size_t>(t) * M + e] = s;
    }
  }
}

// fp32 inputs: one wavefront per (token, expert) dot product, lanes stride the
// reduction dimension with 16-byte loads.  Serves the small fp32 configuration.
__global__ __launch_bounds__(256) void router_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ wr, const float* __restrict__ bias,
    float* __restrict__ logits, int T, int D, int M) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int t = blockIdx.x;
  const float4* xp = reinterpret_cast<const float4*>(x + static_cast<size_t>(t) * D);
  const int nv = D / 4;
  for (int e = blockIdx.y * 4 + wave; e < M; e += gridDim.y * 4) {
    const float4* wp = reinterpret_cast<const float4*>(wr + static_cast<size_t>(e) * D);
    float s = 0.f;
    for (int v = lane; v < nv; v += 64) {
      float4 a = xp[v], b = wp[v];
      s = fmaf(a.x, b.x, s);
      s = fmaf(a.y, b.y, s);
      s = fmaf(a.z, b.z, s);
      s = fmaf(a.w, b.w, s);
    }
    s = wave_sum_f32(s);
    if (lane == 0) logits[static_cast<size_t>(t) * M + e] = s + (bias ? bias[e] : 0.f);
  }
}

// probs[t][:] = softmax(logits[t][:]); one wavefront per token.
__global__ __launch_bounds__(64) void softmax_kernel(const float* __restrict__ logits,
                                                     float* __restrict__ probs, int M) {
  const int lane = threadIdx.x;
  const float* row = logits + static_cast<size_t>(blockIdx.x) * M;
  float* out = probs + static_cast<size_t>(blockIdx.x) * M;
  uint32_t mk = 0;
  for (int i = lane; i < M; i += 64) mk = max(mk, order_key(row[i]));
  mk = wave_max_u32(mk);
  // invert the key map to recover the maximum value
  const uint32_t mu = (mk & 0x80000000u) ? (mk & 0x7FFFFFFFu) : ~mk;
  const float mx = __uint_as_float(mu);
  float s = 0.f;
  for (int i = lane; i < M; i += 64) s += expf(row[i] - mx);
  s = wave_sum_f32(s);
  const float inv = 1.0f / s;
  for (int i = lane; i < M; i += 64) out[i] = expf(row[i] - mx) * inv;
}

int launch_router(const des_shape_t& s, const void* x, const void* w_router, const float* bias,
                  float* logits, hipStream_t st) {
  const int T = s.n_seqs * s.n_tokens;
  if (s.dtype == DES_BF16) {
    dim3 grid((s.n_experts + 15) / 16, (T + 15) / 16);
    hipLaunchKernelGGL(router_bf16_kernel, grid, dim3(kRouterWaves * kWave), 0, st,
                       static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_router),
                       bias, logits, T, s.hidden, s.n_experts);
  } else {
    dim3 grid(T, (s.n_experts + 3) / 4);
    hipLaunchKernelGGL(router_f32_kernel, grid, dim3(256), 0, st, static_cast<const float*>(x),
                       static_cast<const float*>(w_router), bias, logits, T, s.hidden,
                       s.n_experts);
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "router launch");
}

int launch_softmax(const des_shape_t& s, const float* logits, float* probs, hipStream_t st) {
  const int T = s.n_seqs * s.n_tokens;
  hipLaunchKernelGGL(softmax_kernel, dim3(T), dim3(64), 0, st, logits, probs, s.n_experts);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DES_OK : hip_fail(e, "softmax launch");
}

}  // namespace des
