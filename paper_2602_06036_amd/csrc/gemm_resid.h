// O and down projections for a single band of rows (M <= 16), unsplit, with the residual update and the input of
// the following RMSNorm folded into the epilogue:
//     h[m, n] += sum_k a[m, k] W[n, k]                       (residual stream, fp32, in place)
//     a_out[m, n] = h[m, n] * gain_next[n]                   (GEMM operand, hi + lo bf16 pair; NOT divided by the rms)
//     ssq[m, workgroup] = sum over the workgroup's 16 columns of h[m, n]^2
// RMSNorm(h) W' = (1 / rms(h)) * ((h * gain) W'): the GEMM that consumes a_out multiplies its result rows by
// 1 / sqrt(sum(ssq[m, :]) / D + eps) in its own epilogue (EpiArgs::ssq), so no kernel ever has to see a whole row
// between the two GEMMs and the separate normalisation launch disappears.  A workgroup owns ONE 16-row band of W over
// the whole K (N / 16 workgroups: 256 for the 8B shape, one per CU); its NW wavefronts split K, each streaming U k
// tiles at a time with the next U in flight, and meet in LDS.  Every element of h has exactly one writer, every sum a
// fixed order: results do not depend on timing.
#pragma once
#include "gemm.h"

struct ResidArgs {
  float* h;                 // [M, N] residual stream, updated in place
  const float* gain_next;   // [N] gain of the RMSNorm that reads the new h (next layer's first norm, or the final norm)
  bf16_t* a_out;            // operand tiles, row length N
  float* ssq;               // [M, N / 16]
  bf16_t* taps;             // nullable: the new h is also stored as tapped hidden state `tap_idx` (operand, row length tap_K)
  int tap_idx, tap_K;
};

template <int U>
struct ResidBuf {
  u32x4 w[U], ah[U], al[U];
};

template <int U, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_bf16_resid_kernel(const bf16_t* __restrict__ W, const bf16_t* __restrict__ A, int M,
                                                                  int N, int K, ResidArgs ra) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = blockIdx.x, n_tiles = N >> 4, KT = K >> 5;
  const int per = (KT + NW - 1) / NW;
  const int kb = min(KT, wave * per), ke = min(KT, kb + per);
  const int mrow = lane & 15, g = lane >> 4;
  const int col = n * 16 + 4 * g;
  const bool live = mrow < M;

  // the finishing wavefront asks for its piece of h and of the gain before the sweep: no dependent round trip at the end
  float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f), g4 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (wave == 0) {
    if (live) h4 = *reinterpret_cast<const float4*>(ra.h + (size_t)mrow * N + col);
    g4 = *reinterpret_cast<const float4*>(ra.gain_next + col);
  }

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const u32x4* Wp = reinterpret_cast<const u32x4*>(W) + (size_t)n * 64 + lane;
  const size_t w_step = (size_t)n_tiles * 64;   // weight tiles are k-tile-major
  const u32x4* Ap = reinterpret_cast<const u32x4*>(A) + lane;
  auto load = [&](ResidBuf<U>& b, int k0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = k0 + u < ke;
      const int kt = in ? k0 + u : ke - 1;   // past the range: the last tile again, against zeroed activations
      b.w[u] = __builtin_nontemporal_load(Wp + (size_t)kt * w_step);
      const u32x4 hi = Ap[(size_t)kt * 128];
      b.ah[u] = in ? hi : (u32x4){0u, 0u, 0u, 0u};
      const u32x4 lo = Ap[(size_t)kt * 128 + 64];
      b.al[u] = in ? lo : (u32x4){0u, 0u, 0u, 0u};
    }
  };
  auto compute = [&](const ResidBuf<U>& b) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b.w[u]), __builtin_bit_cast(bf16x8, b.ah[u]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b.w[u]), __builtin_bit_cast(bf16x8, b.al[u]), acc, 0, 0, 0);
    }
  };
  // two register buffers; no load inside the loop is conditional (the tail is peeled), see gemm_bf16_kernel
  if (kb < ke) {
    ResidBuf<U> b0, b1;
    load(b0, kb);
    int k0 = kb;
    for (; k0 + 2 * U < ke; k0 += 2 * U) {
      load(b1, k0 + U);
      compute(b0);
      load(b0, k0 + 2 * U);
      compute(b1);
    }
    load(b1, k0 + U);
    compute(b0);
    compute(b1);
  }

  __shared__ float4 red[NW][64];
  red[wave][lane] = make_float4(acc[0], acc[1], acc[2], acc[3]);
  __syncthreads();
  if (wave != 0) return;
  float4 s = red[0][lane];
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    const float4 a = red[w][lane];
    s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
  }
  const float4 hn = make_float4(h4.x + s.x, h4.y + s.y, h4.z + s.z, h4.w + s.w);
  float q = hn.x * hn.x + hn.y * hn.y + hn.z * hn.z + hn.w * hn.w;
  q += __shfl_xor(q, 16, 64);
  q += __shfl_xor(q, 32, 64);
  if (!live) return;
  *reinterpret_cast<float4*>(ra.h + (size_t)mrow * N + col) = hn;
  Act<bf16_t>::store4(ra.a_out, mrow, col, N, make_float4(hn.x * g4.x, hn.y * g4.y, hn.z * g4.z, hn.w * g4.w));
  if (ra.taps) Act<bf16_t>::store4(ra.taps, mrow, ra.tap_idx * N + col, ra.tap_K, hn);
  if (g == 0) ra.ssq[(size_t)mrow * gridDim.x + n] = q;
}
