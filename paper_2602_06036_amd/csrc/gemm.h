// Weight-streaming GEMMs: y[M,N] = a[M,K] * W[N,K]^T with fused epilogues.
//   bf16: MFMA 16x16x32, weights in the tiled layout of common.h, activations as hi+lo bf16 pairs
//         (two MFMAs per weight tile), fp32 accumulation.
//   fp32: one wavefront per output column (tiny models only).
#pragma once
#include "common.h"

enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

struct EpiArgs {
  float* out;   // STORE: out[m*ld + n] = y ; RESID: out[m*ld + n] += y
  int ld;
  void* act;    // SWIGLU: act (tile layout, row length act_K) [m, j] = silu(gate_j) * up_j
  int act_K;
};

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel.  A workgroup of 4 wavefronts owns NT 16-row bands of W (N tiles) and MT 16-row
// bands of the activations; each wavefront streams one quarter of K and the four partial sums are
// added in a fixed order through LDS (deterministic).  The MFMA computes D^T = W_tile * a_tile^T:
// lane l ends up holding y[m = l%16][n = 4*(l/16) .. +3].
// SWIGLU: W rows alternate 16 gate rows / 16 up rows, so tiles (2p, 2p+1) of a workgroup are the
// gate and up values of the same 16 activation columns.
// ------------------------------------------------------------------------------------------------
template <int NT, int MT, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ W, const bf16_t* __restrict__ A,
                                                        int M, int N, int K, EpiArgs ep) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nt0 = blockIdx.x * NT, mt0 = blockIdx.y * MT;
  const int KT = K >> 5;
  const int m_tiles = (M + 15) >> 4;
  const int kt_per = (KT + 3) >> 2;
  const int kt_begin = wave * kt_per;
  const int kt_end = min(KT, kt_begin + kt_per);

  f32x4 acc[NT][MT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const u32x4* Wp = reinterpret_cast<const u32x4*>(W) + lane;
  const u32x4* Ap = reinterpret_cast<const u32x4*>(A) + lane;
  // activation bands past the last one alias the last band (their results are never stored);
  // a band holds, per k tile, the hi tile then the lo tile (64 lanes x 16 bytes each)
  size_t a_band[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) a_band[j] = (size_t)min(mt0 + j, m_tiles - 1) * KT * 128;

#pragma unroll 4
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    u32x4 wf[NT], ah[MT], al[MT];
#pragma unroll
    for (int i = 0; i < NT; ++i) wf[i] = __builtin_nontemporal_load(Wp + ((size_t)(nt0 + i) * KT + kt) * 64);
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      ah[j] = Ap[a_band[j] + (size_t)kt * 128];
      al[j] = Ap[a_band[j] + (size_t)kt * 128 + 64];
    }
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]),
                                                            __builtin_bit_cast(bf16x8, ah[j]), acc[i][j], 0, 0, 0);
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]),
                                                            __builtin_bit_cast(bf16x8, al[j]), acc[i][j], 0, 0, 0);
      }
  }

  __shared__ float4 red[4][NT * MT][64];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j)
      red[wave][i * MT + j][lane] = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
  __syncthreads();

  const int mrow = lane & 15, g = lane >> 4;
  if (EPI == EPI_SWIGLU) {
    bf16_t* act = reinterpret_cast<bf16_t*>(ep.act);
    for (int t = wave; t < (NT / 2) * MT; t += 4) {
      const int p = t / MT, j = t % MT;
      float4 gs = red[0][(2 * p) * MT + j][lane], us = red[0][(2 * p + 1) * MT + j][lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        float4 a = red[w][(2 * p) * MT + j][lane], b = red[w][(2 * p + 1) * MT + j][lane];
        gs.x += a.x; gs.y += a.y; gs.z += a.z; gs.w += a.w;
        us.x += b.x; us.y += b.y; us.z += b.z; us.w += b.w;
      }
      const int m = (mt0 + j) * 16 + mrow;
      if (mt0 + j < m_tiles && m < M) {
        const int col = ((nt0 + 2 * p) >> 1) * 16 + 4 * g;
        Act<bf16_t>::store4(act, m, col, ep.act_K,
                            make_float4(silu_f(gs.x) * us.x, silu_f(gs.y) * us.y, silu_f(gs.z) * us.z, silu_f(gs.w) * us.w));
      }
    }
  } else {
    for (int t = wave; t < NT * MT; t += 4) {
      const int i = t / MT, j = t % MT;
      float4 s = red[0][t][lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        float4 a = red[w][t][lane];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
      }
      const int m = (mt0 + j) * 16 + mrow;
      if (mt0 + j < m_tiles && m < M) {
        float4* dst = reinterpret_cast<float4*>(ep.out + (size_t)m * ep.ld + (nt0 + i) * 16 + 4 * g);
        if (EPI == EPI_RESID) {
          float4 h = *dst;
          s.x += h.x; s.y += h.y; s.z += h.z; s.w += h.w;
        }
        *dst = s;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// fp32 kernel: block = 4 wavefronts, one output column (SWIGLU: one activation column = a gate row
// and the up row 16 below it) per wavefront; lanes stride over K; rows in chunks of 8.
// ------------------------------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ W, const float* __restrict__ A, int M,
                                                       int N, int K, EpiArgs ep) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.x * 4 + wave;
  const int n_cols = (EPI == EPI_SWIGLU) ? N / 2 : N;
  if (col >= n_cols) return;
  const int row0 = (EPI == EPI_SWIGLU) ? (col >> 4) * 32 + (col & 15) : col;
  const float* w0 = W + (size_t)row0 * K;
  const float* w1 = w0 + (size_t)16 * K;  // SWIGLU only
  for (int m0 = 0; m0 < M; m0 += 8) {
    float acc0[8], acc1[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) acc0[r] = acc1[r] = 0.f;
    for (int k = lane * 4; k < K; k += 256) {
      const float4 wa = *reinterpret_cast<const float4*>(w0 + k);
      float4 wb = make_float4(0.f, 0.f, 0.f, 0.f);
      if (EPI == EPI_SWIGLU) wb = *reinterpret_cast<const float4*>(w1 + k);
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        if (m0 + r < M) {
          const float4 a = *reinterpret_cast<const float4*>(A + (size_t)(m0 + r) * K + k);
          acc0[r] += a.x * wa.x + a.y * wa.y + a.z * wa.z + a.w * wa.w;
          if (EPI == EPI_SWIGLU) acc1[r] += a.x * wb.x + a.y * wb.y + a.z * wb.z + a.w * wb.w;
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const float s0 = wave_reduce_sum(acc0[r]);
      const float s1 = (EPI == EPI_SWIGLU) ? wave_reduce_sum(acc1[r]) : 0.f;
      const int m = m0 + r;
      if (lane == 0 && m < M) {
        if (EPI == EPI_SWIGLU) {
          reinterpret_cast<float*>(ep.act)[(size_t)m * ep.act_K + col] = silu_f(s0) * s1;
        } else if (EPI == EPI_RESID) {
          ep.out[(size_t)m * ep.ld + col] += s0;
        } else {
          ep.out[(size_t)m * ep.ld + col] = s0;
        }
      }
    }
  }
}
