// Weight-streaming GEMMs: y[M,N] = a[M,K] * W[N,K]^T with fused epilogues.
//   bf16: MFMA 16x16x32, weights in the tiled layout of common.h, activations as hi+lo bf16 pairs
//         (two MFMAs per weight tile), fp32 accumulation.
//   fp32: one wavefront per output column (tiny models only).
#pragma once
#include <type_traits>

#include "common.h"

enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

struct EpiArgs {
  float* out;   // STORE: out[z*slab + m*ld + n] = partial y of K range z ; RESID (fp32 kernel): out[m*ld + n] += y
  int ld;
  size_t slab;  // elements between the partial results of consecutive K ranges (grid.z)
  void* act;    // SWIGLU: act (GEMM activation operand, row length act_K) [m, j] = silu(gate_j) * up_j
  int act_K;
  // STORE with a single K range, LM head only: fused row argmax.  Every workgroup also writes the best
  // (score, column) of its columns for each of its rows to amax[m * gridDim.x-many parts + part]; score = y
  // (mode 0) or y * inv_T + Gumbel(key, m / B, m % B, purpose 0, column) (mode 1).  out may then be null
  // (logits not wanted).  A second, tiny kernel combines the parts (ties -> lowest column).
  float2* amax = nullptr;
  int amax_mode = 0;
  float amax_inv_T = 1.f;
  const uint64_t* amax_key = nullptr;
  int amax_B = 1;
  // STORE with a single K range, LM head only: fused softmax statistics.  Every workgroup also writes, for each of its
  // rows, (max, sum of exp(y * lse_inv_T - max)) over its columns to lse[m * parts + part] (same partition as amax); a
  // second, tiny kernel combines the parts in ascending order into (max, log-sum-exp).
  float2* lse = nullptr;
  float lse_inv_T = 1.f;
  // grouped launch (routed experts): a 1-D grid over (work item, column block); grp_items[item] = (expert, first band,
  // end band, -) replaces the fixed band range; the workgroup multiplies those bands by the expert's matrix W + expert * grp_w_stride
  // (elements), an item with expert < 0 has nothing to do.  grp_rows (nullable) [bands * 16]: the activation row
  // behind each row of a band (the operand is then read through this list; < 0 = padding, any row will do).
  const int4* grp_items = nullptr;
  int grp_n_items = 0;
  size_t grp_w_stride = 0;
  const int32_t* grp_rows = nullptr;
  // Deferred RMSNorm (streaming kernel only): the operand holds x * gain without the division by the row's rms; row m
  // of the result is multiplied by 1 / sqrt(sum_p ssq[m * ssq_parts + p] * ssq_inv_D + ssq_eps) before any epilogue
  // sees it (the sums of squares come in ssq_parts pieces, added in ascending order; see gemm_resid.h).
  const float* ssq = nullptr;
  int ssq_parts = 0;
  float ssq_inv_D = 0.f, ssq_eps = 0.f;
};

// score of logit y at (row m, column col) for the fused argmax
__device__ __forceinline__ float amax_score(const EpiArgs& ep, uint64_t key, float y, int m, int col) {
  return ep.amax_mode ? y * ep.amax_inv_T + gumbel(counter_uniform(key, m / ep.amax_B, m % ep.amax_B, 0, (uint32_t)col)) : y;
}

// Split of K across workgroups (grid.z ranges): the STORE epilogue writes one partial slab per range and
// the kernel that consumes the result (RMSNorm, q/k-norm + RoPE) adds the slabs in ascending order.
// The kernel boundary provides the ordering: no atomics, no fences, and a sum that does not depend on
// which workgroup finished first.

// (max, sum of exponentials relative to that max) of the union of two sets; an empty set is (-inf, 0)
__device__ __forceinline__ void lse_combine(float& m, float& s, float m2, float s2) {
  const float M = fmaxf(m, m2);
  s = (m == -INFINITY ? 0.f : s * __expf(m - M)) + (m2 == -INFINITY ? 0.f : s2 * __expf(m2 - M));
  m = M;
}
// the same over the 4 lanes that hold the other columns of a row (lane bits 4 and 5)
__device__ __forceinline__ void lse_combine_row(float& m, float& s) {
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
    const float om = __shfl_xor(m, o, 64), os = __shfl_xor(s, o, 64);
    lse_combine(m, s, om, os);
  }
}
__device__ __forceinline__ void lse_add4(float& m, float& s, float4 y, float inv_T) {
  const float a = y.x * inv_T, b = y.y * inv_T, c = y.z * inv_T, d = y.w * inv_T;
  const float mx = fmaxf(fmaxf(a, b), fmaxf(c, d));
  lse_combine(m, s, mx, __expf(a - mx) + __expf(b - mx) + __expf(c - mx) + __expf(d - mx));
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel.  A workgroup of 4 wavefronts owns NT 16-row bands of W (N tiles) and MT 16-row
// bands of the activations for one K range (grid.z ranges); each wavefront streams a quarter of that
// range, U k-tiles at a time with the next U already in flight, every activation fragment reused for
// the NT weight tiles.  The four partial sums are added in a fixed order through LDS.  The MFMA
// computes D^T = W_tile * a_tile^T: lane l ends up holding y[m = l%16][n = 4*(l/16) .. +3].
// SWIGLU: W rows alternate 16 gate rows / 16 up rows, so tiles (2p, 2p+1) of a workgroup are the
// gate and up values of the same 16 activation columns.
// ------------------------------------------------------------------------------------------------
template <int NT, int MT, int U>
struct GemmBuf {
  u32x4 w[U][NT], ah[U][MT], al[U][MT];
};

template <int NT, int MT, int U, int EPI, bool GRP = false, int PH = 1, int NW = 4>
__global__ __launch_bounds__(64 * NW, (NW > 4 ? 1 : PH)) void gemm_bf16_kernel(const bf16_t* __restrict__ W, const bf16_t* __restrict__ A,
                                                        int M, int N, int K, EpiArgs ep) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kz = blockIdx.z;
  const int KT = K >> 5, n_tiles = N >> 4;
  int nt0 = blockIdx.x * NT;
  int mt0 = blockIdx.y * MT, m_tiles = (M + 15) >> 4;   // bands mt0 .. min(mt0 + MT, m_tiles) - 1 are this workgroup's
  if constexpr (GRP) {
    // 1-D grid; consecutive workgroup ids go to different XCDs (round-robin dispatch), so id = 8*j + x is work item
    // 8*(j / columns) + x, column block j % columns: the workgroups that share an item's activation rows run back to
    // back on one XCD and fetch them into one L2 instead of eight
    const int cols = n_tiles / NT, x = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int it = (j / cols) * 8 + x;
    if (it >= ep.grp_n_items) return;
    const int4 item = ep.grp_items[it];
    if (item.x < 0) return;
    W += (size_t)item.x * ep.grp_w_stride;
    nt0 = (j % cols) * NT;
    mt0 = item.y;
    m_tiles = item.z;
  }
  const int ks = gridDim.z;
  const int per = (KT + ks * NW - 1) / (ks * NW);
  const int kb = min(KT, (kz * NW + wave) * per);
  const int ke = min(KT, kb + per);

  f32x4 acc[NT][MT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const u32x4* Wp = reinterpret_cast<const u32x4*>(W) + lane;
  const u32x4* Ap = reinterpret_cast<const u32x4*>(A) + (GRP && ep.grp_rows ? 0 : lane);   // row lists carry the lane's offset
  // activation bands past the last one alias the last band (their results are never stored);
  // a band holds, per k tile, the hi tile then the lo tile (64 lanes x 16 bytes each)
  size_t a_band[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    const int band = min(mt0 + j, m_tiles - 1);
    a_band[j] = (size_t)band * KT * 128;
    if constexpr (GRP) {
      if (ep.grp_rows) {   // lane (row r = lane % 16, k chunk lane / 16) of the fragment reads row grp_rows[16 * band + r]
        const int t = max(ep.grp_rows[band * 16 + (lane & 15)], 0);
        a_band[j] = (size_t)(t >> 4) * KT * 128 + (size_t)((lane >> 4) * 16 + (t & 15));
      }
    }
  }

  auto load = [&](GemmBuf<NT, MT, U>& b, int k0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = k0 + u < ke;
      const int kt = in ? k0 + u : ke - 1;   // past the range: re-read the last tile, with zeroed activations
#pragma unroll
      for (int i = 0; i < NT; ++i) b.w[u][i] = __builtin_nontemporal_load(Wp + ((size_t)kt * n_tiles + nt0 + i) * 64);
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const u32x4 h = Ap[a_band[j] + (size_t)kt * 128], l = Ap[a_band[j] + (size_t)kt * 128 + 64];
        b.ah[u][j] = in ? h : (u32x4){0u, 0u, 0u, 0u};
        b.al[u][j] = in ? l : (u32x4){0u, 0u, 0u, 0u};
      }
    }
  };
  // all hi products of a k tile, then all lo products: two MFMAs on the same accumulator are never back to back (the
  // second would wait out the first one's passes)
  auto compute = [&](const GemmBuf<NT, MT, U>& b) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b.w[u][i]),
                                                              __builtin_bit_cast(bf16x8, b.ah[u][j]), acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b.w[u][i]),
                                                              __builtin_bit_cast(bf16x8, b.al[u][j]), acc[i][j], 0, 0, 0);
    }
  };

  // Deferred RMSNorm: 1 / rms of this workgroup's rows, 16 threads per row, each adding every 16th piece in
  // ascending order, then the 16 partial sums by a fixed shuffle tree.  Written to LDS here, read after the
  // barrier of the cross-wavefront sum.
  __shared__ float s_rstd[MT * 16];
  if (ep.ssq && threadIdx.x < 256) {
    const int r = threadIdx.x >> 4, c = threadIdx.x & 15;
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      const int m = min((mt0 + j) * 16 + r, M - 1);
      const float* pp = ep.ssq + (size_t)m * ep.ssq_parts;
      float t = 0.f;
      if ((ep.ssq_parts & 3) == 0 && ep.ssq_parts <= 512) {
        // all requests of the thread go out together (up to 8 pieces of 4 values, 64 values apart)
        float4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int p = (c + 16 * i) * 4;
          v[i] = p < ep.ssq_parts ? *reinterpret_cast<const float4*>(pp + p) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) t += (v[i].x + v[i].y) + (v[i].z + v[i].w);
      } else {
        for (int p = c; p < ep.ssq_parts; p += 16) t += pp[p];
      }
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) t += __shfl_xor(t, o, 64);
      if (c == 0) s_rstd[j * 16 + r] = 1.0f / sqrtf(t * ep.ssq_inv_D + ep.ssq_eps);
    }
  }

  // Two register buffers, one being multiplied while the other is on its way.  No load inside the loop is
  // conditional: a load that is skipped on some path would make the number of loads in flight unknown at compile
  // time, and the wait for the older buffer would then have to drain the newer one as well.  The last one or two
  // stages are peeled off; if the range has an odd number of stages the final load re-reads the last tile
  // (still in cache) and meets zeroed activations.
  if constexpr (PH == 2 && NW == 4) {
    // one buffer only (and the cross-wavefront sum below in two halves): half the registers and half the LDS, so that
    // two workgroups share a CU and their wavefronts cover each other's waits
    GemmBuf<NT, MT, U> b;
    for (int k0 = kb; k0 < ke; k0 += U) {
      load(b, k0);
      compute(b);
    }
  } else if (kb < ke) {
    GemmBuf<NT, MT, U> b0, b1;
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

  // The four wavefronts' partial sums meet in LDS, PH phases of NT / PH weight tiles each (PH = 2 halves the buffer).
  constexpr int HT = NT / PH;
  static_assert(NT % PH == 0 && (EPI != EPI_SWIGLU || HT % 2 == 0), "phases");
  __shared__ float4 red[NW][HT * MT][64];
  const int mrow = lane & 15, g = lane >> 4;
  // the four wavefronts' partial sums of tile t (= weight tile * MT + band) of the current phase, in wavefront order,
  // times the row's deferred 1 / rms
  auto tile_sum = [&](int t) {
    float4 s = red[0][t][lane];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
      const float4 a = red[w][t][lane];
      s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
    if (ep.ssq) {
      const float rs = s_rstd[(t % MT) * 16 + mrow];
      s.x *= rs; s.y *= rs; s.z *= rs; s.w *= rs;
    }
    return s;
  };
  auto phase = [&](auto phc) {
    constexpr int ph = decltype(phc)::value;
    if (ph) __syncthreads();   // everybody is done reading the previous phase
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j)
        red[wave][i * MT + j][lane] = make_float4(acc[ph * HT + i][j][0], acc[ph * HT + i][j][1], acc[ph * HT + i][j][2], acc[ph * HT + i][j][3]);
    __syncthreads();
    if (EPI == EPI_SWIGLU) {
      bf16_t* act = reinterpret_cast<bf16_t*>(ep.act);
      for (int t = wave; t < (HT / 2) * MT; t += NW) {
        const int p = t / MT, j = t % MT;
        const float4 gs = tile_sum((2 * p) * MT + j), us = tile_sum((2 * p + 1) * MT + j);
        const int m = (mt0 + j) * 16 + mrow;
        if (mt0 + j < m_tiles && m < M) {
          const int col = ((nt0 + ph * HT + 2 * p) >> 1) * 16 + 4 * g;
          Act<bf16_t>::store4(act, m, col, ep.act_K,
                              make_float4(silu_f(gs.x) * us.x, silu_f(gs.y) * us.y, silu_f(gs.z) * us.z, silu_f(gs.w) * us.w));
        }
      }
    } else if (ep.out) {
      for (int t = wave; t < HT * MT; t += NW) {
        const int i = t / MT, j = t % MT;
        const float4 s = tile_sum(t);
        const int m = (mt0 + j) * 16 + mrow;
        if (mt0 + j < m_tiles && m < M) {
          float4* dst = reinterpret_cast<float4*>(ep.out + (size_t)kz * ep.slab + (size_t)m * ep.ld + (nt0 + ph * HT + i) * 16 + 4 * g);
          *dst = s;
        }
      }
    }
  };
  phase(std::integral_constant<int, 0>{});
  if constexpr (PH >= 2) phase(std::integral_constant<int, 1>{});
  if constexpr (PH >= 3) phase(std::integral_constant<int, 2>{});
  static_assert(PH <= 3, "phases");

  if constexpr (EPI != EPI_SWIGLU && PH == 1) {
    if (ep.amax) {   // fused argmax over this workgroup's NT*16 columns (host guarantees a single K range)
      __shared__ float2 wbest[NW][MT * 16];
      const uint64_t key = ep.amax_mode ? ep.amax_key[0] : 0ull;
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const int m = (mt0 + j) * 16 + mrow;
        float bv = -INFINITY;
        int bi = 0x7FFFFFFF;
        for (int i = wave; i < NT; i += NW) {
          const float4 s = tile_sum(i * MT + j);
          const int col = (nt0 + i) * 16 + 4 * g;
          argmax_combine(bv, bi, amax_score(ep, key, s.x, m, col), col);
          argmax_combine(bv, bi, amax_score(ep, key, s.y, m, col + 1), col + 1);
          argmax_combine(bv, bi, amax_score(ep, key, s.z, m, col + 2), col + 2);
          argmax_combine(bv, bi, amax_score(ep, key, s.w, m, col + 3), col + 3);
        }
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
          const float ov = __shfl_xor(bv, o, 64);
          const int oi = __shfl_xor(bi, o, 64);
          argmax_combine(bv, bi, ov, oi);
        }
        if (g == 0) wbest[wave][j * 16 + mrow] = make_float2(bv, __int_as_float(bi));
      }
      __syncthreads();
      for (int r = threadIdx.x; r < MT * 16; r += 64 * NW) {
        const int m = mt0 * 16 + r;
        if (m >= M) continue;
        float bv = wbest[0][r].x;
        int bi = __float_as_int(wbest[0][r].y);
#pragma unroll
        for (int w = 1; w < NW; ++w) argmax_combine(bv, bi, wbest[w][r].x, __float_as_int(wbest[w][r].y));
        ep.amax[(size_t)m * gridDim.x + blockIdx.x] = make_float2(bv, __int_as_float(bi));
      }
    }
    if (ep.lse) {   // fused softmax statistics over this workgroup's NT*16 columns (single K range)
      __shared__ float2 wl[NW][MT * 16];
      __syncthreads();
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        float lm = -INFINITY, ls = 0.f;
        for (int i = wave; i < NT; i += NW) lse_add4(lm, ls, tile_sum(i * MT + j), ep.lse_inv_T);
        lse_combine_row(lm, ls);
        if (g == 0) wl[wave][j * 16 + mrow] = make_float2(lm, ls);
      }
      __syncthreads();
      for (int r = threadIdx.x; r < MT * 16; r += 64 * NW) {
        const int m = mt0 * 16 + r;
        if (m >= M) continue;
        float lm = wl[0][r].x, ls = wl[0][r].y;
#pragma unroll
        for (int w = 1; w < NW; ++w) lse_combine(lm, ls, wl[w][r].x, wl[w][r].y);
        ep.lse[(size_t)m * gridDim.x + blockIdx.x] = make_float2(lm, ls);
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
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
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
