// Routed-expert FFN of a mixture-of-experts target (the Qwen3-Coder-30B-A3B target of Section 5): routing and the
// weighted combination.  The expert GEMMs themselves are grouped launches of the weight-streaming kernel (gemm.h).
//
// Routing rule (that model family's; the paper does not restate it): a token goes to the top_k experts by router
// logit (ties -> lowest index) with weights softmax(chosen logits); y_t = sum_j w_tj FFN_{e_tj}(a_t).
#pragma once
#include "common.h"

constexpr int MOE_MAX_EXPERTS = 256;
constexpr int MOE_MAX_TOPK = 16;

struct MoeRoute {
  const float* logits;   // router logits as K-range slabs: logits[z * stride + t * E + e], z < ks
  int ks;
  size_t stride;
  int M, E, k;
  int MT;                // bands per work item of the grouped GEMMs
  int32_t* sel_e;        // [M * k] chosen experts of row t, by decreasing logit
  float* sel_w;          // [M * k] their weights
  int32_t* sel_pos;      // [M * k] row of the expert-sorted list that holds (t, j)
  int32_t* row_of;       // [n_pos_max] expert-sorted list: token row behind each position, -1 = padding
  int4* items;           // [max_items] (expert, first band, end band, 0), expert = -1: unused
  int max_items;
};

// One workgroup of 16 wavefronts.  Wavefront w owns a contiguous range of token rows; it picks their experts and counts
// them per expert (its own counters: the experts of one row are distinct and its rows come one after the other, so
// plain increments do).  The counts become, per expert, a 16-row-padded range of the sorted list with the wavefronts'
// shares in row order inside it, so that the list -- and everything downstream -- is the same in every run.
__global__ __launch_bounds__(1024) void moe_route_kernel(MoeRoute a) {
  __shared__ int cnt[16][MOE_MAX_EXPERTS];
  __shared__ int tot[MOE_MAX_EXPERTS], base[MOE_MAX_EXPERTS], item0[MOE_MAX_EXPERTS];
  __shared__ int n_items;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 16 * MOE_MAX_EXPERTS; i += 1024) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const int chunk = (a.M + 15) / 16, r0 = min(a.M, wave * chunk), r1 = min(a.M, r0 + chunk);
  for (int t = r0; t < r1; ++t) {
    float v[4];   // lane holds experts lane, lane + 64, ...
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      float x = -INFINITY;
      if (e < a.E) {
        x = 0.f;
        for (int z = 0; z < a.ks; ++z) x += a.logits[(size_t)z * a.stride + (size_t)t * a.E + e];
        x = x == x ? fmaxf(x, -3.0e38f) : -3.0e38f;   // a real expert always beats the padding, whatever the logit
      }
      v[i] = x;
    }
    float mine = 0.f, top = 0.f;
    int mine_e = 0;
    for (int j = 0; j < a.k; ++j) {
      float bv = v[0];
      int bi = lane;
#pragma unroll
      for (int i = 1; i < 4; ++i)
        if (v[i] > bv) { bv = v[i]; bi = lane + 64 * i; }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      if (j == 0) top = bv;
      if (lane == j) { mine = bv; mine_e = bi; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (bi == lane + 64 * i) v[i] = -INFINITY;
    }
    float ex = lane < a.k ? __expf(mine - top) : 0.f, sum = ex;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (lane < a.k) {
      a.sel_e[(size_t)t * a.k + lane] = mine_e;
      a.sel_w[(size_t)t * a.k + lane] = ex / sum;
      cnt[wave][mine_e] += 1;
    }
  }
  __syncthreads();
  if (tid < a.E) {   // per expert: total, and each wavefront's offset inside the expert's range
    int s = 0;
    for (int w = 0; w < 16; ++w) {
      const int n = cnt[w][tid];
      cnt[w][tid] = s;
      s += n;
    }
    tot[tid] = s;
  }
  __syncthreads();
  if (tid == 0) {
    int p = 0, it = 0;
    for (int e = 0; e < a.E; ++e) {
      base[e] = p;
      item0[e] = it;
      const int nb = (tot[e] + 15) >> 4;
      p += nb * 16;
      it += (nb + a.MT - 1) / a.MT;
    }
    n_items = it;
  }
  __syncthreads();
  if (tid < a.E && tot[tid] > 0) {
    const int b0 = base[tid] >> 4, nb = (tot[tid] + 15) >> 4;
    for (int q = 0; q * a.MT < nb; ++q)
      if (item0[tid] + q < a.max_items) a.items[item0[tid] + q] = make_int4(tid, b0 + q * a.MT, min(b0 + (q + 1) * a.MT, b0 + nb), 0);
    for (int p = base[tid] + tot[tid]; p < base[tid] + nb * 16; ++p) a.row_of[p] = -1;
  }
  for (int i = n_items + tid; i < a.max_items; i += 1024) a.items[i] = make_int4(-1, 0, 0, 0);
  for (int t = r0; t < r1; ++t) {
    if (lane < a.k) {
      const int e = a.sel_e[(size_t)t * a.k + lane];   // written by this very lane above
      const int pos = base[e] + cnt[wave][e];
      cnt[wave][e] += 1;
      a.sel_pos[(size_t)t * a.k + lane] = pos;
      a.row_of[pos] = t;
    }
  }
}

// out[t, :] = sum_j w[t, j] * y[pos[t, j], :], j ascending (decreasing router logit)
__global__ __launch_bounds__(256) void moe_combine_kernel(const float* __restrict__ y, const int32_t* __restrict__ pos,
                                                          const float* __restrict__ w, int k, int D, float* __restrict__ out) {
  const int t = blockIdx.x;
  for (int d4 = threadIdx.x; d4 < D / 4; d4 += 256) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
      const float wj = w[(size_t)t * k + j];
      const float4 v = reinterpret_cast<const float4*>(y + (size_t)pos[(size_t)t * k + j] * D)[d4];
      acc.x += wj * v.x; acc.y += wj * v.y; acc.z += wj * v.z; acc.w += wj * v.w;
    }
    reinterpret_cast<float4*>(out + (size_t)t * D)[d4] = acc;
  }
}
