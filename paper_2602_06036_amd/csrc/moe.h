// Routed-expert FFN of a mixture-of-experts target (the Qwen3-Coder-30B-A3B target of Section 5): routing.  The expert
// GEMMs themselves are grouped launches of the weight-streaming kernel (gemm.h); the weighted sum of a row's experts'
// outputs is taken by the RMSNorm kernel that follows (misc.h).
//
// Routing rule (that model family's; the paper does not restate it): a token goes to the top_k experts by router
// logit (ties -> lowest index) with weights softmax(chosen logits); y_t = sum_j w_tj FFN_{e_tj}(a_t).
#pragma once
#include "common.h"

constexpr int MOE_MAX_EXPERTS = 256;
constexpr int MOE_MAX_TOPK = 16;

constexpr int MOE_MASK_WORDS = 8192;    // LDS words of the (expert x row) bitmap: n_experts * ceil(rows / 32) must fit
constexpr int MOE_FUSED_ROWS = 64;      // up to this many rows the routing kernel also picks the experts itself

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
  unsigned long long* counters;   // [5] running totals: routing launches, experts reached, 16-row bands, work items; [4] = bands per work item of the last launch (statistics)
  int32_t* n_bands_out;           // [1] bands of the list this launch built
};

// One wavefront picks row t's experts: lane j < k ends up with the j-th best (expert, weight); returns the expert.
__device__ __forceinline__ int moe_topk_row(const MoeRoute& a, int t, int lane, float& weight) {
  float v[4] = {0.f, 0.f, 0.f, 0.f};   // lane holds experts lane, lane + 64, ...
  for (int z0 = 0; z0 < a.ks; z0 += 4) {   // four slabs' loads in flight at a time, added in ascending order
    float part[4][4];
#pragma unroll
    for (int zz = 0; zz < 4; ++zz)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        part[zz][i] = (e < a.E && z0 + zz < a.ks) ? a.logits[(size_t)(z0 + zz) * a.stride + (size_t)t * a.E + e] : 0.f;
      }
#pragma unroll
    for (int zz = 0; zz < 4; ++zz)
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] += part[zz][i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float x = v[i];
    // a real expert always beats the padding, whatever the logit
    v[i] = lane + 64 * i < a.E ? (x == x ? fmaxf(x, -3.0e38f) : -3.0e38f) : -INFINITY;
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
  weight = ex / sum;
  return mine_e;
}

// Expert choice for many rows: one wavefront per row, four rows per workgroup.
__global__ __launch_bounds__(256) void moe_topk_kernel(MoeRoute a) {
  const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= a.M) return;
  float w;
  const int e = moe_topk_row(a, t, lane, w);
  if (lane < a.k) {
    a.sel_e[(size_t)t * a.k + lane] = e;
    a.sel_w[(size_t)t * a.k + lane] = w;
  }
}

// Builds the expert-sorted row list: one workgroup.  A bitmap (expert x row) in LDS records who goes where; an entry's
// place inside its expert's 16-row-padded range is the number of lower rows with the same expert (a popcount over the
// bitmap), so the list -- and everything downstream -- is the same in every run.  FUSED: also picks the experts
// (few rows; saves a launch), else reads the choices moe_topk_kernel left.
template <bool FUSED>
__global__ __launch_bounds__(1024) void moe_route_kernel(MoeRoute a) {
  __shared__ uint32_t mask[MOE_MASK_WORDS];
  __shared__ uint16_t before[MOE_MASK_WORDS];   // rows of the same expert in lower words
  __shared__ int tot[MOE_MAX_EXPERTS], base[MOE_MAX_EXPERTS], item0[MOE_MAX_EXPERTS];
  __shared__ int sel_l[FUSED ? MOE_FUSED_ROWS * MOE_MAX_TOPK : 1];
  __shared__ int n_items, n_bands, n_used;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int W = (a.M + 31) >> 5, n_entries = a.M * a.k;
  for (int i = tid; i < a.E * W; i += 1024) mask[i] = 0u;
  __syncthreads();
  if constexpr (FUSED) {
    for (int t = wave; t < a.M; t += 16) {
      float w;
      const int e = moe_topk_row(a, t, lane, w);
      if (lane < a.k) {
        a.sel_e[(size_t)t * a.k + lane] = e;
        a.sel_w[(size_t)t * a.k + lane] = w;
        sel_l[t * a.k + lane] = e;
        atomicOr(&mask[e * W + (t >> 5)], 1u << (t & 31));
      }
    }
  } else {
    for (int i = tid; i < n_entries; i += 1024) {
      const int t = i / a.k, e = min(max(a.sel_e[i], 0), a.E - 1);
      atomicOr(&mask[e * W + (t >> 5)], 1u << (t & 31));
    }
  }
  __syncthreads();
  if (tid < a.E) {
    int s = 0;
    for (int w = 0; w < W; ++w) {
      before[tid * W + w] = (uint16_t)s;
      s += __popc(mask[tid * W + w]);
    }
    tot[tid] = s;
  }
  __syncthreads();
  if (wave == 0) {   // exclusive scans over the experts (bands, work items): lane owns experts 4*lane .. 4*lane+3
    int nb[4], ni[4], sb = 0, si = 0, su = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = 4 * lane + i;
      nb[i] = e < a.E ? (tot[e] + 15) >> 4 : 0;
      ni[i] = (nb[i] + a.MT - 1) / a.MT;
      sb += nb[i]; si += ni[i]; su += nb[i] > 0;
    }
    int ib = sb, ii = si;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int ob = __shfl_up(ib, o, 64), oi = __shfl_up(ii, o, 64);
      if (lane >= o) { ib += ob; ii += oi; }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) su += __shfl_xor(su, o, 64);
    int eb = ib - sb, ei = ii - si;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = 4 * lane + i;
      if (e < a.E) { base[e] = eb * 16; item0[e] = ei; }
      eb += nb[i]; ei += ni[i];
    }
    if (lane == 63) { n_items = ii; n_bands = ib; n_used = su; }
  }
  __syncthreads();
  if (tid < a.E && tot[tid] > 0) {
    const int b0 = base[tid] >> 4, nb = (tot[tid] + 15) >> 4;
    for (int q = 0; q * a.MT < nb; ++q)
      if (item0[tid] + q < a.max_items) a.items[item0[tid] + q] = make_int4(tid, b0 + q * a.MT, min(b0 + (q + 1) * a.MT, b0 + nb), 0);
    for (int p = base[tid] + tot[tid]; p < base[tid] + nb * 16; ++p) a.row_of[p] = -1;
  }
  for (int i = n_items + tid; i < a.max_items; i += 1024) a.items[i] = make_int4(-1, 0, 0, 0);
  for (int i = tid; i < n_entries; i += 1024) {
    const int t = i / a.k;
    int e;
    if constexpr (FUSED) e = sel_l[i];
    else e = min(max(a.sel_e[i], 0), a.E - 1);
    const int pos = base[e] + before[e * W + (t >> 5)] + __popc(mask[e * W + (t >> 5)] & ((1u << (t & 31)) - 1u));
    a.sel_pos[i] = pos;
    a.row_of[pos] = t;
  }
  if (tid == 0) {
    a.n_bands_out[0] = n_bands;
    a.counters[0] += 1ull;
    a.counters[1] += (unsigned long long)n_used;
    a.counters[2] += (unsigned long long)n_bands;
    a.counters[3] += (unsigned long long)n_items;
    a.counters[4] = (unsigned long long)a.MT;   // not a total: the bands per work item of this launch
  }
}

// Copies the listed rows of a GEMM operand (hi+lo bf16 tiles, layout of common.h) into list order, so that the grouped
// GEMM reads whole 1 KB fragments instead of sixteen-byte pieces of sixteen different rows.  One wavefront per
// (band, k tile), both planes; padding rows become zeros.  grid = (ceil(KT / 4), bands bound).
__global__ __launch_bounds__(256) void moe_gather_kernel(const u32x4* __restrict__ src, const int32_t* __restrict__ row_of,
                                                         const int32_t* __restrict__ n_bands, int KT, u32x4* __restrict__ dst) {
  const int band = blockIdx.y, kt = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (band >= n_bands[0] || kt >= KT) return;
  const int t = row_of[band * 16 + (lane & 15)];
  u32x4 hi = {0u, 0u, 0u, 0u}, lo = {0u, 0u, 0u, 0u};
  if (t >= 0) {
    const u32x4* p = src + ((size_t)(t >> 4) * KT + kt) * 128 + (lane >> 4) * 16 + (t & 15);
    hi = p[0];
    lo = p[64];
  }
  u32x4* q = dst + ((size_t)band * KT + kt) * 128 + lane;
  q[0] = hi;
  q[64] = lo;
}
