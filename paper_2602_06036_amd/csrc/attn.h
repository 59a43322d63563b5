// Block attention over the paged cache, split along the context ("split-KV") with a deterministic
// log-sum-exp merge.  Used for both halves of the step:
//   verify (Section 3.1): causal -- block row j sees positions 0 .. n_s + j
//   draft  (Section 4.2, Appendix A.3): no mask -- every block row sees the n_s context-feature rows
//                                       and all B block rows (positions 0 .. n_s + B - 1)
// In both cases the block's own K/V rows have already been written to the pool at n_s .. n_s+B-1.
#pragma once
#include "common.h"

struct AttnArgs {
  int n_q_heads, n_kv_heads, head_dim;
  int layer;     // layer inside the pool
  int causal;
  int chunk;     // context tokens per split (multiple of 64)
  int n_splits;
  float scale;   // 1/sqrt(head_dim)
  int q_shift = 0;   // MFMA kernels: the query heads of one kv head are shared out over 2^q_shift workgroups (a workgroup
                     // holds at most 64 query rows = block_size * heads; 8 heads per kv head at block size 16 need two)
};

// partial results: for pr = (m*Hq + hq)*n_splits + split : ml[pr] = (running max, sum exp), o[pr*hd + d]
// (o unnormalised, relative to the running max)

// ------------------------------------------------------------------------------------------------
// Generic kernel (any storage type; plain ALU math).  grid (n_splits, Hkv, S), block 256.
// A wavefront takes query rows r = wave, wave+4, ... of the B*group rows that share this kv head.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_partial_simple_kernel(const T* __restrict__ q, const T* __restrict__ pool,
                                                                  SeqGeom geo, AttnArgs aa, float* __restrict__ part_o,
                                                                  float2* __restrict__ part_ml) {
  const int split = blockIdx.x, kvh = blockIdx.y, s = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hd = aa.head_dim, B = geo.block_size;
  const int group = aa.n_q_heads / aa.n_kv_heads;
  const int rows = B * group;
  const int n_s = geo.seq_lens[s];
  const int cap = geo.max_pages_per_seq * DF_PAGE;
  const int n_tok = min(n_s + B, cap);
  const int c0 = split * aa.chunk;
  const int c1 = min(n_tok, c0 + aa.chunk);
  __shared__ float qs[4][128];
  const int32_t* table = geo.block_table + (size_t)s * geo.max_pages_per_seq;

  for (int r = wave; r < rows; r += 4) {
    const int slot = r / group, hq = kvh * group + r % group;
    const int m = s * B + slot;
    const size_t pr = ((size_t)m * aa.n_q_heads + hq) * aa.n_splits + split;
    const T* qrow = q + ((size_t)m * aa.n_q_heads + hq) * hd;
    for (int d = lane; d < hd; d += 64) qs[wave][d] = Store<T>::to(qrow[d]);
    // (same wavefront writes and reads qs[wave]; LDS ops of one wavefront complete in order)
    const int last_vis = aa.causal ? min(n_s + slot, n_tok - 1) : n_tok - 1;
    float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;
    for (int t0 = c0; t0 < c1; t0 += 64) {
      const int pos = t0 + lane;
      const bool vis = pos < c1 && pos <= last_vis;
      int page = -1;
      if (vis) page = table[pos / DF_PAGE];
      const bool ok = vis && page >= 0 && page < geo.n_pages;
      float sc = -INFINITY;
      if (ok) {
        const T* kb = pool + kv_head_base(aa.layer, geo.n_pages, page, aa.n_kv_heads, kvh, hd);
        const int key = pos % DF_PAGE;
        float acc = 0.f;
        for (int d = 0; d < hd; d += 8) {
          const T* kp = kb + k_in_page(key, d);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc += qs[wave][d + e] * Store<T>::to(kp[e]);
        }
        sc = acc * aa.scale;
      }
      const float tmax = wave_reduce_max(sc);
      if (tmax == -INFINITY) continue;   // uniform across the wavefront
      const float m_new = fmaxf(m_run, tmax);
      const float corr = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
      const float p = ok ? expf(sc - m_new) : 0.f;
      l_run = l_run * corr + wave_reduce_sum(p);
      o0 *= corr;
      o1 *= corr;
      m_run = m_new;
      const int n_in_tile = min(64, c1 - t0);
      for (int kk = 0; kk < n_in_tile; ++kk) {
        const float pk = __shfl(p, kk, 64);
        if (pk == 0.f) continue;         // uniform
        const int kpos = t0 + kk;
        const int pg = table[kpos / DF_PAGE];
        const T* vb = pool + kv_head_base(aa.layer, geo.n_pages, pg, aa.n_kv_heads, kvh, hd) + DF_PAGE * hd;
        const int key = kpos % DF_PAGE;
        if (lane < hd) o0 += pk * Store<T>::to(vb[v_in_page(key, lane)]);
        if (lane + 64 < hd) o1 += pk * Store<T>::to(vb[v_in_page(key, lane + 64)]);
      }
    }
    if (lane == 0) part_ml[pr] = make_float2(m_run, l_run);
    if (lane < hd) part_o[pr * hd + lane] = o0;
    if (lane + 64 < hd) part_o[pr * hd + lane + 64] = o1;
  }
}

// ------------------------------------------------------------------------------------------------
// Merge of the splits in ascending split order, few rows (M < 128, where the number of workgroups matters more than
// the shape of the stores): grid (M*Hq), block 128 (one thread per head dim).
// The (max, sum) pairs are fetched by the first wavefront with one load per split, the partial
// outputs with independent loads four at a time, so the kernel is not a chain of dependent loads.
// Output as GEMM activation operand (Act<T>), row length Hq*hd.  n_splits <= 64.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(128) void attn_merge_rows_kernel(const float* __restrict__ part_o, const float2* __restrict__ part_ml,
                                                         T* __restrict__ out, int n_q_heads, int hd, int n_splits) {
  const int row = blockIdx.x;  // m*Hq + hq
  const int m = row / n_q_heads, hq = row % n_q_heads;
  const int d = threadIdx.x;
  __shared__ float wgt[64];
  __shared__ float s_L;
  // the first PRE splits' outputs are requested before the weights are known: their loads do not depend on the
  // (max, sum) loads, so the two memory round trips overlap instead of following each other
  constexpr int PRE = 20;
  float pre[PRE];
  const float* po = part_o + (size_t)row * n_splits * hd + (d < hd ? d : 0);
#pragma unroll
  for (int c = 0; c < PRE; ++c) pre[c] = c < n_splits ? po[(size_t)c * hd] : 0.f;
  if (threadIdx.x < 64) {
    const int c = threadIdx.x;
    float2 ml = make_float2(-INFINITY, 0.f);
    if (c < n_splits) ml = part_ml[(size_t)row * n_splits + c];
    const float mx = wave_reduce_max(ml.y > 0.f ? ml.x : -INFINITY);
    const float w = (ml.y > 0.f) ? expf(ml.x - mx) : 0.f;
    wgt[c] = w;
    // sum in ascending split order (fixed order, independent of the wavefront reduction tree)
    float L = 0.f;
    for (int i = 0; i < n_splits; ++i) L += __shfl(ml.y * w, i, 64);
    if (c == 0) s_L = L;
  }
  __syncthreads();
  if (d < hd) {
    float o = 0.f;
#pragma unroll
    for (int c = 0; c < PRE; ++c)
      if (c < n_splits) o += wgt[c] * pre[c];
    int c = PRE;
    for (; c + 4 <= n_splits; c += 4) {
      const float a0 = po[(size_t)(c + 0) * hd], a1 = po[(size_t)(c + 1) * hd], a2 = po[(size_t)(c + 2) * hd], a3 = po[(size_t)(c + 3) * hd];
      o += wgt[c] * a0;
      o += wgt[c + 1] * a1;
      o += wgt[c + 2] * a2;
      o += wgt[c + 3] * a3;
    }
    for (; c < n_splits; ++c) o += wgt[c] * po[(size_t)c * hd];
    const float L = s_L;
    Act<T>::store(out, m, hq * hd + d, n_q_heads * hd, L > 0.f ? o / L : 0.f);
  }
}

// ------------------------------------------------------------------------------------------------
// Merge of the splits in ascending split order.  One workgroup per (band of 16 rows, query head): thread
// (r = tid % 16, c = tid / 16) owns 4 head dims of row r, so that the 16 rows of a band write one contiguous piece
// of the operand tile (the band's rows are interleaved inside a tile) instead of scattered 2-byte stores.
// grid (ceil(M/16), Hq), block 16 * hd/4.  The (max, sum) pairs of a row are fetched by one wavefront with one
// load per split; the partial outputs are requested before the weights are known (their loads do not depend on
// the (max, sum) loads, so the two memory round trips overlap).  Output as GEMM activation operand (Act<T>), row
// length Hq*hd.  n_splits <= 64.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(512) void attn_merge_kernel(const float* __restrict__ part_o, const float2* __restrict__ part_ml,
                                                         T* __restrict__ out, int n_q_heads, int hd, int n_splits, int M) {
  const int r = threadIdx.x & 15, c = threadIdx.x >> 4, hq = blockIdx.y;
  const int m_raw = blockIdx.x * 16 + r;
  const bool live = m_raw < M;
  const int m = live ? m_raw : M - 1;
  __shared__ float wgt[16][64];
  __shared__ float s_L[16];
  constexpr int PRE = 8;
  float4 pre[PRE];
  const float* po = part_o + ((size_t)m * n_q_heads + hq) * n_splits * hd + c * 4;
#pragma unroll
  for (int i = 0; i < PRE; ++i) pre[i] = i < n_splits ? *reinterpret_cast<const float4*>(po + (size_t)i * hd) : make_float4(0.f, 0.f, 0.f, 0.f);
  {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    for (int rr = wave; rr < 16; rr += n_waves) {
      const int mm = min(blockIdx.x * 16 + rr, M - 1);
      float2 ml = make_float2(-INFINITY, 0.f);
      if (lane < n_splits) ml = part_ml[((size_t)mm * n_q_heads + hq) * n_splits + lane];
      const float mx = wave_reduce_max(ml.y > 0.f ? ml.x : -INFINITY);
      const float w = (ml.y > 0.f) ? expf(ml.x - mx) : 0.f;
      wgt[rr][lane] = w;
      // sum in ascending split order (fixed order, independent of the wavefront reduction tree)
      float L = 0.f;
      for (int i = 0; i < n_splits; ++i) L += __shfl(ml.y * w, i, 64);
      if (lane == 0) s_L[rr] = L;
    }
  }
  __syncthreads();
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int i = 0; i < PRE; ++i)
    if (i < n_splits) {
      const float w = wgt[r][i];
      o.x += w * pre[i].x; o.y += w * pre[i].y; o.z += w * pre[i].z; o.w += w * pre[i].w;
    }
  int i = PRE;
  for (; i + 4 <= n_splits; i += 4) {
    float4 a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) a[u] = *reinterpret_cast<const float4*>(po + (size_t)(i + u) * hd);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = wgt[r][i + u];
      o.x += w * a[u].x; o.y += w * a[u].y; o.z += w * a[u].z; o.w += w * a[u].w;
    }
  }
  for (; i < n_splits; ++i) {
    const float4 a = *reinterpret_cast<const float4*>(po + (size_t)i * hd);
    const float w = wgt[r][i];
    o.x += w * a.x; o.y += w * a.y; o.z += w * a.z; o.w += w * a.w;
  }
  if (live) {
    const float L = s_L[r];
    Act<T>::store4(out, m, hq * hd + c * 4, n_q_heads * hd,
                   L > 0.f ? make_float4(o.x / L, o.y / L, o.z / L, o.w / L) : make_float4(0.f, 0.f, 0.f, 0.f));
  }
}
