// Small memory-bound kernels of the step: embedding gather, RMSNorm, q/k-norm + RoPE + KV page
// write, row argmax / Gumbel-max, acceptance, commit bookkeeping, weight packing and
// KV import/export.
#pragma once
#include "common.h"

// ---- block assembly + embedding gather -------------------------------------------------------
// tokens_out[s, 0] = anchor[s], tokens_out[s, j>0] = mask_id   (Section 4.2: clean anchor + masks)
__global__ void build_block_kernel(const int32_t* __restrict__ anchor, int32_t* __restrict__ tokens_out, int S, int B,
                                   int mask_id) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < S * B) tokens_out[i] = (i % B == 0) ? anchor[i / B] : mask_id;
}

// Rotary table of one model for the rows of a call: out[m * hd/2 + i] = (cos, sin) of pos(m) * theta^(-2i/hd),
// pos(m) = seq_lens[m / B] + m % B.  Angles are formed in double precision (reduced by sincos) so that long
// contexts do not lose phase accuracy; every layer and head of the call then reads the same rounded pair.
struct RopeTab {
  float2* out;   // null: no table
  double log_theta;
  int hd;
};

// h[m, :] = float(E[tokens[m], :]); ids outside the vocabulary raise the status flag and read row 0; so does a sequence
// longer than the host's hint.
// The first two wavefronts also write the row's entries of up to two rotary tables.
// With `fuse.a_out` the row is also handed on as the first layer's GEMM operand with the RMSNorm deferred (see
// gemm_resid.h): a_out[m, :] = h * gain, ssq[m] = sum of squares of the row (one piece per row).
struct EmbedFuse {
  const float* gain = nullptr;
  void* a_out = nullptr;
  float* ssq = nullptr;
};

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tokens,
                                                    float* __restrict__ h, int D, int vocab, int32_t* status,
                                                    const int32_t* __restrict__ seq_lens, int B, int len_hint, RopeTab t0, RopeTab t1,
                                                    EmbedFuse fuse = EmbedFuse{}) {
  const int m = blockIdx.x;
  // the host sized the attention launches of this call for sequences of at most len_hint committed tokens: a longer
  // one would have its last keys left out, so it is reported
  if (threadIdx.x == 0 && seq_lens[m / B] > len_hint) atomicOr(status, DF_STATUS_CAPACITY);
  {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const RopeTab rt = w == 0 ? t0 : t1;
    if (w < 2 && rt.out && lane < (rt.hd >> 1)) {
      const int pos = seq_lens[m / B] + m % B;
      double sn, cs;
      sincos((double)pos * exp(-rt.log_theta * (2.0 * lane / rt.hd)), &sn, &cs);
      rt.out[(size_t)m * (rt.hd >> 1) + lane] = make_float2((float)cs, (float)sn);
    }
  }
  int tok = tokens[m];
  if (tok < 0 || tok >= vocab) {
    if (threadIdx.x == 0) atomicOr(status, DF_STATUS_CAPACITY);
    tok = 0;
  }
  const T* src = E + (size_t)tok * D;
  float ss = 0.f;
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    const float v = Store<T>::to(src[d]);
    h[(size_t)m * D + d] = v;
    if (fuse.a_out) {
      Act<T>::store(reinterpret_cast<T*>(fuse.a_out), m, d, D, v * fuse.gain[d]);
      ss += v * v;
    }
  }
  if (fuse.a_out) {   // uniform over the workgroup
    __shared__ float part[4];
    ss = wave_reduce_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) fuse.ssq[m] = (part[0] + part[1]) + (part[2] + part[3]);
  }
}

// ---- RMSNorm with pending-sum reduction -----------------------------------------------------------
// x[m,:] = base[m,:] (if base) + sum_z delta[z*slab + m*D + :] (ascending z: the K-range partial results of
// the preceding GEMM).  When delta is given the completed row is written to h_out (the residual stream).
// Optionally the completed row is also stored as tap `tap_idx` (GEMM activation operand, row length tap_K).
// out[m,:] = x * gain / sqrt(mean(x^2) + eps) as GEMM activation operand (Act<T>).
// MIX (routed experts): the pending sum of row m is instead sum_j mix.w[m*k + j] * delta[mix.pos[m*k + j] * D + :], j
// ascending -- the weighted sum of the row's experts' outputs, which sit at the row's positions of the expert-sorted list.
struct RowMix {
  const int32_t* pos = nullptr;
  const float* w = nullptr;
  int k = 0;
};

template <typename T, int NTHR, bool MIX = false>
__global__ __launch_bounds__(NTHR) void rmsnorm_kernel(const float* base, const float* __restrict__ delta, int ks,
                                                      size_t slab, float* h_out, const float* __restrict__ gain,
                                                      T* __restrict__ out, int D, float eps, T* __restrict__ taps, int tap_idx,
                                                      int tap_K, RowMix mix = RowMix{}) {
  // Consecutive workgroup ids go to different XCDs (round-robin dispatch), and the 16 rows of a band share the cache
  // lines of an operand tile: with many rows, XCD x takes the rows [x * M/8, (x+1) * M/8), so that the 16-byte pieces
  // of a line are merged in one L2 and leave it as whole lines instead of eight partial writes from eight L2s.
  const int n_rows = (int)gridDim.x;
  const int m = (n_rows % 128 == 0) ? (int)(blockIdx.x & 7) * (n_rows >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  const size_t ro = (size_t)m * D;
  // completed row chunk d..d+3: base + pending slabs (four independent loads in flight, added in ascending order)
  auto gather = [&](int d) {
    float4 v = base ? *reinterpret_cast<const float4*>(base + ro + d) : make_float4(0.f, 0.f, 0.f, 0.f);
    if constexpr (MIX) {
      const int32_t* pj = mix.pos + (size_t)m * mix.k;
      const float* wj = mix.w + (size_t)m * mix.k;
      int j = 0;
      for (; j + 4 <= mix.k; j += 4) {   // four experts' rows in flight at a time
        const float4 p0 = *reinterpret_cast<const float4*>(delta + (size_t)pj[j] * D + d);
        const float4 p1 = *reinterpret_cast<const float4*>(delta + (size_t)pj[j + 1] * D + d);
        const float4 p2 = *reinterpret_cast<const float4*>(delta + (size_t)pj[j + 2] * D + d);
        const float4 p3 = *reinterpret_cast<const float4*>(delta + (size_t)pj[j + 3] * D + d);
        const float w0 = wj[j], w1 = wj[j + 1], w2 = wj[j + 2], w3 = wj[j + 3];
        v.x += w0 * p0.x; v.y += w0 * p0.y; v.z += w0 * p0.z; v.w += w0 * p0.w;
        v.x += w1 * p1.x; v.y += w1 * p1.y; v.z += w1 * p1.z; v.w += w1 * p1.w;
        v.x += w2 * p2.x; v.y += w2 * p2.y; v.z += w2 * p2.z; v.w += w2 * p2.w;
        v.x += w3 * p3.x; v.y += w3 * p3.y; v.z += w3 * p3.z; v.w += w3 * p3.w;
      }
      for (; j < mix.k; ++j) {
        const float4 p = *reinterpret_cast<const float4*>(delta + (size_t)pj[j] * D + d);
        const float w0 = wj[j];
        v.x += w0 * p.x; v.y += w0 * p.y; v.z += w0 * p.z; v.w += w0 * p.w;
      }
      *reinterpret_cast<float4*>(h_out + ro + d) = v;
      if (taps) Act<T>::store4(taps, m, tap_idx * D + d, tap_K, v);
      return v;
    }
    int z = 0;
    for (; z + 4 <= ks; z += 4) {
      const float* pz = delta + (size_t)z * slab + ro + d;
      const float4 p0 = *reinterpret_cast<const float4*>(pz), p1 = *reinterpret_cast<const float4*>(pz + slab);
      const float4 p2 = *reinterpret_cast<const float4*>(pz + 2 * slab), p3 = *reinterpret_cast<const float4*>(pz + 3 * slab);
      v.x += p0.x; v.y += p0.y; v.z += p0.z; v.w += p0.w;
      v.x += p1.x; v.y += p1.y; v.z += p1.z; v.w += p1.w;
      v.x += p2.x; v.y += p2.y; v.z += p2.z; v.w += p2.w;
      v.x += p3.x; v.y += p3.y; v.z += p3.z; v.w += p3.w;
    }
    for (; z < ks; ++z) {
      const float4 p = *reinterpret_cast<const float4*>(delta + (size_t)z * slab + ro + d);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (ks > 0) *reinterpret_cast<float4*>(h_out + ro + d) = v;
    if (taps) Act<T>::store4(taps, m, tap_idx * D + d, tap_K, v);
    return v;
  };
  // NTHR threads per row (1024 for wide rows: one 16-byte chunk per thread keeps every load independent).
  // The first KEEP chunks of a thread stay in registers between the two passes (rows up to 8192 wide);
  // wider rows re-read the rest from where it was written
  constexpr int KEEP = 8192 / (NTHR * 4);
  float4 keep[KEEP], gk[KEEP];   // the gains are requested together with the row: no extra round trip after the barrier
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < KEEP; ++c) {
    const int d = (c * NTHR + (int)threadIdx.x) * 4;
    gk[c] = d < D ? *reinterpret_cast<const float4*>(gain + d) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int c = 0; c < KEEP; ++c) {
    const int d = (c * NTHR + (int)threadIdx.x) * 4;
    keep[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (d < D) {
      keep[c] = gather(d);
      ss += keep[c].x * keep[c].x + keep[c].y * keep[c].y + keep[c].z * keep[c].z + keep[c].w * keep[c].w;
    }
  }
  for (int d = (KEEP * NTHR + (int)threadIdx.x) * 4; d < D; d += NTHR * 4) {
    const float4 v = gather(d);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  __shared__ float part[NTHR / 64];
  ss = wave_reduce_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < NTHR / 64; ++w) tot += part[w];
  const float rstd = 1.0f / sqrtf(tot / (float)D + eps);
#pragma unroll
  for (int c = 0; c < KEEP; ++c) {
    const int d = (c * NTHR + (int)threadIdx.x) * 4;
    if (d < D) {
      const float4 v = keep[c], g = gk[c];
      Act<T>::store4(out, m, d, D, make_float4(v.x * rstd * g.x, v.y * rstd * g.y, v.z * rstd * g.z, v.w * rstd * g.w));
    }
  }
  const float* src = ks > 0 ? h_out : base;   // each thread re-reads exactly what it wrote
  for (int d = (KEEP * NTHR + (int)threadIdx.x) * 4; d < D; d += NTHR * 4) {
    const float4 v = *reinterpret_cast<const float4*>(src + ro + d);
    const float4 g = *reinterpret_cast<const float4*>(gain + d);
    Act<T>::store4(out, m, d, D, make_float4(v.x * rstd * g.x, v.y * rstd * g.y, v.z * rstd * g.z, v.w * rstd * g.w));
  }
}

// ---- q/k RMSNorm + RoPE + cache write ------------------------------------------------------------
// One wavefront per (row m, head), four heads per workgroup; lane i owns the rotate-half pair (i, i + hd/2) [hd <= 128].
// Input row: fp32 [.. q heads | k heads | v heads ..] starting at in + m*in_ld, given as `ks` partial
// slabs (K ranges of the producing GEMM) `slab` elements apart that are added in ascending order.
// q heads -> q_out [M, Hq, hd] row-major storage type; k/v heads -> page of position seq_len + slot.
// (cos, sin) come from the call's rotary table (RopeTab), written by embed_kernel.
struct RopeArgs {
  int n_q_heads, n_kv_heads, head_dim;
  int q_off, k_off, v_off;  // element offsets inside an input row
  int qk_norm;
  float eps;
  const float2* rope;       // rotary table [M, hd/2] of this model for the rows of the call
  int layer;                // layer index inside the pool
  // grid.z > 1 handles several layers in one launch (the draft's context K/V at commit): layer z reads its
  // k/v columns z * col_stride further along the input row and its k-norm gain kn_stride floats further on
  int col_stride = 0;
  size_t kn_stride = 0;
};

template <typename T>
__global__ __launch_bounds__(256) void qkv_post_kernel(const float* __restrict__ in, int in_ld, const float* __restrict__ qn,
                                                       const float* __restrict__ kn, T* __restrict__ q_out,
                                                       T* __restrict__ pool, SeqGeom geo, RopeArgs ra, int ks, size_t slab) {
  // rows of one 16-key page on one XCD (see rmsnorm_kernel): their 16-byte pieces of a K/V page line meet in one L2
  const int n_rows = (int)gridDim.x;
  const int m = (n_rows % 128 == 0) ? (int)(blockIdx.x & 7) * (n_rows >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  const int head = blockIdx.y * 4 + (int)(threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (head >= ra.n_q_heads + 2 * ra.n_kv_heads) return;   // no barrier in this kernel
  ra.layer += blockIdx.z;
  ra.k_off += blockIdx.z * ra.col_stride;
  ra.v_off += blockIdx.z * ra.col_stride;
  kn += blockIdx.z * ra.kn_stride;
  const int hd = ra.head_dim, half = hd >> 1;
  const int s = m / geo.block_size, slot = m % geo.block_size;
  const int pos = geo.seq_lens[s] + slot;
  const bool is_q = head < ra.n_q_heads;
  const bool is_k = !is_q && head < ra.n_q_heads + ra.n_kv_heads;
  const int kvh = is_q ? 0 : (is_k ? head - ra.n_q_heads : head - ra.n_q_heads - ra.n_kv_heads);
  const float* src = in + (size_t)m * in_ld + (is_q ? ra.q_off + head * hd : (is_k ? ra.k_off : ra.v_off) + kvh * hd);
  const bool active = lane < half;
  float x1 = 0.f, x2 = 0.f;
  if (active)
    for (int z = 0; z < ks; ++z) {
      x1 += src[(size_t)z * slab + lane];
      x2 += src[(size_t)z * slab + lane + half];
    }
  if (!is_q) {
    const int pidx = pos / DF_PAGE;
    int page = -1;
    if (pos >= 0 && pidx < geo.max_pages_per_seq) page = geo.block_table[(size_t)s * geo.max_pages_per_seq + pidx];
    if (page < 0 || page >= geo.n_pages) {
      if (lane == 0) atomicOr(geo.status, DF_STATUS_CAPACITY);
      return;
    }
    T* base = pool + kv_head_base(ra.layer, geo.n_pages, page, ra.n_kv_heads, kvh, hd);
    const int key = pos % DF_PAGE;
    if (!is_k) {
      if (active) {
        base[DF_PAGE * hd + v_in_page(key, lane)] = Store<T>::from(x1);
        base[DF_PAGE * hd + v_in_page(key, lane + half)] = Store<T>::from(x2);
      }
      return;
    }
    if (ra.qk_norm) {
      const float ss = wave_reduce_sum(x1 * x1 + x2 * x2);
      const float rstd = 1.0f / sqrtf(ss / (float)hd + ra.eps);
      if (active) { x1 *= rstd * kn[lane]; x2 *= rstd * kn[lane + half]; }
    }
    if (active) {
      const float2 r = ra.rope[(size_t)m * half + lane];
      const float c = r.x, sf = r.y;
      base[k_in_page(key, lane)] = Store<T>::from(x1 * c - x2 * sf);
      base[k_in_page(key, lane + half)] = Store<T>::from(x2 * c + x1 * sf);
    }
    return;
  }
  if (ra.qk_norm) {
    const float ss = wave_reduce_sum(x1 * x1 + x2 * x2);
    const float rstd = 1.0f / sqrtf(ss / (float)hd + ra.eps);
    if (active) { x1 *= rstd * qn[lane]; x2 *= rstd * qn[lane + half]; }
  }
  if (active) {
    const float2 r = ra.rope[(size_t)m * half + lane];
    const float c = r.x, sf = r.y;
    T* dst = q_out + ((size_t)m * ra.n_q_heads + head) * hd;
    dst[lane] = Store<T>::from(x1 * c - x2 * sf);
    dst[lane + half] = Store<T>::from(x2 * c + x1 * sf);
  }
}

// ---- row argmax (ties -> lowest index), optionally of logit/T + Gumbel noise ---------------------
// block-wide argmax (up to 1024 threads); result valid in thread 0
__device__ __forceinline__ void block_argmax(float& bv, int& bi) {
  __shared__ float sv[16];
  __shared__ int si[16];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    argmax_combine(bv, bi, ov, oi);
  }
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) { sv[wave] = bv; si[wave] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < nw; ++w) argmax_combine(bv, bi, sv[w], si[w]);
  }
}

// mode 0: greedy.  mode 1: draft sampling, score = logit * inv_T + Gumbel(key, seq, slot, purpose 0).
// Stage 1: grid (n_chunks, M): best (score, index) of one chunk of row m -> part[m * n_chunks + chunk].
// Stage 2 (argmax_finish_kernel): combines the chunks in ascending order (ties -> lowest index) and writes out[m]
// unless (skip_slot0 && slot == 0).
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ logits, int V, int B, float2* __restrict__ part,
                                                          int mode, float inv_T, const uint64_t* __restrict__ rng_key) {
  const int chunk = blockIdx.x, n_chunks = gridDim.x, m = blockIdx.y, slot = m % B, seq = m / B;
  const int per = (V + n_chunks - 1) / n_chunks, i0 = chunk * per, i1 = min(V, i0 + per);
  const float* row = logits + (size_t)m * V;
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  const uint64_t key = mode ? rng_key[0] : 0ull;
  for (int i = i0 + threadIdx.x; i < i1; i += blockDim.x) {
    float v = row[i];
    if (mode) v = v * inv_T + gumbel(counter_uniform(key, seq, slot, 0, (uint32_t)i));
    argmax_combine(bv, bi, v, i);
  }
  block_argmax(bv, bi);
  if (threadIdx.x == 0) part[(size_t)m * n_chunks + chunk] = make_float2(bv, __int_as_float(bi));
}

__global__ __launch_bounds__(64) void argmax_finish_kernel(const float2* __restrict__ part, int n_chunks, int B, int32_t* __restrict__ out,
                                                           int skip_slot0) {
  const int m = blockIdx.x;
  if (skip_slot0 && m % B == 0) return;
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int c = threadIdx.x; c < n_chunks; c += 64) {
    const float2 p = part[(size_t)m * n_chunks + c];
    argmax_combine(bv, bi, p.x, __float_as_int(p.y));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    argmax_combine(bv, bi, ov, oi);
  }
  if (threadIdx.x == 0) out[m] = bi;
}

// ---- greedy acceptance (Section 3.1) ---------------------------------------------------------------
__global__ void accept_greedy_kernel(const int32_t* __restrict__ draft, const int32_t* __restrict__ tgt, int S, int B,
                                     int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= S) return;
  const int32_t* d = draft + (size_t)s * B;
  const int32_t* t = tgt + (size_t)s * B;
  int a = 0;
  while (a + 1 < B && d[a + 1] == t[a]) ++a;
  accept_len[s] = a;
  for (int j = 0; j < B; ++j) out_tokens[(size_t)s * B + j] = (j < a) ? d[j + 1] : (j == a ? t[a] : -1);
}

// ---- speculative sampling ---------------------------------------------------------------------------
// per-row softmax statistics of logits * inv_T: stats[m] = (max, log-sum-exp)
__global__ __launch_bounds__(1024) void row_lse_kernel(const float* __restrict__ logits, int V, float inv_T,
                                                       float2* __restrict__ stats) {
  const int m = blockIdx.x;
  const float* row = logits + (size_t)m * V;
  __shared__ float sh[16];
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < V; i += blockDim.x) mx = fmaxf(mx, row[i] * inv_T);
  mx = wave_reduce_max(mx);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) mx = fmaxf(mx, sh[w]);
  __syncthreads();
  float sum = 0.f;
  for (int i = threadIdx.x; i < V; i += blockDim.x) sum += expf(row[i] * inv_T - mx);
  sum = wave_reduce_sum(sum);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += sh[w];
    stats[m] = make_float2(mx, mx + logf(tot));
  }
}

// combines the per-workgroup (max, sum) partials that the LM-head epilogue left for row m, in ascending order of the
// column blocks: stats[m] = (max, log-sum-exp) of logits * inv_T, the pair row_lse_kernel computes from stored logits
__global__ __launch_bounds__(64) void lse_finish_kernel(const float2* __restrict__ part, int n_parts, float2* __restrict__ stats) {
  const int m = blockIdx.x, lane = threadIdx.x;
  float mx = -INFINITY;
  for (int c = lane; c < n_parts; c += 64) mx = fmaxf(mx, part[(size_t)m * n_parts + c].x);
  mx = wave_reduce_max(mx);
  // every lane sums its stride of the parts in ascending order, then the 64 lane sums are added in lane order
  float s = 0.f;
  for (int c = lane; c < n_parts; c += 64) {
    const float2 p = part[(size_t)m * n_parts + c];
    s += p.x == -INFINITY ? 0.f : p.y * expf(p.x - mx);
  }
  float tot = 0.f;
  for (int i = 0; i < 64; ++i) tot += __shfl(s, i, 64);
  if (lane == 0) stats[m] = make_float2(mx, mx + logf(tot));
}

// One block per sequence.  Thread 0 walks the slots: slot j accepted iff u_j * q_j(d_j) < p_{j-1}(d_j).
// Then the whole block draws the final token by Gumbel-max over
//   first rejected slot j: log max(p_{j-1} - q_j, 0)   (purpose 1, slot j)
//   none rejected:         log p_{B-1}                 (purpose 2, slot B)
__global__ __launch_bounds__(1024) void accept_sampling_kernel(const float* __restrict__ p_logits, const float* __restrict__ q_logits,
                                                               const float2* __restrict__ p_stats, const float2* __restrict__ q_stats,
                                                               const int32_t* __restrict__ draft, const float* __restrict__ uniforms,
                                                               const uint64_t* __restrict__ rng_key, int V, int B, float inv_T,
                                                               int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens) {
  const int s = blockIdx.x;
  __shared__ int sh_a;
  if (threadIdx.x == 0) {
    int a = B - 1;
    for (int j = 1; j < B; ++j) {
      const int d = draft[(size_t)s * B + j];
      const size_t mp = (size_t)s * B + j - 1, mq = (size_t)s * B + j;
      const float p = expf(p_logits[mp * V + d] * inv_T - p_stats[mp].y);
      const float q = expf(q_logits[mq * V + d] * inv_T - q_stats[mq].y);
      if (!(uniforms[(size_t)s * B + j] * q < p)) { a = j - 1; break; }
    }
    sh_a = a;
  }
  __syncthreads();
  const int a = sh_a;
  const bool bonus = (a == B - 1);
  // a rejection at slot j gives a = j-1 <= B-2, so a == B-1 means every slot was accepted
  const uint64_t key = rng_key[0];
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  if (bonus) {
    const size_t mp = (size_t)s * B + (B - 1);
    for (int i = threadIdx.x; i < V; i += blockDim.x) {
      const float v = p_logits[mp * V + i] * inv_T - p_stats[mp].y + gumbel(counter_uniform(key, s, B, 2, (uint32_t)i));
      argmax_combine(bv, bi, v, i);
    }
  } else {
    const int j = a + 1;
    const size_t mp = (size_t)s * B + j - 1, mq = (size_t)s * B + j;
    for (int i = threadIdx.x; i < V; i += blockDim.x) {
      const float p = expf(p_logits[mp * V + i] * inv_T - p_stats[mp].y);
      const float q = expf(q_logits[mq * V + i] * inv_T - q_stats[mq].y);
      const float r = p - q;
      if (r > 0.f) {
        const float v = logf(r) + gumbel(counter_uniform(key, s, j, 1, (uint32_t)i));
        argmax_combine(bv, bi, v, i);
      }
    }
  }
  block_argmax(bv, bi);
  if (threadIdx.x == 0) {
    accept_len[s] = a;
    for (int j = 0; j < B; ++j)
      out_tokens[(size_t)s * B + j] = (j < a) ? draft[(size_t)s * B + j + 1] : (j == a ? bi : -1);
  }
}

// ---- commit bookkeeping ----------------------------------------------------------------------------
__global__ void commit_update_kernel(SeqGeom geo, int32_t* __restrict__ seq_lens, int32_t* __restrict__ anchor,
                                     const int32_t* __restrict__ accept_len, const int32_t* __restrict__ out_tokens, int S,
                                     int64_t* __restrict__ kv_slots) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= S) return;
  const int B = geo.block_size;
  const int n = seq_lens[s];
  int a = accept_len[s];
  a = max(-1, min(a, B - 1));   // -1: nothing of this sequence is committed, anchor kept
  if (kv_slots) {
    for (int j = 0; j < B; ++j) {
      int64_t slot = -1;
      const int pos = n + j, pidx = pos / DF_PAGE;
      if (j <= a && pidx < geo.max_pages_per_seq) {
        const int page = geo.block_table[(size_t)s * geo.max_pages_per_seq + pidx];
        if (page >= 0 && page < geo.n_pages) slot = (int64_t)page * DF_PAGE + pos % DF_PAGE;
      }
      kv_slots[(size_t)s * B + j] = slot;
    }
  }
  if (a >= 0) anchor[s] = out_tokens[(size_t)s * B + a];
  seq_lens[s] = n + a + 1;
}

// ---- weight packing ---------------------------------------------------------------------------------
// dst row r of the packed matrix comes from source matrix/row:
//   mode 0 (concat):      sources stacked in order
//   mode 1 (interleave):  16 rows of src0, 16 rows of src1, 16 rows of src0, ...
struct PackSrc {
  const void* src[3];
  int rows[3];
  int n_src;
  int mode;
};
template <typename T>
__global__ __launch_bounds__(256) void pack_kernel(PackSrc ps, int K, int total_rows, T* __restrict__ dst, int dst_row0,
                                                   int dst_rows) {
  const size_t chunk = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 8-element chunk
  const int chunks_per_row = K >> 3;
  const size_t n_chunks = (size_t)total_rows * chunks_per_row;
  if (chunk >= n_chunks) return;
  const int r = (int)(chunk / chunks_per_row), k = (int)(chunk % chunks_per_row) * 8;
  int si = 0, sr = r;
  if (ps.mode == 1) {
    si = (r >> 4) & 1;
    sr = ((r >> 5) << 4) + (r & 15);
  } else {
    while (si + 1 < ps.n_src && sr >= ps.rows[si]) { sr -= ps.rows[si]; ++si; }
  }
  const T* s = reinterpret_cast<const T*>(ps.src[si]) + (size_t)sr * K + k;
  T* d = dst + tile_index<T>(dst_row0 + r, k, K, dst_rows);   // rows land at dst_row0.. of a dst_rows-row matrix
#pragma unroll
  for (int i = 0; i < 8; ++i) d[i] = s[i];
}

// ---- KV import / export -------------------------------------------------------------------------------
// dir 0: pool -> canonical fp32 [count, Hkv, hd]; dir 1: canonical -> pool
template <typename T>
__global__ __launch_bounds__(128) void kv_copy_kernel(T* __restrict__ pool, SeqGeom geo, int layer, int n_kv_heads, int hd, int seq,
                                                      int start, float* __restrict__ k, float* __restrict__ v, int dir) {
  const int pos = start + blockIdx.x, kvh = blockIdx.y;
  const int pidx = pos / DF_PAGE;
  if (pidx >= geo.max_pages_per_seq) return;
  const int page = geo.block_table[(size_t)seq * geo.max_pages_per_seq + pidx];
  if (page < 0 || page >= geo.n_pages) return;
  T* base = pool + kv_head_base(layer, geo.n_pages, page, n_kv_heads, kvh, hd);
  const int key = pos % DF_PAGE;
  const size_t row = ((size_t)blockIdx.x * n_kv_heads + kvh) * hd;
  for (int d = threadIdx.x; d < hd; d += blockDim.x) {
    if (dir == 0) {
      k[row + d] = Store<T>::to(base[k_in_page(key, d)]);
      v[row + d] = Store<T>::to(base[DF_PAGE * hd + v_in_page(key, d)]);
    } else {
      base[k_in_page(key, d)] = Store<T>::from(k[row + d]);
      base[DF_PAGE * hd + v_in_page(key, d)] = Store<T>::from(v[row + d]);
    }
  }
}

// ---- machine probes ---------------------------------------------------------------------------------
// where the probes drop a value when an impossible condition holds, so that the compiler keeps their work
__device__ unsigned g_probe_sink;

// read-only streaming: wavefronts interleave 8 KB pieces across the whole grid
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ p, size_t n_chunks) {
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  const size_t n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
  unsigned acc = 0;
  for (size_t c = wave * 8; c < n_chunks; c += n_waves * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + (c + u < n_chunks ? c + u : c) * 64 + lane);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][3];
  }
  if (acc == 0x12345677u) g_probe_sink = acc;   // keeps the loads alive; practically never true
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters) {
  const u32x4 a = {threadIdx.x, 1u, 2u, 3u}, b = {4u, 5u, threadIdx.x, 7u};
  f32x4 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  if (s == 12345.678f) g_probe_sink = 1u;   // keeps the MFMAs alive
}

typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void probe_mfma32_kernel(int iters) {
  const u32x4 a = {threadIdx.x, 1u, 2u, 3u}, b = {4u, 5u, threadIdx.x, 7u};
  probe_f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  if (s == 12345.678f) g_probe_sink = 1u;   // keeps the MFMAs alive
}

// ---- prefill as a many-row pass (Section 4.1: the standard prefill gives the first token and the target's hidden
// features of every prompt token) ------------------------------------------------------------------------------
// The new tokens of all prompts are cut into chunks of B rows; chunk c (counted over all prompts, in order) becomes
// pseudo-sequence c - chunk0 of one verification-shaped pass: committed length = the prompt's cached length + the
// chunk's offset, block-table row = the prompt's.  Inside a layer every K/V row is in the pages before attention runs,
// so the causal block attention of the chunks is a causal prefill.  One workgroup per pseudo-sequence.
struct PrefillPlan {
  const int32_t* lens;         // [S] new tokens per prompt (device copy of the host's array)
  const int32_t* seq_lens;     // [S] tokens already cached
  const int32_t* block_table;  // [S, mpps]
  const int32_t* tokens;       // new tokens of all prompts, concatenated
  int S, B, mpps, chunk0, n_chunks;
  int32_t* p_lens;             // [n_chunks]
  int32_t* p_table;            // [n_chunks, mpps]
  int32_t* p_tokens;           // [n_chunks, B], zero-padded
  int32_t* end_row;            // [.] row (in this pass) of the last token of every prompt that ends in this pass, in prompt order
  int32_t* end_seq;            // [.] and that prompt's index
};

__global__ __launch_bounds__(256) void prefill_plan_kernel(PrefillPlan p) {
  const int i = blockIdx.x, c = p.chunk0 + i;
  __shared__ int sh[4];
  if (threadIdx.x == 0) {
    int first = 0, s = 0, n_end_before = 0;
    for (; s < p.S; ++s) {
      const int nc = (p.lens[s] + p.B - 1) / p.B;
      if (c < first + nc) break;
      // a prompt before ours whose last chunk lies in this pass takes an earlier place in the end list
      if (nc > 0 && first + nc - 1 >= p.chunk0) ++n_end_before;
      first += nc;
    }
    sh[0] = s;
    sh[1] = (c - first) * p.B;       // offset of the chunk inside the prompt's new tokens
    sh[2] = n_end_before;
    int tok0 = 0;
    for (int t = 0; t < s && t < p.S; ++t) tok0 += p.lens[t];
    sh[3] = tok0;
  }
  __syncthreads();
  const int s = sh[0], off = sh[1];
  if (s >= p.S) return;              // cannot happen when the host counted the chunks from the same lengths
  const int len = p.lens[s], rows = min(p.B, len - off);
  for (int j = threadIdx.x; j < p.mpps; j += blockDim.x) p.p_table[(size_t)i * p.mpps + j] = p.block_table[(size_t)s * p.mpps + j];
  for (int j = threadIdx.x; j < p.B; j += blockDim.x) p.p_tokens[(size_t)i * p.B + j] = j < rows ? p.tokens[sh[3] + off + j] : 0;
  if (threadIdx.x == 0) {
    p.p_lens[i] = p.seq_lens[s] + off;
    if (off + rows == len) {
      p.end_row[sh[2]] = i * p.B + rows - 1;
      p.end_seq[sh[2]] = s;
    }
  }
}

// out row r (GEMM operand, row length K) = row rows[r] of `a`
template <typename T>
__global__ __launch_bounds__(256) void gather_operand_rows_kernel(const T* __restrict__ a, const int32_t* __restrict__ rows, T* __restrict__ out, int K) {
  const int r = blockIdx.x, m = rows[r];
  for (int k = threadIdx.x; k < K; k += blockDim.x) {
    if constexpr (sizeof(T) == 2) {
      const size_t src = Act<bf16_t>::index(m, k, K), dst = Act<bf16_t>::index(r, k, K);
      out[dst] = a[src];
      out[dst + 512] = a[src + 512];
    } else {
      out[(size_t)r * K + k] = a[(size_t)m * K + k];
    }
  }
}

// first generated token of the prompts that ended in a pass: anchor and (optionally) the caller's array
__global__ void prefill_first_kernel(const int32_t* __restrict__ first, const int32_t* __restrict__ end_seq, int n_end, int32_t* anchor,
                                     int32_t* first_out) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_end) return;
  const int s = end_seq[r];
  anchor[s] = first[r];
  if (first_out) first_out[s] = first[r];
}

__global__ void prefill_advance_kernel(int32_t* seq_lens, const int32_t* __restrict__ lens, int S) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s < S) seq_lens[s] += lens[s];
}
