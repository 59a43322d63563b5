// MFMA block attention for bf16 caches (see attn.h for the split / merge contract).
//
// One workgroup = one (split, kv head, sequence): the B*group query rows that share the kv head
// (<= 64, in QG groups of 16) against the chunk's keys.  The four wavefronts take 32-key page pairs
// round-robin, each with its own online-softmax state, and are merged in a fixed order through LDS.
//
// Everything streams from the pool in MFMA operand order (page layout in common.h), nothing is
// transposed:  S^T = K . Q^T   (A = 16 keys x 32 dims of a page, B = Q^T), so a lane ends up with
//              4 consecutive keys of one query column for each of the two pages -- exactly the 8
//              k-slots it must supply as B operand of  O^T += V^T . P^T  (A = 16 dims x 32 keys).
// P is fed as a hi+lo bf16 pair (two MFMAs) so that the attention output keeps ~16 significant bits,
// like every other GEMM input of the bf16 model.
#pragma once
#include "attn.h"

template <int QG, int HD>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ pool,
                                                        SeqGeom geo, AttnArgs aa, float* __restrict__ part_o,
                                                        float2* __restrict__ part_ml) {
  constexpr int KT = HD / 32, DT = HD / 16, LDO = HD + 4;
  const int split = blockIdx.x, kvh = blockIdx.y, s = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, g = lane >> 4;
  const int B = geo.block_size;
  const int group = aa.n_q_heads / aa.n_kv_heads;
  const int rows = B * group;
  const int n_s = geo.seq_lens[s];
  const int cap = geo.max_pages_per_seq * DF_PAGE;
  const int n_tok = min(n_s + B, cap);
  const int c0 = split * aa.chunk;
  const int c1 = min(n_tok, c0 + aa.chunk);
  const int32_t* table = geo.block_table + (size_t)s * geo.max_pages_per_seq;

  __shared__ float osum[64 * LDO];
  __shared__ float sm[4][64];
  __shared__ float lsum[64];

  // ---- query fragments (B operand of S^T): lane (n, g) holds Q[row qg*16+n][kt*32 + g*8 .. +8]
  u32x4 qf[QG][KT];
  int last_vis[QG];
#pragma unroll
  for (int qg = 0; qg < QG; ++qg) {
    const int r = qg * 16 + n;
    const bool valid = r < rows;
    const int slot = valid ? r / group : 0, hq = kvh * group + (valid ? r % group : 0);
    const u32x4* qp = reinterpret_cast<const u32x4*>(q + ((size_t)(s * B + slot) * aa.n_q_heads + hq) * HD);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) qf[qg][kt] = valid ? qp[kt * 4 + g] : (u32x4){0u, 0u, 0u, 0u};
    last_vis[qg] = valid ? (aa.causal ? n_s + slot : 0x7FFFFFFF) : -1;
  }

  float m_run[QG], l_run[QG];
  f32x4 acc[DT][QG];
#pragma unroll
  for (int qg = 0; qg < QG; ++qg) {
    m_run[qg] = -INFINITY;
    l_run[qg] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[dt][qg] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const int n_pairs = c1 > c0 ? (c1 - c0 + 31) >> 5 : 0;
  for (int p = wave; p < n_pairs; p += 4) {
    const int base = c0 + p * 32;           // first key of page A; page B starts at base + 16
    const int ia = base >> 4;
    int pa = table[ia];
    const bool ok_a = pa >= 0 && pa < geo.n_pages;
    if (!ok_a) pa = 0;
    const bool has_b = base + 16 < c1;
    int pb = has_b ? table[ia + 1] : pa;
    const bool ok_b = has_b && pb >= 0 && pb < geo.n_pages;
    if (!ok_b) pb = pa;
    const bf16_t* ka = pool + kv_head_base(aa.layer, geo.n_pages, pa, aa.n_kv_heads, kvh, HD);
    const bf16_t* kb = pool + kv_head_base(aa.layer, geo.n_pages, pb, aa.n_kv_heads, kvh, HD);
    u32x4 kfa[KT], kfb[KT];
    uint2 vfa[DT], vfb[DT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      kfa[kt] = reinterpret_cast<const u32x4*>(ka)[kt * 64 + lane];
      kfb[kt] = reinterpret_cast<const u32x4*>(kb)[kt * 64 + lane];
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      vfa[dt] = reinterpret_cast<const uint2*>(ka + DF_PAGE * HD)[dt * 64 + lane];
      vfb[dt] = reinterpret_cast<const uint2*>(kb + DF_PAGE * HD)[dt * 64 + lane];
    }
    // rows at or beyond n_tok were never written (and an invalid page is not ours): 0 * garbage must not
    // become NaN, so clear those V elements.  Only the last pair of a sequence takes this path.
    if (base + 32 > n_tok || !ok_a || !ok_b) {
      const int pos_a = base + 4 * g, pos_b = base + 16 + 4 * g;
      uint32_t ma0 = 0u, ma1 = 0u, mb0 = 0u, mb1 = 0u;
      if (ok_a && pos_a + 0 < n_tok) ma0 |= 0x0000FFFFu;
      if (ok_a && pos_a + 1 < n_tok) ma0 |= 0xFFFF0000u;
      if (ok_a && pos_a + 2 < n_tok) ma1 |= 0x0000FFFFu;
      if (ok_a && pos_a + 3 < n_tok) ma1 |= 0xFFFF0000u;
      if (ok_b && pos_b + 0 < n_tok) mb0 |= 0x0000FFFFu;
      if (ok_b && pos_b + 1 < n_tok) mb0 |= 0xFFFF0000u;
      if (ok_b && pos_b + 2 < n_tok) mb1 |= 0x0000FFFFu;
      if (ok_b && pos_b + 3 < n_tok) mb1 |= 0xFFFF0000u;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        vfa[dt].x &= ma0; vfa[dt].y &= ma1;
        vfb[dt].x &= mb0; vfb[dt].y &= mb1;
      }
    }

#pragma unroll
    for (int qg = 0; qg < QG; ++qg) {
      f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kfa[kt]), __builtin_bit_cast(bf16x8, qf[qg][kt]), sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kfb[kt]), __builtin_bit_cast(bf16x8, qf[qg][kt]), sb, 0, 0, 0);
      }
      float v[8];
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int pos_a = base + 4 * g + i, pos_b = pos_a + 16;
        v[i] = (ok_a && pos_a < c1 && pos_a <= last_vis[qg]) ? sa[i] * aa.scale : -INFINITY;
        v[4 + i] = (ok_b && pos_b < c1 && pos_b <= last_vis[qg]) ? sb[i] * aa.scale : -INFINITY;
        mx = fmaxf(mx, fmaxf(v[i], v[4 + i]));
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[qg], mx);
      float corr = 1.f, psum = 0.f;
      float pv[8];
      if (m_new == -INFINITY) {
#pragma unroll
        for (int i = 0; i < 8; ++i) pv[i] = 0.f;
      } else {
        corr = (m_run[qg] == -INFINITY) ? 0.f : __expf(m_run[qg] - m_new);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pv[i] = __expf(v[i] - m_new);   // exp(-inf) = 0 for masked keys
          psum += pv[i];
        }
      }
      l_run[qg] = l_run[qg] * corr + psum;
      m_run[qg] = m_new;
      u32x4 ph, pl;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bf16_t h0 = float_to_bf16_bits(pv[2 * i]), h1 = float_to_bf16_bits(pv[2 * i + 1]);
        const bf16_t l0 = float_to_bf16_bits(pv[2 * i] - bf16_bits_to_float(h0));
        const bf16_t l1 = float_to_bf16_bits(pv[2 * i + 1] - bf16_bits_to_float(h1));
        ph[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        pl[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const u32x4 vf = {vfa[dt].x, vfa[dt].y, vfb[dt].x, vfb[dt].y};
        f32x4 a = acc[dt][qg];
        a[0] *= corr; a[1] *= corr; a[2] *= corr; a[3] *= corr;
        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), __builtin_bit_cast(bf16x8, ph), a, 0, 0, 0);
        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), __builtin_bit_cast(bf16x8, pl), a, 0, 0, 0);
        acc[dt][qg] = a;
      }
    }
  }

  // ---- merge the four wavefronts in the order 0,1,2,3 -------------------------------------------------
#pragma unroll
  for (int qg = 0; qg < QG; ++qg)
    if (g == 0) sm[wave][qg * 16 + n] = m_run[qg];
  __syncthreads();
  float sc[QG], lw[QG];
#pragma unroll
  for (int qg = 0; qg < QG; ++qg) {
    const int r = qg * 16 + n;
    const float mg = fmaxf(fmaxf(sm[0][r], sm[1][r]), fmaxf(sm[2][r], sm[3][r]));
    sc[qg] = (m_run[qg] == -INFINITY) ? 0.f : __expf(m_run[qg] - mg);
    float l = l_run[qg];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    lw[qg] = l * sc[qg];
  }
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int qg = 0; qg < QG; ++qg) {
        const int r = qg * 16 + n;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          float4* dst = reinterpret_cast<float4*>(&osum[r * LDO + dt * 16 + 4 * g]);
          float4 o = make_float4(acc[dt][qg][0] * sc[qg], acc[dt][qg][1] * sc[qg], acc[dt][qg][2] * sc[qg], acc[dt][qg][3] * sc[qg]);
          if (w > 0) {
            const float4 prev = *dst;
            o.x += prev.x; o.y += prev.y; o.z += prev.z; o.w += prev.w;
          }
          *dst = o;
        }
        if (g == 0) lsum[r] = (w > 0 ? lsum[r] : 0.f) + lw[qg];
      }
    }
    __syncthreads();
  }
  for (int idx = threadIdx.x; idx < rows * HD; idx += 256) {
    const int r = idx / HD, d = idx % HD;
    const int slot = r / group, hq = kvh * group + r % group;
    const size_t pr = ((size_t)(s * B + slot) * aa.n_q_heads + hq) * aa.n_splits + split;
    part_o[pr * HD + d] = osum[r * LDO + d];
  }
  if (threadIdx.x < rows) {
    const int r = threadIdx.x;
    const int slot = r / group, hq = kvh * group + r % group;
    const size_t pr = ((size_t)(s * B + slot) * aa.n_q_heads + hq) * aa.n_splits + split;
    const float mg = fmaxf(fmaxf(sm[0][r], sm[1][r]), fmaxf(sm[2][r], sm[3][r]));
    part_ml[pr] = make_float2(mg, lsum[r]);
  }
}

// Returns true when it launched a kernel for this configuration; false -> caller uses the generic kernel.
template <typename T>
inline bool attn_mfma_launch(hipStream_t, const T*, const T*, SeqGeom, AttnArgs, int, float*, float2*) {
  return false;
}

template <>
inline bool attn_mfma_launch<bf16_t>(hipStream_t st, const bf16_t* q, const bf16_t* pool, SeqGeom geo, AttnArgs aa, int S,
                                     float* part_o, float2* part_ml) {
  const int rows = geo.block_size * (aa.n_q_heads / aa.n_kv_heads);
  if (rows > 64 || (aa.head_dim != 128 && aa.head_dim != 64)) return false;
  const int qg = (rows + 15) / 16;
  const dim3 grid(aa.n_splits, aa.n_kv_heads, S), block(256);
#define DF_ATTN_CASE(QG_, HD_)                                                                                          \
  hipLaunchKernelGGL((attn_mfma_kernel<QG_, HD_>), grid, block, 0, st, q, pool, geo, aa, part_o, part_ml)
  if (aa.head_dim == 128) {
    if (qg == 1) DF_ATTN_CASE(1, 128);
    else if (qg == 2) DF_ATTN_CASE(2, 128);
    else DF_ATTN_CASE(4, 128);
  } else {
    if (qg == 1) DF_ATTN_CASE(1, 64);
    else if (qg == 2) DF_ATTN_CASE(2, 64);
    else DF_ATTN_CASE(4, 64);
  }
#undef DF_ATTN_CASE
  return true;
}
