// MFMA block attention for bf16 caches (see attn.h for the split / merge contract).
//
// One workgroup = one (split, kv head, sequence): the B*group query rows that share the kv head
// (<= 64) against the chunk's keys.  Wavefront w owns query rows 16w .. 16w+15 for the whole chunk, so
// the four wavefronts never have to be merged; they read the same K/V tiles (the second to fourth read
// hit the CU's L1) and the next 32-key page pair is in flight while the current one is processed.
//
// Everything streams from the pool in MFMA operand order (page layout in common.h), nothing is
// transposed:  S^T = K . Q^T   (A = 16 keys x 32 dims of a page, B = Q^T), so a lane ends up with
//              4 consecutive keys of one query column for each of the two pages -- exactly the 8
//              k-slots it must supply as B operand of  O^T += V^T . P^T  (A = 16 dims x 32 keys).
// P is fed as a hi+lo bf16 pair (two MFMAs) so that the attention output keeps ~16 significant bits,
// like every other GEMM input of the bf16 model.
#pragma once
#include "attn.h"

template <int HD>
struct KvFrags {
  u32x4 ka[HD / 32], kb[HD / 32];
  u32x4 v[HD / 16];   // (4 keys of page A, 4 keys of page B) x one dim per lane: the A operand of P.V
  int ok_a, ok_b;
};

struct AttnLane {          // per-lane constants of the kernel below
  const int32_t* table;
  int c0, c1, n_tok, last_vis, g, lane, kvh;
};

// issues the loads of page pair (pa, pb); pb < 0 means the chunk ends after page A.  STREAM: the fragments are
// used by this wavefront only (key-split kernel), so they are loaded non-temporally and do not displace anything
// from the caches; the row-split kernel's four wavefronts read the same fragments and want them cached.
template <int HD, bool STREAM = false>
__device__ __forceinline__ void attn_load_pages(KvFrags<HD>& f, int pa, int pb, bool has_b, const bf16_t* __restrict__ pool,
                                                const SeqGeom& geo, const AttnArgs& aa, const AttnLane& L) {
  f.ok_a = pa >= 0 && pa < geo.n_pages;
  if (!f.ok_a) pa = 0;
  f.ok_b = has_b && pb >= 0 && pb < geo.n_pages;
  if (!f.ok_b) pb = pa;
  const bf16_t* ka = pool + kv_head_base(aa.layer, geo.n_pages, pa, aa.n_kv_heads, L.kvh, HD);
  const bf16_t* kb = pool + kv_head_base(aa.layer, geo.n_pages, pb, aa.n_kv_heads, L.kvh, HD);
  if constexpr (STREAM) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int kt = 0; kt < HD / 32; ++kt) {
      f.ka[kt] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ka) + kt * 64 + L.lane);
      f.kb[kt] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb) + kt * 64 + L.lane);
    }
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt) {
      const u32x2 a = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(ka + DF_PAGE * HD) + dt * 64 + L.lane);
      const u32x2 b = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(kb + DF_PAGE * HD) + dt * 64 + L.lane);
      f.v[dt] = (u32x4){a[0], a[1], b[0], b[1]};
    }
  } else {
#pragma unroll
    for (int kt = 0; kt < HD / 32; ++kt) {
      f.ka[kt] = reinterpret_cast<const u32x4*>(ka)[kt * 64 + L.lane];
      f.kb[kt] = reinterpret_cast<const u32x4*>(kb)[kt * 64 + L.lane];
    }
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt) {
      const uint2 a = reinterpret_cast<const uint2*>(ka + DF_PAGE * HD)[dt * 64 + L.lane];
      const uint2 b = reinterpret_cast<const uint2*>(kb + DF_PAGE * HD)[dt * 64 + L.lane];
      f.v[dt] = (u32x4){a.x, a.y, b.x, b.y};
    }
  }
}

template <int HD>
__device__ __forceinline__ void attn_load_pair(KvFrags<HD>& f, int p, const bf16_t* __restrict__ pool, const SeqGeom& geo,
                                               const AttnArgs& aa, const AttnLane& L) {
  const int base = L.c0 + p * 32;           // first key of page A; page B starts at base + 16
  const int ia = base >> 4;
  const bool has_b = base + 16 < L.c1;
  const int pa = L.table[ia];
  const int pb = has_b ? L.table[ia + 1] : pa;
  attn_load_pages<HD>(f, pa, pb, has_b, pool, geo, aa, L);
}

template <int HD>
__device__ __forceinline__ void attn_process_pair(KvFrags<HD>& f, int p, const u32x4 (&qf)[HD / 32], f32x4 (&acc)[HD / 16],
                                                  float& m_run, float& l_run, float scale, const AttnLane& L) {
  constexpr int KT = HD / 32, DT = HD / 16;
  const int base = L.c0 + p * 32;
  // rows at or beyond n_tok were never written (and an invalid page is not ours): 0 * garbage must not
  // become NaN, so clear those V elements.  Only the last pair of a sequence takes this path.
  if (base + 32 > L.n_tok || !f.ok_a || !f.ok_b) {
    const int pos_a = base + 4 * L.g, pos_b = base + 16 + 4 * L.g;
    uint32_t ma0 = 0u, ma1 = 0u, mb0 = 0u, mb1 = 0u;
    if (f.ok_a && pos_a + 0 < L.n_tok) ma0 |= 0x0000FFFFu;
    if (f.ok_a && pos_a + 1 < L.n_tok) ma0 |= 0xFFFF0000u;
    if (f.ok_a && pos_a + 2 < L.n_tok) ma1 |= 0x0000FFFFu;
    if (f.ok_a && pos_a + 3 < L.n_tok) ma1 |= 0xFFFF0000u;
    if (f.ok_b && pos_b + 0 < L.n_tok) mb0 |= 0x0000FFFFu;
    if (f.ok_b && pos_b + 1 < L.n_tok) mb0 |= 0xFFFF0000u;
    if (f.ok_b && pos_b + 2 < L.n_tok) mb1 |= 0x0000FFFFu;
    if (f.ok_b && pos_b + 3 < L.n_tok) mb1 |= 0xFFFF0000u;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      f.v[dt] &= (u32x4){ma0, ma1, mb0, mb1};
    }
  }
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.ka[kt]), __builtin_bit_cast(bf16x8, qf[kt]), sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.kb[kt]), __builtin_bit_cast(bf16x8, qf[kt]), sb, 0, 0, 0);
  }
  const int pa0 = base + 4 * L.g;
  float v0, v1, v2, v3, v4, v5, v6, v7;
#define DF_VIS(ok, pos) ((ok) && (pos) < L.c1 && (pos) <= L.last_vis)
  v0 = DF_VIS(f.ok_a, pa0 + 0) ? sa[0] * scale : -INFINITY;
  v1 = DF_VIS(f.ok_a, pa0 + 1) ? sa[1] * scale : -INFINITY;
  v2 = DF_VIS(f.ok_a, pa0 + 2) ? sa[2] * scale : -INFINITY;
  v3 = DF_VIS(f.ok_a, pa0 + 3) ? sa[3] * scale : -INFINITY;
  v4 = DF_VIS(f.ok_b, pa0 + 16) ? sb[0] * scale : -INFINITY;
  v5 = DF_VIS(f.ok_b, pa0 + 17) ? sb[1] * scale : -INFINITY;
  v6 = DF_VIS(f.ok_b, pa0 + 18) ? sb[2] * scale : -INFINITY;
  v7 = DF_VIS(f.ok_b, pa0 + 19) ? sb[3] * scale : -INFINITY;
#undef DF_VIS
  float mx = fmaxf(fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)), fmaxf(fmaxf(v4, v5), fmaxf(v6, v7)));
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float m_new = fmaxf(m_run, mx);
  // all keys so far masked: exponent base 0 gives exp(-inf) = 0 for every (masked) key and corr 1
  const float mb = (m_new == -INFINITY) ? 0.f : m_new;
  const float corr = (m_run == -INFINITY) ? (m_new == -INFINITY ? 1.f : 0.f) : __expf(m_run - m_new);
  const float p0 = __expf(v0 - mb), p1 = __expf(v1 - mb), p2 = __expf(v2 - mb), p3 = __expf(v3 - mb);
  const float p4 = __expf(v4 - mb), p5 = __expf(v5 - mb), p6 = __expf(v6 - mb), p7 = __expf(v7 - mb);
  l_run = l_run * corr + (((p0 + p1) + (p2 + p3)) + ((p4 + p5) + (p6 + p7)));
  m_run = m_new;
  u32x4 ph, pl;
#define DF_PACK(i, a, b)                                                                        \
  {                                                                                             \
    const bf16_t h0 = float_to_bf16_bits(a), h1 = float_to_bf16_bits(b);                        \
    const bf16_t l0 = float_to_bf16_bits((a) - bf16_bits_to_float(h0));                         \
    const bf16_t l1 = float_to_bf16_bits((b) - bf16_bits_to_float(h1));                         \
    ph[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);                                                \
    pl[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);                                                \
  }
  DF_PACK(0, p0, p1) DF_PACK(1, p2, p3) DF_PACK(2, p4, p5) DF_PACK(3, p6, p7)
#undef DF_PACK
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const u32x4 vf = f.v[dt];
    f32x4 a = acc[dt];
    a[0] *= corr; a[1] *= corr; a[2] *= corr; a[3] *= corr;
    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), __builtin_bit_cast(bf16x8, ph), a, 0, 0, 0);
    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), __builtin_bit_cast(bf16x8, pl), a, 0, 0, 0);
    acc[dt] = a;
  }
}

template <int HD>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ pool,
                                                        SeqGeom geo, AttnArgs aa, float* __restrict__ part_o,
                                                        float2* __restrict__ part_ml) {
  constexpr int KT = HD / 32, DT = HD / 16;
  // grid = (splits, kv heads, parts * sequences): the 2^q_shift workgroups that share a kv head's K/V (each with its
  // share of the query heads) differ in blockIdx.z only, by a multiple of the (even) sequence count, and so land on the
  // same XCD and read the K/V pages through one L2; "kvh" below counts head groups (kv head * parts + part)
  const int n_seq = (int)gridDim.z >> aa.q_shift;
  const int part = aa.q_shift ? (int)blockIdx.z / n_seq : 0;
  const int split = blockIdx.x, kvh = ((int)blockIdx.y << aa.q_shift) + part, s = (int)blockIdx.z - part * n_seq;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int B = geo.block_size;
  const int group = (aa.n_q_heads / aa.n_kv_heads) >> aa.q_shift;   // query heads of this workgroup: blockIdx.y ("kvh") counts such head groups
  const int rows = B * group;
  const int n_s = geo.seq_lens[s];
  const int cap = geo.max_pages_per_seq * DF_PAGE;

  // ---- this lane's query column: row r of the kv head's row set
  const int r = wave * 16 + n;
  const bool valid = r < rows;
  const int slot = valid ? r / group : 0, hq = kvh * group + (valid ? r % group : 0);
  const size_t pr = ((size_t)(s * B + slot) * aa.n_q_heads + hq) * aa.n_splits + split;

  AttnLane L;
  L.table = geo.block_table + (size_t)s * geo.max_pages_per_seq;
  L.n_tok = min(n_s + B, cap);
  L.c0 = split * aa.chunk;
  L.c1 = min(L.n_tok, L.c0 + aa.chunk);
  L.last_vis = valid ? (aa.causal ? n_s + slot : 0x7FFFFFFF) : -1;
  L.g = g;
  L.lane = lane;
  L.kvh = kvh >> aa.q_shift;

  // query fragments (B operand of S^T): lane (n, g) holds Q[row][kt*32 + g*8 .. +8]
  u32x4 qf[KT];
  {
    const u32x4* qp = reinterpret_cast<const u32x4*>(q + ((size_t)(s * B + slot) * aa.n_q_heads + hq) * HD);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) qf[kt] = valid ? qp[kt * 4 + g] : (u32x4){0u, 0u, 0u, 0u};
  }

  float m_run = -INFINITY, l_run = 0.f;   // l_run: this lane's share (its 8 keys per pair) of the row sum
  f32x4 acc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) acc[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int n_pairs = L.c1 > L.c0 ? (L.c1 - L.c0 + 31) >> 5 : 0;
  // Two fragment sets, one multiplied while the other is on its way.  Inside the loop no load is conditional (a
  // load skipped on some path would force every wait to drain all loads in flight); the last one or two pairs
  // are peeled off.
  if (n_pairs > 0) {
    KvFrags<HD> f0, f1;
    attn_load_pair<HD>(f0, 0, pool, geo, aa, L);
    int p = 0;
    for (; p + 2 < n_pairs; p += 2) {
      attn_load_pair<HD>(f1, p + 1, pool, geo, aa, L);
      attn_process_pair<HD>(f0, p, qf, acc, m_run, l_run, aa.scale, L);
      attn_load_pair<HD>(f0, p + 2, pool, geo, aa, L);
      attn_process_pair<HD>(f1, p + 1, qf, acc, m_run, l_run, aa.scale, L);
    }
    if (p + 1 < n_pairs) {
      attn_load_pair<HD>(f1, p + 1, pool, geo, aa, L);
      attn_process_pair<HD>(f0, p, qf, acc, m_run, l_run, aa.scale, L);
      attn_process_pair<HD>(f1, p + 1, qf, acc, m_run, l_run, aa.scale, L);
    } else {
      attn_process_pair<HD>(f0, p, qf, acc, m_run, l_run, aa.scale, L);
    }
  }

  // ---- partial result of this split: (max, sum) and the unnormalised output row -------------------------
  float l = l_run;
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  if (valid) {
    if (g == 0) part_ml[pr] = make_float2(m_run, l);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      *reinterpret_cast<float4*>(part_o + pr * HD + dt * 16 + 4 * g) = make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]);
  }
}

// ------------------------------------------------------------------------------------------------
// Long-chunk variant (hundreds of keys or more per workgroup).  The kernel above keeps only one page pair
// of unique bytes in flight per CU (its four wavefronts read the same keys), which is latency-bound once a
// chunk is long.  Here the four wavefronts split the KEYS instead: wavefront w takes page pairs w, w+4, ...
// of the chunk for all RB = 4 blocks of 16 query rows, each with its own pair in flight (4x the bytes in
// flight, K/V fragments read from HBM exactly once per workgroup), and the four partial (max, sum, O) sets
// are merged through LDS at the end with the same log-sum-exp rule as the cross-split merge.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bf16_pair(float a, float b) {   // RNE, a in the low half
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t r = __builtin_convertvector((f32x2_t){a, b}, bf16x2_t);
  return __builtin_bit_cast(uint32_t, r);
}

template <int HD, int RB>
__device__ __forceinline__ void attn_process_pair_wide(KvFrags<HD>& f, int base, const u32x4* __restrict__ q_lds,
                                                       f32x4 (&acc)[RB][HD / 16], float (&m_run)[RB], float (&l_run)[RB],
                                                       const int (&last_vis)[RB], int n_all_vis, float scale2, const AttnLane& L, f32x4* rescale_lds) {
  constexpr int KT = HD / 32, DT = HD / 16;
  if (base + 32 > L.n_tok || !f.ok_a || !f.ok_b) {   // never-written rows / foreign pages: clear V (0 * garbage != NaN)
    const int pos_a = base + 4 * L.g, pos_b = base + 16 + 4 * L.g;
    uint32_t ma0 = 0u, ma1 = 0u, mb0 = 0u, mb1 = 0u;
    if (f.ok_a && pos_a + 0 < L.n_tok) ma0 |= 0x0000FFFFu;
    if (f.ok_a && pos_a + 1 < L.n_tok) ma0 |= 0xFFFF0000u;
    if (f.ok_a && pos_a + 2 < L.n_tok) ma1 |= 0x0000FFFFu;
    if (f.ok_a && pos_a + 3 < L.n_tok) ma1 |= 0xFFFF0000u;
    if (f.ok_b && pos_b + 0 < L.n_tok) mb0 |= 0x0000FFFFu;
    if (f.ok_b && pos_b + 1 < L.n_tok) mb0 |= 0xFFFF0000u;
    if (f.ok_b && pos_b + 2 < L.n_tok) mb1 |= 0x0000FFFFu;
    if (f.ok_b && pos_b + 3 < L.n_tok) mb1 |= 0xFFFF0000u;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) f.v[dt] &= (u32x4){ma0, ma1, mb0, mb1};
  }
  // every key of the pair visible to every row (the bulk of a long context): no per-element masking
  const bool all_vis = f.ok_a && f.ok_b && base + 32 <= n_all_vis;
  const int pa0 = base + 4 * L.g;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
    u32x4 qf[KT];   // query fragments of this row block, kept in LDS between uses
    asm volatile("" ::: "memory");   // keep these reads inside the loop: hoisted, they would cost 64 registers
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) qf[kt] = q_lds[(rb * KT + kt) * 64 + L.lane];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.ka[kt]), __builtin_bit_cast(bf16x8, qf[kt]), sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.kb[kt]), __builtin_bit_cast(bf16x8, qf[kt]), sb, 0, 0, 0);
    }
    float v[8];   // raw scores q.k; the base-2 exponent domain value is v * scale2, scale2 = log2(e) / sqrt(head_dim) > 0
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = sa[i];
      v[4 + i] = sb[i];
    }
    if (!all_vis) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!(f.ok_a && pa0 + i < L.c1 && pa0 + i <= last_vis[rb])) v[i] = -INFINITY;
        if (!(f.ok_b && pa0 + 16 + i < L.c1 && pa0 + 16 + i <= last_vis[rb])) v[4 + i] = -INFINITY;
      }
    }
    // Lazy reference maximum: m_run only moves when the true row maximum has grown by more than 8 (a factor 256),
    // so the accumulators (which live in the MFMA accumulation registers, out of reach of plain ALU ops) are
    // rescaled once or twice per sweep instead of after every pair.  exp2(v - m_run) <= 256 meanwhile.  A row's
    // maximum has grown that much exactly when the maximum of one of its four lanes has, so the common case is
    // decided from each lane's own scores and the cross-lane exchange happens only inside the rare branch.
    const float lmx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7]))) * scale2;
    const float m_old = m_run[rb];
    if (__builtin_amdgcn_ballot_w64(lmx > m_old + 8.f) != 0ull) {
      float mx = lmx;   // the maximum commutes with the positive scale
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const bool grow = mx > m_old + 8.f;
      const float corr = grow ? (m_old == -INFINITY ? 0.f : exp2f(m_old - mx)) : 1.f;
      l_run[rb] *= corr;
      // through LDS: the accumulators can be stored from and loaded into the accumulation registers directly, so
      // the common path never has to shuttle them to ordinary registers on behalf of this rare one
      f32x4* scr = rescale_lds + L.lane;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) scr[dt * 64] = acc[rb][dt];
      asm volatile("" ::: "memory");
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        f32x4 a = scr[dt * 64];
        a[0] *= corr; a[1] *= corr; a[2] *= corr; a[3] *= corr;
        scr[dt * 64] = a;
      }
      asm volatile("" ::: "memory");
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) acc[rb][dt] = scr[dt * 64];
      if (grow) m_run[rb] = mx;
    }
    const float mb = (m_run[rb] == -INFINITY) ? 0.f : m_run[rb];   // nothing visible yet: exp2(-inf - 0) = 0
    float pe[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pe[i] = __builtin_amdgcn_exp2f(fmaf(v[i], scale2, -mb));   // -inf stays -inf -> 0
    l_run[rb] += ((pe[0] + pe[1]) + (pe[2] + pe[3])) + ((pe[4] + pe[5]) + (pe[6] + pe[7]));
    u32x4 ph, pl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t h = pack_bf16_pair(pe[2 * i], pe[2 * i + 1]);
      ph[i] = h;
      pl[i] = pack_bf16_pair(pe[2 * i] - __uint_as_float(h << 16), pe[2 * i + 1] - __uint_as_float(h & 0xFFFF0000u));
    }
    // all hi products, then all lo products: two MFMAs on the same accumulator are never back to back
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      acc[rb][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.v[dt]), __builtin_bit_cast(bf16x8, ph), acc[rb][dt], 0, 0, 0);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      acc[rb][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.v[dt]), __builtin_bit_cast(bf16x8, pl), acc[rb][dt], 0, 0, 0);
  }
}

template <int HD>
__global__ __launch_bounds__(256, 1) void attn_mfma_wide_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ pool,
                                                                SeqGeom geo, AttnArgs aa, float* __restrict__ part_o,
                                                                float2* __restrict__ part_ml) {
  constexpr int KT = HD / 32, DT = HD / 16, RB = 4, LD = HD + 4;
  __shared__ float2 s_ml[4][64];
  __shared__ __attribute__((aligned(16))) float s_raw[4 * 64 * LD];   // query fragments during the sweep, outputs in the merge
  float (*s_o)[64][LD] = reinterpret_cast<float (*)[64][LD]>(s_raw);
  u32x4* q_lds = reinterpret_cast<u32x4*>(s_raw);                      // [rb][kt][lane]
  int32_t* s_pages = reinterpret_cast<int32_t*>(s_raw) + RB * KT * 64 * 4;   // page ids of this chunk (behind the queries)
  // grid = (splits, kv heads, parts * sequences): the 2^q_shift workgroups that share a kv head's K/V (each with its
  // share of the query heads) differ in blockIdx.z only, by a multiple of the (even) sequence count, and so land on the
  // same XCD and read the K/V pages through one L2; "kvh" below counts head groups (kv head * parts + part)
  const int n_seq = (int)gridDim.z >> aa.q_shift;
  const int part = aa.q_shift ? (int)blockIdx.z / n_seq : 0;
  const int split = blockIdx.x, kvh = ((int)blockIdx.y << aa.q_shift) + part, s = (int)blockIdx.z - part * n_seq;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int B = geo.block_size;
  const int group = (aa.n_q_heads / aa.n_kv_heads) >> aa.q_shift;   // query heads of this workgroup: blockIdx.y ("kvh") counts such head groups
  const int rows = B * group;
  const int n_s = geo.seq_lens[s];
  const int cap = geo.max_pages_per_seq * DF_PAGE;
  // per-wavefront staging for the rare accumulator rescale (behind room for 16384 page ids)
  f32x4* rescale_lds = reinterpret_cast<f32x4*>(s_raw + RB * KT * 64 * 4 + 16384) + wave * (DT * 64);

  AttnLane L;
  L.table = geo.block_table + (size_t)s * geo.max_pages_per_seq;
  L.n_tok = min(n_s + B, cap);
  L.c0 = split * aa.chunk;
  L.c1 = min(L.n_tok, L.c0 + aa.chunk);
  L.last_vis = 0;
  L.g = g;
  L.lane = lane;
  L.kvh = kvh >> aa.q_shift;
  const int n_all_vis = min(L.c1, aa.causal ? n_s : L.n_tok);   // keys below this are visible to every row

  // query fragments of the RB row blocks: lane (n, g) holds Q[row rb*16 + n][kt*32 + g*8 .. +8]; wavefront w
  // stages row block w in LDS for everybody
  int last_vis[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = rb * 16 + n;
    const bool valid = r < rows;
    const int slot = valid ? r / group : 0, hq = kvh * group + (valid ? r % group : 0);
    last_vis[rb] = valid ? (aa.causal ? n_s + slot : 0x7FFFFFFF) : -1;
    if (rb == wave) {
      const u32x4* qp = reinterpret_cast<const u32x4*>(q + ((size_t)(s * B + slot) * aa.n_q_heads + hq) * HD);
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) q_lds[(rb * KT + kt) * 64 + lane] = valid ? qp[kt * 4 + g] : (u32x4){0u, 0u, 0u, 0u};
    }
  }
  // the chunk's slice of the page table: the sweep then never waits on a dependent table load from memory
  {
    const int first = L.c0 >> 4, count = L.c1 > L.c0 ? ((L.c1 - L.c0 + 15) >> 4) : 0;
    for (int i = threadIdx.x; i < count; i += 256) s_pages[i] = L.table[first + i];
  }
  __syncthreads();

  float m_run[RB], l_run[RB];
  f32x4 acc[RB][DT];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = -INFINITY;
    l_run[rb] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[rb][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const int n_pairs = L.c1 > L.c0 ? (L.c1 - L.c0 + 31) >> 5 : 0;
  const float scale2 = aa.scale * 1.44269504088896341f;   // scores and running maxima in the base-2 exponent domain
  auto load = [&](KvFrags<HD>& f, int p) {
    const bool has_b = L.c0 + p * 32 + 16 < L.c1;
    // the same for every lane: tell the compiler, so addresses and validity branches stay scalar
    const int pa = __builtin_amdgcn_readfirstlane(s_pages[2 * p]);
    const int pb = has_b ? __builtin_amdgcn_readfirstlane(s_pages[2 * p + 1]) : pa;
    attn_load_pages<HD, true>(f, pa, pb, has_b, pool, geo, aa, L);
  };
  // Two fragment sets per wavefront; no conditional load inside the loop (see the kernel above), tail peeled off.
  if (wave < n_pairs) {
    KvFrags<HD> f0, f1;
    auto process = [&](KvFrags<HD>& f, int p) {
      attn_process_pair_wide<HD, RB>(f, L.c0 + p * 32, q_lds, acc, m_run, l_run, last_vis, n_all_vis, scale2, L, rescale_lds);
    };
    load(f0, wave);
    int p = wave;
    for (; p + 8 < n_pairs; p += 8) {
      load(f1, p + 4);
      process(f0, p);
      load(f0, p + 8);
      process(f1, p + 4);
    }
    if (p + 4 < n_pairs) {
      load(f1, p + 4);
      process(f0, p);
      process(f1, p + 4);
    } else {
      process(f0, p);
    }
  }

  // ---- merge the four wavefronts' partial results (each over its own keys) --------------------------------
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float l = l_run[rb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (g == 0) s_ml[wave][rb * 16 + n] = make_float2(m_run[rb], l);
  }
  __syncthreads();   // also: every wavefront is done with the query fragments that s_o overlays
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = rb * 16 + n;
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) m_all = fmaxf(m_all, s_ml[w][r].x);
    const float mine = (m_run[rb] == -INFINITY) ? 0.f : exp2f(m_run[rb] - m_all);   // m_all is finite whenever m_run is
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      *reinterpret_cast<float4*>(&s_o[wave][r][dt * 16 + 4 * g]) =
          make_float4(acc[rb][dt][0] * mine, acc[rb][dt][1] * mine, acc[rb][dt][2] * mine, acc[rb][dt][3] * mine);
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * (HD / 4); idx += 256) {
    const int r = idx / (HD / 4), d4 = idx % (HD / 4);
    if (r >= rows) continue;
    const int slot = r / group, hq = kvh * group + r % group;
    const size_t pr = ((size_t)(s * B + slot) * aa.n_q_heads + hq) * aa.n_splits + split;
    float4 o = *reinterpret_cast<const float4*>(&s_o[0][r][d4 * 4]);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float4 a = *reinterpret_cast<const float4*>(&s_o[w][r][d4 * 4]);
      o.x += a.x; o.y += a.y; o.z += a.z; o.w += a.w;
    }
    *reinterpret_cast<float4*>(part_o + pr * HD + d4 * 4) = o;
    if (d4 == 0) {
      float m_all = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) m_all = fmaxf(m_all, s_ml[w][r].x);
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float2 ml = s_ml[w][r];
        l += (ml.x == -INFINITY) ? 0.f : ml.y * exp2f(ml.x - m_all);
      }
      part_ml[pr] = make_float2(m_all * 0.69314718055994531f, l);   // the cross-split merge works with natural exponents
    }
  }
}

// Returns true when it launched a kernel for this configuration; false -> caller uses the generic kernel.
template <typename T>
inline bool attn_mfma_launch(hipStream_t, const T*, const T*, SeqGeom, AttnArgs, int, float*, float2*, int) {
  return false;
}

template <>
inline bool attn_mfma_launch<bf16_t>(hipStream_t st, const bf16_t* q, const bf16_t* pool, SeqGeom geo, AttnArgs aa, int S,
                                     float* part_o, float2* part_ml, int wide_min_chunk) {
  const int rows = (geo.block_size * (aa.n_q_heads / aa.n_kv_heads)) >> aa.q_shift;
  if (rows > 64 || (aa.n_q_heads / aa.n_kv_heads) % (1 << aa.q_shift) || (aa.head_dim != 128 && aa.head_dim != 64)) return false;
  const dim3 grid(aa.n_splits, aa.n_kv_heads, S << aa.q_shift), block(256);
  // long chunks: wavefronts split the keys (the chunk's page ids must fit the kernel's LDS slice)
  if (aa.head_dim == 128 && aa.chunk >= wide_min_chunk && aa.chunk / DF_PAGE + 2 <= 16384)
    hipLaunchKernelGGL(attn_mfma_wide_kernel<128>, grid, block, 0, st, q, pool, geo, aa, part_o, part_ml);
  else if (aa.head_dim == 128)
    hipLaunchKernelGGL(attn_mfma_kernel<128>, grid, block, 0, st, q, pool, geo, aa, part_o, part_ml);
  else
    hipLaunchKernelGGL(attn_mfma_kernel<64>, grid, block, 0, st, q, pool, geo, aa, part_o, part_ml);
  return true;
}
