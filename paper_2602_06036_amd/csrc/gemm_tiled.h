// Compute-bound GEMM for many activation rows (M > 64): y[M,N] = a[M,K] * W[N,K]^T, bf16 MFMA 16x16x32 with
// hi+lo activation pairs, fp32 accumulation, the same operand layouts and epilogues as the streaming kernel.
//
// A workgroup of 2*WY wavefronts (WY = 2 or 4 along N x 2 along M) owns a tile of WY*WN weight row bands x 2*WM
// activation row bands for one K range (grid.y).  Both operands already sit in HBM in MFMA fragment order (1 KB per
// 16x32 fragment), so a k tile is staged by copying whole fragments: global -> registers (PD k tiles in flight)
// -> one of two LDS slots; every wavefront reads the WN weight and 2*WM activation fragments of its part of the tile
// (each lane its own 16 bytes: conflict-free ds_read_b128) and issues WN*WM*2 MFMAs per k tile.  The eight-wavefront
// form (WY = 4) is two four-wavefront workgroups fused along N: one activation stage for twice the weight rows,
// i.e. a third less operand traffic from L2 per flop, at one workgroup per CU.
// Schedule of a k tile, register-staged variant (NS = 2; one barrier per k tile, order pinned with scheduling
// barriers): barrier -> all WN + 2*WM fragment reads of the k tile -> the LDS writes of the next k tile (from
// registers loaded PD k tiles earlier) and the global loads of k tile t+1+PD -> the WN*WM*2 MFMAs.  LDS operations
// of a wavefront complete in order and a 1 KB ds_write occupies the LDS path several times longer than a read, so
// the reads go first: the MFMAs wait for the reads only and the writes drain behind the MFMA stream; the second
// workgroup on the CU fills the gaps around the barrier.
// Ring variant (NS >= 3): the k tiles arrive by direct-to-LDS loads, see the comment at the loop.  It is used where
// NS slots fit next to a second workgroup on the CU (128 x 128 and the 64-row tiles) and for the 128-row tiles of
// an unsplit GEMM whose workgroups each have a CU to themselves.
//
// Workgroup order: consecutive workgroup ids go to different XCDs (round-robin dispatch), so id = 8*j + x
// is mapped to weight band block 8*(j / m_blocks) + x and activation block j % m_blocks: the workgroups that
// re-read one weight block run back to back on one XCD and share its L2.
#pragma once
#include "gemm.h"

template <int WN, int WM, int PD, int EPI, int NS = 2, bool GRP = false, int WY = 2>
__global__ __launch_bounds__(128 * WY, (WY == 2 && NS * (2 * WN + 4 * WM) <= 80 ? 2 : 1)) void gemm_bf16_tiled_kernel(
    const bf16_t* __restrict__ W, const bf16_t* __restrict__ A, int M, int N, int K, int n_blocks, int m_blocks, EpiArgs ep) {
  constexpr int NWV = 2 * WY;                       // wavefronts: WY along N x 2 along M
  constexpr int BNT = WY * WN, BMT = 2 * WM;        // fragments of a stage: BNT weight + 2*BMT activation (hi, lo)
  constexpr int FR = BNT + 2 * BMT, PER = FR / NWV; // fragments copied by each wavefront
  static_assert(WN % 2 == 0 && WM % 2 == 0 && FR % NWV == 0 && (PD == 1 || PD == 2) && NS >= 2 && NS * FR <= 160 && (WY == 2 || WY == 4),
                "tile shape");
  __shared__ u32x4 stage[NS][FR][64];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), wy = wave >> 1, wx = wave & 1;
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  int nb = (j / m_blocks) * 8 + xcd, mb = j % m_blocks;
  const int KT = K >> 5, n_tiles = N >> 4;
  int m_tiles = (M + 15) >> 4, mt0 = mb * BMT;
  if constexpr (GRP) {
    // grouped launch (routed experts, see EpiArgs): m_blocks counts work items of up to BMT bands; the workgroups of
    // one item (its n_blocks weight blocks) run back to back on one XCD and share the item's activation rows there
    mb = (j / n_blocks) * 8 + xcd;
    nb = j % n_blocks;
    if (mb >= m_blocks) return;
    const int4 item = ep.grp_items[mb];
    if (item.x < 0) return;
    W += (size_t)item.x * ep.grp_w_stride;
    mt0 = item.y;
    m_tiles = item.z;
  }
  if (nb >= n_blocks) return;                      // whole workgroup leaves before any barrier
  const int ks = gridDim.y, kz = blockIdx.y;
  const int per = (KT + ks - 1) / ks;
  const int kb = min(KT, kz * per), ke = min(KT, kb + per);
  const int nt0 = nb * BNT;

  // the PER fragments this wavefront copies per stage: offset at k tile 0 and stride per k tile (u32x4 units)
  size_t g_off[PER];
  int g_step[PER];
  const u32x4* g_base[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int f = wave * PER + i;
    if (f < BNT) {   // weight fragment: bands past the matrix alias the last band (never stored)
      g_base[i] = reinterpret_cast<const u32x4*>(W);
      g_off[i] = (size_t)min(nt0 + f, n_tiles - 1) * 64 + lane;
      g_step[i] = n_tiles * 64;
    } else {         // activation fragment: band (f - BNT) / 2, plane (f - BNT) % 2
      const int a = f - BNT;
      g_base[i] = reinterpret_cast<const u32x4*>(A);
      g_off[i] = (size_t)min(mt0 + (a >> 1), m_tiles - 1) * KT * 128 + (a & 1) * 64 + lane;
      g_step[i] = 128;
    }
  }
  auto load_global = [&](u32x4 (&g)[PER], int kt) {
#pragma unroll
    for (int i = 0; i < PER; ++i) g[i] = g_base[i][g_off[i] + (size_t)kt * g_step[i]];
  };
  auto write_lds = [&](int slot, const u32x4 (&g)[PER]) {
#pragma unroll
    for (int i = 0; i < PER; ++i) stage[slot][wave * PER + i][lane] = g[i];
  };

  f32x4 acc[WN][WM];
#pragma unroll
  for (int i = 0; i < WN; ++i)
#pragma unroll
    for (int jj = 0; jj < WM; ++jj) acc[i][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (kb < ke) {
   if constexpr (NS == 2) {
    u32x4 g[PD][PER];   // k tiles t+1 .. t+PD on their way from global memory while k tile t is multiplied
    load_global(g[0], kb);
    write_lds(0, g[0]);
#pragma unroll
    for (int d = 0; d < PD; ++d) load_global(g[d], min(kb + 1 + d, ke - 1));

    // One k tile out of LDS slot S0; k tile t+1 goes from register set G into the other slot meanwhile.
    // Order inside a k tile, pinned with scheduling barriers: barrier (k tile t is complete in S0, everybody is done
    // with the other slot) -> all fragment reads of the k tile -> the LDS writes of k tile t+1 and the global loads
    // of k tile t+1+PD -> the MFMAs.  LDS operations of a wavefront complete in order, so the reads must be issued
    // before the (slow) writes: the MFMAs then wait for the reads only, and the writes drain behind the MFMA stream.
    // Straight-line body: past the end of the K range the global loads repeat the last k tile and the write fills a
    // slot nobody reads any more.
    auto k_tile = [&](auto s0_c, auto g_c, int kt) {
      constexpr int s0 = decltype(s0_c)::value, s1 = s0 ^ 1, G = decltype(g_c)::value;
      u32x4 wf[WN], ap[WM][2];
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < WN; ++i) wf[i] = stage[s0][wy * WN + i][lane];
#pragma unroll
      for (int jj = 0; jj < WM; ++jj) {
        ap[jj][0] = stage[s0][BNT + 2 * (wx * WM + jj)][lane];
        ap[jj][1] = stage[s0][BNT + 2 * (wx * WM + jj) + 1][lane];
      }
      __builtin_amdgcn_sched_barrier(0);
      write_lds(s1, g[G]);
      load_global(g[G], min(kt + 1 + PD, ke - 1));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jj = 0; jj < WM; ++jj) {
#pragma unroll
        for (int i = 0; i < WN; ++i)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]), __builtin_bit_cast(bf16x8, ap[jj][0]),
                                                               acc[i][jj], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < WN; ++i)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]), __builtin_bit_cast(bf16x8, ap[jj][1]),
                                                               acc[i][jj], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using IG = std::integral_constant<int, PD - 1>;
    int kt = kb;
    for (; kt + 1 < ke; kt += 2) {
      k_tile(I0{}, I0{}, kt);
      k_tile(I1{}, IG{}, kt + 1);
    }
    if (kt < ke) k_tile(I0{}, I0{}, kt);
   } else {
    // ---- ring of NS LDS slots filled by direct-to-LDS loads (global_load_lds_dwordx4: every lane's 16 bytes go
    // straight to consecutive LDS addresses, which is exactly a fragment in operand order) -------------------
    // No staging registers, no ds_write (a 1 KB ds_write holds up the wavefront's SIMD several times longer than the
    // issue of such a load), k tiles t+1 .. t+NS-1 in flight while k tile t is multiplied.  The loads are inline
    // assembly so that the compiler does not count them: it would otherwise wait for ALL of them before every LDS
    // read.  Completion is tracked by hand: each wavefront issues PER loads per k tile, in order, so "at most
    // PER*(NS-2) outstanding" means its share of k tile t has landed; the barrier extends that to the whole
    // workgroup and also says that everybody is done reading k tile t-1, whose slot is refilled next.
    const unsigned lds_base = (unsigned)(size_t)&stage[0][0][0];
    auto dma_tile = [&](int slot, int kt) {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const u32x4* src = g_base[i] + g_off[i] + (size_t)kt * g_step[i];
        const unsigned dst = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)((slot * FR + wave * PER + i) * 1024));
        // m0 carries the LDS address; whatever the compiler keeps in it is put back, so the statement clobbers nothing
        unsigned keep_m0;
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_nop 0\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep_m0)
                     : "s"(dst), "v"(src)
                     : "memory");
      }
    };
#pragma unroll
    for (int d = 0; d < NS - 1; ++d) dma_tile(d, min(kb + d, ke - 1));
    int slot = 0;
    for (int kt = kb; kt < ke; ++kt) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER * (NS - 2)) : "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      u32x4 wf[WN], ap[WM][2];
      const u32x4* sp = &stage[0][0][0] + (size_t)slot * (FR * 64) + lane;
#pragma unroll
      for (int i = 0; i < WN; ++i) wf[i] = sp[(wy * WN + i) * 64];
#pragma unroll
      for (int jj = 0; jj < WM; ++jj) {
        ap[jj][0] = sp[(BNT + 2 * (wx * WM + jj)) * 64];
        ap[jj][1] = sp[(BNT + 2 * (wx * WM + jj) + 1) * 64];
      }
      // past the end of the K range the last k tile is fetched again into a slot nobody reads any more
      dma_tile(slot == 0 ? NS - 1 : slot - 1, min(kt + NS - 1, ke - 1));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jj = 0; jj < WM; ++jj) {
#pragma unroll
        for (int i = 0; i < WN; ++i)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]), __builtin_bit_cast(bf16x8, ap[jj][0]),
                                                               acc[i][jj], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < WN; ++i)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]), __builtin_bit_cast(bf16x8, ap[jj][1]),
                                                               acc[i][jj], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      slot = slot == NS - 1 ? 0 : slot + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be on its way into LDS when the slots are reused or released
   }
  }

  // lane l holds y[m = band*16 + l%16][n = tile*16 + 4*(l/16) .. +3]
  const int mrow = lane & 15, gq = lane >> 4;
#pragma unroll
  for (int jj = 0; jj < WM; ++jj) {
    const int mt = mt0 + wx * WM + jj, m = mt * 16 + mrow;
    if (mt >= m_tiles || m >= M) continue;
    if (EPI == EPI_SWIGLU) {
      bf16_t* act = reinterpret_cast<bf16_t*>(ep.act);
#pragma unroll
      for (int p = 0; p < WN / 2; ++p) {
        const int nt = nt0 + wy * WN + 2 * p;      // gate tile; the up tile follows it
        if (nt + 1 >= n_tiles) continue;
        const f32x4 gs = acc[2 * p][jj], us = acc[2 * p + 1][jj];
        Act<bf16_t>::store4(act, m, (nt >> 1) * 16 + 4 * gq, ep.act_K,
                            make_float4(silu_f(gs[0]) * us[0], silu_f(gs[1]) * us[1], silu_f(gs[2]) * us[2], silu_f(gs[3]) * us[3]));
      }
    } else {
#pragma unroll
      for (int i = 0; i < WN; ++i) {
        const int nt = nt0 + wy * WN + i;
        if (nt >= n_tiles || !ep.out) continue;
        const f32x4 s = acc[i][jj];
        *reinterpret_cast<float4*>(ep.out + (size_t)kz * ep.slab + (size_t)m * ep.ld + nt * 16 + 4 * gq) = make_float4(s[0], s[1], s[2], s[3]);
      }
    }
  }
  if (EPI == EPI_STORE && ep.amax) {   // fused argmax over this workgroup's columns (host guarantees a single K range)
    __syncthreads();                   // the staging slots are free now: reuse them for the two N halves' bests
    float2* wbest = reinterpret_cast<float2*>(&stage[0][0][0]);   // [wy][BMT * 16 rows]: the bests of the WY column groups
    const uint64_t key = ep.amax_mode ? ep.amax_key[0] : 0ull;
#pragma unroll
    for (int jj = 0; jj < WM; ++jj) {
      const int mt = mt0 + wx * WM + jj, m = mt * 16 + mrow;
      float bv = -INFINITY;
      int bi = 0x7FFFFFFF;
#pragma unroll
      for (int i = 0; i < WN; ++i) {
        const int nt = nt0 + wy * WN + i;
        if (nt >= n_tiles) continue;
        const int col = nt * 16 + 4 * gq;
#pragma unroll
        for (int e = 0; e < 4; ++e) argmax_combine(bv, bi, amax_score(ep, key, acc[i][jj][e], m, col + e), col + e);
      }
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        argmax_combine(bv, bi, ov, oi);
      }
      if (gq == 0) wbest[wy * (BMT * 16) + (wx * WM + jj) * 16 + mrow] = make_float2(bv, __int_as_float(bi));
    }
    __syncthreads();
    for (int r = threadIdx.x; r < BMT * 16; r += 64 * NWV) {
      const int m = mt0 * 16 + r;
      if (m >= M) continue;
      float bv = wbest[r].x;
      int bi = __float_as_int(wbest[r].y);
#pragma unroll
      for (int y = 1; y < WY; ++y) argmax_combine(bv, bi, wbest[y * BMT * 16 + r].x, __float_as_int(wbest[y * BMT * 16 + r].y));
      ep.amax[(size_t)m * n_blocks + nb] = make_float2(bv, __int_as_float(bi));
    }
  }
  if (EPI == EPI_STORE && ep.lse) {   // fused softmax statistics over this workgroup's columns (single K range)
    __syncthreads();                  // the staging slots (and the argmax scratch in them) are free now
    float2* wl = reinterpret_cast<float2*>(&stage[0][0][0]);   // [wy][BMT * 16 rows]
#pragma unroll
    for (int jj = 0; jj < WM; ++jj) {
      float lm = -INFINITY, ls = 0.f;
#pragma unroll
      for (int i = 0; i < WN; ++i) {
        if (nt0 + wy * WN + i >= n_tiles) continue;
        lse_add4(lm, ls, make_float4(acc[i][jj][0], acc[i][jj][1], acc[i][jj][2], acc[i][jj][3]), ep.lse_inv_T);
      }
      lse_combine_row(lm, ls);
      if (gq == 0) wl[wy * (BMT * 16) + (wx * WM + jj) * 16 + mrow] = make_float2(lm, ls);
    }
    __syncthreads();
    for (int r = threadIdx.x; r < BMT * 16; r += 64 * NWV) {
      const int m = mt0 * 16 + r;
      if (m >= M) continue;
      float lm = wl[r].x, ls = wl[r].y;
#pragma unroll
      for (int y = 1; y < WY; ++y) lse_combine(lm, ls, wl[y * BMT * 16 + r].x, wl[y * BMT * 16 + r].y);
      ep.lse[(size_t)m * n_blocks + nb] = make_float2(lm, ls);
    }
  }
}
