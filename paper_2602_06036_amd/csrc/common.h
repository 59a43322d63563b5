// Shared device/host helpers of the DFlash HIP path: storage types, tile and KV-page layouts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // raw bfloat16 bits
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Wavefront index inside a workgroup: kernels compute it as readfirstlane(threadIdx.x >> 6) so that the compiler
// knows it is the same for all 64 lanes; loop bounds, slot numbers and base addresses derived from it then stay
// in scalar registers and the branches on them are plain scalar branches.
#define DF_WAVE 64
#define DF_PAGE 16

__host__ __device__ __forceinline__ float bf16_bits_to_float(bf16_t b) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)b << 16;
  return c.f;
}
// round-to-nearest-even; inputs are finite on this path
__host__ __device__ __forceinline__ bf16_t float_to_bf16_bits(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Store;
template <> struct Store<float> {
  static __host__ __device__ __forceinline__ float from(float f) { return f; }
  static __host__ __device__ __forceinline__ float to(float v) { return v; }
};
template <> struct Store<bf16_t> {
  static __host__ __device__ __forceinline__ bf16_t from(float f) { return float_to_bf16_bits(f); }
  static __host__ __device__ __forceinline__ float to(bf16_t v) { return bf16_bits_to_float(v); }
};

// ---- GEMM weight layout -------------------------------------------------------------------------
// A matrix of N rows x K (K contiguous in the canonical form).  fp32: plain row-major.  bf16: cut into
// 16-row x 32-column tiles; a tile is 1 KB holding, for lane = (k%32)/8*16 + r%16 of a 64-wide
// wavefront, the 8 consecutive k values that lane feeds to v_mfma_f32_16x16x32_bf16.  Tiles are stored
// k-tile-major: all N/16 tiles of k-tile 0, then all tiles of k-tile 1, ...  A wavefront that owns NT
// adjacent row bands reads NT KB contiguously per k step and neighbouring workgroups read the neighbouring
// KBs, so the whole grid sweeps each k slab of the matrix sequentially (DRAM-friendly), instead of
// thousands of independent 1 KB streams.
template <typename T> __host__ __device__ __forceinline__ size_t tile_index(int r, int k, int K, int N);
template <> __host__ __device__ __forceinline__ size_t tile_index<float>(int r, int k, int K, int) {
  return (size_t)r * K + k;
}
template <> __host__ __device__ __forceinline__ size_t tile_index<bf16_t>(int r, int k, int, int N) {
  return ((size_t)(k >> 5) * (N >> 4) + (r >> 4)) * 512 + (size_t)(((((k & 31) >> 3) << 4) + (r & 15)) * 8 + (k & 7));
}
// rows that a buffer in this layout must provide for M logical rows
template <typename T> __host__ __device__ __forceinline__ int tile_rows(int M) { return M; }
template <> __host__ __device__ __forceinline__ int tile_rows<bf16_t>(int M) { return (M + 15) & ~15; }

// ---- GEMM activation operand ---------------------------------------------------------------------
// fp32 models: plain row-major fp32.  bf16 models: every activation that feeds a GEMM is kept as a
// PAIR of bf16 numbers hi + lo (hi = bf16(x), lo = bf16(x - hi)), i.e. ~16 significand bits, and the
// GEMM issues two MFMAs per weight tile.  Single-bf16 inputs make two correct evaluations of the
// same model drift apart by percents of the logit spread (one flipped rounding perturbs every later
// rounding); the pair removes that at no cost while the GEMM is bandwidth-bound.  Layout: the tile
// layout above with the hi tile (1 KB) immediately followed by the lo tile.
template <typename T> struct Act;
template <> struct Act<float> {
  static constexpr int planes = 1;
  static __host__ __device__ __forceinline__ size_t elems(int M, int K) { return (size_t)M * K; }
  static __device__ __forceinline__ void store(float* base, int m, int k, int K, float v) { base[(size_t)m * K + k] = v; }
  // 4 consecutive k (k % 4 == 0)
  static __device__ __forceinline__ void store4(float* base, int m, int k, int K, float4 v) {
    *reinterpret_cast<float4*>(base + (size_t)m * K + k) = v;
  }
};
template <> struct Act<bf16_t> {
  static constexpr int planes = 2;
  static __host__ __device__ __forceinline__ size_t elems(int M, int K) { return (size_t)((M + 15) & ~15) * K * 2; }
  static __host__ __device__ __forceinline__ size_t index(int m, int k, int K) {  // hi element; lo is 512 further
    return ((size_t)(m >> 4) * (K >> 5) + (k >> 5)) * 1024 + (size_t)(((((k & 31) >> 3) << 4) + (m & 15)) * 8 + (k & 7));
  }
  static __device__ __forceinline__ void split(float v, bf16_t& hi, bf16_t& lo) {
    hi = float_to_bf16_bits(v);
    lo = float_to_bf16_bits(v - bf16_bits_to_float(hi));
  }
  static __device__ __forceinline__ void store(bf16_t* base, int m, int k, int K, float v) {
    bf16_t hi, lo;
    split(v, hi, lo);
    const size_t i = index(m, k, K);
    base[i] = hi;
    base[i + 512] = lo;
  }
  static __device__ __forceinline__ void store4(bf16_t* base, int m, int k, int K, float4 v) {
    ushort4 hi, lo;
    split(v.x, hi.x, lo.x);
    split(v.y, hi.y, lo.y);
    split(v.z, hi.z, lo.z);
    split(v.w, hi.w, lo.w);
    const size_t i = index(m, k, K);
    *reinterpret_cast<ushort4*>(base + i) = hi;
    *reinterpret_cast<ushort4*>(base + i + 512) = lo;
  }
};

// ---- KV page layout ----------------------------------------------------------------------------
// A pool holds, per layer, n_pages pages; a page holds for each kv head 16 keys then 16 values:
//   pool[layer][page][kv_head][K|V][16*hd]
// K part: [hd/8][16 keys][8 dims]   -> a 16-key x 32-dim MFMA A-operand tile is 1 KB contiguous
// V part: [hd/16][4][16 dims][4 keys] -> lane (dim%16, key/4) of the P.V MFMA reads 4 keys contiguously
__host__ __device__ __forceinline__ int k_in_page(int key, int d) { return (d >> 3) * 128 + key * 8 + (d & 7); }
__host__ __device__ __forceinline__ int v_in_page(int key, int d) {
  return (d >> 4) * 256 + (key >> 2) * 64 + (d & 15) * 4 + (key & 3);
}
__host__ __device__ __forceinline__ size_t kv_head_base(int layer, int n_pages, int page, int n_kv_heads, int kvh, int hd) {
  return ((((size_t)layer * n_pages + page) * n_kv_heads + kvh) * 2) * (size_t)(DF_PAGE * hd);
}

struct SeqGeom {          // passed by value to kernels that walk the page table
  const int32_t* seq_lens;
  const int32_t* block_table;
  int32_t max_pages_per_seq;
  int32_t n_pages;
  int32_t block_size;
  int32_t* status;        // sticky device status word
};

#define DF_STATUS_CAPACITY 1

__device__ __forceinline__ float wave_reduce_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_reduce_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- counter-based random numbers and the argmax combine rule (shared by the LM-head epilogues and misc.h) ----
// Draws are a hash of (key, sequence, block slot, purpose, index): the same number whichever kernel asks for it.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
// u in (0,1), 23 bits (so that x + 0.5 is exact in fp32): counter c = (((seq*64 + slot)*4 + purpose) << 32) | idx
__device__ __forceinline__ float counter_uniform(uint64_t key, int seq, int slot, int purpose, uint32_t idx) {
  const uint64_t c = ((uint64_t)(((uint32_t)seq * 64u + (uint32_t)slot) * 4u + (uint32_t)purpose) << 32) | idx;
  const uint64_t z = mix64(key + 0x9E3779B97F4A7C15ull * (c + 1ull));
  return ((float)(z >> 41) + 0.5f) * 1.1920928955078125e-7f;  // 2^-23
}
__device__ __forceinline__ float gumbel(float u) { return -logf(-logf(u)); }

__device__ __forceinline__ void argmax_combine(float& bv, int& bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}
