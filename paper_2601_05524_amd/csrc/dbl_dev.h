// Device-side helpers shared by the HIP kernels of libdbl (gfx950 / CDNA4 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dbl {

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int WAVE = 64;
constexpr int TILE_N = 16;   // output features per MFMA tile
constexpr int TILE_K = 32;   // contraction elements per tile block
constexpr int BLOCK_ELEMS = TILE_N * TILE_K;  // 512 elements per weight block

// KV cache layout, per (sequence, kv head): max_ctx * head_dim elements each for K and V, both
// stored in the order the attention kernel's MFMA operands want them, so that every wave-level
// load is 1 KiB (bf16) of consecutive memory -- 8 full cache lines instead of 16 half-used ones.
//   K: tiles of 16 tokens x 32 dims; inside a tile lane l = 16*(d%32/8) + t%16 owns its 8 dims.
//   V: tiles of 32 tokens x 16 dims (V^T is the operand); lane l = 16*(t%16/4) + d%16 owns tokens
//      {4q .. 4q+3} and {16+4q .. 16+4q+3} of the tile (q = t%16/4), in that order.
// t = position in the sequence, d = dim, hd = head_dim; max_ctx is a multiple of 64.
// Paged cache: a page holds KV_PAGE consecutive positions of every kv head in the same tiled
// order (t = position inside the page); KV_PAGE is a multiple of both tile lengths, so a
// 32-token attention step never straddles two pages.
constexpr int KV_PAGE = 256;
__host__ __device__ inline size_t kc_offset(int t, int d, int hd) {
  return ((size_t)((t >> 4) * (hd >> 5) + (d >> 5)) * 64 + (((d & 31) >> 3) * 16 + (t & 15))) * 8 + (d & 7);
}
__host__ __device__ inline size_t vt_offset(int t, int d, int hd) {
  const int tt = t & 31;
  return ((size_t)((t >> 5) * (hd >> 4) + (d >> 4)) * 64 + (((tt & 15) >> 2) * 16 + (d & 15))) * 8 + ((tt >> 4) * 4 + (tt & 3));
}

// Activations of passes with more than 16 rows (inputs of gemm_rows_kernel) are stored as the
// MFMA B fragments that kernel loads: blocks of 16 rows x 32 inputs, lane l = 16*(k%32/8) + m%16
// owns its 8 inputs, block (m/16, k/32) at ((m/16) * (ld/32) + k/32) * 512.  ld = row length in
// elements (a multiple of 32); the buffer holds a multiple of 16 rows.
__host__ __device__ inline size_t xt_offset(int m, int k, int ld) {
  return ((size_t)((m >> 4) * (ld >> 5) + (k >> 5)) * 64 + (((k & 31) >> 3) * 16 + (m & 15))) * 8 + (k & 7);
}

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even float -> bfloat16
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats -> packed bf16 pair (x in the low half), round-to-nearest-even (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float x, float y) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x, y}, bf16x2_t));
}
// two floats -> packed fp16 pair (x in the low half), round-to-nearest-even (v_cvt_pk_f16_f32)
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ uint32_t pack_f16(float x, float y) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x, y}, f16x2_t));
}
// a packed bf16 pair as a packed fp16 pair: exact for magnitudes in [2^-14, 65504] (fp16 has the longer
// significand), smaller ones lose bits or vanish, larger ones saturate at 65504
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u)));
}
// 2^x by the hardware instruction (about 1 ulp; -inf -> 0)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float to_f(bf16_t v) { return bf2f(v); }
  static __device__ __forceinline__ bf16_t from_f(float f) { return f2bf(f); }
};
template <> struct Elem<float> {
  static __device__ __forceinline__ float to_f(float v) { return v; }
  static __device__ __forceinline__ float from_f(float f) { return f; }
};

// ---------------------------------------------------------------------------
// MFMA fragments.  A fragment is the 8 contraction elements one lane contributes
// to a 16 x 16 x 32 tile product: lane l = 16*g + r holds, for tile row r (of A)
// or tile column r (of B), the elements k = 8*g .. 8*g+7 of the 32-wide block.
// bf16: one v_mfma_f32_16x16x32_bf16.  fp32: eight v_mfma_f32_16x16x4_f32, the
// e-th using element e of every lane (lane group g supplies k-index g of that
// instruction), so both types share one data layout.
// Result lane l holds D[4*g + i][r], i = 0..3.
// ---------------------------------------------------------------------------
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { u32x4 v; };
template <> struct Frag<float> { f32x4 lo, hi; };

__device__ __forceinline__ void frag_zero(Frag<bf16_t>& f) { f.v = u32x4{0, 0, 0, 0}; }
__device__ __forceinline__ void frag_zero(Frag<float>& f) { f.lo = f32x4{0, 0, 0, 0}; f.hi = f.lo; }

__device__ __forceinline__ f32x4 mma(const Frag<bf16_t>& a, const Frag<bf16_t>& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a.v),
                                                 __builtin_bit_cast(bf16x8, b.v), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma(const Frag<float>& a, const Frag<float>& b, f32x4 c) {
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.x, b.lo.x, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.y, b.lo.y, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.z, b.lo.z, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.w, b.lo.w, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.x, b.hi.x, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.y, b.hi.y, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.z, b.hi.z, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.w, b.hi.w, c, 0, 0, 0);
  return c;
}

// swap lanes c and c^8 inside every 16-lane row (DPP row rotate by 8)
__device__ __forceinline__ uint32_t dpp_swap8(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128 /* row_ror:8 */, 0xf, 0xf, false);
}
__device__ __forceinline__ Frag<bf16_t> frag_swap_halves(const Frag<bf16_t>& f) {
  Frag<bf16_t> r;
  r.v = u32x4{dpp_swap8(f.v.x), dpp_swap8(f.v.y), dpp_swap8(f.v.z), dpp_swap8(f.v.w)};
  return r;
}
__device__ __forceinline__ Frag<float> frag_swap_halves(const Frag<float>& f) {
  Frag<float> r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r.lo[i] = __uint_as_float(dpp_swap8(__float_as_uint(f.lo[i])));
    r.hi[i] = __uint_as_float(dpp_swap8(__float_as_uint(f.hi[i])));
  }
  return r;
}

// four values rounded to the element type, stored contiguously
__device__ __forceinline__ void st_round4(float* p, const f32x4& v) { *reinterpret_cast<f32x4*>(p) = v; }
__device__ __forceinline__ void st_round4(bf16_t* p, const f32x4& v) {
  *reinterpret_cast<u32x2*>(p) = u32x2{pack_bf16(v.x, v.y), pack_bf16(v.z, v.w)};
}
// one value rounded to the element type
__device__ __forceinline__ void st_round1(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_round1(bf16_t* p, float v) { *p = f2bf(v); }

// 8 consecutive elements of a row-major array (16-byte aligned for bf16, 32 for fp32)
__device__ __forceinline__ Frag<bf16_t> frag_load_row(const bf16_t* p) {
  Frag<bf16_t> f;
  f.v = *reinterpret_cast<const u32x4*>(p);
  return f;
}
__device__ __forceinline__ Frag<float> frag_load_row(const float* p) {
  Frag<float> f;
  f.lo = *reinterpret_cast<const f32x4*>(p);
  f.hi = *reinterpret_cast<const f32x4*>(p + 4);
  return f;
}

// ---------------------------------------------------------------------------
// Tiled weight storage.  A logical [N][K] matrix is cut into blocks of 16 output
// features x 32 inputs; block (t, kb) sits at element offset (t*KBp + kb) * 512.
// Inside a bf16 block lane l's 8 elements are contiguous (16 B per lane, 1 KiB per
// wave load).  Inside an fp32 block the two 16-byte halves of each lane's
// fragment are stored as two 1 KiB planes, so every wave load is again 1 KiB
// contiguous.  These two functions are the single definition of that layout.
// ---------------------------------------------------------------------------
template <typename T>
__host__ __device__ inline size_t tiled_offset(int row, int k, int KBp);
template <>
__host__ __device__ inline size_t tiled_offset<bf16_t>(int row, int k, int KBp) {
  const int t = row >> 4, r = row & 15, kb = k >> 5, kk = k & 31, g = kk >> 3, e = kk & 7;
  return ((size_t)t * KBp + kb) * BLOCK_ELEMS + (size_t)(g * 16 + r) * 8 + e;
}
template <>
__host__ __device__ inline size_t tiled_offset<float>(int row, int k, int KBp) {
  const int t = row >> 4, r = row & 15, kb = k >> 5, kk = k & 31, g = kk >> 3, e = kk & 7;
  return ((size_t)t * KBp + kb) * BLOCK_ELEMS + (size_t)(e >> 2) * 256 + (size_t)(g * 16 + r) * 4 + (e & 3);
}

// streaming (non-temporal) load of one lane's fragment of weight block `blk`
__device__ __forceinline__ Frag<bf16_t> frag_load_w(const bf16_t* W, size_t blk, int lane) {
  Frag<bf16_t> f;
  f.v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(W + blk * BLOCK_ELEMS) + lane);
  return f;
}
__device__ __forceinline__ Frag<float> frag_load_w(const float* W, size_t blk, int lane) {
  Frag<float> f;
  const f32x4* p = reinterpret_cast<const f32x4*>(W + blk * BLOCK_ELEMS);
  f.lo = __builtin_nontemporal_load(p + lane);
  f.hi = __builtin_nontemporal_load(p + 64 + lane);
  return f;
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11)
// ---------------------------------------------------------------------------
struct Philox4 { uint32_t x, y, z, w; };

__host__ __device__ inline Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return Philox4{c0, c1, c2, c3};
}

// uniform in (0,1) from the top 23 bits
__device__ __forceinline__ float u01(uint32_t x) { return ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f); }
// standard Gumbel noise
__device__ __forceinline__ float gumbel(uint32_t x) { return -logf(-logf(u01(x))); }

// (value, id) ordering used for every arg-max: larger value first, then lower id
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
  return v > bv || (v == bv && i < bi);
}

}  // namespace dbl
