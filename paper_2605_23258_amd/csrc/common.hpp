// Shared device helpers for the gfx950 kernels: element types, 16-byte operand
// chunks for the 32x32 MFMA tiles, and wave-level reductions (wave = 64 lanes).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/vector.h"

namespace vec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage type of VECTOR_BF16 tensors

template <typename T> struct Elem;
template <> struct Elem<float>  { static constexpr int kPerChunk = 4; static constexpr int kDtype = VECTOR_F32; };
template <> struct Elem<bf16_t> { static constexpr int kPerChunk = 8; static constexpr int kDtype = VECTOR_BF16; };

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// two floats -> two bf16 in one word (low half first), round to nearest even, in hardware
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ void store_elem(float* p, float x) { *p = x; }
__device__ __forceinline__ void store_elem(bf16_t* p, float x) { p->bits = f32_to_bf16_bits(x); }

// ---------------------------------------------------------------------------
// Operand chunks.  One 32x32 MFMA tile contracts over head_dim in "chunks": a
// chunk is what the two lane halves of a wave hold for one row in 16 bytes each
// (2 x 8 bf16 or 2 x 4 fp32 elements).  Lane l carries row (l & 31); lane half
// (l >> 5) carries elements [c*2E + half*E, +E) of that row, E = elements per
// 16 bytes.  Both MFMA operands use the same mapping, so the contraction pairs
// equal element indices whatever order the hardware walks them in.
// ---------------------------------------------------------------------------
typedef uint4 chunk_t;

template <typename T> __device__ __forceinline__ constexpr int chunks_per_row(int d) {
  return d / (2 * Elem<T>::kPerChunk);
}

// element offset (within a row) of the 16 bytes lane half `half` holds for chunk c
template <typename T> __device__ __forceinline__ int chunk_elem_offset(int c, int half) {
  return (c * 2 + half) * Elem<T>::kPerChunk;
}

// Workgroups go to the eight XCDs in turn by their linear index (x fastest), and every XCD has an
// L2 of its own.  This permutation of a (chunks, heads) grid puts all chunks of a head on one XCD
// (the heads are dealt out over the XCDs, or the XCDs over a head's chunks when there are fewer
// heads than XCDs): what the head's workgroups share (query rows, W, partial results) is then
// fetched into one L2 instead of eight, and a launch finds what the launch before it wrote
// for the same head in the L2 it was written through.  Any grid it does not divide evenly keeps
// the plain order.
constexpr int kXcds = 8;
__device__ __forceinline__ void xcd_chunk_head(int& chunk, int& h) {
  const int gx = gridDim.x, gy = gridDim.y;
  chunk = blockIdx.x; h = blockIdx.y;
  const int id = chunk + gx * h, x = id % kXcds, k = id / kXcds;
  if (gy % kXcds == 0) {
    h = x + kXcds * (k / gx);
    chunk = k % gx;
  } else if (kXcds % gy == 0 && gx % (kXcds / gy) == 0) {
    const int s = kXcds / gy;                  // XCDs per head
    h = x % gy;
    chunk = (x / gy) * (gx / s) + k;
  }
}

__device__ __forceinline__ chunk_t load_chunk(const void* p) { return *reinterpret_cast<const chunk_t*>(p); }

// acc += A(32 x chunk) * B(chunk x 32): a holds rows of the M side, b rows of the N side.
template <typename T> __device__ __forceinline__ void mma_chunk(f32x16& acc, const chunk_t& a, const chunk_t& b);

template <> __device__ __forceinline__ void mma_chunk<bf16_t>(f32x16& acc, const chunk_t& a, const chunk_t& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ void mma_chunk<float>(f32x16& acc, const chunk_t& a, const chunk_t& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// acc = A * B for the first chunk of a contraction: the zero goes in as the MFMA's
// constant C operand instead of sixteen register moves.
template <typename T> __device__ __forceinline__ void mma_chunk_first(f32x16& acc, const chunk_t& a, const chunk_t& b);
template <> __device__ __forceinline__ void mma_chunk_first<bf16_t>(f32x16& acc, const chunk_t& a, const chunk_t& b) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), zero, 0, 0, 0);
}
template <> __device__ __forceinline__ void mma_chunk_first<float>(f32x16& acc, const chunk_t& a, const chunk_t& b) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), zero, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// Row of the 32x32 accumulator tile that register v of this lane holds
// (column = lane & 31).
__device__ __forceinline__ int acc_row(int v, int lane_half) { return (v >> 2) * 8 + lane_half * 4 + (v & 3); }

// 16 bytes of a row -> floats (8 for bf16, 4 for fp32)
template <typename T> struct Unpack16;
template <> struct Unpack16<bf16_t> {
  static __device__ __forceinline__ void run(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
  }
};
template <> struct Unpack16<float> {
  static __device__ __forceinline__ void run(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

// ---------------------------------------------------------------------------
// wave reductions
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
  return x;
}
__device__ __forceinline__ int wave_sum_i(int x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}
// inclusive prefix sum across the 64 lanes
__device__ __forceinline__ int wave_incl_scan_i(int x, int lane) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    int y = __shfl_up(x, o, kWave);
    if (lane >= o) x += y;
  }
  return x;
}

// Smallest / largest of a value over the wave on the DPP network (no LDS traffic); every lane
// gets the result.  Lanes that a step does not feed take the identity (`idle`).
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_take_f(float idle, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(idle), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_min_dpp(float v) {
  v = fminf(v, dpp_take_f<0x111, 0xf>(INFINITY, v));   // row_shr:1 .. 8: lane 15 of each row of 16 holds the row's
  v = fminf(v, dpp_take_f<0x112, 0xf>(INFINITY, v));
  v = fminf(v, dpp_take_f<0x114, 0xf>(INFINITY, v));
  v = fminf(v, dpp_take_f<0x118, 0xf>(INFINITY, v));
  v = fminf(v, dpp_take_f<0x142, 0xa>(INFINITY, v));   // row_bcast:15 into rows 1 and 3
  v = fminf(v, dpp_take_f<0x143, 0xc>(INFINITY, v));   // row_bcast:31 into rows 2 and 3: lane 63 holds the wave's
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_dpp(float v) {
  v = fmaxf(v, dpp_take_f<0x111, 0xf>(-INFINITY, v));
  v = fmaxf(v, dpp_take_f<0x112, 0xf>(-INFINITY, v));
  v = fmaxf(v, dpp_take_f<0x114, 0xf>(-INFINITY, v));
  v = fmaxf(v, dpp_take_f<0x118, 0xf>(-INFINITY, v));
  v = fmaxf(v, dpp_take_f<0x142, 0xa>(-INFINITY, v));
  v = fmaxf(v, dpp_take_f<0x143, 0xc>(-INFINITY, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float wave_sum_dpp(float v) {    // one fixed order of additions: the same bits every time
  v += dpp_take_f<0x111, 0xf>(0.f, v);
  v += dpp_take_f<0x112, 0xf>(0.f, v);
  v += dpp_take_f<0x114, 0xf>(0.f, v);
  v += dpp_take_f<0x118, 0xf>(0.f, v);
  v += dpp_take_f<0x142, 0xa>(0.f, v);
  v += dpp_take_f<0x143, 0xc>(0.f, v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------------------
// Rotary position embedding of cached keys (Section 3.1, RoPE decoupling): the value map
// was fitted on keys as projected, so a cached key is turned back by its position before
// the map is applied.  Frequencies travel as turns (cycles) per position, split into two
// floats (48 bits together); position * frequency is reduced to its fractional turn with an
// exact product (fma) so that the angle is good to about 2^-24 of a turn for any position
// below 2^24.  The hardware sine and cosine take their argument in turns.
// ---------------------------------------------------------------------------
constexpr int kMaxRotaryPairs = 64;      // head_dim / 2 at head_dim = 128

struct RopeParams {
  float turns_hi[kMaxRotaryPairs];       // inv_freq[i] / (2 pi), leading 24 bits
  float turns_lo[kMaxRotaryPairs];       // the next 24 bits
  const int32_t* positions;              // device, or null: the row index
  int32_t pos_offset;
  int32_t interleaved;                   // 0: pair i = (x[i], x[i + d/2]); 1: pair i = (x[2i], x[2i + 1])
};

// (cos, sin) of position * frequency; pos_f = the position as a float (exact below 2^24)
__device__ __forceinline__ void rotary_cos_sin(float pos_f, float t_hi, float t_lo, float& c, float& s) {
  const float p = pos_f * t_hi;
  const float err = fmaf(pos_f, t_hi, -p);                 // exact: the bits the product dropped
  const float u = __builtin_amdgcn_fractf(p) + fmaf(pos_f, t_lo, err);
  c = __builtin_amdgcn_cosf(u);
  s = __builtin_amdgcn_sinf(u);
}
// the inverse rotation of one pair
__device__ __forceinline__ void rotary_back(float a, float b, float c, float s, float& a_pre, float& b_pre) {
  a_pre = fmaf(a, c, b * s);
  b_pre = fmaf(b, c, -(a * s));
}

constexpr float kLog2e = 1.4426950408889634f;

}  // namespace vec
