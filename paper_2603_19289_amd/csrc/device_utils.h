// Device helpers shared by the kernel files: packed 16-byte weight chunks, bf16 rounding,
// wavefront reductions with data-parallel primitives (DPP).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe_spec {

constexpr int kWave = 64;

// 16 bytes of stored weights: 8 bf16 (uint16_t bit patterns) or 4 floats.  Chunks stay packed in
// registers while their loads are in flight and are unpacked to float where they are used.
template <typename WT> struct Packed;
template <> struct Packed<uint16_t> {
  using Raw = uint4;
  static constexpr int N = 8;
  __device__ static __forceinline__ void unpack(const uint4 &v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  // x must already be a bf16 value held in a float
  __device__ static __forceinline__ uint16_t pack_one(float x) { return uint16_t(__float_as_uint(x) >> 16); }
};
template <> struct Packed<float> {
  using Raw = float4;
  static constexpr int N = 4;
  __device__ static __forceinline__ void unpack(const float4 &v, float (&f)[4]) {
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  __device__ static __forceinline__ float pack_one(float x) { return x; }
};

template <typename WT>
__device__ __forceinline__ void load_chunk(const WT *p, float (&f)[Packed<WT>::N]) {
  Packed<WT>::unpack(*reinterpret_cast<const typename Packed<WT>::Raw *>(p), f);
}

// 16-byte load of data that is read once (expert weights streamed from the slots): the
// nontemporal hint keeps such lines from displacing what the caches should hold and measurably
// raises the streaming rate (pure read of 50 MB: 5.0 -> 5.2 TB/s; of 470 MB: 6.3 -> 7.0 TB/s).
typedef __attribute__((ext_vector_type(4))) unsigned int vec4u_t;
template <typename RAW>
__device__ __forceinline__ RAW load_stream(const void *p) {
  static_assert(sizeof(RAW) == 16, "16-byte chunks only");
  const vec4u_t v = __builtin_nontemporal_load(reinterpret_cast<const vec4u_t *>(p));
  return __builtin_bit_cast(RAW, v);
}

// Dot product of one packed weight chunk with one packed activation chunk of the same dtype,
// added to acc in float.  bf16: four two-element dot instructions per 16 bytes (both operands
// stay packed; every product is exact in float).  float: four multiply-adds.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t w, uint32_t a, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w), __builtin_bit_cast(bf16x2_t, a), acc, false);
}

__device__ __forceinline__ float dot_chunk(const uint4 &w, const uint4 &a, float acc) {
  acc = dot2_bf16(w.x, a.x, acc);
  acc = dot2_bf16(w.y, a.y, acc);
  acc = dot2_bf16(w.z, a.z, acc);
  return dot2_bf16(w.w, a.w, acc);
}

__device__ __forceinline__ float dot_chunk(const float4 &w, const float4 &a, float acc) {
  acc += w.x * a.x;
  acc += w.y * a.y;
  acc += w.z * a.z;
  return acc + w.w * a.w;
}


// float -> nearest bfloat16 (ties to even) -> float; finite inputs.
__device__ __forceinline__ float round_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xffff0000u);
}

// double -> nearest bfloat16 (8 significant bits, ties to even), straight from the double so
// that nothing is rounded twice; normal-range inputs.
__device__ __forceinline__ double round_to_bf16(double x) {
  if (x == 0.0) return x;
  int e;
  const double m = frexp(x, &e);
  return ldexp(rint(m * 256.0), e - 8);
}

// The same rounding on the bits of the double: the 45 mantissa bits below bfloat16's seven are
// rounded away to nearest, ties to even (a carry runs into the exponent as it should).  Finite
// inputs whose magnitude is a normal float; zero stays zero.
__device__ __forceinline__ double round_to_bf16_fast(double x) {
  unsigned long long u = static_cast<unsigned long long>(__double_as_longlong(x));
  u += 0x00000fffffffffffull + ((u >> 45) & 1ull);
  u &= ~0x00001fffffffffffull;
  return __longlong_as_double(static_cast<long long>(u));
}

// DPP controls used below: quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.  After the four steps every lane of a row of 16
// holds the row's sum; one lane per row is then read through scalar registers.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, true);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, true);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ float readlane(float v, int src_lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

__device__ __forceinline__ double readlane(double v, int src_lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src_lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src_lane);
  return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes; every lane gets the same value.
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  return (readlane(v, 0) + readlane(v, 16)) + (readlane(v, 32) + readlane(v, 48));
}

// ---- Hand-over slots: "the data is the flag".  A slot of global memory holds all ones (a NaN pattern no
// result can have) until its producer overwrites it with one relaxed device-scope atomic store; consumers read
// it with relaxed device-scope atomic loads until it no longer holds that pattern.  Each slot is a single
// atomic object: nothing has to be ordered against anything else.
constexpr unsigned long long kEmpty64 = ~0ull;

__device__ __forceinline__ void raise_status(unsigned int *status) {      // a word in pinned host memory
  __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ __forceinline__ void publish64(unsigned long long *slot, double v) {
  if (!(v == v)) v = -INFINITY;                // a result that is not a number must not look like an empty slot
  v += 0.0;                                    // -0.0 becomes +0.0: equal logits must be equal bit patterns
  __hip_atomic_store(slot, static_cast<unsigned long long>(__double_as_longlong(v)), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void arm64(unsigned long long *slot) {
  __hip_atomic_store(slot, kEmpty64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ unsigned long long peek64(const unsigned long long *slot) {
  return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits (boundedly) until the slot holds a value.  A look at memory takes about a microsecond to come back;
// four looks are kept in flight 80 ns apart (3 x 64 cycles), so that a value is noticed that soon after it lands
// instead of a whole round trip later (measured on the fused routing launch: 11.2 us with gaps of 1 to 3 units,
// 11.5 with 5, 11.9 with 8, 12.2 with 12).
__device__ __forceinline__ unsigned long long await64(const unsigned long long *slot, unsigned int limit,
                                                      unsigned int *status) {
  unsigned long long v = peek64(slot);
  for (unsigned int spins = 0; v == kEmpty64; spins += 4) {
    if (spins >= limit) { raise_status(status); break; }
    const unsigned long long v0 = peek64(slot);
    __builtin_amdgcn_s_sleep(3);
    const unsigned long long v1 = peek64(slot);
    __builtin_amdgcn_s_sleep(3);
    const unsigned long long v2 = peek64(slot);
    __builtin_amdgcn_s_sleep(3);
    const unsigned long long v3 = peek64(slot);
    if (v0 != kEmpty64) v = v0;
    else if (v1 != kEmpty64) v = v1;
    else if (v2 != kEmpty64) v = v2;
    else v = v3;
  }
  return v;
}

// In-register rank sort of one token's logits.  Every wavefront holds all candidates in
// registers (element i = r*64 + lane, R per lane) and counts, for each of its candidates, how
// many candidates broadcast from source lanes [src_begin, src_end) rank before it: larger logit
// first, equal logits by lower index.  The four wavefronts of the workgroup split the source
// lanes and add their counts in LDS; a candidate's total is its position in the sorted order.
template <int R>
__device__ __forceinline__ void rank_counts(const double (&key)[R], int lane, int src_begin, int src_end,
                                            int (&cnt)[R]) {
#pragma unroll
  for (int r = 0; r < R; ++r) cnt[r] = 0;
  for (int j = src_begin; j < src_end; ++j) {
#pragma unroll
    for (int r2 = 0; r2 < R; ++r2) {
      const double zj = readlane(key[r2], j);
      const int ij = r2 * kWave + j;
#pragma unroll
      for (int r = 0; r < R; ++r)
        cnt[r] += (zj > key[r] || (zj == key[r] && ij < r * kWave + lane)) ? 1 : 0;
    }
  }
}

}  // namespace moe_spec
