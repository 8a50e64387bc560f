// Device-side helpers shared by the A2SF kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace a2sf {

typedef uint16_t bf16_t;  // storage type of bf16 elements (bit pattern)

constexpr int kWave = 64;
constexpr int kThreads = 256;  // every kernel here runs 4 waves per workgroup
constexpr int kWaves = kThreads / kWave;

// ---- element conversion ----------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// round to nearest even; inputs are finite in every caller
__device__ __forceinline__ uint32_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// two floats -> packed bf16 pair (lo in bits 0..15), hardware round-to-nearest-even
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerLane = 4;  // elements in one 16-byte access
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ void store(float* p, float x) { *p = x; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPerLane = 8;
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xFFFF0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xFFFF0000u);
  }
  __device__ static __forceinline__ void store(bf16_t* p, float x) { *p = (bf16_t)f32_to_bf16(x); }
};

// 16 bytes of packed elements from EPL floats (inverse of Elem<T>::unpack)
__device__ __forceinline__ uint4 pack16(const float* f, float) {
  return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
}
__device__ __forceinline__ uint4 pack16(const float* f, bf16_t) {
  return make_uint4(pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7]));
}

// ---- lane exchanges ---------------------------------------------------------------------
// Reductions over the wave stay in the vector pipe: inside a row of 16 lanes DPP lane
// permutations folded into the operation (quad swaps, then mirrors inside half rows and rows:
// a mirror pairs each lane with one holding the other half's partial result), across rows the
// two swap instructions of gfx950 (odd with even rows of 16 lanes, upper with lower half of
// the wave).  A butterfly through the LDS crossbar (ds_bpermute) costs ~100 cycles of latency
// per step instead of a handful.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
// the value of lane l ^ 16 / l ^ 32
__device__ __forceinline__ uint32_t lane_xor16_u32(uint32_t v) {
  const u32x2_t r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return ((threadIdx.x >> 4) & 1) ? r[0] : r[1];   // r[0] = rows (0,0,2,2), r[1] = rows (1,1,3,3)
}
__device__ __forceinline__ uint32_t lane_xor32_u32(uint32_t v) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return ((threadIdx.x >> 5) & 1) ? r[0] : r[1];   // r[0] = halves (lo, lo), r[1] = (hi, hi)
}
// op(v of this lane, v of the partner lane) for commutative op, both steps across rows
template <typename Op>
__device__ __forceinline__ float across_rows(float v, Op op, bool rows16, bool halves) {
  if (rows16) {
    const u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
  if (halves) {
    const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
  return v;
}
struct OpAdd { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };

// Sum over aligned groups of N consecutive lanes (N = 8, 16, 32 or 64); every lane of a
// group gets the group's total.
template <int N>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_move<0xB1>(v);                  // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);                  // quad_perm [2,3,0,1]
  if (N >= 8) v += dpp_move<0x141>(v);     // row_half_mirror
  if (N >= 16) v += dpp_move<0x140>(v);    // row_mirror
  return across_rows(v, OpAdd(), N >= 32, N >= 64);
}

// ---- ordering ---------------------------------------------------------------------------
// Monotone map float -> uint32 (larger float = larger key); -0 is folded onto +0.
__device__ __forceinline__ uint32_t ordered_key(float s) {
  uint32_t u = __float_as_uint(s + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---- wave / block reductions ------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  return across_rows(v, OpMax(), true, true);
}
__device__ __forceinline__ float wave_sum(float v) { return group_sum<64>(v); }
__device__ __forceinline__ int wave_sum_i(int v) {
  uint32_t u = (uint32_t)v;
  u += dpp_move_u32<0xB1>(u);
  u += dpp_move_u32<0x4E>(u);
  u += dpp_move_u32<0x141>(u);
  u += dpp_move_u32<0x140>(u);
  u32x2_t r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  u = r[0] + r[1];
  r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return (int)(r[0] + r[1]);
}
__device__ __forceinline__ int wave_max_i(int v) {
  v = ::max(v, (int)dpp_move_u32<0xB1>((uint32_t)v));
  v = ::max(v, (int)dpp_move_u32<0x4E>((uint32_t)v));
  v = ::max(v, (int)dpp_move_u32<0x141>((uint32_t)v));
  v = ::max(v, (int)dpp_move_u32<0x140>((uint32_t)v));
  u32x2_t r = __builtin_amdgcn_permlane16_swap((uint32_t)v, (uint32_t)v, false, false);
  v = ::max((int)r[0], (int)r[1]);
  r = __builtin_amdgcn_permlane32_swap((uint32_t)v, (uint32_t)v, false, false);
  return ::max((int)r[0], (int)r[1]);
}
// lane `src` (the same for the whole wave) hands its value to every lane
__device__ __forceinline__ float wave_broadcast(float v, int src) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), __builtin_amdgcn_readfirstlane(src)));
}
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
  uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
  const auto take = [&](uint32_t olo, uint32_t ohi) {
    const unsigned long long other = ((unsigned long long)ohi << 32) | olo;
    const unsigned long long mine = ((unsigned long long)hi << 32) | lo;
    if (other < mine) { lo = olo; hi = ohi; }
  };
  take(dpp_move_u32<0xB1>(lo), dpp_move_u32<0xB1>(hi));
  take(dpp_move_u32<0x4E>(lo), dpp_move_u32<0x4E>(hi));
  take(dpp_move_u32<0x141>(lo), dpp_move_u32<0x141>(hi));
  take(dpp_move_u32<0x140>(lo), dpp_move_u32<0x140>(hi));
  take(lane_xor16_u32(lo), lane_xor16_u32(hi));
  take(lane_xor32_u32(lo), lane_xor32_u32(hi));
  return ((unsigned long long)hi << 32) | lo;
}

// Block-wide reductions over 4 waves; `red` is a shared array of >= 8 floats / u64.
// All threads get the result.  Contain two barriers each.
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ int block_sum_i(int v, int* red) {
  v = wave_sum_i(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ unsigned long long block_min_u64(unsigned long long v,
                                                            unsigned long long* red) {
  v = wave_min_u64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long a = red[0] < red[1] ? red[0] : red[1];
  unsigned long long b = red[2] < red[3] ? red[2] : red[3];
  return a < b ? a : b;
}

// Row window and exponent slope of one head's forgotten score (Section 3.3 Eq.5): rows before
// `first_row` have a weight alpha^(n-1-i) below the smallest fp32 subnormal and add exactly 0.
// On entry first_row / log2_alpha are the host's values for its bound alpha_max (log2_alpha is 0
// for both alpha_max = 1, with first_row 0, and alpha_max = 0, with first_row n-1).  With
// alpha_heads the head's own factor narrows the window; a factor above the bound is computed
// as the bound.
__device__ __forceinline__ void head_window(const float* alpha_heads, int g, int n, int& first_row,
                                            float& log2_alpha) {
  if (!alpha_heads) return;  // host values apply to every head
  const float a = alpha_heads[g];
  if (!(a > 0.f)) { first_row = n - 1; log2_alpha = 0.f; return; }   // alpha = 0: the newest row only
  if (log2_alpha == 0.f && first_row >= n - 1) return;               // bound is 0 (or n = 1)
  float l2 = a < 1.f ? log2f(a) : 0.f;
  if (log2_alpha < 0.f) l2 = fminf(l2, log2_alpha);                  // bound below 1: clamp
  log2_alpha = l2;
  if (l2 == 0.f) return;                                             // alpha = 1 under a bound of 1: all rows
  const float rows = 160.0f / (-l2);
  const int own = rows >= (float)n ? 0 : n - ((int)rows + 1);
  first_row = own > first_row ? own : first_row;
}

__device__ __forceinline__ uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// 16 bytes that are read once and not again soon (the streamed rows of a KV cache): the
// non-temporal hint keeps them from displacing other lines on their way through the caches.
// Measured on MI355X with reads of 1.7 GB: 7.0-7.1 TB/s with the hint, 6.2-6.3 TB/s without.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
template <bool STREAM>
__device__ __forceinline__ uint4 load16_as(const void* p) {
  return STREAM ? load16_stream(p) : load16(p);
}
__device__ __forceinline__ void store16(void* p, const uint4& v) { *reinterpret_cast<uint4*>(p) = v; }

}  // namespace a2sf
