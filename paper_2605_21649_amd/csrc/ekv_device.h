// Device-side helpers shared by the gfx950 kernels: 16-byte row loads, wavefront (64-lane)
// reductions built on DPP row operations, order-preserving float<->uint keys.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ekv {

constexpr int kD = 128;            // head_dim the kernels are written for
constexpr int kLanesPerRow = 16;   // 16 lanes x 8 channels cover one 128-channel row
constexpr int kRowsPerWave = 4;    // a 64-lane wavefront covers 4 rows per step
constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even float -> bf16 bits (finite inputs; NaN is kept quiet)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Wave-uniform read of an int32 in device memory that nothing in the running launch writes (page lists, block
// table, lengths written by earlier launches): a load through the constant address space with a uniform address
// is a scalar load, which does not queue behind the vector loads in flight and costs no vector register.
typedef const int32_t __attribute__((address_space(4)))* const_i32_ptr;
__device__ __forceinline__ int32_t uniform_load(const int32_t* p) { return *(const_i32_ptr)(uintptr_t)p; }

// Load 8 consecutive channels (one lane's share of a 128-channel row) as float.
template <typename T> __device__ __forceinline__ void load8(const T* p, float (&x)[8]);

template <> __device__ __forceinline__ void load8<float>(const float* p, float (&x)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
  x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float (&x)[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);     // one 16-byte load: 8 bf16
  x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xffff0000u);
  x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xffff0000u);
  x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xffff0000u);
  x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xffff0000u);
}

// The same 8 channels kept as loaded (16 or 32 bytes), to be widened only where they are consumed:
// a batch of rows in flight then costs 4 (bf16) or 8 (f32) registers per row, not 8 floats.
template <typename T> struct Raw8;
template <> struct Raw8<float> { float4 a, b; };
template <> struct Raw8<bf16_t> { uint4 a; };
__device__ __forceinline__ void load_raw8(const float* p, Raw8<float>& r) {
  r.a = *reinterpret_cast<const float4*>(p);
  r.b = *reinterpret_cast<const float4*>(p + 4);
}
__device__ __forceinline__ void load_raw8(const bf16_t* p, Raw8<bf16_t>& r) { r.a = *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void widen8(const Raw8<float>& r, float (&x)[8]) {
  x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w;
  x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
}
__device__ __forceinline__ void widen8(const Raw8<bf16_t>& r, float (&x)[8]) {
  x[0] = __uint_as_float(r.a.x << 16); x[1] = __uint_as_float(r.a.x & 0xffff0000u);
  x[2] = __uint_as_float(r.a.y << 16); x[3] = __uint_as_float(r.a.y & 0xffff0000u);
  x[4] = __uint_as_float(r.a.z << 16); x[5] = __uint_as_float(r.a.z & 0xffff0000u);
  x[6] = __uint_as_float(r.a.w << 16); x[7] = __uint_as_float(r.a.w & 0xffff0000u);
}

template <typename T> __device__ __forceinline__ void store8(T* p, const float (&x)[8]);

template <> __device__ __forceinline__ void store8<float>(float* p, const float (&x)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}

template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t* p, const float (&x)[8]) {
  uint4 a;
  a.x = float_to_bf16_bits(x[0]) | ((uint32_t)float_to_bf16_bits(x[1]) << 16);
  a.y = float_to_bf16_bits(x[2]) | ((uint32_t)float_to_bf16_bits(x[3]) << 16);
  a.z = float_to_bf16_bits(x[4]) | ((uint32_t)float_to_bf16_bits(x[5]) << 16);
  a.w = float_to_bf16_bits(x[6]) | ((uint32_t)float_to_bf16_bits(x[7]) << 16);
  *reinterpret_cast<uint4*>(p) = a;
}

// ---- 8-bit bounds: OCP E4M3 (bias 7, 3 mantissa bits, subnormals, max 448, 0x7f = NaN) -----------
// Directed rounding of a float: UP gives the code of the smallest format value >= x, otherwise of the
// largest <= x; the NaN code when no finite format value qualifies (or x is NaN).
template <bool UP> __device__ __forceinline__ uint32_t f32_to_e4m3_directed(float x) {
  const uint32_t bits = __float_as_uint(x);
  const uint32_t sign = bits >> 31, abits = bits & 0x7fffffffu;
  const float a = __uint_as_float(abits);
  const bool away = UP ? sign == 0u : sign != 0u;        // the magnitude is rounded up
  if (!(a <= 448.0f)) return (a != a || away) ? 0x7fu : ((sign << 7) | 0x7eu);
  uint32_t mag;
  if (a < 0.015625f) {                                   // below 2^-6: multiples of 2^-9 (codes 0..8)
    const float s = a * 512.0f, f = floorf(s);
    mag = (uint32_t)f + ((away && s != f) ? 1u : 0u);
  } else {
    uint32_t t = abits & ~0xfffffu;                      // three mantissa bits kept
    if (away && t != abits) t += 0x100000u;              // next format value; a carry moves to the next binade
    mag = (t >> 20) - (120u << 3);                       // exponent field = float exponent - 127 + 7
  }
  return (sign << 7) | mag;
}

// One 16-byte unit of the 8-bit bounds: k_min of 8 channels (rounded down), then k_max (rounded up).
__device__ __forceinline__ void store_box8_unit(uint8_t* p, const float (&mn)[8], const float (&mx)[8]) {
  uint4 u;
  u.x = f32_to_e4m3_directed<false>(mn[0]) | (f32_to_e4m3_directed<false>(mn[1]) << 8) |
        (f32_to_e4m3_directed<false>(mn[2]) << 16) | (f32_to_e4m3_directed<false>(mn[3]) << 24);
  u.y = f32_to_e4m3_directed<false>(mn[4]) | (f32_to_e4m3_directed<false>(mn[5]) << 8) |
        (f32_to_e4m3_directed<false>(mn[6]) << 16) | (f32_to_e4m3_directed<false>(mn[7]) << 24);
  u.z = f32_to_e4m3_directed<true>(mx[0]) | (f32_to_e4m3_directed<true>(mx[1]) << 8) |
        (f32_to_e4m3_directed<true>(mx[2]) << 16) | (f32_to_e4m3_directed<true>(mx[3]) << 24);
  u.w = f32_to_e4m3_directed<true>(mx[4]) | (f32_to_e4m3_directed<true>(mx[5]) << 8) |
        (f32_to_e4m3_directed<true>(mx[6]) << 16) | (f32_to_e4m3_directed<true>(mx[7]) << 24);
  *reinterpret_cast<uint4*>(p) = u;
}

// ---- DPP cross-lane moves (no LDS traffic) -------------------------------------------------
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL> __device__ __forceinline__ int dpp_move_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}

// Sum over each aligned group of 16 lanes (a DPP "row"); every lane of the row gets the total.
// Fixed butterfly order: xor 1, xor 2, half-row mirror, row mirror.
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return v;
}

// Wavefront reductions: DPP butterflies inside each 16-lane row, then the two cross-row DPP broadcasts
// (lane 15 of a row into the next row, lane 31 into the upper half), which leave the result in lane 63;
// it is returned to every lane through a scalar register.  No LDS traffic, fixed order.  All 64 lanes of
// the wavefront must be active at the call (every call site is wavefront-uniform).
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_rows(float old, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK> __device__ __forceinline__ int dpp_rows_i(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  v += dpp_rows<0x142, 0xa>(0.f, v);     // row_bcast15 into rows 1 and 3
  v += dpp_rows<0x143, 0xc>(0.f, v);     // row_bcast31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  v = fmaxf(v, dpp_rows<0x142, 0xa>(v, v));
  v = fmaxf(v, dpp_rows<0x143, 0xc>(v, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ int wave_sum_i(int v) {
  v += dpp_move_i<0xB1>(v);
  v += dpp_move_i<0x4E>(v);
  v += dpp_move_i<0x141>(v);
  v += dpp_move_i<0x140>(v);
  v += dpp_rows_i<0x142, 0xa>(0, v);
  v += dpp_rows_i<0x143, 0xc>(0, v);
  return __builtin_amdgcn_readlane(v, 63);
}

// Block-wide reductions through a small LDS array (one slot per wavefront); all threads get the
// result.  The combination order is fixed (wavefront 0,1,2,...), so results are reproducible.
// `buf` must hold blockDim.x/64 floats and must not be in use by a pending reduction.
__device__ __forceinline__ float block_sum(float v, float* buf) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += buf[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* buf) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[w] = v;
  __syncthreads();
  float t = buf[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, buf[i]);
  return t;
}
__device__ __forceinline__ int block_sum_i(int v, int* buf) {
  v = wave_sum_i(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[w] = v;
  __syncthreads();
  int t = 0;
  for (int i = 0; i < nw; ++i) t += buf[i];
  return t;
}

// Exclusive prefix over `U` counts produced by `count_of(u)`, written to pre[0..U] (pre[U] = total); `wsum` holds
// one int per wavefront.  Called by every thread of the workgroup.
template <int THREADS, typename F>
__device__ __forceinline__ void block_exclusive_prefix(int U, F&& count_of, int* pre, int* wsum) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (U <= THREADS) {
    // one unit per thread (the usual launch): a wavefront scan, the wavefront totals, two barriers; every workgroup
    // of the launch runs this before its first load, so it is kept to a few dozen instructions
    const int c = tid < U ? count_of(tid) : 0;
    int inc = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(inc, d); if (lane >= d) inc += t; }
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    int base = inc - c;
#pragma unroll
    for (int i = 0; i < THREADS / 64; ++i) base += i < w ? wsum[i] : 0;
    if (tid < U) pre[tid] = base;
    if (tid == U - 1) pre[U] = base + c;
    __syncthreads();
    return;
  }
  for (int u = tid; u < U; u += THREADS) pre[u] = count_of(u);
  __syncthreads();
  const int upt = (U + THREADS - 1) / THREADS;          // a contiguous segment per thread
  const int s0 = min(tid * upt, U), s1 = min(s0 + upt, U);
  int s = 0;
  for (int u = s0; u < s1; ++u) s += pre[u];
  int inc = s;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(inc, d); if (lane >= d) inc += t; }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  int base = inc - s;
  for (int i = 0; i < w; ++i) base += wsum[i];
  for (int u = s0; u < s1; ++u) { const int c = pre[u]; pre[u] = base; base += c; }
  if (tid == THREADS - 1) pre[U] = base;                // the last segment ends at U
  __syncthreads();
}

// Order-preserving map float -> uint32 (larger float <=> larger key); -inf maps near 0.
__device__ __forceinline__ uint32_t float_to_key(float f) {
  const uint32_t u0 = __float_as_uint(f);
  const uint32_t u = u0 == 0x80000000u ? 0u : u0;        // -0.0 and +0.0 are one value (a tie), not two
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// x^beta for x > 0 with the small integer exponents special-cased (exact products).
__device__ __forceinline__ float pow_beta(float x, float beta, int ibeta) {
  switch (ibeta) {
    case 1: return x;
    case 2: return x * x;
    case 3: return x * x * x;
    case 4: { const float y = x * x; return y * y; }
    default: return __builtin_exp2f(beta * __builtin_log2f(x));
  }
}
// x^(beta-1)
__device__ __forceinline__ float pow_beta_m1(float x, float beta, int ibeta) {
  switch (ibeta) {
    case 1: return 1.f;
    case 2: return x;
    case 3: return x * x;
    case 4: return x * x * x;
    default: return __builtin_exp2f((beta - 1.f) * __builtin_log2f(x));
  }
}

}  // namespace ekv
