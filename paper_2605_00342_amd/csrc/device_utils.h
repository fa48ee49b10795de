// Device-side helpers: storage-type traits (fp32 / bf16), MFMA wrappers for gfx950,
// wavefront reductions, an LDS-only barrier.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evict {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

struct F32 { typedef float elem; static constexpr int kBytes = 4; static constexpr int kBlockElems = 16; };
struct BF16 { typedef uint16_t elem; static constexpr int kBytes = 2; static constexpr int kBlockElems = 32; };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round-to-nearest-even, by the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// two values rounded and packed into one dword (lo in the low half): one instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const bf16x2_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

template <typename ST> __device__ __forceinline__ float load_elem(const void* p, size_t i);
template <> __device__ __forceinline__ float load_elem<F32>(const void* p, size_t i) { return ((const float*)p)[i]; }
template <> __device__ __forceinline__ float load_elem<BF16>(const void* p, size_t i) { return bf16_to_f32(((const uint16_t*)p)[i]); }

template <typename ST> __device__ __forceinline__ void store_elem(void* p, size_t i, float v);
template <> __device__ __forceinline__ void store_elem<F32>(void* p, size_t i, float v) { ((float*)p)[i] = v; }
template <> __device__ __forceinline__ void store_elem<BF16>(void* p, size_t i, float v) { ((uint16_t*)p)[i] = f32_to_bf16(v); }

// value after rounding to the storage type
template <typename ST> __device__ __forceinline__ float round_store(float v);
template <> __device__ __forceinline__ float round_store<F32>(float v) { return v; }
template <> __device__ __forceinline__ float round_store<BF16>(float v) { return bf16_to_f32(f32_to_bf16(v)); }

// Store 4 consecutive elements (16-byte aligned destination for fp32, 8-byte for bf16).
template <typename ST> __device__ __forceinline__ void store4(void* p, size_t i, f32x4 v);
template <> __device__ __forceinline__ void store4<F32>(void* p, size_t i, f32x4 v) {
  *reinterpret_cast<f32x4*>((float*)p + i) = v;
}
template <> __device__ __forceinline__ void store4<BF16>(void* p, size_t i, f32x4 v) {
  uint2 o;
  o.x = pack_bf16x2(v[0], v[1]);
  o.y = pack_bf16x2(v[2], v[3]);
  *reinterpret_cast<uint2*>((uint16_t*)p + i) = o;
}
template <typename ST> __device__ __forceinline__ f32x4 load4(const void* p, size_t i);
template <> __device__ __forceinline__ f32x4 load4<F32>(const void* p, size_t i) {
  return *reinterpret_cast<const f32x4*>((const float*)p + i);
}
template <> __device__ __forceinline__ f32x4 load4<BF16>(const void* p, size_t i) {
  uint2 o = *reinterpret_cast<const uint2*>((const uint16_t*)p + i);
  f32x4 v;
  v[0] = __uint_as_float(o.x << 16); v[1] = __uint_as_float(o.x & 0xFFFF0000u);
  v[2] = __uint_as_float(o.y << 16); v[3] = __uint_as_float(o.y & 0xFFFF0000u);
  return v;
}

// One 1 KiB operand block: each lane holds 16 bytes. With A[m][k] (16 rows) and B[k][n]
// (16 columns), lane l carries row/column l%16 and the (l/16)-th quarter of the block's
// contraction range; both operands use the same mapping so any k order cancels out.
template <typename ST> __device__ __forceinline__ f32x4 mfma_block(u32x4 a, u32x4 b, f32x4 c);
template <> __device__ __forceinline__ f32x4 mfma_block<BF16>(u32x4 a, u32x4 b, f32x4 c) {
  union { u32x4 u; bf16x8 v; } ua, ub;
  ua.u = a; ub.u = b;
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua.v, ub.v, c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mfma_block<F32>(u32x4 a, u32x4 b, f32x4 c) {
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[0]), __uint_as_float(b[0]), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[1]), __uint_as_float(b[1]), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[2]), __uint_as_float(b[2]), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[3]), __uint_as_float(b[3]), c, 0, 0, 0);
  return c;
}

// Wavefront-wide sum / maximum of a float through DPP row operations (no LDS traffic): butterflies
// inside each row of 16 lanes, then row broadcasts into the later rows; the total ends up in the
// last lane and is returned to every lane as a scalar. Lanes a step leaves out read the identity.
#define EVICT_DPP_F32(old_, v_, ctrl_, rows_) \
  __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old_), __float_as_int(v_), ctrl_, rows_, 0xF, false))
__device__ __forceinline__ float wave_sum(float v) {
  v += EVICT_DPP_F32(0.0f, v, 0xB1, 0xF);   // quad_perm [1,0,3,2]
  v += EVICT_DPP_F32(0.0f, v, 0x4E, 0xF);   // quad_perm [2,3,0,1]
  v += EVICT_DPP_F32(0.0f, v, 0x141, 0xF);  // row_half_mirror
  v += EVICT_DPP_F32(0.0f, v, 0x140, 0xF);  // row_mirror
  v += EVICT_DPP_F32(0.0f, v, 0x142, 0xA);  // row_bcast:15 into rows 1, 3
  v += EVICT_DPP_F32(0.0f, v, 0x143, 0xC);  // row_bcast:31 into rows 2, 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0xB1, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x4E, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x141, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x140, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x142, 0xA));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x143, 0xC));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Sum / maximum over each row of 16 lanes, result in every lane of the row (four DPP butterflies).
__device__ __forceinline__ float row16_sum(float v) {
  v += EVICT_DPP_F32(0.0f, v, 0xB1, 0xF);
  v += EVICT_DPP_F32(0.0f, v, 0x4E, 0xF);
  v += EVICT_DPP_F32(0.0f, v, 0x141, 0xF);
  v += EVICT_DPP_F32(0.0f, v, 0x140, 0xF);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0xB1, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x4E, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x141, 0xF));
  v = fmaxf(v, EVICT_DPP_F32(-INFINITY, v, 0x140, 0xF));
  return v;
}

// Wavefront-wide maximum of an unsigned value through DPP row operations (no LDS traffic):
// butterflies inside each row of 16 lanes, then row broadcasts; the result is read from the
// last lane as a scalar. (Lanes a DPP step leaves out read 0, the identity of an unsigned maximum,
// which lets the compiler fold each step into a single v_max_u32 with a DPP operand.)
__device__ __forceinline__ unsigned wave_max_u32(unsigned v) {
  auto mx = [](unsigned a, unsigned b) { return a > b ? a : b; };
  v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));  // row_mirror
  v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false));  // row_bcast:15 into rows 1, 3
  v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false));  // row_bcast:31 into rows 2, 3
  return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

// Token count of a call: the host's T, or -- when the caller has pointed the context at a device word
// (evict_dynamic_tokens) -- the value found there when the kernel runs, clamped to [1, T] (T is then the
// upper bound every grid and buffer was sized for).
__device__ __forceinline__ int dyn_tokens(const int* t_dev, int t_max) {
  if (!t_dev) return t_max;
  const int v = *t_dev;
  return v < 1 ? 1 : (v > t_max ? t_max : v);
}

// Workgroup barrier that waits for LDS traffic only, so that global loads already in
// flight (weight prefetch) stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace evict
