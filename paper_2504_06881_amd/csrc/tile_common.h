// Helpers shared by the tiled 3x3 forward kernels (gfx950): lane geometry constants, raw buffer
// loads of x, and the vectorised row stores of the epilogue.
#pragma once
#include <type_traits>

#include "tconv_internal.h"

namespace tconv {
namespace tile {

constexpr int WAVES = 4;  // waves per workgroup, each a different c_out group

// f(integral_constant<int, I>) for I = FIRST, FIRST + STEP, ... below LAST: a loop whose index is a compile-time
// constant in the body whatever the optimiser decides about unrolling
template <int FIRST, int LAST, int STEP, typename F>
__device__ __forceinline__ void static_steps(F&& f) {
  if constexpr (FIRST < LAST) {
    f(std::integral_constant<int, FIRST>{});
    static_steps<FIRST + STEP, LAST, STEP>(f);
  }
}

typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f2u __attribute__((ext_vector_type(2), aligned(4)));

__device__ __forceinline__ float nan_or(float v, unsigned m) {
  return __uint_as_float(__float_as_uint(v) | m);
}

// ---- input loads go through a raw buffer resource: a wave-uniform 128-bit descriptor of the whole x
// tensor in SGPRs, a per-lane 32-bit byte offset in a VGPR and a wave-uniform channel offset in an SGPR
// (buffer_load ... offen).  No 64-bit per-lane address arithmetic, and nothing loop-invariant for
// the compiler to hoist into VGPR pairs.
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// contiguous run of N values starting at byte offset voff (+ uniform soff) -> fp32 registers
template <int N, typename T>
__device__ __forceinline__ void load_run(float* dst, rsrc_t r, unsigned voff, unsigned soff) {
  if constexpr (sizeof(T) == 4) {  // fp32 storage, 4-byte aligned
    if constexpr (N >= 4) {
      const u4v v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
      dst[0] = __uint_as_float(v.x); dst[1] = __uint_as_float(v.y);
      dst[2] = __uint_as_float(v.z); dst[3] = __uint_as_float(v.w);
      load_run<N - 4, T>(dst + 4, r, voff + 16, soff);
    } else if constexpr (N >= 2) {
      const u2v v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
      dst[0] = __uint_as_float(v.x); dst[1] = __uint_as_float(v.y);
      load_run<N - 2, T>(dst + 2, r, voff + 8, soff);
    } else if constexpr (N == 1) {
      dst[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
    }
  } else {  // bf16 storage: 2-byte aligned, widened exactly
#pragma unroll
    for (int i = 0; i < N; ++i)
      dst[i] = __uint_as_float(((unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff + 2 * i, soff, 0)) << 16);
  }
}

// The same loads without the widening: a register receives the stored bits (fp32: the value; bf16: its 16 bits,
// zero-extended), so that no arithmetic instruction follows the load where it is issued; the main loop widens when
// it masks the padding, just before the first use.
template <int N, typename T>
__device__ __forceinline__ void load_raw_run(float* dst, rsrc_t r, unsigned voff, unsigned soff) {
  if constexpr (sizeof(T) == 4) {
    load_run<N, T>(dst, r, voff, soff);
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i)
      dst[i] = __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff + 2 * i, soff, 0));
  }
}

template <typename T>
__device__ __forceinline__ float load_raw_one(rsrc_t r, unsigned voff, unsigned soff) {
  if constexpr (sizeof(T) == 4)
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
  else
    return __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0));
}

template <typename T>
__device__ __forceinline__ float load_one(rsrc_t r, unsigned voff, unsigned soff) {
  if constexpr (sizeof(T) == 4)
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
  else
    return __uint_as_float(((unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0)) << 16);
}

// ---- a lane's NP (4 or 8) consecutive outputs -> memory.  Pixels q < first_q belong to the
// neighbouring lane (shifted last segment of a row): then single predicated stores, else 16-byte stores.
// The (base, off) forms take a wave-uniform base and the lane's 32-bit element offset, which is what a store
// instruction with a scalar base address wants: no 64-bit per-lane address arithmetic.
typedef int i4u __attribute__((ext_vector_type(4), aligned(4)));
typedef unsigned u4h __attribute__((ext_vector_type(4), aligned(2)));
typedef unsigned u2h __attribute__((ext_vector_type(2), aligned(2)));

template <int NP>
__device__ __forceinline__ void store_row(float* p, const float (&v)[NP], int first_q) {
  if (first_q == 0) {
#pragma unroll
    for (int h = 0; h < NP / 4; ++h) {
      f4u a;
      a.x = v[4 * h]; a.y = v[4 * h + 1]; a.z = v[4 * h + 2]; a.w = v[4 * h + 3];
      *(f4u*)(p + 4 * h) = a;
    }
  } else {
#pragma unroll
    for (int q = 0; q < NP; ++q)
      if (q >= first_q) p[q] = v[q];
  }
}

template <int NP>
__device__ __forceinline__ void store_row(int32_t* p, const int (&v)[NP], int first_q) {
  if (first_q == 0) {
#pragma unroll
    for (int h = 0; h < NP / 4; ++h) {
      i4u a;
      a.x = v[4 * h]; a.y = v[4 * h + 1]; a.z = v[4 * h + 2]; a.w = v[4 * h + 3];
      *(i4u*)(p + 4 * h) = a;
    }
  } else {
#pragma unroll
    for (int q = 0; q < NP; ++q)
      if (q >= first_q) p[q] = v[q];
  }
}

__device__ __forceinline__ unsigned bf16_bits(float v) {  // round to nearest even
  unsigned u = __float_as_uint(v);
  if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

template <int NP>
__device__ __forceinline__ void store_row(bf16_t* p, const float (&v)[NP], int first_q) {
  if (first_q == 0) {
#pragma unroll
    for (int h = 0; h < NP / 4; ++h) {
      u2h a;
      a.x = bf16_bits(v[4 * h]) | (bf16_bits(v[4 * h + 1]) << 16);
      a.y = bf16_bits(v[4 * h + 2]) | (bf16_bits(v[4 * h + 3]) << 16);
      *(u2h*)(p + 4 * h) = a;
    }
  } else {
#pragma unroll
    for (int q = 0; q < NP; ++q)
      if (q >= first_q) p[q] = (bf16_t)bf16_bits(v[q]);
  }
}

// element offset -> byte offset in 32 bits (the caller keeps tensors below 4 GiB), added to the uniform base
template <int NP, typename T, typename V>
__device__ __forceinline__ void store_row(T* base, unsigned off, const V (&v)[NP], int first_q) {
  store_row<NP>((T*)((char*)base + (size_t)(off * (unsigned)sizeof(T))), v, first_q);
}

}  // namespace tile
}  // namespace tconv
