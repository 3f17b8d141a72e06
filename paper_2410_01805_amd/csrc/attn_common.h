// Pieces shared by the bf16 MFMA attention kernels: vector types, bf16 packing, the half-wave
// max exchange and the LDS tile layout.
#pragma once
#include "device_util.h"

namespace locret {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int KT = 64;   // keys per tile
constexpr float RESCALE_LOG2 = 8.f;
// The matrix-core kernels raise a query's running max only when its probability sum over one key tile reaches this
// (2^30): probabilities are formed against a max that may be up to 30 binary orders too low, which float32
// accumulators and bf16 probabilities (same exponent range) hold with room to spare (2^30 * 2^15 keys * |v| << 2^127),
// and which any overflow also trips.  At 2^8 the path was taken in a quarter of the tiles of a workload whose
// large logits arrive late (keys planted 4x larger), each time rescaling the accumulators and redoing the tile's
// exponentials.
constexpr float RESCALE_SUM = 1073741824.f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 x = {a, b};
  bf16x2 y = __builtin_convertvector(x, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
  return *(uint32_t*)&y;
}

// max over the two half-waves: after the swap one register holds the low half's value in both
// halves and the other the high half's
__device__ __forceinline__ float max_across_halves(float x) {
  uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int D>
struct AttnSmem {
  static constexpr int KSTR = D + 8;                 // bf16 elements per K row
  static constexpr int VSTR = KT + 8;                // bf16 elements per V^T row
  bf16_t K[2][KT * KSTR];
  bf16_t Vt[2][D * VSTR];
};

template <int I> struct IntC { static constexpr int value = I; };

}  // namespace locret
