// Pieces shared by the matrix-core variants of the fused apply pass (fp32 MFMA and split-fp16 MFMA):
// lane/unit mapping of the 32x32 MFMA accumulator, the lane-half swap, the hoisting of the
// row/column-constant features and the per-tile LDS set-up.
#pragma once

#include "lopt_internal.h"
#include "lopt_device.h"

namespace lopt {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void swap32(unsigned& a, unsigned& b) {
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}

// Eight swaps (register i with register 4+i of both arrays) and two swaps as single asm blocks: the
// wait states are needed only before the first and after the last swap of a block, and every
// s_nop costs an issue slot.
__device__ __forceinline__ void swap32x8(unsigned (&h)[8], unsigned (&l)[8]) {
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %4\n\tv_permlane32_swap_b32 %1, %5\n\t"
      "v_permlane32_swap_b32 %2, %6\n\tv_permlane32_swap_b32 %3, %7\n\t"
      "v_permlane32_swap_b32 %8, %12\n\tv_permlane32_swap_b32 %9, %13\n\t"
      "v_permlane32_swap_b32 %10, %14\n\tv_permlane32_swap_b32 %11, %15\n\ts_nop 1"
      : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]), "+v"(h[7]),
        "+v"(l[0]), "+v"(l[1]), "+v"(l[2]), "+v"(l[3]), "+v"(l[4]), "+v"(l[5]), "+v"(l[6]), "+v"(l[7]));
}

__device__ __forceinline__ void swap32x2(float& a0, float& b0, float& a1, float& b1) {
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\ts_nop 1"
      : "+v"(a0), "+v"(b0), "+v"(a1), "+v"(b1));
}

__device__ __forceinline__ void swap32(float& a, float& b) {
  // v_permlane32_swap: a.hi <-> b.lo, i.e. afterwards a = [a.lo | b.lo], b = [a.hi | b.hi]
  // (lo = lanes 0..31). Written as inline assembly because the compiler's builtin returns the first
  // result twice (checked on ROCm 7.2); the s_nop pairs cover the VALU <-> permlane-swap wait states
  // that the compiler cannot see inside an asm block.
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}

__device__ __forceinline__ int unit_of(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// ReLU as one integer max on the bit pattern (negative floats are negative integers); fmaxf costs
// two instructions because of its NaN canonicalisation.
__device__ __forceinline__ float relu(float x) {
  const int i = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(float, i > 0 ? i : 0);
}

constexpr int kNF = LOPT_N_ELEM_FEATS;  // 28
constexpr int kH = 32;
constexpr int kNE = 16;  // features that vary per element and go through the matrix cores

// Feature indices by kind. The 12 features that are constant along a row (r_k, 1/sqrt(r_k)) or along
// a column (c_k, 1/sqrt(c_k)) do not need a per-element contraction: their first-layer contribution
// is a 32-vector per row plus a 32-vector per column, added as the C operand of layer 1.
__device__ __forceinline__ constexpr int elem_feat(int i) { return i < 13 ? i : 12 + i; }          // 0..12, 25..27
__device__ __forceinline__ constexpr int row_feat(int i) { return i < 3 ? 13 + i : 16 + i; }       // 13..15, 19..21
__device__ __forceinline__ constexpr int col_feat(int i) { return i < 3 ? 16 + i : 19 + i; }       // 16..18, 22..24

struct ApplyLds {
  float4 colv[4][2][4][64];  // [unit group q][half][element e of the lane][lane]: units 8q+4half..+3
  float4 w1row[6][2][4];     // [row feature][half][q]: W1s[row_feat][unit_of(4q.., half)]
  float4 w3[2][8];           // [half][v/2]: d(v) m(v) d(v+1) m(v+1)
};

template <bool VEC>
__device__ __forceinline__ void load_row(const TensorDev& T, size_t ro, int col, int n, float4 (&d)[6]) {
  const size_t pN = T.padN;
  d[0] = load4s<VEC>(T.g + ro, col, n);
  d[1] = load4s<VEC>(T.p + ro, col, n);
  d[2] = load4s<VEC>(T.st + ro, col, n);
  d[3] = load4s<VEC>(T.st + pN + ro, col, n);
  d[4] = load4s<VEC>(T.st + 2 * pN + ro, col, n);
  d[5] = load4s<VEC>(T.st + 3 * pN + ro, col, n);
}

// Per-tile set-up shared by the matrix-core apply kernels: the column vectors of the hoisted
// column-constant features, the row-feature weights and W3, all into LDS. Ends with a barrier.
__device__ __forceinline__ void apply_tile_setup(const TensorDev& T, const TileDev& tile, const float* __restrict__ ws,
                                                 const float* __restrict__ prep, const float* __restrict__ tail,
                                                 ApplyLds& L) {
  const int n = T.n;
  {
    const int t = threadIdx.x;
    const int c = tile.tj * kTileCols + t;
    float cf[6];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      cf[k] = c < n ? T.st[4 * (size_t)T.padN + 3 * (size_t)T.padm + (size_t)k * T.padn + c] : 0.f;
      cf[3 + k] = c < n ? ws[T.oRC + (size_t)k * T.padn + c] : 0.f;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int u = 8 * q + 4 * hf + j;
          float a = 0.f;
#pragma unroll
          for (int f = 0; f < 6; ++f) a += cf[f] * prep[col_feat(f) * kH + u];
          o[j] = a;
        }
        L.colv[q][hf][t & 3][t >> 2] = make_float4(o[0], o[1], o[2], o[3]);
      }
    }
    if (t < 48) {
      const int f = t >> 3, hf = (t >> 2) & 1, q = t & 3;
      float o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = prep[row_feat(f) * kH + 8 * q + 4 * hf + j];
      L.w1row[f][hf][q] = make_float4(o[0], o[1], o[2], o[3]);
    }
    if (t >= 64 && t < 80) {
      const int hf = (t >> 3) & 1, v2 = t & 7;
      const float* w3g = tail + kH * kH + kH;
      const int u0 = unit_of(2 * v2, hf), u1 = unit_of(2 * v2 + 1, hf);
      L.w3[hf][v2] = make_float4(w3g[2 * u0], w3g[2 * u0 + 1], w3g[2 * u1], w3g[2 * u1 + 1]);
    }
  }
  __syncthreads();

}

}  // namespace lopt
