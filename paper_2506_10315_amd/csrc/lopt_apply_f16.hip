// Split-fp16 matrix-core variant of the fused apply pass for small_fc_lopt, hidden width 32
// (paper: "Kernel 2: fused feature construction and network application"; its H100 appendix puts
// the MLP contraction on tensor cores).
//
// Why not the fp32 MFMA: on gfx950 v_mfma_f32_32x32x2_f32 runs at the rate of the vector FP32 lanes
// and does not overlap with vector-ALU work of the same SIMD (measured: time = MFMA time + VALU
// time), while the 16-bit MFMAs run on the matrix engine at 16x the rate and DO overlap with the
// vector ALU. So the two contractions are done in fp16 with fp32 accumulation, and every operand is
// carried as an unevaluated sum of two fp16 numbers, x = hi + lo with hi = fp16_rtz(x) and
// lo = fp16_rtz(x - hi): 22 significand bits. A product keeps the three leading terms
//   x*w = hi*Whi + lo*Whi + hi*Wlo            (dropped lo*Wlo is below 2^-22 relative)
// i.e. three v_mfma_f32_32x32x16_f16 per 16 values of k. Accuracy is that of fp32 arithmetic to within
// a small factor; range is fp16's, which is why features are normalized BEFORE the contraction here
// (normalized features are bounded by sqrt(N) < 46341 < 65504) instead of folding the normalization into W1.
//
// Layout (same idea as the fp32 kernel): products are computed transposed, D[unit, element] =
// W^T[unit, k] X^T[k, element]. One MFMA takes 16 values of k: lanes 0..31 hold k 0..7 of element
// (lane & 31) as four packed registers, lanes 32..63 hold k 8..15 of the same element.
//   * layer 1 (k = the 16 per-element features): each lane packs its own element's features into 8
//     registers (hi) + 8 (lo); v_permlane32_swap of register i with register 4+i yields the B operands of
//     the wave's two 32-element tiles.
//   * the accumulator leaves lane l with 16 hidden units of element (l & 31): registers 0..7 are k 0..7 of
//     layer 2's first MFMA for this lane half, registers 8..15 those of its second MFMA; ReLU, split and
//     pack happen in place, no cross-lane traffic. The weights are packed per lane in that order.
//   * row/column-constant features, biases: as in the fp32 kernel (C operand of the first MFMA).
//   * layer 3 and the update: vector ALU, fp32.
#include "lopt_apply_common.h"

namespace lopt {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f16x8 as_f16x8(unsigned a, unsigned b, unsigned c, unsigned d) {
  u32x4 v = {a, b, c, d};
  return __builtin_bit_cast(f16x8, v);
}

// (a, b) -> packed hi pair and packed lo pair, hi = rtz_fp16(x), lo = rtz_fp16(x - hi).
// The residual x - float(hi) is one mixed-precision FMA (v_fma_mix_f32 reads the fp16 half directly):
// the compiler only forms it when x itself is a product, so it is written out here.
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a, b));
  float ra, rb;
  asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(ra) : "v"(hi), "v"(a));
  asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(rb) : "v"(hi), "v"(b));
  lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(ra, rb));
}

__device__ __forceinline__ f32x16 mfma3(const f16x8& ah, const f16x8& al, const f16x8& bh, const f16x8& bl,
                                        f32x16 c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c, 0, 0, 0);
  return c;
}

// ReLU, split and pack 8 accumulator registers (k 0..7 of one MFMA) of a tile
__device__ __forceinline__ void pack_relu8(const f32x16& h, int base, f16x8& hi, f16x8& lo) {
  unsigned ph[4], pl[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split2(relu(h[base + 2 * i]), relu(h[base + 2 * i + 1]), ph[i], pl[i]);
  hi = as_f16x8(ph[0], ph[1], ph[2], ph[3]);
  lo = as_f16x8(pl[0], pl[1], pl[2], pl[3]);
}

template <bool VEC>
__device__ __forceinline__ void apply_f16_tile(const TensorDev& T, const TileDev& tile, const float* __restrict__ ws,
                                               const StepArgs& A, const float* __restrict__ tail, ApplyLds& L) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const float* __restrict__ prep = ws + T.oPrep;  // W1s[28][32] (normalization folded in), b1'[32]
  const int n = T.n, m = T.m;

  apply_tile_setup(T, tile, ws, prep, tail, L);

  // ---- weights of this lane, split and packed (once per tile)
  const float* __restrict__ w1raw = tail + (kH * kH + kH + 2 * kH + 2 + 2);  // W1[28][32], not normalized
  f16x8 a1h, a1l, a2h[2], a2l[2];
  {
    unsigned ph[4], pl[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // k slot 8*half + 2i (+1) -> per-element feature
      const float w0 = half ? w1raw[elem_feat(8 + 2 * i) * kH + l32] : w1raw[elem_feat(2 * i) * kH + l32];
      const float w1 = half ? w1raw[elem_feat(9 + 2 * i) * kH + l32] : w1raw[elem_feat(2 * i + 1) * kH + l32];
      split2(w0, w1, ph[i], pl[i]);
    }
    a1h = as_f16x8(ph[0], ph[1], ph[2], ph[3]);
    a1l = as_f16x8(pl[0], pl[1], pl[2], pl[3]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float w0 = tail[unit_of(8 * j + 2 * i, half) * kH + l32];
        const float w1 = tail[unit_of(8 * j + 2 * i + 1, half) * kH + l32];
        split2(w0, w1, ph[i], pl[i]);
      }
      a2h[j] = as_f16x8(ph[0], ph[1], ph[2], ph[3]);
      a2l[j] = as_f16x8(pl[0], pl[1], pl[2], pl[3]);
    }
  }
  f32x16 cb2;
#pragma unroll
  for (int v = 0; v < 16; ++v) cb2[v] = tail[kH * kH + unit_of(v, half)];
  // Row part of layer 1's C operand (bias + the six row-constant features): one value per hidden
  // unit and row, injected through the matrix engine as k slot 0 of an extra MFMA against a constant
  // B operand that is 1 in that slot. Lane l < 32 carries unit l.
  float w1r[6];
#pragma unroll
  for (int f = 0; f < 6; ++f) w1r[f] = prep[row_feat(f) * kH + l32];
  const float b1l = prep[kNF * kH + l32];
  const f16x8 b_one = as_f16x8(half ? 0u : 0x3C00u, 0u, 0u, 0u);   // fp16 1.0 in k slot 0
  const float b3d = tail[kH * kH + kH + 2 * kH], b3m = tail[kH * kH + kH + 2 * kH + 1];
  float sc[kNE];  // normalization factors of the per-element features (wave-uniform)
#pragma unroll
  for (int i = 0; i < kNE; ++i) sc[i] = ws[T.oScale + elem_feat(i)];

  const int col = tile.tj * kTileCols + 4 * lane;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  float4 rc[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) rc[k] = load4<VEC>(ws + T.oRC + (size_t)k * T.padn, col, n);
  const float* rst = T.st + 4 * (size_t)T.padN;
  const float eps = A.eps_acc, lr = A.lr, wd = A.wd;

  int r = r0 + wave;
  float4 cur[6];
  if (r < r1) load_row<VEC>(T, (size_t)r * n, col, n, cur);
  for (; r < r1; r += 4) {
    const size_t ro = (size_t)r * n;
    float4 nxt[6];
    if (r + 4 < r1) load_row<VEC>(T, (size_t)(r + 4) * n, col, n, nxt);   // next row in flight during the MLP
    float rr[3], rv[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      rr[k] = ws[T.oRR + (size_t)k * T.padm + r];
      rv[k] = rst[(size_t)k * T.padm + r];
    }
    // bias + row-constant features of this row for hidden unit (lane & 31), split into fp16 hi + lo
    f16x8 rbh, rbl;
    {
      float rb = b1l;
#pragma unroll
      for (int f = 0; f < 6; ++f) rb += (f < 3 ? rv[f] : rr[f - 3]) * w1r[f];
      unsigned h, l;
      split2(half ? 0.f : rb, 0.f, h, l);
      rbh = as_f16x8(h, 0u, 0u, 0u);
      rbl = as_f16x8(l, 0u, 0u, 0u);
    }
    float pn[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      unsigned ph[8], pl[8];
      {
        const float g = get(cur[0], e);
        const float q1 = get(cur[2], e), q2 = get(cur[3], e), q3 = get(cur[4], e), v = get(cur[5], e);
        const float rs = rsqrtf(v + eps);
        const float f0 = rr[0] * get(rc[0], e), f1 = rr[1] * get(rc[1], e), f2 = rr[2] * get(rc[2], e);
        float x[kNE];
        x[0] = g; x[1] = get(cur[1], e); x[2] = q1; x[3] = q2; x[4] = q3; x[5] = v;
        x[6] = q1 * rs; x[7] = q2 * rs; x[8] = q3 * rs; x[9] = rs;
        x[10] = g * f0; x[11] = g * f1; x[12] = g * f2;
        x[13] = q1 * f0; x[14] = q2 * f1; x[15] = q3 * f2;
#pragma unroll
        for (int i = 0; i < 8; ++i) split2(x[2 * i] * sc[2 * i], x[2 * i + 1] * sc[2 * i + 1], ph[i], pl[i]);
      }
      // registers 0..3 -> B operand of tile E1, registers 4..7 -> B operand of tile E2
      swap32x8(ph, pl);
      // C operand of layer 1: the column vector of the tile's element straight from LDS; the row part
      // (bias + row-constant features) comes in through two extra MFMAs
      f32x16 h1a, h1b;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 ca = L.colv[q][half][e][l32];
        const float4 cb = L.colv[q][half][e][32 + l32];
        h1a[4 * q] = ca.x; h1a[4 * q + 1] = ca.y; h1a[4 * q + 2] = ca.z; h1a[4 * q + 3] = ca.w;
        h1b[4 * q] = cb.x; h1b[4 * q + 1] = cb.y; h1b[4 * q + 2] = cb.z; h1b[4 * q + 3] = cb.w;
      }
      h1a = __builtin_amdgcn_mfma_f32_32x32x16_f16(rbl, b_one, h1a, 0, 0, 0);
      h1b = __builtin_amdgcn_mfma_f32_32x32x16_f16(rbl, b_one, h1b, 0, 0, 0);
      h1a = __builtin_amdgcn_mfma_f32_32x32x16_f16(rbh, b_one, h1a, 0, 0, 0);
      h1b = __builtin_amdgcn_mfma_f32_32x32x16_f16(rbh, b_one, h1b, 0, 0, 0);
      h1a = mfma3(a1h, a1l, as_f16x8(ph[0], ph[1], ph[2], ph[3]), as_f16x8(pl[0], pl[1], pl[2], pl[3]), h1a);
      h1b = mfma3(a1h, a1l, as_f16x8(ph[4], ph[5], ph[6], ph[7]), as_f16x8(pl[4], pl[5], pl[6], pl[7]), h1b);
      f32x16 h2a = cb2, h2b = cb2;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        f16x8 bh, bl;
        pack_relu8(h1a, 8 * j, bh, bl);
        h2a = mfma3(a2h[j], a2l[j], bh, bl, h2a);
        pack_relu8(h1b, 8 * j, bh, bl);
        h2b = mfma3(a2h[j], a2l[j], bh, bl, h2b);
      }
      float da = 0.f, ma = 0.f, db = 0.f, mb = 0.f;
#pragma unroll
      for (int v2 = 0; v2 < 8; ++v2) {
        const float4 w = L.w3[half][v2];
        const float ha0 = relu(h2a[2 * v2]), ha1 = relu(h2a[2 * v2 + 1]);
        const float hb0 = relu(h2b[2 * v2]), hb1 = relu(h2b[2 * v2 + 1]);
        da += ha0 * w.x; ma += ha0 * w.y; da += ha1 * w.z; ma += ha1 * w.w;
        db += hb0 * w.x; mb += hb0 * w.y; db += hb1 * w.z; mb += hb1 * w.w;
      }
      swap32x2(da, db, ma, mb);
      const float d = (da + db) + b3d, mg = (ma + mb) + b3m;
      const float delta = d * expf(mg * A.exp_mult) * A.step_mult;
      const float p = get(cur[1], e);
      pn[e] = p - lr * (delta + wd * p);
      __builtin_amdgcn_sched_barrier(0);   // keep the four rounds apart: bounds register pressure
    }
    store4s<VEC>(T.p + ro, col, n, make_float4(pn[0], pn[1], pn[2], pn[3]));
#pragma unroll
    for (int i = 0; i < 6; ++i) cur[i] = nxt[i];
  }
}

__global__ void __launch_bounds__(kBlock, 2) k_apply_f16x3(const TensorDev* __restrict__ tensors,
                                                           const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                           StepArgs A, const float* __restrict__ tail) {
  __shared__ ApplyLds L;
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  if (T.vec) apply_f16_tile<true>(T, tile, ws, A, tail, L);
  else apply_f16_tile<false>(T, tile, ws, A, tail, L);
}

void launch_apply_f16x3(const Launch& L, const StepArgs& A, const WeightsDev& W, hipStream_t s) {
  if (L.n_tiles == 0) return;
  hipLaunchKernelGGL(k_apply_f16x3, dim3(L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles, L.ws, A, W.mlp_tail);
}

}  // namespace lopt
