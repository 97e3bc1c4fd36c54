// Matrix-core variant of the fused apply pass for small_fc_lopt with (padded) hidden width 32
// (paper: "Kernel 2: fused feature construction and network application"; the appendix on H100
// moves the MLP contraction to tensor cores, which is what this does on gfx950's MFMA units).
//
// Per element the MLP is [28 normalized features] x W1[28,32] -> ReLU -> W2[32,32] -> ReLU ->
// W3[32,2]. Layers 1 and 2 run on v_mfma_f32_32x32x2_f32 in fp32 (no precision is given up);
// layer 3 (2 outputs) and everything else run on the vector ALU.
//
// Layout. The products are computed transposed, D[unit, element] = W^T[unit, k] * X^T[k, element],
// so that the output of one layer is already laid out as the B operand of the next:
//   * A wavefront evaluates 64 elements per round as two 32-element tiles: tile E1 is owned by
//     lanes 0..31, tile E2 by lanes 32..63 (each lane builds the 28 features of its own element).
//   * One MFMA consumes two k values: lanes 0..31 supply k_a, lanes 32..63 supply k_b, both for
//     element (lane & 31). v_permlane32_swap on the feature pair (2s, 2s+1) turns the two
//     "own element" registers into the B operands of step s for E1 and for E2.
//   * The 32x32 result leaves lane l with element (l & 31) and the 16 hidden units
//     u(v, half) = 8*(v/4) + 4*half + (v%4), half = l >> 5, in accumulator register v. Register v
//     (after ReLU) is therefore directly the B operand of layer 2's step v with k_a = u(v,0),
//     k_b = u(v,1); the A operands (weights) are loaded in that order once per tile.
//   * Only the 16 features that vary per element go through layer 1's MFMAs (8 steps). The 12
//     features that are constant along a row or a column contribute a 32-vector per row and a
//     32-vector per column; with the bias they form the C operand of the first MFMA of the chain
//     (column vectors are computed once per tile into LDS, laid out so that each ds_read_b128 is
//     conflict-free; row vectors once per row). Layer 2's bias is the C operand of its first MFMA.
//   * Layer 3: each lane holds half of its element's hidden units; the two partial dot products
//     are exchanged with one more v_permlane32_swap.
#include "lopt_apply_common.h"

namespace lopt {

template <bool VEC>
__device__ __forceinline__ void apply_mfma_tile(const TensorDev& T, const TileDev& tile, const float* __restrict__ ws,
                                                const StepArgs& A, const float* __restrict__ tail,
                                                ApplyLds& L) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const float* __restrict__ prep = ws + T.oPrep;  // W1s[28][32] (normalization folded in), b1'[32]
  const int n = T.n, m = T.m;

  apply_tile_setup(T, tile, ws, prep, tail, L);

  float a1[kNE / 2], a2[kH / 2];
  f32x16 cb1, cb2;
#pragma unroll
  for (int s = 0; s < kNE / 2; ++s) a1[s] = prep[(half ? elem_feat(2 * s + 1) : elem_feat(2 * s)) * kH + l32];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int u = unit_of(v, half);
    a2[v] = tail[u * kH + l32];
    cb1[v] = prep[kNF * kH + u];
    cb2[v] = tail[kH * kH + u];
  }
  const float b3d = tail[kH * kH + kH + 2 * kH], b3m = tail[kH * kH + kH + 2 * kH + 1];

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
    // bias + row-constant features for this row, for the lane's 16 hidden units
    f32x16 cbr = cb1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int f = 0; f < 6; ++f) {
        const float4 w = L.w1row[f][half][q];
        const float xf = f < 3 ? rv[f] : rr[f - 3];
        cbr[4 * q] += xf * w.x; cbr[4 * q + 1] += xf * w.y; cbr[4 * q + 2] += xf * w.z; cbr[4 * q + 3] += xf * w.w;
      }
    }
    float pn[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x[kNE];
      {
        const float g = get(cur[0], e);
        const float q1 = get(cur[2], e), q2 = get(cur[3], e), q3 = get(cur[4], e), v = get(cur[5], e);
        const float rs = rsqrtf(v + eps);
        const float f0 = rr[0] * get(rc[0], e), f1 = rr[1] * get(rc[1], e), f2 = rr[2] * get(rc[2], e);
        x[0] = g; x[1] = get(cur[1], e); x[2] = q1; x[3] = q2; x[4] = q3; x[5] = v;
        x[6] = q1 * rs; x[7] = q2 * rs; x[8] = q3 * rs; x[9] = rs;
        x[10] = g * f0; x[11] = g * f1; x[12] = g * f2;
        x[13] = q1 * f0; x[14] = q2 * f1; x[15] = q3 * f2;
      }
      // x[2s] -> B operand of step s for tile E1, x[2s+1] -> for tile E2
#pragma unroll
      for (int s = 0; s < kNE / 2; ++s) swap32(x[2 * s], x[2 * s + 1]);
      // C operand of layer 1: bias + row vector + column vector of the tile's element
      f32x16 h1a, h1b;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 ca = L.colv[q][half][e][l32];
        const float4 cb = L.colv[q][half][e][32 + l32];
        h1a[4 * q] = cbr[4 * q] + ca.x; h1a[4 * q + 1] = cbr[4 * q + 1] + ca.y;
        h1a[4 * q + 2] = cbr[4 * q + 2] + ca.z; h1a[4 * q + 3] = cbr[4 * q + 3] + ca.w;
        h1b[4 * q] = cbr[4 * q] + cb.x; h1b[4 * q + 1] = cbr[4 * q + 1] + cb.y;
        h1b[4 * q + 2] = cbr[4 * q + 2] + cb.z; h1b[4 * q + 3] = cbr[4 * q + 3] + cb.w;
      }
#pragma unroll
      for (int s = 0; s < kNE / 2; ++s) {
        h1a = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], x[2 * s], h1a, 0, 0, 0);
        h1b = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], x[2 * s + 1], h1b, 0, 0, 0);
      }
      f32x16 h2a = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[0], relu(h1a[0]), cb2, 0, 0, 0);
      f32x16 h2b = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[0], relu(h1b[0]), cb2, 0, 0, 0);
#pragma unroll
      for (int v = 1; v < 16; ++v) {
        h2a = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[v], relu(h1a[v]), h2a, 0, 0, 0);
        h2b = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[v], relu(h1b[v]), h2b, 0, 0, 0);
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
      swap32(da, db);
      swap32(ma, mb);
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

__global__ void __launch_bounds__(kBlock, 2) k_apply_mfma(const TensorDev* __restrict__ tensors,
                                                          const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                          StepArgs A, const float* __restrict__ tail) {
  __shared__ ApplyLds L;
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  if (T.vec) apply_mfma_tile<true>(T, tile, ws, A, tail, L);
  else apply_mfma_tile<false>(T, tile, ws, A, tail, L);
}

bool apply_mfma_available(const StepArgs& A) { return A.kind == LOPT_SMALL_FC && A.HP == kH; }

void launch_apply_mfma(const Launch& L, const StepArgs& A, const WeightsDev& W, hipStream_t s) {
  if (L.n_tiles == 0) return;
  hipLaunchKernelGGL(k_apply_mfma, dim3(L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles, L.ws, A, W.mlp_tail);
}

}  // namespace lopt
