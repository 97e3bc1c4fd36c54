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
//   * Biases enter as the C operand of the first MFMA of each chain.
//   * Layer 3: each lane holds half of its element's hidden units; the two partial dot products
//     are exchanged with one more v_permlane32_swap.
#include "lopt_internal.h"
#include "lopt_device.h"

namespace lopt {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void swap32(float& a, float& b) {
  // v_permlane32_swap: a.hi <-> b.lo, i.e. afterwards a = [a.lo | b.lo], b = [a.hi | b.hi]
  // (lo = lanes 0..31). Written as inline assembly because the compiler's builtin returns the first
  // result twice (checked on ROCm 7.2); the s_nop pairs cover the VALU <-> permlane-swap wait states
  // that the compiler cannot see inside an asm block.
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}

__device__ __forceinline__ int unit_of(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

constexpr int kNF = LOPT_N_ELEM_FEATS;  // 28
constexpr int kH = 32;

template <bool VEC>
__device__ __forceinline__ void apply_mfma_tile(const TensorDev& T, const TileDev& tile, const float* __restrict__ ws,
                                                const StepArgs& A, const float* __restrict__ tail,
                                                const float* __restrict__ w3s) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const float* __restrict__ prep = ws + T.oPrep;  // W1s[28][32] (normalization folded in), b1'[32]
  float a1[kNF / 2], a2[kH / 2];
  f32x16 cb1, cb2;
#pragma unroll
  for (int s = 0; s < kNF / 2; ++s) a1[s] = prep[(2 * s + half) * kH + l32];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int u = unit_of(v, half);
    a2[v] = tail[u * kH + l32];
    cb1[v] = prep[kNF * kH + u];
    cb2[v] = tail[kH * kH + u];
  }
  const float b3d = tail[kH * kH + kH + 2 * kH], b3m = tail[kH * kH + kH + 2 * kH + 1];
  const float4* __restrict__ w3 = reinterpret_cast<const float4*>(w3s) + half * 8;  // [v/2]: d(v) m(v) d(v+1) m(v+1)

  const int n = T.n, m = T.m;
  const int col = tile.tj * kTileCols + 4 * lane;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  float4 rc[3], cc[3];
  const float* cst = T.st + 4 * (size_t)T.padN + 3 * (size_t)T.padm;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    rc[k] = load4<VEC>(ws + T.oRC + (size_t)k * T.padn, col, n);
    cc[k] = load4<VEC>(cst + (size_t)k * T.padn, col, n);
  }
  const float* __restrict__ M1 = T.st;
  const float* __restrict__ M2 = T.st + (size_t)T.padN;
  const float* __restrict__ M3 = T.st + 2 * (size_t)T.padN;
  const float* __restrict__ Vp = T.st + 3 * (size_t)T.padN;
  const float* rst = T.st + 4 * (size_t)T.padN;
  const float eps = A.eps_acc, lr = A.lr, wd = A.wd;
  const float zero = 0.f;

  for (int r = r0 + wave; r < r1; r += 4) {
    const size_t ro = (size_t)r * n;
    const float4 g4 = load4<VEC>(T.g + ro, col, n);
    const float4 p4 = load4<VEC>(T.p + ro, col, n);
    const float4 m1 = load4<VEC>(M1 + ro, col, n);
    const float4 m2 = load4<VEC>(M2 + ro, col, n);
    const float4 m3 = load4<VEC>(M3 + ro, col, n);
    const float4 v4 = load4<VEC>(Vp + ro, col, n);
    float rr[3], rv[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      rr[k] = ws[T.oRR + (size_t)k * T.padm + r];
      rv[k] = rst[(size_t)k * T.padm + r];
    }
    float pn[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x[kNF];
      {
        const float g = get(g4, e), p = get(p4, e);
        const float q1 = get(m1, e), q2 = get(m2, e), q3 = get(m3, e), v = get(v4, e);
        const float rs = rsqrtf(v + eps);
        const float c0 = get(rc[0], e), c1 = get(rc[1], e), c2 = get(rc[2], e);
        const float f0 = rr[0] * c0, f1 = rr[1] * c1, f2 = rr[2] * c2;
        x[0] = g; x[1] = p; x[2] = q1; x[3] = q2; x[4] = q3; x[5] = v;
        x[6] = q1 * rs; x[7] = q2 * rs; x[8] = q3 * rs; x[9] = rs;
        x[10] = g * f0; x[11] = g * f1; x[12] = g * f2;
        x[13] = rv[0]; x[14] = rv[1]; x[15] = rv[2];
        x[16] = get(cc[0], e); x[17] = get(cc[1], e); x[18] = get(cc[2], e);
        x[19] = rr[0]; x[20] = rr[1]; x[21] = rr[2];
        x[22] = c0; x[23] = c1; x[24] = c2;
        x[25] = q1 * f0; x[26] = q2 * f1; x[27] = q3 * f2;
      }
      // x[2s] -> B operand of step s for tile E1, x[2s+1] -> for tile E2
#pragma unroll
      for (int s = 0; s < kNF / 2; ++s) swap32(x[2 * s], x[2 * s + 1]);
      f32x16 h1a = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[0], x[0], cb1, 0, 0, 0);
      f32x16 h1b = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[0], x[1], cb1, 0, 0, 0);
#pragma unroll
      for (int s = 1; s < kNF / 2; ++s) {
        h1a = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], x[2 * s], h1a, 0, 0, 0);
        h1b = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], x[2 * s + 1], h1b, 0, 0, 0);
      }
      f32x16 h2a = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[0], fmaxf(h1a[0], zero), cb2, 0, 0, 0);
      f32x16 h2b = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[0], fmaxf(h1b[0], zero), cb2, 0, 0, 0);
#pragma unroll
      for (int v = 1; v < 16; ++v) {
        h2a = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[v], fmaxf(h1a[v], zero), h2a, 0, 0, 0);
        h2b = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[v], fmaxf(h1b[v], zero), h2b, 0, 0, 0);
      }
      float da = 0.f, ma = 0.f, db = 0.f, mb = 0.f;
#pragma unroll
      for (int v2 = 0; v2 < 8; ++v2) {
        const float4 w = w3[v2];
        const float ha0 = fmaxf(h2a[2 * v2], zero), ha1 = fmaxf(h2a[2 * v2 + 1], zero);
        const float hb0 = fmaxf(h2b[2 * v2], zero), hb1 = fmaxf(h2b[2 * v2 + 1], zero);
        da += ha0 * w.x; ma += ha0 * w.y; da += ha1 * w.z; ma += ha1 * w.w;
        db += hb0 * w.x; mb += hb0 * w.y; db += hb1 * w.z; mb += hb1 * w.w;
      }
      swap32(da, db);
      swap32(ma, mb);
      const float d = (da + db) + b3d, mg = (ma + mb) + b3m;
      const float delta = d * expf(mg * A.exp_mult) * A.step_mult;
      const float p = get(p4, e);
      pn[e] = p - lr * (delta + wd * p);
    }
    store4<VEC>(T.p + ro, col, n, make_float4(pn[0], pn[1], pn[2], pn[3]));
  }
}

__global__ void __launch_bounds__(kBlock, 2) k_apply_mfma(const TensorDev* __restrict__ tensors,
                                                          const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                          StepArgs A, const float* __restrict__ tail) {
  // W3 per half-wave: w3s[half][v][2] = W3[unit_of(v, half)][0..1]
  __shared__ __attribute__((aligned(16))) float w3s[2 * 16 * 2];
  if (threadIdx.x < 64) {
    const int half = threadIdx.x >> 5, v = (threadIdx.x >> 1) & 15, j = threadIdx.x & 1;
    w3s[threadIdx.x] = tail[kH * kH + kH + 2 * unit_of(v, half) + j];
  }
  __syncthreads();
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  if (T.vec) apply_mfma_tile<true>(T, tile, ws, A, tail, w3s);
  else apply_mfma_tile<false>(T, tile, ws, A, tail, w3s);
}

bool apply_mfma_available(const StepArgs& A) { return A.kind == LOPT_SMALL_FC && A.HP == kH; }

void launch_apply_mfma(const Launch& L, const StepArgs& A, const WeightsDev& W, hipStream_t s) {
  if (L.n_tiles == 0) return;
  hipLaunchKernelGGL(k_apply_mfma, dim3(L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles, L.ws, A, W.mlp_tail);
}

}  // namespace lopt
