// Fused apply pass for VeLO with per-element MLP width 4 (paper: "Kernel 2"; per-tensor weights from
// the hypernetwork). The three tiny layers run on v_mfma_f32_4x4x1_16B_f32: the instruction performs
// 16 independent 4x4 outer-product accumulations, D_b[i][j] += A_b[i] * B_b[j], one per group of four
// lanes. With A = W[k][i] (i = lane & 3, the same in every group) and B = feature k of the lane's OWN
// element, lane l ends up with all four hidden pre-activations of its own element in the four
// accumulator registers: no cross-lane traffic at all, exact fp32, and twice the FMA rate of the
// vector ALU (which is what bounds this pass once the weights are per tensor and only 28 to 44 bytes per
// element move). The 12 row/column-constant features enter through the C operand (4 values per row
// and 4 per column), so layer 1 is 17 MFMAs per element instead of 29.
#include "lopt_internal.h"
#include "lopt_device.h"

#ifndef LOPT_V4_STORE
#define LOPT_V4_STORE store4s
#endif
#ifndef LOPT_V4_STATE_STORE
#define LOPT_V4_STATE_STORE store4s
#endif

namespace lopt {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kVF = LOPT_D_VELO;  // 29
constexpr int kVH = 4;
constexpr int kVE = 17;           // features that vary per element: 0..12, 25..27, 28

__device__ __forceinline__ constexpr int velo_elem_feat(int i) { return i < 13 ? i : 12 + i; }   // 0..12, 25..28
__device__ __forceinline__ constexpr int velo_row_feat(int i) { return i < 3 ? 13 + i : 16 + i; }  // 13..15, 19..21
__device__ __forceinline__ constexpr int velo_col_feat(int i) { return i < 3 ? 16 + i : 19 + i; }  // 16..18, 22..24

__device__ __forceinline__ float relu1(float x) {
  const int i = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(float, i > 0 ? i : 0);
}

// UPDATE_STATE: the statistics pass left M_1..3 and V as they were; this pass forms the new values (the statistics
// pass's operations, in its order: the same bits), builds the features from them and writes them back.
template <bool VEC, bool RAW_RSQ, bool UPDATE_STATE>
__device__ __forceinline__ void apply_velo4_tile(const TensorDev& T, const TileDev& tile, const float* __restrict__ ws,
                                                 const StepArgs& A) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i4 = lane & 3;
  // prepared per-tensor MLP: W1s[29][4] (normalization folded in) b1[4] W2[4][4] b2[4] W3[4][2] b3[2]
  const float* __restrict__ prep = ws + T.oPrep;
  const float* __restrict__ W2 = prep + (kVF + 1) * kVH;
  const float* __restrict__ B2 = W2 + kVH * kVH;
  const float* __restrict__ W3 = B2 + kVH;
  const float* __restrict__ B3 = W3 + 2 * kVH;
  float a1[kVE], a2[kVH], a3[kVH];
#pragma unroll
  for (int k = 0; k < kVE; ++k) a1[k] = prep[velo_elem_feat(k) * kVH + i4];
#pragma unroll
  for (int k = 0; k < kVH; ++k) {
    a2[k] = W2[k * kVH + i4];
    a3[k] = i4 < 2 ? W3[2 * k + i4] : 0.f;
  }
  const f32x4 c2 = {B2[0], B2[1], B2[2], B2[3]};
  const f32x4 c3 = {B3[0], B3[1], 0.f, 0.f};

  const int n = T.n, m = T.m;
  const int col = tile.tj * kTileCols + 4 * lane;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  float4 rc[3];
  f32x4 colv[4];   // per column of this lane: sum over the 6 column-constant features, for the 4 hidden units
  {
    float4 cc[3];
    const float* cst = T.st + 4 * (size_t)T.padN + 3 * (size_t)T.padm;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      rc[k] = load4<VEC>(ws + T.oRC + (size_t)k * T.padn, col, n);
      cc[k] = load4<VEC>(cst + (size_t)k * T.padn, col, n);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
#pragma unroll
      for (int u = 0; u < kVH; ++u) {
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          a += get(cc[k], e) * prep[velo_col_feat(k) * kVH + u];
          a += get(rc[k], e) * prep[velo_col_feat(3 + k) * kVH + u];
        }
        colv[e][u] = a;
      }
    }
  }
  float* __restrict__ M1 = T.st;
  float* __restrict__ M2 = T.st + (size_t)T.padN;
  float* __restrict__ M3 = T.st + 2 * (size_t)T.padN;
  float* __restrict__ Vp = T.st + 3 * (size_t)T.padN;
  const float* rst = T.st + 4 * (size_t)T.padN;
  const float eps = A.eps_acc, lr = A.lr, wd = A.wd;
  const float bm1 = A.mom_decay[0], bm2 = A.mom_decay[1], bm3 = A.mom_decay[2], bv = A.rms_decay;
  const float am1 = 1.0f - bm1, am2 = 1.0f - bm2, am3 = 1.0f - bm3, av = 1.0f - bv;

  for (int r = r0 + wave; r < r1; r += 4) {
    const size_t ro = (size_t)r * n;
    const float4 g4 = load4s<VEC>(T.g + ro, col, n);
    const float4 p4 = load4s<VEC>(T.p + ro, col, n);
    const float4 m1 = load4s<VEC>(M1 + ro, col, n);
    const float4 m2 = load4s<VEC>(M2 + ro, col, n);
    const float4 m3 = load4s<VEC>(M3 + ro, col, n);
    const float4 v4 = load4s<VEC>(Vp + ro, col, n);
    float rr[3], rv[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      rr[k] = ws[T.oRR + (size_t)k * T.padm + r];
      rv[k] = rst[(size_t)k * T.padm + r];
    }
    // bias + row-constant features (wave-uniform)
    f32x4 rowv;
#pragma unroll
    for (int u = 0; u < kVH; ++u) {
      float a = prep[kVF * kVH + u];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        a += rv[k] * prep[velo_row_feat(k) * kVH + u];
        a += rr[k] * prep[velo_row_feat(3 + k) * kVH + u];
      }
      rowv[u] = a;
    }
    float x[4][kVE];
    f32x4 h[4];
    float n1[4], n2[4], n3[4], nv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float g = get(g4, e);
      float q1 = get(m1, e), q2 = get(m2, e), q3 = get(m3, e), v = get(v4, e);
      if (UPDATE_STATE) {
        q1 = __builtin_fmaf(bm1, q1, am1 * g);
        q2 = __builtin_fmaf(bm2, q2, am2 * g);
        q3 = __builtin_fmaf(bm3, q3, am3 * g);
        v = __builtin_fmaf(bv, v, av * (g * g));
        n1[e] = q1; n2[e] = q2; n3[e] = q3; nv[e] = v;
      }
      const float rs = RAW_RSQ ? __builtin_amdgcn_rsqf(v + eps) : rsqrtf(v + eps);
      const float f0 = rr[0] * get(rc[0], e), f1 = rr[1] * get(rc[1], e), f2 = rr[2] * get(rc[2], e);
      x[e][0] = g; x[e][1] = get(p4, e); x[e][2] = q1; x[e][3] = q2; x[e][4] = q3; x[e][5] = v;
      x[e][6] = q1 * rs; x[e][7] = q2 * rs; x[e][8] = q3 * rs; x[e][9] = rs;
      x[e][10] = g * f0; x[e][11] = g * f1; x[e][12] = g * f2;
      x[e][13] = q1 * f0; x[e][14] = q2 * f1; x[e][15] = q3 * f2;
      x[e][16] = fminf(fmaxf(g, -0.1f), 0.1f);
      h[e] = rowv + colv[e];
    }
    if (UPDATE_STATE) {   // stored while the values are live as features anyway
      LOPT_V4_STATE_STORE<VEC>(M1 + ro, col, n, make_float4(n1[0], n1[1], n1[2], n1[3]));
      LOPT_V4_STATE_STORE<VEC>(M2 + ro, col, n, make_float4(n2[0], n2[1], n2[2], n2[3]));
      LOPT_V4_STATE_STORE<VEC>(M3 + ro, col, n, make_float4(n3[0], n3[1], n3[2], n3[3]));
      LOPT_V4_STATE_STORE<VEC>(Vp + ro, col, n, make_float4(nv[0], nv[1], nv[2], nv[3]));
    }
    // layer 1: the four elements of the lane are four independent accumulation chains
#pragma unroll
    for (int k = 0; k < kVE; ++k) {
#pragma unroll
      for (int e = 0; e < 4; ++e) h[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(a1[k], x[e][k], h[e], 0, 0, 0);
    }
    f32x4 h2[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) h2[e] = c2;
#pragma unroll
    for (int k = 0; k < kVH; ++k) {
#pragma unroll
      for (int e = 0; e < 4; ++e) h2[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(a2[k], relu1(h[e][k]), h2[e], 0, 0, 0);
    }
    f32x4 o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = c3;
#pragma unroll
    for (int k = 0; k < kVH; ++k) {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(a3[k], relu1(h2[e][k]), o[e], 0, 0, 0);
    }
    float pn[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float delta = o[e][0] * __expf(o[e][1] * A.exp_mult) * A.step_mult;
      const float p = get(p4, e);
      pn[e] = p - lr * (delta + wd * p);
    }
    LOPT_V4_STORE<VEC>(T.p + ro, col, n, make_float4(pn[0], pn[1], pn[2], pn[3]));
  }
}

template <bool RAW_RSQ, bool UPDATE_STATE>
__global__ void __launch_bounds__(kBlock, 4) k_apply_velo4(const TensorDev* __restrict__ tensors,
                                                        const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                        StepArgs A) {
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  if (T.vec) apply_velo4_tile<true, RAW_RSQ, UPDATE_STATE>(T, tile, ws, A);
  else apply_velo4_tile<false, RAW_RSQ, UPDATE_STATE>(T, tile, ws, A);
}

bool apply_velo4_available(const StepArgs& A) { return A.kind == LOPT_VELO && A.H == kVH && A.HP == kVH; }

void launch_apply_velo4(const Launch& L, const StepArgs& A, bool update_state, hipStream_t s) {
  if (L.n_tiles == 0) return;
  // v_rsq_f32 treats inputs below the smallest normal float as zero; with eps_acc that small the kernel takes the
  // library reciprocal square root (which rescales such inputs) instead of the bare instruction
  const bool raw = A.eps_acc >= 1e-30f;
#define LOPT_LAUNCH_V4(R, U) \
  hipLaunchKernelGGL((k_apply_velo4<R, U>), dim3(L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles, L.ws, A)
  if (raw && update_state) LOPT_LAUNCH_V4(true, true);
  else if (raw) LOPT_LAUNCH_V4(true, false);
  else if (update_state) LOPT_LAUNCH_V4(false, true);
  else LOPT_LAUNCH_V4(false, false);
#undef LOPT_LAUNCH_V4
}

}  // namespace lopt
