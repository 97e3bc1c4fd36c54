// Vector-ALU variant of the fused apply pass (paper: "Kernel 2: fused feature construction and
// network application"): rebuild the features of each element in registers, scale, evaluate the
// MLP and write the updated parameter.
#include "lopt_internal.h"
#include "lopt_device.h"

namespace lopt {

// ----------------------------------------------------------------------------- apply (vector ALU)

// Generic fused normalize + MLP + update for any padded hidden width HP in {4,8,16,32,64}.
// The prepared weights of the tile's tensor sit in LDS and are read as wave-uniform float4
// broadcasts; E elements are evaluated together so that each weight read feeds E FMAs.
template <int NF, int HP, int E, bool VEC>
__device__ __forceinline__ void apply_tile(const TensorDev& T, const TileDev& tile, const float* __restrict__ ws,
                                           const StepArgs& A, const float* __restrict__ sw) {
  constexpr int H4 = HP / 4;
  const float4* __restrict__ W1 = reinterpret_cast<const float4*>(sw);           // [NF][H4]
  const float4* __restrict__ B1 = W1 + NF * H4;                                    // [H4]
  const float4* __restrict__ W2 = B1 + H4;                                         // [HP][H4]
  const float4* __restrict__ B2 = W2 + HP * H4;                                    // [H4]
  const float* __restrict__ W3 = reinterpret_cast<const float*>(B2 + H4);          // [HP][2]
  const float* __restrict__ B3 = W3 + 2 * HP;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
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
  const float eps = A.eps_acc;
  const float lr = A.lr, wd = A.wd;
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
    float pn[4];
#pragma unroll
    for (int e0 = 0; e0 < 4; e0 += E) {
      float x[E][NF];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int ee = e0 + e;
        const float g = get(g4, ee), p = get(p4, ee);
        const float a1 = get(m1, ee), a2 = get(m2, ee), a3 = get(m3, ee), v = get(v4, ee);
        const float rs = rsqrtf(v + eps);
        const float f0 = rr[0] * get(rc[0], ee), f1 = rr[1] * get(rc[1], ee), f2 = rr[2] * get(rc[2], ee);
        x[e][0] = g; x[e][1] = p; x[e][2] = a1; x[e][3] = a2; x[e][4] = a3; x[e][5] = v;
        x[e][6] = a1 * rs; x[e][7] = a2 * rs; x[e][8] = a3 * rs; x[e][9] = rs;
        x[e][10] = g * f0; x[e][11] = g * f1; x[e][12] = g * f2;
        x[e][13] = rv[0]; x[e][14] = rv[1]; x[e][15] = rv[2];
        x[e][16] = get(cc[0], ee); x[e][17] = get(cc[1], ee); x[e][18] = get(cc[2], ee);
        x[e][19] = rr[0]; x[e][20] = rr[1]; x[e][21] = rr[2];
        x[e][22] = get(rc[0], ee); x[e][23] = get(rc[1], ee); x[e][24] = get(rc[2], ee);
        x[e][25] = a1 * f0; x[e][26] = a2 * f1; x[e][27] = a3 * f2;
        if (NF == 29) x[e][NF - 1] = fminf(fmaxf(g, -0.1f), 0.1f);
      }
      float h1[E][HP];
#pragma unroll
      for (int u4 = 0; u4 < H4; ++u4) {
        const float4 b = B1[u4];
#pragma unroll
        for (int e = 0; e < E; ++e) { h1[e][4 * u4] = b.x; h1[e][4 * u4 + 1] = b.y; h1[e][4 * u4 + 2] = b.z; h1[e][4 * u4 + 3] = b.w; }
      }
#pragma unroll
      for (int f = 0; f < NF; ++f) {
#pragma unroll
        for (int u4 = 0; u4 < H4; ++u4) {
          const float4 w = W1[f * H4 + u4];
#pragma unroll
          for (int e = 0; e < E; ++e) {
            h1[e][4 * u4] += x[e][f] * w.x; h1[e][4 * u4 + 1] += x[e][f] * w.y;
            h1[e][4 * u4 + 2] += x[e][f] * w.z; h1[e][4 * u4 + 3] += x[e][f] * w.w;
          }
        }
      }
      float h2[E][HP];
#pragma unroll
      for (int u4 = 0; u4 < H4; ++u4) {
        const float4 b = B2[u4];
#pragma unroll
        for (int e = 0; e < E; ++e) { h2[e][4 * u4] = b.x; h2[e][4 * u4 + 1] = b.y; h2[e][4 * u4 + 2] = b.z; h2[e][4 * u4 + 3] = b.w; }
      }
#pragma unroll
      for (int a = 0; a < HP; ++a) {
#pragma unroll
        for (int u4 = 0; u4 < H4; ++u4) {
          const float4 w = W2[a * H4 + u4];
#pragma unroll
          for (int e = 0; e < E; ++e) {
            const float h = fmaxf(h1[e][a], 0.f);
            h2[e][4 * u4] += h * w.x; h2[e][4 * u4 + 1] += h * w.y;
            h2[e][4 * u4 + 2] += h * w.z; h2[e][4 * u4 + 3] += h * w.w;
          }
        }
      }
#pragma unroll
      for (int e = 0; e < E; ++e) {
        float d = B3[0], mg = B3[1];
#pragma unroll
        for (int a = 0; a < HP; ++a) {
          const float h = fmaxf(h2[e][a], 0.f);
          d += h * W3[2 * a];
          mg += h * W3[2 * a + 1];
        }
        const float delta = d * expf(mg * A.exp_mult) * A.step_mult;
        const float p = get(p4, e0 + e);
        pn[e0 + e] = p - lr * (delta + wd * p);
      }
    }
    store4s<VEC>(T.p + ro, col, n, make_float4(pn[0], pn[1], pn[2], pn[3]));
  }
}

template <int NF, int HP, int E>
__global__ void __launch_bounds__(kBlock) k_apply(const TensorDev* __restrict__ tensors,
                                                  const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                  StepArgs A, const float* __restrict__ shared_tail) {
  constexpr int kHead = (NF + 1) * HP;                 // W1s, b1'
  constexpr int kTail = HP * HP + HP + 2 * HP + 2;     // W2, b2, W3, b3
  __shared__ __attribute__((aligned(16))) float sw[kHead + kTail + 2];
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  const float* prep = ws + T.oPrep;
  const float* tail = shared_tail ? shared_tail : prep + kHead;
  for (int i = threadIdx.x; i < kHead; i += kBlock) sw[i] = prep[i];
  for (int i = threadIdx.x; i < kTail; i += kBlock) sw[kHead + i] = tail[i];
  __syncthreads();
  if (T.vec) apply_tile<NF, HP, E, true>(T, tile, ws, A, sw);
  else apply_tile<NF, HP, E, false>(T, tile, ws, A, sw);
}

template <int NF>
static void launch_apply_nf(const Launch& L, const StepArgs& A, const float* tail, hipStream_t s) {
  dim3 grid(L.n_tiles), block(kBlock);
  switch (A.HP) {
    case 4: hipLaunchKernelGGL((k_apply<NF, 4, 4>), grid, block, 0, s, L.tensors, L.tiles, L.ws, A, tail); break;
    case 8: hipLaunchKernelGGL((k_apply<NF, 8, 2>), grid, block, 0, s, L.tensors, L.tiles, L.ws, A, tail); break;
    case 16: hipLaunchKernelGGL((k_apply<NF, 16, 1>), grid, block, 0, s, L.tensors, L.tiles, L.ws, A, tail); break;
    default: hipLaunchKernelGGL((k_apply<NF, 32, 1>), grid, block, 0, s, L.tensors, L.tiles, L.ws, A, tail); break;
  }
}

// This file is compiled once per optimizer kind (LOPT_APPLY_KIND = 0: small_fc_lopt, 1: VeLO)
// so that the two sets of instantiations build in parallel.
#if LOPT_APPLY_KIND == 0
void launch_apply_small_fc(const Launch& L, const StepArgs& A, const WeightsDev& W, hipStream_t s) {
  if (L.n_tiles == 0) return;
  launch_apply_nf<LOPT_N_ELEM_FEATS>(L, A, W.mlp_tail, s);
}
#else
void launch_apply_velo(const Launch& L, const StepArgs& A, const WeightsDev&, hipStream_t s) {
  if (L.n_tiles == 0) return;
  launch_apply_nf<LOPT_D_VELO>(L, A, nullptr, s);
}
#endif

}  // namespace lopt
