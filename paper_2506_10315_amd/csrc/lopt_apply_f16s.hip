// Column-strip form of the split-fp16 matrix-core apply pass for small_fc_lopt, hidden width 32
// (paper: "Kernel 2: fused feature construction and network application"; its H100 appendix puts
// the MLP contraction on tensor cores).
//
// Arithmetic: identical to the row form (lopt_apply_f16.hip): every operand of the two hidden-layer
// contractions is an unevaluated sum of two fp16 numbers and a product keeps hi*Whi + lo*Whi + hi*Wlo
// with fp32 accumulation on v_mfma_f32_32x32x16_f16; features are normalized before the contraction.
//
// What changes is who owns what, chosen so that the kernel needs few registers (three wavefronts per
// SIMD instead of two) and so that almost nothing but the per-element arithmetic is left on the vector ALU:
//   * A wavefront owns a strip of 32 columns and sweeps its rows two at a time: lane (h, c) holds the
//     element (row r + h, column c). The wave's two 32-element MFMA tiles are therefore two ROWS of
//     the same 32 columns, so the first-layer contribution of the six column-constant features is ONE
//     set of 16 accumulator registers per strip, used as the C operand of both tiles for every row
//     (no LDS traffic for it), and each lane's column factors are three registers.
//   * The row-dependent part of the first layer (bias, time features, six row-constant features) is one
//     32-vector per row. It is computed once per 64-row chunk by the whole workgroup, stored in LDS as
//     packed (hi, lo) fp16 pairs, and enters through ONE extra MFMA per tile: A carries (hi, lo) in k
//     slots 0 and 1 of the row's lane half, B is the constant (1, 1) there and 0 elsewhere.
//   * Loads are one dword per array, lane and round (a 128-byte line per row), issued two rounds ahead.
// Workgroup = 4 wavefronts = 128 columns of a planner tile (two workgroups per 256-column tile).
#include "lopt_apply_common.h"

namespace lopt {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kStripCols = 32;
constexpr int kChunkRows = 64;

__device__ __forceinline__ f16x8 pk8(unsigned a, unsigned b, unsigned c, unsigned d) {
  u32x4 v = {a, b, c, d};
  return __builtin_bit_cast(f16x8, v);
}

// (a, b) -> packed hi pair and packed lo pair: hi = rtz_fp16(x), lo = rne_fp16(x - hi). The residual
// is formed and rounded by one mixed-precision FMA per value that writes its fp16 result straight into
// the low or the high half of the destination.
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a, b));
  asm("v_fma_mixlo_f16 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(lo) : "v"(hi), "v"(a));
  asm("v_fma_mixhi_f16 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(lo) : "v"(hi), "v"(b));
}

// one value -> (hi in bits 0..15, lo in bits 16..31)
__device__ __forceinline__ unsigned split1(float a) {
  unsigned pk = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a, 0.f));
  asm("v_fma_mixhi_f16 %0, %0, -1.0, %1 op_sel_hi:[1,0,0]" : "+v"(pk) : "v"(a));
  return pk;
}

__device__ __forceinline__ f32x16 mfma3(const f16x8& ah, const f16x8& al, const f16x8& bh, const f16x8& bl,
                                        f32x16 c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c, 0, 0, 0);
  return c;
}

__device__ __forceinline__ void pack_relu8(const f32x16& h, int base, f16x8& hi, f16x8& lo) {
  unsigned ph[4], pl[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split2(relu(h[base + 2 * i]), relu(h[base + 2 * i + 1]), ph[i], pl[i]);
  hi = pk8(ph[0], ph[1], ph[2], ph[3]);
  lo = pk8(pl[0], pl[1], pl[2], pl[3]);
}

struct StripLds {
  unsigned rowinj[2][kChunkRows][32];  // [buffer][row of the chunk][unit]: packed (hi, lo) of bias + row part
  float4 rowrs[2][kChunkRows];         // rsqrt(r_k + eps) of the row, k = 0..2
  float w1row[6][32];                  // prepared first layer, rows of the row-constant features
  float b1[32];                        // prepared bias (time features folded in)
  float4 w3[2][8];                     // [half][v/2]: d(v) m(v) d(v+1) m(v+1)
};

struct Elem { float g, p, m1, m2, m3, v; };

// The streamed arrays, as global-memory pointers: a wave-uniform base plus a 32-bit lane offset is then one
// global_load with a scalar base, and the loads do not touch the LDS/scalar wait counter.
typedef const float __attribute__((address_space(1)))* gcf32;
typedef float __attribute__((address_space(1)))* gf32;
struct Streams { gcf32 g, p, m1, m2, m3, v; };

__device__ __forceinline__ Elem load_elem(const Streams& S, size_t rowoff, unsigned voff) {
  Elem e;
  e.g = __builtin_nontemporal_load(S.g + rowoff + voff);
  e.p = __builtin_nontemporal_load(S.p + rowoff + voff);
  e.m1 = __builtin_nontemporal_load(S.m1 + rowoff + voff);
  e.m2 = __builtin_nontemporal_load(S.m2 + rowoff + voff);
  e.m3 = __builtin_nontemporal_load(S.m3 + rowoff + voff);
  e.v = __builtin_nontemporal_load(S.v + rowoff + voff);
  return e;
}

}  // namespace

template <bool RAW_RSQ>
__global__ void __launch_bounds__(kBlock, 3) k_apply_f16s(const TensorDev* __restrict__ tensors,
                                                          const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                          StepArgs A, const float* __restrict__ tail) {
  __shared__ StripLds L;
  const TileDev tile = tiles[blockIdx.x >> 1];
  const TensorDev& T = tensors[tile.tensor];
  const int n = T.n, m = T.m;
  const int cblk = tile.tj * kTileCols + (int)(blockIdx.x & 1) * (kTileCols / 2);
  if (cblk >= n) return;  // the right half of a ragged last column tile: nothing to do (whole workgroup)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const float* __restrict__ prep = ws + T.oPrep;  // W1s[28][32] (normalization folded in), b1'[32]
  const int col = cblk + wave * kStripCols + l32;
  const bool col_ok = col < n;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  const float eps = A.eps_acc, lr = A.lr, wd = A.wd;
  const float* __restrict__ rst = T.st + 4 * (size_t)T.padN;   // r_k[3][padm] then c_k[3][padn]

  // ---- tables shared by the workgroup
  {
    const int t = threadIdx.x;
    if (t < 192) L.w1row[t >> 5][t & 31] = prep[row_feat(t >> 5) * kH + (t & 31)];
    else if (t < 224) L.b1[t - 192] = prep[kNF * kH + (t - 192)];
    else if (t < 240) {
      const int hf = (t >> 3) & 1, v2 = t & 7;
      const float* w3g = tail + kH * kH + kH;
      const int u0 = unit_of(2 * v2, hf), u1 = unit_of(2 * v2 + 1, hf);
      L.w3[hf][v2] = make_float4(w3g[2 * u0], w3g[2 * u0 + 1], w3g[2 * u1], w3g[2 * u1 + 1]);
    }
  }

  // ---- weights of this lane, split and packed (the same packing as the row form)
  const float* __restrict__ w1raw = tail + (kH * kH + kH + 2 * kH + 2 + 2);  // W1[28][32], not normalized
  f16x8 a1h, a1l, a2h[2], a2l[2];
  {
    unsigned ph[4], pl[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float w0 = half ? w1raw[elem_feat(8 + 2 * i) * kH + l32] : w1raw[elem_feat(2 * i) * kH + l32];
      const float w1 = half ? w1raw[elem_feat(9 + 2 * i) * kH + l32] : w1raw[elem_feat(2 * i + 1) * kH + l32];
      split2(w0, w1, ph[i], pl[i]);
    }
    a1h = pk8(ph[0], ph[1], ph[2], ph[3]);
    a1l = pk8(pl[0], pl[1], pl[2], pl[3]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float w0 = tail[unit_of(8 * j + 2 * i, half) * kH + l32];
        const float w1 = tail[unit_of(8 * j + 2 * i + 1, half) * kH + l32];
        split2(w0, w1, ph[i], pl[i]);
      }
      a2h[j] = pk8(ph[0], ph[1], ph[2], ph[3]);
      a2l[j] = pk8(pl[0], pl[1], pl[2], pl[3]);
    }
  }
  // layer 2's bias enters like the row part of layer 1: (hi, lo) of b2[unit l32] in k slots 0 and 1
  const unsigned b2pk = split1(tail[kH * kH + l32]);
  const float b3d = tail[kH * kH + kH + 2 * kH], b3m = tail[kH * kH + kH + 2 * kH + 1];

  // ---- column part of layer 1's C operand for this lane's column: units unit_of(v, half), v = 0..15
  f32x16 colc;
  float fg[3], fm[3];   // rsqrt(c_k + eps) of the column times the scale of features 10+k / 25+k
  {
    float cf[6];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      cf[k] = col_ok ? rst[3 * (size_t)T.padm + (size_t)k * T.padn + col] : 0.f;
      cf[3 + k] = col_ok ? ws[T.oRC + (size_t)k * T.padn + col] : 0.f;
      fg[k] = cf[3 + k] * ws[T.oScale + 10 + k];
      fm[k] = cf[3 + k] * ws[T.oScale + 25 + k];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int f = 0; f < 6; ++f) {
        const float4 w = *reinterpret_cast<const float4*>(prep + col_feat(f) * kH + 8 * q + 4 * half);
        a.x += cf[f] * w.x; a.y += cf[f] * w.y; a.z += cf[f] * w.z; a.w += cf[f] * w.w;
      }
      colc[4 * q] = a.x; colc[4 * q + 1] = a.y; colc[4 * q + 2] = a.z; colc[4 * q + 3] = a.w;
    }
  }
  float sc[10];  // normalization factors of features 0..9 (wave-uniform)
#pragma unroll
  for (int i = 0; i < 10; ++i) sc[i] = ws[T.oScale + i];

  // constant B operands that pick k slots (0, 1) of the lower / upper lane half
  const unsigned one2 = 0x3C003C00u;   // fp16 (1.0, 1.0)
  const f16x8 b_one_lo = pk8(half ? 0u : one2, 0u, 0u, 0u);
  const f16x8 b_one_hi = pk8(half ? one2 : 0u, 0u, 0u, 0u);

  // row part of one 64-row chunk -> LDS buffer `buf` (every thread: unit t & 31, rows (t >> 5) + 8 j)
  auto fill_chunk = [&](int rb0, int buf) {
    const int u = threadIdx.x & 31, rg = threadIdx.x >> 5;
    float w1r[6];
#pragma unroll
    for (int f = 0; f < 6; ++f) w1r[f] = L.w1row[f][u];
    const float b1u = L.b1[u];
#pragma unroll
    for (int j = 0; j < kChunkRows / 8; ++j) {
      const int lrow = rg + 8 * j, row = rb0 + lrow;
      unsigned pk = 0u;
      float4 rs4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row < r1) {
        float rb = b1u;
        float rr[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          rr[k] = ws[T.oRR + (size_t)k * T.padm + row];
          rb += rst[(size_t)k * T.padm + row] * w1r[k];
        }
#pragma unroll
        for (int k = 0; k < 3; ++k) rb += rr[k] * w1r[3 + k];
        pk = split1(rb);
        rs4 = make_float4(rr[0], rr[1], rr[2], 0.f);
      }
      L.rowinj[buf][lrow][u] = pk;   // rows past the end hold zeros: the injection MFMA multiplies them by 0
      if (u == 0) L.rowrs[buf][lrow] = rs4;
    }
  };

  __syncthreads();          // tables
  fill_chunk(r0, 0);
  __syncthreads();

  // ---- streaming: lanes of the lower half read row q, lanes of the upper half row q + 1 (q even relative to
  // r0, wave-uniform). Loads are unconditional: a column past the end reads the last column, the upper half of a
  // tensor's last odd row reads the lower half's row, rows past the end read the last row; such lanes compute on
  // real (finite) values and never store.
  Streams S;
  S.g = (gcf32)T.g; S.p = (gcf32)T.p;
  S.m1 = (gcf32)T.st; S.m2 = S.m1 + T.padN; S.m3 = S.m2 + T.padN; S.v = S.m3 + T.padN;
  const gf32 pout = (gf32)T.p;
  const unsigned colc_ = (unsigned)(col_ok ? col : n - 1);
  const unsigned voff_pair = colc_ + (half ? (unsigned)n : 0u);
  auto fetch = [&](int q) {
    const int qc = q < m ? q : m - 1;
    return load_elem(S, (size_t)qc * (size_t)n, qc + 1 < m ? voff_pair : colc_);
  };

  // one round: rows (q, q + 1) of the chunk that starts at rb0; `e` holds their streamed values on entry and
  // those of rows (q + 4, q + 5) on exit
  auto round = [&](Elem& e, int q, int rb0, int buf) {
    const int r = q + half;
    const int lrow = r - rb0;   // < kChunkRows: an odd tail's upper row is the zero-filled row r1 of the chunk
    const unsigned inj = L.rowinj[buf][lrow][l32];
    const float4 rr4 = L.rowrs[buf][lrow];
    // ---- the 16 per-element features, normalized, split, packed
    unsigned ph[8], pl[8];
    const float p_old = e.p;
    {
      const float g = e.g, q1 = e.m1, q2 = e.m2, q3 = e.m3, v = e.v;
      const float rs = RAW_RSQ ? __builtin_amdgcn_rsqf(v + eps) : rsqrtf(v + eps);
      const float tg0 = rr4.x * fg[0], tg1 = rr4.y * fg[1], tg2 = rr4.z * fg[2];
      const float tm0 = rr4.x * fm[0], tm1 = rr4.y * fm[1], tm2 = rr4.z * fm[2];
      split2(g * sc[0], p_old * sc[1], ph[0], pl[0]);
      split2(q1 * sc[2], q2 * sc[3], ph[1], pl[1]);
      split2(q3 * sc[4], v * sc[5], ph[2], pl[2]);
      split2((q1 * rs) * sc[6], (q2 * rs) * sc[7], ph[3], pl[3]);
      split2((q3 * rs) * sc[8], rs * sc[9], ph[4], pl[4]);
      split2(g * tg0, g * tg1, ph[5], pl[5]);
      split2(g * tg2, q1 * tm0, ph[6], pl[6]);
      split2(q2 * tm1, q3 * tm2, ph[7], pl[7]);
    }
    // the streamed values of this round are consumed: fetch this register set's next round
    e = fetch(q + 4);
    // registers 0..3 -> B operand of tile A (row q), registers 4..7 -> B operand of tile B (row q + 1)
    swap32x8(ph, pl);
    f32x16 h1a = __builtin_amdgcn_mfma_f32_32x32x16_f16(pk8(inj, 0u, 0u, 0u), b_one_lo, colc, 0, 0, 0);
    f32x16 h1b = __builtin_amdgcn_mfma_f32_32x32x16_f16(pk8(inj, 0u, 0u, 0u), b_one_hi, colc, 0, 0, 0);
    h1a = mfma3(a1h, a1l, pk8(ph[0], ph[1], ph[2], ph[3]), pk8(pl[0], pl[1], pl[2], pl[3]), h1a);
    h1b = mfma3(a1h, a1l, pk8(ph[4], ph[5], ph[6], ph[7]), pk8(pl[4], pl[5], pl[6], pl[7]), h1b);
    // layer 2, one tile after the other (bounds the live accumulators), then layer 3 of both on the vector ALU
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto layer2 = [&](const f32x16& h1) {
      f32x16 h2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(pk8(b2pk, 0u, 0u, 0u), b_one_lo, zero16, 0, 0, 0);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        f16x8 bh, bl;
        pack_relu8(h1, 8 * j, bh, bl);
        h2 = mfma3(a2h[j], a2l[j], bh, bl, h2);
      }
      return h2;
    };
    __builtin_amdgcn_sched_barrier(0);
    const f32x16 h2a = layer2(h1a);
    __builtin_amdgcn_sched_barrier(0);
    const f32x16 h2b = layer2(h1b);
    __builtin_amdgcn_sched_barrier(0);
    float da = 0.f, ma = 0.f, db = 0.f, mb = 0.f;
#pragma unroll
    for (int v2 = 0; v2 < 8; ++v2) {
      const float4 w = L.w3[half][v2];
      const float ha0 = relu(h2a[2 * v2]), ha1 = relu(h2a[2 * v2 + 1]);
      const float hb0 = relu(h2b[2 * v2]), hb1 = relu(h2b[2 * v2 + 1]);
      da += ha0 * w.x; ma += ha0 * w.y; da += ha1 * w.z; ma += ha1 * w.w;
      db += hb0 * w.x; mb += hb0 * w.y; db += hb1 * w.z; mb += hb1 * w.w;
    }
    // lower lanes keep tile A (their own row), upper lanes tile B (theirs): both halves of each sum meet
    swap32x2(da, db, ma, mb);
    const float d = (da + db) + b3d, mg = (ma + mb) + b3m;
    const float delta = d * __expf(mg * A.exp_mult) * A.step_mult;
    if (col_ok && r < r1)
      __builtin_nontemporal_store(p_old - lr * (delta + wd * p_old), pout + (size_t)q * (size_t)n + voff_pair);
  };

  Elem ea = fetch(r0), eb = fetch(r0 + 2);
  int buf = 0;
  for (int rb0 = r0; rb0 < r1; rb0 += kChunkRows, buf ^= 1) {
    if (rb0 + kChunkRows < r1) fill_chunk(rb0 + kChunkRows, buf ^ 1);
    const int rend = min(rb0 + kChunkRows, r1);
    for (int q = rb0; q < rend; q += 4) {   // a chunk holds an even number of rounds unless it is the last
      round(ea, q, rb0, buf);
      if (q + 2 < rend) round(eb, q + 2, rb0, buf);
    }
    __syncthreads();   // everyone is done with buffer `buf`; the other buffer is complete
  }
}

void launch_apply_f16s(const Launch& L, const StepArgs& A, const WeightsDev& W, hipStream_t s) {
  if (L.n_tiles == 0) return;
  // v_rsq_f32 treats inputs below the smallest normal float as zero; with eps_acc that small the kernel
  // takes the library reciprocal square root (which rescales such inputs) instead of the bare instruction
  if (A.eps_acc >= 1e-30f)
    hipLaunchKernelGGL(k_apply_f16s<true>, dim3(2 * (unsigned)L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles,
                       L.ws, A, W.mlp_tail);
  else
    hipLaunchKernelGGL(k_apply_f16s<false>, dim3(2 * (unsigned)L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles,
                       L.ws, A, W.mlp_tail);
}

}  // namespace lopt
