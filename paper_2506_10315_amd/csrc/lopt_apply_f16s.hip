// Column-strip, software-pipelined form of the split-fp16 matrix-core apply pass for small_fc_lopt,
// hidden width 32 (paper: "Kernel 2: fused feature construction and network application"; its H100
// appendix puts the MLP contraction on tensor cores).
//
// Why not the fp32 MFMA: on gfx950 v_mfma_f32_32x32x2_f32 runs at the rate of the vector FP32 lanes and does not
// overlap with vector-ALU work of the same SIMD (measured: time = MFMA time + VALU time), while the 16-bit MFMAs run
// on the matrix engine at 16x the rate and DO overlap with the vector ALU. So the two hidden-layer contractions are
// done in fp16 with fp32 accumulation, and every operand is carried as an unevaluated sum of two fp16 numbers,
// x = hi + lo with hi = fp16_rtz(x) and lo = fp16_rtz(x - hi): 22 significand bits. A product keeps the three
// leading terms
//   x*w = hi*Whi + lo*Whi + hi*Wlo            (the dropped lo*Wlo is below 2^-22 relative)
// i.e. three v_mfma_f32_32x32x16_f16 per 16 values of k. Accuracy is that of fp32 arithmetic to within a small factor;
// the range is fp16's, which is why features are normalized BEFORE the contraction (normalized features are bounded by
// sqrt(N) < 46341 < 65504) instead of folding the normalization into W1, and why lopt_create rescales the hidden
// units by powers of two (no pre-activation can leave the range).
//
// Layout: products are computed transposed, D[unit, element] = W^T[unit, k] X^T[k, element]. One MFMA takes 16 values
// of k: lanes 0..31 hold k 0..7 of element (lane & 31) as four packed registers, lanes 32..63 hold k 8..15 of the same
// element.
//   * layer 1 (k = the 16 per-element features): each lane packs its own element's features into 8 registers (hi) + 8
//     (lo); v_permlane32_swap of register i with register 4+i yields the B operands of the wave's two 32-element tiles.
//   * the accumulator leaves lane l with 16 hidden units of element (l & 31): registers 0..7 are k 0..7 of layer 2's
//     first MFMA for this lane half, registers 8..15 those of its second MFMA; ReLU, split and pack happen in place,
//     no cross-lane traffic. The weights are packed per lane in that order.
//   * layer 3 and the update: vector ALU, fp32.
//
// Ownership (what makes the kernel small in registers and in vector-ALU work):
//   * A wavefront owns a strip of 32 columns and sweeps its rows two at a time: lane (h, c) holds the
//     element (row q + h, column c). The wave's two 32-element MFMA tiles are therefore two ROWS of the
//     same 32 columns: the first-layer contribution of the six column-constant features is ONE set of 16
//     accumulator registers per strip, used as the C operand of both tiles in every round.
//   * The row-dependent part of the first layer (bias, time features, six row-constant features) is one
//     32-vector per row. The workgroup computes it once per tile into LDS as packed (hi, lo) fp16 pairs;
//     it enters through ONE extra MFMA per tile: A carries (hi, lo) in k slots 0 and 1 of the row's lane
//     half, B is the constant (1, 1) there and 0 elsewhere.
//   * Loads are one dword per array, lane and round (a 128-byte line per row), issued kSets rounds ahead. Stores
//     (the parameter, and with UPDATE_STATE the four accumulators) are raw buffer stores relative to the round's row
//     address; lanes outside the tile are dropped by the descriptor's range check, not by a branch.
//
// Schedule. Measured on gfx950: the 16-bit MFMA costs a wavefront about two issue slots when
// independent vector instructions of the SAME wavefront follow it in program order, and its full 32
// cycles when the wave has nothing else to issue; MFMAs of different wavefronts of a SIMD do not hide
// behind each other's vector work. So the loop is software-pipelined by hand: every MFMA is followed by
// a slice of vector work that belongs to another round,
//     layer-1 MFMAs of round i+1   |  layer 3 + update of round i
//     (ReLU/split of tile A, round i+1: vector ALU only)
//     layer-2 MFMAs, tile A, i+1   |  ReLU/split of tile B, round i+1
//     layer-2 MFMAs, tile B, i+1   |  features of round i+2
// and __builtin_amdgcn_sched_barrier(0) between the slices keeps the compiler from regrouping them.
// Workgroup = 4 wavefronts; it works through apply tiles of up to kApplyRows rows x 128 columns, one at a time.
#include <type_traits>

#include "lopt_apply_common.h"

namespace lopt {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kStripCols = 32;
constexpr int kRowSlack = 16;   // rows of zeros after the tile in the LDS row tables (read by the pipeline's run-out)

#ifndef LOPT_F16S_NSETS
#define LOPT_F16S_NSETS 2
#endif
constexpr int kSets = LOPT_F16S_NSETS;   // register sets of streamed values = rounds of loads in flight

#define LOPT_SB() __builtin_amdgcn_sched_barrier(0)

__device__ __forceinline__ f16x8 pk8(unsigned a, unsigned b, unsigned c, unsigned d) {
  u32x4 v = {a, b, c, d};
  return __builtin_bit_cast(f16x8, v);
}

// (a, b) -> packed hi pair and packed lo pair, hi = rtz_fp16(x), lo = rtz_fp16(x - hi). The residual
// x - float(hi) is one mixed-precision FMA (v_fma_mix_f32 reads the fp16 half directly, full rate; the
// variants that write an fp16 result run at half rate). One assembly block for the four instructions: after a
// separate asm statement the compiler has to assume an instruction whose result needs a wait state before its
// next use and pads every split with an s_nop; none of these four needs one.
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  // the residuals overwrite the registers of a and b, the packed lo pair that of a
  asm("v_cvt_pkrtz_f16_f32 %0, %1, %2\n\t"
      "v_fma_mix_f32 %1, %0, -1.0, %1 op_sel_hi:[1,0,0]\n\t"
      "v_fma_mix_f32 %2, %0, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
      "v_cvt_pkrtz_f16_f32 %1, %1, %2"
      : "=&v"(hi), "+v"(a), "+v"(b));
  lo = __builtin_bit_cast(unsigned, a);
}

// one value -> (hi in bits 0..15, lo in bits 16..31)
__device__ __forceinline__ unsigned split1(float a) {
  unsigned pk = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a, 0.f));
  asm("v_fma_mixhi_f16 %0, %0, -1.0, %1 op_sel_hi:[1,0,0]" : "+v"(pk) : "v"(a));
  return pk;
}

__device__ __forceinline__ f32x16 mfma(const f16x8& a, const f16x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

struct StripLds {
  unsigned rowinj[kApplyRows + kRowSlack][32];  // [row of the tile][unit]: packed (hi, lo) of bias + row part
  float4 rowrs[kApplyRows + kRowSlack];         // rsqrt(r_k + eps) of the row, k = 0..2
  float w1row[6][32];                           // prepared first layer, rows of the row-constant features
  float w1col[6][32];                           // prepared first layer, rows of the column-constant features
  float b1[32];                                 // prepared bias (time features folded in)
  float4 w3[2][8];                              // [half][v/2]: W3 rows d(v) m(v) d(v+1) m(v+1) of units unit_of(v, half)
};

struct Elem { float g, p, m1, m2, m3, v; };

// The streamed arrays as global-memory pointers (wave-uniform base + lane offset).
typedef const float __attribute__((address_space(1)))* gcf32;
typedef float __attribute__((address_space(1)))* gf32;
typedef char __attribute__((address_space(1)))* gc8;
struct Streams { gcf32 g, p, m1, m2, m3, v; };

typedef const char __attribute__((address_space(1)))* gcc8;

// One dword per array at (wave-uniform row offset in elements) + (lane offset in BYTES, 32 bits): written so
// that the address is scalar base + zero-extended 32-bit vector offset, the form a global load takes directly.
__device__ __forceinline__ float ld_stream(gcf32 base, size_t rowoff, unsigned voff_bytes) {
  return __builtin_nontemporal_load((gcf32)((gcc8)(base + rowoff) + voff_bytes));
}
__device__ __forceinline__ Elem load_elem(const Streams& S, size_t rowoff, unsigned voff_bytes) {
  Elem e;
  e.g = ld_stream(S.g, rowoff, voff_bytes);
  e.p = ld_stream(S.p, rowoff, voff_bytes);
  e.m1 = ld_stream(S.m1, rowoff, voff_bytes);
  e.m2 = ld_stream(S.m2, rowoff, voff_bytes);
  e.m3 = ld_stream(S.m3, rowoff, voff_bytes);
  e.v = ld_stream(S.v, rowoff, voff_bytes);
  return e;
}

// Per-lane constants of a strip.
struct Consts {
  f16x8 a1h, a1l, a2h[2], a2l[2];   // split and packed W1 (16 per-element rows) and W2
  f32x16 colc, cb2;                 // C operands: column part of layer 1, bias of layer 2
  float fg[3], fm[3];               // rsqrt(c_k + eps) of the column times the scale of features 10+k / 25+k
  float sc[10];                     // normalization factors of features 0..9 (wave-uniform)
  f16x8 b_one_lo, b_one_hi;         // B operands selecting k slots (0, 1) of the lower / upper lane half
  float eps, lr, wd, exp_mult, step_mult, b3d, b3m;
  float bm[3], am[3], bv, av;       // decays beta_1..3, beta_4 and 1 - beta (UPDATE_STATE: the accumulators move in this pass)
};

// Features of one round, normalized, split and packed: after the lane-half swap registers 0..3 are the B
// operand of tile A (row q), registers 4..7 that of tile B (row q + 1).
struct Feat { unsigned ph[8], pl[8]; float p_old; };

struct FeatTmp { float rs; };

// A wave-uniform global pointer, held in scalar registers.
__device__ __forceinline__ gc8 uniform_ptr(gc8 p) {
  const unsigned long long a = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  return (gc8)(((unsigned long long)hi << 32) | lo);
}

// Stores go out as raw buffer stores whose descriptor starts at the round's (wave-uniform) row address: a lane that
// must not store passes an offset beyond the descriptor's range and the hardware drops its write. No branch and no
// change of the execution mask surrounds the store, so the compiler counts the memory operations in flight exactly
// (with a skipped region it has to assume the fewest, and every wait for a load then also waits for the stores issued
// before it to be acknowledged). Lane offsets of real elements stay below kStoreRange (the launcher's shape check).
constexpr unsigned kStoreRange = 0xFFFFFE00u;
constexpr unsigned kNoStore = 0xFFFFFFFFu;
__device__ __forceinline__ void store_stream(float v, gc8 row_base, unsigned voff_or_none) {
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)uniform_ptr(row_base), 0, (int)kStoreRange,
                                                                      0x00020000);   // raw buffer, 32-bit data
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, (int)voff_or_none, 0, 2 /* nontemporal */);
}

// UPDATE_STATE: the momentum and second-moment accumulators of this round's elements are updated HERE, from the
// values of the previous step, in the same arithmetic as the statistics pass (which then only reads them), and stored:
// M_i <- beta_i M_i + (1 - beta_i) g, V <- beta_4 V + (1 - beta_4) g^2. The features below are built from the new values.
// `keep`: this lane's element lies inside the tile (the run-out rounds and the padding lanes compute, but store nothing).
__device__ __forceinline__ void update_state(const Consts& C, Elem& e, const Streams& S, size_t rowoff, unsigned voff_bytes,
                                             bool keep) {
  const float g = e.g;
  e.m1 = __builtin_fmaf(C.bm[0], e.m1, C.am[0] * g);   // the statistics pass's operations, in its order
  e.m2 = __builtin_fmaf(C.bm[1], e.m2, C.am[1] * g);
  e.m3 = __builtin_fmaf(C.bm[2], e.m3, C.am[2] * g);
  e.v = __builtin_fmaf(C.bv, e.v, C.av * (g * g));
  const unsigned vo = keep ? voff_bytes : kNoStore;
  store_stream(e.m1, (gc8)((gf32)S.m1 + rowoff), vo);
  store_stream(e.m2, (gc8)((gf32)S.m2 + rowoff), vo);
  store_stream(e.m3, (gc8)((gf32)S.m3 + rowoff), vo);
  store_stream(e.v, (gc8)((gf32)S.v + rowoff), vo);
}

// The feature computation in six slices (one per MFMA of the phase it hides behind). The products of the row and
// column factors are formed in the slice that uses them (fewer values live across slices).
template <int PIECE, bool RAW_RSQ>
__device__ __forceinline__ void feat_piece(const Consts& C, const Elem& e, const float4& rr4, FeatTmp& t, Feat& f) {
  if (PIECE == 0) {
    t.rs = RAW_RSQ ? __builtin_amdgcn_rsqf(e.v + C.eps) : rsqrtf(e.v + C.eps);
    // an explicit copy: otherwise the old parameter value stays in the load's register, the next load of this
    // set lands elsewhere, and the loop's back edge needs a copy of a value that is still in flight
    asm volatile("v_mov_b32 %0, %1" : "=v"(f.p_old) : "v"(e.p));
    split2(e.g * C.sc[0], e.p * C.sc[1], f.ph[0], f.pl[0]);
  } else if (PIECE == 1) {
    split2(e.m1 * C.sc[2], e.m2 * C.sc[3], f.ph[1], f.pl[1]);
    split2(e.m3 * C.sc[4], e.v * C.sc[5], f.ph[2], f.pl[2]);
  } else if (PIECE == 2) {
    split2((e.m1 * t.rs) * C.sc[6], (e.m2 * t.rs) * C.sc[7], f.ph[3], f.pl[3]);
  } else if (PIECE == 3) {
    split2((e.m3 * t.rs) * C.sc[8], t.rs * C.sc[9], f.ph[4], f.pl[4]);
    split2(e.g * (rr4.x * C.fg[0]), e.g * (rr4.y * C.fg[1]), f.ph[5], f.pl[5]);
  } else if (PIECE == 4) {
    split2(e.g * (rr4.z * C.fg[2]), e.m1 * (rr4.x * C.fm[0]), f.ph[6], f.pl[6]);
    split2(e.m2 * (rr4.y * C.fm[1]), e.m3 * (rr4.z * C.fm[2]), f.ph[7], f.pl[7]);
  } else {
    swap32x8(f.ph, f.pl);
  }
}

// ReLU, split and pack one pair of accumulator registers of layer 1
__device__ __forceinline__ void relu_split_pair(const f32x16& h, int idx, unsigned& hi, unsigned& lo) {
  split2(relu(h[idx]), relu(h[idx + 1]), hi, lo);
}

// Layer 3 for two units (accumulator registers 2*V2, 2*V2+1) of both tiles; w = d(v) m(v) d(v+1) m(v+1)
template <int V2>
__device__ __forceinline__ void layer3_piece(const float4& w, const f32x16& h2a, const f32x16& h2b, float& da, float& ma,
                                             float& db, float& mb) {
  const float ha0 = relu(h2a[2 * V2]), ha1 = relu(h2a[2 * V2 + 1]);
  const float hb0 = relu(h2b[2 * V2]), hb1 = relu(h2b[2 * V2 + 1]);
  da += ha0 * w.x; ma += ha0 * w.y; da += ha1 * w.z; ma += ha1 * w.w;
  db += hb0 * w.x; mb += hb0 * w.y; db += hb1 * w.z; mb += hb1 * w.w;
}

}  // namespace

template <bool RAW_RSQ, bool UPDATE_STATE>
__global__ void __launch_bounds__(kBlock, 2) k_apply_f16s(const TensorDev* __restrict__ tensors,
                                                          const ApplyTileDev* __restrict__ atiles, int n_atiles,
                                                          int* __restrict__ next_tile, float* __restrict__ ws,
                                                          StepArgs A, const float* __restrict__ tail) {
  __shared__ StripLds L;
  __shared__ int s_tile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;

  // ---- what does not depend on the tile: W3 table, packed weights, scalars
  if (threadIdx.x < 16) {
    const int hf = (threadIdx.x >> 3) & 1, v2 = threadIdx.x & 7;
    const float* w3g = tail + kH * kH + kH;
    const int u0 = unit_of(2 * v2, hf), u1 = unit_of(2 * v2 + 1, hf);
    L.w3[hf][v2] = make_float4(w3g[2 * u0], w3g[2 * u0 + 1], w3g[2 * u1], w3g[2 * u1 + 1]);
  }
  Consts C;
  C.eps = A.eps_acc; C.lr = A.lr; C.wd = A.wd; C.exp_mult = A.exp_mult; C.step_mult = A.step_mult;
#pragma unroll
  for (int i = 0; i < 3; ++i) { C.bm[i] = A.mom_decay[i]; C.am[i] = 1.0f - A.mom_decay[i]; }
  C.bv = A.rms_decay; C.av = 1.0f - A.rms_decay;
  C.b3d = tail[kH * kH + kH + 2 * kH]; C.b3m = tail[kH * kH + kH + 2 * kH + 1];
  // ---- weights of this lane, split and packed in the order the accumulator layout asks for
  {
    const float* __restrict__ w1raw = tail + (kH * kH + kH + 2 * kH + 2 + 2);  // W1[28][32], not normalized
    unsigned ph[4], pl[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float w0 = half ? w1raw[elem_feat(8 + 2 * i) * kH + l32] : w1raw[elem_feat(2 * i) * kH + l32];
      const float w1 = half ? w1raw[elem_feat(9 + 2 * i) * kH + l32] : w1raw[elem_feat(2 * i + 1) * kH + l32];
      split2(w0, w1, ph[i], pl[i]);
    }
    C.a1h = pk8(ph[0], ph[1], ph[2], ph[3]);
    C.a1l = pk8(pl[0], pl[1], pl[2], pl[3]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float w0 = tail[unit_of(8 * j + 2 * i, half) * kH + l32];
        const float w1 = tail[unit_of(8 * j + 2 * i + 1, half) * kH + l32];
        split2(w0, w1, ph[i], pl[i]);
      }
      C.a2h[j] = pk8(ph[0], ph[1], ph[2], ph[3]);
      C.a2l[j] = pk8(pl[0], pl[1], pl[2], pl[3]);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) C.cb2[v] = tail[kH * kH + unit_of(v, half)];
  }
  const unsigned one2 = 0x3C003C00u;   // fp16 (1.0, 1.0)
  C.b_one_lo = pk8(half ? 0u : one2, 0u, 0u, 0u);
  C.b_one_hi = pk8(half ? one2 : 0u, 0u, 0u, 0u);

  // ---- tiles are handed out through a counter: a workgroup takes the next one when it is done with its last,
  // so the launch is as many workgroups as fit on the chip and ends without a ragged last round
  for (;;) {
  if (threadIdx.x == 0) s_tile = atomicAdd(next_tile, 1);
  __syncthreads();   // also: every wavefront is done with the previous tile's LDS tables
  const int tile_id = s_tile;
  if (tile_id >= n_atiles) break;
  const ApplyTileDev at = atiles[tile_id];
  const TensorDev& T = tensors[at.tensor];
  const int n = T.n, m = T.m;
  const float* __restrict__ prep = ws + T.oPrep;  // W1s[28][32] (normalization folded in), b1'[32]
  const int col = at.c0 + wave * kStripCols + l32;
  const bool col_ok = col < n;
  const int r0 = at.r0, r1 = at.r0 + at.rows;
  const float* __restrict__ rst = T.st + 4 * (size_t)T.padN;   // r_k[3][padm] then c_k[3][padn]
  {
    const int t = threadIdx.x;
    if (t < 192) {
      L.w1row[t >> 5][t & 31] = prep[row_feat(t >> 5) * kH + (t & 31)];
      L.w1col[t >> 5][t & 31] = prep[col_feat(t >> 5) * kH + (t & 31)];
    } else if (t < 224) L.b1[t - 192] = prep[kNF * kH + (t - 192)];
  }
#pragma unroll
  for (int i = 0; i < 10; ++i) C.sc[i] = ws[T.oScale + i];
  __syncthreads();   // w1row, w1col, b1
  // ---- column part of layer 1's C operand for this lane's column: units unit_of(v, half), v = 0..15
  {
    float cf[6];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      cf[k] = col_ok ? rst[3 * (size_t)T.padm + (size_t)k * T.padn + col] : 0.f;
      cf[3 + k] = col_ok ? ws[T.oRC + (size_t)k * T.padn + col] : 0.f;
      C.fg[k] = cf[3 + k] * ws[T.oScale + 10 + k];
      C.fm[k] = cf[3 + k] * ws[T.oScale + 25 + k];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int f = 0; f < 6; ++f) {
        const float4 w = *reinterpret_cast<const float4*>(&L.w1col[f][8 * q + 4 * half]);
        a.x += cf[f] * w.x; a.y += cf[f] * w.y; a.z += cf[f] * w.z; a.w += cf[f] * w.w;
      }
      C.colc[4 * q] = a.x; C.colc[4 * q + 1] = a.y; C.colc[4 * q + 2] = a.z; C.colc[4 * q + 3] = a.w;
    }
  }
  // ---- row part of the tile's rows -> LDS (thread: unit t & 31, rows (t >> 5), +8, ...); rows past the tile
  // hold zeros: the injection MFMA multiplies them by 0, and the pipeline's run-out rounds read them
  {
    const int u = threadIdx.x & 31;
    float w1r[6];
#pragma unroll
    for (int f = 0; f < 6; ++f) w1r[f] = L.w1row[f][u];
    const float b1u = L.b1[u];
    for (int lrow = threadIdx.x >> 5; lrow < at.rows + kRowSlack; lrow += kBlock / 32) {
      const int row = r0 + lrow;
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
      L.rowinj[lrow][u] = pk;
      if (u == 0) L.rowrs[lrow] = rs4;
    }
  }
  __syncthreads();

  // ---- streaming: lanes of the lower half read row q, lanes of the upper half row q + 1 (q - r0 even,
  // wave-uniform). Loads are unconditional: a column past the end reads the last column, the upper half of a
  // tensor's last odd row reads the lower half's row, rounds past the tile read the tile's last row; such lanes
  // compute on real (finite) values and never store.
  Streams S;
  S.g = (gcf32)T.g; S.p = (gcf32)T.p;
  S.m1 = (gcf32)T.st; S.m2 = S.m1 + T.padN; S.m3 = S.m2 + T.padN; S.v = S.m3 + T.padN;
  const gf32 pout = (gf32)T.p;
  // lane offsets in bytes, relative to the tile's first column (which goes into the wave-uniform row offset): at most
  // 4 (127 + n) <= kStoreRange - 4 whenever a tensor has a second row (the launcher sends wider ones to another kernel)
  const size_t c0 = (size_t)at.c0;
  const unsigned colc_ = 4u * (unsigned)((col_ok ? col : n - 1) - at.c0);
  const unsigned voff_pair = colc_ + (half ? 4u * (unsigned)n : 0u);
  // wave-uniform element offset of round q's first row (the tile's first column included); only used for rows inside the tile
  auto rowoff_of = [&](int q) __attribute__((always_inline)) { return (size_t)q * (size_t)n + c0; };
  // the pipeline's run-out rounds (q >= r1) read the tile's last row once more: a cache hit, not HBM traffic
  auto fetch = [&](int q) __attribute__((always_inline)) {
    const bool in_tile = q < r1;
    const int qc = in_tile ? q : r1 - 1;
    return load_elem(S, (size_t)qc * (size_t)n + c0, in_tile && qc + 1 < m ? voff_pair : colc_);
  };

  // One step of the pipeline. On entry: h2a/h2b/p_e belong to the round of rows qe, qe+1 (layer 3 and update
  // pending, if DO_E), `f` holds the swapped features of the round at qe + 2 (its layer 1 pending) and `e` the
  // streamed values of the round at qe + 4. On exit everything has moved on by one round and `e` holds the
  // round at qe + 8 (the next one that uses this register set).
  f32x16 h2a, h2b;
  float p_e = 0.f;
  Feat f;
  auto step = [&](auto do_e, Elem& e, int qe) __attribute__((always_inline)) {
    constexpr bool DO_E = decltype(do_e)::value;
    const int qn = qe + 2, qf = qe + 4;
    // ---- phase 1: layer-1 MFMAs of round qn | layer 3 + update of round qe
    const unsigned inj = L.rowinj[qn + half - r0][l32];
    const float4 rr4 = L.rowrs[qf + half - r0];
    f32x16 h1a, h1b;
    float da = 0.f, ma = 0.f, db = 0.f, mb = 0.f;
    const f16x8 injA = pk8(inj, 0u, 0u, 0u);
    const f16x8 bha = pk8(f.ph[0], f.ph[1], f.ph[2], f.ph[3]), bla = pk8(f.pl[0], f.pl[1], f.pl[2], f.pl[3]);
    const f16x8 bhb = pk8(f.ph[4], f.ph[5], f.ph[6], f.ph[7]), blb = pk8(f.pl[4], f.pl[5], f.pl[6], f.pl[7]);
    const float p_n = f.p_old;
    float4 wn = L.w3[half][0];   // W3 comes from LDS one slice ahead of its use (two distinct addresses per wave)
    LOPT_SB();
    h1a = mfma(injA, C.b_one_lo, C.colc);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][1]; layer3_piece<0>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1b = mfma(injA, C.b_one_hi, C.colc);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][2]; layer3_piece<1>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1a = mfma(C.a1l, bha, h1a);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][3]; layer3_piece<2>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1b = mfma(C.a1l, bhb, h1b);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][4]; layer3_piece<3>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1a = mfma(C.a1h, bla, h1a);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][5]; layer3_piece<4>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1b = mfma(C.a1h, blb, h1b);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][6]; layer3_piece<5>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1a = mfma(C.a1h, bha, h1a);
    LOPT_SB();
    if (DO_E) { const float4 w = wn; wn = L.w3[half][7]; layer3_piece<6>(w, h2a, h2b, da, ma, db, mb); }
    LOPT_SB();
    h1b = mfma(C.a1h, bhb, h1b);
    LOPT_SB();
    if (DO_E) {
      layer3_piece<7>(wn, h2a, h2b, da, ma, db, mb);
      // lower lanes keep tile A (their own row), upper lanes tile B (theirs): both halves of each sum meet
      swap32x2(da, db, ma, mb);
      const float d = (da + db) + C.b3d, mg = (ma + mb) + C.b3m;
      const float delta = d * __expf(mg * C.exp_mult) * C.step_mult;
      store_stream(p_e - C.lr * (delta + C.wd * p_e), (gc8)(pout + ((size_t)qe * (size_t)n + c0)),
                   col_ok && qe + half < r1 ? voff_pair : kNoStore);
    }
    p_e = p_n;
    LOPT_SB();
    // ---- phase 2: ReLU/split of tile A (vector ALU only)
    unsigned ah[8], al[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) relu_split_pair(h1a, 2 * i, ah[i], al[i]);
    LOPT_SB();
    // ---- phase 3: layer-2 MFMAs of tile A | ReLU/split of tile B
    unsigned bh[8], bl[8];
    h2a = mfma(C.a2l[0], pk8(ah[0], ah[1], ah[2], ah[3]), C.cb2);
    LOPT_SB();
    relu_split_pair(h1b, 0, bh[0], bl[0]);
    relu_split_pair(h1b, 2, bh[1], bl[1]);
    LOPT_SB();
    h2a = mfma(C.a2h[0], pk8(al[0], al[1], al[2], al[3]), h2a);
    LOPT_SB();
    relu_split_pair(h1b, 4, bh[2], bl[2]);
    LOPT_SB();
    h2a = mfma(C.a2h[0], pk8(ah[0], ah[1], ah[2], ah[3]), h2a);
    LOPT_SB();
    relu_split_pair(h1b, 6, bh[3], bl[3]);
    LOPT_SB();
    h2a = mfma(C.a2l[1], pk8(ah[4], ah[5], ah[6], ah[7]), h2a);
    LOPT_SB();
    relu_split_pair(h1b, 8, bh[4], bl[4]);
    relu_split_pair(h1b, 10, bh[5], bl[5]);
    LOPT_SB();
    h2a = mfma(C.a2h[1], pk8(al[4], al[5], al[6], al[7]), h2a);
    LOPT_SB();
    relu_split_pair(h1b, 12, bh[6], bl[6]);
    LOPT_SB();
    h2a = mfma(C.a2h[1], pk8(ah[4], ah[5], ah[6], ah[7]), h2a);
    LOPT_SB();
    relu_split_pair(h1b, 14, bh[7], bl[7]);
    LOPT_SB();
    // ---- phase 4: layer-2 MFMAs of tile B | features of round qf
    FeatTmp t;
    h2b = mfma(C.a2l[0], pk8(bh[0], bh[1], bh[2], bh[3]), C.cb2);
    LOPT_SB();
    if (UPDATE_STATE) update_state(C, e, S, rowoff_of(qf), voff_pair, col_ok && qf + half < r1);
    feat_piece<0, RAW_RSQ>(C, e, rr4, t, f);
    LOPT_SB();
    h2b = mfma(C.a2h[0], pk8(bl[0], bl[1], bl[2], bl[3]), h2b);
    LOPT_SB();
    feat_piece<1, RAW_RSQ>(C, e, rr4, t, f);
    LOPT_SB();
    h2b = mfma(C.a2h[0], pk8(bh[0], bh[1], bh[2], bh[3]), h2b);
    LOPT_SB();
    feat_piece<2, RAW_RSQ>(C, e, rr4, t, f);
    LOPT_SB();
    h2b = mfma(C.a2l[1], pk8(bh[4], bh[5], bh[6], bh[7]), h2b);
    LOPT_SB();
    feat_piece<3, RAW_RSQ>(C, e, rr4, t, f);
    LOPT_SB();
    h2b = mfma(C.a2h[1], pk8(bl[4], bl[5], bl[6], bl[7]), h2b);
    LOPT_SB();
    feat_piece<4, RAW_RSQ>(C, e, rr4, t, f);
    LOPT_SB();
    h2b = mfma(C.a2h[1], pk8(bh[4], bh[5], bh[6], bh[7]), h2b);
    LOPT_SB();
    e = fetch(qf + 2 * kSets);   // this register set's next round
    feat_piece<5, RAW_RSQ>(C, e, rr4, t, f);
    LOPT_SB();
  };

  // ---- prologue: features of the first round with nothing to hide behind, then one step without layer 3.
  // Round k (rows r0 + 2k, +1) streams through register set k % kSets.
  Elem es[kSets];
#pragma unroll
  for (int s = 0; s < kSets; ++s) es[s] = fetch(r0 + 2 * s);
  {
    const float4 rr4 = L.rowrs[half];
    FeatTmp t;
    if (UPDATE_STATE) update_state(C, es[0], S, rowoff_of(r0), voff_pair, col_ok && r0 + half < r1);
    feat_piece<0, RAW_RSQ>(C, es[0], rr4, t, f);
    feat_piece<1, RAW_RSQ>(C, es[0], rr4, t, f);
    feat_piece<2, RAW_RSQ>(C, es[0], rr4, t, f);
    feat_piece<3, RAW_RSQ>(C, es[0], rr4, t, f);
    feat_piece<4, RAW_RSQ>(C, es[0], rr4, t, f);
    es[0] = fetch(r0 + 2 * kSets);
    feat_piece<5, RAW_RSQ>(C, es[0], rr4, t, f);
  }
  step(std::false_type{}, es[1 % kSets], r0 - 2);   // layers 1-2 of the first row pair, features of the second
  for (int q = r0; q < r1; q += 2 * kSets) {
#pragma unroll
    for (int s = 0; s < kSets; ++s)   // update rows q + 2s, +1 (nothing is stored past the tile); features of round +2
      step(std::true_type{}, es[(s + 2) % kSets], q + 2 * s);
  }
  }   // tile loop
}

// L.apply_counter must be zero when the kernel starts (k_finalize of the same sub-list clears it).
// update_state: the statistics pass left M_1..3 and V as they were (launch_accum_stats with write_state = false) and this
// pass moves them.
void launch_apply_f16s(const Launch& L, const StepArgs& A, const WeightsDev& W, bool update_state, hipStream_t s) {
  if (L.n_atiles == 0) return;
  const int grid = L.n_atiles < L.resident_wgs ? L.n_atiles : L.resident_wgs;
  // v_rsq_f32 treats inputs below the smallest normal float as zero; with eps_acc that small the kernel
  // takes the library reciprocal square root (which rescales such inputs) instead of the bare instruction
  const bool raw = A.eps_acc >= 1e-30f;
#define LOPT_LAUNCH_F16S(R, U)                                                                                  \
  hipLaunchKernelGGL((k_apply_f16s<R, U>), dim3(grid), dim3(kBlock), 0, s, L.tensors, L.atiles, L.n_atiles,       \
                     L.apply_counter, L.ws, A, W.mlp_tail)
  if (raw && update_state) LOPT_LAUNCH_F16S(true, true);
  else if (raw) LOPT_LAUNCH_F16S(true, false);
  else if (update_state) LOPT_LAUNCH_F16S(false, true);
  else LOPT_LAUNCH_F16S(false, false);
#undef LOPT_LAUNCH_F16S
}

}  // namespace lopt
