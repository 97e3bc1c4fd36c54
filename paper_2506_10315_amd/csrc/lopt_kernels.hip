// gfx950 kernels of the learned-optimizer step (paper: section "Optimized Kernel Design").
//
// The paper's two CUDA kernels (feature statistics; fused apply) are re-cut here into a
// fixed sequence of launches that each cover ALL tensors of the step through a table of
// work items (one workgroup = one tile of one tensor):
//   rowcol_sums  : per tile, sum of g^2 over the tile's columns (per row) and rows (per column)
//                  (+ VeLO: extra workgroups sum the tensors' previous LSTM outputs, slice by slice)
//   rc_update    : per row / per column: finish the means, update r_k, c_k, keep rsqrt(r_k+eps),
//                  rsqrt(c_k+eps), and partial sums for the row/column-constant features
//                  (+ VeLO: extra workgroups finish the cross-tensor mean and its gate contribution)
//   accum_stats  : M_i, V update + per-tile sums of squares of the per-element features
//   finalize     : per tensor, fixed-order reduction of all partials -> s_f, scale factors,
//                  first MLP layer with the normalization folded in (small_fc_lopt), LSTM input incl. time and
//                  loss features (VeLO)
//   velo_lstm, velo_head : the per-tensor hypernetwork (VeLO only)
//   apply        : rebuild features, MLP, exponentiated update (lopt_apply_mfma.hip has the
//                  matrix-core variant for hidden width 32)
// A tile is TR rows x 256 columns; a wavefront owns whole rows of the tile (lane l holds the
// four consecutive columns 4l..4l+3 as one float4), so row indices are wave-uniform and the
// column factors are loaded once per tile.
#include "lopt_internal.h"
#include "lopt_device.h"

namespace lopt {

// ----------------------------------------------------------------------------- fill

__global__ void __launch_bounds__(kBlock) k_fill_zero(const TensorDev* __restrict__ tensors, int H2) {
  const TensorDev T = tensors[blockIdx.y];
  size_t total = 4 * (size_t)T.padN + 3 * (size_t)T.padm + 3 * (size_t)T.padn + (size_t)H2 * T.padH;
  size_t n4 = total / 4;  // every section is a multiple of 4 floats
  float4* dst = reinterpret_cast<float4*>(T.st);
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock)
    dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

void launch_fill_zero(const Launch& L, const StepArgs& A, hipStream_t s) {
  if (L.n_tensors == 0) return;
  // grid.y is limited to 65535: loop over slabs of tensors
  for (int t0 = 0; t0 < L.n_tensors; t0 += 32768) {
    int nt = L.n_tensors - t0 < 32768 ? L.n_tensors - t0 : 32768;
    hipLaunchKernelGGL(k_fill_zero, dim3(64, nt), dim3(kBlock), 0, s, L.tensors + t0,
                       A.kind == LOPT_VELO ? 2 : 0);
  }
}

// ----------------------------------------------------------------------------- VeLO cross-tensor term

// The cross-tensor input of VeLO's LSTM depends on nothing this step computes (it reads the LSTM outputs h the previous
// step left in the state blobs), so its two stages ride along as extra workgroups of the first two launches of the
// step instead of taking launches of their own: slice sums of h behind the tiles of k_rowcol_sums, the final mean and
// the gate bias b_eff = b + hbar Wg behind the row/column blocks of k_rc_update. Both have a fixed summation order.
struct MixArgs {
  const float* Wg;        // [HL][4 HL]
  const float* b;         // [4 HL]
  float* part;            // [n_slices][HL] slice sums of h
  float* b_eff;           // [kMixJSplit][4 HL]: hbar Wg summed over a quarter of the units j each
  int HL, n_tensors, per_slice, n_slices;   // n_slices == 0: not VeLO, no extra workgroups
};

// Workgroup (chunk of 64 units, slice of the tensor list): lane = unit j, the four wavefronts take every fourth tensor
// of the slice, four tensors in flight each, and meet in LDS.
__device__ __forceinline__ void mix_hbar_block(const TensorDev* __restrict__ tensors, const MixArgs& M, int blk,
                                               float (*red)[kWave]) {
  const int n_chunks = (M.HL + kWave - 1) / kWave;
  const int chunk = blk % n_chunks, slice = blk / n_chunks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = min(chunk * kWave + lane, M.HL - 1);   // lanes past the end repeat the last unit (dropped below)
  const int t0 = slice * M.per_slice, t1 = min(t0 + M.per_slice, M.n_tensors);
  float a = 0.f;
  for (int t = t0 + wave; t < t1; t += 16) {
    float v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int tt = min(t + 4 * k, t1 - 1);
      const TensorDev& T = tensors[tt];
      v[k] = T.st[4 * (size_t)T.padN + 3 * (size_t)T.padm + 3 * (size_t)T.padn + j];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) a += t + 4 * k < t1 ? v[k] : 0.f;
  }
  red[wave][lane] = a;
  __syncthreads();
  if (wave == 0 && chunk * kWave + lane < M.HL)
    M.part[(size_t)slice * M.HL + j] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

// Workgroup = 64 gate columns (lane = column: coalesced rows of Wg) x one quarter of the units j; its four wavefronts
// take every fourth unit of the quarter, eight rows in flight each, and meet in LDS in a fixed order. The quarters
// are added up (with the bias b) by k_velo_lstm, again in a fixed order.
__device__ __forceinline__ void mix_bias_block(const MixArgs& M, int blk, float* hbar, float (*red)[kWave]) {
  const int HL = M.HL, G = 4 * HL;
  const int n_colblk = (G + kWave - 1) / kWave;
  const int colblk = blk % n_colblk, quarter = blk / n_colblk;
  const int jq = (HL + kMixJSplit - 1) / kMixJSplit;
  const int j0 = quarter * jq, j1 = min(j0 + jq, HL);
  for (int j = j0 + (int)threadIdx.x; j < j1; j += kBlock) {
    double a = 0.0;
    for (int s = 0; s < M.n_slices; ++s) a += (double)M.part[(size_t)s * HL + j];
    hbar[j - j0] = (float)(a / (double)M.n_tensors);
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = min(colblk * kWave + lane, G - 1);
  const float* __restrict__ wg = M.Wg + col;
  float a = 0.f;
  for (int j = j0 + wave; j < j1; j += 32) {
    float w[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = wg[(size_t)min(j + 4 * k, j1 - 1) * G];
#pragma unroll
    for (int k = 0; k < 8; ++k) a += j + 4 * k < j1 ? hbar[j + 4 * k - j0] * w[k] : 0.f;
  }
  red[wave][lane] = a;
  __syncthreads();
  if (wave == 0 && colblk * kWave + lane < G)
    M.b_eff[(size_t)quarter * G + col] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

static MixArgs make_mix(const Launch& L, const StepArgs& A, const WeightsDev& W, float* hbar_part, float* b_eff) {
  MixArgs M{};
  if (A.kind != LOPT_VELO || L.n_tensors == 0) return M;
  M.Wg = W.Wg; M.b = W.b; M.part = hbar_part; M.b_eff = b_eff;
  M.HL = A.HL; M.n_tensors = L.n_tensors;
  int per_slice = (L.n_tensors + kMixSlices - 1) / kMixSlices;
  if (per_slice < 16) per_slice = 16;   // four tensors in flight on each of four wavefronts
  M.per_slice = per_slice;
  M.n_slices = (L.n_tensors + per_slice - 1) / per_slice;
  return M;
}

// ----------------------------------------------------------------------------- rowcol_sums

template <bool VEC>
__device__ __forceinline__ void rowcol_tile(const TensorDev& T, const TileDev& tile, float* __restrict__ ws,
                                            float (*colred)[kTileCols]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = T.n, m = T.m;
  const int col = tile.tj * kTileCols + 4 * lane;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  float* __restrict__ rowpart = ws + T.oRowPart + (size_t)tile.tj * m;
  float c0 = 0.f, c1 = 0.f, c2 = 0.f, c3 = 0.f;
  int r = r0 + wave;
  // two rows in flight per wavefront
  for (; r + 4 < r1; r += 8) {
    float4 a = load4s<VEC>(T.g + (size_t)r * n, col, n);
    float4 b = load4s<VEC>(T.g + (size_t)(r + 4) * n, col, n);
    float ax = a.x * a.x, ay = a.y * a.y, az = a.z * a.z, aw = a.w * a.w;
    float bx = b.x * b.x, by = b.y * b.y, bz = b.z * b.z, bw = b.w * b.w;
    c0 += ax; c1 += ay; c2 += az; c3 += aw;
    c0 += bx; c1 += by; c2 += bz; c3 += bw;
    float sa = wave_sum((ax + ay) + (az + aw));
    float sb = wave_sum((bx + by) + (bz + bw));
    if (lane == 0) { rowpart[r] = sa; rowpart[r + 4] = sb; }
  }
  for (; r < r1; r += 4) {
    float4 a = load4s<VEC>(T.g + (size_t)r * n, col, n);
    float ax = a.x * a.x, ay = a.y * a.y, az = a.z * a.z, aw = a.w * a.w;
    c0 += ax; c1 += ay; c2 += az; c3 += aw;
    float sa = wave_sum((ax + ay) + (az + aw));
    if (lane == 0) rowpart[r] = sa;
  }
  colred[wave][4 * lane + 0] = c0;
  colred[wave][4 * lane + 1] = c1;
  colred[wave][4 * lane + 2] = c2;
  colred[wave][4 * lane + 3] = c3;
  __syncthreads();
  const int c = tile.tj * kTileCols + threadIdx.x;
  if (c < n) {
    float s = (colred[0][threadIdx.x] + colred[1][threadIdx.x]) + (colred[2][threadIdx.x] + colred[3][threadIdx.x]);
    ws[T.oColPart + (size_t)tile.ti * n + c] = s;
  }
}

__global__ void __launch_bounds__(kBlock) k_rowcol_sums(const TensorDev* __restrict__ tensors,
                                                        const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                        int n_tiles, MixArgs M) {
  __shared__ float colred[4][kTileCols];
  if ((int)blockIdx.x >= n_tiles) {   // the extra workgroups of a VeLO step: slice sums of the LSTM outputs
    mix_hbar_block(tensors, M, (int)blockIdx.x - n_tiles, reinterpret_cast<float (*)[kWave]>(&colred[0][0]));
    return;
  }
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  if (T.vec) rowcol_tile<true>(T, tile, ws, colred);
  else rowcol_tile<false>(T, tile, ws, colred);
}

void launch_rowcol_sums(const Launch& L, const StepArgs& A, const WeightsDev& W, float* hbar_part, float* b_eff,
                        hipStream_t s) {
  if (L.n_tiles == 0) return;
  const MixArgs M = make_mix(L, A, W, hbar_part, b_eff);
  const int extra = M.n_slices * ((M.HL + kWave - 1) / kWave);
  hipLaunchKernelGGL(k_rowcol_sums, dim3(L.n_tiles + extra), dim3(kBlock), 0, s, L.tensors, L.tiles, L.ws, L.n_tiles, M);
}

// ----------------------------------------------------------------------------- rc_update

// Block-wide sums of NV values per thread; thread 0 of the block gets them in out[].
template <int NV>
__device__ __forceinline__ void block_sum(float (&v)[NV], float (*red)[4], float* out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    float s = wave_sum(v[q]);
    if (lane == 0) red[q][wave] = s;
  }
  __syncthreads();
  if (threadIdx.x < NV) {
    const int q = threadIdx.x;
    out[q] = (red[q][0] + red[q][1]) + (red[q][2] + red[q][3]);
  }
}

// Sum of part[0], part[stride], ... (count terms) in double, always in index order. The loads of a batch issue
// ahead of the adds: batches of 32 while that many terms are left (the loop is bound by load latency), then 8.
__device__ __forceinline__ double strided_sum(const float* __restrict__ part, int count, size_t stride) {
  double acc = 0.0;
  int j = 0;
  for (; j + 32 <= count; j += 32) {
    float t[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) t[k] = part[(size_t)(j + k) * stride];
#pragma unroll
    for (int k = 0; k < 32; ++k) acc += (double)t[k];
  }
#pragma unroll 8
  for (; j < count; ++j) acc += (double)part[(size_t)j * stride];
  return acc;
}

// The same sum formed by the whole workgroup (for one row or column at a time): thread t adds the terms t, t + 256, ...
// in index order, then a fixed tree over the 256 threads. Every thread gets the result. For tensors of extreme aspect
// ratio (a 1 x 2^28 vector has a million column tiles): one lane summing them all would take milliseconds.
__device__ __forceinline__ double strided_sum_coop(const float* __restrict__ part, int count, size_t stride, double* tree) {
  double a = 0.0;
  int j = threadIdx.x;
  for (; j + 7 * kBlock < count; j += 8 * kBlock) {
    float t[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = part[(size_t)(j + k * kBlock) * stride];
#pragma unroll
    for (int k = 0; k < 8; ++k) a += (double)t[k];
  }
  for (; j < count; j += kBlock) a += (double)part[(size_t)j * stride];
  __syncthreads();   // the previous use of the tree is over
  tree[threadIdx.x] = a;
  __syncthreads();
  for (int w = kBlock / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) tree[threadIdx.x] += tree[threadIdx.x + w];
    __syncthreads();
  }
  return tree[0];
}

// A block of rows (or columns) takes the cooperative sum when there are at least 64 partials per row of the block and
// more than 512 in all (decided by the shapes alone, so a given tensor list always takes the same path).
__device__ __forceinline__ bool rc_sum_coop(int count, int valid) { return count > 512 && count >= 64 * valid; }

__global__ void __launch_bounds__(kBlock) k_rc_update(const TensorDev* __restrict__ tensors,
                                                      const RcItemDev* __restrict__ items, float* __restrict__ ws,
                                                      StepArgs A, int n_items, MixArgs M) {
  __shared__ float red[9][4];
  __shared__ double tree[kBlock];
  if ((int)blockIdx.x >= n_items) {   // the extra workgroups of a VeLO step: mean of the LSTM outputs, gate bias
    __shared__ float hbar[1024];
    __shared__ float mred[4][kWave];
    mix_bias_block(M, (int)blockIdx.x - n_items, hbar, mred);
    return;
  }
  const RcItemDev it = items[blockIdx.x];
  const TensorDev& T = tensors[it.tensor];
  const int idx = it.blk * kBlock + threadIdx.x;
  float v[9];
#pragma unroll
  for (int q = 0; q < 9; ++q) v[q] = 0.f;
  float* st = T.st;
  const int dim = it.is_col ? T.n : T.m, count = it.is_col ? T.nrt : T.nct;
  const int valid = min(kBlock, dim - it.blk * kBlock);
  const float* __restrict__ pbase = ws + (it.is_col ? T.oColPart : T.oRowPart) + (size_t)it.blk * kBlock;
  double acc = 0.0;
  if (rc_sum_coop(count, valid)) {   // workgroup-uniform
    for (int i = 0; i < valid; ++i) {
      const double v1 = strided_sum_coop(pbase + i, count, (size_t)dim, tree);
      if ((int)threadIdx.x == i) acc = v1;
    }
  } else if (idx < dim) {
    acc = strided_sum(pbase + threadIdx.x, count, (size_t)dim);
  }
  if (!it.is_col) {
    if (idx < T.m) {
      const float R = (float)(acc / (double)T.n);
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        float* rk = st + 4 * (size_t)T.padN + (size_t)k * T.padm;
        const float b = A.fac_decay[k];
        const float r = b * rk[idx] + (1.0f - b) * R;
        rk[idx] = r;
        const float rr = rsqrtf(r + A.eps_acc);
        ws[T.oRR + (size_t)k * T.padm + idx] = rr;
        v[k] = r;
        v[3 + k] = r * r;
        v[6 + k] = rr * rr;
      }
    }
  } else {
    if (idx < T.n) {
      const float C = (float)(acc / (double)T.m);
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        float* ck = st + 4 * (size_t)T.padN + 3 * (size_t)T.padm + (size_t)k * T.padn;
        const float b = A.fac_decay[k];
        const float c = b * ck[idx] + (1.0f - b) * C;
        ck[idx] = c;
        const float rc = rsqrtf(c + A.eps_acc);
        ws[T.oRC + (size_t)k * T.padn + idx] = rc;
        v[3 + k] = c * c;
        v[6 + k] = rc * rc;
      }
    }
  }
  const int slot = it.is_col ? T.nrblk + it.blk : it.blk;
  block_sum<9>(v, red, ws + T.oRcPart + (size_t)slot * kRcStride);
}

void launch_rc_update(const Launch& L, const StepArgs& A, const WeightsDev& W, float* hbar_part, float* b_eff,
                      hipStream_t s) {
  if (L.n_rcitems == 0) return;
  const MixArgs M = make_mix(L, A, W, hbar_part, b_eff);
  const int extra = M.n_slices ? kMixJSplit * ((4 * M.HL + kWave - 1) / kWave) : 0;
  hipLaunchKernelGGL(k_rc_update, dim3(L.n_rcitems + extra), dim3(kBlock), 0, s, L.tensors, L.rcitems, L.ws, A,
                     L.n_rcitems, M);
}

// ----------------------------------------------------------------------------- accum_stats

// The per-element features that need a statistic of their own (the row/column-constant ones
// follow from r_k, c_k alone). rrc[k] = rsqrt(r_k[i]+eps) * rsqrt(c_k[j]+eps); the common
// factor sqrt(mean(r_k)+eps) of the factored features is applied per tensor in k_finalize.
// Streaming accesses of this pass: nontemporal loads, ordinary stores (measured: 0.649 ms on the ViT-B/16 set
// against 0.670 plain/plain, 0.670 plain/nontemporal, 0.680 nontemporal/nontemporal).

// Rows that are not 16-byte aligned (n % 4 != 0; a small share of any list): one column per lane and sweep, four
// sweeps of 64 columns over the tile, every access a coalesced dword. Kept small in registers on purpose: the
// kernel's register count is the larger of its two paths, and it decides how many of its workgroups fit beside the
// apply kernel of another tensor group.
template <bool WRITE>
__device__ __forceinline__ void accum_tile(const TensorDev& T, const TileDev& tile, float* __restrict__ ws,
                                           const StepArgs& A, float (&acc)[kNStat]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = T.n, m = T.m;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  const size_t pN = T.padN;
  const float b1 = A.mom_decay[0], b2 = A.mom_decay[1], b3 = A.mom_decay[2], b4 = A.rms_decay;
  const float eps = A.eps_acc;
#pragma unroll 1
  for (int sweep = 0; sweep < kTileCols / kWave; ++sweep) {
    const int c = tile.tj * kTileCols + sweep * kWave + lane;
    if (c >= n) break;   // columns only grow with the sweep
    float rc[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) rc[k] = ws[T.oRC + (size_t)k * T.padn + c];
#pragma unroll 1
    for (int r = r0 + wave; r < r1; r += 4) {
      const size_t ro = (size_t)r * n + c;
      const float g = __builtin_nontemporal_load(T.g + ro), p = __builtin_nontemporal_load(T.p + ro);
      // explicit fused multiply-adds: the apply pass may form the same values again (lopt_state_pass), bit for bit
      const float nm1 = __builtin_fmaf(b1, __builtin_nontemporal_load(T.st + ro), (1.0f - b1) * g);
      const float nm2 = __builtin_fmaf(b2, __builtin_nontemporal_load(T.st + pN + ro), (1.0f - b2) * g);
      const float nm3 = __builtin_fmaf(b3, __builtin_nontemporal_load(T.st + 2 * pN + ro), (1.0f - b3) * g);
      const float nv = __builtin_fmaf(b4, __builtin_nontemporal_load(T.st + 3 * pN + ro), (1.0f - b4) * (g * g));
      const float rs = rsqrtf(nv + eps);
      const float f0 = ws[T.oRR + r] * rc[0], f1 = ws[T.oRR + (size_t)T.padm + r] * rc[1];
      const float f2 = ws[T.oRR + 2 * (size_t)T.padm + r] * rc[2];
      const float gc = fminf(fmaxf(g, -0.1f), 0.1f);
      float t;
      acc[0] += g * g;
      acc[1] += p * p;
      acc[2] += nm1 * nm1;
      acc[3] += nm2 * nm2;
      acc[4] += nm3 * nm3;
      acc[5] += nv * nv;
      t = nm1 * rs; acc[6] += t * t;
      t = nm2 * rs; acc[7] += t * t;
      t = nm3 * rs; acc[8] += t * t;
      acc[9] += rs * rs;
      t = g * f0; acc[10] += t * t;
      t = g * f1; acc[11] += t * t;
      t = g * f2; acc[12] += t * t;
      t = nm1 * f0; acc[13] += t * t;
      t = nm2 * f1; acc[14] += t * t;
      t = nm3 * f2; acc[15] += t * t;
      acc[16] += gc * gc;
      if (WRITE) {
        T.st[ro] = nm1;
        T.st[pN + ro] = nm2;
        T.st[2 * pN + ro] = nm3;
        T.st[3 * pN + ro] = nv;
      }
    }
  }
}

// The same pass for tensors whose rows are 16-byte aligned (n % 4 == 0), which is nearly all of the work: a lane's
// four columns are either all inside the tensor or all outside, so lanes past the last column sit the tile out
// and nothing in the loop is predicated. The sums of squares are taken in the form that needs the fewest vector
// instructions: (M_i rsqrt(V+eps))^2 = M_i^2 / (V+eps), (g a_i b_j)^2 = g^2 a_i^2 b_j^2 (squared row and column
// factors are formed once per row / per tile), clip(g, +-0.1)^2 = min(g^2, 0.01). RAW_RCP: the bare v_rcp_f32 (it
// treats inputs below the smallest normal float as zero, so the launcher asks for it only when eps_acc >= 1e-30).
typedef float __attribute__((ext_vector_type(4))) f32x4v;
typedef const f32x4v __attribute__((address_space(1)))* gcv4;
typedef f32x4v __attribute__((address_space(1)))* gv4;

template <bool RAW_RCP, bool WRITE>
__device__ __forceinline__ void accum_tile_vec(const TensorDev& T, const TileDev& tile, float* __restrict__ ws,
                                               const StepArgs& A, float (&acc)[kNStat]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = T.n, m = T.m;
  const int col = tile.tj * kTileCols + 4 * lane;
  if (col >= n) return;
  const int r0 = tile.ti * T.TR;
  const int r1 = min(r0 + T.TR, m);
  float rc2[3][4];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const float4 c = *reinterpret_cast<const float4*>(ws + T.oRC + (size_t)k * T.padn + col);
    rc2[k][0] = c.x * c.x; rc2[k][1] = c.y * c.y; rc2[k][2] = c.z * c.z; rc2[k][3] = c.w * c.w;
  }
  const size_t pN = T.padN;
  const float b1 = A.mom_decay[0], b2 = A.mom_decay[1], b3 = A.mom_decay[2], b4 = A.rms_decay;
  const float a1 = 1.0f - b1, a2 = 1.0f - b2, a3 = 1.0f - b3, a4 = 1.0f - b4;
  const float eps = A.eps_acc;
  const float clip2 = 0.1f * 0.1f;
  for (int r = r0 + wave; r < r1; r += 4) {
    const size_t ro = (size_t)r * n + col;   // a multiple of 4: every section starts 16-byte aligned
    const f32x4v g4 = __builtin_nontemporal_load((gcv4)(T.g + ro));
    const f32x4v p4 = __builtin_nontemporal_load((gcv4)(T.p + ro));
    const f32x4v m1 = __builtin_nontemporal_load((gcv4)(T.st + ro));
    const f32x4v m2 = __builtin_nontemporal_load((gcv4)(T.st + pN + ro));
    const f32x4v m3 = __builtin_nontemporal_load((gcv4)(T.st + 2 * pN + ro));
    const f32x4v v4 = __builtin_nontemporal_load((gcv4)(T.st + 3 * pN + ro));
    float rr2[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const float rr = ws[T.oRR + (size_t)k * T.padm + r];
      rr2[k] = rr * rr;
    }
    f32x4v o1, o2, o3, ov;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float g = g4[e], p = p4[e];
      const float g2 = g * g;
      // explicit fused multiply-adds: the apply pass may form the same values again (lopt_state_pass), bit for bit
      const float nm1 = __builtin_fmaf(b1, m1[e], a1 * g);
      const float nm2 = __builtin_fmaf(b2, m2[e], a2 * g);
      const float nm3 = __builtin_fmaf(b3, m3[e], a3 * g);
      const float nv = __builtin_fmaf(b4, v4[e], a4 * g2);
      o1[e] = nm1; o2[e] = nm2; o3[e] = nm3; ov[e] = nv;
      const float s1 = nm1 * nm1, s2 = nm2 * nm2, s3 = nm3 * nm3;
      const float rs2 = RAW_RCP ? __builtin_amdgcn_rcpf(nv + eps) : 1.0f / (nv + eps);
      const float f0 = rr2[0] * rc2[0][e], f1 = rr2[1] * rc2[1][e], f2 = rr2[2] * rc2[2][e];
      acc[0] += g2;
      acc[1] += p * p;
      acc[2] += s1; acc[3] += s2; acc[4] += s3;
      acc[5] += nv * nv;
      acc[6] += s1 * rs2; acc[7] += s2 * rs2; acc[8] += s3 * rs2;
      acc[9] += rs2;
      acc[10] += g2 * f0; acc[11] += g2 * f1; acc[12] += g2 * f2;
      acc[13] += s1 * f0; acc[14] += s2 * f1; acc[15] += s3 * f2;
      acc[16] += fminf(g2, clip2);
    }
    if (WRITE) {
      *(gv4)(T.st + ro) = o1;
      *(gv4)(T.st + pN + ro) = o2;
      *(gv4)(T.st + 2 * pN + ro) = o3;
      *(gv4)(T.st + 3 * pN + ro) = ov;
    }
  }
}

// WRITE = false: the accumulators are only read (their new values are formed for the statistics and dropped); the apply
// pass of the same step forms them again and writes them (the two default apply kernels can; a read-only stream
// sustains a higher share of the HBM rate than a read-write one, and 16 of this pass's 40 bytes per element move there).
template <bool RAW_RCP, bool WRITE>
__global__ void __launch_bounds__(kBlock) k_accum_stats(const TensorDev* __restrict__ tensors,
                                                        const TileDev* __restrict__ tiles, float* __restrict__ ws,
                                                        StepArgs A) {
  __shared__ float red[kNStat][4];
  const TileDev tile = tiles[blockIdx.x];
  const TensorDev& T = tensors[tile.tensor];
  float acc[kNStat];
#pragma unroll
  for (int q = 0; q < kNStat; ++q) acc[q] = 0.f;
  if (T.vec) accum_tile_vec<RAW_RCP, WRITE>(T, tile, ws, A, acc);
  else accum_tile<WRITE>(T, tile, ws, A, acc);
  const int lt = tile.ti * T.nct + tile.tj;
  block_sum<kNStat>(acc, red, ws + T.oStatPart + (size_t)lt * kStatStride);
}

void launch_accum_stats(const Launch& L, const StepArgs& A, bool write_state, hipStream_t s) {
  if (L.n_tiles == 0) return;
  const bool raw = A.eps_acc >= 1e-30f;
#define LOPT_LAUNCH_ACC(R, Wr) \
  hipLaunchKernelGGL((k_accum_stats<R, Wr>), dim3(L.n_tiles), dim3(kBlock), 0, s, L.tensors, L.tiles, L.ws, A)
  if (raw && write_state) LOPT_LAUNCH_ACC(true, true);
  else if (raw) LOPT_LAUNCH_ACC(true, false);
  else if (write_state) LOPT_LAUNCH_ACC(false, true);
  else LOPT_LAUNCH_ACC(false, false);
#undef LOPT_LAUNCH_ACC
}

// ----------------------------------------------------------------------------- finalize

// One workgroup per tensor. Reduces every partial in a fixed order (double accumulation),
// then writes s_f, the per-feature scale factors and the prepared first layer.
__global__ void __launch_bounds__(kBlock) k_finalize(const TensorDev* __restrict__ tensors, float* __restrict__ ws,
                                                     StepArgs A, WeightsDev W, float* __restrict__ lstm_u, int tensor0,
                                                     int* __restrict__ apply_counter) {
  __shared__ double part[8][32];
  __shared__ double tot[48];
  __shared__ float s_stats[32], s_scale[32], s_tfeat[LOPT_N_TIME], s_lfeat[LOPT_N_LOSS];
  const int ti = tensor0 + (int)blockIdx.x;
  const TensorDev& T = tensors[ti];
  if (blockIdx.x == 0 && threadIdx.x == 0) *apply_counter = 0;   // the apply pass of this sub-list starts at its first tile
  if (threadIdx.x >= 64 && threadIdx.x < 64 + LOPT_N_TIME) {
    // time features tanh(t/x) (feature table of small_fc_lopt, row "Time Features")
    const double xs[LOPT_N_TIME] = {1, 3, 10, 30, 100, 300, 1000, 3000, 1e4, 3e4, 1e5};
    s_tfeat[threadIdx.x - 64] = (float)tanh((double)A.step / xs[threadIdx.x - 64]);
  }
  if (threadIdx.x >= 96 && threadIdx.x < 96 + LOPT_N_LOSS) {
    // loss features tanh(psi / x), psi = sign(loss) ln(1 + |loss|) (the loss value VeLO's step is given)
    const double xs[LOPT_N_LOSS] = {1, 3, 10};
    const double l = (double)A.loss;
    const double psi = copysign(log1p(fabs(l)), l);
    s_lfeat[threadIdx.x - 96] = (float)tanh(psi / xs[threadIdx.x - 96]);
  }
  const int q = threadIdx.x & 31, seg = threadIdx.x >> 5;
  const int ntiles = T.nrt * T.nct;
  // per-element statistics: 17 sums over the tiles
  double a = 0.0;
  if (q < kNStat && seg < ntiles)   // thread (seg, q): tiles seg, seg + 8, ...
    a = strided_sum(ws + T.oStatPart + q + (size_t)seg * kStatStride, (ntiles - seg + 7) / 8, (size_t)8 * kStatStride);
  part[seg][q] = a;
  __syncthreads();
  if (threadIdx.x < 32) {
    double s = 0.0;
    for (int k = 0; k < 8; ++k) s += part[k][q];
    tot[q] = s;
  }
  __syncthreads();
  // row partials (9 sums over the row blocks) then column partials (slots 3..8 used)
  a = 0.0;
  if (q < 9) {
    const float* rp = ws + T.oRcPart + q;
#pragma unroll 4
    for (int i = seg; i < T.nrblk; i += 8) a += (double)rp[(size_t)i * kRcStride];
  } else if (q >= 16 && q < 25) {
    const float* cp = ws + T.oRcPart + (size_t)T.nrblk * kRcStride + (q - 16);
#pragma unroll 4
    for (int i = seg; i < T.ncblk; i += 8) a += (double)cp[(size_t)i * kRcStride];
  }
  part[seg][q] = a;
  __syncthreads();
  if (threadIdx.x < 32) {
    double s = 0.0;
    for (int k = 0; k < 8; ++k) s += part[k][q];
    if (q < 9) tot[17 + q] = s;                    // 17..19 sum r, 20..22 sum r^2, 23..25 sum 1/(r+eps)
    else if (q >= 19 && q < 25) tot[26 + (q - 19)] = s;  // 26..28 sum c^2, 29..31 sum 1/(c+eps)
  }
  __syncthreads();
  if (threadIdx.x < 32) {
    const int f = threadIdx.x;
    const double N = (double)T.m * (double)T.n;
    double s = 0.0;
    double pre = 1.0;  // factor between the raw feature the kernels build and the feature itself
    if (f < 10) s = tot[f] / N;
    else if (f < 13 || (f >= 25 && f < 28)) {
      const int k = f < 13 ? f - 10 : f - 25;
      const double rbar = tot[17 + k] / (double)T.m + (double)A.eps_acc;
      s = tot[f < 13 ? f : f - 12] / N * rbar;
      pre = sqrt(rbar);
    } else if (f < 16) s = tot[20 + (f - 13)] / (double)T.m;
    else if (f < 19) s = tot[26 + (f - 16)] / (double)T.n;
    else if (f < 22) s = tot[23 + (f - 19)] / (double)T.m;
    else if (f < 25) s = tot[29 + (f - 22)] / (double)T.n;
    else if (f == 28) s = tot[16] / N;
    const float sf = (float)s;
    const float scale = (float)(pre / sqrt((double)sf + (double)A.eps_norm));
    s_stats[f] = sf;
    s_scale[f] = f < A.F ? scale : 0.f;
    ws[T.oStats + f] = f < A.F ? sf : 0.f;
    ws[T.oScale + f] = f < A.F ? scale : 0.f;
  }
  __syncthreads();
  if (A.kind == LOPT_SMALL_FC) {
    // first layer with the normalization folded in, hidden width padded with zeros to HP;
    // the un-normalized time features only shift the bias.
    const int H = A.H, HP = A.HP;
    float* prep = ws + T.oPrep;
    for (int i = threadIdx.x; i < LOPT_N_ELEM_FEATS * HP; i += kBlock) {
      const int f = i / HP, u = i - f * HP;
      prep[i] = u < H ? W.mlp[f * H + u] * s_scale[f] : 0.f;
    }
    for (int u = threadIdx.x; u < HP; u += kBlock) {
      float b = 0.f;
      if (u < H) {
        b = W.mlp[LOPT_D_SMALL_FC * H + u];
        for (int i = 0; i < LOPT_N_TIME; ++i) b += s_tfeat[i] * W.mlp[(LOPT_N_ELEM_FEATS + i) * H + u];
      }
      prep[LOPT_N_ELEM_FEATS * HP + u] = b;
    }
  } else {
    // LSTM input: 0.05*ln(s_f + 1e-30), time features, one-hot of min(ndim, 4), loss features
    float* u = lstm_u + (size_t)ti * kLstmInPad;
    const int t = threadIdx.x;
    if (t < LOPT_D_VELO) u[t] = 0.05f * logf(s_stats[t] + 1e-30f);
    else if (t < LOPT_D_VELO + LOPT_N_TIME) u[t] = s_tfeat[t - LOPT_D_VELO];
    else if (t < LOPT_D_VELO + LOPT_N_TIME + 5) {
      const int nd = T.ndim < 4u ? (int)T.ndim : 4;
      u[t] = (t - (LOPT_D_VELO + LOPT_N_TIME)) == nd ? 1.f : 0.f;
    } else if (t < LOPT_VELO_LSTM_IN) u[t] = s_lfeat[t - (LOPT_D_VELO + LOPT_N_TIME + 5)];
    else if (t < kLstmInPad) u[t] = 0.f;
  }
}

void launch_finalize(const Launch& L, const StepArgs& A, const WeightsDev& W, float* lstm_u, hipStream_t s) {
  if (L.n_tensors == 0) return;
  hipLaunchKernelGGL(k_finalize, dim3(L.n_tensors), dim3(kBlock), 0, s, L.tensors, L.ws, A, W, lstm_u, L.tensor0,
                     L.apply_counter);
}

// ----------------------------------------------------------------------------- VeLO hypernetwork

// One LSTM-cell step for all tensors: Z[T, 4 H_L] = [u | h_prev] [Wx ; Wh] is a dense contraction and runs on the
// matrix cores in fp32 (v_mfma_f32_32x32x2_f32: exact fp32 products, fp32 accumulation). A workgroup owns 32 tensors x
// 16 hidden units (two 32-column MFMA tiles of 8 units x 4 gates); its four wavefronts split the 48 + H_L input slots
// and meet in LDS in a fixed order; one thread per (tensor, unit pair) then applies the cell equations.
// Operands go from global memory straight into the MFMA layout: lane (k-half, t) holds input slot 2p + k-half of tensor
// t (A operand) and of column (gate, unit) = (lane%32 / 8, u0 + 8 tile + lane%8) (B operand). Loads are unconditional
// (clamped to a valid row, multiplied by 0 where a slot carries nothing: the padding slots 45..47, slots past H_L,
// tensors or units past the end), sixteen slot pairs = 48 loads in flight per wavefront: the kernel is bound by the
// latency of those loads, not by arithmetic.
constexpr int kLstmTensors = 32;
constexpr int kLstmUnits = 16;
constexpr int kLstmPairsPerTrip = 16;
typedef float f32x16_l __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(kBlock) k_velo_lstm(const TensorDev* __restrict__ tensors, StepArgs A, WeightsDev W,
                                                      const float* __restrict__ lstm_u, const float* __restrict__ b_eff,
                                                      float* __restrict__ h_new) {
  __shared__ float part[4][2][32][32];   // [wavefront][column tile][tensor][column]: 32 KB
  const int HL = A.HL, G = 4 * HL;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int khalf = lane >> 5, l32 = lane & 31;
  const int t0 = blockIdx.x * kLstmTensors, u0 = blockIdx.y * kLstmUnits;
  // A side: the tensor of this lane (clamped: rows past the list compute on the last tensor and are dropped)
  const int tA = min(t0 + l32, A.n_tensors - 1);
  const TensorDev& T = tensors[tA];
  const float* __restrict__ hsrc = T.st + 4 * (size_t)T.padN + 3 * (size_t)T.padm + 3 * (size_t)T.padn;
  const float* __restrict__ usrc = lstm_u + (size_t)tA * kLstmInPad;
  // B side: the two columns of this lane
  const int gate = l32 >> 3;
  const int ua = min(u0 + (l32 & 7), HL - 1), ub = min(u0 + 8 + (l32 & 7), HL - 1);
  const size_t cola = (size_t)gate * HL + ua, colb = (size_t)gate * HL + ub;

  f32x16_l acc0, acc1;
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
  // slot pairs of this wavefront; slots 0..47 are u (45 used), slots 48.. are h_prev; 48 is even, so a pair never straddles
  const int n_pairs = (kLstmInPad + HL + 1) / 2;
  const int per_wave = (n_pairs + 3) / 4;
  const int p_begin = wave * per_wave, p_end = min(p_begin + per_wave, n_pairs);
  for (int pb = p_begin; pb < p_end; pb += kLstmPairsPerTrip) {
    float a[kLstmPairsPerTrip], b0[kLstmPairsPerTrip], b1[kLstmPairsPerTrip];
#pragma unroll
    for (int j = 0; j < kLstmPairsPerTrip; ++j) {
      const int p = pb + j < p_end ? pb + j : p_end - 1;   // a repeated pair is multiplied by 0 below
      const int k = 2 * p + khalf;
      const bool isu = 2 * p < kLstmInPad;                  // wave-uniform
      const int ku = k < LOPT_VELO_LSTM_IN ? k : LOPT_VELO_LSTM_IN - 1;
      const int kh = k - kLstmInPad;
      const int khc = kh < 0 ? 0 : kh < HL ? kh : HL - 1;
      const float keep = (pb + j < p_end && (isu ? k < LOPT_VELO_LSTM_IN : kh < HL)) ? 1.f : 0.f;
      const float* __restrict__ wrow = isu ? W.Wx + (size_t)ku * G : W.Wh + (size_t)khc * G;
      a[j] = (isu ? usrc[ku] : hsrc[khc]) * keep;
      b0[j] = wrow[cola];
      b1[j] = wrow[colb];
    }
#pragma unroll
    for (int j = 0; j < kLstmPairsPerTrip; ++j) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b0[j], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b1[j], acc1, 0, 0, 0);
    }
  }
  // accumulator register v of lane (k-half, c) is row 8 (v / 4) + 4 k-half + v % 4, column c
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v >> 2) + 4 * khalf + (v & 3);
    part[wave][0][row][l32] = acc0[v];
    part[wave][1][row][l32] = acc1[v];
  }
  __syncthreads();
  {
    const int tt = threadIdx.x >> 3, uu = threadIdx.x & 7;
    if (t0 + tt < A.n_tensors) {
      const TensorDev& Tt = tensors[t0 + tt];
      float* cl = Tt.st + 4 * (size_t)Tt.padN + 3 * (size_t)Tt.padm + 3 * (size_t)Tt.padn + Tt.padH;
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) {
        const int unit = u0 + 8 * tile + uu;
        if (unit < HL) {
          float zz[4];
#pragma unroll
          for (int g2 = 0; g2 < 4; ++g2) {
            const int c = g2 * 8 + uu;
            const int gc = g2 * HL + unit;   // bias + cross-tensor term (its four partial sums, in order)
            const float be = W.b[gc] + ((b_eff[gc] + b_eff[G + gc]) + (b_eff[2 * G + gc] + b_eff[3 * G + gc]));
            zz[g2] = be + ((part[0][tile][tt][c] + part[1][tile][tt][c]) + (part[2][tile][tt][c] + part[3][tile][tt][c]));
          }
          const float ig = 1.f / (1.f + expf(-zz[0]));
          const float fg = 1.f / (1.f + expf(-zz[1]));
          const float gg = tanhf(zz[2]);
          const float og = 1.f / (1.f + expf(-zz[3]));
          const float c = fg * cl[unit] + ig * gg;
          cl[unit] = c;
          h_new[(size_t)(t0 + tt) * HL + unit] = og * tanhf(c);
        }
      }
    }
  }
}

void launch_velo_lstm(const Launch& L, const StepArgs& A, const WeightsDev& W, const float* lstm_u, const float* b_eff,
                      float* h_new, hipStream_t s) {
  if (L.n_tensors == 0) return;
  dim3 grid((L.n_tensors + kLstmTensors - 1) / kLstmTensors, (A.HL + kLstmUnits - 1) / kLstmUnits);
  // a sub-list starts at tensor L.tensor0: the kernel indexes tensors, inputs and outputs from there
  StepArgs As = A;
  As.n_tensors = L.n_tensors;
  hipLaunchKernelGGL(k_velo_lstm, grid, dim3(kBlock), 0, s, L.tensors + L.tensor0, As, W,
                     lstm_u + (size_t)L.tensor0 * kLstmInPad, b_eff, h_new + (size_t)L.tensor0 * A.HL);
}

// Partial matrix-vector product for the hypernetwork head: out[w][c0 + 64 c + lane] = sum over rows
// k = w, w+nw, ... of x[k] * M[k][col], for the four columns c = 0..3 of this lane. Columns past the
// end are clamped for the loads (their results are never read); four rows per trip keep sixteen
// independent coalesced loads in flight (the kernel is bound by their latency).
__device__ __forceinline__ void matvec4(const float* __restrict__ x, int n_in, const float* __restrict__ M, int ld,
                                        int c0, int wave, int nw, int lane, float* __restrict__ part, int W64) {
  const float* wp[4];
  float acc[4][4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int col = c0 + 64 * c + lane;
    wp[c] = M + (col < ld ? col : ld - 1);
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r][c] = 0.f;
  }
  int k = wave;
  for (; k + 3 * nw < n_in; k += 4 * nw) {
    float xv[4], w[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      xv[r] = x[k + r * nw];
#pragma unroll
      for (int c = 0; c < 4; ++c) w[r][c] = wp[c][(size_t)(k + r * nw) * ld];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[r][c] += xv[r] * w[r][c];
  }
  for (int r = 0; k < n_in; k += nw, ++r) {   // at most three rows left
    const float x0 = x[k];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float wv = wp[c][(size_t)k * ld];
      if (r == 0) acc[0][c] += x0 * wv; else if (r == 1) acc[1][c] += x0 * wv; else acc[2][c] += x0 * wv;
    }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (c0 + 64 * c < W64) part[wave * W64 + c0 + 64 * c + lane] = (acc[0][c] + acc[1][c]) + (acc[2][c] + acc[3][c]);
}

// Head of the hypernetwork for one tensor: alpha = h W_a + b_a, theta = alpha B, written as the
// prepared (zero-padded, first layer scaled) per-tensor MLP; the step-size multiplier lam = exp(h . ws + bs)
// is folded into the direction column of the last layer (W3[:, 0], b3[0]), so the apply pass does not see it.
// Also stores the new h into the state.
// Both products split their reduction across the workgroup's wavefronts (combined through LDS in a
// fixed order); lanes own output columns, so weight reads are coalesced.
__global__ void __launch_bounds__(1024) k_velo_head(const TensorDev* __restrict__ tensors, float* __restrict__ ws,
                                                      StepArgs A, WeightsDev W, const float* __restrict__ h_new) {
  extern __shared__ float sh[];  // h[HL] | alpha[K] | part[nw][max(K, P) rounded up to 64]
  __shared__ float s_lam;
  const TensorDev& T = tensors[blockIdx.x];
  const int HL = A.HL, K = A.K, H = A.H, HP = A.HP, F = LOPT_D_VELO, P = A.P;
  const int W64 = ((K > P ? K : P) + 63) & ~63;
  float* sh_h = sh;
  float* sh_a = sh + HL;
  float* part = sh_a + K;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  float* hstate = T.st + 4 * (size_t)T.padN + 3 * (size_t)T.padm + 3 * (size_t)T.padn;
  for (int i = threadIdx.x; i < HL; i += blockDim.x) {
    const float v = h_new[(size_t)blockIdx.x * HL + i];
    sh_h[i] = v;
    hstate[i] = v;
  }
  // zero the padded layout (padding must be zero); disjoint from everything read below
  float* prep = ws + T.oPrep;
  const int prep_n = (F + 1) * HP + HP * HP + HP + 2 * HP + 2;
  for (int i = threadIdx.x; i < prep_n; i += blockDim.x) prep[i] = 0.f;
  __syncthreads();
  if (wave == 0) {
    float a = 0.f;
    for (int i = lane; i < HL; i += kWave) a += sh_h[i] * W.ws[i];
    a = wave_sum(a);
    if (lane == 0) s_lam = expf(a + W.bs[0]);
  }
  // alpha = h W_a: wavefront w reduces rows w, w+nw, ...; a lane owns four output columns 64 apart
  for (int q0 = 0; q0 < K; q0 += 256) matvec4(sh_h, HL, W.Wa, K, q0, wave, nw, lane, part, W64);
  __syncthreads();
  for (int q = threadIdx.x; q < K; q += blockDim.x)
  {
    float a = W.ba[q];
    for (int w = 0; w < nw; ++w) a += part[w * W64 + q];
    sh_a[q] = a;
  }
  __syncthreads();
  // theta = alpha B, same scheme
  for (int i0 = 0; i0 < P; i0 += 256) matvec4(sh_a, K, W.B, P, i0, wave, nw, lane, part, W64);
  __syncthreads();
  const float* scale = ws + T.oScale;
  for (int i = threadIdx.x; i < P; i += blockDim.x) {
    float th = 0.f;
    for (int w = 0; w < nw; ++w) th += part[w * W64 + i];
    // scatter from the compact layout (W1[F,H] b1[H] W2[H,H] b2[H] W3[H,2] b3[2]) to the padded one
    int o = i, dst;
    if (o < F * H) { const int f = o / H, u = o - f * H; dst = f * HP + u; th *= scale[f]; }
    else if ((o -= F * H) < H) dst = F * HP + o;
    else if ((o -= H) < H * H) { const int a = o / H, u = o - a * H; dst = (F + 1) * HP + a * HP + u; }
    else if ((o -= H * H) < H) dst = (F + 1) * HP + HP * HP + o;
    else if ((o -= H) < 2 * H) { dst = (F + 1) * HP + HP * HP + HP + o; if (!(o & 1)) th *= s_lam; }   // W3[a][0]: direction
    else { o -= 2 * H; dst = (F + 1) * HP + HP * HP + HP + 2 * HP + o; if (o == 0) th *= s_lam; }       // b3[0]
    prep[dst] = th;
  }
}

// ---- the head for long tensor lists: alpha = H' W_a + b_a and theta = alpha B as two batched products on the matrix
// cores (fp32), then one small workgroup per tensor that scatters theta into the prepared layout.

// Y[r][c] = bias[c] + sum_k X[r][k] Wm[k][c] with exact fp32 products (v_mfma_f32_32x32x2_f32), the scheme of
// k_velo_lstm: a workgroup owns 32 rows x 64 columns (two 32-column tiles), its four wavefronts split the k range and
// meet in LDS in a fixed order. Lane (k-half, i) holds X[row i][2p + k-half] (A operand) and Wm[2p + k-half][column i] (B
// operand); loads are unconditional (rows, columns and k clamped, surplus k multiplied by 0).
__global__ void __launch_bounds__(kBlock) k_rows_matmul(const float* __restrict__ X, int ldx, int n_rows, int n_in,
                                                        const float* __restrict__ Wm, int ldw, int n_cols,
                                                        const float* __restrict__ bias, float* __restrict__ Y, int ldy) {
  __shared__ float part[4][2][32][32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int khalf = lane >> 5, l32 = lane & 31;
  const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 64;
  const float* __restrict__ xrow = X + (size_t)min(r0 + l32, n_rows - 1) * ldx;
  const int ca = min(c0 + l32, n_cols - 1), cb = min(c0 + 32 + l32, n_cols - 1);
  f32x16_l acc0, acc1;
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
  const int n_pairs = (n_in + 1) / 2;
  const int per_wave = (n_pairs + 3) / 4;
  const int p_begin = wave * per_wave, p_end = min(p_begin + per_wave, n_pairs);
  for (int pb = p_begin; pb < p_end; pb += kLstmPairsPerTrip) {
    float a[kLstmPairsPerTrip], b0[kLstmPairsPerTrip], b1[kLstmPairsPerTrip];
#pragma unroll
    for (int j = 0; j < kLstmPairsPerTrip; ++j) {
      const int pp = pb + j < p_end ? pb + j : p_end - 1;   // a repeated pair is multiplied by 0 below
      const int k = 2 * pp + khalf;
      const int kc = k < n_in ? k : n_in - 1;
      const float keep = (pb + j < p_end && k < n_in) ? 1.f : 0.f;
      a[j] = xrow[kc] * keep;
      b0[j] = Wm[(size_t)kc * ldw + ca];
      b1[j] = Wm[(size_t)kc * ldw + cb];
    }
#pragma unroll
    for (int j = 0; j < kLstmPairsPerTrip; ++j) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b0[j], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b1[j], acc1, 0, 0, 0);
    }
  }
  // accumulator register v of lane (k-half, c) is row 8 (v / 4) + 4 k-half + v % 4, column c
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v >> 2) + 4 * khalf + (v & 3);
    part[wave][0][row][l32] = acc0[v];
    part[wave][1][row][l32] = acc1[v];
  }
  __syncthreads();
  const int rr = threadIdx.x >> 3, cc = threadIdx.x & 7;
  if (r0 + rr < n_rows) {
#pragma unroll
    for (int tile = 0; tile < 2; ++tile)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int cl = 8 * q + cc, col = c0 + 32 * tile + cl;
        if (col < n_cols)
          Y[(size_t)(r0 + rr) * ldy + col] = (bias ? bias[col] : 0.f) + ((part[0][tile][rr][cl] + part[1][tile][rr][cl]) +
                                                                          (part[2][tile][rr][cl] + part[3][tile][rr][cl]));
      }
  }
}

// One workgroup per tensor: new h into the state, step-size multiplier, theta[P] scattered into the prepared layout.
__global__ void __launch_bounds__(kBlock) k_velo_head_scatter(const TensorDev* __restrict__ tensors, float* __restrict__ ws,
                                                              StepArgs A, WeightsDev W, const float* __restrict__ h_new,
                                                              const float* __restrict__ theta) {
  __shared__ float s_lam;
  const TensorDev& T = tensors[blockIdx.x];
  const int HL = A.HL, H = A.H, HP = A.HP, F = LOPT_D_VELO, P = A.P;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* hstate = T.st + 4 * (size_t)T.padN + 3 * (size_t)T.padm + 3 * (size_t)T.padn;
  const float* __restrict__ hn = h_new + (size_t)blockIdx.x * HL;
  for (int i = threadIdx.x; i < HL; i += kBlock) hstate[i] = hn[i];
  float* prep = ws + T.oPrep;
  const int prep_n = (F + 1) * HP + HP * HP + HP + 2 * HP + 2;
  for (int i = threadIdx.x; i < prep_n; i += kBlock) prep[i] = 0.f;   // the padding must be zero
  if (wave == 0) {
    float a = 0.f;
    for (int i = lane; i < HL; i += kWave) a += hn[i] * W.ws[i];
    a = wave_sum(a);
    if (lane == 0) s_lam = expf(a + W.bs[0]);
  }
  __syncthreads();
  const float* scale = ws + T.oScale;
  const float* __restrict__ th_row = theta + (size_t)blockIdx.x * P;
  for (int i = threadIdx.x; i < P; i += kBlock) {
    float th = th_row[i];
    int o = i, dst;
    if (o < F * H) { const int f = o / H, u = o - f * H; dst = f * HP + u; th *= scale[f]; }
    else if ((o -= F * H) < H) dst = F * HP + o;
    else if ((o -= H) < H * H) { const int a = o / H, u = o - a * H; dst = (F + 1) * HP + a * HP + u; }
    else if ((o -= H * H) < H) dst = (F + 1) * HP + HP * HP + o;
    else if ((o -= H) < 2 * H) { dst = (F + 1) * HP + HP * HP + HP + o; if (!(o & 1)) th *= s_lam; }   // W3[a][0]: direction
    else { o -= 2 * H; dst = (F + 1) * HP + HP * HP + HP + 2 * HP + o; if (o == 0) th *= s_lam; }       // b3[0]
    prep[dst] = th;
  }
}

// alpha / theta: scratch of n_tensors x K and n_tensors x P floats for the batched form, null for lists below
// kHeadBatchMin tensors (one workgroup per tensor then does everything; cheaper in launches, dearer in weight reads).
void launch_velo_head(const Launch& L, const StepArgs& A, const WeightsDev& W, const float* h_new, float* alpha,
                      float* theta, hipStream_t s) {
  if (L.n_tensors == 0) return;
  if (alpha && theta && L.n_tensors >= kHeadBatchMin) {
    const int T = L.n_tensors;
    const float* hn = h_new + (size_t)L.tensor0 * A.HL;
    float* al = alpha + (size_t)L.tensor0 * A.K;
    float* th = theta + (size_t)L.tensor0 * A.P;
    hipLaunchKernelGGL(k_rows_matmul, dim3((T + 31) / 32, (A.K + 63) / 64), dim3(kBlock), 0, s, hn, A.HL, T, A.HL, W.Wa, A.K,
                       A.K, W.ba, al, A.K);
    hipLaunchKernelGGL(k_rows_matmul, dim3((T + 31) / 32, (A.P + 63) / 64), dim3(kBlock), 0, s, al, A.K, T, A.K, W.B, A.P,
                       A.P, (const float*)nullptr, th, A.P);
    hipLaunchKernelGGL(k_velo_head_scatter, dim3(T), dim3(kBlock), 0, s, L.tensors + L.tensor0, L.ws, A, W, hn, th);
    return;
  }
  const int W64 = ((A.K > A.P ? A.K : A.P) + 63) & ~63;
  int nw = 16;  // wavefronts per workgroup = ways the reductions are split; bounded by 48 KB of partials
  while (nw > 1 && (size_t)nw * W64 * sizeof(float) > 48 * 1024) nw >>= 1;
  size_t shmem = (size_t)(A.HL + A.K + nw * W64) * sizeof(float);
  hipLaunchKernelGGL(k_velo_head, dim3(L.n_tensors), dim3(64 * nw), shmem, s, L.tensors + L.tensor0, L.ws, A, W,
                     h_new + (size_t)L.tensor0 * A.HL);
}

}  // namespace lopt
