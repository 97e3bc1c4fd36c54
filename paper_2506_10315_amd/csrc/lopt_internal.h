// Internal declarations shared by the host planner and the gfx950 kernels of the
// learned-optimizer step library. Not part of the public boundary (see include/lopt.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lopt.h"

namespace lopt {

constexpr int kBlock = 256;       // threads per workgroup (4 wavefronts of 64)
constexpr int kWave = 64;
constexpr int kTileCols = 256;    // one wavefront row-segment: 64 lanes x float4
constexpr int kRowUnit = 64;      // standard tile height (taller for tall tensors, shorter for small lists)
constexpr int kMaxRowTiles = 256; // tile height grows so that a large tensor has at most this many row tiles ...
constexpr int kMaxTileRows = 1024; // ... up to this height (bounds the length of the per-lane fp32 partial sums)
constexpr int kStatStride = 20;   // floats per tile in the per-tile statistics partials (17 used)
constexpr int kRcStride = 12;     // floats per block in the row/column partials (9 used)
constexpr int kNStat = 17;        // per-element statistics accumulated per tile
constexpr int kStatsPerTensor = 32;
constexpr int kLstmInPad = 48;    // LOPT_VELO_LSTM_IN rounded up to a multiple of 4
constexpr int kMixSlices = 64;    // at most this many slices of the tensor list in the cross-tensor mean
constexpr int kHeadBatchMin = 1024;  // tensor lists from this length on take the batched form of the hypernetwork head
constexpr int kMixJSplit = 4;     // the LSTM units are cut into this many ranges when hbar Wg is formed
#ifndef LOPT_APPLY_ROWS
#define LOPT_APPLY_ROWS 128
#endif
constexpr int kApplyRows = LOPT_APPLY_ROWS;   // tile of the strip-form apply kernel: up to this many rows x 128 columns
constexpr int kApplyCols = 128;

// Per-tensor record in device memory. Offsets o* are in floats from the workspace base.
struct TensorDev {
  float* p;
  const float* g;
  float* st;
  int m, n;
  uint32_t padN, padm, padn, padH;  // state section strides in floats
  uint32_t ndim;
  int vec;                          // n % 4 == 0: rows are 16-byte aligned
  int TR, nrt, nct, tile0;          // tile height, tile grid, first global tile id
  int rc0, nrblk, ncblk;            // first row/col block id, number of row and column blocks
  uint64_t oRowPart;                // [nct][m]   sum over the tile's columns of g^2
  uint64_t oColPart;                // [nrt][n]   sum over the tile's rows of g^2
  uint64_t oRR;                     // [3][padm]  rsqrt(r_k + eps_acc)
  uint64_t oRC;                     // [3][padn]  rsqrt(c_k + eps_acc)
  uint64_t oRcPart;                 // [nrblk + ncblk][kRcStride]
  uint64_t oStatPart;               // [nrt*nct][kStatStride]
  uint64_t oStats;                  // [kStatsPerTensor] s_f
  uint64_t oScale;                  // [kStatsPerTensor] factor applied to the raw feature
  uint64_t oPrep;                   // prepared first layer: W1s[F][HP] then b1'[HP]
};

struct TileDev { int tensor, ti, tj, pad; };
struct RcItemDev { int tensor, is_col, blk, pad; };
struct ApplyTileDev { int tensor, r0, c0, rows; };   // rows <= kApplyRows

// Scalars of one step, passed by value to the kernels.
struct StepArgs {
  float mom_decay[3];
  float rms_decay;
  float fac_decay[3];
  float eps_acc, eps_norm;
  float exp_mult, step_mult;
  float lr, wd;
  long long step;             // number of updates already applied (time features tanh(step/x))
  int kind, H, HP, F;         // F = number of normalized per-element features (28 or 29)
  int HL, K, P;               // VeLO: LSTM width, bank rows, floats per per-tensor MLP
  int n_tensors;
  float loss;                 // VeLO: loss value that goes with this step's gradients
};

// Device weights of the optimizer, owned by the context.
struct WeightsDev {
  // small_fc_lopt (original layout, as uploaded)
  const float* mlp;    // W1[39,H] b1[H] W2[H,H] b2[H] W3[H,2] b3[2]
  const float* mlp_tail;  // W2[HP,HP] b2[HP] W3[HP,2] b3[2] pad[2] W1[28,HP]: zero-padded to the padded width HP
  // VeLO
  const float* Wx; const float* Wh; const float* Wg; const float* b; const float* Wa; const float* ba;
  const float* ws; const float* bs; const float* B;
};

struct Launch {
  const TensorDev* tensors;
  const TileDev* tiles;
  const RcItemDev* rcitems;
  float* ws;
  int n_tensors, n_tiles, n_rcitems;
  const ApplyTileDev* atiles;
  int n_atiles;
  int tensor0;   // first tensor of the sub-list this launch covers (the per-tensor kernels index from it)
  int* apply_counter;     // tile counter of the strip-form apply kernel for this sub-list (cleared by k_finalize)
  int resident_wgs;       // workgroups of the strip-form apply kernel that are resident at once (2 per CU)
};

// kernels (lopt_kernels.hip / lopt_apply_mfma.hip)
void launch_fill_zero(const Launch&, const StepArgs&, hipStream_t);
// VeLO: the two stages of the cross-tensor term (hbar = mean of the tensors' LSTM outputs of the previous step,
// b_eff = b + hbar Wg) ride along as extra workgroups of these two launches, which always cover the WHOLE list and
// come before any tensor's LSTM state is rewritten
void launch_rowcol_sums(const Launch&, const StepArgs&, const WeightsDev&, float* hbar_part, float* b_eff, hipStream_t);
void launch_rc_update(const Launch&, const StepArgs&, const WeightsDev&, float* hbar_part, float* b_eff, hipStream_t);
// write_state = false: M_1..3 and V stay as they are (the strip-form apply pass updates them, see launch_apply_f16s)
void launch_accum_stats(const Launch&, const StepArgs&, bool write_state, hipStream_t);
void launch_finalize(const Launch&, const StepArgs&, const WeightsDev&, float* lstm_u, hipStream_t);
void launch_velo_lstm(const Launch&, const StepArgs&, const WeightsDev&, const float* lstm_u, const float* b_eff,
                      float* h_new, hipStream_t);
void launch_velo_head(const Launch&, const StepArgs&, const WeightsDev&, const float* h_new, float* alpha,
                      float* theta, hipStream_t);
void launch_apply_small_fc(const Launch&, const StepArgs&, const WeightsDev&, hipStream_t);
void launch_apply_velo(const Launch&, const StepArgs&, const WeightsDev&, hipStream_t);
bool apply_mfma_available(const StepArgs&);
void launch_apply_mfma(const Launch&, const StepArgs&, const WeightsDev&, hipStream_t);
bool apply_velo4_available(const StepArgs&);
void launch_apply_velo4(const Launch&, const StepArgs&, bool update_state, hipStream_t);
void launch_apply_f16s(const Launch&, const StepArgs&, const WeightsDev&, bool update_state, hipStream_t);

}  // namespace lopt
