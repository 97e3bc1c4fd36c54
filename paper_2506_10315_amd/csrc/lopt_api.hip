// Host side of the C boundary declared in include/lopt.h: argument validation, the planner that
// turns a tensor list into the device tables the kernels walk, and the launch sequence of a step.
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <mutex>
#include <string>
#include <vector>

#include "lopt_internal.h"

using namespace lopt;

namespace {

thread_local std::string g_last_error;

constexpr int kMaxGroups = 16;

// ---- fixed scratch of lopt_step_static: device tables followed by the workspace. One copy per GPU, at an address
// of its own on each; host code reaches it only through the pointer hipGetSymbolAddress returns for the current
// device (the array's name is a host-side stand-in, not a device address).
constexpr size_t kStaticScratchBytes = LOPT_STATIC_SCRATCH_BYTES;
constexpr size_t kStageInitBytes = 4u << 20;   // pinned staging every context starts with (tables of ~100 k tiles)
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];        // per device: address of `scratch` there (null until a context is created on it)
uint64_t g_scratch_owner[kMaxDevices];   // per device: id of the context whose tables the array holds (0 = none)
std::atomic<uint64_t> g_next_ctx_id{1};

inline uint32_t pad4(uint64_t x) { return (uint32_t)((x + 3) & ~(uint64_t)3); }
inline uint64_t align64(uint64_t x) { return (x + 63) & ~(uint64_t)63; }

int padded_hidden(int H) {
  for (int hp : {4, 8, 16, 32})
    if (H <= hp) return hp;
  return 0;
}

size_t mlp_count(int d, int H) { return (size_t)d * H + H + (size_t)H * H + H + 2 * (size_t)H + 2; }

bool config_ok(const lopt_config* c, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (!c) return bad("config is null");
  if (c->struct_size != sizeof(lopt_config)) return bad("config.struct_size does not match sizeof(lopt_config)");
  if (c->kind != LOPT_SMALL_FC && c->kind != LOPT_VELO) return bad("config.kind is not a lopt_kind");
  if (c->hidden < 1 || c->hidden > 32) return bad("config.hidden must be in [1, 32]");
  const float d[7] = {c->mom_decay[0], c->mom_decay[1], c->mom_decay[2], c->rms_decay,
                      c->fac_decay[0], c->fac_decay[1], c->fac_decay[2]};
  for (float v : d)
    if (!(v >= 0.f && v < 1.f)) return bad("every decay must be in [0, 1)");
  if (!(c->eps_acc >= 0.f) || !(c->eps_norm >= 0.f)) return bad("eps_acc and eps_norm must be >= 0");
  if (!std::isfinite(c->exp_mult) || !std::isfinite(c->step_mult)) return bad("exp_mult/step_mult must be finite");
  if (c->apply_kernel > LOPT_APPLY_MFMA_F16S) return bad("config.apply_kernel is not a lopt_apply_kernel");
  if (c->groups > (uint32_t)kMaxGroups) return bad("config.groups must be in [0, 16]");
  if (c->state_pass > LOPT_STATE_IN_APPLY) return bad("config.state_pass is not a lopt_state_pass");
  if (c->kind == LOPT_VELO) {
    if (c->lstm_hidden < 1 || c->lstm_hidden > 1024) return bad("config.lstm_hidden must be in [1, 1024]");
    if (c->n_bank < 1 || c->n_bank > 1024) return bad("config.n_bank must be in [1, 1024]");
  }
  return true;
}

// Device copy of the plan's tables and what it currently holds.
struct TableStore {
  char* base = nullptr;
  size_t cap = 0;
  bool growable = false;           // library-allocated (may be reallocated) or a fixed region
  TensorDev* d_tensors = nullptr;
  TileDev* d_tiles = nullptr;
  RcItemDev* d_rcitems = nullptr;
  ApplyTileDev* d_atiles = nullptr;
  bool static_uploaded = false;    // tiles, row/column blocks and apply tiles are on the device
  bool tensors_uploaded = false;
  std::vector<TensorDev> last_tensors;  // what d_tensors currently holds
};

// The small_fc_lopt MLP rewritten into an equivalent one whose hidden units are rescaled by powers of two (ReLU is
// positively homogeneous, so W1 diag(s1), b1 s1, diag(1/s1) W2 diag(s2), b2 s2, diag(1/s2) W3 computes the same
// function; scaling by a power of two is exact in fp32). The default apply kernel carries both hidden-layer
// contractions' operands as pairs of fp16 numbers (range 2^-24 .. 65504):
//   s1_u makes the worst case of unit u's first-layer pre-activation, |b1_u| + sum_t |W1[28+t][u]| (time features are
//        at most 1) + sqrt(N_max) sum_f |W1[f][u]| (a normalized feature is at most sqrt(N) in magnitude, N <= 2^31),
//        at most 2^15: no input can make a hidden activation leave the fp16 range, and a typical activation (features
//        of unit mean square) still sits 2^-2 .. 2^0, far above the 2^-24 grid of the low halves;
//   s2_u puts the largest rescaled second-layer weight of output unit u between 2^12 and 2^13, so that weights many
//        orders of magnitude below it still keep their leading bits; layer 2's result stays in fp32.
// All apply kernels run the rewritten network (for the fp32 ones it changes nothing but exponents).
std::vector<float> equilibrate_small_fc(const float* w, int H) {
  const int d = LOPT_D_SMALL_FC, ne = LOPT_N_ELEM_FEATS;
  const size_t oB1 = (size_t)d * H, oW2 = oB1 + H, oB2 = oW2 + (size_t)H * H, oW3 = oB2 + H, oB3 = oW3 + 2 * (size_t)H;
  std::vector<float> out(w, w + oB3 + 2);
  const double xmax = 46341.0;   // sqrt(2^31 - 1), rounded up
  auto pow2_below = [](double target, double v) {   // largest power of two s with v * s <= target (1 if v is 0)
    if (!(v > 0.0)) return 1.0;
    int e = (int)std::floor(std::log2(target / v));
    e = e < -60 ? -60 : e > 60 ? 60 : e;
    return std::ldexp(1.0, e);
  };
  std::vector<double> s1(H), s2(H);
  for (int u = 0; u < H; ++u) {
    double b = std::fabs((double)w[oB1 + u]);
    for (int f = 0; f < d; ++f) b += std::fabs((double)w[(size_t)f * H + u]) * (f < ne ? xmax : 1.0);
    s1[u] = pow2_below(32768.0, b);
  }
  for (int u = 0; u < H; ++u) {
    double cm = 0.0;
    for (int a = 0; a < H; ++a) cm = std::fmax(cm, std::fabs((double)w[oW2 + (size_t)a * H + u]) / s1[a]);
    s2[u] = pow2_below(8192.0, cm);
  }
  for (int u = 0; u < H; ++u) {
    for (int f = 0; f < d; ++f) out[(size_t)f * H + u] = (float)((double)w[(size_t)f * H + u] * s1[u]);
    out[oB1 + u] = (float)((double)w[oB1 + u] * s1[u]);
    for (int a = 0; a < H; ++a) out[oW2 + (size_t)a * H + u] = (float)((double)w[oW2 + (size_t)a * H + u] / s1[a] * s2[u]);
    out[oB2 + u] = (float)((double)w[oB2 + u] * s2[u]);
    out[oW3 + 2 * (size_t)u] = (float)((double)w[oW3 + 2 * (size_t)u] / s2[u]);
    out[oW3 + 2 * (size_t)u + 1] = (float)((double)w[oW3 + 2 * (size_t)u + 1] / s2[u]);
  }
  return out;
}

struct Plan {
  std::vector<lopt_tensor_desc> descs;
  std::vector<TensorDev> tensors;   // pointers filled per call
  std::vector<TileDev> tiles;
  std::vector<RcItemDev> rcitems;
  std::vector<ApplyTileDev> atiles;   // tiles of the strip-form apply kernel
  std::vector<int> atile0;            // first apply tile of every tensor
  uint64_t total_elems = 0;
  std::vector<size_t> state_bytes;
  uint64_t oLstmU = 0, oHNew = 0;   // VeLO scratch (floats)
  uint64_t oHbarPart = 0, oBeff = 0; // VeLO cross-tensor term: slice sums of h, gate bias with the term added
  uint64_t oAlpha = 0, oTheta = 0;   // VeLO, long lists: bank coefficients [T][K] and per-tensor MLPs [T][P]
  bool head_batched = false;
  uint64_t oCounters = 0;           // kMaxGroups ints: tile counters of the strip-form apply kernel
  uint64_t ws_floats = 0;
};

}  // namespace

struct lopt_ctx {
  lopt_config cfg;
  int device = 0;
  int n_cu = 256;
  int HP = 0, F = 0, P = 0;
  float* d_weights = nullptr;      // the uploaded blob
  float* d_tail = nullptr;         // small_fc_lopt: padded W2 b2 W3 b3
  WeightsDev W{};
  // cached plan + device tables: `heap` is library-allocated and grows with the list, `fixed` is the front of the
  // file-scope scratch array (lopt_step_static)
  Plan plan;
  bool plan_valid = false;
  TableStore heap, fixed;
  bool state_in_apply = true;      // the strip-form apply kernel writes M_1..3, V (configuration field state_pass)
  bool failed = false;             // a HIP call failed in the middle of a launch sequence: the context refuses further steps
  float loss = 0.f;                // lopt_set_loss: goes with the gradients of the following steps (VeLO)
  uint64_t id = 0;                 // names this context as the owner of the static scratch's contents
  void* static_scratch = nullptr;  // device address of `scratch` on ctx->device
  void* h_stage = nullptr;         // pinned staging
  size_t h_stage_bytes = 0;
  hipEvent_t stage_ev = nullptr;
  bool stage_pending = false;
  int apply_variant = 0;           // lopt_apply_kernel (configuration field, else LOPT_APPLY in the environment at create)
  // Group pipeline (small_fc_lopt, strip-form apply): the tensor list is cut into groups; the HBM-bound passes of
  // group g+1 run on `aux_stream` while the compute-bound apply pass of group g runs on the caller's stream.
  int groups_override = 0;         // configuration field, else LOPT_GROUPS in the environment at create (0 = choose by size)
  hipStream_t aux_stream = nullptr;
  hipEvent_t ev_fork = nullptr;
  std::vector<hipEvent_t> ev_start, ev_pre;   // per group: "previous group's passes are enqueued" / "this group's passes are done"
  // optional per-pass timing
  bool profiling = false;
  std::vector<hipEvent_t> prof_events;   // (LOPT_N_PASSES + 1) events per recorded step
  size_t prof_steps = 0;
  std::string err, err_first;
};

namespace {

lopt_status fail(lopt_ctx* ctx, lopt_status st, const std::string& msg) {
  if (ctx) ctx->err = msg;
  g_last_error = msg;
  return st;
}

#define HIP_TRY(ctx, call)                                                                   \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail(ctx, e_ == hipErrorOutOfMemory ? LOPT_ENOMEM : LOPT_EHIP,                  \
                  std::string(#call) + ": " + hipGetErrorString(e_));                        \
  } while (0)

lopt_status check_descs(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* d) {
  if (n > 0 && !d) return fail(ctx, LOPT_EINVAL, "descs_host is null");
  if (n > (size_t)1 << 24) return fail(ctx, LOPT_EINVAL, "too many tensors");
  for (size_t i = 0; i < n; ++i) {
    if (d[i].rows < 1 || d[i].cols < 1 || d[i].rows > 0x7fffffffLL || d[i].cols > 0x7fffffffLL ||
        d[i].rows * d[i].cols > 0x7fffffffLL) {
      char buf[160];
      snprintf(buf, sizeof buf, "tensor %zu: rows=%lld cols=%lld outside [1, 2^31-1] elements", i,
               (long long)d[i].rows, (long long)d[i].cols);
      return fail(ctx, LOPT_ESHAPE, buf);
    }
    if (d[i].ndim < 1) return fail(ctx, LOPT_EINVAL, "tensor ndim must be >= 1");
  }
  return LOPT_OK;
}

// Number of tensor groups of the two-stream pipeline for a list of `total` elements (0 override = by size).
int planned_groups(int override_g, uint64_t total, size_t n) {
  int G = override_g ? override_g : total >= (1024u << 20) ? 16 : total >= (256u << 20) ? 8 : total >= (32u << 20) ? 4 : 1;
  if ((size_t)G > n) G = (int)n;
  return G < 1 ? 1 : G;
}

// Contiguous tensor ranges [bound[g], bound[g+1]) of about equal element count.
void group_bounds(const lopt_tensor_desc* d, size_t n, int G, uint64_t total, int* bound) {
  uint64_t cum = 0;
  int g = 1;
  bound[0] = 0;
  for (size_t i = 0; i < n && g < G; ++i) {
    cum += (uint64_t)d[i].rows * (uint64_t)d[i].cols;
    if (cum * (uint64_t)G >= total * (uint64_t)g && (int)i + 1 > bound[g - 1]) bound[g++] = (int)i + 1;
  }
  while (g <= G) bound[g++] = (int)n;
}

// Lay out tiles, row/column blocks and workspace regions for a tensor list.
void build_plan(const lopt_ctx* ctx, size_t n, const lopt_tensor_desc* d, Plan* pl) {
  pl->descs.assign(d, d + n);
  pl->tensors.assign(n, TensorDev{});
  pl->tiles.clear();
  pl->rcitems.clear();
  pl->atiles.clear();
  pl->atile0.assign(n, 0);
  pl->total_elems = 0;
  pl->state_bytes.assign(n, 0);
  const bool velo = ctx->cfg.kind == LOPT_VELO;
  const int HP = ctx->HP;
  const uint64_t prep_floats = (uint64_t)(LOPT_D_VELO + 1) * HP + (uint64_t)HP * HP + HP + 2 * HP + 2;
  uint64_t off = 0;
  auto take = [&](uint64_t nfloats) { uint64_t o = off; off = align64(off + nfloats); return o; };
  pl->oCounters = take(kMaxGroups);
  if (velo) {
    pl->oLstmU = take((uint64_t)n * kLstmInPad);
    pl->oHNew = take((uint64_t)n * ctx->cfg.lstm_hidden);
    pl->oHbarPart = take((uint64_t)kMixSlices * ctx->cfg.lstm_hidden);
    pl->oBeff = take((uint64_t)kMixJSplit * 4ull * ctx->cfg.lstm_hidden);
    pl->head_batched = n >= (size_t)kHeadBatchMin;
    if (pl->head_batched) {
      pl->oAlpha = take((uint64_t)n * ctx->cfg.n_bank);
      pl->oTheta = take((uint64_t)n * (uint64_t)ctx->P);
    }
  }
  // Apply tiles get shorter towards the end of every tensor group of the pipeline (a single group if it is off): the
  // strip apply kernel hands tiles out in table order, so the last tiles of a launch decide how long the chip idles
  // while the final workgroups finish (a 128-row tile is about 90 us of work, a 32-row tile a quarter of that).
  uint64_t total = 0;
  for (size_t i = 0; i < n; ++i) total += (uint64_t)d[i].rows * (uint64_t)d[i].cols;
  const int G_plan = ctx->cfg.kind == LOPT_SMALL_FC ? planned_groups(ctx->groups_override, total, n) : 1;
  int gbound[kMaxGroups + 1];
  group_bounds(d, n, G_plan, total, gbound);
  std::vector<uint64_t> gtotal(G_plan, 0), gbefore(n, 0);
  for (int g = 0; g < G_plan; ++g)
    for (int i = gbound[g]; i < gbound[g + 1]; ++i) {
      gbefore[i] = gtotal[g];
      gtotal[g] += (uint64_t)d[i].rows * (uint64_t)d[i].cols;
    }
  std::vector<int> group_of(n, 0);
  for (int g = 0; g < G_plan; ++g)
    for (int i = gbound[g]; i < gbound[g + 1]; ++i) group_of[i] = g;
  // Small parameter sets: with the standard 64-row tiles there may be fewer tiles than the chip has workgroup
  // slots (256 CUs x 2..8), so the tile height is halved until the list yields about 2048 tiles or reaches 8 rows.
  uint64_t std_tiles = 0;
  for (size_t i = 0; i < n; ++i)
    std_tiles += (uint64_t)((d[i].rows + kRowUnit - 1) / kRowUnit) * (uint64_t)((d[i].cols + kTileCols - 1) / kTileCols);
  int shrink = 1;
  while (shrink < 8 && std_tiles * shrink < 2048) shrink *= 2;
  for (size_t i = 0; i < n; ++i) {
    TensorDev& T = pl->tensors[i];
    const int m = (int)d[i].rows, nn = (int)d[i].cols;
    const uint64_t N = (uint64_t)m * nn;
    T.m = m; T.n = nn;
    T.padN = pad4(N); T.padm = pad4(m); T.padn = pad4(nn);
    T.padH = velo ? pad4(ctx->cfg.lstm_hidden) : 0;
    T.ndim = d[i].ndim;
    T.vec = (nn % 4 == 0) ? 1 : 0;
    const int units = (m + kRowUnit - 1) / kRowUnit;
    const int q = (units + kMaxRowTiles - 1) / kMaxRowTiles;
    T.TR = kRowUnit * (q < 1 ? 1 : q) / shrink;   // a multiple of 8: every wavefront of a tile owns whole rows
    // ... but never more than kMaxRowTiles row tiles per tensor (the second-stage reductions loop over them; a small
    // list, whose tiles were made shorter above, may have `shrink` times as many) ...
    const int max_rt = kMaxRowTiles * shrink;
    const int min_tr = ((m + max_rt - 1) / max_rt + 7) & ~7;
    if (T.TR < min_tr) T.TR = min_tr;
    // ... unless that makes a tile taller than kMaxTileRows: a lane sums a quarter of the tile's rows in fp32
    // (four values per row), and such a partial sum must stay at about a thousand terms. Tensors of more than
    // kMaxRowTiles * kMaxTileRows rows get more row tiles instead.
    if (T.TR > kMaxTileRows) T.TR = kMaxTileRows;
    T.nrt = (m + T.TR - 1) / T.TR;
    T.nct = (nn + kTileCols - 1) / kTileCols;
    T.tile0 = (int)pl->tiles.size();
    for (int ti = 0; ti < T.nrt; ++ti)
      for (int tj = 0; tj < T.nct; ++tj) pl->tiles.push_back(TileDev{(int)i, ti, tj, 0});
    T.nrblk = (m + kBlock - 1) / kBlock;
    T.ncblk = (nn + kBlock - 1) / kBlock;
    T.rc0 = (int)pl->rcitems.size();
    for (int b = 0; b < T.nrblk; ++b) pl->rcitems.push_back(RcItemDev{(int)i, 0, b, 0});
    for (int b = 0; b < T.ncblk; ++b) pl->rcitems.push_back(RcItemDev{(int)i, 1, b, 0});
    // apply tiles: up to kApplyRows x kApplyCols, shorter for small lists like the statistics tiles
    pl->atile0[i] = (int)pl->atiles.size();
    pl->total_elems += N;
    for (int ar0 = 0; ar0 < m;) {
      // position of this row block inside its group: full height for the first 70 %, half to 88 %, a quarter after
      const uint64_t pos = gbefore[i] + (uint64_t)ar0 * (uint64_t)nn, gt = gtotal[group_of[i]];
      int AR = kApplyRows / shrink;
      if (pos * 100 >= gt * 88) AR /= 4;
      else if (pos * 100 >= gt * 70) AR /= 2;
      if (AR < 8) AR = 8;
      const int rows = m - ar0 < AR ? m - ar0 : AR;
      for (int ac0 = 0; ac0 < nn; ac0 += kApplyCols) pl->atiles.push_back(ApplyTileDev{(int)i, ar0, ac0, rows});
      ar0 += rows;
    }
    T.oRowPart = take((uint64_t)T.nct * m);
    T.oColPart = take((uint64_t)T.nrt * nn);
    T.oRR = take(3ull * T.padm);
    T.oRC = take(3ull * T.padn);
    T.oRcPart = take((uint64_t)(T.nrblk + T.ncblk) * kRcStride);
    T.oStatPart = take((uint64_t)T.nrt * T.nct * kStatStride);
    T.oStats = take(kStatsPerTensor);
    T.oScale = take(kStatsPerTensor);
    T.oPrep = take(prep_floats);
    pl->state_bytes[i] = sizeof(float) * (4ull * T.padN + 3ull * T.padm + 3ull * T.padn + 2ull * T.padH);
  }
  pl->ws_floats = off;
}

bool same_descs(const Plan& pl, size_t n, const lopt_tensor_desc* d) {
  if (pl.descs.size() != n) return false;
  for (size_t i = 0; i < n; ++i)
    if (pl.descs[i].ndim != d[i].ndim || pl.descs[i].rows != d[i].rows || pl.descs[i].cols != d[i].cols)
      return false;
  return true;
}

lopt_status ensure_plan(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* d) {
  if (ctx->plan_valid && same_descs(ctx->plan, n, d)) return LOPT_OK;
  try {
    build_plan(ctx, n, d, &ctx->plan);
  } catch (const std::bad_alloc&) {
    ctx->plan_valid = false;
    return fail(ctx, LOPT_ENOMEM, "out of host memory while planning");
  }
  ctx->plan_valid = true;
  for (TableStore* st : {&ctx->heap, &ctx->fixed}) st->static_uploaded = st->tensors_uploaded = false;
  return LOPT_OK;
}

size_t table_bytes(const Plan& pl) {
  return align64(pl.tensors.size() * sizeof(TensorDev)) + align64(pl.tiles.size() * sizeof(TileDev)) +
         align64(pl.rcitems.size() * sizeof(RcItemDev)) + align64(pl.atiles.size() * sizeof(ApplyTileDev));
}

// Make sure the device tables of `st` hold the current plan and pointers. A growable store and the pinned staging
// buffer are reallocated when the list outgrows them; a fixed store never allocates (the caller has checked that the
// tables fit both).
lopt_status upload_tables(lopt_ctx* ctx, TableStore& st, hipStream_t stream) {
  Plan& pl = ctx->plan;
  const size_t nT = pl.tensors.size(), nTi = pl.tiles.size(), nRc = pl.rcitems.size(), nAt = pl.atiles.size();
  const size_t bT = align64(nT * sizeof(TensorDev)), bTi = align64(nTi * sizeof(TileDev)),
               bRc = align64(nRc * sizeof(RcItemDev)), bAt = align64(nAt * sizeof(ApplyTileDev));
  const size_t need = bT + bTi + bRc + bAt;
  if (need == 0) return LOPT_OK;
  if (need > st.cap) {
    if (!st.growable) return fail(ctx, LOPT_ELIMIT, "device tables do not fit the fixed scratch region");
    if (ctx->stage_pending) { HIP_TRY(ctx, hipEventSynchronize(ctx->stage_ev)); ctx->stage_pending = false; }
    if (st.base) { HIP_TRY(ctx, hipStreamSynchronize(stream)); HIP_TRY(ctx, hipFree(st.base)); st.base = nullptr; }
    st.cap = 0;
    HIP_TRY(ctx, hipMalloc((void**)&st.base, need));
    st.cap = need;
    st.static_uploaded = false;
    st.tensors_uploaded = false;
  }
  if (need > ctx->h_stage_bytes) {
    if (!st.growable) return fail(ctx, LOPT_ELIMIT, "device tables do not fit the pinned staging buffer");
    if (ctx->stage_pending) { HIP_TRY(ctx, hipEventSynchronize(ctx->stage_ev)); ctx->stage_pending = false; }
    if (ctx->h_stage) { HIP_TRY(ctx, hipHostFree(ctx->h_stage)); ctx->h_stage = nullptr; }
    ctx->h_stage_bytes = 0;
    HIP_TRY(ctx, hipHostMalloc(&ctx->h_stage, need, hipHostMallocDefault));
    ctx->h_stage_bytes = need;
  }
  char* dbase = st.base;
  st.d_tensors = (TensorDev*)dbase;
  st.d_tiles = (TileDev*)(dbase + bT);
  st.d_rcitems = (RcItemDev*)(dbase + bT + bTi);
  st.d_atiles = (ApplyTileDev*)(dbase + bT + bTi + bRc);
  const bool need_tensors = !st.tensors_uploaded || st.last_tensors.size() != nT ||
                            memcmp(st.last_tensors.data(), pl.tensors.data(), nT * sizeof(TensorDev)) != 0;
  const bool need_static = !st.static_uploaded;
  if (!need_tensors && !need_static) return LOPT_OK;
  if (ctx->stage_pending) { HIP_TRY(ctx, hipEventSynchronize(ctx->stage_ev)); ctx->stage_pending = false; }
  char* hbase = (char*)ctx->h_stage;
  if (need_tensors) {
    memcpy(hbase, pl.tensors.data(), nT * sizeof(TensorDev));
    HIP_TRY(ctx, hipMemcpyAsync(st.d_tensors, hbase, nT * sizeof(TensorDev), hipMemcpyHostToDevice, stream));
    st.last_tensors = pl.tensors;
    st.tensors_uploaded = true;
  }
  if (need_static) {
    memcpy(hbase + bT, pl.tiles.data(), nTi * sizeof(TileDev));
    memcpy(hbase + bT + bTi, pl.rcitems.data(), nRc * sizeof(RcItemDev));
    HIP_TRY(ctx, hipMemcpyAsync(st.d_tiles, hbase + bT, nTi * sizeof(TileDev) , hipMemcpyHostToDevice, stream));
    if (nRc) HIP_TRY(ctx, hipMemcpyAsync(st.d_rcitems, hbase + bT + bTi, nRc * sizeof(RcItemDev), hipMemcpyHostToDevice, stream));
    memcpy(hbase + bT + bTi + bRc, pl.atiles.data(), nAt * sizeof(ApplyTileDev));
    if (nAt) HIP_TRY(ctx, hipMemcpyAsync(st.d_atiles, hbase + bT + bTi + bRc, nAt * sizeof(ApplyTileDev), hipMemcpyHostToDevice, stream));
    st.static_uploaded = true;
  }
  HIP_TRY(ctx, hipEventRecord(ctx->stage_ev, stream));
  ctx->stage_pending = true;
  return LOPT_OK;
}

StepArgs make_args(const lopt_ctx* ctx, int64_t step, float lr, float wd, int n_tensors) {
  StepArgs A{};
  const lopt_config& c = ctx->cfg;
  for (int i = 0; i < 3; ++i) { A.mom_decay[i] = c.mom_decay[i]; A.fac_decay[i] = c.fac_decay[i]; }
  A.rms_decay = c.rms_decay;
  A.eps_acc = c.eps_acc; A.eps_norm = c.eps_norm;
  A.exp_mult = c.exp_mult; A.step_mult = c.step_mult;
  A.lr = lr; A.wd = wd;
  A.step = (long long)step;
  A.kind = (int)c.kind; A.H = (int)c.hidden; A.HP = ctx->HP; A.F = ctx->F;
  A.HL = (int)c.lstm_hidden; A.K = (int)c.n_bank; A.P = ctx->P;
  A.n_tensors = n_tensors;
  A.loss = ctx->loss;
  return A;
}

}  // namespace

extern "C" {

lopt_status lopt_default_config(uint32_t kind, lopt_config* cfg) {
  if (!cfg) return fail(nullptr, LOPT_EINVAL, "cfg is null");
  if (kind != LOPT_SMALL_FC && kind != LOPT_VELO) return fail(nullptr, LOPT_EINVAL, "unknown kind");
  memset(cfg, 0, sizeof *cfg);
  cfg->struct_size = sizeof(lopt_config);
  cfg->kind = kind;
  cfg->hidden = kind == LOPT_SMALL_FC ? 32 : 4;
  cfg->mom_decay[0] = 0.9f; cfg->mom_decay[1] = 0.99f; cfg->mom_decay[2] = 0.999f;
  cfg->rms_decay = 0.999f;
  cfg->fac_decay[0] = 0.9f; cfg->fac_decay[1] = 0.99f; cfg->fac_decay[2] = 0.999f;
  cfg->eps_acc = 1e-16f;
  cfg->eps_norm = 1e-30f;
  cfg->exp_mult = 0.01f;
  cfg->step_mult = 0.01f;
  cfg->lstm_hidden = 512;
  cfg->n_bank = 256;
  return LOPT_OK;
}

size_t lopt_weights_count(const lopt_config* c) {
  if (!config_ok(c, nullptr)) return 0;
  if (c->kind == LOPT_SMALL_FC) return mlp_count(LOPT_D_SMALL_FC, (int)c->hidden);
  const size_t HL = c->lstm_hidden, K = c->n_bank, P = mlp_count(LOPT_D_VELO, (int)c->hidden);
  return (size_t)LOPT_VELO_LSTM_IN * 4 * HL + 2 * (HL * 4 * HL) + 4 * HL + HL * K + K + HL + 1 + K * P;
}

lopt_status lopt_create(const lopt_config* cfg, const float* weights_host, size_t n_weights, lopt_ctx** out) {
  std::string why;
  if (!out) return fail(nullptr, LOPT_EINVAL, "out is null");
  if (!config_ok(cfg, &why)) return fail(nullptr, LOPT_EINVAL, why);
  if (!weights_host) return fail(nullptr, LOPT_EINVAL, "weights_host is null");
  const size_t want = lopt_weights_count(cfg);
  if (n_weights != want) {
    char buf[128];
    snprintf(buf, sizeof buf, "n_weights=%zu but this configuration needs %zu floats", n_weights, want);
    return fail(nullptr, LOPT_ESTATE, buf);
  }
  for (size_t i = 0; i < n_weights; ++i)
    if (!std::isfinite(weights_host[i])) return fail(nullptr, LOPT_EINVAL, "weights_host holds a non-finite value");
  std::vector<float> eq;
  if (cfg->kind == LOPT_SMALL_FC) {
    try { eq = equilibrate_small_fc(weights_host, (int)cfg->hidden); } catch (const std::bad_alloc&) { return fail(nullptr, LOPT_ENOMEM, "out of host memory"); }
    weights_host = eq.data();   // from here on: the equivalent, rescaled network
  }
  // the configuration's fields select kernel and launch plan; the environment fills in fields left at 0
  int apply_variant = (int)cfg->apply_kernel, groups_override = (int)cfg->groups, state_pass = (int)cfg->state_pass;
  if (const char* e = getenv("LOPT_APPLY")) {
    const int v = !strcmp(e, "auto") ? LOPT_APPLY_AUTO : !strcmp(e, "valu") ? LOPT_APPLY_VALU
                : !strcmp(e, "mfma_f32") ? LOPT_APPLY_MFMA_F32 : !strcmp(e, "mfma_f16s") ? LOPT_APPLY_MFMA_F16S : -1;
    if (v < 0)
      return fail(nullptr, LOPT_EINVAL, std::string("LOPT_APPLY=") + e + " is not one of auto, valu, mfma_f32, mfma_f16s");
    if (!apply_variant) apply_variant = v;
  }
  if (const char* e = getenv("LOPT_GROUPS")) {
    char* end = nullptr;
    const long g = strtol(e, &end, 10);
    if (end == e || *end || g < 0 || g > kMaxGroups)
      return fail(nullptr, LOPT_EINVAL, std::string("LOPT_GROUPS=") + e + " is not an integer in [0, 16]");
    if (!groups_override) groups_override = (int)g;
  }
  if (const char* e = getenv("LOPT_STATE_PASS")) {
    const int v = !strcmp(e, "auto") ? LOPT_STATE_AUTO : !strcmp(e, "stats") ? LOPT_STATE_IN_STATS
                : !strcmp(e, "apply") ? LOPT_STATE_IN_APPLY : -1;
    if (v < 0) return fail(nullptr, LOPT_EINVAL, std::string("LOPT_STATE_PASS=") + e + " is not one of auto, stats, apply");
    if (!state_pass) state_pass = v;
  }
  lopt_ctx* ctx = new (std::nothrow) lopt_ctx();
  if (!ctx) return fail(nullptr, LOPT_ENOMEM, "out of host memory");
  ctx->cfg = *cfg;
  ctx->apply_variant = apply_variant;
  ctx->state_in_apply = state_pass != LOPT_STATE_IN_STATS;
  ctx->groups_override = groups_override;
  const int H = (int)cfg->hidden;
  ctx->HP = padded_hidden(H);
  ctx->F = cfg->kind == LOPT_SMALL_FC ? LOPT_N_ELEM_FEATS : LOPT_D_VELO;
  ctx->P = (int)mlp_count(LOPT_D_VELO, H);
  lopt_status st = LOPT_OK;
  auto cleanup = [&](lopt_status s) { std::string m = ctx->err; lopt_destroy(ctx); g_last_error = m; return s; };
#define CREATE_TRY(call)                                                                      \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess) {                                                                   \
      fail(ctx, e_ == hipErrorOutOfMemory ? LOPT_ENOMEM : LOPT_EHIP,                          \
           std::string(#call) + ": " + hipGetErrorString(e_));                                \
      return cleanup(e_ == hipErrorOutOfMemory ? LOPT_ENOMEM : LOPT_EHIP);                    \
    }                                                                                         \
  } while (0)
  CREATE_TRY(hipGetDevice(&ctx->device));
  CREATE_TRY(hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device));
  CREATE_TRY(hipMalloc((void**)&ctx->d_weights, n_weights * sizeof(float)));
  CREATE_TRY(hipMemcpy(ctx->d_weights, weights_host, n_weights * sizeof(float), hipMemcpyHostToDevice));
  CREATE_TRY(hipEventCreateWithFlags(&ctx->stage_ev, hipEventDisableTiming));
  CREATE_TRY(hipHostMalloc(&ctx->h_stage, kStageInitBytes, hipHostMallocDefault));
  ctx->h_stage_bytes = kStageInitBytes;
  ctx->heap.growable = true;
  ctx->id = g_next_ctx_id.fetch_add(1);
  if (ctx->device >= 0 && ctx->device < kMaxDevices) {
    // the fixed scratch of lopt_step_static: resolve this device's copy once, with this device current
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[ctx->device]) {
      void* sp = nullptr;
      CREATE_TRY(hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)));
      g_scratch_ptr[ctx->device] = sp;
    }
    ctx->static_scratch = g_scratch_ptr[ctx->device];
    ctx->fixed.base = (char*)ctx->static_scratch;
  }
  {
    CREATE_TRY(hipStreamCreateWithFlags(&ctx->aux_stream, hipStreamNonBlocking));
    CREATE_TRY(hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming));
    for (int g = 0; g < kMaxGroups; ++g) {
      hipEvent_t a = nullptr, b = nullptr;
      CREATE_TRY(hipEventCreateWithFlags(&a, hipEventDisableTiming));
      ctx->ev_start.push_back(a);
      CREATE_TRY(hipEventCreateWithFlags(&b, hipEventDisableTiming));
      ctx->ev_pre.push_back(b);
    }
  }
  if (cfg->kind == LOPT_SMALL_FC) {
    const int HP = ctx->HP;
    // W2 b2 W3 b3 zero-padded to HP, followed by the un-normalized first layer W1[28][HP] (padded)
    const size_t tail_n = (size_t)HP * HP + HP + 2 * HP + 2;
    std::vector<float> tail(tail_n + 2 + (size_t)LOPT_N_ELEM_FEATS * HP, 0.f);
    const float* W2 = weights_host + (size_t)LOPT_D_SMALL_FC * H + H;
    const float* b2 = W2 + (size_t)H * H;
    const float* W3 = b2 + H;
    const float* b3 = W3 + 2 * H;
    for (int a = 0; a < H; ++a)
      for (int u = 0; u < H; ++u) tail[(size_t)a * HP + u] = W2[a * H + u];
    for (int u = 0; u < H; ++u) tail[(size_t)HP * HP + u] = b2[u];
    for (int a = 0; a < H; ++a) { tail[(size_t)HP * HP + HP + 2 * a] = W3[2 * a]; tail[(size_t)HP * HP + HP + 2 * a + 1] = W3[2 * a + 1]; }
    tail[(size_t)HP * HP + HP + 2 * HP] = b3[0];
    tail[(size_t)HP * HP + HP + 2 * HP + 1] = b3[1];
    for (int f = 0; f < LOPT_N_ELEM_FEATS; ++f)
      for (int u = 0; u < H; ++u) tail[tail_n + 2 + (size_t)f * HP + u] = weights_host[(size_t)f * H + u];
    CREATE_TRY(hipMalloc((void**)&ctx->d_tail, tail.size() * sizeof(float)));
    CREATE_TRY(hipMemcpy(ctx->d_tail, tail.data(), tail.size() * sizeof(float), hipMemcpyHostToDevice));
    ctx->W.mlp = ctx->d_weights;
    ctx->W.mlp_tail = ctx->d_tail;
  } else {
    const size_t HL = cfg->lstm_hidden, K = cfg->n_bank;
    const float* w = ctx->d_weights;
    ctx->W.Wx = w; w += (size_t)LOPT_VELO_LSTM_IN * 4 * HL;
    ctx->W.Wh = w; w += HL * 4 * HL;
    ctx->W.Wg = w; w += HL * 4 * HL;
    ctx->W.b = w; w += 4 * HL;
    ctx->W.Wa = w; w += HL * K;
    ctx->W.ba = w; w += K;
    ctx->W.ws = w; w += HL;
    ctx->W.bs = w; w += 1;
    ctx->W.B = w;
  }
#undef CREATE_TRY
  (void)st;
  *out = ctx;
  return LOPT_OK;
}

void lopt_destroy(lopt_ctx* ctx) {
  if (!ctx) return;
  if (ctx->d_weights) (void)hipFree(ctx->d_weights);
  if (ctx->d_tail) (void)hipFree(ctx->d_tail);
  if (ctx->heap.base) (void)hipFree(ctx->heap.base);
  if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
  if (ctx->stage_ev) (void)hipEventDestroy(ctx->stage_ev);
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  if (ctx->aux_stream) { (void)hipStreamSynchronize(ctx->aux_stream); (void)hipStreamDestroy(ctx->aux_stream); }
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  for (hipEvent_t e : ctx->ev_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : ctx->ev_pre) (void)hipEventDestroy(e);
  delete ctx;
}

lopt_status lopt_state_bytes(const lopt_ctx* cctx, size_t n, const lopt_tensor_desc* descs, size_t* per_tensor,
                             size_t* workspace_bytes) {
  lopt_ctx* ctx = const_cast<lopt_ctx*>(cctx);
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  lopt_status st = check_descs(ctx, n, descs);
  if (st != LOPT_OK) return st;
  Plan tmp;
  const Plan* pl = &tmp;
  if (ctx->plan_valid && same_descs(ctx->plan, n, descs)) pl = &ctx->plan;
  else {
    try { build_plan(ctx, n, descs, &tmp); } catch (const std::bad_alloc&) { return fail(ctx, LOPT_ENOMEM, "out of host memory while planning"); }
  }
  if (per_tensor) for (size_t i = 0; i < n; ++i) per_tensor[i] = pl->state_bytes[i];
  if (workspace_bytes) *workspace_bytes = (size_t)(pl->ws_floats * sizeof(float)) + 256;
  return LOPT_OK;
}

lopt_status lopt_stats_offsets(const lopt_ctx* cctx, size_t n, const lopt_tensor_desc* descs, size_t* offsets) {
  lopt_ctx* ctx = const_cast<lopt_ctx*>(cctx);
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  if (n > 0 && !offsets) return fail(ctx, LOPT_EINVAL, "offsets_bytes is null");
  lopt_status st = check_descs(ctx, n, descs);
  if (st != LOPT_OK) return st;
  Plan tmp;
  const Plan* pl = &tmp;
  if (ctx->plan_valid && same_descs(ctx->plan, n, descs)) pl = &ctx->plan;
  else {
    try { build_plan(ctx, n, descs, &tmp); } catch (const std::bad_alloc&) { return fail(ctx, LOPT_ENOMEM, "out of host memory while planning"); }
  }
  for (size_t i = 0; i < n; ++i) offsets[i] = (size_t)pl->tensors[i].oStats * sizeof(float);
  return LOPT_OK;
}

static lopt_status check_ptrs(lopt_ctx* ctx, size_t n, const void* const* arr, const char* name) {
  if (n > 0 && !arr) return fail(ctx, LOPT_EINVAL, std::string(name) + " is null");
  for (size_t i = 0; i < n; ++i) {
    if (!arr[i]) return fail(ctx, LOPT_EINVAL, std::string(name) + "[" + std::to_string(i) + "] is null");
    if ((uintptr_t)arr[i] & 15) return fail(ctx, LOPT_EINVAL, std::string(name) + "[" + std::to_string(i) + "] is not 16-byte aligned");
  }
  return LOPT_OK;
}

lopt_status lopt_init_state(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs, void* const* state, void* workspace,
                            void* hip_stream) {
  (void)workspace;
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  lopt_status st = check_descs(ctx, n, descs);
  if (st != LOPT_OK) return st;
  st = check_ptrs(ctx, n, (const void* const*)state, "state_host");
  if (st != LOPT_OK) return st;
  if (n == 0) return LOPT_OK;
  st = ensure_plan(ctx, n, descs);
  if (st != LOPT_OK) return st;
  hipStream_t stream = (hipStream_t)hip_stream;
  for (size_t i = 0; i < n; ++i) {
    TensorDev& T = ctx->plan.tensors[i];
    T.st = (float*)state[i];
  }
  st = upload_tables(ctx, ctx->heap, stream);
  if (st != LOPT_OK) return st;
  const TableStore& tb = ctx->heap;
  Launch L{tb.d_tensors, tb.d_tiles, tb.d_rcitems, nullptr, (int)n, (int)ctx->plan.tiles.size(),
           (int)ctx->plan.rcitems.size(), tb.d_atiles, (int)ctx->plan.atiles.size(), 0, nullptr, 0};
  StepArgs A = make_args(ctx, 0, 0.f, 0.f, (int)n);
  launch_fill_zero(L, A, stream);
  HIP_TRY(ctx, hipGetLastError());
  return LOPT_OK;
}

}  // extern "C"

// One step. use_static: tables and workspace live in the file-scope scratch array of this device (`workspace` is
// ignored) and nothing on this path allocates.
static lopt_status step_impl(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs, float* const* params,
                             const float* const* grads, void* const* state, void* workspace, int64_t step, float lr,
                             float weight_decay, void* hip_stream, bool use_static) {
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  if (ctx->failed) return fail(ctx, LOPT_EHIP, "this context failed in the middle of an earlier step (" + ctx->err_first + "); create a new one");
  lopt_status st = check_descs(ctx, n, descs);
  if (st != LOPT_OK) return st;
  if (step < 0) return fail(ctx, LOPT_EINVAL, "step must be >= 0");
  if (!std::isfinite(lr) || !std::isfinite(weight_decay)) return fail(ctx, LOPT_EINVAL, "lr and weight_decay must be finite");
  if ((st = check_ptrs(ctx, n, (const void* const*)params, "params_host")) != LOPT_OK) return st;
  if ((st = check_ptrs(ctx, n, (const void* const*)grads, "grads_host")) != LOPT_OK) return st;
  if ((st = check_ptrs(ctx, n, (const void* const*)state, "state_host")) != LOPT_OK) return st;
  if (n == 0) return LOPT_OK;
  if (use_static) {
    if (!ctx->static_scratch) return fail(ctx, LOPT_EINVAL, "no static scratch on this device");
  } else {
    if (!workspace) return fail(ctx, LOPT_EINVAL, "workspace is null");
    if ((uintptr_t)workspace & 15) return fail(ctx, LOPT_EINVAL, "workspace is not 16-byte aligned");
  }
  if ((st = ensure_plan(ctx, n, descs)) != LOPT_OK) return st;
  hipStream_t stream = (hipStream_t)hip_stream;
  Plan& pl = ctx->plan;
  TableStore& tb = use_static ? ctx->fixed : ctx->heap;
  if (use_static) {
    // layout of the array: [tables, rounded up to 256 bytes | workspace]
    const size_t tbytes = (table_bytes(pl) + 255) & ~(size_t)255;
    const size_t need = tbytes + (size_t)pl.ws_floats * sizeof(float);
    if (need > kStaticScratchBytes || table_bytes(pl) > ctx->h_stage_bytes) {
      char buf[200];
      snprintf(buf, sizeof buf, "this tensor list needs %zu bytes of scratch (%zu of them tables); lopt_step_static has %zu "
               "(tables: %zu)", need, table_bytes(pl), kStaticScratchBytes, ctx->h_stage_bytes);
      return fail(ctx, LOPT_ELIMIT, buf);
    }
    tb.cap = tbytes;
    workspace = ctx->fixed.base + tbytes;
    // another context may have used the array since this one last did: then nothing of ours is left in it
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_owner[ctx->device] != ctx->id) tb.static_uploaded = tb.tensors_uploaded = false;
    g_scratch_owner[ctx->device] = ctx->id;
  }
  for (size_t i = 0; i < n; ++i) {
    TensorDev& T = pl.tensors[i];
    T.p = params[i];
    T.g = grads[i];
    T.st = (float*)state[i];
  }
  if ((st = upload_tables(ctx, tb, stream)) != LOPT_OK) return st;
  // workspace base rounded up to 256 bytes (lopt_state_bytes adds the slack)
  float* ws = (float*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  Launch L{tb.d_tensors, tb.d_tiles, tb.d_rcitems, ws, (int)n, (int)pl.tiles.size(), (int)pl.rcitems.size(),
           tb.d_atiles, (int)pl.atiles.size(), 0, (int*)(ws + pl.oCounters), 2 * ctx->n_cu};
  const bool profiling = ctx->profiling && !use_static;   // per-pass timing creates events: not on the static path
  StepArgs A = make_args(ctx, step, lr, weight_decay, (int)n);
  const bool mfma_ok = apply_mfma_available(A);
  // the strip-form kernel addresses a row pair with 32-bit byte offsets from the tile's first column: 4 (127 + cols)
  // must stay below the range of its store descriptors (2^32 - 512), which only a tensor of two or more rows and
  // 2^30 - 255 or more columns breaks (it takes the fp32 kernel)
  bool strip_ok = mfma_ok && (ctx->apply_variant == LOPT_APPLY_AUTO || ctx->apply_variant == LOPT_APPLY_MFMA_F16S);
  for (size_t i = 0; strip_ok && i < n; ++i) strip_ok = descs[i].rows == 1 || descs[i].cols <= (1 << 30) - 256;
  // With the two default apply kernels the momentum / second-moment accumulators are written by the apply pass and the
  // statistics pass only reads them: 24 + 44 instead of 40 + 28 bytes per element (configuration field state_pass).
  // The read-only statistics stream runs at 83 % of the HBM rate against 67 % for the read-write one; the strip-form
  // kernel is bound by instruction issue and takes the extra stores in its stride, the VeLO kernel is HBM-bound and
  // gives part of the gain back.
  const bool velo4_ok = ctx->cfg.kind == LOPT_VELO && ctx->apply_variant != LOPT_APPLY_VALU && apply_velo4_available(A);
  const bool state_in_apply = (strip_ok || velo4_ok) && ctx->state_in_apply;
  auto launch_apply = [&](const Launch& La) {
    if (strip_ok) launch_apply_f16s(La, A, ctx->W, state_in_apply, stream);
    else if (mfma_ok && ctx->apply_variant != LOPT_APPLY_VALU) launch_apply_mfma(La, A, ctx->W, stream);
    else if (ctx->cfg.kind == LOPT_SMALL_FC) launch_apply_small_fc(La, A, ctx->W, stream);
    else if (velo4_ok) launch_apply_velo4(La, A, state_in_apply, stream);
    else launch_apply_velo(La, A, ctx->W, stream);
  };
  // ---- group pipeline: only where the apply pass is compute-bound (strip form), the list is large enough to
  // pay for the extra launches, and per-pass timing is off (its events assume one pass after the other)
  int G = 1;
  const bool velo = ctx->cfg.kind == LOPT_VELO;
  if (ctx->aux_stream && !profiling) {
    if (strip_ok) G = planned_groups(ctx->groups_override, pl.total_elems, n);
    else if (velo && ctx->groups_override) G = planned_groups(ctx->groups_override, pl.total_elems, n);
  }
  // From here on kernels are in flight: a HIP error leaves params and state partly updated. The context is marked
  // failed, and the second stream (if it was forked) is joined back so that the caller's stream semantics hold.
  bool forked = false;
  auto launch_failed = [&](hipError_t e, const char* what) {
    if (forked) {
      (void)hipEventRecord(ctx->ev_pre[0], ctx->aux_stream);
      (void)hipStreamWaitEvent(stream, ctx->ev_pre[0], 0);
    }
    ctx->failed = true;
    ctx->err_first = std::string(what) + ": " + hipGetErrorString(e);
    return fail(ctx, e == hipErrorOutOfMemory ? LOPT_ENOMEM : LOPT_EHIP, ctx->err_first);
  };
#define LAUNCH_TRY(call)                                              \
  do {                                                                \
    hipError_t e_ = (call);                                           \
    if (e_ != hipSuccess) return launch_failed(e_, #call);            \
  } while (0)
  if (G > 1) {
    // contiguous tensor ranges of about equal element count
    int bound[kMaxGroups + 1];
    group_bounds(descs, n, G, pl.total_elems, bound);
    auto sub = [&](int g) {
      const int t0 = bound[g], t1 = bound[g + 1];
      Launch S = L;
      if (t0 >= t1) { S.n_tensors = S.n_tiles = S.n_rcitems = S.n_atiles = 0; return S; }
      const int tile0 = pl.tensors[t0].tile0, tile1 = t1 < (int)n ? pl.tensors[t1].tile0 : (int)pl.tiles.size();
      const int rc0 = pl.tensors[t0].rc0, rc1 = t1 < (int)n ? pl.tensors[t1].rc0 : (int)pl.rcitems.size();
      const int at0 = pl.atile0[t0], at1 = t1 < (int)n ? pl.atile0[t1] : (int)pl.atiles.size();
      S.tiles = L.tiles + tile0; S.n_tiles = tile1 - tile0;
      S.rcitems = L.rcitems + rc0; S.n_rcitems = rc1 - rc0;
      S.atiles = L.atiles + at0; S.n_atiles = at1 - at0;
      S.tensor0 = t0; S.n_tensors = t1 - t0;
      S.apply_counter = L.apply_counter + g;
      return S;
    };
    // accumulator update + statistics + per-tensor finalize of one group: what its apply pass waits for
    auto stats_passes = [&](const Launch& S, hipStream_t s) {
      launch_accum_stats(S, A, !state_in_apply, s);
      launch_finalize(S, A, ctx->W, ws + pl.oLstmU, s);
      if (velo) {
        launch_velo_lstm(S, A, ctx->W, ws + pl.oLstmU, ws + pl.oBeff, ws + pl.oHNew, s);
        launch_velo_head(S, A, ctx->W, ws + pl.oHNew, pl.head_batched ? ws + pl.oAlpha : nullptr,
                         pl.head_batched ? ws + pl.oTheta : nullptr, s);
      }
    };
    hipStream_t aux = ctx->aux_stream;
    // the row/column pass reads only the gradients (4 of the step's 72 bytes per element): whole list, up front
    // (VeLO: the cross-tensor term rides along in these two launches, before any group rewrites its LSTM outputs)
    launch_rowcol_sums(L, A, ctx->W, ws + pl.oHbarPart, ws + pl.oBeff, stream);
    launch_rc_update(L, A, ctx->W, ws + pl.oHbarPart, ws + pl.oBeff, stream);
    LAUNCH_TRY(hipEventRecord(ctx->ev_fork, stream));       // aux joins the caller's stream here ...
    LAUNCH_TRY(hipStreamWaitEvent(aux, ctx->ev_fork, 0));
    forked = true;
    stats_passes(sub(0), stream);
    for (int g = 0; g < G; ++g) {
      if (g + 1 < G) {
        // the next group's HBM-bound passes start when this group's are done, i.e. together with its apply pass
        LAUNCH_TRY(hipEventRecord(ctx->ev_start[g + 1], stream));
        LAUNCH_TRY(hipStreamWaitEvent(aux, ctx->ev_start[g + 1], 0));
        stats_passes(sub(g + 1), aux);
        LAUNCH_TRY(hipEventRecord(ctx->ev_pre[g + 1], aux));
      }
      launch_apply(sub(g));
      if (g + 1 < G) LAUNCH_TRY(hipStreamWaitEvent(stream, ctx->ev_pre[g + 1], 0));   // ... and is joined back here
    }
    LAUNCH_TRY(hipGetLastError());
    return LOPT_OK;
  }
  hipEvent_t* ev = nullptr;
  if (profiling) {
    const size_t need = (ctx->prof_steps + 1) * (LOPT_N_PASSES + 1);
    while (ctx->prof_events.size() < need) {
      hipEvent_t e;
      HIP_TRY(ctx, hipEventCreate(&e));   // nothing is in flight yet
      ctx->prof_events.push_back(e);
    }
    ev = ctx->prof_events.data() + ctx->prof_steps * (LOPT_N_PASSES + 1);
    ctx->prof_steps++;
  }
#define MARK(i) do { if (ev) LAUNCH_TRY(hipEventRecord(ev[i], stream)); } while (0)
  MARK(0);
  launch_rowcol_sums(L, A, ctx->W, ws + pl.oHbarPart, ws + pl.oBeff, stream);
  MARK(1);
  launch_rc_update(L, A, ctx->W, ws + pl.oHbarPart, ws + pl.oBeff, stream);
  MARK(2);
  launch_accum_stats(L, A, !state_in_apply, stream);
  MARK(3);
  launch_finalize(L, A, ctx->W, ws + pl.oLstmU, stream);
  MARK(4);
  if (ctx->cfg.kind == LOPT_VELO) {
    launch_velo_lstm(L, A, ctx->W, ws + pl.oLstmU, ws + pl.oBeff, ws + pl.oHNew, stream);
    MARK(5);
    launch_velo_head(L, A, ctx->W, ws + pl.oHNew, pl.head_batched ? ws + pl.oAlpha : nullptr,
                     pl.head_batched ? ws + pl.oTheta : nullptr, stream);
    MARK(6);
  } else {
    MARK(5);
    MARK(6);
  }
  launch_apply(L);
  MARK(7);
#undef MARK
  LAUNCH_TRY(hipGetLastError());
  return LOPT_OK;
#undef LAUNCH_TRY
}

extern "C" {

lopt_status lopt_step(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs, float* const* params,
                      const float* const* grads, void* const* state, void* workspace, int64_t step, float lr,
                      float weight_decay, void* hip_stream) {
  return step_impl(ctx, n, descs, params, grads, state, workspace, step, lr, weight_decay, hip_stream, false);
}

lopt_status lopt_step_static(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs, float* const* params,
                             const float* const* grads, void* const* state, int64_t step, float lr,
                             float weight_decay, void* hip_stream) {
  return step_impl(ctx, n, descs, params, grads, state, nullptr, step, lr, weight_decay, hip_stream, true);
}

lopt_status lopt_set_loss(lopt_ctx* ctx, float loss) {
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  if (!std::isfinite(loss)) return fail(ctx, LOPT_EINVAL, "loss must be finite");
  ctx->loss = loss;
  return LOPT_OK;
}

lopt_status lopt_profile_enable(lopt_ctx* ctx, int on) {
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  ctx->profiling = on != 0;
  return LOPT_OK;
}

lopt_status lopt_profile_read(lopt_ctx* ctx, double* ms_per_pass, uint64_t* n_steps) {
  if (!ctx) return fail(nullptr, LOPT_EINVAL, "ctx is null");
  if (!ms_per_pass) return fail(ctx, LOPT_EINVAL, "ms_per_pass is null");
  for (int i = 0; i < LOPT_N_PASSES; ++i) ms_per_pass[i] = 0.0;
  for (size_t s = 0; s < ctx->prof_steps; ++s) {
    hipEvent_t* ev = ctx->prof_events.data() + s * (LOPT_N_PASSES + 1);
    HIP_TRY(ctx, hipEventSynchronize(ev[LOPT_N_PASSES]));
    for (int i = 0; i < LOPT_N_PASSES; ++i) {
      float ms = 0.f;
      HIP_TRY(ctx, hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
      ms_per_pass[i] += (double)ms;
    }
  }
  if (n_steps) *n_steps = ctx->prof_steps;
  ctx->prof_steps = 0;
  return LOPT_OK;
}

const char* lopt_pass_name(int pass) {
  static const char* names[LOPT_N_PASSES] = {"rowcol_sums", "rc_update", "accum_stats", "finalize",
                                             "velo_lstm", "velo_head", "apply"};
  return pass >= 0 && pass < LOPT_N_PASSES ? names[pass] : nullptr;
}

const char* lopt_last_error(const lopt_ctx* ctx) {
  if (ctx) return ctx->err.c_str();
  return g_last_error.c_str();
}

}  // extern "C"
