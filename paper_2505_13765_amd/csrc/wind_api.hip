// Host side of libwind: the C ABI of include/wind.h, weight upload, workspace, the decode loop
// (replayed from a captured HIP graph), statistics and the debug entry point.
#include "../../include/wind.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <algorithm>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <exception>
#include <map>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "wind_kernels.h"
#include "wind_beam.h"

using namespace wind;

namespace {

thread_local std::string g_err;

int fail(int code, const std::string &msg) {
  g_err = msg;
  return code;
}

#define HIP_TRY(expr)                                                                         \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(WIND_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));           \
  } while (0)

using JointCfg = TileCfg<128, 128, 64, 64>;            // debug store kernel
using EncBigCfg = Ring5Cfg<256, 64, 128>;               // encoder projection of large calls: 256 x 256 tiles
using EncCfg = TileCfg<128, 128, 64, 64>;
using EncSmallCfg = TileCfg<64, 64, 32, 32>;   // calls whose 128 x 128 tiles would leave most CUs idle (same sums, same order)
using PredCfg = DmaCfg<64, 64, 32, 32, 64, 4>;   // 32 utterances (hi and lo rows) x 64 columns, 4-stage ring
constexpr int kPredMfmaMinBatch = 1;       // below this the FMA prediction network is used
constexpr size_t kEncRing5MinRows = 16384;   // B * T from which the encoder projection uses 256 x 256 tiles
constexpr int kIterRowsCap = 16384;   // iterations whose row counts profile mode records
constexpr int kRowPad = 256;  // window-row buffers are padded to a multiple of every tile height, plus one block

uint16_t host_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
float host_bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct GraphKey {
  CallDev call;
  int unroll;
  bool operator==(const GraphKey &o) const { return std::memcmp(this, &o, sizeof(GraphKey)) == 0; }
};

}  // namespace

// Scratch memory of the entry point that allocates nothing: one array per GPU, in the code object.  In
// host code the name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[WIND_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
char *g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

// The address of `scratch` on the current device, looked up once per device.
int static_scratch_address(char **out) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(WIND_ERR_UNSUPPORTED, "device ordinal above 63");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch_ptr[dev] = (char *)p;
  }
  *out = g_scratch_ptr[dev];
  return WIND_OK;
}
}  // namespace

// Beam search: state slots of the label sequences it has touched, and staging for its round trips.
struct BeamPool {
  float *h = nullptr, *c = nullptr;   // [cap][L][Hp]
  float *p = nullptr;                 // [cap][Hj]
  int cap = 0;
  float *e_all = nullptr;             // [T][Hj] every frame through the encoder projection
  size_t e_bytes = 0;
  int *d_stage = nullptr, *h_stage = nullptr;   // index lists of a large batch, device and pinned host
  void *h_res = nullptr, *d_res = nullptr;      // results of a pass: pinned host memory and its device address
};

struct wind_model {
  ModelDev dev{};
  int dtype = WIND_BF16;
  hipStream_t load_stream = nullptr;   // wind_load_weights: the stream its copies and kernels go to
  std::vector<void *> allocs;
  // workspace
  void *ws = nullptr;
  size_t ws_bytes = 0;
  CallDev call{};
  // loop replay
  hipStream_t cap_stream = nullptr;
  hipGraph_t graph[2] = {nullptr, nullptr};            // [1]: the iterations with joint_wide_kernel
  hipGraphExec_t graph_exec[2] = {nullptr, nullptr};
  GraphKey graph_key{};
  bool graph_valid = false;
  int opt_enc_wide = 1;         // large calls: encoder projection on the 256-column tile core (where the model allows)
  int opt_joint_wide = 1;       // 0: never, 1: iterations with more than wide_rows window rows, 2: always (where the model allows)
  long long prev_wide_iters = 0, last_wide_iters = 0;   // iterations of the previous / last call that had more than wide_rows window rows
  int opt_graph = 1, opt_unroll = 16;
  int opt_host_sync = 0;   // 1: kernels one by one and the host reads the active count after every iteration
  hipEvent_t ev_call[3] = {nullptr, nullptr, nullptr};   // last decode call: start, loop start, loop end
  bool have_call_times = false;
  // an asynchronous decode that wind_get_stats has not completed yet
  bool async_pending = false, async_loop = false;
  hipStream_t async_stream = nullptr;
  unsigned *async_bar = nullptr;
  int opt_pred_mfma_min_batch = kPredMfmaMinBatch;
  int opt_loop_kernel = 1;
  int opt_loop_one_xcd = 1;
  int opt_loop_fused = 1;
  long long opt_loop_spin_limit = 1ll << 21;
  int opt_debug_stamps = 0;
  int opt_lstm_rec = 1;
  int opt_atomic_lists = 1;
  int opt_slot_rows = 1;        // the iteration's prediction-network launches take their rows by slot (CallDev::slot_rows)
  int opt_decide_two = 1;       // rows of 65 .. 128 key parts: both halves of a row's keys in the decision kernel's first round trip
  bool fma_pred_step = false;   // this call's prediction-network steps keep their state in fp32 (the resident loop kernel reads it)
  LoopDev loop{};
  int *dbg_len = nullptr, *dbg_out = nullptr;   // lengths and outputs of the debug entry points (inside the workspace)
  void *beam_ws = nullptr;   // workspace of the beam scoring step
  BeamPool beam_pool{};
  int opt_beam_exact = 0;
  size_t beam_ws_bytes = 0;
  double kappa = 8.0;
  double wnorm_max = 0.0;
  int *h_flag = nullptr;  // pinned
  unsigned long long *h_stats = nullptr;   // pinned, behind h_flag in the same allocation: the call's counters
  int cu_count = 0;            // CUs of the device the model was loaded on (the resident loop kernel wants one per workgroup)
  int loop_info[2] = {0, 0};   // last decode call: workgroups of the resident loop kernel (0: not used), whether they shared one L2
  long long prev_iters = 0;
  int prev_B = 0, prev_T = 0, prev_W = 0;
  wind_stats last_stats{};
  bool have_stats = false;
  // per-kernel timing (option "profile"): event pairs recorded around each launch, read at every poll
  int opt_profile = 0;
  std::vector<hipEvent_t> ev_pool;
  std::vector<int> ev_kind;   // kind of pair i (events 2i, 2i+1)
  double prof_ms[WIND_NUM_KERNELS] = {0};
  long long prof_n[WIND_NUM_KERNELS] = {0};
  std::vector<float> joint_us;      // last profiled decode: duration of every joint launch, in launch order
  std::vector<int> joint_rows;      // and the window rows of its iteration
};

namespace {

template <class T>
int upload(wind_model *m, const std::vector<T> &host, const void **dev_out) {
  void *d = nullptr;
  HIP_TRY(hipMalloc(&d, host.size() * sizeof(T) + 256));
  m->allocs.push_back(d);
  // on the caller's stream; the host array is a temporary, so the copy is awaited here
  HIP_TRY(hipMemcpyAsync(d, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice, m->load_stream));
  HIP_TRY(hipStreamSynchronize(m->load_stream));
  *dev_out = d;
  return WIND_OK;
}

// matrix [rows, cols] fp32 -> model storage type, optionally padded with zero rows
int upload_matrix(wind_model *m, const float *src, size_t rows, size_t cols, size_t rows_pad, const void **out) {
  if (m->dtype == WIND_BF16) {
    std::vector<uint16_t> h(rows_pad * cols, 0);
    for (size_t i = 0; i < rows * cols; ++i) h[i] = host_bf16(src[i]);
    return upload(m, h, out);
  }
  std::vector<float> h(rows_pad * cols, 0.f);
  std::memcpy(h.data(), src, rows * cols * sizeof(float));
  return upload(m, h, out);
}

void set_tau(wind_model *m) {
  // bf16 rounding of the hidden vector: relative error uniform within half an ulp (2^-8), rms
  // about 1.5e-3 of the value; the difference of two screened logits then has standard deviation
  // about 2.1e-3 * |w| * |z| / sqrt(Hj) for weights that are not aligned with z.  kappa such
  // deviations make the band.
  m->dev.tau_scale = (float)(m->kappa * 2.1e-3 * m->wnorm_max / std::sqrt((double)m->dev.Hj));
}

// Where everything of a decode call lives inside the one workspace slab.
struct WsLayout {
  size_t total, Mpad, st;
  bool big_enc;
  int slot_stride, nparts, nparts_tiny;
  size_t o_e, o_encb, o_len, o_nact, o_eidx, o_eltok, o_slot, o_slotc, o_rst, o_raux, o_nemit, o_ticket, o_h, o_c, o_hn, o_hb,
      o_hz, o_rec, o_p, o_z, o_bl, o_zn, o_parts, o_rl, o_stats, o_dbg, o_iter, o_dbglen, o_dbgout, o_lbar, o_lh, o_lp, o_lparts;
};

WsLayout workspace_layout(const wind_model *m, int B, int T, int W) {
  const ModelDev &d = m->dev;
  WsLayout w{};
  w.Mpad = round_up((size_t)B * W, kRowPad) + kRowPad;   // a 192-row tile may run past the 256 multiple
  const int ntiles = (d.V + WsCfg<1>::BN - 1) / WsCfg<1>::BN;
  w.nparts = ntiles * WsCfg<1>::WAVES_N;
  w.nparts_tiny = (d.V + kTinyCols - 1) / kTinyCols;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += round_up(bytes, 256);
    return o;
  };
  w.o_e = take((size_t)B * T * d.Hj * 4);
  w.big_enc = m->dtype == WIND_BF16 && (size_t)B * T >= kEncRing5MinRows;
  w.o_encb = take(w.big_enc ? ((size_t)B * T + EncBigCfg::BM) * d.D * 2 : 0);
  w.slot_stride = B > kTinyRows ? B : kTinyRows;
  w.o_len = take((size_t)B * 4);
  w.o_nact = take(8); w.o_eidx = take((size_t)B * 4);
  w.o_eltok = take((size_t)B * 4);
  w.o_slot = take((size_t)2 * w.slot_stride * 16); w.o_slotc = take((size_t)2 * w.slot_stride * 4);
  w.o_rst = take((size_t)B * 16); w.o_raux = take((size_t)B * 16);
  w.o_nemit = take(4); w.o_ticket = take(8);
  w.st = (size_t)d.L * B * d.Hp * 4;
  w.o_h = take(w.st); w.o_c = take(w.st); w.o_hn = take(w.st);
  w.o_hb = take(2 * w.st);   // four bf16 arrays
  w.o_hz = take((size_t)(d.E > d.Hp ? d.E : d.Hp) * 2 + 256);
  w.o_rec = take((size_t)d.L * B * 4 * d.Hp * 4);
  w.o_p = take((size_t)B * d.Hj * 4);
  w.o_z = take(w.Mpad * d.Hj * 2);
  w.o_bl = take(w.Mpad * 4); w.o_zn = take(w.Mpad * 4);
  w.o_parts = take(w.Mpad * (size_t)std::max(w.nparts_tiny * 8, w.nparts * 16));   // two keys of 32 columns, or three (+ pad) of 64
  w.o_rl = take(w.Mpad * 4);
  w.o_stats = take(kNumStats * 8);
  w.o_dbg = take(128);
  w.o_iter = take((size_t)kIterRowsCap * 4);
  w.o_dbglen = take((size_t)B * 4);             // debug entry points: lengths and outputs of their own
  w.o_dbgout = take((size_t)(3 * B + 2) * 4);
  w.o_lbar = take((size_t)(1 + 256) * kLoopFlagStride * 4); w.o_lh = take((size_t)kLoopMaxB * d.Hp * 4);
  w.o_lp = take((size_t)kLoopMaxB * d.Hj * 4);
  w.o_lparts = take((size_t)2 * kLoopRows * w.nparts_tiny * 8);
  w.total = off;
  return w;
}

void carve_workspace(wind_model *m, const WsLayout &w, char *base, int B);

// The model's own workspace: allocated on first use, regrown when a call needs more.
int ensure_workspace(wind_model *m, int B, int T, int W) {
  const WsLayout w = workspace_layout(m, B, T, W);
  if (w.total > m->ws_bytes) {
    HIP_TRY(hipDeviceSynchronize());
    if (m->ws) HIP_TRY(hipFree(m->ws));
    m->ws = nullptr;
    m->ws_bytes = 0;
    m->graph_valid = false;
    HIP_TRY(hipMalloc(&m->ws, w.total));
    m->ws_bytes = w.total;
    // window-row buffers are read tile-wide: start them defined
    HIP_TRY(hipMemset(m->ws, 0, w.total));
  }
  carve_workspace(m, w, (char *)m->ws, B);
  return WIND_OK;
}

// Points the call's arrays into a workspace laid out by workspace_layout.
void carve_workspace(wind_model *m, const WsLayout &w, char *base, int B) {
  const ModelDev &d = m->dev;
  const size_t st = w.st;
  const bool big_enc = w.big_enc;
  const int slot_stride = w.slot_stride, nparts = w.nparts, nparts_tiny = w.nparts_tiny;
  const size_t o_e = w.o_e, o_encb = w.o_encb, o_len = w.o_len, o_nact = w.o_nact, o_eidx = w.o_eidx, o_eltok = w.o_eltok,
               o_slot = w.o_slot, o_slotc = w.o_slotc, o_rst = w.o_rst, o_raux = w.o_raux, o_nemit = w.o_nemit,
               o_ticket = w.o_ticket, o_h = w.o_h, o_c = w.o_c, o_hn = w.o_hn, o_hb = w.o_hb, o_hz = w.o_hz, o_p = w.o_p,
               o_z = w.o_z, o_bl = w.o_bl, o_zn = w.o_zn, o_parts = w.o_parts, o_rl = w.o_rl, o_stats = w.o_stats,
               o_dbg = w.o_dbg, o_lbar = w.o_lbar, o_lh = w.o_lh, o_lp = w.o_lp, o_lparts = w.o_lparts;
  (void)d;
  CallDev &c = m->call;
  c.Mpad = (int)w.Mpad;
  c.e = (float *)(base + o_e);
  c.enc_b = big_enc ? (bf16_t *)(base + o_encb) : nullptr;
  c.len = (int *)(base + o_len);
  c.n_active = (int *)(base + o_nact);
  c.slot_stride = slot_stride;
  c.res_state = (int4 *)(base + o_rst); c.res_aux = (int4 *)(base + o_raux);
  c.emit_idx = (int *)(base + o_eidx); c.n_emit = (int *)(base + o_nemit);
  c.emit_list_tok = (int *)(base + o_eltok);
  c.slot_state = (int4 *)(base + o_slot); c.slot_count = (int *)(base + o_slotc);
  c.ticket = (unsigned *)(base + o_ticket);
  c.h = (float *)(base + o_h); c.c = (float *)(base + o_c); c.hn = (float *)(base + o_hn);
  c.hb_hi = (bf16_t *)(base + o_hb); c.hb_lo = c.hb_hi + st / 4; c.hbn_hi = c.hb_lo + st / 4; c.hbn_lo = c.hbn_hi + st / 4;
  c.hb_zero = (const bf16_t *)(base + o_hz);
  // recurrent gate sums kept ahead of the step: where the prediction network runs on MFMA tiles and the
  // iteration is the graph of kernels with its own decision kernel
  c.rec = m->opt_lstm_rec && m->dtype == WIND_BF16 && B >= m->opt_pred_mfma_min_batch
              ? (float *)(base + w.o_rec) : nullptr;
  c.p = (float *)(base + o_p);
  c.z = (bf16_t *)(base + o_z);
  c.blank_logit = (float *)(base + o_bl); c.znorm = (float *)(base + o_zn);
  c.parts = (float *)(base + o_parts);
  c.nparts = nparts;
  c.part_width = WsCfg<1>::WN;
  c.nparts_tiny = nparts_tiny;
  c.row_label = (int *)(base + o_rl);
  c.stats = (unsigned long long *)(base + o_stats);
  c.dbg = m->opt_debug_stamps ? (long long *)(base + o_dbg) : nullptr;
  c.iter_rows = m->opt_profile ? (int *)(base + w.o_iter) : nullptr;
  c.iter_rows_cap = kIterRowsCap;
  m->dbg_len = (int *)(base + w.o_dbglen);
  m->dbg_out = (int *)(base + w.o_dbgout);
  c.lists_atomic = m->opt_atomic_lists && m->dtype == WIND_BF16;   // the path with build_z_kernel
  c.slot_rows = m->opt_slot_rows && c.lists_atomic && c.rec != nullptr && m->dev.L > 1;   // only layers above the first use it
  m->loop.bar = (unsigned *)(base + o_lbar);
  m->loop.h_x = (float *)(base + o_lh);
  m->loop.p_x = (float *)(base + o_lp);
  m->loop.parts_x = (float2 *)(base + o_lparts);
}

int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(WIND_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
  return WIND_OK;
}

// ---- per-kernel timing -------------------------------------------------------------------------
// Launches a kernel; with option "profile" the launch carries an event pair that receives the
// dispatch's own begin and end time stamps (the duration a profiler reports for the kernel).
template <class... KArgs, class... Args>
void launch(wind_model *m, hipStream_t s, int kind, bool capturing, void (*kernel)(KArgs...), dim3 grid, dim3 block,
            size_t smem, Args... args) {
  if (m->opt_profile && !capturing) {
    const size_t i = m->ev_kind.size();
    bool ok = true;
    while (ok && m->ev_pool.size() < 2 * (i + 1)) {
      hipEvent_t e = nullptr;
      ok = hipEventCreate(&e) == hipSuccess;
      if (ok) m->ev_pool.push_back(e);
    }
    if (ok) {
      m->ev_kind.push_back(kind);
      hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, s, m->ev_pool[2 * i], m->ev_pool[2 * i + 1], 0,
                            static_cast<KArgs>(args)...);
      return;
    }
  }
  hipLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, s, static_cast<KArgs>(args)...);
}

// call after the stream has been synchronised
void prof_collect(wind_model *m) {
  for (size_t i = 0; i < m->ev_kind.size(); ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, m->ev_pool[2 * i], m->ev_pool[2 * i + 1]) == hipSuccess) {
      m->prof_ms[m->ev_kind[i]] += ms;
      m->prof_n[m->ev_kind[i]] += 1;
      if (m->ev_kind[i] == WIND_K_JOINT) m->joint_us.push_back(ms * 1000.f);
    }
  }
  m->ev_kind.clear();
}

// prediction-network step for the utterances on the emit list, then their projection
int enqueue_pred_step(wind_model *m, hipStream_t s, bool capturing, bool first = false, int parity = 0) {
  const ModelDev &d = m->dev;
  const CallDev &c = m->call;
  const int lstm_blocks = (d.Hp + 3) / 4, proj_blocks = (d.Hj + 3) / 4;
  const bool mfma = m->dtype == WIND_BF16 && c.B >= m->opt_pred_mfma_min_batch && !m->fma_pred_step;
  const bool small_k = 2 * d.Hp <= 512 * kSmallKSteps;   // the low-latency kernels' K range
  constexpr int R = PredCfg::BM / 2;
  const unsigned mtiles = (unsigned)((c.B + R - 1) / R);
  if (mfma && c.rec) {
    // the first layer's step was taken by the decision kernel (first step of a call: by the full
    // kernels below, from the zero state); the layers above add their input half to the recurrent
    // sums; the projection launch also renews those sums for the utterances that emitted
    const unsigned rec_tiles = (unsigned)(d.L * (4 * d.Hp / PredCfg::BN)), proj_tiles = (unsigned)(d.Hj / PredCfg::BN);
    if (first) {
      CallDev c0 = c;
      c0.rec = nullptr;
      for (int l = 0; l < d.L; ++l)
        launch(m, s, WIND_K_LSTM, capturing, lstm_layer_dma_kernel<PredCfg>, dim3((unsigned)(4 * d.Hp / PredCfg::BN), mtiles),
               dim3(PredCfg::NT), PredCfg::SMEM_BYTES, d, c0, l, 0, 0);
      launch(m, s, WIND_K_PRED_PROJ, capturing, pred_proj_dma_kernel<PredCfg>, dim3(proj_tiles, mtiles), dim3(PredCfg::NT),
             PredCfg::SMEM_BYTES, d, c0, 0, (int)proj_tiles);
      launch(m, s, WIND_K_LSTM, capturing, pred_proj_dma_kernel<PredCfg>, dim3(rec_tiles, mtiles), dim3(PredCfg::NT),
             PredCfg::SMEM_BYTES, d, c, 1, 0);
    } else {
      // the layers above the first take their rows by slot (asked for at once) or through the emit list; the
      // projection launch always goes through the list (by slot it was slower: 6.6 -> 7.0 us on the B = 128 workload)
      for (int l = 1; l < d.L; ++l)
        launch(m, s, WIND_K_LSTM, capturing, lstm_layer_dma_kernel<PredCfg>, dim3((unsigned)(4 * d.Hp / PredCfg::BN), mtiles),
               dim3(PredCfg::NT), PredCfg::SMEM_BYTES, d, c, l, c.slot_rows ? 2 : 1, parity);
      launch(m, s, WIND_K_PRED_PROJ, capturing, pred_proj_dma_kernel<PredCfg>, dim3(proj_tiles + rec_tiles, mtiles),
             dim3(PredCfg::NT), PredCfg::SMEM_BYTES, d, c, 1, (int)proj_tiles);
    }
    return check_launch("prediction step");
  }
  for (int l = 0; l < d.L; ++l) {
    if (mfma)
      launch(m, s, WIND_K_LSTM, capturing, lstm_layer_dma_kernel<PredCfg>, dim3((unsigned)(4 * d.Hp / PredCfg::BN), mtiles),
             dim3(PredCfg::NT), PredCfg::SMEM_BYTES, d, c, l, 0, 0);
    else if (m->dtype == WIND_BF16 && small_k)
      launch(m, s, WIND_K_LSTM, capturing, lstm_small_kernel<2>, dim3(lstm_blocks), dim3(256), 0, d, c, l);
    else if (m->dtype == WIND_BF16)
      launch(m, s, WIND_K_LSTM, capturing, lstm_layer_kernel<bf16_t, 4>, dim3(lstm_blocks), dim3(256), 0, d, c, l);
    else
      launch(m, s, WIND_K_LSTM, capturing, lstm_layer_kernel<float, 4>, dim3(lstm_blocks), dim3(256), 0, d, c, l);
  }
  if (mfma)
    launch(m, s, WIND_K_PRED_PROJ, capturing, pred_proj_dma_kernel<PredCfg>, dim3((unsigned)(d.Hj / PredCfg::BN), mtiles),
           dim3(PredCfg::NT), PredCfg::SMEM_BYTES, d, c, 0, d.Hj / PredCfg::BN);
  else if (m->dtype == WIND_BF16 && small_k)
    launch(m, s, WIND_K_PRED_PROJ, capturing, pred_small_kernel<2>, dim3(proj_blocks), dim3(256), 0, d, c);
  else if (m->dtype == WIND_BF16)
    launch(m, s, WIND_K_PRED_PROJ, capturing, pred_proj_kernel<bf16_t, 4>, dim3(proj_blocks), dim3(256), 0, d, c);
  else
    launch(m, s, WIND_K_PRED_PROJ, capturing, pred_proj_kernel<float, 4>, dim3(proj_blocks), dim3(256), 0, d, c);
  return check_launch("prediction step");
}

// Large calls of bf16 models whose input size the 256-column tile core takes (ten K stages of 32 at least, buffer
// descriptors with 32-bit sizes) run the encoder projection on it (option enc_wide).
bool enc_wide_ok(const wind_model *m, int B, int T) {
  const ModelDev &d = m->dev;
  if (!m->opt_enc_wide || !d.w_enc_slab || d.D < kWideMinK || d.D % 32) return false;
  return ((unsigned long long)B * T + 256) * d.D * 2 < (1ull << 32);
}

int enqueue_prologue(wind_model *m, hipStream_t s) {
  const ModelDev &d = m->dev;
  const CallDev &c = m->call;
  {
    const size_t nstate = (size_t)d.L * c.B * d.Hp;
    init_state_kernel<<<(unsigned)std::min<size_t>(64, (nstate + 4095) / 4096 + 1), 256, 0, s>>>(d, c);
  }
  if (c.T > 0) {
    if (m->dtype == WIND_BF16 && c.enc_b) {
      const long long rows = (long long)c.B * c.T;
      const bool wide = enc_wide_ok(m, c.B, c.T);
      launch(m, s, WIND_K_ENC_PROJ, false, enc_round_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, d, c, wide ? 1 : 0);
      if (wide) {
        const int tiles_per_utt = (c.T + 255) / 256, n_row_tiles = c.B * tiles_per_utt, n_col_tiles = (d.Hj + 255) / 256;
        launch(m, s, WIND_K_ENC_PROJ, false, enc_proj_wide_kernel, dim3((unsigned)((n_row_tiles + 7) / 8 * 8 * n_col_tiles)), dim3(256),
               kWideSmemBytes, d, c, tiles_per_utt, n_row_tiles, n_col_tiles);
      } else {
        const int tiles_per_utt = (c.T + EncBigCfg::BM - 1) / EncBigCfg::BM;
        dim3 grid((unsigned)(c.B * tiles_per_utt), (unsigned)((d.Hj + EncBigCfg::BN - 1) / EncBigCfg::BN));
        launch(m, s, WIND_K_ENC_PROJ, false, enc_proj_ring5_kernel<EncBigCfg>, grid, dim3(EncBigCfg::NT),
               EncBigCfg::SMEM_BYTES, d, c, tiles_per_utt);
      }
    } else if (m->dtype == WIND_BF16) {
      const int tiles_per_utt = (c.T + EncCfg::BM - 1) / EncCfg::BM;
      dim3 grid((unsigned)(c.B * tiles_per_utt), (unsigned)((d.Hj + EncCfg::BN - 1) / EncCfg::BN));
      if (grid.x * grid.y < 128) {   // a single short utterance: a quarter of the tile on four times the workgroups
        const int small_per_utt = (c.T + EncSmallCfg::BM - 1) / EncSmallCfg::BM;
        dim3 sgrid((unsigned)(c.B * small_per_utt), (unsigned)((d.Hj + EncSmallCfg::BN - 1) / EncSmallCfg::BN));
        launch(m, s, WIND_K_ENC_PROJ, false, enc_proj_mfma_kernel<EncSmallCfg>, sgrid, dim3(EncSmallCfg::NT), EncSmallCfg::SMEM_BYTES,
               d, c, small_per_utt);
      } else {
        launch(m, s, WIND_K_ENC_PROJ, false, enc_proj_mfma_kernel<EncCfg>, grid, dim3(EncCfg::NT), EncCfg::SMEM_BYTES, d, c,
               tiles_per_utt);
      }
    } else {
      launch(m, s, WIND_K_ENC_PROJ, false, enc_proj_f32_kernel, dim3((unsigned)c.T, (unsigned)c.B), dim3(256),
             (size_t)d.D * 4, d, c);
    }
  }
  int rc = check_launch("prologue");
  if (rc) return rc;
  return enqueue_pred_step(m, s, false, true);
}

// The joint kernel on 256-column tiles (joint_wide_kernel) pays off from 192-row tiles on: with `wfill` row
// tiles filling the chip, for iterations with more than 128 wfill window rows.  Returns that threshold (0 with
// option joint_wide = 2: every iteration), or -1 if the model or the call never runs the kernel.
int wide_threshold_rows(const wind_model *m, int B, int W) {
  const ModelDev &d = m->dev;
  if (m->dtype != WIND_BF16 || !d.w_out_slab || m->opt_joint_wide == 0) return -1;
  const int NT = (d.V + WideCfg<1>::BN - 1) / WideCfg<1>::BN, wfill = NT >= 256 ? 1 : 256 / NT;
  const int thr = m->opt_joint_wide == 2 ? 0 : 128 * wfill;
  const unsigned long long z_bytes = (round_up((size_t)B * W, kRowPad) + kRowPad) * (unsigned long long)d.Hj * 2;
  if (z_bytes >= (1ull << 32)) return -1;   // the kernel's buffer descriptors take 32-bit sizes
  return (long long)B * W > thr ? thr : -1;
}

// the output contraction with its row argmax folded in, for the window rows build_z_kernel wrote
// (wide: in slab layout, for joint_wide_kernel)
void enqueue_joint(wind_model *m, hipStream_t s, int parity, bool capturing, bool wide) {
  const ModelDev &d = m->dev;
  const CallDev &c = m->call;
  if (wide) {
    const int NT = (d.V + WideCfg<1>::BN - 1) / WideCfg<1>::BN, fill = NT >= 256 ? 1 : 256 / NT;
    launch(m, s, WIND_K_JOINT, capturing, joint_wide_kernel, dim3((unsigned)((fill * NT + 7) / 8 * 8)), dim3(WideCfg<1>::NT),
           kWideSmemBytes, d, c, parity, fill, NT);
    return;
  }
  // fill x NT workgroups, each walking as many row tiles as the iteration's row count needs
  const int NT = (d.V + WsCfg<1>::BN - 1) / WsCfg<1>::BN, fill = NT >= 256 ? 1 : 256 / NT;
  launch(m, s, WIND_K_JOINT, capturing, joint_ws_kernel, dim3((unsigned)((fill * NT + 7) / 8 * 8)), dim3(WsCfg<1>::NT),
         kWsSmemBytes, d, c, parity, fill, NT);
}

int enqueue_iteration(wind_model *m, hipStream_t s, int parity, bool capturing, bool wide) {
  const ModelDev &d = m->dev;
  const CallDev &c = m->call;
  const int max_rows = c.B * c.W;
  const int decide_threads = 64 * (c.W < 16 ? c.W : 16);
  if (m->dtype == WIND_BF16) {
    launch(m, s, WIND_K_BUILD_Z, capturing, build_z_kernel, dim3((unsigned)((max_rows + 3) / 4)), dim3(256), 0, d, c, parity,
           wide ? 1 : 0, wide_threshold_rows(m, c.B, c.W));
    enqueue_joint(m, s, parity, capturing, wide);
    if (d.Hj <= 1024 && c.nparts > 64 && c.nparts <= 128 && c.W <= 16 && m->opt_decide_two)   // one row per wave, two key loads per lane
      launch(m, s, WIND_K_DECIDE, capturing, decide_kernel<bf16_t, false, true>, dim3((unsigned)c.B), dim3(decide_threads), 0, d, c, parity, 0);
    else if (d.Hj <= 1024)
      launch(m, s, WIND_K_DECIDE, capturing, decide_kernel<bf16_t, false>, dim3((unsigned)c.B), dim3(decide_threads), 0, d, c, parity, 0);
    else
      launch(m, s, WIND_K_DECIDE, capturing, decide_kernel<bf16_t, true>, dim3((unsigned)c.B), dim3(decide_threads), 0, d, c, parity, 0);
  } else {
    launch(m, s, WIND_K_JOINT, capturing, joint_exact_kernel<float>, dim3((unsigned)max_rows), dim3(256), (size_t)d.Hj * 4,
           d, c, parity, 1, 0, 0, 0, (const float *)nullptr, 0, (float *)nullptr, (bf16_t *)nullptr);
    launch(m, s, WIND_K_DECIDE, capturing, decide_kernel<float, false>, dim3((unsigned)c.B), dim3(decide_threads), 0, d, c, parity, 1);
  }
  int rc = check_launch("iteration");
  if (rc) return rc;
  return enqueue_pred_step(m, s, capturing, false, parity);
}

// The loop's graphs: `unroll` iterations with joint_ws_kernel, and, where the call can have iterations
// for joint_wide_kernel, the same with that kernel (either graph is right for any row count).
int ensure_graph(wind_model *m) {
  GraphKey key{};
  key.call = m->call;
  key.unroll = m->opt_unroll;
  if (m->graph_valid && key == m->graph_key) return WIND_OK;
  for (int g = 0; g < 2; ++g) {
    if (m->graph_exec[g]) { (void)hipGraphExecDestroy(m->graph_exec[g]); m->graph_exec[g] = nullptr; }
    if (m->graph[g]) { (void)hipGraphDestroy(m->graph[g]); m->graph[g] = nullptr; }
  }
  m->graph_valid = false;
  if (!m->cap_stream) HIP_TRY(hipStreamCreateWithFlags(&m->cap_stream, hipStreamNonBlocking));
  const int wide_rows = wide_threshold_rows(m, m->call.B, m->call.W);
  const bool want[2] = {wide_rows != 0, wide_rows >= 0};
  for (int w = 0; w < 2; ++w) {
    if (!want[w]) continue;
    HIP_TRY(hipStreamBeginCapture(m->cap_stream, hipStreamCaptureModeThreadLocal));
    int rc = WIND_OK;
    for (int it = 0; it < m->opt_unroll && rc == WIND_OK; ++it) rc = enqueue_iteration(m, m->cap_stream, it & 1, true, w == 1);
    hipGraph_t g = nullptr;
    hipError_t e = hipStreamEndCapture(m->cap_stream, &g);
    if (rc != WIND_OK) { if (g) (void)hipGraphDestroy(g); return rc; }
    if (e != hipSuccess) return fail(WIND_ERR_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
    m->graph[w] = g;
    HIP_TRY(hipGraphInstantiate(&m->graph_exec[w], m->graph[w], nullptr, nullptr, 0));
  }
  m->graph_key = key;
  m->graph_valid = true;
  return WIND_OK;
}

// The call's counters on their way to pinned memory (h_stats); read_stats takes them from there once
// the stream has passed the copy.
int enqueue_stats_copy(wind_model *m, hipStream_t s) {
  HIP_TRY(hipMemcpyAsync(m->h_stats, m->call.stats, kNumStats * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
  return WIND_OK;
}

int read_stats(wind_model *m) {
  const unsigned long long *h = m->h_stats;
  wind_stats &st = m->last_stats;
  std::memset(&st, 0, sizeof(st));
  st.iterations = (int64_t)h[ST_ITER];
  st.windows = (int64_t)h[ST_WINDOWS];
  st.rows = (int64_t)h[ST_ROWS];
  st.useful_rows = (int64_t)h[ST_USEFUL];
  st.labels = (int64_t)h[ST_LABELS];
  st.forced_advances = (int64_t)h[ST_FORCED];
  st.rechecks = (int64_t)h[ST_RECHECK];
  m->last_wide_iters = (long long)h[ST_WIDE];
  for (int i = 0; i <= WIND_MAX_WINDOW; ++i) st.jump_hist[i] = (int64_t)h[kStatJump0 + i];
  m->have_stats = true;
  if (m->call.dbg) {
    long long d[16];
    if (hipMemcpy(d, m->call.dbg, sizeof(d), hipMemcpyDeviceToHost) == hipSuccess && d[10] > 0)
      std::fprintf(stderr, "[wind debug] resident loop, workgroup 0, avg us per iteration: gather %.2f  mfma+keys %.2f  barrier1 %.2f  decide %.2f | per emitting iteration: lstm %.2f  barrier2 %.2f  hcopy+pred %.2f  barrier3 %.2f  pcopy %.2f  (%lld iterations, %lld emitting)\n",
                   d[0] / 100.0 / d[10], d[1] / 100.0 / d[10], d[2] / 100.0 / d[10], d[3] / 100.0 / d[10], d[4] / 100.0 / (d[11] ? d[11] : 1),
                   d[5] / 100.0 / (d[11] ? d[11] : 1), d[6] / 100.0 / (d[11] ? d[11] : 1), d[7] / 100.0 / (d[11] ? d[11] : 1), d[8] / 100.0 / (d[11] ? d[11] : 1), d[10], d[11]);
    else if (d[3] > 0 && d[10] == 0 && d[8] == 0)
      std::fprintf(stderr, "[wind debug] decide kernel, last workgroup avg us: rows %.2f  ticket %.2f  compaction %.2f (%lld launches); rows phase of workgroups with a near-tie %.2f (%lld), without %.2f (%lld)\n",
                   d[0] / 100.0 / d[3], d[1] / 100.0 / d[3], d[2] / 100.0 / d[3], d[3], d[4] / 100.0 / (d[5] ? d[5] : 1), d[5],
                   d[6] / 100.0 / (d[7] ? d[7] : 1), d[7]);
    (void)hipMemset(m->call.dbg, 0, 128);
  }
  return h[ST_OVERFLOW] ? WIND_ERR_OVERFLOW : WIND_OK;
}

int fetch_stats(wind_model *m, hipStream_t s) {
  int rc = enqueue_stats_copy(m, s);
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(s));
  return read_stats(m);
}

// Shape of the resident loop kernel for this call, or false if the call does not qualify: bf16, one
// LSTM layer, at most 2 utterances and 32 window rows, every workgroup's weight slice within LDS,
// at most one workgroup per CU.  First choice: at most 32 workgroups, which fit the CUs of one XCD
// and then exchange through its L2 (window rows limited to 16 so that the larger weight slices
// still fit LDS); otherwise 16 units per workgroup, spread over the chip.
bool loop_kernel_shape(const wind_model *m, int B, int T, int W, LoopDev *lp, size_t *smem) {
  const ModelDev &d = m->dev;
  // the kernel indexes the projected frames, the label table and the exchange buffers with 32 bits
  if ((unsigned long long)B * (unsigned long long)T * d.Hj >= (1ull << 31) || (unsigned long long)(d.V + 1) * 4 * d.Hp >= (1ull << 31)) return false;
  if (m->dtype != WIND_BF16 || d.L != 1 || B > kLoopMaxB || B * W > kLoopRows || d.Hj > kTinyMaxHj) return false;
  if (!m->opt_loop_kernel || m->opt_profile || !m->opt_graph || m->opt_host_sync) return false;
  const int nparts_tiny = (d.V + kTinyCols - 1) / kTinyCols;
  if (nparts_tiny * 8 > (d.Hj + 8) * 2) return false;              // a row's keys fit where its hidden vector was
  if (d.Hp % 64 || d.Hj % 64) return false;                        // K of every matrix-core product splits over four waves in steps of 16
  const int widest = d.Hp > d.Hj ? d.Hp : d.Hj;
  // at most 16 window rows and a joint width in steps of 128: the rows go straight into matrix-core operands
  const bool fused = m->opt_loop_fused && B * W <= 16 && d.Hj % 128 == 0 && d.Hj <= 128 * kFusedSteps;
  for (int near = m->opt_loop_one_xcd ? 1 : 0; near >= 0; --near) {
    if (near && m->cu_count < 8 * kLoopNearG) continue;   // eight XCDs of at least 32 CUs each
    int G = near ? kLoopNearG : (widest + 15) / 16;
    if (G < nparts_tiny) { if (near) continue; G = nparts_tiny; }
    if (G > 256 || G > m->cu_count) return false;
    lp->G = G;
    lp->step = near ? 8 : 1;
    lp->zrows = fused ? 0 : near && B * W <= 16 ? 16 : kLoopRows;
    lp->upw = ((d.Hp + G - 1) / G + 3) / 4 * 4;
    lp->ppw = ((d.Hj + G - 1) / G + 3) / 4 * 4;
    *smem = loop_smem_bytes(d.Hp, d.Hj, B, lp->upw, lp->ppw, lp->zrows);
    if (lp->upw * 4 + lp->ppw > kLoopProdRows) continue;             // gate rows and projection rows go through the matrix cores in one pass
    if (*smem + 6144 <= 160 * 1024 && *smem <= kLoopMaxSmem) return true;   // room for the kernel's static LDS
  }
  return false;
}

// One decode call.  ext_ws null: the model's own workspace, and the call returns when the decode has
// finished.  ext_ws given: the caller's workspace, at most max_iters loop iterations are enqueued and
// the call returns at once; wind_get_stats completes it (finish_async).
int decode(wind_model *m, const float *enc, const int32_t *lengths, int B, int T, int W, int S,
           int32_t *out_tokens, int32_t *out_frames, int32_t *out_counts, int cap, void *stream,
           void *ext_ws = nullptr, size_t ext_bytes = 0, long long async_iters = 0) {
  if (!m) return fail(WIND_ERR_ARG, "model is null");
  if (m->async_pending) return fail(WIND_ERR_ARG, "an asynchronous decode is pending on this model: call wind_get_stats first");
  if (!lengths || !out_tokens || !out_frames || !out_counts) return fail(WIND_ERR_ARG, "null pointer argument");
  if (B < 1 || T < 0 || cap < 1) return fail(WIND_ERR_ARG, "B >= 1, T >= 0, cap >= 1 required");
  if (T > 0 && !enc) return fail(WIND_ERR_ARG, "enc_out is null");
  if (W < 1 || W > WIND_MAX_WINDOW) return fail(WIND_ERR_ARG, "W must be in 1..64");
  if (S < 1) return fail(WIND_ERR_ARG, "max_symbols_per_step must be >= 1");
  if ((long long)B * T > (1ll << 31) - 1) return fail(WIND_ERR_ARG, "B*T too large");
  if (m->dtype == WIND_BF16 && m->dev.Hj > kDecideMaxHj) return fail(WIND_ERR_UNSUPPORTED, "Hj > 2048");
  hipStream_t s = (hipStream_t)stream;
  const bool async = ext_ws != nullptr;
  int rc = WIND_OK;
  if (async) {
    const WsLayout w = workspace_layout(m, B, T, W);
    if (ext_bytes < w.total)
      return fail(WIND_ERR_ARG, "workspace of " + std::to_string(ext_bytes) + " bytes, this shape needs " + std::to_string(w.total));
    if ((uintptr_t)ext_ws % 256) return fail(WIND_ERR_ARG, "workspace must be 256-byte aligned");
    if (async_iters < 1) return fail(WIND_ERR_ARG, "max_iterations must be >= 1");
    carve_workspace(m, w, (char *)ext_ws, B);
    // the caller's memory may hold anything: the window rows are fetched tile-wide, so they start defined
    const size_t zi = w.Mpad * (size_t)m->dev.Hj / 2;
    fill_int_kernel<<<(unsigned)std::min<size_t>((zi + 255) / 256, 2048), 256, 0, s>>>((int *)m->call.z, (int)zi, 0);
  } else {
    rc = ensure_workspace(m, B, T, W);
    if (rc) return rc;
  }
  CallDev &c = m->call;
  c.B = B; c.T = T; c.W = W; c.S = S; c.cap = cap;
  c.enc = enc; c.lengths = lengths;
  c.out_tokens = out_tokens; c.out_frames = out_frames; c.out_counts = out_counts;

  LoopDev lp = m->loop;
  size_t loop_smem = 0;
  const bool use_loop = loop_kernel_shape(m, B, T, W, &lp, &loop_smem);
  const long long max_iters = (long long)T * ((long long)S + 1) + 2;   // every iteration moves some pointer or emits
  m->loop_info[0] = m->loop_info[1] = 0;
  m->fma_pred_step = use_loop;   // the resident kernel starts from the fp32 state of the start-token step
  if (use_loop) { c.rec = nullptr; c.lists_atomic = 0; c.slot_rows = 0; }
  m->have_call_times = false;
  HIP_TRY(hipEventRecord(m->ev_call[0], s));
  rc = enqueue_prologue(m, s);
  if (rc) return rc;
  HIP_TRY(hipEventRecord(m->ev_call[1], s));   // the loop starts here: state set up, every frame projected
  if (use_loop) {
    // the whole loop as one resident kernel
    lp.max_iters = (int)std::min<long long>(async ? std::min(async_iters, max_iters) : max_iters, 1 << 30);
    lp.spin_limit = (unsigned)m->opt_loop_spin_limit;
    {
      const int bar_ints = (1 + lp.G) * kLoopFlagStride;
      // the key exchange starts out as "two iterations old": all tag bits set, the first iterations' tag is 0
      const int key_ints = 2 * kLoopRows * ((m->dev.V + kTinyCols - 1) / kTinyCols) * 2;
      loop_prepare_kernel<<<(unsigned)((bar_ints + key_ints + 255) / 256), 256, 0, s>>>((int *)lp.bar, bar_ints, (int *)lp.parts_x, key_ints);
    }
    {
      const dim3 grid((unsigned)(lp.G * lp.step));
      switch (lp.zrows == 0 ? m->dev.Hj / 128 : 0) {   // fused form: one instance per number of K steps
        case 0: wind_loop_kernel<0><<<grid, 256, loop_smem, s>>>(m->dev, c, lp); break;
        case 1: wind_loop_kernel<1><<<grid, 256, loop_smem, s>>>(m->dev, c, lp); break;
        case 2: wind_loop_kernel<2><<<grid, 256, loop_smem, s>>>(m->dev, c, lp); break;
        case 3: wind_loop_kernel<3><<<grid, 256, loop_smem, s>>>(m->dev, c, lp); break;
        case 4: wind_loop_kernel<4><<<grid, 256, loop_smem, s>>>(m->dev, c, lp); break;
        case 5: wind_loop_kernel<5><<<grid, 256, loop_smem, s>>>(m->dev, c, lp); break;
        default: return fail(WIND_ERR_UNSUPPORTED, "resident loop: no fused instance for this joint width");
      }
    }
    rc = check_launch("resident loop");
    if (rc) return rc;
    HIP_TRY(hipEventRecord(m->ev_call[2], s));
    if (async) {
      m->async_pending = true; m->async_loop = true; m->async_stream = s; m->async_bar = lp.bar;
      m->loop_info[0] = lp.G; m->loop_info[1] = 0;
      return WIND_OK;
    }
    static_assert(kNumStats <= 128, "loop_collect_kernel: one thread per counter");
    loop_collect_kernel<<<1, 128, 0, s>>>(c.n_active, lp.bar, c.stats, kNumStats, m->h_flag, m->h_stats);   // one launch, one wait
    rc = check_launch("resident loop results");
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(s));
    m->loop_info[0] = lp.G; m->loop_info[1] = m->h_flag[2] == 2;
    if (m->h_flag[1] != 0) return fail(WIND_ERR_HIP, "resident loop: a grid barrier timed out (workgroups not all resident?)");
    if (m->h_flag[0] != 0) return fail(WIND_ERR_HIP, "decode loop did not terminate");
    m->have_call_times = true;
    rc = read_stats(m);
    if (rc == WIND_ERR_OVERFLOW) return fail(rc, "an utterance produced more labels than cap");
    return rc;
  }
  const int U = m->opt_unroll;
  const bool use_graph = m->opt_graph && !m->opt_profile && !m->opt_host_sync;   // events cannot sit between graph nodes
  // Which joint kernel the iterations of a block of U run (either is right for any row count; the choice is
  // about speed): joint_wide_kernel while the call has more than wide_rows window rows per iteration.  The
  // row count only falls during a call, so from a count read back, active utterances x W; for blocks enqueued
  // ahead of any count, from how many such iterations the previous call of the same shape had.
  const int wide_rows = wide_threshold_rows(m, B, W);
  const bool same_shape = m->prev_B == B && m->prev_T == T && m->prev_W == W && m->prev_iters > 0;
  auto wide_by_count = [&](long long active) { return wide_rows >= 0 && active * W > wide_rows; };
  auto wide_by_history = [&](long long block) {
    if (wide_rows < 0) return false;
    if (wide_rows == 0) return true;
    return same_shape ? block * U + U / 2 < m->prev_wide_iters : block == 0 && wide_by_count(B);
  };
  m->joint_us.clear();
  m->joint_rows.clear();
  if (use_graph) {
    rc = ensure_graph(m);
    if (rc) return rc;
  }
  if (async) {
    // no polling: the iterations the caller allows, in whole replays; kernels of iterations past the
    // end of the decode find no active utterance and leave at once
    if (!use_graph) return fail(WIND_ERR_UNSUPPORTED, "the asynchronous decode needs graph replay (options graph, profile, host_sync)");
    const long long replays = (std::min(async_iters, max_iters) + U - 1) / U;
    for (long long i = 0; i < replays; ++i) HIP_TRY(hipGraphLaunch(m->graph_exec[wide_by_history(i) ? 1 : 0], s));
    HIP_TRY(hipEventRecord(m->ev_call[2], s));
    m->async_pending = true; m->async_loop = false; m->async_stream = s;
    return WIND_OK;
  }
  if (m->opt_host_sync) {
    // The loop as a framework runs it without graphs (Analysis, "Incorporation with CUDA-graphs", the
    // rows without graph of Table 5): the kernels of one iteration, then the host waits for them and
    // reads how many utterances are still active before it launches the next iteration.
    for (long long it = 0;; ++it) {
      const int parity = (int)(it & 1);
      rc = enqueue_iteration(m, s, parity, false, wide_by_count(it == 0 ? B : *m->h_flag));
      if (rc) return rc;
      HIP_TRY(hipEventRecord(m->ev_call[2], s));
      HIP_TRY(hipMemcpyAsync(m->h_flag, c.n_active + (parity ^ 1), sizeof(int), hipMemcpyDeviceToHost, s));
      HIP_TRY(hipStreamSynchronize(s));
      prof_collect(m);
      if (*m->h_flag == 0) break;
      if (it > max_iters) return fail(WIND_ERR_HIP, "decode loop did not terminate");
    }
  } else {
    // Launch ahead by what the previous call of the same shape needed, then poll once per replay.
    long long ahead = 1;
    if (m->prev_B == B && m->prev_T == T && m->prev_W == W && m->prev_iters > 0) ahead = m->prev_iters / U;
    if (ahead < 1) ahead = 1;
    const long long max_launches = (max_iters + 2 * U) / U + 2;
    long long launches = 0;
    bool polled = false;
    for (;;) {
      for (long long i = 0; i < ahead; ++i, ++launches) {
        const bool wide = polled ? wide_by_count(*m->h_flag) : wide_by_history(launches);
        if (use_graph) {
          HIP_TRY(hipGraphLaunch(m->graph_exec[wide ? 1 : 0], s));
        } else {
          for (int it = 0; it < U; ++it) {
            rc = enqueue_iteration(m, s, it & 1, false, wide);
            if (rc) return rc;
          }
        }
      }
      ahead = 1;
      polled = true;
      HIP_TRY(hipEventRecord(m->ev_call[2], s));
      HIP_TRY(hipMemcpyAsync(m->h_flag, c.n_active, sizeof(int), hipMemcpyDeviceToHost, s));
      rc = enqueue_stats_copy(m, s);   // final once the count is zero: the last poll needs no second wait
      if (rc) return rc;
      HIP_TRY(hipStreamSynchronize(s));
      prof_collect(m);
      if (*m->h_flag == 0) break;
      if (launches > max_launches) return fail(WIND_ERR_HIP, "decode loop did not terminate");
    }
  }
  m->have_call_times = true;
  rc = m->opt_host_sync ? fetch_stats(m, s) : read_stats(m);
  if (c.iter_rows && (rc == WIND_OK || rc == WIND_ERR_OVERFLOW)) {
    const size_t n = (size_t)std::min<long long>(m->last_stats.iterations, kIterRowsCap);
    m->joint_rows.resize(n);
    if (n) HIP_TRY(hipMemcpy(m->joint_rows.data(), c.iter_rows, n * sizeof(int), hipMemcpyDeviceToHost));
  }
  m->prev_B = B; m->prev_T = T; m->prev_W = W;
  m->prev_iters = m->last_stats.iterations;
  m->prev_wide_iters = m->last_wide_iters;
  if (rc == WIND_ERR_OVERFLOW) return fail(rc, "an utterance produced more labels than cap");
  return rc;
}

}  // namespace

#include "wind_beam_search.h"

extern "C" {

const char *wind_last_error(void) { return g_err.c_str(); }

// The host-side conversion of the weights uses standard containers; nothing they throw may cross the C boundary.
int wind_load_weights(const wind_weights *w, void *stream, wind_model **out) try {
  if (!w || !out) return fail(WIND_ERR_ARG, "null argument");
  *out = nullptr;
  if (w->L < 1 || w->L > WIND_MAX_LAYERS) return fail(WIND_ERR_ARG, "L must be in 1..4");
  if (w->D < 1 || w->E < 1 || w->Hp < 1 || w->Hj < 1 || w->V < 1) return fail(WIND_ERR_ARG, "sizes must be >= 1");
  if (w->dtype != WIND_F32 && w->dtype != WIND_BF16) return fail(WIND_ERR_ARG, "unknown dtype");
  if (!w->emb || !w->w_enc || !w->b_enc || !w->w_pred || !w->b_pred || !w->w_out || !w->b_out)
    return fail(WIND_ERR_ARG, "null weight pointer");
  for (int l = 0; l < w->L; ++l)
    if (!w->w_ih[l] || !w->w_hh[l] || !w->b_ih[l] || !w->b_hh[l]) return fail(WIND_ERR_ARG, "null LSTM weight pointer");
  if (w->dtype == WIND_BF16 && (w->D % 64 || w->E % 64 || w->Hp % 64 || w->Hj % 64))
    return fail(WIND_ERR_UNSUPPORTED, "bf16 models need D, E, Hp, Hj to be multiples of 64");
  if ((long long)(w->V + 1) * w->Hj > (1ll << 31) - 1) return fail(WIND_ERR_UNSUPPORTED, "(V+1)*Hj too large");

  wind_model *m = new wind_model();
  m->dtype = w->dtype;
  m->load_stream = (hipStream_t)stream;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
      m->cu_count = cus;
  }
  ModelDev &d = m->dev;
  d.D = w->D; d.E = w->E; d.Hp = w->Hp; d.L = w->L; d.Hj = w->Hj; d.V = w->V;
  d.Vpad = (int)round_up((size_t)w->V + 1, 256);
  int rc = WIND_OK;
  auto chk = [&](int r) { if (rc == WIND_OK) rc = r; };
  const int Hp = w->Hp;
  chk(upload_matrix(m, w->emb, (size_t)w->V + 1, w->E, (size_t)w->V + 1, &d.emb));
  for (int l = 0; l < w->L && rc == WIND_OK; ++l) {
    // layer 0 keeps only its recurrent half here; its input half becomes the emb_gates table below
    const int in = l == 0 ? 0 : Hp, K = in + Hp;
    std::vector<float> cat((size_t)4 * Hp * K), bias((size_t)4 * Hp);
    for (int g = 0; g < 4; ++g)
      for (int j = 0; j < Hp; ++j) {
        const size_t src = (size_t)g * Hp + j, dst = (size_t)j * 4 + g;
        if (in) std::memcpy(&cat[dst * K], w->w_ih[l] + src * in, sizeof(float) * in);
        std::memcpy(&cat[dst * K + in], w->w_hh[l] + src * Hp, sizeof(float) * Hp);
        bias[dst] = w->b_ih[l][src] + w->b_hh[l][src];
      }
    chk(upload_matrix(m, cat.data(), (size_t)4 * Hp, K, (size_t)4 * Hp, &d.w_cat[l]));
    const void *bp = nullptr;
    chk(upload(m, bias, &bp));
    d.b_cat[l] = (const float *)bp;
    if (l == 0 && rc == WIND_OK) {
      // emb_gates[v][4j+g] = b_ih + b_hh + w_ih[gate g of unit j] . emb[v], in the model's storage precision
      std::vector<float> ih((size_t)4 * Hp * w->E);
      for (int g = 0; g < 4; ++g)
        for (int j = 0; j < Hp; ++j)
          std::memcpy(&ih[((size_t)j * 4 + g) * w->E], w->w_ih[0] + ((size_t)g * Hp + j) * w->E, sizeof(float) * w->E);
      const void *d_ih = nullptr;
      chk(upload_matrix(m, ih.data(), (size_t)4 * Hp, w->E, (size_t)4 * Hp, &d_ih));
      void *table = nullptr;
      if (rc == WIND_OK) {
        hipError_t e = hipMalloc(&table, (size_t)(w->V + 1) * 4 * Hp * sizeof(float));
        if (e != hipSuccess) rc = fail(WIND_ERR_HIP, std::string("hipMalloc(emb_gates): ") + hipGetErrorString(e));
        else m->allocs.push_back(table);
      }
      if (rc == WIND_OK) {
        dim3 grid((unsigned)((w->V + 1 + 63) / 64), (unsigned)((4 * Hp + 63) / 64));
        if (m->dtype == WIND_BF16)
          emb_gates_kernel<bf16_t><<<grid, 256, 0, m->load_stream>>>((const bf16_t *)d.emb, (const bf16_t *)d_ih, d.b_cat[0], (float *)table,
                                                  w->V + 1, 4 * Hp, w->E);
        else
          emb_gates_kernel<float><<<grid, 256, 0, m->load_stream>>>((const float *)d.emb, (const float *)d_ih, d.b_cat[0], (float *)table,
                                                 w->V + 1, 4 * Hp, w->E);
        chk(check_launch("emb_gates"));
        hipError_t e = hipStreamSynchronize(m->load_stream);
        if (rc == WIND_OK && e != hipSuccess) rc = fail(WIND_ERR_HIP, std::string("emb_gates: ") + hipGetErrorString(e));
        d.emb_gates = (const float *)table;
      }
    }
    if (m->dtype == WIND_BF16) {
      // MFMA layout: tile column n0 + g*UB + u = gate g of unit n0/4 + u
      constexpr int UB = PredCfg::BN / 4;
      std::vector<float> cat_t((size_t)4 * Hp * K), bias_t((size_t)4 * Hp);
      for (int g = 0; g < 4; ++g)
        for (int j = 0; j < Hp; ++j) {
          const size_t src = (size_t)j * 4 + g, dst = (size_t)(j / UB) * PredCfg::BN + (size_t)g * UB + j % UB;
          std::memcpy(&cat_t[dst * K], &cat[src * K], sizeof(float) * K);
          bias_t[dst] = bias[src];
        }
      chk(upload_matrix(m, cat_t.data(), (size_t)4 * Hp, K, (size_t)4 * Hp, &d.w_cat_t[l]));
      chk(upload(m, bias_t, &bp));
      d.b_cat_t[l] = (const float *)bp;
    }
  }
  const void *tmp = nullptr;
  chk(upload_matrix(m, w->w_enc, w->Hj, w->D, round_up(w->Hj, 256), &d.w_enc));
  d.w_enc_slab = nullptr;
  if (m->dtype == WIND_BF16 && w->D >= kWideMinK && w->D % 32 == 0) {
    // the same rows in slabs of 32 inputs, for enc_proj_wide_kernel
    const size_t hj_pad = round_up(w->Hj, 256);
    std::vector<uint16_t> h(hj_pad * w->D, 0);
    for (size_t j = 0; j < (size_t)w->Hj; ++j)
      for (size_t k = 0; k < (size_t)w->D; ++k) h[((k >> 5) * hj_pad + j) * 32 + (k & 31)] = host_bf16(w->w_enc[j * w->D + k]);
    chk(upload(m, h, &d.w_enc_slab));
  }
  chk(upload(m, std::vector<float>(w->b_enc, w->b_enc + w->Hj), &tmp)); d.b_enc = (const float *)tmp;
  chk(upload_matrix(m, w->w_pred, w->Hj, Hp, w->Hj, &d.w_pred));
  chk(upload(m, std::vector<float>(w->b_pred, w->b_pred + w->Hj), &tmp)); d.b_pred = (const float *)tmp;
  chk(upload_matrix(m, w->w_out, (size_t)w->V + 1, w->Hj, d.Vpad, &d.w_out));
  d.w_out_slab = nullptr;
  if (m->dtype == WIND_BF16 && w->Hj >= kWideMinK && (unsigned long long)d.Vpad * w->Hj * 2 < (1ull << 32)) {
    // the same rows in slabs of 32 hidden units, for joint_wide_kernel
    std::vector<uint16_t> h((size_t)d.Vpad * w->Hj, 0);
    for (size_t v = 0; v <= (size_t)w->V; ++v)
      for (size_t k = 0; k < (size_t)w->Hj; ++k) h[((k >> 5) * d.Vpad + v) * 32 + (k & 31)] = host_bf16(w->w_out[v * w->Hj + k]);
    chk(upload(m, h, &d.w_out_slab));
  }
  chk(upload(m, std::vector<float>(w->b_out, w->b_out + w->V + 1), &tmp)); d.b_out = (const float *)tmp;
  {
    std::vector<float> wb(w->Hj);
    for (int k = 0; k < w->Hj; ++k) {
      float x = w->w_out[(size_t)w->V * w->Hj + k];
      wb[k] = m->dtype == WIND_BF16 ? host_bf16_to_f32(host_bf16(x)) : x;
    }
    chk(upload(m, wb, &tmp)); d.w_blank = (const float *)tmp;
    double wmax = 0.0;
    for (int v = 0; v < w->V; ++v) {
      double s2 = 0.0;
      for (int k = 0; k < w->Hj; ++k) { double x = w->w_out[(size_t)v * w->Hj + k]; s2 += x * x; }
      wmax = s2 > wmax ? s2 : wmax;
    }
    m->wnorm_max = std::sqrt(wmax);
    set_tau(m);
  }
  for (int i = 0; i < 3 && rc == WIND_OK; ++i) {
    hipError_t e = hipEventCreate(&m->ev_call[i]);
    if (e != hipSuccess) rc = fail(WIND_ERR_HIP, std::string("hipEventCreate: ") + hipGetErrorString(e));
  }
  if (rc == WIND_OK) {
    char *unused = nullptr;
    rc = static_scratch_address(&unused);   // once per device, here rather than in a call that must not stall
  }
  if (rc == WIND_OK) {
    hipError_t e = hipHostMalloc((void **)&m->h_flag, 64 + kNumStats * sizeof(unsigned long long), hipHostMallocDefault);
    if (e != hipSuccess) rc = fail(WIND_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));
    else m->h_stats = reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(m->h_flag) + 64);
  }
  if (rc == WIND_OK) {
    hipError_t e = hipFuncSetAttribute((const void *)joint_ws_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kWsSmemBytes);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)joint_wide_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kWideSmemBytes);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)enc_proj_wide_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kWideSmemBytes);
    static_assert(kFusedSteps == 5, "one resident loop instance per number of fused K steps: here and at the launch");
    const void *loop_instances[] = {(const void *)wind_loop_kernel<0>, (const void *)wind_loop_kernel<1>, (const void *)wind_loop_kernel<2>,
                                    (const void *)wind_loop_kernel<3>, (const void *)wind_loop_kernel<4>, (const void *)wind_loop_kernel<5>};
    for (const void *k : loop_instances)
      if (e == hipSuccess) e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLoopMaxSmem);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)joint_mfma_store_kernel<JointCfg>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, JointCfg::SMEM_BYTES);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)beam_logits_tiny_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              2 * 32 * (kBeamTinyMaxHj + 8) * 2);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)enc_proj_ring5_kernel<EncBigCfg>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              EncBigCfg::SMEM_BYTES);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)enc_proj_mfma_kernel<EncCfg>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, EncCfg::SMEM_BYTES);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)enc_proj_mfma_kernel<EncSmallCfg>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, EncSmallCfg::SMEM_BYTES);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)lstm_layer_dma_kernel<PredCfg>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, PredCfg::SMEM_BYTES);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)pred_proj_dma_kernel<PredCfg>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, PredCfg::SMEM_BYTES);
    if (e != hipSuccess) rc = fail(WIND_ERR_HIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
  }
  if (rc != WIND_OK) {
    std::string keep = g_err;
    wind_free(m);
    g_err = keep;
    return rc;
  }
  *out = m;
  return WIND_OK;
} catch (const std::exception &e) {
  return fail(WIND_ERR_HIP, std::string("wind_load_weights: ") + e.what());
}

int wind_free(wind_model *m) {
  if (!m) return WIND_OK;
  (void)hipDeviceSynchronize();
  for (int g = 0; g < 2; ++g) {
    if (m->graph_exec[g]) (void)hipGraphExecDestroy(m->graph_exec[g]);
    if (m->graph[g]) (void)hipGraphDestroy(m->graph[g]);
  }
  if (m->cap_stream) (void)hipStreamDestroy(m->cap_stream);
  for (void *p : m->allocs) (void)hipFree(p);
  if (m->ws) (void)hipFree(m->ws);
  if (m->beam_ws) (void)hipFree(m->beam_ws);
  beam_pool_free(m);
  if (m->h_flag) (void)hipHostFree(m->h_flag);
  for (hipEvent_t e : m->ev_pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : m->ev_call) if (e) (void)hipEventDestroy(e);
  delete m;
  return WIND_OK;
}

int wind_greedy_decode(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, int W,
                       int max_symbols_per_step, int32_t *out_tokens, int32_t *out_frames,
                       int32_t *out_counts, int cap, void *stream) {
  return decode(m, enc_out, lengths, B, T, W, max_symbols_per_step, out_tokens, out_frames, out_counts, cap, stream);
}

int wind_sequential_decode(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T,
                           int max_symbols_per_step, int32_t *out_tokens, int32_t *out_frames,
                           int32_t *out_counts, int cap, void *stream) {
  return decode(m, enc_out, lengths, B, T, 1, max_symbols_per_step, out_tokens, out_frames, out_counts, cap, stream);
}

static int beam_scores_check(const wind_model *m, const float *enc_window, int n, const float *dec_out, int Bh, int K,
                             const int32_t *out_labels, const int32_t *out_jumps, const float *out_scores) {
  if (!m || !enc_window || !dec_out || !out_labels || !out_jumps || !out_scores) return fail(WIND_ERR_ARG, "null argument");
  if (n < 1 || n > kBeamMaxWindow) return fail(WIND_ERR_ARG, "window must have 1..64 frames");
  if (K < 1 || K > kBeamMaxK) return fail(WIND_ERR_ARG, "K must be in 1..32");
  if (Bh < 1 || (long long)Bh * n > 65536) return fail(WIND_ERR_ARG, "Bh >= 1 and Bh * n <= 65536 required");
  return WIND_OK;
}

// the scoring step's kernels, on a workspace that is already laid out
static int beam_scores_enqueue(wind_model *m, const BeamWs &ws, const float *enc_window, int n, const float *dec_out,
                               int Bh, int K, int32_t *out_labels, int32_t *out_jumps, float *out_scores, hipStream_t s) {
  const ModelDev &d = m->dev;
  beam_enqueue_linear(m, d.w_enc, d.b_enc, enc_window, ws.e, n, d.Hj, d.D, true, s);
  beam_enqueue_linear(m, d.w_pred, d.b_pred, dec_out, ws.p, Bh, d.Hj, d.Hp, false, s);
  beam_enqueue_logits(m, ws, ws.e, n, ws.p, beam_identity(), Bh, s);
  beam_enqueue_topk(m, ws, n, Bh, K, out_labels, out_jumps, out_scores, s);
  return check_launch("beam window scores");
}

int wind_beam_window_scores(wind_model *m, const float *enc_window, int n, const float *dec_out, int Bh, int K,
                            int32_t *out_labels, int32_t *out_jumps, float *out_scores, void *stream) {
  int rc = beam_scores_check(m, enc_window, n, dec_out, Bh, K, out_labels, out_jumps, out_scores);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  BeamWs ws;
  rc = beam_workspace(m, (size_t)n, (size_t)Bh, (size_t)Bh * n, &ws);
  if (rc) return rc;
  rc = beam_scores_enqueue(m, ws, enc_window, n, dec_out, Bh, K, out_labels, out_jumps, out_scores, s);
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(s));
  return WIND_OK;
}

int wind_beam_window_scores_static(wind_model *m, const float *enc_window, int n, const float *dec_out, int Bh, int K,
                                   int32_t *out_labels, int32_t *out_jumps, float *out_scores, void *stream) {
  int rc = beam_scores_check(m, enc_window, n, dec_out, Bh, K, out_labels, out_jumps, out_scores);
  if (rc) return rc;
  const size_t rows = (size_t)Bh * n;
  const size_t need = beam_carve(m, (size_t)n, (size_t)Bh, rows, nullptr, nullptr);
  if (need > (size_t)WIND_STATIC_SCRATCH_BYTES)
    return fail(WIND_ERR_ARG, "wind_beam_window_scores_static: this shape needs " + std::to_string(need) +
                                  " bytes of scratch memory, the static buffer has " +
                                  std::to_string((size_t)WIND_STATIC_SCRATCH_BYTES));
  char *base = nullptr;
  rc = static_scratch_address(&base);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  BeamWs ws;
  beam_carve(m, (size_t)n, (size_t)Bh, rows, base, &ws);
  // The buffer keeps the last call's contents.  The one place read before it is written: the rows
  // between `rows` and the next multiple of the MFMA tile height (whole row tiles are fetched).
  const size_t rows_pad = round_up(rows, JointCfg::BM), pad_ints = (rows_pad - rows) * m->dev.Hj / 2;   // bf16 pairs
  if (pad_ints) {
    const unsigned blocks = (unsigned)std::min<size_t>((pad_ints + 255) / 256, 256);
    fill_int_kernel<<<blocks, 256, 0, s>>>((int *)(ws.z + rows * m->dev.Hj), (int)pad_ints, 0);
    fill_int_kernel<<<blocks, 256, 0, s>>>((int *)(ws.z_lo + rows * m->dev.Hj), (int)pad_ints, 0);
  }
  return beam_scores_enqueue(m, ws, enc_window, n, dec_out, Bh, K, out_labels, out_jumps, out_scores, s);
}

int wind_workspace_bytes(const wind_model *m, int B, int T, int W, size_t *bytes) {
  if (!m || !bytes) return fail(WIND_ERR_ARG, "null argument");
  if (B < 1 || T < 0 || W < 1 || W > WIND_MAX_WINDOW || (long long)B * T > (1ll << 31) - 1)
    return fail(WIND_ERR_ARG, "B >= 1, T >= 0, 1 <= W <= 64, B*T < 2^31 required");
  *bytes = workspace_layout(m, B, T, W).total;
  return WIND_OK;
}

// Completes an asynchronous decode: waits for its stream, reads the counters and the loop's end state.
static int finish_async(wind_model *m) {
  hipStream_t s = m->async_stream;
  m->async_pending = false;
  m->h_flag[0] = m->h_flag[1] = 0;
  HIP_TRY(hipMemcpyAsync(m->h_flag, m->call.n_active, sizeof(int), hipMemcpyDeviceToHost, s));
  if (m->async_loop) HIP_TRY(hipMemcpyAsync(m->h_flag + 2, m->async_bar, 2 * sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  if (m->async_loop) m->loop_info[1] = m->h_flag[3] == 2;
  if (m->async_loop && m->h_flag[2] != 0)
    return fail(WIND_ERR_HIP, "resident loop: a grid barrier timed out (workgroups not all resident?)");
  int rc = fetch_stats(m, s);
  m->have_call_times = true;
  m->prev_B = m->call.B; m->prev_T = m->call.T; m->prev_W = m->call.W;
  m->prev_iters = m->last_stats.iterations;
  // whole replays are an even number of iterations, so the last one left its count in the first slot
  if (m->h_flag[0] != 0) {
    if (rc == WIND_OK || rc == WIND_ERR_OVERFLOW)
      return fail(WIND_ERR_UNFINISHED, "the decode did not finish within max_iterations: outputs hold the labels found so far");
  }
  if (rc == WIND_ERR_OVERFLOW) return fail(rc, "an utterance produced more labels than cap");
  return rc;
}

int wind_get_loop_info(wind_model *m, int *workgroups, int *one_l2) {
  if (!m || !workgroups || !one_l2) return fail(WIND_ERR_ARG, "null argument");
  if (m->async_pending) { const int rc = finish_async(m); if (rc != WIND_OK && rc != WIND_ERR_OVERFLOW && rc != WIND_ERR_UNFINISHED) return rc; }
  *workgroups = m->loop_info[0];
  *one_l2 = m->loop_info[1];
  return WIND_OK;
}

int wind_get_stats(wind_model *m, wind_stats *out) {
  if (!m || !out) return fail(WIND_ERR_ARG, "null argument");
  int rc = WIND_OK;
  if (m->async_pending) rc = finish_async(m);
  if (!m->have_stats) return rc != WIND_OK ? rc : fail(WIND_ERR_ARG, "no decode call yet");
  *out = m->last_stats;
  return rc;
}

int wind_greedy_decode_async(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, int W,
                             int max_symbols_per_step, int32_t *out_tokens, int32_t *out_frames, int32_t *out_counts,
                             int cap, void *workspace, size_t workspace_bytes, int64_t max_iterations, void *stream) {
  if (!workspace) return fail(WIND_ERR_ARG, "workspace is null");
  return decode(m, enc_out, lengths, B, T, W, max_symbols_per_step, out_tokens, out_frames, out_counts, cap, stream,
                workspace, workspace_bytes, (long long)max_iterations);
}

int wind_get_kernel_times(wind_model *m, double *ms, int64_t *launches) {
  if (!m || !ms || !launches) return fail(WIND_ERR_ARG, "null argument");
  for (int k = 0; k < WIND_NUM_KERNELS; ++k) { ms[k] = m->prof_ms[k]; launches[k] = m->prof_n[k]; }
  return WIND_OK;
}

int wind_get_call_times(wind_model *m, double *total_ms, double *loop_ms) {
  if (!m || !total_ms || !loop_ms) return fail(WIND_ERR_ARG, "null argument");
  if (!m->have_call_times) return fail(WIND_ERR_ARG, "no completed decode call yet");
  float a = 0.f, b = 0.f;
  HIP_TRY(hipEventElapsedTime(&a, m->ev_call[0], m->ev_call[2]));
  HIP_TRY(hipEventElapsedTime(&b, m->ev_call[1], m->ev_call[2]));
  *total_ms = a;
  *loop_ms = b;
  return WIND_OK;
}

int wind_get_joint_launches(wind_model *m, int32_t *rows, float *us, int cap, int *n) {
  if (!m || !rows || !us || !n || cap < 0) return fail(WIND_ERR_ARG, "null argument");
  // launches past the last iteration found no active utterance and are left out
  const size_t have = std::min(m->joint_rows.size(), m->joint_us.size());
  const size_t k = std::min<size_t>(have, (size_t)cap);
  for (size_t i = 0; i < k; ++i) { rows[i] = m->joint_rows[i]; us[i] = m->joint_us[i]; }
  *n = (int)have;
  return WIND_OK;
}

int wind_set_option(wind_model *m, const char *key, int64_t value) {
  if (!m || !key) return fail(WIND_ERR_ARG, "null argument");
  if (!std::strcmp(key, "graph")) { m->opt_graph = value != 0; return WIND_OK; }
  if (!std::strcmp(key, "host_sync")) { m->opt_host_sync = value != 0; return WIND_OK; }
  if (!std::strcmp(key, "profile")) {
    m->opt_profile = value != 0;
    for (int k = 0; k < WIND_NUM_KERNELS; ++k) { m->prof_ms[k] = 0.0; m->prof_n[k] = 0; }
    return WIND_OK;
  }
  if (!std::strcmp(key, "unroll")) {
    if (value < 2 || value > 256 || (value & 1)) return fail(WIND_ERR_ARG, "unroll must be even, 2..256");
    m->opt_unroll = (int)value;
    return WIND_OK;
  }
  if (!std::strcmp(key, "beam_exact")) {
    m->opt_beam_exact = value != 0;
    return WIND_OK;
  }
  if (!std::strcmp(key, "debug_stamps")) {
    m->opt_debug_stamps = value != 0;
    m->graph_valid = false;
    return WIND_OK;
  }
  if (!std::strcmp(key, "loop_kernel")) {
    m->opt_loop_kernel = value != 0;
    return WIND_OK;
  }
  if (!std::strcmp(key, "loop_fused")) {
    m->opt_loop_fused = value != 0;
    return WIND_OK;
  }
  if (!std::strcmp(key, "loop_one_xcd")) {
    m->opt_loop_one_xcd = value != 0;
    return WIND_OK;
  }
  if (!std::strcmp(key, "loop_spin_limit")) {
    if (value < 0 || value > (1ll << 30)) return fail(WIND_ERR_ARG, "loop_spin_limit must be in 0..2^30");
    m->opt_loop_spin_limit = value;
    return WIND_OK;
  }
  if (!std::strcmp(key, "enc_wide")) {
    m->opt_enc_wide = value != 0;
    return WIND_OK;
  }
  if (!std::strcmp(key, "joint_wide")) {
    if (value < 0 || value > 2) return fail(WIND_ERR_ARG, "joint_wide must be 0 (never), 1 (iterations with many rows) or 2 (always)");
    m->opt_joint_wide = (int)value;
    m->graph_valid = false;
    m->prev_iters = 0;
    return WIND_OK;
  }
  if (!std::strcmp(key, "atomic_lists")) {
    m->opt_atomic_lists = value != 0;
    m->graph_valid = false;
    return WIND_OK;
  }
  if (!std::strcmp(key, "slot_rows")) {
    m->opt_slot_rows = value != 0;
    m->graph_valid = false;
    return WIND_OK;
  }
  if (!std::strcmp(key, "decide_two")) {
    m->opt_decide_two = value != 0;
    m->graph_valid = false;
    return WIND_OK;
  }
  if (!std::strcmp(key, "lstm_rec")) {
    m->opt_lstm_rec = value != 0;
    m->graph_valid = false;
    return WIND_OK;
  }
  if (!std::strcmp(key, "pred_mfma_min_batch")) {
    m->opt_pred_mfma_min_batch = (int)value;
    m->graph_valid = false;
    return WIND_OK;
  }
  if (!std::strcmp(key, "recheck_kappa_milli")) {
    if (value < 0) return fail(WIND_ERR_ARG, "kappa must be >= 0");
    m->kappa = (double)value / 1000.0;
    set_tau(m);
    m->graph_valid = false;
    return WIND_OK;
  }
  return fail(WIND_ERR_ARG, std::string("unknown option ") + key);
}

// Common start of the debug entry points: workspace for the shape, the call's fields, and a decode
// prologue (state, encoder projection, start-token step) with the library's own outputs.
static int debug_prologue(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, int W, hipStream_t s) {
  int rc = ensure_workspace(m, B, T, W);
  if (rc) return rc;
  CallDev &c = m->call;
  c.B = B; c.T = T; c.W = W; c.S = 1; c.cap = 1;
  c.rec = nullptr;   // whole prediction-network steps: no decision kernel runs between them
  c.lists_atomic = 0;
  c.slot_rows = 0;
  m->fma_pred_step = false;
  m->graph_valid = false;
  c.enc = enc_out;
  if (lengths) {
    c.lengths = lengths;
  } else {   // every frame of every utterance
    fill_int_kernel<<<(unsigned)((B + 255) / 256), 256, 0, s>>>(m->dbg_len, B, T);
    c.lengths = m->dbg_len;
  }
  c.out_tokens = m->dbg_out; c.out_frames = m->dbg_out + B; c.out_counts = m->dbg_out + 2 * B;
  return enqueue_prologue(m, s);
}

int wind_debug_joint_logits(wind_model *m, const float *enc_out, int B, int T, int b, int t0, int n,
                            const int32_t *prefix, int prefix_len, int exact, float *logits, void *stream) try {
  if (!m || !enc_out || !logits) return fail(WIND_ERR_ARG, "null argument");
  if (B < 1 || T < 1 || b < 0 || b >= B || t0 < 0 || n < 1 || t0 + n > T || n > WIND_MAX_WINDOW)
    return fail(WIND_ERR_ARG, "window out of range");
  if ((long long)B * T > (1ll << 31) - 1) return fail(WIND_ERR_ARG, "B*T too large");
  if (prefix_len < 0 || (prefix_len > 0 && !prefix)) return fail(WIND_ERR_ARG, "bad prefix");
  for (int i = 0; i < prefix_len; ++i)
    if (prefix[i] < 0 || prefix[i] >= m->dev.V) return fail(WIND_ERR_ARG, "prefix label out of range");
  hipStream_t s = (hipStream_t)stream;
  int rc = debug_prologue(m, enc_out, nullptr, B, T, WIND_MAX_WINDOW, s);   // start-token step on every utterance
  CallDev &c = m->call;
  for (int i = 0; i < prefix_len && rc == WIND_OK; ++i) {
    // feed prefix[i] to utterance b only: an emit list of one entry
    fill_int_kernel<<<1, 256, 0, s>>>(c.n_emit, 1, 1);
    fill_int_kernel<<<1, 256, 0, s>>>(c.emit_idx, 1, b);
    fill_int_kernel<<<1, 256, 0, s>>>(c.emit_list_tok, 1, prefix[i]);
    rc = enqueue_pred_step(m, s, false);
  }
  if (rc == WIND_OK) {
    const ModelDev &d = m->dev;
    const float *pb = c.p + (size_t)b * d.Hj;
    if (m->dtype == WIND_F32) {
      joint_exact_kernel<float><<<n, 256, (size_t)d.Hj * 4, s>>>(d, c, 0, 0, b, t0, n, pb, 0, logits, nullptr);
    } else if (exact) {
      joint_exact_kernel<bf16_t><<<n, 256, (size_t)d.Hj * 4, s>>>(d, c, 0, 0, b, t0, n, pb, 0, logits, nullptr);
    } else {
      // hidden vectors rounded to bf16 into the window buffer, then the MFMA tile core with stores
      joint_exact_kernel<bf16_t><<<n, 256, (size_t)d.Hj * 4, s>>>(d, c, 0, 0, b, t0, n, pb, 1, nullptr, c.z);
      dim3 grid(1, (unsigned)((d.V + 1 + JointCfg::BN - 1) / JointCfg::BN));
      joint_mfma_store_kernel<JointCfg><<<grid, JointCfg::NT, JointCfg::SMEM_BYTES, s>>>(d, c.z, nullptr, n, logits);
    }
    rc = check_launch("debug joint");
  }
  hipError_t e = hipStreamSynchronize(s);
  if (rc == WIND_OK && e != hipSuccess) return fail(WIND_ERR_HIP, std::string("debug sync: ") + hipGetErrorString(e));
  return rc;
} catch (const std::exception &e) {
  return fail(WIND_ERR_HIP, std::string("wind_debug_joint_logits: ") + e.what());
}

int wind_debug_enc_proj(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, float *e_out,
                        void *stream) try {
  if (!m || !enc_out || !lengths || !e_out) return fail(WIND_ERR_ARG, "null argument");
  if (B < 1 || T < 1 || (long long)B * T > (1ll << 31) - 1) return fail(WIND_ERR_ARG, "B >= 1, T >= 1, B*T < 2^31 required");
  hipStream_t s = (hipStream_t)stream;
  int rc = debug_prologue(m, enc_out, lengths, B, T, 1, s);
  if (rc) return rc;
  HIP_TRY(hipMemcpyAsync(e_out, m->call.e, (size_t)B * T * m->dev.Hj * sizeof(float), hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipStreamSynchronize(s));
  return WIND_OK;
} catch (const std::exception &e) {
  return fail(WIND_ERR_HIP, std::string("wind_debug_enc_proj: ") + e.what());
}

int wind_debug_joint_keys(wind_model *m, const float *enc_out, const int32_t *lengths, int B, int T, int W,
                          float *keys, int32_t *nparts, int32_t *part_width, void *stream) try {
  if (!m || !nparts || !part_width) return fail(WIND_ERR_ARG, "null argument");
  if (m->dtype != WIND_BF16) return fail(WIND_ERR_UNSUPPORTED, "fp32 models take the argmax directly: there are no keys");
  if (m->dev.Hj > kDecideMaxHj) return fail(WIND_ERR_UNSUPPORTED, "Hj > 2048");
  if (B < 1 || T < 1 || W < 1 || W > WIND_MAX_WINDOW || (long long)B * T > (1ll << 31) - 1)
    return fail(WIND_ERR_ARG, "B >= 1, T >= 1, 1 <= W <= 64, B*T < 2^31 required");
  {
    const WsLayout w = workspace_layout(m, B, T, W);
    *nparts = w.nparts;
    *part_width = WsCfg<1>::WN;
  }
  if (!keys) return WIND_OK;
  if (!enc_out || !lengths) return fail(WIND_ERR_ARG, "null argument");
  hipStream_t s = (hipStream_t)stream;
  int rc = debug_prologue(m, enc_out, lengths, B, T, W, s);
  if (rc) return rc;
  const CallDev &c = m->call;
  // the first loop iteration's window rows and their keys, by the kernels a decode call launches
  const bool wide = wide_threshold_rows(m, B, W) >= 0 && (long long)B * W > wide_threshold_rows(m, B, W);
  build_z_kernel<<<(unsigned)((B * W + 3) / 4), 256, 0, s>>>(m->dev, c, 0, wide ? 1 : 0, -1);
  enqueue_joint(m, s, 0, true, wide);
  rc = check_launch("debug joint keys");
  if (rc) return rc;
  HIP_TRY(hipMemcpyAsync(keys, c.parts, (size_t)B * W * c.nparts * sizeof(float4), hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipStreamSynchronize(s));
  return WIND_OK;
} catch (const std::exception &e) {
  return fail(WIND_ERR_HIP, std::string("wind_debug_joint_keys: ") + e.what());
}

}  // extern "C"
