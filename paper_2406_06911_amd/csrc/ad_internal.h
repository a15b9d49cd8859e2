// Internal declarations shared by the host logic, the runtime and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "asyncdiff.h"

namespace ad {

void set_error(const char* fmt, ...);

#define AD_FAIL(code, ...)          \
  do {                              \
    ::ad::set_error(__VA_ARGS__);   \
    return (code);                  \
  } while (0)

#define AD_HIP(expr)                                                                             \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) AD_FAIL(AD_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

constexpr int kTrainSteps = 1000;
constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
inline int round_up(int v, int a) { return (v + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == AD_BF16 ? 2 : 4; }

// GEMM tiling constants the packing and the kernels agree on.
constexpr int kRowBytes = 128;                      // bytes of K per LDS row per k-tile
inline int bk_elems(int dtype) { return kRowBytes / (int)esize(dtype); }   // 64 (bf16) / 32 (fp32)
constexpr int kNPad = 128;                          // packed weight rows are padded to this multiple
constexpr int kConvInK = 64;                        // padded K of the im2col'ed first convolution

struct Unit {
  ad_unit_info info;
  int comp = 0;            // owning component, 1-based
  // weight indices into Ctx::weights (manifest order); -1 when absent
  int w_first = -1;
  int temb_row = 0;        // row offset of this ResBlock in the fused time-embedding projection
};

enum WeightRole {
  W_CONV3,       // [O][I][3][3] -> packed GEMM operand
  W_CONV1,       // [O][I][1][1] or linear [O][I] -> packed GEMM operand
  W_CONV_IN,     // first convolution: packed against the im2col'ed latent
  W_GEGLU,       // ff1: rows interleaved value/gate in blocks of 32
  W_SMALL,       // [O][I] kept row-major in storage dtype (time MLP)
  W_TEMB,        // ResBlock time projection, rows gathered into one matrix
  W_VEC_F32,     // bias / gamma / beta, fp32 (padded to kNPad when used as a GEMM bias)
  W_GEGLU_BIAS,  // ff1 bias, interleaved like its weight
  W_TEMB_BIAS,
  W_QKV_Q,       // self-attention q: holds the fused [q; k; v] GEMM operand
  W_QKV_KV       // self-attention k and v: stored inside the fused operand of q
};

struct Weight {
  ad_weight_info info;
  int role = W_VEC_F32;
  size_t dev_off = 0;     // offset in the weight arena
  size_t dev_bytes = 0;
  int n_pad = 0, k_pad = 0;
};

struct Component {
  int first = 0, last = 0;
  std::vector<int> in_units, out_units;
  int temb_row0 = 0, temb_rows = 0;    // rows of the fused time projection this component needs
};

// Activation workspace of one (component, lane): offsets into the work arena.
constexpr int kNumTemps = 10;
struct Workspace {
  std::vector<size_t> unit_off;        // per unit of the component (index unit - first); SIZE_MAX = external output
  size_t temp_off[kNumTemps] = {0};
  size_t temp_bytes[kNumTemps] = {0};
  size_t f32_off = 0;                  // small fp32 area: sinusoid, time MLP, projections
  size_t gn_off = 0;                   // GroupNorm scratch
};

struct Ctx {
  ad_unet_cfg cfg{};
  int N = 1, warmup = 0, stride = 1;   // N: evaluations per step (segments); equals `devices` unless wrapped
  int devices = 1;                      // components that run side by side (streams of an asynchronous round)
  bool wrap = false;                    // wrapped segmentation: segments 1 and N are one component
  std::vector<Unit> units;
  std::vector<Component> comps;
  std::vector<Weight> weights;
  int temb_dim = 0, temb_rows_total = 0;
  // combined weights (not in the manifest): fused time projection matrix and bias
  size_t temb_w_off = 0, temb_b_off = 0;

  // memory plan
  size_t weight_bytes = 0, work_bytes = 0;
  std::vector<size_t> slot_off[3];     // per unit; SIZE_MAX when the unit's output never crosses components (the third
                                       // copy is used by the per-edge mode only)
  std::vector<size_t> eps_off;         // per stride lane
  // cross-attention keys / values of the text embedding (constant over the steps): per unit, per layer
  std::vector<std::vector<size_t>> text_k_off, text_v_off;
  const void* text_cached = nullptr;   // text embedding the cache was computed from
  std::vector<std::vector<Workspace>> ws;   // [component][lane]
  size_t f32_bytes = 0, gn_bytes = 0;

  char* weights_dev = nullptr;
  char* work_dev = nullptr;
  bool weights_loaded = false;

  // run state
  int T = 0, sampler = AD_DDIM, beta_kind = AD_BETA_LINEAR, time_shift = 0;
  float cfg_scale = 1.f;
  std::vector<int> taus;
  std::vector<double> acp;             // cumulative alpha products, 1000 entries
  std::vector<ad_sched_row> rows;
  size_t next_row = 0;
  int steps_done = 0;
  std::vector<hipEvent_t> events;      // one per stream used + helpers
  hipEvent_t ev_pack = nullptr;
  void* profiler = nullptr;            // ad::Profiler*, owned

  // per-step scalars on the device (timestep, input scale, sampler coefficients) and the step counter the
  // kernels index them with; uploaded at the first round of a run
  size_t step_table_off = 0, step_counter_off = 0;
  bool step_table_ready = false;

  // captured asynchronous rounds, one per slot parity (graph mode)
  bool use_graphs = false;
  struct RoundGraph {
    hipGraphExec_t exec = nullptr;
    hipGraph_t graph = nullptr;
    const void* latent = nullptr; const void* text = nullptr; const void* pooled = nullptr;
    std::vector<hipStream_t> streams;
    float cfg_scale = 0.f;
    std::vector<int> offsets;            // per row: component and (tau, latent, eps) step relative to the round's first step
  } round_graph[2];

  // per-edge mode (ad_set_edge_mode): an asynchronous round is not bracketed by a barrier; every evaluation waits for the
  // evaluations whose stored tensors it reads (previous round) and for the readers of the copy it overwrites (two rounds
  // back; three copies of the stored tensors, copy = round mod 3).  Events by [component - 1][round mod 4], the sampler's by
  // [round mod 4]; one device step counter per component (the components are in different rounds at the same time).
  bool edge_mode = false;
  std::vector<hipEvent_t> ev_done;
  hipEvent_t ev_sampler[4] = {nullptr, nullptr, nullptr, nullptr};
  struct CompGraph {
    hipGraphExec_t exec = nullptr;
    hipGraph_t graph = nullptr;
    const void* latent = nullptr; const void* text = nullptr; const void* pooled = nullptr;
    hipStream_t stream = nullptr;
    float cfg_scale = 0.f;
    int tau_off = 0, latent_off = 0, eps_off = 0;
  };
  std::vector<CompGraph> comp_graph;   // [evaluation of the round * 3 + copy written]
};

// host logic
int64_t unit_flops(const ad_unet_cfg& c, const ad_unit_info& u);
std::vector<int> partition_cuts(const std::vector<int64_t>& costs, int n);
void build_schedule(int T, int N, int w, int S, bool time_shift, bool wrap, std::vector<ad_sched_row>& rows);
std::vector<int> partition_cuts_wrapped(const std::vector<int64_t>& costs, int n);
void sampler_coeffs(const Ctx& c, int step, double* cx, double* ce, double* in_scale, double* init_scale);
size_t tensor_bytes(const Ctx& c, int unit);

// weight packing (host)
size_t packed_conv_bytes(int dtype, int n_out, int c_in, int ksize);
void pack_conv(int dtype, const float* w, int n_out, int c_in, int ksize, bool geglu, void* out);
void pack_rows(int dtype, const float* w, size_t n, void* out);   // plain conversion
uint16_t f32_to_bf16(float f);

}  // namespace ad
