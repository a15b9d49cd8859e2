// Launchers of the HIP kernels (device pointers, explicit stream).  Shapes are validated here,
// on the host, before any launch.
#pragma once

#include "ad_internal.h"

namespace ad {

// Optional per-launch timing: when a profiler is installed and switched on, every kernel launch
// is bracketed by HIP events on its own stream and tagged with its algorithmic work.
struct ProfRec {
  const char* name;
  double flops;      // algorithmic floating-point operations of the launch
  double bytes;      // algorithmic HBM bytes of the launch
  hipEvent_t start, stop;
  int m = 0, n = 0, k = 0;   // GEMM view of the launch (attention: queries, keys, channels), else 0
};
struct Profiler {
  bool on = false;
  std::vector<ProfRec> recs;
};
void set_profiler(Profiler* p);   // per host thread; nullptr removes it
struct ProfLaunch {
  ProfLaunch(const char* name, double flops, double bytes, hipStream_t s, int m = 0, int n = 0, int k = 0);
  ~ProfLaunch();
  hipEvent_t stop_ = nullptr;
  hipStream_t s_ = nullptr;
};

struct ConvArgs {
  int dtype;
  const void* src0; const void* src1;   // NHWC sources, concatenated on channels
  int c0, c1;
  int batch, hs, ws;                    // stored spatial size of the sources
  int up;                               // 1: logical input = nearest-2x of the stored one
  int ksize, stride;
  const void* w;                        // packed [n_pad][k_pad]
  int n_out;                            // GEMM N (for GEGLU: the 2x-wide packed projection)
  const float* bias; const float* rowvec; int rowvec_ld;   // rowvec [batch][rowvec_ld]; 0: ld = n_out, < 0: one row for every sample
  const void* residual;
  void* out; int out_mode; int ld_t;
  void* splitk_ws = nullptr;            // fp32 scratch for split-K partial sums (optional)
  size_t splitk_bytes = 0;
  void* out2 = nullptr; void* out3 = nullptr;   // OUT_QKV: columns [n/3, 2n/3) and [2n/3, n)
  int k_real = 0;                       // > 0: K without zero padding, for the profiler's FLOP count (the im2col'ed first convolution)
};
// OUT_QKV: n_out = 3c; thirds go to out [m][c], out2 [m][c] and out3 ([batch][c][ld_t] when ld_t > 0, else [m][c])
enum { OUT_ROWMAJOR = 0, OUT_GEGLU = 1, OUT_TRANSPOSED = 2, OUT_TRANSPOSED_F32 = 3, OUT_QKV = 4 };

ad_status launch_conv(const ConvArgs& a, hipStream_t s);
void set_tile_override(int tile);     // -1 = choose automatically
void set_attn_variant(int variant);   // -1 automatic, 0 first-generation kernel, 1 / 2 second generation with 32 / 64 queries per wavefront
void set_order_override(int order);   // -1 automatic, 0 row-tile-major, 1 column-tile-major workgroup order
// scratch a convolution of this shape wants for split-K (0 = it will not split); k = taps * channels
size_t conv_workspace_bytes(int dtype, long long m, int n, int k, int out_mode);

ad_status launch_groupnorm(int dtype, const void* src0, const void* src1, int c0, int c1, int batch, int hw, int groups,
                           const float* gamma, const float* beta, float eps, int silu, void* out, void* scratch,
                           size_t scratch_bytes, hipStream_t s);
// the same with the partial sums in the library's fixed device array (no caller scratch, no allocation)
ad_status launch_groupnorm_static(int dtype, const void* src0, const void* src1, int c0, int c1, int batch, int hw, int groups,
                                  const float* gamma, const float* beta, float eps, int silu, void* out, hipStream_t s);
ad_status launch_layernorm(int dtype, const void* src, int rows, int c, const float* gamma, const float* beta, float eps,
                           void* out, hipStream_t s);
ad_status launch_attention(int dtype, const void* q, const void* k, const void* v, int v_t, int batch, int l, int lk, int c,
                           int head_dim, int ldq, int ldk, int ldv, int ldo, void* out, hipStream_t s);
// attention over the frame axis: row (f, p) = f * positions + p of q / k / v / out; heads = c / head width
ad_status launch_attention_frames(int dtype, const void* q, const void* k, const void* v, int frames, int positions, int c,
                                  int heads, int ldq, int ldk, int ldv, int ldo, void* out, hipStream_t s);
// out[r][n] = act_out(bias[n] + sum_k act_in(in[r*in_ld + k]) w[n][k]); in/out fp32, w in dtype; rows <= 16;
// in_ld = 0 feeds every row the same input
ad_status launch_linear_rows(int dtype, const float* in, int in_ld, int rows, int k, const void* w, const float* bias, int n,
                             int silu_in, int silu_out, int accumulate, float* out, hipStream_t s);
// Per-step scalars can be passed as immediates or looked up on the device: table[*counter + offset].  The
// second form keeps the launch arguments identical from round to round, which a captured graph needs.
struct StepRec { float tau, in_scale, cx, ce; };
struct StepRef {
  const StepRec* table = nullptr;   // nullptr: use the immediate value
  const int* counter = nullptr;
  int offset = 0;
};
ad_status launch_sinusoid(float tau, StepRef ref, int dim, float* out, hipStream_t s);
ad_status launch_advance(int* counter, int by, hipStream_t s);
// im2col of the fp32 latent (times scale) for the first 3x3 convolution: out [batch*h*w][kConvInK]; the latent is
// [cl][h][w] shared by all batch rows, or [batch][cl][h][w] when per_sample is set
ad_status launch_pack_latent(int dtype, const float* latent, int per_sample, float scale, StepRef ref, int cl, int h, int w, int batch,
                             void* out, hipStream_t s);
ad_status launch_sampler(float* x, const float* eps, size_t n, int batch, float cx, float ce, StepRef ref, float g, hipStream_t s);

}  // namespace ad
