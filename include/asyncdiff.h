/*
 * asyncdiff.h - C ABI of the MI355X (gfx950) asynchronous-denoising library.
 *
 * The library runs the noise-prediction UNet of a latent diffusion model cut into N
 * sequential components (AsyncDiff, arXiv 2406.06911, Section 3.2, Eq. 4), under the paper's
 * asynchronous schedule: w sequential warm-up steps, then component n of a step consumes what
 * component n-1 (and every other producer of its skip features) stored in the previous
 * parallel round (Section 3.2 "Asynchronous Denoising", Eq. 5, "Multi-Device Communication"),
 * optionally with stride denoising (Section 3.2 "Stride Denoising", Appendix A) and time
 * shifting (Appendix A), followed by the sampler update S(x_t, eps_t, t) (Section 3.1, Eq. 3).
 * The paper spreads the components over GPUs; here one GPU runs them concurrently on the
 * HIP streams the caller passes.
 *
 * Conventions
 *   - Every pointer argument says whether it is HOST or DEVICE memory.  The library never
 *     allocates device memory: the caller allocates the two arenas whose sizes
 *     ad_device_bytes() reports and hands them over with ad_bind_device_memory().
 *   - Hidden states are DEVICE tensors in NHWC order [batch][H][W][C], element type = cfg.dtype.
 *     The latent is DEVICE fp32 [latent_channels][H][W] (one image; the batch rows of
 *     classifier-free guidance share it).  The noise prediction is DEVICE fp32
 *     [batch][latent_channels][H][W].  The text embedding is DEVICE, element type = cfg.dtype,
 *     [batch][ctx_len][ctx_dim]; the pooled embedding DEVICE fp32 [batch][pooled_dim].
 *     Video model (cfg.frames > 0): latent and noise prediction are both fp32 [frames][latent_channels][H][W],
 *     the text embedding is [1][ctx_len][ctx_dim], the sampler applies no guidance.
 *   - Steps are numbered i = 0..T-1 in execution order; tau_i is the training timestep of step i.
 *   - Calls that take a stream only enqueue work; they never synchronise.
 *   - Every call returns an ad_status; no exception crosses the boundary.  ad_last_error()
 *     returns a HOST string describing the last failure on the calling thread.
 *   - A context is not thread-safe; use one per host thread or serialise calls.
 */
#ifndef ASYNCDIFF_H
#define ASYNCDIFF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ad_status {
  AD_OK = 0,
  AD_ERR_INVALID = 1, /* bad argument or configuration */
  AD_ERR_NOMEM = 2,   /* bound arenas too small / host allocation failed */
  AD_ERR_HIP = 3,     /* a HIP runtime call failed */
  AD_ERR_DONE = 4,    /* ad_step called after the last step */
  AD_ERR_STATE = 5    /* call order violated (e.g. forward before weights are loaded) */
} ad_status;

typedef enum ad_dtype { AD_F32 = 0, AD_BF16 = 1 } ad_dtype;
typedef enum ad_sampler_kind { AD_DDIM = 0, AD_EULER = 1 } ad_sampler_kind;
typedef enum ad_beta_kind { AD_BETA_LINEAR = 0, AD_BETA_SCALED_LINEAR = 1 } ad_beta_kind;
typedef enum ad_unit_kind {
  AD_UNIT_CONV_IN = 0, AD_UNIT_RES = 1, AD_UNIT_TFM = 2, AD_UNIT_DOWN = 3, AD_UNIT_UP = 4, AD_UNIT_OUT = 5
} ad_unit_kind;

#define AD_MAX_LEVELS 4
#define AD_NAME_LEN 64

/* Shape of the UNet.  The paper uses the denoiser as a black box (Section 4.1); this struct
 * describes the Stable-Diffusion-shaped family it is evaluated on. */
typedef struct ad_unet_cfg {
  int latent_channels;                  /* 4 */
  int height, width;                    /* latent size */
  int batch;                            /* 2 with classifier-free guidance, else 1 */
  int n_levels;                         /* <= AD_MAX_LEVELS */
  int channels[AD_MAX_LEVELS];          /* per level; multiples of 32 (fp32) / 64 (bf16) */
  int layers_per_block;                 /* ResBlocks per down level (up levels have one more) */
  int transformer_depth[AD_MAX_LEVELS]; /* transformer layers after each ResBlock of the level; 0 = none */
  int mid_depth;                        /* transformer layers in the middle block; 0 = none */
  int head_dim;                         /* attention head width; channels[l] % head_dim == 0 */
  int gn_groups;
  int ctx_len, ctx_dim;                 /* text embedding */
  int pooled_dim;                       /* 0 = no pooled-embedding branch */
  float gn_eps, ln_eps;
  int dtype;                            /* ad_dtype: storage type of weights and hidden states */
  /* Video model (Section 4, "Experimental Results on Video Diffusion Models", Table 4: the same schedule on a UNet
   * with temporal layers).  frames > 0: the batch axis is the frame axis (batch == frames <= 16), every frame has its own latent,
   * there is no guidance pair, one text embedding [1][ctx_len][ctx_dim] serves all frames.  temporal_heads > 0 adds,
   * after every spatial transformer, a temporal attention layer: LayerNorm, multi-head attention whose tokens are
   * the frames of one spatial position (head width = channels / temporal_heads, no positional term), output
   * projection, residual.  Both 0: image model. */
  int frames;
  int temporal_heads;
} ad_unet_cfg;

typedef struct ad_unit_info {
  char name[AD_NAME_LEN];
  int kind;        /* ad_unit_kind */
  int c_in, c_skip, c_out;
  int h_in, w_in, h_out, w_out;
  int depth;       /* transformer layers */
  int skip_from;   /* unit whose output is concatenated to the main input, or -1 */
  int64_t flops;   /* 2 per multiply-accumulate: convolutions, linear layers, attention matmuls */
} ad_unit_info;

typedef struct ad_weight_info {
  char name[AD_NAME_LEN];
  int ndim;
  int shape[4];    /* conv: [out][in][k][k]; linear: [out][in]; vectors: [n] */
} ad_weight_info;

/* One component evaluation of the schedule table (Section 3.2; Appendix A). */
typedef struct ad_sched_row {
  int round;       /* parallel round; warm-up steps are rounds 0..w-1 */
  int comp;        /* 1..N */
  int tau_step;    /* step whose timestep feeds the time embedding */
  int read_slot;   /* 0/1: which stored-state slot the inputs come from */
  int write_slot;  /* 0/1, or -1 when only the noise prediction of this evaluation is kept */
  int latent_step; /* step index of the latent read by component 1, else -1 */
  int eps_step;    /* step whose noise prediction this evaluation yields (component N), else -1 */
  int fresh_from;  /* wrapped segmentation: evaluation of the same round whose outputs are read fresh (0 = none) */
} ad_sched_row;

typedef struct ad_ctx ad_ctx;
typedef void* ad_stream; /* a hipStream_t */

/* ---- life cycle (host only, no GPU needed) -------------------------------------------------- */

/* Builds the unit list, the FLOP-balanced contiguous partition into n_components (Section 3.2:
 * components of comparable load; Appendix A "Model Segmentation") and the memory plan.
 * warmup >= 1 is required when n_components > 1 (the stored states must exist before the first
 * asynchronous round); stride >= 1.  cfg: HOST.  *out receives a context owned by the library. */
ad_status ad_create(const ad_unet_cfg* cfg, int n_components, int warmup, int stride, ad_ctx** out);
/* The same with the partition given by the caller (Section 3.2 asks for components of comparable load and leaves
 * the measure open; a caller that has timed the units can balance by time instead of FLOPs).  cuts: HOST,
 * n_components - 1 unit indices, cuts[k] = first unit of component k + 2, strictly increasing, inside
 * (0, number of units); ignored (may be NULL) when n_components is 1.  Everything else as ad_create. */
ad_status ad_create_with_cuts(const ad_unet_cfg* cfg, int n_components, const int* cuts, int warmup, int stride, ad_ctx** out);
/* The partition rule of ad_create applied to arbitrary per-unit costs (FLOPs, measured microseconds, ...): the
 * contiguous split of n_units costs into n_components parts that minimises the largest part; among optimal
 * splits the lexicographically smallest cut vector.  costs: HOST, non-negative; cuts: HOST, receives
 * n_components - 1 first-unit indices (the format ad_create_with_cuts takes). */
ad_status ad_balance_cuts(const int64_t* costs, int n_units, int n_components, int* cuts);
/* Wrapped segmentation (Appendix A "Model Segmentation": for SDXL the first and the last blocks are one segment, the
 * rest is split sequentially).  The unit list is cut into n_components + 1 contiguous segments; segment 1 (head)
 * and segment n_components + 1 (tail) are one component, run back to back on one stream; segments 2..n_components
 * are the other components.  The schedule table, ad_component_forward and ad_component_io number the segments
 * 1..n_components + 1 (ad_num_segments); in an asynchronous round the tail reads the head's outputs of the same
 * round (fresh skip features) and everything else from the previous round, and yields the noise prediction.
 * cuts: HOST, n_components first-unit indices of segments 2..n_components + 1, or NULL for the split that minimises
 * the largest component cost in FLOPs (ties: lexicographically smallest; exhaustive search, n_components <= 6).
 * Stride is 1 (the paper does not say how stride and this segmentation combine); n_components >= 2. */
ad_status ad_create_wrapped(const ad_unet_cfg* cfg, int n_components, const int* cuts, int warmup, ad_ctx** out);
/* Number of unit ranges ad_get_partition fills: n_components, or n_components + 1 for the wrapped segmentation. */
int ad_num_segments(const ad_ctx* ctx);
void ad_destroy(ad_ctx* ctx); /* NULL is allowed */
const char* ad_last_error(void);

/* ---- introspection (host only; integer results are bit-exact by contract) ------------------- */
int ad_num_units(const ad_ctx* ctx);
ad_status ad_get_unit(const ad_ctx* ctx, int unit, ad_unit_info* out);
/* first[k], last[k]: unit range of component k+1; arrays of n_components ints (HOST). */
/* first/last: HOST arrays of ad_num_segments() entries. */
ad_status ad_get_partition(const ad_ctx* ctx, int* first, int* last);
/* Tensors a component reads from earlier components / offers to later ones, named by producing
 * unit (-1 = the latent).  Arrays HOST, capacity cap each; n_in and n_out receive the counts.
 * The main hidden state (previous unit / last unit) is always listed.  Order: ascending. */
ad_status ad_component_io(const ad_ctx* ctx, int comp, int cap, int* in_units, int* n_in, int* out_units, int* n_out);
/* Shape and byte size of the tensor unit `unit` produces (unit -1: the latent, fp32). */
ad_status ad_tensor_shape(const ad_ctx* ctx, int unit, int* b, int* h, int* w, int* c, size_t* bytes);
int ad_num_weights(const ad_ctx* ctx);
ad_status ad_get_weight(const ad_ctx* ctx, int index, ad_weight_info* out);

/* ---- device memory and weights --------------------------------------------------------------- */
ad_status ad_device_bytes(const ad_ctx* ctx, size_t* weight_bytes, size_t* work_bytes);
/* weights_dev, work_dev: DEVICE, 256-byte aligned, at least the sizes above; owned by the caller and
 * must outlive the context's use.  The work arena holds the stored-state slots, the per-component
 * activations and the noise predictions. */
ad_status ad_bind_device_memory(ad_ctx* ctx, void* weights_dev, size_t weight_bytes, void* work_dev, size_t work_bytes);
/* host_ptrs[i]: HOST fp32 array of weight i in manifest order and manifest shape.  The library
 * converts to cfg.dtype, re-lays-out for its kernels and copies to the weight arena (synchronous). */
ad_status ad_load_weights(ad_ctx* ctx, const float* const* host_ptrs, int n);

/* ---- run set-up -------------------------------------------------------------------------------- */
/* Fixes the number of steps T, the sampler and the noise schedule, builds the schedule table and
 * rewinds the step counter.  Timesteps: tau_i = (T-1-i) * (1000 / T); betas over 1000 training steps
 * from 0.00085 to 0.012 (linear, or linear in sqrt(beta)).  time_shift: Appendix A "Time Shifting". */
ad_status ad_reset(ad_ctx* ctx, int T, int sampler_kind, int beta_kind, float cfg_scale, int time_shift);
ad_status ad_get_timesteps(const ad_ctx* ctx, int* tau, int cap);           /* HOST out, T entries */
int ad_num_sched_rows(const ad_ctx* ctx);
ad_status ad_get_schedule(const ad_ctx* ctx, ad_sched_row* rows, int cap);  /* HOST out */
/* Sampler coefficients of step i: x' = c_x * x + c_eps * eps; in_scale multiplies the latent before it
 * enters the model (1 for DDIM); init_scale multiplies the initial noise (1 for DDIM).  HOST out. */
ad_status ad_get_sampler_coeffs(const ad_ctx* ctx, int step, double* c_x, double* c_eps, double* in_scale, double* init_scale);

/* ---- the hot path ------------------------------------------------------------------------------ */

/* One evaluation of component `comp` (1..N) = eps_theta^comp(., t) of Eq. 4.
 *   lane        which private activation workspace to use: 0, or 0..stride-1 for the last component
 *               (two evaluations that run concurrently must use different lanes);
 *   hidden_in   HOST array of DEVICE pointers, one per input of ad_component_io() in its order
 *               (for component 1 the single entry is the fp32 latent, [frames][C][H][W] for the video model);
 *   t_index     step index i whose timestep tau_i feeds the time embedding (0..T-1);
 *   latent_scale  factor applied to the latent on entry (component 1 only; ad_get_sampler_coeffs);
 *   text_emb, pooled_emb  DEVICE (pooled_emb may be NULL when cfg.pooled_dim == 0);
 *   hidden_out  HOST array of DEVICE pointers, one per output of ad_component_io() in its order
 *               (the last component's single output is the fp32 noise prediction);
 *   stream      all work is enqueued here.
 * Inputs are only read, outputs only written; nothing else outside the lane's workspace changes. */
ad_status ad_component_forward(ad_ctx* ctx, int comp, int lane, const void* const* hidden_in, int t_index,
                               float latent_scale, const void* text_emb, const void* pooled_emb,
                               void* const* hidden_out, ad_stream stream);

/* The cross-attention keys and values depend only on the text embedding, not on the step: this call
 * computes them once into the work arena.  ad_step does it by itself at the first round of a run;
 * ad_component_forward uses the cache when it is called with the same text_emb pointer and recomputes
 * the projections otherwise.  ad_reset drops the cache.  text_emb: DEVICE. */
ad_status ad_precompute_text(ad_ctx* ctx, const void* text_emb, ad_stream stream);

/* One parallel round of the schedule (one step during warm-up, `stride` steps afterwards, fewer in a
 * trailing partial round): evaluates the round's components concurrently on the given streams
 * (evaluation e runs on streams[e % n_streams]; n_streams = 1 gives the serial order), stores their
 * outputs in the slot the table names, then applies the sampler once per completed step.
 *   latent      DEVICE fp32 [C][H][W] ([frames][C][H][W] for the video model), updated in place;
 *   streams     HOST array of hipStream_t;
 *   steps_done  HOST out: total steps completed after this call.
 * On return all work is enqueued; the last used event is waited on by streams[0], so synchronising
 * streams[0] is enough to observe the round.  Returns AD_ERR_DONE once T steps are complete. */
ad_status ad_step(ad_ctx* ctx, void* latent, const void* text_emb, const void* pooled_emb,
                  const ad_stream* streams, int n_streams, int* steps_done);

/* Graph mode (off by default): full asynchronous rounds are captured into a HIP graph the first time each
 * slot parity is met (per-step scalars are read from a device table through a device-side step counter, so
 * the captured launch arguments do not change from round to round) and replayed afterwards with one
 * hipGraphLaunch on streams[0]; the host then enqueues one call per round instead of ~500 launches.  Warm-up
 * rounds, trailing partial rounds and rounds under ad_profile_enable are launched directly.  The graphs are
 * tied to the latent / text / pooled pointers, the streams and the run; a change re-captures. */
ad_status ad_set_graph_mode(ad_ctx* ctx, int on);

/* Per-edge mode (off by default; Section 3.2, Eq. 7: a component needs nothing but the outputs its predecessors produced
 * in the previous step): full asynchronous rounds are enqueued without the barrier that otherwise opens and closes a
 * round.  Evaluation e of a round runs on streams[e % n_streams]; before it starts it waits (events) for the evaluations of
 * the previous round whose stored outputs it reads - component 1 for the previous round's sampler - and for the
 * evaluations of two rounds back that read the copy of its outputs it overwrites: the stored tensors are kept in three
 * copies (copy = round mod 3) instead of two.  A component whose producers are done therefore starts its next round while
 * slower components still work on the current one.  Results are bit-identical to the barrier rounds.  With graph mode on,
 * one graph per (component, copy) is replayed.  Differences for the caller: streams[0] is NOT joined with the other
 * streams when ad_step returns - synchronise every stream (or the device) before reading the latent - and
 * ad_get_slot_tensor's slot is the copy 0..2.  With stride S the S evaluations of the last component run on the streams
 * after those of the components, the sampler behind all of them; with the wrapped segmentation the tail waits for the head
 * of its own round.  Cannot be switched in the middle of a run (AD_ERR_STATE).  Warm-up rounds and a trailing partial round
 * are enqueued as before, behind everything the rounds before them left running. */
ad_status ad_set_edge_mode(ad_ctx* ctx, int on);

/* Sampler update of step `step_index` (Section 3.1, Eq. 3, read as deterministic DDIM; or Euler),
 * fused with the guidance combination eps = eps_u + g (eps_c - eps_u) (batch row 0 = conditional):
 *   x  DEVICE fp32 [C][H][W] in place;  eps  DEVICE fp32 [batch][C][H][W].
 * Video model: x and eps are both [frames][C][H][W] and cfg_scale is ignored (no guidance pair). */
ad_status ad_ddim_update(ad_ctx* ctx, void* x, const void* eps, int step_index, float cfg_scale, ad_stream stream);
/* The same kernel on an arbitrary element count (used to measure it at a bandwidth-bound size):
 *   x DEVICE fp32 [n] in place; eps DEVICE fp32 [batch][n]; x' = c_x * x + c_eps * guided eps. */
ad_status ad_sampler_update_raw(void* x, const void* eps, size_t n, int batch, float c_x, float c_eps,
                                float cfg_scale, ad_stream stream);

/* After ad_step: DEVICE pointer of the stored output of `unit` in slot 0/1 (valid for units listed as a
 * component output), and of noise-prediction buffer j (0..stride-1). */
ad_status ad_get_slot_tensor(const ad_ctx* ctx, int slot, int unit, void** ptr, size_t* bytes);
ad_status ad_get_eps_buffer(const ad_ctx* ctx, int j, void** ptr, size_t* bytes);

/* ---- per-launch timing --------------------------------------------------------------------------- *
 * While enabled, every kernel the context launches (ad_component_forward, ad_step, ad_ddim_update) is
 * bracketed by HIP events recorded on the kernel's own stream and tagged with its algorithmic work.
 * ad_profile_get waits for record `index` to finish.  Off by default; costs two event records per launch. */
typedef struct ad_profile_rec {
  char kernel[32];  /* kernel class, e.g. "igemm_bf16_128x128" */
  double flops;     /* algorithmic floating-point operations of the launch (2 per multiply-accumulate) */
  double bytes;     /* algorithmic HBM bytes of the launch (operands read once, results written once) */
  float ms;         /* duration between the two events */
  int m, n, k;      /* GEMM view of the launch (attention: queries, keys, channels); 0 otherwise */
} ad_profile_rec;
ad_status ad_profile_enable(ad_ctx* ctx, int on);
ad_status ad_profile_clear(ad_ctx* ctx);
int ad_profile_count(const ad_ctx* ctx);
ad_status ad_profile_get(const ad_ctx* ctx, int index, ad_profile_rec* out); /* HOST out */

/* ---- single kernels (entry points for kernel-level parity tests and measurements) -------------- *
 * All pointers DEVICE; element type `dtype` (ad_dtype) unless stated.  Tensors NHWC. */

/* Implicit-GEMM convolution / linear layer:  out[m][n] = sum_k A[m][k] W[n][k] (+bias +rowvec +residual).
 *   src0/src1  inputs concatenated on channels (src1 may be NULL, c1 = 0); stored spatial size hs x ws;
 *   up         1: the logical input is the nearest-2x upsampling of the stored one;
 *   ksize 1|3, stride 1|2, padding ksize/2;  w_packed: weights as produced by ad_pack_conv_weight;
 *   bias fp32 [n] or NULL; rowvec fp32 [batch][n] or NULL; residual [m][n] or NULL;
 *   out_mode 0: [m][n] dtype; 1: GEGLU (weights packed with geglu=1) -> [m][n/2]; 2: transposed
 *   [batch][n][ld_t] in dtype; 3: transposed fp32 [batch][n][ld_t]; 4: fused q/k/v projection, n_out = 3c:
 *   columns [0,c) -> out [m][c], [c,2c) -> out2 [m][c], [2c,3c) -> out3, [batch][c][ld_t] when ld_t > 0 else [m][c]
 *   (out2, out3 are ignored by the other modes).
 *   splitk_ws: optional fp32 scratch of splitk_bytes (ad_conv_workspace_bytes); with it, GEMMs with few output
 *   tiles and a long K are split along K and reduced in a second kernel (fixed summation order). */
size_t ad_conv_workspace_bytes(int dtype, int batch, int h_out, int w_out, int n_out, int c_in_total, int ksize, int out_mode);
ad_status ad_conv_forward(int dtype, const void* src0, const void* src1, int c0, int c1, int batch, int hs, int ws,
                          int up, int ksize, int stride, const void* w_packed, int n_out, const float* bias,
                          const float* rowvec, const void* residual, void* out, void* out2, void* out3, int out_mode,
                          int ld_t, void* splitk_ws, size_t splitk_bytes, ad_stream stream);
/* Tuning knob for measurements: forces the block tile of ad_conv_forward and of every convolution / linear
 * layer of the process (1: 128x128 register-staged tiles, 3: 64x64 register-staged tiles, 4: 128x128 two-stage
 * LDS-DMA, 5: 128x128 three-stage LDS-DMA, 6: 256x128 three-stage LDS-DMA, 7: 64x64 three-stage LDS-DMA,
 * 8 / 9: as 5 / 6, with 3x3 stride-1 convolutions on the halo-staged kernel (128 / 256 output positions per workgroup),
 * 10 / 11: as 6 / 5 with four wavefronts per workgroup instead of eight, 12: as 6 with sixteen,
 * -1: automatic choice, the default (3x3 convolutions on the per-tap kernels 5 / 6: measured faster than 8 / 9 on the SD-sized models)).
 * 4 to 9 apply to bf16 GEMMs with a row-major, GEGLU or fused q/k/v output; other calls keep the automatic
 * choice.  Results are the same up to rounding order.  Process-global, not thread-safe: for tests and measurements. */
ad_status ad_tune_conv_tile(int tile);
/* Tuning knob for measurements: order in which the workgroups of a GEMM walk its output tiles.  0: an XCD owns a
 * run of row tiles and every column tile of them (the weights are fetched into every L2); 1: an XCD owns a run of
 * column tiles (the activations are fetched into every L2); -1: automatic, the default (the smaller operand is
 * the one fetched everywhere).  Results are bit-identical. */
ad_status ad_tune_conv_order(int order);
/* Tuning knob for measurements and tests (process-global, not thread-safe): which MFMA attention kernel serves bf16,
 * head_dim 64, transposed v.  0: 32 queries per wavefront, register-staged tiles; 1 / 2: tiles filled by the load
 * unit, lazy maximum, 32 / 64 queries per wavefront; 3: as 1 with the scores of the next 32 keys computed while the
 * exponentials of the current ones run (two workgroups per CU; 4-10 % faster than 1 alone on the GPU, no faster inside the
 * concurrent schedule); -1: automatic, the default (1 beyond 256 keys, else 0).  Same results up to rounding. */
ad_status ad_tune_attention(int variant);
/* Packs HOST fp32 weights [n_out][c_in][k][k] into the kernel layout (HOST out, dtype elements).
 * Returns the packed size in bytes through *bytes when out == NULL. */
ad_status ad_pack_conv_weight(int dtype, const float* w, int n_out, int c_in, int ksize, int geglu, void* out, size_t* bytes);
/* GroupNorm (+SiLU when silu != 0) over the channel concatenation of src0/src1; gamma/beta fp32;
 * scratch: fp32, at least ad_groupnorm_scratch_bytes(); out [batch][hw][c0+c1]. */
size_t ad_groupnorm_scratch_bytes(int batch, int hw, int c);
ad_status ad_groupnorm_forward(int dtype, const void* src0, const void* src1, int c0, int c1, int batch, int hw,
                               int groups, const float* gamma, const float* beta, float eps, int silu,
                               void* out, void* scratch, ad_stream stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): ad_groupnorm_forward with the partial sums kept in a fixed 512 KiB device array of the
 * library instead of a caller-supplied scratch buffer.  Same kernels, same results bit for bit.  Calls no
 * hipMalloc / hipFree.  Limit: 2 * batch * min(64, max(1, hw / 8)) * groups * 8 bytes <= 512 KiB (e.g. batch 16 with
 * 32 groups), else AD_ERR_NOMEM.  Every call on a GPU shares that GPU's array: calls that overlap on one GPU
 * (different streams, or threads) race; calls on one stream are ordered and need no clearing in between. */
ad_status ad_groupnorm_forward_static(int dtype, const void* src0, const void* src1, int c0, int c1, int batch, int hw,
                                      int groups, const float* gamma, const float* beta, float eps, int silu,
                                      void* out, ad_stream stream);
ad_status ad_layernorm_forward(int dtype, const void* src, int rows, int c, const float* gamma, const float* beta,
                               float eps, void* out, ad_stream stream);
/* Multi-head attention out[b][l][h*d+j] = softmax(q k^T / sqrt(d)) v, heads = c / head_dim.
 *   q [batch][l][ldq], k [batch][lk][ldk], out [batch][l][ldo] (leading dimensions in elements);
 *   v_is_transposed 0: v [batch][lk][ldv]; 1: v [batch][c][ldv] (keys contiguous, ldv >= lk rounded up to 64).
 *   The MFMA kernel is used for bf16, head_dim 64, transposed v; the generic kernel otherwise. */
ad_status ad_attention_forward(int dtype, const void* q, const void* k, const void* v, int v_is_transposed,
                               int batch, int l, int lk, int c, int head_dim, int ldq, int ldk, int ldv, int ldo,
                               void* out, ad_stream stream);

/* Attention over the frame axis (temporal layer of the video model): at each of `positions` spatial positions the
 * `frames` (<= 16) rows f * positions + p, f = 0..frames-1, are one sequence; heads of width c / heads;
 * out[row][h*d+j] = softmax(q k^T / sqrt(d)) v within the sequence.  q, k, v, out: [frames*positions][ld*]. */
ad_status ad_attention_frames_forward(int dtype, const void* q, const void* k, const void* v, int frames, int positions,
                                      int c, int heads, int ldq, int ldk, int ldv, int ldo, void* out, ad_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* ASYNCDIFF_H */
