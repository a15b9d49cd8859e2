// Component runtime: weight upload, evaluation of one component (a contiguous unit range) on a
// stream, and the round driver that runs the schedule table over the caller's streams with the
// double-buffered stored states.
#include <cstdio>
#include <cstring>

#include "ad_internal.h"
#include "ad_kernels.h"

namespace ad {

static inline Ctx* C(ad_ctx* p) { return reinterpret_cast<Ctx*>(p); }
static inline const Ctx* C(const ad_ctx* p) { return reinterpret_cast<const Ctx*>(p); }

#define AD_TRY(expr)                  \
  do {                                \
    ad_status st_ = (expr);           \
    if (st_ != AD_OK) return st_;     \
  } while (0)

// Device-side view of the weights of one evaluation.
struct WView {
  const Ctx& c;
  const void* at(int idx) const { return c.weights_dev + c.weights[idx].dev_off; }
  const float* f32(int idx) const { return (const float*)at(idx); }
};

struct Eval {
  Ctx& c;
  const Component& cp;
  const Workspace& ws;
  const void* const* in;
  void* const* out;
  const void* text;
  hipStream_t s;
  int dt;
  const float* proj = nullptr;   // fused time projection of the component's ResBlocks [batch][proj_ld]
  int proj_ld = 0;

  char* work(size_t off) const { return c.work_dev + off; }
  void* temp(int t) const { return ws.temp_bytes[t] ? work(ws.temp_off[t]) : nullptr; }
  float* f32area() const { return (float*)work(ws.f32_off); }

  // tensor produced by `unit` (may live outside this component)
  const void* tensor_in(int unit) const {
    if (unit >= cp.first && unit <= cp.last) return tensor_out(unit);
    for (size_t i = 0; i < cp.in_units.size(); ++i)
      if (cp.in_units[i] == unit) return in[i];
    return nullptr;
  }
  void* tensor_out(int unit) const {
    const size_t off = ws.unit_off[unit - cp.first];
    if (off != SIZE_MAX) return work(off);
    for (size_t i = 0; i < cp.out_units.size(); ++i)
      if (cp.out_units[i] == unit) return out[i];
    return nullptr;
  }

  ad_status conv(const void* src0, const void* src1, int c0, int c1, int hs, int wsz, int up, int ksize, int stride,
                 int w_idx, int b_idx, const float* rowvec, const void* residual, void* dst, int mode = OUT_ROWMAJOR,
                 int ld_t = 0) const {
    WView wv{c};
    ConvArgs a{dt, src0, src1, c0, c1, c.cfg.batch, hs, wsz, up, ksize, stride, wv.at(w_idx), c.weights[w_idx].info.shape[0],
               b_idx >= 0 ? wv.f32(b_idx) : nullptr, rowvec, proj_ld, residual, dst, mode, ld_t, temp(9), ws.temp_bytes[9]};
    return launch_conv(a, s);
  }
  // linear layer on a [rows][cin] matrix
  ad_status linear(const void* src, int rows, int cin, int w_idx, int b_idx, const void* residual, void* dst,
                   int mode = OUT_ROWMAJOR, int batch = 1, int ld_t = 0) const {
    WView wv{c};
    ConvArgs a{dt, src, nullptr, cin, 0, batch, rows / batch, 1, 0, 1, 1, wv.at(w_idx), c.weights[w_idx].info.shape[0],
               b_idx >= 0 ? wv.f32(b_idx) : nullptr, nullptr, 0, residual, dst, mode, ld_t, temp(9), ws.temp_bytes[9]};
    return launch_conv(a, s);
  }
  ad_status gn(const void* src0, const void* src1, int c0, int c1, int hw, int g_idx, int silu, void* dst) const {
    WView wv{c};
    return launch_groupnorm(dt, src0, src1, c0, c1, c.cfg.batch, hw, c.cfg.gn_groups, wv.f32(g_idx), wv.f32(g_idx + 1),
                            c.cfg.gn_eps, silu, dst, work(ws.gn_off), c.gn_bytes, s);
  }
  ad_status ln(const void* src, int rows, int ch, int g_idx, void* dst) const {
    WView wv{c};
    return launch_layernorm(dt, src, rows, ch, wv.f32(g_idx), wv.f32(g_idx + 1), c.cfg.ln_eps, dst, s);
  }

  ad_status res(const Unit& u, int ui) const {
    const ad_unit_info& f = u.info;
    const int hw = f.h_in * f.w_in, ci = f.c_in + f.c_skip, w0 = u.w_first;
    const void* x0 = tensor_in(ui - 1);
    const void* x1 = f.skip_from >= 0 ? tensor_in(f.skip_from) : nullptr;
    if (!x0 || (f.skip_from >= 0 && !x1)) AD_FAIL(AD_ERR_STATE, "unit %s: missing input", f.name);
    // manifest order: gn1.g gn1.b conv1.w conv1.b temb.w temb.b gn2.g gn2.b conv2.w conv2.b [short.w short.b]
    AD_TRY(gn(x0, x1, f.c_in, f.c_skip, hw, w0 + 0, 1, temp(0)));
    // conv1 adds this block's slice of the fused time projection per (sample, channel)
    const float* rowvec = proj + (u.temb_row - cp.temb_row0);
    AD_TRY(conv(temp(0), nullptr, ci, 0, f.h_in, f.w_in, 0, 3, 1, w0 + 2, w0 + 3, rowvec, nullptr, temp(1)));
    AD_TRY(gn(temp(1), nullptr, f.c_out, 0, hw, w0 + 6, 1, temp(0)));
    const void* shortcut = x0;
    if (ci != f.c_out) {
      AD_TRY(conv(x0, x1, f.c_in, f.c_skip, f.h_in, f.w_in, 0, 1, 1, w0 + 10, w0 + 11, nullptr, nullptr, temp(2)));
      shortcut = temp(2);
    }
    return conv(temp(0), nullptr, f.c_out, 0, f.h_in, f.w_in, 0, 3, 1, w0 + 8, w0 + 9, nullptr, shortcut, tensor_out(ui));
  }
  // cross-attention key / value projections of the text embedding for the layer whose weights start at w
  ad_status text_kv(int w, void* kdst, void* vdst) const {
    const int B = c.cfg.frames > 0 ? 1 : c.cfg.batch;        // a video has one text embedding for all frames
    const int Lk = c.cfg.ctx_len, lkp = round_up(Lk, 64);
    const bool vt = dt == AD_BF16 && c.cfg.head_dim == 64;
    AD_TRY(linear(text, B * Lk, c.cfg.ctx_dim, w + 10, -1, nullptr, kdst));
    if (vt) return linear(text, B * Lk, c.cfg.ctx_dim, w + 11, -1, nullptr, vdst, OUT_TRANSPOSED, B, lkp);
    return linear(text, B * Lk, c.cfg.ctx_dim, w + 11, -1, nullptr, vdst);
  }

  ad_status tfm(const Unit& u, int ui) const {
    const ad_unit_info& f = u.info;
    const int B = c.cfg.batch, L = f.h_in * f.w_in, Cc = f.c_in, M = B * L, d = c.cfg.head_dim;
    const int Lk = c.cfg.ctx_len, lp = round_up(L, 64), lkp = round_up(Lk, 64);
    const bool vt = dt == AD_BF16 && d == 64;          // transposed V feeds the MFMA attention kernel
    const void* x = tensor_in(ui - 1);
    if (!x) AD_FAIL(AD_ERR_STATE, "unit %s: missing input", f.name);
    int w = u.w_first;
    // gn.g gn.b proj_in.w proj_in.b | per layer 20 entries | proj_out.w proj_out.b
    AD_TRY(gn(x, nullptr, Cc, 0, L, w + 0, 0, temp(0)));
    AD_TRY(linear(temp(0), M, Cc, w + 2, w + 3, nullptr, temp(1)));
    w += 4;
    void* h = temp(1);
    for (int k = 0; k < f.depth; ++k, w += 20) {
      // ln1.g ln1.b a1.q a1.k a1.v a1.o.w a1.o.b ln2.g ln2.b a2.q a2.k a2.v a2.o.w a2.o.b ln3.g ln3.b ff1.w ff1.b ff2.w ff2.b
      AD_TRY(ln(h, M, Cc, w + 0, temp(0)));
      {   // q, k, v of the self-attention in one GEMM; v lands transposed when the MFMA attention kernel follows
        WView wv{c};
        ConvArgs a{dt, temp(0), nullptr, Cc, 0, B, L, 1, 0, 1, 1, wv.at(w + 2), 3 * Cc, nullptr, nullptr, 0, nullptr, temp(2), OUT_QKV,
                   vt ? lp : 0, temp(9), ws.temp_bytes[9], temp(3), temp(4)};
        AD_TRY(launch_conv(a, s));
      }
      AD_TRY(launch_attention(dt, temp(2), temp(3), temp(4), vt, B, L, L, Cc, d, Cc, Cc, vt ? lp : Cc, Cc, temp(5), s));
      AD_TRY(linear(temp(5), M, Cc, w + 5, w + 6, h, h));
      AD_TRY(ln(h, M, Cc, w + 7, temp(0)));
      AD_TRY(linear(temp(0), M, Cc, w + 9, -1, nullptr, temp(2)));
      // keys / values of the text: taken from the per-run cache when it was built from this embedding
      const void* tk = temp(7);
      const void* tv = temp(8);
      if (c.text_cached == text) {
        tk = work(c.text_k_off[ui][k]);
        tv = work(c.text_v_off[ui][k]);
      } else {
        AD_TRY(text_kv(w, temp(7), temp(8)));
      }
      // video: every frame attends to the one text embedding, so the frames' tokens form one long query sequence
      if (c.cfg.frames > 0) AD_TRY(launch_attention(dt, temp(2), tk, tv, vt, 1, M, Lk, Cc, d, Cc, Cc, vt ? lkp : Cc, Cc, temp(5), s));
      else AD_TRY(launch_attention(dt, temp(2), tk, tv, vt, B, L, Lk, Cc, d, Cc, Cc, vt ? lkp : Cc, Cc, temp(5), s));
      AD_TRY(linear(temp(5), M, Cc, w + 12, w + 13, h, h));
      AD_TRY(ln(h, M, Cc, w + 14, temp(0)));
      AD_TRY(linear(temp(0), M, Cc, w + 16, w + 17, nullptr, temp(6), OUT_GEGLU));
      AD_TRY(linear(temp(6), M, 4 * Cc, w + 18, w + 19, h, h));
    }
    void* z = tensor_out(ui);
    AD_TRY(linear(h, M, Cc, w + 0, w + 1, x, z));
    if (c.cfg.temporal_heads == 0) return AD_OK;
    // temporal layer: temp.ln.g temp.ln.b temp.q temp.k temp.v temp.o.w temp.o.b; tokens = the frames of one position
    w += 2;
    AD_TRY(ln(z, M, Cc, w + 0, temp(0)));
    {
      WView wv{c};
      ConvArgs a{dt, temp(0), nullptr, Cc, 0, B, L, 1, 0, 1, 1, wv.at(w + 2), 3 * Cc, nullptr, nullptr, 0, nullptr, temp(2), OUT_QKV,
                 0, temp(9), ws.temp_bytes[9], temp(3), temp(4)};
      AD_TRY(launch_conv(a, s));
    }
    AD_TRY(launch_attention_frames(dt, temp(2), temp(3), temp(4), c.cfg.frames, L, Cc, c.cfg.temporal_heads, Cc, Cc, Cc, Cc, temp(5), s));
    return linear(temp(5), M, Cc, w + 5, w + 6, z, z);
  }
};

// temb = Lin2(SiLU(Lin1(sinusoid(tau)))) (+ pooled branch), then every ResBlock projection of the
// component in one launch: proj[b][row] = temb_b[row] + sum_k SiLU(temb[b][k]) W[row][k].
static ad_status time_projection(Eval& e, int tau, StepRef tau_ref, const void* pooled) {
  Ctx& c = e.c;
  // without the pooled branch every batch row has the same embedding: one row is computed and shared
  const int B = c.cfg.pooled_dim > 0 ? c.cfg.batch : 1;
  const int td = c.temb_dim, c0 = c.cfg.channels[0], dt = e.dt;
  float* sinus = e.f32area();
  float* t1 = sinus + c0;
  float* temb = t1 + (size_t)B * td;
  float* pool1 = temb + (size_t)B * td;
  float* proj = pool1 + 2 * (size_t)B * td;
  WView wv{c};
  AD_TRY(launch_sinusoid((float)tau, tau_ref, c0, sinus, e.s));
  // the sinusoid is the same for every batch row: evaluate the MLP on one row, broadcast below
  AD_TRY(launch_linear_rows(dt, sinus, 0, 1, c0, wv.at(0), wv.f32(1), td, 0, 1, 0, t1, e.s));
  AD_TRY(launch_linear_rows(dt, t1, 0, B, td, wv.at(2), wv.f32(3), td, 0, 0, 0, temb, e.s));
  if (c.cfg.pooled_dim > 0) {
    if (!pooled) AD_FAIL(AD_ERR_INVALID, "pooled embedding required by this configuration");
    AD_TRY(launch_linear_rows(dt, (const float*)pooled, c.cfg.pooled_dim, B, c.cfg.pooled_dim, wv.at(4), wv.f32(5), td, 0, 1, 0, pool1, e.s));
    AD_TRY(launch_linear_rows(dt, pool1, td, B, td, wv.at(6), wv.f32(7), td, 0, 0, 1, temb, e.s));
  }
  e.proj = proj;
  e.proj_ld = c.cfg.pooled_dim > 0 ? e.cp.temb_rows : -1;
  if (e.cp.temb_rows > 0) {
    const char* wmat = c.weights_dev + c.temb_w_off + (size_t)e.cp.temb_row0 * td * esize(dt);
    const float* bvec = (const float*)(c.weights_dev + c.temb_b_off) + e.cp.temb_row0;
    AD_TRY(launch_linear_rows(dt, temb, td, B, td, wmat, bvec, e.cp.temb_rows, 1, 0, 0, proj, e.s));
  }
  return AD_OK;
}

static ad_status run_component(Ctx& c, int comp, int lane, const void* const* in, int tau, float latent_scale,
                               const void* text, const void* pooled, void* const* out, hipStream_t s,
                               hipEvent_t latent_consumed = nullptr, StepRef tau_ref = StepRef{}, StepRef scale_ref = StepRef{}) {
  const Component& cp = c.comps[comp - 1];
  Eval e{c, cp, c.ws[comp - 1][lane], in, out, text, s, c.cfg.dtype};
  const ad_unet_cfg& g = c.cfg;
  AD_TRY(time_projection(e, tau, tau_ref, pooled));
  for (int ui = cp.first; ui <= cp.last; ++ui) {
    const Unit& u = c.units[ui];
    const ad_unit_info& f = u.info;
    switch (f.kind) {
      case AD_UNIT_CONV_IN: {
        const void* latent = e.tensor_in(-1);
        if (!latent) AD_FAIL(AD_ERR_STATE, "conv_in: missing latent");
        AD_TRY(launch_pack_latent(e.dt, (const float*)latent, g.frames > 0, latent_scale, scale_ref, g.latent_channels, g.height, g.width, g.batch, e.temp(0), s));
        if (latent_consumed) AD_HIP(hipEventRecord(latent_consumed, s));
        {   // a 1x1 GEMM over the im2col'ed latent: K = 9 latent channels zero-padded to kConvInK
          WView wv{c};
          ConvArgs a{e.dt, e.temp(0), nullptr, kConvInK, 0, g.batch, g.height, g.width, 0, 1, 1, wv.at(u.w_first), c.weights[u.w_first].info.shape[0],
                     wv.f32(u.w_first + 1), nullptr, 0, nullptr, e.tensor_out(ui), OUT_ROWMAJOR, 0, e.temp(9), e.ws.temp_bytes[9]};
          a.k_real = 9 * g.latent_channels;
          AD_TRY(launch_conv(a, s));
        }
        break;
      }
      case AD_UNIT_RES: {
        AD_TRY(e.res(u, ui));
        break;
      }
      case AD_UNIT_TFM: AD_TRY(e.tfm(u, ui)); break;
      case AD_UNIT_DOWN:
        AD_TRY(e.conv(e.tensor_in(ui - 1), nullptr, f.c_in, 0, f.h_in, f.w_in, 0, 3, 2, u.w_first, u.w_first + 1, nullptr, nullptr, e.tensor_out(ui)));
        break;
      case AD_UNIT_UP:
        AD_TRY(e.conv(e.tensor_in(ui - 1), nullptr, f.c_in, 0, f.h_in, f.w_in, 1, 3, 1, u.w_first, u.w_first + 1, nullptr, nullptr, e.tensor_out(ui)));
        break;
      case AD_UNIT_OUT:
        AD_TRY(e.gn(e.tensor_in(ui - 1), nullptr, f.c_in, 0, f.h_in * f.w_in, u.w_first, 1, e.temp(0)));
        AD_TRY(e.conv(e.temp(0), nullptr, f.c_in, 0, f.h_in, f.w_in, 0, 3, 1, u.w_first + 2, u.w_first + 3, nullptr, nullptr,
                      e.tensor_out(ui), OUT_TRANSPOSED_F32, f.h_out * f.w_out));
        break;
    }
  }
  return AD_OK;
}

// Cross-attention keys and values depend only on the text embedding: compute them once per run.
static ad_status precompute_text(Ctx& c, const void* text, hipStream_t s) {
  static const void* const no_in[1] = {nullptr};
  static void* const no_out[1] = {nullptr};
  c.text_cached = nullptr;
  for (int ui = 0; ui < (int)c.units.size(); ++ui) {
    const Unit& u = c.units[ui];
    if (u.info.kind != AD_UNIT_TFM) continue;
    const int comp = u.comp;
    Eval e{c, c.comps[comp - 1], c.ws[comp - 1][0], no_in, no_out, text, s, c.cfg.dtype};
    for (int k = 0; k < u.info.depth; ++k)
      AD_TRY(e.text_kv(u.w_first + 4 + 20 * k, c.work_dev + c.text_k_off[ui][k], c.work_dev + c.text_v_off[ui][k]));
  }
  c.text_cached = text;
  return AD_OK;
}

}  // namespace ad

using namespace ad;

extern "C" {

static Profiler* prof_of(const Ctx& c) { return (Profiler*)c.profiler; }

static void prof_clear(Profiler* p) {
  for (ProfRec& r : p->recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  p->recs.clear();
}

ad_status ad_profile_enable(ad_ctx* ctx, int on) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (!c.profiler) c.profiler = new Profiler();
  prof_of(c)->on = on != 0;
  return AD_OK;
}

ad_status ad_profile_clear(ad_ctx* ctx) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (C(ctx)->profiler) prof_clear(prof_of(*C(ctx)));
  return AD_OK;
}

int ad_profile_count(const ad_ctx* ctx) { return (ctx && C(ctx)->profiler) ? (int)prof_of(*C(ctx))->recs.size() : 0; }

ad_status ad_profile_get(const ad_ctx* ctx, int index, ad_profile_rec* out) {
  if (!ctx || !out) AD_FAIL(AD_ERR_INVALID, "null argument");
  const Ctx& c = *C(ctx);
  if (!c.profiler || index < 0 || index >= (int)prof_of(c)->recs.size()) AD_FAIL(AD_ERR_INVALID, "record %d out of range", index);
  const ProfRec& r = prof_of(c)->recs[index];
  AD_HIP(hipEventSynchronize(r.stop));
  float ms = 0.f;
  AD_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
  std::snprintf(out->kernel, sizeof(out->kernel), "%s", r.name);
  out->flops = r.flops; out->bytes = r.bytes; out->ms = ms;
  out->m = r.m; out->n = r.n; out->k = r.k;
  return AD_OK;
}

void ad_destroy(ad_ctx* ctx) {
  if (!ctx) return;
  Ctx* c = C(ctx);
  if (c->profiler) { prof_clear(prof_of(*c)); delete prof_of(*c); }
  for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
  if (c->ev_pack) (void)hipEventDestroy(c->ev_pack);
  bool replayed = c->round_graph[0].exec || c->round_graph[1].exec;
  for (auto& g : c->comp_graph) replayed = replayed || g.exec;
  if (replayed) (void)hipDeviceSynchronize();
  for (auto& g : c->round_graph) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.graph) (void)hipGraphDestroy(g.graph);
  }
  for (auto& g : c->comp_graph) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.graph) (void)hipGraphDestroy(g.graph);
  }
  for (hipEvent_t e : c->ev_done)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_sampler)
    if (e) (void)hipEventDestroy(e);
  delete c;
}

ad_status ad_bind_device_memory(ad_ctx* ctx, void* weights_dev, size_t weight_bytes, void* work_dev, size_t work_bytes) {
  if (!ctx || !weights_dev || !work_dev) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (weight_bytes < c.weight_bytes || work_bytes < c.work_bytes)
    AD_FAIL(AD_ERR_NOMEM, "arenas too small: need %zu + %zu bytes", c.weight_bytes, c.work_bytes);
  if (((uintptr_t)weights_dev | (uintptr_t)work_dev) % kAlign) AD_FAIL(AD_ERR_INVALID, "arenas must be %zu-byte aligned", kAlign);
  c.weights_dev = (char*)weights_dev;
  c.work_dev = (char*)work_dev;
  c.weights_loaded = false;
  return AD_OK;
}

ad_status ad_load_weights(ad_ctx* ctx, const float* const* host_ptrs, int n) {
  if (!ctx || !host_ptrs) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (!c.weights_dev) AD_FAIL(AD_ERR_STATE, "ad_bind_device_memory has not been called");
  if (n != (int)c.weights.size()) AD_FAIL(AD_ERR_INVALID, "expected %zu weight tensors, got %d", c.weights.size(), n);
  const int dt = c.cfg.dtype;
  std::vector<char> stage;
  for (int i = 0; i < n; ++i)
    if (!host_ptrs[i]) AD_FAIL(AD_ERR_INVALID, "weight %d (%s) is null", i, c.weights[i].info.name);
  // the fused time-projection matrix is assembled from the ResBlocks' rows
  std::vector<char> temb_w((size_t)c.temb_rows_total * c.temb_dim * esize(dt));
  std::vector<float> temb_b((size_t)c.temb_rows_total);
  size_t temb_row = 0;
  for (int i = 0; i < n; ++i) {
    const Weight& w = c.weights[i];
    const int* sh = w.info.shape;
    const float* src = host_ptrs[i];
    if (w.role == W_TEMB) {
      pack_rows(dt, src, (size_t)sh[0] * sh[1], temb_w.data() + temb_row * c.temb_dim * esize(dt));
      continue;
    }
    if (w.role == W_QKV_KV) continue;     // packed together with q
    if (w.role == W_QKV_Q) {
      const size_t each = (size_t)sh[0] * sh[1];
      std::vector<float> cat(3 * each);
      for (int j = 0; j < 3; ++j) std::memcpy(cat.data() + j * each, host_ptrs[i + j], each * 4);
      stage.assign(w.dev_bytes, 0);
      pack_conv(dt, cat.data(), 3 * sh[0], sh[1], 1, false, stage.data());
      AD_HIP(hipMemcpy(c.weights_dev + w.dev_off, stage.data(), w.dev_bytes, hipMemcpyHostToDevice));
      continue;
    }
    if (w.role == W_TEMB_BIAS) {
      std::memcpy(temb_b.data() + temb_row, src, (size_t)sh[0] * 4);
      temb_row += sh[0];
      continue;
    }
    stage.assign(w.dev_bytes, 0);
    switch (w.role) {
      case W_CONV3: pack_conv(dt, src, sh[0], sh[1], 3, false, stage.data()); break;
      case W_CONV1: pack_conv(dt, src, sh[0], sh[1], 1, false, stage.data()); break;
      case W_GEGLU: pack_conv(dt, src, sh[0], sh[1], 1, true, stage.data()); break;
      case W_CONV_IN: {
        // K index = tap * c_in + channel, padded to kConvInK
        std::vector<float> tmp((size_t)sh[0] * kConvInK, 0.f);
        for (int o = 0; o < sh[0]; ++o)
          for (int ci = 0; ci < sh[1]; ++ci)
            for (int t = 0; t < 9; ++t) tmp[(size_t)o * kConvInK + t * sh[1] + ci] = src[((size_t)o * sh[1] + ci) * 9 + t];
        pack_rows(dt, tmp.data(), tmp.size(), stage.data());
        break;
      }
      case W_SMALL: pack_rows(dt, src, (size_t)sh[0] * sh[1], stage.data()); break;
      case W_VEC_F32: std::memcpy(stage.data(), src, (size_t)sh[0] * 4); break;
      case W_GEGLU_BIAS: {
        float* dst = (float*)stage.data();
        const int half = sh[0] / 2;
        for (int r = 0; r < sh[0]; ++r) {
          const int blk = r / 64, in = r % 64;
          dst[r] = src[in < 32 ? blk * 32 + in : half + blk * 32 + in - 32];
        }
        break;
      }
      default: break;
    }
    AD_HIP(hipMemcpy(c.weights_dev + w.dev_off, stage.data(), w.dev_bytes, hipMemcpyHostToDevice));
  }
  if (c.temb_rows_total > 0) {
    AD_HIP(hipMemcpy(c.weights_dev + c.temb_w_off, temb_w.data(), temb_w.size(), hipMemcpyHostToDevice));
    AD_HIP(hipMemcpy(c.weights_dev + c.temb_b_off, temb_b.data(), temb_b.size() * 4, hipMemcpyHostToDevice));
  }
  AD_HIP(hipDeviceSynchronize());
  c.weights_loaded = true;
  return AD_OK;
}

ad_status ad_component_forward(ad_ctx* ctx, int comp, int lane, const void* const* hidden_in, int t_index,
                               float latent_scale, const void* text_emb, const void* pooled_emb,
                               void* const* hidden_out, ad_stream stream) {
  if (!ctx || !hidden_in || !hidden_out) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (!c.weights_loaded) AD_FAIL(AD_ERR_STATE, "weights are not loaded");
  if (c.T == 0) AD_FAIL(AD_ERR_STATE, "ad_reset has not been called");
  if (comp < 1 || comp > c.N) AD_FAIL(AD_ERR_INVALID, "component %d out of range", comp);
  if (lane < 0 || lane >= (int)c.ws[comp - 1].size()) AD_FAIL(AD_ERR_INVALID, "lane %d out of range for component %d", lane, comp);
  if (t_index < 0 || t_index >= c.T) AD_FAIL(AD_ERR_INVALID, "t_index %d out of range", t_index);
  const Component& cp = c.comps[comp - 1];
  for (size_t i = 0; i < cp.in_units.size(); ++i) if (!hidden_in[i]) AD_FAIL(AD_ERR_INVALID, "hidden_in[%zu] is null", i);
  for (size_t i = 0; i < cp.out_units.size(); ++i) if (!hidden_out[i]) AD_FAIL(AD_ERR_INVALID, "hidden_out[%zu] is null", i);
  bool needs_text = false;
  for (int i = cp.first; i <= cp.last; ++i) needs_text |= c.units[i].info.kind == AD_UNIT_TFM;
  if (needs_text && !text_emb) AD_FAIL(AD_ERR_INVALID, "text_emb is null");
  set_profiler(prof_of(c));
  ad_status st = run_component(c, comp, lane, hidden_in, c.taus[t_index], latent_scale, text_emb, pooled_emb, hidden_out, (hipStream_t)stream);
  set_profiler(nullptr);
  return st;
}

ad_status ad_precompute_text(ad_ctx* ctx, const void* text_emb, ad_stream stream) {
  if (!ctx || !text_emb) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (!c.weights_loaded) AD_FAIL(AD_ERR_STATE, "weights are not loaded");
  set_profiler(prof_of(c));
  ad_status st = precompute_text(c, text_emb, (hipStream_t)stream);
  set_profiler(nullptr);
  return st;
}

ad_status ad_ddim_update(ad_ctx* ctx, void* x, const void* eps, int step_index, float cfg_scale, ad_stream stream) {
  if (!ctx || !x || !eps) AD_FAIL(AD_ERR_INVALID, "null argument");
  const Ctx& c = *C(ctx);
  if (c.T == 0) AD_FAIL(AD_ERR_STATE, "ad_reset has not been called");
  if (step_index < 0 || step_index >= c.T) AD_FAIL(AD_ERR_INVALID, "step %d out of range", step_index);
  double cx, ce, s0, s1;
  sampler_coeffs(c, step_index, &cx, &ce, &s0, &s1);
  // video: one latent per frame and no guidance, i.e. one long vector with a single row of predictions
  const size_t n = (size_t)(c.cfg.frames > 0 ? c.cfg.frames : 1) * c.cfg.latent_channels * c.cfg.height * c.cfg.width;
  set_profiler(prof_of(c));
  ad_status st = launch_sampler((float*)x, (const float*)eps, n, c.cfg.frames > 0 ? 1 : c.cfg.batch, (float)cx, (float)ce, StepRef{}, cfg_scale, (hipStream_t)stream);
  set_profiler(nullptr);
  return st;
}

ad_status ad_get_slot_tensor(const ad_ctx* ctx, int slot, int unit, void** ptr, size_t* bytes) {
  if (!ctx || !ptr) AD_FAIL(AD_ERR_INVALID, "null argument");
  const Ctx& c = *C(ctx);
  if (slot < 0 || slot > 2 || unit < 0 || unit >= (int)c.units.size()) AD_FAIL(AD_ERR_INVALID, "slot/unit out of range");
  if (c.slot_off[slot][unit] == SIZE_MAX) AD_FAIL(AD_ERR_INVALID, "unit %d is not a stored component output", unit);
  if (!c.work_dev) AD_FAIL(AD_ERR_STATE, "no device memory bound");
  *ptr = c.work_dev + c.slot_off[slot][unit];
  if (bytes) *bytes = tensor_bytes(c, unit);
  return AD_OK;
}

ad_status ad_get_eps_buffer(const ad_ctx* ctx, int j, void** ptr, size_t* bytes) {
  if (!ctx || !ptr) AD_FAIL(AD_ERR_INVALID, "null argument");
  const Ctx& c = *C(ctx);
  if (j < 0 || j >= c.stride) AD_FAIL(AD_ERR_INVALID, "buffer %d out of range", j);
  if (!c.work_dev) AD_FAIL(AD_ERR_STATE, "no device memory bound");
  *ptr = c.work_dev + c.eps_off[j];
  if (bytes) *bytes = tensor_bytes(c, (int)c.units.size() - 1);
  return AD_OK;
}

// Which copy of the stored tensors a schedule row reads and writes.  Barrier mode: the table's two slots.  Per-edge mode:
// copy = round mod 3 for what a round writes, the round before for what an asynchronous round reads (a warm-up round
// reads what it has just written).
static inline int phys_write(const Ctx& c, const ad_sched_row& row) { return c.edge_mode ? row.round % 3 : row.write_slot; }
static inline int phys_read(const Ctx& c, const ad_sched_row& row) {
  if (!c.edge_mode) return row.read_slot;
  return row.read_slot == row.write_slot ? row.round % 3 : (row.round + 2) % 3;
}
static inline hipEvent_t& ev_done_of(Ctx& c, int comp, int round) { return c.ev_done[(size_t)(comp - 1) * 4 + (round & 3)]; }

// One asynchronous round without a barrier (per-edge mode).  Component n runs on
// streams[(n - 1) % ns], the S evaluations of the last component (stride S) on the streams after it.  Before an
// evaluation starts it waits for (a) the evaluations of the previous round whose stored tensors it reads - for component 1
// that is the sampler of the previous round, which also stands for the last component - and (b) the evaluations of two
// rounds back that read the copy it is about to overwrite.  The sampler follows the last evaluation of the last component
// on its stream, behind the other ones of that component and behind this round's component 1 (which has read the latent).
// Nothing joins the streams: a component whose producers are done starts its next round while slower components still work
// on this one.  graphs: replay one captured graph per (evaluation, copy) instead of launching the kernels.
static ad_status enqueue_round_edges(Ctx& c, size_t r0, size_t r1, void* latent, const void* text_emb, const void* pooled_emb,
                                     const ad_stream* streams, int ns, bool graphs, std::vector<int>* steps_out) {
  const int nu = (int)c.units.size();
  const int S = c.stride;
  const StepRec* table = (const StepRec*)(c.work_dev + c.step_table_off);
  int* counters = (int*)(c.work_dev + c.step_counter_off);
  const int base = c.steps_done;
  const int g = c.rows[r0].round;
  const size_t n = (size_t)(c.cfg.frames > 0 ? c.cfg.frames : 1) * c.cfg.latent_channels * c.cfg.height * c.cfg.width;
  std::vector<hipStream_t> lane_stream;
  std::vector<int> lane_eps_off, lane_step;
  for (size_t r = r0; r < r1; ++r) {
    const ad_sched_row& row = c.rows[r];
    const int e = (int)(r - r0);                       // evaluation index within the round
    const int lane = e < c.N - 1 ? 0 : e - (c.N - 1);
    if (row.comp != (e < c.N - 1 ? e + 1 : c.N)) AD_FAIL(AD_ERR_STATE, "per-edge mode: a round lists its components in order");
    const Component& cp = c.comps[row.comp - 1];
    hipStream_t s = (hipStream_t)streams[e % ns];
    if (cp.in_units.size() > 64 || cp.out_units.size() > 64) AD_FAIL(AD_ERR_INVALID, "too many component tensors");
    // (a) producers of the previous round; the tail of the wrapped segmentation reads the head of its own round
    bool waited[64] = {false};
    for (int u : cp.in_units) {
      if (u < 0) { AD_HIP(hipStreamWaitEvent(s, c.ev_sampler[(g + 3) & 3], 0)); continue; }
      const int m = c.units[u].comp;
      if (m == row.comp || waited[m]) continue;
      waited[m] = true;
      AD_HIP(hipStreamWaitEvent(s, ev_done_of(c, m, m == row.fresh_from ? g : g - 1), 0));
    }
    // the noise-prediction buffer of this lane was read by the previous round's sampler, possibly on another stream
    if (row.comp == c.N && c.N > 1) AD_HIP(hipStreamWaitEvent(s, c.ev_sampler[(g + 3) & 3], 0));
    // (b) readers, two rounds back, of the copy written now
    bool reader[64] = {false};
    for (int m = 1; m <= c.N; ++m) {
      if (m == row.comp) continue;
      for (int u : c.comps[m - 1].in_units)
        if (u >= 0 && c.units[u].comp == row.comp) reader[m] = true;
    }
    for (int m = 1; m <= c.N; ++m)
      if (reader[m]) AD_HIP(hipStreamWaitEvent(s, ev_done_of(c, m, g - 2), 0));

    const void* in[64];
    void* out[64];
    for (size_t i = 0; i < cp.in_units.size(); ++i) {
      const int u = cp.in_units[i];
      if (u < 0) { in[i] = latent; continue; }
      const bool fresh = row.fresh_from > 0 && c.units[u].comp == row.fresh_from;
      in[i] = c.work_dev + c.slot_off[fresh ? phys_write(c, row) : phys_read(c, row)][u];
    }
    for (size_t i = 0; i < cp.out_units.size(); ++i) {
      const int u = cp.out_units[i];
      if (u == nu - 1) out[i] = c.work_dev + c.eps_off[lane];
      else if (row.write_slot >= 0) out[i] = c.work_dev + c.slot_off[phys_write(c, row)][u];
      else AD_FAIL(AD_ERR_STATE, "schedule row drops a stored tensor");
    }
    int* counter = counters + row.comp;
    const int tau_off = row.tau_step - base, latent_off = row.latent_step >= 0 ? row.latent_step - base : 0;
    const int eps_off = row.eps_step >= 0 ? row.eps_step - base : INT32_MIN;
    auto work = [&]() -> ad_status {
      AD_TRY(run_component(c, row.comp, lane, in, c.taus[row.tau_step], 1.f, text_emb, pooled_emb, out, s, nullptr,
                           StepRef{table, counter, tau_off}, StepRef{table, counter, latent_off}));
      if (row.eps_step < 0) AD_TRY(launch_advance(counter, S, s));      // a full round is S steps for every component
      return AD_OK;
    };
    if (graphs) {
      Ctx::CompGraph& cg = c.comp_graph[(size_t)e * 3 + g % 3];
      const bool same = cg.exec && cg.latent == latent && cg.text == text_emb && cg.pooled == pooled_emb && cg.stream == s &&
                        cg.cfg_scale == c.cfg_scale && cg.tau_off == tau_off && cg.latent_off == latent_off && cg.eps_off == eps_off;
      if (!same) {
        if (cg.exec) AD_HIP(hipStreamSynchronize(s));    // a replay of the old graph may still be running
        if (cg.exec) (void)hipGraphExecDestroy(cg.exec);
        if (cg.graph) (void)hipGraphDestroy(cg.graph);
        cg.exec = nullptr; cg.graph = nullptr;
        AD_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed));
        const ad_status st = work();
        hipGraph_t graph = nullptr;
        const hipError_t err = hipStreamEndCapture(s, &graph);
        if (st != AD_OK) { if (graph) (void)hipGraphDestroy(graph); return st; }
        if (err != hipSuccess) AD_FAIL(AD_ERR_HIP, "hipStreamEndCapture failed: %s", hipGetErrorString(err));
        cg.graph = graph;
        AD_HIP(hipGraphInstantiate(&cg.exec, cg.graph, nullptr, nullptr, 0));
        cg.latent = latent; cg.text = text_emb; cg.pooled = pooled_emb; cg.stream = s; cg.cfg_scale = c.cfg_scale;
        cg.tau_off = tau_off; cg.latent_off = latent_off; cg.eps_off = eps_off;
      }
      AD_HIP(hipGraphLaunch(cg.exec, s));
    } else {
      AD_TRY(work());
    }
    if (row.eps_step >= 0) {
      lane_stream.push_back(s); lane_eps_off.push_back(eps_off); lane_step.push_back(row.eps_step);
    } else {
      AD_HIP(hipEventRecord(ev_done_of(c, row.comp, g), s));
    }
  }
  if (lane_stream.empty()) AD_FAIL(AD_ERR_STATE, "per-edge mode: a full round ends with the last component");
  // sampler updates in step order on the stream of the last evaluation, behind the other evaluations of the last component
  hipStream_t ss = lane_stream.back();
  for (size_t j = 0; j + 1 < lane_stream.size(); ++j)
    if (lane_stream[j] != ss) {
      AD_HIP(hipEventRecord(c.events[1 + j], lane_stream[j]));
      AD_HIP(hipStreamWaitEvent(ss, c.events[1 + j], 0));
    }
  // the sampler overwrites the latent: this round's component 1 has to be done with it
  if (c.N > 1) AD_HIP(hipStreamWaitEvent(ss, ev_done_of(c, 1, g), 0));
  int* counter = counters + c.N;
  for (size_t j = 0; j < lane_stream.size(); ++j) {
    AD_TRY(launch_sampler((float*)latent, (const float*)(c.work_dev + c.eps_off[j]), n, c.cfg.frames > 0 ? 1 : c.cfg.batch, 0.f, 0.f,
                          StepRef{table, counter, lane_eps_off[j]}, c.cfg_scale, ss));
    if (steps_out) steps_out->push_back(lane_step[j]);
  }
  AD_TRY(launch_advance(counter, (int)lane_stream.size(), ss));
  AD_TRY(launch_advance(counters, (int)lane_stream.size(), ss));          // the counter of the barrier rounds moves along
  AD_HIP(hipEventRecord(c.ev_sampler[g & 3], ss));
  AD_HIP(hipEventRecord(ev_done_of(c, c.N, g), ss));
  return AD_OK;
}

// One round of the table.  Streams: evaluation e of the round runs on streams[e % n]; every stream
// first waits for the event that opened the round (recorded on streams[0] behind the previous round, which
// this round reads from and whose read slot it overwrites), the sampler runs behind the last-component
// evaluations and behind the latent read of component 1, and streams[0] joins the other streams at the end.
// Every per-step scalar is looked up on the device (table[counter + offset]) so that the launch arguments of
// an asynchronous round depend only on its slot parity: such a round can be captured once and replayed.
static ad_status enqueue_round(Ctx& c, size_t r0, size_t r1, void* latent, const void* text_emb, const void* pooled_emb,
                               const ad_stream* streams, int ns, std::vector<int>* steps_out) {
  const bool warm = c.rows[r0].read_slot == c.rows[r0].write_slot;
  const int nu = (int)c.units.size();
  const int max_par = c.devices + c.stride - 1;
  hipStream_t s0 = (hipStream_t)streams[0];
  const StepRec* table = (const StepRec*)(c.work_dev + c.step_table_off);
  int* counter = (int*)(c.work_dev + c.step_counter_off);
  const int base = c.steps_done;             // the device counter holds this value when the round runs

  if (c.edge_mode) {
    // a barrier round inside a per-edge run (warm-up, a profiled round): the rounds before it were not joined, so
    // streams[0] first gets behind everything they may still be doing
    const int g = c.rows[r0].round;
    for (int m = 1; m <= c.N; ++m)
      for (int back = 1; back <= 2; ++back) AD_HIP(hipStreamWaitEvent(s0, ev_done_of(c, m, g - back), 0));
    AD_HIP(hipStreamWaitEvent(s0, c.ev_sampler[(g + 3) & 3], 0));
  }
  // open the round: the other streams start behind everything streams[0] has been given so far
  AD_HIP(hipEventRecord(c.events[0], s0));
  for (int k = 1; k < ns; ++k) AD_HIP(hipStreamWaitEvent((hipStream_t)streams[k], c.events[0], 0));

  std::vector<hipStream_t> comp_stream(c.N + 1, s0);
  std::vector<int> eps_steps, eps_lane;
  std::vector<hipStream_t> eps_stream;
  int lane_next = 0;
  bool pack_recorded = false;
  hipStream_t pack_stream = nullptr;
  for (size_t r = r0; r < r1; ++r) {
    const ad_sched_row& row = c.rows[r];
    const Component& cp = c.comps[row.comp - 1];
    hipStream_t s = warm ? s0 : (hipStream_t)streams[(r - r0) % ns];
    // an evaluation that reads another one of its own round fresh follows it on its stream (wrapped segmentation)
    if (!warm && row.fresh_from > 0) s = comp_stream[row.fresh_from];
    comp_stream[row.comp] = s;
    const void* in[64];
    void* out[64];
    if (cp.in_units.size() > 64 || cp.out_units.size() > 64) AD_FAIL(AD_ERR_INVALID, "too many component tensors");
    for (size_t i = 0; i < cp.in_units.size(); ++i) {
      if (cp.in_units[i] < 0) { in[i] = latent; continue; }
      const int u = cp.in_units[i];
      const int slot = (row.fresh_from > 0 && c.units[u].comp == row.fresh_from) ? phys_write(c, row) : phys_read(c, row);
      in[i] = c.work_dev + c.slot_off[slot][u];
    }
    int lane = 0;
    if (row.comp == c.N) lane = lane_next++;
    for (size_t i = 0; i < cp.out_units.size(); ++i) {
      const int u = cp.out_units[i];
      if (u == nu - 1) out[i] = c.work_dev + c.eps_off[lane];
      else if (row.write_slot >= 0) out[i] = c.work_dev + c.slot_off[phys_write(c, row)][u];
      else AD_FAIL(AD_ERR_STATE, "schedule row drops a stored tensor");
    }
    const StepRef tau_ref{table, counter, row.tau_step - base};
    const StepRef scale_ref{table, counter, row.latent_step >= 0 ? row.latent_step - base : 0};
    // the sampler may overwrite the latent only after component 1 has consumed it
    AD_TRY(run_component(c, row.comp, lane, in, c.taus[row.tau_step], 1.f, text_emb, pooled_emb, out, s,
                         row.latent_step >= 0 ? c.ev_pack : nullptr, tau_ref, scale_ref));
    if (row.latent_step >= 0) { pack_recorded = true; pack_stream = s; }
    if (row.eps_step >= 0) { eps_steps.push_back(row.eps_step); eps_lane.push_back(lane); eps_stream.push_back(s); }
  }
  // sampler updates, in step order, on the stream of the last head evaluation
  hipStream_t ss = eps_stream.empty() ? s0 : eps_stream.back();
  for (size_t j = 0; j + 1 < eps_stream.size(); ++j)
    if (eps_stream[j] != ss) {
      AD_HIP(hipEventRecord(c.events[1 + j], eps_stream[j]));
      AD_HIP(hipStreamWaitEvent(ss, c.events[1 + j], 0));
    }
  if (pack_recorded && pack_stream != ss) AD_HIP(hipStreamWaitEvent(ss, c.ev_pack, 0));
  const size_t n = (size_t)(c.cfg.frames > 0 ? c.cfg.frames : 1) * c.cfg.latent_channels * c.cfg.height * c.cfg.width;
  for (size_t j = 0; j < eps_steps.size(); ++j)
    AD_TRY(launch_sampler((float*)latent, (const float*)(c.work_dev + c.eps_off[eps_lane[j]]), n, c.cfg.frames > 0 ? 1 : c.cfg.batch, 0.f, 0.f,
                          StepRef{table, counter, eps_steps[j] - base}, c.cfg_scale, ss));
  // close the round: streams[0] joins every other stream, then moves the step counter on
  for (int k = 1; k < ns; ++k) {
    AD_HIP(hipEventRecord(c.events[max_par + k], (hipStream_t)streams[k]));
    AD_HIP(hipStreamWaitEvent(s0, c.events[max_par + k], 0));
  }
  AD_TRY(launch_advance(counter, (int)eps_steps.size(), s0));
  if (c.edge_mode) {
    // a barrier round inside a per-edge run (warm-up): the per-component counters move along, and everything the next
    // round may wait for counts as done here
    for (int m = 1; m <= c.N; ++m) {
      AD_TRY(launch_advance(counter + m, (int)eps_steps.size(), s0));
      AD_HIP(hipEventRecord(ev_done_of(c, m, c.rows[r0].round), s0));
    }
    AD_HIP(hipEventRecord(c.ev_sampler[c.rows[r0].round & 3], s0));
  }
  if (steps_out) *steps_out = eps_steps;
  return AD_OK;
}

static void drop_graph(Ctx::RoundGraph& g) {
  if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (g.graph) (void)hipGraphDestroy(g.graph);
  g.exec = nullptr; g.graph = nullptr;
}

static void drop_comp_graphs(Ctx& c) {
  for (auto& g : c.comp_graph) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.graph) (void)hipGraphDestroy(g.graph);
    g.exec = nullptr; g.graph = nullptr;
  }
}

ad_status ad_set_edge_mode(ad_ctx* ctx, int on) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (on && c.N > 60) AD_FAIL(AD_ERR_INVALID, "the per-edge mode holds at most 60 components");
  if (c.next_row != 0 && c.next_row < c.rows.size()) AD_FAIL(AD_ERR_STATE, "the mode cannot change in the middle of a run");
  c.edge_mode = on != 0;
  return AD_OK;
}

ad_status ad_set_graph_mode(ad_ctx* ctx, int on) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  c.use_graphs = on != 0;
  if (!c.use_graphs && (c.round_graph[0].exec || c.round_graph[1].exec)) {
    AD_HIP(hipDeviceSynchronize());
    for (auto& g : c.round_graph) drop_graph(g);
  }
  return AD_OK;
}

ad_status ad_step(ad_ctx* ctx, void* latent, const void* text_emb, const void* pooled_emb, const ad_stream* streams,
                  int n_streams, int* steps_done) {
  if (!ctx || !latent || !streams || n_streams < 1) AD_FAIL(AD_ERR_INVALID, "bad argument");
  Ctx& c = *C(ctx);
  if (!c.weights_loaded) AD_FAIL(AD_ERR_STATE, "weights are not loaded");
  if (c.T == 0) AD_FAIL(AD_ERR_STATE, "ad_reset has not been called");
  if (c.next_row >= c.rows.size()) {
    if (steps_done) *steps_done = c.steps_done;
    return AD_ERR_DONE;
  }
  const int max_par = c.devices + c.stride - 1;
  const int ns = n_streams < max_par ? n_streams : max_par;
  while ((int)c.events.size() < 2 * max_par + 2) {
    hipEvent_t ev;
    AD_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    c.events.push_back(ev);
  }
  if (!c.ev_pack) AD_HIP(hipEventCreateWithFlags(&c.ev_pack, hipEventDisableTiming));
  hipStream_t s0 = (hipStream_t)streams[0];
  if (c.edge_mode) {
    // events of the per-edge rounds (the warm-up rounds of such a run record them too) and the per-component graphs
    if ((int)c.ev_done.size() < 4 * c.N) c.ev_done.resize((size_t)4 * c.N, nullptr);
    for (auto& ev : c.ev_done)
      if (!ev) AD_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    for (auto& ev : c.ev_sampler)
      if (!ev) AD_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    const size_t n_graphs = (size_t)3 * (c.N + c.stride - 1);
    if (c.comp_graph.size() != n_graphs) { drop_comp_graphs(c); c.comp_graph.assign(n_graphs, Ctx::CompGraph{}); }
  }

  if (!c.step_table_ready) {
    // first round of a run: per-step scalars and the step counter go to the device (once, synchronously)
    std::vector<StepRec> tab(c.T);
    for (int i = 0; i < c.T; ++i) {
      double cx, ce, in_scale, init_scale;
      sampler_coeffs(c, i, &cx, &ce, &in_scale, &init_scale);
      tab[i] = StepRec{(float)c.taus[i], (float)in_scale, (float)cx, (float)ce};
    }
    int zero[64];                                       // the round counter and one counter per component
    for (int& z : zero) z = c.steps_done;
    AD_HIP(hipDeviceSynchronize());
    AD_HIP(hipMemcpy(c.work_dev + c.step_table_off, tab.data(), tab.size() * sizeof(StepRec), hipMemcpyHostToDevice));
    AD_HIP(hipMemcpy(c.work_dev + c.step_counter_off, zero, sizeof(zero), hipMemcpyHostToDevice));
    AD_HIP(hipDeviceSynchronize());
    c.step_table_ready = true;
    for (auto& g : c.round_graph) drop_graph(g);      // the table belongs to the run; so do its graphs
    drop_comp_graphs(c);
  }
  if (text_emb && c.text_cached != text_emb) {
    // first round of a run (or a new embedding): build the text key / value cache ahead of everything else
    set_profiler(prof_of(c));
    ad_status st = precompute_text(c, text_emb, s0);
    set_profiler(nullptr);
    if (st != AD_OK) return st;
  }

  const size_t r0 = c.next_row;
  size_t r1 = r0;
  while (r1 < c.rows.size() && c.rows[r1].round == c.rows[r0].round) ++r1;
  const bool warm = c.rows[r0].read_slot == c.rows[r0].write_slot;
  const bool full = !warm && (int)(r1 - r0) == c.N + c.stride - 1;
  Profiler* prof = prof_of(c);
  const bool profiling = prof && prof->on;
  std::vector<int> done;
  ad_status st = AD_OK;
  if (c.edge_mode && full && !profiling) {
    st = enqueue_round_edges(c, r0, r1, latent, text_emb, pooled_emb, streams, ns, c.use_graphs, &done);
    if (st != AD_OK) return st;
  } else if (c.use_graphs && full && !profiling) {
    // an asynchronous full round depends on the step only through the device-side counter: capture it once
    // per slot parity (and per set of caller pointers), then replay
    Ctx::RoundGraph& g = c.round_graph[c.rows[r0].write_slot & 1];
    // what a captured round bakes in besides the pointers: every row's step indices relative to the device counter
    // (they differ between rounds when time shifting starts, or for the round right after a warm-up of zero steps)
    std::vector<int> offsets;
    for (size_t r = r0; r < r1; ++r) {
      const ad_sched_row& row = c.rows[r];
      offsets.push_back(row.comp);
      offsets.push_back(row.tau_step - c.steps_done);
      offsets.push_back(row.latent_step >= 0 ? row.latent_step - c.steps_done : INT32_MIN);
      offsets.push_back(row.eps_step >= 0 ? row.eps_step - c.steps_done : INT32_MIN);
      offsets.push_back(row.fresh_from);
    }
    bool same = g.exec && g.latent == latent && g.text == text_emb && g.pooled == pooled_emb && g.cfg_scale == c.cfg_scale &&
                (int)g.streams.size() == ns && g.offsets == offsets;
    for (int k = 0; same && k < ns; ++k) same = g.streams[k] == (hipStream_t)streams[k];
    if (!same) {
      if (g.exec) AD_HIP(hipStreamSynchronize(s0));   // a replay of the old graph may still be running
      drop_graph(g);
      AD_HIP(hipStreamBeginCapture(s0, hipStreamCaptureModeRelaxed));
      st = enqueue_round(c, r0, r1, latent, text_emb, pooled_emb, streams, ns, &done);
      hipGraph_t graph = nullptr;
      const hipError_t e = hipStreamEndCapture(s0, &graph);
      if (st != AD_OK) { if (graph) (void)hipGraphDestroy(graph); return st; }
      if (e != hipSuccess) AD_FAIL(AD_ERR_HIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
      g.graph = graph;
      AD_HIP(hipGraphInstantiate(&g.exec, g.graph, nullptr, nullptr, 0));
      g.latent = latent; g.text = text_emb; g.pooled = pooled_emb; g.cfg_scale = c.cfg_scale;
      g.streams.assign((const hipStream_t*)streams, (const hipStream_t*)streams + ns);
      g.offsets = offsets;
    } else {
      for (size_t r = r0; r < r1; ++r)
        if (c.rows[r].eps_step >= 0) done.push_back(c.rows[r].eps_step);
    }
    AD_HIP(hipGraphLaunch(g.exec, s0));
  } else {
    set_profiler(prof);
    st = enqueue_round(c, r0, r1, latent, text_emb, pooled_emb, streams, ns, &done);
    set_profiler(nullptr);
    if (st != AD_OK) return st;
  }
  for (int i : done) c.steps_done = i + 1 > c.steps_done ? i + 1 : c.steps_done;
  c.next_row = r1;
  if (steps_done) *steps_done = c.steps_done;
  return AD_OK;
}

}  // extern "C"
