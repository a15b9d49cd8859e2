// Host-side logic of the library: configuration checks, unit list, FLOP-balanced partition,
// schedule table, sampler coefficients, weight manifest / packing and the memory plan.
// Nothing here touches the GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <limits>

#include "ad_internal.h"
#include "ad_kernels.h"

namespace ad {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

// ------------------------------------------------------------------------------------------------
// Unit list: the UNet as an ordered sequence of blocks with explicit skip wiring.
// ------------------------------------------------------------------------------------------------
static Unit make_unit(int kind, const std::string& name, int c_in, int c_skip, int c_out, int h_in, int w_in,
                      int h_out, int w_out, int depth, int skip_from) {
  Unit u;
  std::memset(&u.info, 0, sizeof(u.info));
  std::snprintf(u.info.name, AD_NAME_LEN, "%s", name.c_str());
  u.info.kind = kind;
  u.info.c_in = c_in; u.info.c_skip = c_skip; u.info.c_out = c_out;
  u.info.h_in = h_in; u.info.w_in = w_in; u.info.h_out = h_out; u.info.w_out = w_out;
  u.info.depth = depth; u.info.skip_from = skip_from;
  return u;
}

static void build_units(const ad_unet_cfg& c, std::vector<Unit>& units) {
  std::vector<int> skips;
  int h = c.height, w = c.width;
  auto nm = [](const char* pre, int l, int j, const char* suf) {
    char b[AD_NAME_LEN];
    if (j >= 0) std::snprintf(b, sizeof(b), "%s%d.%d.%s", pre, l, j, suf);
    else std::snprintf(b, sizeof(b), "%s%d.%s", pre, l, suf);
    return std::string(b);
  };
  units.push_back(make_unit(AD_UNIT_CONV_IN, "conv_in", c.latent_channels, 0, c.channels[0], h, w, h, w, 0, -1));
  skips.push_back(0);
  int ch = c.channels[0];
  for (int l = 0; l < c.n_levels; ++l) {
    for (int j = 0; j < c.layers_per_block; ++j) {
      units.push_back(make_unit(AD_UNIT_RES, nm("d", l, j, "res"), ch, 0, c.channels[l], h, w, h, w, 0, -1));
      ch = c.channels[l];
      if (c.transformer_depth[l] > 0)
        units.push_back(make_unit(AD_UNIT_TFM, nm("d", l, j, "tfm"), ch, 0, ch, h, w, h, w, c.transformer_depth[l], -1));
      skips.push_back((int)units.size() - 1);
    }
    if (l < c.n_levels - 1) {
      units.push_back(make_unit(AD_UNIT_DOWN, nm("d", l, -1, "ds"), ch, 0, ch, h, w, h / 2, w / 2, 0, -1));
      skips.push_back((int)units.size() - 1);
      h /= 2; w /= 2;
    }
  }
  units.push_back(make_unit(AD_UNIT_RES, "mid.res0", ch, 0, ch, h, w, h, w, 0, -1));
  if (c.mid_depth > 0) units.push_back(make_unit(AD_UNIT_TFM, "mid.tfm", ch, 0, ch, h, w, h, w, c.mid_depth, -1));
  units.push_back(make_unit(AD_UNIT_RES, "mid.res1", ch, 0, ch, h, w, h, w, 0, -1));
  for (int l = c.n_levels - 1; l >= 0; --l) {
    for (int j = 0; j <= c.layers_per_block; ++j) {
      int s = skips.back();
      skips.pop_back();
      units.push_back(make_unit(AD_UNIT_RES, nm("u", l, j, "res"), ch, units[s].info.c_out, c.channels[l], h, w, h, w, 0, s));
      ch = c.channels[l];
      if (c.transformer_depth[l] > 0)
        units.push_back(make_unit(AD_UNIT_TFM, nm("u", l, j, "tfm"), ch, 0, ch, h, w, h, w, c.transformer_depth[l], -1));
    }
    if (l > 0) {
      units.push_back(make_unit(AD_UNIT_UP, nm("u", l, -1, "us"), ch, 0, ch, h, w, 2 * h, 2 * w, 0, -1));
      h *= 2; w *= 2;
    }
  }
  units.push_back(make_unit(AD_UNIT_OUT, "out", ch, 0, c.latent_channels, h, w, h, w, 0, -1));
}

// 2 FLOPs per multiply-accumulate of every convolution, linear layer and attention matmul.
int64_t unit_flops(const ad_unet_cfg& c, const ad_unit_info& u) {
  const int64_t B = c.batch;
  auto conv = [&](int64_t ci, int64_t co, int64_t k) { return 2 * B * u.h_out * u.w_out * co * ci * k * k; };
  switch (u.kind) {
    case AD_UNIT_CONV_IN: case AD_UNIT_DOWN: case AD_UNIT_UP: case AD_UNIT_OUT:
      return conv(u.c_in, u.c_out, 3);
    case AD_UNIT_RES: {
      int64_t ci = u.c_in + u.c_skip;
      int64_t f = conv(ci, u.c_out, 3) + conv(u.c_out, u.c_out, 3) + 2 * B * (4 * c.channels[0]) * u.c_out;
      if (ci != u.c_out) f += conv(ci, u.c_out, 1);
      return f;
    }
    case AD_UNIT_TFM: {
      int64_t C = u.c_in, L = (int64_t)u.h_in * u.w_in, Lk = c.ctx_len;
      int64_t lin = 2 * B * L * C * C;
      const int64_t Bt = c.frames > 0 ? 1 : B;                                     // rows of the text embedding
      int64_t per = 4 * lin + 4 * B * L * L * C;                                  // self attention
      per += 2 * lin + 2 * (2 * Bt * Lk * C * c.ctx_dim) + 4 * B * L * Lk * C;     // cross attention
      per += 24 * B * L * C * C;                                                  // GEGLU feed-forward
      int64_t f = 2 * lin + u.depth * per;
      if (c.temporal_heads > 0) f += 4 * lin + 4 * B * L * c.frames * C;           // temporal layer: q, k, v, o + scores over frames
      return f;
    }
  }
  return 0;
}

// Minimise the largest component over contiguous cuts; among optimal cut vectors take the
// lexicographically smallest.  Returns the N-1 positions where a new component starts.
std::vector<int> partition_cuts(const std::vector<int64_t>& costs, int n) {
  const int m = (int)costs.size();
  std::vector<int64_t> pre(m + 1, 0);
  for (int i = 0; i < m; ++i) pre[i + 1] = pre[i] + costs[i];
  const int64_t INF = std::numeric_limits<int64_t>::max();
  // tail[k][i]: smallest achievable maximum when units i.. are split into k parts
  std::vector<std::vector<int64_t>> tail(n + 1, std::vector<int64_t>(m + 1, INF));
  tail[0][m] = 0;
  for (int k = 1; k <= n; ++k)
    for (int i = m - k; i >= 0; --i) {
      int64_t best = INF;
      for (int e = i + 1; e <= m - (k - 1); ++e) {
        if (tail[k - 1][e] == INF) continue;
        int64_t v = std::max(pre[e] - pre[i], tail[k - 1][e]);
        if (v < best) best = v;
      }
      tail[k][i] = best;
    }
  const int64_t opt = tail[n][0];
  std::vector<int> cuts;
  int i = 0;
  for (int k = n; k > 1; --k)
    for (int e = i + 1; e <= m - (k - 1); ++e)
      if (pre[e] - pre[i] <= opt && tail[k - 1][e] <= opt) {
        cuts.push_back(e);
        i = e;
        break;
      }
  return cuts;
}

// Schedule table (Section 3.2; Appendix A "Stride Denoising", "Time Shifting").
// Wrapped segmentation: the n cuts of the unit list into n + 1 segments that minimise
// max(cost(first) + cost(last), cost of each middle segment); ties -> lexicographically smallest cut vector.
// Cut vectors are enumerated in lexicographic order, the first optimum is kept.
std::vector<int> partition_cuts_wrapped(const std::vector<int64_t>& costs, int n) {
  const int m = (int)costs.size();
  std::vector<int64_t> pre(m + 1, 0);
  for (int i = 0; i < m; ++i) pre[i + 1] = pre[i] + costs[i];
  std::vector<int> cuts(n), best;
  for (int k = 0; k < n; ++k) cuts[k] = k + 1;
  int64_t best_cost = -1;
  while (true) {
    int64_t worst = pre[cuts[0]] + (pre[m] - pre[cuts[n - 1]]);
    for (int k = 0; k + 1 < n; ++k) worst = std::max(worst, pre[cuts[k + 1]] - pre[cuts[k]]);
    if (best_cost < 0 || worst < best_cost) { best_cost = worst; best = cuts; }
    int k = n - 1;                                   // next combination of n values out of 1..m-1
    while (k >= 0 && cuts[k] == m - 1 - (n - 1 - k)) --k;
    if (k < 0) break;
    ++cuts[k];
    for (int j = k + 1; j < n; ++j) cuts[j] = cuts[j - 1] + 1;
  }
  return best;
}

void build_schedule(int T, int N, int w, int S, bool time_shift, bool wrap, std::vector<ad_sched_row>& rows) {
  rows.clear();
  auto tau_of = [&](int i) { return (time_shift && i >= w && i >= 1) ? i - 1 : i; };
  int g = 0;
  const int wu = w < T ? w : T;
  for (int i = 0; i < wu; ++i, ++g)
    for (int n = 1; n <= N; ++n)
      rows.push_back(ad_sched_row{g, n, i, g & 1, g & 1, n == 1 ? i : -1, n == N ? i : -1, 0});
  if (wrap) {
    // N evaluations per step (head, middle segments, tail); the tail reads the head of its own round
    for (int b = wu; b < T; ++b, ++g) {
      const int rd = (g - 1) & 1, wr = g & 1;
      for (int n = 1; n < N; ++n) rows.push_back(ad_sched_row{g, n, tau_of(b), rd, wr, n == 1 ? b : -1, -1, 0});
      rows.push_back(ad_sched_row{g, N, tau_of(b), rd, wr, -1, b, 1});
    }
    return;
  }
  for (int b = wu; b < T; ++g) {
    const int steps = (T - b < S) ? T - b : S;
    const bool full = steps == S;
    const int rd = (g - 1) & 1, wr = g & 1;
    if (full)
      for (int n = 1; n < N; ++n)
        rows.push_back(ad_sched_row{g, n, tau_of(b + S - 1), rd, wr, n == 1 ? b : -1, -1, 0});
    for (int j = 0; j < steps; ++j)
      rows.push_back(ad_sched_row{g, N, tau_of(b + j), rd, (full && j == S - 1) ? wr : -1, N == 1 ? b : -1, b + j, 0});
    b += steps;
  }
}

static void alphas_cumprod(int kind, std::vector<double>& acp) {
  acp.resize(kTrainSteps);
  const double b0 = 0.00085, b1 = 0.012;
  double prod = 1.0;
  for (int k = 0; k < kTrainSteps; ++k) {
    double f = (double)k / (kTrainSteps - 1), beta;
    if (kind == AD_BETA_LINEAR) beta = b0 + (b1 - b0) * f;
    else { double r = std::sqrt(b0) + (std::sqrt(b1) - std::sqrt(b0)) * f; beta = r * r; }
    prod *= 1.0 - beta;
    acp[k] = prod;
  }
}

// x' = cx * x + ce * eps.  DDIM (eta = 0): x' = sqrt(a')(x - sqrt(1-a) eps)/sqrt(a) + sqrt(1-a') eps with
// a' = 1 after the last step.  Euler: x' = x + (sigma' - sigma) eps, sigma = sqrt((1-a)/a), final sigma' = 0.
void sampler_coeffs(const Ctx& c, int step, double* cx, double* ce, double* in_scale, double* init_scale) {
  const double a = c.acp[c.taus[step]];
  const double a2 = step + 1 < c.T ? c.acp[c.taus[step + 1]] : 1.0;
  const double sig = std::sqrt((1 - a) / a), sig2 = step + 1 < c.T ? std::sqrt((1 - a2) / a2) : 0.0;
  if (c.sampler == AD_DDIM) {
    *cx = std::sqrt(a2) / std::sqrt(a);
    *ce = std::sqrt(1 - a2) - std::sqrt(a2) * std::sqrt(1 - a) / std::sqrt(a);
    *in_scale = 1.0;
    *init_scale = 1.0;
  } else {
    *cx = 1.0;
    *ce = sig2 - sig;
    *in_scale = 1.0 / std::sqrt(sig * sig + 1.0);
    const double a0 = c.acp[c.taus[0]];
    *init_scale = std::sqrt((1 - a0) / a0 + 1.0);
  }
}

// ------------------------------------------------------------------------------------------------
// Weight manifest.
// ------------------------------------------------------------------------------------------------
static void add_w(Ctx& c, const std::string& name, int role, std::initializer_list<int> shape) {
  Weight w;
  std::memset(&w.info, 0, sizeof(w.info));
  std::snprintf(w.info.name, AD_NAME_LEN, "%s", name.c_str());
  w.info.ndim = (int)shape.size();
  int i = 0;
  for (int s : shape) w.info.shape[i++] = s;
  w.role = role;
  c.weights.push_back(w);
}

static void build_manifest(Ctx& c) {
  const ad_unet_cfg& g = c.cfg;
  const int td = c.temb_dim, c0 = g.channels[0];
  add_w(c, "time.lin1.w", W_SMALL, {td, c0});   add_w(c, "time.lin1.b", W_VEC_F32, {td});
  add_w(c, "time.lin2.w", W_SMALL, {td, td});   add_w(c, "time.lin2.b", W_VEC_F32, {td});
  if (g.pooled_dim > 0) {
    add_w(c, "pool.lin1.w", W_SMALL, {td, g.pooled_dim}); add_w(c, "pool.lin1.b", W_VEC_F32, {td});
    add_w(c, "pool.lin2.w", W_SMALL, {td, td});           add_w(c, "pool.lin2.b", W_VEC_F32, {td});
  }
  int temb_row = 0;
  for (Unit& u : c.units) {
    const ad_unit_info& f = u.info;
    const std::string n = f.name;
    u.w_first = (int)c.weights.size();
    switch (f.kind) {
      case AD_UNIT_CONV_IN:
        add_w(c, n + ".conv.w", W_CONV_IN, {f.c_out, f.c_in, 3, 3}); add_w(c, n + ".conv.b", W_VEC_F32, {f.c_out});
        break;
      case AD_UNIT_DOWN: case AD_UNIT_UP:
        add_w(c, n + ".conv.w", W_CONV3, {f.c_out, f.c_in, 3, 3}); add_w(c, n + ".conv.b", W_VEC_F32, {f.c_out});
        break;
      case AD_UNIT_OUT:
        add_w(c, n + ".gn.g", W_VEC_F32, {f.c_in}); add_w(c, n + ".gn.b", W_VEC_F32, {f.c_in});
        add_w(c, n + ".conv.w", W_CONV3, {f.c_out, f.c_in, 3, 3}); add_w(c, n + ".conv.b", W_VEC_F32, {f.c_out});
        break;
      case AD_UNIT_RES: {
        const int ci = f.c_in + f.c_skip;
        add_w(c, n + ".gn1.g", W_VEC_F32, {ci}); add_w(c, n + ".gn1.b", W_VEC_F32, {ci});
        add_w(c, n + ".conv1.w", W_CONV3, {f.c_out, ci, 3, 3}); add_w(c, n + ".conv1.b", W_VEC_F32, {f.c_out});
        add_w(c, n + ".temb.w", W_TEMB, {f.c_out, td}); add_w(c, n + ".temb.b", W_TEMB_BIAS, {f.c_out});
        add_w(c, n + ".gn2.g", W_VEC_F32, {f.c_out}); add_w(c, n + ".gn2.b", W_VEC_F32, {f.c_out});
        add_w(c, n + ".conv2.w", W_CONV3, {f.c_out, f.c_out, 3, 3}); add_w(c, n + ".conv2.b", W_VEC_F32, {f.c_out});
        if (ci != f.c_out) {
          add_w(c, n + ".short.w", W_CONV1, {f.c_out, ci, 1, 1}); add_w(c, n + ".short.b", W_VEC_F32, {f.c_out});
        }
        u.temb_row = temb_row;
        temb_row += f.c_out;
        break;
      }
      case AD_UNIT_TFM: {
        const int C = f.c_in;
        add_w(c, n + ".gn.g", W_VEC_F32, {C}); add_w(c, n + ".gn.b", W_VEC_F32, {C});
        add_w(c, n + ".proj_in.w", W_CONV1, {C, C}); add_w(c, n + ".proj_in.b", W_VEC_F32, {C});
        for (int k = 0; k < f.depth; ++k) {
          const std::string p = n + "." + std::to_string(k);
          add_w(c, p + ".ln1.g", W_VEC_F32, {C}); add_w(c, p + ".ln1.b", W_VEC_F32, {C});
          add_w(c, p + ".attn1.q.w", W_QKV_Q, {C, C}); add_w(c, p + ".attn1.k.w", W_QKV_KV, {C, C});
          add_w(c, p + ".attn1.v.w", W_QKV_KV, {C, C});
          add_w(c, p + ".attn1.o.w", W_CONV1, {C, C}); add_w(c, p + ".attn1.o.b", W_VEC_F32, {C});
          add_w(c, p + ".ln2.g", W_VEC_F32, {C}); add_w(c, p + ".ln2.b", W_VEC_F32, {C});
          add_w(c, p + ".attn2.q.w", W_CONV1, {C, C}); add_w(c, p + ".attn2.k.w", W_CONV1, {C, g.ctx_dim});
          add_w(c, p + ".attn2.v.w", W_CONV1, {C, g.ctx_dim});
          add_w(c, p + ".attn2.o.w", W_CONV1, {C, C}); add_w(c, p + ".attn2.o.b", W_VEC_F32, {C});
          add_w(c, p + ".ln3.g", W_VEC_F32, {C}); add_w(c, p + ".ln3.b", W_VEC_F32, {C});
          add_w(c, p + ".ff1.w", W_GEGLU, {8 * C, C}); add_w(c, p + ".ff1.b", W_GEGLU_BIAS, {8 * C});
          add_w(c, p + ".ff2.w", W_CONV1, {C, 4 * C}); add_w(c, p + ".ff2.b", W_VEC_F32, {C});
        }
        add_w(c, n + ".proj_out.w", W_CONV1, {C, C}); add_w(c, n + ".proj_out.b", W_VEC_F32, {C});
        if (g.temporal_heads > 0) {
          const std::string p = n + ".temp";
          add_w(c, p + ".ln.g", W_VEC_F32, {C}); add_w(c, p + ".ln.b", W_VEC_F32, {C});
          add_w(c, p + ".q.w", W_QKV_Q, {C, C}); add_w(c, p + ".k.w", W_QKV_KV, {C, C}); add_w(c, p + ".v.w", W_QKV_KV, {C, C});
          add_w(c, p + ".o.w", W_CONV1, {C, C}); add_w(c, p + ".o.b", W_VEC_F32, {C});
        }
        break;
      }
    }
  }
  c.temb_rows_total = temb_row;
}

// ------------------------------------------------------------------------------------------------
// Packing of GEMM operands: rows = output channels padded to kNPad, K ordered (tap, channel).
// ------------------------------------------------------------------------------------------------
uint16_t f32_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                            // round to nearest even
  return (uint16_t)(u >> 16);
}

static inline void put(int dtype, void* out, size_t idx, float v) {
  if (dtype == AD_BF16) ((uint16_t*)out)[idx] = f32_to_bf16(v);
  else ((float*)out)[idx] = v;
}

size_t packed_conv_bytes(int dtype, int n_out, int c_in, int ksize) {
  return (size_t)round_up(n_out, kNPad) * round_up(ksize * ksize * c_in, bk_elems(dtype)) * esize(dtype);
}

void pack_conv(int dtype, const float* w, int n_out, int c_in, int ksize, bool geglu, void* out) {
  const int taps = ksize * ksize;
  const int kp = round_up(taps * c_in, bk_elems(dtype));
  std::memset(out, 0, packed_conv_bytes(dtype, n_out, c_in, ksize));
  const int half = n_out / 2;
  for (int r = 0; r < n_out; ++r) {
    int src = r;
    if (geglu) {   // packed rows alternate 32 value rows, 32 gate rows
      const int blk = r / 64, in = r % 64;
      src = in < 32 ? blk * 32 + in : half + blk * 32 + in - 32;
    }
    const float* ws = w + (size_t)src * c_in * taps;
    for (int t = 0; t < taps; ++t)
      for (int i = 0; i < c_in; ++i) put(dtype, out, (size_t)r * kp + (size_t)t * c_in + i, ws[(size_t)i * taps + t]);
  }
}

void pack_rows(int dtype, const float* w, size_t n, void* out) {
  for (size_t i = 0; i < n; ++i) put(dtype, out, i, w[i]);
}

// ------------------------------------------------------------------------------------------------
// Memory plan.
// ------------------------------------------------------------------------------------------------
size_t tensor_bytes(const Ctx& c, int unit) {
  const ad_unet_cfg& g = c.cfg;
  if (unit < 0) return (size_t)(g.frames > 0 ? g.frames : 1) * g.latent_channels * g.height * g.width * 4;
  const ad_unit_info& u = c.units[unit].info;
  if (unit == (int)c.units.size() - 1) return (size_t)g.batch * u.c_out * u.h_out * u.w_out * 4;
  return (size_t)g.batch * u.h_out * u.w_out * u.c_out * esize(g.dtype);
}

static void plan_weights(Ctx& c) {
  const int dt = c.cfg.dtype;
  size_t off = 0;
  for (Weight& w : c.weights) {
    const int* s = w.info.shape;
    size_t bytes = 0;
    switch (w.role) {
      case W_CONV3:   bytes = packed_conv_bytes(dt, s[0], s[1], 3); w.n_pad = round_up(s[0], kNPad); w.k_pad = round_up(9 * s[1], bk_elems(dt)); break;
      case W_CONV1: case W_GEGLU:
        bytes = packed_conv_bytes(dt, s[0], s[1], 1); w.n_pad = round_up(s[0], kNPad); w.k_pad = round_up(s[1], bk_elems(dt)); break;
      case W_CONV_IN: w.n_pad = round_up(s[0], kNPad); w.k_pad = kConvInK; bytes = (size_t)w.n_pad * kConvInK * esize(dt); break;
      case W_SMALL:   bytes = (size_t)s[0] * s[1] * esize(dt); break;
      case W_TEMB: case W_TEMB_BIAS: case W_QKV_KV: bytes = 0; break;   // live in a fused matrix
      case W_QKV_Q: bytes = packed_conv_bytes(dt, 3 * s[0], s[1], 1); w.n_pad = round_up(3 * s[0], kNPad); w.k_pad = round_up(s[1], bk_elems(dt)); break;
      case W_VEC_F32: case W_GEGLU_BIAS: bytes = (size_t)round_up(s[0], kNPad) * 4; break;
    }
    w.dev_off = off;
    w.dev_bytes = bytes;
    off += align_up(bytes);
  }
  c.temb_w_off = off;
  off += align_up((size_t)c.temb_rows_total * c.temb_dim * esize(dt));
  c.temb_b_off = off;
  off += align_up((size_t)c.temb_rows_total * 4);
  c.weight_bytes = off;
}

static void plan_work(Ctx& c) {
  const ad_unet_cfg& g = c.cfg;
  const size_t es = esize(g.dtype);
  const int nu = (int)c.units.size();
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  // stored-state slots: every tensor that leaves its component (the noise prediction has its own buffers)
  for (int s = 0; s < 3; ++s) c.slot_off[s].assign(nu, SIZE_MAX);
  for (const Component& cp : c.comps)
    for (int u : cp.out_units)
      if (u != nu - 1)
        for (int s = 0; s < 3; ++s) c.slot_off[s][u] = take(tensor_bytes(c, u));
  c.eps_off.clear();
  for (int j = 0; j < c.stride; ++j) c.eps_off.push_back(take(tensor_bytes(c, nu - 1)));
  c.step_table_off = take((size_t)(kTrainSteps + 8) * sizeof(StepRec));
  c.step_counter_off = take(256);
  c.text_k_off.assign(nu, {});
  c.text_v_off.assign(nu, {});
  for (int ui = 0; ui < nu; ++ui) {
    const ad_unit_info& u = c.units[ui].info;
    if (u.kind != AD_UNIT_TFM) continue;
    const bool vt = g.dtype == AD_BF16 && g.head_dim == 64;
    const size_t bt = g.frames > 0 ? 1 : g.batch;          // rows of the text embedding
    for (int k = 0; k < u.depth; ++k) {
      c.text_k_off[ui].push_back(take(bt * g.ctx_len * u.c_in * es));
      c.text_v_off[ui].push_back(take(vt ? bt * u.c_in * round_up(g.ctx_len, 64) * es : bt * g.ctx_len * u.c_in * es));
    }
  }
  // per (component, lane) activation workspaces
  int cmax = 0;
  for (const Unit& u : c.units) cmax = std::max(cmax, std::max(u.info.c_in + u.info.c_skip, u.info.c_out));
  c.f32_bytes = ((size_t)g.channels[0] + 4ull * g.batch * c.temb_dim + (size_t)g.batch * c.temb_rows_total) * 4;
  c.gn_bytes = ad_groupnorm_scratch_bytes(g.batch, g.height * g.width, cmax);
  c.ws.assign(c.N, {});
  for (int n = 0; n < c.N; ++n) {
    const Component& cp = c.comps[n];
    size_t need[kNumTemps] = {0};
    auto want = [&](int t, size_t bytes) { if (bytes > need[t]) need[t] = bytes; };
    for (int ui = cp.first; ui <= cp.last; ++ui) {
      const ad_unit_info& u = c.units[ui].info;
      const size_t B = g.batch;
      const size_t m_in = B * u.h_in * u.w_in, m_out = B * u.h_out * u.w_out;
      // split-K scratch: the largest need over the epilogues a GEMM of this shape can be launched with, so that
      // the split chosen for a layer (and with it the rounding order) never depends on what else shares its component
      auto gemm = [&](size_t m, int n, int k, int mode = OUT_ROWMAJOR) {
        for (int md : {mode, (int)OUT_ROWMAJOR, (int)OUT_TRANSPOSED, (int)OUT_TRANSPOSED_F32})
          want(9, conv_workspace_bytes(g.dtype, (long long)m, n, k, md));
      };
      switch (u.kind) {
        case AD_UNIT_CONV_IN: want(0, m_out * kConvInK * es); break;
        case AD_UNIT_DOWN: case AD_UNIT_UP: gemm(m_out, u.c_out, 9 * u.c_in); break;
        case AD_UNIT_OUT: want(0, m_in * u.c_in * es); gemm(m_out, u.c_out, 9 * u.c_in); break;
        case AD_UNIT_RES:
          want(0, m_in * std::max(u.c_in + u.c_skip, u.c_out) * es);
          want(1, m_out * u.c_out * es);
          want(2, m_out * u.c_out * es);
          gemm(m_out, u.c_out, 9 * (u.c_in + u.c_skip));
          gemm(m_out, u.c_out, 9 * u.c_out);
          gemm(m_out, u.c_out, u.c_in + u.c_skip);
          break;
        case AD_UNIT_TFM: {
          const size_t L = (size_t)u.h_in * u.w_in, C = u.c_in;
          const size_t lp = round_up((int)L, 64), lkp = round_up(g.ctx_len, 64);
          for (int t : {0, 1, 2, 3, 5}) want(t, m_in * C * es);
          want(4, B * C * lp * es);
          want(6, m_in * 4 * C * es);
          want(7, B * g.ctx_len * C * es);
          want(8, B * C * lkp * es);
          gemm(m_in, (int)C, (int)C);
          gemm(m_in, (int)(3 * C), (int)C, OUT_QKV);
          gemm(m_in, (int)C, (int)(4 * C));
          gemm(B * g.ctx_len, (int)C, g.ctx_dim);
          break;
        }
        default: break;
      }
    }
    const int lanes = (n == c.N - 1) ? c.stride : 1;
    for (int lane = 0; lane < lanes; ++lane) {
      Workspace w;
      for (int ui = cp.first; ui <= cp.last; ++ui) {
        bool external = false;
        for (int o : cp.out_units) external |= (o == ui);
        w.unit_off.push_back(external ? SIZE_MAX : take(tensor_bytes(c, ui)));
      }
      for (int t = 0; t < kNumTemps; ++t) { w.temp_bytes[t] = need[t]; w.temp_off[t] = need[t] ? take(need[t]) : 0; }
      w.f32_off = take(c.f32_bytes);
      w.gn_off = take(c.gn_bytes);
      c.ws[n].push_back(w);
    }
  }
  c.work_bytes = off;
}

static void component_io(const Ctx& c, int first, int last, std::vector<int>& ins, std::vector<int>& outs) {
  const int nu = (int)c.units.size();
  std::vector<char> in_mark(nu + 1, 0), out_mark(nu, 0);
  in_mark[first] = 1;   // index shifted by one: entry i stands for unit i-1
  for (int i = first; i <= last; ++i) {
    int s = c.units[i].info.skip_from;
    if (s >= 0 && s < first) in_mark[s + 1] = 1;
  }
  out_mark[last] = 1;
  for (int i = last + 1; i < nu; ++i) {
    int s = c.units[i].info.skip_from;
    if (s >= first && s <= last) out_mark[s] = 1;
  }
  ins.clear(); outs.clear();
  for (int i = 0; i <= nu; ++i) if (in_mark[i]) ins.push_back(i - 1);
  for (int i = 0; i < nu; ++i) if (out_mark[i]) outs.push_back(i);
}

static ad_status validate(const ad_unet_cfg& g, int n, int warmup, int stride) {
  if (g.latent_channels < 1 || g.latent_channels > 7) AD_FAIL(AD_ERR_INVALID, "latent_channels must be 1..7");
  if (g.n_levels < 1 || g.n_levels > AD_MAX_LEVELS) AD_FAIL(AD_ERR_INVALID, "n_levels must be 1..%d", AD_MAX_LEVELS);
  if (g.batch < 1 || g.batch > 16) AD_FAIL(AD_ERR_INVALID, "batch must be 1..16");
  if (g.dtype != AD_F32 && g.dtype != AD_BF16) AD_FAIL(AD_ERR_INVALID, "dtype must be AD_F32 or AD_BF16");
  const int div = 1 << (g.n_levels - 1);
  if (g.height < div || g.width < div || g.height % div || g.width % div)
    AD_FAIL(AD_ERR_INVALID, "latent %dx%d must be a positive multiple of %d", g.height, g.width, div);
  if (g.layers_per_block < 1) AD_FAIL(AD_ERR_INVALID, "layers_per_block must be >= 1");
  if (g.gn_groups < 1 || g.head_dim < 1) AD_FAIL(AD_ERR_INVALID, "gn_groups and head_dim must be positive");
  const int cm = bk_elems(g.dtype);
  bool any_attn = g.mid_depth > 0;
  for (int l = 0; l < g.n_levels; ++l) {
    if (g.channels[l] < cm || g.channels[l] % cm)
      AD_FAIL(AD_ERR_INVALID, "channels[%d]=%d must be a positive multiple of %d for this dtype", l, g.channels[l], cm);
    if (g.channels[l] % g.gn_groups) AD_FAIL(AD_ERR_INVALID, "channels[%d] not divisible by gn_groups", l);
    if (g.transformer_depth[l] < 0) AD_FAIL(AD_ERR_INVALID, "transformer_depth[%d] negative", l);
    if (g.transformer_depth[l] > 0) {
      any_attn = true;
      if (g.channels[l] % g.head_dim) AD_FAIL(AD_ERR_INVALID, "channels[%d] not divisible by head_dim", l);
    }
  }
  if (g.mid_depth < 0) AD_FAIL(AD_ERR_INVALID, "mid_depth negative");
  if (g.mid_depth > 0 && g.channels[g.n_levels - 1] % g.head_dim) AD_FAIL(AD_ERR_INVALID, "mid channels not divisible by head_dim");
  if (any_attn) {
    if (g.ctx_len < 1 || g.ctx_dim < 1) AD_FAIL(AD_ERR_INVALID, "ctx_len and ctx_dim must be positive");
    if (g.ctx_dim % cm) AD_FAIL(AD_ERR_INVALID, "ctx_dim must be a multiple of %d for this dtype", cm);
    if (g.head_dim > 128 || g.head_dim % 8) AD_FAIL(AD_ERR_INVALID, "head_dim must be a multiple of 8, at most 128");
  }
  if (g.pooled_dim < 0 || g.pooled_dim % 8) AD_FAIL(AD_ERR_INVALID, "pooled_dim must be a non-negative multiple of 8");
  if (g.frames < 0 || g.frames > 16) AD_FAIL(AD_ERR_INVALID, "frames must be 0 (image model) or 1..16");
  if (g.frames > 0 && g.batch != g.frames) AD_FAIL(AD_ERR_INVALID, "a video model has batch == frames");
  if (g.frames == 0 && g.batch > 2) AD_FAIL(AD_ERR_INVALID, "an image model has batch 1 (no guidance) or 2 (guidance pair)");
  if (g.frames > 0 && g.pooled_dim > 0) AD_FAIL(AD_ERR_INVALID, "the pooled-embedding branch is not defined for the video model");
  if (g.temporal_heads < 0 || (g.temporal_heads > 0 && g.frames == 0)) AD_FAIL(AD_ERR_INVALID, "temporal_heads needs frames > 0");
  if (g.temporal_heads > 0) {
    for (int l = 0; l < g.n_levels; ++l)
      if (g.transformer_depth[l] > 0 && (g.channels[l] % g.temporal_heads || g.channels[l] / g.temporal_heads > 320))
        AD_FAIL(AD_ERR_INVALID, "channels[%d] must split into temporal_heads heads of at most 320 channels", l);
    const int cm_ = g.channels[g.n_levels - 1];
    if (g.mid_depth > 0 && (cm_ % g.temporal_heads || cm_ / g.temporal_heads > 320))
      AD_FAIL(AD_ERR_INVALID, "mid channels must split into temporal_heads heads of at most 320 channels");
  }
  if (!(g.gn_eps > 0) || !(g.ln_eps > 0)) AD_FAIL(AD_ERR_INVALID, "eps values must be positive");
  if (n < 1) AD_FAIL(AD_ERR_INVALID, "n_components must be >= 1");
  if (stride < 1 || stride > 8) AD_FAIL(AD_ERR_INVALID, "stride must be 1..8");
  if (warmup < 0) AD_FAIL(AD_ERR_INVALID, "warmup must be >= 0");
  if (n > 1 && warmup < 1) AD_FAIL(AD_ERR_INVALID, "warmup >= 1 is required with more than one component");
  return AD_OK;
}

}  // namespace ad

using namespace ad;

extern "C" {

const char* ad_last_error(void) { return g_err; }

static ad_status create_ctx(const ad_unet_cfg* cfg, int n_components, const int* user_cuts, int warmup, int stride, ad_ctx** out,
                            bool wrap = false) {
  if (!cfg || !out) AD_FAIL(AD_ERR_INVALID, "null argument");
  *out = nullptr;
  ad_status st = validate(*cfg, n_components, warmup, stride);
  if (st != AD_OK) return st;
  Ctx* c = new (std::nothrow) Ctx();
  if (!c) AD_FAIL(AD_ERR_NOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->devices = n_components; c->wrap = wrap;
  if (wrap) ++n_components;             // from here on: the number of segments
  c->N = n_components; c->warmup = warmup; c->stride = stride;
  c->temb_dim = 4 * cfg->channels[0];
  build_units(c->cfg, c->units);
  const int nu = (int)c->units.size();
  if (n_components > nu) { delete c; AD_FAIL(AD_ERR_INVALID, "n_components %d exceeds the %d units", n_components, nu); }
  for (const Unit& u : c->units)
    if (u.info.kind == AD_UNIT_RES && (u.info.c_in + u.info.c_skip) % cfg->gn_groups) {
      delete c;
      AD_FAIL(AD_ERR_INVALID, "concatenated channels not divisible by gn_groups");
    }
  std::vector<int64_t> costs;
  for (Unit& u : c->units) { u.info.flops = unit_flops(c->cfg, u.info); costs.push_back(u.info.flops); }
  std::vector<int> cuts;
  if (user_cuts) {
    for (int k = 0; k + 1 < n_components; ++k) {
      const int lo = k == 0 ? 0 : user_cuts[k - 1];
      if (user_cuts[k] <= lo || user_cuts[k] >= nu) {
        delete c;
        AD_FAIL(AD_ERR_INVALID, "cuts must be strictly increasing and inside (0, %d)", nu);
      }
      cuts.push_back(user_cuts[k]);
    }
  } else {
    cuts = wrap ? partition_cuts_wrapped(costs, n_components - 1) : partition_cuts(costs, n_components);
  }
  std::vector<int> edges{0};
  edges.insert(edges.end(), cuts.begin(), cuts.end());
  edges.push_back(nu);
  c->comps.resize(n_components);
  for (int k = 0; k < n_components; ++k) {
    Component& cp = c->comps[k];
    cp.first = edges[k]; cp.last = edges[k + 1] - 1;
    for (int i = cp.first; i <= cp.last; ++i) c->units[i].comp = k + 1;
    component_io(*c, cp.first, cp.last, cp.in_units, cp.out_units);
  }
  build_manifest(*c);
  for (Component& cp : c->comps) {
    cp.temb_row0 = -1; cp.temb_rows = 0;
    for (int i = cp.first; i <= cp.last; ++i)
      if (c->units[i].info.kind == AD_UNIT_RES) {
        if (cp.temb_row0 < 0) cp.temb_row0 = c->units[i].temb_row;
        cp.temb_rows += c->units[i].info.c_out;
      }
    if (cp.temb_row0 < 0) cp.temb_row0 = 0;
  }
  plan_weights(*c);
  plan_work(*c);
  *out = reinterpret_cast<ad_ctx*>(c);
  return AD_OK;
}

ad_status ad_create(const ad_unet_cfg* cfg, int n_components, int warmup, int stride, ad_ctx** out) {
  return create_ctx(cfg, n_components, nullptr, warmup, stride, out);
}

ad_status ad_balance_cuts(const int64_t* costs, int n_units, int n_components, int* cuts) {
  if (!costs || n_units < 1 || n_components < 1 || n_components > n_units || (n_components > 1 && !cuts))
    AD_FAIL(AD_ERR_INVALID, "bad argument");
  std::vector<int64_t> c(costs, costs + n_units);
  for (int64_t v : c)
    if (v < 0) AD_FAIL(AD_ERR_INVALID, "costs must not be negative");
  const std::vector<int> r = partition_cuts(c, n_components);
  for (size_t k = 0; k < r.size(); ++k) cuts[k] = r[k];
  return AD_OK;
}

ad_status ad_create_wrapped(const ad_unet_cfg* cfg, int n_components, const int* cuts, int warmup, ad_ctx** out) {
  if (n_components < 2) AD_FAIL(AD_ERR_INVALID, "the wrapped segmentation needs at least two components");
  if (!cuts && n_components > 6) AD_FAIL(AD_ERR_INVALID, "automatic wrapped cuts are searched exhaustively: n_components <= 6");
  return create_ctx(cfg, n_components, cuts, warmup, 1, out, true);
}

ad_status ad_create_with_cuts(const ad_unet_cfg* cfg, int n_components, const int* cuts, int warmup, int stride, ad_ctx** out) {
  if (n_components > 1 && !cuts) AD_FAIL(AD_ERR_INVALID, "null argument");
  return create_ctx(cfg, n_components, n_components > 1 ? cuts : nullptr, warmup, stride, out);
}

static inline const Ctx* C(const ad_ctx* p) { return reinterpret_cast<const Ctx*>(p); }
static inline Ctx* C(ad_ctx* p) { return reinterpret_cast<Ctx*>(p); }

int ad_num_units(const ad_ctx* ctx) { return ctx ? (int)C(ctx)->units.size() : 0; }
int ad_num_segments(const ad_ctx* ctx) { return ctx ? C(ctx)->N : 0; }

ad_status ad_get_unit(const ad_ctx* ctx, int unit, ad_unit_info* out) {
  if (!ctx || !out) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (unit < 0 || unit >= (int)C(ctx)->units.size()) AD_FAIL(AD_ERR_INVALID, "unit %d out of range", unit);
  *out = C(ctx)->units[unit].info;
  return AD_OK;
}

ad_status ad_get_partition(const ad_ctx* ctx, int* first, int* last) {
  if (!ctx || !first || !last) AD_FAIL(AD_ERR_INVALID, "null argument");
  for (int k = 0; k < C(ctx)->N; ++k) { first[k] = C(ctx)->comps[k].first; last[k] = C(ctx)->comps[k].last; }
  return AD_OK;
}

ad_status ad_component_io(const ad_ctx* ctx, int comp, int cap, int* in_units, int* n_in, int* out_units, int* n_out) {
  if (!ctx || !in_units || !n_in || !out_units || !n_out) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (comp < 1 || comp > C(ctx)->N) AD_FAIL(AD_ERR_INVALID, "component %d out of range", comp);
  const Component& cp = C(ctx)->comps[comp - 1];
  if ((int)cp.in_units.size() > cap || (int)cp.out_units.size() > cap) AD_FAIL(AD_ERR_INVALID, "capacity %d too small", cap);
  *n_in = (int)cp.in_units.size(); *n_out = (int)cp.out_units.size();
  for (int i = 0; i < *n_in; ++i) in_units[i] = cp.in_units[i];
  for (int i = 0; i < *n_out; ++i) out_units[i] = cp.out_units[i];
  return AD_OK;
}

ad_status ad_tensor_shape(const ad_ctx* ctx, int unit, int* b, int* h, int* w, int* c, size_t* bytes) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  const Ctx& x = *C(ctx);
  if (unit < -1 || unit >= (int)x.units.size()) AD_FAIL(AD_ERR_INVALID, "unit %d out of range", unit);
  int bb, hh, ww, cc;
  if (unit < 0) { bb = x.cfg.frames > 0 ? x.cfg.frames : 1; hh = x.cfg.height; ww = x.cfg.width; cc = x.cfg.latent_channels; }
  else { const ad_unit_info& u = x.units[unit].info; bb = x.cfg.batch; hh = u.h_out; ww = u.w_out; cc = u.c_out; }
  if (b) *b = bb; if (h) *h = hh; if (w) *w = ww; if (c) *c = cc;
  if (bytes) *bytes = tensor_bytes(x, unit);
  return AD_OK;
}

int ad_num_weights(const ad_ctx* ctx) { return ctx ? (int)C(ctx)->weights.size() : 0; }

ad_status ad_get_weight(const ad_ctx* ctx, int index, ad_weight_info* out) {
  if (!ctx || !out) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (index < 0 || index >= (int)C(ctx)->weights.size()) AD_FAIL(AD_ERR_INVALID, "weight %d out of range", index);
  *out = C(ctx)->weights[index].info;
  return AD_OK;
}

ad_status ad_device_bytes(const ad_ctx* ctx, size_t* weight_bytes, size_t* work_bytes) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (weight_bytes) *weight_bytes = C(ctx)->weight_bytes;
  if (work_bytes) *work_bytes = C(ctx)->work_bytes;
  return AD_OK;
}

ad_status ad_reset(ad_ctx* ctx, int T, int sampler_kind, int beta_kind, float cfg_scale, int time_shift) {
  if (!ctx) AD_FAIL(AD_ERR_INVALID, "null argument");
  Ctx& c = *C(ctx);
  if (T < 1 || T > kTrainSteps) AD_FAIL(AD_ERR_INVALID, "T must be 1..%d", kTrainSteps);
  if (sampler_kind != AD_DDIM && sampler_kind != AD_EULER) AD_FAIL(AD_ERR_INVALID, "unknown sampler");
  if (beta_kind != AD_BETA_LINEAR && beta_kind != AD_BETA_SCALED_LINEAR) AD_FAIL(AD_ERR_INVALID, "unknown beta schedule");
  c.T = T; c.sampler = sampler_kind; c.beta_kind = beta_kind; c.cfg_scale = cfg_scale; c.time_shift = time_shift ? 1 : 0;
  c.taus.resize(T);
  for (int i = 0; i < T; ++i) c.taus[i] = (T - 1 - i) * (kTrainSteps / T);
  alphas_cumprod(beta_kind, c.acp);
  build_schedule(T, c.N, c.warmup, c.stride, c.time_shift != 0, c.wrap, c.rows);
  c.next_row = 0;
  c.steps_done = 0;
  c.text_cached = nullptr;
  c.step_table_ready = false;
  return AD_OK;
}

ad_status ad_get_timesteps(const ad_ctx* ctx, int* tau, int cap) {
  if (!ctx || !tau) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (C(ctx)->T == 0) AD_FAIL(AD_ERR_STATE, "ad_reset has not been called");
  if (cap < C(ctx)->T) AD_FAIL(AD_ERR_INVALID, "capacity %d too small", cap);
  for (int i = 0; i < C(ctx)->T; ++i) tau[i] = C(ctx)->taus[i];
  return AD_OK;
}

int ad_num_sched_rows(const ad_ctx* ctx) { return ctx ? (int)C(ctx)->rows.size() : 0; }

ad_status ad_get_schedule(const ad_ctx* ctx, ad_sched_row* rows, int cap) {
  if (!ctx || !rows) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (C(ctx)->T == 0) AD_FAIL(AD_ERR_STATE, "ad_reset has not been called");
  if (cap < (int)C(ctx)->rows.size()) AD_FAIL(AD_ERR_INVALID, "capacity %d too small", cap);
  for (size_t i = 0; i < C(ctx)->rows.size(); ++i) rows[i] = C(ctx)->rows[i];
  return AD_OK;
}

ad_status ad_get_sampler_coeffs(const ad_ctx* ctx, int step, double* c_x, double* c_eps, double* in_scale, double* init_scale) {
  if (!ctx || !c_x || !c_eps || !in_scale || !init_scale) AD_FAIL(AD_ERR_INVALID, "null argument");
  if (C(ctx)->T == 0) AD_FAIL(AD_ERR_STATE, "ad_reset has not been called");
  if (step < 0 || step >= C(ctx)->T) AD_FAIL(AD_ERR_INVALID, "step %d out of range", step);
  sampler_coeffs(*C(ctx), step, c_x, c_eps, in_scale, init_scale);
  return AD_OK;
}

ad_status ad_pack_conv_weight(int dtype, const float* w, int n_out, int c_in, int ksize, int geglu, void* out, size_t* bytes) {
  if (dtype != AD_F32 && dtype != AD_BF16) AD_FAIL(AD_ERR_INVALID, "bad dtype");
  if (n_out < 1 || c_in < 1 || (ksize != 1 && ksize != 3)) AD_FAIL(AD_ERR_INVALID, "bad shape");
  if (geglu && (n_out % 64)) AD_FAIL(AD_ERR_INVALID, "GEGLU packing needs n_out divisible by 64");
  if (bytes) *bytes = packed_conv_bytes(dtype, n_out, c_in, ksize);
  if (!out) return AD_OK;
  if (!w) AD_FAIL(AD_ERR_INVALID, "null weights");
  pack_conv(dtype, w, n_out, c_in, ksize, geglu != 0, out);
  return AD_OK;
}

}  // extern "C"
