"""ctypes binding of libasyncdiff.so.  Names follow include/asyncdiff.h one to one."""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- before the library: PyTorch ships its own HIP runtime, and the process must hold one copy.
# Loaded in this order the library binds to the runtime PyTorch brought; loaded first, it would pull in the system's
# runtime, PyTorch would then mix the two, and the first HIP call fails with "no ROCm-capable device is detected".

AD_F32, AD_BF16 = 0, 1
AD_DDIM, AD_EULER = 0, 1
AD_BETA_LINEAR, AD_BETA_SCALED_LINEAR = 0, 1
AD_OK, AD_ERR_INVALID, AD_ERR_NOMEM, AD_ERR_HIP, AD_ERR_DONE, AD_ERR_STATE = range(6)
UNIT_KINDS = ["conv_in", "res", "tfm", "down", "up", "out"]
OUT_ROWMAJOR, OUT_GEGLU, OUT_TRANSPOSED, OUT_TRANSPOSED_F32, OUT_QKV = 0, 1, 2, 3, 4

lib_path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libasyncdiff.so")


class AsyncDiffError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"asyncdiff status {status}: {message}")
        self.status = status


class UNetCfg(C.Structure):
    _fields_ = [("latent_channels", C.c_int), ("height", C.c_int), ("width", C.c_int), ("batch", C.c_int),
                ("n_levels", C.c_int), ("channels", C.c_int * 4), ("layers_per_block", C.c_int),
                ("transformer_depth", C.c_int * 4), ("mid_depth", C.c_int), ("head_dim", C.c_int),
                ("gn_groups", C.c_int), ("ctx_len", C.c_int), ("ctx_dim", C.c_int), ("pooled_dim", C.c_int),
                ("gn_eps", C.c_float), ("ln_eps", C.c_float), ("dtype", C.c_int),
                ("frames", C.c_int), ("temporal_heads", C.c_int)]

    @classmethod
    def from_dict(cls, d, dtype):
        c = cls()
        c.latent_channels, c.height, c.width, c.batch = d["latent_channels"], d["height"], d["width"], d["batch"]
        c.n_levels = len(d["channels"])
        for i, v in enumerate(d["channels"]):
            c.channels[i] = v
        for i, v in enumerate(d["transformer_depth"]):
            c.transformer_depth[i] = v
        c.layers_per_block, c.mid_depth, c.head_dim = d["layers_per_block"], d["mid_depth"], d["head_dim"]
        c.gn_groups, c.ctx_len, c.ctx_dim, c.pooled_dim = d["gn_groups"], d["ctx_len"], d["ctx_dim"], d.get("pooled_dim", 0)
        c.gn_eps, c.ln_eps = d.get("gn_eps", 1e-5), d.get("ln_eps", 1e-5)
        c.dtype = dtype
        c.frames, c.temporal_heads = d.get("frames", 0), d.get("temporal_heads", 0)
        return c


class UnitInfo(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("kind", C.c_int), ("c_in", C.c_int), ("c_skip", C.c_int), ("c_out", C.c_int),
                ("h_in", C.c_int), ("w_in", C.c_int), ("h_out", C.c_int), ("w_out", C.c_int), ("depth", C.c_int),
                ("skip_from", C.c_int), ("flops", C.c_int64)]


class WeightInfo(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("ndim", C.c_int), ("shape", C.c_int * 4)]


class SchedRow(C.Structure):
    _fields_ = [("round", C.c_int), ("comp", C.c_int), ("tau_step", C.c_int), ("read_slot", C.c_int),
                ("write_slot", C.c_int), ("latent_step", C.c_int), ("eps_step", C.c_int), ("fresh_from", C.c_int)]

    def as_tuple(self):
        return (self.round, self.comp, self.tau_step, self.read_slot, self.write_slot, self.latent_step, self.eps_step,
                self.fresh_from)


class ProfileRec(C.Structure):
    _fields_ = [("kernel", C.c_char * 32), ("flops", C.c_double), ("bytes", C.c_double), ("ms", C.c_float), ("m", C.c_int), ("n", C.c_int), ("k", C.c_int)]


EXPORTS = [
    "ad_create", "ad_destroy", "ad_last_error", "ad_num_units", "ad_get_unit", "ad_get_partition", "ad_component_io",
    "ad_tensor_shape", "ad_num_weights", "ad_get_weight", "ad_device_bytes", "ad_bind_device_memory", "ad_load_weights",
    "ad_reset", "ad_get_timesteps", "ad_num_sched_rows", "ad_get_schedule", "ad_get_sampler_coeffs",
    "ad_component_forward", "ad_step", "ad_ddim_update", "ad_sampler_update_raw", "ad_get_slot_tensor", "ad_get_eps_buffer",
    "ad_conv_forward", "ad_conv_workspace_bytes", "ad_pack_conv_weight", "ad_groupnorm_scratch_bytes", "ad_groupnorm_forward", "ad_layernorm_forward",
    "ad_attention_forward", "ad_profile_enable", "ad_profile_clear", "ad_profile_count", "ad_profile_get", "ad_tune_conv_tile", "ad_precompute_text", "ad_set_graph_mode", "ad_set_edge_mode", "ad_create_with_cuts", "ad_balance_cuts", "ad_tune_conv_order", "ad_create_wrapped", "ad_num_segments",
    "ad_attention_frames_forward", "ad_groupnorm_forward_static", "ad_tune_attention",
]


def _load():
    if not os.path.exists(lib_path):
        raise ImportError(f"{lib_path} is missing: build it with `python -m paper_2406_06911_amd.build` "
                          "(there is no fallback implementation)")
    L = C.CDLL(lib_path)
    vp, ci, cf, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    P = C.POINTER
    L.ad_last_error.restype = C.c_char_p
    L.ad_create.argtypes = [P(UNetCfg), ci, ci, ci, P(vp)]
    L.ad_create_with_cuts.argtypes = [P(UNetCfg), ci, P(ci), ci, ci, P(vp)]
    L.ad_tune_conv_order.argtypes = [ci]
    L.ad_create_wrapped.argtypes = [P(UNetCfg), ci, P(ci), ci, P(vp)]
    L.ad_num_segments.argtypes = [vp]
    L.ad_balance_cuts.argtypes = [P(C.c_int64), ci, ci, P(ci)]
    L.ad_destroy.argtypes = [vp]; L.ad_destroy.restype = None
    L.ad_num_units.argtypes = [vp]
    L.ad_get_unit.argtypes = [vp, ci, P(UnitInfo)]
    L.ad_get_partition.argtypes = [vp, P(ci), P(ci)]
    L.ad_component_io.argtypes = [vp, ci, ci, P(ci), P(ci), P(ci), P(ci)]
    L.ad_tensor_shape.argtypes = [vp, ci, P(ci), P(ci), P(ci), P(ci), P(sz)]
    L.ad_num_weights.argtypes = [vp]
    L.ad_get_weight.argtypes = [vp, ci, P(WeightInfo)]
    L.ad_device_bytes.argtypes = [vp, P(sz), P(sz)]
    L.ad_bind_device_memory.argtypes = [vp, vp, sz, vp, sz]
    L.ad_load_weights.argtypes = [vp, P(vp), ci]
    L.ad_reset.argtypes = [vp, ci, ci, ci, cf, ci]
    L.ad_get_timesteps.argtypes = [vp, P(ci), ci]
    L.ad_num_sched_rows.argtypes = [vp]
    L.ad_get_schedule.argtypes = [vp, P(SchedRow), ci]
    L.ad_get_sampler_coeffs.argtypes = [vp, ci, P(C.c_double), P(C.c_double), P(C.c_double), P(C.c_double)]
    L.ad_component_forward.argtypes = [vp, ci, ci, P(vp), ci, cf, vp, vp, P(vp), vp]
    L.ad_step.argtypes = [vp, vp, vp, vp, P(vp), ci, P(ci)]
    L.ad_ddim_update.argtypes = [vp, vp, vp, ci, cf, vp]
    L.ad_sampler_update_raw.argtypes = [vp, vp, sz, ci, cf, cf, cf, vp]
    L.ad_get_slot_tensor.argtypes = [vp, ci, ci, P(vp), P(sz)]
    L.ad_get_eps_buffer.argtypes = [vp, ci, P(vp), P(sz)]
    L.ad_conv_forward.argtypes = [ci, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, ci, vp, vp, vp, vp, vp, vp, ci, ci, vp, sz, vp]
    L.ad_conv_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci]; L.ad_conv_workspace_bytes.restype = sz
    L.ad_pack_conv_weight.argtypes = [ci, vp, ci, ci, ci, ci, vp, P(sz)]
    L.ad_groupnorm_scratch_bytes.argtypes = [ci, ci, ci]; L.ad_groupnorm_scratch_bytes.restype = sz
    L.ad_groupnorm_forward.argtypes = [ci, vp, vp, ci, ci, ci, ci, ci, vp, vp, cf, ci, vp, vp, vp]
    L.ad_groupnorm_forward_static.argtypes = [ci, vp, vp, ci, ci, ci, ci, ci, vp, vp, cf, ci, vp, vp]
    L.ad_layernorm_forward.argtypes = [ci, vp, ci, ci, vp, vp, cf, vp, vp]
    L.ad_attention_forward.argtypes = [ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp]
    L.ad_attention_frames_forward.argtypes = [ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp]
    L.ad_tune_conv_tile.argtypes = [ci]
    L.ad_tune_attention.argtypes = [ci]
    L.ad_precompute_text.argtypes = [vp, vp, vp]
    L.ad_set_graph_mode.argtypes = [vp, ci]
    L.ad_set_edge_mode.argtypes = [vp, ci]
    L.ad_profile_enable.argtypes = [vp, ci]
    L.ad_profile_clear.argtypes = [vp]
    L.ad_profile_count.argtypes = [vp]
    L.ad_profile_get.argtypes = [vp, ci, P(ProfileRec)]
    return L


lib = _load()


def check(status):
    if status != AD_OK:
        raise AsyncDiffError(status, lib.ad_last_error().decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def balance_cuts(costs, n_components):
    """Minimax contiguous split of integer per-unit costs (ad_balance_cuts); returns the n_components - 1 cuts."""
    costs = [int(c) for c in costs]
    arr = (C.c_int64 * len(costs))(*costs)
    out = (C.c_int * max(n_components - 1, 1))()
    check(lib.ad_balance_cuts(arr, len(costs), n_components, out))
    return [out[k] for k in range(n_components - 1)]


class AsyncDiff:
    """Owns an ad_ctx plus the torch tensors that back its two device arenas."""

    def __init__(self, cfg_dict, n_components, warmup, stride, dtype=AD_F32, cuts=None, wrap=False):
        self.cfg = UNetCfg.from_dict(cfg_dict, dtype)
        self.N, self.warmup, self.stride, self.dtype = n_components, warmup, stride, dtype
        self._h = C.c_void_p()
        if wrap:
            if stride != 1:
                raise ValueError("the wrapped segmentation is defined for stride 1")
            if cuts is not None and len(cuts) != n_components:
                raise ValueError("cuts must hold n_components unit indices for the wrapped segmentation")
            arr = (C.c_int * n_components)(*cuts) if cuts is not None else None
            check(lib.ad_create_wrapped(C.byref(self.cfg), n_components, arr, warmup, C.byref(self._h)))
        elif cuts is None:
            check(lib.ad_create(C.byref(self.cfg), n_components, warmup, stride, C.byref(self._h)))
        else:
            if len(cuts) != n_components - 1:
                raise ValueError("cuts must hold n_components - 1 unit indices")
            arr = (C.c_int * max(len(cuts), 1))(*cuts)
            check(lib.ad_create_with_cuts(C.byref(self.cfg), n_components, arr, warmup, stride, C.byref(self._h)))
        self._weights_t = self._work_t = None

    def close(self):
        if self._h:
            lib.ad_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- introspection -----------------------------------------------------------------------
    def units(self):
        out = []
        for i in range(lib.ad_num_units(self._h)):
            u = UnitInfo()
            check(lib.ad_get_unit(self._h, i, C.byref(u)))
            out.append(u)
        return out

    def partition(self):
        n = lib.ad_num_segments(self._h)
        a, b = (C.c_int * n)(), (C.c_int * n)()
        check(lib.ad_get_partition(self._h, a, b))
        return [(a[i], b[i]) for i in range(n)]

    def component_io(self, comp):
        cap = 128
        i, o, ni, no = (C.c_int * cap)(), (C.c_int * cap)(), C.c_int(), C.c_int()
        check(lib.ad_component_io(self._h, comp, cap, i, C.byref(ni), o, C.byref(no)))
        return list(i[:ni.value]), list(o[:no.value])

    def tensor_shape(self, unit):
        b, h, w, c, n = C.c_int(), C.c_int(), C.c_int(), C.c_int(), C.c_size_t()
        check(lib.ad_tensor_shape(self._h, unit, C.byref(b), C.byref(h), C.byref(w), C.byref(c), C.byref(n)))
        return (b.value, h.value, w.value, c.value), n.value

    def weight_manifest(self):
        out = []
        for i in range(lib.ad_num_weights(self._h)):
            w = WeightInfo()
            check(lib.ad_get_weight(self._h, i, C.byref(w)))
            out.append((w.name.decode(), tuple(w.shape[:w.ndim])))
        return out

    def device_bytes(self):
        a, b = C.c_size_t(), C.c_size_t()
        check(lib.ad_device_bytes(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    # ---- memory and weights --------------------------------------------------------------------
    def allocate(self, device="cuda:0"):
        import torch
        wb, kb = self.device_bytes()
        self._weights_t = torch.zeros(wb + 256, dtype=torch.uint8, device=device)
        self._work_t = torch.zeros(kb + 256, dtype=torch.uint8, device=device)
        al = lambda t: (t.data_ptr() + 255) // 256 * 256
        check(lib.ad_bind_device_memory(self._h, C.c_void_p(al(self._weights_t)), wb, C.c_void_p(al(self._work_t)), kb))

    def load_weights(self, weights):
        """weights: {name: float32 ndarray} covering the manifest."""
        man = self.weight_manifest()
        arrs = []
        for name, shape in man:
            a = np.ascontiguousarray(weights[name], dtype=np.float32)
            if tuple(a.shape) != tuple(shape):
                raise ValueError(f"{name}: shape {a.shape} != {shape}")
            arrs.append(a)
        ptrs = (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
        check(lib.ad_load_weights(self._h, ptrs, len(arrs)))

    # ---- run set-up ------------------------------------------------------------------------------
    def reset(self, T, sampler=AD_DDIM, beta=AD_BETA_LINEAR, cfg_scale=1.0, time_shift=False):
        self.T = T
        check(lib.ad_reset(self._h, T, sampler, beta, float(cfg_scale), int(time_shift)))

    def timesteps(self):
        a = (C.c_int * self.T)()
        check(lib.ad_get_timesteps(self._h, a, self.T))
        return list(a)

    def schedule(self):
        n = lib.ad_num_sched_rows(self._h)
        rows = (SchedRow * n)()
        check(lib.ad_get_schedule(self._h, rows, n))
        return [r.as_tuple() for r in rows]

    def sampler_coeffs(self, step):
        a, b, c, d = C.c_double(), C.c_double(), C.c_double(), C.c_double()
        check(lib.ad_get_sampler_coeffs(self._h, step, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
        return a.value, b.value, c.value, d.value

    # ---- hot path ---------------------------------------------------------------------------------
    def component_forward(self, comp, hidden_in, t_index, text_emb, hidden_out, stream, lane=0, latent_scale=1.0, pooled=None):
        pin = (C.c_void_p * len(hidden_in))(*[t.data_ptr() for t in hidden_in])
        pout = (C.c_void_p * len(hidden_out))(*[t.data_ptr() for t in hidden_out])
        check(lib.ad_component_forward(self._h, comp, lane, pin, t_index, float(latent_scale), _ptr(text_emb), _ptr(pooled),
                                       pout, C.c_void_p(stream.cuda_stream)))

    def step(self, latent, text_emb, streams, pooled=None):
        ps = (C.c_void_p * len(streams))(*[s.cuda_stream for s in streams])
        done = C.c_int()
        st = lib.ad_step(self._h, _ptr(latent), _ptr(text_emb), _ptr(pooled), ps, len(streams), C.byref(done))
        if st == AD_ERR_DONE:
            return None
        check(st)
        return done.value

    def set_graph_mode(self, on):
        check(lib.ad_set_graph_mode(self._h, int(on)))

    def set_edge_mode(self, on):
        check(lib.ad_set_edge_mode(self._h, int(on)))

    def precompute_text(self, text_emb, stream):
        check(lib.ad_precompute_text(self._h, _ptr(text_emb), C.c_void_p(stream.cuda_stream)))

    def ddim_update(self, x, eps, step_index, cfg_scale, stream):
        check(lib.ad_ddim_update(self._h, _ptr(x), _ptr(eps), step_index, float(cfg_scale), C.c_void_p(stream.cuda_stream)))

    def profile(self, on):
        check(lib.ad_profile_enable(self._h, int(on)))

    def profile_records(self, clear=True):
        """[(kernel, flops, bytes, ms)] of every launch recorded so far (waits for them to finish)."""
        out = []
        r = ProfileRec()
        for i in range(lib.ad_profile_count(self._h)):
            check(lib.ad_profile_get(self._h, i, C.byref(r)))
            out.append((r.kernel.decode(), r.flops, r.bytes, r.ms, (r.m, r.n, r.k)))
        if clear:
            check(lib.ad_profile_clear(self._h))
        return out

    def slot_tensor_ptr(self, slot, unit):
        p, n = C.c_void_p(), C.c_size_t()
        check(lib.ad_get_slot_tensor(self._h, slot, unit, C.byref(p), C.byref(n)))
        return p.value, n.value

    def eps_buffer_ptr(self, j):
        p, n = C.c_void_p(), C.c_size_t()
        check(lib.ad_get_eps_buffer(self._h, j, C.byref(p), C.byref(n)))
        return p.value, n.value


def pack_conv_weight(dtype, w, geglu=False):
    """Returns the packed weight as a uint8 ndarray (host)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim == 2:
        w = w[:, :, None, None]
    n_out, c_in, k, _ = w.shape
    nbytes = C.c_size_t()
    check(lib.ad_pack_conv_weight(dtype, None, n_out, c_in, k, int(geglu), None, C.byref(nbytes)))
    out = np.zeros(nbytes.value, np.uint8)
    check(lib.ad_pack_conv_weight(dtype, C.c_void_p(w.ctypes.data), n_out, c_in, k, int(geglu), C.c_void_p(out.ctypes.data), C.byref(nbytes)))
    return out
