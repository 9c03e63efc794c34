"""ctypes binding of libhsd.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used to own device
memory and the stream.  Importing this module fails loudly when the library has not been built
(python -m paper_2510_19705_amd.build); there is no CPU fallback.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhsd.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libhsd.so is not built: run `python -m paper_2510_19705_amd.build` (needs hipcc)")
lib = C.CDLL(LIB_PATH)

F32, BF16 = 0, 1
LAYOUT_TILES, LAYOUT_ROWS = 0, 1
MAX_LEVELS, MAX_PASS_ROWS, KV_PAGE = 8, 64, 64


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("d", C.c_int), ("n_q", C.c_int), ("n_kv", C.c_int), ("hd", C.c_int),
                ("ffn", C.c_int), ("vocab", C.c_int), ("dtype", C.c_int), ("rope_base", C.c_float), ("eps", C.c_float),
                ("max_seq", C.c_int), ("max_rows", C.c_int), ("rows_copy_layers", C.c_int)]


class LayerWeights(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("norm1_dev", "wq_dev", "wk_dev", "wv_dev", "wo_dev", "norm2_dev", "wg_dev",
                                          "wu_dev", "wd_dev")]


class Level(C.Structure):
    _fields_ = [("model", C.c_void_p), ("exit_layer", C.c_int)]


N_SITES = 6
SITE_NAMES = ("qkv", "attn", "o", "gateup", "down", "head")


class SiteTimes(C.Structure):
    _fields_ = [("launches", C.c_int64 * N_SITES), ("ms", C.c_double * N_SITES), ("empty_bracket_ms", C.c_double)]


class KernelTuning(C.Structure):
    """hsd_kernel_tuning (include/hsd_dev.h): launch heuristics of one model / one stand-alone call."""
    _fields_ = [("gemm_nt", C.c_int * 4), ("gemm_ksplit", C.c_int * 4), ("gemm_deep", C.c_int), ("gemm_interleave", C.c_int * 4),
                ("gemv_max_m_qkv", C.c_int), ("gemv_max_m_o", C.c_int), ("gemv_max_m_down", C.c_int),
                ("halves_max_groups", C.c_int), ("attn_qt1_rows", C.c_int), ("attn_steps_per_wave", C.c_int),
                ("attn_target_wgs", C.c_int), ("attn_fused_merge", C.c_int), ("wide_min_rows", C.c_int), ("wide_cols", C.c_int)]


class DriverTuning(C.Structure):
    """hsd_driver_tuning: the round driver's choices for one hierarchy."""
    _fields_ = [("fused_sampler_max_v", C.c_int), ("preembed", C.c_int), ("poll_mailbox", C.c_int)]


class Stats(C.Structure):
    _fields_ = [("passes", C.c_int64 * MAX_LEVELS), ("pass_rows", C.c_int64 * MAX_LEVELS),
                ("drafted", C.c_int64 * MAX_LEVELS), ("accepted", C.c_int64 * MAX_LEVELS),
                ("tested", C.c_int64 * MAX_LEVELS), ("reused_rows", C.c_int64 * MAX_LEVELS), ("rounds", C.c_int64),
                ("tokens", C.c_int64)]


_vp, _i, _sz, _f, _d = C.c_void_p, C.c_int, C.c_size_t, C.c_float, C.c_double
_ip, _dp = C.POINTER(C.c_int), C.POINTER(C.c_double)
_SIGS = {
    "hsd_model_weight_bytes": (_sz, [C.POINTER(ModelDesc)]),
    "hsd_model_kv_bytes": (_sz, [C.POINTER(ModelDesc)]),
    "hsd_model_scratch_bytes": (_sz, [C.POINTER(ModelDesc)]),
    "hsd_model_create": (_i, [C.POINTER(ModelDesc), _vp, _vp, _vp, _vp, C.POINTER(_vp)]),
    "hsd_model_destroy": (None, [_vp]),
    "hsd_model_load_layer": (_i, [_vp, _i, C.POINTER(LayerWeights)]),
    "hsd_model_load_head": (_i, [_vp, _vp, _vp, _vp]),
    "hsd_model_set_pages": (_i, [_vp, C.POINTER(C.c_int32), _i]),
    "hsd_model_pass": (_i, [_vp, _vp, _i, _i, _i, _i, _vp]),
    "hsd_model_set_batch": (_i, [_vp, _i, _i, C.POINTER(C.c_int32)]),
    "hsd_model_pass_batch": (_i, [_vp, _vp, C.POINTER(C.c_int32), _i, _i, _i, _vp]),
    "hsd_hier_set_reuse": (_i, [_vp, _i]),
    "hsd_hier_set_ablation": (_i, [_vp, C.POINTER(C.c_float), _i]),
    "hsd_hier_set_distilled": (_i, [_vp, _i, _i, _f]),
    "hsd_stats_cost": (C.c_double, [C.POINTER(Stats), _i, C.POINTER(C.c_double)]),
    "hsd_model_pass_exits": (_i, [_vp, _vp, _i, _i, C.POINTER(C.c_int), _i, _i, _vp]),
    "hsd_overlap": (_i, [_vp, _i, _i, _i, _vp, _vp]),
    "hsd_calibrate_workspace_bytes": (C.c_size_t, [_vp, _i, _i, _i]),
    "hsd_calibrate_levels_workspace_bytes": (C.c_size_t, [_i, C.POINTER(Level), _i, _i]),
    "hsd_calibrate_levels": (_i, [_i, C.POINTER(Level), _vp, _i, _i, C.c_float, _i, _vp, C.c_size_t, C.POINTER(C.c_double),
                                  C.POINTER(C.c_double)]),
    "hsd_calibrate": (_i, [_vp, C.POINTER(C.c_int), _i, _vp, _i, _i, C.c_float, _i, _vp, C.c_size_t, C.POINTER(C.c_double),
                           C.POINTER(C.c_double)]),
    "hsd_profile_begin": (_i, [_vp, _i]),
    "hsd_profile_end": (_i, [_vp, C.POINTER(SiteTimes)]),
    "hsd_measure_site": (_i, [_vp, _i, _i, _i, _i, _dp]),
    "hsd_site_kernel": (_i, [_vp, _i, _i, C.c_char_p, _i]),
    "hsd_softmax_scratch_bytes": (_sz, [_i, _i]),
    "hsd_softmax": (_i, [_vp, _vp, _i, _i, _f, _vp, _vp]),
    "hsd_sampler_scratch_bytes": (_sz, [_i]),
    "hsd_accept_resample": (_i, [_vp, _vp, _vp, _i, _i, C.c_uint64, C.c_uint32, C.c_uint32, _vp, _vp, _vp]),
    "hsd_accept_resample_static": (_i, [_vp, _vp, _vp, _i, _i, C.c_uint64, C.c_uint32, C.c_uint32, _vp, _vp]),
    "hsd_softmax_verify": (_i, [_vp, _vp, _vp, _i, _i, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32, _vp, _vp, _vp, _vp, _vp]),
    "hsd_kv_layer_bytes": (_sz, [_i, _i, _i, _i]),
    "hsd_attention_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "hsd_kv_write": (_i, [_vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp]),
    "hsd_attention": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp]),
    "hsd_packed_bytes": (_sz, [_i, _i, _i]),
    "hsd_gemm_workspace_bytes": (_sz, [_i, _i, _i]),
    "hsd_pack_weight": (_i, [_vp, _vp, _i, _i, _i, _i, _vp]),
    "hsd_gemm": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp]),
    "hsd_kernel_tuning_default": (None, [C.POINTER(KernelTuning)]),
    "hsd_driver_tuning_default": (None, [C.POINTER(DriverTuning)]),
    "hsd_model_set_tuning": (_i, [_vp, C.POINTER(KernelTuning)]),
    "hsd_hier_set_tuning": (_i, [_vp, C.POINTER(DriverTuning)]),
    "hsd_gemm_tuned": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, C.POINTER(KernelTuning)]),
    "hsd_attention_tuned": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, C.POINTER(KernelTuning)]),
    "hsd_hier_workspace_bytes": (_sz, [_i, C.POINTER(Level), _ip]),
    "hsd_hier_create": (_i, [_i, C.POINTER(Level), _ip, _f, C.c_uint64, _vp, _sz, _vp, C.POINTER(_vp)]),
    "hsd_hier_destroy": (None, [_vp]),
    "hsd_prefill": (_i, [_vp, C.POINTER(C.c_int32), _i]),
    "hsd_prefill_cached": (_i, [_vp, C.POINTER(C.c_int32), _i, _i]),
    "hsd_rewind": (_i, [_vp, _i]),
    "hsd_hier_set_seed": (_i, [_vp, C.c_uint64]),
    "hsd_draft": (_i, [_vp, _i, _i, C.POINTER(C.c_int32), C.POINTER(_vp)]),
    "hsd_verify": (_i, [_vp, _i, C.POINTER(C.c_int32), _vp, _i, _i, C.POINTER(C.c_int32), _ip, C.POINTER(_vp)]),
    "hsd_run": (_i, [_vp, _i, C.POINTER(C.c_int32), _i, _ip, C.POINTER(_vp)]),
    "hsd_generate": (_i, [_vp, _i, C.POINTER(C.c_int32), C.POINTER(Stats)]),
    "hsd_batch_workspace_bytes": (_sz, [_i, C.POINTER(Level), _ip, _i, _i]),
    "hsd_batch_create": (_i, [_i, C.POINTER(Level), _ip, _i, _i, _f, C.POINTER(C.c_uint64), _vp, _sz, _vp, C.POINTER(_vp)]),
    "hsd_batch_destroy": (None, [_vp]),
    "hsd_batch_prefill": (_i, [_vp, C.POINTER(C.c_int32), _i, _ip]),
    "hsd_batch_generate": (_i, [_vp, _i, C.POINTER(C.c_int32), C.POINTER(Stats)]),
    "hsd_batch_sequence_length": (_i, [_vp, _i]),
    "hsd_get_stats": (_i, [_vp, C.POINTER(Stats)]),
    "hsd_sequence_length": (_i, [_vp]),
    "hsd_measure_pass": (_i, [_vp, _i, _i, _i, _dp]),
    "hsd_gamma": (_d, [_d, _i, _i]),
    "hsd_expected_latency": (_d, [_i, _dp, _dp, _ip, _i]),
    "hsd_select_hierarchy": (_i, [_i, _dp, _dp, _i, _i, _ip, _ip, _ip, _dp]),
    "hsd_best_single_draft": (_i, [_i, _dp, _dp, _i, _ip, _ip, _dp]),
    "hsd_last_error": (C.c_char_p, []),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args
EXPORTS = tuple(_SIGS)


class HsdError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__("libhsd error %d: %s" % (code, lib.hsd_last_error().decode()))


def _check(rc):
    if rc != 0:
        raise HsdError(rc)


def kernel_tuning(**settings):
    """The library's default launch heuristics with the given fields replaced (gemm_nt / gemm_ksplit / gemm_interleave: dict epilogue -> value)."""
    k = KernelTuning()
    lib.hsd_kernel_tuning_default(C.byref(k))
    for name, v in settings.items():
        if name in ("gemm_nt", "gemm_ksplit", "gemm_interleave"):
            for epi, val in v.items():
                getattr(k, name)[epi] = val
        else:
            if not hasattr(k, name):
                raise AttributeError(name)
            setattr(k, name, v)
    return k


def driver_tuning(**settings):
    d = DriverTuning()
    lib.hsd_driver_tuning_default(C.byref(d))
    for name, v in settings.items():
        if not hasattr(d, name):
            raise AttributeError(name)
        setattr(d, name, v)
    return d


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _buf(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def _rows_view(ptr, rows, vocab, keepalive):
    """Zero-copy torch view of `rows` fp32 distribution rows at a borrowed device pointer."""
    base = keepalive.data_ptr()
    off = ptr - base
    assert 0 <= off and off + rows * vocab * 4 <= keepalive.numel(), "borrowed pointer outside the workspace"
    return keepalive[off:off + rows * vocab * 4].view(torch.float32).view(rows, vocab)


# ---- model -----------------------------------------------------------------------------------
class Model:
    def __init__(self, shape, dtype, max_seq, max_rows, rope_base=10000.0, eps=1e-5, rows_copy_layers=0):
        self.desc = ModelDesc(shape["n_layers"], shape["d"], shape["n_q"], shape["n_kv"], shape["hd"], shape["ffn"],
                              shape["vocab"], dtype, rope_base, eps, max_seq, max_rows, rows_copy_layers)
        self.dtype = dtype
        self.tdtype = torch.bfloat16 if dtype == BF16 else torch.float32
        self.stream = _stream()
        nbytes = [lib.hsd_model_weight_bytes(C.byref(self.desc)), lib.hsd_model_kv_bytes(C.byref(self.desc)),
                  lib.hsd_model_scratch_bytes(C.byref(self.desc))]
        if 0 in nbytes:
            raise HsdError(-1)
        self.weights, self.kv, self.scratch = (_buf(n) for n in nbytes)
        self.handle = C.c_void_p()
        _check(lib.hsd_model_create(C.byref(self.desc), self.weights.data_ptr(), self.kv.data_ptr(),
                                    self.scratch.data_ptr(), self.stream, C.byref(self.handle)))

    def close(self):
        if self.handle:
            lib.hsd_model_destroy(self.handle)
            self.handle = C.c_void_p()

    def _dev(self, a, norm=False):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        return t if norm else t.to(self.tdtype).contiguous()

    def load_layer(self, layer, w):
        """hsd_model_load_layer with host fp32 arrays (already bf16-representable for bf16 models)."""
        keep = {k: self._dev(w[k], norm=k.startswith("norm")) for k in
                ("norm1", "wq", "wk", "wv", "wo", "norm2", "wg", "wu", "wd")}
        lw = LayerWeights(*[keep[k].data_ptr() for k in ("norm1", "wq", "wk", "wv", "wo", "norm2", "wg", "wu", "wd")])
        torch.cuda.current_stream().synchronize()
        _check(lib.hsd_model_load_layer(self.handle, layer, C.byref(lw)))

    def load_layer_dev(self, layer, t):
        """hsd_model_load_layer with cuda tensors already in the model's element type (norms fp32)."""
        order = ("norm1", "wq", "wk", "wv", "wo", "norm2", "wg", "wu", "wd")
        lw = LayerWeights(*[t[k].contiguous().data_ptr() for k in order])
        torch.cuda.current_stream().synchronize()
        _check(lib.hsd_model_load_layer(self.handle, layer, C.byref(lw)))

    def load_head_dev(self, embed, head, norm_f):
        torch.cuda.current_stream().synchronize()
        _check(lib.hsd_model_load_head(self.handle, embed.data_ptr(), head.data_ptr(), norm_f.data_ptr()))

    def load_head(self, embed, head, norm_f):
        e, h, n = self._dev(embed), self._dev(head), self._dev(norm_f, norm=True)
        torch.cuda.current_stream().synchronize()
        _check(lib.hsd_model_load_head(self.handle, e.data_ptr(), h.data_ptr(), n.data_ptr()))

    def load(self, weights):
        for i, lw in enumerate(weights["layers"]):
            self.load_layer(i, lw)
        self.load_head(weights["embed"], weights["head"], weights["norm_f"])

    def profile_begin(self, max_launches):
        _check(lib.hsd_profile_begin(self.handle, max_launches))

    def profile_end(self):
        st = SiteTimes()
        _check(lib.hsd_profile_end(self.handle, C.byref(st)))
        out = {SITE_NAMES[i]: (st.launches[i], st.ms[i]) for i in range(N_SITES)}
        out["empty_bracket_ms"] = st.empty_bracket_ms
        return out

    def measure_site(self, site, rows, pos0, iters):
        us = C.c_double()
        _check(lib.hsd_measure_site(self.handle, SITE_NAMES.index(site), rows, pos0, iters, C.byref(us)))
        return us.value

    def set_tuning(self, **settings):
        """hsd_model_set_tuning: this model's launch heuristics = the defaults with `settings` replaced (none: defaults)."""
        _check(lib.hsd_model_set_tuning(self.handle, C.byref(kernel_tuning(**settings)) if settings else None))

    def site_kernel(self, site, rows):
        buf = C.create_string_buffer(128)
        _check(lib.hsd_site_kernel(self.handle, SITE_NAMES.index(site), rows, buf, 128))
        return buf.value.decode()

    def set_pages(self, table):
        a, p = _i32(table)
        _check(lib.hsd_model_set_pages(self.handle, p, len(a)))

    def model_pass(self, tokens_dev, pos0, exit_layer, n_logit_rows):
        """hsd_model_pass; tokens_dev: int32 cuda tensor.  Returns fp32 logits [n_logit_rows, vocab]."""
        logits = torch.empty((max(n_logit_rows, 1), self.desc.vocab), dtype=torch.float32, device="cuda")
        _check(lib.hsd_model_pass(self.handle, tokens_dev.data_ptr(), pos0, tokens_dev.numel(), exit_layer, n_logit_rows,
                                  logits.data_ptr()))
        return logits[:n_logit_rows]

    def set_batch(self, batch, pages_per_seq=0, page_table=None):
        """hsd_model_set_batch; page_table: [batch, pages_per_seq] ints (default: consecutive pages per sequence)."""
        if batch == 0:
            _check(lib.hsd_model_set_batch(self.handle, 0, 0, None))
            return
        if page_table is None:
            page_table = np.arange(batch * pages_per_seq, dtype=np.int32)
        a, p = _i32(np.asarray(page_table).reshape(-1))
        _check(lib.hsd_model_set_batch(self.handle, batch, pages_per_seq, p))

    def model_pass_batch(self, tokens_dev, pos0, exit_layer, with_logits=True):
        """hsd_model_pass_batch; tokens_dev: int32 cuda tensor [batch, m]; pos0: host ints [batch].
        Returns fp32 logits [batch, m, vocab] (None without logits)."""
        batch, m = tokens_dev.shape
        a, p = _i32(pos0)
        logits = torch.empty((batch, m, self.desc.vocab), dtype=torch.float32, device="cuda") if with_logits else None
        _check(lib.hsd_model_pass_batch(self.handle, tokens_dev.contiguous().data_ptr(), p, m, exit_layer, int(with_logits),
                                        logits.data_ptr() if with_logits else None))
        return logits

    def model_pass_exits(self, tokens_dev, pos0, exits, n_logit_rows):
        """hsd_model_pass_exits.  Returns fp32 logits [len(exits), n_logit_rows, vocab]."""
        logits = torch.empty((len(exits), max(n_logit_rows, 1), self.desc.vocab), dtype=torch.float32, device="cuda")
        arr = (C.c_int * len(exits))(*exits)
        _check(lib.hsd_model_pass_exits(self.handle, tokens_dev.data_ptr(), pos0, tokens_dev.numel(), arr, len(exits),
                                        n_logit_rows, logits.data_ptr()))
        return logits[:, :n_logit_rows]

    def calibrate(self, exits, tokens_dev, n_ctx, temperature, cost_rows=0):
        """hsd_calibrate.  Returns (alpha [n, n] numpy fp64, costs in ms [n] or None)."""
        n, n_tokens = len(exits), tokens_dev.numel()
        nbytes = lib.hsd_calibrate_workspace_bytes(self.handle, n, n_tokens, n_ctx)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        arr = (C.c_int * n)(*exits)
        alpha = (C.c_double * (n * n))()
        cost = (C.c_double * n)() if cost_rows > 0 else None
        _check(lib.hsd_calibrate(self.handle, arr, n, tokens_dev.data_ptr(), n_tokens, n_ctx, float(temperature), cost_rows,
                                 ws.data_ptr(), nbytes, alpha, cost))
        return np.array(alpha[:]).reshape(n, n), (np.array(cost[:]) if cost is not None else None)


def calibrate_levels(levels, tokens_dev, n_ctx, temperature, cost_rows=0):
    """hsd_calibrate_levels.  levels: list of (Model, exit_layer).  Returns (alpha [n, n] numpy fp64, costs in ms or None)."""
    n, n_tokens = len(levels), tokens_dev.numel()
    lv = (Level * n)(*[Level(m.handle, e) for m, e in levels])
    nbytes = lib.hsd_calibrate_levels_workspace_bytes(n, lv, n_tokens, n_ctx)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    alpha = (C.c_double * (n * n))()
    cost = (C.c_double * n)() if cost_rows > 0 else None
    _check(lib.hsd_calibrate_levels(n, lv, tokens_dev.data_ptr(), n_tokens, n_ctx, float(temperature), cost_rows, ws.data_ptr(),
                                    nbytes, alpha, cost))
    return np.array(alpha[:]).reshape(n, n), (np.array(cost[:]) if cost is not None else None)


def overlap(rows):
    """hsd_overlap.  rows: fp32 cuda tensor [n_dists, n_rows, vocab].  Returns fp64 cuda tensor [n_pairs, n_rows]."""
    rows = rows.contiguous()
    n, r, v = rows.shape
    out = torch.empty((n * (n - 1) // 2, r), dtype=torch.float64, device="cuda")
    _check(lib.hsd_overlap(rows.data_ptr(), n, r, v, out.data_ptr(), _stream()))
    return out


# ---- stand-alone kernels ----------------------------------------------------------------------
def softmax(logits, temperature):
    logits = logits.contiguous()
    out = torch.empty_like(logits)
    nb = lib.hsd_softmax_scratch_bytes(logits.shape[0], logits.shape[1])
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda") if nb else None
    _check(lib.hsd_softmax(logits.data_ptr(), out.data_ptr(), logits.shape[0], logits.shape[1], float(temperature),
                           scratch.data_ptr() if nb else None, _stream()))
    return out


_sampler_scratch = {}


def accept_resample(p, q, x, seed, level, call):
    """p [t+1, V], q [t, V] fp32 cuda tensors, x int32 cuda tensor [t+1] (x_1..x_t, one spare).
    Returns (n, m) after synchronising; x[n] = m on the device."""
    t, V = p.shape[0] - 1, p.shape[1]
    key = (V, torch.cuda.current_device())
    if key not in _sampler_scratch:
        _sampler_scratch[key] = torch.zeros(lib.hsd_sampler_scratch_bytes(V), dtype=torch.uint8, device="cuda")
    res = torch.empty(2, dtype=torch.int32, device="cuda")
    _check(lib.hsd_accept_resample(p.data_ptr(), q.data_ptr() if t > 0 else None, x.data_ptr(), t, V, seed, level, call,
                                   res.data_ptr(), _sampler_scratch[key].data_ptr(), _stream()))
    n, m = res.cpu().tolist()
    return n, m


def accept_resample_static(p, q, x, seed, level, call):
    """hsd_accept_resample_static: as accept_resample, with the library's built-in scratch (no buffer is created here:
    the result words are the caller's).  Returns the int32 cuda tensor [2] (n, m); x[n] = m on the device."""
    t, V = p.shape[0] - 1, p.shape[1]
    res = torch.empty(2, dtype=torch.int32, device="cuda")
    _check(lib.hsd_accept_resample_static(p.data_ptr(), q.data_ptr() if t > 0 else None, x.data_ptr(), t, V, seed, level, call,
                                          res.data_ptr(), _stream()))
    return res


def softmax_verify(z, q, x, temperature, seed, level, call, want_probs=True, mailbox=None):
    """hsd_softmax + hsd_accept_resample in one launch.  z [t+1, V] fp32 logits, q [t, V] fp32, x int32 [t+1] (cuda).
    mailbox: optional pinned int32 host tensor (t + 3 entries).  Returns (n, m, probs or None) after synchronising."""
    t, V = z.shape[0] - 1, z.shape[1]
    key = (V, torch.cuda.current_device())
    if key not in _sampler_scratch:
        _sampler_scratch[key] = torch.zeros(lib.hsd_sampler_scratch_bytes(V), dtype=torch.uint8, device="cuda")
    res = torch.empty(2, dtype=torch.int32, device="cuda")
    probs = torch.empty_like(z) if want_probs else None
    _check(lib.hsd_softmax_verify(z.data_ptr(), q.data_ptr() if t > 0 else None, x.data_ptr(), t, V, temperature, seed, level,
                                  call, probs.data_ptr() if want_probs else None, res.data_ptr(),
                                  _sampler_scratch[key].data_ptr(), mailbox.data_ptr() if mailbox is not None else None,
                                  _stream()))
    n, m = res.cpu().tolist()
    return n, m, probs


class KvLayer:
    """One layer's paged KV cache for a batch of sequences (stand-alone attention tests and micro-benchmarks)."""

    def __init__(self, batch, max_len, n_kv, hd, dtype, page_perm=None):
        self.batch, self.n_kv, self.hd, self.dtype = batch, n_kv, hd, dtype
        self.max_pages = (max_len + KV_PAGE - 1) // KV_PAGE
        n_pages = batch * self.max_pages
        self.buf = torch.zeros(lib.hsd_kv_layer_bytes(n_pages, n_kv, hd, dtype), dtype=torch.uint8, device="cuda")
        table = np.arange(n_pages, dtype=np.int32) if page_perm is None else np.asarray(page_perm, dtype=np.int32)
        self.pages = torch.from_numpy(table.reshape(batch, self.max_pages).copy()).cuda()

    def write(self, pos0, k, v):
        """k, v: cuda tensors [batch, n, n_kv, hd] of the cache's element type; pos0: int32 cuda tensor [batch]."""
        _check(lib.hsd_kv_write(self.buf.data_ptr(), self.pages.data_ptr(), self.max_pages, pos0.data_ptr(), self.batch,
                                k.shape[1], self.n_kv, self.hd, self.dtype, k.contiguous().data_ptr(),
                                v.contiguous().data_ptr(), _stream()))

    def attention(self, q, pos0, max_len, ws=None, tuning=None):
        """q: [batch, m, n_q, hd]; returns att of the same shape and type.  tuning: a KernelTuning (hsd_attention_tuned)."""
        b, m, n_q, hd = q.shape
        if ws is None:       # zero on first use: the workspace begins with arrival counters
            ws = torch.zeros(max(256, lib.hsd_attention_workspace_bytes(b, m, n_q, self.n_kv, hd, max_len)), dtype=torch.uint8, device="cuda")
        out = torch.empty_like(q)
        args = (q.contiguous().data_ptr(), self.buf.data_ptr(), self.pages.data_ptr(), self.max_pages, pos0.data_ptr(), b, m, max_len,
                n_q, self.n_kv, hd, self.dtype, out.data_ptr(), ws.data_ptr(), _stream())
        _check(lib.hsd_attention(*args) if tuning is None else lib.hsd_attention_tuned(*args, C.byref(tuning)))
        return out


def pack_weight(w, dtype, layout=LAYOUT_TILES):
    """w: cuda tensor [n, k] of the dtype's element type; returns the packed buffer."""
    n, k = w.shape
    out = _buf(lib.hsd_packed_bytes(n, k, dtype))
    _check(lib.hsd_pack_weight(w.contiguous().data_ptr(), out.data_ptr(), n, k, dtype, layout, _stream()))
    return out


def gemm(x, packed, n, dtype, ws=None, layout=LAYOUT_TILES, tuning=None):
    m, k = x.shape
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    if ws is None:
        ws = _buf(lib.hsd_gemm_workspace_bytes(m, n, k))
    args = (x.contiguous().data_ptr(), packed.data_ptr(), y.data_ptr(), m, n, k, dtype, layout, ws.data_ptr(), _stream())
    _check(lib.hsd_gemm(*args) if tuning is None else lib.hsd_gemm_tuned(*args, C.byref(tuning)))
    return y


# ---- hierarchy --------------------------------------------------------------------------------
class Hierarchy:
    def __init__(self, levels, T, temperature, seed):
        """levels: list of (Model, exit_layer) from the smallest drafter to the target."""
        self.models = [m for m, _ in levels]
        self.n = len(levels)
        self.K = self.n - 1
        self.T = list(T)
        self.vocab = levels[0][0].desc.vocab
        self._lv = (Level * self.n)(*[Level(m.handle, e) for m, e in levels])
        self._T = (C.c_int * max(1, self.K))(*self.T)
        nbytes = lib.hsd_hier_workspace_bytes(self.n, self._lv, self._T)
        self.handle = C.c_void_p()
        if nbytes == 0:      # invalid hierarchy: let create report the status code
            _check(lib.hsd_hier_create(self.n, self._lv, self._T, float(temperature), seed, None, 0,
                                       self.models[0].stream, C.byref(self.handle)))
        self.workspace = _buf(nbytes)
        _check(lib.hsd_hier_create(self.n, self._lv, self._T, float(temperature), seed, self.workspace.data_ptr(),
                                   self.workspace.numel(), self.models[0].stream, C.byref(self.handle)))

    def close(self):
        if self.handle:
            lib.hsd_hier_destroy(self.handle)
            self.handle = C.c_void_p()

    def prefill(self, prompt):
        a, p = _i32(prompt)
        _check(lib.hsd_prefill(self.handle, p, len(a)))

    def prefill_cached(self, prompt, n_cached):
        """hsd_prefill_cached: the first n_cached tokens' K/V are already in every network's cache."""
        a, p = _i32(prompt)
        _check(lib.hsd_prefill_cached(self.handle, p, len(a), n_cached))

    def rewind(self, n):
        _check(lib.hsd_rewind(self.handle, n))

    def set_seed(self, seed):
        _check(lib.hsd_hier_set_seed(self.handle, seed))

    def draft(self, k, level=0):
        toks = np.zeros(k, dtype=np.int32)
        ptr = C.c_void_p()
        _check(lib.hsd_draft(self.handle, level, k, toks.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(ptr)))
        return toks, _rows_view(ptr.value, k, self.vocab, self.workspace)

    def verify(self, level, draft_tokens, draft_probs, t, append=False):
        """draft_tokens: host ids to append first, or None when the drafts are already the last t tokens."""
        out = np.zeros(t + 1, dtype=np.int32)
        n1 = C.c_int()
        ptr = C.c_void_p()
        dt = None
        if draft_tokens is not None:
            keep, dt = _i32(draft_tokens)
        _check(lib.hsd_verify(self.handle, level, dt, draft_probs.data_ptr(), t, int(append),
                              out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n1), C.byref(ptr)))
        return out[:n1.value], _rows_view(ptr.value, n1.value, self.vocab, self.workspace)

    def run(self, level, cap=256):
        out = np.zeros(cap, dtype=np.int32)
        n = C.c_int()
        ptr = C.c_void_p()
        _check(lib.hsd_run(self.handle, level, out.ctypes.data_as(C.POINTER(C.c_int32)), cap, C.byref(n), C.byref(ptr)))
        return out[:n.value], _rows_view(ptr.value, n.value, self.vocab, self.workspace)

    def generate(self, n_tokens):
        out = np.zeros(n_tokens, dtype=np.int32)
        st = Stats()
        _check(lib.hsd_generate(self.handle, n_tokens, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(st)))
        return out, st

    def set_distilled(self, level, source_level, noise_std):
        """hsd_hier_set_distilled: level's logits = source level's logits + seeded Gaussian noise (synthetic drafter)."""
        _check(lib.hsd_hier_set_distilled(self.handle, level, source_level, float(noise_std)))

    def set_tuning(self, **settings):
        """hsd_hier_set_tuning: the driver's choices for this hierarchy = the defaults with `settings` replaced."""
        _check(lib.hsd_hier_set_tuning(self.handle, C.byref(driver_tuning(**settings)) if settings else None))

    def set_reuse(self, on=True):
        """hsd_hier_set_reuse: verifier passes resume from the hidden states the shallower exit below has kept."""
        _check(lib.hsd_hier_set_reuse(self.handle, int(on)))

    def set_ablation(self, coin=None, exactly_T=False):
        """hsd_hier_set_ablation: coin = per-level fixed acceptance probabilities (entry 0 ignored, negative = real)."""
        arr = None
        if coin is not None:
            arr = (C.c_float * MAX_LEVELS)(*([float(c) for c in coin] + [-1.0] * (MAX_LEVELS - len(coin))))
        _check(lib.hsd_hier_set_ablation(self.handle, arr, int(exactly_T)))

    def stats(self):
        st = Stats()
        _check(lib.hsd_get_stats(self.handle, C.byref(st)))
        return st

    def sequence_length(self):
        return lib.hsd_sequence_length(self.handle)

    def measure_pass(self, level, m, iters):
        ms = C.c_double()
        _check(lib.hsd_measure_pass(self.handle, level, m, iters, C.byref(ms)))
        return ms.value


# ---- host-side latency model ------------------------------------------------------------------
class BatchHierarchy:
    """hsd_batch_*: HSD over several sequences in lockstep; sequence b is decoded as Hierarchy would decode it alone
    with seeds[b].  Every model needs max_seq >= batch * max_len."""

    def __init__(self, levels, T, temperature, seeds, max_len):
        self.models = [m for m, _ in levels]
        self.n, self.K, self.B = len(levels), len(levels) - 1, len(seeds)
        self.vocab = levels[0][0].desc.vocab
        self._lv = (Level * self.n)(*[Level(m.handle, e) for m, e in levels])
        self._T = (C.c_int * max(1, self.K))(*list(T))
        self._seeds = (C.c_uint64 * self.B)(*[int(x) for x in seeds])
        nbytes = lib.hsd_batch_workspace_bytes(self.n, self._lv, self._T, self.B, max_len)
        self.handle = C.c_void_p()
        if nbytes == 0:      # invalid configuration: let create report the status code
            _check(lib.hsd_batch_create(self.n, self._lv, self._T, self.B, max_len, float(temperature), self._seeds, None, 0,
                                        self.models[0].stream, C.byref(self.handle)))
        self.workspace = _buf(nbytes)
        _check(lib.hsd_batch_create(self.n, self._lv, self._T, self.B, max_len, float(temperature), self._seeds,
                                    self.workspace.data_ptr(), self.workspace.numel(), self.models[0].stream, C.byref(self.handle)))

    def close(self):
        if self.handle:
            lib.hsd_batch_destroy(self.handle)
            self.handle = C.c_void_p()
            for m in set(self.models):
                m.set_batch(0)

    def prefill(self, prompts):
        """prompts: one sequence of token ids per batch entry (lengths may differ)."""
        assert len(prompts) == self.B
        lens = np.array([len(p) for p in prompts], dtype=np.int32)
        flat = np.zeros((self.B, int(lens.max())), dtype=np.int32)
        for b, p in enumerate(prompts):
            flat[b, :len(p)] = np.asarray(p, dtype=np.int32)
        _check(lib.hsd_batch_prefill(self.handle, flat.ctypes.data_as(C.POINTER(C.c_int32)), flat.shape[1],
                                     lens.ctypes.data_as(C.POINTER(C.c_int))))

    def generate(self, n_tokens):
        out = np.zeros((self.B, n_tokens), dtype=np.int32)
        st = Stats()
        _check(lib.hsd_batch_generate(self.handle, n_tokens, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(st)))
        return out, st

    def sequence_length(self, b):
        return lib.hsd_batch_sequence_length(self.handle, b)


def stats_cost(st, cost):
    """hsd_stats_cost: sum of passes[i] * cost[i]."""
    c, cp = _f64(cost)
    return lib.hsd_stats_cost(C.byref(st), len(c), cp)


def gamma(alpha, Ti, Tj):
    return lib.hsd_gamma(alpha, Ti, Tj)


def expected_latency(cost, alpha_adj, T, exact_overshoot=False):
    c, cp = _f64(cost)
    a, ap = _f64(alpha_adj if len(alpha_adj) else [0.0])
    Ta = (C.c_int * max(1, len(T)))(*T)
    return lib.hsd_expected_latency(len(c), cp, ap, Ta, int(exact_overshoot))


def select_hierarchy(cost, alpha, Tbar, monotone_T=True):
    n = len(cost)
    c, cp = _f64(cost)
    a, ap = _f64(np.asarray(alpha, dtype=np.float64).reshape(n, n))
    sig, Ts = (C.c_int * n)(), (C.c_int * max(1, n - 1))()
    ns, lat = C.c_int(), C.c_double()
    _check(lib.hsd_select_hierarchy(n, cp, ap, Tbar, int(monotone_T), sig, Ts, C.byref(ns), C.byref(lat)))
    return lat.value, list(sig[:ns.value]), list(Ts[:ns.value - 1])


def best_single_draft(cost, alpha, Tbar):
    n = len(cost)
    c, cp = _f64(cost)
    a, ap = _f64(np.asarray(alpha, dtype=np.float64).reshape(n, n))
    dr, T, lat = C.c_int(), C.c_int(), C.c_double()
    _check(lib.hsd_best_single_draft(n, cp, ap, Tbar, C.byref(dr), C.byref(T), C.byref(lat)))
    return lat.value, dr.value, T.value
