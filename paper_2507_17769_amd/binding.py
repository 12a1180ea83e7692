"""ctypes binding over libpolystep.so: argument marshalling only.

Function names and argument order mirror include/polystep.h.  Device buffers are passed as
integer addresses (e.g. torch.Tensor.data_ptr()); every step of the path runs inside the
library's HIP kernels.  Importing this module fails loudly if the library has not been built
(`python -m paper_2507_17769_amd.build`): there is no fallback path.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- first, on purpose: the process must hold ONE HIP runtime.  torch ships its own
#                libamdhip64; loading it before libpolystep makes the dynamic loader resolve our
#                dependency to that same copy, so device pointers and streams are shared.

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpolystep.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_17769_amd.build`")
lib = C.CDLL(LIB_PATH)

PS_OK, PS_EINVAL, PS_ERANGE, PS_ENOMEM, PS_ESTATE, PS_EDEVICE = range(6)
STATUS_NAMES = ["PS_OK", "PS_EINVAL", "PS_ERANGE", "PS_ENOMEM", "PS_ESTATE", "PS_EDEVICE"]
PS_PAGE_SIZE = 16
PS_N_STAGES = 8
PS_GRID_MAX_DRAWS = 8
PS_STATIC_SCRATCH_BYTES = 64 << 20
PS_FLAG_HOST_ONLY = 1
STAGE_NAMES = ["rmsnorm_attn", "gemm_qkv", "rope_append", "attention", "gemm_o", "rmsnorm_ffn", "gemm_gate_up", "gemm_down"]


class ps_model_desc(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("n_layers", C.c_int32), ("page_size", C.c_int32), ("max_position", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("flags", C.c_uint32)]


class ps_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "g_attn", "g_ffn")]


class ps_head_weights(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("g_final", C.c_void_p), ("w_out", C.c_void_p), ("vocab", C.c_int32)]


class ps_sim_config(C.Structure):
    _fields_ = [("mode", C.c_int32), ("n_servers", C.c_int32), ("n_tiers", C.c_int32), ("tpot_ms", C.POINTER(C.c_double)),
                ("avg_decode_len", C.c_int32), ("kv_capacity", C.c_double), ("check_period_ms", C.c_int32), ("max_steps", C.c_int64),
                ("prefill_budget", C.c_int32)]


class ps_sim_request(C.Structure):
    _fields_ = [("arrival_ms", C.c_double), ("prompt_len", C.c_int32), ("output_len", C.c_int32), ("ttft_ms", C.c_double),
                ("tier", C.c_int32)]


class ps_sim_summary(C.Structure):
    _fields_ = [("end_ms", C.c_int64), ("cost_ms", C.c_double), ("scale_ups", C.c_int64), ("scale_downs", C.c_int64),
                ("promotions", C.c_int64), ("dropped", C.c_int64), ("iterations", C.c_int64), ("admission_tests", C.c_int64)]


class ps_running_req(C.Structure):
    _fields_ = [("kv_len", C.c_int32), ("generated", C.c_int32)]


class ps_seq(C.Structure):
    _fields_ = [("req_id", C.c_int64), ("n_new", C.c_int32), ("kv_len", C.c_int32),
                ("page_table", C.POINTER(C.c_int32)), ("n_pages", C.c_int32)]


class ps_clock_reading(C.Structure):
    _fields_ = [("shader_mhz", C.c_double), ("ticks_per_mfma", C.c_double), ("mfma_tflops", C.c_double), ("elapsed_ms", C.c_double),
                ("compute_units", C.c_int32), ("wavefronts_per_simd", C.c_int32)]


class ps_step_stats(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("total_kv", C.c_int64), ("n_attn_items", C.c_int32),
                ("n_attn_partials", C.c_int32), ("ms_total", C.c_float), ("ms_stage", C.c_float * PS_N_STAGES)]


class ps_taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("xn", "q", "attn", "x1", "xn2", "act", "x_in", "x_out")]


class ps_grid_cell_spec(C.Structure):
    _fields_ = [("chunk", C.c_int32), ("n_decode", C.c_int32), ("n_draws", C.c_int32),
                ("chunk_prefix", C.POINTER(C.c_int32)), ("decode_kv", C.POINTER(C.c_int32))]


class ps_grid_opts(C.Structure):
    _fields_ = [("warmup", C.c_int32), ("iters", C.c_int32)]


class ps_grid_cell(C.Structure):
    _fields_ = [("chunk", C.c_int32), ("n_decode", C.c_int32), ("n_tokens", C.c_int32), ("n_draws", C.c_int32),
                ("total_kv", C.c_int64), ("median_ms", C.c_float), ("stage_ms", C.c_float * PS_N_STAGES),
                ("draw_ms", C.c_float * PS_GRID_MAX_DRAWS), ("draw_total_kv", C.c_int64 * PS_GRID_MAX_DRAWS)]


_P = C.c_void_p
_I32P = C.POINTER(C.c_int32)
_SIGS = {
    "ps_create": (C.c_int, [C.POINTER(ps_model_desc), _P, C.POINTER(_P)]),
    "ps_sync": (C.c_int, [_P]),
    "ps_destroy": (None, [_P]),
    "ps_last_error": (C.c_char_p, [_P]),
    "ps_set_option": (C.c_int, [_P, C.c_char_p, C.c_int64]),
    "ps_init_layer": (C.c_int, [_P, C.c_int32, C.POINTER(ps_layer_weights)]),
    "ps_kv_alloc": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_uint64]),
    "ps_kv_reserve": (C.c_int, [_P, C.c_int64, C.c_int32, _I32P, C.c_int32, _I32P]),
    "ps_kv_release": (C.c_int, [_P, C.c_int64]),
    "ps_kv_free_pages": (C.c_int32, [_P]),
    "ps_kv_write": (C.c_int, [_P, C.c_int32, C.POINTER(ps_seq), C.c_int32, C.c_int32, _P, _P]),
    "ps_kv_read": (C.c_int, [_P, C.c_int32, C.POINTER(ps_seq), C.c_int32, C.c_int32, _P, _P]),
    "ps_step": (C.c_int, [_P, C.POINTER(ps_seq), C.c_int32, _P, _P, C.POINTER(ps_step_stats)]),
    "ps_step_static": (C.c_int, [_P, C.POINTER(ps_seq), C.c_int32, _P, _P]),
    "ps_init_head": (C.c_int, [_P, C.POINTER(ps_head_weights)]),
    "ps_step_tokens": (C.c_int, [_P, C.POINTER(ps_seq), C.c_int32, _I32P, _P, _P, _P, C.POINTER(ps_step_stats), C.POINTER(C.c_float)]),
    "ps_step_indices": (C.c_int, [_P, C.POINTER(ps_seq), C.c_int32, _I32P, _I32P, _I32P]),
    "ps_plan_attention": (C.c_int, [_P, C.POINTER(ps_seq), C.c_int32, _I32P, C.c_int32, _I32P]),
    "ps_set_taps": (C.c_int, [_P, C.c_int32, C.POINTER(ps_taps)]),
    "ps_attention_times": (C.c_int, [_P, C.POINTER(C.c_float), C.c_int32, _I32P]),
    "ps_gemm_times": (C.c_int, [_P, C.POINTER(C.c_float), C.c_int32, _I32P]),
    "ps_clock_under_load": (C.c_int, [_P, C.c_int32, C.c_int32, C.POINTER(ps_clock_reading)]),
    "ps_hbm_read_rate": (C.c_int, [_P, C.c_int64, C.c_int32, C.POINTER(C.c_double)]),
    "ps_profile_grid": (C.c_int, [_P, C.POINTER(ps_grid_cell_spec), C.c_int32, C.POINTER(ps_grid_opts), _P, _P,
                                  C.POINTER(ps_grid_cell)]),
}
_D = C.c_double
_SCHED_SIGS = {
    "ps_profile_create": (C.c_int, [_I32P, C.c_int32, C.POINTER(C.c_int64), C.c_int32, C.POINTER(C.c_float), C.POINTER(_P)]),
    "ps_profile_destroy": (None, [_P]),
    "ps_profile_lookup": (_D, [_P, _D, _D]),
    "ps_max_future_kv": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int64), _I32P]),
    "ps_predict_admit": (C.c_int, [_P, _P, C.c_int32, C.c_int32, C.c_int32, _D, _D, _I32P, C.POINTER(_D), C.POINTER(C.c_int64)]),
    "ps_chunk_plan": (C.c_int, [_I32P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _I32P, C.c_int32, _I32P, _I32P]),
    "ps_predict_chunked_prefill": (C.c_int, [_P, _P, C.c_int32, C.c_int32, C.c_int32, _D, _D, _D, _I32P, _I32P, _I32P, C.POINTER(_D)]),
    "ps_batch_limit_pd": (C.c_int32, [_P, _D, _D, _D, _D, C.c_int32]),
    "ps_batch_limit_co": (C.c_int32, [_P, _D, _D, _D, _D, _D, C.c_int32]),
    "ps_cost_pd": (_D, [_P, _D, _D, _D, _D]),
    "ps_cost_co": (_D, [_P, _D, _D, _D]),
    "ps_optimal_cost_pd": (_D, [_P, _D, _D, _D, _D, _D, C.c_int32]),
    "ps_optimal_cost_co": (_D, [_P, _D, _D, _D, _D, _D, C.c_int32]),
    "ps_sim_run": (C.c_int, [_P, _P, _P, C.c_int32, _P, _P, _P, _P, _P, _P]),
}
EXPORTS = sorted(_SIGS)
SCHED_EXPORTS = sorted(_SCHED_SIGS)
for _name, (_res, _args) in _SCHED_SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args


class PolystepError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {message}")
        self.status = status


def _as_i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class SeqArray:
    """A C array of ps_seq plus the int32 page tables it points into (kept alive here)."""

    def __init__(self, seqs):
        """seqs: iterable of (req_id, n_new, kv_len, pages) or objects with those attributes."""
        rows = [s if isinstance(s, tuple) else (s.req_id, s.n_new, s.kv_len, s.pages) for s in seqs]
        self.n = len(rows)
        self._tables = [_as_i32(r[3]) for r in rows]
        self.array = (ps_seq * max(self.n, 1))()
        for i, (r, t) in enumerate(zip(rows, self._tables)):
            self.array[i] = ps_seq(int(r[0]), int(r[1]), int(r[2]), t.ctypes.data_as(_I32P), len(t))
        self.n_tokens = sum(int(r[1]) for r in rows)


class Context:
    """Owns one ps_ctx.  Methods are the C entry points with the ps_ prefix dropped."""

    def __init__(self, hidden, n_q_heads, n_kv_heads, head_dim, ffn, n_layers=1, max_position=8192, rms_eps=1e-5,
                 rope_base=10000.0, host_only=False, stream=0):
        self.desc = ps_model_desc(hidden, n_q_heads, n_kv_heads, head_dim, ffn, n_layers, PS_PAGE_SIZE, max_position,
                                  rms_eps, rope_base, PS_FLAG_HOST_ONLY if host_only else 0)
        h = _P()
        st = lib.ps_create(C.byref(self.desc), _P(stream), C.byref(h))
        if st != PS_OK:
            raise PolystepError(st, lib.ps_last_error(None).decode())
        self.handle = h

    def _check(self, st):
        if st != PS_OK:
            raise PolystepError(st, lib.ps_last_error(self.handle).decode())

    def destroy(self):
        if getattr(self, "handle", None):
            lib.ps_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.destroy()

    def sync(self):
        self._check(lib.ps_sync(self.handle))

    def set_option(self, name, value):
        self._check(lib.ps_set_option(self.handle, name.encode(), int(value)))

    def init_layer(self, layer, **ptrs):
        w = ps_layer_weights(*[int(ptrs[n]) for n, _ in ps_layer_weights._fields_])
        self._check(lib.ps_init_layer(self.handle, layer, C.byref(w)))

    def kv_alloc(self, n_pages, n_kv_layers=1, perm_seed=0):
        self._check(lib.ps_kv_alloc(self.handle, n_pages, n_kv_layers, perm_seed))

    def kv_reserve(self, req_id, kv_len):
        cap = max(1, (kv_len + PS_PAGE_SIZE - 1) // PS_PAGE_SIZE + 4096)
        buf = np.zeros(cap, dtype=np.int32)
        n = C.c_int32(0)
        self._check(lib.ps_kv_reserve(self.handle, req_id, kv_len, buf.ctypes.data_as(_I32P), cap, C.byref(n)))
        return buf[:n.value].copy()

    def kv_release(self, req_id):
        self._check(lib.ps_kv_release(self.handle, req_id))

    def kv_free_pages(self):
        return lib.ps_kv_free_pages(self.handle)

    def kv_write(self, layer, pages, pos0, n, k_ptr, v_ptr):
        sa = SeqArray([(0, 1, 1, pages)])
        self._check(lib.ps_kv_write(self.handle, layer, sa.array, pos0, n, _P(k_ptr), _P(v_ptr)))

    def kv_read(self, layer, pages, pos0, n, k_ptr, v_ptr):
        sa = SeqArray([(0, 1, 1, pages)])
        self._check(lib.ps_kv_read(self.handle, layer, sa.array, pos0, n, _P(k_ptr), _P(v_ptr)))

    def step(self, seqs, x_in_ptr, x_out_ptr, want_stats=False):
        sa = seqs if isinstance(seqs, SeqArray) else SeqArray(seqs)
        stats = ps_step_stats() if want_stats else None
        self._check(lib.ps_step(self.handle, sa.array, sa.n, _P(x_in_ptr), _P(x_out_ptr),
                                C.byref(stats) if want_stats else None))
        return stats

    def step_static(self, seqs, x_in_ptr, x_out_ptr):
        sa = seqs if isinstance(seqs, SeqArray) else SeqArray(seqs)
        self._check(lib.ps_step_static(self.handle, sa.array, sa.n, _P(x_in_ptr), _P(x_out_ptr)))

    def init_head(self, embedding, g_final, w_out, vocab):
        w = ps_head_weights(int(embedding), int(g_final), int(w_out), int(vocab))
        self._check(lib.ps_init_head(self.handle, C.byref(w)))

    def step_tokens(self, seqs, token_ids, next_tokens_ptr=None, logits_ptr=None, hidden_ptr=None, want_stats=False, want_parts=False):
        """token_ids: host int32 array [T].  Returns (stats or None, [ms embedding, ms layers, ms head] or None)."""
        sa = seqs if isinstance(seqs, SeqArray) else SeqArray(seqs)
        ids = np.ascontiguousarray(token_ids, dtype=np.int32)
        if ids.shape != (sa.n_tokens,):
            raise ValueError("token_ids must hold one id per new token")
        stats = ps_step_stats() if want_stats else None
        parts = (C.c_float * 3)() if want_parts else None
        self._check(lib.ps_step_tokens(self.handle, sa.array, sa.n, ids.ctypes.data_as(_I32P), _P(next_tokens_ptr), _P(logits_ptr),
                                       _P(hidden_ptr), C.byref(stats) if want_stats else None, parts))
        return stats, ([parts[i] for i in range(3)] if want_parts else None)

    def step_indices(self, seqs):
        sa = seqs if isinstance(seqs, SeqArray) else SeqArray(seqs)
        cu = np.zeros(sa.n + 1, dtype=np.int32)
        pos = np.zeros(max(sa.n_tokens, 1), dtype=np.int32)
        slots = np.zeros(max(sa.n_tokens, 1), dtype=np.int32)
        self._check(lib.ps_step_indices(self.handle, sa.array, sa.n, cu.ctypes.data_as(_I32P),
                                        pos.ctypes.data_as(_I32P), slots.ctypes.data_as(_I32P)))
        return cu, pos[:sa.n_tokens], slots[:sa.n_tokens]

    def plan_attention(self, seqs):
        sa = seqs if isinstance(seqs, SeqArray) else SeqArray(seqs)
        n = C.c_int32(0)
        self._check(lib.ps_plan_attention(self.handle, sa.array, sa.n, None, 0, C.byref(n)))
        items = np.zeros((max(n.value, 1), 8), dtype=np.int32)
        self._check(lib.ps_plan_attention(self.handle, sa.array, sa.n, items.ctypes.data_as(_I32P), n.value, C.byref(n)))
        return items[:n.value]

    def attention_times(self, cap=2048):
        buf = (C.c_float * cap)()
        n = C.c_int32(0)
        self._check(lib.ps_attention_times(self.handle, buf, cap, C.byref(n)))
        return [buf[i] for i in range(n.value)]

    def gemm_times(self, cap=1024):
        """-> list of [qkv, o, gate_up, down] ms, one per layer of every timed step"""
        buf = (C.c_float * (4 * cap))()
        n = C.c_int32(0)
        self._check(lib.ps_gemm_times(self.handle, buf, cap, C.byref(n)))
        return [[buf[4 * i + k] for k in range(4)] for i in range(n.value)]

    def clock_under_load(self, mfma_per_wavefront=400000, wavefronts_per_simd=2):
        r = ps_clock_reading()
        self._check(lib.ps_clock_under_load(self.handle, mfma_per_wavefront, wavefronts_per_simd, C.byref(r)))
        return {n: getattr(r, n) for n, _ in ps_clock_reading._fields_}

    def hbm_read_rate(self, n_bytes=2 << 30, passes=4):
        g = C.c_double(0.0)
        self._check(lib.ps_hbm_read_rate(self.handle, n_bytes, passes, C.byref(g)))
        return g.value

    def set_taps(self, layer, **ptrs):
        if not ptrs:
            self._check(lib.ps_set_taps(self.handle, layer, None))
            return
        t = ps_taps(*[int(ptrs.get(n, 0)) or None for n, _ in ps_taps._fields_])
        self._check(lib.ps_set_taps(self.handle, layer, C.byref(t)))

    def profile_grid(self, cells, x_in_ptr, x_out_ptr, warmup=2, iters=5):
        """cells: list of (chunk, n_decode, chunk_prefix[n_draws], decode_kv[n_draws][n_decode])."""
        n = len(cells)
        specs = (ps_grid_cell_spec * max(n, 1))()
        keep = []
        for i, (chunk, n_dec, prefixes, dkv) in enumerate(cells):
            pf = _as_i32(prefixes)
            dk = _as_i32(dkv).reshape(len(pf), n_dec) if n_dec else np.zeros((len(pf), 0), dtype=np.int32)
            keep += [pf, dk]
            specs[i] = ps_grid_cell_spec(chunk, n_dec, len(pf), pf.ctypes.data_as(_I32P), dk.ctypes.data_as(_I32P))
        out = (ps_grid_cell * max(n, 1))()
        opts = ps_grid_opts(warmup, iters)
        self._check(lib.ps_profile_grid(self.handle, specs, n, C.byref(opts), _P(x_in_ptr), _P(x_out_ptr), out))
        return [out[i] for i in range(n)]


# ---- polysched: host-side consumers of the latency profile (include/polysched.h) -------------
def _running(reqs):
    arr = (ps_running_req * max(1, len(reqs)))()
    for i, (kv, g) in enumerate(reqs):
        arr[i].kv_len, arr[i].generated = int(kv), int(g)
    return arr


def _sched_check(status, what):
    if status != PS_OK:
        raise PolystepError(status, what)


class Profile:
    """(batch size, KV cache size) -> time table and the decisions taken with it."""

    def __init__(self, batch_sizes, kv_sizes, ms):
        b = np.ascontiguousarray(batch_sizes, dtype=np.int32)
        k = np.ascontiguousarray(kv_sizes, dtype=np.int64)
        t = np.ascontiguousarray(ms, dtype=np.float32).reshape(len(b), len(k))
        h = _P()
        _sched_check(lib.ps_profile_create(b.ctypes.data_as(_I32P), len(b), k.ctypes.data_as(C.POINTER(C.c_int64)), len(k),
                                           t.ctypes.data_as(C.POINTER(C.c_float)), C.byref(h)), "ps_profile_create")
        self.handle = h

    def close(self):
        if self.handle:
            lib.ps_profile_destroy(self.handle)
            self.handle = None

    def lookup(self, batch, kv):
        return lib.ps_profile_lookup(self.handle, float(batch), float(kv))

    def predict_admit(self, running, new_prompt, avg_decode, tpot_ms, wait_ms=0.0):
        admit, t, kv = C.c_int32(0), _D(0), C.c_int64(0)
        _sched_check(lib.ps_predict_admit(self.handle, _running(running), len(running), int(new_prompt), int(avg_decode), float(tpot_ms),
                                          float(wait_ms), C.byref(admit), C.byref(t), C.byref(kv)), "ps_predict_admit")
        return bool(admit.value), t.value, kv.value

    def predict_chunked_prefill(self, running, prompt, avg_decode, tpot_ms, ttft_ms, wait_ms=0.0):
        admit, chunk, n, t = C.c_int32(0), C.c_int32(0), C.c_int32(0), _D(0)
        _sched_check(lib.ps_predict_chunked_prefill(self.handle, _running(running), len(running), int(prompt), int(avg_decode), float(tpot_ms),
                                                    float(ttft_ms), float(wait_ms), C.byref(admit), C.byref(chunk), C.byref(n), C.byref(t)),
                     "ps_predict_chunked_prefill")
        return bool(admit.value), chunk.value, n.value, t.value

    def cost_pd(self, p, d, b_pf, b_dc):
        return lib.ps_cost_pd(self.handle, float(p), float(d), float(b_pf), float(b_dc))

    def cost_co(self, p, d, b):
        return lib.ps_cost_co(self.handle, float(p), float(d), float(b))

    def optimal_cost_pd(self, p, d, tpot_ms, capacity, b_pf, b_max=4096):
        return lib.ps_optimal_cost_pd(self.handle, float(p), float(d), float(tpot_ms), float(capacity), float(b_pf), int(b_max))

    def optimal_cost_co(self, p, d, tpot_ms, ttft_ms, capacity, b_max=4096):
        return lib.ps_optimal_cost_co(self.handle, float(p), float(d), float(tpot_ms), float(ttft_ms), float(capacity), int(b_max))

    def simulate(self, arrival, prompt, output, ttft, tier, tpots, n_servers, avg_decode, kv_capacity, check_period=1000,
                 max_steps=10 ** 9, disaggregated=False, prefill_budget=0):
        """ps_sim_run on parallel per-request sequences; returns a dict with the per-request arrays and the summary."""
        n = len(arrival)
        reqs = (ps_sim_request * max(1, n))()
        for i in range(n):
            reqs[i] = ps_sim_request(float(arrival[i]), int(prompt[i]), int(output[i]), float(ttft[i]), int(tier[i]))
        tp = (C.c_double * len(tpots))(*[float(t) for t in tpots])
        cfg = ps_sim_config(1 if disaggregated else 0, int(n_servers), len(tpots), tp, int(avg_decode), float(kv_capacity),
                            int(check_period), int(max_steps), int(prefill_budget))
        att = np.zeros(n, dtype=np.uint8)
        first, fin = np.zeros(n), np.zeros(n)
        srv, dsrv = np.zeros(n, dtype=np.int32), np.zeros(n, dtype=np.int32)
        summ = ps_sim_summary()
        _sched_check(lib.ps_sim_run(self.handle, C.byref(cfg), reqs, n, att.ctypes.data, first.ctypes.data, fin.ctypes.data,
                                    srv.ctypes.data, dsrv.ctypes.data, C.byref(summ)), "ps_sim_run")
        out = {name: getattr(summ, name) for name, _ in ps_sim_summary._fields_}
        out.update(attained=att, first_token_ms=first, finish_ms=fin, server=srv, decode_server=dsrv)
        return out

    def batch_limit_pd(self, p, d, tpot_ms, capacity, b_max=4096):
        return lib.ps_batch_limit_pd(self.handle, float(p), float(d), float(tpot_ms), float(capacity), int(b_max))

    def batch_limit_co(self, p, d, tpot_ms, ttft_ms, capacity, b_max=4096):
        return lib.ps_batch_limit_co(self.handle, float(p), float(d), float(tpot_ms), float(ttft_ms), float(capacity), int(b_max))


def max_future_kv(running, new_prompt, avg_decode):
    kv, n = C.c_int64(0), C.c_int32(0)
    _sched_check(lib.ps_max_future_kv(_running(running), len(running), -1 if new_prompt is None else int(new_prompt), int(avg_decode),
                                      C.byref(kv), C.byref(n)), "ps_max_future_kv")
    return kv.value, n.value


def chunk_plan(prompts, budget, dynamic, first_iteration_used=0):
    """-> list of iterations, each a list of (request, tokens)"""
    pr = np.ascontiguousarray(prompts, dtype=np.int32)
    n_chunks, n_iter = C.c_int32(0), C.c_int32(0)
    _sched_check(lib.ps_chunk_plan(pr.ctypes.data_as(_I32P), len(pr), int(budget), int(bool(dynamic)), int(first_iteration_used), None, 0,
                                   C.byref(n_chunks), C.byref(n_iter)), "ps_chunk_plan")
    buf = np.zeros((max(1, n_chunks.value), 3), dtype=np.int32)
    _sched_check(lib.ps_chunk_plan(pr.ctypes.data_as(_I32P), len(pr), int(budget), int(bool(dynamic)), int(first_iteration_used),
                                   buf.ctypes.data_as(_I32P), n_chunks.value, C.byref(n_chunks), C.byref(n_iter)), "ps_chunk_plan")
    out = [[] for _ in range(n_iter.value)]
    for it, r, t in buf[:n_chunks.value].tolist():
        out[it].append((r, t))
    return out
