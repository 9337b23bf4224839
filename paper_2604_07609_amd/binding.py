"""ctypes binding of include/blink.h. Same names as the C ABI, numpy arrays in and out."""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

FLAG_TRACE, FLAG_EXIT_WHEN_IDLE, FLAG_KEEP_LOGITS, FLAG_NO_GRAPH, FLAG_CHUNKED_PREFILL, FLAG_PREEMPTION, FLAG_PREFIX_CACHE, FLAG_SPECULATIVE = 1, 2, 8, 16, 32, 64, 128, 256
FLAG_HOST_STEP = 512
ERR_INVAL, ERR_TOO_LARGE, ERR_FULL, ERR_DEVICE, ERR_STATE = -1, -2, -3, -4, -5
EVENT_FIRST, EVENT_LAST = 1, 2

EXPORTS = ["blink_init", "blink_submit", "blink_run", "blink_set_exit_when_idle", "blink_wait", "blink_stop", "blink_poll_outputs", "blink_shutdown",
           "blink_get_trace", "blink_get_stats", "blink_debug_read", "blink_time_phase", "blink_get_phase_times", "blink_calibration_copy",
           "blink_calibration_rates", "blink_clock_sync", "blink_sample_rows", "blink_sample_rows_static", "blink_last_error"]


class DBG:
    LOGITS, FREE_STACK, INPUT_IDS, POSITIONS, SLOT_MAPPING, SEQ_BATCH_SLOT, BLOCK_TABLES, SEQ_LENS, CU_SEQLENS, \
        SLOT_STATES, HIDDEN, ROUTING, ATTN_ITEMS = range(1, 14)


class Config(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "dtype")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("weights", C.c_void_p), ("weights_bytes", C.c_uint64),
        ("kv_block_size", C.c_uint32), ("kv_num_blocks", C.c_uint32), ("max_batch", C.c_uint32), ("max_seq_len", C.c_uint32),
        ("max_prefill_tokens", C.c_uint32), ("ring_slots", C.c_uint32), ("eos_token_id", C.c_int32), ("device", C.c_int32),
        ("flags", C.c_uint32), ("trace_capacity", C.c_uint32), ("idle_poll_us", C.c_uint32), ("pump_depth", C.c_uint32),
        ("tune", C.c_uint32), ("n_experts", C.c_uint32), ("n_active", C.c_uint32), ("spec_tokens", C.c_uint32)]


class Sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_k", C.c_uint32), ("top_p", C.c_float), ("seed", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [("iterations", C.c_uint64), ("prefill_iterations", C.c_uint64), ("tokens_out", C.c_uint64),
                ("tokens_prefilled", C.c_uint64), ("next_ticket", C.c_uint64), ("n_running", C.c_uint32),
                ("free_blocks", C.c_uint32), ("committed_blocks", C.c_uint32), ("device_error", C.c_uint32),
                ("running", C.c_uint32), ("windows", C.c_uint32), ("kv_bytes", C.c_uint64), ("weight_bytes", C.c_uint64),
                ("ring_bytes", C.c_uint64), ("prefix_hit_blocks", C.c_uint64), ("prefix_evictions", C.c_uint64),
                ("pinned_blocks", C.c_uint32), ("pad1", C.c_uint32), ("spec_drafted", C.c_uint64), ("spec_accepted", C.c_uint64)]


EVENT_DTYPE = np.dtype([("request_id", "<u8"), ("index", "<u4"), ("token", "<i4"), ("flags", "<u4"), ("iteration", "<u4"),
                        ("device_ns", "<u8")], align=True)
TRACE_DTYPE = np.dtype([("iteration", "<u4"), ("kind", "<u4"), ("tail", "<u8"), ("n_admitted", "<u4"), ("n_seqs", "<u4"),
                        ("n_tokens", "<u4"), ("free_blocks", "<u4"), ("first_admitted", "<u8"), ("t_sched_begin_ns", "<u8"),
                        ("t_sched_end_ns", "<u8"), ("t_forward_end_ns", "<u8"), ("t_publish_end_ns", "<u8"), ("ctx_tokens", "<u8"),
                        ("chain", "<u8"), ("n_resumed", "<u4"), ("n_preempted", "<u4")],
                       align=True)


class BlinkError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"blink error {code}: {msg}")
        self.code = code


def lib_path():
    return os.path.join(HERE, "libblink.so")


_lib = None


def load_library():
    """Loads libblink.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    p = lib_path()
    if not os.path.exists(p):
        raise ImportError(f"{p} is missing: build it with `python -m paper_2604_07609_amd.build`")
    lib = C.CDLL(p)
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    lib.blink_init.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    lib.blink_submit.argtypes = [vp, vp, u32, u32, C.POINTER(Sampling), C.POINTER(u64)]
    lib.blink_run.argtypes = [vp, u64]
    lib.blink_wait.argtypes = [vp]
    lib.blink_set_exit_when_idle.argtypes = [vp, u32]
    lib.blink_stop.argtypes = [vp]
    lib.blink_poll_outputs.argtypes = [vp, vp, u32, C.POINTER(u32)]
    lib.blink_shutdown.argtypes = [vp]
    lib.blink_get_trace.argtypes = [vp, vp, u64, C.POINTER(u64)]
    lib.blink_get_stats.argtypes = [vp, C.POINTER(Stats)]
    lib.blink_debug_read.argtypes = [vp, u32, vp, u64, C.POINTER(u64)]
    lib.blink_time_phase.argtypes = [vp, C.c_int32]
    lib.blink_calibration_copy.argtypes = [vp, u64]
    lib.blink_calibration_rates.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.blink_get_phase_times.argtypes = [vp, vp, u64, C.POINTER(u64)]
    lib.blink_clock_sync.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64)]
    lib.blink_sample_rows.argtypes = [C.c_int32, vp, u32, u32, vp, vp, vp]
    lib.blink_sample_rows_static.argtypes = [C.c_int32, vp, u32, u32, vp, vp, vp]
    lib.blink_last_error.restype = C.c_char_p
    for n in EXPORTS[:-1]:
        getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


def _check(lib, rc):
    if rc != 0:
        raise BlinkError(rc, lib.blink_last_error().decode())


def _sample_rows(fn_name, logits, params, token_index, device=0):
    lib = load_library()
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    n, v = logits.shape
    ps = (Sampling * n)(*[Sampling(float(p["temperature"]), int(p["top_k"]), float(p["top_p"]), int(p["seed"]) & 0xFFFFFFFFFFFFFFFF) for p in params])
    ti = np.ascontiguousarray(token_index, dtype=np.uint32)
    assert ti.size == n
    out = np.zeros(n, dtype=np.int32)
    _check(lib, getattr(lib, fn_name)(int(device), logits.ctypes.data, n, v, C.cast(ps, C.c_void_p), ti.ctypes.data, out.ctypes.data))
    return out


def sample_rows(logits, params, token_index, device=0):
    """blink_sample_rows: logits float32 [n][vocab], params: list of dicts (temperature, top_k, top_p, seed),
    token_index: output index per row. Returns int32 [n]."""
    return _sample_rows("blink_sample_rows", logits, params, token_index, device)


def sample_rows_static(logits, params, token_index, device=0):
    """blink_sample_rows_static: as sample_rows, staging in the library's static device array (no allocation)."""
    return _sample_rows("blink_sample_rows_static", logits, params, token_index, device)


class Engine:
    """One serving engine on one GPU. model/engine: dicts as in synth.configs; blob: uint8 array (synth.pack_blob)."""

    def __init__(self, model, engine, blob, flags=0, device=0, trace_capacity=0, idle_poll_us=0, pump_depth=0, tune=0):
        self.lib = load_library()
        self.model, self.engine = dict(model), dict(engine)
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        cfg = Config()
        for k in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "dtype", "rms_eps", "rope_theta"):
            setattr(cfg, k, model[k])
        for k in ("kv_block_size", "kv_num_blocks", "max_batch", "max_seq_len", "max_prefill_tokens", "ring_slots", "eos_token_id"):
            setattr(cfg, k, engine[k])
        cfg.weights = blob.ctypes.data
        cfg.weights_bytes = blob.nbytes
        if engine.get("chunked_prefill"):
            flags |= FLAG_CHUNKED_PREFILL
        if engine.get("preemption"):
            flags |= FLAG_PREEMPTION
        if engine.get("prefix_cache"):
            flags |= FLAG_PREFIX_CACHE
        if engine.get("speculative"):
            flags |= FLAG_SPECULATIVE
            cfg.spec_tokens = int(engine["speculative"])
        cfg.device, cfg.flags, cfg.trace_capacity, cfg.idle_poll_us = device, flags, trace_capacity, idle_poll_us
        cfg.pump_depth, cfg.tune = pump_depth, tune
        cfg.n_experts, cfg.n_active = model.get("n_experts", 0), model.get("n_active", 0)
        self.h = C.c_void_p()
        _check(self.lib, self.lib.blink_init(C.byref(cfg), C.byref(self.h)))

    def submit(self, prompt, max_new_tokens, temperature=0.0, top_k=0, top_p=1.0, seed=0):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        s = Sampling(float(temperature), int(top_k), float(top_p), int(seed) & 0xFFFFFFFFFFFFFFFF)
        rid = C.c_uint64()
        _check(self.lib, self.lib.blink_submit(self.h, p.ctypes.data, p.size, int(max_new_tokens), C.byref(s), C.byref(rid)))
        return rid.value

    def submit_request(self, r):
        return self.submit(r["prompt"], r["max_new_tokens"], r["temperature"], r["top_k"], r["top_p"], r["seed"])

    def run(self, max_iterations=0):
        _check(self.lib, self.lib.blink_run(self.h, int(max_iterations)))

    def set_exit_when_idle(self, on):
        _check(self.lib, self.lib.blink_set_exit_when_idle(self.h, 1 if on else 0))

    def wait(self):
        _check(self.lib, self.lib.blink_wait(self.h))

    def stop(self):
        _check(self.lib, self.lib.blink_stop(self.h))

    def poll(self, cap=4096):
        buf = np.zeros(cap, dtype=EVENT_DTYPE)
        n = C.c_uint32()
        _check(self.lib, self.lib.blink_poll_outputs(self.h, buf.ctypes.data, cap, C.byref(n)))
        return buf[: n.value]

    def drain(self, cap=4096):
        """Polls until a poll returns nothing. Returns all events as one array."""
        out = []
        while True:
            ev = self.poll(cap)
            if ev.size == 0:
                break
            out.append(ev.copy())
        return np.concatenate(out) if out else np.zeros(0, dtype=EVENT_DTYPE)

    def trace(self, cap=1 << 16):
        buf = np.zeros(cap, dtype=TRACE_DTYPE)
        n = C.c_uint64()
        _check(self.lib, self.lib.blink_get_trace(self.h, buf.ctypes.data, cap, C.byref(n)))
        return buf[: n.value]

    def stats(self):
        s = Stats()
        _check(self.lib, self.lib.blink_get_stats(self.h, C.byref(s)))
        return {k: getattr(s, k) for k, _ in Stats._fields_}

    def debug_read(self, what, dtype, max_bytes=None):
        if max_bytes is None:
            m, e = self.model, self.engine
            max_t = max(e["max_prefill_tokens"], e["max_seq_len"], e["max_batch"])
            max_bytes = 8 + 4 * max(e["max_batch"] * (1 + int(e.get("speculative", 0))) * m["vocab"], e["kv_num_blocks"] + 1, max_t * m["d_model"],
                                    m["n_layers"] * max_t * m.get("n_active", 0),
                                    e["max_batch"] * ((e["max_seq_len"] + 15) // 16), e["ring_slots"])
        buf = np.zeros(max_bytes, dtype=np.uint8)
        n = C.c_uint64()
        _check(self.lib, self.lib.blink_debug_read(self.h, int(what), buf.ctypes.data, buf.nbytes, C.byref(n)))
        return buf[: n.value].view(dtype).copy()

    def time_phase(self, phase):
        _check(self.lib, self.lib.blink_time_phase(self.h, int(phase)))

    def calibration_copy(self, nbytes):
        _check(self.lib, self.lib.blink_calibration_copy(self.h, int(nbytes)))

    def calibration_rates(self):
        """(GB/s of a plain 1 GiB copy kernel, read + written; TFLOP/s of a register-only bf16 MFMA loop; GB/s of a plain
        read of 1 GiB) on this device."""
        c, m, r = C.c_double(), C.c_double(), C.c_double()
        _check(self.lib, self.lib.blink_calibration_rates(self.h, C.byref(c), C.byref(m), C.byref(r)))
        return c.value, m.value, r.value

    def clock_sync(self):
        """(device_ns, host_ns on CLOCK_MONOTONIC, uncertainty_ns): the device clock read no later than host_ns."""
        d, h, u = C.c_uint64(), C.c_uint64(), C.c_uint64()
        _check(self.lib, self.lib.blink_clock_sync(self.h, C.byref(d), C.byref(h), C.byref(u)))
        return d.value, h.value, u.value

    def phase_times_ms(self, cap=1 << 20):
        buf = np.zeros(cap, dtype=np.float32)
        n = C.c_uint64()
        _check(self.lib, self.lib.blink_get_phase_times(self.h, buf.ctypes.data, cap, C.byref(n)))
        return buf[: n.value].copy()

    def shutdown(self):
        if self.h:
            _check(self.lib, self.lib.blink_shutdown(self.h))
            self.h = C.c_void_p()

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.shutdown()
