"""ctypes binding of libpahq.so.  Argument marshalling only: every step of the
method runs inside the library's HIP kernels.  torch is used to allocate the
device workspace and to provide the stream."""
from __future__ import annotations

import ctypes as C
import os
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpahq.so")

ALL_FP32, ALL_FP8, PAHQ = 0, 1, 2
MMA_FP8, MMA_F16_EXACT = 0, 1
METRIC_KL, METRIC_LOGIT_DIFF = 0, 1
W_Q, W_K, W_V, W_O, W_IN, W_GATE, W_OUT, W_U = range(8)


class PahqError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {lib().pahq_strerror(code).decode()} ({code})")


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "n_heads", "d_head", "d_model", "d_mlp", "vocab", "n_ctx",
                                         "norm", "act", "pos")] + \
               [("norm_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("split_qkv", "precision", "max_batch_edges", "mma", "low_bits", "nonattn_bf16", "fp32_residency")]

    @classmethod
    def from_shape(cls, shape, precision=PAHQ, max_batch_edges=32, mma=MMA_F16_EXACT, low_bits=8, nonattn_bf16=False,
                   split_qkv=True, fp32_on_host=False):
        return cls(n_layers=shape.n_layers, n_heads=shape.n_heads, d_head=shape.d_head, d_model=shape.d_model,
                   d_mlp=shape.d_mlp, vocab=shape.vocab, n_ctx=shape.n_ctx, norm=shape.norm, act=shape.act,
                   pos=shape.pos, norm_eps=shape.norm_eps, rope_theta=shape.rope_theta, split_qkv=1 if split_qkv else 0,
                   precision=precision, max_batch_edges=max_batch_edges, mma=mma, low_bits=low_bits,
                   nonattn_bf16=1 if nonattn_bf16 else 0, fp32_residency=1 if fp32_on_host else 0)


_W_NAMES = ("W_E", "W_pos", "W_Q", "W_K", "W_V", "W_O", "b_Q", "b_K", "b_V", "b_O", "ln1_g", "ln1_b", "ln2_g",
            "ln2_b", "W_in", "b_in", "W_gate", "W_out", "b_out", "lnf_g", "lnf_b", "W_U", "b_U")


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_NAMES] + [("on_device", C.c_int32)]


class TraceRec(C.Structure):
    _fields_ = [("receiver", C.c_int32), ("sender", C.c_int32), ("kl_new", C.c_float), ("kl_cur", C.c_float),
                ("removed", C.c_int32)]


class KernelStat(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double), ("bytes", C.c_double)]


KERNEL_CLASSES = ("gather_norm_quant", "edge_patch", "gemm_fp8", "gemm_f32", "attention", "stream_update",
                  "hidden_quant", "logsumexp", "kl", "oproj_fused")

_lib = None


def lib():
    """Loads libpahq.so (built in-tree by paper_2510_23264_amd.build).  There is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: run `python -m paper_2510_23264_amd.build` first")
        L = C.CDLL(_LIB_PATH)
        cfgp, i32p, i64p, u8p, f32p = C.POINTER(Config), C.POINTER(C.c_int32), C.POINTER(C.c_int64), \
            C.POINTER(C.c_uint8), C.POINTER(C.c_float)
        sig = {
            "pahq_n_senders": [cfgp, i32p], "pahq_n_receivers": [cfgp, i32p],
            "pahq_n_upstream": [cfgp, C.c_int32, i32p], "pahq_edge_count": [cfgp, i64p],
            "pahq_edge_id": [cfgp, C.c_int32, C.c_int32, i64p], "pahq_node_of_receiver": [cfgp, C.c_int32, i32p],
            "pahq_workspace_bytes": [cfgp, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)],
            "pahq_init_model": [cfgp, C.POINTER(Weights), C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                C.POINTER(C.c_void_p)],
            "pahq_clean_cache": [C.c_void_p, i32p, i32p],
            "pahq_eval_edges": [C.c_void_p, C.c_int32, i32p, C.c_int32, f32p],
            "pahq_eval_edge_list": [C.c_void_p, C.c_int64, i32p, i32p, f32p],
            "pahq_get_weight_bf16": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_uint16)],
            "pahq_round_rows_bf16": [C.c_void_p, C.c_int32, f32p, C.c_int32, C.c_int32, C.POINTER(C.c_uint16)],
            "pahq_eval_current": [C.c_void_p, C.c_int32, f32p],
            "pahq_acdc_sweep": [C.c_void_p, C.c_float, i32p, C.c_int32, u8p, i64p, C.POINTER(TraceRec), C.c_int64],
            "pahq_acdc_sweep_resume": [C.c_void_p, C.c_float, i32p, C.c_int32, u8p, i64p, C.POINTER(TraceRec), C.c_int64],
            "pahq_eval_edges_sender_policy": [C.c_void_p, C.c_int32, i32p, C.c_int32, f32p, f32p],
            "pahq_acdc_sweep_sender_policy": [C.c_void_p, C.c_float, i32p, C.c_int32, u8p, i64p, C.POINTER(TraceRec), C.c_int64],
            "pahq_acdc_sweep_grid": [C.c_void_p, f32p, C.c_int32, i32p, C.c_int32, u8p, i64p],
            "pahq_eval_circuit": [C.c_void_p, u8p, u8p, f32p, f32p],
            "pahq_set_metric": [C.c_void_p, C.c_int32, i32p, i32p],
            "pahq_set_removed": [C.c_void_p, u8p], "pahq_get_removed": [C.c_void_p, u8p],
            "pahq_set_dead_node_skipping": [C.c_void_p, C.c_int32],
            "pahq_prefetch_heads": [C.c_void_p, C.c_int32, C.c_uint64],
            "pahq_set_attention_form": [C.c_void_p, C.c_int32],
            "pahq_get_transfer_stats": [C.c_void_p, i64p],
            "pahq_get_weight_q": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, u8p, f32p],
            "pahq_quantize_rows": [C.c_void_p, f32p, C.c_int32, C.c_int32, u8p, f32p],
            "pahq_quantize_rows_site": [C.c_void_p, C.c_int32, f32p, C.c_int32, C.c_int32, u8p, f32p],
            "pahq_gemm_codes": [C.c_void_p, u8p, u8p, C.c_int32, C.c_int32, C.c_int32, f32p],
            "pahq_get_logits": [C.c_void_p, C.c_int32, f32p],
            "pahq_get_sender_output": [C.c_void_p, C.c_int32, C.c_int32, f32p],
            "pahq_get_counters": [C.c_void_p, i64p],
            "pahq_set_profiling": [C.c_void_p, C.c_int32],
            "pahq_set_profiling_sample": [C.c_void_p, C.c_uint32, C.c_int32],
            "pahq_get_profile": [C.c_void_p, C.POINTER(KernelStat)],
            "pahq_quantize_rows_noalloc": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
            "pahq_compare_encoders": [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)],
            "pahq_measure_ceilings": [C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double)],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes, fn.restype = args, C.c_int
        L.pahq_strerror.argtypes, L.pahq_strerror.restype = [C.c_int], C.c_char_p
        L.pahq_free.argtypes, L.pahq_free.restype = [C.c_void_p], None
        _lib = L
    return _lib


def _chk(code, what):
    if code != 0:
        raise PahqError(code, what)


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _scalar(fn, ctype, cfg, *args):
    out = ctype()
    _chk(fn(C.byref(cfg), *args, C.byref(out)), fn.__name__)
    return out.value


def n_senders(cfg): return _scalar(lib().pahq_n_senders, C.c_int32, cfg)
def n_receivers(cfg): return _scalar(lib().pahq_n_receivers, C.c_int32, cfg)
def n_upstream(cfg, r): return _scalar(lib().pahq_n_upstream, C.c_int32, cfg, r)
def edge_count(cfg): return _scalar(lib().pahq_edge_count, C.c_int64, cfg)
def edge_id(cfg, s, r): return _scalar(lib().pahq_edge_id, C.c_int64, cfg, s, r)
def node_of_receiver(cfg, r): return _scalar(lib().pahq_node_of_receiver, C.c_int32, cfg, r)
def workspace_bytes(cfg, B, S): return _scalar(lib().pahq_workspace_bytes, C.c_size_t, cfg, B, S)


def measure_ceilings(scratch_mib=1024):
    """(fp16 matrix-core issue-loop TFLOP/s, streaming-copy GB/s read + written) of cuda:0, measured now."""
    import torch
    buf = torch.empty(int(scratch_mib) << 20, dtype=torch.uint8, device="cuda:0")
    tf, gb = C.c_double(), C.c_double()
    _chk(lib().pahq_measure_ceilings(C.c_void_p(torch.cuda.current_stream().cuda_stream), C.c_void_p(buf.data_ptr()),
                                     C.c_size_t(buf.numel()), C.byref(tf), C.byref(gb)), "pahq_measure_ceilings")
    return tf.value, gb.value


def tau_grid(n=21, lo=1e-3, hi=10 ** 0.5):
    """The threshold grid of the paper's ROC scans: n log-spaced values from lo to hi (21 values in [0.001, 3.16])."""
    return np.exp(np.linspace(np.log(lo), np.log(hi), n)).astype(np.float32)


def compare_encoders():
    """(mismatches, example pattern) of the hardware E4M3 conversion against the defining encoder over all finite binary32."""
    import torch
    buf = torch.zeros(4, dtype=torch.int64, device="cuda:0")
    n, ex = C.c_uint64(), C.c_uint32()
    _chk(lib().pahq_compare_encoders(C.c_void_p(torch.cuda.current_stream().cuda_stream), C.c_void_p(buf.data_ptr()),
                                     C.byref(n), C.byref(ex)), "pahq_compare_encoders")
    return n.value, ex.value


def quantize_rows_noalloc(x, codes, scales, stream=None):
    """pahq_quantize_rows_noalloc on device tensors the caller owns: x float32 [rows][cols], codes uint8
    [rows][cols], scales float32 [rows], all contiguous on the current device.  Enqueues; does not wait."""
    import torch
    rows, cols = x.shape
    if not (x.is_cuda and codes.is_cuda and scales.is_cuda and x.is_contiguous() and codes.is_contiguous()
            and scales.is_contiguous() and x.dtype == torch.float32 and codes.dtype == torch.uint8
            and scales.dtype == torch.float32 and codes.shape == x.shape and scales.numel() == rows):
        raise ValueError("x float32 [rows][cols], codes uint8 [rows][cols], scales float32 [rows], contiguous, on the device")
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _chk(lib().pahq_quantize_rows_noalloc(C.c_void_p(st), C.c_void_p(x.data_ptr()), rows, cols,
                                          C.c_void_p(codes.data_ptr()), C.c_void_p(scales.data_ptr())),
         "pahq_quantize_rows_noalloc")


class Model:
    """pahq_init_model + the calls on the handle.  `weights`: dict of float32 numpy arrays
    (layouts as in include/pahq.h)."""

    def __init__(self, shape, weights, B, S, precision=PAHQ, max_batch_edges=32, mma=MMA_F16_EXACT, device="cuda:0",
                 workspace_bytes_override=None, low_bits=8, nonattn_bf16=False, split_qkv=True, fp32_on_host=False):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no HIP device: libpahq has no CPU path")
        self.cfg = Config.from_shape(shape, precision, max_batch_edges, mma, low_bits, nonattn_bf16, split_qkv, fp32_on_host)
        self.B, self.S, self.T = B, S, B * S
        self.n_edges = edge_count(self.cfg)
        nbytes = workspace_bytes(self.cfg, B, S)
        if workspace_bytes_override is not None:       # hand the library a workspace of another size (its size check)
            nbytes = int(workspace_bytes_override)
        self._torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(self.device)
        w = Weights()
        self._keep = []
        for n in _W_NAMES:
            a = weights.get(n)
            if a is None:
                setattr(w, n, None)
            else:
                a = np.ascontiguousarray(a, dtype=np.float32)
                self._keep.append(a)
                setattr(w, n, a.ctypes.data)
        w.on_device = 0
        h = C.c_void_p()
        _chk(lib().pahq_init_model(C.byref(self.cfg), C.byref(w), B, S, C.c_void_p(base), C.c_size_t(nbytes),
                                   C.c_void_p(self.stream.cuda_stream), C.byref(h)), "pahq_init_model")
        self.h = h
        self._keep = []
        self.workspace_bytes = nbytes

    def close(self):
        if getattr(self, "h", None):
            self._torch.cuda.synchronize(self.device)
            lib().pahq_free(self.h)
            self.h = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def clean_cache(self, clean_tok, corrupt_tok):
        a = np.ascontiguousarray(clean_tok, dtype=np.int32)
        b = np.ascontiguousarray(corrupt_tok, dtype=np.int32)
        if a.shape != (self.B, self.S) or b.shape != (self.B, self.S):
            raise ValueError("token arrays must be [B][S]")
        _chk(lib().pahq_clean_cache(self.h, _ptr(a, C.c_int32), _ptr(b, C.c_int32)), "pahq_clean_cache")

    def set_metric(self, metric, answer_ids=None, distractor_ids=None):
        """METRIC_KL or METRIC_LOGIT_DIFF (then with one answer and one distractor token id per sequence);
        call before clean_cache."""
        a = d = None
        if answer_ids is not None:
            a = np.ascontiguousarray(answer_ids, dtype=np.int32)
            d = np.ascontiguousarray(distractor_ids, dtype=np.int32)
            if a.shape != (self.B,) or d.shape != (self.B,):
                raise ValueError("one answer and one distractor id per sequence")
        _chk(lib().pahq_set_metric(self.h, int(metric), None if a is None else _ptr(a, C.c_int32),
                                   None if d is None else _ptr(d, C.c_int32)), "pahq_set_metric")

    def eval_edges(self, receiver, sender_ids):
        s = np.ascontiguousarray(sender_ids, dtype=np.int32)
        out = np.empty(s.size, dtype=np.float32)
        _chk(lib().pahq_eval_edges(self.h, int(receiver), _ptr(s, C.c_int32), s.size, _ptr(out, C.c_float)),
             "pahq_eval_edges")
        return out

    def eval_edge_list(self, receivers, sender_ids):
        r = np.ascontiguousarray(receivers, dtype=np.int32)
        s = np.ascontiguousarray(sender_ids, dtype=np.int32)
        if r.shape != s.shape or r.ndim != 1:
            raise ValueError("receivers and sender_ids: one entry per edge")
        out = np.empty(s.size, dtype=np.float32)
        _chk(lib().pahq_eval_edge_list(self.h, s.size, _ptr(r, C.c_int32), _ptr(s, C.c_int32), _ptr(out, C.c_float)),
             "pahq_eval_edge_list")
        return out

    def eval_current(self, receiver):
        out = C.c_float()
        _chk(lib().pahq_eval_current(self.h, int(receiver), C.byref(out)), "pahq_eval_current")
        return out.value

    def eval_edges_sender_policy(self, receiver, sender_ids):
        """(kl_new, kl_cur) per candidate, each under the precision set of its own sender."""
        s = np.ascontiguousarray(sender_ids, dtype=np.int32)
        new = np.empty(s.size, dtype=np.float32)
        cur = np.empty(s.size, dtype=np.float32)
        _chk(lib().pahq_eval_edges_sender_policy(self.h, int(receiver), _ptr(s, C.c_int32), s.size, _ptr(new, C.c_float),
                                                 _ptr(cur, C.c_float)), "pahq_eval_edges_sender_policy")
        return new, cur

    def acdc_sweep(self, tau, receivers=None, trace_cap=None, sender_policy=False, resume=False):
        """Returns (kept uint8[n_edges], n_evals, trace structured array).  resume: start from the current removed set."""
        kept = np.empty(self.n_edges, dtype=np.uint8)
        n_evals = C.c_int64()
        cap = self.n_edges if trace_cap is None else int(trace_cap)
        trace = (TraceRec * max(cap, 1))()
        if receivers is None:
            rp, rn = None, 0
        else:
            r = np.ascontiguousarray(receivers, dtype=np.int32)
            rp, rn = _ptr(r, C.c_int32), r.size
        fn = lib().pahq_acdc_sweep_sender_policy if sender_policy else \
            (lib().pahq_acdc_sweep_resume if resume else lib().pahq_acdc_sweep)
        _chk(fn(self.h, C.c_float(tau), rp, rn, _ptr(kept, C.c_uint8), C.byref(n_evals), trace, cap), "pahq_acdc_sweep")
        n = min(n_evals.value, cap)
        tr = np.ctypeslib.as_array(trace)[:n].copy() if n else np.zeros(0, dtype=np.dtype(TraceRec))
        return kept, n_evals.value, tr

    def acdc_sweep_grid(self, taus, receivers=None):
        """Sweeps at every threshold of `taus` on one set of caches.  Returns (kept uint8[n_taus][n_edges], n_evals[n_taus])."""
        t = np.ascontiguousarray(taus, dtype=np.float32)
        kept = np.empty((t.size, self.n_edges), dtype=np.uint8)
        n_evals = np.zeros(t.size, dtype=np.int64)
        if receivers is None:
            rp, rn = None, 0
        else:
            r = np.ascontiguousarray(receivers, dtype=np.int32)
            rp, rn = _ptr(r, C.c_int32), r.size
        _chk(lib().pahq_acdc_sweep_grid(self.h, _ptr(t, C.c_float), t.size, rp, rn, _ptr(kept, C.c_uint8),
                                        _ptr(n_evals, C.c_int64)), "pahq_acdc_sweep_grid")
        return kept, n_evals

    def eval_circuit(self, kept=None, f32_heads=None, want_logits=False):
        """KL of the pruned graph under a set of fp32 heads (and its logits when asked for)."""
        kp = hp = lp = None
        if kept is not None:
            k = np.ascontiguousarray(kept, dtype=np.uint8)
            if k.size != self.n_edges:
                raise ValueError("kept must have one byte per edge")
            kp = _ptr(k, C.c_uint8)
        if f32_heads is not None:
            h = np.ascontiguousarray(f32_heads, dtype=np.uint8)
            if h.shape != (self.cfg.n_layers, self.cfg.n_heads):
                raise ValueError("f32_heads must be [n_layers][n_heads]")
            hp = _ptr(h, C.c_uint8)
        logits = np.empty((self.B, self.cfg.vocab), dtype=np.float32) if want_logits else None
        if want_logits:
            lp = _ptr(logits, C.c_float)
        out = C.c_float()
        _chk(lib().pahq_eval_circuit(self.h, kp, hp, C.byref(out), lp), "pahq_eval_circuit")
        return (out.value, logits) if want_logits else out.value

    def set_dead_node_skipping(self, on):
        _chk(lib().pahq_set_dead_node_skipping(self.h, 1 if on else 0), "pahq_set_dead_node_skipping")

    def set_attention_form(self, form):
        _chk(lib().pahq_set_attention_form(self.h, int(form)), "pahq_set_attention_form")

    def prefetch_heads(self, layer, heads):
        """heads: iterable of head indices of `layer` whose fp32 weights will be needed next (host residency)."""
        mask = 0
        for h in heads:
            mask |= 1 << int(h)
        _chk(lib().pahq_prefetch_heads(self.h, int(layer), C.c_uint64(mask)), "pahq_prefetch_heads")

    def transfer_stats(self):
        out = (C.c_int64 * 6)()
        _chk(lib().pahq_get_transfer_stats(self.h, out), "pahq_get_transfer_stats")
        return dict(zip(("head_uses", "demand_transfers", "transfers_ahead", "bytes_moved", "host_bytes", "slot_bytes"), out))

    def set_removed(self, removed):
        r = np.ascontiguousarray(removed, dtype=np.uint8)
        if r.size != self.n_edges:
            raise ValueError("removed must have one byte per edge")
        _chk(lib().pahq_set_removed(self.h, _ptr(r, C.c_uint8)), "pahq_set_removed")

    def get_removed(self):
        r = np.empty(self.n_edges, dtype=np.uint8)
        _chk(lib().pahq_get_removed(self.h, _ptr(r, C.c_uint8)), "pahq_get_removed")
        return r

    def get_weight_q(self, which, layer, head, shape):
        codes = np.empty(shape, dtype=np.uint8)
        scale = C.c_float()
        _chk(lib().pahq_get_weight_q(self.h, which, layer, head, _ptr(codes, C.c_uint8), C.byref(scale)),
             "pahq_get_weight_q")
        return codes, np.float32(scale.value)

    def quantize_rows(self, x, site=None):
        """site None: pahq_quantize_rows; 0 / 1 / 2: pahq_quantize_rows_site (hidden, norm, attention quantiser)."""
        x = np.ascontiguousarray(x, dtype=np.float32)
        rows, cols = x.shape
        codes = np.empty((rows, cols), dtype=np.uint8)
        scales = np.empty(rows, dtype=np.float32)
        if site is None:
            _chk(lib().pahq_quantize_rows(self.h, _ptr(x, C.c_float), rows, cols, _ptr(codes, C.c_uint8),
                                          _ptr(scales, C.c_float)), "pahq_quantize_rows")
        else:
            _chk(lib().pahq_quantize_rows_site(self.h, int(site), _ptr(x, C.c_float), rows, cols, _ptr(codes, C.c_uint8),
                                               _ptr(scales, C.c_float)), "pahq_quantize_rows_site")
        return codes, scales

    def get_weight_bf16(self, which, layer, shape, head=0):
        """bfloat16 patterns uint16 [K][N] of an MLP matrix or the unembedding (nonattn_bf16 models), or of a head's
        projection (low_bits = 16)."""
        out = np.empty(shape, dtype=np.uint16)
        _chk(lib().pahq_get_weight_bf16(self.h, int(which), int(layer), int(head), _ptr(out, C.c_uint16)), "pahq_get_weight_bf16")
        return out

    def round_rows_bf16(self, x, site):
        x = np.ascontiguousarray(x, dtype=np.float32)
        out = np.empty(x.shape, dtype=np.uint16)
        _chk(lib().pahq_round_rows_bf16(self.h, int(site), _ptr(x, C.c_float), x.shape[0], x.shape[1], _ptr(out, C.c_uint16)),
             "pahq_round_rows_bf16")
        return out

    def gemm_codes(self, a, w):
        """a uint8 [m][k], w uint8 [n][k] -> float32 [m][n] = sum_k dec(a) dec(w)."""
        a = np.ascontiguousarray(a, dtype=np.uint8)
        w = np.ascontiguousarray(w, dtype=np.uint8)
        m, k = a.shape
        n, k2 = w.shape
        if k != k2:
            raise ValueError("a and w must share k")
        out = np.empty((m, n), dtype=np.float32)
        _chk(lib().pahq_gemm_codes(self.h, _ptr(a, C.c_uint8), _ptr(w, C.c_uint8), m, n, k, _ptr(out, C.c_float)),
             "pahq_gemm_codes")
        return out

    def get_logits(self, which):
        out = np.empty((self.B, self.cfg.vocab), dtype=np.float32)
        _chk(lib().pahq_get_logits(self.h, which, _ptr(out, C.c_float)), "pahq_get_logits")
        return out

    def get_sender_output(self, which, sender):
        out = np.empty((self.T, self.cfg.d_model), dtype=np.float32)
        _chk(lib().pahq_get_sender_output(self.h, which, sender, _ptr(out, C.c_float)), "pahq_get_sender_output")
        return out

    def set_profiling(self, on):
        _chk(lib().pahq_set_profiling(self.h, 1 if on else 0), "pahq_set_profiling")

    def set_profiling_sample(self, classes=None, every_nth_pass=1):
        """Record only the named kernel classes (None = all), in every n-th pass."""
        mask = 0xFFFFFFFF if classes is None else sum(1 << KERNEL_CLASSES.index(c) for c in classes)
        _chk(lib().pahq_set_profiling_sample(self.h, mask, every_nth_pass), "pahq_set_profiling_sample")

    def get_profile(self):
        """dict: kernel class -> (launches, ms, algorithmic flops, algorithmic bytes)."""
        out = (KernelStat * len(KERNEL_CLASSES))()
        _chk(lib().pahq_get_profile(self.h, out), "pahq_get_profile")
        return {n: dict(launches=o.launches, ms=o.ms, flops=o.flops, bytes=o.bytes)
                for n, o in zip(KERNEL_CLASSES, out)}

    def counters(self):
        out = (C.c_int64 * 3)()
        _chk(lib().pahq_get_counters(self.h, out), "pahq_get_counters")
        return tuple(out)
