"""ctypes binding with the same names as include/blockbatch.h (argument marshalling only)."""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

BB_INIT, BB_PERIODIC = 0, 1
BB_MAX_BRANCHES = 8
_ERR = {-1: "BB_EINVAL", -2: "BB_ESTATE", -3: "BB_ENOMEM", -4: "BB_EHIP"}


class BBError(RuntimeError):
    pass


class bb_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("qkv_bias", C.c_int), ("mask_id", C.c_int)]


class bb_decode_cfg(C.Structure):
    _fields_ = [("tau_dec", C.c_float), ("tau_merge", C.c_float), ("tau_sync", C.c_int),
                ("refresh_interval", C.c_int), ("leader_rule", C.c_int), ("eos_id", C.c_int)]


class bb_limits(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("max_requests", "max_branches", "max_seq_len", "max_gen_len", "max_step_rows")]


class bb_tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("data", C.c_void_p), ("on_device", C.c_int), ("rows", C.c_long), ("cols", C.c_long)]


class BranchState(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("block", "start", "end", "done", "tokens_decoded", "tokens_merged",
                                       "committed_threshold", "committed_fallback", "synced_from")] + [("mean_conf", C.c_float)]


class RequestStats(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_branches", "refresh_due", "all_done", "nfe_init", "nfe_block", "nfe_refresh",
                                             "finished", "winner", "eos_pos")] + \
               [("branch", BranchState * BB_MAX_BRANCHES)]


class bb_step_view(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("counts_dev", "row_branch_dev", "row_pos_dev", "lm_row_dev", "argmax_dev",
                                          "conf_dev", "lse_dev", "logits_dev")] + [("rows_capacity", C.c_int)]


@dataclass
class Limits:
    max_requests: int = 1
    max_branches: int = 4
    max_seq_len: int = 128
    max_gen_len: int = 64
    max_step_rows: int = 64


def lib_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libblockbatch.so")


_LIB = None
EXPORTS = ("bb_workspace_bytes", "bb_create", "bb_destroy", "bb_last_error", "bb_load_weights", "bb_request_open",
           "bb_request_close", "bb_refresh", "bb_denoise_step", "bb_merge_commit", "bb_get_tokens", "bb_get_stats",
           "bb_get_view", "bb_set_state", "bb_get_kv", "bb_set_kv", "bb_read_device", "bb_synchronize", "bb_debug_gemm", "bb_debug_gemm_wide", "bb_debug_wide_format", "bb_profile_enable", "bb_profile_read", "bb_debug_set_gemm_plan", "bb_debug_gemm_plan", "bb_debug_copy16", "bb_generate", "bb_kv_diag_scratch_bytes", "bb_kv_diagnostics", "bb_gemm_static", "bb_debug_mfma_rate", "bb_debug_keep_logits")
KERNEL_CLASSES = ("gemm_skinny", "gemm_wide", "attention", "glue", "policy")


class bb_profile_entry(C.Structure):
    _fields_ = [("klass", C.c_int), ("launches", C.c_int), ("total_ms", C.c_double), ("bytes", C.c_double), ("flops", C.c_double)]


def load_library():
    """Load libblockbatch.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is None:
        p = lib_path()
        if not os.path.exists(p):
            raise BBError(f"{p} is missing: build it with `python -m paper_2605_29233_amd.build` (there is no CPU fallback)")
        lib = C.CDLL(p)
        lib.bb_workspace_bytes.restype = C.c_size_t
        lib.bb_workspace_bytes.argtypes = [C.POINTER(bb_model_cfg), C.POINTER(bb_limits)]
        lib.bb_last_error.restype = C.c_char_p
        lib.bb_last_error.argtypes = [C.c_void_p]
        lib.bb_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(bb_model_cfg), C.POINTER(bb_decode_cfg),
                                  C.POINTER(bb_limits), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.bb_destroy.argtypes = [C.c_void_p]
        lib.bb_load_weights.argtypes = [C.c_void_p, C.POINTER(bb_tensor), C.c_int]
        lib.bb_request_open.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.POINTER(C.c_int)]
        lib.bb_request_close.argtypes = [C.c_void_p, C.c_int]
        lib.bb_refresh.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        lib.bb_denoise_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(bb_step_view)]
        lib.bb_merge_commit.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        lib.bb_get_view.argtypes = [C.c_void_p, C.POINTER(bb_step_view)]
        lib.bb_get_tokens.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        lib.bb_get_stats.argtypes = [C.c_void_p, C.c_int, C.POINTER(RequestStats)]
        lib.bb_set_state.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.bb_get_kv.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        lib.bb_set_kv.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        lib.bb_read_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
        lib.bb_synchronize.argtypes = [C.c_void_p]
        lib.bb_debug_set_gemm_plan.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        lib.bb_profile_enable.argtypes = [C.c_void_p, C.c_int]
        lib.bb_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int)]
        lib.bb_debug_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]
        lib.bb_debug_gemm_wide.argtypes = lib.bb_debug_gemm.argtypes
        lib.bb_debug_wide_format.argtypes = [C.c_void_p, C.c_int]
        lib.bb_debug_gemm_plan.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int)]
        lib.bb_kv_diag_scratch_bytes.restype = C.c_size_t
        lib.bb_kv_diag_scratch_bytes.argtypes = [C.c_void_p, C.c_int]
        lib.bb_kv_diagnostics.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.bb_generate.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        lib.bb_debug_copy16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
        lib.bb_debug_keep_logits.argtypes = [C.c_void_p, C.c_int]
        lib.bb_debug_mfma_rate.argtypes = [C.c_void_p, C.POINTER(C.c_double)]
        lib.bb_gemm_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]
        _LIB = lib
    return _LIB


def gemm_static(A, W_bits, C_out, split_k=0, stream=None):
    """bb_gemm_static on torch CUDA tensors: A fp32 [M][K], W_bits int16 (bf16 bit patterns) [N][K], C_out fp32
    [M][N] (written in place).  Marshalling only; returns the library's return code."""
    import torch
    assert A.is_cuda and W_bits.is_cuda and C_out.is_cuda and A.is_contiguous() and W_bits.is_contiguous() and C_out.is_contiguous()
    assert A.dtype == torch.float32 and C_out.dtype == torch.float32 and W_bits.element_size() == 2
    M, K = A.shape
    N = W_bits.shape[0]
    assert W_bits.shape[1] == K and tuple(C_out.shape) == (M, N)
    st = stream if stream is not None else torch.cuda.current_stream(A.device)
    return load_library().bb_gemm_static(C.c_void_p(A.data_ptr()), C.c_void_p(W_bits.data_ptr()), C.c_void_p(C_out.data_ptr()),
                                         M, N, K, int(split_k), C.c_void_p(st.cuda_stream))


def gemm_plan(M, N, K, wide=True, fusable=False):
    """bb_debug_gemm_plan: dict(split_k, chunks_per_split, nt, mt, workgroups) of the launch the library would take
    (host-only, no device needed)."""
    out = (C.c_int * 5)()
    rc = load_library().bb_debug_gemm_plan(int(M), int(N), int(K), int(wide), int(fusable), out)
    if rc != 0:
        raise ValueError(f"bb_debug_gemm_plan({M}, {N}, {K}) -> {rc}")
    return dict(split_k=out[0], chunks_per_split=out[1], nt=out[2], mt=out[3], workgroups=out[4])


class StepView:
    """Results of the latest forward, copied to the host on demand."""

    def __init__(self, bb, raw):
        self._bb, self._raw = bb, raw
        counts = bb._read(raw.counts_dev, 2, np.int32)
        self.m_q, self.m_lm = int(counts[0]), int(counts[1])

    def rows(self):
        gbr = self._bb._read(self._raw.row_branch_dev, self.m_q, np.int32)
        pos = self._bb._read(self._raw.row_pos_dev, self.m_q, np.int32)
        return gbr, pos

    def lm_rows(self):
        return self._bb._read(self._raw.lm_row_dev, self.m_lm, np.int32)

    def argmax(self):
        return self._bb._read(self._raw.argmax_dev, self.m_lm, np.int32)

    def conf(self):
        return self._bb._read(self._raw.conf_dev, self.m_lm, np.float32)

    def lse(self):
        return self._bb._read(self._raw.lse_dev, self.m_lm, np.float32)

    def logits(self):
        if not self._raw.logits_dev:
            raise BBError("the logits were not stored: call keep_logits() before the forward")
        v = self._bb.model.vocab
        return self._bb._read(self._raw.logits_dev, self.m_lm * v, np.float32).reshape(self.m_lm, v)


class BlockBatch:
    def __init__(self, model, decode, limits: Limits, device="cuda:0", stream=None, poison_workspace=False):
        import torch
        self.lib = load_library()
        self.model, self.decode, self.limits = model, decode, limits
        self._mc = bb_model_cfg(model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads, model.head_dim,
                                model.d_ffn, model.vocab, model.rope_base, model.rms_eps, int(model.qkv_bias), model.mask_id)
        self._dc = bb_decode_cfg(decode.tau_dec, decode.tau_merge, decode.tau_sync, decode.refresh_interval, decode.leader_rule,
                                 getattr(decode, "eos_id", -1))
        self._lim = bb_limits(limits.max_requests, limits.max_branches, limits.max_seq_len, limits.max_gen_len, limits.max_step_rows)
        nbytes = self.lib.bb_workspace_bytes(C.byref(self._mc), C.byref(self._lim))
        if nbytes == 0:
            raise BBError("unsupported model shape or limits")
        self.workspace_bytes = nbytes
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        if poison_workspace:        # tests: the library must not rely on what the caller's memory held (0xFF.. = NaN patterns)
            self._ws.fill_(0xFF)
        base = (self._ws.data_ptr() + 255) // 256 * 256
        self._stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._ctx = C.c_void_p()
        rc = self.lib.bb_create(C.byref(self._ctx), C.byref(self._mc), C.byref(self._dc), C.byref(self._lim),
                                C.c_void_p(base), C.c_size_t(nbytes), C.c_void_p(self._stream.cuda_stream))
        if rc != 0:
            raise BBError(f"bb_create failed: {_ERR.get(rc, rc)}")
        self._req = {}

    # -- helpers ------------------------------------------------------------------------------
    def _chk(self, rc, what):
        if rc != 0:
            msg = self.lib.bb_last_error(self._ctx)
            raise BBError(f"{what}: {_ERR.get(rc, rc)}: {msg.decode() if msg else ''}")

    def _read(self, ptr, n, dtype):
        out = np.empty(n, dtype=dtype)
        if n:
            self._chk(self.lib.bb_read_device(self._ctx, C.c_void_p(ptr), out.ctypes.data_as(C.c_void_p), out.nbytes), "bb_read_device")
        return out

    @staticmethod
    def _ids(ids):
        a = np.ascontiguousarray(ids, dtype=np.int32)
        return a, a.ctypes.data_as(C.c_void_p), len(a)

    def close(self):
        if self._ctx:
            self.lib.bb_destroy(self._ctx)
            self._ctx = C.c_void_p()
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the boundary -------------------------------------------------------------------------
    def load_weights(self, named_tensors):
        """named_tensors: iterable of (name, torch bf16 tensor on the CPU or on this device)."""
        import torch
        for name, t in named_tensors:
            t = t.contiguous()
            assert t.dtype == torch.bfloat16
            rows, cols = (t.shape[0], t.shape[1]) if t.dim() == 2 else (1, t.numel())
            bt = bb_tensor(name.encode(), C.c_void_p(t.data_ptr()), int(t.is_cuda), rows, cols)
            self._chk(self.lib.bb_load_weights(self._ctx, C.byref(bt), 1), f"bb_load_weights({name})")

    def request_open(self, prompt, gen_len, block_sizes):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        b = np.ascontiguousarray(block_sizes, dtype=np.int32)
        rid = C.c_int(-1)
        self._chk(self.lib.bb_request_open(self._ctx, p.ctypes.data_as(C.c_void_p), len(p), int(gen_len),
                                           b.ctypes.data_as(C.c_void_p), len(b), C.byref(rid)), "bb_request_open")
        self._req[rid.value] = (len(b), len(p) + int(gen_len))
        return rid.value

    def request_close(self, rid):
        self._chk(self.lib.bb_request_close(self._ctx, rid), "bb_request_close")
        self._req.pop(rid, None)

    def refresh(self, ids, mode):
        a, p, n = self._ids(ids)
        self._chk(self.lib.bb_refresh(self._ctx, p, n, mode), "bb_refresh")

    def denoise_step(self, ids, want_view=True):
        a, p, n = self._ids(ids)
        raw = bb_step_view()
        self._chk(self.lib.bb_denoise_step(self._ctx, p, n, C.byref(raw) if want_view else None), "bb_denoise_step")
        return StepView(self, raw) if want_view else None

    def latest_view(self):
        """View of the rows of the latest forward (use after refresh(BB_INIT) of one request)."""
        raw = bb_step_view()
        self._chk(self.lib.bb_get_view(self._ctx, C.byref(raw)), "bb_get_view")
        return StepView(self, raw)

    def merge_commit(self, ids, want_stats=True):
        a, p, n = self._ids(ids)
        if not want_stats:
            self._chk(self.lib.bb_merge_commit(self._ctx, p, n, None), "bb_merge_commit")
            return None
        st = (RequestStats * n)()
        self._chk(self.lib.bb_merge_commit(self._ctx, p, n, C.cast(st, C.c_void_p)), "bb_merge_commit")
        return list(st)

    def generate(self, ids, max_block_forwards=1 << 30):
        """Alg. 1 from the initial forward to the end for opened, uninitialised requests; returns their stats."""
        a, p, n = self._ids(ids)
        st = (RequestStats * n)()
        self._chk(self.lib.bb_generate(self._ctx, p, n, int(max_block_forwards), C.cast(st, C.c_void_p)), "bb_generate")
        return list(st)

    def kv_diagnostics(self, rid, want_error=True):
        """(E [N] or None, pairwise squared distances [N][N], D_t) of App. A.2; want_error runs a refresh."""
        import torch
        n, _ = self._req[rid]
        Dp = np.zeros((n, n), dtype=np.float64)
        Da = C.c_double(0.0)
        E, scratch, nbytes = None, None, 0
        if want_error:
            E = np.zeros(n, dtype=np.float64)
            nbytes = self.lib.bb_kv_diag_scratch_bytes(self._ctx, rid)
            scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._chk(self.lib.bb_kv_diagnostics(self._ctx, rid, C.c_void_p(scratch.data_ptr()) if want_error else None, nbytes,
                                             E.ctypes.data_as(C.c_void_p) if want_error else None,
                                             Dp.ctypes.data_as(C.c_void_p), C.byref(Da)), "bb_kv_diagnostics")
        return E, Dp, Da.value

    # -- inspection ---------------------------------------------------------------------------
    def synchronize(self):
        self._chk(self.lib.bb_synchronize(self._ctx), "bb_synchronize")

    def set_gemm_plan(self, kind, nt, split_k):
        self._chk(self.lib.bb_debug_set_gemm_plan(self._ctx, kind, nt, split_k), "bb_debug_set_gemm_plan")

    def profile_enable(self, on=True):
        self._chk(self.lib.bb_profile_enable(self._ctx, int(on)), "bb_profile_enable")

    def profile_read(self):
        """{class name: dict(launches, total_ms, bytes, flops)} of the launches recorded since the last read."""
        arr = (bb_profile_entry * len(KERNEL_CLASSES))()
        n = C.c_int(0)
        self._chk(self.lib.bb_profile_read(self._ctx, C.cast(arr, C.c_void_p), len(KERNEL_CLASSES), C.byref(n)), "bb_profile_read")
        return {KERNEL_CLASSES[e.klass]: dict(launches=e.launches, total_ms=e.total_ms, bytes=e.bytes, flops=e.flops)
                for e in list(arr)[:n.value]}

    def get_tokens(self, rid):
        n, L = self._req[rid]
        X = np.empty((n, L), dtype=np.int32)
        self._chk(self.lib.bb_get_tokens(self._ctx, rid, X.ctypes.data_as(C.c_void_p)), "bb_get_tokens")
        return X

    def get_stats(self, rid):
        st = RequestStats()
        self._chk(self.lib.bb_get_stats(self._ctx, rid, C.byref(st)), "bb_get_stats")
        return st

    def set_state(self, rid, X, branches):
        n, L = self._req[rid]
        X = np.ascontiguousarray(X, dtype=np.int32)
        assert X.shape == (n, L)
        arr = (BranchState * n)()
        for k, b in enumerate(branches):
            arr[k].start, arr[k].end, arr[k].done, arr[k].mean_conf = int(b.start), int(b.end), int(b.done), float(b.mean_conf)
        self._chk(self.lib.bb_set_state(self._ctx, rid, X.ctypes.data_as(C.c_void_p), C.cast(arr, C.c_void_p)), "bb_set_state")

    def get_kv(self, rid, branch, layer):
        n, L = self._req[rid]
        shp = (L, self.model.n_kv_heads, self.model.head_dim)
        K = np.empty(shp, dtype=np.float32)
        V = np.empty(shp, dtype=np.float32)
        self._chk(self.lib.bb_get_kv(self._ctx, rid, branch, layer, K.ctypes.data_as(C.c_void_p), V.ctypes.data_as(C.c_void_p)), "bb_get_kv")
        return K, V

    def set_kv(self, rid, branch, layer, K, V):
        n, L = self._req[rid]
        shp = (L, self.model.n_kv_heads, self.model.head_dim)
        K = np.ascontiguousarray(K, dtype=np.float32)
        V = np.ascontiguousarray(V, dtype=np.float32)
        assert K.shape == shp and V.shape == shp
        self._chk(self.lib.bb_set_kv(self._ctx, rid, branch, layer, K.ctypes.data_as(C.c_void_p), V.ctypes.data_as(C.c_void_p)), "bb_set_kv")

    def debug_copy16(self, src, dst):
        """Plain 16-byte-per-lane device copy of one torch tensor into another (traffic-counter reference)."""
        assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
        nbytes = src.numel() * src.element_size()
        assert nbytes == dst.numel() * dst.element_size()
        self._chk(self.lib.bb_debug_copy16(self._ctx, C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), nbytes), "bb_debug_copy16")

    def keep_logits(self, on=True):
        """Tests: make the forwards store the fp32 logits too (StepView.logits needs it)."""
        self._chk(self.lib.bb_debug_keep_logits(self._ctx, int(on)), "bb_debug_keep_logits")

    def debug_mfma_rate(self):
        """TFLOP/s of a pure 32x32x16 bf16 MFMA loop on this chip (measured peak)."""
        out = C.c_double(0.0)
        self._chk(self.lib.bb_debug_mfma_rate(self._ctx, C.byref(out)), "bb_debug_mfma_rate")
        return out.value

    def debug_gemm(self, A, W_bits, split_k=0, wide=False):
        A = np.ascontiguousarray(A, dtype=np.float32)
        W = np.ascontiguousarray(W_bits, dtype=np.uint16)
        M, K = A.shape
        N = W.shape[0]
        out = np.empty((M, N), dtype=np.float32)
        fn = self.lib.bb_debug_gemm_wide if wide else self.lib.bb_debug_gemm
        self._chk(fn(self._ctx, A.ctypes.data_as(C.c_void_p), W.ctypes.data_as(C.c_void_p),
                     out.ctypes.data_as(C.c_void_p), M, N, K, split_k), "bb_debug_gemm_wide" if wide else "bb_debug_gemm")
        return out

    def wide_format(self, on=True):
        self._chk(self.lib.bb_debug_wide_format(self._ctx, int(on)), "bb_debug_wide_format")
