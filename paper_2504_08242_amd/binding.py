"""ctypes binding of libjupiter_stage.so (see include/jupiter_stage.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch provides device memory and streams.  There is no fallback:
if the library is missing, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libjupiter_stage.so")

JUP_F32, JUP_BF16, JUP_BF16_W4 = 0, 1, 2
JUP_OK, JUP_EINVAL, JUP_EPOS, JUP_ECAP, JUP_EDEVICE, JUP_ENOMEM = 0, -1, -2, -3, -4, -5
STATUS_NAMES = {0: "JUP_OK", -1: "JUP_EINVAL", -2: "JUP_EPOS", -3: "JUP_ECAP", -4: "JUP_EDEVICE", -5: "JUP_ENOMEM"}
KERNEL_IDS = {"rmsnorm": 0, "gemm_qkv": 1, "attention": 2, "gemm_o": 3, "gemm_gate_up": 4, "gemm_down": 5}
WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")


class StageConfig(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32), ("rms_eps", ctypes.c_float),
                ("rope_theta", ctypes.c_float), ("dtype", ctypes.c_int32), ("w4_expanded", ctypes.c_int32)]


MATRIX_NAMES = WEIGHT_NAMES[:7]
SCALE_FIELDS = ("sq", "sk", "sv", "so", "s_gate", "s_up", "s_down")  # jup_layer_weights_t, in MATRIX_NAMES order


class LayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_NAMES + SCALE_FIELDS]


class JupiterError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib():
    """Loads the C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_08242_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        cfgp = ctypes.POINTER(StageConfig)
        sig = {
            "jup_stage_packed_bytes": (sz, [cfgp]),
            "jup_stage_workspace_bytes": (sz, [cfgp, i32]),
            "jup_stage_create": (i32, [cfgp, ctypes.POINTER(LayerWeights), vp, sz, vp, sz, i32, vp,
                                       ctypes.POINTER(vp)]),
            "jup_stage_destroy": (None, [vp]),
            "jup_kv_bytes": (sz, [cfgp, i32]),
            "jup_kv_create": (i32, [cfgp, i32, vp, sz, ctypes.POINTER(vp)]),
            "jup_kv_fork_bytes": (sz, [vp, i32, i32]),
            "jup_kv_fork": (i32, [vp, i32, i32, vp, sz, ctypes.POINTER(vp)]),
            "jup_kv_reset": (i32, [vp]),
            "jup_kv_truncate": (i32, [vp, i32]),
            "jup_kv_keep": (i32, [vp, i32, i32, ctypes.POINTER(i32), vp]),
            "jup_kv_len": (i32, [vp]),
            "jup_kv_capacity": (i32, [vp]),
            "jup_kv_check_append": (i32, [vp, i32, i32]),
            "jup_kv_destroy": (i32, [vp]),
            "jup_stage_prefill_chunk": (i32, [vp, vp, i32, i32, vp, vp, vp]),
            "jup_stage_prefill_chunk_static": (i32, [vp, vp, i32, i32, vp, vp, vp]),
            "jup_stage_prefill_branches": (i32, [vp, i32, vp, i32, ctypes.POINTER(i32), ctypes.POINTER(vp), vp, vp]),
            "jup_stage_prefill_chunks": (i32, [vp, vp, i32, ctypes.POINTER(i32), i32, vp, vp, vp]),
            "jup_stage_enable_overlap": (i32, [vp, i32, vp, sz]),
            "jup_stage_prefill_tree": (i32, [vp, vp, i32, i32, ctypes.POINTER(i32), vp, vp, vp]),
            "jup_stage_trace": (i32, [vp, i32, i32]),
            "jup_stage_trace_read": (i32, [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32),
                                           ctypes.POINTER(i32)]),
            "jup_diag_mfma_loop": (i32, [vp, sz, i32, ctypes.c_int64, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]),
            "jup_diag_clock_probe": (i32, [ctypes.c_int64, vp, vp]),
            "jup_diag_fill_probe": (i32, [vp, sz, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double)]),
            "jup_diag_stream_probe": (i32, [vp, sz, i32, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double)]),
            "jup_diag_lds_read_probe": (i32, [i32, i32, i32, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]),
            "jup_diag_kernel_name": (i32, [vp, i32, i32, i32, ctypes.c_char_p, sz]),
            "jup_last_error": (ctypes.c_char_p, []),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def last_error():
    return lib().jup_last_error().decode()


def _check(status):
    if status != JUP_OK:
        raise JupiterError(status, last_error())


def make_config(cfg, dtype, w4_expanded=False):
    """cfg: dict with n_layers, d_model, n_heads, head_dim, d_ffn, rms_eps, rope_theta; dtype: 'f32' | 'bf16' |
    'w4' (bf16 activations and cache, 4-bit projection matrices); w4_expanded: jup_stage_config_t.w4_expanded."""
    return StageConfig(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"],
                       cfg["rms_eps"], cfg["rope_theta"], {"f32": JUP_F32, "bf16": JUP_BF16, "w4": JUP_BF16_W4}[dtype],
                       int(bool(w4_expanded)))


def _torch_dtype(dtype):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16, "w4": torch.bfloat16}[dtype]


def _stream_handle(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class KvCache:
    """jup_kv_t plus the torch tensor that backs it (layout: [layer][K|V][head][position][head_dim])."""

    def __init__(self, cfg, dtype, max_positions, device="cuda:0", _fork_of=None, _n_shared=0):
        import torch
        self.cfg, self.dtype, self.max_positions = dict(cfg), dtype, int(max_positions)
        self.parent, self.n_shared = _fork_of, int(_n_shared)
        L = lib()
        ccfg = make_config(cfg, dtype)
        es = 4 if dtype == "f32" else 2
        self.handle = ctypes.c_void_p()
        if _fork_of is None:
            nbytes = L.jup_kv_bytes(ctypes.byref(ccfg), self.max_positions)
            if nbytes == 0:
                raise JupiterError(JUP_EINVAL, "jup_kv_bytes rejected the configuration")
            slots = self.max_positions
            self.buf = torch.zeros(nbytes // es, dtype=_torch_dtype(dtype), device=device)
            _check(L.jup_kv_create(ctypes.byref(ccfg), self.max_positions, ctypes.c_void_p(self.buf.data_ptr()),
                                   nbytes, ctypes.byref(self.handle)))
        else:
            nbytes = L.jup_kv_fork_bytes(_fork_of.handle, self.n_shared, self.max_positions)
            if nbytes == 0:
                raise JupiterError(JUP_EINVAL, "jup_kv_fork_bytes rejected the arguments")
            slots = self.max_positions - self.n_shared
            self.buf = torch.zeros(nbytes // es, dtype=_torch_dtype(dtype), device=device)
            _check(L.jup_kv_fork(_fork_of.handle, self.n_shared, self.max_positions,
                                 ctypes.c_void_p(self.buf.data_ptr()), nbytes, ctypes.byref(self.handle)))
        self.slots = slots

    def fork(self, n_shared, max_positions):
        return KvCache(self.cfg, self.dtype, max_positions, device=self.buf.device, _fork_of=self, _n_shared=n_shared)

    def view(self):
        """Own buffer as [n_layers, 2, n_heads, slots, head_dim]."""
        c = self.cfg
        return self.buf.view(c["n_layers"], 2, c["n_heads"], self.slots, c["head_dim"])

    def __len__(self):
        return int(lib().jup_kv_len(self.handle))

    def reset(self):
        _check(lib().jup_kv_reset(self.handle))

    def truncate(self, new_len):
        _check(lib().jup_kv_truncate(self.handle, int(new_len)))

    def keep(self, base_len, slots, stream=None):
        """Keeps the first base_len entries and, behind them, the entries base_len + slots[j] (a tree's accepted path)."""
        k = len(slots)
        arr = (ctypes.c_int32 * max(1, k))(*[int(x) for x in slots])
        _check(lib().jup_kv_keep(self.handle, int(base_len), k, arr, _stream_handle(stream)))

    def check_append(self, n_tokens, pos_offset):
        return int(lib().jup_kv_check_append(self.handle, int(n_tokens), int(pos_offset)))

    def destroy(self):
        if self.handle:
            _check(lib().jup_kv_destroy(self.handle))
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            if self.handle:
                lib().jup_kv_destroy(self.handle)
        except Exception:
            pass


class Stage:
    """jup_stage_t plus the torch tensors that back its packed weights and workspace."""

    def __init__(self, cfg, dtype, layers, max_chunk_tokens, device="cuda:0", stream=None, w4_expanded=False):
        """layers: list of dicts keyed by WEIGHT_NAMES holding torch tensors of the stage dtype on `device`; for
        dtype 'w4' the seven matrices are uint8 code pairs and every matrix ``name`` comes with an fp32
        ``name + '_scale'`` (see upload_w4_layers).  w4_expanded: a 'w4' stage also keeps a bf16 copy of its matrices
        for chunks of more than 64 rows (jup_stage_config_t.w4_expanded)."""
        import torch
        self.cfg, self.dtype, self.max_chunk_tokens = dict(cfg), dtype, int(max_chunk_tokens)
        L = lib()
        ccfg = make_config(cfg, dtype, w4_expanded)
        pb = L.jup_stage_packed_bytes(ctypes.byref(ccfg))
        wb = L.jup_stage_workspace_bytes(ctypes.byref(ccfg), self.max_chunk_tokens)
        if pb == 0 or wb == 0:
            # let the library produce the message
            self.packed = self.workspace = None
        else:
            self.packed = torch.empty(pb, dtype=torch.uint8, device=device)
            self.workspace = torch.empty(wb, dtype=torch.uint8, device=device)
        td = _torch_dtype(dtype)
        arr = (LayerWeights * max(1, len(layers)))()
        for i, w in enumerate(layers):
            for n in WEIGHT_NAMES:
                t = w[n]
                want = torch.uint8 if dtype == "w4" and n in MATRIX_NAMES else td
                assert t.dtype == want and t.is_contiguous() and t.device.type == "cuda", n
                setattr(arr[i], n, t.data_ptr())
            if dtype == "w4":
                for n, field in zip(MATRIX_NAMES, SCALE_FIELDS):
                    t = w[n + "_scale"]
                    assert t.dtype == torch.float32 and t.is_contiguous() and t.device.type == "cuda", n
                    setattr(arr[i], field, t.data_ptr())
        self.handle = ctypes.c_void_p()
        _check(L.jup_stage_create(ctypes.byref(ccfg), arr,
                                  ctypes.c_void_p(self.packed.data_ptr() if self.packed is not None else 0), pb,
                                  ctypes.c_void_p(self.workspace.data_ptr() if self.workspace is not None else 0), wb,
                                  self.max_chunk_tokens, _stream_handle(stream), ctypes.byref(self.handle)))

    def prefill_chunk(self, hidden_in, pos_offset, kv, hidden_out=None, stream=None):
        """hidden_in: [n_tokens, d_model] tensor of the stage dtype on the GPU. Returns hidden_out."""
        import torch
        n = int(hidden_in.shape[0])
        assert hidden_in.is_contiguous() and hidden_in.dtype == _torch_dtype(self.dtype)
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        _check(lib().jup_stage_prefill_chunk(self.handle, ctypes.c_void_p(hidden_in.data_ptr()), n, int(pos_offset),
                                             kv.handle, ctypes.c_void_p(hidden_out.data_ptr()),
                                             _stream_handle(stream)))
        return hidden_out

    def prefill_chunk_static(self, hidden_in, pos_offset, kv, hidden_out, stream=None):
        """jup_stage_prefill_chunk_static: the same call on the library's static scratch.  hidden_out is required (the
        entry point exists for callers that cannot allocate, so the binding does not allocate for them either)."""
        n = int(hidden_in.shape[0])
        assert hidden_in.is_contiguous() and hidden_in.dtype == _torch_dtype(self.dtype)
        _check(lib().jup_stage_prefill_chunk_static(self.handle, ctypes.c_void_p(hidden_in.data_ptr()), n,
                                                    int(pos_offset), kv.handle, ctypes.c_void_p(hidden_out.data_ptr()),
                                                    _stream_handle(stream)))
        return hidden_out

    def enable_overlap(self, n_lanes=2):
        """Scratch buffers (and, inside the library, streams) for n_lanes - 1 further lanes of prefill_chunks."""
        import torch
        ccfg = make_config(self.cfg, self.dtype)
        nbytes = lib().jup_stage_workspace_bytes(ctypes.byref(ccfg), self.max_chunk_tokens) * max(1, int(n_lanes) - 1)
        self.lane_workspaces = torch.empty(nbytes, dtype=torch.uint8, device=self.workspace.device)
        _check(lib().jup_stage_enable_overlap(self.handle, int(n_lanes), ctypes.c_void_p(self.lane_workspaces.data_ptr()),
                                              nbytes))

    def prefill_chunks(self, hidden_in, chunk_tokens, pos_offset, kv, hidden_out=None, stream=None):
        """hidden_in: [sum(chunk_tokens), d_model]; the chunks follow each other from pos_offset. Returns hidden_out."""
        import torch
        k = len(chunk_tokens)
        assert int(hidden_in.shape[0]) == sum(int(c) for c in chunk_tokens)
        assert hidden_in.is_contiguous() and hidden_in.dtype == _torch_dtype(self.dtype)
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        arr = (ctypes.c_int32 * max(1, k))(*[int(c) for c in chunk_tokens])
        _check(lib().jup_stage_prefill_chunks(self.handle, ctypes.c_void_p(hidden_in.data_ptr()), k, arr, int(pos_offset),
                                              kv.handle, ctypes.c_void_p(hidden_out.data_ptr()), _stream_handle(stream)))
        return hidden_out

    def prefill_tree(self, hidden_in, pos_offset, parents, kv, hidden_out=None, stream=None):
        """hidden_in: [n_tokens, d_model] candidate tokens of a token tree; parents[t] is -1 or an earlier row."""
        import torch
        n = int(hidden_in.shape[0])
        assert len(parents) == n
        assert hidden_in.is_contiguous() and hidden_in.dtype == _torch_dtype(self.dtype)
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        par = (ctypes.c_int32 * max(1, n))(*[int(x) for x in parents])
        _check(lib().jup_stage_prefill_tree(self.handle, ctypes.c_void_p(hidden_in.data_ptr()), n, int(pos_offset), par,
                                            kv.handle, ctypes.c_void_p(hidden_out.data_ptr()),
                                            _stream_handle(stream)))
        return hidden_out

    def prefill_branches(self, hidden_in, n_tokens, pos_offsets, kvs, hidden_out=None, stream=None):
        """hidden_in: [len(kvs) * n_tokens, d_model]; rows b*n_tokens.. belong to branch b. Returns hidden_out."""
        import torch
        nb = len(kvs)
        assert len(pos_offsets) == nb and hidden_in.shape[0] == nb * n_tokens
        assert hidden_in.is_contiguous() and hidden_in.dtype == _torch_dtype(self.dtype)
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        pos = (ctypes.c_int32 * nb)(*[int(p) for p in pos_offsets])
        handles = (ctypes.c_void_p * nb)(*[k.handle for k in kvs])
        _check(lib().jup_stage_prefill_branches(self.handle, nb, ctypes.c_void_p(hidden_in.data_ptr()), int(n_tokens),
                                                pos, handles, ctypes.c_void_p(hidden_out.data_ptr()),
                                                _stream_handle(stream)))
        return hidden_out

    def trace(self, kernel_id, max_launches=4096):
        """Times every launch of one kernel class (KERNEL_IDS) with HIP events; -1 stops."""
        _check(lib().jup_stage_trace(self.handle, int(kernel_id), int(max_launches)))

    def trace_read(self):
        """(total milliseconds, launches timed, launches dropped) since the last read."""
        ms, n, dr = ctypes.c_double(), ctypes.c_int32(), ctypes.c_int32()
        _check(lib().jup_stage_trace_read(self.handle, ctypes.byref(ms), ctypes.byref(n), ctypes.byref(dr)))
        return ms.value, n.value, dr.value

    def kernel_name(self, kernel_id, n_tokens, overlapped=False):
        """Name of the projection kernel instantiation a chunk of n_tokens runs as (jup_diag_kernel_name)."""
        buf = ctypes.create_string_buffer(96)
        _check(lib().jup_diag_kernel_name(self.handle, int(kernel_id), int(n_tokens), int(bool(overlapped)), buf, 96))
        return buf.value.decode()

    def destroy(self):
        if self.handle:
            lib().jup_stage_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def upload_layers(layers_np, dtype, device="cuda:0"):
    """numpy fp32 layer dicts (already bf16-representable when dtype == 'bf16') -> torch tensors on the GPU."""
    import torch
    td = _torch_dtype(dtype)
    return [{n: torch.from_numpy(w[n]).to(device=device, dtype=td).contiguous() for n in WEIGHT_NAMES}
            for w in layers_np]


def upload_w4_layers(layers_np, device="cuda:0"):
    """Layer dicts of a 4-bit stage (uint8 code pairs, fp32 ``*_scale`` arrays, fp32 bf16-representable gains)
    -> torch tensors on the GPU."""
    import torch
    out = []
    for w in layers_np:
        d = {}
        for n in MATRIX_NAMES:
            d[n] = torch.from_numpy(w[n]).to(device=device).contiguous()
            d[n + "_scale"] = torch.from_numpy(w[n + "_scale"]).to(device=device, dtype=torch.float32).contiguous()
        for n in ("g_attn", "g_mlp"):
            d[n] = torch.from_numpy(w[n]).to(device=device, dtype=torch.bfloat16).contiguous()
        out.append(d)
    return out


def diag_mfma_loop(operands, n_workgroups, iters_per_wave, ticks, sink, stream=None):
    """Enqueues the bare MFMA loop (jup_diag_mfma_loop); returns its flop count.  operands: bf16 tensor, ticks: int64
    tensor [n_workgroups, 2], sink: float32 tensor [1], all on the GPU."""
    flop = ctypes.c_double()
    _check(lib().jup_diag_mfma_loop(ctypes.c_void_p(operands.data_ptr()), operands.numel() * operands.element_size(),
                                    int(n_workgroups), int(iters_per_wave), ctypes.c_void_p(ticks.data_ptr()),
                                    ctypes.c_void_p(sink.data_ptr()), _stream_handle(stream), ctypes.byref(flop)))
    return flop.value


def diag_fill_probe(buf, n_workgroups, depth, pieces_per_wave, stream=None):
    """Enqueues the operand-fill probe (jup_diag_fill_probe) over the whole of `buf` (uint8 tensor on the GPU);
    returns the bytes the launch moves."""
    nbytes = ctypes.c_double()
    _check(lib().jup_diag_fill_probe(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), int(n_workgroups),
                                     int(depth), int(pieces_per_wave), _stream_handle(stream), ctypes.byref(nbytes)))
    return nbytes.value


def diag_stream_probe(buf, n_workgroups, depth, pieces_per_wave, n_launches=1, stream=None):
    """Enqueues the weight-stream probe (jup_diag_stream_probe) n_launches times back to back: n_workgroups disjoint
    regions of `buf` (uint8 tensor on the GPU) streamed once into LDS per launch, successive launches on successive parts
    of the buffer; returns the bytes all launches move."""
    nbytes = ctypes.c_double()
    _check(lib().jup_diag_stream_probe(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), int(n_workgroups),
                                       int(depth), int(pieces_per_wave), int(n_launches), _stream_handle(stream),
                                       ctypes.byref(nbytes)))
    return nbytes.value


def diag_lds_read_probe(n_workgroups, threads, trips, ticks, sink, stream=None):
    """Enqueues the LDS read probe (jup_diag_lds_read_probe); ticks: int64 tensor [n_workgroups], sink: int32 tensor
    [1], both on the GPU.  Returns the bytes one workgroup reads."""
    nbytes = ctypes.c_double()
    _check(lib().jup_diag_lds_read_probe(int(n_workgroups), int(threads), int(trips), ctypes.c_void_p(ticks.data_ptr()),
                                         ctypes.c_void_p(sink.data_ptr()), _stream_handle(stream), ctypes.byref(nbytes)))
    return nbytes.value


def diag_clock_probe(ref_ticks, ticks, stream=None):
    """Enqueues the one-wave clock probe (jup_diag_clock_probe); ticks: int64 tensor [2] on the GPU."""
    _check(lib().jup_diag_clock_probe(int(ref_ticks), ctypes.c_void_p(ticks.data_ptr()), _stream_handle(stream)))
