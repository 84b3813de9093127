"""ctypes binding of libssd.so (include/ssd.h).  Argument marshalling only."""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
EXPORTED_SYMBOLS = [
    "ssd_model_workspace_bytes", "ssd_model_create", "ssd_model_destroy", "ssd_kv_pool_bytes",
    "ssd_kv_workspace_bytes", "ssd_kv_create", "ssd_kv_destroy", "ssd_prefill", "ssd_draft_step", "ssd_verify",
    "ssd_kv_rollback", "ssd_kv_follow", "ssd_verify_from_probs", "ssd_warp_probs", "ssd_kv_state",
    "ssd_kv_free_stack", "ssd_profile_begin", "ssd_profile_end", "ssd_kv_last_forward_path", "ssd_trace_barriers", "ssd_strerror", "ssd_last_error",
    "ssd_verify_noalloc", "ssd_kv_clear_error", "ssd_kv_test_hook", "ssd_cycle_create", "ssd_cycle_launch", "ssd_cycle_captures", "ssd_cycle_destroy",
]


class SSDError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libssd error {code}: {msg}")
        self.code = code


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                         "vocab", "n_embed", "dtype", "qkv_bias")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float)]


class SampleConfig(C.Structure):
    _fields_ = [("beta", C.c_float), ("temperature", C.c_float), ("top_k", C.c_int32), ("greedy", C.c_int32),
                ("seed", C.c_uint64)]


def sample_config(beta=0.0, temperature=1.0, top_k=0, greedy=False, seed=0):
    return SampleConfig(float(beta), float(temperature), int(top_k), int(bool(greedy)), int(seed))


def library_path():
    return os.path.join(_HERE, "libssd.so")


_LIB = None


def load_library():
    """Load the in-tree HIP library.  There is no fallback: without it nothing here works."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(path)
    vp, i32p, f32p, sz, i32, u64 = C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_uint64
    sig = {
        "ssd_model_workspace_bytes": (sz, [C.POINTER(ModelConfig), i32]),
        "ssd_model_create": (i32, [C.POINTER(ModelConfig), C.POINTER(vp), i32, i32, vp, sz, vp, C.POINTER(vp)]),
        "ssd_model_destroy": (i32, [vp]),
        "ssd_kv_pool_bytes": (sz, [vp, i32, i32]),
        "ssd_kv_workspace_bytes": (sz, [vp, i32, i32, i32, i32]),
        "ssd_kv_create": (i32, [vp, i32, i32, i32, i32, i32, i32, vp, sz, vp, sz, vp, C.POINTER(vp)]),
        "ssd_kv_destroy": (i32, [vp]),
        "ssd_prefill": (i32, [vp, vp, i32, i32p, i32, vp]),
        "ssd_draft_step": (i32, [vp, vp, i32, C.POINTER(SampleConfig), u64, i32, i32p, i32, f32p, sz, vp]),
        "ssd_verify": (i32, [vp, vp, i32, C.POINTER(C.c_int32), i32p, f32p, i32, C.POINTER(SampleConfig), u64,
                             i32p, i32p, f32p, f32p, vp]),
        "ssd_verify_noalloc": (i32, [vp, vp, i32, i32p, f32p, i32, C.POINTER(SampleConfig), u64, i32p, i32p, vp]),
        "ssd_kv_rollback": (i32, [vp, i32, i32, i32, vp]),
        "ssd_kv_follow": (i32, [vp, i32, i32, i32p, i32p, i32p, vp]),
        "ssd_verify_from_probs": (i32, [f32p, f32p, i32p, f32p, i32, i32, i32, C.c_float, i32p, i32p, i32p, vp]),
        "ssd_warp_probs": (i32, [f32p, i32, i32, C.POINTER(SampleConfig), f32p, vp]),
        "ssd_kv_state": (i32, [vp, i32, vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                               C.POINTER(C.c_int32), C.POINTER(C.c_int32), i32]),
        "ssd_kv_free_stack": (i32, [vp, vp, C.POINTER(C.c_int32), i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
        "ssd_profile_begin": (i32, [i32]),
        "ssd_profile_end": (i32, [C.POINTER(C.c_double), C.POINTER(C.c_int)]),
        "ssd_kv_last_forward_path": (i32, [vp]),
        "ssd_trace_barriers": (i32, [vp, i32, vp, C.POINTER(C.c_uint64), i32, C.POINTER(C.c_int), C.POINTER(C.c_int)]),
        "ssd_kv_clear_error": (i32, [vp, vp]),
        "ssd_kv_test_hook": (i32, [vp, i32, C.c_longlong, vp]),
        "ssd_cycle_create": (i32, [vp, vp, vp, vp, i32, i32, C.POINTER(SampleConfig), C.POINTER(SampleConfig), i32p, f32p,
                                   i32p, i32p, u64, vp, C.POINTER(vp)]),
        "ssd_cycle_launch": (i32, [vp, vp]),
        "ssd_cycle_captures": (i32, [vp]),
        "ssd_cycle_destroy": (i32, [vp]),
        "ssd_strerror": (C.c_char_p, [i32]),
        "ssd_last_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _LIB = lib
    return lib


def _check(rc):
    if rc != 0:
        raise SSDError(rc, load_library().ssd_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev_bytes(n, device):
    """Device buffer of n bytes, 256-byte aligned (torch's caching allocator aligns to 512), filled with 0xFF:
    a kernel that read a workspace entry nobody wrote would see NaN (floats) or -1 (ints), not stale data."""
    t = torch.full((max(int(n), 256),), 0xFF, dtype=torch.uint8, device=device)
    assert t.data_ptr() % 256 == 0
    return t


def upload_weights(shape, weights, device="cuda"):
    """numpy fp32 tensors (canonical layout, see include/ssd.h) -> device tensors of the model's storage type."""
    store = torch.bfloat16 if shape["dtype"] == "bf16" else torch.float32
    out = {}
    for k, v in weights.items():
        if v is None:
            out[k] = None
            continue
        t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32))
        is_matrix = v.ndim == 2
        out[k] = t.to(store).to(device) if is_matrix else t.to(device)
    return out


class Model:
    """ssd_model handle.  `dev_weights`: dict name -> device tensor (see upload_weights)."""

    def __init__(self, shape, dev_weights, max_positions, device="cuda"):
        lib = load_library()
        self.shape = dict(shape)
        self.cfg = ModelConfig(shape["n_layers"], shape["d_model"], shape["n_q_heads"], shape["n_kv_heads"],
                               shape["head_dim"], shape["d_ffn"], shape["vocab"], shape["n_embed"],
                               1 if shape["dtype"] == "bf16" else 0, int(shape["qkv_bias"]),
                               float(shape["rope_base"]), float(shape["rms_eps"]))
        names = ["embed", "final_norm", "head"]
        for l in range(shape["n_layers"]):
            names += [f"l{l}.{n}" for n in ("ln1", "wqkv", "bqkv", "wo", "ln2", "wgate", "wup", "wdown")]
        ptrs = (C.c_void_p * len(names))(*[0 if dev_weights[n] is None else dev_weights[n].data_ptr() for n in names])
        need = lib.ssd_model_workspace_bytes(C.byref(self.cfg), max_positions)
        if need == 0:
            raise SSDError(-1, lib.ssd_last_error().decode())
        self.ws = _dev_bytes(need, device)
        self.max_positions = max_positions
        h = C.c_void_p()
        _check(lib.ssd_model_create(C.byref(self.cfg), ptrs, len(names), max_positions, _ptr(self.ws), need, _stream(),
                                    C.byref(h)))
        torch.cuda.current_stream().synchronize()      # the canonical weights may be dropped from here on
        self.handle = h
        self.device = device

    def __del__(self):
        if getattr(self, "handle", None) and _LIB is not None:
            _LIB.ssd_model_destroy(self.handle)
            self.handle = None


class KVCache:
    """ssd_kv handle with its pool and workspace."""

    def __init__(self, model, max_seqs, max_rows, n_blocks, block_tokens=16, max_blocks_per_seq=None, pending_cap=1):
        lib = load_library()
        self.model = model
        if max_blocks_per_seq is None:
            max_blocks_per_seq = -(-model.max_positions // block_tokens)
        self.max_seqs, self.max_rows, self.n_blocks = max_seqs, max_rows, n_blocks
        self.block_tokens, self.mbps, self.pending_cap = block_tokens, max_blocks_per_seq, pending_cap
        pool_bytes = lib.ssd_kv_pool_bytes(model.handle, n_blocks, block_tokens)
        ws_bytes = lib.ssd_kv_workspace_bytes(model.handle, max_seqs, max_rows, n_blocks, max_blocks_per_seq)
        sh = model.shape
        dt = torch.bfloat16 if sh["dtype"] == "bf16" else torch.float32
        # keys [layer][0][block][kv_head][token][head_dim]; values [layer][1][block][kv_head][head_dim][token]
        self.pool = torch.zeros((sh["n_layers"], 2, n_blocks, sh["n_kv_heads"], block_tokens, sh["head_dim"]),
                                dtype=dt, device=model.device)
        assert self.pool.numel() * self.pool.element_size() == pool_bytes
        self.ws = _dev_bytes(ws_bytes, model.device)
        h = C.c_void_p()
        _check(lib.ssd_kv_create(model.handle, max_seqs, max_rows, n_blocks, block_tokens, max_blocks_per_seq,
                                 pending_cap, _ptr(self.pool), pool_bytes, _ptr(self.ws), ws_bytes, _stream(),
                                 C.byref(h)))
        self.handle = h

    def __del__(self):
        if getattr(self, "handle", None) and _LIB is not None:
            _LIB.ssd_kv_destroy(self.handle)
            self.handle = None

    def state(self, seq):
        lib = load_library()
        ln, npend, own = C.c_int32(), C.c_int32(), C.c_int32()
        pend = (C.c_int32 * 2)()
        table = (C.c_int32 * self.mbps)()
        _check(lib.ssd_kv_state(self.handle, seq, _stream(), C.byref(ln), C.byref(npend), pend, C.byref(own), table,
                                self.mbps))
        return dict(len=ln.value, n_pending=npend.value, pending=list(pend)[:max(npend.value, 0)],
                    n_owned=own.value, table=list(table)[:own.value])

    def last_forward_path(self):
        """1 one launch per operator, 2 persistent kernel with grid barriers, 3 barrier-free persistent kernel,
        4 the same with the attention of a short prefix done without parts."""
        return load_library().ssd_kv_last_forward_path(self.handle)

    def clear_error(self):
        _check(load_library().ssd_kv_clear_error(self.handle, _stream()))

    def test_hook(self, what, value=0):
        _check(load_library().ssd_kv_test_hook(self.handle, int(what), int(value), _stream()))

    def free_stack(self):
        lib = load_library()
        buf = (C.c_int32 * self.n_blocks)()
        n, err = C.c_int32(), C.c_int32()
        _check(lib.ssd_kv_free_stack(self.handle, _stream(), buf, self.n_blocks, C.byref(n), C.byref(err)))
        return list(buf)[:n.value], err.value

    def gather(self, seq, layer, length):
        """Keys and values of positions 0..length-1 as [length, n_kv_heads, head_dim] fp32 host arrays
        (test helper: reads the pool through the block table)."""
        st = self.state(seq)
        bt = self.block_tokens
        nkv, hd = self.model.shape["n_kv_heads"], self.model.shape["head_dim"]
        idx = torch.tensor([st["table"][p // bt] for p in range(length)], device=self.pool.device)
        off = torch.tensor([p % bt for p in range(length)], device=self.pool.device)
        k = self.pool[layer, 0, idx, :, off, :].float().cpu().numpy()
        vt = self.pool[layer, 1].reshape(self.n_blocks, nkv, hd, bt)          # values are stored [dim][token]
        v = vt[idx, :, :, off].float().cpu().numpy()
        return k, v


def ssd_prefill(model, kv, seq, tokens):
    """tokens: int32 device tensor [n]."""
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
    _check(load_library().ssd_prefill(model.handle, kv.handle, seq, _ptr(tokens), tokens.numel(), _stream()))


def ssd_verify(target, kv, n_seqs, draft_tokens, draft_probs, K, cfg, step_ctr, prefix_len=None,
               want_probs=False, want_logits=False, out=None):
    """Returns dict(n_accepted [B] int32, next_token [B] int32, probs [B,K+1,V] | None, logits | None), device tensors."""
    dev = target.device
    V = target.shape["vocab"]
    if out is None:
        out = dict(n_accepted=torch.empty(n_seqs, dtype=torch.int32, device=dev),
                   next_token=torch.empty(n_seqs, dtype=torch.int32, device=dev),
                   probs=torch.empty((n_seqs, K + 1, V), dtype=torch.float32, device=dev) if want_probs else None,
                   logits=torch.empty((n_seqs, K + 1, V), dtype=torch.float32, device=dev) if want_logits else None)
    for name, dt in (("n_accepted", torch.int32), ("next_token", torch.int32), ("probs", torch.float32),
                     ("logits", torch.float32)):
        t = out.get(name)
        assert t is None or (t.dtype == dt and t.is_cuda), f"out[{name!r}] must be a {dt} device tensor"
    pl = None
    if prefix_len is not None:
        pl = (C.c_int32 * n_seqs)(*[int(v) for v in prefix_len])
    if K > 0:
        assert draft_tokens.dtype == torch.int32 and draft_tokens.is_contiguous() and draft_tokens.numel() == n_seqs * K
        assert draft_probs.dtype == torch.float32 and draft_probs.is_contiguous() and draft_probs.numel() == n_seqs * K * V
    _check(load_library().ssd_verify(target.handle, kv.handle, n_seqs, pl, _ptr(draft_tokens), _ptr(draft_probs), K,
                                     C.byref(cfg), int(step_ctr), _ptr(out["n_accepted"]), _ptr(out["next_token"]),
                                     _ptr(out["probs"]), _ptr(out["logits"]), _stream()))
    return out


def ssd_verify_noalloc(target, kv, n_seqs, draft_tokens, draft_probs, K, cfg, step_ctr, n_accepted, next_token):
    """ssd_verify whose staging lives in the library's static device array; outputs go to the given int32 tensors."""
    assert n_accepted.dtype == next_token.dtype == torch.int32 and n_accepted.is_cuda and next_token.is_cuda
    if K > 0:
        assert draft_tokens.dtype == torch.int32 and draft_tokens.is_contiguous() and draft_tokens.numel() == n_seqs * K
        assert draft_probs.dtype == torch.float32 and draft_probs.is_contiguous()
    _check(load_library().ssd_verify_noalloc(target.handle, kv.handle, n_seqs, _ptr(draft_tokens), _ptr(draft_probs), K,
                                             C.byref(cfg), int(step_ctr), _ptr(n_accepted), _ptr(next_token), _stream()))


def ssd_draft_step(draft, kv_d, n_seqs, cfg, step_ctr, draft_idx, token_out, token_stride, probs_out, probs_stride):
    """token_out: int32 device tensor (view) whose element b*token_stride receives sequence b's token;
    probs_out: fp32 device tensor (view) whose row at b*probs_stride receives pd."""
    assert token_out.dtype == torch.int32 and (probs_out is None or probs_out.dtype == torch.float32)
    _check(load_library().ssd_draft_step(draft.handle, kv_d.handle, n_seqs, C.byref(cfg), int(step_ctr), draft_idx,
                                         _ptr(token_out), token_stride, _ptr(probs_out), probs_stride, _stream()))


def ssd_kv_rollback(kv, seq, new_len, pending_token):
    _check(load_library().ssd_kv_rollback(kv.handle, seq, new_len, pending_token, _stream()))


def ssd_kv_follow(kv_d, n_seqs, K, n_accepted, next_token, draft_tokens):
    assert n_accepted.dtype == next_token.dtype == draft_tokens.dtype == torch.int32
    _check(load_library().ssd_kv_follow(kv_d.handle, n_seqs, K, _ptr(n_accepted), _ptr(next_token),
                                        _ptr(draft_tokens), _stream()))


HOOK_TIMEOUT, HOOK_LAUNCH_NUMBER, HOOK_LAUNCH_NUMBER_DEVICE_ONLY = 1, 2, 3


class Cycle:
    """ssd_cycle handle: one SSD cycle captured as a graph; launch() replays it on the current stream."""

    def __init__(self, target, kv, draft, kv_d, n_seqs, K, cfg, dcfg, draft_tokens, draft_probs, n_accepted, next_token,
                 first_step=0):
        for t, dt in ((draft_tokens, torch.int32), (draft_probs, torch.float32), (n_accepted, torch.int32),
                      (next_token, torch.int32)):
            assert t.dtype == dt and t.is_cuda and t.is_contiguous()
        assert draft_tokens.numel() == n_seqs * K and draft_probs.numel() == n_seqs * K * target.shape["vocab"]
        self._keep = (target, kv, draft, kv_d, draft_tokens, draft_probs, n_accepted, next_token)
        h = C.c_void_p()
        _check(load_library().ssd_cycle_create(target.handle, kv.handle, draft.handle, kv_d.handle, n_seqs, K, C.byref(cfg),
                                               C.byref(dcfg), _ptr(draft_tokens), _ptr(draft_probs), _ptr(n_accepted),
                                               _ptr(next_token), int(first_step), _stream(), C.byref(h)))
        self.handle = h

    def launch(self):
        _check(load_library().ssd_cycle_launch(self.handle, _stream()))

    def captures(self):
        return load_library().ssd_cycle_captures(self.handle)

    def __del__(self):
        if getattr(self, "handle", None) and _LIB is not None:
            _LIB.ssd_cycle_destroy(self.handle)
            self.handle = None


def ssd_verify_from_probs(pt, pd, tokens, uniforms, beta):
    """pt [B,K+1,V], pd [B,K,V], tokens [B,K] int32, uniforms [B,K+1]: device tensors.  Returns (n, next, flags)."""
    B, K1, V = pt.shape
    K = K1 - 1
    dev = pt.device
    n = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    flags = torch.empty(B, dtype=torch.int32, device=dev)
    for t, dt in ((pt, torch.float32), (pd, torch.float32), (tokens, torch.int32), (uniforms, torch.float32)):
        assert t is None or (t.is_contiguous() and t.dtype == dt)
    _check(load_library().ssd_verify_from_probs(_ptr(pt), _ptr(pd if K else None), _ptr(tokens if K else None),
                                                _ptr(uniforms), B, K, V, float(beta), _ptr(n), _ptr(nxt), _ptr(flags),
                                                _stream()))
    return n, nxt, flags


def ssd_warp_probs(logits, cfg):
    rows, V = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    probs = torch.empty_like(logits)
    _check(load_library().ssd_warp_probs(_ptr(logits), rows, V, C.byref(cfg), _ptr(probs), _stream()))
    return probs


PROFILE_KINDS = {"qkv": 0, "attention": 1, "o": 2, "gate_up": 3, "down": 4, "head": 5, "persistent": 6}


def ssd_profile_begin(kind):
    _check(load_library().ssd_profile_begin(PROFILE_KINDS[kind]))


def ssd_profile_end():
    """Returns (summed kernel milliseconds, launches)."""
    ms, n = C.c_double(), C.c_int()
    _check(load_library().ssd_profile_end(C.byref(ms), C.byref(n)))
    return ms.value, n.value


def ssd_trace_barriers(kv, enable, read=False):
    """Switch the persistent kernel's barrier trace on/off; with read=True return the last forward's samples as a
    numpy array [workgroups, barriers, 2] of 100 MHz clock ticks (arrival, release)."""
    lib = load_library()
    if not read:
        _check(lib.ssd_trace_barriers(kv.handle, int(enable), _stream(), None, 0, None, None))
        return None
    cap = 256 * 512
    buf = (C.c_uint64 * cap)()
    g, n = C.c_int(), C.c_int()
    _check(lib.ssd_trace_barriers(kv.handle, int(enable), _stream(), buf, cap, C.byref(g), C.byref(n)))
    raw = np.frombuffer(buf, dtype=np.uint64)[:g.value * 512].reshape(g.value, 512).copy()
    kv._trace_raw = raw
    return raw[:, :n.value].reshape(g.value, n.value // 2, 2)
