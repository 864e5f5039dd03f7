"""ctypes binding of libpod.so: the same calls as include/pod.h, argument marshalling only.

Tensors are torch CUDA tensors (PyTorch serves as the device allocator and stream
provider, nothing else); every step of the path runs inside libpod's HIP kernels.
There is no CPU fallback: without the built library, importing the symbols fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

OK, ERR_INVALID_ARG, ERR_CAPACITY, ERR_STATE, ERR_HIP = 0, -1, -2, -3, -4

EXPORTS = [
    "pod_last_error", "pod_cache_bytes", "pod_cache_live_bytes", "pod_cache_init", "pod_cache_destroy",
    "pod_cache_reset", "pod_cache_seq_len", "pod_cache_check", "pod_workspace_bytes", "pod_cache_append",
    "pod_cache_fill", "pod_decode_attention", "pod_prefill_attention", "pod_cache_export_logical",
    "pod_profile_enable", "pod_profile_disable", "pod_profile_read", "pod_profile_read_each", "pod_profile_stream_read", "pod_profile_set_trace", "pod_profile_mfma_feed",
    "pod_score_buffer_bytes", "pod_decode_attention_reuse", "pod_decode_attention_gated", "pod_score_skip_offset",
    "pod_group_layers", "pod_layer_similarity",
    "pod_decode_attention_static", "pod_cache_region_counts", "pod_decode_step", "pod_cache_set_length_source", "pod_cache_launch_info",
    "pod_cache_sync_lengths", "pod_cache_append_many", "pod_prefill_chunk_workspace_bytes", "pod_prefill_chunk_in_place_bytes", "pod_prefill_attention_chunk", "pod_decode_even_plan",
    "pod_decode_plan", "pod_decode_step_reuse",
    "pod_select_workspace_bytes", "pod_select_votes", "pod_select_top", "pod_cache_compact",
]


class PodConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("num_layers", "group_size", "num_q_heads", "num_kv_heads", "head_dim",
                                          "sink", "window", "max_batch", "max_context")] + \
               [("block_lowest", C.POINTER(C.c_int32))]


class PodError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libpod error {code}: {msg}")
        self.code = code


_lib = None


def lib_path() -> str:
    return _build.LIB


def load():
    """Load libpod.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    L = C.CDLL(_build.LIB)
    vp, i32p, szp = C.c_void_p, C.c_void_p, C.POINTER(C.c_size_t)
    cfgp = C.POINTER(PodConfig)
    L.pod_last_error.restype = C.c_char_p
    L.pod_last_error.argtypes = []
    sig = {
        "pod_cache_bytes": [cfgp, szp],
        "pod_cache_live_bytes": [cfgp, C.c_int64, szp, szp],
        "pod_cache_init": [cfgp, vp, C.c_size_t, vp, C.POINTER(vp)],
        "pod_cache_destroy": [vp],
        "pod_cache_reset": [vp, C.c_int, vp],
        "pod_cache_seq_len": [vp, C.c_int, C.c_int, C.POINTER(C.c_int64)],
        "pod_cache_check": [vp, vp],
        "pod_cache_region_counts": [vp, C.c_int, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int)],
        "pod_cache_sync_lengths": [vp, vp],
        "pod_workspace_bytes": [cfgp, szp],
        "pod_decode_plan": [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32)],
        "pod_decode_even_plan": [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)],
        "pod_cache_append": [vp, C.c_int, vp, vp, i32p, C.c_int, vp],
        "pod_cache_fill": [vp, C.c_int, C.c_int, C.c_int, vp, vp, vp],
        "pod_decode_attention": [vp, C.c_int, vp, vp, i32p, C.c_int, C.c_int, C.c_float, vp, C.c_size_t, vp, vp],
        "pod_decode_step": [vp, C.c_int, vp, vp, vp, vp, i32p, C.c_int, C.c_int, C.c_float, vp, C.c_size_t, vp, vp],
        "pod_decode_step_reuse": [vp, C.c_int, vp, vp, vp, i32p, C.c_int, C.c_int, C.c_float, vp, C.c_size_t, vp, C.c_size_t, vp, vp],
        "pod_cache_set_length_source": [vp, C.c_int],
        "pod_cache_launch_info": [vp, C.POINTER(C.c_int32)],
        "pod_decode_attention_static": [vp, C.c_int, vp, vp, i32p, C.c_int, C.c_int, C.c_float, vp, vp],
        "pod_prefill_attention": [vp, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp, C.c_float, vp, C.c_int, vp],
        "pod_cache_export_logical": [vp, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, vp],
        "pod_score_buffer_bytes": [cfgp, szp],
        "pod_decode_attention_gated": [vp, C.c_int, vp, i32p, C.c_int, C.c_int, C.c_float, C.c_float, vp, C.c_size_t,
                                       vp, C.c_size_t, vp, vp],
        "pod_score_skip_offset": [cfgp, szp],
        "pod_group_layers": [vp, C.c_int, C.c_int, C.c_int, C.c_float, vp],
        "pod_layer_similarity": [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp],
        "pod_decode_attention_reuse": [vp, C.c_int, vp, i32p, C.c_int, C.c_int, C.c_float, vp, C.c_size_t, vp,
                                       C.c_size_t, vp, vp],
        "pod_cache_append_many": [vp, C.c_int, vp, vp, i32p, i32p, C.c_int, C.c_int, vp],
        "pod_prefill_chunk_workspace_bytes": [cfgp, C.c_int64, szp],
        "pod_prefill_chunk_in_place_bytes": [cfgp, C.c_int64, C.c_int64, szp],
        "pod_prefill_attention_chunk": [vp, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp, C.c_float, vp, C.c_size_t, vp,
                                        C.c_int, vp],
        "pod_select_workspace_bytes": [cfgp, C.c_int64, C.c_int, C.c_int, szp],
        "pod_select_votes": [vp, C.c_int, C.c_int, C.c_int, vp, C.c_int, vp, C.c_float, vp, vp, C.c_size_t, vp],
        "pod_select_top": [vp, C.c_int, C.c_int, vp, C.c_int, C.c_int, C.c_int, vp, vp, C.c_size_t, vp],
        "pod_cache_compact": [vp, C.c_int, C.c_int, vp, C.c_int, vp, C.c_size_t, vp],
        "pod_profile_enable": [vp, C.c_int],
        "pod_profile_disable": [vp],
        "pod_profile_read": [vp, C.POINTER(C.c_double), C.POINTER(C.c_int)],
        "pod_profile_read_each": [vp, C.POINTER(C.c_float), C.c_int, C.POINTER(C.c_int)],
        "pod_profile_stream_read": [vp, vp, C.c_size_t, vp],
        "pod_profile_set_trace": [vp, vp, C.c_size_t],
        "pod_profile_mfma_feed": [C.c_int, C.c_int, vp, C.c_size_t, vp],
    }
    for name, args in sig.items():
        fn = getattr(L, name)
        fn.restype = C.c_int
        fn.argtypes = args
    _lib = L
    return L


def _check(rc):
    if rc != OK:
        raise PodError(rc, load().pod_last_error().decode())


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def make_config(num_layers, group_size, num_q_heads, num_kv_heads, head_dim, sink, window, max_batch,
                max_context, block_lowest=None) -> PodConfig:
    """block_lowest: optional int [num_layers][num_kv_heads] table of head-wise blocks (see pod.h)."""
    cfg = PodConfig(num_layers, group_size, num_q_heads, num_kv_heads, head_dim, sink, window, max_batch,
                    max_context, None)
    if block_lowest is not None:
        import numpy as np
        tab = np.ascontiguousarray(block_lowest, dtype=np.int32)
        if tab.shape != (num_layers, num_kv_heads):
            raise ValueError(f"block_lowest must have shape ({num_layers}, {num_kv_heads})")
        cfg._block_lowest_keepalive = tab           # the struct only holds the pointer
        cfg.block_lowest = tab.ctypes.data_as(C.POINTER(C.c_int32))
    return cfg


def pod_group_layers(sim, num_kv_heads, threshold=0.5):
    """Greedy grouping of layers into head-wise blocks; sim: float [num_q_heads][L][L]; returns int32 [L][num_kv_heads]."""
    import numpy as np
    sim = np.ascontiguousarray(sim, dtype=np.float32)
    Hq, L, L2 = sim.shape
    assert L == L2
    out = np.zeros((L, num_kv_heads), dtype=np.int32)
    _check(load().pod_group_layers(sim.ctypes.data_as(C.c_void_p), L, Hq, num_kv_heads, float(threshold),
                                   out.ctypes.data_as(C.c_void_p)))
    return out


def pod_layer_similarity(att: torch.Tensor) -> torch.Tensor:
    """att: CUDA float32 [L][H][rows][n] attention rows; returns CUDA float32 sim [H][L][L]."""
    L, H, R, n = att.shape
    sim = torch.empty((H, L, L), dtype=torch.float32, device=att.device)
    _check(load().pod_layer_similarity(_ptr(att, torch.float32), L, H, R, n, _ptr(sim, torch.float32), _stream()))
    return sim


def pod_cache_bytes(cfg: PodConfig) -> int:
    out = C.c_size_t()
    _check(load().pod_cache_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def pod_cache_live_bytes(cfg: PodConfig, n: int):
    a, b = C.c_size_t(), C.c_size_t()
    _check(load().pod_cache_live_bytes(C.byref(cfg), n, C.byref(a), C.byref(b)))
    return a.value, b.value


def pod_score_buffer_bytes(cfg: PodConfig) -> int:
    out = C.c_size_t()
    _check(load().pod_score_buffer_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def pod_prefill_chunk_workspace_bytes(cfg: PodConfig, n_total: int) -> int:
    b = C.c_size_t()
    _check(load().pod_prefill_chunk_workspace_bytes(C.byref(cfg), n_total, C.byref(b)))
    return b.value


def pod_prefill_chunk_in_place_bytes(cfg: PodConfig, n_total: int, T: int) -> int:
    b = C.c_size_t(0)
    _check(load().pod_prefill_chunk_in_place_bytes(C.byref(cfg), n_total, T, C.byref(b)))
    return b.value


def pod_select_workspace_bytes(cfg: PodConfig, n: int, obs: int, keep: int) -> int:
    b = C.c_size_t(0)
    _check(load().pod_select_workspace_bytes(C.byref(cfg), n, obs, keep, C.byref(b)))
    return b.value


POOL_AVG, POOL_MAX = 0, 1


def pod_workspace_bytes(cfg: PodConfig) -> int:
    out = C.c_size_t()
    _check(load().pod_workspace_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def pod_decode_plan(num_cus: int, batch: int, num_kv_heads: int, proximal_rows: int, max_context_len: int) -> dict:
    plan = (C.c_int32 * 6)()
    _check(load().pod_decode_plan(num_cus, batch, num_kv_heads, proximal_rows, max_context_len, plan))
    return dict(waves=plan[0], chunk=plan[1], chunk_prox=plan[2], distant_pieces=plan[3], pieces=plan[4], merge_inside=bool(plan[5]))


def pod_decode_even_plan(num_cus: int, num_kv_heads: int, proximal_rows: int, context_lens, distant_unit_tokens: int = 128) -> dict:
    """Host logic (no GPU): the even split of a decode launch over several rounds' worth of rows."""
    B = len(context_lens)
    lens = (C.c_int32 * B)(*[int(n) for n in context_lens])
    plan = (C.c_int32 * 4)()
    cum = (C.c_int32 * (B + 1))()
    _check(load().pod_decode_even_plan(num_cus, B, num_kv_heads, proximal_rows, distant_unit_tokens, lens, plan, cum))
    return dict(units_per_workgroup=plan[0], workgroups=plan[1], units=plan[2], partials_per_pair=plan[3], unit_cum=list(cum))


def pod_profile_stream_read(buf: torch.Tensor, nbytes: int, cache=None):
    """Enqueue one plain streaming read of the first nbytes of a CUDA tensor on the current stream; with a PodCache
    whose profiling is enabled the launch is recorded like a decode launch."""
    _check(load().pod_profile_stream_read(cache.handle if cache is not None else None, buf.data_ptr(), nbytes, _stream()))


def pod_profile_mfma_feed(variant: int, iters: int, scratch: torch.Tensor):
    """Enqueue the synthetic MFMA loop `variant` (see pod.h) on the current stream; scratch: CUDA tensor of >= 2048 bytes per CU."""
    _check(load().pod_profile_mfma_feed(variant, iters, scratch.data_ptr(), scratch.numel() * scratch.element_size(), _stream()))


GUARD_BYTE = 0xA5
_guarded = []   # (weak reference to the owner, name, whole tensor, guard bytes): every guarded buffer handed out


def guarded_empty(nbytes: int, device, guard_bytes: int, owner=None, name="buffer") -> torch.Tensor:
    """nbytes of device memory, 256-byte aligned; with guard_bytes > 0 the allocation carries that many bytes of a
    fixed pattern in front of and behind the part that is handed out, which guards_intact() checks afterwards."""
    if guard_bytes <= 0:
        return torch.empty(nbytes, dtype=torch.uint8, device=device)
    import weakref
    g = (guard_bytes + 255) // 256 * 256
    whole = torch.full((nbytes + 2 * g,), GUARD_BYTE, dtype=torch.uint8, device=device)
    _guarded.append((weakref.ref(owner) if owner is not None else None, name, whole, g))
    return whole[g:g + nbytes]


def guards_intact(clear: bool = True):
    """Names of the guarded buffers whose guard bands were written to (empty list = all intact)."""
    torch.cuda.synchronize()
    bad = []
    for ref, name, whole, g in _guarded:
        if not (bool((whole[:g] == GUARD_BYTE).all()) and bool((whole[-g:] == GUARD_BYTE).all())):
            bad.append(name)
    if clear:
        _guarded.clear()
    return bad


class PodCache:
    """Owns the torch buffers (cache + decode workspace) and the libpod handle.  guard_bytes > 0: every buffer this
    object hands to the library sits between guard bands (see guards_intact)."""

    def __init__(self, cfg: PodConfig, device="cuda:0", guard_bytes=0):
        self.cfg = cfg
        self.device = torch.device(device)
        self.guard_bytes = guard_bytes
        nbytes = pod_cache_bytes(cfg)
        self.buf = guarded_empty(nbytes, self.device, guard_bytes, self, "cache")
        self.workspace = guarded_empty(pod_workspace_bytes(cfg), self.device, guard_bytes, self, "decode workspace")
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(load().pod_cache_init(C.byref(cfg), self.buf.data_ptr(), nbytes, _stream(), C.byref(h)))
        self.handle = h

    def __del__(self):
        h = getattr(self, "handle", None)
        if h:
            load().pod_cache_destroy(h)
            self.handle = None

    # -- the C ABI, one method per call -------------------------------------------------
    def pod_cache_reset(self, seq_slot=-1):
        _check(load().pod_cache_reset(self.handle, seq_slot, _stream()))

    def pod_cache_seq_len(self, layer, seq_slot) -> int:
        n = C.c_int64()
        _check(load().pod_cache_seq_len(self.handle, layer, seq_slot, C.byref(n)))
        return n.value

    def pod_cache_region_counts(self, layer, seq_slot):
        """((sink, recent, distant) token counts, keeps_distant_keys) of (layer, seq_slot)."""
        cnt, low = (C.c_int64 * 3)(), C.c_int()
        _check(load().pod_cache_region_counts(self.handle, layer, seq_slot, cnt, C.byref(low)))
        return (cnt[0], cnt[1], cnt[2]), bool(low.value)

    def pod_cache_check(self):
        _check(load().pod_cache_check(self.handle, _stream()))

    def pod_cache_sync_lengths(self):
        _check(load().pod_cache_sync_lengths(self.handle, _stream()))

    def pod_cache_append(self, layer, k_new, v_new, positions):
        B = positions.shape[0]
        _check(load().pod_cache_append(self.handle, layer, _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
                                       _ptr(positions, torch.int32), B, _stream()))

    def pod_cache_append_many(self, layer, k_new, v_new, positions, counts=None):
        """k_new, v_new: [B][T][Hkv][d]; positions: device int32 [B]; counts: host sequence of B ints or None."""
        B, T = k_new.shape[0], k_new.shape[1]
        cp = None
        if counts is not None:
            assert len(counts) == B
            cp = (C.c_int32 * B)(*[int(x) for x in counts])
        _check(load().pod_cache_append_many(self.handle, layer, _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
                                            _ptr(positions, torch.int32), cp, T, B, _stream()))

    def pod_cache_fill(self, layer, seq_slot, k, v):
        n = k.shape[0]
        _check(load().pod_cache_fill(self.handle, layer, seq_slot, n, _ptr(k, torch.bfloat16),
                                     _ptr(v, torch.bfloat16), _stream()))

    def pod_decode_attention(self, layer, q, q_shared, context_lens, scale, out=None, max_context_len=0):
        B = q.shape[0]
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_decode_attention(self.handle, layer, _ptr(q, torch.bfloat16), _ptr(q_shared, torch.bfloat16),
                                           _ptr(context_lens, torch.int32), B, max_context_len, scale,
                                           self.workspace.data_ptr(), self.workspace.numel(), _ptr(out, torch.bfloat16),
                                           _stream()))
        return out

    def pod_decode_step(self, layer, k_new, v_new, q, q_shared, positions, scale, out=None, max_context_len=0):
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_decode_step(self.handle, layer, _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
                                      _ptr(q, torch.bfloat16), _ptr(q_shared, torch.bfloat16), _ptr(positions, torch.int32),
                                      q.shape[0], max_context_len, scale, self.workspace.data_ptr(), self.workspace.numel(),
                                      _ptr(out, torch.bfloat16), _stream()))
        return out

    def pod_decode_step_reuse(self, layer, k_new, v_new, q, positions, scale, scores, out=None, max_context_len=0):
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_decode_step_reuse(self.handle, layer, _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
                                            _ptr(q, torch.bfloat16), _ptr(positions, torch.int32), q.shape[0], max_context_len,
                                            scale, self.workspace.data_ptr(), self.workspace.numel(), scores.data_ptr(),
                                            scores.numel() * scores.element_size(), _ptr(out, torch.bfloat16), _stream()))
        return out

    def pod_cache_launch_info(self):
        info = (C.c_int32 * 4)()
        _check(load().pod_cache_launch_info(self.handle, info))
        return dict(xcds=info[0], xcd_local=bool(info[1]), fused_merge=bool(info[2]), device_lengths=bool(info[3]))

    def pod_cache_set_length_source(self, from_device):
        _check(load().pod_cache_set_length_source(self.handle, int(bool(from_device))))

    def pod_decode_attention_static(self, layer, q, q_shared, context_lens, scale, out, max_context_len=0):
        """pod_decode_attention on the library's own fixed scratch array; `out` is the caller's (nothing is allocated)."""
        _check(load().pod_decode_attention_static(self.handle, layer, _ptr(q, torch.bfloat16), _ptr(q_shared, torch.bfloat16),
                                                  _ptr(context_lens, torch.int32), q.shape[0], max_context_len, scale,
                                                  _ptr(out, torch.bfloat16), _stream()))
        return out

    def pod_decode_attention_reuse(self, layer, q, context_lens, scale, scores, out=None, max_context_len=0):
        B = q.shape[0]
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_decode_attention_reuse(self.handle, layer, _ptr(q, torch.bfloat16),
                                                 _ptr(context_lens, torch.int32), B, max_context_len, scale,
                                                 self.workspace.data_ptr(), self.workspace.numel(),
                                                 scores.data_ptr(), scores.numel() * scores.element_size(),
                                                 _ptr(out, torch.bfloat16), _stream()))
        return out

    def pod_decode_attention_gated(self, layer, q, context_lens, scale, tau, scores, out=None, max_context_len=0):
        B = q.shape[0]
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_decode_attention_gated(self.handle, layer, _ptr(q, torch.bfloat16),
                                                 _ptr(context_lens, torch.int32), B, max_context_len, scale, tau,
                                                 self.workspace.data_ptr(), self.workspace.numel(),
                                                 scores.data_ptr(), scores.numel() * scores.element_size(),
                                                 _ptr(out, torch.bfloat16), _stream()))
        return out

    def skip_flags(self, scores):
        """View of the int32 [max_batch][num_q_heads] flags the last gated upper-layer call left in `scores`."""
        off = C.c_size_t()
        _check(load().pod_score_skip_offset(C.byref(self.cfg), C.byref(off)))
        nb = self.cfg.max_batch * self.cfg.num_q_heads * 4
        return scores[off.value:off.value + nb].view(torch.int32).view(self.cfg.max_batch, self.cfg.num_q_heads)

    def new_score_buffer(self):
        """Device buffer for pod_decode_attention_reuse (one block's distant logits)."""
        return guarded_empty(pod_score_buffer_bytes(self.cfg), self.device, self.guard_bytes, self, "score buffer")

    def new_chunk_workspace(self, n_total, in_place_chunk=0):
        """Device buffer for pod_prefill_attention_chunk of a sequence that holds n_total tokens after the chunk;
        in_place_chunk = T > 0: the smaller one that suffices when chunks of at most T tokens are stored by the call."""
        size = (pod_prefill_chunk_in_place_bytes(self.cfg, n_total, in_place_chunk) if in_place_chunk > 0
                else pod_prefill_chunk_workspace_bytes(self.cfg, n_total))
        return guarded_empty(size, self.device, self.guard_bytes, self, "chunk workspace")

    def new_select_workspace(self, n, obs, keep):
        """Device buffer for pod_select_votes, pod_select_top and pod_cache_compact on a prompt of n tokens."""
        return guarded_empty(pod_select_workspace_bytes(self.cfg, n, obs, keep), self.device, self.guard_bytes, self,
                             "selection workspace")

    def pod_select_votes(self, layer, q_obs, k, scale, workspace, votes=None, seq_slot=0, n=None):
        """q_obs: bf16 [obs][Hq][d] (the prompt's last queries at `layer`); k: bf16 [n][Hkv][d], or None with n given:
        keys from the cache of (layer, seq_slot).  Returns float [Hkv][n - S - W] (rows of heads whose block does not
        start at `layer` are not written)."""
        c, obs = self.cfg, q_obs.shape[0]
        n = k.shape[0] if k is not None else n
        if votes is None:
            votes = torch.zeros((c.num_kv_heads, n - c.sink - c.window), dtype=torch.float32, device=self.device)
        _check(load().pod_select_votes(self.handle, layer, seq_slot, n, _ptr(q_obs, torch.bfloat16), obs,
                                       _ptr(k, torch.bfloat16), scale, _ptr(votes, torch.float32), workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream()))
        return votes

    def pod_select_top(self, layer, n, votes, pool_width, pool_kind, keep, sel, workspace):
        """sel: int32 [num_layers][Hkv][keep]; rows (layer, h) of the heads whose block starts at `layer` are written."""
        c = self.cfg
        assert tuple(sel.shape) == (c.num_layers, c.num_kv_heads, keep)
        assert tuple(votes.shape) == (c.num_kv_heads, n - c.sink - c.window)
        _check(load().pod_select_top(self.handle, layer, n, _ptr(votes, torch.float32), pool_width, pool_kind, keep,
                                     _ptr(sel, torch.int32), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream()))
        return sel

    def pod_cache_compact(self, layer, seq_slot, sel, workspace):
        c = self.cfg
        assert sel.dim() == 3 and tuple(sel.shape[:2]) == (c.num_layers, c.num_kv_heads)
        _check(load().pod_cache_compact(self.handle, layer, seq_slot, _ptr(sel, torch.int32), sel.shape[2],
                                        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()))

    def pod_prefill_attention(self, layer, seq_slot, q, k, v, q_shared, k_shared, scale, out=None, write_cache=False):
        n = q.shape[0]
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_prefill_attention(self.handle, layer, seq_slot, n, _ptr(q, torch.bfloat16),
                                            _ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16),
                                            _ptr(q_shared, torch.bfloat16), _ptr(k_shared, torch.bfloat16), scale,
                                            _ptr(out, torch.bfloat16), int(bool(write_cache)), _stream()))
        return out

    def pod_prefill_attention_chunk(self, layer, seq_slot, q, k, v, q_shared, k_shared, scale, workspace, out=None,
                                    write_cache=False):
        """Chunk of T new tokens of a sequence whose earlier tokens are in the cache; workspace: device uint8 tensor of
        pod_prefill_chunk_workspace_bytes(cfg, tokens after the chunk) bytes."""
        T = q.shape[0]
        if out is None:
            out = torch.empty_like(q)
        _check(load().pod_prefill_attention_chunk(self.handle, layer, seq_slot, T, _ptr(q, torch.bfloat16),
                                                  _ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16),
                                                  _ptr(q_shared, torch.bfloat16), _ptr(k_shared, torch.bfloat16), scale,
                                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                  _ptr(out, torch.bfloat16), int(bool(write_cache)), _stream()))
        return out

    def pod_profile_enable(self, max_records):
        _check(load().pod_profile_enable(self.handle, max_records))

    def pod_profile_disable(self):
        _check(load().pod_profile_disable(self.handle))

    def pod_profile_read(self):
        ms, cnt = C.c_double(), C.c_int()
        _check(load().pod_profile_read(self.handle, C.byref(ms), C.byref(cnt)))
        return ms.value, cnt.value

    def pod_profile_set_trace(self, buf):
        """buf: CUDA int64 tensor (8 words per workgroup) or None."""
        _check(load().pod_profile_set_trace(self.handle, buf.data_ptr() if buf is not None else None,
                                            buf.numel() * buf.element_size() if buf is not None else 0))

    def pod_profile_read_each(self, capacity):
        """Kernel time in ms of each recorded launch, in call order."""
        buf, cnt = (C.c_float * capacity)(), C.c_int()
        _check(load().pod_profile_read_each(self.handle, buf, capacity, C.byref(cnt)))
        return [buf[i] for i in range(cnt.value)]

    def pod_cache_export_logical(self, layer, seq_slot):
        """dict of bf16 tensors [tokens][Hkv][d]: sinkK, sinkV, recentK, recentV, distV (+ distK at a lowest layer)."""
        c = self.cfg
        (ns, nr, nd), lowest = self.pod_cache_region_counts(layer, seq_slot)
        mk = lambda t: torch.zeros((t, c.num_kv_heads, c.head_dim), dtype=torch.bfloat16, device=self.device)
        out = dict(sinkK=mk(ns), sinkV=mk(ns), recentK=mk(nr), recentV=mk(nr), distV=mk(nd))
        if lowest:
            out["distK"] = mk(nd)                              # (heads that are not lowest at this layer: zeros)
        _check(load().pod_cache_export_logical(self.handle, layer, seq_slot, _ptr(out["sinkK"]), _ptr(out["sinkV"]),
                                               _ptr(out["recentK"]), _ptr(out["recentV"]),
                                               _ptr(out["distK"]) if lowest else None, _ptr(out["distV"]), _stream()))
        return out
