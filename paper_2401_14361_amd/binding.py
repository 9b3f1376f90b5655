"""ctypes binding of libmoei.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/moei.h) and
takes torch CUDA tensors for device buffers; outputs are allocated with torch
(device memory plumbing) and filled by the library's kernels.  A missing library
is an error: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

__all__ = [
    "MoeiError", "ModelDesc", "lib", "lib_path", "Eamc", "Cache",
    "moe_route_topk", "eam_update", "eamc_match", "eamc_match_topm", "expert_priority", "expert_ffn_gemv",
    "expert_ffn_gemv_static",
    "moe_decode_layer", "moe_prefill_layer", "expert_ffn_grouped", "WDTYPE_FP32", "WDTYPE_BF16", "EXPORTS", "expert_pack", "profile_enable", "profile_disable", "profile_read", "profile_samples",
]

WDTYPE_FP32, WDTYPE_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))

EXPORTS = [
    "moei_last_error", "moei_version",
    "moei_eamc_create", "moei_eamc_load", "moei_eamc_insert", "moei_eamc_export", "moei_eamc_save", "moei_eamc_restore", "moei_eamc_size", "moei_eamc_destroy",
    "moe_route_topk", "eam_update", "eamc_match", "eamc_match_topm", "expert_priority",
    "moei_cache_create", "moei_cache_destroy", "moei_expert_pack", "moei_cache_reset", "moei_cache_slot_ptr", "moei_cache_slot_table",
    "moei_cache_get_slots", "moei_cache_retrieve", "expert_ffn_gemv", "expert_ffn_gemv_static", "expert_ffn_grouped", "moei_cache_error_flags",
    "moe_decode_layer", "moei_cache_last_step", "moei_cache_last_heads", "moei_cache_join", "moei_cache_sync",
    "moei_cache_set_match_count", "moei_cache_last_matches",
    "moe_prefill_layer", "moei_cache_set_policy", "moei_cache_prefetch", "moei_cache_set_prefetch", "moei_cache_last_prefetch",
    "moei_profile_enable", "moei_profile_disable", "moei_profile_kernels", "moei_profile_kernel_name",
    "moei_profile_read", "moei_profile_samples",
]


class MoeiError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moei error {code}: {msg}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [("L", C.c_int32), ("E", C.c_int32), ("k", C.c_int32), ("n_shared", C.c_int32),
                ("H", C.c_int32), ("I", C.c_int32), ("wdtype", C.c_int32), ("renorm_topk", C.c_int32),
                ("eps", C.c_float)]

    @classmethod
    def from_config(cls, cfg, eps: float = 2.0 ** -20) -> "ModelDesc":
        return cls(cfg.L, cfg.E, cfg.k, cfg.n_shared, cfg.H, cfg.I,
                   WDTYPE_FP32 if cfg.wdtype == "fp32" else WDTYPE_BF16, int(cfg.renorm), eps)


def lib_path() -> str:
    return os.path.join(_HERE, "libmoei.so")


_lib = None


def lib() -> C.CDLL:
    """The loaded HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        p = lib_path()
        if not os.path.exists(p):
            raise FileNotFoundError(f"{p} is missing: run `python -m paper_2401_14361_amd.build` "
                                    "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = C.CDLL(p)
        L.moei_last_error.restype = C.c_char_p
        L.moei_version.restype = C.c_char_p
        for name in EXPORTS[2:]:
            getattr(L, name).restype = C.c_int
        L.moei_profile_kernel_name.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise MoeiError(rc, lib().moei_last_error().decode())
    return rc


def _p(t) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous(), "tensors handed to the library must be contiguous"
        return C.c_void_p(t.data_ptr())
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return C.c_void_p(t.ctypes.data)
    return C.c_void_p(int(t))


def _stream(stream=None) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype, dtype)
    return t


# ---------------------------------------------------------------------------- objects
class Eamc:
    """Owner of a moei_eamc handle."""

    def __init__(self, desc: ModelDesc, n_cap: int, cell_bytes: int = 4):
        self.desc, self.n_cap, self.cell_bytes = desc, n_cap, cell_bytes
        self.h = C.c_void_p(0)
        _check(lib().moei_eamc_create(C.byref(desc), n_cap, cell_bytes, C.byref(self.h)))

    def load(self, traces: np.ndarray) -> None:
        traces = np.ascontiguousarray(traces, dtype=np.int32)
        N = traces.shape[0]
        assert traces.shape[1:] == (self.desc.L, self.desc.E) or N == 0
        _check(lib().moei_eamc_load(self.h, _p(traces), N))

    def insert(self, eam: np.ndarray, victim: int = -1) -> None:
        eam = np.ascontiguousarray(eam, dtype=np.int32)
        assert eam.shape == (self.desc.L, self.desc.E)
        _check(lib().moei_eamc_insert(self.h, _p(eam), victim))

    def export(self) -> np.ndarray:
        out = np.zeros((self.size, self.desc.L, self.desc.E), dtype=np.int32)
        _check(lib().moei_eamc_export(self.h, _p(out), out.shape[0]))
        return out

    def save(self, path: str) -> None:
        """Checkpoint file of the collection (failure recovery)."""
        _check(lib().moei_eamc_save(self.h, os.fsencode(path)))

    def restore(self, path: str) -> None:
        _check(lib().moei_eamc_restore(self.h, os.fsencode(path)))

    @property
    def size(self) -> int:
        return _check(lib().moei_eamc_size(self.h))

    def close(self) -> None:
        if self.h:
            lib().moei_eamc_destroy(self.h)
            self.h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Cache:
    """Owner of a moei_cache handle (slot pool, slot table, per-layer scratch)."""

    def __init__(self, desc: ModelDesc, n_slots: int, h_experts: torch.Tensor | np.ndarray | None = None,
                 h_shared: torch.Tensor | np.ndarray | None = None):
        self.desc, self.n_slots = desc, n_slots
        self._keep = (h_experts, h_shared)      # the library reads the host copy on every miss
        n_host = 0 if h_experts is None else int(h_experts.shape[0])
        self.h = C.c_void_p(0)
        _check(lib().moei_cache_create(C.byref(desc), n_slots, _p(h_experts), n_host, _p(h_shared), C.byref(self.h)))
        self.slot_elems = 3 * desc.H * desc.I

    def reset(self, n_resident: int) -> None:
        _check(lib().moei_cache_reset(self.h, n_resident))

    def slot_ptr(self, slot: int) -> int:
        out = C.c_void_p(0)
        _check(lib().moei_cache_slot_ptr(self.h, slot, C.byref(out)))
        return out.value

    def slot_tensor(self, slot: int) -> torch.Tensor:
        """A torch view of one slot's weights on the device (no copy, no ownership)."""
        fp32 = self.desc.wdtype == WDTYPE_FP32

        class _View:
            pass

        v = _View()
        v.__cuda_array_interface__ = {"shape": (self.slot_elems,), "typestr": "<f4" if fp32 else "<i2",
                                      "data": (self.slot_ptr(slot), False), "version": 2}
        t = torch.as_tensor(v, device="cuda")
        return t if fp32 else t.view(torch.bfloat16)

    def slot_table(self) -> int:
        out = C.c_void_p(0)
        _check(lib().moei_cache_slot_table(self.h, C.byref(out)))
        return out.value

    def get_slots(self) -> np.ndarray:
        out = np.empty(self.desc.L * self.desc.E, dtype=np.int32)
        _check(lib().moei_cache_get_slots(self.h, _p(out)))
        return out

    def retrieve(self, layer: int, idx, ev_order, stream=None):
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        ev = np.ascontiguousarray(ev_order, dtype=np.int32)
        n = idx.shape[0]
        slots = np.empty(n, dtype=np.int32)
        victims = np.empty(n, dtype=np.int32)
        n_miss = C.c_int32(0)
        _check(lib().moei_cache_retrieve(self.h, layer, _p(idx), n, _p(ev), ev.shape[0], _p(slots), _p(victims),
                                         C.byref(n_miss), _stream(stream)))
        return slots, victims, n_miss.value

    def error_flags(self, stream=None) -> int:
        f = C.c_int32(0)
        _check(lib().moei_cache_error_flags(self.h, C.byref(f), _stream(stream)))
        return f.value

    def join(self, stream=None) -> None:
        _check(lib().moei_cache_join(self.h, _stream(stream)))

    def sync(self) -> None:
        _check(lib().moei_cache_sync(self.h))

    def last_heads(self, stream=None):
        """(pf_head, ev_head): the leading entries of the two orders as the last layer step selected them."""
        pf = np.empty(64, dtype=np.int32)
        ev = np.empty(128, dtype=np.int32)
        n_pf, n_ev = C.c_int32(0), C.c_int32(0)
        _check(lib().moei_cache_last_heads(self.h, _p(pf), pf.size, C.byref(n_pf), _p(ev), ev.size, C.byref(n_ev),
                                           _stream(stream)))
        return pf[:n_pf.value].copy(), ev[:n_ev.value].copy()

    def last_step(self, stream=None) -> dict:
        LE, k = self.desc.L * self.desc.E, self.desc.k
        w = np.empty(k, dtype=np.float32)
        sim = C.c_float(0)
        P = np.empty(LE, dtype=np.float32)
        V = np.empty(LE, dtype=np.float32)
        pf = np.empty(LE, dtype=np.int32)
        ev = np.empty(LE, dtype=np.int32)
        n_pf, n_ev = C.c_int32(0), C.c_int32(0)
        _check(lib().moei_cache_last_step(self.h, _p(w), C.byref(sim), _p(P), _p(V), _p(pf), C.byref(n_pf), _p(ev),
                                          C.byref(n_ev), _stream(stream)))
        return dict(w=w, sim=sim.value, P=P.reshape(self.desc.L, self.desc.E), V=V.reshape(self.desc.L, self.desc.E),
                    pf_order=pf[:n_pf.value].copy(), ev_order=ev[:n_ev.value].copy())

    POLICIES = {"eam": 0, "lru": 1, "count": 2}

    def set_policy(self, policy: str) -> None:
        """Eviction rule: "eam" (Alg. 1, default), "lru" or "count" (the comparison rules)."""
        _check(lib().moei_cache_set_policy(self.h, self.POLICIES[policy]))

    def set_prefetch(self, depth: int) -> None:
        """Prefetch candidates considered after each synchronous layer step (0 = off)."""
        _check(lib().moei_cache_set_prefetch(self.h, int(depth)))

    def prefetch(self, pf_order, ev_order, V, depth: int, protect=(), stream=None):
        """Sec. 4.6 prefetch step from host-side orders and fp32 scores -> list of (fid, victim, slot)."""
        pf = np.ascontiguousarray(np.asarray(pf_order, dtype=np.int32).reshape(-1))
        ev = np.ascontiguousarray(np.asarray(ev_order, dtype=np.int32).reshape(-1))
        Vf = np.ascontiguousarray(np.asarray(V, dtype=np.float32).reshape(-1))
        assert Vf.size == self.desc.L * self.desc.E
        pr = np.ascontiguousarray(np.asarray(list(protect), dtype=np.int32).reshape(-1))
        n = max(int(depth), 1)
        fids, vic, slots = (np.empty(n, dtype=np.int32) for _ in range(3))
        issued = C.c_int32(0)
        _check(lib().moei_cache_prefetch(self.h, _p(pf) if pf.size else None, pf.size, _p(ev) if ev.size else None,
                                         ev.size, _p(Vf), int(depth), _p(pr) if pr.size else None, pr.size,
                                         _p(fids), _p(vic), _p(slots), C.byref(issued), _stream(stream)))
        m = issued.value
        return [(int(fids[i]), int(vic[i]), int(slots[i])) for i in range(m)]

    def last_prefetch(self):
        fids, vic = np.empty(32, dtype=np.int32), np.empty(32, dtype=np.int32)
        n = C.c_int32(0)
        _check(lib().moei_cache_last_prefetch(self.h, _p(fids), _p(vic), 32, C.byref(n)))
        return [(int(fids[i]), int(vic[i])) for i in range(n.value)]

    def set_match_count(self, m: int) -> None:
        """Traces aggregated by the layer step's prediction (Sec. 4.5 step 2); default 1."""
        _check(lib().moei_cache_set_match_count(self.h, int(m)))

    def last_matches(self, stream=None):
        """(trace indices, similarities) matched by the last layer step, most similar first."""
        top = np.empty(16, dtype=np.int32)
        sim = np.empty(16, dtype=np.float32)
        m = C.c_int32(0)
        _check(lib().moei_cache_last_matches(self.h, _p(top), _p(sim), 16, C.byref(m), _stream(stream)))
        return top[:m.value].copy(), sim[:m.value].copy()

    def close(self) -> None:
        if self.h:
            lib().moei_cache_destroy(self.h)
            self.h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ------------------------------------------------------------------------ entry points
def expert_pack(desc: ModelDesc, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
                out: np.ndarray | None = None) -> np.ndarray:
    """W_gate [I][H], W_up [I][H], W_down [H][I] (host arrays in the storage dtype) -> one
    expert in slot layout, flat [3*H*I].  Data movement only."""
    H, I = desc.H, desc.I
    dt = np.float32 if desc.wdtype == WDTYPE_FP32 else np.uint16
    g = np.ascontiguousarray(w_gate, dtype=dt)
    u = np.ascontiguousarray(w_up, dtype=dt)
    d = np.ascontiguousarray(w_down, dtype=dt)
    assert g.shape == (I, H) and u.shape == (I, H) and d.shape == (H, I)
    if out is None:
        out = np.empty(3 * H * I, dtype=dt)
    assert out.dtype == dt and out.size == 3 * H * I and out.flags["C_CONTIGUOUS"]
    _check(lib().moei_expert_pack(C.byref(desc), _p(g), _p(u), _p(d), _p(out)))
    return out



def moe_route_topk(logits: torch.Tensor, k: int, renorm: bool, stream=None):
    """logits [B][E] fp32 (device) -> (idx [B][k] int32, w [B][k] fp32) on the device."""
    _dev(logits, torch.float32)
    B, E = logits.shape
    idx = torch.empty((B, k), dtype=torch.int32, device=logits.device)
    w = torch.empty((B, k), dtype=torch.float32, device=logits.device)
    _check(lib().moe_route_topk(_p(logits), B, E, k, int(renorm), _p(idx), _p(w), _stream(stream)))
    return idx, w


def eam_update(eam: torch.Tensor, layer: int, idx: torch.Tensor, stream=None) -> None:
    """eam [B][L][E] int32 (device), updated in place with the picks idx [B][k]."""
    _dev(eam, torch.int32)
    _dev(idx, torch.int32)
    if eam.dim() == 2:
        eam = eam.unsqueeze(0)
    B, L, E = eam.shape
    assert idx.shape[0] == B
    _check(lib().eam_update(_p(eam), B, L, E, layer, _p(idx), idx.shape[1], _stream(stream)))


def eamc_match(eamc: Eamc, eam: torch.Tensor, layer_hi: int | None = None, want_sims: bool = False, stream=None):
    """eam [B][L][E] int32 (device) -> (best [B] int32, best_sim [B] fp32, sims [B][N] fp32 or None)."""
    _dev(eam, torch.int32)
    if eam.dim() == 2:
        eam = eam.unsqueeze(0)
    B = eam.shape[0]
    assert tuple(eam.shape[1:]) == (eamc.desc.L, eamc.desc.E)
    best = torch.empty(B, dtype=torch.int32, device=eam.device)
    sim = torch.empty(B, dtype=torch.float32, device=eam.device)
    sims = torch.empty((B, eamc.size), dtype=torch.float32, device=eam.device) if want_sims else None
    lh = eamc.desc.L - 1 if layer_hi is None else layer_hi
    _check(lib().eamc_match(eamc.h, _p(eam), B, lh, _p(best), _p(sim), _p(sims), _stream(stream)))
    return best, sim, sims


def eamc_match_topm(eamc: Eamc, eam: torch.Tensor, m: int, layer_hi: int | None = None, want_sims: bool = False,
                    stream=None):
    """eam [L][E] int32 (device) -> (top [m] int32, top_sim [m] fp32, sims [N] fp32 or None): the m most
    similar traces, most similar first; entries beyond the stored traces are -1."""
    _dev(eam, torch.int32)
    assert tuple(eam.shape) == (eamc.desc.L, eamc.desc.E)
    n = max(int(m), 1)
    top = torch.empty(n, dtype=torch.int32, device=eam.device)
    sim = torch.empty(n, dtype=torch.float32, device=eam.device)
    sims = torch.empty(eamc.size, dtype=torch.float32, device=eam.device) if want_sims else None
    lh = eamc.desc.L - 1 if layer_hi is None else layer_hi
    _check(lib().eamc_match_topm(eamc.h, _p(eam), lh, int(m), _p(top), _p(sim), _p(sims), _stream(stream)))
    return top, sim, sims


def expert_priority(eamc: Eamc, best: torch.Tensor, cur_layer: int, slot_of, eps: float,
                    cur_idx: torch.Tensor | None = None, stream=None):
    """-> (P [L][E] fp32, V [L][E] fp32, pf_order, n_pf, ev_order, n_ev), all device tensors.
    slot_of: device int32 tensor [L*E] or a raw device address (Cache.slot_table())."""
    _dev(best, torch.int32)
    L, E = eamc.desc.L, eamc.desc.E
    dev = best.device
    P = torch.empty((L, E), dtype=torch.float32, device=dev)
    V = torch.empty((L, E), dtype=torch.float32, device=dev)
    pf = torch.empty(L * E, dtype=torch.int32, device=dev)
    ev = torch.empty(L * E, dtype=torch.int32, device=dev)
    n_pf = torch.zeros(1, dtype=torch.int32, device=dev)
    n_ev = torch.zeros(1, dtype=torch.int32, device=dev)
    k = 0
    if cur_idx is not None:
        _dev(cur_idx, torch.int32)
        k = cur_idx.numel()
    _check(lib().expert_priority(eamc.h, _p(best), best.shape[0], cur_layer, _p(slot_of), C.c_float(eps),
                                 _p(cur_idx), k, _p(P), _p(V), _p(pf), _p(n_pf), _p(ev), _p(n_ev), _stream(stream)))
    return P, V, pf, n_pf, ev, n_ev


def expert_ffn_gemv(cache: Cache, slot_ids: torch.Tensor, gate_w: torch.Tensor, x: torch.Tensor, stream=None,
                    out: torch.Tensor | None = None) -> torch.Tensor:
    """x [H] in the weight dtype (device) -> y [H] fp32 over the given slots."""
    _dev(slot_ids, torch.int32)
    _dev(gate_w, torch.float32)
    assert x.is_cuda and x.is_contiguous() and x.numel() == cache.desc.H
    y = out if out is not None else torch.empty(cache.desc.H, dtype=torch.float32, device=x.device)
    _check(lib().expert_ffn_gemv(cache.h, _p(slot_ids), _p(gate_w), slot_ids.numel(), _p(x), _p(y), _stream(stream)))
    return y


def expert_ffn_gemv_static(cache: Cache, slot_ids: torch.Tensor, gate_w: torch.Tensor, x: torch.Tensor, out: torch.Tensor,
                           stream=None) -> torch.Tensor:
    """expert_ffn_gemv with its scratch in the library's static device array: allocates nothing,
    so the output tensor is the caller's."""
    _dev(slot_ids, torch.int32)
    _dev(gate_w, torch.float32)
    _dev(out, torch.float32)
    assert x.is_cuda and x.is_contiguous() and x.numel() == cache.desc.H and out.numel() == cache.desc.H
    _check(lib().expert_ffn_gemv_static(cache.h, _p(slot_ids), _p(gate_w), slot_ids.numel(), _p(x), _p(out),
                                        _stream(stream)))
    return out


def expert_ffn_grouped(cache: Cache, layer: int, idx: torch.Tensor, w: torch.Tensor, x: torch.Tensor,
                       stream=None) -> torch.Tensor:
    """Decode batch: idx [B][k] int32, w [B][k] fp32, x [B][H] weight dtype (device) -> y [B][H] fp32."""
    _dev(idx, torch.int32)
    _dev(w, torch.float32)
    B = idx.shape[0]
    assert x.is_cuda and x.is_contiguous() and x.numel() == B * cache.desc.H
    y = torch.empty((B, cache.desc.H), dtype=torch.float32, device=x.device)
    _check(lib().expert_ffn_grouped(cache.h, layer, _p(idx), _p(w), B, _p(x), _p(y), _stream(stream)))
    return y


def moe_decode_layer(cache: Cache, eamc: Eamc, eam: torch.Tensor, layer: int, router_w: torch.Tensor,
                     router_bias: torch.Tensor | None, x: torch.Tensor, y: torch.Tensor, sync: bool = True,
                     stream=None):
    """One fused layer step. sync=True returns (topk_idx [k] np.int32, best, n_miss); else None."""
    _dev(eam, torch.int32)
    assert router_w.is_cuda and x.is_cuda and y.is_cuda and y.dtype == torch.float32
    if not sync:
        _check(lib().moe_decode_layer(cache.h, eamc.h, _p(eam), layer, _p(router_w), _p(router_bias), _p(x), _p(y),
                                      None, None, None, _stream(stream)))
        return None
    idx = np.empty(cache.desc.k, dtype=np.int32)
    best, n_miss = C.c_int32(0), C.c_int32(0)
    _check(lib().moe_decode_layer(cache.h, eamc.h, _p(eam), layer, _p(router_w), _p(router_bias), _p(x), _p(y),
                                  _p(idx), C.byref(best), C.byref(n_miss), _stream(stream)))
    return idx, best.value, n_miss.value


# -------------------------------------------------------------------- kernel timing
def moe_prefill_layer(cache: Cache, eam: torch.Tensor, layer: int, router_w: torch.Tensor, router_bias,
                      X: torch.Tensor, Y: torch.Tensor | None = None, want_picks: bool = False, stream=None):
    """Prefill iteration of one layer: X [n][H] (bf16 bits) -> Y [n][H] fp32; eam [L][E] int32 updated in
    place.  Returns Y, or (Y, idx [n][k], w [n][k]) with want_picks."""
    _dev(eam, torch.int32)
    n, H = X.shape
    assert H == cache.desc.H and X.is_contiguous()
    if Y is None:
        Y = torch.empty((n, H), dtype=torch.float32, device=X.device)
    idx = torch.empty((n, cache.desc.k), dtype=torch.int32, device=X.device) if want_picks else None
    w = torch.empty((n, cache.desc.k), dtype=torch.float32, device=X.device) if want_picks else None
    _check(lib().moe_prefill_layer(cache.h, _p(eam), layer, _p(router_w), _p(router_bias), _p(X), n, _p(Y),
                                   _p(idx), _p(w), _stream(stream)))
    return (Y, idx, w) if want_picks else Y


def profile_enable(max_samples: int) -> None:
    _check(lib().moei_profile_enable(max_samples))


def profile_disable() -> None:
    _check(lib().moei_profile_disable())


def profile_samples(name: str) -> np.ndarray:
    """Durations (microseconds) of the recorded launches of one kernel, in launch order."""
    for i in range(lib().moei_profile_kernels()):
        if lib().moei_profile_kernel_name(i).decode() == name:
            n = C.c_int32(0)
            _check(lib().moei_profile_samples(i, None, 0, C.byref(n)))
            out = np.empty(max(n.value, 1), dtype=np.float32)
            _check(lib().moei_profile_samples(i, _p(out), n.value, C.byref(n)))
            return out[:n.value].astype(np.float64) * 1e3
    raise KeyError(name)


def profile_read() -> dict:
    """{kernel name: (launches recorded, total milliseconds between their event brackets)}"""
    out = {}
    for i in range(lib().moei_profile_kernels()):
        t, n = C.c_double(0), C.c_int32(0)
        _check(lib().moei_profile_read(i, C.byref(t), C.byref(n)))
        out[lib().moei_profile_kernel_name(i).decode()] = (n.value, t.value)
    return out
