"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

__all__ = [
    "LZ_F32", "LZ_BF16", "LZ_GELU", "LZ_SWIGLU", "LzError", "Shape", "lib", "lib_path",
    "lz_strerror", "lz_version", "lz_plan_workspace_bytes", "lz_ffn_workspace_bytes",
    "lz_route", "lz_plan_dispatch", "lz_plan_dispatch_noalloc", "LZ_PLAN_NOALLOC_SCRATCH_BYTES", "lz_permute", "lz_permute_scatter", "lz_expert_ffn", "lz_unpermute_combine",
    "lz_ffn_tiles", "lz_ffn_up", "lz_ffn_down", "lz_ffn_up_gather", "lz_expert_ffn_gather", "lz_allocate_replicas", "lz_place_mro", "lz_place_spread", "lz_place_compact", "lz_recovery_probability",
    "lz_replan", "lz_apply_transfers", "MoELayer",
    "lz_pack_weights", "lz_train_workspace_bytes", "lz_ffn_forward_train", "lz_combine_backward",
    "lz_ffn_backward", "lz_ffn_backward_accumulate", "lz_permute_backward", "lz_route_backward", "lz_reduce_replica_grads",
    "lz_reduce_replica_grads_dtype", "lz_debug_xcc_ids",
]

LZ_F32, LZ_BF16 = 0, 1
LZ_GELU, LZ_SWIGLU = 0, 1
LZ_PLAN_NOALLOC_SCRATCH_BYTES = 4 << 20
LZ_OK, LZ_EINVAL, LZ_ESHAPE, LZ_EWORKSPACE, LZ_EUNRECOVERABLE, LZ_EINFEASIBLE, LZ_EHIP = 0, -1, -2, -3, -4, -5, -6


class LzError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lz_strerror(code)} ({code})")


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("T", "d", "ffn", "E", "k", "N", "c", "dtype", "act")]


class _Transfer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dst_slot", "src_slot", "expert", "remote")]


@dataclass(frozen=True)
class Shape:
    T: int
    d: int
    ffn: int
    E: int
    k: int
    N: int
    c: int
    dtype: int
    act: int

    @property
    def S(self):
        return self.N * self.c

    @property
    def P(self):
        return self.T * self.k

    def c_struct(self):
        return _Shape(self.T, self.d, self.ffn, self.E, self.k, self.N, self.c, self.dtype, self.act)

    @staticmethod
    def from_config(cfg):
        return Shape(cfg.T, cfg.d, cfg.ffn, cfg.E, cfg.k, cfg.N, cfg.c,
                     LZ_F32 if cfg.dtype == "f32" else LZ_BF16,
                     LZ_GELU if cfg.act == "gelu" else LZ_SWIGLU)


def lib_path() -> str:
    """The in-tree library, or the build LAZARUS_MOE_LIB points at (same ABI, other build flags)."""
    override = os.environ.get("LAZARUS_MOE_LIB")
    if override:
        return override
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblazarus_moe.so")


def _load():
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it first (python paper_2407_04656_amd/build.py or "
            "__graft_entry__.build()); there is no fallback path")
    # PyTorch-ROCm ships its own HIP runtime.  Load it first when torch is installed, so that this
    # library binds to the same runtime as the tensors and streams it is handed (with two
    # runtimes in one process every launch on a torch stream fails).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(path)
    vp, i32, u64 = C.c_void_p, C.c_int32, C.c_size_t
    sp = C.POINTER(_Shape)
    sig = {
        "lz_strerror": (C.c_char_p, [i32]),
        "lz_version": (i32, []),
        "lz_plan_workspace_bytes": (u64, [sp]),
        "lz_ffn_workspace_bytes": (u64, [sp]),
        "lz_route": (i32, [vp, i32, i32, i32, vp, vp, vp]),
        "lz_plan_dispatch": (i32, [vp, sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u64, vp]),
        "lz_plan_dispatch_noalloc": (i32, [vp, sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "lz_permute": (i32, [vp, vp, sp, vp, vp]),
        "lz_permute_scatter": (i32, [vp, vp, sp, vp, vp]),
        "lz_expert_ffn": (i32, [vp, vp, vp, vp, sp, vp, vp, u64, vp]),
        "lz_unpermute_combine": (i32, [vp, vp, vp, sp, vp, vp]),
        "lz_ffn_tiles": (i32, [vp, sp, vp, u64, vp]),
        "lz_ffn_up": (i32, [vp, vp, sp, vp, u64, vp]),
        "lz_ffn_down": (i32, [vp, sp, vp, vp, u64, vp]),
        "lz_ffn_up_gather": (i32, [vp, vp, vp, sp, vp, u64, vp]),
        "lz_expert_ffn_gather": (i32, [vp, vp, vp, vp, vp, sp, vp, vp, u64, vp]),
        "lz_allocate_replicas": (i32, [vp, i32, i32, i32, i32, vp]),
        "lz_place_mro": (i32, [vp, vp, i32, i32, i32, vp]),
        "lz_place_spread": (i32, [vp, i32, i32, i32, vp]),
        "lz_place_compact": (i32, [vp, i32, i32, i32, vp]),
        "lz_recovery_probability": (i32, [vp, i32, i32, i32, i32, vp, vp]),
        "lz_replan": (i32, [vp, i32, i32, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]),
        "lz_apply_transfers": (i32, [vp, i32, vp, vp, i32, vp, vp, i32, sp, vp]),
        "lz_pack_weights": (i32, [vp, i32, i32, i32, i32, vp, vp]),
        "lz_train_workspace_bytes": (u64, [sp]),
        "lz_ffn_forward_train": (i32, [vp, vp, vp, vp, sp, vp, vp, vp, vp, u64, vp]),
        "lz_combine_backward": (i32, [vp, vp, vp, vp, sp, vp, vp, vp]),
        "lz_ffn_backward": (i32, [vp, vp, vp, vp, vp, vp, vp, sp, vp, vp, vp, vp, u64, vp]),
        "lz_ffn_backward_accumulate": (i32, [vp, vp, vp, vp, vp, vp, vp, sp, vp, vp, vp, vp, u64, vp]),
        "lz_permute_backward": (i32, [vp, vp, sp, vp, vp]),
        "lz_route_backward": (i32, [vp, vp, vp, sp, vp, vp]),
        "lz_reduce_replica_grads": (i32, [vp, vp, i32, i32, C.c_int64, vp, vp]),
        "lz_reduce_replica_grads_dtype": (i32, [vp, vp, i32, i32, C.c_int64, i32, vp, vp]),
        "lz_debug_xcc_ids": (i32, [vp, i32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()
def lz_strerror(code: int) -> str:
    return lib.lz_strerror(int(code)).decode()


def lz_version() -> int:
    return int(lib.lz_version())


def _check(code: int, where: str):
    if code != LZ_OK:
        raise LzError(code, where)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array, None -> NULL."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    assert t.is_contiguous()
    return t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def lz_plan_workspace_bytes(shape: Shape) -> int:
    return int(lib.lz_plan_workspace_bytes(C.byref(shape.c_struct())))


def lz_ffn_workspace_bytes(shape: Shape) -> int:
    return int(lib.lz_ffn_workspace_bytes(C.byref(shape.c_struct())))


# ------------------------------------------------------------------ device hot path
def lz_route(logits, T, E, k, topk_ids, topk_gates, stream=None):
    _check(lib.lz_route(_ptr(logits), T, E, k, _ptr(topk_ids), _ptr(topk_gates),
                        _stream() if stream is None else stream), "lz_route")


def lz_plan_dispatch(topk_ids, shape, rank_tok_off, slot_expert, slot_counts, slot_offsets, pair_to_row,
                     row_to_pair, Tej_opt, D_opt, status_opt, ws, ws_bytes, stream=None):
    _check(lib.lz_plan_dispatch(_ptr(topk_ids), C.byref(shape.c_struct()), _ptr(rank_tok_off),
                                _ptr(slot_expert), _ptr(slot_counts), _ptr(slot_offsets),
                                _ptr(pair_to_row), _ptr(row_to_pair), _ptr(Tej_opt), _ptr(D_opt),
                                _ptr(status_opt), _ptr(ws), ws_bytes,
                                _stream() if stream is None else stream), "lz_plan_dispatch")


def lz_plan_dispatch_noalloc(topk_ids, shape, rank_tok_off, slot_expert, slot_counts, slot_offsets, pair_to_row,
                             row_to_pair, Tej_opt, D_opt, status_opt, stream=None):
    _check(lib.lz_plan_dispatch_noalloc(_ptr(topk_ids), C.byref(shape.c_struct()), _ptr(rank_tok_off),
                                        _ptr(slot_expert), _ptr(slot_counts), _ptr(slot_offsets),
                                        _ptr(pair_to_row), _ptr(row_to_pair), _ptr(Tej_opt), _ptr(D_opt),
                                        _ptr(status_opt), _stream() if stream is None else stream),
           "lz_plan_dispatch_noalloc")


def lz_permute(x, row_to_pair, shape, xp, stream=None):
    _check(lib.lz_permute(_ptr(x), _ptr(row_to_pair), C.byref(shape.c_struct()), _ptr(xp),
                          _stream() if stream is None else stream), "lz_permute")


def lz_permute_scatter(x, pair_to_row, shape, xp, stream=None):
    _check(lib.lz_permute_scatter(_ptr(x), _ptr(pair_to_row), C.byref(shape.c_struct()), _ptr(xp),
                                  _stream() if stream is None else stream), "lz_permute_scatter")


def lz_pack_weights(w, S, rows, cols, dtype, packed, stream=None):
    _check(lib.lz_pack_weights(_ptr(w), S, rows, cols, dtype, _ptr(packed),
                               _stream() if stream is None else stream), "lz_pack_weights")


def lz_expert_ffn(xp, slot_offsets, w1, w2, shape, yp, ws, ws_bytes, stream=None):
    _check(lib.lz_expert_ffn(_ptr(xp), _ptr(slot_offsets), _ptr(w1), _ptr(w2), C.byref(shape.c_struct()),
                             _ptr(yp), _ptr(ws), ws_bytes,
                             _stream() if stream is None else stream), "lz_expert_ffn")


def lz_ffn_tiles(slot_offsets, shape, ws, ws_bytes, stream=None):
    _check(lib.lz_ffn_tiles(_ptr(slot_offsets), C.byref(shape.c_struct()), _ptr(ws), ws_bytes,
                            _stream() if stream is None else stream), "lz_ffn_tiles")


def lz_ffn_up(xp, w1, shape, ws, ws_bytes, stream=None):
    _check(lib.lz_ffn_up(_ptr(xp), _ptr(w1), C.byref(shape.c_struct()), _ptr(ws), ws_bytes,
                         _stream() if stream is None else stream), "lz_ffn_up")


def lz_ffn_up_gather(x, row_to_pair, w1, shape, ws, ws_bytes, stream=None):
    _check(lib.lz_ffn_up_gather(_ptr(x), _ptr(row_to_pair), _ptr(w1), C.byref(shape.c_struct()), _ptr(ws), ws_bytes,
                                _stream() if stream is None else stream), "lz_ffn_up_gather")


def lz_expert_ffn_gather(x, row_to_pair, slot_offsets, w1, w2, shape, yp, ws, ws_bytes, stream=None):
    _check(lib.lz_expert_ffn_gather(_ptr(x), _ptr(row_to_pair), _ptr(slot_offsets), _ptr(w1), _ptr(w2),
                                    C.byref(shape.c_struct()), _ptr(yp), _ptr(ws), ws_bytes,
                                    _stream() if stream is None else stream), "lz_expert_ffn_gather")


def lz_ffn_down(w2, shape, yp, ws, ws_bytes, stream=None):
    _check(lib.lz_ffn_down(_ptr(w2), C.byref(shape.c_struct()), _ptr(yp), _ptr(ws), ws_bytes,
                           _stream() if stream is None else stream), "lz_ffn_down")


def lz_unpermute_combine(yp, pair_to_row, topk_gates, shape, y, stream=None):
    _check(lib.lz_unpermute_combine(_ptr(yp), _ptr(pair_to_row), _ptr(topk_gates),
                                    C.byref(shape.c_struct()), _ptr(y),
                                    _stream() if stream is None else stream), "lz_unpermute_combine")


# ------------------------------------------------------------------ training
def lz_train_workspace_bytes(shape: Shape) -> int:
    return int(lib.lz_train_workspace_bytes(C.byref(shape.c_struct())))


def lz_ffn_forward_train(xp, slot_offsets, w1, w2, shape, z, h, yp, ws, ws_bytes, stream=None):
    _check(lib.lz_ffn_forward_train(_ptr(xp), _ptr(slot_offsets), _ptr(w1), _ptr(w2), C.byref(shape.c_struct()),
                                    _ptr(z), _ptr(h), _ptr(yp), _ptr(ws), ws_bytes,
                                    _stream() if stream is None else stream), "lz_ffn_forward_train")


def lz_combine_backward(dy, yp, pair_to_row, topk_gates, shape, dyp, dgates, stream=None):
    _check(lib.lz_combine_backward(_ptr(dy), _ptr(yp), _ptr(pair_to_row), _ptr(topk_gates),
                                   C.byref(shape.c_struct()), _ptr(dyp), _ptr(dgates),
                                   _stream() if stream is None else stream), "lz_combine_backward")


def lz_ffn_backward(dyp, xp, z, h, slot_offsets, w1, w2, shape, dxp, dw1, dw2, ws, ws_bytes, stream=None):
    _check(lib.lz_ffn_backward(_ptr(dyp), _ptr(xp), _ptr(z), _ptr(h), _ptr(slot_offsets), _ptr(w1), _ptr(w2),
                               C.byref(shape.c_struct()), _ptr(dxp), _ptr(dw1), _ptr(dw2), _ptr(ws), ws_bytes,
                               _stream() if stream is None else stream), "lz_ffn_backward")


def lz_ffn_backward_accumulate(dyp, xp, z, h, slot_offsets, w1, w2, shape, dxp, dw1_acc, dw2_acc, ws, ws_bytes,
                               stream=None):
    _check(lib.lz_ffn_backward_accumulate(_ptr(dyp), _ptr(xp), _ptr(z), _ptr(h), _ptr(slot_offsets), _ptr(w1),
                                          _ptr(w2), C.byref(shape.c_struct()), _ptr(dxp), _ptr(dw1_acc),
                                          _ptr(dw2_acc), _ptr(ws), ws_bytes,
                                          _stream() if stream is None else stream), "lz_ffn_backward_accumulate")


def lz_permute_backward(dxp, pair_to_row, shape, dx, stream=None):
    _check(lib.lz_permute_backward(_ptr(dxp), _ptr(pair_to_row), C.byref(shape.c_struct()), _ptr(dx),
                                   _stream() if stream is None else stream), "lz_permute_backward")


def lz_route_backward(dgates, topk_gates, topk_ids, shape, dlogits, stream=None):
    _check(lib.lz_route_backward(_ptr(dgates), _ptr(topk_gates), _ptr(topk_ids), C.byref(shape.c_struct()),
                                 _ptr(dlogits), _stream() if stream is None else stream), "lz_route_backward")


def lz_reduce_replica_grads(dw_slot, slot_expert, S, E, elems_per_slot, dw, stream=None):
    _check(lib.lz_reduce_replica_grads(_ptr(dw_slot), _ptr(slot_expert), S, E, elems_per_slot, _ptr(dw),
                                       _stream() if stream is None else stream), "lz_reduce_replica_grads")


def lz_reduce_replica_grads_dtype(dw_slot, slot_expert, S, E, elems_per_slot, dtype, dw, stream=None):
    _check(lib.lz_reduce_replica_grads_dtype(_ptr(dw_slot), _ptr(slot_expert), S, E, elems_per_slot, dtype, _ptr(dw),
                                             _stream() if stream is None else stream),
           "lz_reduce_replica_grads_dtype")


def lz_debug_xcc_ids(xcc_of_workgroup, n_workgroups, stream=None):
    _check(lib.lz_debug_xcc_ids(_ptr(xcc_of_workgroup), n_workgroups, _stream() if stream is None else stream),
           "lz_debug_xcc_ids")


# ------------------------------------------------------------------ host planning
def _i64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def lz_allocate_replicas(t_e, N, c, f):
    t = _i64(t_e)
    r = np.zeros(len(t), dtype=np.int32)
    _check(lib.lz_allocate_replicas(t.ctypes.data, len(t), N, c, f, r.ctypes.data), "lz_allocate_replicas")
    return r


def lz_place_mro(r_e, t_e, N, c):
    r, t = _i32(r_e), _i64(t_e)
    out = np.full(N * c, -1, dtype=np.int32)
    _check(lib.lz_place_mro(r.ctypes.data, t.ctypes.data, len(r), N, c, out.ctypes.data), "lz_place_mro")
    return out


def lz_place_spread(r_e, N, c):
    r = _i32(r_e)
    out = np.full(N * c, -1, dtype=np.int32)
    _check(lib.lz_place_spread(r.ctypes.data, len(r), N, c, out.ctypes.data), "lz_place_spread")
    return out


def lz_place_compact(r_e, N, c):
    r = _i32(r_e)
    out = np.full(N * c, -1, dtype=np.int32)
    _check(lib.lz_place_compact(r.ctypes.data, len(r), N, c, out.ctypes.data), "lz_place_compact")
    return out


def lz_recovery_probability(slot_expert, E, N, c, n_alive):
    se = _i32(slot_expert)
    good, total = C.c_uint64(0), C.c_uint64(0)
    _check(lib.lz_recovery_probability(se.ctypes.data, E, N, c, n_alive, C.addressof(good),
                                       C.addressof(total)), "lz_recovery_probability")
    return good.value, total.value


def lz_replan(old_slot_expert, N_old, c_old, alive, t_e, c_new, f):
    old, t = _i32(old_slot_expert), _i64(t_e)
    al = np.ascontiguousarray(np.asarray(alive, dtype=np.uint8))
    n_max = int(al.astype(bool).sum())
    new = np.full(max(1, n_max * c_new), -1, dtype=np.int32)
    plan2phys = np.full(max(1, n_max), -1, dtype=np.int32)
    xf = (_Transfer * max(1, n_max * c_new))()
    n_x = C.c_int32(n_max * c_new)
    n_new = C.c_int32(0)
    _check(lib.lz_replan(old.ctypes.data, N_old, c_old, al.ctypes.data, t.ctypes.data, len(t), c_new, f,
                         new.ctypes.data, plan2phys.ctypes.data, C.addressof(xf), C.addressof(n_x),
                         C.addressof(n_new)), "lz_replan")
    transfers = [(x.dst_slot, x.src_slot, x.expert, x.remote) for x in xf[:n_x.value]]
    return {"new_slot_expert": new[:n_new.value * c_new], "plan2phys": plan2phys[:n_new.value],
            "transfers": transfers, "N_new": n_new.value}


def lz_apply_transfers(transfers, w1_old, w2_old, S_old, w1_new, w2_new, S_new, shape, stream=None):
    arr = (_Transfer * max(1, len(transfers)))()
    for i, (d, s, e, r) in enumerate(transfers):
        arr[i] = _Transfer(d, s, e, r)
    _check(lib.lz_apply_transfers(C.addressof(arr), len(transfers), _ptr(w1_old), _ptr(w2_old), S_old,
                                  _ptr(w1_new), _ptr(w2_new), S_new, C.byref(shape.c_struct()),
                                  _stream() if stream is None else stream), "lz_apply_transfers")


# ------------------------------------------------------------------ convenience
class MoELayer:
    """Owns the device buffers of one layer shape and runs the five calls in order.

    Buffer management only: torch allocates, the library computes.  Weights are per-slot
    copies laid out input-major, w1[S, d, n1], w2[S, ffn, d] (see include/lazarus_moe.h).
    """

    def __init__(self, shape: Shape, device="cuda:0"):
        import torch
        self.shape = shape
        self.device = torch.device(device)
        s = shape
        tdt = torch.float32 if s.dtype == LZ_F32 else torch.bfloat16
        dev = self.device
        i32 = torch.int32
        self.topk_ids = torch.empty((s.T, s.k), dtype=i32, device=dev)
        self.topk_gates = torch.empty((s.T, s.k), dtype=torch.float32, device=dev)
        self.slot_counts = torch.empty(s.S, dtype=i32, device=dev)
        self.slot_offsets = torch.empty(s.S + 1, dtype=i32, device=dev)
        self.pair_to_row = torch.empty(s.P, dtype=i32, device=dev)
        self.row_to_pair = torch.empty(s.P, dtype=i32, device=dev)
        self.Tej = torch.empty((s.E, s.N), dtype=i32, device=dev)
        self.D = torch.empty((s.E, s.N, s.N), dtype=i32, device=dev)
        self.status = torch.zeros(1, dtype=i32, device=dev)
        self.xp = torch.empty((s.P, s.d), dtype=tdt, device=dev)
        self.yp = torch.empty((s.P, s.d), dtype=tdt, device=dev)
        self.y = torch.empty((s.T, s.d), dtype=tdt, device=dev)
        self.plan_ws_bytes = lz_plan_workspace_bytes(shape)
        self.ffn_ws_bytes = lz_ffn_workspace_bytes(shape)
        self.plan_ws = torch.empty(self.plan_ws_bytes, dtype=torch.uint8, device=dev)
        self.ffn_ws = torch.empty(self.ffn_ws_bytes, dtype=torch.uint8, device=dev)
        self.rank_tok_off = None
        self.slot_expert = None
        self.w1 = None
        self.w2 = None

    def set_plan(self, slot_expert, rank_tok_off):
        import torch
        self.slot_expert = torch.as_tensor(np.asarray(slot_expert, dtype=np.int32), device=self.device)
        self.rank_tok_off = torch.as_tensor(np.asarray(rank_tok_off, dtype=np.int32), device=self.device)

    def set_slot_weights(self, w1, w2):
        self.w1, self.w2 = w1, w2

    def load_expert_weights(self, w1_experts, w2_experts, slot_expert):
        """Give every slot its own copy of its expert's weights.  The host arrays are indexed by
        expert and come in the usual [out, in] layout (w1 [E, n1, d], w2 [E, d, ffn]); every expert
        is converted once with lz_pack_weights and copied to its slots."""
        import torch
        s = self.shape
        tdt = torch.float32 if s.dtype == LZ_F32 else torch.bfloat16

        def to_dev(a):
            t = torch.from_numpy(a)
            if s.dtype == LZ_BF16:
                t = t.view(torch.bfloat16)
            t = t.to(self.device)
            packed = torch.empty((t.shape[1], t.shape[0]), dtype=t.dtype, device=self.device)
            lz_pack_weights(t, 1, t.shape[0], t.shape[1], s.dtype, packed)
            return packed

        n1 = w1_experts.shape[1]
        self.w1 = torch.empty((s.S, s.d, n1), dtype=tdt, device=self.device)
        self.w2 = torch.empty((s.S, s.ffn, s.d), dtype=tdt, device=self.device)
        cache = {}
        for slot, e in enumerate(np.asarray(slot_expert)):
            e = int(e)
            if e not in cache:
                cache[e] = (to_dev(w1_experts[e]), to_dev(w2_experts[e]))
            self.w1[slot].copy_(cache[e][0])
            self.w2[slot].copy_(cache[e][1])

    # the five calls
    def route(self, logits):
        s = self.shape
        lz_route(logits, s.T, s.E, s.k, self.topk_ids, self.topk_gates)

    def plan_dispatch(self):
        lz_plan_dispatch(self.topk_ids, self.shape, self.rank_tok_off, self.slot_expert, self.slot_counts,
                         self.slot_offsets, self.pair_to_row, self.row_to_pair, self.Tej, self.D,
                         self.status, self.plan_ws, self.plan_ws_bytes)

    def permute(self, x):
        lz_permute_scatter(x, self.pair_to_row, self.shape, self.xp)

    def expert_ffn(self):
        lz_expert_ffn(self.xp, self.slot_offsets, self.w1, self.w2, self.shape, self.yp, self.ffn_ws,
                      self.ffn_ws_bytes)

    def unpermute_combine(self):
        lz_unpermute_combine(self.yp, self.pair_to_row, self.topk_gates, self.shape, self.y)

    def forward(self, logits, x):
        self.route(logits)
        self.plan_dispatch()
        self.permute(x)
        self.expert_ffn()
        self.unpermute_combine()
        return self.y

    # ---- training: forward that keeps its intermediates, then the backward chain
    def enable_training(self):
        """Allocate what the backward needs."""
        import torch
        s, dev = self.shape, self.device
        bf = torch.float32 if s.dtype == LZ_F32 else torch.bfloat16
        n1 = self.w1.shape[2]
        self.train_ws_bytes = lz_train_workspace_bytes(s)
        if self.train_ws_bytes == 0:
            raise LzError(LZ_ESHAPE, "lz_train_workspace_bytes")
        self.train_ws = torch.empty(self.train_ws_bytes, dtype=torch.uint8, device=dev)
        self.z = torch.empty((s.P, n1), dtype=bf, device=dev)
        self.h = torch.empty((s.P, s.ffn), dtype=bf, device=dev)
        self.dyp = torch.empty((s.P, s.d), dtype=bf, device=dev)
        self.dxp = torch.empty((s.P, s.d), dtype=bf, device=dev)
        self.dx = torch.empty((s.T, s.d), dtype=bf, device=dev)
        self.dgates = torch.empty((s.T, s.k), dtype=torch.float32, device=dev)
        self.dlogits = torch.empty((s.T, s.E), dtype=torch.float32, device=dev)
        self.dw1_slot = torch.empty((s.S, s.d, n1), dtype=bf, device=dev)
        self.dw2_slot = torch.empty((s.S, s.ffn, s.d), dtype=bf, device=dev)
        self.dw1 = torch.empty((s.E, s.d, n1), dtype=bf, device=dev)
        self.dw2 = torch.empty((s.E, s.ffn, s.d), dtype=bf, device=dev)

    def forward_fused(self, logits, x):
        """The same pass with the reshuffle done by the first GEMM's loads (no permute call, xp unused)."""
        self.route(logits)
        self.plan_dispatch()
        lz_expert_ffn_gather(x, self.row_to_pair, self.slot_offsets, self.w1, self.w2, self.shape, self.yp,
                             self.ffn_ws, self.ffn_ws_bytes)
        self.unpermute_combine()
        return self.y

    def forward_train(self, logits, x):
        self.route(logits)
        self.plan_dispatch()
        self.permute(x)
        lz_ffn_forward_train(self.xp, self.slot_offsets, self.w1, self.w2, self.shape, self.z, self.h, self.yp,
                             self.train_ws, self.train_ws_bytes)
        self.unpermute_combine()
        return self.y

    def enable_accumulation(self):
        """fp32 accumulators for the slots' weight gradients (micro-batches), zeroed."""
        import torch
        self.dw1_acc = torch.zeros(tuple(self.dw1_slot.shape), dtype=torch.float32, device=self.device)
        self.dw2_acc = torch.zeros(tuple(self.dw2_slot.shape), dtype=torch.float32, device=self.device)
        self.dw1_sum = torch.empty(tuple(self.dw1.shape), dtype=torch.float32, device=self.device)
        self.dw2_sum = torch.empty(tuple(self.dw2.shape), dtype=torch.float32, device=self.device)

    def backward_accumulate(self, dy):
        """One micro-batch: data gradients as in backward(), weight gradients added to the fp32 accumulators."""
        s = self.shape
        lz_combine_backward(dy, self.yp, self.pair_to_row, self.topk_gates, s, self.dyp, self.dgates)
        lz_ffn_backward_accumulate(self.dyp, self.xp, self.z, self.h, self.slot_offsets, self.w1, self.w2, s,
                                   self.dxp, self.dw1_acc, self.dw2_acc, self.train_ws, self.train_ws_bytes)
        lz_permute_backward(self.dxp, self.pair_to_row, s, self.dx)
        lz_route_backward(self.dgates, self.topk_gates, self.topk_ids, s, self.dlogits)
        return self.dx

    def reduce_accumulated(self):
        """Per-expert sums of the accumulators over the replicas (fp32)."""
        s = self.shape
        lz_reduce_replica_grads_dtype(self.dw1_acc, self.slot_expert, s.S, s.E, self.dw1_acc[0].numel(), LZ_F32,
                                      self.dw1_sum)
        lz_reduce_replica_grads_dtype(self.dw2_acc, self.slot_expert, s.S, s.E, self.dw2_acc[0].numel(), LZ_F32,
                                      self.dw2_sum)
        return self.dw1_sum, self.dw2_sum

    def backward(self, dy):
        s = self.shape
        lz_combine_backward(dy, self.yp, self.pair_to_row, self.topk_gates, s, self.dyp, self.dgates)
        lz_ffn_backward(self.dyp, self.xp, self.z, self.h, self.slot_offsets, self.w1, self.w2, s, self.dxp,
                        self.dw1_slot, self.dw2_slot, self.train_ws, self.train_ws_bytes)
        lz_permute_backward(self.dxp, self.pair_to_row, s, self.dx)
        lz_route_backward(self.dgates, self.topk_gates, self.topk_ids, s, self.dlogits)
        lz_reduce_replica_grads_dtype(self.dw1_slot, self.slot_expert, s.S, s.E, self.dw1_slot[0].numel(), s.dtype,
                                      self.dw1)
        lz_reduce_replica_grads_dtype(self.dw2_slot, self.slot_expert, s.S, s.E, self.dw2_slot[0].numel(), s.dtype,
                                      self.dw2)
        return self.dx
