"""ctypes binding of libflexlink.so: same names as the C ABI, argument
marshalling only.  Every step of the collectives runs inside the library.

torch is used for device memory and streams; it is imported first so that the
library binds to the HIP runtime torch has already loaded.
"""
import ctypes
import os

import torch  # noqa: F401  (must precede loading the library)

from . import build as _build

FLEX_MAX_RANKS = 8
FLEX_MAX_PATHS = 4

FLEX_OK, FLEX_ERR_INVALID_ARG, FLEX_ERR_UNSUPPORTED, FLEX_ERR_HIP, FLEX_ERR_NOMEM, FLEX_ERR_STATE = range(6)
FLEX_F32, FLEX_BF16, FLEX_F16 = 0, 1, 2
FLEX_SUM = 0
FLEX_ALLREDUCE, FLEX_ALLGATHER, FLEX_REDUCESCATTER, FLEX_ALLTOALL = 0, 1, 2, 3
FLEX_PATH_DEVICE, FLEX_PATH_HOST, FLEX_PATH_HOST2 = 0, 1, 2
FLEX_SPLIT_STATIC, FLEX_SPLIT_ADAPTIVE = 0, 1
FLEX_STAGE_TUNING, FLEX_STAGE_RUNTIME = 1, 2
FLEX_ENGINE_KERNEL, FLEX_ENGINE_HYBRID, FLEX_ENGINE_SDMA = 0, 1, 2
FLEX_SHAPE_WAVE, FLEX_SHAPE_BLOCK = 0, 1
FLEX_SYNC_EVENTS, FLEX_SYNC_COUNTERS = 0, 1

u32, u64, i32, f64 = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int32, ctypes.c_double


class _Struct(ctypes.Structure):
    def as_dict(self):
        out = {}
        for name, _ in self._fields_:
            v = getattr(self, name)
            if isinstance(v, _Struct):
                v = v.as_dict()
            elif isinstance(v, ctypes.Array):
                v = list(v)
            out[name] = v
        return out


class BalancerCfg(_Struct):
    _fields_ = [("share_total", u32), ("initial_step", u32), ("stability_required", u32),
                ("max_tune_iters", u32), ("window", u32), ("runtime_step", u32),
                ("aux_share_cap", u32), ("reserved", u32),
                ("convergence_threshold", f64), ("runtime_threshold", f64)]


class BalancerState(_Struct):
    _fields_ = [("npaths", u32), ("stage", u32), ("tune_iters", u32), ("step", u32),
                ("stability_count", u32), ("prev_slowest", i32), ("active_mask", u32),
                ("window_fill", u32), ("adjustments", u64), ("shares", u32 * FLEX_MAX_PATHS)]


class Config(_Struct):
    _fields_ = [("struct_size", u32), ("num_slots", u32), ("chunk_bytes", u64), ("min_split_bytes", u64),
                ("max_host_units", u32), ("split_align_elems", u32), ("tune_reps", u32), ("probe_units", u32),
                ("tune_accept_check", u32), ("accept_pairs", u32), ("launch_shape", u32),
                ("reduce_serial_loads", u32), ("reduce_nontemporal", u32), ("copy_nontemporal", u32),
                ("reduce_lds_reserve", u32), ("reserved", u32),
                ("host_engine", u32), ("host_blocks", u32), ("host_die_shift", u32), ("min_step_bytes", u32),
                ("slot_sync", u32), ("num_aux_paths", u32), ("host_down_blocks", u32), ("sample_every", u32),
                ("balancer", BalancerCfg)]


class Stats(_Struct):
    _fields_ = [("calls", u64), ("split_calls", u64), ("samples", u64), ("blocking_reads", u64),
                ("last_count", u64), ("last_split", u64), ("mode", u32), ("static_host_units", u32),
                ("last_time_s", f64 * FLEX_MAX_PATHS), ("mean_time_s", f64 * FLEX_MAX_PATHS),
                ("npaths", u32), ("static_units", u32 * FLEX_MAX_PATHS), ("reserved", u32),
                ("last_start", u64 * FLEX_MAX_PATHS),
                ("balancer", BalancerState)]


class TuneResult(_Struct):
    _fields_ = [("path_bw", f64 * FLEX_MAX_PATHS), ("initial_shares", u32 * FLEX_MAX_PATHS),
                ("shares", u32 * FLEX_MAX_PATHS), ("active_mask", u32), ("iterations", u32),
                ("path_time_s", f64 * FLEX_MAX_PATHS), ("balanced_shares", u32 * FLEX_MAX_PATHS),
                ("device_alone_s", f64), ("combined_s", f64), ("device_alone_mad_s", f64),
                ("combined_mad_s", f64), ("accept_samples", u32), ("reverted", u32)]


class TuneRound(_Struct):
    _fields_ = [("path_time_s", f64 * FLEX_MAX_PATHS), ("shares_before", u32 * FLEX_MAX_PATHS),
                ("shares_after", u32 * FLEX_MAX_PATHS), ("step_after", u32), ("active_after", u32)]


class FlexError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("flexlink status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built: there is no
    fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        raise RuntimeError(
            "libflexlink.so is not built (%s missing); run `python -m paper_2510_15882_amd.build` "
            "or __graft_entry__.build()" % path)
    L = ctypes.CDLL(path)
    vp, pvp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
    sz, ci = ctypes.c_size_t, ctypes.c_int
    P = ctypes.POINTER
    sigs = {
        "flex_balancer_cfg_default": [P(BalancerCfg)],
        "flex_balancer_init": [pvp, ci, P(f64), P(BalancerCfg)],
        "flex_balancer_init_shares": [pvp, ci, P(u32), P(BalancerCfg)],
        "flex_balancer_update": [vp, P(f64), P(u32)],
        "flex_balancer_finish_tuning": [vp],
        "flex_balancer_revert_to_primary": [vp],
        "flex_balancer_get": [vp, P(BalancerState)],
        "flex_balancer_destroy": [vp],
        "flex_partition": [u64, u32, u32, u32, u64, P(u64)],
        "flex_partition_paths": [u64, P(u32), ci, u32, u32, u64, P(u64)],
        "flex_set_split_paths": [vp, ci, ci, P(u32), ci],
        "flex_struct_sizes": [P(sz)],
        "flex_config_default": [P(Config)],
        "flex_comm_create": [pvp, ci, ci, sz, P(Config)],
        "flex_comm_destroy": [vp],
        "flex_allreduce_local": [vp, pvp, vp, sz, ci, ci, vp],
        "flex_allgather_local": [vp, pvp, vp, sz, ci, vp],
        "flex_reducescatter_local": [vp, pvp, vp, sz, ci, ci, vp],
        "flex_alltoall_local": [vp, pvp, vp, sz, ci, vp],
        "flex_allreduce_staged_noalloc": [pvp, ci, ci, vp, sz, ci, ci, u32, vp],
        "flex_set_split": [vp, ci, ci, u32],
        "flex_comm_tune": [vp, ci, pvp, vp, sz, ci, vp, P(TuneResult)],
        "flex_comm_set_shares": [vp, ci, sz, ci, P(u32)],
        "flex_comm_tune_trace": [vp, ci, sz, ci, P(TuneRound), u32, P(u32)],
        "flex_pipeline_plan": [u64, u64, u64, P(u64), u32, P(u32)],
        "flex_evaluator_poll": [vp],
        "flex_evaluator_drain": [vp],
        "flex_get_stats": [vp, ci, sz, ci, P(Stats)],
    }
    for name, argtypes in sigs.items():
        fn = getattr(L, name)
        fn.argtypes = argtypes
        fn.restype = ci
    L.flex_status_string.argtypes = [ci]
    L.flex_status_string.restype = ctypes.c_char_p
    L.flex_last_error.argtypes = []
    L.flex_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(status):
    if status != FLEX_OK:
        raise FlexError(status, lib().flex_last_error().decode())


def flex_status_string(status):
    return lib().flex_status_string(status).decode()


def flex_last_error():
    return lib().flex_last_error().decode()


# ------------------------------------------------------------------ balancer

def flex_balancer_cfg_default():
    cfg = BalancerCfg()
    _check(lib().flex_balancer_cfg_default(ctypes.byref(cfg)))
    return cfg


def _cfg_ref(cfg):
    return ctypes.byref(cfg) if cfg is not None else None


def flex_balancer_init(path_bw, cfg=None):
    h = ctypes.c_void_p()
    arr = (f64 * len(path_bw))(*path_bw)
    _check(lib().flex_balancer_init(ctypes.byref(h), len(path_bw), arr, _cfg_ref(cfg)))
    return h


def flex_balancer_init_shares(shares, cfg=None):
    h = ctypes.c_void_p()
    arr = (u32 * len(shares))(*shares)
    _check(lib().flex_balancer_init_shares(ctypes.byref(h), len(shares), arr, _cfg_ref(cfg)))
    return h


def flex_balancer_update(b, path_time_s):
    n = len(path_time_s)
    t = (f64 * n)(*path_time_s)
    s = (u32 * n)()
    _check(lib().flex_balancer_update(b, t, s))
    return list(s)


def flex_balancer_finish_tuning(b):
    _check(lib().flex_balancer_finish_tuning(b))


def flex_balancer_revert_to_primary(b):
    _check(lib().flex_balancer_revert_to_primary(b))


def flex_balancer_get(b):
    st = BalancerState()
    _check(lib().flex_balancer_get(b, ctypes.byref(st)))
    return st


def flex_balancer_destroy(b):
    _check(lib().flex_balancer_destroy(b))


def flex_struct_sizes():
    out = (ctypes.c_size_t * 6)()
    _check(lib().flex_struct_sizes(out))
    return list(out)


def flex_partition(count, host_units, share_total=10000, align_elems=2048, min_count=32768):
    out = u64()
    _check(lib().flex_partition(count, host_units, share_total, align_elems, min_count, ctypes.byref(out)))
    return out.value


# -------------------------------------------------------------- communicator

def flex_config_default():
    cfg = Config()
    _check(lib().flex_config_default(ctypes.byref(cfg)))
    return cfg


def dtype_code(dtype):
    if dtype == torch.float32:
        return FLEX_F32
    if dtype == torch.bfloat16:
        return FLEX_BF16
    if dtype == torch.float16:
        return FLEX_F16
    raise ValueError("unsupported dtype %r" % (dtype,))


def flex_comm_create(nranks, rank, max_bytes_per_rank, cfg=None):
    h = ctypes.c_void_p()
    _check(lib().flex_comm_create(ctypes.byref(h), nranks, rank, max_bytes_per_rank, _cfg_ref(cfg)))
    return h


def flex_comm_destroy(comm):
    _check(lib().flex_comm_destroy(comm))


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(stream)


def _pointer_array(tensors):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr() if isinstance(t, torch.Tensor) else int(t)
    return arr


def _marshal(coll, tensors, out, count, require_device=True):
    """Check the tensors of one collective call and return the array of rank
    pointers, in one pass (this runs on every call).  The C ABI takes plain
    pointers and trusts the count: a count beyond a tensor's end would make
    the kernels read or write outside it, so that is caught here."""
    n = len(tensors)
    need_in = count * (n if coll in (FLEX_REDUCESCATTER, FLEX_ALLTOALL) else 1)
    need_out = count * (n if coll in (FLEX_ALLGATHER, FLEX_ALLTOALL) else 1)
    dtype = out.dtype
    if (require_device and not out.is_cuda) or not out.is_contiguous():
        raise ValueError("tensors must be contiguous CUDA tensors")
    if count < 0 or out.numel() < need_out:
        raise ValueError("out holds %d elements, the call writes %d" % (out.numel(), need_out))
    arr = (ctypes.c_void_p * n)()
    r = 0
    for t in tensors:
        if (require_device and not t.is_cuda) or not t.is_contiguous():
            raise ValueError("tensors must be contiguous CUDA tensors")
        if t.dtype != dtype:
            raise ValueError("dtype mismatch")
        if t.numel() < need_in:
            raise ValueError("rank %d holds %d elements, the call reads %d" % (r, t.numel(), need_in))
        arr[r] = t.data_ptr()
        r += 1
    return arr


def flex_allreduce_local(comm, rank_bufs, out, count=None, op=FLEX_SUM, stream=None):
    """rank_bufs: list of device tensors (one per rank); out: device tensor."""
    count = rank_bufs[0].numel() if count is None else count
    _check(lib().flex_allreduce_local(comm, _marshal(FLEX_ALLREDUCE, rank_bufs, out, count), out.data_ptr(), count,
                                      dtype_code(out.dtype), op, _stream_handle(stream)))


def flex_allreduce_staged_noalloc(rank_bufs, rank, out, count=None, staged_units=0, op=FLEX_SUM, stream=None):
    """No communicator: the staged part goes through the library's built-in transit buffer."""
    count = rank_bufs[0].numel() if count is None else count
    _check(lib().flex_allreduce_staged_noalloc(_marshal(FLEX_ALLREDUCE, rank_bufs, out, count), len(rank_bufs), rank, out.data_ptr(), count,
                                               dtype_code(out.dtype), op, staged_units, _stream_handle(stream)))


def flex_reducescatter_local(comm, rank_bufs, out, recv_count=None, op=FLEX_SUM, stream=None):
    """rank_bufs: list of nranks device tensors of nranks * recv_count elements."""
    recv_count = rank_bufs[0].numel() // len(rank_bufs) if recv_count is None else recv_count
    _check(lib().flex_reducescatter_local(comm, _marshal(FLEX_REDUCESCATTER, rank_bufs, out, recv_count),
                                          out.data_ptr(), recv_count,
                                          dtype_code(out.dtype), op, _stream_handle(stream)))


def flex_allgather_local(comm, rank_slices, out, slice_count=None, stream=None):
    slice_count = rank_slices[0].numel() if slice_count is None else slice_count
    _check(lib().flex_allgather_local(comm, _marshal(FLEX_ALLGATHER, rank_slices, out, slice_count), out.data_ptr(),
                                      slice_count,
                                      dtype_code(out.dtype), _stream_handle(stream)))


def flex_alltoall_local(comm, rank_bufs, out, count=None, stream=None):
    """rank_bufs: list of nranks device tensors of nranks * count elements."""
    count = rank_bufs[0].numel() // len(rank_bufs) if count is None else count
    _check(lib().flex_alltoall_local(comm, _marshal(FLEX_ALLTOALL, rank_bufs, out, count), out.data_ptr(), count,
                                     dtype_code(out.dtype), _stream_handle(stream)))


def flex_set_split(comm, coll, mode, host_units=0):
    _check(lib().flex_set_split(comm, coll, mode, host_units))


def flex_comm_tune(comm, coll, rank_bufs, out, count=None, stream=None):
    if count is None:
        count = rank_bufs[0].numel() // (len(rank_bufs) if coll in (FLEX_REDUCESCATTER, FLEX_ALLTOALL) else 1)
    res = TuneResult()
    _check(lib().flex_comm_tune(comm, coll, _marshal(coll, rank_bufs, out, count), out.data_ptr(), count,
                                dtype_code(out.dtype), _stream_handle(stream), ctypes.byref(res)))
    return res


def flex_partition_paths(count, units, share_total=10000, align_elems=2048, min_count=32768):
    n = len(units)
    arr = (u32 * n)(*units)
    out = (u64 * (n + 1))()
    _check(lib().flex_partition_paths(count, arr, n, share_total, align_elems, min_count, out))
    return list(out)


def flex_set_split_paths(comm, coll, mode, aux_units=()):
    arr = (u32 * max(len(aux_units), 1))(*aux_units)
    _check(lib().flex_set_split_paths(comm, coll, mode, arr, len(aux_units)))


def flex_comm_set_shares(comm, coll, count, dtype, shares):
    arr = (u32 * FLEX_MAX_PATHS)(*shares)
    _check(lib().flex_comm_set_shares(comm, coll, count, dtype_code(dtype), arr))


def flex_comm_tune_trace(comm, coll, count, dtype, max_rounds=128):
    """The iterations of the last flex_comm_tune of that size class (list of TuneRound) and how many it ran."""
    arr = (TuneRound * max_rounds)()
    n = u32()
    _check(lib().flex_comm_tune_trace(comm, coll, count, dtype_code(dtype), arr, max_rounds, ctypes.byref(n)))
    return [arr[k] for k in range(min(n.value, max_rounds))], n.value


def flex_pipeline_plan(nbytes, chunk_bytes=4 << 20, min_step_bytes=256 << 10):
    n = u32()
    _check(lib().flex_pipeline_plan(nbytes, chunk_bytes, min_step_bytes, None, 0, ctypes.byref(n)))
    arr = (u64 * max(n.value, 1))()
    _check(lib().flex_pipeline_plan(nbytes, chunk_bytes, min_step_bytes, arr, n.value, ctypes.byref(n)))
    return list(arr)[:n.value]


def flex_evaluator_poll(comm):
    _check(lib().flex_evaluator_poll(comm))


def flex_evaluator_drain(comm):
    _check(lib().flex_evaluator_drain(comm))


def flex_get_stats(comm, coll, count, dtype):
    st = Stats()
    _check(lib().flex_get_stats(comm, coll, count, dtype_code(dtype), ctypes.byref(st)))
    return st
