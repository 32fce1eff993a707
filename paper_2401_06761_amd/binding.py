"""ctypes binding of include/apar.h.  Names and argument order follow the header."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libapar.so")

APAR_F32, APAR_BF16, APAR_BF16_FP8KV = 0, 1, 2


class AparError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        msg = f"{where}: {apar_status_string(status)} ({status})"
        if detail:
            msg += f": {detail}"
        super().__init__(msg)


class AparPoolConfig(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("dtype", C.c_int32), ("max_threads", C.c_int32),
                ("num_blocks", C.c_int64), ("softmax_scale", C.c_float)]


class AparStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("total_blocks", "used_blocks", "free_blocks", "live_threads",
                                         "threads_issued", "cow_copies", "block_bytes", "bytes_resident",
                                         "bytes_vanilla")]


class AparPlanInfo(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n_threads", "n_segments", "n_units", "n_partial_rows", "unique_blocks",
                                         "unique_tokens", "path_tokens", "algorithmic_bytes")]


class AparGroupStepInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_forked", "n_finished", "n_rows_appended", "n_unfinished")]


class AparGroupInfo(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n_sequences", "n_unfinished", "n_nodes", "steps", "prompt_tokens",
                                         "generated_tokens", "attended_tokens", "cached_tokens",
                                         "max_cached_tokens")]


APAR_TOKEN_FORK, APAR_TOKEN_CHILD, APAR_TOKEN_EOS = -1, -2, -3


class AparServerConfig(C.Structure):
    _fields_ = [("max_running", C.c_int32), ("watermark_blocks", C.c_int32)]


class AparServerSeq(C.Structure):
    _fields_ = [("request_id", C.c_int32), ("thread", C.c_int32), ("seq_index", C.c_int32), ("last_token", C.c_int32),
                ("length", C.c_int64), ("start_len", C.c_int64), ("group_size", C.c_int32), ("reserved", C.c_int32)]


class AparServerStepInfo(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_preempted", "n_forked", "n_finished_sequences", "n_finished_requests",
                                         "n_rows_appended", "n_running")]


class AparServerStats(C.Structure):
    _fields_ = [(k, C.c_int64) for k in ("steps", "n_submitted", "n_waiting", "n_running", "n_finished",
                                         "n_admissions", "n_preemptions", "generated_tokens",
                                         "batch_sequences_total", "peak_used_blocks", "peak_running", "peak_threads")]


class AparProfile(C.Structure):
    _fields_ = [("n_decode_calls", C.c_int64), ("attention_kernel_ms", C.c_double), ("merge_kernel_ms", C.c_double),
                ("plan_host_ms", C.c_double), ("n_append_calls", C.c_int64), ("append_kernels_ms", C.c_double),
                ("host_wait_ms", C.c_double)]


def library_path() -> str:
    return _LIB_PATH


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(or python paper_2401_06761_amd/build.py).  There is no fallback path.")
    # PyTorch ships its own HIP runtime.  Import it first so that libapar binds to that
    # copy (the loader matches it by soname); two runtimes in one process do not share devices.
    import torch  # noqa: F401

    lib = C.CDLL(_LIB_PATH)
    P, I, V = C.c_void_p, C.c_int, C.c_void_p
    I32P = C.POINTER(C.c_int32)
    sig = {
        "apar_pool_create": [C.POINTER(AparPoolConfig), V, C.c_size_t, C.POINTER(P)],
        "apar_pool_destroy": [P],
        "apar_thread_create": [P, I32P],
        "apar_fork": [P, C.c_int32, I, I32P],
        "apar_append_kv": [P, C.c_int32, V, V, I, V],
        "apar_append_kv_batch": [P, I32P, I, V, V, V],
        "apar_decode_attention": [P, V, I32P, I, V, V],
        "apar_decode_attention_fixed": [P, V, I32P, I, V, V],
        "apar_decode_attention_spec": [P, V, V, V, V, I, I32P, I, V, V],
        "apar_commit_candidates": [P, I32P, I, V, V, I, C.POINTER(C.c_uint8), V],
        "apar_prefill_attention": [P, V, I32P, I32P, I, V, V],
        "apar_free_thread": [P, C.c_int32],
        "apar_thread_len": [P, C.c_int32, C.POINTER(C.c_int64)],
        "apar_thread_block_table": [P, C.c_int32, I32P, I, C.POINTER(C.c_int)],
        "apar_block_refcount": [P, C.c_int32, I32P],
        "apar_pool_stats": [P, C.POINTER(AparStats)],
        "apar_last_plan_info": [P, C.POINTER(AparPlanInfo)],
        "apar_read_kv_rows": [P, C.c_int32, C.c_int64, I, V, V, V],
        "apar_last_plan_export": [P, I, I32P, C.c_int64, C.POINTER(C.c_int64)],
        "apar_profile_enable": [P, I],
        "apar_profile_read": [P, C.POINTER(AparProfile)],
        "apar_profile_attention_calls": [P, C.POINTER(C.c_float), C.c_int64, C.POINTER(C.c_int64)],
        "apar_set_chunk_blocks": [P, I],
        "apar_set_prefill_kernel": [P, I],
        "apar_set_matrix_units": [P, I, I],
        "apar_set_inline_shared": [P, I],
        "apar_set_write_checks": [P, I],
        "apar_set_plan_reuse": [P, I],
        "apar_plan_counts": [P, C.POINTER(C.c_int64), C.POINTER(C.c_int64)],
        "apar_last_prefill_kernel": [P],
        "apar_append_kv_gather": [P, I32P, I32P, I, V, V, V],
        "apar_server_create": [P, C.POINTER(AparServerConfig), C.POINTER(P)],
        "apar_server_destroy": [P],
        "apar_server_submit": [P, C.c_int32, I32P, I],
        "apar_server_admit": [P, V, V, C.c_int64, V, C.POINTER(C.c_int32), C.POINTER(C.c_int64)],
        "apar_server_batch": [P, C.POINTER(AparServerSeq), I, C.POINTER(C.c_int)],
        "apar_server_step": [P, I32P, I, V, V, V, C.POINTER(AparServerStepInfo)],
        "apar_server_pop_finished": [P, C.POINTER(C.c_int32), I32P, C.c_int64, C.POINTER(C.c_int64),
                                     C.POINTER(AparGroupInfo)],
        "apar_server_get_stats": [P, C.POINTER(AparServerStats)],
        "apar_group_create": [P, I32P, I, V, V, V, C.POINTER(P)],
        "apar_group_destroy": [P],
        "apar_group_unfinished": [P, I32P, I, C.POINTER(C.c_int)],
        "apar_group_step": [P, I32P, I, V, V, V, C.POINTER(AparGroupStepInfo)],
        "apar_group_restore": [P, I32P, C.c_int64, C.POINTER(C.c_int64)],
        "apar_group_get_info": [P, C.POINTER(AparGroupInfo)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.apar_plan_record_version.argtypes = []
    lib.apar_plan_record_version.restype = C.c_int
    lib.apar_status_string.argtypes = [C.c_int]
    lib.apar_status_string.restype = C.c_char_p
    lib.apar_last_hip_error.argtypes = []
    lib.apar_last_hip_error.restype = C.c_char_p
    return lib


_lib: Optional[C.CDLL] = None


def _L() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = _load()
    return _lib


def exported_symbols() -> List[str]:
    """Names the loaded library resolves, out of those apar.h declares."""
    import re

    hdr = open(os.path.join(os.path.dirname(_HERE), "include", "apar.h")).read()
    names = re.findall(r"\b(apar_[a-z_0-9]+)\s*\(", hdr)
    lib = _L()
    return [n for n in dict.fromkeys(names) if hasattr(lib, n)]


def apar_status_string(status: int) -> str:
    return _L().apar_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        detail = _L().apar_last_hip_error().decode() if status == -5 else ""
        raise AparError(status, where, detail)


def _ids(seq):
    """Host array of thread ids as int32*; numpy int32 arrays are passed without a copy."""
    import numpy as np

    arr = np.ascontiguousarray(seq, dtype=np.int32)
    if arr.ndim != 1:
        raise ValueError("thread ids must be a 1-d sequence")
    ptr = arr.ctypes.data_as(C.POINTER(C.c_int32))
    ptr._keepalive = arr  # the array must outlive the call
    return ptr, int(arr.shape[0])


def _ptr(t) -> int:
    """Device pointer of a torch tensor (must be contiguous and on the GPU)."""
    if t is None:
        return 0
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return t.data_ptr()


_HAVE_GPU = None  # torch.cuda.is_available(), asked once


def _stream(stream) -> int:
    global _HAVE_GPU
    if stream is None:
        import torch

        if _HAVE_GPU is None:
            _HAVE_GPU = bool(torch.cuda.is_available())
        if not _HAVE_GPU:
            return 0  # only dry-run pools can be used without a GPU; they ignore the stream
        return torch.cuda.current_stream().cuda_stream
    return int(getattr(stream, "cuda_stream", stream))


def apar_pool_create(cfg: AparPoolConfig, kv_dev, kv_bytes: Optional[int] = None) -> C.c_void_p:
    """kv_dev: a GPU tensor, a raw device address, or None for a dry-run (bookkeeping-only) pool."""
    if kv_dev is None:
        ptr, kv_bytes = 0, 0
    else:
        ptr = kv_dev if isinstance(kv_dev, int) else _ptr(kv_dev)
        if kv_bytes is None:
            kv_bytes = kv_dev.numel() * kv_dev.element_size()
    out = C.c_void_p()
    _check(_L().apar_pool_create(C.byref(cfg), ptr, kv_bytes, C.byref(out)), "apar_pool_create")
    return out


def apar_pool_destroy(pool) -> None:
    _check(_L().apar_pool_destroy(pool), "apar_pool_destroy")


def apar_thread_create(pool) -> int:
    out = C.c_int32()
    _check(_L().apar_thread_create(pool, C.byref(out)), "apar_thread_create")
    return out.value


def apar_fork(pool, parent: int, n_children: int) -> List[int]:
    out = (C.c_int32 * max(n_children, 1))()
    _check(_L().apar_fork(pool, parent, n_children, out), "apar_fork")
    return list(out[:n_children])


def apar_append_kv(pool, thread: int, k, v, n_tokens: Optional[int] = None, stream=None) -> None:
    if n_tokens is None:
        n_tokens = k.shape[0]
    _check(_L().apar_append_kv(pool, thread, _ptr(k), _ptr(v), n_tokens, _stream(stream)), "apar_append_kv")


def apar_append_kv_batch(pool, threads: Sequence[int], k, v, stream=None) -> None:
    arr, n = _ids(threads)
    _check(_L().apar_append_kv_batch(pool, arr, n, _ptr(k), _ptr(v), _stream(stream)), "apar_append_kv_batch")


def apar_decode_attention(pool, q, threads: Sequence[int], out, stream=None) -> None:
    arr, n = _ids(threads)
    _check(_L().apar_decode_attention(pool, _ptr(q), arr, n, _ptr(out), _stream(stream)), "apar_decode_attention")


def apar_decode_attention_fixed(pool, q, threads: Sequence[int], out, stream=None) -> None:
    arr, n = _ids(threads)
    _check(_L().apar_decode_attention_fixed(pool, _ptr(q), arr, n, _ptr(out), _stream(stream)),
           "apar_decode_attention_fixed")


def apar_decode_attention_spec(pool, q, cand_k, cand_v, mask, n_cand: int, threads: Sequence[int], out,
                               stream=None) -> None:
    arr, n = _ids(threads)
    _check(_L().apar_decode_attention_spec(pool, _ptr(q), _ptr(cand_k), _ptr(cand_v), _ptr(mask), n_cand, arr, n,
                                           _ptr(out), _stream(stream)), "apar_decode_attention_spec")


def apar_commit_candidates(pool, threads: Sequence[int], cand_k, cand_v, n_cand: int, accept_masks, stream=None) -> None:
    """accept_masks: one byte per listed thread (host), bit c set iff candidate c is accepted."""
    import numpy as np

    arr, n = _ids(threads)
    masks = np.ascontiguousarray(accept_masks, dtype=np.uint8)
    if masks.shape != (n,):
        raise ValueError("accept_masks must hold one byte per listed thread")
    _check(_L().apar_commit_candidates(pool, arr, n, _ptr(cand_k), _ptr(cand_v), n_cand,
                                       masks.ctypes.data_as(C.POINTER(C.c_uint8)), _stream(stream)),
           "apar_commit_candidates")


def apar_prefill_attention(pool, q, threads: Sequence[int], m: Sequence[int], out, stream=None) -> None:
    arr, n = _ids(threads)
    marr, nm = _ids(m)
    if nm != n:
        raise ValueError("one m per listed thread")
    _check(_L().apar_prefill_attention(pool, _ptr(q), arr, marr, n, _ptr(out), _stream(stream)),
           "apar_prefill_attention")


def apar_free_thread(pool, thread: int) -> None:
    _check(_L().apar_free_thread(pool, thread), "apar_free_thread")


def apar_thread_len(pool, thread: int) -> int:
    out = C.c_int64()
    _check(_L().apar_thread_len(pool, thread, C.byref(out)), "apar_thread_len")
    return out.value


def apar_thread_block_table(pool, thread: int) -> List[int]:
    n = C.c_int()
    st = _L().apar_thread_block_table(pool, thread, None, 0, C.byref(n))
    if st not in (0, -1):
        _check(st, "apar_thread_block_table")
    if st == -1 and n.value == 0:
        _check(st, "apar_thread_block_table")
    buf = (C.c_int32 * max(n.value, 1))()
    _check(_L().apar_thread_block_table(pool, thread, buf, n.value, C.byref(n)), "apar_thread_block_table")
    return list(buf[: n.value])


def apar_block_refcount(pool, block: int) -> int:
    out = C.c_int32()
    _check(_L().apar_block_refcount(pool, block, C.byref(out)), "apar_block_refcount")
    return out.value


def apar_pool_stats(pool) -> AparStats:
    out = AparStats()
    _check(_L().apar_pool_stats(pool, C.byref(out)), "apar_pool_stats")
    return out


def apar_last_plan_info(pool) -> AparPlanInfo:
    out = AparPlanInfo()
    _check(_L().apar_last_plan_info(pool, C.byref(out)), "apar_last_plan_info")
    return out


(APAR_PLAN_WORKGROUPS, APAR_PLAN_TILES, APAR_PLAN_DFS_THREADS, APAR_PLAN_PATH_OFS, APAR_PLAN_PATH_IDS,
 APAR_PLAN_GEOMETRY, APAR_PLAN_CHANGED_WORKGROUP_WORDS, APAR_PLAN_CHANGED_TILE_WORDS) = range(8)


def apar_last_plan_export(pool, which: int) -> List[int]:
    if apar_plan_record_version() != APAR_PLAN_RECORD_VERSION:
        raise RuntimeError("the library's plan tables have another layout than this binding reads")
    n = C.c_int64()
    _L().apar_last_plan_export(pool, which, None, 0, C.byref(n))
    buf = (C.c_int32 * max(n.value, 1))()
    _check(_L().apar_last_plan_export(pool, which, buf, n.value, C.byref(n)), "apar_last_plan_export")
    return list(buf[: n.value])


def apar_read_kv_rows(pool, thread: int, first: int, n: int, k_out, v_out, stream=None) -> None:
    _check(_L().apar_read_kv_rows(pool, thread, first, n, _ptr(k_out), _ptr(v_out), _stream(stream)),
           "apar_read_kv_rows")


def apar_profile_enable(pool, on: bool) -> None:
    _check(_L().apar_profile_enable(pool, int(bool(on))), "apar_profile_enable")


def apar_profile_read(pool) -> AparProfile:
    out = AparProfile()
    _check(_L().apar_profile_read(pool, C.byref(out)), "apar_profile_read")
    return out


def apar_profile_attention_calls(pool) -> List[float]:
    n = C.c_int64()
    _L().apar_profile_attention_calls(pool, None, 0, C.byref(n))
    buf = (C.c_float * max(n.value, 1))()
    _check(_L().apar_profile_attention_calls(pool, buf, n.value, C.byref(n)), "apar_profile_attention_calls")
    return list(buf[: n.value])


def apar_set_chunk_blocks(pool, blocks_per_unit: int) -> None:
    _check(_L().apar_set_chunk_blocks(pool, blocks_per_unit), "apar_set_chunk_blocks")


APAR_PREFILL_AUTO, APAR_PREFILL_ROW_TILES, APAR_PREFILL_MATRIX = 0, 1, 2


def apar_set_inline_shared(pool, on: bool) -> None:
    _check(_L().apar_set_inline_shared(pool, 1 if on else 0), "apar_set_inline_shared")


def apar_set_write_checks(pool, on: bool) -> None:
    _check(_L().apar_set_write_checks(pool, 1 if on else 0), "apar_set_write_checks")


def apar_set_plan_reuse(pool, on: bool) -> None:
    _check(_L().apar_set_plan_reuse(pool, 1 if on else 0), "apar_set_plan_reuse")


def apar_plan_counts(pool) -> Tuple[int, int]:
    """(decode calls that built their plan, decode calls that carried the previous one over)."""
    built, carried = C.c_int64(0), C.c_int64(0)
    _check(_L().apar_plan_counts(pool, C.byref(built), C.byref(carried)), "apar_plan_counts")
    return int(built.value), int(carried.value)


APAR_PLAN_RECORD_VERSION = 2  # the layout apar_last_plan_export's readers here were written for


def apar_plan_record_version() -> int:
    return int(_L().apar_plan_record_version())


def apar_set_matrix_units(pool, min_rows: int, min_blocks: int) -> None:
    _check(_L().apar_set_matrix_units(pool, min_rows, min_blocks), "apar_set_matrix_units")


def apar_set_prefill_kernel(pool, which: int) -> None:
    _check(_L().apar_set_prefill_kernel(pool, which), "apar_set_prefill_kernel")


def apar_last_prefill_kernel(pool) -> int:
    return int(_L().apar_last_prefill_kernel(pool))


def apar_group_create(pool, prompt_tokens: Sequence[int], k, v, stream=None) -> C.c_void_p:
    arr, n = _ids(prompt_tokens)
    out = C.c_void_p()
    _check(_L().apar_group_create(pool, arr, n, _ptr(k), _ptr(v), _stream(stream), C.byref(out)), "apar_group_create")
    return out


def apar_group_destroy(group) -> None:
    _check(_L().apar_group_destroy(group), "apar_group_destroy")


def apar_group_unfinished(group) -> List[int]:
    n = C.c_int()
    _L().apar_group_unfinished(group, None, 0, C.byref(n))
    buf = (C.c_int32 * max(n.value, 1))()
    _check(_L().apar_group_unfinished(group, buf, n.value, C.byref(n)), "apar_group_unfinished")
    return list(buf[: n.value])


def apar_group_step(group, sampled: Sequence[int], k, v, stream=None) -> AparGroupStepInfo:
    arr, n = _ids(sampled)
    info = AparGroupStepInfo()
    _check(_L().apar_group_step(group, arr, n, _ptr(k), _ptr(v), _stream(stream), C.byref(info)), "apar_group_step")
    return info


def apar_group_restore(group) -> List[int]:
    n = C.c_int64()
    _L().apar_group_restore(group, None, 0, C.byref(n))
    buf = (C.c_int32 * max(n.value, 1))()
    _check(_L().apar_group_restore(group, buf, n.value, C.byref(n)), "apar_group_restore")
    return list(buf[: n.value])


def apar_group_get_info(group) -> AparGroupInfo:
    out = AparGroupInfo()
    _check(_L().apar_group_get_info(group, C.byref(out)), "apar_group_get_info")
    return out


def apar_append_kv_gather(pool, threads: Sequence[int], src_rows: Sequence[int], k, v, stream=None) -> None:
    arr, n = _ids(threads)
    src, ns = _ids(src_rows)
    if ns != n:
        raise ValueError("one source row per listed thread")
    _check(_L().apar_append_kv_gather(pool, arr, src, n, _ptr(k), _ptr(v), _stream(stream)), "apar_append_kv_gather")


def apar_server_create(pool, max_running: int, watermark_blocks: int) -> C.c_void_p:
    cfg = AparServerConfig(max_running, watermark_blocks)
    out = C.c_void_p()
    _check(_L().apar_server_create(pool, C.byref(cfg), C.byref(out)), "apar_server_create")
    return out


def apar_server_destroy(server) -> None:
    _check(_L().apar_server_destroy(server), "apar_server_destroy")


def apar_server_submit(server, request_id: int, prompt_tokens: Sequence[int]) -> None:
    arr, n = _ids(prompt_tokens)
    _check(_L().apar_server_submit(server, request_id, arr, n), "apar_server_submit")


def apar_server_admit(server, k, v, rows_available: int, stream=None):
    """Returns (requests admitted, prompt rows consumed from k, v)."""
    n, used = C.c_int32(), C.c_int64()
    _check(_L().apar_server_admit(server, _ptr(k), _ptr(v), rows_available, _stream(stream), C.byref(n), C.byref(used)),
           "apar_server_admit")
    return n.value, used.value


def apar_server_batch(server):
    """The batch as a numpy structured array (fields as apar_server_seq)."""
    import numpy as np

    n = C.c_int()
    _L().apar_server_batch(server, None, 0, C.byref(n))
    buf = (AparServerSeq * max(n.value, 1))()
    _check(_L().apar_server_batch(server, buf, n.value, C.byref(n)), "apar_server_batch")
    dt = np.dtype([("request_id", "<i4"), ("thread", "<i4"), ("seq_index", "<i4"), ("last_token", "<i4"),
                   ("length", "<i8"), ("start_len", "<i8"), ("group_size", "<i4"), ("reserved", "<i4")])
    return np.frombuffer(buf, dtype=dt, count=n.value).copy()


def apar_server_step(server, sampled, k, v, stream=None) -> AparServerStepInfo:
    arr, n = _ids(sampled)
    info = AparServerStepInfo()
    _check(_L().apar_server_step(server, arr, n, _ptr(k), _ptr(v), _stream(stream), C.byref(info)), "apar_server_step")
    return info


def apar_server_pop_finished(server):
    """(request id, tokens in Restore order, AparGroupInfo) of the oldest completed request, or None."""
    rid, n = C.c_int32(), C.c_int64()
    rc = _L().apar_server_pop_finished(server, C.byref(rid), None, 0, C.byref(n), None)
    if rid.value < 0:
        _check(rc, "apar_server_pop_finished")
        return None
    buf = (C.c_int32 * max(n.value, 1))()
    info = AparGroupInfo()
    _check(_L().apar_server_pop_finished(server, C.byref(rid), buf, n.value, C.byref(n), C.byref(info)),
           "apar_server_pop_finished")
    return rid.value, list(buf[: n.value]), info


def apar_server_get_stats(server) -> AparServerStats:
    out = AparServerStats()
    _check(_L().apar_server_get_stats(server, C.byref(out)), "apar_server_get_stats")
    return out


class Pool:
    """Owns the KV buffer (a torch tensor: device memory is PyTorch's job here) and the handle."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str, num_blocks: int,
                 max_threads: int = 1 << 20, softmax_scale: float = 0.0, device: str = "cuda:0",
                 dry_run: bool = False):
        import torch

        # "bf16_fp8kv": bf16 at the interface, full blocks cached in fp8 (APAR_BF16_FP8KV)
        self.torch_dtype = {"f32": torch.float32, "bf16": torch.bfloat16, "bf16_fp8kv": torch.bfloat16}[dtype]
        e = 4 if dtype == "f32" else 2
        self.block_bytes = 2 * n_kv_heads * 16 * head_dim * e
        self.kv = None if dry_run else torch.empty(num_blocks * self.block_bytes, dtype=torch.uint8, device=device)
        self.cfg = AparPoolConfig(n_q_heads, n_kv_heads, head_dim, 16,
                                  {"f32": APAR_F32, "bf16": APAR_BF16, "bf16_fp8kv": APAR_BF16_FP8KV}[dtype],
                                  max_threads, num_blocks, softmax_scale)
        self.n_q, self.n_kv, self.d = n_q_heads, n_kv_heads, head_dim
        self.device = device
        self.handle = apar_pool_create(self.cfg, self.kv)

    def close(self) -> None:
        if self.handle is not None:
            apar_pool_destroy(self.handle)
            self.handle = None
            self.kv = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
