"""ctypes binding of include/ha_rag.h: same names, argument marshalling only.

Device and pinned buffers are torch tensors (or raw integer addresses); this
module passes their addresses through and never computes on them.  If the built
library is missing the import of this module still works, but the first call
raises: there is no CPU fallback.
"""
import ctypes as C
import os

from . import build as _build

OK, EINVAL, ENOENT, ENOSPC, EFORMAT, EHIP, EIO = 0, -1, -2, -3, -4, -5, -6
PREC_16, PREC_INT8, PREC_INT4, PREC_FP8_E4M3, PREC_FP8_E5M2, PREC_GSE8 = 0, 1, 2, 3, 4, 5
TIER_HBM, TIER_PINNED, TIER_PAGEABLE, TIER_DISK, TIER_NONE = 0, 1, 2, 3, 255
PART_KV, PART_K, PART_V = 0, 1, 2
NO_CHUNK = 2**64 - 1
ATTEND_COUNT = 1
ATTEND_STATIC_SCRATCH_BYTES, ATTEND_STATIC_MAX_REQUESTS, ATTEND_STATIC_MAX_DOCS = 32 << 20, 64, 416
PLACE_DEVICE_VISIBLE = 1
BITS = {PREC_16: 16, PREC_INT8: 8, PREC_INT4: 4, PREC_FP8_E4M3: 8, PREC_FP8_E5M2: 8,
        PREC_GSE8: 8}  # storage bits
PREC_OF_BITS = {16: PREC_16, 8: PREC_INT8, 4: PREC_INT4}

# every function include/ha_rag.h declares
SYMBOLS = [
    "ha_rag_chunk_bytes", "ha_rag_alg1_classes", "ha_rag_strerror", "ha_rag_version",
    "ha_rag_create", "ha_rag_destroy", "ha_rag_last_hip_error", "ha_rag_set_launch_params",
    "ha_rag_quantize_chunk", "ha_rag_load_packed", "ha_rag_register_slab",
    "ha_rag_register_staging", "ha_rag_pool_insert", "ha_rag_pool_slot", "ha_rag_pool_promote",
    "ha_rag_pool_evict", "ha_rag_pool_query", "ha_rag_touch",
    "ha_rag_set_counts", "ha_rag_rerank", "ha_rag_get_rank", "ha_rag_load_chunks",
    "ha_rag_load_batch", "ha_rag_register_disk", "ha_rag_register_bounce", "ha_rag_pool_lru",
    "ha_rag_quantize_half", "ha_rag_pool_insert_half", "ha_rag_load_packed_paged",
    "ha_rag_load_chunks_paged", "ha_rag_chunk_sq_error", "ha_rag_pool_save_index",
    "ha_rag_pool_load_index", "ha_rag_pool_remove", "ha_rag_attend_packed",
    "ha_rag_attend_workspace_bytes", "ha_rag_attend_chunks", "ha_rag_attend_chunks_workspace_bytes",
    "ha_rag_place_chunks", "ha_rag_attend_packed_static", "ha_rag_register_external",
    "ha_rag_pool_insert_external", "ha_rag_pool_repoint_external", "ha_rag_forget_stream",
    "ha_rag_quantize_chunks",
]


class Config(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in (
        "n_layers", "n_kv_heads", "head_dim", "max_chunk_tokens", "group_int8", "group_int4",
        "tau_gpu_ppm", "rerank_interval", "n_copy_streams", "dry_run", "tau_pin_ppm",
        "tau_page_ppm", "disk_o_direct", "half_slots", "pinned_dma", "io_threads")]


class LaunchParams(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in (
        "threads", "planes16", "planes8", "nt_store", "nt_load")]


class PackedChunk(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("n_tokens", C.c_uint32), ("prec", C.c_uint32),
                ("group", C.c_uint32), ("part", C.c_uint32)]


class AttendRequest(C.Structure):
    _fields_ = [("q", C.c_void_p), ("out", C.c_void_p), ("lse", C.c_void_p), ("n_q", C.c_uint32),
                ("n_chunks", C.c_uint32)]


class PagedCache(C.Structure):
    _fields_ = [("base", C.c_void_p), ("page_table", C.c_void_p), ("bad_pages", C.c_void_p),
                ("page_stride", C.c_uint64), ("tile_stride", C.c_uint64),
                ("page_tokens", C.c_uint32), ("n_table", C.c_uint32), ("n_pages", C.c_uint32),
                ("reserved", C.c_uint32)]


class ChunkInfo(C.Structure):
    _fields_ = [("prec", C.c_uint32), ("group", C.c_uint32), ("n_tokens", C.c_uint32),
                ("in_hbm", C.c_uint32), ("in_pinned", C.c_uint32), ("rank", C.c_uint32),
                ("in_pageable", C.c_uint32), ("on_disk", C.c_uint32),
                ("part", C.c_uint32), ("disk_slot", C.c_uint32), ("count", C.c_uint64), ("bytes", C.c_uint64),
                ("hbm_ptr", C.c_void_p), ("pinned_ptr", C.c_void_p)]


class ChunkTrace(C.Structure):
    _fields_ = [("tok_off", C.c_uint64), ("evicted_id", C.c_uint64), ("found_tier", C.c_uint8),
                ("promoted", C.c_uint8), ("promote_skipped", C.c_uint8),
                ("placed_tier", C.c_uint8), ("reserved", C.c_uint8 * 4)]


class LoadStats(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in (
        "n_chunks", "n_hbm_hits", "n_pinned_hits", "n_promoted", "n_evicted",
        "n_promote_skipped", "n_kernel_launches", "n_pageable_hits", "n_disk_hits",
        "n_placed_host")] + [("reserved", C.c_uint32 * 2)] + [(n, C.c_uint64) for n in (
            "tokens", "bytes_h2d", "bytes_d2d", "packed_bytes_read", "bf16_bytes_written",
            "bytes_disk_read", "bytes_host_copied")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if not n.startswith("reserved")}


class HaRagError(RuntimeError):
    def __init__(self, code, where, detail=""):
        self.code = code
        msg = f"{where}: {strerror(code)} ({code})"
        if detail:
            msg += f" [{detail}]"
        super().__init__(msg)


_lib = None


def lib_path():
    return _build.LIB


def lib():
    """Loads lib/libha_rag.so.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build it first (python -m paper_2510_20878_amd.build or "
                "__graft_entry__.build()); there is no fallback path")
        # PyTorch ships its own HIP runtime.  Device memory and streams come from
        # torch, so the library must bind to that same runtime: import torch first,
        # then the loader resolves libamdhip64 to the copy torch already mapped.
        import torch  # noqa: F401
        L = C.CDLL(path)
        vp, u32, u64, sz = C.c_void_p, C.c_uint32, C.c_uint64, C.c_size_t
        P = C.POINTER
        sig = {
            "ha_rag_chunk_bytes": (C.c_int, [u32] * 6 + [P(sz)] * 3),
            "ha_rag_alg1_classes": (C.c_int, [P(u64), sz, P(u32), u32, P(C.c_uint8), P(u32)]),
            "ha_rag_strerror": (C.c_char_p, [C.c_int]),
            "ha_rag_version": (C.c_char_p, []),
            "ha_rag_create": (C.c_int, [P(Config), P(vp)]),
            "ha_rag_destroy": (C.c_int, [vp]),
            "ha_rag_last_hip_error": (C.c_char_p, [vp]),
            "ha_rag_set_launch_params": (C.c_int, [vp, P(LaunchParams)]),
            "ha_rag_quantize_chunk": (C.c_int, [vp, vp, u32, u32, u32, vp, vp, vp]),
            "ha_rag_quantize_half": (C.c_int, [vp, vp, u32, u32, u32, vp, vp, vp]),
            "ha_rag_quantize_chunks": (C.c_int, [vp, P(vp), P(vp), P(u32), u32, u32, u32, vp, vp]),
            "ha_rag_pool_insert_half": (C.c_int, [vp, u64, u32, u32, u32, vp, C.c_int, u32, vp]),
            "ha_rag_load_packed": (C.c_int, [vp, P(PackedChunk), u32, vp, u64, u64, vp]),
            "ha_rag_chunk_sq_error": (C.c_int, [vp, vp, vp, u32, u32, u32, u32, vp, vp]),
            "ha_rag_load_packed_paged": (C.c_int, [vp, P(PackedChunk), u32, P(PagedCache), u64, vp]),
            "ha_rag_attend_packed": (C.c_int, [vp, P(PackedChunk), P(AttendRequest), u32, u32, u32,
                                               C.c_float, vp, C.c_size_t, vp]),
            "ha_rag_attend_packed_static": (C.c_int, [vp, P(PackedChunk), P(AttendRequest), u32, u32,
                                                      u32, C.c_float, vp]),
            "ha_rag_attend_workspace_bytes": (C.c_int, [vp, P(PackedChunk), P(AttendRequest), u32, u32,
                                                        P(C.c_size_t)]),
            "ha_rag_attend_chunks": (C.c_int, [vp, P(u64), P(AttendRequest), u32, u32, u32, C.c_float,
                                               u32, vp, C.c_size_t, vp]),
            "ha_rag_attend_chunks_workspace_bytes": (C.c_int, [vp, P(u64), P(AttendRequest), u32, u32,
                                                               P(C.c_size_t)]),
            "ha_rag_load_chunks_paged": (C.c_int, [vp, P(u64), P(C.c_uint8), u32, P(PagedCache), u64, vp,
                                                   P(LoadStats), P(ChunkTrace)]),
            "ha_rag_register_slab": (C.c_int, [vp, u32, u32, vp, sz]),
            "ha_rag_register_staging": (C.c_int, [vp, vp, sz]),
            "ha_rag_register_bounce": (C.c_int, [vp, vp, sz]),
            "ha_rag_register_disk": (C.c_int, [vp, u32, C.c_char_p, sz]),
            "ha_rag_pool_save_index": (C.c_int, [vp, C.c_char_p]),
            "ha_rag_pool_load_index": (C.c_int, [vp, C.c_char_p, P(sz)]),
            "ha_rag_pool_lru": (C.c_int, [vp, u32, P(u64), sz, P(sz)]),
            "ha_rag_pool_insert": (C.c_int, [vp, u64, u32, u32, vp, C.c_int, u32, vp]),
            "ha_rag_pool_slot": (C.c_int, [vp, u64, u32, P(vp), P(sz)]),
            "ha_rag_pool_promote": (C.c_int, [vp, u64, vp]),
            "ha_rag_pool_evict": (C.c_int, [vp, u64, u32]),
            "ha_rag_pool_remove": (C.c_int, [vp, u64]),
            "ha_rag_pool_query": (C.c_int, [vp, u64, P(ChunkInfo)]),
            "ha_rag_forget_stream": (C.c_int, [vp, vp]),
            "ha_rag_register_external": (C.c_int, [vp, u32]),
            "ha_rag_pool_insert_external": (C.c_int, [vp, u64, u32, u32, u32, vp]),
            "ha_rag_pool_repoint_external": (C.c_int, [vp, P(u64), P(vp), sz]),
            "ha_rag_touch": (C.c_int, [vp, P(u64), sz]),
            "ha_rag_set_counts": (C.c_int, [vp, P(u64), P(u64), sz]),
            "ha_rag_rerank": (C.c_int, [vp]),
            "ha_rag_get_rank": (C.c_int, [vp, u64, P(u32)]),
            "ha_rag_place_chunks": (C.c_int, [vp, P(u64), P(C.c_uint8), u32, u32, vp, P(LoadStats),
                                              P(ChunkTrace)]),
            "ha_rag_load_chunks": (C.c_int, [vp, P(u64), P(C.c_uint8), u32, vp, u64, u64, vp,
                                             P(LoadStats), P(ChunkTrace)]),
            "ha_rag_load_batch": (C.c_int, [vp, P(u64), P(C.c_uint8), P(u32), u32, P(vp), P(u64),
                                            P(u64), vp, P(LoadStats), P(ChunkTrace)]),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def paged_cache(base, page_table, page_tokens, n_pages, layout, n_layers, n_kv_heads, head_dim,
                bad_pages=None, n_table=None):
    """A PagedCache for one of the two pool layouts the header describes: "page_major"
    (every page one [L][2][H][P][D] block) or "tile_major" ([L][2][H][n_pages][P][D])."""
    row = head_dim * 2
    if layout == "page_major":
        tile_stride = page_tokens * row
        page_stride = 2 * n_layers * n_kv_heads * tile_stride
    elif layout == "tile_major":
        page_stride = page_tokens * row
        tile_stride = n_pages * page_stride
    else:
        raise ValueError(layout)
    if n_table is None:
        n_table = page_table.numel() if hasattr(page_table, "numel") else len(page_table)
    return PagedCache(_addr(base), _addr(page_table), _addr(bad_pages), page_stride, tile_stride,
                      page_tokens, n_table, n_pages, 0)


def strerror(code):
    return lib().ha_rag_strerror(code).decode()


def version():
    return lib().ha_rag_version().decode()


def _addr(x):
    """Address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(type(x))


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream  # torch.cuda.Stream


def _u64s(ids):
    return (C.c_uint64 * len(ids))(*[int(i) for i in ids])


def ha_rag_chunk_bytes(L, H, D, prec, group, n_tokens):
    """Returns (payload, meta, total) bytes."""
    p, m, t = C.c_size_t(), C.c_size_t(), C.c_size_t()
    rc = lib().ha_rag_chunk_bytes(L, H, D, prec, group, n_tokens, C.byref(p), C.byref(m), C.byref(t))
    if rc:
        raise HaRagError(rc, "ha_rag_chunk_bytes")
    return p.value, m.value, t.value


def ha_rag_alg1_classes(af, tau_ppm):
    """Returns (classes, ranks) lists."""
    n = len(af)
    a = _u64s(af)
    t = (C.c_uint32 * len(tau_ppm))(*tau_ppm)
    cls = (C.c_uint8 * max(n, 1))()
    rk = (C.c_uint32 * max(n, 1))()
    rc = lib().ha_rag_alg1_classes(a, n, t, len(tau_ppm), cls, rk)
    if rc:
        raise HaRagError(rc, "ha_rag_alg1_classes")
    return list(cls[:n]), list(rk[:n])


class Context:
    """Owns one ha_rag_ctx.  Methods carry the C names without the prefix."""

    def __init__(self, n_layers, n_kv_heads, head_dim, max_chunk_tokens, group_int8=128,
                 group_int4=128, tau_gpu_ppm=50_000, rerank_interval=0, n_copy_streams=0,
                 dry_run=False, tau_pin_ppm=0, tau_page_ppm=0, disk_o_direct=False,
                 half_slots=False, pinned_dma=False, io_threads=0):
        self.cfg = Config(n_layers, n_kv_heads, head_dim, max_chunk_tokens, group_int8, group_int4,
                          tau_gpu_ppm, rerank_interval, n_copy_streams, int(dry_run),
                          tau_pin_ppm, tau_page_ppm, 1 if disk_o_direct else 0,
                          1 if half_slots else 0, 1 if pinned_dma else 0, io_threads)
        self._h = C.c_void_p()
        rc = lib().ha_rag_create(C.byref(self.cfg), C.byref(self._h))
        if rc:
            detail = lib().ha_rag_last_hip_error(None).decode() if rc == EHIP else ""
            raise HaRagError(rc, "ha_rag_create", detail)
        self._keep = []  # tensors registered as slabs stay alive with the context

    def _chk(self, rc, where):
        if rc:
            detail = lib().ha_rag_last_hip_error(self._h).decode() if rc in (EHIP, EIO) else ""
            raise HaRagError(rc, where, detail)

    def destroy(self):
        if self._h:
            lib().ha_rag_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def group_of(self, prec):
        return {PREC_INT8: self.cfg.group_int8, PREC_INT4: self.cfg.group_int4}.get(prec, 0)

    def chunk_bytes(self, prec, n_tokens, group=None, part=PART_KV):
        g = self.group_of(prec) if group is None else group
        whole = ha_rag_chunk_bytes(self.cfg.n_layers, self.cfg.n_kv_heads, self.cfg.head_dim, prec,
                                   g, n_tokens)[2]
        return whole if part == PART_KV else whole // 2

    def forget_stream(self, stream):
        self._chk(lib().ha_rag_forget_stream(self._h, _stream(stream)), "ha_rag_forget_stream")

    def set_launch_params(self, threads=64, planes16=0, planes8=0, nt_store=1, nt_load=1):
        lp = LaunchParams(threads, planes16, planes8, int(nt_store), int(nt_load))
        self._chk(lib().ha_rag_set_launch_params(self._h, C.byref(lp)), "ha_rag_set_launch_params")

    def quantize_chunk(self, src, n_tokens, prec, group, dst, saturated=None, stream=None):
        self._chk(lib().ha_rag_quantize_chunk(self._h, _addr(src), n_tokens, prec, group, _addr(dst),
                                              _addr(saturated), _stream(stream)),
                  "ha_rag_quantize_chunk")

    def quantize_chunks(self, srcs, n_tokens, prec, group, dsts, saturated=None, stream=None):
        """One launch for a list of chunks of one tag: srcs / dsts lists of tensors or addresses,
        n_tokens a list."""
        n = len(srcs)
        sp = (C.c_void_p * max(n, 1))(*[_addr(x) for x in srcs])
        dp = (C.c_void_p * max(n, 1))(*[_addr(x) for x in dsts])
        nt = (C.c_uint32 * max(n, 1))(*[int(t) for t in n_tokens])
        self._chk(lib().ha_rag_quantize_chunks(self._h, sp, dp, nt, n, prec, group, _addr(saturated),
                                               _stream(stream)), "ha_rag_quantize_chunks")

    def quantize_half(self, src, n_tokens, prec, group, dst, saturated=None, stream=None):
        self._chk(lib().ha_rag_quantize_half(self._h, _addr(src), n_tokens, prec, group, _addr(dst),
                                             _addr(saturated), _stream(stream)),
                  "ha_rag_quantize_half")

    def chunk_sq_error(self, src, packed, n_tokens, prec, group, sum_sq, part=PART_KV, stream=None):
        self._chk(lib().ha_rag_chunk_sq_error(self._h, _addr(src), _addr(packed), n_tokens, prec, group,
                                              part, _addr(sum_sq), _stream(stream)),
                  "ha_rag_chunk_sq_error")

    def load_packed(self, chunks, out, cap_tokens, tok_base=0, stream=None):
        """chunks: list of (packed, n_tokens, prec, group[, part])."""
        arr = (PackedChunk * max(len(chunks), 1))()
        for i, ch in enumerate(chunks):
            p, t, prec, g = ch[:4]
            arr[i] = PackedChunk(_addr(p), t, prec, g, ch[4] if len(ch) > 4 else PART_KV)
        self._chk(lib().ha_rag_load_packed(self._h, arr, len(chunks), _addr(out), cap_tokens,
                                           tok_base, _stream(stream)), "ha_rag_load_packed")

    def load_packed_paged(self, chunks, cache, tok_base=0, stream=None):
        """chunks as in load_packed; cache: a PagedCache (see paged_cache())."""
        arr = (PackedChunk * max(len(chunks), 1))()
        for i, ch in enumerate(chunks):
            p, t, prec, g = ch[:4]
            arr[i] = PackedChunk(_addr(p), t, prec, g, ch[4] if len(ch) > 4 else PART_KV)
        self._chk(lib().ha_rag_load_packed_paged(self._h, arr, len(chunks), C.byref(cache), tok_base,
                                                 _stream(stream)), "ha_rag_load_packed_paged")

    @staticmethod
    def attend_lists(requests):
        """requests: list of (chunks, q, out, lse, n_q) with chunks as in load_packed.  Returns
        the marshalled lists, which attend_packed accepts in place of `requests` (a caller that
        repeats a call layer after layer marshals once)."""
        if isinstance(requests, tuple) and len(requests) == 3 and isinstance(requests[2], int):
            return requests
        n_chunks = sum(len(r[0]) for r in requests)
        arr = (PackedChunk * max(n_chunks, 1))()
        reqs = (AttendRequest * max(len(requests), 1))()
        k = 0
        for i, (chunks, q, out, lse, n_q) in enumerate(requests):
            for ch in chunks:
                p, t, prec, g = ch[:4]
                arr[k] = PackedChunk(_addr(p), t, prec, g, ch[4] if len(ch) > 4 else PART_KV)
                k += 1
            reqs[i] = AttendRequest(_addr(q), _addr(out), _addr(lse), n_q, len(chunks))
        return arr, reqs, len(requests)

    def attend_workspace_bytes(self, requests, n_q_heads):
        arr, reqs, n_reqs = self.attend_lists(requests)
        n = C.c_size_t(0)
        self._chk(lib().ha_rag_attend_workspace_bytes(self._h, arr, reqs, n_reqs, n_q_heads,
                                                      C.byref(n)), "ha_rag_attend_workspace_bytes")
        return n.value

    def attend_packed(self, requests, layer, n_q_heads, sm_scale, workspace, workspace_bytes=None,
                      stream=None):
        arr, reqs, n_reqs = self.attend_lists(requests)
        if workspace_bytes is None:
            workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        self._chk(lib().ha_rag_attend_packed(self._h, arr, reqs, n_reqs, layer, n_q_heads,
                                             sm_scale, _addr(workspace), workspace_bytes,
                                             _stream(stream)), "ha_rag_attend_packed")

    def attend_packed_static(self, requests, layer, n_q_heads, sm_scale, stream=None):
        arr, reqs, n_reqs = self.attend_lists(requests)
        rc = lib().ha_rag_attend_packed_static(self._h, arr, reqs, n_reqs, layer, n_q_heads,
                                               sm_scale, _stream(stream))
        if rc:
            detail = lib().ha_rag_last_hip_error(self._h).decode() if rc in (EHIP, ENOSPC) else ""
            raise HaRagError(rc, "ha_rag_attend_packed_static", detail)

    @staticmethod
    def attend_id_lists(requests):
        """requests: list of (ids, q, out, lse, n_q).  Returns the marshalled lists, which
        attend_chunks accepts in place of `requests`."""
        if isinstance(requests, tuple) and len(requests) == 3 and isinstance(requests[2], int):
            return requests
        ids = [i for r in requests for i in r[0]]
        reqs = (AttendRequest * max(len(requests), 1))()
        for k, (rid, q, out, lse, n_q) in enumerate(requests):
            reqs[k] = AttendRequest(_addr(q), _addr(out), _addr(lse), n_q, len(rid))
        return _u64s(ids), reqs, len(requests)

    def attend_chunks_workspace_bytes(self, requests, n_q_heads):
        ids, reqs, n_reqs = self.attend_id_lists(requests)
        n = C.c_size_t(0)
        self._chk(lib().ha_rag_attend_chunks_workspace_bytes(self._h, ids, reqs, n_reqs, n_q_heads,
                                                             C.byref(n)),
                  "ha_rag_attend_chunks_workspace_bytes")
        return n.value

    def attend_chunks(self, requests, layer, n_q_heads, sm_scale, workspace, workspace_bytes=None,
                      count=False, stream=None):
        ids, reqs, n_reqs = self.attend_id_lists(requests)
        if workspace_bytes is None:
            workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        self._chk(lib().ha_rag_attend_chunks(self._h, ids, reqs, n_reqs, layer, n_q_heads, sm_scale,
                                             ATTEND_COUNT if count else 0, _addr(workspace),
                                             workspace_bytes, _stream(stream)), "ha_rag_attend_chunks")

    def load_chunks_paged(self, ids, cache, tok_base=0, tags=None, stream=None, want_trace=False):
        n = len(ids)
        st = LoadStats()
        tr = (ChunkTrace * max(n, 1))() if want_trace else None
        tg = (C.c_uint8 * max(n, 1))(*tags) if tags is not None else None
        self._chk(lib().ha_rag_load_chunks_paged(self._h, _u64s(ids), tg, n, C.byref(cache), tok_base,
                                                 _stream(stream), C.byref(st), tr),
                  "ha_rag_load_chunks_paged")
        return st.as_dict(), (list(tr[:n]) if want_trace else None)

    def register_slab(self, tier, prec, base, nbytes=None):
        if nbytes is None:
            nbytes = base.numel() * base.element_size()
        self._chk(lib().ha_rag_register_slab(self._h, tier, prec, _addr(base), nbytes),
                  "ha_rag_register_slab")
        self._keep.append(base)

    def register_staging(self, base, nbytes=None):
        if nbytes is None:
            nbytes = base.numel() * base.element_size()
        self._chk(lib().ha_rag_register_staging(self._h, _addr(base), nbytes),
                  "ha_rag_register_staging")
        self._keep.append(base)

    def register_bounce(self, base, nbytes=None):
        if nbytes is None:
            nbytes = base.numel() * base.element_size()
        self._chk(lib().ha_rag_register_bounce(self._h, _addr(base), nbytes),
                  "ha_rag_register_bounce")
        self._keep.append(base)

    def register_disk(self, prec, path, nbytes):
        self._chk(lib().ha_rag_register_disk(self._h, prec, os.fsencode(path), nbytes),
                  "ha_rag_register_disk")

    def pool_insert(self, cid, prec, n_tokens, packed, tier, packed_is_device=False, stream=None):
        self._chk(lib().ha_rag_pool_insert(self._h, cid, prec, n_tokens, _addr(packed),
                                           1 if packed_is_device else 0, tier, _stream(stream)),
                  "ha_rag_pool_insert")

    def pool_insert_half(self, cid, part, prec, n_tokens, packed, tier, packed_is_device=False,
                         stream=None):
        self._chk(lib().ha_rag_pool_insert_half(self._h, cid, part, prec, n_tokens, _addr(packed),
                                                1 if packed_is_device else 0, tier, _stream(stream)),
                  "ha_rag_pool_insert_half")

    def pool_slot(self, cid, tier):
        p, n = C.c_void_p(), C.c_size_t()
        self._chk(lib().ha_rag_pool_slot(self._h, cid, tier, C.byref(p), C.byref(n)),
                  "ha_rag_pool_slot")
        return p.value, n.value

    def pool_promote(self, cid, stream=None):
        self._chk(lib().ha_rag_pool_promote(self._h, cid, _stream(stream)), "ha_rag_pool_promote")

    def pool_evict(self, cid, tier=TIER_HBM):
        self._chk(lib().ha_rag_pool_evict(self._h, cid, tier), "ha_rag_pool_evict")

    def pool_remove(self, cid):
        self._chk(lib().ha_rag_pool_remove(self._h, cid), "ha_rag_pool_remove")

    def pool_query(self, cid):
        info = ChunkInfo()
        self._chk(lib().ha_rag_pool_query(self._h, cid, C.byref(info)), "ha_rag_pool_query")
        return info

    def pool_save_index(self, path):
        self._chk(lib().ha_rag_pool_save_index(self._h, os.fsencode(path)), "ha_rag_pool_save_index")

    def pool_load_index(self, path):
        n = C.c_size_t()
        self._chk(lib().ha_rag_pool_load_index(self._h, os.fsencode(path), C.byref(n)),
                  "ha_rag_pool_load_index")
        return n.value

    def pool_lru(self, tier, cap=1 << 16):
        ids = (C.c_uint64 * cap)()
        n = C.c_size_t()
        self._chk(lib().ha_rag_pool_lru(self._h, tier, ids, cap, C.byref(n)), "ha_rag_pool_lru")
        return list(ids[:n.value])

    def pool_hbm_lru(self, cap=1 << 16):
        return self.pool_lru(TIER_HBM, cap)

    def register_external(self, prec):
        self._chk(lib().ha_rag_register_external(self._h, prec), "ha_rag_register_external")

    def pool_insert_external(self, cid, prec, n_tokens, pinned, part=PART_KV):
        """pinned: address (int) or pinned tensor holding the packed bytes; stays the caller's."""
        self._chk(lib().ha_rag_pool_insert_external(self._h, cid, part, prec, n_tokens, _addr(pinned)),
                  "ha_rag_pool_insert_external")

    def pool_repoint_external(self, ids, addrs):
        n = len(ids)
        arr = (C.c_void_p * max(n, 1))(*[int(a) for a in addrs])
        self._chk(lib().ha_rag_pool_repoint_external(self._h, _u64s(ids), arr, n),
                  "ha_rag_pool_repoint_external")

    def touch(self, ids):
        self._chk(lib().ha_rag_touch(self._h, _u64s(ids), len(ids)), "ha_rag_touch")

    def set_counts(self, ids, counts):
        self._chk(lib().ha_rag_set_counts(self._h, _u64s(ids), _u64s(counts), len(ids)),
                  "ha_rag_set_counts")

    def rerank(self):
        self._chk(lib().ha_rag_rerank(self._h), "ha_rag_rerank")

    def get_rank(self, cid):
        r = C.c_uint32()
        self._chk(lib().ha_rag_get_rank(self._h, cid, C.byref(r)), "ha_rag_get_rank")
        return r.value

    def load_chunks(self, ids, out, cap_tokens, tok_base=0, tags=None, stream=None,
                    want_trace=False):
        """Returns (stats dict, trace list or None)."""
        n = len(ids)
        st = LoadStats()
        tr = (ChunkTrace * max(n, 1))() if want_trace else None
        tg = (C.c_uint8 * max(n, 1))(*tags) if tags is not None else None
        self._chk(lib().ha_rag_load_chunks(self._h, _u64s(ids), tg, n, _addr(out), cap_tokens,
                                           tok_base, _stream(stream), C.byref(st), tr),
                  "ha_rag_load_chunks")
        return st.as_dict(), (list(tr[:n]) if want_trace else None)

    def place_chunks(self, ids, device_visible=False, tags=None, stream=None, want_trace=False):
        """Algorithm 2's bookkeeping and copies for `ids` without a decode.  Returns (stats dict,
        trace list or None)."""
        n = len(ids)
        st = LoadStats()
        tr = (ChunkTrace * max(n, 1))() if want_trace else None
        tg = (C.c_uint8 * max(n, 1))(*tags) if tags is not None else None
        self._chk(lib().ha_rag_place_chunks(self._h, _u64s(ids), tg, n,
                                            PLACE_DEVICE_VISIBLE if device_visible else 0,
                                            _stream(stream), C.byref(st), tr), "ha_rag_place_chunks")
        return st.as_dict(), (list(tr[:n]) if want_trace else None)

    def load_batch(self, requests, outs, cap_tokens, tok_base=None, tags=None, stream=None,
                   want_trace=False):
        """requests: list of id lists; outs: one cache per request."""
        flat = [i for r in requests for i in r]
        starts = [0]
        for r in requests:
            starts.append(starts[-1] + len(r))
        n, nr = len(flat), len(requests)
        st = LoadStats()
        tr = (ChunkTrace * max(n, 1))() if want_trace else None
        tg = (C.c_uint8 * max(n, 1))(*tags) if tags is not None else None
        outp = (C.c_void_p * max(nr, 1))(*[_addr(o) for o in outs])
        caps = _u64s(cap_tokens)
        base = _u64s(tok_base) if tok_base is not None else None
        self._chk(lib().ha_rag_load_batch(self._h, _u64s(flat), tg, (C.c_uint32 * (nr + 1))(*starts),
                                          nr, outp, caps, base, _stream(stream), C.byref(st), tr),
                  "ha_rag_load_batch")
        return st.as_dict(), (list(tr[:n]) if want_trace else None)
