"""ctypes binding of the C ABI declared in include/heddle.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

OK, E_INVAL, E_NOMEM, E_HIP, E_UNSUPPORTED = 0, -1, -2, -3, -4


def lib_path() -> str:
    return os.path.join(HERE, "libheddle.so")


def _load():
    # PyTorch ships its own HIP runtime; two runtimes in one process cannot both open the
    # GPU.  Import torch first so that libheddle's libamdhip64.so.7 dependency resolves to
    # the copy torch has already loaded.
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it first (python -m paper_2603_28101_amd.build, or "
            "__graft_entry__.build()); there is no fallback implementation")
    return C.CDLL(path)


lib = _load()

i32p = C.POINTER(C.c_int32)
vp = C.c_void_p


class Config(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("block_tokens", C.c_int32), ("n_blocks", C.c_int32), ("device", C.c_int32),
        ("kv_pool", vp),
        ("n_cu", C.c_int32), ("wg_per_cu", C.c_int32), ("min_chunk_blk", C.c_int32),
        ("tile_blk", C.c_int32), ("max_split", C.c_int32),
        ("scale", C.c_float),
        ("min_share_blk", C.c_int32), ("group_wg_per_cu", C.c_int32),
        ("append_wg_per_cu", C.c_int32), ("append_min_steps", C.c_int32),
    ]


class Plan(C.Structure):
    _fields_ = [
        ("cap_items", C.c_int32), ("n_items", C.c_int32), ("chunk", C.c_int32),
        ("item_b", i32p), ("item_s", i32p), ("item_blk_begin", i32p), ("item_blk_end", i32p),
        ("nsplit", i32p), ("part_off", i32p),
    ]


_SHARED_ITEM = ("item_b", "item_s", "item_blk_begin", "item_blk_end")
_SHARED_GITEM = ("gitem_g", "gitem_k", "gitem_blk_begin", "gitem_blk_end", "gitem_m0", "gitem_mn")
_SHARED_GROUP = ("group_leader", "group_prefix", "group_parts")
_SHARED_TRAJ = ("members", "traj_group", "traj_prefix", "nsplit")


class SharedPlan(C.Structure):
    _fields_ = (
        [(k, C.c_int32) for k in ("cap_items", "cap_gitems", "cap_groups", "n_items", "n_gitems", "n_groups",
                                  "chunk", "chunk_g")]
        + [(k, i32p) for k in _SHARED_ITEM + _SHARED_GITEM + _SHARED_GROUP]
        + [("member_off", i32p)] + [(k, i32p) for k in _SHARED_TRAJ] + [("part_off", i32p)]
    )


_SPLIT_TILE = ("tile_b", "tile_row0", "tile_rows_n", "tile_extent", "tile_nsplit", "tile_part_base")
_SPLIT_ITEM = ("item_tile", "item_k", "item_step_begin", "item_step_end")


class AppendSplitPlan(C.Structure):
    _fields_ = ([(k, C.c_int32) for k in ("cap_tiles", "cap_items", "n_tiles", "n_items", "n_slots", "tile_rows")]
                + [(k, i32p) for k in _SPLIT_TILE + _SPLIT_ITEM])


class AppendPlan(C.Structure):
    _fields_ = [
        ("cap_tiles", C.c_int32), ("n_tiles", C.c_int32), ("tile_rows", C.c_int32),
        ("tile_b", i32p), ("tile_row0", i32p), ("tile_rows_n", i32p), ("tile_extent", i32p),
    ]


class DecodeArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32),
        ("len_host", i32p), ("row_off_host", i32p),
        ("row_off", vp), ("block_ids", vp),
        ("q", vp), ("k_new", vp), ("v_new", vp), ("out", vp), ("lse", vp),
    ]


class AppendArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32),
        ("ctx_len_host", i32p), ("cu_chunk_host", i32p), ("row_off_host", i32p),
        ("row_off", vp), ("block_ids", vp),
        ("q", vp), ("k", vp), ("v", vp), ("out", vp), ("lse", vp),
    ]


lib.heddle_ctx_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
lib.heddle_ctx_destroy.argtypes = [vp]
lib.heddle_ctx_reserve.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32]
lib.heddle_kv_alloc.argtypes = [vp, C.c_int32, i32p]
lib.heddle_kv_free.argtypes = [vp, C.c_int32, i32p]
lib.heddle_kv_retain.argtypes = [vp, C.c_int32, i32p]
lib.heddle_ctx_set_kv_pool.argtypes = [vp, vp]
lib.heddle_kv_num_free.argtypes = [vp, i32p]
lib.heddle_plan_decode.argtypes = [vp, C.c_int32, i32p, C.POINTER(Plan)]
lib.heddle_plan_append.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int32, C.POINTER(AppendPlan)]
lib.heddle_attn_decode.argtypes = [vp, C.POINTER(DecodeArgs), vp]
lib.heddle_attn_decode_static.argtypes = [vp, C.POINTER(DecodeArgs), vp]
lib.heddle_plan_append_split.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int32, C.POINTER(AppendSplitPlan)]
lib.heddle_plan_decode_shared.argtypes = [vp, C.c_int32, i32p, i32p, i32p, C.POINTER(SharedPlan)]
lib.heddle_attn_decode_shared.argtypes = [vp, C.POINTER(DecodeArgs), i32p, vp]
lib.heddle_attn_append.argtypes = [vp, C.POINTER(AppendArgs), vp]
lib.heddle_kv_pack.argtypes = [vp, C.c_int32, i32p, vp, vp]
lib.heddle_kv_unpack.argtypes = [vp, C.c_int32, i32p, vp, vp]
lib.heddle_kv_copy.argtypes = [vp, C.c_int32, i32p, i32p, vp]
f64p = C.POINTER(C.c_double)
lib.heddle_placement_dp.argtypes = [C.c_int32, f64p, i32p, C.c_int32, f64p, C.c_int32, C.c_double, C.c_int32,
                                    i32p, f64p]
lib.heddle_placement_aggregate.argtypes = [C.c_int32, f64p, C.c_double, C.c_int32, i32p, i32p, i32p]
lib.heddle_interference_table.argtypes = [C.c_int32, f64p, f64p, C.c_int32, f64p]
lib.heddle_simulate_group.argtypes = [C.c_int32, i32p, C.c_int32, f64p, f64p, f64p]
lib.heddle_timing_enable.argtypes = [vp, C.c_int32]
lib.heddle_timing_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
lib.heddle_timing_samples.argtypes = [vp, C.c_int32, C.c_int64, C.POINTER(C.c_float), C.POINTER(C.c_int64)]
lib.heddle_stream_read.argtypes = [vp, C.c_uint64, vp, vp]
lib.heddle_ctx_scratch_bytes.argtypes = [vp, C.POINTER(C.c_uint64)]
lib.heddle_ctx_scratch_bytes.restype = C.c_int
lib.heddle_strerror.argtypes = [C.c_int]
lib.heddle_strerror.restype = C.c_char_p
lib.heddle_last_error_detail.restype = C.c_char_p
for _f in ("heddle_ctx_create", "heddle_ctx_destroy", "heddle_ctx_reserve", "heddle_ctx_set_kv_pool", "heddle_kv_alloc", "heddle_kv_free",
           "heddle_kv_retain",
           "heddle_kv_num_free", "heddle_plan_decode", "heddle_plan_append", "heddle_attn_decode",
           "heddle_attn_decode_static",
           "heddle_attn_append", "heddle_plan_decode_shared", "heddle_attn_decode_shared", "heddle_plan_append_split", "heddle_kv_pack", "heddle_kv_unpack", "heddle_kv_copy", "heddle_timing_enable",
           "heddle_timing_read", "heddle_timing_samples", "heddle_stream_read", "heddle_placement_dp", "heddle_placement_aggregate",
           "heddle_interference_table", "heddle_simulate_group",
           "heddle_version"):
    getattr(lib, _f).restype = C.c_int


class HeddleError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        # the detail text belongs to a failed HIP call, or names the limit a static-scratch call exceeded
        detail = (lib.heddle_last_error_detail().decode()
                  if code == E_HIP or (code == E_NOMEM and where.endswith("_static")) else "")
        super().__init__(f"{where}: {lib.heddle_strerror(code).decode()} ({code}) {detail}")


def _check(code: int, where: str):
    if code != OK:
        raise HeddleError(code, where)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(i32p)


def _dptr(t, what="tensor", itemsize=None, min_elems=0):
    """Device pointer of a torch tensor (or a raw integer address / None).  The C ABI takes plain
    pointers and cannot see what is behind them, so a tensor is checked here: it must live on a
    GPU, be contiguous, have elements of `itemsize` bytes and hold at least `min_elems` of them --
    a host tensor or a short one would otherwise end in a GPU memory fault, not in an error."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError(f"{what}: expected a device tensor, got one on {t.device}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: device tensors must be contiguous")
    if itemsize is not None and t.element_size() != itemsize:
        raise ValueError(f"{what}: elements of {itemsize} bytes expected, got {t.dtype}")
    if t.numel() < min_elems:
        raise ValueError(f"{what}: {t.numel()} elements, the call reads or writes {min_elems}")
    return t.data_ptr()


def _stream_ptr(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(f64p)


def placement_dp(lengths_desc, m, F, T=1.0, counts=None, full_scan=False):
    """(makespan, sizes[m]) of the presorted dynamic programming over descending lengths."""
    L, Lp = _f64(lengths_desc)
    Ft, Fp = _f64(F)
    cp = None
    if counts is not None:
        cnt, cp = _i32(counts)
    sizes = np.zeros(max(int(m), 1), dtype=np.int32)
    mk = C.c_double()
    _check(lib.heddle_placement_dp(L.shape[0], Lp, cp, int(m), Fp, Ft.shape[0], float(T), 1 if full_scan else 0,
                                   sizes.ctypes.data_as(i32p), C.byref(mk)), "heddle_placement_dp")
    return mk.value, sizes


def placement_aggregate(lengths_desc, threshold, bundle):
    L, Lp = _f64(lengths_desc)
    first = np.empty(max(L.shape[0], 1), dtype=np.int32)
    count = np.empty(max(L.shape[0], 1), dtype=np.int32)
    n = C.c_int32()
    _check(lib.heddle_placement_aggregate(L.shape[0], Lp, float(threshold), int(bundle), first.ctypes.data_as(i32p),
                                          count.ctypes.data_as(i32p), C.byref(n)), "heddle_placement_aggregate")
    return first[: n.value].copy(), count[: n.value].copy()


def interference_table(batch_sizes, step_time, n):
    bs, bsp = _f64(batch_sizes)
    ts, tsp = _f64(step_time)
    if bs.shape != ts.shape:
        raise ValueError("one step time per batch size")
    F = np.empty(int(n) + 1, dtype=np.float64)
    _check(lib.heddle_interference_table(bs.shape[0], bsp, tsp, int(n), F.ctypes.data_as(f64p)),
           "heddle_interference_table")
    return F


def simulate_group(lengths, batch_sizes, step_time):
    L, Lp = _i32(lengths)
    bs, bsp = _f64(batch_sizes)
    ts, tsp = _f64(step_time)
    out = C.c_double()
    _check(lib.heddle_simulate_group(L.shape[0], Lp, bs.shape[0], bsp, tsp, C.byref(out)), "heddle_simulate_group")
    return out.value


class Context:
    """One paged KV pool with its block manager, planners and attention calls."""

    def __init__(self, n_q_heads, n_kv_heads, head_dim, n_blocks, kv_pool=None, device=-1, *,
                 n_cu=0, wg_per_cu=0, min_chunk_blk=0, tile_blk=0, max_split=0, scale=0.0,
                 min_share_blk=0, group_wg_per_cu=0, append_wg_per_cu=0, append_min_steps=0):
        self.n_q_heads, self.n_kv_heads, self.head_dim, self.n_blocks = n_q_heads, n_kv_heads, head_dim, n_blocks
        pool_elems = int(n_blocks) * int(n_kv_heads) * 2 * 16 * int(head_dim)
        self.cfg = Config(n_q_heads, n_kv_heads, head_dim, 16, n_blocks, device, _dptr(kv_pool, "kv_pool", 2, pool_elems),
                          n_cu, wg_per_cu, min_chunk_blk, tile_blk, max_split, scale,
                          min_share_blk, group_wg_per_cu, append_wg_per_cu, append_min_steps)
        self._pool = kv_pool  # keep the tensor alive
        self._h = vp()
        _check(lib.heddle_ctx_create(C.byref(self.cfg), C.byref(self._h)), "heddle_ctx_create")
        self.max_split = max_split or 64

    def close(self):
        if self._h:
            h, self._h = self._h, vp()
            _check(lib.heddle_ctx_destroy(h), "heddle_ctx_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reserve(self, max_trajectories: int, max_chunk_rows: int = 0, with_shared_prefix: bool = False) -> None:
        """Sizes the scratch for the largest batch: no later call within these limits allocates or synchronises."""
        _check(lib.heddle_ctx_reserve(self._h, int(max_trajectories), int(max_chunk_rows), 1 if with_shared_prefix else 0),
               "heddle_ctx_reserve")

    def set_kv_pool(self, kv_pool) -> None:
        """Another pool of the same shape (one per layer of a model); later calls read and write it."""
        pool_elems = self.n_blocks * self.n_kv_heads * 2 * 16 * self.head_dim
        _check(lib.heddle_ctx_set_kv_pool(self._h, _dptr(kv_pool, "kv_pool", 2, pool_elems)), "heddle_ctx_set_kv_pool")
        self._pool = kv_pool  # keep the tensor alive

    # ---- block manager
    def kv_alloc(self, n: int) -> np.ndarray:
        out = np.empty(max(n, 0), dtype=np.int32)
        _check(lib.heddle_kv_alloc(self._h, n, out.ctypes.data_as(i32p)), "heddle_kv_alloc")
        return out

    def kv_retain(self, ids) -> None:
        a, p = _i32(ids)
        _check(lib.heddle_kv_retain(self._h, a.shape[0], p), "heddle_kv_retain")

    def kv_free(self, ids) -> None:
        a, p = _i32(ids)
        _check(lib.heddle_kv_free(self._h, a.shape[0], p), "heddle_kv_free")

    def kv_num_free(self) -> int:
        n = C.c_int32()
        _check(lib.heddle_kv_num_free(self._h, C.byref(n)), "heddle_kv_num_free")
        return n.value

    # ---- planners
    def plan_decode(self, lens) -> dict:
        lens_a, lens_p = _i32(lens)
        B = lens_a.shape[0]
        cap = max(B * self.max_split, 1)
        arrs = {k: np.empty(cap, dtype=np.int32) for k in ("item_b", "item_s", "item_blk_begin", "item_blk_end")}
        nsplit = np.empty(B, dtype=np.int32)
        part_off = np.empty(B + 1, dtype=np.int32)
        p = Plan(cap, 0, 0, *(arrs[k].ctypes.data_as(i32p) for k in ("item_b", "item_s", "item_blk_begin", "item_blk_end")),
                 nsplit.ctypes.data_as(i32p), part_off.ctypes.data_as(i32p))
        _check(lib.heddle_plan_decode(self._h, B, lens_p, C.byref(p)), "heddle_plan_decode")
        out = {k: v[: p.n_items].copy() for k, v in arrs.items()}
        out.update(n_items=p.n_items, chunk=p.chunk, nsplit=nsplit, part_off=part_off)
        return out

    def plan_decode_shared(self, lens, row_off, block_ids) -> dict:
        lens_a, lens_p = _i32(lens)
        ro_a, ro_p = _i32(row_off)
        ids_a, ids_p = _i32(block_ids)
        B = lens_a.shape[0]
        cap_items = max(B * self.max_split, 1)
        cap_gitems = max(B * self.max_split, 1)
        cap_groups = max(B // 2, 1)
        arrs = {k: np.empty(cap_items, dtype=np.int32) for k in _SHARED_ITEM}
        arrs.update({k: np.empty(cap_gitems, dtype=np.int32) for k in _SHARED_GITEM})
        arrs.update({k: np.empty(cap_groups, dtype=np.int32) for k in _SHARED_GROUP})
        arrs["member_off"] = np.empty(cap_groups + 1, dtype=np.int32)
        arrs.update({k: np.empty(B, dtype=np.int32) for k in _SHARED_TRAJ})
        arrs["part_off"] = np.empty(B + 1, dtype=np.int32)
        p = SharedPlan(cap_items, cap_gitems, cap_groups, 0, 0, 0, 0, 0,
                       *(arrs[k].ctypes.data_as(i32p) for k in _SHARED_ITEM + _SHARED_GITEM + _SHARED_GROUP),
                       arrs["member_off"].ctypes.data_as(i32p),
                       *(arrs[k].ctypes.data_as(i32p) for k in _SHARED_TRAJ),
                       arrs["part_off"].ctypes.data_as(i32p))
        _check(lib.heddle_plan_decode_shared(self._h, B, lens_p, ro_p, ids_p, C.byref(p)),
               "heddle_plan_decode_shared")
        out = {k: arrs[k][: p.n_items].copy() for k in _SHARED_ITEM}
        out.update({k: arrs[k][: p.n_gitems].copy() for k in _SHARED_GITEM})
        out.update({k: arrs[k][: p.n_groups].copy() for k in _SHARED_GROUP})
        out["member_off"] = arrs["member_off"][: p.n_groups + 1].copy()
        out["members"] = arrs["members"][: int(out["member_off"][-1])].copy()
        out.update({k: arrs[k] for k in ("traj_group", "traj_prefix", "nsplit", "part_off")})
        out.update(n_items=p.n_items, n_gitems=p.n_gitems, n_groups=p.n_groups, chunk=p.chunk, chunk_g=p.chunk_g)
        return out

    def plan_append(self, ctx_lens, cu_chunk, tile_rows: int = 0) -> dict:
        L, Lp = _i32(ctx_lens)
        cu, cup = _i32(cu_chunk)
        B = L.shape[0]
        tr = tile_rows if tile_rows > 0 else 1
        cap = int(sum(-(-int(cu[b + 1] - cu[b]) // tr) for b in range(B))) if tile_rows > 0 else int(cu[-1])
        cap = max(cap, 1)
        arrs = {k: np.empty(cap, dtype=np.int32) for k in ("tile_b", "tile_row0", "tile_rows_n", "tile_extent")}
        p = AppendPlan(cap, 0, 0, *(arrs[k].ctypes.data_as(i32p) for k in ("tile_b", "tile_row0", "tile_rows_n", "tile_extent")))
        _check(lib.heddle_plan_append(self._h, B, Lp, cup, tile_rows, C.byref(p)), "heddle_plan_append")
        out = {k: v[: p.n_tiles].copy() for k, v in arrs.items()}
        out.update(n_tiles=p.n_tiles, tile_rows=p.tile_rows)
        return out

    def plan_append_split(self, ctx_lens, cu_chunk, tile_rows: int = 0) -> dict:
        L, Lp = _i32(ctx_lens)
        cu, cup = _i32(cu_chunk)
        B = L.shape[0]
        cap_tiles = max(int(cu[-1]), 1)
        cap_items = cap_tiles * self.max_split
        arrs = {k: np.empty(cap_tiles, dtype=np.int32) for k in _SPLIT_TILE}
        arrs.update({k: np.empty(cap_items, dtype=np.int32) for k in _SPLIT_ITEM})
        p = AppendSplitPlan(cap_tiles, cap_items, 0, 0, 0, 0,
                            *(arrs[k].ctypes.data_as(i32p) for k in _SPLIT_TILE + _SPLIT_ITEM))
        _check(lib.heddle_plan_append_split(self._h, B, Lp, cup, tile_rows, C.byref(p)), "heddle_plan_append_split")
        out = {k: arrs[k][: p.n_tiles].copy() for k in _SPLIT_TILE}
        out.update({k: arrs[k][: p.n_items].copy() for k in _SPLIT_ITEM})
        out.update(n_tiles=p.n_tiles, n_items=p.n_items, n_slots=p.n_slots, tile_rows=p.tile_rows)
        return out

    # ---- attention
    def attn_decode(self, lens, row_off_host, row_off, block_ids, q, out, lse=None, k_new=None,
                    v_new=None, stream=None) -> None:
        lens_a, lens_p = _i32(lens)
        ro_a, ro_p = _i32(row_off_host)
        args = self._decode_args(lens_a, lens_p, ro_a, ro_p, row_off, block_ids, q, out, lse, k_new, v_new)
        _check(lib.heddle_attn_decode(self._h, C.byref(args), _stream_ptr(stream)), "heddle_attn_decode")

    def attn_decode_static(self, lens, row_off_host, row_off, block_ids, q, out, lse=None, k_new=None,
                           v_new=None, stream=None) -> None:
        """heddle_attn_decode with the library's static device scratch: allocates nothing."""
        lens_a, lens_p = _i32(lens)
        ro_a, ro_p = _i32(row_off_host)
        args = self._decode_args(lens_a, lens_p, ro_a, ro_p, row_off, block_ids, q, out, lse, k_new, v_new)
        _check(lib.heddle_attn_decode_static(self._h, C.byref(args), _stream_ptr(stream)),
               "heddle_attn_decode_static")

    def _decode_args(self, lens_a, lens_p, ro_a, ro_p, row_off, block_ids, q, out, lse, k_new, v_new):
        B = lens_a.shape[0]
        if ro_a.shape[0] != B + 1:
            raise ValueError("row_off_host must have one more entry than lens")
        nq, nkv = B * self.n_q_heads * self.head_dim, B * self.n_kv_heads * self.head_dim
        return DecodeArgs(B, lens_p, ro_p, _dptr(row_off, "row_off", 4, B + 1),
                          _dptr(block_ids, "block_ids", 4, max(int(ro_a[-1]), 0)), _dptr(q, "q", 2, nq),
                          _dptr(k_new, "k_new", 2, nkv), _dptr(v_new, "v_new", 2, nkv), _dptr(out, "out", 2, nq),
                          _dptr(lse, "lse", 4, B * self.n_q_heads))

    def attn_decode_shared(self, lens, row_off_host, block_ids_host, row_off, block_ids, q, out, lse=None,
                           k_new=None, v_new=None, stream=None) -> None:
        lens_a, lens_p = _i32(lens)
        ro_a, ro_p = _i32(row_off_host)
        ids_a, ids_p = _i32(block_ids_host)
        if ro_a.shape[0] and ids_a.shape[0] < int(ro_a[-1]):
            raise ValueError("block_ids_host is shorter than the table row_off_host describes")
        args = self._decode_args(lens_a, lens_p, ro_a, ro_p, row_off, block_ids, q, out, lse, k_new, v_new)
        _check(lib.heddle_attn_decode_shared(self._h, C.byref(args), ids_p, _stream_ptr(stream)),
               "heddle_attn_decode_shared")

    def attn_append(self, ctx_lens, cu_chunk, row_off_host, row_off, block_ids, q, k, v, out, lse=None,
                    stream=None) -> None:
        L, Lp = _i32(ctx_lens)
        cu, cup = _i32(cu_chunk)
        ro_a, ro_p = _i32(row_off_host)
        B = L.shape[0]
        if cu.shape[0] != B + 1 or ro_a.shape[0] != B + 1:
            raise ValueError("cu_chunk and row_off_host must have one more entry than ctx_lens")
        rows = max(int(cu[-1]), 0)
        nq, nkv = rows * self.n_q_heads * self.head_dim, rows * self.n_kv_heads * self.head_dim
        args = AppendArgs(B, Lp, cup, ro_p, _dptr(row_off, "row_off", 4, B + 1),
                          _dptr(block_ids, "block_ids", 4, max(int(ro_a[-1]), 0)), _dptr(q, "q", 2, nq),
                          _dptr(k, "k", 2, nkv), _dptr(v, "v", 2, nkv), _dptr(out, "out", 2, nq),
                          _dptr(lse, "lse", 4, rows * self.n_q_heads))
        _check(lib.heddle_attn_append(self._h, C.byref(args), _stream_ptr(stream)), "heddle_attn_append")

    # ---- pack / unpack
    def kv_pack(self, block_ids, staging, stream=None) -> None:
        a, p = _i32(block_ids)
        need = a.shape[0] * self.n_kv_heads * 2 * 16 * self.head_dim
        _check(lib.heddle_kv_pack(self._h, a.shape[0], p, _dptr(staging, "staging", 2, need), _stream_ptr(stream)),
               "heddle_kv_pack")

    def kv_unpack(self, block_ids, staging, stream=None) -> None:
        a, p = _i32(block_ids)
        need = a.shape[0] * self.n_kv_heads * 2 * 16 * self.head_dim
        _check(lib.heddle_kv_unpack(self._h, a.shape[0], p, _dptr(staging, "staging", 2, need), _stream_ptr(stream)),
               "heddle_kv_unpack")

    def kv_copy(self, src_block_ids, dst_block_ids, stream=None) -> None:
        s, sp = _i32(src_block_ids)
        d, dp = _i32(dst_block_ids)
        if s.shape[0] != d.shape[0]:
            raise ValueError("kv_copy: as many destinations as sources")
        _check(lib.heddle_kv_copy(self._h, s.shape[0], sp, dp, _stream_ptr(stream)), "heddle_kv_copy")

    # ---- measurement
    def scratch_bytes(self):
        """(plan buffer, split-K partials, pinned staging ring) in bytes, as allocated right now."""
        out = (C.c_uint64 * 3)()
        _check(lib.heddle_ctx_scratch_bytes(self._h, out), "heddle_ctx_scratch_bytes")
        return tuple(int(x) for x in out)

    def timing_enable(self, every: int = 1) -> None:
        """every = N >= 1: record every N-th launch of each kernel; 0 / False: off."""
        _check(lib.heddle_timing_enable(self._h, int(every)), "heddle_timing_enable")

    def timing_read(self, which: int):
        us, n = C.c_double(), C.c_int64()
        _check(lib.heddle_timing_read(self._h, which, C.byref(us), C.byref(n)), "heddle_timing_read")
        return us.value, n.value

    def timing_samples(self, which: int) -> np.ndarray:
        """Durations in microseconds of the recorded launches of one kernel (at most the last 2048)."""
        n = C.c_int64()
        _check(lib.heddle_timing_samples(self._h, which, 0, None, C.byref(n)), "heddle_timing_samples")
        out = np.empty(min(n.value, 2048), dtype=np.float32)
        _check(lib.heddle_timing_samples(self._h, which, out.shape[0], out.ctypes.data_as(C.POINTER(C.c_float)),
                                         C.byref(n)), "heddle_timing_samples")
        return out


def stream_read(src, nbytes: int, sink, stream=None) -> None:
    _check(lib.heddle_stream_read(_dptr(src), nbytes, _dptr(sink), _stream_ptr(stream)), "heddle_stream_read")
