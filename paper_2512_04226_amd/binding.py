"""ctypes binding of include/gemm.h: same names, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device buffers: bf16 operands as
torch.bfloat16 (or int16/uint16 bit patterns), fp8 operands as torch.uint8 or
torch.float8_e4m3fn.  Every computation happens inside libgemm355.so; if the library is
missing this module raises at import.
"""
import ctypes
import os

# PyTorch bundles its own HIP runtime.  Loading it first makes libgemm355.so resolve
# libamdhip64 to that same copy: one runtime per process, so that streams and device
# pointers handed over by torch belong to the runtime that launches the kernels.
import torch  # noqa: F401

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("GEMM355_LIB") or os.path.join(_PKG, "libgemm355.so")   # override: a differently built copy

GEMM_BF16 = 0
GEMM_FP8_E4M3 = 1
GEMM_FP16 = 2
GEMM_ABI_VERSION = 8
GEMM_B_ROW_MAJOR = 0
GEMM_B_K_CONTIGUOUS = 1

STATUS = {0: "GEMM_OK", -1: "GEMM_ERR_NULL", -2: "GEMM_ERR_SHAPE", -3: "GEMM_ERR_DTYPE", -4: "GEMM_ERR_CFG_ILLEGAL",
          -5: "GEMM_ERR_ALIGN", -6: "GEMM_ERR_WORKSPACE", -7: "GEMM_ERR_ABI", -8: "GEMM_ERR_HIP", -9: "GEMM_ERR_INDEX"}
BOTTLENECKS = ("compute_full", "compute_under_occupied", "ls_issue", "lds", "l2", "mall", "hbm", "launch")


class GemmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        RuntimeError.__init__(self, "%s: %s (%d: %s)" % (where, STATUS.get(status, "?"), status,
                                                         gemm_strerror(status)))


class gemm_hw(ctypes.Structure):
    _fields_ = [("n_cu", ctypes.c_int32), ("n_xcd", ctypes.c_int32), ("simd_per_cu", ctypes.c_int32),
                ("reserved0", ctypes.c_int32), ("lds_bytes", ctypes.c_double), ("l2_bytes", ctypes.c_double),
                ("mall_bytes", ctypes.c_double), ("clk_ghz", ctypes.c_double),
                ("hbm_bytes_per_clk", ctypes.c_double), ("mall_bytes_per_clk", ctypes.c_double),
                ("l2_bytes_per_clk", ctypes.c_double), ("lds_bytes_per_clk", ctypes.c_double),
                ("lds_tr_bytes_per_clk", ctypes.c_double),
                ("vmem_bytes_per_clk", ctypes.c_double), ("mem_latency_clk", ctypes.c_double),
                ("cache_eff_frac", ctypes.c_double), ("launch_clk", ctypes.c_double),
                ("wg_overhead_clk", ctypes.c_double), ("epilogue_clk", ctypes.c_double),
                ("reduce_launch_clk", ctypes.c_double), ("under_occ_frac", ctypes.c_double),
                ("seg_eff_lo", ctypes.c_double), ("overlap_frac", ctypes.c_double),
                ("l_mi_clk", (ctypes.c_double * 2) * 2), ("fill_issue_bytes_per_clk", ctypes.c_double),
                ("slab_sync_clk", ctypes.c_double)]


class gemm_cfg(ctypes.Structure):
    _fields_ = [("abi_version", ctypes.c_uint32), ("dtype", ctypes.c_int32), ("M", ctypes.c_int64),
                ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64),
                ("ldc", ctypes.c_int64), ("kernel_id", ctypes.c_int32), ("block_m", ctypes.c_uint16),
                ("block_n", ctypes.c_uint16), ("block_k", ctypes.c_uint16), ("waves_m", ctypes.c_uint8),
                ("waves_n", ctypes.c_uint8), ("mfma", ctypes.c_uint8), ("k_unroll", ctypes.c_uint8),
                ("split_k", ctypes.c_uint16), ("group_m", ctypes.c_uint16), ("group_n", ctypes.c_uint16),
                ("xcd_remap", ctypes.c_uint8), ("stages", ctypes.c_uint8),
                ("reserved1", ctypes.c_uint16), ("b_layout", ctypes.c_uint8), ("stream_k", ctypes.c_uint8),
                ("sk_workers", ctypes.c_uint16), ("alpha", ctypes.c_float),
                ("bottleneck", ctypes.c_int32), ("beta", ctypes.c_float), ("predicted_us", ctypes.c_double),
                ("batch", ctypes.c_int32), ("groups", ctypes.c_int32), ("stride_a", ctypes.c_int64),
                ("stride_b", ctypes.c_int64), ("stride_c", ctypes.c_int64)]

    def describe(self):
        return ("%dx%dx%d w%dx%d mfma%d s%d %s g%d%s%s" % (
            self.block_m, self.block_n, self.block_k, self.waves_m, self.waves_n, self.mfma, self.stages,
            ("streamk%d" % self.sk_workers) if self.stream_k else ("split%d" % self.split_k), self.group_m,
            "" if self.xcd_remap else " noxcd", " Bkc" if self.b_layout else "")
                + (" batch%d" % self.batch if self.batch > 1 else "")
                + (" groups%d" % self.groups if self.groups else ""))

    def copy(self):
        c = gemm_cfg()
        ctypes.memmove(ctypes.byref(c), ctypes.byref(self), ctypes.sizeof(gemm_cfg))
        return c


class gemm_prediction(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in (
        "n_mi", "l_mt_ideal", "l_compute", "tiles", "waves", "active_cu", "f_m", "f_n", "h_l2", "h_mall", "l_issue", "l_lds",
        "l_l2", "l_mall", "l_hbm", "l_mem", "l_mem_tail", "l_prologue", "l_epilogue", "l_iter", "iters", "l_tile",
        "l_tile_tail", "l_reduce", "l_total", "total_us")] + [("bottleneck", ctypes.c_int32),
                                                              ("occupancy", ctypes.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError("libgemm355.so is not built: run `python -m paper_2512_04226_amd.build` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_i64, _int, _vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
_lib.gemm_abi_version.restype = ctypes.c_uint32
_lib.gemm_abi_version.argtypes = []
_lib.gemm_strerror.restype = ctypes.c_char_p
_lib.gemm_strerror.argtypes = [_int]
_lib.gemm_select.restype = _int
_lib.gemm_select.argtypes = [_i64, _i64, _i64, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_select_ex.restype = _int
_lib.gemm_select_ex.argtypes = [_i64, _i64, _i64, _int, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_cfg_at_ex.restype = _int
_lib.gemm_cfg_at_ex.argtypes = [_int, _i64, _i64, _i64, _int, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_run.restype = _int
_lib.gemm_run.argtypes = [ctypes.POINTER(gemm_cfg), _vp, _vp, _vp, _vp]
_lib.gemm_run_noalloc.restype = _int
_lib.gemm_run_noalloc.argtypes = [ctypes.POINTER(gemm_cfg), _vp, _vp, _vp, _vp]
GEMM_NOALLOC_WORKSPACE_BYTES = 64 << 20
_lib.gemm_workspace_bytes.restype = ctypes.c_size_t
_lib.gemm_workspace_bytes.argtypes = [ctypes.POINTER(gemm_cfg)]
_lib.gemm_set_workspace.restype = _int
_lib.gemm_set_workspace.argtypes = [_vp, ctypes.c_size_t]
_lib.gemm_cfg_count.restype = _int
_lib.gemm_cfg_count.argtypes = [_int]
_lib.gemm_cfg_at.restype = _int
_lib.gemm_cfg_at.argtypes = [_int, _i64, _i64, _i64, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_predict.restype = _int
_lib.gemm_predict.argtypes = [ctypes.POINTER(gemm_cfg), ctypes.POINTER(gemm_prediction)]
_lib.gemm_hw_get.restype = _int
_lib.gemm_hw_get.argtypes = [ctypes.POINTER(gemm_hw)]
_lib.gemm_hw_set.restype = _int
_lib.gemm_hw_set.argtypes = [ctypes.POINTER(gemm_hw)]
_lib.gemm_hw_reset.restype = _int
_lib.gemm_hw_reset.argtypes = []
_lib.gemm_hw_preset.restype = _int
_lib.gemm_hw_preset.argtypes = [_int, ctypes.POINTER(gemm_hw)]


_lib.gemm_probe_mfma.restype = _int
_lib.gemm_probe_mfma.argtypes = [_int, _int, _vp, _vp, ctypes.POINTER(ctypes.c_double)]
_lib.gemm_probe_stream.restype = _int
_lib.gemm_probe_stream.argtypes = [_vp, ctypes.c_size_t, _vp, _vp, ctypes.POINTER(ctypes.c_double)]


_lib.gemm_variant_occupancy.restype = _int
_lib.gemm_variant_occupancy.argtypes = [_int, _int, _int, ctypes.POINTER(_int)]


def gemm_variant_occupancy(dtype, variant, b_layout=GEMM_B_ROW_MAJOR):
    """Workgroups of a compiled variant the HIP runtime keeps resident on one CU (needs the GPU)."""
    out = _int()
    _check(_lib.gemm_variant_occupancy(dtype, variant, b_layout, ctypes.byref(out)), "gemm_variant_occupancy")
    return out.value


_lib.gemm_probe_mfma_ex.restype = _int
_lib.gemm_probe_mfma_ex.argtypes = [_int, _int, _int, ctypes.c_double, ctypes.c_double, _vp, _vp,
                                    ctypes.POINTER(ctypes.c_double)]
_lib.gemm_probe_read.restype = _int
_lib.gemm_probe_read.argtypes = [_vp, ctypes.c_size_t, _int, _vp, _vp, ctypes.POINTER(ctypes.c_double)]
_lib.gemm_probe_lds.restype = _int
_lib.gemm_probe_lds.argtypes = [_int, _int, _vp, _vp, ctypes.POINTER(ctypes.c_double)]
_lib.gemm_probe_fill.restype = _int
_lib.gemm_probe_fill.argtypes = [_int, _int, _int, _int, _vp, ctypes.c_size_t, ctypes.c_size_t, _vp, _vp,
                                 ctypes.POINTER(ctypes.c_double)]
_lib.gemm_probe_latency.restype = _int
_lib.gemm_probe_latency.argtypes = [_vp, ctypes.c_size_t, _vp, _vp, ctypes.POINTER(ctypes.c_double)]


def gemm_probe_mfma_ex(dtype, mfma, operands, scratch, warm_ms=30.0, timed_ms=20.0, stream=None):
    """TFLOP/s of the MFMA loop on constant (operands=0) or workload-like (operands=1) register contents,
    in the settled state."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_mfma_ex(dtype, mfma, operands, warm_ms, timed_ms, _ptr(scratch),
                                   ctypes.c_void_p(_stream_handle(stream)), ctypes.byref(out)), "gemm_probe_mfma_ex")
    return out.value


def gemm_probe_read(buf, passes, scratch, stream=None):
    """GB/s of `passes` reads of the whole tensor by one launch."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_read(_ptr(buf), buf.numel() * buf.element_size(), passes, _ptr(scratch),
                                ctypes.c_void_p(_stream_handle(stream)), ctypes.byref(out)), "gemm_probe_read")
    return out.value


def gemm_probe_lds(kind, waves_per_cu, scratch, stream=None):
    """Device-wide GB/s of LDS fragment reads (kind 0 b128, 1 b64, 2 tr_b16, 3 tr_b8)."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_lds(kind, waves_per_cu, _ptr(scratch), ctypes.c_void_p(_stream_handle(stream)),
                               ctypes.byref(out)), "gemm_probe_lds")
    return out.value


def gemm_probe_fill(kind, pattern, buf, footprint, scratch, wgs_per_cu=1, sync=0, stream=None):
    """Device-wide GB/s of 8-wave workgroups moving 64 KiB slabs from the tensor towards LDS (kind 0 direct
    to LDS 16 B per lane, 1 direct 4 B per lane, 2 into registers, 3 registers then ds_write; pattern 0
    consecutive bytes inside `footprint`, 1 rows of 128 B 16 KiB apart)."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_fill(kind, pattern, wgs_per_cu, sync, _ptr(buf), buf.numel() * buf.element_size(), footprint,
                                _ptr(scratch), ctypes.c_void_p(_stream_handle(stream)), ctypes.byref(out)),
           "gemm_probe_fill")
    return out.value


def gemm_probe_latency(buf, scratch, stream=None):
    """Nanoseconds per dependent load through the tensor (which is overwritten)."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_latency(_ptr(buf), buf.numel() * buf.element_size(), _ptr(scratch),
                                   ctypes.c_void_p(_stream_handle(stream)), ctypes.byref(out)), "gemm_probe_latency")
    return out.value


def gemm_probe_mfma(dtype, mfma, scratch, stream=None):
    """Device-wide TFLOP/s of a register-resident MFMA loop (scratch: any device tensor)."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_mfma(dtype, mfma, _ptr(scratch), ctypes.c_void_p(_stream_handle(stream)),
                                ctypes.byref(out)), "gemm_probe_mfma")
    return out.value


def gemm_probe_stream(buf, scratch, stream=None):
    """GB/s of a streaming read over the device tensor buf."""
    out = ctypes.c_double()
    _check(_lib.gemm_probe_stream(_ptr(buf), buf.numel() * buf.element_size(), _ptr(scratch),
                                  ctypes.c_void_p(_stream_handle(stream)), ctypes.byref(out)), "gemm_probe_stream")
    return out.value


def _stream_handle(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def gemm_abi_version():
    return int(_lib.gemm_abi_version())


def gemm_strerror(status):
    return _lib.gemm_strerror(int(status)).decode()


def _check(rc, where):
    if rc != 0:
        raise GemmError(rc, where)


def gemm_select(M, N, K, dtype):
    cfg = gemm_cfg()
    _check(_lib.gemm_select(M, N, K, dtype, ctypes.byref(cfg)), "gemm_select")
    return cfg


def gemm_select_ex(M, N, K, dtype, b_layout):
    cfg = gemm_cfg()
    _check(_lib.gemm_select_ex(M, N, K, dtype, b_layout, ctypes.byref(cfg)), "gemm_select_ex")
    return cfg


def gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout):
    """Returns the cfg, or None when variant idx is not legal for the shape."""
    cfg = gemm_cfg()
    rc = _lib.gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout, ctypes.byref(cfg))
    if rc == -4:
        return None
    _check(rc, "gemm_cfg_at_ex")
    return cfg


_lib.gemm_select_batched.restype = _int
_lib.gemm_select_batched.argtypes = [_i64, _i64, _i64, _i64, _int, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_cfg_at_batched.restype = _int
_lib.gemm_cfg_at_batched.argtypes = [_int, _i64, _i64, _i64, _i64, _int, _int, ctypes.POINTER(gemm_cfg)]


def gemm_select_batched(M, N, K, batch, dtype, b_layout=0):
    cfg = gemm_cfg()
    _check(_lib.gemm_select_batched(M, N, K, batch, dtype, b_layout, ctypes.byref(cfg)), "gemm_select_batched")
    return cfg


def gemm_cfg_at_batched(idx, M, N, K, batch, dtype, b_layout=0):
    """Returns the cfg, or None when variant idx is not legal for the shape and batch."""
    cfg = gemm_cfg()
    rc = _lib.gemm_cfg_at_batched(idx, M, N, K, batch, dtype, b_layout, ctypes.byref(cfg))
    if rc == -4:
        return None
    _check(rc, "gemm_cfg_at_batched")
    return cfg


def gemm_cfg_count(dtype):
    n = _lib.gemm_cfg_count(dtype)
    if n < 0:
        raise GemmError(n, "gemm_cfg_count")
    return n


def gemm_cfg_at(idx, M, N, K, dtype):
    """Returns the cfg, or None when variant idx is not legal for the shape."""
    cfg = gemm_cfg()
    rc = _lib.gemm_cfg_at(idx, M, N, K, dtype, ctypes.byref(cfg))
    if rc == -4:
        return None
    _check(rc, "gemm_cfg_at")
    return cfg


def gemm_predict(cfg):
    p = gemm_prediction()
    _check(_lib.gemm_predict(ctypes.byref(cfg), ctypes.byref(p)), "gemm_predict")
    return p


def gemm_hw_get():
    h = gemm_hw()
    _check(_lib.gemm_hw_get(ctypes.byref(h)), "gemm_hw_get")
    return h


def gemm_hw_set(h):
    _check(_lib.gemm_hw_set(ctypes.byref(h)), "gemm_hw_set")


GEMM_HW_MI355X, GEMM_HW_MI300X_LIKE = 0, 1


def gemm_hw_preset(hw_id):
    hw = gemm_hw()
    _check(_lib.gemm_hw_preset(int(hw_id), ctypes.byref(hw)), "gemm_hw_preset")
    return hw


def gemm_hw_reset():
    _check(_lib.gemm_hw_reset(), "gemm_hw_reset")


class gemm_sk_segment(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("tile_m", "tile_n", "slab0", "count", "complete", "sk_tile")]


_lib.gemm_stream_k_plan.restype = _int
_lib.gemm_stream_k_plan.argtypes = [ctypes.POINTER(gemm_cfg), ctypes.POINTER(ctypes.c_int32)]
_lib.gemm_stream_k_segments.restype = _int
_lib.gemm_stream_k_segments.argtypes = [ctypes.POINTER(gemm_cfg), _int, ctypes.POINTER(gemm_sk_segment)]


_lib.gemm_stream_k_contributors.restype = _int
_lib.gemm_stream_k_contributors.argtypes = [ctypes.POINTER(gemm_cfg), _int, ctypes.POINTER(ctypes.c_int32)]


def gemm_stream_k_contributors(cfg, sk_tile):
    """(first worker, last worker, segment number of the first worker's partial) of a stream-K tile."""
    out = (ctypes.c_int32 * 3)()
    _check(_lib.gemm_stream_k_contributors(ctypes.byref(cfg), int(sk_tile), out), "gemm_stream_k_contributors")
    return tuple(out)


def gemm_stream_k_plan(cfg):
    """(workers, sk_tiles, dp_tiles, slabs) of a stream-K cfg."""
    out = (ctypes.c_int32 * 4)()
    _check(_lib.gemm_stream_k_plan(ctypes.byref(cfg), out), "gemm_stream_k_plan")
    return tuple(out)


def gemm_stream_k_segments(cfg, worker):
    """Worker's segments as a list of gemm_sk_segment (at most two)."""
    seg = (gemm_sk_segment * 2)()
    n = _lib.gemm_stream_k_segments(ctypes.byref(cfg), int(worker), seg)
    if n < 0:
        raise GemmError(n, "gemm_stream_k_segments")
    return [seg[i] for i in range(n)]


def gemm_workspace_bytes(cfg):
    return int(_lib.gemm_workspace_bytes(ctypes.byref(cfg)))


def gemm_set_workspace(tensor):
    """Register a caller-owned device tensor (or None) as the split-K workspace."""
    if tensor is None:
        _check(_lib.gemm_set_workspace(None, 0), "gemm_set_workspace")
    else:
        _check(_lib.gemm_set_workspace(tensor.data_ptr(), tensor.numel() * tensor.element_size()),
               "gemm_set_workspace")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def gemm_run(cfg, A, B, C, stream=None):
    """Enqueue C = alpha * A * B + beta * C (cfg.batch problems, cfg.stride_* apart).  stream: a torch.cuda.Stream, a raw hipStream_t int, or
    None for torch's current stream."""
    _check(_lib.gemm_run(ctypes.byref(cfg), _ptr(A), _ptr(B), _ptr(C), ctypes.c_void_p(_stream_handle(stream))),
           "gemm_run")


def gemm_run_noalloc(cfg, A, B, C, stream=None):
    """gemm_run with the library's own built-in workspace (at most GEMM_NOALLOC_WORKSPACE_BYTES); allocates nothing."""
    _check(_lib.gemm_run_noalloc(ctypes.byref(cfg), _ptr(A), _ptr(B), _ptr(C), ctypes.c_void_p(_stream_handle(stream))),
           "gemm_run_noalloc")


class gemm_problem(ctypes.Structure):
    _fields_ = [("M", _i64), ("N", _i64), ("K", _i64), ("lda", _i64), ("ldb", _i64), ("ldc", _i64),
                ("A", _vp), ("B", _vp), ("C", _vp)]


class gemm_group_rec(ctypes.Structure):
    _fields_ = [("A", ctypes.c_uint64), ("B", ctypes.c_uint64), ("C", ctypes.c_uint64)] + [
        (n, ctypes.c_int32) for n in ("M", "N", "K", "lda", "ldb", "ldc", "tiles_m", "tiles_n", "tile_start", "group_m")]


_lib.gemm_variant_count.restype = _int
_lib.gemm_variant_count.argtypes = [_int]
_lib.gemm_select_grouped.restype = _int
_lib.gemm_select_grouped.argtypes = [_int, ctypes.POINTER(gemm_problem), _int, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_cfg_at_grouped.restype = _int
_lib.gemm_cfg_at_grouped.argtypes = [_int, _int, ctypes.POINTER(gemm_problem), _int, _int, ctypes.POINTER(gemm_cfg)]
_lib.gemm_grouped_plan.restype = _int
_lib.gemm_grouped_plan.argtypes = [ctypes.POINTER(gemm_cfg), _int, ctypes.POINTER(gemm_problem),
                                   ctypes.POINTER(gemm_group_rec), ctypes.POINTER(_i64)]
_lib.gemm_grouped_locate.restype = _int
_lib.gemm_grouped_locate.argtypes = [ctypes.POINTER(gemm_cfg), _int, ctypes.POINTER(gemm_group_rec), _i64,
                                     ctypes.POINTER(ctypes.c_int32)]
_lib.gemm_run_grouped.restype = _int
_lib.gemm_run_grouped.argtypes = [ctypes.POINTER(gemm_cfg), _int, ctypes.POINTER(gemm_group_rec), _vp, _vp]


def gemm_variant_count(dtype):
    n = _lib.gemm_variant_count(dtype)
    if n < 0:
        raise GemmError(n, "gemm_variant_count")
    return n


def make_problems(shapes, b_layout=0, tensors=None):
    """ctypes array of gemm_problem from [(M, N, K), ...] with dense leading dimensions; tensors:
    optional [(A, B, C), ...] of device tensors (None entries allowed for empty groups)."""
    arr = (gemm_problem * len(shapes))()
    for i, (M, N, K) in enumerate(shapes):
        arr[i].M, arr[i].N, arr[i].K = M, N, K
        arr[i].lda, arr[i].ldb, arr[i].ldc = K, (K if b_layout else N), N
        if tensors is not None:
            A, B, C = tensors[i]
            arr[i].A = A.data_ptr() if A is not None else None
            arr[i].B = B.data_ptr() if B is not None else None
            arr[i].C = C.data_ptr() if C is not None else None
    return arr


def gemm_select_grouped(problems, dtype, b_layout=0):
    cfg = gemm_cfg()
    _check(_lib.gemm_select_grouped(len(problems), problems, dtype, b_layout, ctypes.byref(cfg)), "gemm_select_grouped")
    return cfg


def gemm_cfg_at_grouped(variant, problems, dtype, b_layout=0):
    """Returns the grouped cfg of a variant, or None when it cannot run every group."""
    cfg = gemm_cfg()
    rc = _lib.gemm_cfg_at_grouped(variant, len(problems), problems, dtype, b_layout, ctypes.byref(cfg))
    if rc == -4:
        return None
    _check(rc, "gemm_cfg_at_grouped")
    return cfg


def gemm_grouped_locate(cfg, table, workgroup):
    """(record index, tile_m, tile_n) of a workgroup of the grouped launch, or (-1, -1, -1) when idle."""
    out = (ctypes.c_int32 * 3)()
    _check(_lib.gemm_grouped_locate(ctypes.byref(cfg), len(table), table, int(workgroup), out), "gemm_grouped_locate")
    return tuple(out)


def gemm_grouped_plan(cfg, problems):
    """(host table as a ctypes array of gemm_group_rec, workgroups of the launch)."""
    table = (gemm_group_rec * len(problems))()
    total = _i64()
    _check(_lib.gemm_grouped_plan(ctypes.byref(cfg), len(problems), problems, table, ctypes.byref(total)),
           "gemm_grouped_plan")
    return table, total.value


def table_to_device(table, device="cuda"):
    """The plan's records, byte for byte, in a device tensor (the caller keeps it alive)."""
    raw = bytes(table)
    return torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(device)


def gemm_run_grouped(cfg, table, dev_table, stream=None):
    """Enqueue the grouped launch: table from gemm_grouped_plan, dev_table its copy in device memory."""
    _check(_lib.gemm_run_grouped(ctypes.byref(cfg), len(table), table, _ptr(dev_table),
                                 ctypes.c_void_p(_stream_handle(stream))), "gemm_run_grouped")
