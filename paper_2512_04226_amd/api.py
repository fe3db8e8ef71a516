"""`matmul`: the call a user of the paper's library makes -- hand over two tensors, get the product,
with the kernel chosen analytically for the shape (Section V-C: selection costs microseconds and
is cached per shape, no tuning run).  A thin convenience layer over `binding`: it looks up or
makes the cfg, keeps one workspace tensor per device and calls gemm_run; every step of the
computation runs in libgemm355.so.

    C = matmul(A, B)                       # A (M, K), B (K, N): bf16, fp16 or float8_e4m3fn
    C = matmul(X, W, b_k_contiguous=True)  # W stored (N, K), as an nn.Linear weight
"""
import torch

from . import binding as g

_DTYPES = {torch.bfloat16: g.GEMM_BF16, torch.float16: g.GEMM_FP16}
if hasattr(torch, "float8_e4m3fn"):
    _DTYPES[torch.float8_e4m3fn] = g.GEMM_FP8_E4M3

_cfg_cache = {}       # (M, N, K, dtype, b_layout) -> cfg; the selector is deterministic, so this is exact
_workspace = {}       # device index -> tensor


def select(M, N, K, dtype, b_layout=g.GEMM_B_ROW_MAJOR):
    """The analytic pick for a shape, memoised."""
    key = (M, N, K, dtype, b_layout)
    cfg = _cfg_cache.get(key)
    if cfg is None:
        cfg = _cfg_cache[key] = g.gemm_select_ex(M, N, K, dtype, b_layout)
    return cfg


def _ensure_workspace(cfg, device):
    need = g.gemm_workspace_bytes(cfg)
    if not need:
        return
    idx = device.index if device.index is not None else torch.cuda.current_device()
    cur = _workspace.get(idx)
    if cur is None or cur.numel() * 4 < need:
        # A larger buffer replaces the old one.  Launches enqueued earlier -- on whatever stream the caller
        # gave them -- may still be using the old one, and the allocator only knows about torch's current
        # stream: wait for the device before the old buffer can be handed out again.  (Rare: the buffer
        # only ever grows.)
        if cur is not None:
            torch.cuda.synchronize(device)
        cur = _workspace[idx] = torch.empty((need + 3) // 4, dtype=torch.float32, device=device)
    g.gemm_set_workspace(cur)


def matmul(A, B, out=None, alpha=1.0, beta=0.0, b_k_contiguous=False, stream=None):
    """out = alpha * A @ B + beta * out.  A: (M, K) row-major; B: (K, N) row-major, or (N, K)
    row-major with b_k_contiguous=True.  bf16 / fp8 inputs give a bf16 result, fp16 gives fp16."""
    if A.dtype not in _DTYPES or B.dtype != A.dtype:
        raise TypeError("matmul takes two tensors of one dtype out of %s" % sorted(str(d) for d in _DTYPES))
    if A.dim() != 2 or B.dim() != 2 or not A.is_cuda or not B.is_cuda or A.device != B.device:
        raise ValueError("matmul takes two 2-D tensors on one GPU")
    if A.stride(1) != 1 or B.stride(1) != 1:
        raise ValueError("rows of A and B must be contiguous (leading dimensions are free)")
    M, K = A.shape
    N = B.shape[0] if b_k_contiguous else B.shape[1]
    if (B.shape[1] if b_k_contiguous else B.shape[0]) != K:
        raise ValueError("inner dimensions differ")
    dtype = _DTYPES[A.dtype]
    out_dtype = torch.float16 if dtype == g.GEMM_FP16 else torch.bfloat16
    if out is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs out")
        # rows of C start on 16-byte boundaries: a ragged N gets a padded row stride (the result is a view)
        out = torch.empty((M, -(-N // 8) * 8), dtype=out_dtype, device=A.device)[:, :N]
    elif out.shape != (M, N) or out.dtype != out_dtype or out.stride(1) != 1 or out.device != A.device:
        raise ValueError("out must be a (%d, %d) %s tensor with contiguous rows" % (M, N, out_dtype))
    layout = g.GEMM_B_K_CONTIGUOUS if b_k_contiguous else g.GEMM_B_ROW_MAJOR
    cfg = select(M, N, K, dtype, layout).copy()
    cfg.lda, cfg.ldb, cfg.ldc = A.stride(0), B.stride(0), out.stride(0)
    cfg.alpha, cfg.beta = alpha, beta
    with torch.cuda.device(A.device):
        _ensure_workspace(cfg, A.device)
        g.gemm_run(cfg, A, B, out, stream)
    return out
