"""ctypes binding of the BitLinear C-ABI (include/bitlinear.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
libbitlinear_hip.so.  PyTorch supplies device memory and the current stream.
There is no CPU fallback: if the library is missing, load() raises.
"""
import ctypes
import os

from . import build as _build

BL_OK = 0
BL_LAYOUT_ROWMAJOR, BL_LAYOUT_K16, BL_LAYOUT_TRIT5, BL_LAYOUT_KMAJOR = 0, 1, 2, 3
BL_IN_FP32_LATENT, BL_IN_INT8_TERNARY = 0, 1
BL_OP_PACK, BL_OP_QUANT, BL_OP_GEMV, BL_OP_GEMM = 0, 1, 2, 3

_i64, _vp, _ci, _sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/bitlinear.h one to one
SIGNATURES = {
    "bl_version": (_ci, []),
    "bl_status_str": (ctypes.c_char_p, [_ci]),
    "bl_packed_bytes": (_sz, [_i64, _i64, _ci]),
    "bl_padded_k": (_i64, [_i64]),
    "bl_workspace_bytes": (_sz, [_ci, _i64, _i64, _i64]),
    "bl_pack_ternary": (_ci, [_vp, _ci, _i64, _i64, _ci, _vp, _vp, _vp, _vp]),
    "bl_unpack_ternary": (_ci, [_vp, _i64, _i64, _ci, _vp, _vp, _vp]),
    "bl_quant_act_int8": (_ci, [_vp, _i64, _i64, _vp, _vp, _vp, _vp]),
    "bl_gemv_w158a8": (_ci, [_vp, _vp, _ci, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp]),
    "bl_gemm_w158a8": (_ci, [_vp, _vp, _ci, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp]),
    "bl_bitlinear_decode": (_ci, [_vp, _vp, _ci, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "bl_bitlinear_decode_group": (_ci, [_vp, _ci, _ci, _i64, _vp]),
    "bl_quant_act_ex": (_ci, [_vp, _i64, _i64, _vp, _vp, _vp, _vp]),
    "bl_gemm_w158a8_res": (_ci, [_vp, _vp, _ci, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "bl_gemm_w158a8_fused": (_ci, [_vp, _vp, _ci, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp]),
    "bl_quant_from_absmax": (_ci, [_vp, _vp, _i64, _i64, _vp, _vp, _vp, _vp]),
    "bl_stack_table_bytes": (_sz, [_vp, _ci]),
    "bl_stack_table_bytes_batched": (_sz, [_vp, _ci, _i64]),
    "bl_stack_build": (_ci, [_vp, _ci, _ci, _i64, _vp, _vp, _vp]),
    "bl_stack_run": (_ci, [_vp, _vp, _vp]),
    "bl_debug_force_path": (_ci, [_ci]),
    "bl_probe_stream_read": (_ci, [_vp, _sz, _ci, _vp, _vp]),
    "bl_probe_stream_write": (_ci, [_vp, _i64, _i64, _ci, _vp]),
    "bl_probe_mfma_i8": (_ci, [_ci, _vp, _vp, _vp]),
    "bl_probe_mfma_i8_ex": (_ci, [_ci, _vp, _vp, _vp, _vp, _vp]),
    "bl_probe_wall_clock_khz": (_ci, []),
    "bl_debug_clock_stamps": (_ci, [_vp]),
    "bl_gemm_w158a8_noalloc": (_ci, [_vp, _vp, _ci, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp]),
}

BL_PROD_BF16, BL_PROD_F32, BL_PROD_ATTN_V, BL_PROD_RESIDUAL, BL_PROD_RELU2_GATE = 0, 1, 2, 3, 4


class Producer(ctypes.Structure):
    """Mirror of bl_producer."""
    _fields_ = [("kind", _ci), ("in0", _vp), ("in1", _vp), ("aux_out", _vp),
                ("n_q", _ci), ("n_kv", _ci), ("head_dim", _ci),
                ("norm", _ci), ("gain", _vp), ("eps", ctypes.c_float)]


def make_producer(kind, in0, in1=None, aux_out=None, n_q=0, n_kv=0, head_dim=0, norm=False, gain=None, eps=1e-5):
    """norm=True: RMS normalisation (optional fp32 gains [K]) in front of the quantiser."""
    p = Producer()
    p.kind, p.in0, p.in1, p.aux_out = int(kind), _ptr(in0), _ptr(in1), _ptr(aux_out)
    p.n_q, p.n_kv, p.head_dim = int(n_q), int(n_kv), int(head_dim)
    p.norm, p.gain, p.eps = int(bool(norm)), _ptr(gain), float(eps)
    return p


class DecodeDesc(ctypes.Structure):
    """Mirror of bl_decode_desc."""
    _fields_ = [("packed", _vp), ("beta", _vp), ("X", _vp), ("q", _vp), ("scale", _vp), ("rowsum", _vp),
                ("N", _i64), ("K", _i64), ("acc", _vp), ("y", _vp), ("q_out", _vp), ("scale_out", _vp),
                ("fixed_scale", ctypes.c_float), ("prod", Producer), ("residual", _vp)]


BL_EPI_RESIDUAL, BL_EPI_RELU2_GATE = 1, 2


class GemmEpilogue(ctypes.Structure):
    """Mirror of bl_gemm_epilogue."""
    _fields_ = [("kind", _ci), ("residual", _vp), ("y", _vp), ("x_bf16", _vp), ("absmax", _vp)]


class StackPlan(ctypes.Structure):
    """Mirror of bl_stack_plan."""
    _fields_ = [("count", ctypes.c_int32), ("blocks", ctypes.c_int32), ("prep_count", ctypes.c_int32),
                ("inline_count", ctypes.c_int32), ("norm", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
                ("layout", ctypes.c_int32), ("red_ints", ctypes.c_int32),
                ("wg_offset", _i64), ("prep_offset", _i64),
                ("packed_bytes", _i64), ("table_bytes", _i64),
                ("tokens", ctypes.c_int32), ("entries", ctypes.c_int32)]


class BitLinearError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s failed: %s" % (where, status_str(status)))


_lib = None


def load():
    """Load the built library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_PATH):
            raise RuntimeError("libbitlinear_hip.so is not built (run __graft_entry__.build()); "
                               "this package has no fallback path")
        lib = ctypes.CDLL(_build.LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def status_str(status):
    return load().bl_status_str(int(status)).decode()


def _check(status, where):
    if status != BL_OK:
        raise BitLinearError(status, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def bl_version():
    return load().bl_version()


def bl_packed_bytes(N, K, layout=BL_LAYOUT_K16):
    return load().bl_packed_bytes(N, K, layout)


def bl_padded_k(K):
    return load().bl_padded_k(K)


def bl_workspace_bytes(op, M, N, K):
    return load().bl_workspace_bytes(op, M, N, K)


def _workspace(nbytes, device):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def bl_pack_ternary(W, layout=BL_LAYOUT_K16, beta=None):
    """W: cuda fp32 [N][K] latent weights, or cuda int8 ternary with `beta` given.
    Returns (packed uint8 [N*K/4], beta fp32 [1])."""
    import torch
    N, K = W.shape
    assert W.is_cuda and W.is_contiguous()
    nbytes = bl_packed_bytes(N, K, layout)
    if nbytes == 0:
        raise BitLinearError(2 if layout in (0, 1, 2, 3) else 3, "bl_packed_bytes")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    if W.dtype == torch.float32:
        kind = BL_IN_FP32_LATENT
        beta_t = torch.empty(1, dtype=torch.float32, device=W.device)
    elif W.dtype == torch.int8:
        kind = BL_IN_INT8_TERNARY
        beta_t = torch.as_tensor([float(beta)], dtype=torch.float32, device=W.device) \
            if not isinstance(beta, torch.Tensor) else beta
    else:
        raise TypeError("W must be float32 or int8")
    ws = _workspace(bl_workspace_bytes(BL_OP_PACK, 0, N, K), W.device)
    _check(load().bl_pack_ternary(_ptr(W), kind, N, K, layout, _ptr(packed), _ptr(beta_t), _ptr(ws), _stream()),
           "bl_pack_ternary")
    return packed, beta_t


def bl_unpack_ternary(packed, N, K, layout=BL_LAYOUT_K16):
    """Returns (Wt int8 [N][K], bad int32 [1])."""
    import torch
    Wt = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    bad = torch.empty(1, dtype=torch.int32, device=packed.device)
    _check(load().bl_unpack_ternary(_ptr(packed), N, K, layout, _ptr(Wt), _ptr(bad), _stream()),
           "bl_unpack_ternary")
    return Wt, bad


def bl_quant_act_int8(X, want_rowsum=True):
    """X: cuda bfloat16 [M][K].  Returns (q int8 [M][Kp] with Kp = bl_padded_k(K) and zeros in the padding,
    scale fp32 [M], rowsum int32 [M] or None)."""
    import torch
    assert X.is_cuda and X.is_contiguous() and X.dtype == torch.bfloat16
    M, K = X.shape
    q = torch.empty((M, bl_padded_k(K)), dtype=torch.int8, device=X.device)
    scale = torch.empty(M, dtype=torch.float32, device=X.device)
    rowsum = torch.empty(M, dtype=torch.int32, device=X.device) if want_rowsum else None
    _check(load().bl_quant_act_int8(_ptr(X), M, K, _ptr(q), _ptr(scale), _ptr(rowsum), _stream()),
           "bl_quant_act_int8")
    return q, scale, rowsum


def _matmul(fn_name, op, packed, beta, layout, q, scale, rowsum, N, want_acc, want_y, acc, y, workspace, K=None):
    import torch
    M = q.shape[0]
    K = q.shape[1] if K is None else K          # q is [M][Kp]: pass the true K of a ragged matrix explicitly
    assert q.shape[1] == bl_padded_k(K)
    assert q.is_cuda and q.is_contiguous() and q.dtype == torch.int8
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=q.device)
    if want_y and y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=q.device)
    if workspace is None and rowsum is None:
        workspace = _workspace(bl_workspace_bytes(op, M, N, K), q.device)
    fn = getattr(load(), fn_name)
    _check(fn(_ptr(packed), _ptr(beta), layout, _ptr(q), _ptr(scale), _ptr(rowsum), M, N, K,
              _ptr(acc), _ptr(y), _ptr(workspace), _stream()), fn_name)
    return acc, y


def bl_gemv_w158a8(packed, beta, layout, q, scale, rowsum, N, want_acc=True, want_y=True,
                   acc=None, y=None, workspace=None, K=None):
    """Decode product, 1 <= M <= 64.  Returns (acc int32 [M][N] or None, y fp32 [M][N] or None)."""
    return _matmul("bl_gemv_w158a8", BL_OP_GEMV, packed, beta, layout, q, scale, rowsum, N, want_acc, want_y,
                   acc, y, workspace, K)


def bl_gemm_w158a8(packed, beta, layout, q, scale, rowsum, N, want_acc=True, want_y=True,
                   acc=None, y=None, workspace=None, K=None):
    """Prefill product, any M.  Returns (acc, y) like bl_gemv_w158a8."""
    return _matmul("bl_gemm_w158a8", BL_OP_GEMM, packed, beta, layout, q, scale, rowsum, N, want_acc, want_y,
                   acc, y, workspace, K)


def bl_bitlinear_decode(packed, beta, layout, X, N, want_acc=False, want_y=True, want_q=False, acc=None, y=None):
    """Fused decode BitLinear, M <= 4: bf16 X [M][K] -> (acc, y, q, scale)."""
    import torch
    assert X.is_cuda and X.is_contiguous() and X.dtype == torch.bfloat16
    M, K = X.shape
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=X.device)
    if want_y and y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=X.device)
    q = torch.empty((M, K), dtype=torch.int8, device=X.device) if want_q else None
    scale = torch.empty(M, dtype=torch.float32, device=X.device) if want_q else None
    _check(load().bl_bitlinear_decode(_ptr(packed), _ptr(beta), layout, _ptr(X), M, N, K, _ptr(acc), _ptr(y),
                                      _ptr(q), _ptr(scale), _stream()), "bl_bitlinear_decode")
    return acc, y, q, scale


def make_decode_descs(items):
    """items: list of dicts with tensor values for the bl_decode_desc fields
    (packed, beta, X or q/scale/rowsum, acc, y, q_out, scale_out) and int N, K.
    Returns a ctypes array usable with bl_bitlinear_decode_group."""
    arr = (DecodeDesc * len(items))()
    for d, it in zip(arr, items):
        for f in ("packed", "beta", "X", "q", "scale", "rowsum", "acc", "y", "q_out", "scale_out", "residual"):
            setattr(d, f, _ptr(it.get(f)))
        d.N, d.K = int(it["N"]), int(it["K"])
        d.fixed_scale = float(it.get("fixed_scale", 0.0))
        if it.get("prod") is not None:
            d.prod = it["prod"]
    return arr


def bl_bitlinear_decode_group(descs, layout, M):
    """descs: ctypes array from make_decode_descs (host memory)."""
    _check(load().bl_bitlinear_decode_group(descs, len(descs), layout, M, _stream()), "bl_bitlinear_decode_group")


def bl_quant_act_ex(prod, M, K, device, want_rowsum=True, q=None, scale=None, rowsum=None):
    """Producer + quantiser (prefill side).  prod: Producer from make_producer.
    Returns (q int8 [M][K], scale fp32 [M], rowsum int32 [M] or None)."""
    import torch
    if q is None:
        q = torch.empty((M, K), dtype=torch.int8, device=device)
    if scale is None:
        scale = torch.empty(M, dtype=torch.float32, device=device)
    if rowsum is None and want_rowsum:
        rowsum = torch.empty(M, dtype=torch.int32, device=device)
    _check(load().bl_quant_act_ex(ctypes.byref(prod), M, K, _ptr(q), _ptr(scale), _ptr(rowsum), _stream()),
           "bl_quant_act_ex")
    return q, scale, rowsum


def bl_gemm_w158a8_res(packed, beta, layout, q, scale, rowsum, N, residual, want_acc=False, want_y=True,
                       acc=None, y=None, workspace=None):
    """Prefill product with a residual added in the epilogue.  Returns (acc, y)."""
    import torch
    M, K = q.shape
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=q.device)
    if want_y and y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=q.device)
    if workspace is None and rowsum is None:
        workspace = _workspace(bl_workspace_bytes(BL_OP_GEMM, M, N, K), q.device)
    _check(load().bl_gemm_w158a8_res(_ptr(packed), _ptr(beta), layout, _ptr(q), _ptr(scale), _ptr(rowsum), M, N, K,
                                     _ptr(residual), _ptr(acc), _ptr(y), _ptr(workspace), _stream()),
           "bl_gemm_w158a8_res")
    return acc, y


def bl_gemm_w158a8_noalloc(packed, beta, layout, q, scale, N, acc=None, y=None):
    """Prefill product through the entry point that allocates nothing (row sums in the
    library's static device scratch).  The caller passes the outputs; returns (acc, y)."""
    M, K = q.shape
    _check(load().bl_gemm_w158a8_noalloc(_ptr(packed), _ptr(beta), layout, _ptr(q), _ptr(scale), M, N, K,
                                         _ptr(acc), _ptr(y), _stream()), "bl_gemm_w158a8_noalloc")
    return acc, y


class Stack:
    """A product table of the persistent streaming decode kernel: bl_stack_build once,
    bl_stack_run per step.  Holds the device table and keeps the descriptors' tensors alive."""

    def __init__(self, items, layout, M, device):
        import torch
        self.items = items                      # keeps every tensor of the table alive
        self.descs = make_decode_descs(items)
        nbytes = load().bl_stack_table_bytes(self.descs, len(items)) if M == 1 else \
            load().bl_stack_table_bytes_batched(self.descs, len(items), M)
        if nbytes == 0:
            raise BitLinearError(2, "bl_stack_table_bytes")
        self.table = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.plan = StackPlan()
        _check(load().bl_stack_build(self.descs, len(items), layout, M, _ptr(self.table), ctypes.byref(self.plan),
                                     _stream()), "bl_stack_build")

    def run(self):
        _check(load().bl_stack_run(_ptr(self.table), ctypes.byref(self.plan), _stream()), "bl_stack_run")


def bl_gemm_w158a8_fused(packed, beta, layout, q, scale, rowsum, N, kind, x_bf16, absmax, residual=None, y=None,
                         acc=None):
    """Prefill product with a fused producer epilogue (bl_gemm_w158a8_fused).  x_bf16: bf16 [M][N_out]
    out; absmax: fp32 [M], zero before the call."""
    M, K = q.shape
    ep = GemmEpilogue()
    ep.kind, ep.residual, ep.y, ep.x_bf16, ep.absmax = int(kind), _ptr(residual), _ptr(y), _ptr(x_bf16), _ptr(absmax)
    _check(load().bl_gemm_w158a8_fused(_ptr(packed), _ptr(beta), layout, _ptr(q), _ptr(scale), _ptr(rowsum), M, N, K,
                                       ctypes.byref(ep), _ptr(acc), _stream()), "bl_gemm_w158a8_fused")


def bl_quant_from_absmax(X, absmax, q=None, scale=None, rowsum=None):
    """One-pass quantiser of bf16 rows X [M][K] with known row maxima (cleared by the call)."""
    import torch
    M, K = X.shape
    if q is None:
        q = torch.empty((M, K), dtype=torch.int8, device=X.device)
    if scale is None:
        scale = torch.empty(M, dtype=torch.float32, device=X.device)
    if rowsum is None:
        rowsum = torch.empty(M, dtype=torch.int32, device=X.device)
    _check(load().bl_quant_from_absmax(_ptr(X), _ptr(absmax), M, K, _ptr(q), _ptr(scale), _ptr(rowsum), _stream()),
           "bl_quant_from_absmax")
    return q, scale, rowsum
