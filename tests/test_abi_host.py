"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, sizes are right and argument errors are
reported as status codes before any GPU work."""
import ctypes
import os
import re

import pytest

from paper_2504_12285_amd import binding as bl
from paper_2504_12285_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hip_build.LIB_PATH):
        hip_build.build()
    return bl.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bitlinear.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bl_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = _declared_symbols()
    assert {"bl_pack_ternary", "bl_quant_act_int8", "bl_gemv_w158a8", "bl_gemm_w158a8"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
        assert n in bl.SIGNATURES, "binding lacks " + n
    assert sorted(bl.SIGNATURES) == names


def test_sizes(lib):
    assert lib.bl_version() >= 100
    for layout in (0, 1):
        assert lib.bl_packed_bytes(2560, 2560, layout) == 2560 * 2560 // 4
        assert lib.bl_packed_bytes(13824, 2560, layout) == 8847360
        assert lib.bl_packed_bytes(2560, 6912, layout) == 4423680
    assert lib.bl_packed_bytes(2560, 2560, 7) == 0
    # ragged shapes are padded: rows of ceil(K/64)*64 weights, ceil(N/4)*4 rows
    assert lib.bl_packed_bytes(2560, 100, 0) == 2560 * 128 // 4
    assert lib.bl_packed_bytes(6, 128, 0) == 8 * 128 // 4
    assert lib.bl_packed_bytes(1, 1, 1) == 4 * 64 // 4
    assert lib.bl_packed_bytes(0, 64, 0) == 0 and lib.bl_packed_bytes(64, 0, 0) == 0
    assert lib.bl_packed_bytes((1 << 24) + 1, 64, 0) == 0
    assert [lib.bl_padded_k(k) for k in (1, 63, 64, 65, 2560, 6912, 6913)] == [64, 64, 64, 128, 2560, 6912, 6976]
    assert lib.bl_padded_k(0) == 0 and lib.bl_padded_k((1 << 24) + 1) == 0
    assert lib.bl_workspace_bytes(bl.BL_OP_PACK, 0, 2560, 2560) >= 8192
    assert lib.bl_workspace_bytes(bl.BL_OP_GEMM, 2048, 2560, 2560) >= 2048 * 4
    assert b"BL_ERR_SHAPE" in lib.bl_status_str(2)


def test_argument_errors_need_no_gpu(lib):
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) & ~255  # an aligned host address: never dereferenced on error paths
    NULL = None
    # NULL pointers
    assert lib.bl_pack_ternary(NULL, 0, 64, 64, 0, p, p, p, NULL) == 1
    assert lib.bl_quant_act_int8(p, 1, 64, NULL, p, NULL, NULL) == 1
    assert lib.bl_gemv_w158a8(p, p, 0, p, p, NULL, 1, 64, 64, NULL, NULL, NULL, NULL) == 1  # no output
    assert lib.bl_gemv_w158a8(p, p, 0, p, NULL, NULL, 1, 64, 64, NULL, p, NULL, NULL) == 1  # y without scale
    # shapes
    assert lib.bl_pack_ternary(p, 0, 64, 0, 0, p, p, p, NULL) == 2
    assert lib.bl_pack_ternary(p, 0, 0, 64, 0, p, p, p, NULL) == 2
    assert lib.bl_pack_ternary(p, 0, (1 << 24) + 1, 64, 0, p, p, p, NULL) == 2
    assert lib.bl_pack_ternary(p, 0, 6, 100, 0, p, p, NULL, NULL) == 7       # ragged shape: same workspace rule
    assert lib.bl_quant_act_int8(p, 0, 64, p, p, NULL, NULL) == 2
    assert lib.bl_quant_act_int8(p, 1, 0, p, p, NULL, NULL) == 2
    assert lib.bl_gemv_w158a8(p, p, 0, p, p, NULL, 65, 64, 64, p, NULL, NULL, NULL) == 2   # M > 64
    assert lib.bl_gemv_w158a8(p, p, 0, p, p, NULL, 0, 64, 64, p, NULL, NULL, NULL) == 2
    assert lib.bl_gemm_w158a8(p, p, 0, p, p, NULL, 8, 64, 0, p, NULL, NULL, NULL) == 2
    assert lib.bl_gemm_w158a8(p, p, 0, p, p, NULL, 8, 0, 96, p, NULL, NULL, NULL) == 2
    # layout / kind
    assert lib.bl_pack_ternary(p, 0, 64, 64, 5, p, p, p, NULL) == 3
    assert lib.bl_gemv_w158a8(p, p, 9, p, p, NULL, 1, 64, 64, p, NULL, NULL, NULL) == 3
    assert lib.bl_pack_ternary(p, 3, 64, 64, 0, p, p, p, NULL) == 5
    # alignment
    assert lib.bl_gemv_w158a8(p + 4, p, 0, p, p, NULL, 1, 64, 64, p, NULL, NULL, NULL) == 4
    assert lib.bl_gemm_w158a8(p, p, 0, p + 1, p, NULL, 1, 64, 64, p, NULL, NULL, NULL) == 4
    # workspace
    assert lib.bl_pack_ternary(p, 0, 64, 64, 0, p, p, NULL, NULL) == 7


def test_producer_and_group_descriptors_are_checked_on_the_host(lib):
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) & ~255   # never dereferenced on these error paths

    class T:   # stands in for a tensor: only data_ptr() is used by the marshalling code
        def __init__(self, a):
            self.a = a

        def data_ptr(self):
            return self.a
    t = T(p)

    def quant_ex(prod, M=1, K=2560):
        return lib.bl_quant_act_ex(ctypes.byref(prod), M, K, p, p, None, None)
    assert quant_ex(bl.make_producer(9, t)) == 5                                  # unknown kind
    assert quant_ex(bl.make_producer(bl.BL_PROD_RESIDUAL, t)) == 5                # no second operand
    assert quant_ex(bl.make_producer(bl.BL_PROD_ATTN_V, t, n_q=20, n_kv=5, head_dim=64)) == 5   # geometry != K
    assert quant_ex(bl.make_producer(bl.BL_PROD_F32, t, norm=True, eps=-1.0)) == 5             # negative eps
    assert quant_ex(bl.make_producer(bl.BL_PROD_F32, t, norm=True, gain=T(p + 4))) == 5        # misaligned gains
    assert quant_ex(bl.make_producer(bl.BL_PROD_F32, T(0))) == 1                  # no input
    assert quant_ex(bl.make_producer(bl.BL_PROD_F32, t), K=100) == 2
    # grouped decode: count, M limits per input kind, layout
    beta = t
    d_q = bl.make_decode_descs([dict(packed=t, beta=beta, N=64, K=64, y=t, q=t, scale=t)])
    d_x = bl.make_decode_descs([dict(packed=t, beta=beta, N=64, K=64, y=t, X=t)])
    assert lib.bl_bitlinear_decode_group(d_q, 0, 1, 1, None) == 2
    assert lib.bl_bitlinear_decode_group(d_q, 5, 1, 1, None) == 2
    assert lib.bl_bitlinear_decode_group(d_q, 1, 1, 65, None) == 2                # int8 inputs: M <= 64
    assert lib.bl_bitlinear_decode_group(d_x, 1, 1, 17, None) == 2                # fused inputs: M <= 16
    d_x100 = bl.make_decode_descs([dict(packed=t, beta=beta, N=64, K=100, y=t, X=t)])
    assert lib.bl_bitlinear_decode_group(d_x100, 1, 1, 1, None) == 2              # fused inputs: K % 64 == 0
    d_q100 = bl.make_decode_descs([dict(packed=t, beta=beta, N=7, K=100, y=t, q=t, scale=t)])
    assert lib.bl_bitlinear_decode_group(d_q100, 1, 9, 1, None) == 3              # int8 inputs: any N, K (layout checked)
    assert lib.bl_bitlinear_decode_group(d_q, 1, 7, 1, None) == 3
    assert lib.bl_bitlinear_decode_group(None, 1, 1, 1, None) == 1


def test_binding_raises_with_status():
    with pytest.raises(bl.BitLinearError) as e:
        bl._check(2, "bl_gemv_w158a8")
    assert e.value.status == 2 and "BL_ERR_SHAPE" in str(e.value)


def test_noalloc_entry_point_checks_arguments_before_any_gpu_work(lib):
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) & ~255
    assert lib.bl_gemm_w158a8_noalloc(None, p, 1, p, p, 1, 64, 64, p, p, None) == 1      # NULL packed
    assert lib.bl_gemm_w158a8_noalloc(p, p, 1, p, p, 16385, 64, 64, p, p, None) == 2     # beyond the scratch
    assert lib.bl_gemm_w158a8_noalloc(p, p, 1, p, p, 0, 64, 64, p, p, None) == 2
    assert lib.bl_gemm_w158a8_noalloc(p, p, 9, p, p, 1, 64, 64, p, p, None) == 3         # layout
    assert lib.bl_gemm_w158a8_noalloc(p + 4, p, 1, p, p, 1, 64, 64, p, p, None) == 4     # alignment


def test_debug_hook_and_gemv_workspace_status(lib):
    assert lib.bl_debug_force_path(4) == 5 and lib.bl_debug_force_path(-1) == 5
    assert lib.bl_debug_force_path(2) == 0 and lib.bl_debug_force_path(0) == 0
    # a decode product with K > 8192 and no row sums needs the workspace: reported before any GPU work
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) & ~255
    assert lib.bl_gemv_w158a8(p, p, 1, p, p, None, 1, 64, 8256, p, p, None, None) == 7


def test_stack_tables_are_sized_and_checked_on_the_host(lib):
    """bl_stack_* (one-token and batched form): table sizes, descriptor errors and malformed plans are
    host work; nothing here reaches a GPU call."""
    buf = (ctypes.c_char * 8192)()
    p = (ctypes.addressof(buf) + 255) & ~255
    d = (bl.DecodeDesc * 2)()
    for e in d:
        e.packed = e.beta = e.q = e.scale = e.rowsum = e.y = p
        e.N, e.K = 2560, 2560
    d[1].K = 6912
    one = lib.bl_stack_table_bytes(d, 2)
    assert one > 0 and one % 256 == 0
    assert lib.bl_stack_table_bytes(d, 0) == 0 and lib.bl_stack_table_bytes(d, 1025) == 0
    # batched form: more table entries than products once rows are split, scratch for the k parts
    sizes = {M: lib.bl_stack_table_bytes_batched(d, 2, M) for M in (2, 8, 32, 64)}
    assert all(v > 0 and v % 256 == 0 for v in sizes.values())
    assert sizes[32] >= sizes[8] + 32 * 2560 * 4          # the long-k product collects partial sums at M = 32
    assert lib.bl_stack_table_bytes_batched(d, 2, 1) == 0 and lib.bl_stack_table_bytes_batched(d, 2, 65) == 0
    assert lib.bl_stack_table_bytes_batched(d, 0, 8) == 0 and lib.bl_stack_table_bytes_batched(None, 2, 8) == 0
    plan = bl.StackPlan()
    assert lib.bl_stack_build(d, 2, 1, 65, p, ctypes.byref(plan), None) == 2
    assert lib.bl_stack_build(d, 2, 0, 8, p, ctypes.byref(plan), None) == 3        # batched: layout 1 only
    assert lib.bl_stack_build(d, 2, 1, 8, p + 8, ctypes.byref(plan), None) == 4
    d[0].rowsum = None
    assert lib.bl_stack_build(d, 2, 1, 8, p, ctypes.byref(plan), None) == 1        # batched: row sums required
    d[0].rowsum = p
    d[0].X = p
    assert lib.bl_stack_build(d, 2, 1, 8, p, ctypes.byref(plan), None) == 5        # batched: int8 inputs only
    d[0].X = None
    d[1].y = None
    assert lib.bl_stack_build(d, 2, 1, 8, p, ctypes.byref(plan), None) == 1        # no output at all
    # a plan that no build call produced
    bad = bl.StackPlan()
    assert lib.bl_stack_run(p, ctypes.byref(bad), None) == 5
    bad.tokens, bad.count, bad.entries, bad.blocks, bad.lds_bytes, bad.layout = 8, 2, 2, 16, 100, 1
    assert lib.bl_stack_run(p, ctypes.byref(bad), None) == 5
    assert lib.bl_stack_run(None, ctypes.byref(bad), None) == 1
    # the tile route of the batched form (more than 48 tokens): more workgroups than tiles, offsets that
    # no build call laid out, fewer tokens than the route takes
    tile = bl.StackPlan()
    tile.tokens, tile.count, tile.entries, tile.norm, tile.layout, tile.red_ints, tile.blocks = 64, 2, 2, 3, 1, 40, 41
    assert lib.bl_stack_run(p, ctypes.byref(tile), None) == 5
    tile.blocks = 40
    assert lib.bl_stack_run(p, ctypes.byref(tile), None) == 5
    tile.tokens = 8
    assert lib.bl_stack_run(p, ctypes.byref(tile), None) == 5


def test_probe_arguments_are_checked_on_the_host(lib):
    """The measurement aids reject bad arguments before any GPU call."""
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) & ~255
    assert lib.bl_probe_stream_write(None, 128, 128, 0, None) == 1
    assert lib.bl_probe_stream_write(p, 100, 128, 0, None) == 2          # rows not a multiple of 128
    assert lib.bl_probe_stream_write(p, 128, 64, 0, None) == 2
    assert lib.bl_probe_stream_write(p, 128, 128, 9, None) == 2
    assert lib.bl_probe_stream_write(p + 2, 128, 128, 0, None) == 4
    assert lib.bl_probe_stream_read(None, 1024, 0, p, None) == 1
    assert lib.bl_probe_stream_read(p, 24, 0, p, None) == 2
