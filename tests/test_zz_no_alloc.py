"""The entry point that allocates nothing (bl_gemm_w158a8_noalloc) against the existing one
(bl_gemm_w158a8 with a caller workspace): identical int32 accumulators and identical fp32
outputs, on two calls in a row, the second with a smaller input (the static scratch keeps
the first call's contents)."""
import numpy as np
import pytest

import oracle
import synth
from helpers import to_dev

pytestmark = pytest.mark.gpu


def _case(seed, M, N, K, dev):
    import torch
    from paper_2504_12285_amd import binding as bl
    W = synth.latent_weights(seed, N, K, layer=3, matrix="o")
    X = synth.activations_bf16(seed, M, K, layer=3, matrix="o")
    packed, beta = bl.bl_pack_ternary(to_dev(W), bl.BL_LAYOUT_K16)
    q, scale, _ = bl.bl_quant_act_int8(to_dev(X))
    return packed, beta, q, scale


def test_noalloc_matches_workspace_entry_point_twice():
    import torch
    from paper_2504_12285_amd import binding as bl
    dev = torch.device("cuda:0")
    lib = bl.load()
    for seed, M, N, K in ((11, 300, 640, 1280), (12, 37, 132, 448)):   # second call: smaller, ragged
        packed, beta, q, scale = _case(seed, M, N, K, dev)
        acc_ref, y_ref = bl.bl_gemm_w158a8(packed, beta, bl.BL_LAYOUT_K16, q, scale, None, N)
        acc = torch.full((M, N), -7, dtype=torch.int32, device=dev)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        rc = lib.bl_gemm_w158a8_noalloc(packed.data_ptr(), beta.data_ptr(), bl.BL_LAYOUT_K16, q.data_ptr(),
                                        scale.data_ptr(), M, N, K, acc.data_ptr(), y.data_ptr(),
                                        torch.cuda.current_stream().cuda_stream)
        assert rc == 0, bl.status_str(rc)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
        assert np.array_equal(acc.cpu().numpy(), acc_ref.cpu().numpy())
        assert np.array_equal(y.cpu().numpy().view(np.uint32), y_ref.cpu().numpy().view(np.uint32))
        # and against the oracle itself
        Wt = oracle.ternarize(synth.latent_weights(seed, N, K, layer=3, matrix="o"),
                              oracle.absmean_beta(synth.latent_weights(seed, N, K, layer=3, matrix="o")))
        assert np.array_equal(acc.cpu().numpy(), oracle.matmul_i32(q.cpu().numpy(), Wt))


def test_noalloc_rejects_sizes_beyond_the_scratch():
    import torch
    from paper_2504_12285_amd import binding as bl
    dev = torch.device("cuda:0")
    lib = bl.load()
    t = torch.zeros(4096, dtype=torch.uint8, device=dev)
    p = t.data_ptr()
    assert lib.bl_gemm_w158a8_noalloc(p, p, 1, p, p, 16385, 64, 64, p, p, None) == 2
