"""Call sequences for the synthetic 2B-style layer chain (benchmark config 4):
four BitLinears per layer joined by fused producers.  Orchestration only: every
arithmetic step runs inside the HIP kernels reached through the C-ABI.

Layer, per token (tokens are independent; the glue is a stand-in, not the
model's attention):  qkv = BL_qkv(bf16(x));  o = BL_o(bf16(V broadcast over its
GQA group));  h1 = x + o;  gu = BL_gu(bf16(h1));  x' = h1 + BL_down(bf16(relu(g)^2 * u)).
Without gains every BitLinear rescales with 1/127 instead of absmax/127 (norm
stand-in).  With gains (a dict name -> fp32 [K] device tensor or None per layer) the
producers apply the RMS normalisation in front of each quantiser and the rescale uses the
true absmax/127.
"""
import numpy as np

from . import binding as bl

SHAPES = {"qkv": (3840, 2560), "o": (2560, 2560), "gate_up": (13824, 2560), "down": (2560, 6912)}
N_Q, N_KV, HEAD_DIM = 20, 5, 128
UNIT_SCALE = float(np.float32(1.0) / np.float32(127.0))


class ChainBuffers:
    """Device tensors reused by every layer of a chain run."""

    def __init__(self, M, device, trace=False):
        import torch
        f32 = dict(dtype=torch.float32, device=device)
        self.M, self.device, self.trace = M, device, trace
        self.qkv = torch.empty((M, 3840), **f32)
        self.o = torch.empty((M, 2560), **f32)
        self.h1 = torch.empty((M, 2560), **f32)
        self.gu = torch.empty((M, 13824), **f32)
        self.x_next = torch.empty((M, 2560), **f32)
        self.unit = torch.full((M,), UNIT_SCALE, **f32)
        # prefill path scratch
        self.q = {k: torch.empty((M, K), dtype=torch.int8, device=device) for k, K in (("h", 2560), ("f", 6912))}
        self.scale = torch.empty(M, **f32)
        self.rowsum = torch.empty(M, dtype=torch.int32, device=device)
        # fused producer epilogues: bf16 inputs of the next BitLinear and their row maxima (kept at zero
        # between uses: the one-pass quantiser clears what the epilogue accumulated)
        self.xb = {k: torch.empty((M, K), dtype=torch.bfloat16, device=device) for k, K in (("h", 2560), ("f", 6912))}
        self.absmax = torch.zeros(M, **f32)
        self.q_valid_for = None       # data_ptr of the residual stream whose int8 form sits in q["h"]


def _producers(x, B, gains=None, eps=1e-5):
    def n(name):
        return {} if gains is None else dict(norm=True, gain=gains.get(name), eps=eps)
    return {
        "qkv": bl.make_producer(bl.BL_PROD_F32, x, **n("qkv")),
        "o": bl.make_producer(bl.BL_PROD_ATTN_V, B.qkv, n_q=N_Q, n_kv=N_KV, head_dim=HEAD_DIM, **n("o")),
        "gate_up": bl.make_producer(bl.BL_PROD_RESIDUAL, x, B.o, B.h1, **n("gate_up")),
        "down": bl.make_producer(bl.BL_PROD_RELU2_GATE, B.gu, **n("down")),
    }


def layer_decode(weights, layout, x, B, records=None, gains=None):
    """One layer for M <= 16 tokens: four fused launches (producer + quantiser +
    product + rescale [+ residual]).  weights: name -> (packed, beta).  x: fp32
    [M][2560].  Returns B.x_next (swap with x for the next layer).  If records is
    a list, int32 accumulators and quantised inputs of each BitLinear are kept."""
    import torch
    M = B.M
    prods = _producers(x, B, gains)
    outs = {"qkv": B.qkv, "o": B.o, "gate_up": B.gu, "down": B.x_next}
    for name in ("qkv", "o", "gate_up", "down"):
        N, K = SHAPES[name]
        packed, beta = weights[name]
        item = dict(packed=packed, beta=beta, N=N, K=K, y=outs[name], prod=prods[name],
                    fixed_scale=UNIT_SCALE if gains is None else 0.0,
                    residual=B.h1 if name == "down" else None)
        if records is not None:
            item["acc"] = torch.empty((M, N), dtype=torch.int32, device=B.device)
            item["q_out"] = torch.empty((M, K), dtype=torch.int8, device=B.device)
            item["scale_out"] = torch.empty(M, dtype=torch.float32, device=B.device)
            records.append(dict(name=name, acc=item["acc"], q=item["q_out"], scale=item["scale_out"], y=outs[name]))
        bl.bl_bitlinear_decode_group(bl.make_decode_descs([item]), layout, M)
        if records is not None:
            records[-1]["y"] = outs[name].clone()
    return B.x_next


def layer_prefill(weights, layout, x, B, records=None, gains=None):
    """One layer for any M.  Without gains (and with the kernel-native layout) the elementwise glue
    runs in the products' epilogues: o -> h1 = x + o, gate_up -> relu(g)^2 * u, down -> x' = h1 + down,
    each written once as bf16 with its row maximum, then quantised in one pass (the input of the qkv
    product of the NEXT layer included).  With gains (RMS normalisation, a float reduction over the
    row) or layout 0: producer + quantiser kernel in front of every product."""
    import torch
    if gains is not None or layout != bl.BL_LAYOUT_K16:
        return _layer_prefill_unfused(weights, layout, x, B, records, gains)
    M, dev = B.M, B.device

    def rec(name, acc, q, y):
        if records is not None:
            records.append(dict(name=name, acc=acc, q=q.clone(), scale=B.scale.clone(), y=y))

    def new_acc(N):
        return torch.empty((M, N), dtype=torch.int32, device=dev) if records is not None else None

    qh, qf = B.q["h"], B.q["f"]
    # qkv: its input was quantised by the previous layer's down epilogue, or comes from outside
    if B.q_valid_for != x.data_ptr():
        bl.bl_quant_act_ex(bl.make_producer(bl.BL_PROD_F32, x), M, 2560, dev, q=qh, scale=B.scale, rowsum=B.rowsum)
    packed, beta = weights["qkv"]
    acc = new_acc(3840)
    bl.bl_gemm_w158a8_res(packed, beta, layout, qh, B.unit, B.rowsum, 3840, None, want_acc=records is not None,
                          acc=acc, y=B.qkv)
    rec("qkv", acc, qh, B.qkv.clone() if records is not None else None)
    # o: context-length-1 attention = V broadcast (a gather, not an epilogue of qkv), then h1 = x + o
    bl.bl_quant_act_ex(bl.make_producer(bl.BL_PROD_ATTN_V, B.qkv, n_q=N_Q, n_kv=N_KV, head_dim=HEAD_DIM), M, 2560, dev,
                       q=qh, scale=B.scale, rowsum=B.rowsum)
    packed, beta = weights["o"]
    acc = new_acc(2560)
    bl.bl_gemm_w158a8_fused(packed, beta, layout, qh, B.unit, B.rowsum, 2560, bl.BL_EPI_RESIDUAL, B.xb["h"], B.absmax,
                            residual=x, y=B.h1, acc=acc)
    rec("o", acc, qh, None)
    # gate_up: input bf16(h1); epilogue relu(g)^2 * u
    bl.bl_quant_from_absmax(B.xb["h"], B.absmax, q=qh, scale=B.scale, rowsum=B.rowsum)
    packed, beta = weights["gate_up"]
    acc = new_acc(13824)
    bl.bl_gemm_w158a8_fused(packed, beta, layout, qh, B.unit, B.rowsum, 13824, bl.BL_EPI_RELU2_GATE, B.xb["f"], B.absmax,
                            acc=acc)
    rec("gate_up", acc, qh, None)
    # down: epilogue x' = h1 + down, and the int8 form of x' for the next layer's qkv
    bl.bl_quant_from_absmax(B.xb["f"], B.absmax, q=qf, scale=B.scale, rowsum=B.rowsum)
    packed, beta = weights["down"]
    acc = new_acc(2560)
    bl.bl_gemm_w158a8_fused(packed, beta, layout, qf, B.unit, B.rowsum, 2560, bl.BL_EPI_RESIDUAL, B.xb["h"], B.absmax,
                            residual=B.h1, y=B.x_next, acc=acc)
    rec("down", acc, qf, None)
    bl.bl_quant_from_absmax(B.xb["h"], B.absmax, q=qh, scale=B.scale, rowsum=B.rowsum)
    B.q_valid_for = B.x_next.data_ptr()
    return B.x_next


def _layer_prefill_unfused(weights, layout, x, B, records=None, gains=None):
    """One layer for any M: producer+quantiser kernel, then the matrix-core
    product (residual fused into the last epilogue)."""
    import torch
    M = B.M
    B.q_valid_for = None
    prods = _producers(x, B, gains)
    outs = {"qkv": B.qkv, "o": B.o, "gate_up": B.gu, "down": B.x_next}
    for name in ("qkv", "o", "gate_up", "down"):
        N, K = SHAPES[name]
        packed, beta = weights[name]
        q = B.q["f" if K == 6912 else "h"]
        bl.bl_quant_act_ex(prods[name], M, K, B.device, q=q, scale=B.scale, rowsum=B.rowsum)
        acc = torch.empty((M, N), dtype=torch.int32, device=B.device) if records is not None else None
        bl.bl_gemm_w158a8_res(packed, beta, layout, q, B.unit if gains is None else B.scale, B.rowsum, N,
                              B.h1 if name == "down" else None,
                              want_acc=records is not None, acc=acc, y=outs[name])
        if records is not None:
            records.append(dict(name=name, acc=acc, q=q.clone(), scale=B.scale.clone(), y=outs[name].clone()))
    return B.x_next


def run_chain(layer_weights, layout, x0, mode="decode", records=None, layer_gains=None):
    """Runs x0 (fp32 [M][2560], device) through the given layers.  mode: "decode"
    (M <= 16, fused launches) or "prefill".  layer_gains: None, or one gains dict per layer
    (RMS normalisation on).  Returns the final x (a device tensor)."""
    M = x0.shape[0]
    B = ChainBuffers(M, x0.device)
    x = x0.clone()
    step = layer_decode if mode == "decode" else layer_prefill
    for li, w in enumerate(layer_weights):
        rec = [] if records is not None else None
        out = step(w, layout, x, B, rec, None if layer_gains is None else layer_gains[li])
        if records is not None:
            records.append(rec)
        B.x_next, x = x, out          # ping-pong: the old input becomes the next output buffer
    return x
