"""Device-side copies of a seeded layer (inputs.make_layer) and one helper that calls a layer
entry point on them.  Marshalling only: tensors are created with PyTorch (device memory), every
step of the layer runs in the HIP library through binding.py.  Used by bench.py, by
__graft_entry__.smoke() and by the GPU tests."""
import numpy as np
import torch

from . import binding as B
from . import inputs

DEV = "cuda:0"

def to_dev(a, dtype, ld=None):
    """float32 numpy array whose values are representable in `dtype` -> device tensor.  With
    `ld` the rows (last axis) are stored `ld` elements apart and the result is a view of the
    padded storage; the padding holds a huge value, so that a kernel that reads it is caught."""
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = inputs.bf16_bits(a)
        t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(DEV)
    else:
        t = torch.from_numpy(a).to(DEV)
    if ld is None or ld == a.shape[-1]:
        return t
    store = torch.full(a.shape[:-1] + (ld,), 3.0e38, dtype=t.dtype, device=DEV)
    store[..., :a.shape[-1]] = t
    return store[..., :a.shape[-1]]


def to_host(t):
    return t.detach().float().cpu().numpy()


class DevLayer:
    """Device copies of a layer dict from inputs.make_layer, plus the weights struct."""

    def __init__(self, L, dtype, pad_weights=False):
        self.dtype = dtype
        self.code = B.BF16 if dtype == "bf16" else B.F32
        act = lambda k: to_dev(L.get(k), dtype)
        # expert weights, optionally with the padded row stride the library recommends
        wgt = lambda k: to_dev(L.get(k), dtype,
                               B.scmoe_padded_ld(L[k].shape[-1], self.code) if pad_weights and L.get(k) is not None
                               else None)
        f32 = lambda k: to_dev(L.get(k), "f32")
        self.x_prev, self.x_cur = act("x_prev"), act("x_cur")
        self.Wg, self.bias = f32("Wg"), f32("bias")
        self.W1, self.W2, self.W1s, self.W2s = wgt("W1"), wgt("W2"), wgt("W1s"), wgt("W2s")
        self.b1, self.b2, self.b1s, self.b2s = f32("b1"), f32("b2"), f32("b1s"), f32("b2s")
        self.Wcg = f32("Wcg")
        self.weights = B.make_weights(self.Wg, self.W1, self.W2, self.W1s, self.W2s, self.bias, self.b1,
                                      self.b2, self.b1s, self.b2s, self.Wcg)
        self.E, self.F, self.d = self.W1.shape
        self.T = self.x_cur.shape[0]
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32


def run_layer(D, k=1, capacity=None, shared=True, normalize=0, cg_mode=0, gelu_mode=0, residual=False,
              two_streams=False):
    """Call the layer entry point; returns (y numpy float32, routing dict of numpy arrays)."""
    T, E = D.T, D.E
    C_ = T * k if capacity is None else capacity
    desc = B.make_desc(T, D.d, D.F, E, k, C_, D.code, gelu_mode, normalize, cg_mode)
    ws = torch.empty(B.scmoe_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    y = torch.full((T, D.d), float("nan"), dtype=D.tdtype, device=DEV)   # a row left unwritten fails the comparison
    rows = min(T * k, E * C_)
    r = dict(expert_idx=torch.empty(T * k, dtype=torch.int32, device=DEV),
             gate_w=torch.empty(T * k, dtype=torch.float32, device=DEV),
             counts=torch.empty(E, dtype=torch.int32, device=DEV),
             offsets=torch.empty(E + 1, dtype=torch.int32, device=DEV),
             dst_row=torch.empty(T * k, dtype=torch.int32, device=DEV),
             src_token=torch.full((max(rows, 1),), -1, dtype=torch.int32, device=DEV))
    rout = B.make_routing_out(**r)
    if shared:
        aux = torch.cuda.Stream() if two_streams else None
        B.scmoe_layer_forward(desc, D.x_prev, D.x_cur, D.weights, y, ws,
                              residual=D.x_cur if residual else None, routing=rout, stream_aux=aux)
    else:
        B.moe_topk_layer_forward(desc, D.x_cur, D.weights, y, ws, routing=rout)
    torch.cuda.synchronize()
    out = {n: t.cpu().numpy() for n, t in r.items()}
    Kk = int(out["offsets"][E])
    routing = dict(idx=out["expert_idx"].reshape(T, k), w=out["gate_w"].reshape(T, k), counts=out["counts"],
                   offsets=out["offsets"], dst_row=out["dst_row"].reshape(T, k),
                   src_token=out["src_token"][:Kk])
    return to_host(y), routing
