"""The library under HIP graph capture: its calls allocate nothing, never synchronise and keep no state, so a
sequence of them recorded once into a graph must give, on every replay, the bits the same calls give when
issued directly.  Each replay runs on fresh input bytes written into the captured buffers, with ordinary eager
work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import paper_2503_20354_amd as surgeon
import surgeon_workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layer_cases():
    # (kind, dtype, shape parameters, group_len, r): one case per family of kernels
    return [
        ("conv", "f32", dict(Nb=4, Ci=32, H=16, W=16, Co=48, k=3, stride=1, pad=1), 4096, 0.9),    # run staging, fp32 MFMA
        ("conv", "bf16", dict(Nb=4, Ci=64, H=8, W=8, Co=128, k=1, stride=1, pad=0), 4096, 0.5),     # un-pack + dense contraction
        ("conv", "bf16", dict(Nb=2, Ci=16, H=14, W=14, Co=32, k=3, stride=2, pad=1), 512, 0.7),     # element staging, strided
        ("linear", "bf16", dict(M=300, K=320, N=136), 320, 0.9),                                  # grouped un-pack, bf16 MFMA
        ("linear", "f32", dict(M=128, K=512, N=256), 512, 0.5),
        ("linear", "f32", dict(M=64, K=512, N=64), 64 * 512, 0.8),                                # whole-tensor selection
    ]


class _Layer:
    def __init__(self, kind, dtype, sh, g, r, seed):
        self.kind, self.dtype, self.sh, self.g, self.r = kind, dtype, sh, g, r
        self.tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        self.dt = surgeon.F32 if dtype == "f32" else surgeon.BF16
        if kind == "conv":
            oh = (sh["H"] + 2 * sh["pad"] - sh["k"]) // sh["stride"] + 1
            ow = (sh["W"] + 2 * sh["pad"] - sh["k"]) // sh["stride"] + 1
            self.a_shape = (sh["Nb"], sh["Ci"], sh["H"], sh["W"])
            self.dy_shape = (sh["Nb"], sh["Co"], oh, ow)
            self.dw_shape = (sh["Co"], sh["Ci"], sh["k"], sh["k"])
        else:
            self.a_shape, self.dy_shape, self.dw_shape = (sh["M"], sh["K"]), (sh["M"], sh["N"]), (sh["N"], sh["K"])
        self.n = int(np.prod(self.a_shape))
        k, _, mask_bytes, ws_sel = surgeon.surgeon_packed_sizes(self.n, g, r, self.dt)
        if kind == "conv":
            self.desc = surgeon.conv2d_desc(sh["Nb"], sh["Ci"], sh["H"], sh["W"], sh["Co"], sh["k"], sh["k"], sh["stride"],
                                            sh["pad"], self.dt, k, group_len=g, r=r)
        else:
            self.desc = surgeon.linear_desc(sh["M"], sh["K"], sh["N"], self.dt, k, group_len=g, r=r)
        self.ws_bytes = max(16, ws_sel, surgeon.surgeon_dw_ws_bytes(self.desc))
        self.A = torch.empty(self.a_shape, dtype=self.tdt, device=DEV)
        self.dY = torch.empty(self.dy_shape, dtype=self.tdt, device=DEV)
        self.seed = seed
        self.out = [self._outputs() for _ in range(2)]  # [0]: written by the graph, [1]: written eagerly

    def _outputs(self):
        return {"vals": torch.zeros(max(self.desc.k_total, 1), dtype=self.tdt, device=DEV),
                "mask": torch.zeros((self.n + 63) // 64, dtype=torch.int64, device=DEV),
                "dW": torch.zeros(self.dw_shape, dtype=torch.float32, device=DEV)}

    def fill(self, round_no):
        self.A.copy_(wl.draw(self.a_shape, "relu" if self.kind == "conv" else "normal", self.dtype,
                             self.seed * 100 + 2 * round_no))
        self.dY.copy_(wl.draw(self.dy_shape, "normal", self.dtype, self.seed * 100 + 2 * round_no + 1))

    def enqueue(self, which, ws):
        o = self.out[which]
        surgeon.surgeon_prune_pack(self.A, self.g, self.r, o["vals"], o["mask"], None, ws)
        surgeon.surgeon_dw_from_packed(self.desc, o["vals"], o["mask"], self.dY, o["dW"], ws)


def test_replays_match_direct_calls():
    surgeon.load_library()
    layers = [_Layer(*c, seed=40 + i) for i, c in enumerate(_layer_cases())]
    G = [torch.zeros(len(layers), dtype=torch.float32, device=DEV) for _ in range(2)]
    ws_bytes = max([L.ws_bytes for L in layers] +
                   [surgeon.surgeon_grad_importance_batched_ws_bytes([L.out[0]["dW"] for L in layers])])
    ws = [torch.empty(ws_bytes, dtype=torch.uint8, device=DEV) for _ in range(2)]

    def enqueue_all(which):
        for L in layers:
            L.enqueue(which, ws[which])
        surgeon.surgeon_grad_importance_batched([L.out[which]["dW"] for L in layers], G[which], ws[which])

    for L in layers:
        L.fill(0)
    enqueue_all(0)  # once outside capture, so that anything the runtime sets up lazily exists already
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue_all(0)
    torch.cuda.synchronize()

    for round_no in range(1, 4):
        print("replay", round_no, flush=True)
        for L in layers:
            L.fill(round_no)
            for t in L.out[0].values():
                t.fill_(-1 if t.dtype == torch.int64 else 7.0)  # stale results must not survive the replay
        G[0].fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        enqueue_all(1)  # the same calls issued directly, into the other set of outputs
        torch.cuda.synchronize()
        for i, L in enumerate(layers):
            k = L.desc.k_total
            for name in ("mask", "vals", "dW"):
                a, b = L.out[0][name], L.out[1][name]
                if name == "vals":
                    a, b = a[:k], b[:k]
                assert np.array_equal(wl.to_numpy_bits(a).view(np.uint8), wl.to_numpy_bits(b).view(np.uint8)), \
                    "layer %d %s differs on replay %d" % (i, name, round_no)
            assert L.out[1]["dW"].abs().sum().item() > 0
        assert torch.equal(G[0], G[1])
        assert bool((G[1] > 0).all())
