"""A stack of MoE layers driven through the C library: the multi-layer workload of the benchmark.

The MoE layers are the library's (`moe_layer`, one call per layer, with the next layer's gate for
the prediction of DAOP Sec. III observation 3).  What sits between them in a real model
(attention, normalisation) is outside this build, so the harness replaces it by parameter-free
glue, computed here with torch ops and stated as a stand-in:

    u_l = h_l / sqrt(mean(h_l^2) + 1e-6)   (fp32, rounded to the storage type)  -> the layer input x
    h_{l+1} = h_l + MoE_l(u_l)             (fp32, kept by the harness)

The prediction for layer l+1 is made from u_l (the hidden state layer l's gate sees); the "actual"
routing of layer l+1 sees u_{l+1}.  Per layer the harness keeps the expert activation counts
(prefill and decode separately: the two L x E matrices of Eq. 1) and the agreement between
predicted and actual experts.
"""
from __future__ import annotations

import torch

from . import moe, synth


def rms_norm(h: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    """The glue's parameter-free RMS normalisation (fp32 arithmetic, one rounding)."""
    return (h * torch.rsqrt(h.pow(2).mean(dim=1, keepdim=True) + 1e-6)).to(dtype)


class MoeStack:
    """`n_layers` resident MoE layers of one shape with seeded synthetic weights (seed = layer index)
    and a Zipf gate bias whose expert ranking is permuted per layer."""

    def __init__(self, n_layers: int, H: int, F: int, E: int, k: int, dtype=torch.bfloat16, device="cuda",
                 zipf_s: float | None = 1.2, max_tokens: int = 1024):
        self.L, self.H, self.F, self.E, self.k, self.dtype, self.device = n_layers, H, F, E, k, dtype, device
        self.shape = moe.make_shape(H, F, E, k, dtype)
        self.layers = []
        for l in range(n_layers):
            d = synth.moe_layer_inputs(1, H, F, E, dtype, device, seed=l, zipf_s=None, with_next=False)
            d.pop("x")
            d["bias"] = None if zipf_s is None else synth.zipf_gate_bias(E, zipf_s, device, perm_seed=l)
            self.layers.append(d)
        self.max_tokens = max_tokens
        self.y = torch.empty((max_tokens, H), dtype=dtype, device=device)
        self.idx = torch.empty((n_layers, max_tokens, k), dtype=torch.int32, device=device)
        self.w = torch.empty((max_tokens, k), dtype=torch.float32, device=device)
        self.pred = torch.empty((n_layers, max_tokens, k), dtype=torch.int32, device=device)
        self.workspace = moe.alloc_workspace(self.shape, max_tokens, device)
        self._epad = (E + 3) // 4 * 4   # rows of the count matrices stay 16-byte aligned

    def new_counts(self) -> torch.Tensor:
        """A zeroed L x E count matrix (int32; row stride padded to 16 bytes, use counts[:, :E])."""
        return torch.zeros((self.L, self._epad), dtype=torch.int32, device=self.device)

    def weight_bytes(self) -> int:
        return sum(t.numel() * t.element_size() for d in self.layers for t in d.values() if t is not None)

    def forward(self, h0: torch.Tensor, counts: torch.Tensor, keep_inputs: bool = False, keep_outputs: bool = False):
        """Runs all layers on the fp32 hidden states h0 [T, H]; adds each layer's activation counts to
        its row of `counts` (from new_counts()).  Returns a dict with the final hidden state, the
        selections idx [L, T, k], the predictions pred [L - 1, T, k] (pred[l] = layer l's prediction
        of layer l + 1) and, on request, the per-layer inputs u_l and outputs y_l."""
        T = h0.shape[0]
        assert T <= self.max_tokens and h0.dtype == torch.float32
        h = h0
        inputs, outputs = [], []
        for l, d in enumerate(self.layers):
            u = rms_norm(h, self.dtype)
            nxt = self.layers[l + 1] if l + 1 < self.L else None
            moe.moe_layer(self.shape, u, d["wg"], d["bias"], nxt["wg"] if nxt else None, nxt["bias"] if nxt else None,
                          d["w1"], d["w3"], d["w2"], self.y[:T], self.idx[l, :T], self.w[:T],
                          counts[l, : self.E], True, self.pred[l, :T] if nxt else None, self.workspace)
            h = h + self.y[:T].float()
            if keep_inputs:
                inputs.append(u)
            if keep_outputs:
                outputs.append((self.y[:T].clone(), self.w[:T].clone()))
        return {"h": h, "idx": self.idx[:, :T], "pred": self.pred[: self.L - 1, :T], "inputs": inputs, "outputs": outputs}


class CapturedStep:
    """One forward pass of a MoeStack on `tokens` tokens recorded into a HIP graph: a decode step of a
    deep stack is a few hundred short launches, which the host cannot issue as fast as the GPU runs
    them.  Write the hidden states into `h_in`, call replay(), read `out` (the dict forward() returns,
    in static buffers) and `counts` (accumulated over the replays)."""

    def __init__(self, st: MoeStack, tokens: int, counts: torch.Tensor):
        self.h_in = torch.zeros((tokens, st.H), dtype=torch.float32, device=st.device)
        self.counts = counts
        scratch = st.new_counts()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):      # warm-up outside the capture (one-time kernel attribute calls)
            st.forward(self.h_in, scratch)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.out = st.forward(self.h_in, counts)
        torch.cuda.synchronize()
        counts.zero_()      # a capture executes nothing, but leave no doubt about where the counts start

    def replay(self):
        self.graph.replay()
        return self.out


def agreement(pred: torch.Tensor, actual: torch.Tensor):
    """Agreement of predicted with actual expert sets.  pred [L - 1, T, k] (layer l's prediction of
    layer l + 1), actual [L, T, k].  Returns per-layer (exact-set match rate, mean overlap / k) for
    layers 1 .. L - 1, as fp64 tensors."""
    act = actual[1:]
    k = pred.shape[-1]
    common = (pred.unsqueeze(-1) == act.unsqueeze(-2)).any(-1).sum(-1)   # [L - 1, T] experts in both sets
    exact = (common == k).double().mean(dim=1)
    overlap = common.double().mean(dim=1) / k
    return exact, overlap


def forward_precalc(st: MoeStack, h0: torch.Tensor, on_gpu: torch.Tensor, first_predicted_layer: int = 5,
                    keep_layers: bool = False):
    """The decode-phase approximation of DAOP (Sec. IV-C) on the stack, for measuring what it does
    to the outputs.

    on_gpu: uint8 [L, E] expert cache.  Layers below `first_predicted_layer` run exactly (the paper
    uses the original gate for the first blocks: prediction for block i + 1 is applied when i >= 4).
    From that layer on, the experts of layer l are the ones PREDICTED from layer l - 1's input
    u_{l-1} with layer l's gate, gracefully degraded against the cache (`daop_predict_degraded`),
    with the predicted weights; a selected expert that is outside the cache is evaluated on the stale
    input u_{l-1} (it was pre-calculated one layer ahead), one inside the cache on the true input
    u_l (one `moe_expert_ffn_precalc` call per layer).  Returns the final hidden state (fp32) and the number of (token, selection) pairs evaluated
    on stale input; with keep_layers also the per-layer (u_prev, u, idx, w, stale mask, y).
    """
    from . import policy

    T = h0.shape[0]
    dev, dt, k, E = st.device, st.dtype, st.k, st.E
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    w = torch.empty((T, k), dtype=torch.float32, device=dev)
    counts = torch.zeros((st._epad,), dtype=torch.int32, device=dev)
    y = torch.empty((T, st.H), dtype=dt, device=dev)
    h = h0
    u_prev = None
    n_stale = 0
    layers = []
    for l, d in enumerate(st.layers):
        u = rms_norm(h, dt)
        if l < first_predicted_layer or u_prev is None:
            moe.moe_route(st.shape, u, d["wg"], d["bias"], idx, w, counts[:E], False, st.workspace)
            moe.moe_expert_ffn(st.shape, u, idx, w, d["w1"], d["w3"], d["w2"], y, st.workspace)
            out = y.float()
            stale = None
        else:
            row = on_gpu[l].clone()   # its own allocation: the library wants 16-byte aligned pointers
            policy.daop_predict_degraded(st.shape, u_prev, d["wg"], d["bias"], row, idx, w)
            stale = (row[idx.long()] == 0).to(torch.uint8)     # [T, k]: selected expert is outside the cache
            moe.moe_expert_ffn_precalc(st.shape, u, u_prev, stale, idx, w, d["w1"], d["w3"], d["w2"], y, st.workspace)
            out = y.float()
            n_stale += int(stale.sum().item())
        if keep_layers:
            layers.append((u_prev, u, idx.clone(), w.clone(), None if stale is None else stale.clone(), out.clone()))
        h = h + out
        u_prev = u
    return {"h": h, "stale_selections": n_stale, "layers": layers}
