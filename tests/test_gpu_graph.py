"""The layer step captured in a HIP graph (through torch's capture stream): the library allocates nothing, clears
nothing with memset nodes and forks/joins its helper stream with events, so a captured forward + backward must
replay to the bits of the plain launches, on every replay, with other work on the GPU between the replays."""
import pytest
import torch

import workloads as W
from paper_2302_08005_amd import binding as B

pytestmark = pytest.mark.gpu

CASES = [
    W.LayerConfig("graph-postln-bf16", 2, 200, 384, 6, 1000, causal=0, dropout_p=0.1, dtype=W.BF16, len_lo=50, len_hi=200, config_id=51),
    W.LayerConfig("graph-llama-bf16-checkpoint", 2, 128, 256, 4, 344, causal=1, dropout_p=0.1, dtype=W.BF16, pre_ln=1,
                  ln_eps=1e-6, arch=W.LLAMA, config_id=52),
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_captured_step_replays_to_the_same_bits(cfg):
    params = W.make_params(cfg, perturbed=True)
    x_np, dy_np, sl_np = W.make_inputs(cfg)
    layer = B.Layer(cfg, params, checkpoint=1 if "checkpoint" in cfg.name else 0)
    x, dy = layer.to_device(x_np), layer.to_device(dy_np)
    sl = None if sl_np is None else torch.from_numpy(sl_np).to("cuda:0")
    y, dx = torch.empty_like(x), torch.empty_like(x)

    def step():
        B.slapo_layer_fwd(layer.desc, layer.params, x, sl, y, layer.saved, layer.scratch)
        B.slapo_layer_bwd(layer.desc, layer.params, x, sl, dy, layer.saved, dx, layer.grads, layer.scratch)

    step()
    torch.cuda.synchronize()
    want = [y.clone(), dx.clone()] + [layer.grads[k].clone() for k in W.param_names(cfg)]

    side = torch.cuda.Stream()                      # warm-up on a side stream, as torch's capture protocol asks
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        for t in [y, dx] + [layer.grads[k] for k in W.param_names(cfg)]:
            t.fill_(7.0)                            # eager work between the replays; results must come from the graph
        layer.scratch.fill_(0x3C)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [y, dx] + [layer.grads[k] for k in W.param_names(cfg)]
        for i, (g, w) in enumerate(zip(got, want)):
            assert torch.equal(g, w), (replay, i)
