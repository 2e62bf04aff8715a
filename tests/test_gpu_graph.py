"""HIP-graph replays of a whole training step of the layer against the same step launched
eagerly.  bench.py times graph replays, so a replay must do exactly the work of an eager step:
every replay is compared bit for bit with an eager run on the same inputs (the kernels use no
atomics, so results do not depend on timing), with the program's own eager work and
synchronizations between the replays and new inputs written into the captured buffers each time.
The shapes cover the launch configurations: the 128 x 64 producer / consumer kernel, the
streaming kernels (M <= 16, one and two quantization groups per backward tile; two passes for 24
tokens), the 256 x 256 kernel and its 128-row instantiation with a split contraction and the second launch, and the projection kernel's two forms
(one row tile per workgroup; four that share the factor, with its finish launch), each with the
adapter-gradient launches."""
import pytest
import torch

from paper_2309_16119_amd import binding as b

from gpu_util import to_device
from test_gpu_parity import layer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits,K,N,M,r,group", [
    (3, 2112, 2136, 300, 8, 64),
    (3, 1024, 768, 16, 8, 128),
    (4, 320, 8232, 300, 16, 64),
    (4, 512, 640, 16, 16, 64),        # streaming kernels, two quantization groups per backward tile
    (2, 6400, 520, 1100, 8, 64),      # projection with four row tiles per workgroup, slices of the contraction + finish
    (3, 4096, 1024, 128, 8, 128),     # 128-row instantiation of the 256-column kernel, split contraction + fix-up
    (3, 4096, 4096, 24, 8, 128),      # two passes of the streaming kernels that share the scratch
])
def test_graph_replays_equal_eager_steps(bits, K, N, M, r, group):
    L = layer(bits, K, N, M, r, group, seed=4)
    D = to_device(L)
    s = L["lora_scale"]
    X, dY = D["Xd"].clone(), D["dYd"].clone()
    out = {
        "Y": torch.empty((M, N), dtype=torch.bfloat16, device="cuda"),
        "dX": torch.empty((M, K), dtype=torch.bfloat16, device="cuda"),
        "XA": torch.empty((M, r), dtype=torch.float32, device="cuda"),
        "T": torch.empty((M, r), dtype=torch.float32, device="cuda"),
        "dA": torch.empty((K, r), dtype=torch.float32, device="cuda"),
        "dB": torch.empty((r, N), dtype=torch.float32, device="cuda"),
    }

    def step():
        b.modulora_fwd(D["w"], X, D["Ad"], D["Bd"], s, Y=out["Y"], XA=out["XA"])
        b.modulora_bwd_input(D["w"], dY, D["Ad"], D["Bd"], s, dX=out["dX"], dYBt=out["T"])
        b.modulora_bwd_lora(X, dY, D["Ad"], D["Bd"], s, XA=out["XA"], dYBt=out["T"], dA=out["dA"], dB=out["dB"])

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                   # eager first, on the capture stream: kernel attributes and that stream's
    torch.cuda.synchronize()     # cached workspace exist before the capture
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    gen = torch.Generator(device="cuda").manual_seed(17)
    for rep in range(3):
        X.copy_(torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16))
        dY.copy_(torch.randn((M, N), generator=gen, device="cuda").to(torch.bfloat16))
        for t in out.values():
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        replayed = {k: v.clone() for k, v in out.items()}
        for t in out.values():
            t.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        for k, v in out.items():
            assert not torch.isnan(v.float()).any(), (k, rep)
            assert torch.equal(replayed[k].view(torch.int16) if v.dtype == torch.bfloat16 else replayed[k],
                               v.view(torch.int16) if v.dtype == torch.bfloat16 else v), (k, rep)
