"""rq_block_forward under stream capture: the pass (one stream, and the two halves of the batch forked onto the context's second
stream and joined again) recorded into a HIP graph and replayed gives the bits of the eager pass, on every replay and with
other work in between."""
import pytest
import torch

from paper_2402_05628_amd import synth
from tests.helpers import dev

pytestmark = pytest.mark.gpu


def _raw_to_device(raw):
    return {k: (None if v is None else dev(v)) for k, v in raw.items() if k != "x"}


@pytest.mark.parametrize("streams", [1, 3])
def test_block_forward_replays_from_a_graph(streams):
    from paper_2402_05628_amd import binding as b
    cfg = synth.CONFIGS[1].with_batch(8)
    print("case streams", streams, flush=True)
    raw = synth.make_block(cfg, cfg_id=1, seed=5)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x = dev(raw["x"])
        ctx = b.Context(0, stream=side)
        blk = b.calibrate_block(ctx, cfg, _raw_to_device(raw), x, cfg.batch, cfg.seq)
        b.set_block_streams(ctx, streams)
        want = torch.zeros_like(x)
        blk.forward(x, want, cfg.batch, cfg.seq)          # also takes the workspace and does the kernels' one-time set-up
        side.synchronize()
        y = torch.full_like(x, float("nan"))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        blk.forward(x, y, cfg.batch, cfg.seq)
    for rep in range(3):
        y.fill_(float("nan"))
        junk = torch.randn(1 << 20, device="cuda")
        junk.mul_(3.0).sum().item()                       # eager work and a synchronization between the replays
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), "replay %d differs from the eager pass" % rep
    ctx.close()
