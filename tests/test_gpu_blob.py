"""The block-parameter blob: save a calibrated block, load it into one device arena, same bits out."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2402_05628_amd import synth
from tests.helpers import dev

pytestmark = pytest.mark.gpu


def _raw_to_device(raw):
    return {k: (None if v is None else dev(v)) for k, v in raw.items() if k != "x"}


@pytest.mark.parametrize("cfg_id,batch", [(0, 0), (1, 2), (2, 16), (4, 2)])
def test_saved_and_loaded_block_gives_the_same_bits(tmp_path, cfg_id, batch):
    from paper_2402_05628_amd import binding as b
    cfg = synth.CONFIGS[cfg_id] if batch == 0 else synth.CONFIGS[cfg_id].with_batch(batch)
    print("case", cfg.name, flush=True)
    raw = synth.make_block(cfg, cfg_id=cfg_id, seed=5)
    x = dev(raw["x"])
    ctx = b.Context(0)
    blk = b.calibrate_block(ctx, cfg, _raw_to_device(raw), x, cfg.batch, cfg.seq)
    y = torch.zeros_like(x)
    blk.forward(x, y, cfg.batch, cfg.seq)
    path = tmp_path / "block.rqb"
    n = b.save_block(blk, str(path))
    data = path.read_bytes()
    assert len(data) == n == b.block_blob_bytes(blk)
    assert b.check_block_blob(data) == n
    h = b.BlobHeader.from_buffer_copy(data)
    assert (h.D, h.H, h.Dm, h.bits_a, h.bits_p) == (cfg.D, cfg.H, cfg.Dm, cfg.bits_a, cfg.bits_p)
    assert (h.rel_bias_elems > 0) == (raw.get("rel_bias") is not None)
    # the arrays in the file are the device arrays
    s_w = np.frombuffer(data, np.float32, count=h.lin[0][0], offset=h.off[5])
    assert np.array_equal(s_w, blk.P["qkv"]["s_w"].cpu().numpy())
    g1 = np.frombuffer(data, np.float32, count=cfg.D, offset=h.off[0])
    assert np.array_equal(g1, blk.P["ln1"]["gamma_t"].cpu().numpy())
    # a second context loads the file and runs the block: same bits, and the loaded block saves to the same bytes
    ctx2 = b.Context(0)
    blk2 = b.load_block(ctx2, str(path))
    del blk
    y2 = torch.zeros_like(x)
    blk2.forward(x, y2, cfg.batch, cfg.seq)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    buf = (C.c_char * n)()
    ctx2.check(b._rq_blob_save(ctx2.handle, C.byref(blk2.bp), h.rel_bias_elems, C.cast(buf, C.c_void_p), n))
    assert bytes(buf) == data


def test_damaged_blob_is_refused_before_anything_is_copied(tmp_path):
    from paper_2402_05628_amd import binding as b
    cfg = synth.CONFIGS[0]
    raw = synth.make_block(cfg, cfg_id=0, seed=5)
    x = dev(raw["x"])
    ctx = b.Context(0)
    blk = b.calibrate_block(ctx, cfg, _raw_to_device(raw), x, cfg.batch, cfg.seq)
    path = tmp_path / "block.rqb"
    b.save_block(blk, str(path))
    data = bytearray(path.read_bytes())
    h = b.BlobHeader.from_buffer_copy(bytes(data))
    for field, value in (("total_bytes", h.total_bytes + 1), ("D", h.D + 4), ("version", 7)):
        bad = b.BlobHeader.from_buffer_copy(bytes(data))
        setattr(bad, field, value)
        p = tmp_path / ("bad_%s.rqb" % field)
        p.write_bytes(bytes(bad) + bytes(data[C.sizeof(b.BlobHeader):]))
        with pytest.raises(b.RqError):
            b.load_block(ctx, str(p))
    short = tmp_path / "short.rqb"
    short.write_bytes(bytes(data[:len(data) // 2]))
    with pytest.raises(b.RqError):
        b.load_block(ctx, str(short))
