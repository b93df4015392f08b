"""The memory probe (tidal_hbm_probe): the LoRA kernels' walk with the arithmetic taken out.  Its three
forms must touch exactly what they claim: the read form nothing, two read-modify-write passes nothing
net, one such pass one bit per 32-bit word, the write form every word of the matrices and nothing
beyond them."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402


@pytest.mark.parametrize("walk", [1, 3, 16])
def test_probe_forms_touch_what_they_claim(walk):
    assert torch.cuda.is_available()
    rows, cols, n = 96, 768, 5                            # 3 row blocks (a ragged last run for walk 16), 3 strips
    guard = 4096
    g = torch.Generator(device="cpu").manual_seed(walk)
    host = torch.randint(-2 ** 15, 2 ** 15 - 1, (guard + n * rows * cols + guard,), dtype=torch.int16, generator=g)
    mem = host.to("cuda:0")
    body = mem[guard:guard + n * rows * cols]
    assert body.data_ptr() % 16 == 0
    before = host.numpy().copy()
    assert tb.tidal_hbm_probe(body, rows, cols, n, walk, tb.TIDAL_PROBE_READ, 2) > 0
    assert np.array_equal(mem.cpu().numpy(), before)
    assert tb.tidal_hbm_probe(body, rows, cols, n, walk, tb.TIDAL_PROBE_RMW, 1) > 0     # warm-up + 1 pass = 2 passes
    assert np.array_equal(mem.cpu().numpy(), before)
    assert tb.tidal_hbm_probe(body, rows, cols, n, walk, tb.TIDAL_PROBE_RMW, 2) > 0     # 3 passes: one bit per word flipped
    after = mem.cpu().numpy()
    want = before.copy()
    w32 = want[guard:guard + n * rows * cols].view(np.uint32)
    w32 ^= 1
    assert np.array_equal(after, want)
    assert tb.tidal_hbm_probe(body, rows, cols, n, walk, tb.TIDAL_PROBE_WRITE, 1) > 0
    final = mem.cpu().numpy()
    assert np.array_equal(final[:guard], before[:guard]) and np.array_equal(final[-guard:], before[-guard:])
    words = final[guard:guard + n * rows * cols].view(np.uint32).reshape(n, rows, cols // 2)
    # every 16-byte vector holds (row, strip, lane's column group, 0)
    assert np.array_equal(words[:, :, 0::4], np.broadcast_to(np.arange(rows, dtype=np.uint32)[None, :, None], (n, rows, cols // 8)))
    strip = (np.arange(cols // 8) // 32).astype(np.uint32)
    assert np.array_equal(words[:, :, 1::4], np.broadcast_to(strip[None, None, :], (n, rows, cols // 8)))
    assert not words[:, :, 3::4].any()


def test_probe_rejects_bad_arguments():
    mem = torch.zeros(32 * 256, dtype=torch.int16, device="cuda:0")
    for kw in (dict(rows=33), dict(cols=300), dict(walk=0), dict(mode=3), dict(n=0)):
        a = dict(rows=32, cols=256, n=1, walk=1, mode=0)
        a.update(kw)
        with pytest.raises(tb.TidalError):
            tb.tidal_hbm_probe(mem, a["rows"], a["cols"], a["n"], a["walk"], a["mode"], 1)
