"""tidal_lora_apply_static under HIP graph capture: the use the allocation-free entry point exists for.

A layer loop of applies (decode segments and one prompt, three adapters) is captured once and replayed
several times, with the program's own eager work and synchronisations between the replays; every
replay must give the eager call's bits.  The adapters' uploads are finished and seen before the capture
(one eager pass), so the captured calls consist of kernel launches only.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from tests.gpu_util import Template                       # noqa: E402


def bf16_bits(rng, shape, scale):
    return (rng.normal(0, scale, shape).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def test_captured_layer_loop_replays_to_the_eager_bits():
    assert torch.cuda.is_available()
    rng = np.random.default_rng(99)
    layers, out, inn = 4, 512, 1024
    with Template([(out, inn)] * layers, max_adapter_bytes=0) as T:
        T.materialize({l: rng.normal(0, 0.02, (out, inn)).astype(np.float32) for l in range(layers)})
        handles = []
        for r, al in ((8, 16.0), (16, 32.0), (64, 128.0)):
            items = [(l, al, rng.normal(0, 0.05, (r, inn)).astype(np.float32), rng.normal(0, 0.05, (out, r)).astype(np.float32))
                     for l in range(layers)]
            handles.append(T.upload_adapter(items))
        T.sync()
        segs = [(i % 3, i, i + 1) for i in range(16)] + [(2, 16, 56), (-1, 56, 60), (1, 60, 64)]
        n = 64
        arrays = tb.lora_apply_arrays(handles, segs)              # marshalled once: nothing is built during capture
        x = [torch.from_numpy(bf16_bits(rng, (n, inn), 1.0).view(np.int16)).to("cuda:0") for _ in range(layers)]
        y0 = [torch.from_numpy(bf16_bits(rng, (n, out), 1.0).view(np.int16)).to("cuda:0") for _ in range(layers)]
        y = [t.clone() for t in y0]
        s = torch.cuda.Stream()

        def run_layers(stream):
            for l in range(layers):
                tb.tidal_lora_apply_static(T.h, l, arrays[0], arrays[1], x[l], y[l], n, stream)

        run_layers(s)                                             # eager: the reference, and the uploads are seen done
        s.synchronize()
        want = [t.cpu().numpy().copy() for t in y]
        assert any(np.mean(w != t0.cpu().numpy()) > 0.3 for w, t0 in zip(want, y0))
        for l in range(layers):
            y[l].copy_(y0[l])
        torch.cuda.synchronize()

        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            run_layers(torch.cuda.current_stream())
        torch.cuda.synchronize()
        for replay in range(4):
            for l in range(layers):                               # eager work between the replays
                y[l].copy_(y0[l])
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for l in range(layers):
                got = y[l].cpu().numpy()
                assert np.array_equal(got, want[l]), "replay %d, layer %d: %d elements differ" % (replay, l, int(np.sum(got != want[l])))
        del g
