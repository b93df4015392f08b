"""GPU parity at full size, in the launch configuration bench.py times (default config: 128 MiB
chunks, matrix-core LoRA kernels, pinned host pool, adapters by host pointers).

Llama2-7B-shaped stack (13.48 GB fp16 -> bf16, r=16 on q and v of 32 layers):
  * every one of the 226 slots is compared bit for bit with the oracle's conversion,
  * after attach and after swap, every element of every targeted slot (64 slots, 1.07 G
    elements) is recomputed by the oracle from the GPU's previous state -- in blocks of 512 rows,
    one oracle call each, on several host threads -- and compared within 2^-7 * max|W| (and one
    bf16 ulp per element),
  * every untargeted slot must be bit-identical to its materialised state (compared on device),
  * a second cold start with the adapter folded into the load (tidal_materialize_attach) is
    checked on every element too, against the oracle's one-rounding result from the fp16 source.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from paper_2503_06421_amd import workloads as wl_mod      # noqa: E402


def f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_llama2_7b_shaped_materialize_attach_swap(orc):
    assert torch.cuda.is_available()
    wl = wl_mod.llama2_7b()
    isz = wl_mod.ITEMSIZE[wl.host_dtype]
    pool = torch.empty(wl.source_bytes, dtype=torch.uint8, pin_memory=True)
    pool_np = pool.numpy()
    views, off = [], 0
    for t in wl.tensors:
        n = t.numel * isz
        views.append(pool_np[off:off + n].view(np.float16).reshape(t.rows, t.cols))
        off += n
    wl_mod.draw_all(wl, views, threads=16)
    print("drawn", flush=True)

    ads = [[(s, wl.alpha) + wl_mod.draw_adapter(wl, a, s) for s in wl.lora_slots] for a in (0, 1)]
    cfg0 = tb.make_config()
    need0 = tb.tidal_template_required_bytes(wl.shapes, cfg0)
    # size of the packed adapter: in x 16 + out x 16 bf16 per target
    adapter_bytes = sum(2 * 16 * (wl.tensors[s].rows + wl.tensors[s].cols) for s in wl.lora_slots)
    cfg = tb.make_config(max_adapter_bytes=adapter_bytes)
    need = tb.tidal_template_required_bytes(wl.shapes, cfg)
    assert need > need0
    arena = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    T = tb.tidal_template_create(wl.shapes, arena, need, cfg)
    copy_s, comp_s = torch.cuda.Stream(), torch.cuda.Stream()

    def dev_slot(i):
        p, nb = tb.tidal_template_slot_ptr(T, i)
        o = p - arena.data_ptr()
        return arena[o:o + nb]

    try:
        tb.tidal_materialize(T, [(i, wl.host_dtype, tb.host_ptr(v)) for i, v in enumerate(views)], copy_s, comp_s)
        tb.tidal_template_sync(T)
        torch.cuda.synchronize()
        print("materialised", flush=True)
        for i, v in enumerate(views):
            got = dev_slot(i).cpu().numpy().view(np.uint16).reshape(v.shape)
            assert np.array_equal(got, orc.convert_to_bf16(v)), "slot %d (%s)" % (i, wl.tensors[i].name)
        print("conversion and placement bit-exact on all %d slots" % len(views), flush=True)
        end = tb.tidal_template_slot_ptr(T, len(views) - 1)
        slot_area = end[0] - arena.data_ptr() + end[1]
        pristine = arena[:slot_area].clone()

        def host_slot(i):
            t = wl.tensors[i]
            return dev_slot(i).cpu().numpy().view(np.uint16).reshape(t.rows, t.cols)

        blocks = [(r0, min(r0 + 512, 4096)) for r0 in range(0, 4096, 512)]       # the whole tensor
        tasks = [(idx, s, b) for idx, s in enumerate(wl.lora_slots) for b in blocks]
        prev = {s: host_slot(s) for s in wl.lora_slots}

        def check(tag, old, new):
            cur = {s: host_slot(s) for s in wl.lora_slots}

            def one(task):
                idx, s, b = task
                before = prev[s][b[0]:b[1]]
                want = before.copy()
                mid = 0.0
                if old is not None:
                    _, al, A, B = old[idx]
                    orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(np.ascontiguousarray(B[b[0]:b[1]])), al, -1)
                    mid = np.abs(f32(want))          # a swap rounds twice: the state between the two roundings
                _, al, A, B = new[idx]
                orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(np.ascontiguousarray(B[b[0]:b[1]])), al, +1)
                got = cur[s][b[0]:b[1]]
                g, w = f32(got), f32(want)
                assert np.max(np.abs(g - w)) <= 2.0 ** -7 * np.max(np.abs(w)), (tag, s, b)
                # per element: one bf16 ulp of the result, and for a swap one more of the state in between
                # (where fp32 and fp64 accumulation round that state to neighbouring values)
                assert np.all(np.abs(g - w) <= (np.abs(w) + mid) * 2.0 ** -7 + 2.0 ** -20 * np.max(np.abs(w))), (tag, s, b)
                assert np.mean(got != want) < 2e-3, (tag, s, b)
                assert np.any(got != before), (tag, s, b)                    # the update happened
                return float(np.max(np.abs(g - w)) / np.max(np.abs(w)))

            with ThreadPoolExecutor(max_workers=16) as ex:
                worst = max(ex.map(one, tasks))
            prev.update(cur)
            print("%s: %d whole slots checked, worst max-abs-err / max|W| = %.3g" % (tag, len(cur), worst), flush=True)

        def untouched():
            targeted = set(wl.lora_slots)
            for i in range(len(views)):
                if i in targeted:
                    continue
                p, nb = tb.tidal_template_slot_ptr(T, i)
                o = p - arena.data_ptr()
                assert torch.equal(arena[o:o + nb], pristine[o:o + nb]), "untargeted slot %d changed" % i

        tb.tidal_lora_attach(T, tb.targets_from_arrays(ads[0]), comp_s)
        tb.tidal_template_sync(T)
        check("attach", None, ads[0])
        untouched()
        tb.tidal_lora_swap(T, tb.targets_from_arrays(ads[1]), comp_s)
        tb.tidal_template_sync(T)
        check("swap", ads[0], ads[1])
        untouched()
        st = tb.tidal_get_stats(T)
        # every targeted element was passed over exactly twice; attach and swap each upload and merge
        # in a few groups of targets (one launch per group, all slots have one shape)
        assert st["rmw_elems"] == 2 * wl.lora_w_elements
        n_launch = st["lora_launches"]
        assert 2 <= n_launch <= 16 and n_launch % 2 == 0
        # 101 chunks of 128 MiB for the stack; each adapter (16.8 MB of fp16 factors) is one more per group
        assert st["chunks"] == -(-wl.source_bytes // (128 << 20)) + n_launch

        # cold start again, adapter 0 folded into the load (re-materialising resets the template)
        tb.tidal_materialize_attach(T, [(i, wl.host_dtype, tb.host_ptr(v)) for i, v in enumerate(views)],
                                    tb.targets_from_arrays(ads[0]), copy_s, comp_s)
        tb.tidal_template_sync(T)
        torch.cuda.synchronize()
        cur = {s: host_slot(s) for s in wl.lora_slots}

        def one_fused(task):
            idx, s, b = task
            _, al, A, B = ads[0][idx]
            src = views[s][b[0]:b[1]]
            want = orc.materialize_merge(src, orc.convert_to_bf16(A), orc.convert_to_bf16(np.ascontiguousarray(B[b[0]:b[1]])), al)
            got = cur[s][b[0]:b[1]]
            g, w = f32(got), f32(want)
            assert np.max(np.abs(g - w)) <= 2.0 ** -7 * np.max(np.abs(w)), ("fused", s, b)
            assert np.mean(got != want) < 2e-3, ("fused", s, b)
            assert np.mean(got != orc.convert_to_bf16(src)) > 0.3, ("fused", s, b)
            return float(np.max(np.abs(g - w)) / np.max(np.abs(w)))

        with ThreadPoolExecutor(max_workers=16) as ex:
            worst = max(ex.map(one_fused, tasks))
        print("fused cold start: %d whole slots checked, worst max-abs-err / max|W| = %.3g" % (len(cur), worst), flush=True)
        untouched()
        assert tb.tidal_get_stats(T)["lora_launches"] == n_launch              # no read-modify-write pass was added
    finally:
        torch.cuda.synchronize()
        tb.tidal_template_destroy(T)
