"""GPU parity of the LoRA passes in the launch geometry the full-size workloads run with.

The walk length of a wave (32-row blocks per 256-column strip), the kernel variant and the number
of waves per SIMD are chosen from the size of a launch, so small test shapes only ever see one block
per wave.  Here the launches are as large as those of the resident-adapter workload (Sec. 5.2,
keep-alive: only the dynamic part is redone per invocation), and WHOLE tensors are compared with the
oracle:

  * every padded-rank instantiation -- the 16 ordered pairs of ranks {8, 16, 32, 64} as fused swaps,
    the four merges, the four unmerges and the four copy-on-write fork applies -- on 33 slots of
    4096 x 4096 and on 24 slots of 5152 x 5120 (a row pitch that is no power of two, and a last
    row block that ends a walk early), fused swaps also bit-identical to a two-pass template;
  * the full 200-invocation Zipf schedule on 128 slots of 4096 x 4096.

Slots fall into a few classes that share base values and factors, so that every slot of a launch
can be checked: one whole slot per class against the oracle (restarted from the GPU's previous state
each step, so one-ulp differences of the matrix-core path do not compound), all others bit for bit
against their class's slot on the device.  The oracle runs as it stands, one slot per host thread.
"""
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from paper_2503_06421_amd import workloads as wl_mod      # noqa: E402

TOL = 2.0 ** -7
RANKS = (8, 16, 32, 64)
# cyclic sequence over four symbols in which every ordered pair (self pairs included) occurs once
PAIR_WALK = (0, 0, 1, 0, 2, 0, 3, 1, 1, 2, 1, 3, 2, 2, 3, 3)
ORACLE_THREADS = 16


def f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


class Stack:
    """n slots of out x in over one arena; class of slot s = s % n_classes."""

    def __init__(self, out, inn, n, n_classes, flags=0, seed=0):
        self.out, self.inn, self.n, self.k = out, inn, n, n_classes
        self.shapes = [(out, inn)] * n
        self.cfg = tb.make_config(flags=flags)
        need = tb.tidal_template_required_bytes(self.shapes, self.cfg)
        self.arena = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        self.h = tb.tidal_template_create(self.shapes, self.arena, need, self.cfg)
        self.copy_s, self.comp_s = torch.cuda.Stream(), torch.cuda.Stream()
        self.slot_bytes = 2 * out * inn
        p0, _ = tb.tidal_template_slot_ptr(self.h, 0)
        for s in range(n):                                   # slots are back to back (sizes are multiples of 256)
            p, nb = tb.tidal_template_slot_ptr(self.h, s)
            assert p - p0 == s * self.slot_bytes and nb == self.slot_bytes
        self.base_off = p0 - self.arena.data_ptr()
        rng = np.random.default_rng(seed)
        self.base = [torch.from_numpy(rng.normal(0, 0.02, (out, inn)).astype(np.float16)).pin_memory()
                     for _ in range(n_classes)]
        tb.tidal_materialize(self.h, [(s, tb.TIDAL_F16, self.base[s % n_classes].data_ptr()) for s in range(n)],
                             self.copy_s, self.comp_s)
        self.sync()
        self.keep = []

    def sync(self):
        tb.tidal_template_sync(self.h)
        torch.cuda.synchronize()

    def slots_dev(self):
        """All slots as an (n, out*in) int16 view of the arena."""
        return self.arena[self.base_off: self.base_off + self.n * self.slot_bytes].view(torch.int16).view(self.n, -1)

    def slot_host(self, s):
        return self.slots_dev()[s].cpu().numpy().view(np.uint16).reshape(self.out, self.inn)

    def upload(self, factors, alpha):
        """factors: per class (A, B) host fp16 arrays.  Returns a resident adapter over all slots."""
        tg = tb.targets_from_arrays([(s, alpha) + factors[s % self.k] for s in range(self.n)])
        nb = tb.tidal_adapter_required_bytes(self.h, tg)
        mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
        a = tb.tidal_adapter_upload(self.h, tg, mem, nb, self.comp_s)
        self.sync()
        self.keep.append((mem, a))
        return a

    def classes_agree(self, dev=None):
        dev = self.slots_dev() if dev is None else dev
        for c in range(self.k):
            members = dev[c::self.k]
            if not bool(torch.all(members == members[0:1])):
                return False
        return True

    def close(self):
        torch.cuda.synchronize()
        for _, a in self.keep:
            try:
                tb.tidal_adapter_destroy(a)
            except tb.TidalError:                            # still attached after a failed test: the template goes first
                pass
        tb.tidal_template_destroy(self.h)
        self.keep = []


def draw_factors(seed, r, out, inn, n_classes):
    g = np.random.default_rng(seed)
    return [(g.normal(0, 0.01, (r, inn)).astype(np.float16), g.normal(0, 0.01, (out, r)).astype(np.float16))
            for _ in range(n_classes)]


def oracle_step(orc, before, old, new):
    """before: bf16 bits; old/new: (alpha, A, B) host fp16 or None.  Returns the oracle's result."""
    want = before.copy()
    if old is not None:
        al, A, B = old
        orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(B), al, -1)
    if new is not None:
        al, A, B = new
        orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(B), al, +1)
    return want


def compare(got, want, before, what, changes=True):
    g, w = f32(got), f32(want)
    err = float(np.max(np.abs(g - w)) / np.max(np.abs(w)))
    assert err <= TOL, (what, err)
    frac = float(np.mean(got != want))
    assert frac < 5e-3, (what, frac)                         # the rest is one rounding step away
    if changes:                                              # and the pass did something (a swap to the
        assert float(np.mean(got != before)) > 0.3, what     # attached adapter itself changes next to nothing)
    return err, frac


@pytest.mark.parametrize("out,inn,n", [(4096, 4096, 33), (5152, 5120, 24)], ids=["4096x4096x33", "5152x5120x24"])
def test_every_instantiation_whole_tensors(orc, out, inn, n):
    assert torch.cuda.is_available()
    K = 3
    T = Stack(out, inn, n, K, seed=1)
    T2 = Stack(out, inn, n, K, flags=tb.TIDAL_FLAG_TWO_PASS_SWAP, seed=1)
    pool = ThreadPoolExecutor(max_workers=ORACLE_THREADS)
    jobs, seen, swap_pairs = [], {}, set()
    try:
        assert torch.equal(T.slots_dev(), T2.slots_dev())
        pairs = {(PAIR_WALK[i], PAIR_WALK[(i + 1) % 16]) for i in range(16)}
        assert len(pairs) == 16
        # the plan: attach, 16 swaps (every ordered rank pair), detach; then merge + unmerge of the other ranks
        steps = [("attach", None, RANKS[PAIR_WALK[0]])]
        steps += [("swap", RANKS[PAIR_WALK[i - 1]], RANKS[PAIR_WALK[i % 16]]) for i in range(1, 17)]
        steps += [("detach", RANKS[PAIR_WALK[0]], None)]
        for r in RANKS[1:]:
            steps += [("attach", None, r), ("detach", r, None)]
        cur = cur2 = None                                    # (factors per class, alpha, handle)
        state = [T.slot_host(c) for c in range(K)]
        for idx, (kind, r_old, r_new) in enumerate(steps):
            new = new2 = None
            if r_new is not None:
                fac = draw_factors(1000 * out + idx, r_new, out, inn, K)
                new = (fac, 2.0 * r_new, T.upload(fac, 2.0 * r_new))
                new2 = (fac, 2.0 * r_new, T2.upload(fac, 2.0 * r_new))
            info = tb.tidal_lora_launch_info(T.h, out, inn, n, r_old or 0, r_new or 0)
            if kind == "swap":
                swap_pairs.add((info["rank_padded_old"], info["rank_padded_new"]))
            if kind == "attach":
                tb.tidal_lora_attach_adapter(T.h, new[2], T.comp_s)
                tb.tidal_lora_attach_adapter(T2.h, new2[2], T2.comp_s)
            elif kind == "swap":
                tb.tidal_lora_swap_adapter(T.h, new[2], T.comp_s)
                tb.tidal_lora_swap_adapter(T2.h, new2[2], T2.comp_s)
            else:
                tb.tidal_lora_detach(T.h, T.comp_s)
                tb.tidal_lora_detach(T2.h, T2.comp_s)
            T.sync()
            T2.sync()
            assert cur is None or r_old == cur[0][0][0].shape[0]
            dev = T.slots_dev()
            assert T.classes_agree(dev), ("slots of one class differ", idx, kind, r_old, r_new)
            assert torch.equal(dev, T2.slots_dev()), ("fused pass != two passes", idx, kind, r_old, r_new)
            after = [T.slot_host(c) for c in range(K)]
            for c in range(K):
                o = (cur[1], cur[0][c][0], cur[0][c][1]) if (cur is not None and kind != "attach") else None
                nw = (new[1], new[0][c][0], new[0][c][1]) if new is not None else None
                what = "%s %s->%s class %d [%s rc=%d]" % (kind, r_old, r_new, c, info["kernel"], info["blocks_per_walk"])
                jobs.append((what, state[c], after[c], pool.submit(oracle_step, orc, state[c], o, nw)))
            seen[(info["kernel"], info["blocks_per_walk"])] = seen.get((info["kernel"], info["blocks_per_walk"]), 0) + 1
            state = after
            cur, cur2 = (new, new2) if new is not None else (None, None)
        # copy-on-write forks: every private copy rewritten from the (now detached) template
        need = tb.tidal_fork_required_bytes(T.h, list(range(n)))
        fmem = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        F = tb.tidal_fork_create(T.h, list(range(n)), fmem, need)
        try:
            p0, _ = tb.tidal_fork_slot_ptr(F, 0)
            for r in RANKS:
                fac = draw_factors(77 * out + r, r, out, inn, K)
                a = T.upload(fac, 2.0 * r)
                info = tb.tidal_lora_launch_info(T.h, out, inn, n, 0, r, fork=True)
                tb.tidal_fork_apply(F, a, T.comp_s)
                T.sync()
                fdev = fmem[p0 - fmem.data_ptr(): p0 - fmem.data_ptr() + n * T.slot_bytes].view(torch.int16).view(n, -1)
                assert T.classes_agree(fdev), ("fork: slots of one class differ", r)
                assert T.classes_agree(), "the template changed under a fork"
                for c in range(K):
                    got = fdev[c].cpu().numpy().view(np.uint16).reshape(out, inn)
                    what = "fork 0->%d class %d [%s rc=%d]" % (r, c, info["kernel"], info["blocks_per_walk"])
                    jobs.append((what, state[c], got, pool.submit(oracle_step, orc, state[c], None, (2.0 * r, fac[c][0], fac[c][1]))))
                seen[(info["kernel"], info["blocks_per_walk"])] = seen.get((info["kernel"], info["blocks_per_walk"]), 0) + 1
        finally:
            tb.tidal_fork_destroy(F)
        worst = 0.0
        for what, before, got, fut in jobs:
            err, frac = compare(got, fut.result(), before, what)
            worst = max(worst, err)
        print("\n%d x %d x %d: %d whole tensors against the oracle, worst max-abs-err / max|W| = %.3g" %
              (n, out, inn, len(jobs), worst), flush=True)
        for (kernel, rc), cnt in sorted(seen.items()):
            print("  %-44s %2d blocks per walk: %d launches" % (kernel, rc, cnt), flush=True)
        assert len(swap_pairs) == 9, sorted(swap_pairs)      # the nine padded-rank swap instantiations
        assert max(rc for _, rc in seen) >= 8 and len({rc for _, rc in seen}) >= 3
    finally:
        pool.shutdown(wait=True, cancel_futures=True)
        T.close()
        T2.close()


def test_adapter_churn_all_200_steps_whole_tensors(orc):
    """Configuration 4 as it runs: 128 slots of 4096 x 4096, pool of 32 resident adapters with ranks
    from {8, 16, 32, 64}, the seeded Zipf(1.1) schedule of 200 invocations (one attach, 199 fused
    swaps).  After every step two whole slots (their position in the launch moves with the step) are
    recomputed by the oracle from the GPU's previous state; every other slot is compared with its
    class's slot on the device."""
    assert torch.cuda.is_available()
    ch = wl_mod.adapter_churn()
    assert len(ch.schedule) == 200 and len(ch.ranks) == 32
    out = inn = 4096
    n, K = 128, 4
    T = Stack(out, inn, n, K, seed=4)
    pool = ThreadPoolExecutor(max_workers=ORACLE_THREADS)
    room = threading.Semaphore(3 * ORACLE_THREADS)            # bounds the snapshots waiting for the oracle
    jobs, pairs = [], {}

    def task(before, old, new):
        try:
            return oracle_step(orc, before, old, new)
        finally:
            room.release()

    try:
        fac, handle = {}, {}
        for a in sorted(set(ch.schedule)):
            fac[a] = draw_factors(5000 + a, ch.ranks[a], out, inn, K)
            handle[a] = T.upload(fac[a], ch.alphas[a])
        cur = None
        for step, a in enumerate(ch.schedule):
            classes = (step % K, (step + 1) % K)
            slots = [c + K * ((7 * step + 3 * c) % (n // K)) for c in classes]      # moves through the launch
            before = [T.slot_host(s) for s in slots]
            if cur is None:
                tb.tidal_lora_attach_adapter(T.h, handle[a], T.comp_s)
            else:
                tb.tidal_lora_swap_adapter(T.h, handle[a], T.comp_s)
            T.sync()
            assert T.classes_agree(), ("slots of one class differ", step)
            r_old = ch.ranks[cur] if cur is not None else 0
            info = tb.tidal_lora_launch_info(T.h, out, inn, n, r_old, ch.ranks[a])
            key = (r_old, ch.ranks[a], info["kernel"], info["blocks_per_walk"])
            pairs[key] = pairs.get(key, 0) + 1
            for s, c, b in zip(slots, classes, before):
                o = (ch.alphas[cur], fac[cur][c][0], fac[cur][c][1]) if cur is not None else None
                nw = (ch.alphas[a], fac[a][c][0], fac[a][c][1])
                room.acquire()
                jobs.append(("step %d adapter %d (%d->%d) slot %d" % (step, a, r_old, ch.ranks[a], s), b, T.slot_host(s),
                             pool.submit(task, b, o, nw), a != cur))
            cur = a
            while jobs and jobs[0][3].done():                 # check and drop finished ones as we go
                what, b, got, fut, changes = jobs.pop(0)
                compare(got, fut.result(), b, what, changes)
            if step % 25 == 24:
                print("churn replay: %d steps enqueued" % (step + 1), flush=True)
        for what, b, got, fut, changes in jobs:
            compare(got, fut.result(), b, what, changes)
        assert tb.tidal_get_stats(T.h)["lora_launches"] == len(ch.schedule)
        print("\nchurn replay: 200 steps, 400 whole tensors against the oracle", flush=True)
        for (r0, r1, kernel, rc), cnt in sorted(pairs.items()):
            print("  %2d -> %2d  %-40s %2d blocks per walk: %3d steps" % (r0, r1, kernel, rc, cnt), flush=True)
        tb.tidal_lora_detach(T.h, T.comp_s)
        T.sync()
    finally:
        pool.shutdown(wait=True, cancel_futures=True)
        T.close()
