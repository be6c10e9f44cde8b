"""Independent contexts used from several host threads at once, each on a stream of its own
(the header's threading convention): every thread runs many steps with table updates in
between, and every step must equal the oracle's.  Contexts share nothing, so nothing but
the library's own global state could make them interfere."""
import threading

import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu
from test_gpu_parity import oracle_step

pytestmark = pytest.mark.gpu


def test_four_threads_four_contexts(oracle):
    n_threads, n_steps = 4, 12
    shapes = [dict(T=256, H=512), dict(T=512, H=256), dict(T=128, H=1024), dict(T=1024, H=128)]
    work, refs = [], []
    for i in range(n_threads):
        sets = synth.churn_inputs(n_steps, **shapes[i])
        work.append(sets)
        dead = synth.active_mask(sets[0].R, (3 + i,))
        repaired = synth.repaired_placement(sets[0].p2l, (3 + i,), sets[0].R, sets[0].S_prim,
                                            sets[0].S_red)
        # steps 4..7 of every thread run with one rank failed (a different one per thread)
        tables = [(repaired, dead) if 4 <= s < 8 else (sets[0].p2l, sets[0].active)
                  for s in range(n_steps)]
        refs.append([oracle_step(oracle, sets[s], p2l=tables[s][0], active=tables[s][1])
                     for s in range(n_steps)])
        work[-1] = (sets, tables)
    errors, results = [], [[None] * n_steps for _ in range(n_threads)]
    start = threading.Barrier(n_threads)

    def run(i):
        try:
            torch.cuda.set_device(0)
            sets, tables = work[i]
            stream = torch.cuda.Stream()
            ctx = gu.make_context(sets[0])
            try:
                gu.apply_tables(ctx, *tables[0], stream)
                devs = [gu.DeviceStep(ctx, wl, stream) for wl in sets]
                torch.cuda.synchronize()
                start.wait()
                for s in range(n_steps):
                    if s == 4:                                   # failure: placement, then mask
                        ctx.update_placement(tables[s][0], stream)
                        ctx.set_membership(tables[s][1], stream)
                    elif s == 8:                                 # rejoin: mask, then placement
                        ctx.set_membership(tables[s][1], stream)
                        ctx.update_placement(tables[s][0], stream)
                    devs[s].step()
                    lay = ctx.read_layout(sets[s].T, stream)     # waits for this thread's stream only
                    results[i][s] = (lay, gu.to_host(devs[s].out, np.uint16).copy())
            finally:
                ctx.destroy()
        except Exception as exc:                                 # surfaced by the main thread
            errors.append((i, repr(exc)))
            try:
                start.abort()
            except Exception:
                pass

    threads = [threading.Thread(target=run, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=300)
    assert not errors, errors
    for i in range(n_threads):
        sets, _ = work[i]
        for s in range(n_steps):
            lay, out = results[i][s]
            gu.assert_layout_equal(lay, refs[i][s]["lay"], sets[s].T, sets[s].k)
            assert np.array_equal(out, refs[i][s]["chain_bits"]), (i, s)
