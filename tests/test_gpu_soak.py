"""Soak of the in-launch hand-off between the projection and its consumers (Sec. 3.3,
Eqs. 8-9: R is produced and consumed inside one launch): about ten thousand launches
through ONE workspace, token counts of every kernel class in seeded random order,
restored and not restored, eager and replayed from captured graphs, back to back without
a synchronisation between the launches of a batch.  Every output is compared bit for bit
with the first result of its class, which is verified against the oracle; the run stops at
its first mismatch and checks the unit's status word after every batch."""
import time

import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from glowq_inputs import UnitShape, gen_activations
from oracle import glowq_oracle as O
from gpu_util import DeviceUnit, dev_bits, stream
from util import recipe_unit, rel_err

pytestmark = pytest.mark.gpu

TOKENS = [1, 2, 4, 9, 16, 32, 48, 130]
N_LAUNCHES = 10000
TIME_CAP_S = 100.0


def test_handshake_soak():
    shape = UnitShape("g", 2304, (72, 40))          # two K parts in every projection flavour
    base = recipe_unit(O, 1, 0, max(TOKENS), r=24, shape=shape, G=128)
    classes = []                                     # (T, restore) -> device unit + reference
    for T in TOKENS:
        for restore in (True, False):
            u = dict(base, X=base["X"][:T], T=T)
            du = DeviceUnit(u)
            classes.append(dict(T=T, restore=restore, du=du, unit=u))
    ws_bytes = max(G.glowq_workspace_bytes([c["du"].desc]) for c in classes)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    G.glowq_workspace_init(ws.data_ptr(), ws_bytes, stream())
    failed = torch.zeros(1, dtype=torch.int32, device="cuda")

    def launch(c, st):
        G.glowq_group_forward(c["du"].desc, c["restore"], ws.data_ptr(), ws_bytes, st)

    # first result of every class: against the oracle; it becomes the class's reference
    for c in classes:
        launch(c, stream())
        ys = c["du"].outputs()
        for y, ref in zip(ys, O.group_forward(c["unit"], c["restore"])):
            assert rel_err(y, ref) <= 2e-3, (c["T"], c["restore"])
        c["ref"] = [y.clone() for y in c["du"].Y]
    # one captured graph per class
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for c in classes:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                launch(c, torch.cuda.current_stream().cuda_stream)
            c["graph"] = g
    torch.cuda.synchronize()

    rng = np.random.default_rng(2024)
    done, t0 = 0, time.time()
    with torch.cuda.stream(side):
        while done < N_LAUNCHES and time.time() - t0 < TIME_CAP_S:
            batch = rng.permutation(len(classes))[:rng.integers(4, len(classes) + 1)]
            for i in batch:
                classes[i]["du"].clear()
            for i in batch:                           # back to back, no synchronisation
                if rng.random() < 0.5:
                    classes[i]["graph"].replay()
                else:
                    launch(classes[i], side.cuda_stream)
            G.glowq_workspace_status([classes[batch[0]]["du"].desc], ws.data_ptr(), ws_bytes,
                                     failed.data_ptr(), side.cuda_stream)
            side.synchronize()
            assert int(failed.item()) == 0, f"status word set after {done} launches"
            for i in batch:
                c = classes[i]
                for y, ref in zip(c["du"].Y, c["ref"]):
                    assert torch.equal(y, ref), f"mismatch after {done} launches: T={c['T']} restore={c['restore']}"
            done += len(batch)
    print(f"soak: {done} launches in {time.time() - t0:.1f} s")
    assert done >= 2000, "the soak was cut short by its time cap far too early"
