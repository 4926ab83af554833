"""A CPU model of the LDS-ring schedule of k_solve_wave_bands_io (rows of a 64-row band pass through four chunks of
16 columns per row; a filling, a solving and a draining wave, coupled by three counters).  The model restates the
schedule (which chunk of which row each block of each wave touches, and what each wave waits for) and runs the three
waves in random legal interleavings, one block at a time.  It checks what the kernel relies on: every read of the
solving wave (including the one-step look-ahead) finds the chunk it expects, still unsolved; a chunk is only refilled
after it has left; every chunk that leaves is completely solved; every pixel leaves exactly once; nothing deadlocks."""
import random

import pytest

CHUNK = 16          # columns per chunk = steps per block
SLOTS = 4           # chunks a row holds in the ring


def rho(r):
    return (r - 1) >> 4


def run_model(band_rows, W, seed):
    rnd = random.Random(seed)
    nsteps = band_rows + W - 1
    nblocks = (nsteps + CHUNK - 1) // CHUNK
    nstore = (W + CHUNK - 1) // CHUNK + 4
    ring = [[None] * SLOTS for _ in range(64)]
    left = set()
    loaded = done = stored = 0              # the three counters
    lm, sj, sm = -1, 0, 0                   # next block of the filling / solving / draining wave

    def can_fill():
        return lm < nblocks and (lm < 3 or stored >= lm - 2)

    def can_solve():
        return sj < nblocks and loaded >= sj + 2

    def can_drain():
        return sm < nstore and done >= min(sm + 1, nblocks)

    while lm < nblocks or sj < nblocks or sm < nstore:
        ready = [name for name, ok in (("fill", can_fill()), ("solve", can_solve()), ("drain", can_drain())) if ok]
        assert ready, f"deadlock at fill {lm} solve {sj} drain {sm}"
        act = rnd.choice(ready)
        if act == "fill":
            for r in range(64):
                q = lm - rho(r)
                if q >= 0 and CHUNK * q < W:
                    old = ring[r][q % SLOTS]
                    if old is not None and r < band_rows:
                        assert old["left"], f"row {r}: chunk {old['chunk']} refilled by {q} before it left"
                    ring[r][q % SLOTS] = {"chunk": q, "solved": set(), "left": False}
            lm += 1
            loaded = lm + 1
        elif act == "solve":
            for r in range(band_rows):
                for t in range(CHUNK * sj, CHUNK * sj + CHUNK + 1):      # the last one is the look-ahead read
                    c = t - r
                    if 0 <= c < W:
                        slot = ring[r][(c // CHUNK) % SLOTS]
                        assert slot is not None and slot["chunk"] == c // CHUNK, f"row {r} column {c} block {sj}"
                        assert c not in slot["solved"]
                        if t < CHUNK * sj + CHUNK and t < nsteps:
                            slot["solved"].add(c)
            sj += 1
            done = sj
        else:
            for r in range(band_rows):
                q = sm - rho(r) - 1
                if q >= 0 and CHUNK * q < W:
                    slot = ring[r][q % SLOTS]
                    assert slot is not None and slot["chunk"] == q, f"row {r}: drain block {sm} expected chunk {q}"
                    cols = set(range(CHUNK * q, min(CHUNK * q + CHUNK, W)))
                    assert slot["solved"] == cols, f"row {r} chunk {q} leaves incomplete"
                    slot["left"] = True
                    for c in cols:
                        assert (r, c) not in left
                        left.add((r, c))
            sm += 1
            stored = sm
    assert len(left) == band_rows * W


@pytest.mark.parametrize("band_rows,W", [(64, 256), (64, 128), (64, 132), (8, 140), (1, 128), (64, 64), (33, 68),
                                         (64, 4), (2, 8), (17, 36), (63, 100)])
def test_ring_schedule_is_hazard_free_under_random_interleavings(band_rows, W):
    for seed in range(12):
        run_model(band_rows, W, seed)
