"""A model of the kernel's ticket protocol, run on the CPU under adversarial
interleavings: waves draw tickets from several counters (ticket t from counter
t mod Q, a wave stays with its own counter until it is empty, then goes round
the others), a ticket is (stage instance, tile) in the schedule's execution
order, and a wave that holds a ticket waits until every tile of the instances
it depends on is finished.  The model checks what the kernel's comments claim:
no interleaving deadlocks, every tile is processed exactly once, and every wave
draws exactly one ticket past the end of every counter (which is what the
host's bookkeeping of the counters' bases relies on).

The dependency structure comes from the library's own per-edge schedules; the
protocol is restated here, it is not the kernel's code."""
import numpy as np
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si


def instances(top, root, n, chunk, tile):
    """(tiles, deps) per stage instance of the library's per-edge AllReduce schedule."""
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)
    steps = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_EDGE).steps()
    out = []
    for s in steps:
        off, ln = int(s["off"]), int(s["len"])
        tiles = (off + ln + tile - 1) // tile - off // tile      # tiles lie on the absolute grid
        out.append((tiles, [int(d) for d in s["deps"][:int(s["n_deps"])]]))
    return out


def simulate(inst, n_waves, n_queues, rng, prefer_waiting):
    """One run.  Each scheduling step picks a wave and lets it take one action."""
    tiles_per_chunk = max(t for t, _ in inst)
    n_items = len(inst) * tiles_per_chunk
    n_queues = min(n_queues, n_waves)
    counter = [0] * n_queues
    done = [0] * len(inst)
    processed = set()
    overdraws = [[0] * n_queues for _ in range(n_waves)]
    # wave state: ("draw", queue, empty_queues) | ("hold", instance, tile, queue, empty) | ("exit",)
    state = [("draw", w % n_queues, 0) for w in range(n_waves)]
    for _ in range(50 * (n_items + n_waves * n_queues) + 1000):
        live = [w for w in range(n_waves) if state[w][0] != "exit"]
        if not live:
            break
        waiting = [w for w in live if state[w][0] == "hold"]
        w = int(rng.choice(waiting)) if (prefer_waiting and waiting and rng.random() < 0.9) else int(rng.choice(live))
        st = state[w]
        if st[0] == "draw":
            _, q, empty = st
            nth = counter[q]
            counter[q] += 1
            t = nth * n_queues + q
            if t >= n_items:
                overdraws[w][q] += 1
                empty += 1
                state[w] = ("exit",) if empty == n_queues else ("draw", (q + 1) % n_queues, empty)
            else:
                state[w] = ("hold", t // tiles_per_chunk, t % tiles_per_chunk, q, empty)
        else:
            _, ii, tile, q, empty = st
            if tile >= inst[ii][0]:                 # this instance has fewer tiles: nothing to do
                state[w] = ("draw", q, empty)
            elif all(done[d] == inst[d][0] for d in inst[ii][1]):
                assert (ii, tile) not in processed
                processed.add((ii, tile))
                done[ii] += 1                        # posted with the wave's next draw in the kernel
                state[w] = ("draw", q, empty)
            # else: keeps polling
    else:
        stuck = [state[w] for w in range(n_waves) if state[w][0] == "hold"]
        pytest.fail(f"no progress: {len(processed)} tiles done, waiting waves {stuck[:4]}")
    assert len(processed) == sum(t for t, _ in inst)
    assert all(done[i] == inst[i][0] for i in range(len(inst)))
    assert all(o == 1 for per_wave in overdraws for o in per_wave)
    return counter


CASES = {
    "chain of 6, 5 chunks": (si.chain(6), 0, 20_000, 4_000, 1_024),
    "cube-mesh, ragged": (si.hybrid_cube_mesh(), 0, 50_003, 3_000, 1_024),
    "16 one-hop trees": (si.complete_graph(16), bl.BLINK_ROOT_ANY, 16 * 700, 256, 256),
}


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("n_queues", [1, 2, 4])
@pytest.mark.parametrize("n_waves", [1, 4, 5, 37])
def test_no_interleaving_deadlocks_and_every_tile_runs_once(case, n_queues, n_waves):
    inst = instances(*CASES[case])
    for seed in range(4):
        rng = np.random.default_rng([5, seed, n_queues, n_waves])
        counter = simulate(inst, n_waves, n_queues, rng, prefer_waiting=bool(seed % 2))
        # what the host adds to each counter's base per call: its tickets + one per wave
        q_used = min(n_queues, n_waves)
        n_items = len(inst) * max(t for t, _ in inst)
        assert counter == [(n_items + q_used - 1 - q) // q_used + n_waves for q in range(q_used)]


def test_the_model_does_detect_a_deadlock():
    """Hand every wave to a counter it does not own (so a counter has no waves of
    its own) and starve the rest: the protocol's precondition, at least as many
    waves as counters, is what the run above depends on."""
    inst = instances(si.chain(4), 0, 1_024, 1_024, 1_024)     # one chunk: every ticket waits for the one before it
    tiles_per_chunk = max(t for t, _ in inst)
    # two counters, ONE wave that never leaves counter 1: ticket 0 (counter 0) is never drawn
    counter, done = [0, 0], [0] * len(inst)
    progressed = True
    held = None
    steps = 0
    while progressed and steps < 1000:
        steps += 1
        progressed = False
        if held is None:
            t = counter[1] * 2 + 1
            counter[1] += 1
            if t < len(inst) * tiles_per_chunk:
                held = (t // tiles_per_chunk, t % tiles_per_chunk)
                progressed = True
        else:
            ii, tile = held
            if tile >= inst[ii][0] or all(done[d] == inst[d][0] for d in inst[ii][1]):
                if tile < inst[ii][0]:
                    done[ii] += 1
                held = None
                progressed = True
    assert held is not None and done[0] == 0          # stuck behind the ticket nobody can draw
