"""Host-side model of the hand-over of tile columns in the dense pass over X (no GPU needed).

In `dense_stream_kernel` the 8 waves of a workgroup share a panel-wide accumulator of X_t^T A that is cut into 8 tile
columns.  In global step g = 8 * round + s wave w works on column (w + s) % 8, so a column passes from wave w + 1 to
wave w.  There is no barrier: every wave publishes the number of steps it has completed, and before it touches the
column of step g it polls until its neighbour w + 1 has completed g steps.  A wave that has nothing to do in a step
(no strip for it in the chunk's last round, or a tile beyond the matrix) waits all the same before its own count
moves.

The model below states that protocol (indexing as in the kernel: tile of a step, strip of a round with the panel's
rotation, the predicate for "has work") as eight little state machines and runs them under schedules drawn at random,
including adversarial ones that let single waves run far ahead.  Invariant checked at every step: a wave that enters
the column phase finds no other wave inside that column.  The same model with the idle waves' wait taken out (the
mistake an earlier version of the kernel had) must violate the invariant on ragged shapes: that is what makes the
check worth something.
"""
import numpy as np
import pytest

K_WAVES = 8
K_TILES = 8
K_PANEL = 128


class Workgroup:
    """One workgroup of the dense pass: panel `panel` of a matrix with n columns, rows [0, rows) of a chunk."""

    def __init__(self, n, rows, panel, idle_waves_wait=True):
        self.tiles = min(K_TILES, (n - panel * K_PANEL + 15) // 16)
        self.nstrips = (rows + 15) // 16
        self.nrounds = (self.nstrips + K_WAVES - 1) // K_WAVES
        self.rnd0 = panel % self.nrounds
        self.nsteps = self.nrounds * K_TILES
        self.idle_waves_wait = idle_waves_wait
        self.done = [0] * K_WAVES                 # steps completed, as published in LDS
        self.step = [0] * K_WAVES                 # the step a wave is in
        self.phase = ["p"] * K_WAVES              # p: products that touch nothing shared; wait; col: inside the column
        self.owner = [None] * K_TILES             # wave inside each column
        self.col_work = np.zeros((K_TILES,), dtype=np.int64)   # column phases carried out per column
        self.strip_tiles = set()                  # (strip, tile) pairs whose column phase was carried out

    def strip_of(self, w, rnd):
        rr = rnd + self.rnd0
        if rr >= self.nrounds:
            rr -= self.nrounds
        return rr * K_WAVES + w

    def has_work(self, w, g):
        rnd, s = divmod(g, K_TILES)
        return self.strip_of(w, rnd) < self.nstrips and ((w + s) % K_TILES) < self.tiles

    def finished(self, w):
        return self.step[w] >= self.nsteps

    def advance(self, w):
        """One scheduling quantum of wave w.  Returns False if the wave could not move (its poll failed)."""
        g = self.step[w]
        col = (w + g) % K_TILES
        work = self.has_work(w, g)
        if self.phase[w] == "p":
            self.phase[w] = "wait" if (work or self.idle_waves_wait) else "publish"
            return True
        if self.phase[w] == "wait":
            if self.done[(w + 1) % K_WAVES] < g:
                return False
            if work:
                assert self.owner[col] is None, f"wave {w} enters column {col} in step {g} while wave {self.owner[col]} is in it"
                self.owner[col] = w
                self.phase[w] = "col"
            else:
                self.phase[w] = "publish"
            return True
        if self.phase[w] == "col":
            self.owner[col] = None
            self.col_work[col] += 1
            self.strip_tiles.add((self.strip_of(w, g // K_TILES), col))
            self.phase[w] = "publish"
            return True
        self.done[w] = g + 1                      # publish
        self.step[w] = g + 1
        self.phase[w] = "p"
        return True


def run(wg, rng, style):
    """Drive the eight waves until all have finished; `style` picks the scheduler."""
    quanta = 0
    while not all(wg.finished(w) for w in range(K_WAVES)):
        live = [w for w in range(K_WAVES) if not wg.finished(w)]
        if style == "uniform":
            w = live[rng.integers(len(live))]
            wg.advance(w)
        elif style == "bursts":                   # one wave runs as far as it can, then another
            w = live[rng.integers(len(live))]
            for _ in range(int(rng.integers(1, 60))):
                if wg.finished(w) or not wg.advance(w):
                    break
        else:                                     # "laggard": one wave is starved for long stretches
            lag = int(rng.integers(K_WAVES))
            for _ in range(int(rng.integers(20, 400))):
                others = [w for w in range(K_WAVES) if w != lag and not wg.finished(w)]
                if not others:
                    break
                wg.advance(others[rng.integers(len(others))])
            if not wg.finished(lag):
                wg.advance(lag)
        quanta += 1
        assert quanta < 10_000_000, "the waves stopped making progress (a wait that never ends)"


def shapes(rng, count):
    for _ in range(count):
        n = int(rng.integers(17, 1400))
        rows = int(rng.integers(1, 700))
        n_panels = (n + K_PANEL - 1) // K_PANEL
        yield n, rows, int(rng.integers(n_panels))


@pytest.mark.parametrize("style", ["uniform", "bursts", "laggard"])
def test_every_column_has_one_owner_at_any_time(style):
    rng = np.random.default_rng({"uniform": 1, "bursts": 2, "laggard": 3}[style])
    # the shapes of the GPU regression test (ragged last rounds) and random ones
    fixed = [(685, 685, 5), (685, 344, 0), (300, 300, 2), (1000, 504, 7), (130, 130, 1), (17, 17, 0), (2048, 2048, 3)]
    for n, rows, panel in fixed + list(shapes(rng, 60)):
        wg = Workgroup(n, rows, panel)
        run(wg, rng, style)
        # every (strip, tile) of the chunk went through its column phase exactly once, and every wave made every step
        assert len(wg.strip_tiles) == wg.nstrips * wg.tiles and wg.col_work.sum() == wg.nstrips * wg.tiles
        assert wg.done == [wg.nsteps] * K_WAVES and wg.owner == [None] * K_TILES


def test_model_catches_idle_waves_that_do_not_wait():
    """The planted mistake: a wave without work publishes its step without looking at its neighbour.  The wave behind
    it then takes a column over while the wave in front may still be inside it.  On a chunk whose last round has strips
    for only some of the waves, a schedule that starves one working wave runs into it."""
    rng = np.random.default_rng(7)
    hits = 0
    for trial in range(40):
        wg = Workgroup(685, 685, int(rng.integers(6)), idle_waves_wait=False)
        try:
            run(wg, rng, "laggard")
        except AssertionError as err:
            assert "enters column" in str(err)
            hits += 1
    assert hits > 0
