"""Host-side model of the inter-workgroup protocols of the one-pass encoders: the range
words that workgroups exchange through the workspace, the waits on them, and the rule by
which the workspace is left all zero without a clearing pass.  Each wave is a coroutine
that yields at every access to the shared words; a seeded scheduler interleaves the waves
of all workgroups at random.  Checked on thousands of schedules: no wave ever waits for
a word that has already been cleared (that would hang the kernel), every wave sees all
words of its chunk, and every word and counter is zero at the end.

The model restates the protocol, it shares nothing with the kernels:
  rotated kernels   per item: [workgroup barrier] publish, wait for all words of the chunk,
                    clear the own word of the workgroup's PREVIOUS chunk
  one word per workgroup (more than 16 workers): wave 0 publishes behind the barrier and clears
  pipelined kernel  (unrotated bf16) no barriers: publish item k + 1, wait for item k,
                    clear the own word of item k - 2
  both              the workgroups of a chunk count themselves off for a workgroup's last
                    chunk(s); the last one clears all of the chunk's words and the counter
and a deliberately wrong variant (the pipelined kernel clearing item k - 1) must be caught.
"""
import random

import pytest


class Hang(Exception):
    pass


class World:
    def __init__(self, W, V, chunks, words_per_workgroup=None):
        self.W, self.V = W, V
        self.P = words_per_workgroup or V     # publishing waves per workgroup
        self.word = {(c, w, v): 0 for c in range(chunks) for w in range(W) for v in range(self.P)}
        self.done = [0] * chunks
        self.seen = {}            # (w, v, c) -> the words a wave saw when its wait ended

    def all_words(self, c):
        return [self.word[(c, w, v)] for w in range(self.W) for v in range(self.P)]


class Barrier:
    def __init__(self, parties):
        self.parties, self.count, self.generation = parties, 0, 0


def _barrier(bar):
    gen = bar.generation
    bar.count += 1
    if bar.count == bar.parties:
        bar.count = 0
        bar.generation += 1
    while bar.generation == gen:
        yield "barrier"


def _wait(world, c, me):
    while True:
        yield "poll"
        words = world.all_words(c)
        if all(x != 0 for x in words):
            world.seen[me + (c,)] = words
            return


def _count_off(world, c):
    yield "atomic"
    arrived = world.done[c]
    world.done[c] += 1
    if arrived == world.W - 1:
        for w in range(world.W):
            for v in range(world.P):
                yield "clear"
                world.word[(c, w, v)] = 0
        world.done[c] = 0


def rotated_wave(world, bar, w, v, items):
    """One word per wave; a workgroup barrier (the rotation's exchanges) in front of every publication."""
    prev = None
    for c in items:
        yield from _barrier(bar)
        yield "publish"
        world.word[(c, w, v)] = 100 + c
        yield from _wait(world, c, (w, v))
        if prev is not None:
            yield "clear"
            world.word[(prev, w, v)] = 0
        prev = c
    yield from _barrier(bar)
    if v == 0 and prev is not None:
        yield from _count_off(world, prev)


def workgroup_word_wave(world, bar, w, v, items):
    """One word per WORKGROUP (more than 16 workers): wave 0 publishes behind the barrier and
    clears; every wave polls."""
    prev = None
    for c in items:
        yield from _barrier(bar)
        if v == 0:
            yield "publish"
            world.word[(c, w, 0)] = 100 + c
        yield from _wait(world, c, (w, v))
        if v == 0 and prev is not None:
            yield "clear"
            world.word[(prev, w, 0)] = 0
        prev = c
    yield from _barrier(bar)
    if v == 0 and prev is not None:
        yield from _count_off(world, prev)


def pipelined_wave(world, bar, w, v, items, clear_lag=2):
    """No barrier between items: the range of item k + 1 is published before the wait for item k."""
    if not items:
        return
    yield "publish"
    world.word[(items[0], w, v)] = 100 + items[0]
    for k, c in enumerate(items):
        if k + 1 < len(items):
            yield "publish"
            world.word[(items[k + 1], w, v)] = 100 + items[k + 1]
        yield from _wait(world, c, (w, v))
        if k >= clear_lag:
            yield "clear"
            world.word[(items[k - clear_lag], w, v)] = 0
    yield from _barrier(bar)
    if v == 0:
        for c in items[-clear_lag:]:
            yield from _count_off(world, c)


def run(kind, W, V, groups, rounds, seed, words_per_workgroup=None, **kw):
    """groups peer groups of W workgroups; group q handles chunks q, q + groups, ..."""
    rng = random.Random(seed)
    chunks = groups * rounds
    world = World(W, V, chunks, words_per_workgroup)
    waves = []
    for q in range(groups):
        items = list(range(q, chunks, groups))
        for w in range(W):
            bar = Barrier(V)
            for v in range(V):
                waves.append(kind(world, bar, w, v, items, **kw))
    idle = 0
    while waves:
        i = rng.randrange(len(waves))
        before = (dict(world.word), list(world.done))
        try:
            step = next(waves[i])
        except StopIteration:
            waves.pop(i)
            idle = 0
            continue
        if step in ("poll", "barrier") and before == (world.word, world.done):
            idle += 1
            if idle > 2000 * len(waves):
                raise Hang(f"no progress: {len(waves)} waves stuck")
        else:
            idle = 0
    assert all(x == 0 for x in world.word.values()), "a range word is left set"
    assert all(x == 0 for x in world.done), "a counter is left set"
    for (w, v, c), words in world.seen.items():
        assert all(x == 100 + c for x in words), "a wave saw a word of another chunk"
    assert len(world.seen) == chunks * W * V
    return world


@pytest.mark.parametrize("W,V,groups,rounds", [(2, 2, 1, 1), (2, 2, 1, 4), (3, 2, 2, 3), (2, 3, 1, 5), (4, 1, 2, 4)])
def test_rotated_protocol_clears_itself_and_never_hangs(W, V, groups, rounds):
    for seed in range(300):
        run(rotated_wave, W, V, groups, rounds, seed)


@pytest.mark.parametrize("W,V,groups,rounds", [(2, 2, 1, 1), (2, 3, 1, 4), (3, 2, 2, 3), (5, 2, 1, 4)])
def test_workgroup_word_protocol_clears_itself_and_never_hangs(W, V, groups, rounds):
    for seed in range(300):
        run(workgroup_word_wave, W, V, groups, rounds, seed, words_per_workgroup=1)


@pytest.mark.parametrize("W,V,groups,rounds", [(2, 2, 1, 1), (2, 2, 1, 2), (2, 2, 1, 3), (3, 2, 2, 4), (2, 3, 1, 6), (4, 1, 2, 5)])
def test_pipelined_protocol_clears_itself_and_never_hangs(W, V, groups, rounds):
    for seed in range(300):
        run(pipelined_wave, W, V, groups, rounds, seed)


def test_the_model_catches_a_word_cleared_one_item_too_early():
    """Clearing the own word of item k - 1 after the wait for item k is wrong for the
    pipelined kernel (a peer may still be waiting for item k - 1): some schedule hangs."""
    caught = 0
    for seed in range(300):
        try:
            run(pipelined_wave, 2, 2, 1, 5, seed, clear_lag=1)
        except (Hang, AssertionError):
            caught += 1
    assert caught > 0
