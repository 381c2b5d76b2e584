"""A small model of how thc_encode_all's workgroups share and clear the range words of
a chunk (CPU only; no kernel code is involved).

The kernel's rules, restated here as a state machine and run under random schedules:

* a chunk has one word per wave of each of its W workgroups, zero = not yet published;
* a wave publishes its word for item k only after a workgroup barrier that all waves of
  its workgroup reach only after finishing their poll of item k - 1;
* a wave's poll of item k succeeds once all words of that chunk are non-zero;
* after its poll of item k succeeds, a wave clears its own word of item k - 1;
* after the last item a workgroup barrier, then one arrival per workgroup on the chunk's
  counter; the W-th arrival clears all words of the last chunk and the counter.

Checked for every schedule tried: no wave waits forever (a word it needs is never
cleared before it has read it), and the words and counters are all zero at the end.
"""
import random

import pytest


def run(W, waves, items, seed):
    rng = random.Random(seed)
    words = [[[0] * waves for _ in range(W)] for _ in range(items)]   # [item][workgroup][wave]
    counter = [0] * items
    # per wave: (phase, item); phases: "publish" -> "poll" -> next item ... -> "arrive" -> "done"
    phase = [[("publish", 0) for _ in range(waves)] for _ in range(W)]
    polled = [[-1] * waves for _ in range(W)]        # last item whose poll this wave finished
    arrived = [False] * W
    steps = 0
    while any(p[0] != "done" for wg in phase for p in wg):
        steps += 1
        assert steps < 200_000, "no progress: some wave waits for a word that was cleared too early"
        g, v = rng.randrange(W), rng.randrange(waves)
        ph, k = phase[g][v]
        if ph == "publish":
            # barrier of item k's rotation: every wave of the workgroup is past its poll of k - 1
            if all(polled[g][u] >= k - 1 for u in range(waves)):
                assert words[k][g][v] == 0
                words[k][g][v] = 1
                phase[g][v] = ("poll", k)
        elif ph == "poll":
            if all(words[k][h][u] for h in range(W) for u in range(waves)):
                if k > 0:
                    assert words[k - 1][g][v] == 1
                    words[k - 1][g][v] = 0           # own word of the previous item
                polled[g][v] = k
                phase[g][v] = ("publish", k + 1) if k + 1 < items else ("arrive", k)
        elif ph == "arrive":
            # barrier after the last item, then one arrival per workgroup (by its first wave)
            if all(polled[g][u] >= k for u in range(waves)):
                if v == 0 and not arrived[g]:
                    arrived[g] = True
                    counter[k] += 1
                    if counter[k] == W:
                        for h in range(W):
                            for u in range(waves):
                                words[k][h][u] = 0
                        counter[k] = 0
                phase[g][v] = ("done", k)
    return words, counter


@pytest.mark.parametrize("W,waves,items", [(1, 1, 1), (1, 8, 3), (2, 2, 1), (3, 2, 4), (8, 8, 3), (4, 3, 6)])
def test_words_are_never_cleared_early_and_end_up_zero(W, waves, items):
    for seed in range(40):
        words, counter = run(W, waves, items, seed)
        assert not any(x for item in words for wg in item for x in wg)
        assert not any(counter)


def test_model_detects_a_rule_that_clears_too_early():
    """The same machine with a wrong rule (a wave clears its own word of the CURRENT item
    right after its own poll) must get stuck: the check above is able to fail."""
    W, waves = 3, 2
    rng = random.Random(0)
    words = [[0] * waves for _ in range(W)]
    waiting = {(g, v) for g in range(W) for v in range(waves)}
    published = set()
    for _ in range(10_000):
        g, v = rng.randrange(W), rng.randrange(waves)
        if (g, v) not in published:
            words[g][v] = 1
            published.add((g, v))
        elif (g, v) in waiting and all(words[h][u] for h in range(W) for u in range(waves)):
            words[g][v] = 0                          # too early: the others have not read it yet
            waiting.discard((g, v))
    assert waiting, "clearing one's own word of the current item should strand the other waves"
