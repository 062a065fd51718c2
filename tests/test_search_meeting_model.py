"""Host model of the meetings between the thread blocks that share a row in the general threshold
search of top-k (Definition 2): every interleaving of the blocks' atomic steps is enumerated for a few
blocks, meetings and poll budgets, and the row's result must be written exactly once in each of them.

The model states the protocol, not the device code: a block arrives at a meeting (one atomic add),
then polls a give-up flag and the arrival counter a bounded number of times; a block whose budget ends
sets the flag and leaves.  In the form `shared_last_meeting` every block waits at the last meeting and
the block whose range holds the rank-th tie writes the result, block 0 repeating the search alone when
its own wait ran out.  That form loses the result when the owner's budget ends just before the final
arrival while block 0 has already seen the counter reach its target -- the model finds that
interleaving.  In the form the kernel uses (`block0_last_meeting`) the other blocks only arrive at the
last meeting and block 0 alone writes, after its wait or after searching alone; no interleaving loses
or doubles the result.
"""
import itertools

import pytest

PASS, FAIL = "pass", "fail"


def _explore(B, meetings, budget, owner, protocol):
    """All reachable final states of the model.  A block's local state is (meeting, phase, polls) or a
    final verdict.  Shared state: arrivals, give-up flag, number of result writes."""
    # phases inside a meeting: 0 arrive, 1 poll the flag, 2 poll the counter
    start = tuple((0, 0, 0) for _ in range(B))
    finals = set()
    seen = set()
    stack = [(start, 0, 0, 0)]
    while stack:
        state = stack.pop()
        if state in seen:
            continue
        seen.add(state)
        blocks, arrivals, flag, writes = state
        runnable = [b for b in range(B) if not isinstance(blocks[b], str)]
        if not runnable:
            finals.add((blocks, writes))
            continue
        for b in runnable:
            m, phase, polls = blocks[b]
            nb, na, nf, nw = list(blocks), arrivals, flag, writes
            last = m == meetings - 1
            target = B * (m + 1)

            def leave(passed):
                """What block b does once the meetings are over for it."""
                nonlocal nw
                if protocol == "shared_last_meeting":
                    if passed and b == owner:
                        nw += 1                      # the owner walks its ties and writes
                    if not passed and b == 0:
                        nw += 1                      # block 0 searches alone and writes
                else:
                    if b == 0:
                        nw += 1                      # after its wait, or after searching alone
                nb[b] = PASS if passed else FAIL

            if phase == 0:
                na += 1
                if protocol == "block0_last_meeting" and last and b != 0:
                    leave(True)                      # arrive and leave without waiting
                else:
                    nb[b] = (m, 1, polls)
            elif phase == 1:
                if polls >= budget:                  # the wait ran out: flag the row and leave
                    nf = 1
                    leave(False)
                elif flag:
                    nf = 1
                    leave(False)
                else:
                    nb[b] = (m, 2, polls)
            else:
                if arrivals >= target:
                    if last:
                        leave(True)
                    else:
                        nb[b] = (m + 1, 0, 0)
                else:
                    nb[b] = (m, 1, polls + 1)
            stack.append((tuple(nb), na, nf, nw))
    return finals


CASES = list(itertools.product([2, 3], [1, 2, 3], [0, 1, 2, 3]))


@pytest.mark.parametrize("B,meetings,budget", CASES)
def test_block0_as_the_only_writer_never_loses_the_result(B, meetings, budget):
    for owner in range(B):
        finals = _explore(B, meetings, budget, owner, "block0_last_meeting")
        assert finals, "the model must terminate"
        for blocks, writes in finals:
            assert writes == 1, f"B={B} meetings={meetings} budget={budget} owner={owner}: {blocks} wrote {writes} times"


def test_a_shared_last_meeting_can_lose_the_result():
    """B = 3, the owner is block 2 and its budget ends between the last two arrivals: blocks 0 and 1 pass,
    block 2 gives up, nobody writes."""
    finals = _explore(3, 2, 1, owner=2, protocol="shared_last_meeting")
    lost = [blocks for blocks, writes in finals if writes == 0]
    assert lost, "the model should find the interleaving in which no block writes the row's result"
    assert any(blocks[0] == PASS and blocks[2] == FAIL for blocks in lost)
    # with the owner being block 0 itself that form is safe: it writes after a pass and after a failure
    for _, writes in _explore(3, 2, 1, owner=0, protocol="shared_last_meeting"):
        assert writes >= 1


def test_a_budget_of_zero_sends_every_row_to_block_0_alone():
    for blocks, writes in _explore(3, 3, 0, owner=1, protocol="block0_last_meeting"):
        assert blocks[0] == FAIL and writes == 1
