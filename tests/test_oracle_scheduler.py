"""Pins for the scheduling oracle (CPU only).

The paper gives the policy in words and a figure (section 4.2, Figure 6) and no
worked example, so the pins are traces worked out by hand from those rules on
tiny workloads, plus the properties the paper states: the switch to decoding
happens only when the CPU store is full (or nothing is left to prefill), the
switch back only when the store has been emptied onto the GPU, a sequence is
decoded only after its cache has been swapped in, and with an unbounded store
the engine changes stage once.
"""
import numpy as np
import pytest

from oracle import scheduler as sc

P, TD, IN, D, TP, F = sc.PREFILL, sc.TO_DECODE, sc.SWAP_IN, sc.DECODE, sc.TO_PREFILL, sc.FINISH


def test_hand_trace_everything_fits():
    trace, st = sc.simulate([4, 4, 4], [3, 3, 3], tier_tokens=100, gpu_pages=100, max_prefill_tokens=8, max_decode_seqs=10)
    assert trace == [(P, [0, 1]), (P, [2]), (TD, []), (IN, [0, 1, 2]), (D, [0, 1, 2]), (D, [0, 1, 2]), (F, [0, 1, 2])]
    assert (st["to_decode"], st["to_prefill"], st["tokens"]) == (1, 0, 9)


def test_hand_trace_store_full_forces_two_rounds():
    trace, st = sc.simulate([10] * 4, [2] * 4, tier_tokens=25, gpu_pages=100, max_prefill_tokens=100, max_decode_seqs=10)
    assert trace == [(P, [0, 1]), (TD, []), (IN, [0, 1]), (D, [0, 1]), (F, [0, 1]), (TP, []),
                     (P, [2, 3]), (TD, []), (IN, [2, 3]), (D, [2, 3]), (F, [2, 3])]
    assert (st["to_decode"], st["to_prefill"], st["max_store_tokens"]) == (2, 1, 20)


def test_hand_trace_gpu_pages_throttle_admission():
    # pages of 4 tokens; final lengths 8, 5, 5 tokens -> 2 pages each; the GPU holds 3 pages
    trace, st = sc.simulate([4, 4, 4], [5, 2, 2], tier_tokens=100, gpu_pages=3, max_prefill_tokens=100,
                            max_decode_seqs=10, page_size=4)
    assert trace == [(P, [0, 1, 2]), (TD, []), (IN, [0]), (D, [0]), (D, [0]), (D, [0]), (D, [0]), (F, [0]),
                     (IN, [1]), (D, [1]), (F, [1]), (IN, [2]), (D, [2]), (F, [2])]
    assert st["max_promised_pages"] == 2 and st["max_running"] == 1


def test_hand_trace_running_sequences_survive_a_prefill_phase():
    trace, st = sc.simulate([8, 8, 8], [4, 2, 2], tier_tokens=16, gpu_pages=100, max_prefill_tokens=100, max_decode_seqs=10)
    assert trace == [(P, [0, 1]), (TD, []), (IN, [0, 1]), (D, [0, 1]), (F, [1]), (TP, []),
                     (P, [2]), (TD, []), (IN, [2]), (D, [0]), (D, [0, 2]), (F, [0, 2])]


def test_single_token_requests_finish_at_prefill_and_skip_the_store():
    trace, st = sc.simulate([5, 5, 5], [1, 1, 3], tier_tokens=5, gpu_pages=10, max_prefill_tokens=100, max_decode_seqs=4)
    assert trace == [(P, [0, 1, 2]), (F, [0, 1]), (TD, []), (IN, [2]), (D, [2]), (D, [2]), (F, [2])]
    assert st["max_store_tokens"] == 5


def test_max_decode_seqs_limits_the_running_set():
    trace, st = sc.simulate([2] * 5, [3] * 5, tier_tokens=100, gpu_pages=100, max_prefill_tokens=100, max_decode_seqs=2)
    assert st["max_running"] == 2
    assert [ids for c, ids in trace if c == IN] == [[0, 1], [2, 3], [4]]


def test_hand_trace_swap_in_groups_let_decoding_start_early():
    trace, st = sc.simulate([4] * 3, [3] * 3, tier_tokens=100, gpu_pages=100, max_prefill_tokens=100, max_decode_seqs=10,
                            swap_in_group=1)
    assert trace == [(P, [0, 1, 2]), (TD, []), (IN, [0]), (IN, [1]), (D, [0]), (IN, [2]), (D, [0, 1]), (F, [0]),
                     (D, [1, 2]), (F, [1]), (D, [2]), (F, [2])]


def test_long_prompt_forms_its_own_batch():
    trace, _ = sc.simulate([3, 50, 3], [2, 2, 2], tier_tokens=100, gpu_pages=100, max_prefill_tokens=10, max_decode_seqs=8)
    assert [ids for c, ids in trace if c == P] == [[0], [1], [2]]


def test_prefill_batch_is_bounded_by_the_gpu_pages():
    # pages of 4 tokens, 3 pages: prompts of 3 tokens take a page each, so a batch holds three of them
    trace, _ = sc.simulate([3] * 5, [2] * 5, tier_tokens=100, gpu_pages=3, max_prefill_tokens=100, max_decode_seqs=8, page_size=4)
    assert [ids for c, ids in trace if c == P] == [[0, 1, 2], [3, 4]]


def _replay_and_check(prompt, out, tier, pages, mpt, mds, page_size=16, group=0):
    trace, st = sc.simulate(prompt, out, tier, pages, mpt, mds, page_size, group)
    n = len(prompt)
    state = ["waiting"] * n            # waiting -> store -> arriving -> running -> done
    produced = [0] * n
    store_tokens, promised = 0, 0
    next_waiting = 0
    stage = "prefill"
    arriving_prev = []
    for code, ids in trace:
        if code == P:
            assert stage == "prefill"
            assert ids == list(range(next_waiting, next_waiting + len(ids)))           # arrival order
            assert sum(prompt[i] for i in ids) <= mpt or len(ids) == 1
            assert sum(sc.pages_of(prompt[i], page_size) for i in ids) <= pages
            next_waiting += len(ids)
            for i in ids:
                assert state[i] == "waiting"
                produced[i] = 1
                if out[i] > 1:
                    state[i] = "store"
                    store_tokens += prompt[i]
                else:
                    state[i] = "last"
            assert store_tokens <= tier
        elif code == TD:
            assert stage == "prefill"
            # only when the store cannot take the next request, or nothing is left to prefill
            if next_waiting < n:
                need = prompt[next_waiting] if out[next_waiting] > 1 else 0
                assert store_tokens + need > tier
            stage = "decode"
            arriving_prev = []
        elif code == IN:
            assert stage == "decode"
            for i in ids:
                assert state[i] == "store"
                state[i] = "arriving"
                promised += sc.pages_of(prompt[i] + out[i] - 1, page_size)
            assert promised <= pages and (group <= 0 or len(ids) <= group)
            # first in first out: everything still in the store arrived later
            assert all(j > max(ids) for j in range(n) if state[j] == "store")
            arriving_prev = arriving_prev + ids
        elif code == D:
            assert stage == "decode" and ids
            for i in ids:
                if state[i] == "arriving":          # requested in an earlier iteration, by construction of the trace
                    assert i in arriving_prev
                    state[i] = "running"
                    store_tokens -= prompt[i]
                assert state[i] == "running"
                produced[i] += 1
                if produced[i] == out[i]:
                    state[i] = "last"
            assert len(ids) <= mds
            # continuous batching: everyone on board decodes in every step
            assert all(state[j] != "running" or j in ids for j in range(n))
        elif code == F:
            for i in ids:
                assert state[i] == "last" and produced[i] == out[i]
                state[i] = "done"
                if out[i] > 1:
                    promised -= sc.pages_of(prompt[i] + out[i] - 1, page_size)
        elif code == TP:
            assert stage == "decode"
            # arrivals of the last iteration count as moved: the store proper is empty and requests are waiting
            assert all(s not in ("store",) for s in state) and next_waiting < n
            stage = "prefill"
    assert all(s == "done" for s in state) and produced == list(out)
    assert st["tokens"] == sum(out)
    return trace, st


@pytest.mark.parametrize("seed", range(8))
def test_invariants_on_random_workloads(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 40))
    prompt = [int(v) for v in rng.integers(1, 200, n)]
    out = [int(v) for v in rng.integers(1, 30, n)]
    tier = int(max(prompt) + rng.integers(0, 600))
    page = 16
    pages = int(max(sc.pages_of(p + o - 1, page) for p, o in zip(prompt, out)) + rng.integers(0, 40))
    _replay_and_check(prompt, out, tier, pages, int(rng.integers(50, 400)), int(rng.integers(1, 12)), page, seed % 3)


def test_unbounded_store_changes_stage_once_and_tight_store_once_per_request():
    prompt, out = [7] * 12, [3] * 12
    _, st = sc.simulate(prompt, out, tier_tokens=10 ** 9, gpu_pages=10 ** 6, max_prefill_tokens=20, max_decode_seqs=100)
    assert (st["to_decode"], st["to_prefill"]) == (1, 0)
    _, st = sc.simulate(prompt, out, tier_tokens=7, gpu_pages=10 ** 6, max_prefill_tokens=20, max_decode_seqs=100)
    assert (st["to_decode"], st["to_prefill"]) == (12, 11)
    # a store of m requests: ceil(12 / m) rounds
    for m in (2, 3, 5):
        _, st = sc.simulate(prompt, out, tier_tokens=7 * m, gpu_pages=10 ** 6, max_prefill_tokens=20, max_decode_seqs=100)
        assert st["to_decode"] == -(-12 // m)


def test_requests_that_cannot_fit_are_refused():
    with pytest.raises(ValueError):
        sc.simulate([100], [2], tier_tokens=50, gpu_pages=100, max_prefill_tokens=10, max_decode_seqs=1)
    with pytest.raises(ValueError):
        sc.simulate([100], [2], tier_tokens=500, gpu_pages=2, max_prefill_tokens=10, max_decode_seqs=1)
    with pytest.raises(ValueError):
        sc.simulate([0], [2], tier_tokens=500, gpu_pages=2, max_prefill_tokens=10, max_decode_seqs=1)
