"""CPU oracle for transition-minimizing scheduling over the tiered KV buffer.
TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product path never does, and shares no code with it.

What is computed: the order of the engine's actions for an offline workload.
The paper fixes the policy in words (section 4.2 "Tiered KV Cache Buffering and
Transition-minimizing Scheduling", Figure 6; section 5.2 "Asynchronous
swap-in"):

  * prefill runs batch after batch and every generated KV cache goes to the CPU
    store; the switch to decoding happens only when that store is full;
  * during decoding continuous batching runs as usual, except that new
    sequences come on board by swapping their cache in from the CPU store
    whenever the GPU store has room; the prefetch is asynchronous and a
    sequence is scheduled for decoding only after its cache has arrived;
  * the switch back to prefilling happens only when the whole CPU store has
    been moved to the GPU.

What the paper leaves open, and the reading taken (each is a deterministic rule
so that two implementations can be compared action by action):

  * batch formation: requests are served in arrival order; a prefill batch takes
    requests while the sum of prompt lengths stays within `max_prefill_tokens`
    (a longer single prompt forms a batch of its own) and the pages of its prompts fit the
    GPU store;
  * "full": the next request's prompt does not fit in what is left of the CPU
    store (capacity counted in tokens; the store is empty whenever a prefill
    phase starts, so there is no fragmentation);
  * a request that wants one token only is finished by its prefill and never
    enters the store;
  * GPU room: a sequence is admitted when the pages of its final length
    (prompt + outputs - 1 cached tokens) fit next to those already promised to
    admitted sequences, and the number of admitted sequences stays within
    `max_decode_seqs`; admission is first-in first-out, at most `swap_in_group`
    sequences per iteration (0: no limit), so that decoding can begin while the
    rest of the store is still on its way;
  * arrival of a prefetch: caches requested during iteration t are on board at
    the start of iteration t + 1;
  * sequences still decoding when the store runs empty keep their GPU pages
    through the next prefill phase and continue in the next decode phase; with
    no request left to prefill, decoding simply runs until all are finished.

Pure Python on integers: every decision is exact.
"""

PREFILL, TO_DECODE, SWAP_IN, DECODE, TO_PREFILL, FINISH = 1, 2, 3, 4, 5, 6


def pages_of(tokens, page_size=16):
    return -(-tokens // page_size)


def simulate(prompt_lens, out_lens, tier_tokens, gpu_pages, max_prefill_tokens, max_decode_seqs, page_size=16,
             swap_in_group=0):
    """Returns (trace, stats).  trace is a list of (code, [request ids]):
    PREFILL batch, TO_DECODE [], SWAP_IN requested, DECODE step over the ids,
    TO_PREFILL [], FINISH ids (after the action that produced their last token)."""
    n = len(prompt_lens)
    for i in range(n):
        if prompt_lens[i] < 1 or out_lens[i] < 1:
            raise ValueError("lengths must be positive")
        if out_lens[i] > 1 and prompt_lens[i] > tier_tokens:
            raise ValueError("request %d does not fit the CPU store" % i)
        if out_lens[i] > 1 and pages_of(prompt_lens[i] + out_lens[i] - 1, page_size) > gpu_pages:
            raise ValueError("request %d does not fit the GPU store" % i)
        if pages_of(prompt_lens[i], page_size) > gpu_pages:
            raise ValueError("prompt %d does not fit the GPU store" % i)
    trace = []
    waiting = list(range(n))            # arrival order
    store = []                          # CPU store, first in first out
    store_used = 0
    running = []                        # on board, in order of admission
    arriving = []                       # requested in the previous iteration
    promised = 0                        # GPU pages promised to admitted sequences
    produced = [0] * n
    stats = {"prefill_batches": 0, "decode_steps": 0, "to_decode": 0, "to_prefill": 0, "tokens": 0,
             "max_store_tokens": 0, "max_promised_pages": 0, "max_running": 0}

    def final_pages(i):
        return pages_of(prompt_lens[i] + out_lens[i] - 1, page_size)

    while waiting or store or running or arriving:
        # ---------------- prefill phase: until the store is full or nothing is left to prefill
        full = False
        while waiting and not full:
            batch, tokens, pages = [], 0, 0
            while waiting:
                r = waiting[0]
                need = prompt_lens[r] if out_lens[r] > 1 else 0
                if store_used + need > tier_tokens:
                    full = True
                    break
                if batch and tokens + prompt_lens[r] > max_prefill_tokens:
                    break
                if batch and pages + pages_of(prompt_lens[r], page_size) > gpu_pages:
                    break
                waiting.pop(0)
                batch.append(r)
                tokens += prompt_lens[r]
                pages += pages_of(prompt_lens[r], page_size)
                store_used += need
            if not batch:
                break
            trace.append((PREFILL, list(batch)))
            stats["prefill_batches"] += 1
            done = []
            for r in batch:
                produced[r] = 1
                stats["tokens"] += 1
                if out_lens[r] == 1:
                    done.append(r)
                else:
                    store.append(r)
            stats["max_store_tokens"] = max(stats["max_store_tokens"], store_used)
            if done:
                trace.append((FINISH, done))
        if not (store or running or arriving):
            continue                     # everything prefilled so far finished at once; more may be waiting
        # ---------------- decode phase
        trace.append((TO_DECODE, []))
        stats["to_decode"] += 1
        while True:
            running.extend(arriving)     # last iteration's prefetches are on board
            for r in arriving:
                store_used -= prompt_lens[r]
            arriving = []
            asked = []
            while store and promised + final_pages(store[0]) <= gpu_pages and \
                    len(running) + len(asked) < max_decode_seqs and \
                    (swap_in_group <= 0 or len(asked) < swap_in_group):
                r = store.pop(0)
                promised += final_pages(r)
                asked.append(r)
            if asked:
                trace.append((SWAP_IN, list(asked)))
                arriving = asked
            stats["max_promised_pages"] = max(stats["max_promised_pages"], promised)
            stepped = bool(running)
            if running:
                trace.append((DECODE, list(running)))
                stats["decode_steps"] += 1
                stats["max_running"] = max(stats["max_running"], len(running))
                done = []
                for r in running:
                    produced[r] += 1
                    stats["tokens"] += 1
                    if produced[r] == out_lens[r]:
                        done.append(r)
                if done:
                    trace.append((FINISH, done))
                    for r in done:
                        promised -= final_pages(r)
                    running = [r for r in running if r not in done]
            if not store and not arriving:
                if waiting:              # the whole store has moved to the GPU: back to prefilling
                    trace.append((TO_PREFILL, []))
                    stats["to_prefill"] += 1
                    break
                if not running:
                    break
            elif not stepped and not asked:
                raise RuntimeError("no progress: head of the store cannot be admitted")
    assert produced == list(out_lens)
    return trace, stats
