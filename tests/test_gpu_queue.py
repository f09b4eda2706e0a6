"""The request queue (batch former + pipelined runner) through the C ABI: batches are formed by the paper's rule
(append to the last batch until it is full, Sec. 4.2), run in order with the next batch's tenants prefetched under the
current batch (Sec. 6.2), and every request's rows come back as its own tenant's layer computes them (oracle)."""
import numpy as np
import pytest
import torch

import synth
from oracle import hmi_oracle as O
from tests.oracle_side import compare, weights_of

pytestmark = pytest.mark.gpu


class TierModel:
    """Host mirror of the pool's residency policy: forward calls and prefetch calls both advance the clock; a tenant
    that is not resident takes a free slot, else the least recently used slot that the current call has not touched
    (ties: lowest tenant id); a prefetch stops quietly when no such slot is left."""

    def __init__(self, slots, resident):
        self.slots, self.clock = slots, 0
        self.stamp = {t: 0 for t in resident}
        self.hits = self.misses = self.evictions = 0

    def _place(self, t):
        if len(self.stamp) >= self.slots:
            old = [(s, v) for v, s in self.stamp.items() if s < self.clock]
            if not old:
                return False
            del self.stamp[min(old)[1]]
            self.evictions += 1
        self.stamp[t] = self.clock
        return True

    def forward(self, distinct):
        self.clock += 1
        for t in distinct:
            if t in self.stamp:
                self.stamp[t] = self.clock
        for t in distinct:
            if t in self.stamp:
                self.hits += 1
            else:
                self.misses += 1
                assert self._place(t)

    def prefetch(self, distinct):
        self.clock += 1
        for t in distinct:
            if t in self.stamp:
                self.stamp[t] = self.clock
        for t in distinct:
            if t not in self.stamp and not self._place(t):
                break


def form_batches(reqs, max_req, max_tok, slots):
    """The batching rule, in Python: -> list of lists of request indices."""
    batches, cur, tok, tenants = [], [], 0, set()
    for i, (t, n) in enumerate(reqs):
        if cur and (len(cur) == max_req or tok + n > max_tok or (t not in tenants and len(tenants) == slots)):
            batches.append(cur)
            cur, tok, tenants = [], 0, set()
        cur.append(i)
        tok += n
        tenants.add(t)
    if cur:
        batches.append(cur)
    return batches


def test_queue_forms_batches_runs_them_in_order_and_prefetches_the_next(hmi):
    from paper_2504_17449_amd import harness
    slots, max_req, max_tok = 5, 8, 200
    wl = synth.Workload(name="queue_small", block=synth.BLOCK_ENC_POSTLN, dtype="bf16", d_model=128, d_ff=256, n_heads=2,
                        n_layers=1, n_tenants=30, n_requests=70, seq_min=1, seq_max=60, popularity="zipf", zipf_s=0.7,
                        ln_eps=1e-12, hbm_slots=slots, host_tier=True, seed=23)
    ids, lens = synth.batch_ids_lens(wl)
    reqs = [(int(t), int(n)) for t, n in zip(ids, lens)]
    want_batches = form_batches(reqs, max_req, max_tok, slots)
    assert len(want_batches) > 8 and any(len(b) < max_req for b in want_batches[:-1])    # tokens / tenants close batches too
    pool = harness.create_pool(wl, max_requests=max_req, max_tokens=max_tok)
    q = None
    try:
        harness.load_tenants(pool, wl)
        model = TierModel(slots, range(slots))                    # tenants 0..4 took the free slots at load
        q = hmi.Queue(pool, max_req, max_tok, max_waiting_batches=2)
        xs = [harness.host_to_device(synth.hidden_states(wl, r, n), "bf16") for r, (_, n) in enumerate(reqs)]
        ys = [torch.empty_like(x) for x in xs]
        tickets, ran = [None] * len(reqs), []

        def run_one():
            b, n = q.run()
            assert b == len(ran) and n == len(want_batches[b])    # in order, formed by the rule
            distinct = list(dict.fromkeys(reqs[i][0] for i in want_batches[b]))
            model.forward(distinct)
            if b + 1 < len(want_batches) and (b + 1 < opened[0]):
                model.prefetch(list(dict.fromkeys(reqs[i][0] for i in want_batches[b + 1])))
            ran.append(b)
            for i in want_batches[b]:
                q.fetch(tickets[i], ys[i])

        opened = [0]                                             # batches the queue has opened so far
        for i, (t, n) in enumerate(reqs):
            ticket = q.push(t, xs[i])
            if ticket is None:                                   # two batches are waiting: run the older one, then push again
                assert q.waiting() == 2
                run_one()
                ticket = q.push(t, xs[i])
                assert ticket is not None
            tickets[i] = ticket
            opened[0] = (ticket >> 20) + 1
            assert ticket >> 20 == next(b for b, members in enumerate(want_batches) if i in members)
        while q.waiting():
            run_one()
        assert q.run() == (-1, 0)
        torch.cuda.synchronize()
        assert len(ran) == len(want_batches)
        st = pool.stats()
        assert (st["hits"], st["misses"], st["evictions"]) == (model.hits, model.misses, model.evictions), (st, vars(model))
        assert st["evictions"] > 10 and st["hits"] > st["misses"]      # the prefetch turned most lookups into hits
        # every request against its own tenant's layer
        wof = weights_of(wl, 0)
        worst = (0.0, 0.0)
        for i, (t, n) in enumerate(reqs):
            y_ref = O.block_forward(wl.block, synth.hidden_states(wl, i, n).astype(np.float64), wof(t), wl.n_heads, wl.ln_eps)
            max_abs, rel, ok = compare(harness.device_to_f64(ys[i]), y_ref, np.arange(n), "bf16")
            assert ok, (i, t, n, max_abs, rel)
            worst = max(worst, (max_abs, rel))
        print(f"  {len(reqs)} requests in {len(want_batches)} batches, stats {st}, worst max_abs {worst[0]:.3e}", flush=True)
        # errors: nothing changes
        assert hmi.hmi_queue_push(q.h, 99, 4, xs[0].data_ptr())[0] == hmi.HMI_ERR_TENANT
        assert hmi.hmi_queue_push(q.h, 1, max_tok + 1, xs[0].data_ptr())[0] == hmi.HMI_ERR_SHAPE
        assert hmi.hmi_queue_fetch(q.h, tickets[0], ys[0].data_ptr()) == hmi.HMI_ERR_ARG      # results of batch 0 were given up long ago
        t_new = q.push(2, xs[0])
        assert hmi.hmi_queue_fetch(q.h, t_new, ys[0].data_ptr()) == hmi.HMI_ERR_ARG           # not run yet
        assert q.waiting() == 1
    finally:
        if q is not None:
            q.close()
        pool.close()


def test_queue_output_is_the_stack_call_on_the_gathered_batch_bit_for_bit(hmi):
    """A pool without host tier (nothing to prefetch), two layers, requests scattered over separate device buffers:
    what a request fetches from the queue is bit for bit what hmi_stack_forward writes for it when the same batch is
    handed over as one packed tensor; batches close on the token limit."""
    from paper_2504_17449_amd import harness
    max_req, max_tok = 16, 300
    wl = synth.Workload(name="queue_resident", block=synth.BLOCK_FFN, dtype="bf16", d_model=256, d_ff=512, n_heads=0,
                        n_layers=2, n_tenants=6, n_requests=40, seq_min=3, seq_max=90, popularity="uniform", zipf_s=0.0,
                        ln_eps=1e-12, hbm_slots=6, host_tier=False, seed=5)
    ids, lens = synth.batch_ids_lens(wl)
    reqs = [(int(t), int(n)) for t, n in zip(ids, lens)]
    want_batches = form_batches(reqs, max_req, max_tok, wl.hbm_slots)
    assert len(want_batches) >= 4 and all(len(b) < max_req for b in want_batches)       # the token limit closes them
    pool = harness.create_pool(wl, max_requests=max_req, max_tokens=max_tok)
    q = None
    try:
        harness.load_tenants(pool, wl)
        q = hmi.Queue(pool, max_req, max_tok, max_waiting_batches=len(want_batches))
        xs = [harness.host_to_device(synth.hidden_states(wl, r, n), "bf16") for r, (_, n) in enumerate(reqs)]
        ys = [torch.zeros_like(x) for x in xs]
        tickets = [q.push(t, xs[i]) for i, (t, _) in enumerate(reqs)]
        assert None not in tickets and q.waiting() == len(want_batches)
        for b, members in enumerate(want_batches):
            assert q.run() == (b, len(members))
            for i in members:
                q.fetch(tickets[i], ys[i])
        torch.cuda.synchronize()
        for members in want_batches:
            xb = torch.cat([xs[i] for i in members])
            yb = torch.empty_like(xb)
            pool.stack_forward(0, wl.n_layers, xb, yb, np.array([reqs[i][0] for i in members], np.int32),
                               np.array([reqs[i][1] for i in members], np.int32))
            torch.cuda.synchronize()
            off = 0
            for i in members:
                n = reqs[i][1]
                assert torch.equal(ys[i].view(torch.int16), yb[off:off + n].view(torch.int16)), i
                off += n
        # and against the oracle, every request
        wofs = [weights_of(wl, l) for l in range(wl.n_layers)]
        for i, (t, n) in enumerate(reqs):
            h = synth.hidden_states(wl, i, n).astype(np.float64)
            for l in range(wl.n_layers):
                h = O.block_forward(wl.block, h, wofs[l](t), wl.n_heads, wl.ln_eps)
            max_abs, rel, ok = compare(harness.device_to_f64(ys[i]), h, np.arange(n), "bf16")
            assert ok, (i, t, n, max_abs, rel)
    finally:
        if q is not None:
            q.close()
        pool.close()
