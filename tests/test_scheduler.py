"""Request scheduler (paper Sec. 4.2.1): the oracle model is pinned to a hand-worked example,
to the closed-form steady state and to invariants; the library's scheduler (host-only C++,
called through the C ABI) must then form exactly the oracle's batches."""
import os

import numpy as np
import pytest

from oracle.batch_formation import BatchFormation
from paper_2408_12757_amd import binding as nf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "batch_formation_example.txt")


def drive(sched, requests, lag, max_iters=100000, arrivals=None):
    """Runs a scheduler model to completion.  arrivals[i] = iteration at which request i is
    submitted (default: all at the start).  Returns the list of batches."""
    arrivals = arrivals or [0] * len(requests)
    order = sorted(range(len(requests)), key=lambda i: (arrivals[i], i))
    batches, nxt = [], 0
    for it in range(max_iters):
        while nxt < len(order) and arrivals[order[nxt]] <= it:
            p, o = requests[order[nxt]]
            sched.submit(p, o)
            nxt += 1
        b = sched.next_batch()
        batches.append(b)
        if it - lag >= 0:
            sched.complete(it - lag)
        if nxt == len(order) and b["n_tokens"] == 0 and not sched.requests:
            # drain the iterations still in flight
            for k in range(max(0, it - lag + 1), it + 1):
                sched.complete(k)
            return batches
    raise AssertionError("scheduler did not finish")


# ------------------------------------------------------------------ oracle pins ---

def test_oracle_reproduces_the_hand_worked_example():
    reqs = [(5, 3), (6, 2), (9, 1), (2, 2)]
    s = BatchFormation(dense_batch=8, page_size=4, num_pages=64, max_requests=16, avg_decode_len=3)
    got = drive(s, reqs, lag=0)
    want = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        want[int(f[0])] = [tuple(e.split(":")) for e in f[1:]]
    assert len(got) >= len(want)
    for it, entries in want.items():
        mine = [(f"r{e['rid']}", "D" if e["decode"] else "P", str(e["q_len"]), str(e["ctx_len"]))
                for e in got[it]["entries"]]
        assert mine == entries, (it, mine, entries)


def check_invariants(batches, requests, dense_batch, page_size, num_pages, lag, expect_full=True):
    """Token conservation, decode-first, exact fill, page exclusivity."""
    n = len(requests)
    prefilled, decoded = [0] * n, [0] * n
    for b in batches:
        assert b["n_tokens"] <= dense_batch
        kinds = [e["decode"] for e in b["entries"]]
        assert kinds == sorted(kinds), "prefill entries come first, then decode entries"
        owners = {}
        for e in b["entries"]:
            rid, q = e["rid"], e["q_len"]
            assert e["ctx_len"] == prefilled[rid] + decoded[rid], "a request's tokens are scheduled in order"
            need = -(-(e["ctx_len"] + q) // page_size)
            assert len(e["pages"]) >= need and len(set(e["pages"])) == len(e["pages"])
            for p in e["pages"]:
                assert 0 <= p < num_pages
                assert owners.setdefault(p, rid) == rid, "a page belongs to one request at a time"
            if e["decode"]:
                assert q == 1 and prefilled[rid] == requests[rid][0]
                decoded[rid] += 1
            else:
                prefilled[rid] += q
                assert prefilled[rid] <= requests[rid][0]
    for rid, (p, o) in enumerate(requests):
        assert prefilled[rid] == p, "every prompt token is prefilled exactly once"
        # o - 1 decode iterations are needed; the end is seen `lag` iterations late
        assert o - 1 <= decoded[rid] <= o - 1 + lag, (rid, decoded[rid], o)
    if expect_full:
        # while prompt tokens are waiting the batch is filled exactly
        remaining = sum(p for p, _ in requests)
        for b in batches:
            pf = sum(e["q_len"] for e in b["entries"] if not e["decode"])
            remaining -= pf
            if remaining > 0:
                assert b["n_tokens"] == dense_batch, (b["iteration"], b["n_tokens"])


@pytest.mark.parametrize("lag", [0, 1, 2])
def test_oracle_invariants_on_random_streams(lag):
    rng = np.random.default_rng(11 + lag)
    reqs = [(int(rng.integers(1, 90)), int(rng.integers(1, 40))) for _ in range(120)]
    s = BatchFormation(dense_batch=64, page_size=4, num_pages=4000, max_requests=64, avg_decode_len=20)
    batches = drive(s, reqs, lag)
    check_invariants(batches, reqs, 64, 4, 4000, lag)
    assert len(s.free) == 4000 and not s.resident and not s.swapped and not s.waiting
    assert all(not b["swap_out"] for b in batches)


def test_oracle_steady_state_matches_the_closed_form():
    """Constant lengths: a request takes p prefill tokens and d - 1 decode tokens, so a full
    batch of B tokens retires B / (p + d - 1) requests per iteration and holds
    B (d - 1) / (p + d - 1) decode requests (Sec. 4.2.1: the numbers of decode and prefill
    requests stabilise)."""
    B, p, d = 64, 24, 9
    reqs = [(p, d)] * 400
    s = BatchFormation(dense_batch=B, page_size=4, num_pages=100000, max_requests=1000, avg_decode_len=d)
    batches = drive(s, reqs, lag=0)
    steady = batches[60:-60]
    n_dec = np.mean([b["n_decode"] for b in steady])
    assert abs(n_dec - B * (d - 1) / (p + d - 1)) < 0.75, n_dec
    assert all(b["n_tokens"] == B for b in steady)


def test_oracle_prediction_prevents_swapping_when_lengths_match_the_average():
    """All outputs equal the average: the predicted peak is exact, so no request is ever
    swapped out, and the pool is used up to what the prediction allows."""
    P, NP, p, d = 4, 120, 30, 11
    reqs = [(p, d)] * 60
    s = BatchFormation(dense_batch=32, page_size=P, num_pages=NP, max_requests=100, avg_decode_len=d)
    batches = drive(s, reqs, lag=0)
    check_invariants(batches, reqs, 32, P, NP, 0, expect_full=False)
    assert all(not b["swap_out"] for b in batches)
    per_req = -(-(p + d - 1) // P)
    peak_resident = max(len({e["rid"] for e in b["entries"]}) for b in batches)
    assert peak_resident <= NP // per_req + 1


def test_oracle_swaps_out_and_reloads_when_outputs_exceed_the_prediction():
    """Outputs far above the average make the prediction optimistic: decode requests are
    swapped out when the pool runs dry and come back; every request still gets all its tokens."""
    rng = np.random.default_rng(5)
    reqs = [(int(rng.integers(8, 24)), int(rng.integers(60, 120))) for _ in range(40)]
    s = BatchFormation(dense_batch=32, page_size=4, num_pages=150, max_requests=64, avg_decode_len=4)
    batches = drive(s, reqs, lag=1)
    check_invariants(batches, reqs, 32, 4, 150, 1, expect_full=False)
    n_out = sum(len(b["swap_out"]) for b in batches)
    n_in = sum(len(b["swap_in"]) for b in batches)
    assert n_out > 0 and n_out == n_in + sum(len(b["released"]) for b in batches)
    # a reloaded request gets as many pages as were saved
    saved = {}
    for b in batches:
        for rid, pages in b["swap_out"]:
            saved[rid] = len(pages)
        for rid, pages in b["swap_in"]:
            assert len(pages) == saved.pop(rid)
    assert len(s.free) == 150


# --------------------------------------------- the library against the oracle ---

def lib_batch_as_dict(fb):
    entries = []
    for i in range(fb.n_prefill_reqs + fb.n_decode_reqs):
        entries.append({"rid": int(fb.request_ids[i]), "q_len": int(fb.q_indptr[i + 1] - fb.q_indptr[i]),
                        "ctx_len": int(fb.ctx_len[i]),
                        "pages": [int(x) for x in fb.page_ids[fb.page_indptr[i]:fb.page_indptr[i + 1]]],
                        "decode": i >= fb.n_prefill_reqs})
    return {"iteration": fb.iteration, "entries": entries, "n_prefill": fb.n_prefill_reqs, "n_decode": fb.n_decode_reqs,
            "n_tokens": fb.n_tokens, "swap_out": [(r, [int(x) for x in p]) for r, p in fb.swap_out],
            "swap_in": [(r, [int(x) for x in p]) for r, p in fb.swap_in], "released": list(fb.released),
            "finished": list(fb.finished)}


def test_a_request_the_prediction_would_never_admit_still_runs_when_alone():
    """Long prompt, short output, tight pool, large average output length: the predicted peak
    (prompt + average output) exceeds the pool although the request itself fits.  With nothing
    resident it must be admitted anyway - submit accepted it - in the oracle and in the library;
    otherwise every batch would be empty for ever."""
    B, P, NP, avg = 32, 4, 30, 64.0          # 120 token slots; prediction wants 100 + 64
    reqs = [(100, 3), (90, 2)]
    oracle = BatchFormation(B, P, NP, 8, 0, 0, avg)
    batches = drive(oracle, reqs, lag=0)
    assert sum(b["n_tokens"] for b in batches) == 100 + 2 + 90 + 1
    assert len(oracle.free) == NP
    s = nf.Scheduler(B, P, NP, 8, 0, 0, avg)
    for p_len, o_len in reqs:
        s.submit(p_len, o_len)
    tokens, it = 0, 0
    for _ in range(64):
        b = s.next_batch()
        tokens += b.n_tokens
        s.complete(it)
        it += 1
        st = s.stats()
        if st["waiting"] + st["resident"] + st["swapped"] == 0:
            break
    assert tokens == 100 + 2 + 90 + 1 and s.stats()["finished"] == 2
    s.close()


CASES = [
    # name, dense_batch, page_size, num_pages, max_requests, max_chunk, reserve, avg, lag, n_req, prompt range, output range
    ("roomy", 64, 4, 5000, 64, 0, 0, 20.0, 0, 150, (1, 90), (1, 40)),
    ("async", 64, 16, 2000, 48, 0, 0, 16.0, 1, 150, (1, 200), (1, 50)),
    ("chunk_cap", 48, 4, 3000, 32, 16, 5, 10.0, 1, 100, (1, 120), (1, 30)),
    ("tight_pool", 32, 4, 150, 64, 0, 0, 4.0, 1, 40, (8, 24), (60, 120)),
    ("tight_pool_sync", 32, 4, 200, 20, 0, 3, 8.0, 0, 60, (4, 40), (1, 150)),
    ("few_slots", 16, 2, 400, 3, 0, 0, 5.0, 2, 30, (1, 30), (1, 12)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_library_scheduler_forms_the_oracle_batches(case):
    name, B, P, NP, maxr, chunk, reserve, avg, lag, n, pr, orng = case
    rng = np.random.default_rng(hash(name) % 1000)
    reqs = [(int(rng.integers(pr[0], pr[1] + 1)), int(rng.integers(orng[0], orng[1] + 1))) for _ in range(n)]
    arrivals = sorted(int(x) for x in rng.integers(0, 40, size=n))
    oracle = BatchFormation(B, P, NP, maxr, chunk, reserve, avg)
    want = drive(oracle, reqs, lag, arrivals=arrivals)

    class LibModel:
        def __init__(self):
            self.s = nf.Scheduler(B, P, NP, maxr, chunk, reserve, avg)
            self.requests = True

        def submit(self, p, o):
            return self.s.submit(p, o)

        def next_batch(self):
            b = lib_batch_as_dict(self.s.next_batch())
            st = self.s.stats()
            self.requests = st["waiting"] + st["resident"] + st["swapped"] > 0
            return b

        def complete(self, k):
            self.s.complete(k)
            st = self.s.stats()
            self.requests = st["waiting"] + st["resident"] + st["swapped"] > 0

    model = LibModel()
    got = drive(model, reqs, lag, arrivals=arrivals)
    assert len(got) == len(want)
    for g, w in zip(got, want):
        assert g == w, (name, g["iteration"])
    st = model.s.stats()
    assert st["finished"] == n and st["free_pages"] == NP and st["wasted_decode_tokens"] == oracle.wasted
    assert st["prefill_tokens"] == sum(p for p, _ in reqs)
    if name.startswith("tight"):
        assert st["swap_outs"] > 0
    model.s.close()


def test_library_scheduler_rejects_bad_calls():
    with pytest.raises(nf.NfError):
        nf.Scheduler(0, 16, 100, 10)
    s = nf.Scheduler(64, 16, 10, 10, avg_decode_len=8)
    with pytest.raises(nf.NfError) as e:
        s.submit(200, 10)          # can never fit 10 pages
    assert e.value.status == nf.NF_EPAGES
    with pytest.raises(nf.NfError):
        s.submit(0, 1)
    with pytest.raises(nf.NfError):
        s.complete(0)              # nothing formed yet
    s.submit(5, 2)
    b = s.next_batch()
    assert b.n_tokens == 5 and b.n_prefill_reqs == 1
    with pytest.raises(nf.NfError):
        s.complete(1)              # out of order
    s.complete(0)
    s.close()
