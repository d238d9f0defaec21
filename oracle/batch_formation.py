"""Oracle of the request scheduler (paper Sec. 4.2.1 "Request scheduling"): a plain,
slow Python model of batch formation, memory prediction and swap-out / reload, written
from the paper's description.  TEST INFRASTRUCTURE ONLY: nothing in the product path may
import it; it shares no code with the C++ scheduler.

What the paper fixes: unfinished decode requests come first, one token each; prefill
requests are cut at token granularity to fill the rest of a fixed dense batch exactly;
new requests are admitted only while the predicted peak memory (decoded tokens tracked per
request, completion estimated from the average decode length) stays within the pool; when
memory still runs out a request is moved to the host and brought back later without
recomputation; with asynchronous scheduling the end of a request is seen one iteration
late, so it decodes one token past its end.

Readings where the paper is silent (the C++ scheduler takes the same ones):
  * order: requests are served in arrival order; among prefill requests those already
    started come before new ones; the batch lists prefill entries, then decode entries;
  * the first generated token comes out of the iteration that processes the last prompt
    token; a request whose output length is n ends with its n-th generated token and has
    then cached prompt + n - 1 tokens;
  * prediction: every resident request is assumed to reach the running average output
    length (prior weighted like 16 finished requests), at least one more iteration; a
    request holds its whole prompt plus the decode iterations scheduled so far plus t
    tokens t iterations from now; the pool must cover the usage just before every
    predicted departure;
  * victim of a swap-out: the youngest decode request scheduled in this iteration that has
    not been given its page yet (possibly the request that needs the page); swapped
    requests return oldest first, once their pages plus one are free and the prediction
    allows; pages are handed out from a stack whose top is initially page 0, and freed
    pages go back on top in the order of the owner's page list;
  * progress: the prediction only guards admission beside other requests.  When no request
    is resident, the oldest swapped-out (else waiting) request is taken whatever the
    prediction says - it fits the pool alone (submission checks that) - so a long-prompt
    request under a large average output length cannot starve.
"""
import math


class Request:
    def __init__(self, rid, prompt, output):
        self.rid, self.prompt, self.output = rid, prompt, output
        self.prefilled = 0      # prompt tokens scheduled
        self.dec_sched = 0      # decode iterations scheduled
        self.generated = 0      # generated tokens the scheduler has been told about
        self.pages = []
        self.where = "waiting"  # waiting | resident | swapped | done

    @property
    def cached(self):
        return self.prefilled + self.dec_sched


class BatchFormation:
    def __init__(self, dense_batch, page_size, num_pages, max_requests, max_chunk=0, reserve_pages=0,
                 avg_decode_len=256.0):
        self.B, self.P, self.NP = dense_batch, page_size, num_pages
        self.max_requests, self.max_chunk, self.reserve = max_requests, max_chunk, reserve_pages
        self.prior_avg = float(avg_decode_len)
        self.free = list(range(num_pages - 1, -1, -1))  # stack, top = end of list = page 0
        self.requests = {}
        self.waiting, self.resident, self.swapped = [], [], []
        self.issued = {}          # iteration -> [(rid, q_len, kind, ends_prompt)]
        self.n_formed = self.n_completed = 0
        self.finished_outputs = []
        self.released_pending = []
        self.finished_pending = []
        self.wasted = 0

    # ---- helpers -------------------------------------------------------------------
    def pages_for(self, tokens):
        return -(-tokens // self.P)

    def average_output(self):
        return (self.prior_avg * 16.0 + sum(self.finished_outputs)) / (16.0 + len(self.finished_outputs))

    def predicted_peak_fits(self, extra=None):
        avg = max(1, math.ceil(self.average_output() - 1e-6))
        group = [self.requests[r] for r in self.resident] + ([extra] if extra is not None else [])
        future = [(max(1, avg - (1 + r.dec_sched)), r.prompt + r.dec_sched) for r in group]
        for leave_at, _ in future:
            usage = sum(self.pages_for(base + leave_at) for rem, base in future if rem >= leave_at)
            if usage > self.NP - self.reserve:
                return False
        return True

    def submit(self, prompt, output):
        rid = len(self.requests) + len(self.finished_outputs)
        if self.pages_for(prompt + output) > self.NP - self.reserve:
            raise ValueError("request can never fit")
        self.requests[rid] = Request(rid, prompt, output)
        self.waiting.append(rid)
        return rid

    # ---- one iteration ---------------------------------------------------------------
    def next_batch(self):
        swap_out, swap_in = [], []
        released, self.released_pending = self.released_pending, []
        finished, self.finished_pending = self.finished_pending, []

        # reload, oldest first
        while self.swapped and len(self.resident) < self.max_requests:
            r = self.requests[self.swapped[0]]
            need = self.pages_for(r.cached)
            if need + 1 > len(self.free) or (self.resident and not self.predicted_peak_fits(r)):
                break
            self.swapped.pop(0)
            r.pages = [self.free.pop() for _ in range(need)]
            r.where = "resident"
            self.resident.append(r.rid)
            swap_in.append((r.rid, list(r.pages)))

        # decode requests first
        decode = [rid for rid in self.resident if self.requests[rid].prefilled == self.requests[rid].prompt]
        decode = decode[:self.B]
        i = 0
        while i < len(decode):
            r = self.requests[decode[i]]
            keep = True
            if self.pages_for(r.cached + 1) > len(r.pages):
                while not self.free:
                    victim = self.requests[decode.pop()]
                    swap_out.append((victim.rid, list(victim.pages)))
                    self.free.extend(victim.pages)
                    victim.pages = []
                    victim.where = "swapped"
                    self.swapped.append(victim.rid)
                    self.resident.remove(victim.rid)
                    if victim is r:
                        keep = False
                        break
                if keep:
                    r.pages.append(self.free.pop())
            if keep:
                i += 1

        # prefill fills the rest
        room_in_batch = self.B - len(decode)
        prefill = []

        def limit(n):
            return min(n, self.max_chunk) if self.max_chunk > 0 else n
        for rid in self.resident:
            if room_in_batch == 0:
                break
            r = self.requests[rid]
            if r.prefilled == r.prompt:
                continue
            want = limit(min(r.prompt - r.prefilled, room_in_batch))
            room_in_pool = len(r.pages) * self.P - r.cached + len(self.free) * self.P
            chunk = min(want, room_in_pool)
            if chunk <= 0:
                continue
            while len(r.pages) < self.pages_for(r.cached + chunk):
                r.pages.append(self.free.pop())
            prefill.append((rid, chunk))
            room_in_batch -= chunk
        while room_in_batch > 0 and self.waiting and len(self.resident) < self.max_requests:
            r = self.requests[self.waiting[0]]
            if self.resident and not self.predicted_peak_fits(r):
                break
            chunk = min(limit(min(r.prompt, room_in_batch)), len(self.free) * self.P)
            if chunk <= 0:
                break
            self.waiting.pop(0)
            r.where = "resident"
            self.resident.append(r.rid)
            while len(r.pages) < self.pages_for(chunk):
                r.pages.append(self.free.pop())
            prefill.append((r.rid, chunk))
            room_in_batch -= chunk

        # the batch
        entries, issued = [], []
        for rid, chunk in prefill:
            r = self.requests[rid]
            entries.append({"rid": rid, "q_len": chunk, "ctx_len": r.cached, "pages": list(r.pages), "decode": False})
            r.prefilled += chunk
            issued.append((rid, chunk, "prefill", r.prefilled == r.prompt))
        for rid in decode:
            r = self.requests[rid]
            entries.append({"rid": rid, "q_len": 1, "ctx_len": r.cached, "pages": list(r.pages), "decode": True})
            r.dec_sched += 1
            issued.append((rid, 1, "decode", False))
        self.issued[self.n_formed] = issued
        batch = {"iteration": self.n_formed, "entries": entries, "n_prefill": len(prefill), "n_decode": len(decode),
                 "n_tokens": sum(e["q_len"] for e in entries), "swap_out": swap_out, "swap_in": swap_in,
                 "released": released, "finished": finished}
        self.n_formed += 1
        return batch

    def complete(self, iteration):
        if iteration != self.n_completed or iteration >= self.n_formed:
            raise ValueError("iterations complete in order")
        for rid, q_len, kind, ends_prompt in self.issued.pop(iteration):
            r = self.requests.get(rid)
            if r is None:
                self.wasted += q_len
                continue
            if kind == "decode":
                r.generated += 1
            elif ends_prompt:
                r.generated = 1
            if r.generated >= r.output:
                if r.where == "resident":
                    self.free.extend(r.pages)
                    self.resident.remove(rid)
                elif r.where == "swapped":
                    self.swapped.remove(rid)
                    self.released_pending.append(rid)
                r.where = "done"
                self.finished_pending.append(rid)
                self.finished_outputs.append(r.output)
                del self.requests[rid]
        self.n_completed += 1
