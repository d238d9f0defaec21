// Continuous batching (paper Sec. 4.2.1 "Request scheduling"): batch formation, memory
// prediction, swap-out / reload decisions and the page allocator.  Pure host code.
//
// Vocabulary.  cached(r) = prompt tokens scheduled for prefill + decode iterations scheduled:
// the tokens whose K/V are in the cache or will be appended by an issued iteration.  A
// resident request whose whole prompt has been scheduled is a decode candidate: every
// iteration appends its last generated token and produces the next one.  The iteration that
// processes the last prompt token produces generated token 1; a request ends with generated
// token output_len, which the scheduler only learns through nf_sched_complete.
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <deque>
#include <map>
#include <new>
#include <vector>

#include "../../include/nf.h"

namespace {

enum ReqState { WAITING = 0, RESIDENT = 1, SWAPPED = 2, DONE = 3 };

struct Req {
  int64_t id = 0;
  int32_t prompt = 0, output = 0;
  int32_t prefilled = 0;  // prompt tokens scheduled so far
  int32_t dec_sched = 0;  // decode iterations scheduled so far
  int32_t gen_known = 0;  // generated tokens confirmed by nf_sched_complete
  int state = WAITING;
  std::vector<int32_t> pages;
  int32_t cached() const { return prefilled + dec_sched; }
};

struct Entry {
  int64_t id;
  int32_t q_len;
  bool decode;
  bool ends_prompt;
};

}  // namespace

struct nf_sched {
  nf_sched_config cfg{};
  std::map<int64_t, Req> reqs;      // every request not yet forgotten
  std::deque<int64_t> waiting;      // submission order
  std::vector<int64_t> resident;    // admission order
  std::deque<int64_t> swapped;      // swap-out order
  std::vector<int32_t> free_pages;  // stack: back() is handed out next
  std::map<int64_t, std::vector<Entry>> inflight;
  int64_t next_id = 0, n_formed = 0, n_completed = 0;
  int64_t n_finished = 0, sum_finished_output = 0;
  nf_sched_stats st{};
  // output arrays of the last batch
  std::vector<int32_t> q_indptr, ctx_len, page_indptr, page_ids;
  std::vector<int64_t> request_ids;
  std::vector<int64_t> so_req, si_req, released, released_pending, finished, finished_pending;
  std::vector<int32_t> so_indptr, so_pages, si_indptr, si_pages;

  int32_t pages_for(int64_t tokens) const {
    return (int32_t)((tokens + cfg.page_size - 1) / cfg.page_size);
  }
  double avg_decode_len() const {
    return ((double)cfg.avg_decode_len * 16.0 + (double)sum_finished_output) / (16.0 + (double)n_finished);
  }
  int32_t take_page() {
    const int32_t p = free_pages.back();
    free_pages.pop_back();
    return p;
  }
  void give_pages(std::vector<int32_t>& pages) {
    for (int32_t p : pages) free_pages.push_back(p);
    pages.clear();
  }

  // Peak of the page pool if every resident request (and `extra`, if not null) runs to the
  // average output length: a request holds base + t tokens t iterations from now and leaves
  // after rem more iterations; the usage just before each departure is compared with the pool.
  bool prediction_fits(const Req* extra) const {
    const int32_t avg = (int32_t)std::max<int64_t>(1, (int64_t)ceil(avg_decode_len() - 1e-6));
    std::vector<std::pair<int32_t, int32_t>> v;  // (rem, base)
    v.reserve(resident.size() + 1);
    auto add = [&](const Req& r) {
      const int32_t base = r.prompt + r.dec_sched;
      const int32_t rem = std::max(1, avg - (1 + r.dec_sched));
      v.emplace_back(rem, base);
    };
    for (int64_t id : resident) add(reqs.at(id));
    if (extra) add(*extra);
    std::sort(v.begin(), v.end());
    const int64_t limit = cfg.num_pages - cfg.reserve_pages;
    for (size_t j = 0; j < v.size(); ++j) {
      if (j > 0 && v[j].first == v[j - 1].first) continue;  // same departure time: already checked
      const int32_t t = v[j].first;
      int64_t usage = 0;
      for (size_t i = j; i < v.size(); ++i) usage += pages_for((int64_t)v[i].second + t);
      if (usage > limit) return false;
    }
    return true;
  }
};

extern "C" int nf_sched_create(const nf_sched_config* cfg, nf_sched** out) try {
  if (!cfg || !out) return NF_EINVAL;
  *out = nullptr;
  if (cfg->dense_batch < 1 || cfg->page_size < 1 || cfg->num_pages < 1 || cfg->num_pages > INT32_MAX ||
      cfg->max_requests < 1 || cfg->max_chunk < 0 || cfg->reserve_pages < 0 || cfg->reserve_pages >= cfg->num_pages ||
      !(cfg->avg_decode_len >= 1.0f))
    return NF_EINVAL;
  nf_sched* s = new (std::nothrow) nf_sched();
  if (!s) return NF_ENOMEM;
  s->cfg = *cfg;
  s->free_pages.resize((size_t)cfg->num_pages);
  for (int64_t i = 0; i < cfg->num_pages; ++i) s->free_pages[(size_t)i] = (int32_t)(cfg->num_pages - 1 - i);
  *out = s;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" void nf_sched_destroy(nf_sched* s) { delete s; }

extern "C" int nf_sched_submit(nf_sched* s, int32_t prompt_len, int32_t output_len, int64_t* request_id) try {
  if (!s || prompt_len < 1 || output_len < 1) return NF_EINVAL;
  // a request alone in the pool must fit with every token it can ever cache
  if (s->pages_for((int64_t)prompt_len + output_len) > s->cfg.num_pages - s->cfg.reserve_pages) return NF_EPAGES;
  Req r;
  r.id = s->next_id++;
  r.prompt = prompt_len;
  r.output = output_len;
  s->reqs[r.id] = r;
  s->waiting.push_back(r.id);
  s->st.submitted++;
  if (request_id) *request_id = r.id;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_sched_next_batch(nf_sched* s, nf_sched_batch* out) try {
  if (!s || !out) return NF_EINVAL;
  const nf_sched_config& c = s->cfg;
  const int32_t P = c.page_size;
  s->so_req.clear();
  s->so_indptr.assign(1, 0);
  s->so_pages.clear();
  s->si_req.clear();
  s->si_indptr.assign(1, 0);
  s->si_pages.clear();
  s->released.swap(s->released_pending);
  s->released_pending.clear();
  s->finished.swap(s->finished_pending);
  s->finished_pending.clear();

  // 1. bring swapped-out requests back, oldest first, while pages and the prediction allow
  while (!s->swapped.empty() && (int)s->resident.size() < c.max_requests) {
    Req& r = s->reqs.at(s->swapped.front());
    const int32_t need = s->pages_for(r.cached());
    // with nothing resident the oldest request comes back whatever the prediction says: submit
    // proved that it fits alone, and refusing it would stall the loop for good
    if ((int64_t)need + 1 > (int64_t)s->free_pages.size() || (!s->resident.empty() && !s->prediction_fits(&r))) break;
    s->swapped.pop_front();
    for (int32_t i = 0; i < need; ++i) r.pages.push_back(s->take_page());
    r.state = RESIDENT;
    s->resident.push_back(r.id);
    s->si_req.push_back(r.id);
    s->si_pages.insert(s->si_pages.end(), r.pages.begin(), r.pages.end());
    s->si_indptr.push_back((int32_t)s->si_pages.size());
    s->st.swap_ins++;
  }

  // 2. decode requests first: one token each, in admission order; a request that needs a new
  // page when none is free swaps out the youngest scheduled decode request behind it (or itself)
  std::vector<int64_t> dec;
  for (int64_t id : s->resident) {
    const Req& r = s->reqs.at(id);
    if (r.prefilled == r.prompt && (int32_t)dec.size() < c.dense_batch) dec.push_back(id);
  }
  auto swap_out = [&](int64_t id) {
    Req& v = s->reqs.at(id);
    s->so_req.push_back(id);
    s->so_pages.insert(s->so_pages.end(), v.pages.begin(), v.pages.end());
    s->so_indptr.push_back((int32_t)s->so_pages.size());
    s->give_pages(v.pages);
    v.state = SWAPPED;
    s->swapped.push_back(id);
    s->resident.erase(std::find(s->resident.begin(), s->resident.end(), id));
    s->st.swap_outs++;
  };
  for (size_t i = 0; i < dec.size();) {
    Req& r = s->reqs.at(dec[i]);
    bool kept = true;
    if (s->pages_for((int64_t)r.cached() + 1) > (int32_t)r.pages.size()) {
      while (s->free_pages.empty()) {
        const int64_t victim = dec.back();
        dec.pop_back();
        swap_out(victim);
        if (victim == r.id) {
          kept = false;
          break;
        }
      }
      if (kept) r.pages.push_back(s->take_page());
    }
    if (kept) ++i;  // else dec[i] was the last element and is gone
  }

  // 3. prefill fills the rest of the dense batch: requests already in prefill, then new ones
  int32_t cap = c.dense_batch - (int32_t)dec.size();
  std::vector<std::pair<int64_t, int32_t>> pf;  // (request, chunk)
  auto chunk_limit = [&](int32_t want) { return c.max_chunk > 0 ? std::min(want, c.max_chunk) : want; };
  for (int64_t id : s->resident) {
    if (cap == 0) break;
    Req& r = s->reqs.at(id);
    if (r.prefilled == r.prompt) continue;
    const int32_t want = chunk_limit(std::min(r.prompt - r.prefilled, cap));
    const int64_t room = (int64_t)r.pages.size() * P - r.cached() + (int64_t)s->free_pages.size() * P;
    const int32_t chunk = (int32_t)std::min<int64_t>(want, room);
    if (chunk <= 0) continue;
    while ((int32_t)r.pages.size() < s->pages_for((int64_t)r.cached() + chunk)) r.pages.push_back(s->take_page());
    pf.emplace_back(id, chunk);
    cap -= chunk;
  }
  while (cap > 0 && !s->waiting.empty() && (int)s->resident.size() < c.max_requests) {
    Req& r = s->reqs.at(s->waiting.front());
    if (!s->resident.empty() && !s->prediction_fits(&r)) break;  // alone, a request is always admitted
    const int32_t want = chunk_limit(std::min(r.prompt, cap));
    const int32_t chunk = (int32_t)std::min<int64_t>(want, (int64_t)s->free_pages.size() * P);
    if (chunk <= 0) break;
    s->waiting.pop_front();
    r.state = RESIDENT;
    s->resident.push_back(r.id);
    while ((int32_t)r.pages.size() < s->pages_for(chunk)) r.pages.push_back(s->take_page());
    pf.emplace_back(r.id, chunk);
    cap -= chunk;
  }

  // 4. the batch arrays: prefill entries, then decode entries
  s->q_indptr.assign(1, 0);
  s->ctx_len.clear();
  s->page_indptr.assign(1, 0);
  s->page_ids.clear();
  s->request_ids.clear();
  std::vector<Entry>& fl = s->inflight[s->n_formed];
  auto emit = [&](Req& r, int32_t q_len, bool decode) {
    s->q_indptr.push_back(s->q_indptr.back() + q_len);
    s->ctx_len.push_back(r.cached());
    s->page_ids.insert(s->page_ids.end(), r.pages.begin(), r.pages.end());
    s->page_indptr.push_back((int32_t)s->page_ids.size());
    s->request_ids.push_back(r.id);
    if (decode) {
      r.dec_sched += 1;
      s->st.decode_tokens += 1;
    } else {
      r.prefilled += q_len;
      s->st.prefill_tokens += q_len;
    }
    fl.push_back(Entry{r.id, q_len, decode, !decode && r.prefilled == r.prompt});
  };
  for (auto& e : pf) emit(s->reqs.at(e.first), e.second, false);
  for (int64_t id : dec) emit(s->reqs.at(id), 1, true);

  out->iteration = s->n_formed++;
  out->n_tokens = s->q_indptr.back();
  out->n_prefill_reqs = (int32_t)pf.size();
  out->n_decode_reqs = (int32_t)dec.size();
  out->q_indptr = s->q_indptr.data();
  out->ctx_len = s->ctx_len.data();
  out->page_indptr = s->page_indptr.data();
  out->page_ids = s->page_ids.data();
  out->request_ids = s->request_ids.data();
  out->n_swap_out = (int32_t)s->so_req.size();
  out->swap_out_req = s->so_req.data();
  out->swap_out_indptr = s->so_indptr.data();
  out->swap_out_pages = s->so_pages.data();
  out->n_swap_in = (int32_t)s->si_req.size();
  out->swap_in_req = s->si_req.data();
  out->swap_in_indptr = s->si_indptr.data();
  out->swap_in_pages = s->si_pages.data();
  out->n_released = (int32_t)s->released.size();
  out->released_req = s->released.data();
  out->n_finished = (int32_t)s->finished.size();
  out->finished_req = s->finished.data();
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_sched_complete(nf_sched* s, int64_t iteration) try {
  if (!s || iteration != s->n_completed || iteration >= s->n_formed) return NF_EINVAL;
  auto it = s->inflight.find(iteration);
  if (it == s->inflight.end()) return NF_EINVAL;
  for (const Entry& e : it->second) {
    auto rit = s->reqs.find(e.id);
    if (rit == s->reqs.end()) {  // retired earlier: this was a token past the end
      s->st.wasted_decode_tokens += e.q_len;
      continue;
    }
    Req& r = rit->second;
    if (e.decode)
      r.gen_known += 1;
    else if (e.ends_prompt)
      r.gen_known = 1;
    if (r.gen_known >= r.output) {
      if (r.state == RESIDENT) {
        s->give_pages(r.pages);
        s->resident.erase(std::find(s->resident.begin(), s->resident.end(), r.id));
      } else if (r.state == SWAPPED) {
        s->swapped.erase(std::find(s->swapped.begin(), s->swapped.end(), r.id));
        s->released_pending.push_back(r.id);
      }
      s->finished_pending.push_back(r.id);
      s->n_finished++;
      s->sum_finished_output += r.output;
      s->st.finished++;
      s->reqs.erase(rit);
    }
  }
  s->inflight.erase(it);
  s->n_completed++;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_sched_get_stats(const nf_sched* s, nf_sched_stats* out) try {
  if (!s || !out) return NF_EINVAL;
  *out = s->st;
  out->iterations_formed = s->n_formed;
  out->iterations_completed = s->n_completed;
  out->waiting = (int64_t)s->waiting.size();
  out->resident = (int64_t)s->resident.size();
  out->swapped = (int64_t)s->swapped.size();
  out->free_pages = (int64_t)s->free_pages.size();
  out->avg_decode_len = s->avg_decode_len();
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}
