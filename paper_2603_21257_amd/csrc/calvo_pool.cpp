// Slot bookkeeping for the paged KV space in HBM (the paper's L1 tier) with the paper's proactive
// allocation (Section 3.1): the destination blocks of a request are reserved at the moment its
// lower-level transfer is issued, so a block that reaches host DRAM can move on at once; when HBM is
// short the scheme falls back to reactive allocation (footnote of Section 3.1) - the request
// waits in a queue and gets its slots when earlier requests release theirs.  Host code only; the
// library's loading and attention calls take the resulting block tables.  See include/calvo.h.
#include <cstdint>
#include <deque>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/calvo.h"

struct calvo_pool {
  std::mutex mu;
  std::vector<int32_t> refs;        // references per slot; 0 = free
  std::vector<char> mark;           // scratch for duplicate checks, all zero between calls
  std::vector<int32_t> free_stack;  // free slot ids; the back is handed out next
  int64_t n_refs = 0;               // sum of refs
  struct Waiter {
    int64_t ticket;
    std::vector<int32_t> shared;
    int32_t n_own;
  };
  std::deque<Waiter> waiters;       // admissions that found HBM short, oldest first
  int64_t next_ticket = 1;
};

namespace {

bool valid_slots(const calvo_pool* p, const int32_t* slots, int32_t n, bool must_be_used) {
  for (int32_t i = 0; i < n; i++) {
    if (slots[i] < 0 || (size_t)slots[i] >= p->refs.size()) return false;
    if (must_be_used && p->refs[(size_t)slots[i]] <= 0) return false;
  }
  return true;
}

// shared slots gain a reference, n_own free slots are taken: table = shared ++ own.  The caller
// has checked that n_own <= free and that the shared slots are in use.
void grant(calvo_pool* p, const int32_t* shared, int32_t n_shared, int32_t n_own, int32_t* table) {
  for (int32_t i = 0; i < n_shared; i++) {
    p->refs[(size_t)shared[i]]++;
    table[i] = shared[i];
  }
  for (int32_t i = 0; i < n_own; i++) {
    const int32_t s = p->free_stack.back();
    p->free_stack.pop_back();
    p->refs[(size_t)s] = 1;
    table[n_shared + i] = s;
  }
  p->n_refs += (int64_t)n_shared + n_own;
}

}  // namespace

extern "C" {

int calvo_pool_create(int64_t n_blocks, calvo_pool** out) {
  if (!out) return CALVO_EINVAL;
  *out = nullptr;
  if (n_blocks <= 0 || n_blocks > INT32_MAX) return CALVO_EINVAL;
  calvo_pool* p = new (std::nothrow) calvo_pool();
  if (!p) return CALVO_ENOMEM;
  p->refs.assign((size_t)n_blocks, 0);
  p->mark.assign((size_t)n_blocks, 0);
  p->free_stack.resize((size_t)n_blocks);
  for (int64_t i = 0; i < n_blocks; i++) p->free_stack[(size_t)i] = (int32_t)(n_blocks - 1 - i);   // slot 0 first
  *out = p;
  return CALVO_OK;
}

int calvo_pool_destroy(calvo_pool* p) {
  if (!p) return CALVO_EINVAL;
  delete p;
  return CALVO_OK;
}

int calvo_pool_reserve(calvo_pool* p, int32_t n, int32_t* slots) {
  if (!p || n < 0 || (n > 0 && !slots)) return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  if ((size_t)n > p->free_stack.size()) return CALVO_ENOMEM;
  grant(p, nullptr, 0, n, slots);
  return CALVO_OK;
}

int calvo_pool_retain(calvo_pool* p, const int32_t* slots, int32_t n) {
  if (!p || n < 0 || (n > 0 && !slots)) return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  if (!valid_slots(p, slots, n, true)) return CALVO_EINVAL;
  for (int32_t i = 0; i < n; i++) p->refs[(size_t)slots[i]]++;
  p->n_refs += n;
  return CALVO_OK;
}

int calvo_pool_release(calvo_pool* p, const int32_t* slots, int32_t n) {
  if (!p || n < 0 || (n > 0 && !slots)) return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  // all or nothing: an entry without a reference left (counting repeats inside the list) undoes the call
  std::vector<int32_t> freed;
  for (int32_t i = 0; i < n; i++) {
    const bool ok = slots[i] >= 0 && (size_t)slots[i] < p->refs.size() && p->refs[(size_t)slots[i]] > 0;
    if (!ok) {
      for (int32_t k = 0; k < i; k++) p->refs[(size_t)slots[k]]++;
      return CALVO_EINVAL;
    }
    if (--p->refs[(size_t)slots[i]] == 0) freed.push_back(slots[i]);
  }
  p->free_stack.insert(p->free_stack.end(), freed.begin(), freed.end());
  p->n_refs -= n;
  return CALVO_OK;
}

int calvo_pool_counts(calvo_pool* p, int64_t* n_free, int64_t* n_used, int64_t* n_refs, int64_t* n_waiting) {
  if (!p) return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  if (n_free) *n_free = (int64_t)p->free_stack.size();
  if (n_used) *n_used = (int64_t)p->refs.size() - (int64_t)p->free_stack.size();
  if (n_refs) *n_refs = p->n_refs;
  if (n_waiting) *n_waiting = (int64_t)p->waiters.size();
  return CALVO_OK;
}

int calvo_pool_admit(calvo_pool* p, const int32_t* shared, int32_t n_shared, int32_t n_own, int32_t* table,
                     int64_t* ticket) {
  if (!p || n_shared < 0 || n_own < 0 || (n_shared > 0 && !shared) || (n_shared + n_own > 0 && !table) || !ticket)
    return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  *ticket = 0;
  if ((size_t)n_own > p->refs.size()) return CALVO_ENOMEM;         // can never be satisfied
  if (!valid_slots(p, shared, n_shared, true)) return CALVO_EINVAL;
  bool dup = false;
  for (int32_t i = 0; i < n_shared; i++) {
    dup |= p->mark[(size_t)shared[i]] != 0;
    p->mark[(size_t)shared[i]] = 1;
  }
  for (int32_t i = 0; i < n_shared; i++) p->mark[(size_t)shared[i]] = 0;
  if (dup) return CALVO_EINVAL;
  // proactive: take the slots now - unless older admissions are still waiting (no overtaking) or
  // HBM is short; then the request queues up and is allocated reactively
  if (p->waiters.empty() && (size_t)n_own <= p->free_stack.size()) {
    grant(p, shared, n_shared, n_own, table);
    return CALVO_OK;
  }
  // the shared run must not disappear while the request waits: it is referenced from now on
  for (int32_t i = 0; i < n_shared; i++) p->refs[(size_t)shared[i]]++;
  p->n_refs += n_shared;
  calvo_pool::Waiter w{p->next_ticket++, std::vector<int32_t>(shared, shared + n_shared), n_own};
  *ticket = w.ticket;
  p->waiters.push_back(std::move(w));
  return CALVO_ENOTREADY;
}

int calvo_pool_retry(calvo_pool* p, int64_t ticket, int32_t* table) {
  if (!p || ticket <= 0) return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  size_t pos = 0;
  while (pos < p->waiters.size() && p->waiters[pos].ticket != ticket) pos++;
  if (pos == p->waiters.size()) return CALVO_EINVAL;
  if (pos != 0) return CALVO_ENOTREADY;                            // strictly in arrival order
  calvo_pool::Waiter& w = p->waiters.front();
  if ((size_t)w.n_own > p->free_stack.size()) return CALVO_ENOTREADY;
  const int32_t ns = (int32_t)w.shared.size();
  if (ns + w.n_own > 0 && !table) return CALVO_EINVAL;
  // the shared references were taken at admission
  for (int32_t i = 0; i < ns; i++) table[i] = w.shared[(size_t)i];
  grant(p, nullptr, 0, w.n_own, table + ns);
  p->waiters.pop_front();
  return CALVO_OK;
}

int calvo_pool_cancel(calvo_pool* p, int64_t ticket) {
  if (!p || ticket <= 0) return CALVO_EINVAL;
  std::lock_guard<std::mutex> lk(p->mu);
  for (size_t pos = 0; pos < p->waiters.size(); pos++)
    if (p->waiters[pos].ticket == ticket) {
      // give back the references on the shared run; a slot nobody else holds any more becomes free
      for (int32_t s : p->waiters[pos].shared)
        if (--p->refs[(size_t)s] == 0) p->free_stack.push_back(s);
      p->n_refs -= (int64_t)p->waiters[pos].shared.size();
      p->waiters.erase(p->waiters.begin() + (long)pos);
      return CALVO_OK;
    }
  return CALVO_EINVAL;
}

}  // extern "C"
