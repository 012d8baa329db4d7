// The multi-request dispatcher of libcalvo (paper Section 3.1 and 3.2): every loading stage and the
// compute stage have a dispatcher-executor pair of their own - a thread that, whenever its resource
// is free, takes the highest-priority request whose input from the stage below is ready and whose
// destination is allocated, moves it, and signals the stage above - so that the (emulated) network
// link, PCIe and the GPU are busy with different requests at the same time.  The destination slots
// in HBM are requested when the lowest stage issues a request's transfer (proactive allocation); if
// HBM is short the request's blocks wait in the stage below until slots come back (reactive).
// See include/calvo.h for the contract.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstring>
#include <deque>
#include <limits>
#include <memory>
#include <new>

#include "calvo_ctx.h"

using namespace calvo;
using namespace calvo::host;

namespace {

using clk = std::chrono::steady_clock;

struct Job {
  int64_t id = 0;
  calvo_dispatch_job spec{};
  calvo_job sched{};                    // what the queue policies look at (absolute times)
  std::vector<int32_t> shared;          // the run it shares (slots already in use)
  std::vector<int32_t> table;           // shared run + own slots, valid once granted
  int n_tab = 0;                        // table entries: prefix blocks + suffix blocks
  bool granted = false;
  int64_t ticket = -1;
  bool load_picked = false, compute_picked = false, finished = false, released = false;
  bool table_uploaded = false;
  int layers_handed = 0;                // layers whose last block has been queued for HBM (their event is recorded)
  std::vector<hipEvent_t> ev_layer;
  hipEvent_t ev_done = nullptr;
  calvo_batch* batch = nullptr;
  calvo_dispatch_result res{};
  std::string err;                      // what the failing call said (the stage threads have their own last-error text)
};

struct Chunk {
  Job* job;
  int layer;
  int64_t j0, nb;          // blocks [j0, j0 + nb) of the job; nb == 0: the job has nothing to load
  int slot;                // pinned ring slot that holds them
  bool last_of_layer;
};

}  // namespace

struct calvo_dispatcher {
  calvo_ctx* c = nullptr;               // NULL: dry run (stages sleep for the jobs' sim_load_s / sim_comp_s)
  calvo_dispatch_config cfg{};
  clk::time_point t0;
  std::mutex mu;
  std::condition_variable cv;
  bool stop = false;
  bool cancel_waiting = false;          // destroy: jobs that still wait for slots nobody will give back are failed
  std::vector<std::unique_ptr<Job>> jobs;
  std::deque<Chunk> pcie_q;             // blocks that have landed in the pinned ring, in link order
  std::deque<Job*> done_q;              // jobs whose compute has been queued, in that order
  // pinned ring slots: 0 free, 1 filled by the link stage and not yet taken by the PCIe stage,
  // 2 taken (its copy's completion event is recorded)
  std::vector<int> slot_state;
  calvo_dispatch_stats stats{};
  double link_first = -1.0, link_last = 0.0;
  std::thread t_link, t_pcie, t_comp, t_done;
  int n_slots = 0, n_threads = 0;
  int64_t chunk_blocks = 0;
  double rate = 0.0;

  double now() const { return std::chrono::duration<double>(clk::now() - t0).count(); }
};

namespace {

// index of the job the policy serves next among those with eligible[i], or -1
int pick_job(calvo_dispatcher* d, const std::vector<char>& eligible) {
  const int n = (int)d->jobs.size();
  std::vector<calvo_job> js((size_t)n);
  std::vector<unsigned char> skip((size_t)n);
  bool any = false;
  for (int i = 0; i < n; i++) {
    js[i] = d->jobs[i]->sched;
    skip[i] = eligible[i] ? 0 : 1;
    any |= eligible[i] != 0;
  }
  if (!any) return -1;
  int idx = -1;
  const double inf = std::numeric_limits<double>::infinity();
  if (calvo_sched_pick(d->cfg.policy, &d->cfg.model, js.data(), skip.data(), n, inf, &idx) != CALVO_OK) return -1;
  return idx;
}

void fail_job(calvo_dispatcher* d, Job* j, int status) {      // d->mu held; called on the thread whose call failed
  if (j->res.status == CALVO_OK) {
    j->res.status = status;
    j->err = calvo_last_error();
  }
  if (!j->finished) {
    j->finished = true;
    j->res.first_token_s = d->now();
  }
  j->layers_handed = d->c ? d->c->cfg.n_layers : 1;
}

// Proactive allocation: called when the lowest stage issues the job's transfer.  d->mu held.
void admit(calvo_dispatcher* d, Job* j) {
  if (!d->cfg.pool) {
    j->granted = true;
    return;
  }
  j->table.assign((size_t)j->n_tab, 0);
  const int n_sh = (int)j->shared.size();
  const int rc = calvo_pool_admit(d->cfg.pool, n_sh ? j->shared.data() : nullptr, n_sh, j->n_tab - n_sh, j->table.data(),
                                  &j->ticket);
  if (rc == CALVO_OK) j->granted = true;
  else if (rc == CALVO_ENOTREADY) j->res.reactive = 1;
  else fail_job(d, j, rc);
}

// Reactive path: the job's blocks wait below until its slots are granted.  Returns false on stop / failure.
bool wait_granted(calvo_dispatcher* d, Job* j, std::unique_lock<std::mutex>& lk) {
  const double t_begin = d->now();
  while (!j->granted && !d->stop && j->res.status == CALVO_OK) {
    const int rc = calvo_pool_retry(d->cfg.pool, j->ticket, j->table.data());
    if (rc == CALVO_OK) { j->granted = true; break; }
    if (rc != CALVO_ENOTREADY) { fail_job(d, j, rc); break; }
    if (d->cancel_waiting) {
      (void)calvo_pool_cancel(d->cfg.pool, j->ticket);
      j->ticket = -1;
      (void)fail(CALVO_ENOMEM, "the dispatcher was destroyed while the job waited for slots that are held outside it");
      fail_job(d, j, CALVO_ENOMEM);
      break;
    }
    d->cv.wait_for(lk, std::chrono::milliseconds(2));       // woken by calvo_dispatch_release
  }
  if (j->res.reactive) j->res.alloc_wait_s += d->now() - t_begin;
  return j->granted && !d->stop;
}

int request_of(const Job* j, calvo_request* r) {
  r->host_kv = j->spec.host_kv;
  r->host_layer_stride = j->spec.host_layer_stride;
  r->block_table = j->table.data();
  r->n_prefix_blocks = j->spec.n_prefix_blocks;
  r->first_ingest_block = (int32_t)j->shared.size();
  r->suffix_len = j->spec.suffix_len;
  return CALVO_OK;
}

// ---- stage L3 -> L2: the emulated link (three-stage mode only)
void link_main(calvo_dispatcher* d) {
  calvo_ctx* c = d->c;
  (void)hipSetDevice(c->device);
  clk::time_point link_free_at{};          // the link has never been used: long free
  uint64_t k = 0;
  std::unique_lock<std::mutex> lk(d->mu);
  for (;;) {
    std::vector<char> el(d->jobs.size());
    for (size_t i = 0; i < d->jobs.size(); i++) el[i] = !d->jobs[i]->load_picked && d->jobs[i]->res.status == CALVO_OK;
    const int idx = d->stop ? -1 : pick_job(d, el);
    if (idx < 0) {
      if (d->stop) return;
      d->cv.wait(lk);
      continue;
    }
    Job* j = d->jobs[(size_t)idx].get();
    j->load_picked = true;
    j->res.load_start_s = d->now();
    admit(d, j);                              // the destination one level up is requested as the transfer is issued
    d->cv.notify_all();
    const int64_t first = (int64_t)j->shared.size(), nblk = j->spec.n_prefix_blocks;
    if (j->res.status != CALVO_OK) continue;
    if (first >= nblk) {
      d->pcie_q.push_back({j, 0, 0, 0, -1, true});
      d->cv.notify_all();
      continue;
    }
    const int L = c->cfg.n_layers;
    // (a job that has failed meanwhile - its admission was refused or withdrawn - is not streamed any further)
    for (int l = 0; l < L && !d->stop && j->res.status == CALVO_OK; l++) {
      for (int64_t j0 = first; j0 < nblk && !d->stop && j->res.status == CALVO_OK; j0 += d->chunk_blocks) {
        const int64_t nb = std::min<int64_t>(d->chunk_blocks, nblk - j0);
        const size_t bytes = (size_t)nb * c->blk_bytes;
        const int slot = (int)(k % (uint64_t)d->n_slots);
        k++;
        const double w0 = d->now();
        d->cv.wait(lk, [&] { return d->slot_state[slot] != 1 || d->stop; });     // the PCIe stage has taken its previous contents
        if (d->stop) return;
        const bool copying = d->slot_state[slot] == 2;
        lk.unlock();
        if (copying) (void)hipEventSynchronize(c->ev_l2_free[slot]);              // ... and copied them to the device
        const auto t1 = clk::now();
        const double waited = std::chrono::duration<double>(t1 - d->t0).count() - w0;
        // the link streams on its own: the short hand-over between two chunks does not hold it up; after
        // a real gap (no request queued, or back-pressure from the stages above) it starts afresh
        const auto start = (t1 - link_free_at > std::chrono::microseconds(200)) ? t1 : link_free_at;
        parallel_copy((unsigned char*)c->l2_ring[slot],
                      (const unsigned char*)j->spec.host_kv + (int64_t)l * j->spec.host_layer_stride + j0 * (int64_t)c->blk_bytes,
                      bytes, d->n_threads);
        if (d->rate > 0.0) {
          link_free_at = start + std::chrono::duration_cast<clk::duration>(std::chrono::duration<double>((double)bytes / d->rate));
          std::this_thread::sleep_until(link_free_at);
        }
        const double busy = std::chrono::duration<double>(clk::now() - t1).count();
        lk.lock();
        d->stats.ring_wait_s += waited;
        d->stats.link_busy_s += busy;
        d->stats.bytes += (int64_t)bytes;
        if (d->link_first < 0) d->link_first = std::chrono::duration<double>(t1 - d->t0).count();
        d->link_last = d->now();
        d->slot_state[slot] = 1;
        d->pcie_q.push_back({j, l, j0, nb, slot, j0 + nb >= nblk});
        d->cv.notify_all();
      }
    }
  }
}

// Every layer of the job counts as handed over (nothing to load, or a failure).  d->mu held.
hipError_t hand_over_all(calvo_dispatcher* d, Job* j) {
  hipError_t e = hipSuccess;
  if (d->c)
    for (size_t l = (size_t)j->layers_handed; l < j->ev_layer.size() && e == hipSuccess; l++) e = hipEventRecord(j->ev_layer[l], d->c->s_scatter);
  j->layers_handed = d->c ? d->c->cfg.n_layers : 1;
  j->res.load_end_s = d->now();
  return e;
}

// ---- stage L2 -> L1: PCIe.  Three-stage mode: takes the blocks the link has delivered, in link order.
// Two-stage mode (the jobs' KV sits in pinned host memory): picks the next job itself when the
// previous job's blocks are all in HBM.
void pcie_main(calvo_dispatcher* d) {
  calvo_ctx* c = d->c;
  if (c) (void)hipSetDevice(c->device);
  Job* prev = nullptr;
  std::unique_lock<std::mutex> lk(d->mu);
  for (;;) {
    if (d->cfg.three_stage && c) {
      d->cv.wait(lk, [&] { return !d->pcie_q.empty() || d->stop; });
      if (d->pcie_q.empty()) return;
      const Chunk ch = d->pcie_q.front();
      d->pcie_q.pop_front();
      Job* j = ch.job;
      // a block moves up only if (1) it has arrived below - it is in the ring - and (2) its destination is allocated
      if (!wait_granted(d, j, lk)) {
        if (ch.slot >= 0) d->slot_state[ch.slot] = 0;
        if (d->stop) return;
        (void)hand_over_all(d, j);
        d->cv.notify_all();
        continue;
      }
      hipError_t e = hipSuccess;
      if (ch.nb == 0) {
        e = hand_over_all(d, j);
      } else {
        lk.unlock();
        int rc = CALVO_OK;
        if (!j->table_uploaded) {
          rc = upload_ingest_table(c, j->table.data() + j->shared.size(), (size_t)(j->spec.n_prefix_blocks - (int64_t)j->shared.size()));
          j->table_uploaded = true;
        }
        unsigned char* pool_layer = (unsigned char*)c->cfg.pool + (int64_t)ch.layer * c->layer_bytes;
        if (rc == CALVO_OK)
          e = enqueue_staged(c, (const unsigned char*)c->l2_ring[ch.slot], pool_layer, c->d_tab_ing + (ch.j0 - (int64_t)j->shared.size()),
                             ch.nb, c->ev_l2_free[ch.slot]);
        if (rc == CALVO_OK && e == hipSuccess && ch.last_of_layer) e = hipEventRecord(j->ev_layer[(size_t)ch.layer], c->s_scatter);
        lk.lock();
        d->slot_state[ch.slot] = (rc == CALVO_OK && e == hipSuccess) ? 2 : 0;
        if (rc != CALVO_OK) fail_job(d, j, rc);
        else if (e == hipSuccess && ch.last_of_layer) {
          j->layers_handed = ch.layer + 1;
          if (ch.layer + 1 == c->cfg.n_layers) j->res.load_end_s = d->now();
        }
      }
      if (e != hipSuccess) { (void)hipGetLastError(); fail_job(d, j, CALVO_EHIP); }
      d->cv.notify_all();
      continue;
    }
    // ---- two stages (and the dry run): this thread is the loading stage
    if (prev && c) {                     // the loading stage is free when the previous job's last block has landed
      lk.unlock();
      (void)hipEventSynchronize(prev->ev_layer.back());
      lk.lock();
      prev->res.load_end_s = d->now();
      prev = nullptr;
      d->cv.notify_all();
    }
    std::vector<char> el(d->jobs.size());
    for (size_t i = 0; i < d->jobs.size(); i++) el[i] = !d->jobs[i]->load_picked && d->jobs[i]->res.status == CALVO_OK;
    const int idx = d->stop ? -1 : pick_job(d, el);
    if (idx < 0) {
      if (d->stop) return;
      d->cv.wait(lk);
      continue;
    }
    Job* j = d->jobs[(size_t)idx].get();
    j->load_picked = true;
    j->res.load_start_s = d->now();
    admit(d, j);
    if (j->res.status == CALVO_OK && !wait_granted(d, j, lk)) {
      if (d->stop) return;
    }
    if (j->res.status != CALVO_OK) { (void)hand_over_all(d, j); d->cv.notify_all(); continue; }
    if (!c) {                            // dry run: the loading stage is busy for the job's loading time
      lk.unlock();
      std::this_thread::sleep_for(std::chrono::duration<double>(j->spec.sim_load_s));
      lk.lock();
      (void)hand_over_all(d, j);
      d->cv.notify_all();
      continue;
    }
    const int64_t first = (int64_t)j->shared.size(), nblk = j->spec.n_prefix_blocks;
    lk.unlock();
    int rc = CALVO_OK;
    hipError_t e = hipSuccess;
    if (nblk > first) rc = upload_ingest_table(c, j->table.data() + first, (size_t)(nblk - first));
    for (int l = 0; l < c->cfg.n_layers && rc == CALVO_OK && e == hipSuccess; l++) {
      unsigned char* pool_layer = (unsigned char*)c->cfg.pool + (int64_t)l * c->layer_bytes;
      const unsigned char* src = (const unsigned char*)j->spec.host_kv + (int64_t)l * j->spec.host_layer_stride;
      for (int64_t j0 = first; j0 < nblk && e == hipSuccess; j0 += c->staging_blocks) {
        const int64_t nb = std::min<int64_t>(c->staging_blocks, nblk - j0);
        e = enqueue_staged(c, src + j0 * (int64_t)c->blk_bytes, pool_layer, c->d_tab_ing + (j0 - first), nb, nullptr);
      }
      if (e == hipSuccess) e = hipEventRecord(j->ev_layer[(size_t)l], c->s_scatter);
      if (e == hipSuccess) {
        std::lock_guard<std::mutex> g(d->mu);
        j->layers_handed = l + 1;
        d->cv.notify_all();
      }
    }
    lk.lock();
    if (rc != CALVO_OK) fail_job(d, j, rc);
    if (e != hipSuccess) { (void)hipGetLastError(); fail_job(d, j, CALVO_EHIP); }
    prev = (j->res.status == CALVO_OK) ? j : nullptr;
    d->cv.notify_all();
  }
}

// ---- compute stage: the highest-priority job whose first layer has been handed over; its layers are
// queued behind their events as the loading stages hand them over
void comp_main(calvo_dispatcher* d) {
  calvo_ctx* c = d->c;
  if (c) (void)hipSetDevice(c->device);
  std::unique_lock<std::mutex> lk(d->mu);
  for (;;) {
    std::vector<char> el(d->jobs.size());
    for (size_t i = 0; i < d->jobs.size(); i++) {
      const Job* j = d->jobs[i].get();
      el[i] = j->load_picked && !j->compute_picked && j->granted && j->layers_handed >= 1 && j->res.status == CALVO_OK;
    }
    const int idx = d->stop ? -1 : pick_job(d, el);
    if (idx < 0) {
      if (d->stop) return;
      d->cv.wait(lk);
      continue;
    }
    Job* j = d->jobs[(size_t)idx].get();
    j->compute_picked = true;
    j->res.compute_start_s = d->now();
    if (!c) {                            // dry run
      lk.unlock();
      std::this_thread::sleep_for(std::chrono::duration<double>(j->spec.sim_comp_s));
      lk.lock();
      j->res.first_token_s = d->now();
      j->finished = true;
      d->stats.jobs_done++;
      d->cv.notify_all();
      continue;
    }
    lk.unlock();
    calvo_request r{};
    request_of(j, &r);
    const int32_t cu[2] = {0, j->spec.suffix_len};
    int rc = calvo_batch_prepare(c, &r, 1, cu, &j->batch);
    const int L = c->cfg.n_layers;
    const int64_t S = j->spec.suffix_len;
    const int64_t q_stride = j->spec.q_layer_stride ? j->spec.q_layer_stride : S * c->cfg.n_q_heads * c->cfg.head_dim * (int64_t)c->elt;
    const int64_t out_stride = j->spec.out_layer_stride ? j->spec.out_layer_stride : S * c->cfg.n_q_heads * c->cfg.head_dim * (int64_t)c->elt;
    const int64_t kv_stride = j->spec.kv_layer_stride ? j->spec.kv_layer_stride : S * c->cfg.n_kv_heads * c->cfg.head_dim * (int64_t)c->elt;
    for (int l = 0; l < L && rc == CALVO_OK; l++) {
      {
        std::unique_lock<std::mutex> g(d->mu);
        d->cv.wait(g, [&] { return j->layers_handed > l || d->stop || j->res.status != CALVO_OK; });
        if (d->stop || j->res.status != CALVO_OK) break;
      }
      const unsigned char* q = (const unsigned char*)j->spec.q + l * q_stride;
      const unsigned char* ks = j->spec.k_suffix ? (const unsigned char*)j->spec.k_suffix + l * kv_stride : nullptr;
      const unsigned char* vs = j->spec.v_suffix ? (const unsigned char*)j->spec.v_suffix + l * kv_stride : nullptr;
      unsigned char* out = (unsigned char*)j->spec.out + l * out_stride;
      rc = prefill_attn_prepared(j->batch, l, S ? q : nullptr, S ? ks : nullptr, S ? vs : nullptr, S ? out : nullptr, j->spec.scale,
                                 j->ev_layer[(size_t)l]);
    }
    hipError_t e = hipSuccess;
    if (rc == CALVO_OK) e = hipEventRecord(j->ev_done, c->s_compute);
    lk.lock();
    if (d->stop) return;
    if (rc != CALVO_OK) fail_job(d, j, rc);
    else if (e != hipSuccess) { (void)hipGetLastError(); fail_job(d, j, CALVO_EHIP); }
    else if (j->res.status == CALVO_OK) d->done_q.push_back(j);     // a job that failed while it loaded is finished already
    d->cv.notify_all();
  }
}

// ---- first-token signal: waits for each job's last launch in the order they were queued
void done_main(calvo_dispatcher* d) {
  (void)hipSetDevice(d->c->device);
  std::unique_lock<std::mutex> lk(d->mu);
  for (;;) {
    d->cv.wait(lk, [&] { return !d->done_q.empty() || d->stop; });
    if (d->done_q.empty()) return;
    Job* j = d->done_q.front();
    d->done_q.pop_front();
    lk.unlock();
    const hipError_t e = hipEventSynchronize(j->ev_done);
    lk.lock();
    j->res.first_token_s = d->now();
    if (e != hipSuccess) { (void)hipGetLastError(); j->res.status = CALVO_EHIP; }
    j->finished = true;
    d->stats.jobs_done++;
    d->cv.notify_all();
  }
}

// [p, p + extent) must lie inside one device allocation: a wrong layer stride is refused here
// instead of faulting in a kernel (an allocator that carves tensors out of larger segments can
// still hide an overrun into a neighbouring tensor).
int check_device_extent(const void* p, int64_t extent, const char* what) {
  if (!p || extent <= 0) return CALVO_OK;
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)p) != hipSuccess) {
    (void)hipGetLastError();
    return fail(CALVO_EINVAL, "%s is not device memory", what);
  }
  const int64_t off = (const unsigned char*)p - (const unsigned char*)base;
  if (off < 0 || off + extent > (int64_t)size)
    return fail(CALVO_EINVAL, "%s: %lld bytes from the pointer over all layers, but its allocation ends after %lld", what,
                (long long)extent, (long long)((int64_t)size - off));
  return CALVO_OK;
}

Job* find_job(calvo_dispatcher* d, int64_t id) {
  return (id >= 0 && id < (int64_t)d->jobs.size()) ? d->jobs[(size_t)id].get() : nullptr;
}

}  // namespace

extern "C" {

int calvo_dispatch_create(calvo_ctx* c, const calvo_dispatch_config* cfg, calvo_dispatcher** out) {
  if (!out) return fail(CALVO_EINVAL, "out is NULL");
  *out = nullptr;
  if (!cfg) return fail(CALVO_EINVAL, "config is NULL");
  if (cfg->policy < CALVO_POLICY_FIFO || cfg->policy > CALVO_POLICY_EDF) return fail(CALVO_EINVAL, "unknown policy %d", cfg->policy);
  if (c && c->n_staging == 0) return fail(CALVO_EINVAL, "the dispatcher needs a context with staging buffers");
  const calvo_l3_config& l3 = cfg->l3;
  if (cfg->three_stage) {
    if (l3.n_slots != 0 && (l3.n_slots < 2 || l3.n_slots > 8)) return fail(CALVO_EINVAL, "l3: n_slots must be 0 or in [2, 8]");
    if (l3.n_threads < 0 || l3.n_threads > 32) return fail(CALVO_EINVAL, "l3: n_threads must be in [0, 32]");
    if (!(l3.l3_GBps >= 0.0)) return fail(CALVO_EINVAL, "l3: l3_GBps must be non-negative");
  }
  calvo_dispatcher* d = new (std::nothrow) calvo_dispatcher();
  if (!d) return fail(CALVO_ENOMEM, "out of host memory");
  d->c = c;
  d->cfg = *cfg;
  d->t0 = clk::now();
  if (c && cfg->three_stage) {
    d->n_slots = l3.n_slots ? l3.n_slots : 3;
    d->n_threads = l3.n_threads ? l3.n_threads : 4;
    d->rate = l3.l3_GBps * 1e9;
    const int64_t want = l3.chunk_bytes ? (int64_t)(l3.chunk_bytes / c->blk_bytes) : c->staging_blocks;
    d->chunk_blocks = std::max<int64_t>(1, std::min<int64_t>(want, c->staging_blocks));
    const int rc = ensure_l2_ring(c, (size_t)d->chunk_blocks * c->blk_bytes, d->n_slots);
    if (rc != CALVO_OK) { delete d; return rc; }
    d->slot_state.assign((size_t)d->n_slots, 0);
  }
  try {
    if (c && cfg->three_stage) d->t_link = std::thread(link_main, d);
    d->t_pcie = std::thread(pcie_main, d);
    d->t_comp = std::thread(comp_main, d);
    if (c) d->t_done = std::thread(done_main, d);
  } catch (...) {
    (void)calvo_dispatch_destroy(d);
    return fail(CALVO_ENOMEM, "cannot start the dispatcher threads");
  }
  *out = d;
  return CALVO_OK;
}

int calvo_dispatch_submit(calvo_dispatcher* d, const calvo_dispatch_job* job, int64_t* id) {
  if (!d || !job || !id) return fail(CALVO_EINVAL, "NULL argument");
  if (job->n_prefix_blocks < 0 || job->suffix_len < 0 || job->n_shared < 0 || job->n_shared > job->n_prefix_blocks)
    return fail(CALVO_EINVAL, "bad block or token counts");
  const int n_tab = job->n_prefix_blocks + (job->suffix_len + kBlockTokens - 1) / kBlockTokens;
  calvo_ctx* c = d->c;
  const int n_given = d->cfg.pool ? job->n_shared : (c ? n_tab : 0);       // a dry run without a pool needs no slots
  if (n_given > 0 && !job->block_table) return fail(CALVO_EINVAL, "block_table is NULL");
  if (c) {
    if (job->n_prefix_blocks > job->n_shared && !job->host_kv) return fail(CALVO_EINVAL, "host_kv is NULL");
    if (job->suffix_len > 0 && (!job->q || !job->out)) return fail(CALVO_EINVAL, "q or out is NULL");
    if ((job->k_suffix == nullptr) != (job->v_suffix == nullptr)) return fail(CALVO_EINVAL, "k_suffix and v_suffix go together");
    if (job->q_layer_stride < 0 || job->kv_layer_stride < 0 || job->out_layer_stride < 0 || job->q_layer_stride % 16 ||
        job->kv_layer_stride % 16 || job->out_layer_stride % 16)
      return fail(CALVO_EINVAL, "layer strides must be non-negative multiples of 16 bytes");
    if ((job->q_layer_stride && job->q_layer_stride < (int64_t)job->suffix_len * c->cfg.n_q_heads * c->cfg.head_dim * (int64_t)c->elt) ||
        (job->out_layer_stride && job->out_layer_stride < (int64_t)job->suffix_len * c->cfg.n_q_heads * c->cfg.head_dim * (int64_t)c->elt) ||
        (job->kv_layer_stride && job->kv_layer_stride < (int64_t)job->suffix_len * c->cfg.n_kv_heads * c->cfg.head_dim * (int64_t)c->elt))
      return fail(CALVO_EINVAL, "a layer stride is smaller than one layer of the job");
    if (job->suffix_len > 0) {
      const int64_t L = c->cfg.n_layers;
      const int64_t q_layer = (int64_t)job->suffix_len * c->cfg.n_q_heads * c->cfg.head_dim * (int64_t)c->elt;
      const int64_t kv_layer = (int64_t)job->suffix_len * c->cfg.n_kv_heads * c->cfg.head_dim * (int64_t)c->elt;
      auto extent = [&](int64_t stride, int64_t layer) { return (L - 1) * (stride ? stride : layer) + layer; };
      int rc = check_device_extent(job->q, extent(job->q_layer_stride, q_layer), "q");
      if (rc == CALVO_OK) rc = check_device_extent(job->out, extent(job->out_layer_stride, q_layer), "out");
      if (rc == CALVO_OK) rc = check_device_extent(job->k_suffix, extent(job->kv_layer_stride, kv_layer), "k_suffix");
      if (rc == CALVO_OK) rc = check_device_extent(job->v_suffix, extent(job->kv_layer_stride, kv_layer), "v_suffix");
      if (rc != CALVO_OK) return rc;
    }
    if (n_tab > c->cfg.pool_blocks) return fail(CALVO_ENOMEM, "the job needs %d slots, the pool has %lld", n_tab, (long long)c->cfg.pool_blocks);
    if (!d->cfg.three_stage && job->n_prefix_blocks > job->n_shared) {
      hipPointerAttribute_t attr;
      const hipError_t e = hipPointerGetAttributes(&attr, job->host_kv);
      if (e != hipSuccess || attr.type != hipMemoryTypeHost) {
        (void)hipGetLastError();
        return fail(CALVO_EINVAL, "host_kv is not page-locked host memory (two-stage dispatcher)");
      }
    }
  } else if (!(job->sim_load_s >= 0.0) || !(job->sim_comp_s >= 0.0) || !std::isfinite(job->sim_load_s) || !std::isfinite(job->sim_comp_s)) {
    return fail(CALVO_EINVAL, "dry run: sim_load_s and sim_comp_s must be finite and non-negative");
  }
  std::unique_ptr<Job> j(new (std::nothrow) Job());
  if (!j) return fail(CALVO_ENOMEM, "out of host memory");
  j->spec = *job;
  j->n_tab = n_tab;
  if (n_given > 0) {
    j->shared.assign(job->block_table, job->block_table + job->n_shared);
    if (!d->cfg.pool) j->table.assign(job->block_table, job->block_table + n_tab);
  }
  j->spec.block_table = nullptr;
  if (c) {
    j->ev_layer.assign((size_t)c->cfg.n_layers, nullptr);
    hipError_t e = hipSuccess;
    for (auto& ev : j->ev_layer)
      if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&j->ev_done, hipEventDisableTiming);
    if (e != hipSuccess) {
      for (auto ev : j->ev_layer) if (ev) (void)hipEventDestroy(ev);
      if (j->ev_done) (void)hipEventDestroy(j->ev_done);
      return fail_hip(e, "hipEventCreate (job)");
    }
  }
  std::lock_guard<std::mutex> lk(d->mu);
  if (d->stop) return fail(CALVO_EINVAL, "the dispatcher is shutting down");
  j->id = (int64_t)d->jobs.size();
  const double t = d->now();
  j->res.submit_s = t;
  j->sched.arrival_s = t;
  j->sched.deadline_s = job->deadline_s > 0.0 ? t + job->deadline_s : std::numeric_limits<double>::infinity();
  j->sched.ctx_tokens = (int64_t)(job->n_prefix_blocks - job->n_shared) * kBlockTokens;
  j->sched.query_tokens = job->suffix_len;
  *id = j->id;
  d->jobs.push_back(std::move(j));
  d->cv.notify_all();
  return CALVO_OK;
}

int calvo_dispatch_wait(calvo_dispatcher* d, int64_t id, calvo_dispatch_result* res) {
  if (!d) return fail(CALVO_EINVAL, "dispatcher is NULL");
  std::unique_lock<std::mutex> lk(d->mu);
  Job* j = find_job(d, id);
  if (!j) return fail(CALVO_EINVAL, "unknown job %lld", (long long)id);
  d->cv.wait(lk, [&] { return j->finished; });
  if (res) *res = j->res;
  if (j->res.status != CALVO_OK) return fail(j->res.status, "job %lld failed: %s", (long long)id, j->err.c_str());
  return CALVO_OK;
}

int calvo_dispatch_poll(calvo_dispatcher* d, int64_t id, calvo_dispatch_result* res) {
  if (!d) return fail(CALVO_EINVAL, "dispatcher is NULL");
  std::lock_guard<std::mutex> lk(d->mu);
  Job* j = find_job(d, id);
  if (!j) return fail(CALVO_EINVAL, "unknown job %lld", (long long)id);
  if (res) *res = j->res;
  if (!j->finished) return CALVO_ENOTREADY;
  if (j->res.status != CALVO_OK) return fail(j->res.status, "job %lld failed: %s", (long long)id, j->err.c_str());
  return CALVO_OK;
}

int calvo_dispatch_table(calvo_dispatcher* d, int64_t id, int32_t* table, int32_t capacity, int32_t* n) {
  if (!d || !n) return fail(CALVO_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> lk(d->mu);
  Job* j = find_job(d, id);
  if (!j) return fail(CALVO_EINVAL, "unknown job %lld", (long long)id);
  if (!j->granted) return fail(CALVO_ENOTREADY, "job %lld has no slots yet", (long long)id);
  *n = j->n_tab;
  if (capacity < j->n_tab || (j->n_tab > 0 && !table)) return fail(CALVO_ENOMEM, "table needs %d entries", j->n_tab);
  if (j->n_tab) memcpy(table, j->table.data(), (size_t)j->n_tab * 4);
  return CALVO_OK;
}

int calvo_dispatch_release(calvo_dispatcher* d, int64_t id) {
  if (!d) return fail(CALVO_EINVAL, "dispatcher is NULL");
  calvo_batch* batch = nullptr;
  int rc = CALVO_OK;
  bool failed = false;
  {
    std::lock_guard<std::mutex> lk(d->mu);
    Job* j = find_job(d, id);
    if (!j) return fail(CALVO_EINVAL, "unknown job %lld", (long long)id);
    if (!j->finished) return fail(CALVO_ENOTREADY, "job %lld has not produced its first token yet", (long long)id);
    if (j->released) return fail(CALVO_EINVAL, "job %lld was released before", (long long)id);
    j->released = true;
    if (d->cfg.pool && j->granted && j->n_tab > 0) rc = calvo_pool_release(d->cfg.pool, j->table.data(), j->n_tab);
    batch = j->batch;
    j->batch = nullptr;
    failed = j->res.status != CALVO_OK;
    d->cv.notify_all();                   // requests that wait for slots try again
  }
  // a finished job's launches are complete (its last event has fired); a failed one may have some in flight
  if (failed && batch) (void)calvo_batch_destroy(batch);
  else batch_free_completed(batch);
  return rc;
}

int calvo_dispatch_stats_get(calvo_dispatcher* d, calvo_dispatch_stats* st) {
  if (!d || !st) return fail(CALVO_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> lk(d->mu);
  *st = d->stats;
  st->link_span_s = d->link_first >= 0 ? d->link_last - d->link_first : 0.0;
  st->jobs_submitted = (int64_t)d->jobs.size();
  return CALVO_OK;
}

int calvo_dispatch_destroy(calvo_dispatcher* d) {
  if (!d) return fail(CALVO_EINVAL, "dispatcher is NULL");
  {
    // let the work that has been submitted finish, then stop the stages; finished jobs that nobody
    // released give their slots back now, so that jobs which wait for slots can go on
    std::unique_lock<std::mutex> lk(d->mu);
    int quiet = 0;                          // consecutive rounds in which only slot waiters were left
    for (;;) {
      bool all = true, only_waiters = true, released_now = false;
      for (auto& j : d->jobs) {
        if (!j->finished) {
          all = false;
          if (!(j->load_picked && !j->granted)) only_waiters = false;      // queued, loading or computing: will move by itself
          continue;
        }
        if (d->cfg.pool && j->granted && !j->released && j->n_tab > 0) {
          (void)calvo_pool_release(d->cfg.pool, j->table.data(), j->n_tab);
          j->released = true;
          released_now = true;
          d->cv.notify_all();
        }
      }
      if (all) break;
      // Everything that can finish has finished and given its slots back, and what is left still waits for
      // slots: they are held outside this dispatcher, so those jobs are failed instead of waiting for ever.
      quiet = (only_waiters && !released_now) ? quiet + 1 : 0;
      if (quiet > 50) {
        d->cancel_waiting = true;
        d->cv.notify_all();
      }
      d->cv.wait_for(lk, std::chrono::milliseconds(2));
    }
    d->stop = true;
  }
  d->cv.notify_all();
  for (std::thread* t : {&d->t_link, &d->t_pcie, &d->t_comp, &d->t_done})
    if (t->joinable()) t->join();
  hipError_t e = hipSuccess, t;
  if (d->c) {
    calvo_ctx* c = d->c;
    for (auto& s : c->s_copy)
      if (s && (t = hipStreamSynchronize(s)) != hipSuccess) e = t;
    if (c->s_scatter && (t = hipStreamSynchronize(c->s_scatter)) != hipSuccess) e = t;
    if (c->s_compute && (t = hipStreamSynchronize(c->s_compute)) != hipSuccess) e = t;
  }
  for (auto& j : d->jobs) {
    batch_free_completed(j->batch);
    for (auto ev : j->ev_layer) if (ev) (void)hipEventDestroy(ev);
    if (j->ev_done) (void)hipEventDestroy(j->ev_done);
    if (d->cfg.pool && !j->granted && j->ticket >= 0) (void)calvo_pool_cancel(d->cfg.pool, j->ticket);
  }
  delete d;
  if (e != hipSuccess) return fail_hip(e, "synchronize at calvo_dispatch_destroy");
  return CALVO_OK;
}

}  // extern "C"
