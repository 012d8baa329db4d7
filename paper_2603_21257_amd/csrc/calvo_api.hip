// Host side of libcalvo: argument validation, the ingest pipeline (paper Section 3.1,
// the L2->L1 loading stage with its per-layer completion signal, and the emulated L3->L2
// stage in front of it), the block-table cache and the launch of the compute stage.
// See include/calvo.h for the contract.
#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "calvo_ctx.h"
#include "ingest_plan.h"

using namespace calvo;
using namespace calvo::host;

namespace {
thread_local std::string g_err;
}

namespace calvo {
namespace host {

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  (void)hipGetLastError();  // clear the sticky per-thread error
  return fail(e == hipErrorOutOfMemory ? CALVO_ENOMEM : CALVO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace host
}  // namespace calvo

namespace {

// ---- device memory for calvo_prefill_attn_noalloc: what calvo_prefill_attn keeps in buffers it
// allocates (the descriptor blob and the split-KV partial results) lives here in one file-scope
// array instead.  Every GPU the library runs on holds its own copy at its own address until the
// process ends; host code only ever uses the address obtained per device from
// hipGetSymbolAddress (the array's name is not a device address on the host side).
constexpr size_t kStaticBlobInts = (size_t)262144;                  // 1 MiB of descriptors: about 80000 table entries
constexpr size_t kStaticPartSlots = 2048;                           // (work item, head group, wave) slots
constexpr size_t kStaticBlobBytes = kStaticBlobInts * 4;
constexpr size_t kStaticPartOBytes = kStaticPartSlots * 32 * 128 * sizeof(float);   // 32 MiB
constexpr size_t kStaticPartMlBytes = kStaticPartSlots * 32 * 2 * sizeof(float);    // 512 KiB
constexpr size_t kScratchBytes = kStaticBlobBytes + kStaticPartOBytes + kStaticPartMlBytes;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Address of this device's copy of the array (looked up once per device, with that device current).
int scratch_for_device(int dev, unsigned char** out) {
  if (dev < 0 || dev >= kMaxDevices) return fail(CALVO_EINVAL, "device index %d not supported", dev);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (cur != dev) return fail(CALVO_EINVAL, "device %d is not the current device (%d)", dev, cur);
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(CALVO_EHIP, "hipGetSymbolAddress returned NULL");
    g_scratch_ptr[dev] = (unsigned char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return CALVO_OK;
}

}  // namespace

namespace {

void destroy_partial(calvo_ctx* c) {
  if (!c) return;
  for (void* p : c->staging)
    if (p) (void)hipFree(p);
  for (auto e : c->ev_filled) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_free) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_layer) if (e) (void)hipEventDestroy(e);
  for (auto& v : c->ev_chunk)
    for (auto e : v) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_t0) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_t1) if (e) (void)hipEventDestroy(e);
  for (void* p : c->l2_ring)
    if (p) (void)hipHostFree(p);
  for (auto e : c->ev_l2_free) if (e) (void)hipEventDestroy(e);
  if (c->ev_tab_ing) (void)hipEventDestroy(c->ev_tab_ing);
  for (auto e : c->ev_att) if (e) (void)hipEventDestroy(e);
  if (c->d_tab_ing) (void)hipFree(c->d_tab_ing);
  if (c->h_tab_ing) (void)hipHostFree(c->h_tab_ing);
  if (c->d_att) (void)hipFree(c->d_att);
  for (auto h : c->h_att) if (h) (void)hipHostFree(h);
  for (auto h : c->h_static) if (h) (void)hipHostFree(h);
  for (auto e : c->ev_static) if (e) (void)hipEventDestroy(e);
  if (c->part_o) (void)hipFree(c->part_o);
  if (c->part_ml) (void)hipFree(c->part_ml);
  for (auto& b : c->blob_free) { (void)hipFree(b.d); (void)hipHostFree(b.h); }
  for (auto& s : c->s_copy) if (s) (void)hipStreamDestroy(s);
  if (c->s_scatter) (void)hipStreamDestroy(c->s_scatter);
  if (c->own_compute && c->s_compute) (void)hipStreamDestroy(c->s_compute);
  (void)hipGetLastError();
  delete c;
}

int validate_config(const calvo_config* cfg) {
  if (!cfg) return fail(CALVO_EINVAL, "config is NULL");
  if (cfg->n_layers <= 0) return fail(CALVO_EINVAL, "n_layers must be positive");
  if (cfg->n_kv_heads <= 0 || cfg->n_q_heads <= 0 || cfg->n_q_heads % cfg->n_kv_heads != 0)
    return fail(CALVO_EINVAL, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", cfg->n_q_heads,
                cfg->n_kv_heads);
  if (cfg->head_dim <= 0 || cfg->head_dim > 256 || cfg->head_dim % 8 != 0)
    return fail(CALVO_EINVAL, "head_dim must be a multiple of 8 in [8, 256]");
  if (cfg->block_tokens != kBlockTokens) return fail(CALVO_EINVAL, "block_tokens must be 16");
  if (cfg->dtype != CALVO_BF16 && cfg->dtype != CALVO_F32) return fail(CALVO_EINVAL, "unknown dtype");
  if (cfg->pool_blocks <= 0 || cfg->pool_blocks > INT32_MAX) return fail(CALVO_EINVAL, "pool_blocks out of range");
  if (!cfg->pool) return fail(CALVO_EINVAL, "pool is NULL");
  if (((uintptr_t)cfg->pool & 15) != 0) return fail(CALVO_EINVAL, "pool must be 16-byte aligned");
  if (cfg->n_staging != 0 && (cfg->n_staging < 2 || cfg->n_staging > 8))
    return fail(CALVO_EINVAL, "n_staging must be 0 or in [2, 8]");
  if (cfg->n_copy_streams < 0 || cfg->n_copy_streams > 1) return fail(CALVO_EINVAL, "n_copy_streams must be 0 or 1");
  const size_t elt = cfg->dtype == CALVO_BF16 ? 2 : 4;
  const size_t blk = (size_t)2 * kBlockTokens * cfg->n_kv_heads * cfg->head_dim * elt;
  if (cfg->staging_bytes != 0 && cfg->staging_bytes < blk)
    return fail(CALVO_EINVAL, "staging_bytes (%zu) is smaller than one block (%zu)", cfg->staging_bytes, blk);
  return CALVO_OK;
}

}  // namespace

namespace calvo {
namespace host {

// Checks shared by ingest and attention.  Nothing is queued before these pass.
int validate_requests(const calvo_ctx* c, const calvo_request* reqs, int n_reqs, bool need_host,
                      std::vector<char>& seen) {
  if (!reqs && n_reqs > 0) return fail(CALVO_EINVAL, "reqs is NULL");
  if (n_reqs < 0) return fail(CALVO_EINVAL, "n_reqs is negative");
  for (int r = 0; r < n_reqs; r++) {
    const calvo_request& q = reqs[r];
    if (q.n_prefix_blocks < 0 || q.suffix_len < 0)
      return fail(CALVO_EINVAL, "request %d: negative block or token count", r);
    if (q.first_ingest_block < 0 || q.first_ingest_block > q.n_prefix_blocks)
      return fail(CALVO_EINVAL, "request %d: first_ingest_block outside [0, n_prefix_blocks]", r);
    const int64_t n_tab = (int64_t)q.n_prefix_blocks + (q.suffix_len + kBlockTokens - 1) / kBlockTokens;
    if (n_tab > c->cfg.pool_blocks)
      return fail(CALVO_ENOMEM, "request %d needs %lld slots, the pool has %lld", r, (long long)n_tab,
                  (long long)c->cfg.pool_blocks);
    if (n_tab > 0 && !q.block_table) return fail(CALVO_EINVAL, "request %d: block_table is NULL", r);
    if ((int64_t)q.n_prefix_blocks * kBlockTokens + q.suffix_len > INT32_MAX)
      return fail(CALVO_EINVAL, "request %d: context too long", r);
    seen.assign((size_t)c->cfg.pool_blocks, 0);
    for (int64_t j = 0; j < n_tab; j++) {
      const int32_t s = q.block_table[j];
      if (s < 0 || s >= c->cfg.pool_blocks)
        return fail(CALVO_EINVAL, "request %d: slot %d at table[%lld] is outside the pool (not allocated)", r, s,
                    (long long)j);
      if (seen[s]) return fail(CALVO_EINVAL, "request %d: slot %d appears twice in its table", r, s);
      seen[s] = 1;
    }
    if (need_host && q.n_prefix_blocks > q.first_ingest_block) {
      if (!q.host_kv) return fail(CALVO_EINVAL, "request %d: host_kv is NULL", r);
      if (((uintptr_t)q.host_kv & 15) != 0 || (q.host_layer_stride & 15) != 0)
        return fail(CALVO_EINVAL, "request %d: host_kv and host_layer_stride must be 16-byte aligned", r);
      if (c->cfg.n_layers > 1 && q.host_layer_stride < (int64_t)q.n_prefix_blocks * (int64_t)c->blk_bytes)
        return fail(CALVO_EINVAL, "request %d: host_layer_stride is smaller than the request's blocks", r);
    }
  }
  return CALVO_OK;
}

}  // namespace host
}  // namespace calvo

namespace {

int ensure_ing_table(calvo_ctx* c, size_t n) {
  if (n <= c->tab_ing_cap) return CALVO_OK;
  if (c->tab_ing_pending) { HIP_TRY(hipEventSynchronize(c->ev_tab_ing)); c->tab_ing_pending = false; }
  HIP_TRY(hipStreamSynchronize(c->s_scatter));
  size_t cap = std::max<size_t>(n, 4096);
  int32_t *d = nullptr, *h = nullptr;
  HIP_TRY(hipMalloc((void**)&d, cap * 4));
  hipError_t e = hipHostMalloc((void**)&h, cap * 4, hipHostMallocDefault);
  if (e != hipSuccess) { (void)hipFree(d); return fail_hip(e, "hipHostMalloc(table shadow)"); }
  if (c->d_tab_ing) (void)hipFree(c->d_tab_ing);
  if (c->h_tab_ing) (void)hipHostFree(c->h_tab_ing);
  c->d_tab_ing = d; c->h_tab_ing = h; c->tab_ing_cap = cap;
  return CALVO_OK;
}

int ensure_att_blob(calvo_ctx* c, size_t n) {
  if (n <= c->att_cap) return CALVO_OK;
  for (int k = 0; k < calvo_ctx::kShadows; k++)
    if (c->att_pending[k]) { HIP_TRY(hipEventSynchronize(c->ev_att[k])); c->att_pending[k] = false; }
  HIP_TRY(hipStreamSynchronize(c->s_compute));
  size_t cap = std::max<size_t>(n, 8192);
  int32_t* d = nullptr;
  int32_t* h[calvo_ctx::kShadows] = {nullptr, nullptr, nullptr, nullptr};
  HIP_TRY(hipMalloc((void**)&d, cap * 4));
  for (int k = 0; k < calvo_ctx::kShadows; k++) {
    hipError_t e = hipHostMalloc((void**)&h[k], cap * 4, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipFree(d);
      for (int j = 0; j < k; j++) (void)hipHostFree(h[j]);
      return fail_hip(e, "hipHostMalloc(descriptor shadow)");
    }
  }
  if (c->d_att) (void)hipFree(c->d_att);
  for (int k = 0; k < calvo_ctx::kShadows; k++) {
    if (c->h_att[k]) (void)hipHostFree(c->h_att[k]);
    c->h_att[k] = h[k];
  }
  c->d_att = d; c->att_cap = cap; c->att_len = 0; c->att_cur = 0;
  return CALVO_OK;
}


// Room for the split-KV partial results of `slots` (work item, head group, wave) triples.  Growing
// frees the old buffers, hence waits for the compute stream; contexts for bf16 / head-dim-128
// pools start with room for the short-query batches (kPartialSlots0), so only long chunk-granular
// layers ever grow it.
constexpr size_t kPartialSlots0 = 4096;      // 68 MB

int ensure_partials(calvo_ctx* c, size_t slots) {
  if (slots <= c->part_slots) return CALVO_OK;
  if (c->part_slots) HIP_TRY(hipStreamSynchronize(c->s_compute));
  if (c->part_o) (void)hipFree(c->part_o);
  if (c->part_ml) (void)hipFree(c->part_ml);
  c->part_o = c->part_ml = nullptr;
  c->part_slots = 0;
  slots = std::max(slots, kPartialSlots0);
  HIP_TRY(hipMalloc((void**)&c->part_o, slots * 32 * 128 * sizeof(float)));
  HIP_TRY(hipMalloc((void**)&c->part_ml, slots * 32 * 2 * sizeof(float)));
  c->part_slots = slots;
  return CALVO_OK;
}

// Waits for a running L3 loader and returns its status (CALVO_OK if none ran).  A failure is
// reported once: the call that returns it also forgets it and un-marks the layers the loader did
// not hand over, so that the context can load again.
int join_loader(calvo_ctx* c) {
  if (c->loader_started) {
    if (c->loader.joinable()) c->loader.join();
    c->loader_started = false;
  }
  std::lock_guard<std::mutex> lk(c->mu);
  const int rc = c->l3_status;
  if (rc != CALVO_OK) {
    g_err = c->l3_err;
    c->l3_status = CALVO_OK;
    c->l3_err.clear();
    for (size_t l = 0; l < c->layer_pending.size(); l++)
      if (c->layer_pending[l]) {
        c->layer_pending[l] = 0;
        c->layer_issued[l] = 0;
        c->chunks_issued[l] = 0;
        c->n_chunks[l] = 0;
        c->chunk_blocks[l] = 0;
      }
  }
  return rc;
}

// Blocks until a running loader has handed `layer` to the L2->L1 stage (or failed; the failure is
// then reported here and forgotten, see join_loader).
int wait_handed_over(calvo_ctx* c, int layer) {
  {
    std::unique_lock<std::mutex> lk(c->mu);
    c->cv.wait(lk, [&] { return !c->layer_pending[layer] || c->l3_status != CALVO_OK; });
    if (!c->layer_pending[layer]) return CALVO_OK;
  }
  return join_loader(c);        // the loader has failed: it is about to exit
}

// Blocks until chunk `chunk` of `layer` has been handed to the L2->L1 stage, i.e. its event has been
// recorded (at once unless a loader is still running), or the loader failed.
int wait_chunk_handed_over(calvo_ctx* c, int layer, int chunk) {
  {
    std::unique_lock<std::mutex> lk(c->mu);
    c->cv.wait(lk, [&] { return c->chunks_issued[layer] > chunk || !c->layer_pending[layer] || c->l3_status != CALVO_OK; });
    if (c->chunks_issued[layer] > chunk) return CALVO_OK;
    if (c->l3_status == CALVO_OK) return fail(CALVO_ENOTREADY, "chunk %d of layer %d was not loaded", chunk, layer);
  }
  return join_loader(c);
}

bool layer_is_issued(calvo_ctx* c, int layer) {
  std::lock_guard<std::mutex> lk(c->mu);
  return c->layer_issued[layer] != 0;
}

}  // namespace

namespace calvo {
namespace host {

// L2->L1 for nb consecutive blocks (nb <= staging_blocks) that sit in page-locked host memory:
// copy engine into the next device staging buffer, then scatter into the pool through the table.
// If done is given it is recorded on the copy stream right after the transfer (the source may be
// overwritten once it fires).
hipError_t enqueue_staged(calvo_ctx* c, const unsigned char* pinned_src, unsigned char* pool_layer,
                          const int32_t* d_table, int64_t nb, hipEvent_t done) {
  const int b = (int)(c->seq % (uint64_t)c->n_staging);
  hipStream_t cs = c->s_copy[c->seq % (uint64_t)c->n_copy];
  hipError_t e;
  if (c->test_ingest_delay_us > 0) std::this_thread::sleep_for(std::chrono::microseconds(c->test_ingest_delay_us));
  if (c->free_recorded[b] && (e = hipStreamWaitEvent(cs, c->ev_free[b], 0)) != hipSuccess) return e;
  if ((e = hipMemcpyAsync(c->staging[b], pinned_src, (size_t)nb * c->blk_bytes, hipMemcpyHostToDevice, cs)) != hipSuccess) return e;
  if (done && (e = hipEventRecord(done, cs)) != hipSuccess) return e;
  if ((e = hipEventRecord(c->ev_filled[b], cs)) != hipSuccess) return e;
  if ((e = hipStreamWaitEvent(c->s_scatter, c->ev_filled[b], 0)) != hipSuccess) return e;
  if (c->test_scatter_delay_us > 0 && (e = launch_delay(c->test_scatter_delay_us, c->s_scatter)) != hipSuccess) return e;
  if ((e = launch_scatter_blocks(c->staging[b], pool_layer, d_table, nb, (int32_t)c->blk_bytes, 1024, c->s_scatter)) != hipSuccess) return e;
  if ((e = hipEventRecord(c->ev_free[b], c->s_scatter)) != hipSuccess) return e;
  c->free_recorded[b] = 1;
  c->seq++;
  return hipSuccess;
}

}  // namespace host
}  // namespace calvo

namespace {

struct L3Request {            // what the loader keeps of a calvo_request after the call has returned
  const unsigned char* src;   // pageable "remote" memory
  int64_t layer_stride;
  int64_t first, nblk;
  int64_t tab_off;            // index of its block 0 in the device table (entries exist from `first` on)
};

struct L3Job {
  std::vector<L3Request> reqs;
  int layer_begin = 0, layer_end = 0;
  int64_t chunk_blocks = 0;
  bool chunk_ready = false;   // chunk-major order over block indices, one event per chunk
  int n_slots = 0, n_threads = 0;
  double rate = 0.0;          // bytes per second, 0 = unthrottled
};

}  // namespace

namespace calvo {
namespace host {

void parallel_copy(unsigned char* dst, const unsigned char* src, size_t n, int n_threads) {
  size_t piece = (n / (size_t)n_threads + 4095) & ~(size_t)4095;
  if (piece == 0 || n_threads <= 1 || n <= piece) {
    memcpy(dst, src, n);
    return;
  }
  std::vector<std::thread> th;
  for (size_t off = piece; off < n; off += piece)
    th.emplace_back([=] { memcpy(dst + off, src + off, std::min(piece, n - off)); });
  memcpy(dst, src, piece);
  for (auto& t : th) t.join();
}

}  // namespace host
}  // namespace calvo

namespace {

// Body of the loader thread: L3 -> L2 (host copy into the pinned ring, rate limited), then the
// hand-over of every landed chunk to the L2 -> L1 stage.
void loader_main(calvo_ctx* c, L3Job job) {
  using clock = std::chrono::steady_clock;
  const auto t_begin = clock::now();
  calvo_l3_stats st{};
  int status = CALVO_OK;
  std::string err;
  auto hip_fail = [&](hipError_t e, const char* what) {
    (void)hipGetLastError();
    status = e == hipErrorOutOfMemory ? CALVO_ENOMEM : CALVO_EHIP;
    err = std::string(what) + ": " + hipGetErrorString(e);
  };
  hipError_t e = hipSetDevice(c->device);
  if (e != hipSuccess) hip_fail(e, "hipSetDevice (loader)");
  auto link_free_at = clock::now();          // when the emulated link can start its next chunk
  uint64_t k = 0;
  // blocks [j0, j0 + nb) of request q, layer l (nb <= chunk_blocks): through one ring slot
  auto move_chunk = [&](int l, const L3Request& q, int64_t j0, int64_t nb) {
    unsigned char* pool_layer = (unsigned char*)c->cfg.pool + (int64_t)l * c->layer_bytes;
    const size_t bytes = (size_t)nb * c->blk_bytes;
    const int slot = (int)(k % (uint64_t)job.n_slots);
    if (c->test_l3_fail_chunk >= 0 && k == (uint64_t)c->test_l3_fail_chunk) {
      status = CALVO_EHIP;
      err = "injected failure of the L3 loader (CALVO_TEST_L3_FAIL_CHUNK)";
      return;
    }
    k++;
    auto t0 = clock::now();
    if (c->l2_free_recorded[slot] && (e = hipEventSynchronize(c->ev_l2_free[slot])) != hipSuccess) {
      hip_fail(e, "hipEventSynchronize (L2 ring slot)");
      return;
    }
    auto t1 = clock::now();
    const double waited = std::chrono::duration<double>(t1 - t0).count();
    st.ring_wait_s += waited;
    // The emulated link streams on its own: the time this thread spends handing a chunk to the
    // next stage does not hold it up.  It starts the next chunk when it is free, unless it had
    // to wait for a ring slot (back-pressure from L2 -> L1), in which case it starts now.
    const auto start = waited > 50e-6 ? std::max(t1, link_free_at) : link_free_at;
    parallel_copy((unsigned char*)c->l2_ring[slot],
                  q.src + (int64_t)l * q.layer_stride + j0 * (int64_t)c->blk_bytes, bytes, job.n_threads);
    if (job.rate > 0.0) {
      link_free_at = start + std::chrono::duration_cast<clock::duration>(std::chrono::duration<double>((double)bytes / job.rate));
      std::this_thread::sleep_until(link_free_at);
    }
    st.l3_busy_s += std::chrono::duration<double>(clock::now() - t1).count();
    st.bytes += (int64_t)bytes;
    st.chunks++;
    e = enqueue_staged(c, (const unsigned char*)c->l2_ring[slot], pool_layer, c->d_tab_ing + q.tab_off + j0, nb,
                       c->ev_l2_free[slot]);
    if (e != hipSuccess) { hip_fail(e, "L2 -> L1 hand-over"); return; }
    c->l2_free_recorded[slot] = 1;
  };
  int64_t max_blocks = 0;
  for (const L3Request& q : job.reqs) max_blocks = std::max(max_blocks, q.nblk);
  for (int l = job.layer_begin; l < job.layer_end && status == CALVO_OK; l++) {
    if (!job.chunk_ready) {
      for (size_t r = 0; r < job.reqs.size() && status == CALVO_OK; r++) {
        const L3Request& q = job.reqs[r];
        for (int64_t j0 = q.first; j0 < q.nblk && status == CALVO_OK; j0 += job.chunk_blocks)
          move_chunk(l, q, j0, std::min<int64_t>(job.chunk_blocks, q.nblk - j0));
      }
    } else {
      // chunk n = block indices [n cb, (n+1) cb) of every request, signalled as soon as it is queued
      const int64_t cb = job.chunk_blocks, nck = (max_blocks + cb - 1) / cb;
      for (int64_t n = 0; n < nck && status == CALVO_OK; n++) {
        for (size_t r = 0; r < job.reqs.size() && status == CALVO_OK; r++) {
          const L3Request& q = job.reqs[r];
          const int64_t j0 = std::max(q.first, n * cb), j1 = std::min(q.nblk, (n + 1) * cb);
          if (j0 < j1) move_chunk(l, q, j0, j1 - j0);
        }
        if (status != CALVO_OK) break;
        if ((e = hipEventRecord(c->ev_chunk[l][(size_t)n], c->s_scatter)) != hipSuccess) { hip_fail(e, "hipEventRecord (chunk)"); break; }
        {
          std::lock_guard<std::mutex> lk(c->mu);
          c->chunks_issued[l] = (int32_t)(n + 1);
        }
        c->cv.notify_all();
      }
    }
    if (status != CALVO_OK) break;
    if ((e = hipEventRecord(c->ev_layer[l], c->s_scatter)) != hipSuccess) { hip_fail(e, "hipEventRecord (layer)"); break; }
    {
      std::lock_guard<std::mutex> lk(c->mu);
      c->layer_issued[l] = 1;
      c->layer_pending[l] = 0;
    }
    c->cv.notify_all();
  }
  st.total_s = std::chrono::duration<double>(clock::now() - t_begin).count();
  {
    std::lock_guard<std::mutex> lk(c->mu);
    c->l3_stats = st;
    c->l3_status = status;
    c->l3_err = err;
  }
  c->cv.notify_all();     // on failure the waiters see the status; pending layers stay pending
}

}  // namespace

extern "C" {

const char* calvo_last_error(void) { return g_err.c_str(); }

int calvo_create(const calvo_config* cfg, calvo_ctx** out) {
  if (!out) return fail(CALVO_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = validate_config(cfg);
  if (rc != CALVO_OK) return rc;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  calvo_ctx* c = new (std::nothrow) calvo_ctx();
  if (!c) return fail(CALVO_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  c->device = dev;
  {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) c->n_cus = cus;
    else (void)hipGetLastError();
  }
  c->elt = cfg->dtype == CALVO_BF16 ? 2 : 4;
  c->blk_bytes = (size_t)2 * kBlockTokens * cfg->n_kv_heads * cfg->head_dim * c->elt;
  c->layer_bytes = (int64_t)cfg->pool_blocks * (int64_t)c->blk_bytes;
  c->n_staging = cfg->staging_bytes ? (cfg->n_staging ? cfg->n_staging : 2) : 0;
  c->n_copy = cfg->n_copy_streams ? cfg->n_copy_streams : 1;
  c->staging_blocks = cfg->staging_bytes / c->blk_bytes;
  if (const char* e = getenv("CALVO_ATTN_SPLITS")) {    // test knob: cut every tile's context into this many pieces
    const int g = atoi(e);
    if (g >= 1 && g <= 64) c->force_splits = g;
  }
  if (const char* e = getenv("CALVO_INGEST_DELAY_US")) { const int g = atoi(e); if (g > 0 && g <= 1000000) c->test_ingest_delay_us = g; }
  if (const char* e = getenv("CALVO_TEST_SCATTER_DELAY_US")) { const int g = atoi(e); if (g > 0 && g <= 20000) c->test_scatter_delay_us = g; }
  if (const char* e = getenv("CALVO_TEST_L3_FAIL_CHUNK")) { const int g = atoi(e); if (g >= 0) c->test_l3_fail_chunk = g; }
  if (const char* e = getenv("CALVO_SPLIT_MIN")) { const int g = atoi(e); if (g >= 1 && g <= 4096) c->split_min = g; }
  if (const char* e = getenv("CALVO_SPLIT_FILL")) { const int g = atoi(e); if (g >= 0 && g <= 4096) c->split_fill = g; }
  if (const char* e = getenv("CALVO_MERGE_MIB")) { const int g = atoi(e); if (g >= 0 && g <= 4096) c->merge_bytes = (size_t)g << 20; }
  if (const char* e = getenv("CALVO_SCATTER_GRID")) {   // tuning knob: workgroups of the zero-copy scatter
    const int g = atoi(e);
    if (g >= 1 && g <= 4096) c->scatter_grid = g;
  }

#define CREATE_TRY(expr)                                                        \
  do {                                                                          \
    hipError_t e_ = (expr);                                                     \
    if (e_ != hipSuccess) { int rc_ = fail_hip(e_, #expr); destroy_partial(c); return rc_; } \
  } while (0)

  for (int i = 0; i < c->n_copy; i++) CREATE_TRY(hipStreamCreateWithFlags(&c->s_copy[i], hipStreamNonBlocking));
  CREATE_TRY(hipStreamCreateWithFlags(&c->s_scatter, hipStreamNonBlocking));
  if (cfg->compute_stream) {
    c->s_compute = (hipStream_t)cfg->compute_stream;
  } else {
    CREATE_TRY(hipStreamCreateWithFlags(&c->s_compute, hipStreamNonBlocking));
    c->own_compute = true;
  }
  c->staging.assign(c->n_staging, nullptr);
  c->ev_filled.assign(c->n_staging, nullptr);
  c->ev_free.assign(c->n_staging, nullptr);
  c->free_recorded.assign(c->n_staging, 0);
  for (int i = 0; i < c->n_staging; i++) {
    CREATE_TRY(hipMalloc(&c->staging[i], (size_t)c->staging_blocks * c->blk_bytes));
    CREATE_TRY(hipEventCreateWithFlags(&c->ev_filled[i], hipEventDisableTiming));
    CREATE_TRY(hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
  }
  c->ev_layer.assign(cfg->n_layers, nullptr);
  c->ev_t0.assign(cfg->n_layers, nullptr);
  c->ev_t1.assign(cfg->n_layers, nullptr);
  c->layer_issued.assign(cfg->n_layers, 0);
  c->chunk_blocks.assign(cfg->n_layers, 0);
  c->n_chunks.assign(cfg->n_layers, 0);
  c->chunks_issued.assign(cfg->n_layers, 0);
  c->ev_chunk.resize(cfg->n_layers);
  c->layer_pending.assign(cfg->n_layers, 0);
  c->timed.assign(cfg->n_layers, 0);
  c->last_variant.assign(cfg->n_layers, -1);
  c->last_wgs.assign(cfg->n_layers, 0);
  for (int l = 0; l < cfg->n_layers; l++) {
    CREATE_TRY(hipEventCreateWithFlags(&c->ev_layer[l], hipEventDisableTiming));
    CREATE_TRY(hipEventCreate(&c->ev_t0[l]));
    CREATE_TRY(hipEventCreate(&c->ev_t1[l]));
  }
  CREATE_TRY(hipEventCreateWithFlags(&c->ev_tab_ing, hipEventDisableTiming));
  for (auto& e : c->ev_att) CREATE_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  for (auto& e : c->ev_static) CREATE_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  for (auto& h : c->h_static) CREATE_TRY(hipHostMalloc((void**)&h, kStaticBlobBytes, hipHostMallocDefault));
#undef CREATE_TRY
  {
    const int src = scratch_for_device(dev, &c->d_static);
    if (src != CALVO_OK) { destroy_partial(c); return src; }
  }
  if (cfg->dtype == CALVO_BF16 && cfg->head_dim == 128) {
    // the pipelined kernels use more dynamic LDS than the default limit (a per-device attribute)
    hipError_t e = attn_pipe_prepare();
    if (e == hipSuccess) e = attn_duo_prepare();
    if (e != hipSuccess) { const int prc = fail_hip(e, "hipFuncSetAttribute(dynamic LDS)"); destroy_partial(c); return prc; }
  }
  if (cfg->dtype == CALVO_BF16 && cfg->head_dim == 128) {
    const int prc = ensure_partials(c, kPartialSlots0);
    if (prc != CALVO_OK) { destroy_partial(c); return prc; }
  }
  *out = c;
  return CALVO_OK;
}

int calvo_destroy(calvo_ctx* c) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  (void)join_loader(c);
  hipError_t e = hipSuccess, t;
  for (auto& s : c->s_copy)
    if (s && (t = hipStreamSynchronize(s)) != hipSuccess) e = t;
  if (c->s_scatter && (t = hipStreamSynchronize(c->s_scatter)) != hipSuccess) e = t;
  if (c->s_compute && (t = hipStreamSynchronize(c->s_compute)) != hipSuccess) e = t;
  destroy_partial(c);
  if (e != hipSuccess) return fail_hip(e, "synchronize at destroy");
  return CALVO_OK;
}

}  // extern "C"

namespace {

}  // namespace

namespace calvo {
namespace host {

int upload_ingest_table(calvo_ctx* c, const int32_t* slots, size_t n) {
  if (n == 0) return CALVO_OK;
  int rc = ensure_ing_table(c, n);
  if (rc != CALVO_OK) return rc;
  // the pinned shadow is read when the scatter stream gets to the previous upload
  if (c->tab_ing_pending) { HIP_TRY(hipEventSynchronize(c->ev_tab_ing)); c->tab_ing_pending = false; }
  memcpy(c->h_tab_ing, slots, n * 4);
  HIP_TRY(hipMemcpyAsync(c->d_tab_ing, c->h_tab_ing, n * 4, hipMemcpyHostToDevice, c->s_scatter));
  HIP_TRY(hipEventRecord(c->ev_tab_ing, c->s_scatter));
  c->tab_ing_pending = true;
  return CALVO_OK;
}

int ensure_l2_ring(calvo_ctx* c, size_t slot_bytes, int n_slots) {
  if (slot_bytes <= c->l2_slot_bytes && (int)c->l2_ring.size() >= n_slots) return CALVO_OK;
  for (auto& s : c->s_copy) if (s) HIP_TRY(hipStreamSynchronize(s));
  for (void* p : c->l2_ring) if (p) (void)hipHostFree(p);
  for (auto e : c->ev_l2_free) if (e) (void)hipEventDestroy(e);
  c->l2_ring.assign(n_slots, nullptr);
  c->ev_l2_free.assign(n_slots, nullptr);
  c->l2_free_recorded.assign(n_slots, 0);
  c->l2_slot_bytes = 0;
  for (int i = 0; i < n_slots; i++) {
    hipError_t e = hipHostMalloc(&c->l2_ring[i], slot_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_l2_free[i], hipEventDisableTiming);
    if (e != hipSuccess) return fail_hip(e, "pinned L2 ring");
  }
  c->l2_slot_bytes = slot_bytes;
  return CALVO_OK;
}

}  // namespace host
}  // namespace calvo

namespace {

// Front part shared by both ingest calls: validation, source pointers, block tables to the device.
// pinned: the sources must be page-locked (and device-mapped for the zero-copy mode).
int prepare_ingest(calvo_ctx* c, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end, bool pinned,
                   std::vector<const unsigned char*>& src, std::vector<int64_t>& tab_off) {
  if (layer_begin < 0 || layer_end > c->cfg.n_layers || layer_begin > layer_end)
    return fail(CALVO_EINVAL, "layer range [%d, %d) outside [0, %d]", layer_begin, layer_end, c->cfg.n_layers);
  std::vector<char> seen;
  int rc = validate_requests(c, reqs, n_reqs, true, seen);
  if (rc != CALVO_OK) return rc;
  src.assign(n_reqs, nullptr);
  tab_off.assign(n_reqs, 0);
  // The device table holds the slots of the blocks that are loaded, request after request, so that
  // requests whose host blocks follow each other also have consecutive table entries (one transfer
  // and one scatter can then serve several of them).  tab_off[r] + j is the entry of block j >= first.
  size_t n_tab = 0;
  for (int r = 0; r < n_reqs; r++) {
    tab_off[r] = (int64_t)n_tab - reqs[r].first_ingest_block;
    n_tab += (size_t)(reqs[r].n_prefix_blocks - reqs[r].first_ingest_block);
    if (reqs[r].n_prefix_blocks == reqs[r].first_ingest_block) continue;
    void* dp = const_cast<void*>(reqs[r].host_kv);
    if (pinned) {
      // the source must be page-locked host memory the device can address
      hipPointerAttribute_t attr;
      hipError_t e = hipPointerGetAttributes(&attr, reqs[r].host_kv);
      if (e != hipSuccess || attr.type != hipMemoryTypeHost) {
        (void)hipGetLastError();
        return fail(CALVO_EINVAL, "request %d: host_kv is not page-locked host memory", r);
      }
      if (c->n_staging == 0) {
        dp = nullptr;
        e = hipHostGetDevicePointer(&dp, const_cast<void*>(reqs[r].host_kv), 0);
        if (e != hipSuccess || !dp) {
          (void)hipGetLastError();
          return fail(CALVO_EINVAL, "request %d: host_kv has no device mapping", r);
        }
      }
    }
    src[r] = (const unsigned char*)dp;
  }
  if (layer_begin == layer_end || n_reqs == 0) return CALVO_OK;
  // block tables -> device (ingest stream)
  if (n_tab > 0) {
    std::vector<int32_t> slots(n_tab);
    for (int r = 0; r < n_reqs; r++)
      if (reqs[r].n_prefix_blocks > reqs[r].first_ingest_block)
        memcpy(slots.data() + tab_off[r] + reqs[r].first_ingest_block, reqs[r].block_table + reqs[r].first_ingest_block,
               (size_t)(reqs[r].n_prefix_blocks - reqs[r].first_ingest_block) * 4);
    rc = upload_ingest_table(c, slots.data(), n_tab);
    if (rc != CALVO_OK) return rc;
  }
  return CALVO_OK;
}

// What the attention kernels read besides Q and the pool, as one array of int32 (offsets in int32):
// request descriptors (ReqDesc x n), work items, first items of the cut tiles, per-launch work item
// lists, block tables, block byte offsets.  Each request's table is followed by copies of its last
// entry (kTablePad of them, one more if that makes the count even) so that a kernel may look
// kTablePad blocks past the end without clamping.  The offsets are slot * block_bytes (the byte
// offset of the block inside a layer of the pool) for the same blocks, split by parity: first those
// of blocks 0, 2, 4, ... then those of blocks 1, 3, 5, ... - a wave that always fetches the same
// half of a 32-key sub-tile reads its offsets from consecutive addresses.
struct BlobLayout {
  size_t items_off = 0, split_off = 0, tables_off = 0, offs_off = 0;
  std::vector<size_t> group_off;
};

BlobLayout build_descriptor_blob(const calvo_ctx* c, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix,
                                 const PlanItems& plan, std::vector<int32_t>& blob) {
  BlobLayout lay;
  auto table_len = [&](int r) { return (int64_t)reqs[r].n_prefix_blocks + (reqs[r].suffix_len + kBlockTokens - 1) / kBlockTokens; };
  blob.clear();
  blob.reserve(4 * n_reqs + 1024);
  size_t n_tab = 0;
  for (int r = 0; r < n_reqs; r++) {
    const int64_t nt = table_len(r);
    blob.push_back((int32_t)n_tab);
    blob.push_back(reqs[r].n_prefix_blocks * kBlockTokens);
    blob.push_back(reqs[r].suffix_len);
    blob.push_back(cu_suffix[r]);
    n_tab += (size_t)nt + kTablePad + (nt & 1);
  }
  lay.items_off = blob.size();
  for (const WorkItem& it : plan.items) {
    const int32_t* w = (const int32_t*)&it;
    blob.insert(blob.end(), w, w + sizeof(WorkItem) / 4);
  }
  lay.split_off = blob.size();
  blob.insert(blob.end(), plan.split_tiles.begin(), plan.split_tiles.end());
  for (const auto& g : plan.groups) {
    lay.group_off.push_back(blob.size());
    blob.insert(blob.end(), g.begin(), g.end());
  }
  lay.tables_off = blob.size();
  for (int r = 0; r < n_reqs; r++) {
    const int64_t nt = table_len(r);
    blob.insert(blob.end(), reqs[r].block_table, reqs[r].block_table + nt);
    blob.insert(blob.end(), kTablePad + (nt & 1), nt > 0 ? reqs[r].block_table[nt - 1] : 0);
  }
  if (blob.size() & 1) blob.push_back(0);                       // 8-byte alignment of the offsets
  lay.offs_off = blob.size();
  size_t base = lay.tables_off;
  for (int r = 0; r < n_reqs; r++) {
    const int64_t nt = table_len(r);
    const size_t padded = (size_t)nt + kTablePad + (nt & 1);
    for (int par = 0; par < 2; par++)
      for (size_t i = par; i < padded; i += 2) {
        const int64_t off = (int64_t)blob[base + i] * (int64_t)c->blk_bytes;
        blob.push_back((int32_t)(uint32_t)(off & 0xffffffff));
        blob.push_back((int32_t)(off >> 32));
      }
    base += padded;
  }
  return lay;
}

}  // namespace

extern "C" {

static int ingest_impl(calvo_ctx* c, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end,
                       const int32_t* chunk_blocks) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  if (chunk_blocks && layer_begin >= 0 && layer_end <= c->cfg.n_layers)
    for (int l = layer_begin; l < layer_end; l++) {
      const int32_t cb = chunk_blocks[l - layer_begin];
      if (cb < 0 || (cb & 1)) return fail(CALVO_EINVAL, "chunk_blocks[%d] = %d must be 0 or a positive even number", l - layer_begin, cb);
    }
  int rc = join_loader(c);
  if (rc != CALVO_OK) return rc;
  std::vector<const unsigned char*> src;
  std::vector<int64_t> tab_off;
  rc = prepare_ingest(c, reqs, n_reqs, layer_begin, layer_end, true, src, tab_off);
  if (rc != CALVO_OK) return rc;
  if (layer_begin == layer_end || n_reqs == 0) return CALVO_OK;
  int64_t max_blocks = 0;
  for (int r = 0; r < n_reqs; r++) max_blocks = std::max<int64_t>(max_blocks, reqs[r].n_prefix_blocks);

  // blocks [j0, j1) of request r, layer l: one scatter launch (zero-copy) or staged pieces
  auto load_range = [&](int l, int r, int64_t j0, int64_t j1) -> int {
    const calvo_request& q = reqs[r];
    unsigned char* pool_layer = (unsigned char*)c->cfg.pool + (int64_t)l * c->layer_bytes;
    const unsigned char* lsrc = src[r] + (int64_t)l * q.host_layer_stride;
    if (c->n_staging == 0) {
      // zero-copy: the scatter kernel reads the pinned blocks over PCIe itself
      HIP_TRY(launch_scatter_blocks(lsrc + j0 * (int64_t)c->blk_bytes, pool_layer, c->d_tab_ing + tab_off[r] + j0,
                                    j1 - j0, (int32_t)c->blk_bytes, c->scatter_grid, c->s_scatter));
      return CALVO_OK;
    }
    for (int64_t j = j0; j < j1; j += c->staging_blocks) {
      const int64_t nb = std::min<int64_t>(c->staging_blocks, j1 - j);
      HIP_TRY(enqueue_staged(c, lsrc + j * (int64_t)c->blk_bytes, pool_layer, c->d_tab_ing + tab_off[r] + j, nb, nullptr));
    }
    return CALVO_OK;
  };

  // Requests whose host blocks (and hence table entries) follow each other load as one run, and
  // consecutive small layers share a transfer: see ingest_plan.cpp.
  std::vector<IngestSrc> isrc((size_t)n_reqs);
  for (int r = 0; r < n_reqs; r++)
    isrc[(size_t)r] = {(uintptr_t)src[r], reqs[r].host_layer_stride, reqs[r].first_ingest_block, reqs[r].n_prefix_blocks,
                       tab_off[r]};
  auto chunk_of = [&](int l) -> int64_t { return chunk_blocks ? chunk_blocks[l - layer_begin] : 0; };
  auto mark_issued = [&](int l, int64_t cb, int64_t nck) {
    std::lock_guard<std::mutex> lk(c->mu);
    c->layer_issued[l] = 1;
    c->chunk_blocks[l] = (int32_t)cb;
    c->n_chunks[l] = (int32_t)nck;
    c->chunks_issued[l] = (int32_t)nck;
  };

  int group = 0;                       // whole-layer transfers issued so far (sets the merge ramp)
  for (int l = layer_begin; l < layer_end;) {
    const int64_t cb = chunk_of(l);
    if (cb > 0) {
      const int64_t nck = (max_blocks + cb - 1) / cb;
      while ((int64_t)c->ev_chunk[l].size() < nck) {       // events of this layer's chunks (kept for later calls)
        hipEvent_t ev = nullptr;
        HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        c->ev_chunk[l].push_back(ev);
      }
      // chunk k = block indices [k cb, (k+1) cb) of every request (a shared run sits at the same
      // indices in every table, so once chunk k is in, all blocks below (k+1) cb are resident)
      for (int64_t k = 0; k < nck; k++) {
        for (int r = 0; r < n_reqs; r++) {
          const int64_t j0 = std::max<int64_t>(reqs[r].first_ingest_block, k * cb);
          const int64_t j1 = std::min<int64_t>(reqs[r].n_prefix_blocks, (k + 1) * cb);
          if (j0 < j1 && (rc = load_range(l, r, j0, j1)) != CALVO_OK) return rc;
        }
        HIP_TRY(hipEventRecord(c->ev_chunk[l][k], c->s_scatter));
      }
      HIP_TRY(hipEventRecord(c->ev_layer[l], c->s_scatter));
      mark_issued(l, cb, nck);
      l++;
      continue;
    }
    const std::vector<IngestRun> runs = ingest_layer_runs(isrc.data(), n_reqs, l, c->blk_bytes);
    const int k = ingest_group_layers(isrc.data(), n_reqs, l, layer_end, chunk_blocks, layer_begin, c->blk_bytes,
                                      c->n_staging > 0 ? c->staging_blocks : 0, c->merge_bytes, group);
    if (k > 1) {
      const IngestRun& u = runs[0];
      const int64_t nb = u.j1 - u.j0;
      const size_t run_bytes = (size_t)nb * c->blk_bytes;
      const int b = (int)(c->seq % (uint64_t)c->n_staging);
      hipStream_t cs = c->s_copy[c->seq % (uint64_t)c->n_copy];
      if (c->free_recorded[b]) HIP_TRY(hipStreamWaitEvent(cs, c->ev_free[b], 0));
      HIP_TRY(hipMemcpyAsync(c->staging[b], (const void*)u.beg, (size_t)k * run_bytes, hipMemcpyHostToDevice, cs));
      HIP_TRY(hipEventRecord(c->ev_filled[b], cs));
      HIP_TRY(hipStreamWaitEvent(c->s_scatter, c->ev_filled[b], 0));
      for (int i = 0; i < k; i++) {
        unsigned char* pool_layer = (unsigned char*)c->cfg.pool + (int64_t)(l + i) * c->layer_bytes;
        HIP_TRY(launch_scatter_blocks((const unsigned char*)c->staging[b] + (size_t)i * run_bytes, pool_layer,
                                      c->d_tab_ing + tab_off[u.r] + u.j0, nb, (int32_t)c->blk_bytes, 1024, c->s_scatter));
        HIP_TRY(hipEventRecord(c->ev_layer[l + i], c->s_scatter));
        mark_issued(l + i, 0, 0);
      }
      HIP_TRY(hipEventRecord(c->ev_free[b], c->s_scatter));
      c->free_recorded[b] = 1;
      c->seq++;
    } else {
      for (const IngestRun& u : runs)
        if ((rc = load_range(l, u.r, u.j0, u.j1)) != CALVO_OK) return rc;
      HIP_TRY(hipEventRecord(c->ev_layer[l], c->s_scatter));
      mark_issued(l, 0, 0);
    }
    group++;
    l += k;
  }
  return CALVO_OK;
}

int calvo_kv_ingest(calvo_ctx* c, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end) {
  return ingest_impl(c, reqs, n_reqs, layer_begin, layer_end, nullptr);
}

int calvo_kv_ingest_chunked(calvo_ctx* c, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end,
                            const int32_t* chunk_blocks) {
  if (!chunk_blocks) return fail(CALVO_EINVAL, "chunk_blocks is NULL");
  return ingest_impl(c, reqs, n_reqs, layer_begin, layer_end, chunk_blocks);
}

int calvo_chunk_count(calvo_ctx* c, int layer, int* n_chunks) {
  if (!c || !n_chunks) return fail(CALVO_EINVAL, "ctx or n_chunks is NULL");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  std::lock_guard<std::mutex> lk(c->mu);
  *n_chunks = c->n_chunks[layer];
  return CALVO_OK;
}

int calvo_chunk_event(calvo_ctx* c, int layer, int chunk, int mode, void* stream) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  if (mode != CALVO_EV_QUERY && mode != CALVO_EV_HOST_WAIT && mode != CALVO_EV_STREAM_WAIT)
    return fail(CALVO_EINVAL, "unknown mode %d", mode);
  int nck;
  {
    std::lock_guard<std::mutex> lk(c->mu);
    nck = c->n_chunks[layer];
  }
  if (chunk < 0 || chunk >= nck) return fail(CALVO_EINVAL, "chunk %d outside [0, %d) of layer %d", chunk, nck, layer);
  if (mode == CALVO_EV_QUERY) {
    std::unique_lock<std::mutex> lk(c->mu);
    if (c->chunks_issued[layer] <= chunk) {              // a running loader has not reached it yet
      if (c->l3_status != CALVO_OK) { lk.unlock(); return join_loader(c); }
      return fail(CALVO_ENOTREADY, "chunk %d of layer %d is still loading", chunk, layer);
    }
  } else {
    const int rc = wait_chunk_handed_over(c, layer, chunk);
    if (rc != CALVO_OK) return rc;
  }
  hipEvent_t ev = c->ev_chunk[layer][chunk];
  if (mode == CALVO_EV_QUERY) {
    hipError_t e = hipEventQuery(ev);
    if (e == hipSuccess) return CALVO_OK;
    if (e == hipErrorNotReady) { (void)hipGetLastError(); return fail(CALVO_ENOTREADY, "chunk %d of layer %d is still loading", chunk, layer); }
    return fail_hip(e, "hipEventQuery");
  }
  if (mode == CALVO_EV_HOST_WAIT) {
    HIP_TRY(hipEventSynchronize(ev));
    return CALVO_OK;
  }
  HIP_TRY(hipStreamWaitEvent(stream ? (hipStream_t)stream : c->s_compute, ev, 0));
  return CALVO_OK;
}

int calvo_kv_ingest_l3(calvo_ctx* c, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end,
                       const calvo_l3_config* l3) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  if (c->n_staging == 0) return fail(CALVO_EINVAL, "three-stage loading needs a context with staging buffers");
  calvo_l3_config cfg{};
  if (l3) cfg = *l3;
  if (cfg.n_slots != 0 && (cfg.n_slots < 2 || cfg.n_slots > 8)) return fail(CALVO_EINVAL, "l3: n_slots must be 0 or in [2, 8]");
  if (cfg.n_threads < 0 || cfg.n_threads > 32) return fail(CALVO_EINVAL, "l3: n_threads must be in [0, 32]");
  if (!(cfg.l3_GBps >= 0.0)) return fail(CALVO_EINVAL, "l3: l3_GBps must be non-negative");
  if (cfg.chunk_bytes != 0 && cfg.chunk_bytes < c->blk_bytes)
    return fail(CALVO_EINVAL, "l3: chunk_bytes (%zu) is smaller than one block (%zu)", cfg.chunk_bytes, c->blk_bytes);
  int rc = join_loader(c);
  if (rc != CALVO_OK) return rc;
  std::vector<const unsigned char*> src;
  std::vector<int64_t> tab_off;
  rc = prepare_ingest(c, reqs, n_reqs, layer_begin, layer_end, false, src, tab_off);
  if (rc != CALVO_OK) return rc;
  {
    std::lock_guard<std::mutex> lk(c->mu);
    c->l3_stats = calvo_l3_stats{};
  }
  if (layer_begin == layer_end || n_reqs == 0) return CALVO_OK;

  L3Job job;
  job.layer_begin = layer_begin;
  job.layer_end = layer_end;
  job.n_slots = cfg.n_slots ? cfg.n_slots : 3;
  job.n_threads = cfg.n_threads ? cfg.n_threads : 4;
  job.rate = cfg.l3_GBps * 1e9;
  const int64_t want = cfg.chunk_bytes ? (int64_t)(cfg.chunk_bytes / c->blk_bytes) : c->staging_blocks;
  job.chunk_blocks = std::min<int64_t>(want, c->staging_blocks);
  job.chunk_ready = cfg.chunk_ready != 0;
  int64_t max_blocks = 0;
  for (int r = 0; r < n_reqs; r++) max_blocks = std::max<int64_t>(max_blocks, reqs[r].n_prefix_blocks);
  if (job.chunk_ready) {
    job.chunk_blocks &= ~(int64_t)1;                    // attention walks the context two blocks at a time
    if (job.chunk_blocks < 2) return fail(CALVO_EINVAL, "l3: chunk-granular readiness needs chunks of at least two blocks");
  }
  for (int r = 0; r < n_reqs; r++)
    if (reqs[r].n_prefix_blocks > reqs[r].first_ingest_block)
      job.reqs.push_back({src[r], reqs[r].host_layer_stride, reqs[r].first_ingest_block, reqs[r].n_prefix_blocks, tab_off[r]});

  // the pinned ring (kept for later calls; regrown if a call asks for more)
  rc = ensure_l2_ring(c, (size_t)job.chunk_blocks * c->blk_bytes, job.n_slots);
  if (rc != CALVO_OK) return rc;
  const int64_t nck_l3 = job.chunk_ready ? (max_blocks + job.chunk_blocks - 1) / job.chunk_blocks : 0;
  for (int l = layer_begin; l < layer_end; l++)
    while ((int64_t)c->ev_chunk[l].size() < nck_l3) {         // the loader records them, this thread makes them
      hipEvent_t ev = nullptr;
      HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
      c->ev_chunk[l].push_back(ev);
    }
  {
    std::lock_guard<std::mutex> lk(c->mu);
    for (int l = layer_begin; l < layer_end; l++) {
      c->layer_pending[l] = 1;
      c->layer_issued[l] = 0;
      c->chunk_blocks[l] = job.chunk_ready ? (int32_t)job.chunk_blocks : 0;
      c->n_chunks[l] = (int32_t)nck_l3;
      c->chunks_issued[l] = 0;
    }
    c->l3_status = CALVO_OK;
    c->l3_err.clear();
  }
  try {
    c->loader = std::thread(loader_main, c, std::move(job));
  } catch (...) {
    std::lock_guard<std::mutex> lk(c->mu);
    for (int l = layer_begin; l < layer_end; l++) c->layer_pending[l] = 0;
    return fail(CALVO_ENOMEM, "cannot start the loader thread");
  }
  c->loader_started = true;
  return CALVO_OK;
}

int calvo_l3_wait(calvo_ctx* c, calvo_l3_stats* stats) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  const int rc = join_loader(c);
  if (stats) {
    std::lock_guard<std::mutex> lk(c->mu);
    *stats = c->l3_stats;
  }
  return rc;
}

int calvo_layer_event(calvo_ctx* c, int layer, int mode, void* stream) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  if (mode != CALVO_EV_QUERY && mode != CALVO_EV_HOST_WAIT && mode != CALVO_EV_STREAM_WAIT)
    return fail(CALVO_EINVAL, "unknown mode %d", mode);
  if (mode == CALVO_EV_QUERY) {
    std::unique_lock<std::mutex> lk(c->mu);
    if (c->layer_pending[layer]) {
      if (c->l3_status != CALVO_OK) { lk.unlock(); return join_loader(c); }
      return fail(CALVO_ENOTREADY, "layer %d is still loading", layer);
    }
  } else {
    const int rc = wait_handed_over(c, layer);
    if (rc != CALVO_OK) return rc;
  }
  if (!layer_is_issued(c, layer)) return CALVO_OK;
  if (mode == CALVO_EV_QUERY) {
    hipError_t e = hipEventQuery(c->ev_layer[layer]);
    if (e == hipSuccess) return CALVO_OK;
    if (e == hipErrorNotReady) { (void)hipGetLastError(); return fail(CALVO_ENOTREADY, "layer %d is still loading", layer); }
    return fail_hip(e, "hipEventQuery");
  }
  if (mode == CALVO_EV_HOST_WAIT) {
    HIP_TRY(hipEventSynchronize(c->ev_layer[layer]));
    return CALVO_OK;
  }
  hipStream_t s = stream ? (hipStream_t)stream : c->s_compute;
  HIP_TRY(hipStreamWaitEvent(s, c->ev_layer[layer], 0));
  return CALVO_OK;
}

}  // extern "C"

namespace {

// What one attention call launches for a batch: decided on the host from the batch's lengths (and, for
// a layer loaded in chunks, from the chunk size), together with the descriptor words the kernels read.
struct AttnPlan {
  bool mfma = false;
  int HW = 1, variant = 0, tile_tokens = 1;
  int n_reqs = 0, total = 0;            // requests, suffix tokens over all of them
  bool chunked = false;
  int nck = 0;
  PlanItems plan;
  std::vector<int32_t> blob;
  BlobLayout lay;
  size_t part_need = 0;                 // split-KV partial-result slots the launch writes
};

// Argument checks of an attention call that do not depend on the layer.  *total = suffix tokens.
int check_batch_args(const calvo_ctx* c, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, int* total) {
  std::vector<char> seen;
  int rc = validate_requests(c, reqs, n_reqs, false, seen);
  if (rc != CALVO_OK) return rc;
  if (n_reqs > 0 && !cu_suffix) return fail(CALVO_EINVAL, "cu_suffix is NULL");
  if (n_reqs > 0 && cu_suffix[0] != 0) return fail(CALVO_EINVAL, "cu_suffix[0] must be 0");
  for (int r = 0; r < n_reqs; r++)
    if (cu_suffix[r + 1] - cu_suffix[r] != reqs[r].suffix_len)
      return fail(CALVO_EINVAL, "cu_suffix[%d+1]-cu_suffix[%d] != suffix_len of request %d", r, r, r);
  *total = n_reqs > 0 ? cu_suffix[n_reqs] : 0;
  return CALVO_OK;
}

int check_pointer_args(const void* q, const void* k_suffix, const void* v_suffix, const void* out, int total) {
  if ((k_suffix == nullptr) != (v_suffix == nullptr))
    return fail(CALVO_EINVAL, "k_suffix and v_suffix must both be given or both be NULL");
  if (total > 0) {
    if (!q || !out) return fail(CALVO_EINVAL, "q or out is NULL");
    if ((((uintptr_t)q | (uintptr_t)out | (uintptr_t)k_suffix | (uintptr_t)v_suffix) & 15) != 0)
      return fail(CALVO_EINVAL, "q, out, k_suffix and v_suffix must be 16-byte aligned");
  }
  return CALVO_OK;
}

// cb > 0: the layer was loaded in nck chunks of cb block indices and attention follows the chunks.
void make_attn_plan(calvo_ctx* c, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, int total, int cb,
                    int nck, AttnPlan& ap) {
  const calvo_config& cf = c->cfg;
  ap.n_reqs = n_reqs;
  ap.total = total;
  ap.mfma = cf.dtype == CALVO_BF16 && cf.head_dim == 128;
  ap.HW = attn_heads_per_wg(cf.n_q_heads, cf.n_kv_heads);
  ap.variant = 0;
  std::vector<int32_t> pblocks(n_reqs), slens(n_reqs);
  for (int r = 0; r < n_reqs; r++) { pblocks[r] = reqs[r].n_prefix_blocks; slens[r] = reqs[r].suffix_len; }
  if (ap.mfma) ap.variant = attn_mfma_choose(slens.data(), n_reqs, ap.HW);
  ap.tile_tokens = ap.mfma ? attn_mfma_tile_tokens(ap.variant, ap.HW) : 1;
  // Work items: tiles of suffix tokens, heaviest first, each possibly cut into split-KV pieces
  // (consecutive work items) that the merge kernel combines; see attn_plan.cpp.
  ap.chunked = ap.mfma && cb > 0 && !c->force_splits;
  ap.nck = nck;
  ap.plan = PlanItems();
  if (ap.mfma) {
    const std::vector<PlanTile> tiles = plan_tiles(pblocks.data(), slens.data(), n_reqs, ap.tile_tokens);
    const PlanParams pp{cf.n_q_heads / ap.HW, c->n_cus * (8 / attn_mfma_waves_per_wg(ap.variant)), c->split_min, c->split_fill,
                        c->force_splits};
    if (ap.chunked) {
      ap.plan = plan_items_chunked(tiles, pblocks.data(), cb, nck);
    } else {
      // the decision (a replay of the launch, attn_plan.cpp) depends only on the batch's lengths and
      // is kept for the following layers
      std::vector<int64_t> key;
      key.reserve(2 * n_reqs + 1);
      key.push_back(ap.variant);
      for (int r = 0; r < n_reqs; r++) { key.push_back(reqs[r].n_prefix_blocks); key.push_back(reqs[r].suffix_len); }
      int want = 1;
      if (!c->force_splits && key == c->plan_key) want = c->plan_want;
      else {
        want = plan_pieces(tiles, pp);
        if (!c->force_splits) { c->plan_key = key; c->plan_want = want; }
      }
      ap.plan = plan_items(tiles, want, pp);
    }
  }
  ap.lay = build_descriptor_blob(c, reqs, n_reqs, cu_suffix, ap.plan, ap.blob);
  ap.part_need = ap.plan.split_tiles.empty()
                     ? 0
                     : ap.plan.items.size() * (size_t)(cf.n_q_heads / ap.HW) * (size_t)attn_mfma_waves_per_wg(ap.variant);
}

hipError_t launch_attn(int variant, const AttnParams& p, hipStream_t stream) {
  return variant == kAttnDuo ? launch_attn_duo(p, stream) : launch_attn_pipe(p, stream);
}

// Queues the suffix append and the attention of one layer on the compute stream.  d_att: the device
// copy of ap.blob.  ready: NULL = the layer's own loading state decides what the stream waits for.
int launch_layer(calvo_ctx* c, int layer, const void* q, const void* k_suffix, const void* v_suffix, void* out, float scale,
                 const AttnPlan& ap, const int32_t* d_att, float* part_o, float* part_ml, hipEvent_t ready) {
  const calvo_config& cf = c->cfg;
  int rc;
  if (ready) {
    HIP_TRY(hipStreamWaitEvent(c->s_compute, ready, 0));   // the caller's own signal for this layer's blocks
  } else if (!ap.chunked) {
    rc = wait_handed_over(c, layer);        // a running L3 loader: until the layer's last chunk is queued
    if (rc != CALVO_OK) return rc;
    // chunk-granular launches wait for their own chunk; everything else for the whole layer.  The
    // suffix rows go to slots no load writes, so they may be stored before the layer is in.
    if (layer_is_issued(c, layer)) HIP_TRY(hipStreamWaitEvent(c->s_compute, c->ev_layer[layer], 0));
  }
  unsigned char* pool_layer = (unsigned char*)cf.pool + (int64_t)layer * c->layer_bytes;
  const ReqDesc* d_reqs = (const ReqDesc*)d_att;
  const int32_t* d_tables = d_att + ap.lay.tables_off;

  if (k_suffix) {
    AppendParams app{};
    app.k_suffix = k_suffix; app.v_suffix = v_suffix; app.pool_layer = pool_layer;
    app.reqs = d_reqs; app.tables = d_tables; app.n_reqs = ap.n_reqs; app.total_tokens = ap.total;
    app.row_chunks = (int32_t)((size_t)cf.n_kv_heads * cf.head_dim * c->elt / 16);
    HIP_TRY(launch_suffix_append(app, c->s_compute));
  }

  AttnParams p{};
  p.q = q; p.out = out; p.pool_layer = pool_layer;
  p.reqs = d_reqs; p.items = (const WorkItem*)(d_att + ap.lay.items_off); p.tables = d_tables;
  p.blk_offs = (const int64_t*)(d_att + ap.lay.offs_off);
  p.n_q_heads = cf.n_q_heads; p.n_kv_heads = cf.n_kv_heads; p.head_dim = cf.head_dim;
  p.heads_per_wg = ap.HW; p.tile_tokens = ap.tile_tokens;
  p.waves_per_wg = attn_mfma_waves_per_wg(ap.variant);
  p.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)cf.head_dim);
  HIP_TRY(hipEventRecord(c->ev_t0[layer], c->s_compute));
  if (ap.mfma) {
    p.part_o = part_o;
    p.part_ml = part_ml;
    const auto& groups = ap.plan.groups;
    if (ap.chunked) {
      for (size_t g = 0; g < groups.size(); g++) {
        // a device-side wait needs a recorded event: with a loader running, this thread follows it chunk by chunk
        if (g < (size_t)ap.nck) {
          if ((rc = wait_chunk_handed_over(c, layer, (int)g)) != CALVO_OK) return rc;
          HIP_TRY(hipStreamWaitEvent(c->s_compute, c->ev_chunk[layer][g], 0));
        } else {
          if ((rc = wait_handed_over(c, layer)) != CALVO_OK) return rc;
          if (layer_is_issued(c, layer)) HIP_TRY(hipStreamWaitEvent(c->s_compute, c->ev_layer[layer], 0));
        }
        if (groups[g].empty()) continue;
        p.n_items = (int32_t)groups[g].size();
        p.item_index = d_att + ap.lay.group_off[g];
        HIP_TRY(launch_attn(ap.variant, p, c->s_compute));
      }
      p.item_index = nullptr;
    } else {
      p.n_items = (int32_t)ap.plan.items.size();
      HIP_TRY(launch_attn(ap.variant, p, c->s_compute));
    }
    HIP_TRY(launch_merge_splits(p, d_att + ap.lay.split_off, (int)ap.plan.split_tiles.size(), c->s_compute));
  } else {
    p.n_items = ap.n_reqs;
    HIP_TRY(launch_attn_simple(p, cf.dtype, ap.total, c->s_compute));
  }
  HIP_TRY(hipEventRecord(c->ev_t1[layer], c->s_compute));
  c->timed[layer] = 1;
  c->last_variant[layer] = ap.mfma ? ap.variant : -1;
  c->last_wgs[layer] = ap.mfma ? (int32_t)(ap.plan.items.size() * (size_t)(cf.n_q_heads / ap.HW)) : 0;
  return CALVO_OK;
}

}  // namespace

// A batch whose requests were validated, planned and described to the device once
// (calvo_batch_prepare): the per-layer call then only queues its launches.
struct PreparedPlan {
  AttnPlan ap;
  int32_t* d_blob = nullptr;                  // device copy of ap.blob (owned)
  int32_t* h_blob = nullptr;                  // its pinned source (read when the compute stream gets to the upload)
  size_t blob_bytes = 0;                      // capacity of both
};

struct calvo_batch {
  calvo_ctx* c = nullptr;
  std::vector<std::vector<int32_t>> tables;   // copies of the block tables
  std::vector<calvo_request> reqs;            // block_table points into `tables`
  std::vector<int32_t> cu;
  PreparedPlan whole;                         // the launch for a layer loaded as a whole
  // launches that follow a layer's chunks, made at the first such layer and kept: key = (chunk size in
  // blocks, number of chunks)
  std::vector<std::pair<std::pair<int, int>, PreparedPlan*>> chunked;
};

namespace {

// device + pinned copies of pp.ap.blob, upload queued on the compute stream
int upload_prepared(calvo_ctx* c, PreparedPlan& pp) {
  const size_t bytes = std::max<size_t>(pp.ap.blob.size(), 4) * 4;
  {
    // the smallest buffer pair that was given back and is large enough
    std::lock_guard<std::mutex> lk(c->blob_mu);
    int best = -1;
    for (int i = 0; i < (int)c->blob_free.size(); i++)
      if (c->blob_free[i].bytes >= bytes && (best < 0 || c->blob_free[i].bytes < c->blob_free[best].bytes)) best = i;
    if (best >= 0) {
      pp.d_blob = c->blob_free[best].d; pp.h_blob = c->blob_free[best].h; pp.blob_bytes = c->blob_free[best].bytes;
      c->blob_free.erase(c->blob_free.begin() + best);
    }
  }
  if (!pp.d_blob) {
    const size_t cap = (bytes + 65535) / 65536 * 65536;
    HIP_TRY(hipMalloc((void**)&pp.d_blob, cap));
    HIP_TRY(hipHostMalloc((void**)&pp.h_blob, cap, hipHostMallocDefault));
    pp.blob_bytes = cap;
  }
  if (pp.ap.part_need) {
    const int rc = ensure_partials(c, pp.ap.part_need);
    if (rc != CALVO_OK) return rc;
  }
  memcpy(pp.h_blob, pp.ap.blob.data(), pp.ap.blob.size() * 4);
  HIP_TRY(hipMemcpyAsync(pp.d_blob, pp.h_blob, pp.ap.blob.size() * 4, hipMemcpyHostToDevice, c->s_compute));
  return CALVO_OK;
}

// The launches that read the buffers have finished (or were never queued).
void free_prepared(calvo_ctx* c, PreparedPlan& pp) {
  constexpr size_t kKeep = 64;
  bool kept = false;
  if (c && pp.d_blob && pp.h_blob) {
    std::lock_guard<std::mutex> lk(c->blob_mu);
    if (c->blob_free.size() < kKeep) { c->blob_free.push_back({pp.d_blob, pp.h_blob, pp.blob_bytes}); kept = true; }
  }
  if (!kept) {
    if (pp.d_blob) (void)hipFree(pp.d_blob);
    if (pp.h_blob) (void)hipHostFree(pp.h_blob);
  }
  pp.d_blob = pp.h_blob = nullptr;
  pp.blob_bytes = 0;
}

}  // namespace

// use_static: descriptors and split-KV partial results go to this device's file-scope array and
// nothing is allocated (calvo_prefill_attn_noalloc); otherwise to buffers the context grows on demand.
int calvo::host::prefill_attn_impl(calvo_ctx* c, int layer, const void* q, const void* k_suffix, const void* v_suffix, void* out,
                                   const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, float scale, bool use_static,
                                   hipEvent_t ready) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  int total = 0;
  int rc = check_batch_args(c, reqs, n_reqs, cu_suffix, &total);
  if (rc != CALVO_OK) return rc;
  rc = check_pointer_args(q, k_suffix, v_suffix, out, total);
  if (rc != CALVO_OK) return rc;
  if (total == 0) {
    // nothing to compute; still order the compute stream after the layer's ingest
    if (ready) { HIP_TRY(hipStreamWaitEvent(c->s_compute, ready, 0)); return CALVO_OK; }
    rc = wait_handed_over(c, layer);
    if (rc != CALVO_OK) return rc;
    if (layer_is_issued(c, layer)) HIP_TRY(hipStreamWaitEvent(c->s_compute, c->ev_layer[layer], 0));
    return CALVO_OK;
  }
  int cb = 0, nck = 0;
  if (!ready) {      // a layer loaded in chunks: attention follows the chunks, one launch behind each chunk's event
    std::lock_guard<std::mutex> lk(c->mu);
    cb = c->chunk_blocks[layer];
    nck = c->n_chunks[layer];
  }
  AttnPlan ap;
  make_attn_plan(c, reqs, n_reqs, cu_suffix, total, cb, nck, ap);
  const std::vector<int32_t>& blob = ap.blob;

  int32_t* d_att = c->d_att;
  float *part_o = c->part_o, *part_ml = c->part_ml;
  if (use_static) {
    // fixed capacity, no allocation: the array is shared by every call on this GPU, so its
    // descriptors are uploaded on every call (another context may have used it in between)
    if (blob.size() > kStaticBlobInts)
      return fail(CALVO_ENOMEM, "calvo_prefill_attn_noalloc: the batch needs %zu descriptor words, the static array holds %zu "
                  "(use calvo_prefill_attn)", blob.size(), kStaticBlobInts);
    if (ap.part_need > kStaticPartSlots)
      return fail(CALVO_ENOMEM, "calvo_prefill_attn_noalloc: the launch needs %zu partial-result slots, the static array holds %zu "
                  "(use calvo_prefill_attn)", ap.part_need, kStaticPartSlots);
    d_att = (int32_t*)c->d_static;
    part_o = (float*)(c->d_static + kStaticBlobBytes);
    part_ml = (float*)(c->d_static + kStaticBlobBytes + kStaticPartOBytes);
    const int k = (c->static_cur + 1) % calvo_ctx::kShadows;
    if (c->static_pending[k]) { HIP_TRY(hipEventSynchronize(c->ev_static[k])); c->static_pending[k] = false; }
    memcpy(c->h_static[k], blob.data(), blob.size() * 4);
    HIP_TRY(hipMemcpyAsync(d_att, c->h_static[k], blob.size() * 4, hipMemcpyHostToDevice, c->s_compute));
    HIP_TRY(hipEventRecord(c->ev_static[k], c->s_compute));
    c->static_pending[k] = true;
    c->static_cur = k;
  } else {
    rc = ensure_att_blob(c, blob.size());
    if (rc != CALVO_OK) return rc;
    if (ap.part_need) {
      rc = ensure_partials(c, ap.part_need);
      if (rc != CALVO_OK) return rc;
    }
    d_att = c->d_att;
    part_o = c->part_o;
    part_ml = c->part_ml;
    const bool same = c->att_len == blob.size() && memcmp(c->h_att[c->att_cur], blob.data(), blob.size() * 4) == 0;
    if (!same) {
      const int k = (c->att_cur + 1) % calvo_ctx::kShadows;      // the shadow whose upload is the oldest
      if (c->att_pending[k]) { HIP_TRY(hipEventSynchronize(c->ev_att[k])); c->att_pending[k] = false; }
      c->att_len = 0;                       // the device copy is unknown until the transfer is queued
      memcpy(c->h_att[k], blob.data(), blob.size() * 4);
      HIP_TRY(hipMemcpyAsync(c->d_att, c->h_att[k], blob.size() * 4, hipMemcpyHostToDevice, c->s_compute));
      c->att_cur = k;
      c->att_len = blob.size();
      HIP_TRY(hipEventRecord(c->ev_att[k], c->s_compute));
      c->att_pending[k] = true;
    }
  }
  return launch_layer(c, layer, q, k_suffix, v_suffix, out, scale, ap, d_att, part_o, part_ml, ready);
}

int calvo::host::prefill_attn_prepared(calvo_batch* b, int layer, const void* q, const void* k_suffix, const void* v_suffix,
                                       void* out, float scale, hipEvent_t ready) {
  if (!b || !b->c) return fail(CALVO_EINVAL, "batch is NULL");
  calvo_ctx* c = b->c;
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  int rc = check_pointer_args(q, k_suffix, v_suffix, out, b->whole.ap.total);
  if (rc != CALVO_OK) return rc;
  PreparedPlan* pp = &b->whole;
  if (!ready && b->whole.ap.total > 0) {
    // a layer that was loaded in chunks gets the launches that follow its chunks: planned and
    // uploaded the first time that chunking is seen, kept for the other layers and steps
    int cb = 0, nck = 0;
    {
      std::lock_guard<std::mutex> lk(c->mu);
      cb = c->chunk_blocks[layer];
      nck = c->n_chunks[layer];
    }
    if (cb > 0 && b->whole.ap.mfma && !c->force_splits) {
      pp = nullptr;
      for (auto& e : b->chunked)
        if (e.first == std::make_pair(cb, nck)) pp = e.second;
      if (!pp) {
        pp = new (std::nothrow) PreparedPlan();
        if (!pp) return fail(CALVO_ENOMEM, "out of host memory");
        make_attn_plan(c, b->reqs.data(), (int)b->reqs.size(), b->cu.data(), b->whole.ap.total, cb, nck, pp->ap);
        rc = upload_prepared(c, *pp);
        if (rc != CALVO_OK) { free_prepared(c, *pp); delete pp; return rc; }
        b->chunked.push_back({{cb, nck}, pp});
      }
    }
  }
  if (b->whole.ap.total == 0) {
    if (ready) { HIP_TRY(hipStreamWaitEvent(c->s_compute, ready, 0)); return CALVO_OK; }
    rc = wait_handed_over(c, layer);
    if (rc != CALVO_OK) return rc;
    if (layer_is_issued(c, layer)) HIP_TRY(hipStreamWaitEvent(c->s_compute, c->ev_layer[layer], 0));
    return CALVO_OK;
  }
  return launch_layer(c, layer, q, k_suffix, v_suffix, out, scale, pp->ap, pp->d_blob, c->part_o, c->part_ml, ready);
}

void calvo::host::batch_free_completed(calvo_batch* b) {
  if (!b) return;
  free_prepared(b->c, b->whole);
  for (auto& e2 : b->chunked) { free_prepared(b->c, *e2.second); delete e2.second; }
  delete b;
}

extern "C" {

int calvo_batch_prepare(calvo_ctx* c, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, calvo_batch** out) {
  if (!out) return fail(CALVO_EINVAL, "out is NULL");
  *out = nullptr;
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  int total = 0;
  int rc = check_batch_args(c, reqs, n_reqs, cu_suffix, &total);
  if (rc != CALVO_OK) return rc;
  calvo_batch* b = new (std::nothrow) calvo_batch();
  if (!b) return fail(CALVO_ENOMEM, "out of host memory");
  b->c = c;
  b->tables.resize((size_t)n_reqs);
  b->reqs.assign(reqs, reqs + n_reqs);
  for (int r = 0; r < n_reqs; r++) {
    const int64_t nt = (int64_t)reqs[r].n_prefix_blocks + (reqs[r].suffix_len + kBlockTokens - 1) / kBlockTokens;
    b->tables[r].assign(reqs[r].block_table, reqs[r].block_table + nt);
    b->reqs[r].block_table = b->tables[r].data();
  }
  b->cu.assign(cu_suffix, cu_suffix + (n_reqs > 0 ? n_reqs + 1 : 0));
  if (n_reqs == 0) b->cu.assign(1, 0);
  make_attn_plan(c, b->reqs.data(), n_reqs, b->cu.data(), total, 0, 0, b->whole.ap);
  rc = upload_prepared(c, b->whole);
  if (rc != CALVO_OK) {
    const std::string msg = calvo_last_error();
    (void)calvo_batch_destroy(b);
    return fail(rc, "%s", msg.c_str());
  }
  *out = b;
  return CALVO_OK;
}

int calvo_batch_destroy(calvo_batch* b) {
  if (!b) return fail(CALVO_EINVAL, "batch is NULL");
  hipError_t e = hipSuccess;
  if (b->c && b->c->s_compute) e = hipStreamSynchronize(b->c->s_compute);   // launches that read its descriptors
  batch_free_completed(b);
  if (e != hipSuccess) return fail_hip(e, "synchronize at calvo_batch_destroy");
  return CALVO_OK;
}

int calvo_prefill_attn_batch(calvo_ctx* c, calvo_batch* b, int layer, const void* q, const void* k_suffix, const void* v_suffix,
                             void* out, float scale) {
  if (!c || !b || b->c != c) return fail(CALVO_EINVAL, "batch does not belong to this context");
  return prefill_attn_prepared(b, layer, q, k_suffix, v_suffix, out, scale, nullptr);
}

int calvo_prefill_attn(calvo_ctx* c, int layer, const void* q, const void* k_suffix, const void* v_suffix, void* out,
                       const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, float scale) {
  return prefill_attn_impl(c, layer, q, k_suffix, v_suffix, out, reqs, n_reqs, cu_suffix, scale, false, nullptr);
}

int calvo_prefill_attn_noalloc(calvo_ctx* c, int layer, const void* q, const void* k_suffix, const void* v_suffix, void* out,
                               const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, float scale) {
  return prefill_attn_impl(c, layer, q, k_suffix, v_suffix, out, reqs, n_reqs, cu_suffix, scale, true, nullptr);
}

int calvo_attn_kernel_info(calvo_ctx* c, int layer, int* kernel, int* n_workgroups) {
  if (!c) return fail(CALVO_EINVAL, "ctx is NULL");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  if (!c->timed[layer]) return fail(CALVO_ENOTREADY, "no attention kernel was queued for layer %d", layer);
  if (kernel) *kernel = c->last_variant[layer];
  if (n_workgroups) *n_workgroups = c->last_wgs[layer];
  return CALVO_OK;
}

int calvo_attn_kernel_ms(calvo_ctx* c, int layer, float* ms) {
  if (!c || !ms) return fail(CALVO_EINVAL, "NULL argument");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(CALVO_EINVAL, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  if (!c->timed[layer]) return fail(CALVO_ENOTREADY, "no attention kernel was queued for layer %d", layer);
  HIP_TRY(hipEventSynchronize(c->ev_t1[layer]));
  HIP_TRY(hipEventElapsedTime(ms, c->ev_t0[layer], c->ev_t1[layer]));
  return CALVO_OK;
}

}  // extern "C"
