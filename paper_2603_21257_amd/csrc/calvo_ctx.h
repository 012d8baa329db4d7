// The context of libcalvo as its host-side translation units see it (calvo_api.hip: loading and
// attention calls; calvo_dispatch.hip: the multi-request dispatcher), and the helpers they share.
// Not part of the public ABI (see include/calvo.h).
#pragma once
#include <condition_variable>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/calvo.h"
#include "calvo_internal.h"

struct calvo_ctx {
  calvo_config cfg{};
  size_t elt = 0, blk_bytes = 0;
  int64_t layer_bytes = 0;
  int n_staging = 0, n_copy = 0;
  int64_t staging_blocks = 0;
  hipStream_t s_copy[1] = {nullptr};
  hipStream_t s_scatter = nullptr;
  hipStream_t s_compute = nullptr;
  bool own_compute = false;
  std::vector<void*> staging;
  std::vector<hipEvent_t> ev_filled, ev_free;
  std::vector<char> free_recorded;
  uint64_t seq = 0;
  std::vector<hipEvent_t> ev_layer;
  std::vector<char> layer_issued;
  // chunk-granular readiness: layer l was loaded in pieces of chunk_blocks[l] block indices
  // (0 = as a whole); ev_chunk[l][k] fires when blocks [0, (k+1) * chunk_blocks[l]) of every
  // request are resident
  std::vector<int32_t> chunk_blocks;
  std::vector<int32_t> n_chunks;
  std::vector<int32_t> chunks_issued;   // chunk events recorded so far (a running loader records them one by one; guarded by mu)
  std::vector<std::vector<hipEvent_t>> ev_chunk;
  // ingest-side table copy (device) and its pinned shadow
  int32_t* d_tab_ing = nullptr;
  int32_t* h_tab_ing = nullptr;
  size_t tab_ing_cap = 0;
  hipEvent_t ev_tab_ing = nullptr;
  bool tab_ing_pending = false;
  // attention-side descriptor blob: [ReqDesc x n][WorkItem x m][tables]
  int32_t* d_att = nullptr;
  // its pinned shadows: an upload reads its shadow when the compute stream gets to it, so a batch that
  // differs from the previous one takes the next shadow instead of waiting for that upload (several
  // requests can be queued on the compute stream without the calling thread blocking)
  static constexpr int kShadows = 4;
  int32_t* h_att[kShadows] = {nullptr, nullptr, nullptr, nullptr};
  size_t att_cap = 0;     // in int32
  size_t att_len = 0;     // valid int32 in shadow att_cur == on device
  int att_cur = 0;
  hipEvent_t ev_att[kShadows] = {nullptr, nullptr, nullptr, nullptr};
  bool att_pending[kShadows] = {false, false, false, false};
  std::vector<hipEvent_t> ev_t0, ev_t1;
  std::vector<char> timed;
  std::vector<int32_t> last_variant, last_wgs;   // per layer: attention kernel chosen, workgroups launched
  int scatter_grid = 64;
  size_t merge_bytes = (size_t)256 << 20;   // consecutive small layers cross PCIe together up to this size (CALVO_MERGE_MIB)
  int force_splits = 0;           // CALVO_ATTN_SPLITS: pieces per tile (0 = automatic)
  int split_min = 48;             // shortest piece of a cut tile, in 32-key sub-tiles
  int split_fill = 30;            // cost of a workgroup's pipeline fill and drain, in sub-tile steps (launch replay)
  int n_cus = 256;                // compute units of the device
  std::vector<int64_t> plan_key;  // lengths of the batch the cached decision belongs to
  int plan_want = 1;
  float* part_o = nullptr;        // split-KV partial results (compute stream only)
  float* part_ml = nullptr;
  size_t part_slots = 0;          // capacity in (work item, head group, wave) slots
  int device = 0;
  // test hooks (environment, read by calvo_create): the host sleeps this long before it queues each
  // transfer of the L2 -> L1 stage (makes the loading stage the slow one without touching the
  // device); the L3 loader reports a failure instead of moving chunk number test_l3_fail_chunk
  int test_ingest_delay_us = 0;
  int test_scatter_delay_us = 0;     // a delay kernel in front of every scatter: the scatter becomes the slow stage
  int test_l3_fail_chunk = -1;
  // ---- calvo_prefill_attn_noalloc: this device's static array and pinned shadows of fixed size
  // (made by calvo_create) for the descriptor uploads
  unsigned char* d_static = nullptr;
  int32_t* h_static[kShadows] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t ev_static[kShadows] = {nullptr, nullptr, nullptr, nullptr};
  bool static_pending[kShadows] = {false, false, false, false};
  int static_cur = 0;
  // ---- emulated L3 -> L2 stage: a loader thread, a ring of pinned buffers, and the hand-over
  // state it shares with the calling thread (layer_issued, l3_*: guarded by mu)
  std::mutex mu;
  std::condition_variable cv;
  std::thread loader;
  bool loader_started = false;
  std::vector<char> layer_pending;           // layers a running loader will still hand over
  int l3_status = CALVO_OK;
  std::string l3_err;
  calvo_l3_stats l3_stats{};
  // descriptor buffers of prepared batches that have been given back, kept for the next batch: a
  // device free waits for the whole device, which a serving loop cannot afford per request
  struct BlobBuf { int32_t* d; int32_t* h; size_t bytes; };
  std::mutex blob_mu;
  std::vector<BlobBuf> blob_free;
  std::vector<void*> l2_ring;
  std::vector<hipEvent_t> ev_l2_free;
  std::vector<char> l2_free_recorded;
  size_t l2_slot_bytes = 0;
};

namespace calvo {
namespace host {

// status + thread-local message (calvo_last_error)
int fail(int code, const char* fmt, ...);
int fail_hip(hipError_t e, const char* what);

#define HIP_TRY(expr)                                               \
  do {                                                              \
    hipError_t e_ = (expr);                                         \
    if (e_ != hipSuccess) return ::calvo::host::fail_hip(e_, #expr); \
  } while (0)

// Checks shared by loading and attention.  Nothing is queued before these pass.
int validate_requests(const calvo_ctx* c, const calvo_request* reqs, int n_reqs, bool need_host, std::vector<char>& seen);

// L2->L1 for nb consecutive blocks (nb <= staging_blocks) that sit in page-locked host memory: copy
// engine into the next device staging buffer, then scatter into the pool through the device table.
// If done is given it is recorded on the copy stream right after the transfer (the source may be
// overwritten once it fires).  One thread at a time.
hipError_t enqueue_staged(calvo_ctx* c, const unsigned char* pinned_src, unsigned char* pool_layer,
                          const int32_t* d_table, int64_t nb, hipEvent_t done);

// n slot ids -> the context's device-side loading table (queued on the scatter stream, in order with
// the scatters that use the previous contents).  The device copy starts at c->d_tab_ing.
int upload_ingest_table(calvo_ctx* c, const int32_t* slots, size_t n);

// the pinned ring of the emulated L3 -> L2 stage: at least n_slots buffers of slot_bytes
int ensure_l2_ring(calvo_ctx* c, size_t slot_bytes, int n_slots);

void parallel_copy(unsigned char* dst, const unsigned char* src, size_t n, int n_threads);

// The compute stage of one layer.  use_static: descriptors and partial results in the static device
// array (calvo_prefill_attn_noalloc).  ready: NULL = wait for the layer's own loading state (events of
// the most recent loading call); otherwise the compute stream waits for this event and the context's
// per-layer loading state is not consulted (the dispatcher keeps one event set per job).
int prefill_attn_impl(calvo_ctx* c, int layer, const void* q, const void* k_suffix, const void* v_suffix, void* out,
                      const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, float scale, bool use_static,
                      hipEvent_t ready);

// The same for a batch prepared with calvo_batch_prepare: no validation, planning or upload per call.
int prefill_attn_prepared(calvo_batch* b, int layer, const void* q, const void* k_suffix, const void* v_suffix, void* out,
                          float scale, hipEvent_t ready);

// Frees a prepared batch whose launches are known to have finished (no wait for the compute stream).
void batch_free_completed(calvo_batch* b);

}  // namespace host
}  // namespace calvo
