// Host side of the library: context, expert images, per-layer LRU cache with
// demand loads and prefetch on a side stream, the cache-size planner, and the
// C entry points declared in include/adapmoe.h.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/adapmoe.h"
#include "launch.h"

using namespace adapmoe;

namespace {

struct Slot {
  char* dev = nullptr;
  hipEvent_t copy_done = nullptr;  // recorded on the side stream after the copy into the slot
  hipEvent_t read_done = nullptr;  // recorded on the compute stream after the last FFN reading the slot
  bool copy_pending = false;       // a copy was issued and no compute stream has been told to wait for it yet
  bool was_read = false;
  std::vector<hipEvent_t> tile_done;  // tile-wise copies: one event per tile, in transfer order (created on first use)
  bool tiled = false;              // the last copy into the slot was issued tile by tile
  uint64_t copy_seq = 0;           // position of the last copy in the side stream's order
  uint64_t stage_seq = 0;          // staged copies: number of the request that fills the slot (0 = none)
};

struct Entry {
  int expert;
  int slot;
  bool by_prefetch;  // filled by a prefetch and not demanded since
};

struct LayerCache {
  int cap = 0;
  std::vector<Entry> order;  // front = least recently used
  // Prefetched experts that could not take one of the layer's own slots: held in spare slots
  // outside the budget until the layer's next demand (the on-demand-load model of Sec. 4.4.2
  // credits a correct prefetch whatever the layer's cache size, Eq.11-14).
  std::vector<Entry> landing;
  int find(int e) const {
    for (size_t i = 0; i < order.size(); ++i)
      if (order[i].expert == e) return (int)i;
    return -1;
  }
  int find_landing(int e) const {
    for (size_t i = 0; i < landing.size(); ++i)
      if (landing[i].expert == e) return (int)i;
    return -1;
  }
  void touch(int pos) {
    Entry en = order[pos];
    order.erase(order.begin() + pos);
    order.push_back(en);
  }
};

struct TimedLaunch {
  int cls;
  hipEvent_t t0, t1;
};

// What the demand phase of one layer step leaves for the expert FFN that follows it and for the
// end of the step (Alg.1: the compute queue of the required experts).
struct StepState {
  bool open = false;
  int layer = -1;
  std::vector<int> used_slots;                 // slots the FFN of this step reads
  std::vector<std::pair<int, int>> transient;  // (expert, slot) to drop right after the FFN
  std::vector<int> demanded;                   // experts needed by this step so far
  int rank_slot[2] = {-1, -1};                 // slot of token 0's expert of rank j (-1: caller memory)
  int k0 = 0;                                  // experts token 0 runs
  void reset(int l) {
    open = true;
    layer = l;
    used_slots.clear();
    transient.clear();
    demanded.clear();
    rank_slot[0] = rank_slot[1] = -1;
    k0 = 0;
  }
};

// Staging of expert images that live in pageable host memory (more experts than the machine lets a
// process pin): a worker thread copies each requested image into one of a few pinned buffers and
// from there to its slot on the side stream, so that the copy of image n+1 into a pinned buffer runs
// while image n crosses the link (Alg.1's transfer queue and communication stream, with the host
// copy as an extra stage).  Requests are served in order.
struct StageBuf {
  char* host = nullptr;
  hipEvent_t done = nullptr;   // the transfer out of this buffer has finished
  bool used = false;
};
struct CopyReq {
  const void* src;
  int slot;
  bool wait_read;              // the slot was read by a kernel: the transfer waits for its read_done event
};
struct Stager {
  std::thread worker;
  std::mutex mu;
  std::condition_variable cv_req, cv_done;
  std::deque<CopyReq> queue;
  bool stop = false;
  uint64_t requested = 0, issued = 0;   // requests queued so far / requests whose transfer is on the side stream
  hipError_t err = hipSuccess;
  std::vector<StageBuf> bufs;
  int next_buf = 0;
  int threads = 6;                      // host threads that share one copy into a pinned buffer
  hipEvent_t last_done = nullptr;       // done event of the latest transfer put on the side stream (the link is idle once it has fired)
  // helper threads of the worker: each copies its share of the job posted last
  std::vector<std::thread> helpers;
  std::mutex pool_mu;
  std::condition_variable pool_job, pool_done;
  char* job_dst = nullptr;
  const char* job_src = nullptr;
  size_t job_bytes = 0, job_share = 0;
  uint64_t job_gen = 0;
  int job_pending = 0;
  bool pool_stop = false;
};

}  // namespace

struct adapmoe_ctx {
  adapmoe_config cfg{};
  size_t image_bytes = 0, w2_offset = 0;
  bool bf16_act = false;
  std::vector<const void*> router;
  std::vector<float> tau;
  std::vector<const void*> host_image;  // [L*N]
  std::vector<const void*> bound;       // [L*N]
  std::vector<int> bound_count;         // [L]
  const void** d_table = nullptr;       // [L*N] device
  int32_t* d_err = nullptr;
  int32_t* d_dec = nullptr;             // ids[2B] k[B], then per look-ahead depth d = 1..3: pred_ids[2B] pred_k[B]
  int lookahead = 1;                    // layers ahead that are predicted and prefetched (Sec. 4.3)
  const void* first_pred = nullptr;     // predictive gate for layer 0 of the following token (Sec. 4.3, Eq.9), device [N,H]
  int tiles = 0;                        // > 1: expert copies are cut into tiles and a waiting FFN runs tile by tile (Alg.1)
  bool poison = false;                  // fill a slot with all-ones bytes before every copy into it (ordering check)
  Stager* stager = nullptr;             // non-null: host images are pageable and go through pinned staging buffers
  uint64_t copy_seq = 0;
  float* d_w = nullptr;                 // [B,2]
  float* d_a = nullptr;                 // [B][2][a_stride]
  ResolvedExperts* d_res = nullptr;     // [B] resolved experts of the last gate of moe_layer_step
  unsigned* d_fused_counter = nullptr;  // arrival counter of the fused kernel's grid barrier (only grows)
  unsigned fused_seq = 0;               // fused launches so far
  unsigned* d_dyn = nullptr;            // [max_B][kDynQueues * kDynStride] row counters of the gate/up GEMV's dynamic tail, zero between steps
  // batched path scratch (bf16, max_B > 1)
  int32_t* d_bkt_count = nullptr;
  int32_t* d_bkt_tok = nullptr;
  float* d_bkt_w = nullptr;
  const void** d_bkt_base = nullptr;
  int32_t* d_bkt_active = nullptr;
  uint16_t* d_xop = nullptr;
  uint16_t* d_ahi = nullptr;
  uint16_t* d_alo = nullptr;
  int32_t* h_dec = nullptr;             // pinned mirror of d_dec
  hipStream_t copy_stream = nullptr;
  LaunchCfg lc{};

  bool cache_ready = false;
  std::vector<Slot> slots;
  std::vector<int> free_slots;
  std::vector<LayerCache> layers;
  std::vector<std::pair<const void**, const void*>> pending_pokes;  // (device address, value), applied before the next FFN
  StepState step;                       // demand phase of the running layer step
  int32_t* dec_log = nullptr;           // caller's device buffer for gate decisions (tracing aid), records of 6*max_B ints
  int dec_log_cap = 0, dec_log_pos = 0;

  std::deque<adapmoe_event> trace;
  adapmoe_counters_t ctr{};
  int token = 0;
  std::string last_error;

  bool profiling = false;
  std::vector<TimedLaunch> timed;
  std::vector<hipEvent_t> event_pool;
};

namespace {

// Two fused kernels must never share the device: each keeps every compute unit
// until all of its workgroups have arrived at its barrier.  Launches on one
// stream are ordered anyway; a launch on another stream (or from another
// context) first waits for everything enqueued so far on the stream of the
// previous fused launch.
std::mutex g_fused_mu;
hipStream_t g_fused_last_stream = nullptr;
bool g_fused_any = false;
hipEvent_t g_fused_event = nullptr;

hipError_t fused_serialise(hipStream_t s) {
  std::lock_guard<std::mutex> lk(g_fused_mu);
  if (g_fused_any && g_fused_last_stream != s) {
    hipError_t e;
    if (!g_fused_event && (e = hipEventCreateWithFlags(&g_fused_event, hipEventDisableTiming)) != hipSuccess) return e;
    if ((e = hipEventRecord(g_fused_event, g_fused_last_stream)) != hipSuccess) return e;
    if ((e = hipStreamWaitEvent(s, g_fused_event, 0)) != hipSuccess) return e;
  }
  g_fused_any = true;
  g_fused_last_stream = s;
  return hipSuccess;
}

int fail(adapmoe_ctx* c, int code, const std::string& msg) {
  if (c) c->last_error = msg;
  return code;
}

#define HIPCHK(ctx, call)                                                                 \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return fail((ctx), ADAPMOE_EHIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
  } while (0)

// No exception crosses the C boundary: the containers of the context allocate, so every entry
// point that can reach an allocation runs inside this pair.
#define ABI_TRY try {
#define ABI_CATCH(ctx)                                                                     \
  }                                                                                        \
  catch (const std::bad_alloc&) {                                                          \
    return fail((ctx), ADAPMOE_ENOMEM, "host memory allocation failed");                   \
  }                                                                                        \
  catch (...) {                                                                            \
    return fail((ctx), ADAPMOE_ESTATE, "unexpected exception inside the library");         \
  }

bool cfg_ok(const adapmoe_config* c) {
  if (!c) return false;
  if (c->dtype != ADAPMOE_F32 && c->dtype != ADAPMOE_BF16 && c->dtype != ADAPMOE_INT4G64 && c->dtype != ADAPMOE_INT2G64) return false;
  const int q = c->dtype == ADAPMOE_BF16 ? 512 : 256;
  if (c->H <= 0 || c->F <= 0 || c->H % q || c->F % q) return false;
  if (c->N < 2 || c->N > 64 || c->L < 1) return false;
  if (c->dtype == ADAPMOE_INT4G64 || c->dtype == ADAPMOE_INT2G64) {
    // a lane owns one group of 64 per block of 4096: at most 2 blocks of x and 4 blocks of a in registers
    if (c->H > 8192 || c->F > 16384) return false;
  } else if ((size_t)2 * c->F * sizeof(float) > 160 * 1024) {
    return false;  // a_j of two experts must fit in LDS
  }
  return true;
}

// bytes per element of activations and of fp32/bf16 weights
size_t elem_size(int dtype) { return dtype == ADAPMOE_F32 ? 4 : 2; }

// code width of the group-quantised formats, 0 for fp32/bf16 weights
int quant_bits(int dtype) { return dtype == ADAPMOE_INT4G64 ? 4 : dtype == ADAPMOE_INT2G64 ? 2 : 0; }

// quantised image: bytes of one row of n weights (codes + fp16 scale/zero per 64)
size_t q_row_bytes(int bits, size_t n) { return n * bits / 8 + n / 16; }

// floats per (token, expert slot) of the a_j scratch
size_t a_stride_for(const adapmoe_config& c) {
  if (!quant_bits(c.dtype)) return (size_t)c.F;
  const size_t blocks = ((size_t)c.F / 64 + 63) / 64;
  return std::max((size_t)c.F, blocks * 2048);  // int4: blocks x 8 vectors x 64 lanes x 8 bf16
}

void record(adapmoe_ctx* c, int layer, int kind, int expert, int victim, int slot) {
  switch (kind) {
    case ADAPMOE_EV_HIT: c->ctr.hits++; break;
    case ADAPMOE_EV_HIT_PF: c->ctr.hits++; c->ctr.hits_after_prefetch++; break;
    case ADAPMOE_EV_MISS: c->ctr.misses++; break;
    case ADAPMOE_EV_BYPASS: c->ctr.bypasses++; break;
    case ADAPMOE_EV_PF_TOUCH: c->ctr.prefetch_touches++; break;
    case ADAPMOE_EV_PF_LOAD: c->ctr.prefetch_loads++; break;
    case ADAPMOE_EV_PF_LAND: c->ctr.prefetch_loads++; c->ctr.prefetch_landed++; break;
  }
  if (c->cfg.trace_capacity <= 0) return;
  if ((int)c->trace.size() >= c->cfg.trace_capacity) c->trace.pop_front();
  c->trace.push_back(adapmoe_event{c->token, layer, kind, expert, victim, slot});
}

// Tile-wise transfer (Sec. 5, Alg.1): the gate/up part of an image (F row pairs) is cut into
// `tiles` blocks of rows and the W2 part (H rows) into tiles/2, all of (nearly) equal size.
int gateup_tiles(const adapmoe_ctx* c) { return c->tiles; }
int down_tiles(const adapmoe_ctx* c) { return std::max(1, c->tiles / 2); }
// rows [*r0, *r1) of tile t: t < gateup_tiles counts row pairs, the others rows of W2
void tile_rows(const adapmoe_ctx* c, int t, int* r0, int* r1) {
  const int tg = gateup_tiles(c), td = down_tiles(c);
  if (t < tg) {
    *r0 = (int)((int64_t)c->cfg.F * t / tg);
    *r1 = (int)((int64_t)c->cfg.F * (t + 1) / tg);
  } else {
    *r0 = (int)((int64_t)c->cfg.H * (t - tg) / td);
    *r1 = (int)((int64_t)c->cfg.H * (t - tg + 1) / td);
  }
}
void tile_bytes(const adapmoe_ctx* c, int t, size_t* b0, size_t* b1) {
  int r0, r1;
  tile_rows(c, t, &r0, &r1);
  if (t < gateup_tiles(c)) {
    const size_t pair = c->w2_offset / (size_t)c->cfg.F;
    *b0 = pair * r0;
    *b1 = pair * r1;
  } else {
    const size_t row = (c->image_bytes - c->w2_offset) / (size_t)c->cfg.H;
    *b0 = c->w2_offset + row * r0;
    *b1 = c->w2_offset + row * r1;
  }
}

// Starts the copy of (layer, expert) into `slot` on the side stream.  The copy
// waits for the last kernel that read the slot; its completion is the slot's
// copy_done event.
int start_copy(adapmoe_ctx* c, int layer, int expert, int slot) {
  const void* src = c->host_image[(size_t)layer * c->cfg.N + expert];
  if (!src) return fail(c, ADAPMOE_ENOTREG, "expert has no registered host image");
  Slot& s = c->slots[slot];
  if (c->stager) {   // the worker thread stages the image and puts the transfer on the side stream
    Stager& st = *c->stager;
    {
      std::lock_guard<std::mutex> lk(st.mu);
      if (st.err != hipSuccess) return fail(c, ADAPMOE_EHIP, std::string("staged copy: ") + hipGetErrorString(st.err));
      st.queue.push_back(CopyReq{src, slot, s.was_read});
      s.stage_seq = ++st.requested;
    }
    st.cv_req.notify_one();
    s.tiled = false;
    s.copy_pending = true;
    s.copy_seq = ++c->copy_seq;
    c->ctr.h2d_bytes += c->image_bytes;
    return ADAPMOE_OK;
  }
  if (s.was_read) HIPCHK(c, hipStreamWaitEvent(c->copy_stream, s.read_done, 0));
  if (c->poison) HIPCHK(c, hipMemsetAsync(s.dev, 0xFF, c->image_bytes, c->copy_stream));
  s.tiled = c->tiles > 1;
  if (s.tiled) {
    // tiles in storage order: row-pair blocks of the interleaved W1/W3 part, then row blocks of W2
    const int tg = gateup_tiles(c), td = down_tiles(c);
    while ((int)s.tile_done.size() < tg + td) {
      hipEvent_t ev = nullptr;
      HIPCHK(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
      s.tile_done.push_back(ev);
    }
    for (int t = 0; t < tg + td; ++t) {
      size_t b0, b1;
      tile_bytes(c, t, &b0, &b1);
      HIPCHK(c, hipMemcpyAsync(s.dev + b0, static_cast<const char*>(src) + b0, b1 - b0, hipMemcpyHostToDevice, c->copy_stream));
      HIPCHK(c, hipEventRecord(s.tile_done[t], c->copy_stream));
    }
  } else {
    HIPCHK(c, hipMemcpyAsync(s.dev, src, c->image_bytes, hipMemcpyHostToDevice, c->copy_stream));
  }
  HIPCHK(c, hipEventRecord(s.copy_done, c->copy_stream));
  s.copy_pending = true;
  s.copy_seq = ++c->copy_seq;
  c->ctr.h2d_bytes += c->image_bytes;
  return ADAPMOE_OK;
}

// Staged copies: blocks until the worker has put the transfer into `sl` on the side stream, so that
// the slot's copy_done event stands for that transfer (an event that has not been recorded yet
// would let a waiting stream through).
int wait_issued(adapmoe_ctx* c, const Slot& sl) {
  if (!c->stager || sl.stage_seq == 0) return ADAPMOE_OK;
  Stager& st = *c->stager;
  std::unique_lock<std::mutex> lk(st.mu);
  st.cv_done.wait(lk, [&] { return st.issued >= sl.stage_seq || st.err != hipSuccess; });
  if (st.err != hipSuccess) return fail(c, ADAPMOE_EHIP, std::string("staged copy: ") + hipGetErrorString(st.err));
  return ADAPMOE_OK;
}

// Blocks until every requested staged copy is on the side stream.
int drain_stager(adapmoe_ctx* c) {
  if (!c->stager) return ADAPMOE_OK;
  Stager& st = *c->stager;
  std::unique_lock<std::mutex> lk(st.mu);
  st.cv_done.wait(lk, [&] { return st.issued >= st.requested || st.err != hipSuccess; });
  if (st.err != hipSuccess) return fail(c, ADAPMOE_EHIP, std::string("staged copy: ") + hipGetErrorString(st.err));
  return ADAPMOE_OK;
}

// Helper i copies share i + 1 of every job; the worker copies share 0 and waits for the others.
void pool_helper(Stager* st, int index) {
  uint64_t seen = 0;
  for (;;) {
    char* dst;
    const char* src;
    size_t bytes, share;
    {
      std::unique_lock<std::mutex> lk(st->pool_mu);
      st->pool_job.wait(lk, [&] { return st->pool_stop || st->job_gen != seen; });
      if (st->pool_stop) return;
      seen = st->job_gen;
      dst = st->job_dst; src = st->job_src; bytes = st->job_bytes; share = st->job_share;
    }
    const size_t off = share * (size_t)(index + 1);
    if (off < bytes) memcpy(dst + off, src + off, std::min(share, bytes - off));
    {
      std::lock_guard<std::mutex> lk(st->pool_mu);
      if (--st->job_pending == 0) st->pool_done.notify_one();
    }
  }
}

// dst[0, bytes) = src[0, bytes) by the worker and its helpers together (only the worker calls this)
void pool_copy(Stager* st, char* dst, const char* src, size_t bytes) {
  const size_t parts = st->helpers.size() + 1;
  const size_t share = ((bytes + parts - 1) / parts + 4095) & ~(size_t)4095;
  if (!st->helpers.empty()) {
    std::lock_guard<std::mutex> lk(st->pool_mu);
    st->job_dst = dst; st->job_src = src; st->job_bytes = bytes; st->job_share = share;
    st->job_pending = (int)st->helpers.size();
    ++st->job_gen;
  }
  st->pool_job.notify_all();
  memcpy(dst, src, std::min(share, bytes));
  if (!st->helpers.empty()) {
    std::unique_lock<std::mutex> lk(st->pool_mu);
    st->pool_done.wait(lk, [&] { return st->job_pending == 0; });
  }
}

// An image that finds the link idle is staged and sent in pieces, so that its first bytes cross
// the link while the rest is still being copied into the pinned buffer (a load that nothing
// overlaps would otherwise take the staging time on top of the transfer time); an image that
// queues behind another transfer is staged whole while that one is under way and sent with one
// command (every further copy command leaves the link idle for some microseconds).
constexpr size_t kStagePiece = (size_t)32 << 20;

void stager_main(adapmoe_ctx* c) {
  Stager& st = *c->stager;
  hipError_t e = hipSetDevice(c->cfg.device);
  for (;;) {
    CopyReq req;
    {
      std::unique_lock<std::mutex> lk(st.mu);
      st.cv_req.wait(lk, [&] { return st.stop || !st.queue.empty(); });
      if (st.queue.empty()) return;   // stop requested and nothing left
      req = st.queue.front();
      st.queue.pop_front();
    }
    StageBuf& b = st.bufs[st.next_buf];
    st.next_buf = (st.next_buf + 1) % (int)st.bufs.size();
    if (e == hipSuccess && b.used) e = hipEventSynchronize(b.done);   // the buffer's previous transfer has left it
    if (e == hipSuccess) {
      bool idle = true;                                                // has the latest transfer finished?
      if (st.last_done) {
        const hipError_t q = hipEventQuery(st.last_done);
        if (q == hipErrorNotReady) idle = false;
        else if (q != hipSuccess) e = q;
      }
      const size_t piece = idle ? kStagePiece : c->image_bytes;
      Slot& s = c->slots[req.slot];
      const char* src = static_cast<const char*>(req.src);
      for (size_t off = 0; off < c->image_bytes && e == hipSuccess; off += piece) {
        const size_t n = std::min(piece, c->image_bytes - off);
        pool_copy(&st, b.host + off, src + off, n);
        if (off == 0) {
          if (req.wait_read) e = hipStreamWaitEvent(c->copy_stream, s.read_done, 0);
          if (e == hipSuccess && c->poison) e = hipMemsetAsync(s.dev, 0xFF, c->image_bytes, c->copy_stream);
        }
        if (e == hipSuccess) e = hipMemcpyAsync(s.dev + off, b.host + off, n, hipMemcpyHostToDevice, c->copy_stream);
      }
      if (e == hipSuccess) e = hipEventRecord(b.done, c->copy_stream);
      if (e == hipSuccess) e = hipEventRecord(s.copy_done, c->copy_stream);
      b.used = true;
      st.last_done = b.done;
    }
    {
      std::lock_guard<std::mutex> lk(st.mu);
      st.issued++;
      if (e != hipSuccess && st.err == hipSuccess) st.err = e;
    }
    st.cv_done.notify_all();
  }
}

void stop_stager(adapmoe_ctx* c) {
  if (!c->stager) return;
  Stager& st = *c->stager;
  {
    std::lock_guard<std::mutex> lk(st.mu);
    st.stop = true;
  }
  st.cv_req.notify_all();
  if (st.worker.joinable()) st.worker.join();
  {
    std::lock_guard<std::mutex> lk(st.pool_mu);
    st.pool_stop = true;
  }
  st.pool_job.notify_all();
  for (std::thread& t : st.helpers)
    if (t.joinable()) t.join();
  hipStreamSynchronize(c->copy_stream);
  for (StageBuf& b : st.bufs) {
    if (b.host) hipHostFree(b.host);
    if (b.done) hipEventDestroy(b.done);
  }
  delete c->stager;
  c->stager = nullptr;
}

void poke_later(adapmoe_ctx* c, int layer, int expert, const void* value) {
  c->pending_pokes.emplace_back(c->d_table + (size_t)layer * c->cfg.N + expert, value);
}

// resolved pointer of (token b, rank j) for the FFN launch of the running step
void poke_resolved(adapmoe_ctx* c, int b, int j, const void* value) {
  c->pending_pokes.emplace_back(&c->d_res[b].base[j], value);
}

int flush_pokes(adapmoe_ctx* c, hipStream_t s) {
  // One launch stores up to 8 values from 8 threads, in no defined order: when an address was given
  // several values since the last flush (an expert evicted and loaded again within one step), only
  // the last one is sent.
  std::vector<std::pair<const void**, const void*>> last;
  last.reserve(c->pending_pokes.size());
  for (size_t i = 0; i < c->pending_pokes.size(); ++i) {
    bool later = false;
    for (size_t j = i + 1; j < c->pending_pokes.size() && !later; ++j) later = c->pending_pokes[j].first == c->pending_pokes[i].first;
    if (!later) last.push_back(c->pending_pokes[i]);
  }
  c->pending_pokes.clear();
  size_t i = 0;
  while (i < last.size()) {
    PokeArgs p{};
    for (p.n = 0; p.n < 8 && i < last.size(); ++p.n, ++i) {
      p.addr[p.n] = last[i].first;
      p.value[p.n] = last[i].second;
    }
    HIPCHK(c, launch_poke(p, s));
  }
  return ADAPMOE_OK;
}

// Prefetch policy for one layer (Sec. 4.3; Alg.1 transfer set), rank order.  At most as many of the
// predicted experts as the layer owns slots are refreshed in or loaded into its LRU set (a prefetch
// never evicts an expert predicted together with it); with `allow_landing` (the prediction for the
// next layer) the others are copied into spare slots outside the budget and kept until the layer's
// next demand, otherwise (deeper look-ahead) they are left out.
int prefetch_layer(adapmoe_ctx* c, int layer, const int32_t* ids, int n, bool allow_landing) {
  LayerCache& lc = c->layers[layer];
  const int N = c->cfg.N;
  int own = 0;
  for (int i = 0; i < n; ++i) {
    const int e = ids[i];
    if (e < 0 || e >= N) return fail(c, ADAPMOE_EINVAL, "prefetch: expert id out of range");
    if (c->bound[(size_t)layer * N + e]) continue;  // lives in caller memory: nothing to do
    const int lpos = lc.find_landing(e);
    if (lpos >= 0) {
      record(c, layer, ADAPMOE_EV_PF_TOUCH, e, -1, lc.landing[lpos].slot);
      continue;
    }
    const int pos = lc.find(e);
    if (own < lc.cap) {
      ++own;
      if (pos >= 0) {
        const int slot = lc.order[pos].slot;
        lc.touch(pos);
        record(c, layer, ADAPMOE_EV_PF_TOUCH, e, -1, slot);
        continue;
      }
      int victim = -1, slot;
      if ((int)lc.order.size() >= lc.cap) {
        victim = lc.order.front().expert;
        slot = lc.order.front().slot;
        lc.order.erase(lc.order.begin());
        poke_later(c, layer, victim, nullptr);
      } else {
        if (c->free_slots.empty()) return fail(c, ADAPMOE_ENOMEM, "no free cache slot");
        slot = c->free_slots.back();
        c->free_slots.pop_back();
      }
      int rc = start_copy(c, layer, e, slot);
      if (rc) return rc;
      lc.order.push_back(Entry{e, slot, true});
      poke_later(c, layer, e, c->slots[slot].dev);
      record(c, layer, ADAPMOE_EV_PF_LOAD, e, victim, slot);
      continue;
    }
    if (!allow_landing) continue;
    if (pos >= 0) {   // listed twice by the caller: on the GPU already
      const int slot = lc.order[pos].slot;
      lc.touch(pos);
      record(c, layer, ADAPMOE_EV_PF_TOUCH, e, -1, slot);
      continue;
    }
    if ((int)lc.landing.size() >= 2 * c->cfg.max_B) continue;   // one step cannot require more than 2 per token
    if (c->free_slots.empty()) return fail(c, ADAPMOE_ENOMEM, "no spare slot for a prefetched expert");
    const int slot = c->free_slots.back();
    c->free_slots.pop_back();
    int rc = start_copy(c, layer, e, slot);
    if (rc) {
      c->free_slots.push_back(slot);
      return rc;
    }
    lc.landing.push_back(Entry{e, slot, true});
    poke_later(c, layer, e, c->slots[slot].dev);
    record(c, layer, ADAPMOE_EV_PF_LAND, e, -1, slot);
  }
  return ADAPMOE_OK;
}

hipEvent_t get_event(adapmoe_ctx* c) {
  if (!c->event_pool.empty()) {
    hipEvent_t e = c->event_pool.back();
    c->event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

struct ScopedTimer {
  adapmoe_ctx* c;
  hipStream_t s;
  TimedLaunch t{};
  bool on;
  ScopedTimer(adapmoe_ctx* c_, int cls, hipStream_t s_) : c(c_), s(s_), on(c_->profiling) {
    if (!on) return;
    t.cls = cls;
    t.t0 = get_event(c);
    t.t1 = get_event(c);
    if (!t.t0 || !t.t1) { on = false; return; }
    hipEventRecord(t.t0, s);
  }
  ~ScopedTimer() {
    if (!on) return;
    hipEventRecord(t.t1, s);
    c->timed.push_back(t);
  }
};

// Launch configuration for one GEMV launch: while the context is profiling it carries a pair of
// events that the launch ties to the kernel's own dispatch (execution time as a profiler reports
// it), registered under the kernel class `cls`.
LaunchCfg timed_cfg(adapmoe_ctx* c, int cls) {
  LaunchCfg lc = c->lc;
  if (!c->profiling) return lc;
  TimedLaunch t{cls, get_event(c), get_event(c)};
  if (!t.t0 || !t.t1) {
    if (t.t0) c->event_pool.push_back(t.t0);
    if (t.t1) c->event_pool.push_back(t.t1);
    return lc;
  }
  lc.timing.start = t.t0;
  lc.timing.stop = t.t1;
  c->timed.push_back(t);
  return lc;
}

FfnArgs ffn_args(adapmoe_ctx* c, int layer, const void* x, int B, const int32_t* ids, const float* w, const int32_t* k,
                 float* y, const ResolvedExperts* res) {
  FfnArgs p{};
  p.table = c->d_table + (size_t)layer * c->cfg.N;
  p.res = res;
  p.x = x;
  p.ids = ids;
  p.w = w;
  p.k = k;
  p.a = c->d_a;
  p.a_stride = a_stride_for(c->cfg);
  p.y = y;
  p.err = c->d_err;
  p.B = B;
  p.H = c->cfg.H;
  p.F = c->cfg.F;
  p.N = c->cfg.N;
  p.w2_offset = c->w2_offset;
  p.j_only = -1;
  p.dyn_pct = c->lc.dyn_pct;
  return p;
}

int launch_ffn(adapmoe_ctx* c, int layer, const void* x, int B, const int32_t* ids, const float* w, const int32_t* k,
               float* y, hipStream_t s, const ResolvedExperts* res = nullptr) {
  if (c->cfg.dtype == ADAPMOE_BF16 && B >= c->lc.batch_min && c->d_xop) {
    // several tokens: bucket by expert, stream every touched expert once (grouped GEMM on the matrix cores)
    const size_t esz = 2;
    for (int b0 = 0; b0 < B; b0 += 16) {
      BatchArgs q{};
      q.table = c->d_table + (size_t)layer * c->cfg.N;
      q.x = static_cast<const char*>(x) + (size_t)b0 * c->cfg.H * esz;
      q.ids = ids + 2 * b0;
      q.w = w + 2 * b0;
      q.k = k + b0;
      q.y = y + (size_t)b0 * c->cfg.H;
      q.err = c->d_err;
      q.B = std::min(16, B - b0);
      q.H = c->cfg.H;
      q.F = c->cfg.F;
      q.N = c->cfg.N;
      q.w2_offset = c->w2_offset;
      q.bkt_count = c->d_bkt_count;
      q.bkt_tok = c->d_bkt_tok;
      q.bkt_w = c->d_bkt_w;
      q.bkt_base = c->d_bkt_base;
      q.bkt_active = c->d_bkt_active;
      q.xop = c->d_xop;
      q.a_hi = c->d_ahi;
      q.a_lo = c->d_alo;
      q.two_terms = c->lc.batch_two_terms;
      HIPCHK(c, launch_bucket_gather(q, s, timed_cfg(c, 3).timing));
      HIPCHK(c, launch_grouped_gateup(q, c->lc.batch_direct, s, timed_cfg(c, 4).timing));
      HIPCHK(c, launch_grouped_down(q, c->lc.batch_two_terms != 0, s, timed_cfg(c, 5).timing));
    }
    c->ctr.ffn_launches++;
    return ADAPMOE_OK;
  }
  FfnArgs p = ffn_args(c, layer, x, B, ids, w, k, y, res);
  if (B == 1 && res != nullptr && c->lc.fused_blocks > 0) {
    // residency of the activated experts is established by the caller (moe_layer_step)
    FusedSync sy{c->d_fused_counter, (c->fused_seq + 1) * (unsigned)c->lc.fused_blocks, 4000000u};
    HIPCHK(c, fused_serialise(s));
    {
      ScopedTimer t(c, 6, s);
      HIPCHK(c, launch_ffn_fused(p, c->cfg.dtype, sy, c->lc.fused_blocks, s));
    }
    c->fused_seq++;
    c->ctr.ffn_launches++;
    return ADAPMOE_OK;
  }
  const int qb = quant_bits(c->cfg.dtype);
  // dynamic tail of the gate/up GEMV: its row counters are zero at launch because the down kernel
  // of the previous step cleared them (both kernels always run as a pair on one stream)
  const bool dyn = c->lc.dyn_pct > 0;
  {
    const LaunchCfg lc = timed_cfg(c, 0);
    p.dyn_ctr = dyn ? c->d_dyn : nullptr;
    p.dyn_clear = nullptr;
    HIPCHK(c, qb ? launch_ffn_gateup_quant(p, qb, lc, s) : launch_ffn_gateup(p, c->cfg.dtype, lc, s));
  }
  {
    const LaunchCfg lc = timed_cfg(c, 1);
    p.dyn_ctr = nullptr;
    p.dyn_clear = dyn ? c->d_dyn : nullptr;
    const hipError_t de = qb ? launch_ffn_down_quant(p, qb, lc, s) : launch_ffn_down(p, c->cfg.dtype, lc, s);
    if (de != hipSuccess) {
      // the gate/up kernel has drawn from its row counters and the kernel that clears them did not
      // start: clear them here, or the next gate/up launch would skip its pool rows
      if (dyn) (void)hipMemsetAsync(c->d_dyn, 0, (size_t)c->cfg.max_B * kDynQueues * kDynStride * sizeof(unsigned), s);
      return fail(c, ADAPMOE_EHIP, std::string("down GEMV launch: ") + hipGetErrorString(de));
    }
  }
  c->ctr.ffn_launches++;
  return ADAPMOE_OK;
}

// One token whose activated experts are partly still on their way (Alg.1, tile-wise scheduling):
// experts already in HBM are evaluated first, then each arriving expert tile by tile in the order
// the side stream delivers them; every launch waits only for the tile it reads.  rank_slot[j] is
// the cache slot of the expert of rank j, or -1 when it lives in caller memory.
int launch_ffn_tiled(adapmoe_ctx* c, int layer, const void* x, int kk, const int* rank_slot, float* y, hipStream_t s) {
  const int qb = quant_bits(c->cfg.dtype);
  int order[2] = {0, 1};
  auto arrival = [&](int j) -> uint64_t {
    if (rank_slot[j] < 0) return 0;
    const Slot& sl = c->slots[rank_slot[j]];
    return sl.copy_pending ? sl.copy_seq : 0;
  };
  if (kk > 1 && arrival(1) < arrival(0)) std::swap(order[0], order[1]);
  auto gateup = [&](FfnArgs& p) -> int {
    ScopedTimer t(c, 0, s);
    HIPCHK(c, qb ? launch_ffn_gateup_quant(p, qb, c->lc, s) : launch_ffn_gateup(p, c->cfg.dtype, c->lc, s));
    return ADAPMOE_OK;
  };
  auto down = [&](FfnArgs& p) -> int {
    ScopedTimer t(c, 1, s);
    HIPCHK(c, qb ? launch_ffn_down_quant(p, qb, c->lc, s) : launch_ffn_down(p, c->cfg.dtype, c->lc, s));
    return ADAPMOE_OK;
  };
  for (int i = 0; i < kk && i < 2; ++i) {
    const int j = order[i];
    FfnArgs p = ffn_args(c, layer, x, 1, nullptr, nullptr, nullptr, y, c->d_res);
    p.j_only = j;
    p.accumulate = i > 0;
    Slot* sl = rank_slot[j] >= 0 ? &c->slots[rank_slot[j]] : nullptr;
    int rc;
    if (sl && sl->copy_pending) {
      rc = wait_issued(c, *sl);
      if (rc) return rc;
    }
    if (sl && sl->copy_pending && hipEventQuery(sl->copy_done) == hipSuccess) sl->copy_pending = false;  // already landed
    (void)hipGetLastError();  // hipErrorNotReady from the query is not an error
    if (sl && sl->copy_pending && sl->tiled) {
      const int tg = gateup_tiles(c), td = down_tiles(c);
      for (int t = 0; t < tg + td; ++t) {
        HIPCHK(c, hipStreamWaitEvent(s, sl->tile_done[t], 0));
        tile_rows(c, t, &p.r0, &p.r1);
        rc = t < tg ? gateup(p) : down(p);
        if (rc) return rc;
      }
      sl->copy_pending = false;
      c->ctr.tiled_ffn++;
    } else {
      if (sl && sl->copy_pending) {
        HIPCHK(c, hipStreamWaitEvent(s, sl->copy_done, 0));
        sl->copy_pending = false;
      }
      p.r0 = 0;
      p.r1 = c->cfg.F;
      if ((rc = gateup(p))) return rc;
      p.r1 = c->cfg.H;
      if ((rc = down(p))) return rc;
    }
  }
  c->ctr.ffn_launches++;
  return ADAPMOE_OK;
}

// Gate of `layer` plus, for depth d = 1..depth, the gate of layer+d on the same input (prediction).
// pred[d-1] = {ids, k} output pointers of depth d.
int launch_gate_both(adapmoe_ctx* c, int layer, const void* x, int B, int32_t* ids, float* w, int32_t* k,
                     int depth, int32_t* const* pred_ids, int32_t* const* pred_k, hipStream_t s, ResolvedExperts* res = nullptr,
                     const NormArgs* norm = nullptr) {
  if (!c->router[layer]) return fail(c, ADAPMOE_ESTATE, "router of this layer not set");
  GateArgs g{};
  g.x = x;
  g.B = B;
  g.H = c->cfg.H;
  g.N = c->cfg.N;
  g.Wg[0] = c->router[layer];
  g.tau[0] = c->tau[layer];
  g.ids[0] = ids;
  g.k[0] = k;
  g.w = w;
  g.res = res;
  g.table = c->d_table + (size_t)layer * c->cfg.N;
  for (int d = 1; d <= depth; ++d) {
    const bool has = layer + d < c->cfg.L && c->router[layer + d];
    g.Wg[d] = has ? c->router[layer + d] : nullptr;
    g.tau[d] = has ? c->tau[layer + d] : 0.f;
    g.ids[d] = pred_ids[d - 1];
    g.k[d] = pred_k[d - 1];
  }
  if (depth >= 1 && layer == c->cfg.L - 1 && c->first_pred) {
    // last layer: its input also goes through the predictive gate of the first layer
    g.Wg[1] = c->first_pred;
    g.tau[1] = c->tau[0];
  }
  if (norm && depth > 0)   // several routers read x: it has to be complete before any of their workgroups starts
    HIPCHK(c, launch_residual_rmsnorm(norm->h, norm->y, norm->gamma, norm->x, c->bf16_act, B, c->cfg.H, s));
  const KernelTiming kt = timed_cfg(c, 2).timing;
  if (norm && depth == 0) HIPCHK(c, launch_norm_gate(g, *norm, c->bf16_act, s, kt));   // one router: normalise and gate in one launch
  else HIPCHK(c, launch_gate(g, c->bf16_act, 1 + depth, s, kt));
  return ADAPMOE_OK;
}

// Demand phase of one layer step (Alg.1: E.in_GPU are computed as they are, E.in_CPU go to the
// transfer queue): for every token, in token order, its k[b] required experts in rank order are
// looked up in the layer's LRU set and landing buffers; missing ones are copied on the side stream
// (evicting the least recently used entry, or into a spare slot when the layer owns none).  Leaves
// in c->step what the FFN has to wait for and what is released after it.  `resolved`: also write the
// experts' addresses into the per-token records the gate left for the FFN kernels.
int demand_tokens(adapmoe_ctx* c, int layer, const int32_t* ids, const int32_t* kk, int B, bool resolved) {
  const int N = c->cfg.N;
  LayerCache& lc = c->layers[layer];
  StepState& st = c->step;
  st.reset(layer);
  st.k0 = kk[0];
  auto& used_slots = st.used_slots;
  auto& transient = st.transient;
  auto& demanded = st.demanded;
  int* rank_slot = st.rank_slot;
  auto resolve = [&](int b, int j, const void* value) {
    if (resolved) poke_resolved(c, b, j, value);
  };
  int rc;
  for (int b = 0; b < B; ++b) {
    for (int j = 0; j < kk[b] && j < 2; ++j) {
      const int e = ids[2 * b + j];
      if (e < 0 || e >= N) return fail(c, ADAPMOE_EINVAL, "demand: expert id out of range");
      if (c->bound[(size_t)layer * N + e]) {
        record(c, layer, ADAPMOE_EV_HIT, e, -1, -2);
        resolve(b, j, c->bound[(size_t)layer * N + e]);
        continue;
      }
      bool is_transient = false;
      for (auto& t : transient) is_transient |= (t.first == e);
      const int pos = lc.find(e);
      if (pos >= 0) {
        Entry& en = lc.order[pos];
        record(c, layer, en.by_prefetch ? ADAPMOE_EV_HIT_PF : ADAPMOE_EV_HIT, e, -1, en.slot);
        en.by_prefetch = false;
        used_slots.push_back(en.slot);
        resolve(b, j, c->slots[en.slot].dev);
        if (b == 0) rank_slot[j] = en.slot;
        lc.touch(pos);
        demanded.push_back(e);
        continue;
      }
      const int lpos = lc.find_landing(e);
      if (lpos >= 0) {   // prefetched into a spare slot: no load; it joins the layer's set if the layer has one
        const Entry en = lc.landing[lpos];
        lc.landing.erase(lc.landing.begin() + lpos);
        int victim = -1;
        if (lc.cap > 0) {
          if ((int)lc.order.size() >= lc.cap) {
            const Entry v = lc.order.front();
            lc.order.erase(lc.order.begin());
            victim = v.expert;
            if (std::find(demanded.begin(), demanded.end(), victim) != demanded.end()) {
              transient.emplace_back(victim, v.slot);   // still read by this step's FFN
            } else {
              poke_later(c, layer, victim, nullptr);
              c->free_slots.push_back(v.slot);
            }
          }
          lc.order.push_back(Entry{e, en.slot, false});
          demanded.push_back(e);
        } else {
          transient.emplace_back(e, en.slot);
        }
        record(c, layer, ADAPMOE_EV_HIT_PF, e, victim, en.slot);
        used_slots.push_back(en.slot);
        resolve(b, j, c->slots[en.slot].dev);
        if (b == 0) rank_slot[j] = en.slot;
        continue;
      }
      if (is_transient) {  // evicted or bypassed earlier in this same step, image still in its slot
        if (lc.cap == 0) {
          for (auto& t : transient)
            if (t.first == e) {
              resolve(b, j, c->slots[t.second].dev);
              if (b == 0) rank_slot[j] = t.second;
            }
          record(c, layer, ADAPMOE_EV_BYPASS, e, -1, -1);
          continue;
        }
        // falls through to a regular miss below: logically it is gone
      }
      int victim = -1, slot = -1;
      if (lc.cap == 0) {
        if (c->free_slots.empty()) return fail(c, ADAPMOE_ENOMEM, "no spare slot for a bypass load");
        slot = c->free_slots.back();
        c->free_slots.pop_back();
        rc = start_copy(c, layer, e, slot);
        if (rc) return rc;
        poke_later(c, layer, e, c->slots[slot].dev);
        transient.emplace_back(e, slot);
        used_slots.push_back(slot);
        resolve(b, j, c->slots[slot].dev);
        if (b == 0) rank_slot[j] = slot;
        record(c, layer, ADAPMOE_EV_BYPASS, e, -1, slot);
        continue;
      }
      if ((int)lc.order.size() >= lc.cap) {
        Entry v = lc.order.front();
        lc.order.erase(lc.order.begin());
        victim = v.expert;
        const bool victim_needed = std::find(demanded.begin(), demanded.end(), victim) != demanded.end();
        if (victim_needed) {  // still read by this step's FFN: keep its image, take another slot
          transient.emplace_back(victim, v.slot);
          if (c->free_slots.empty()) return fail(c, ADAPMOE_ENOMEM, "no spare slot");
          slot = c->free_slots.back();
          c->free_slots.pop_back();
        } else {
          slot = v.slot;
          poke_later(c, layer, victim, nullptr);
        }
      } else {
        if (c->free_slots.empty()) return fail(c, ADAPMOE_ENOMEM, "no free cache slot");
        slot = c->free_slots.back();
        c->free_slots.pop_back();
      }
      if (is_transient) {
        // the expert was pushed out earlier in this step and is demanded again: reuse nothing, load again
        for (auto& t : transient)
          if (t.first == e) t.first = -1 - e;  // its old slot is still released, but the table entry now points to the new one
      }
      rc = start_copy(c, layer, e, slot);
      if (rc) return rc;
      lc.order.push_back(Entry{e, slot, false});
      poke_later(c, layer, e, c->slots[slot].dev);
      used_slots.push_back(slot);
      resolve(b, j, c->slots[slot].dev);
      if (b == 0) rank_slot[j] = slot;
      demanded.push_back(e);
      record(c, layer, ADAPMOE_EV_MISS, e, victim, slot);
    }
  }
  // prefetched experts that this step does not require are dropped; nothing reads them
  for (const Entry& en : lc.landing) {
    poke_later(c, layer, en.expert, nullptr);
    c->free_slots.push_back(en.slot);
  }
  lc.landing.clear();
  return ADAPMOE_OK;
}

// Makes `s` wait for the copies of the experts the running step reads.
int wait_for_step_copies(adapmoe_ctx* c, hipStream_t s) {
  for (int slot : c->step.used_slots) {
    Slot& sl = c->slots[slot];
    if (sl.copy_pending) {
      int rc = wait_issued(c, sl);
      if (rc) return rc;
      HIPCHK(c, hipStreamWaitEvent(s, sl.copy_done, 0));
      sl.copy_pending = false;
    }
  }
  return ADAPMOE_OK;
}

// End of a layer step, after its FFN has been enqueued on `s`: the slots it read are marked, and
// what the step held beyond the layer's own slots goes back to the pool.
int finish_step(adapmoe_ctx* c, hipStream_t s) {
  StepState& st = c->step;
  st.open = false;
  for (int slot : st.used_slots) {
    Slot& sl = c->slots[slot];
    HIPCHK(c, hipEventRecord(sl.read_done, s));
    sl.was_read = true;
  }
  for (auto& t : st.transient) {
    if (t.first >= 0) poke_later(c, st.layer, t.first, nullptr);
    c->free_slots.push_back(t.second);
  }
  if (!st.transient.empty()) {
    int rc = flush_pokes(c, s);
    if (rc) return rc;
  }
  st.used_slots.clear();
  st.transient.clear();
  return ADAPMOE_OK;
}

bool layer_fully_bound(const adapmoe_ctx* c, int layer) { return c->bound_count[layer] == c->cfg.N; }

}  // namespace

// ---- expert FFN without any allocation ------------------------------------------------------

// Scratch memory of moe_expert_ffn_static: the intermediate vectors a_j of up to kStaticMaxB tokens,
// the row counters of the gate/up GEMV's dynamic tail and a flag word, in a fixed array that every
// GPU the library runs on holds until the process ends.
constexpr int kStaticMaxB = 4;
constexpr size_t kStaticMaxStride = 16384;   // floats per (token, expert) of the a_j scratch: F <= 16384
constexpr size_t kStaticABytes = (size_t)kStaticMaxB * 2 * kStaticMaxStride * sizeof(float);
constexpr size_t kStaticDynBytes = (size_t)kStaticMaxB * adapmoe::kDynQueues * adapmoe::kDynStride * sizeof(unsigned);
constexpr size_t kStaticScratchBytes = kStaticABytes + kStaticDynBytes + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices] = {};        // device address of `scratch` on each GPU (each holds its own copy)
unsigned g_static_dtypes[kMaxDevices] = {};  // storage types whose kernels have been prepared on the GPU

// Address of this GPU's copy of `scratch`, looked up once per device with that device current.
// The array's name is only a handle on the host: kernels, memsets and copies get this address.
int static_scratch(int dev, int dtype, char** out) {
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return ADAPMOE_EHIP;
    }
    // the row counters must be zero when a gate/up launch starts (a fresh array is, and every down
    // launch leaves them so; this covers a process that reloads the library's code object)
    if (hipMemset(static_cast<char*>(ptr) + kStaticABytes, 0, kStaticDynBytes + 256) != hipSuccess) {
      (void)hipGetLastError();
      return ADAPMOE_EHIP;
    }
    g_static_ptr[dev] = ptr;
  }
  if (!(g_static_dtypes[dev] & (1u << dtype))) {
    if (ffn_kernels_init(dtype) != hipSuccess) {
      (void)hipGetLastError();
      return ADAPMOE_EHIP;
    }
    g_static_dtypes[dev] |= 1u << dtype;
  }
  *out = static_cast<char*>(g_static_ptr[dev]);
  return ADAPMOE_OK;
}

}  // namespace

// ---------------------------------------------------------------------------

extern "C" {

const char* adapmoe_strerror(int code) {
  switch (code) {
    case ADAPMOE_OK: return "ok";
    case ADAPMOE_EINVAL: return "invalid argument";
    case ADAPMOE_ENOMEM: return "out of memory";
    case ADAPMOE_ENOTREG: return "expert not registered";
    case ADAPMOE_ENORES: return "expert not resident";
    case ADAPMOE_EHIP: return "HIP runtime failure";
    case ADAPMOE_ESTATE: return "invalid state for this call";
    default: return "unknown error";
  }
}

const char* adapmoe_last_error(const adapmoe_ctx* ctx) { return ctx ? ctx->last_error.c_str() : ""; }

int adapmoe_expert_bytes(const adapmoe_config* cfg, size_t* bytes_out) {
  if (!cfg_ok(cfg) || !bytes_out) return ADAPMOE_EINVAL;
  if (const int qb = quant_bits(cfg->dtype)) *bytes_out = (size_t)2 * cfg->F * q_row_bytes(qb, cfg->H) + (size_t)cfg->H * q_row_bytes(qb, cfg->F);
  else *bytes_out = (size_t)3 * cfg->H * cfg->F * elem_size(cfg->dtype);
  return ADAPMOE_OK;
}

int adapmoe_pack_expert(const adapmoe_config* cfg, const void* W1, const void* W3, const void* W2, void* out) {
  if (!cfg_ok(cfg) || !W1 || !W3 || !W2 || !out || quant_bits(cfg->dtype)) return ADAPMOE_EINVAL;
  const size_t row = (size_t)cfg->H * elem_size(cfg->dtype);
  char* o = static_cast<char*>(out);
  for (int f = 0; f < cfg->F; ++f) {
    memcpy(o + (size_t)(2 * f) * row, static_cast<const char*>(W1) + (size_t)f * row, row);
    memcpy(o + (size_t)(2 * f + 1) * row, static_cast<const char*>(W3) + (size_t)f * row, row);
  }
  memcpy(o + (size_t)2 * cfg->F * row, W2, (size_t)cfg->H * cfg->F * elem_size(cfg->dtype));
  return ADAPMOE_OK;
}

// One row of n codes (4 or 2 bits) -> the streaming row format: blocks of up to 64 groups; a
// group's 64 codes take bits/2 vectors of 16 bytes and a block stores vector v of every group
// before vector v+1 of any.  A dword covers 32/bits consecutive elements: field s of its low
// half is element 2s, field s of its high half is element 2s+1.  Then (scale, zero) per group.
static void pack_row_quant(int bits, const uint8_t* q, const uint16_t* sc, const uint16_t* zr, size_t n, char* out) {
  const size_t G = n / 64;
  const int vecs = bits / 2;               // 16-byte vectors per group
  const int per_dword = 32 / bits;         // elements per dword
  const uint32_t cmask = (1u << bits) - 1;
  for (size_t blk = 0; blk * 64 < G; ++blk) {
    const size_t nb = std::min<size_t>(64, G - blk * 64);
    char* cb = out + blk * 64 * (size_t)bits * 8;
    for (size_t l = 0; l < nb; ++l) {
      const uint8_t* gq = q + (blk * 64 + l) * 64;
      for (int v = 0; v < vecs; ++v) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(cb + v * nb * 16 + l * 16);
        for (int d = 0; d < 4; ++d) {
          const uint8_t* e = gq + (v * 4 + d) * per_dword;
          uint32_t w = 0;
          for (int sft = 0; sft < per_dword / 2; ++sft) {
            w |= (uint32_t)(e[2 * sft] & cmask) << (bits * sft);
            w |= (uint32_t)(e[2 * sft + 1] & cmask) << (bits * sft + 16);
          }
          dst[d] = w;
        }
      }
    }
  }
  uint32_t* sz = reinterpret_cast<uint32_t*>(out + n * bits / 8);
  for (size_t g = 0; g < G; ++g) sz[g] = (uint32_t)sc[g] | ((uint32_t)zr[g] << 16);
}

static int pack_expert_quant(const adapmoe_config* cfg, int dtype, const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                             const uint8_t* q3, const uint16_t* s3, const uint16_t* z3, const uint8_t* q2,
                             const uint16_t* s2, const uint16_t* z2, void* out) {
  if (!cfg_ok(cfg) || cfg->dtype != dtype || !q1 || !s1 || !z1 || !q3 || !s3 || !z3 || !q2 || !s2 || !z2 || !out)
    return ADAPMOE_EINVAL;
  const int bits = quant_bits(dtype);
  const size_t H = cfg->H, F = cfg->F;
  const size_t rbH = q_row_bytes(bits, H), rbF = q_row_bytes(bits, F);
  char* o = static_cast<char*>(out);
  for (size_t f = 0; f < F; ++f) {
    pack_row_quant(bits, q1 + f * H, s1 + f * (H / 64), z1 + f * (H / 64), H, o + (2 * f) * rbH);
    pack_row_quant(bits, q3 + f * H, s3 + f * (H / 64), z3 + f * (H / 64), H, o + (2 * f + 1) * rbH);
  }
  char* o2 = o + 2 * F * rbH;
  for (size_t h = 0; h < H; ++h) pack_row_quant(bits, q2 + h * F, s2 + h * (F / 64), z2 + h * (F / 64), F, o2 + h * rbF);
  return ADAPMOE_OK;
}

int adapmoe_pack_expert_int4(const adapmoe_config* cfg, const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                             const uint8_t* q3, const uint16_t* s3, const uint16_t* z3, const uint8_t* q2,
                             const uint16_t* s2, const uint16_t* z2, void* out) {
  return pack_expert_quant(cfg, ADAPMOE_INT4G64, q1, s1, z1, q3, s3, z3, q2, s2, z2, out);
}

int adapmoe_pack_expert_int2(const adapmoe_config* cfg, const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                             const uint8_t* q3, const uint16_t* s3, const uint16_t* z3, const uint8_t* q2,
                             const uint16_t* s2, const uint16_t* z2, void* out) {
  return pack_expert_quant(cfg, ADAPMOE_INT2G64, q1, s1, z1, q3, s3, z3, q2, s2, z2, out);
}

int adapmoe_create(const adapmoe_config* cfg, adapmoe_ctx** out) {
  if (!out) return ADAPMOE_EINVAL;
  *out = nullptr;
  if (!cfg_ok(cfg) || cfg->max_B < 1 || cfg->max_B > 64) return ADAPMOE_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) return ADAPMOE_EHIP;
  adapmoe_ctx* c = new (std::nothrow) adapmoe_ctx();
  if (!c) return ADAPMOE_ENOMEM;
  try {
  c->cfg = *cfg;
  c->bf16_act = cfg->dtype != ADAPMOE_F32;
  adapmoe_expert_bytes(cfg, &c->image_bytes);
  c->w2_offset = quant_bits(cfg->dtype) ? (size_t)2 * cfg->F * q_row_bytes(quant_bits(cfg->dtype), cfg->H)
                                        : (size_t)2 * cfg->F * cfg->H * elem_size(cfg->dtype);
  const size_t LN = (size_t)cfg->L * cfg->N;
  c->router.assign(cfg->L, nullptr);
  c->tau.assign(cfg->L, 0.f);
  c->host_image.assign(LN, nullptr);
  c->bound.assign(LN, nullptr);
  c->bound_count.assign(cfg->L, 0);
  c->layers.resize(cfg->L);
  // defaults measured best on MI355X; adapmoe_set_option changes them
  c->lc.gateup_blocks = quant_bits(cfg->dtype) ? 256 : 512;   // quantised: 16 wavefronts per workgroup, one per compute unit
  c->lc.down_blocks = 256;
  c->lc.batch_min = 3;
  c->lc.batch_two_terms = 0;
  c->lc.batch_direct = 2;
  c->lc.fused_blocks = 0;
  c->lc.dyn_pct = quant_bits(cfg->dtype) ? 0 : 20;   // quantised gate/up: measured 1 us slower per launch with a dynamic tail
  const int B = cfg->max_B;
  bool ok = hipSetDevice(cfg->device) == hipSuccess;
  ok = ok && hipMalloc(&c->d_table, LN * sizeof(void*)) == hipSuccess;
  ok = ok && hipMemset(c->d_table, 0, LN * sizeof(void*)) == hipSuccess;
  ok = ok && hipMalloc(&c->d_err, sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMemset(c->d_err, 0, sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&c->d_dyn, (size_t)B * kDynQueues * kDynStride * sizeof(unsigned)) == hipSuccess;
  ok = ok && hipMemset(c->d_dyn, 0, (size_t)B * kDynQueues * kDynStride * sizeof(unsigned)) == hipSuccess;
  ok = ok && hipMalloc(&c->d_dec, (size_t)12 * B * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&c->d_w, (size_t)2 * B * sizeof(float)) == hipSuccess;
  ok = ok && hipMalloc(&c->d_a, (size_t)2 * B * a_stride_for(*cfg) * sizeof(float)) == hipSuccess;
  ok = ok && hipMalloc(&c->d_res, (size_t)B * sizeof(ResolvedExperts)) == hipSuccess;
  ok = ok && hipMemset(c->d_res, 0, (size_t)B * sizeof(ResolvedExperts)) == hipSuccess;
  ok = ok && hipHostMalloc(reinterpret_cast<void**>(&c->h_dec), (size_t)12 * B * sizeof(int32_t), hipHostMallocDefault) == hipSuccess;
  if (cfg->dtype == ADAPMOE_BF16 && B > 1) {
    const size_t N = cfg->N;
    ok = ok && hipMalloc(&c->d_bkt_count, N * sizeof(int32_t)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_bkt_tok, N * 16 * sizeof(int32_t)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_bkt_w, N * 16 * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_bkt_base, N * sizeof(void*)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_bkt_active, (N + 1) * sizeof(int32_t)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_xop, N * (size_t)cfg->H * 16 * 2) == hipSuccess;
    ok = ok && hipMalloc(&c->d_ahi, N * (size_t)cfg->F * 16 * 2) == hipSuccess;
    ok = ok && hipMalloc(&c->d_alo, N * (size_t)cfg->F * 16 * 2) == hipSuccess;
    ok = ok && batched_kernels_init() == hipSuccess;
  }
  ok = ok && hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) == hipSuccess;
  ok = ok && ffn_kernels_init(cfg->dtype) == hipSuccess;
  if (!ok) {
    adapmoe_destroy(c);
    return ADAPMOE_EHIP;
  }
  } catch (...) {   // a container of the context could not allocate
    adapmoe_destroy(c);
    return ADAPMOE_ENOMEM;
  }
  *out = c;
  return ADAPMOE_OK;
}

int adapmoe_destroy(adapmoe_ctx* c) {
  if (!c) return ADAPMOE_EINVAL;
  hipSetDevice(c->cfg.device);
  stop_stager(c);
  hipDeviceSynchronize();
  for (Slot& s : c->slots) {
    if (s.dev) hipFree(s.dev);
    if (s.copy_done) hipEventDestroy(s.copy_done);
    if (s.read_done) hipEventDestroy(s.read_done);
    for (hipEvent_t ev : s.tile_done) hipEventDestroy(ev);
  }
  for (TimedLaunch& t : c->timed) {
    hipEventDestroy(t.t0);
    hipEventDestroy(t.t1);
  }
  for (hipEvent_t e : c->event_pool) hipEventDestroy(e);
  if (c->copy_stream) hipStreamDestroy(c->copy_stream);
  if (c->d_table) hipFree(c->d_table);
  if (c->d_err) hipFree(c->d_err);
  if (c->d_dec) hipFree(c->d_dec);
  if (c->d_w) hipFree(c->d_w);
  if (c->d_a) hipFree(c->d_a);
  if (c->d_res) hipFree(c->d_res);
  if (c->d_fused_counter) hipFree(c->d_fused_counter);
  if (c->d_dyn) hipFree(c->d_dyn);
  if (c->d_bkt_count) hipFree(c->d_bkt_count);
  if (c->d_bkt_tok) hipFree(c->d_bkt_tok);
  if (c->d_bkt_w) hipFree(c->d_bkt_w);
  if (c->d_bkt_base) hipFree(c->d_bkt_base);
  if (c->d_bkt_active) hipFree(c->d_bkt_active);
  if (c->d_xop) hipFree(c->d_xop);
  if (c->d_ahi) hipFree(c->d_ahi);
  if (c->d_alo) hipFree(c->d_alo);
  if (c->h_dec) hipHostFree(c->h_dec);
  delete c;
  return ADAPMOE_OK;
}

int adapmoe_set_router(adapmoe_ctx* c, int layer, const void* Wg_dev) {
  if (!c || layer < 0 || layer >= c->cfg.L || !Wg_dev) return fail(c, ADAPMOE_EINVAL, "set_router: bad argument");
  c->router[layer] = Wg_dev;
  return ADAPMOE_OK;
}

int adapmoe_set_tau(adapmoe_ctx* c, const float* tau) {
  if (!c || !tau) return fail(c, ADAPMOE_EINVAL, "set_tau: bad argument");
  for (int l = 0; l < c->cfg.L; ++l) {
    if (!(tau[l] >= 0.f)) return fail(c, ADAPMOE_EINVAL, "set_tau: threshold must be >= 0");
    c->tau[l] = tau[l];
  }
  return ADAPMOE_OK;
}

int adapmoe_register_expert(adapmoe_ctx* c, int layer, int expert, const void* image_host, size_t bytes) {
  if (!c || layer < 0 || layer >= c->cfg.L || expert < 0 || expert >= c->cfg.N || !image_host)
    return fail(c, ADAPMOE_EINVAL, "register_expert: bad argument");
  if (bytes != c->image_bytes) return fail(c, ADAPMOE_EINVAL, "register_expert: image size mismatch");
  c->host_image[(size_t)layer * c->cfg.N + expert] = image_host;
  return ADAPMOE_OK;
}

int adapmoe_bind_expert_dev(adapmoe_ctx* c, int layer, int expert, const void* image_dev) {
  if (!c || layer < 0 || layer >= c->cfg.L || expert < 0 || expert >= c->cfg.N || !image_dev)
    return fail(c, ADAPMOE_EINVAL, "bind_expert_dev: bad argument");
  if ((reinterpret_cast<uintptr_t>(image_dev) & 15) != 0) return fail(c, ADAPMOE_EINVAL, "bind_expert_dev: image must be 16-byte aligned");
  const size_t idx = (size_t)layer * c->cfg.N + expert;
  if (c->layers[layer].find(expert) >= 0) return fail(c, ADAPMOE_ESTATE, "bind_expert_dev: expert currently cached");
  if (!c->bound[idx]) c->bound_count[layer]++;
  c->bound[idx] = image_dev;
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipMemcpy(c->d_table + idx, &image_dev, sizeof(void*), hipMemcpyHostToDevice));
  return ADAPMOE_OK;
}

// ---- planner (Sec. 4.4: Eq.10-15 cost, Eq.16-19 knapsack DP, traceback) -------

double cache_cost(int N, int t, double a, double beta) {
  if (N < 2 || t < 0 || t > N) return NAN;
  const double pairs = (double)N * (N - 1);
  const double miss1 = 1.0 - (double)t / N;                          // one given expert absent (Eq.10)
  const double miss2 = std::max((double)(N - t) * (N - t - 1), 0.0) / pairs;  // two given experts both absent
  const double mixed = 2.0 * (N - t) * t / pairs;                    // exactly one of two absent
  const double one = miss1 * (1.0 - beta);                           // Eq.11
  const double two = 2.0 * miss2 * (1.0 - beta)                      // Eq.12
                     + miss2 * beta                                  // Eq.13
                     + mixed * (1.0 - beta);                         // Eq.14
  return a * one + (1.0 - a) * two;                                  // Eq.15
}

int cache_plan(int L, int N, int C, const double* a, const double* beta, int32_t* t_out, double* cost_out) {
  ABI_TRY
  if (L < 1 || N < 2 || C < 0 || !a || !beta || !t_out) return ADAPMOE_EINVAL;
  const double tie = 1e-12;
  std::vector<double> f((size_t)L * (N + 1));
  for (int i = 0; i < L; ++i)
    for (int t = 0; t <= N; ++t) f[(size_t)i * (N + 1) + t] = cache_cost(N, t, a[i], beta[i]);
  const size_t W = (size_t)C + 1;
  std::vector<double> best((size_t)(L + 1) * W, 0.0);  // best[i][j]: first i layers, at most j slots (Eq.19)
  for (int i = 1; i <= L; ++i)
    for (int j = 0; j <= C; ++j) {
      double m = INFINITY;
      for (int k = 0; k <= std::min(j, N); ++k)
        m = std::min(m, best[(size_t)(i - 1) * W + (j - k)] + f[(size_t)(i - 1) * (N + 1) + k]);
      best[(size_t)i * W + j] = m;
    }
  int j = C;
  for (int i = L; i >= 1; --i) {  // traceback from the last layer, smallest slot count attaining the minimum
    int pick = 0;
    for (int k = 0; k <= std::min(j, N); ++k)
      if (best[(size_t)(i - 1) * W + (j - k)] + f[(size_t)(i - 1) * (N + 1) + k] <= best[(size_t)i * W + j] + tie) {
        pick = k;
        break;
      }
    t_out[i - 1] = pick;
    j -= pick;
  }
  if (cost_out) *cost_out = best[(size_t)L * W + C];
  return ADAPMOE_OK;
  ABI_CATCH(nullptr)
}

int cache_alloc(adapmoe_ctx* c, const int32_t* slots_per_layer) {
  ABI_TRY
  if (!c || !slots_per_layer) return fail(c, ADAPMOE_EINVAL, "cache_alloc: bad argument");
  if (c->cache_ready) return fail(c, ADAPMOE_ESTATE, "cache_alloc: already allocated");
  size_t total = 0;
  for (int l = 0; l < c->cfg.L; ++l) {
    if (slots_per_layer[l] < 0 || slots_per_layer[l] > c->cfg.N) return fail(c, ADAPMOE_EINVAL, "cache_alloc: slots per layer must be in 0..N");
    total += slots_per_layer[l];
  }
  total += 4 * (size_t)c->cfg.max_B;  // spare slots: what one step may read beyond the layers' own slots + landing buffers of the next layer
  HIPCHK(c, hipSetDevice(c->cfg.device));
  c->slots.resize(total);
  for (size_t i = 0; i < total; ++i) {
    Slot& s = c->slots[i];
    if (hipMalloc(reinterpret_cast<void**>(&s.dev), c->image_bytes) != hipSuccess ||
        hipEventCreateWithFlags(&s.copy_done, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&s.read_done, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      for (Slot& t : c->slots) {
        if (t.dev) hipFree(t.dev);
        if (t.copy_done) hipEventDestroy(t.copy_done);
        if (t.read_done) hipEventDestroy(t.read_done);
      }
      c->slots.clear();
      return fail(c, ADAPMOE_ENOMEM, "cache_alloc: HBM allocation failed");
    }
  }
  c->free_slots.clear();
  for (int i = (int)total - 1; i >= 0; --i) c->free_slots.push_back(i);
  for (int l = 0; l < c->cfg.L; ++l) {
    c->layers[l].cap = slots_per_layer[l];
    c->layers[l].order.clear();
  }
  c->cache_ready = true;
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

int cache_lookup(adapmoe_ctx* c, int layer, const int32_t* ids, int n, int32_t* slot_out, int touch) {
  ABI_TRY
  if (!c || layer < 0 || layer >= c->cfg.L || !ids || !slot_out || n < 0) return fail(c, ADAPMOE_EINVAL, "cache_lookup: bad argument");
  LayerCache& lc = c->layers[layer];
  for (int i = 0; i < n; ++i) {
    const int e = ids[i];
    if (e < 0 || e >= c->cfg.N) return fail(c, ADAPMOE_EINVAL, "cache_lookup: expert id out of range");
    if (c->bound[(size_t)layer * c->cfg.N + e]) { slot_out[i] = -2; continue; }
    const int pos = lc.find(e);
    if (pos < 0) {
      const int lpos = lc.find_landing(e);   // prefetched into a landing buffer: on the GPU, outside the LRU order
      slot_out[i] = lpos >= 0 ? lc.landing[lpos].slot : -1;
      continue;
    }
    slot_out[i] = lc.order[pos].slot;
    if (touch) lc.touch(pos);
  }
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

// ---- steps ------------------------------------------------------------------

int moe_gate(adapmoe_ctx* c, int layer, const void* x, int B, int32_t* ids, float* w, int32_t* k, int32_t* pred_ids,
             int32_t* pred_k, void* stream) {
  ABI_TRY
  if (!c || layer < 0 || layer >= c->cfg.L || !x || !ids || !w || !k || B < 1 || B > c->cfg.max_B)
    return fail(c, ADAPMOE_EINVAL, "moe_gate: bad argument");
  if ((pred_ids == nullptr) != (pred_k == nullptr)) return fail(c, ADAPMOE_EINVAL, "moe_gate: give both prediction outputs or neither");
  int32_t* pi[1] = {pred_ids};
  int32_t* pk[1] = {pred_k};
  return launch_gate_both(c, layer, x, B, ids, w, k, pred_ids ? 1 : 0, pi, pk, static_cast<hipStream_t>(stream));
  ABI_CATCH(c)
}

int moe_expert_ffn(adapmoe_ctx* c, int layer, const void* x, int B, const int32_t* ids, const float* w, const int32_t* k,
                   float* y, void* stream) {
  ABI_TRY
  if (!c || layer < 0 || layer >= c->cfg.L || !x || !ids || !w || !k || !y || B < 1 || B > c->cfg.max_B)
    return fail(c, ADAPMOE_EINVAL, "moe_expert_ffn: bad argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  int rc = flush_pokes(c, s);
  if (rc) return rc;
  if (c->step.open && c->step.layer == layer) {
    // moe_demand told which experts this step reads: wait for their copies, run, end the step
    rc = wait_for_step_copies(c, s);
    if (rc) return rc;
    rc = launch_ffn(c, layer, x, B, ids, w, k, y, s);
    if (rc) return rc;
    return finish_step(c, s);
  }
  // the ids are on the device only: wait for every copy into this layer's slots that is still unannounced
  LayerCache& lc = c->layers[layer];
  auto each_entry = [&](auto fn) -> int {
    for (Entry& en : lc.order) { int r = fn(c->slots[en.slot]); if (r) return r; }
    for (Entry& en : lc.landing) { int r = fn(c->slots[en.slot]); if (r) return r; }
    return ADAPMOE_OK;
  };
  rc = each_entry([&](Slot& sl) -> int {
    if (sl.copy_pending) {
      int r = wait_issued(c, sl);
      if (r) return r;
      HIPCHK(c, hipStreamWaitEvent(s, sl.copy_done, 0));
      sl.copy_pending = false;
    }
    return ADAPMOE_OK;
  });
  if (rc) return rc;
  rc = launch_ffn(c, layer, x, B, ids, w, k, y, s);
  if (rc) return rc;
  rc = each_entry([&](Slot& sl) -> int {
    HIPCHK(c, hipEventRecord(sl.read_done, s));
    sl.was_read = true;
    return ADAPMOE_OK;
  });
  if (rc) return rc;
  // this was the layer's demand: prefetched experts held outside the layer's own slots are dropped
  for (const Entry& en : lc.landing) {
    poke_later(c, layer, en.expert, nullptr);
    c->free_slots.push_back(en.slot);
  }
  if (!lc.landing.empty()) {
    lc.landing.clear();
    return flush_pokes(c, s);
  }
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

int moe_demand(adapmoe_ctx* c, int layer, const int32_t* ids_host, const int32_t* k_host, int B, int32_t* loads_out) {
  ABI_TRY
  if (!c || layer < 0 || layer >= c->cfg.L || !ids_host || !k_host || B < 1 || B > c->cfg.max_B)
    return fail(c, ADAPMOE_EINVAL, "moe_demand: bad argument");
  if (!c->cache_ready && !layer_fully_bound(c, layer)) return fail(c, ADAPMOE_ESTATE, "moe_demand: cache not allocated");
  for (int b = 0; b < B; ++b)
    if (k_host[b] < 1 || k_host[b] > 2) return fail(c, ADAPMOE_EINVAL, "moe_demand: k must be 1 or 2");
  if (c->step.open) return fail(c, ADAPMOE_ESTATE, "moe_demand: the previous demand has not been followed by moe_expert_ffn");
  const uint64_t before = c->ctr.misses + c->ctr.bypasses;
  const int rc = demand_tokens(c, layer, ids_host, k_host, B, false);
  if (rc) {
    c->step.open = false;
    return rc;
  }
  if (loads_out) *loads_out = (int32_t)(c->ctr.misses + c->ctr.bypasses - before);
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

int moe_prefetch(adapmoe_ctx* c, int layer, const int32_t* ids_host, int n) {
  ABI_TRY
  if (!c || layer < 0 || layer >= c->cfg.L || !ids_host || n < 0) return fail(c, ADAPMOE_EINVAL, "moe_prefetch: bad argument");
  if (!c->cache_ready) return fail(c, ADAPMOE_ESTATE, "moe_prefetch: cache not allocated");
  return prefetch_layer(c, layer, ids_host, n, true);
  ABI_CATCH(c)
}

int moe_expert_ffn_static(int32_t H, int32_t F, int32_t N, int32_t dtype, const void* const* table_dev, const void* x, int B,
                          const int32_t* ids, const float* w, const int32_t* k, float* y, int32_t* err_dev, void* stream) {
  adapmoe_config cfg{};
  cfg.H = H;
  cfg.F = F;
  cfg.N = N;
  cfg.L = 1;
  cfg.dtype = dtype;
  cfg.max_B = B;
  if (!cfg_ok(&cfg) || !table_dev || !x || !ids || !w || !k || !y) return ADAPMOE_EINVAL;
  if (B < 1 || B > kStaticMaxB) return ADAPMOE_EINVAL;          // beyond the fixed scratch array
  if (a_stride_for(cfg) > kStaticMaxStride) return ADAPMOE_EINVAL;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ADAPMOE_EHIP;
  char* base = nullptr;
  int rc = static_scratch(dev, dtype, &base);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int qb = quant_bits(dtype);
  LaunchCfg lc{};
  lc.gateup_blocks = qb ? 256 : 512;
  lc.down_blocks = 256;
  lc.dyn_pct = qb ? 0 : 20;
  unsigned* dyn = reinterpret_cast<unsigned*>(base + kStaticABytes);
  FfnArgs p{};
  p.table = table_dev;
  p.res = nullptr;
  p.x = x;
  p.ids = ids;
  p.w = w;
  p.k = k;
  p.a = reinterpret_cast<float*>(base);
  p.a_stride = a_stride_for(cfg);
  p.y = y;
  p.err = err_dev ? err_dev : reinterpret_cast<int32_t*>(base + kStaticABytes + kStaticDynBytes);
  p.B = B;
  p.H = H;
  p.F = F;
  p.N = N;
  p.w2_offset = qb ? (size_t)2 * F * q_row_bytes(qb, H) : (size_t)2 * F * H * elem_size(dtype);
  p.j_only = -1;
  p.dyn_pct = lc.dyn_pct;
  p.dyn_ctr = lc.dyn_pct > 0 ? dyn : nullptr;
  p.dyn_clear = nullptr;
  if ((qb ? launch_ffn_gateup_quant(p, qb, lc, s) : launch_ffn_gateup(p, dtype, lc, s)) != hipSuccess) {
    (void)hipGetLastError();
    return ADAPMOE_EHIP;
  }
  p.dyn_ctr = nullptr;
  p.dyn_clear = lc.dyn_pct > 0 ? dyn : nullptr;
  if ((qb ? launch_ffn_down_quant(p, qb, lc, s) : launch_ffn_down(p, dtype, lc, s)) != hipSuccess) {
    (void)hipGetLastError();
    return ADAPMOE_EHIP;
  }
  return ADAPMOE_OK;
}

}  // extern "C"

namespace {

// moe_layer_step with an optional residual update + normalisation in front of the gate
// (norm->x must be the x the step reads).
int layer_step_impl(adapmoe_ctx* c, int layer, const void* x, int B, float* y, void* stream, const NormArgs* norm) {
  if (!c || layer < 0 || layer >= c->cfg.L || !x || !y || B < 1 || B > c->cfg.max_B)
    return fail(c, ADAPMOE_EINVAL, "moe_layer_step: bad argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* d_ids = c->d_dec;
  int32_t* d_k = c->d_dec + 2 * B;
  int32_t* d_pids[3] = {c->d_dec + 3 * B, c->d_dec + 6 * B, c->d_dec + 9 * B};
  int32_t* d_pk[3] = {c->d_dec + 5 * B, c->d_dec + 8 * B, c->d_dec + 11 * B};
  const bool wraps = layer == c->cfg.L - 1 && c->first_pred != nullptr;   // prediction for layer 0 of the next token
  const int next = wraps ? 0 : layer + 1;
  const bool next_needs_host = next < c->cfg.L && !layer_fully_bound(c, next) && c->cache_ready;
  const bool host_path = !layer_fully_bound(c, layer) || next_needs_host;

  const int depth = host_path ? c->lookahead : 0;
  int rc = launch_gate_both(c, layer, x, B, d_ids, c->d_w, d_k, depth, d_pids, d_pk, s, c->d_res, norm);
  if (rc) return rc;
  c->ctr.tokens_gated += B;
  if (c->dec_log && c->dec_log_pos < c->dec_log_cap) {
    HIPCHK(c, hipMemcpyAsync(c->dec_log + (size_t)c->dec_log_pos * 6 * c->cfg.max_B, c->d_dec, (size_t)6 * B * sizeof(int32_t),
                             hipMemcpyDeviceToDevice, s));
    c->dec_log_pos++;
  }

  if (!host_path) {  // every expert of the layer lives in HBM: residency is a device-side table lookup
    rc = flush_pokes(c, s);
    if (rc) return rc;
    return launch_ffn(c, layer, x, B, d_ids, c->d_w, d_k, y, s, c->d_res);
  }
  if (!c->cache_ready && !layer_fully_bound(c, layer)) return fail(c, ADAPMOE_ESTATE, "moe_layer_step: cache not allocated");

  // Alg.1: the host needs E and r to decide what to transfer
  HIPCHK(c, hipMemcpyAsync(c->h_dec, c->d_dec, (size_t)(3 + 3 * depth) * B * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipStreamSynchronize(s));
  const int32_t* ids = c->h_dec;
  const int32_t* kk = c->h_dec + 2 * B;

  rc = demand_tokens(c, layer, ids, kk, B, true);
  if (rc) return rc;
  for (int b = 0; b < B; ++b)
    if (kk[b] == 1) c->ctr.single_expert++;

  // Predicted experts go to the transfer queue after the demanded ones (Alg.1).  Look-ahead
  // (Sec. 4.3): the layer after next is served only if nothing had to be loaded for the nearer one.
  if (c->cache_ready) {
    for (int d = 1; d <= depth && (layer + d < c->cfg.L || (wraps && d == 1)); ++d) {
      const int target = wraps ? 0 : layer + d;
      const int32_t* pids = c->h_dec + 3 * B * d;
      const int32_t* pk = pids + 2 * B;
      std::vector<int32_t> r;
      for (int b = 0; b < B; ++b)
        for (int j = 0; j < pk[b] && j < 2; ++j)
          if (std::find(r.begin(), r.end(), pids[2 * b + j]) == r.end()) r.push_back(pids[2 * b + j]);
      const uint64_t loads_before = c->ctr.prefetch_loads;
      rc = prefetch_layer(c, target, r.data(), (int)r.size(), d == 1);
      if (rc) return rc;
      if (c->ctr.prefetch_loads != loads_before) break;
    }
  }

  rc = flush_pokes(c, s);
  if (rc) return rc;
  StepState& st = c->step;
  bool tile_path = false;
  if (c->tiles > 1 && B == 1 && c->lc.fused_blocks == 0)
    for (int slot : st.used_slots) tile_path |= c->slots[slot].copy_pending && c->slots[slot].tiled;
  if (tile_path) {
    rc = launch_ffn_tiled(c, layer, x, kk[0], st.rank_slot, y, s);
  } else {
    rc = wait_for_step_copies(c, s);
    if (rc) return rc;
    rc = launch_ffn(c, layer, x, B, d_ids, c->d_w, d_k, y, s, c->d_res);
  }
  if (rc) return rc;
  return finish_step(c, s);
}

}  // namespace

extern "C" {

int moe_layer_step(adapmoe_ctx* c, int layer, const void* x, int B, float* y, void* stream) {
  ABI_TRY
  return layer_step_impl(c, layer, x, B, y, stream, nullptr);
  ABI_CATCH(c)
}

int moe_residual_rmsnorm(adapmoe_ctx* c, float* h, const float* y, float gamma, void* x, int B, void* stream) {
  if (!c || !h || !x || B < 1 || B > c->cfg.max_B) return fail(c, ADAPMOE_EINVAL, "moe_residual_rmsnorm: bad argument");
  HIPCHK(c, launch_residual_rmsnorm(h, y, gamma, x, c->bf16_act, B, c->cfg.H, static_cast<hipStream_t>(stream)));
  return ADAPMOE_OK;
}

int moe_stack_token(adapmoe_ctx* c, int token, float* h, void* x, float* y, int B, float gamma, void* stream) {
  ABI_TRY
  if (!c || !h || !x || !y || B < 1 || B > c->cfg.max_B) return fail(c, ADAPMOE_EINVAL, "moe_stack_token: bad argument");
  c->token = token;
  hipStream_t s = static_cast<hipStream_t>(stream);
  for (int l = 0; l < c->cfg.L; ++l) {
    const NormArgs norm{h, l > 0 ? y : nullptr, gamma, x};
    int rc = layer_step_impl(c, l, x, B, y, stream, &norm);
    if (rc) return rc;
  }
  // last residual update (x is rewritten with the normalised final state, unused)
  HIPCHK(c, launch_residual_rmsnorm(h, y, gamma, x, c->bf16_act, B, c->cfg.H, s));
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

// ---- bookkeeping ---------------------------------------------------------------

int adapmoe_set_first_layer_predictor(adapmoe_ctx* c, const void* Gpre_dev) {
  if (!c) return ADAPMOE_EINVAL;
  // with one layer the prefetch would target the layer that is running and could evict what its FFN reads
  if (Gpre_dev && c->cfg.L == 1) return fail(c, ADAPMOE_ESTATE, "set_first_layer_predictor: needs at least two layers");
  c->first_pred = Gpre_dev;
  return ADAPMOE_OK;
}

int adapmoe_set_option(adapmoe_ctx* c, int option, int value) {
  if (!c) return ADAPMOE_EINVAL;
  const bool quant = quant_bits(c->cfg.dtype) != 0;
  switch (option) {
    case ADAPMOE_OPT_BATCH_MIN:
      if (value < 1) return fail(c, ADAPMOE_EINVAL, "set_option: BATCH_MIN must be >= 1");
      c->lc.batch_min = value;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_BATCH_TWO_TERMS:
      if (value != 0 && value != 1) return fail(c, ADAPMOE_EINVAL, "set_option: BATCH_TWO_TERMS is 0 or 1");
      c->lc.batch_two_terms = value;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_BATCH_DIRECT:
      if (value < 0 || value > 2) return fail(c, ADAPMOE_EINVAL, "set_option: BATCH_DIRECT is 0, 1 or 2");
      c->lc.batch_direct = value;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_DYN_PCT:
      if (value < 0 || value > 100) return fail(c, ADAPMOE_EINVAL, "set_option: DYN_PCT is 0..100");
      c->lc.dyn_pct = value;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_GATEUP_BLOCKS:
      if (value < 1 || value > 65535) return fail(c, ADAPMOE_EINVAL, "set_option: GATEUP_BLOCKS is 1..65535");
      c->lc.gateup_blocks = value;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_DOWN_BLOCKS:
      if (value < 1 || value > 65535) return fail(c, ADAPMOE_EINVAL, "set_option: DOWN_BLOCKS is 1..65535");
      c->lc.down_blocks = value;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_POISON_SLOTS:
      if (value != 0 && value != 1) return fail(c, ADAPMOE_EINVAL, "set_option: POISON_SLOTS is 0 or 1");
      c->poison = value != 0;
      return ADAPMOE_OK;
    case ADAPMOE_OPT_FUSED: {
      if (value == 0) {
        c->lc.fused_blocks = 0;
        return ADAPMOE_OK;
      }
      if (value != 1) return fail(c, ADAPMOE_EINVAL, "set_option: FUSED is 0 or 1");
      if (quant) return fail(c, ADAPMOE_ESTATE, "set_option: the fused kernel takes fp32/bf16 experts only");
      // Single-token steps run both GEMVs in one launch with a grid-wide barrier in between.
      // Measured slower than two launches on MI355X (114 vs 108 us per Mixtral-shaped step) even
      // though the barrier needs no cache maintenance: every workgroup re-reads a_j past its L2,
      // and the slowest workgroup of the first phase holds up all others.
      HIPCHK(c, hipSetDevice(c->cfg.device));
      int cap = 0;
      const hipError_t fe = ffn_fused_init(c->cfg.dtype);
      if (fe == hipSuccess) cap = ffn_fused_capacity(c->cfg.dtype, c->cfg.H, c->cfg.F, c->cfg.device);
      if (getenv("ADAPMOE_VERBOSE")) fprintf(stderr, "adapmoe: fused init %s, capacity %d\n", hipGetErrorString(fe), cap);
      (void)hipGetLastError();  // a shape the fused kernel does not take is not an error of the runtime
      if (cap <= 0) return fail(c, ADAPMOE_ESTATE, "set_option: shape does not fit the fused kernel");
      if (!c->d_fused_counter) {
        HIPCHK(c, hipMalloc(&c->d_fused_counter, sizeof(unsigned)));
        HIPCHK(c, hipMemset(c->d_fused_counter, 0, sizeof(unsigned)));
        c->fused_seq = 0;
      }
      c->lc.fused_blocks = cap;
      return ADAPMOE_OK;
    }
    default:
      return fail(c, ADAPMOE_EINVAL, "set_option: unknown option");
  }
}

int adapmoe_get_option(adapmoe_ctx* c, int option, int* value_out) {
  if (!c || !value_out) return ADAPMOE_EINVAL;
  switch (option) {
    case ADAPMOE_OPT_BATCH_MIN: *value_out = c->lc.batch_min; break;
    case ADAPMOE_OPT_BATCH_TWO_TERMS: *value_out = c->lc.batch_two_terms; break;
    case ADAPMOE_OPT_BATCH_DIRECT: *value_out = c->lc.batch_direct; break;
    case ADAPMOE_OPT_DYN_PCT: *value_out = c->lc.dyn_pct; break;
    case ADAPMOE_OPT_GATEUP_BLOCKS: *value_out = c->lc.gateup_blocks; break;
    case ADAPMOE_OPT_DOWN_BLOCKS: *value_out = c->lc.down_blocks; break;
    case ADAPMOE_OPT_FUSED: *value_out = c->lc.fused_blocks > 0 ? 1 : 0; break;
    case ADAPMOE_OPT_POISON_SLOTS: *value_out = c->poison ? 1 : 0; break;
    default: return fail(c, ADAPMOE_EINVAL, "get_option: unknown option");
  }
  return ADAPMOE_OK;
}

int adapmoe_set_staging(adapmoe_ctx* c, int buffers, int host_threads) {
  ABI_TRY
  if (!c || buffers < 0 || buffers > 16 || host_threads < 0 || host_threads > 64) return fail(c, ADAPMOE_EINVAL, "set_staging: buffers 0..16, host threads 0..64");
  if (c->step.open) return fail(c, ADAPMOE_ESTATE, "set_staging: a layer step is open");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  if (c->stager) {
    int rc = drain_stager(c);
    if (rc) return rc;
    stop_stager(c);
  }
  if (buffers == 0) return ADAPMOE_OK;
  if (buffers < 2) return fail(c, ADAPMOE_EINVAL, "set_staging: at least two buffers (one fills while the other crosses the link)");
  Stager* st = new Stager();
  st->threads = host_threads > 0 ? host_threads : 6;
  st->bufs.resize(buffers);
  c->stager = st;
  for (StageBuf& b : st->bufs) {
    if (hipHostMalloc(reinterpret_cast<void**>(&b.host), c->image_bytes, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&b.done, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      stop_stager(c);
      return fail(c, ADAPMOE_ENOMEM, "set_staging: pinned buffer allocation failed");
    }
  }
  for (int i = 0; i + 1 < st->threads; ++i) st->helpers.emplace_back(pool_helper, st, i);
  st->worker = std::thread(stager_main, c);
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

int adapmoe_set_tiles(adapmoe_ctx* c, int tiles) {
  if (!c || tiles < 0 || tiles > 64 || tiles > c->cfg.F || tiles / 2 > c->cfg.H)
    return fail(c, ADAPMOE_EINVAL, "set_tiles: tiles must be 0..64 and not exceed the number of rows");
  c->tiles = tiles;
  return ADAPMOE_OK;
}

int adapmoe_set_lookahead(adapmoe_ctx* c, int depth) {
  if (!c || depth < 1 || depth > 3) return fail(c, ADAPMOE_EINVAL, "set_lookahead: depth must be 1, 2 or 3");
  c->lookahead = depth;
  return ADAPMOE_OK;
}

int adapmoe_last_lookahead(adapmoe_ctx* c, int depth, int32_t* pred_ids, int32_t* pred_k, int B) {
  if (!c || depth < 1 || depth > 3 || B < 1 || B > c->cfg.max_B) return fail(c, ADAPMOE_EINVAL, "last_lookahead: bad argument");
  if (pred_ids) memcpy(pred_ids, c->h_dec + 3 * B * depth, (size_t)2 * B * sizeof(int32_t));
  if (pred_k) memcpy(pred_k, c->h_dec + 3 * B * depth + 2 * B, (size_t)B * sizeof(int32_t));
  return ADAPMOE_OK;
}

int adapmoe_set_token(adapmoe_ctx* c, int token) {
  if (!c) return ADAPMOE_EINVAL;
  c->token = token;
  return ADAPMOE_OK;
}

int adapmoe_trace_read(adapmoe_ctx* c, adapmoe_event* buf, size_t cap, size_t* n_out) {
  if (!c || (!buf && cap) || !n_out) return fail(c, ADAPMOE_EINVAL, "trace_read: bad argument");
  size_t n = std::min(cap, c->trace.size());
  for (size_t i = 0; i < n; ++i) {
    buf[i] = c->trace.front();
    c->trace.pop_front();
  }
  *n_out = n;
  return ADAPMOE_OK;
}

int adapmoe_counters(adapmoe_ctx* c, adapmoe_counters_t* out) {
  if (!c || !out) return ADAPMOE_EINVAL;
  *out = c->ctr;
  return ADAPMOE_OK;
}

int adapmoe_last_decision(adapmoe_ctx* c, int32_t* ids, int32_t* k, int32_t* pred_ids, int32_t* pred_k, int B) {
  if (!c || B < 1 || B > c->cfg.max_B) return fail(c, ADAPMOE_EINVAL, "last_decision: bad argument");
  if (ids) memcpy(ids, c->h_dec, (size_t)2 * B * sizeof(int32_t));
  if (k) memcpy(k, c->h_dec + 2 * B, (size_t)B * sizeof(int32_t));
  if (pred_ids) memcpy(pred_ids, c->h_dec + 3 * B, (size_t)2 * B * sizeof(int32_t));
  if (pred_k) memcpy(pred_k, c->h_dec + 5 * B, (size_t)B * sizeof(int32_t));
  return ADAPMOE_OK;
}

int adapmoe_set_decision_log(adapmoe_ctx* c, int32_t* log_dev, int capacity) {
  if (!c || capacity < 0 || (log_dev && capacity < 1)) return fail(c, ADAPMOE_EINVAL, "set_decision_log: bad argument");
  c->dec_log = log_dev;
  c->dec_log_cap = log_dev ? capacity : 0;
  c->dec_log_pos = 0;
  return ADAPMOE_OK;
}

int adapmoe_check(adapmoe_ctx* c, void* stream) {
  if (!c) return ADAPMOE_EINVAL;
  HIPCHK(c, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  int drc = drain_stager(c);
  if (drc) return drc;
  HIPCHK(c, hipStreamSynchronize(c->copy_stream));
  int32_t flags = 0;
  HIPCHK(c, hipMemcpy(&flags, c->d_err, sizeof(flags), hipMemcpyDeviceToHost));
  if (flags) {
    HIPCHK(c, hipMemset(c->d_err, 0, sizeof(int32_t)));
    if (flags & 4) return fail(c, ADAPMOE_EHIP, "fused FFN kernel: grid barrier timed out (device shared with another long-running kernel?)");
    if (flags & 2) return fail(c, ADAPMOE_EINVAL, "expert FFN met an expert id out of range (or the same expert twice for one token)");
    return fail(c, ADAPMOE_ENORES, "expert FFN met a non-resident expert");
  }
  return ADAPMOE_OK;
}

int adapmoe_profile(adapmoe_ctx* c, int on) {
  if (!c) return ADAPMOE_EINVAL;
  c->profiling = on != 0;
  return ADAPMOE_OK;
}

int adapmoe_profile_read(adapmoe_ctx* c, int cls, uint64_t* launches, double* total_ms) {
  ABI_TRY
  if (!c || !launches || !total_ms) return fail(c, ADAPMOE_EINVAL, "profile_read: bad argument");
  uint64_t n = 0;
  double ms = 0.0;
  std::vector<TimedLaunch> keep;
  hipError_t bad = hipSuccess;
  for (TimedLaunch& t : c->timed) {
    if (t.cls != cls) { keep.push_back(t); continue; }
    float d = 0.f;
    hipError_t e = hipEventSynchronize(t.t1);
    if (e == hipSuccess) e = hipEventElapsedTime(&d, t.t0, t.t1);
    if (e == hipSuccess) {
      ms += d;
      ++n;
    } else {
      bad = e;
    }
    c->event_pool.push_back(t.t0);   // every event stays owned by exactly one list
    c->event_pool.push_back(t.t1);
  }
  c->timed.swap(keep);
  *launches = n;
  *total_ms = ms;
  if (bad != hipSuccess) return fail(c, ADAPMOE_EHIP, std::string("profile_read: ") + hipGetErrorString(bad));
  return ADAPMOE_OK;
  ABI_CATCH(c)
}

int adapmoe_stream_probe(const void* buf_dev, int64_t nrows, int row_bytes, int rows_per_unit, int chunk_bytes, int workgroups, int reps,
                         double* us_out, void* stream) {
  ABI_TRY
  const bool whole = chunk_bytes == row_bytes;
  if (!buf_dev || !us_out || nrows < 1 || row_bytes < 512 || rows_per_unit < 1 || reps < 1 || workgroups < 1 || workgroups > 65535)
    return ADAPMOE_EINVAL;
  if (whole ? (chunk_bytes % 1024 != 0 || chunk_bytes > 16384 || 16384 % chunk_bytes != 0) : (chunk_bytes != 512 || row_bytes % 512 != 0))
    return ADAPMOE_EINVAL;
  if (((int64_t)rows_per_unit * chunk_bytes) % 16384 != 0 || nrows % rows_per_unit != 0) return ADAPMOE_EINVAL;
  // parts per wavefront must fit the streamer's 32-bit count
  const int64_t units = nrows / rows_per_unit, parts = (int64_t)(rows_per_unit / (16384 / chunk_bytes)) * (row_bytes / chunk_bytes);
  if ((units / ((int64_t)workgroups * 4) + 1) * parts > 0x7fffffff) return ADAPMOE_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) e = launch_stream_probe(buf_dev, (long)nrows, row_bytes, rows_per_unit, chunk_bytes, workgroups, nullptr, s);   // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, s);
  for (int r = 0; r < reps && e == hipSuccess; ++r)
    e = launch_stream_probe(buf_dev, (long)nrows, row_bytes, rows_per_unit, chunk_bytes, workgroups, nullptr, s);
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  if (e0) hipEventDestroy(e0);
  if (e1) hipEventDestroy(e1);
  if (e != hipSuccess) return ADAPMOE_EHIP;
  *us_out = (double)ms * 1e3 / reps;
  return ADAPMOE_OK;
  ABI_CATCH(nullptr)
}

}  // extern "C"
