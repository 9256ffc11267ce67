// cs_xchannel: the embedding hand-off between an encoder task and an LLM task that run as two
// PROCESSES on one GPU.  The paper's executors are separate processes joined by a per-GPU Sidecar
// (Sec. 2.1 "Data Plane"): the sender's tensor is written to a shared buffer, the receiver is
// notified of its address and reads it into its own memory (Sec. 2.2 "Data Forwarding"), and
// executors wait for tensors that have not arrived (Sec. 2.1 "Request Lifecycle").
//
// Here the shared buffer is a pool of slots in HBM that the producer allocates and the consumer maps
// through an IPC memory handle (rows never leave the GPU); the slot table and the notification queue
// live in a POSIX shared-memory segment both processes map; the notification is the slot number,
// pushed into the queue by a host function the producer's stream runs once everything enqueued
// before publish has finished, so a slot the consumer is told about is complete in memory; the
// consumer's copy is the placement itself (the row scatter reads the slot through its mapping), and a
// host function behind it hands the slot back.  No GPU event crosses the process boundary.
//
// Slot life: FREE -> WRITING (acquire) -> PUBLISHING (publish called, producer's work still running)
// -> READY (work done, notification queued) -> DRAINING (forward called, scatter running) -> FREE.
// Every transition is one atomic store or compare-exchange on the slot's state word; the two
// processes share no lock except a spin flag around queue pushes.
#include <errno.h>
#include <fcntl.h>
#include <hip/hip_runtime.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <time.h>
#include <unistd.h>

#include <atomic>
#include <new>
#include <string>

#include "common.h"

using namespace cs;

namespace {

constexpr uint32_t XCH_MAGIC = 0x43535843u;   // "CXSC"
constexpr int XCH_MAX_SLOTS = 256;
constexpr size_t XCH_MAX_POOL = ((size_t)2 << 30) - 4096;   // one IPC mapping stays under 2 GiB

struct XSlot {
  std::atomic<int32_t> state;
  int32_t hidden, dtype;
  int64_t n_rows;
  uint64_t bytes;                      // what acquire reserved
  std::atomic<int64_t> t_ready_ns;     // CLOCK_MONOTONIC when the producer's work was seen finished
  std::atomic<int64_t> t_placed_ns;    // ... when the consumer's placement was seen finished
};

struct XCtl {
  uint32_t magic;
  int32_t n_slots;
  uint64_t slot_bytes, slot_stride;
  hipIpcMemHandle_t mem;
  std::atomic<int32_t> attached;       // consumers that opened the pool
  // notification queue: slot numbers in the order they became READY (each slot is in it at most once)
  std::atomic<uint32_t> q_head, q_tail;
  std::atomic_flag q_push_lock;
  int32_t queue[XCH_MAX_SLOTS];
  XSlot slots[XCH_MAX_SLOTS];
};

static_assert(std::atomic<int32_t>::is_always_lock_free && std::atomic<int64_t>::is_always_lock_free,
              "the slot table is shared between processes: its atomics must be address-free");

int64_t now_ns() {
  timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (int64_t)ts.tv_sec * 1000000000ll + ts.tv_nsec;
}

std::string shm_name(const char* name) { return std::string("/cornenc-") + name; }

struct HostArg {            // what a stream's host function needs; one per slot and direction, reused
  XCtl* ctl;
  int32_t slot;
};

// Runs on a runtime thread behind the producer's work: the slot is complete in memory.
void on_produced(void* p) {
  HostArg* a = static_cast<HostArg*>(p);
  XCtl* c = a->ctl;
  XSlot& s = c->slots[a->slot];
  s.t_ready_ns.store(now_ns(), std::memory_order_relaxed);
  s.state.store(CS_XSLOT_READY, std::memory_order_release);
  while (c->q_push_lock.test_and_set(std::memory_order_acquire)) {}
  const uint32_t t = c->q_tail.load(std::memory_order_relaxed);
  c->queue[t % XCH_MAX_SLOTS] = a->slot;
  c->q_tail.store(t + 1, std::memory_order_release);
  c->q_push_lock.clear(std::memory_order_release);
}

// Runs behind the consumer's scatter: the slot has been read and may be written again.
void on_placed(void* p) {
  HostArg* a = static_cast<HostArg*>(p);
  XSlot& s = a->ctl->slots[a->slot];
  s.t_placed_ns.store(now_ns(), std::memory_order_relaxed);
  s.state.store(CS_XSLOT_FREE, std::memory_order_release);
}

}  // namespace

struct cs_xchannel {
  bool owner = false;
  std::string name;
  XCtl* ctl = nullptr;
  unsigned char* pool = nullptr;
  HostArg args[XCH_MAX_SLOTS];
};

static void xch_free(cs_xchannel* x) {
  if (!x) return;
  if (x->pool) {
    if (x->owner) (void)hipFree(x->pool);
    else (void)hipIpcCloseMemHandle(x->pool);
  }
  if (x->ctl) munmap(x->ctl, sizeof(XCtl));
  if (x->owner && !x->name.empty()) shm_unlink(shm_name(x->name.c_str()).c_str());
  delete x;
}

static cs_status xslot(cs_xchannel* x, int32_t slot, const char* who, XSlot** out) {
  if (!x) return fail(CS_ERR_INVALID_ARG, std::string(who) + ": NULL channel");
  if (slot < 0 || slot >= x->ctl->n_slots) return fail(CS_ERR_INVALID_ARG, std::string(who) + ": no such slot");
  *out = &x->ctl->slots[slot];
  return CS_OK;
}

static bool name_ok(const char* name) {
  if (!name || !*name) return false;
  size_t n = 0;
  for (const char* p = name; *p; ++p, ++n)
    if (!((*p >= 'a' && *p <= 'z') || (*p >= 'A' && *p <= 'Z') || (*p >= '0' && *p <= '9') || *p == '_' || *p == '-')) return false;
  return n <= 64;
}

extern "C" {

cs_status cs_xchannel_create(const char* name, int32_t n_slots, size_t slot_bytes, cs_xchannel** out) try {
  if (!out) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_create: NULL out");
  *out = nullptr;
  if (!name_ok(name)) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_create: name must be 1..64 characters of [A-Za-z0-9_-]");
  if (n_slots <= 0 || n_slots > XCH_MAX_SLOTS) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_create: n_slots out of range");
  const size_t stride = (slot_bytes + 255) & ~(size_t)255;
  if (slot_bytes == 0 || stride > XCH_MAX_POOL / (size_t)n_slots)
    return fail(CS_ERR_UNSUPPORTED, "cs_xchannel_create: the pool (n_slots * slot_bytes) must stay under 2 GiB");
  cs_xchannel* x = new cs_xchannel();
  x->owner = true;
  const std::string sn = shm_name(name);
  const int fd = shm_open(sn.c_str(), O_CREAT | O_EXCL | O_RDWR, 0600);
  if (fd < 0) {
    delete x;
    return fail(CS_ERR_INVALID_ARG, "cs_xchannel_create: shm_open(" + sn + "): " + strerror(errno));
  }
  x->name = name;
  void* m = MAP_FAILED;
  if (ftruncate(fd, sizeof(XCtl)) == 0) m = mmap(nullptr, sizeof(XCtl), PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
  close(fd);
  if (m == MAP_FAILED) {
    xch_free(x);
    return fail(CS_ERR_NO_MEMORY, std::string("cs_xchannel_create: shared segment: ") + strerror(errno));
  }
  x->ctl = new (m) XCtl();   // the fresh segment is zero-filled; this gives the atomics their start values
  XCtl* c = x->ctl;
  c->n_slots = n_slots;
  c->slot_bytes = slot_bytes;
  c->slot_stride = stride;
  c->q_push_lock.clear();
  for (int i = 0; i < n_slots; ++i) c->slots[i].state.store(CS_XSLOT_FREE);
  hipError_t he = hipMalloc(reinterpret_cast<void**>(&x->pool), stride * (size_t)n_slots);
  if (he == hipSuccess) he = hipIpcGetMemHandle(&c->mem, x->pool);
  if (he != hipSuccess) {
    xch_free(x);
    return fail(CS_ERR_HIP, std::string("cs_xchannel_create: ") + hipGetErrorString(he));
  }
  for (int i = 0; i < n_slots; ++i) x->args[i] = HostArg{c, i};
  std::atomic_thread_fence(std::memory_order_release);
  c->magic = XCH_MAGIC;      // last: an opener that sees it sees everything above
  *out = x;
  return CS_OK;
} CS_CATCH_ALL("cs_xchannel_create")

cs_status cs_xchannel_open(const char* name, cs_xchannel** out) try {
  if (!out) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_open: NULL out");
  *out = nullptr;
  if (!name_ok(name)) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_open: bad name");
  const std::string sn = shm_name(name);
  const int fd = shm_open(sn.c_str(), O_RDWR, 0600);
  if (fd < 0) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_open: shm_open(" + sn + "): " + strerror(errno));
  struct stat st;
  void* m = MAP_FAILED;
  if (fstat(fd, &st) == 0 && (size_t)st.st_size >= sizeof(XCtl))
    m = mmap(nullptr, sizeof(XCtl), PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
  close(fd);
  if (m == MAP_FAILED) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_open: the segment is not a channel (or not complete yet)");
  cs_xchannel* x = new cs_xchannel();
  x->ctl = static_cast<XCtl*>(m);
  std::atomic_thread_fence(std::memory_order_acquire);
  if (x->ctl->magic != XCH_MAGIC || x->ctl->n_slots <= 0 || x->ctl->n_slots > XCH_MAX_SLOTS) {
    xch_free(x);
    return fail(CS_ERR_INVALID_ARG, "cs_xchannel_open: the segment is not a channel (or not complete yet)");
  }
  void* p = nullptr;
  const hipError_t he = hipIpcOpenMemHandle(&p, x->ctl->mem, hipIpcMemLazyEnablePeerAccess);
  if (he != hipSuccess) {
    xch_free(x);
    return fail(CS_ERR_HIP, std::string("cs_xchannel_open: hipIpcOpenMemHandle: ") + hipGetErrorString(he));
  }
  x->pool = static_cast<unsigned char*>(p);
  for (int i = 0; i < x->ctl->n_slots; ++i) x->args[i] = HostArg{x->ctl, i};
  x->ctl->attached.fetch_add(1);
  *out = x;
  return CS_OK;
} CS_CATCH_ALL("cs_xchannel_open")

void cs_xchannel_close(cs_xchannel* x) {
  if (!x) return;
  // host functions of this process that are still queued on a stream refer to this object
  (void)hipDeviceSynchronize();
  if (x->ctl && !x->owner) x->ctl->attached.fetch_sub(1);
  xch_free(x);
}

cs_status cs_xchannel_acquire(cs_xchannel* x, size_t bytes, int32_t* slot, void** dev_ptr) try {
  if (!x || !slot || !dev_ptr) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_acquire: NULL argument");
  *slot = -1;
  *dev_ptr = nullptr;
  XCtl* c = x->ctl;
  if (bytes == 0 || bytes > c->slot_bytes) return fail(CS_ERR_WORKSPACE, "cs_xchannel_acquire: tensor does not fit a slot");
  for (int i = 0; i < c->n_slots; ++i) {
    int32_t want = CS_XSLOT_FREE;
    // FREE is stored only after the consumer's scatter of the slot's last tensor has finished
    if (c->slots[i].state.compare_exchange_strong(want, CS_XSLOT_WRITING, std::memory_order_acq_rel)) {
      c->slots[i].bytes = bytes;
      *slot = i;
      *dev_ptr = x->pool + (size_t)i * c->slot_stride;
      return CS_OK;
    }
  }
  return fail(CS_ERR_BUSY, "cs_xchannel_acquire: every slot is in use");
} CS_CATCH_ALL("cs_xchannel_acquire")

cs_status cs_xchannel_publish(cs_xchannel* x, int32_t slot, int64_t n_rows, int32_t hidden, int32_t dtype,
                              void* producer_stream) try {
  XSlot* s = nullptr;
  if (cs_status st = xslot(x, slot, "cs_xchannel_publish", &s)) return st;
  if (dtype != CS_F32 && dtype != CS_BF16) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_publish: dtype");
  if (n_rows < 0 || hidden <= 0) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_publish: sizes");
  const size_t row_bytes = (size_t)hidden * (dtype == CS_BF16 ? 2 : 4);
  if (row_bytes % 16) return fail(CS_ERR_UNSUPPORTED, "cs_xchannel_publish: a row must be a multiple of 16 bytes");
  if (s->state.load(std::memory_order_acquire) != CS_XSLOT_WRITING)
    return fail(CS_ERR_INVALID_ARG, "cs_xchannel_publish: slot was not acquired");
  if ((uint64_t)n_rows > s->bytes / row_bytes) return fail(CS_ERR_SHAPE, "cs_xchannel_publish: more rows than were reserved");
  s->n_rows = n_rows;
  s->hidden = hidden;
  s->dtype = dtype;
  s->state.store(CS_XSLOT_PUBLISHING, std::memory_order_release);
  const hipError_t he = hipLaunchHostFunc(static_cast<hipStream_t>(producer_stream), on_produced, &x->args[slot]);
  if (he != hipSuccess) {
    s->state.store(CS_XSLOT_WRITING, std::memory_order_release);
    return fail(CS_ERR_HIP, std::string("cs_xchannel_publish: hipLaunchHostFunc: ") + hipGetErrorString(he));
  }
  return CS_OK;
} CS_CATCH_ALL("cs_xchannel_publish")

cs_status cs_xchannel_wait(cs_xchannel* x, int64_t timeout_us, int32_t* slot, int64_t* n_rows, int32_t* hidden,
                           int32_t* dtype) try {
  if (!x || !slot) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_wait: NULL argument");
  *slot = -1;
  XCtl* c = x->ctl;
  const int64_t t0 = now_ns(), limit = timeout_us < 0 ? 0 : timeout_us * 1000;
  for (int spins = 0;; ++spins) {
    const uint32_t h = c->q_head.load(std::memory_order_relaxed);
    if (h != c->q_tail.load(std::memory_order_acquire)) {
      const int32_t sl = c->queue[h % XCH_MAX_SLOTS];
      c->q_head.store(h + 1, std::memory_order_release);
      const XSlot& s = c->slots[sl];
      *slot = sl;
      if (n_rows) *n_rows = s.n_rows;
      if (hidden) *hidden = s.hidden;
      if (dtype) *dtype = s.dtype;
      return CS_OK;
    }
    const int64_t waited = now_ns() - t0;
    if (waited >= limit) return fail(CS_ERR_TIMEOUT, "cs_xchannel_wait: nothing arrived in time");
    if (waited > 200000) {   // after 0.2 ms of polling, sleep between looks
      timespec ts = {0, 50000};
      nanosleep(&ts, nullptr);
    }
  }
} CS_CATCH_ALL("cs_xchannel_wait")

cs_status cs_xchannel_forward(cs_xchannel* x, int32_t slot, const int64_t* placeholder_index, void* dst_seq,
                              int64_t dst_rows, int32_t* err_flag, void* consumer_stream) try {
  XSlot* s = nullptr;
  if (cs_status st = xslot(x, slot, "cs_xchannel_forward", &s)) return st;
  if (dst_rows < 0) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_forward: negative size");
  if (s->state.load(std::memory_order_acquire) != CS_XSLOT_READY)
    return fail(CS_ERR_INVALID_ARG, "cs_xchannel_forward: nothing has arrived in this slot");
  hipStream_t cons = static_cast<hipStream_t>(consumer_stream);
  if (s->n_rows > 0) {
    if (!placeholder_index || !dst_seq) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_forward: NULL argument");
    if (reinterpret_cast<uintptr_t>(dst_seq) & 15) return fail(CS_ERR_INVALID_ARG, "cs_xchannel_forward: dst_seq must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(placeholder_index) & 7) || (reinterpret_cast<uintptr_t>(err_flag) & 3))
      return fail(CS_ERR_INVALID_ARG, "cs_xchannel_forward: misaligned index or flag pointer");
  }
  // everything above returns with the slot still READY: a rejected call can be repeated
  s->state.store(CS_XSLOT_DRAINING, std::memory_order_release);
  if (s->n_rows > 0) {
    const int64_t row_bytes = (int64_t)s->hidden * (s->dtype == CS_BF16 ? 2 : 4);
    if (cs_status st = launch_scatter_rows(x->pool + (size_t)slot * x->ctl->slot_stride, placeholder_index, dst_seq,
                                           s->n_rows, dst_rows, row_bytes, err_flag, cons)) {
      s->state.store(CS_XSLOT_READY, std::memory_order_release);
      return st;
    }
  }
  const hipError_t he = hipLaunchHostFunc(cons, on_placed, &x->args[slot]);
  if (he != hipSuccess) {
    // the scatter may be running: the slot must not be handed back before it ends
    (void)hipStreamSynchronize(cons);
    on_placed(&x->args[slot]);
    return fail(CS_ERR_HIP, std::string("cs_xchannel_forward: hipLaunchHostFunc: ") + hipGetErrorString(he));
  }
  return CS_OK;
} CS_CATCH_ALL("cs_xchannel_forward")

cs_status cs_xchannel_release(cs_xchannel* x, int32_t slot) try {
  XSlot* s = nullptr;
  if (cs_status st = xslot(x, slot, "cs_xchannel_release", &s)) return st;
  int32_t want = CS_XSLOT_WRITING;
  if (!s->state.compare_exchange_strong(want, CS_XSLOT_FREE, std::memory_order_acq_rel))
    return fail(CS_ERR_INVALID_ARG, "cs_xchannel_release: only a slot that was acquired and not yet published can be released");
  return CS_OK;
} CS_CATCH_ALL("cs_xchannel_release")

cs_status cs_xchannel_describe(cs_xchannel* x, int32_t slot, int32_t* state, const void** dev_ptr, int64_t* n_rows,
                               int32_t* hidden, int32_t* dtype, int64_t* t_ready_ns, int64_t* t_placed_ns) try {
  XSlot* s = nullptr;
  if (cs_status st = xslot(x, slot, "cs_xchannel_describe", &s)) return st;
  const int32_t stt = s->state.load(std::memory_order_acquire);
  if (state) *state = stt;
  if (dev_ptr) *dev_ptr = x->pool + (size_t)slot * x->ctl->slot_stride;
  const bool has = stt == CS_XSLOT_PUBLISHING || stt == CS_XSLOT_READY || stt == CS_XSLOT_DRAINING;
  if (n_rows) *n_rows = has ? s->n_rows : 0;
  if (hidden) *hidden = has ? s->hidden : 0;
  if (dtype) *dtype = has ? s->dtype : 0;
  if (t_ready_ns) *t_ready_ns = s->t_ready_ns.load(std::memory_order_relaxed);
  if (t_placed_ns) *t_placed_ns = s->t_placed_ns.load(std::memory_order_relaxed);
  return CS_OK;
} CS_CATCH_ALL("cs_xchannel_describe")

}  // extern "C"
