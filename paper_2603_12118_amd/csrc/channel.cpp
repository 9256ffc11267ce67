// cs_channel: the embedding hand-off between an encoder task and an LLM task that run on two
// streams of one process on one GPU (Sec. 2.2 "Data Forwarding": the producer's tensor
// sits in a shared buffer, the consumer is told where; Sec. 2.1 "Request Lifecycle": executors wait
// for tensors that have not arrived).  Slots live in device memory; "arrival" is a HIP event the consumer's stream waits
// for, so neither side blocks the host and the rows never leave HBM.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>
#include <vector>

#include "common.h"

using namespace cs;

namespace {

struct Slot {
  int32_t state = CS_SLOT_FREE;
  hipEvent_t ready = nullptr;    // recorded by publish on the producer's stream
  hipEvent_t drained = nullptr;  // recorded by forward on the consumer's stream
  bool drained_pending = false;  // a forward has been enqueued since the slot was last acquired
  int64_t n_rows = 0;
  int32_t hidden = 0, dtype = CS_BF16;
  size_t bytes = 0;              // what acquire reserved
};

}  // namespace

struct cs_channel {
  std::mutex mu;
  unsigned char* pool = nullptr;
  size_t slot_bytes = 0;   // what a slot may hold, as asked for at create
  size_t slot_stride = 0;  // distance between slots in the pool
  int device = 0;
  std::vector<Slot> slots;
};

static void free_channel(cs_channel* ch) {
  if (!ch) return;
  for (Slot& s : ch->slots) {
    if (s.ready) (void)hipEventDestroy(s.ready);
    if (s.drained) (void)hipEventDestroy(s.drained);
  }
  if (ch->pool) (void)hipFree(ch->pool);
  delete ch;
}

static cs_status slot_of(cs_channel* ch, int32_t slot, const char* who, Slot** out) {
  if (!ch) return fail(CS_ERR_INVALID_ARG, std::string(who) + ": NULL channel");
  if (slot < 0 || slot >= (int32_t)ch->slots.size()) return fail(CS_ERR_INVALID_ARG, std::string(who) + ": no such slot");
  *out = &ch->slots[slot];
  return CS_OK;
}

extern "C" {

cs_status cs_channel_create(int32_t n_slots, size_t slot_bytes, cs_channel** out) try {
  if (!out) return fail(CS_ERR_INVALID_ARG, "cs_channel_create: NULL out");
  *out = nullptr;
  if (n_slots <= 0 || n_slots > CS_CHANNEL_MAX_SLOTS) return fail(CS_ERR_INVALID_ARG, "cs_channel_create: n_slots out of range");
  if (slot_bytes == 0 || slot_bytes > ((size_t)1 << 40) / (size_t)n_slots) return fail(CS_ERR_INVALID_ARG, "cs_channel_create: slot_bytes out of range");
  cs_channel* ch = new cs_channel();
  ch->slot_bytes = slot_bytes;
  ch->slot_stride = (slot_bytes + 255) & ~(size_t)255;  // every slot starts on a 256-byte boundary
  ch->slots.resize(n_slots);
  hipError_t he = hipGetDevice(&ch->device);
  if (he == hipSuccess) he = hipMalloc(reinterpret_cast<void**>(&ch->pool), ch->slot_stride * (size_t)n_slots);
  for (Slot& s : ch->slots) {
    if (he == hipSuccess) he = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming);
    if (he == hipSuccess) he = hipEventCreateWithFlags(&s.drained, hipEventDisableTiming);
  }
  if (he != hipSuccess) {
    free_channel(ch);
    return fail(CS_ERR_HIP, std::string("cs_channel_create: ") + hipGetErrorString(he));
  }
  *out = ch;
  return CS_OK;
} CS_CATCH_ALL("cs_channel_create")

void cs_channel_destroy(cs_channel* ch) { free_channel(ch); }

cs_status cs_channel_acquire(cs_channel* ch, size_t bytes, void* producer_stream, int32_t* slot, void** dev_ptr) try {
  if (!ch || !slot || !dev_ptr) return fail(CS_ERR_INVALID_ARG, "cs_channel_acquire: NULL argument");
  *slot = -1;
  *dev_ptr = nullptr;
  if (bytes == 0 || bytes > ch->slot_bytes) return fail(CS_ERR_WORKSPACE, "cs_channel_acquire: tensor does not fit a slot");
  std::lock_guard<std::mutex> lock(ch->mu);
  for (size_t i = 0; i < ch->slots.size(); ++i) {
    Slot& s = ch->slots[i];
    if (s.state != CS_SLOT_FREE) continue;
    // The rows the last consumer of this slot still reads must be read before the producer writes.
    if (s.drained_pending) {
      CS_HIP(hipStreamWaitEvent(static_cast<hipStream_t>(producer_stream), s.drained, 0));
      s.drained_pending = false;
    }
    s.state = CS_SLOT_WRITING;
    s.bytes = bytes;
    *slot = (int32_t)i;
    *dev_ptr = ch->pool + i * ch->slot_stride;
    return CS_OK;
  }
  return fail(CS_ERR_BUSY, "cs_channel_acquire: every slot is in use");
} CS_CATCH_ALL("cs_channel_acquire")

cs_status cs_channel_publish(cs_channel* ch, int32_t slot, int64_t n_rows, int32_t hidden, int32_t dtype, void* producer_stream) try {
  Slot* s = nullptr;
  if (cs_status st = slot_of(ch, slot, "cs_channel_publish", &s)) return st;
  if (dtype != CS_F32 && dtype != CS_BF16) return fail(CS_ERR_INVALID_ARG, "cs_channel_publish: dtype");
  if (n_rows < 0 || hidden <= 0) return fail(CS_ERR_INVALID_ARG, "cs_channel_publish: sizes");
  const size_t row_bytes = (size_t)hidden * (dtype == CS_BF16 ? 2 : 4);
  if (row_bytes % 16) return fail(CS_ERR_UNSUPPORTED, "cs_channel_publish: a row must be a multiple of 16 bytes");
  std::lock_guard<std::mutex> lock(ch->mu);
  if (s->state != CS_SLOT_WRITING) return fail(CS_ERR_INVALID_ARG, "cs_channel_publish: slot was not acquired");
  if ((size_t)n_rows > s->bytes / row_bytes) return fail(CS_ERR_SHAPE, "cs_channel_publish: more rows than were reserved");
  CS_HIP(hipEventRecord(s->ready, static_cast<hipStream_t>(producer_stream)));
  s->n_rows = n_rows;
  s->hidden = hidden;
  s->dtype = dtype;
  s->state = CS_SLOT_READY;
  return CS_OK;
} CS_CATCH_ALL("cs_channel_publish")

cs_status cs_channel_release(cs_channel* ch, int32_t slot, void* stream) try {
  Slot* s = nullptr;
  if (cs_status st = slot_of(ch, slot, "cs_channel_release", &s)) return st;
  std::lock_guard<std::mutex> lock(ch->mu);
  if (s->state == CS_SLOT_FREE) return fail(CS_ERR_INVALID_ARG, "cs_channel_release: slot is not in use");
  CS_HIP(hipEventRecord(s->drained, static_cast<hipStream_t>(stream)));
  s->drained_pending = true;
  s->state = CS_SLOT_FREE;
  return CS_OK;
} CS_CATCH_ALL("cs_channel_release")

cs_status cs_channel_describe(cs_channel* ch, int32_t slot, int32_t* state, const void** dev_ptr, int64_t* n_rows,
                              int32_t* hidden, int32_t* dtype, int32_t* arrived) try {
  Slot* s = nullptr;
  if (cs_status st = slot_of(ch, slot, "cs_channel_describe", &s)) return st;
  std::lock_guard<std::mutex> lock(ch->mu);
  if (state) *state = s->state;
  if (dev_ptr) *dev_ptr = ch->pool + (size_t)slot * ch->slot_stride;
  const bool ready = s->state == CS_SLOT_READY;
  if (n_rows) *n_rows = ready ? s->n_rows : 0;
  if (hidden) *hidden = ready ? s->hidden : 0;
  if (dtype) *dtype = ready ? s->dtype : 0;
  if (arrived) {
    *arrived = 0;
    if (ready) {
      const hipError_t he = hipEventQuery(s->ready);
      if (he == hipSuccess) *arrived = 1;
      else if (he != hipErrorNotReady) return fail(CS_ERR_HIP, std::string("cs_channel_describe: ") + hipGetErrorString(he));
    }
  }
  return CS_OK;
} CS_CATCH_ALL("cs_channel_describe")

cs_status cs_channel_forward(cs_channel* ch, int32_t slot, const int64_t* placeholder_index, void* dst_seq,
                             int64_t dst_rows, int32_t* err_flag, void* consumer_stream) try {
  Slot* s = nullptr;
  if (cs_status st = slot_of(ch, slot, "cs_channel_forward", &s)) return st;
  std::lock_guard<std::mutex> lock(ch->mu);
  if (s->state != CS_SLOT_READY) return fail(CS_ERR_INVALID_ARG, "cs_channel_forward: nothing was published in this slot");
  if (dst_rows < 0) return fail(CS_ERR_INVALID_ARG, "cs_channel_forward: negative size");
  hipStream_t cons = static_cast<hipStream_t>(consumer_stream);
  if (s->n_rows > 0) {
    if (!placeholder_index || !dst_seq) return fail(CS_ERR_INVALID_ARG, "cs_channel_forward: NULL argument");
    if (reinterpret_cast<uintptr_t>(dst_seq) & 15) return fail(CS_ERR_INVALID_ARG, "cs_channel_forward: dst_seq must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(placeholder_index) & 7) || (reinterpret_cast<uintptr_t>(err_flag) & 3))
      return fail(CS_ERR_INVALID_ARG, "cs_channel_forward: misaligned index or flag pointer");
    // Everything above returns with the slot still READY: a rejected call can be repeated.
    CS_HIP(hipStreamWaitEvent(cons, s->ready, 0));
    const int64_t row_bytes = (int64_t)s->hidden * (s->dtype == CS_BF16 ? 2 : 4);
    if (cs_status st = launch_scatter_rows(ch->pool + (size_t)slot * ch->slot_stride, placeholder_index, dst_seq, s->n_rows,
                                           dst_rows, row_bytes, err_flag, cons))
      return st;
    CS_HIP(hipEventRecord(s->drained, cons));
    s->drained_pending = true;
  }
  s->state = CS_SLOT_FREE;
  return CS_OK;
} CS_CATCH_ALL("cs_channel_forward")

}  // extern "C"
