// Pinned host ring -> asynchronous H2D copies on a copy stream (see include/tide_ingest.h).
#include "../../include/tide_ingest.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <new>

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

enum SlotState { kFree = 0, kFilling = 1, kCopying = 2 };

}  // namespace

struct tide_ingest {
  size_t slot_bytes;
  int n_slots;
  int device;
  char* ring;             // pinned
  hipStream_t copy_stream;
  hipEvent_t events[64];
  hipEvent_t reader_events[64];   // recorded on the consumer's stream: the last reader of a slot's destination
  int state[64];
  int next;               // round-robin start of the search for a free slot
};

#define ING_HIP(call, what)                                                                   \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess) return fail(TIDE_INGEST_ERR_HIP, "%s: %s", what, hipGetErrorString(e_)); \
  } while (0)

extern "C" {

const char* tide_ingest_last_error(void) { return g_err; }

int tide_ingest_create(tide_ingest** out, size_t slot_bytes, int32_t n_slots) {
  if (!out) return fail(TIDE_INGEST_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (slot_bytes == 0 || n_slots < 2 || n_slots > 64) return fail(TIDE_INGEST_ERR_ARG, "slot_bytes must be > 0 and n_slots in [2, 64]");
  tide_ingest* q = new (std::nothrow) tide_ingest();
  if (!q) return fail(TIDE_INGEST_ERR_HIP, "out of host memory");
  q->slot_bytes = slot_bytes;
  q->n_slots = n_slots;
  q->ring = nullptr;
  q->copy_stream = nullptr;
  q->next = 0;
  int made = 0;
  hipError_t e = hipGetDevice(&q->device);
  if (e == hipSuccess) e = hipHostMalloc((void**)&q->ring, slot_bytes * (size_t)n_slots, hipHostMallocDefault);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&q->copy_stream, hipStreamNonBlocking);   // default priority
  for (; e == hipSuccess && made < n_slots; ++made) {
    q->state[made] = kFree;
    e = hipEventCreateWithFlags(&q->events[made], hipEventDisableTiming);
    if (e != hipSuccess) break;
    e = hipEventCreateWithFlags(&q->reader_events[made], hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipEventDestroy(q->events[made]); break; }
  }
  if (e != hipSuccess) {
    for (int i = 0; i < made; ++i) { (void)hipEventDestroy(q->events[i]); (void)hipEventDestroy(q->reader_events[i]); }
    if (q->copy_stream) (void)hipStreamDestroy(q->copy_stream);
    if (q->ring) (void)hipHostFree(q->ring);
    delete q;
    return fail(TIDE_INGEST_ERR_HIP, "create: %s", hipGetErrorString(e));
  }
  *out = q;
  return TIDE_INGEST_OK;
}

int tide_ingest_destroy(tide_ingest* q) {
  if (!q) return fail(TIDE_INGEST_ERR_NULL, "queue is NULL");
  (void)hipStreamSynchronize(q->copy_stream);   // copies in flight read the ring
  for (int i = 0; i < q->n_slots; ++i) { (void)hipEventDestroy(q->events[i]); (void)hipEventDestroy(q->reader_events[i]); }
  (void)hipStreamDestroy(q->copy_stream);
  (void)hipHostFree(q->ring);
  delete q;
  return TIDE_INGEST_OK;
}

int tide_ingest_done(tide_ingest* q, int32_t slot) {
  if (!q) return fail(TIDE_INGEST_ERR_NULL, "queue is NULL");
  if (slot < 0 || slot >= q->n_slots) return fail(TIDE_INGEST_ERR_ARG, "slot out of range");
  if (q->state[slot] != kCopying) return q->state[slot] == kFree ? 1 : 0;
  const hipError_t e = hipEventQuery(q->events[slot]);
  if (e == hipSuccess) return 1;
  if (e == hipErrorNotReady) return 0;
  return fail(TIDE_INGEST_ERR_HIP, "event query: %s", hipGetErrorString(e));
}

int tide_ingest_acquire(tide_ingest* q, int32_t* slot, void** host_ptr) {
  if (!q || !slot || !host_ptr) return fail(TIDE_INGEST_ERR_NULL, "NULL argument");
  for (int k = 0; k < q->n_slots; ++k) {
    const int i = (q->next + k) % q->n_slots;
    if (q->state[i] == kCopying) {
      const int d = tide_ingest_done(q, i);
      if (d < 0) return d;
      if (d == 1) q->state[i] = kFree;
    }
    if (q->state[i] == kFree) {
      q->state[i] = kFilling;
      q->next = (i + 1) % q->n_slots;
      *slot = i;
      *host_ptr = q->ring + (size_t)i * q->slot_bytes;
      return TIDE_INGEST_OK;
    }
  }
  return fail(TIDE_INGEST_ERR_BUSY, "no free slot: %d slots are filling or copying", q->n_slots);
}

int tide_ingest_submit(tide_ingest* q, int32_t slot, void* device_dst, size_t bytes, void* reader_stream,
                       int32_t after_reader) {
  if (!q || !device_dst) return fail(TIDE_INGEST_ERR_NULL, "NULL argument");
  if (slot < 0 || slot >= q->n_slots) return fail(TIDE_INGEST_ERR_ARG, "slot out of range");
  if (bytes == 0 || bytes > q->slot_bytes) return fail(TIDE_INGEST_ERR_ARG, "bytes must be in [1, slot_bytes]");
  if (q->state[slot] != kFilling) return fail(TIDE_INGEST_ERR_BUSY, "slot %d was not acquired", slot);
  if (after_reader) {
    // the destination may still be read by work already enqueued on the consumer's stream (the step before last of a
    // device double buffer): the copy starts only after everything enqueued there so far
    ING_HIP(hipEventRecord(q->reader_events[slot], (hipStream_t)reader_stream), "reader event record");
    ING_HIP(hipStreamWaitEvent(q->copy_stream, q->reader_events[slot], 0), "copy stream wait");
  }
  ING_HIP(hipMemcpyAsync(device_dst, q->ring + (size_t)slot * q->slot_bytes, bytes, hipMemcpyHostToDevice, q->copy_stream), "H2D copy");
  ING_HIP(hipEventRecord(q->events[slot], q->copy_stream), "event record");
  q->state[slot] = kCopying;
  return TIDE_INGEST_OK;
}

int tide_ingest_wait(tide_ingest* q, int32_t slot, void* compute_stream) {
  if (!q) return fail(TIDE_INGEST_ERR_NULL, "queue is NULL");
  if (slot < 0 || slot >= q->n_slots) return fail(TIDE_INGEST_ERR_ARG, "slot out of range");
  if (q->state[slot] != kCopying) return fail(TIDE_INGEST_ERR_BUSY, "slot %d has no copy submitted", slot);
  ING_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, q->events[slot], 0), "stream wait");
  return TIDE_INGEST_OK;
}

}  // extern "C"
