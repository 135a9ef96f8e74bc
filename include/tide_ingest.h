/* Signal ingest: pinned host ring buffer -> asynchronous host-to-device copies on a copy stream of its own,
 * overlapped with the training step that runs on the caller's compute stream.
 *
 * In the paper's system the inference engine hands captured hidden states of accepted tokens to the
 * training process (Sec. 3.2, Fig. 3: the signals travel from the serving GPUs to the training GPU through
 * host memory).  This is the last hop before the hot path: the producer fills a pinned slot on the host,
 * the slot is copied to a device buffer the caller owns while the previous batch trains, and the compute
 * stream waits on the copy's event only when it reaches the step that consumes it.
 *
 * Ownership: the ring (pinned host memory from hipHostMalloc), one stream at the default priority and two
 * events per slot belong to the object and are released by tide_ingest_destroy.  Device buffers belong to
 * the caller.  Nothing here is called from inside a kernel launch path of the training step: create once,
 * then acquire / submit / wait / (poll) per batch.  Not thread-safe: one producer thread per object.
 * Every function returns 0 on success or a negative TIDE_INGEST_* code; tide_ingest_last_error() gives
 * the text of the last failure on this thread. */
#ifndef TIDE_INGEST_H_
#define TIDE_INGEST_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIDE_INGEST_OK 0
#define TIDE_INGEST_ERR_NULL (-1)
#define TIDE_INGEST_ERR_ARG (-2)
#define TIDE_INGEST_ERR_HIP (-4)
#define TIDE_INGEST_ERR_BUSY (-5)      /* no free slot / slot not in the state the call needs */

typedef struct tide_ingest tide_ingest;

/* n_slots (2..64) pinned slots of slot_bytes each on the current device. */
int tide_ingest_create(tide_ingest **out, size_t slot_bytes, int32_t n_slots);
int tide_ingest_destroy(tide_ingest *q);

/* Next free slot for the producer: *slot gets its index, *host_ptr the pinned memory to fill (slot_bytes).
 * A slot whose copy has completed is recycled here (the completion is polled, never waited for).
 * TIDE_INGEST_ERR_BUSY when every slot is still filling or copying. */
int tide_ingest_acquire(tide_ingest *q, int32_t *slot, void **host_ptr);

/* Enqueue the copy of the first `bytes` of the slot to device_dst (DEVICE pointer, caller-owned, must stay
 * valid until the copy completed) on the copy stream and record the slot's event.  Returns at once.
 * The copy OVERWRITES device_dst, so it must not start while earlier work still reads that buffer (a training
 * step enqueued before, not yet finished, that consumed the buffer's previous contents: the usual state of a
 * device double buffer driven without host synchronisation).  after_reader != 0: the copy is ordered after
 * everything enqueued so far on reader_stream (a hipStream_t, NULL = the default stream), by an event recorded
 * there now that the copy stream waits for.  after_reader == 0: no ordering, reader_stream is ignored; the
 * caller guarantees that nothing in flight reads device_dst. */
int tide_ingest_submit(tide_ingest *q, int32_t slot, void *device_dst, size_t bytes, void *reader_stream,
                       int32_t after_reader);

/* Make `compute_stream` (a hipStream_t) wait for the slot's copy: work enqueued on it afterwards sees the
 * data.  Does not block the host. */
int tide_ingest_wait(tide_ingest *q, int32_t slot, void *compute_stream);

/* 1 if the slot's copy has completed, 0 if it is still in flight (host-side poll, no blocking). */
int tide_ingest_done(tide_ingest *q, int32_t slot);

const char *tide_ingest_last_error(void);

#ifdef __cplusplus
}
#endif
#endif  /* TIDE_INGEST_H_ */
