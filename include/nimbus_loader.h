/*
 * nimbus_loader.h -- C ABI of the asynchronous weight loading of the Nimbus client
 * (arXiv 2411.15707, Section 3.2, paragraph "Asynchronous Weight Loading", and the
 * appendix on the client's burden, paragraph of the same name).
 *
 * What the paper fixes: the encrypted weights are produced once in the setup phase and are
 * larger than the shares they replace, so the client keeps only the weights of the layer it
 * is computing (or of a few layers) in fast memory and loads the next layer's weights from
 * slower storage while the current layer is still busy; the load is hidden behind that work.
 *
 * Here the fast memory is the GPU's HBM and the slower storage is pinned host memory: the
 * (prepared) weight buffer of layer i+1 is copied host -> device on a copy stream while the
 * kernels of layer i run on the compute stream.  A loader object keeps, per device slot,
 * the two events that order the streams:
 *     load(slot)     copy stream:    wait until the slot was released, copy, mark it loaded
 *     acquire(slot)  compute stream: wait until the slot is loaded
 *     release(slot)  compute stream: mark that the work enqueued so far was the last to read it
 * A typical loop over layers with two slots:
 *     load(0, layer 0)
 *     for i: load((i+1) % 2, layer i+1); acquire(i % 2); <enqueue layer i>; release(i % 2)
 *
 * Conventions:
 *   - the loader owns no device memory: slot buffers belong to the caller, and so does the
 *     host memory, which must be pinned (page-locked at allocation, e.g. hipHostMalloc) for
 *     the copy to run asynchronously;
 *   - streams are hipStream_t values (NULL = the default stream), all of default priority;
 *   - no call waits for the GPU; every function returns a nimbus_cop.h status code
 *     (NIMBUS_COP_OK = 0, NIMBUS_COP_ERR_INVALID_ARG for a null handle or pointer, a slot out
 *     of range or zero bytes, NIMBUS_COP_ERR_LAUNCH when the HIP runtime refuses a call);
 *   - one loader serves one (copy stream, compute stream) pair at a time and is not
 *     thread-safe; different loaders are independent.
 */
#ifndef NIMBUS_LOADER_H
#define NIMBUS_LOADER_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nimbus_loader nimbus_loader;

/* Creates a loader with `slots` device slots (1 <= slots <= 64) on the current device:
 * a small host object and two events per slot.  *out receives the handle. */
int nimbus_loader_create(int slots, nimbus_loader **out);

/* Destroys the loader's events and frees the host object.  Work already enqueued is not
 * affected (events that are still pending are released by the runtime when they complete).
 * NULL is allowed. */
int nimbus_loader_destroy(nimbus_loader *loader);

/* Enqueues on copy_stream: wait for the slot's last release (if any), copy `bytes` bytes
 * from src_host (pinned host memory) to dst_device, mark the slot loaded.
 * dst_device may differ from call to call; what is ordered is the slot number. */
int nimbus_loader_load(nimbus_loader *loader, int slot, void *dst_device, const void *src_host,
                       size_t bytes, void *copy_stream);

/* Makes the work enqueued on compute_stream after this call wait for the slot's last load.
 * A slot that was never loaded makes nothing wait. */
int nimbus_loader_acquire(nimbus_loader *loader, int slot, void *compute_stream);

/* Records on compute_stream that everything enqueued there so far has finished reading the
 * slot: the slot's next load waits for this point. */
int nimbus_loader_release(nimbus_loader *loader, int slot, void *compute_stream);

#ifdef __cplusplus
}
#endif
#endif /* NIMBUS_LOADER_H */
