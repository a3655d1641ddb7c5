/*
 * dmi_debug.h -- hooks for tests of the capture-and-stage library; not part of the public ABI
 * of include/dmi.h (the symbols are exported from libdmi.so all the same).
 */
#ifndef DMI_DEBUG_H
#define DMI_DEBUG_H
#include "dmi.h"
#ifdef __cplusplus
extern "C" {
#endif

/* Fill both rings with one byte value (synchronous; nothing may be in flight).  Lets a test see
 * that every byte of every record, pads included, is written by the capture: the record layout
 * (dmi.h) says that every pad byte is zero. */
dmi_status_t dmi_debug_fill_rings(dmi_ring_t *ring, uint8_t value);

/* How many pageable buffers the exporter's copy stage has taken from the allocator, and how many
 * records found an idle buffer instead, since the ring was created [both host]. */
dmi_status_t dmi_debug_exporter_allocs(dmi_ring_t *ring, uint64_t *allocated, uint64_t *reused);

/* The next capture launch issued by the calling thread is timed by the hardware: start_event and
 * stop_event [hipEvent_t, created with timing enabled] take the time stamps at which that kernel
 * began to execute and ended, so that hipEventElapsedTime between them is the kernel's own
 * duration (what a profiler reports), without what two markers recorded around the call add.
 * One launch only; NULL, NULL cancels.  For benchmarks; thread local; not for launches of a
 * replayable step (a stream that is being captured records no events of this kind). */
dmi_status_t dmi_debug_time_next_launch(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* DMI_DEBUG_H */
