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

#ifdef __cplusplus
}
#endif
#endif /* DMI_DEBUG_H */
