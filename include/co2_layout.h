/* co2_layout.h -- optional memory-layout service of libco2.so (MI355X, gfx950).
 *
 * Not part of the CO2 method and not needed by any entry point of co2.h, which
 * work on any device memory and never allocate.  These two calls are the only
 * ones in the library that allocate or free device memory.
 */
#ifndef CO2_LAYOUT_H_
#define CO2_LAYOUT_H_

#include <stddef.h>
#include <stdint.h>

#include "co2.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Buffers placed for the sweep: a service for callers that own their
 * allocation.
 *
 * co2_buffer_set_create allocates `count` device buffers of bytes[i] bytes
 * (HOST array) and stores their DEVICE addresses in bufs_out[i] (HOST array).
 * Each buffer is an ordinary flat, contiguous range of device addresses,
 * 4 KiB aligned, readable and writable by every kernel and copy on the current
 * device.  Physically, every buffer is cut into the same number P of pieces
 * (about piece_bytes each for the largest buffer; 0 = 64 MiB, the size that
 * measured fastest and most reproducible for multi-gigabyte buffers; must be a
 * multiple of 2 MiB) and the pieces are obtained from the driver in the order
 * piece 0 of every buffer, piece 1 of every buffer, ...: the parts of the
 * buffers that the sweep touches at the same time are then neighbours in
 * device memory, which makes the sweep's duration independent of what the
 * driver's allocator would hand out for K + 4 gigabyte-sized allocations
 * (measured at 1.3e9 elements per buffer with the default piece size: 11.8-12.1
 * ms per sweep at K = 8 in every set made, against 11.9-12.9 ms for plain
 * allocations; the piece size matters: 128 MiB pieces were 5 % slower every time).
 * Buffers of different element size (fp32 vectors and bf16 pseudo-gradients)
 * get pieces in the same proportion, so piece j always covers the same element
 * range.  Memory use: sum of bytes[i] rounded up to P * 2 MiB per buffer.
 *
 * Ownership: the set owns the memory until co2_buffer_set_destroy, which the
 * caller invokes after all work on the buffers has completed (it does not
 * synchronise).  These two calls are the only ones in the library that
 * allocate or free; they use HIP's virtual-memory-management calls on the
 * current device and return CO2_EHIP (co2_last_hip_error() holds the
 * hipError_t, e.g. out of memory) after releasing whatever they had obtained.
 */
#define CO2_MAX_BUFFER_SET 64
typedef struct co2_buffer_set co2_buffer_set;
int co2_buffer_set_create(int32_t count, const size_t* bytes, size_t piece_bytes, void** bufs_out,
                          co2_buffer_set** set_out);
int co2_buffer_set_destroy(co2_buffer_set* set);

#ifdef __cplusplus
}
#endif
#endif /* CO2_LAYOUT_H_ */
