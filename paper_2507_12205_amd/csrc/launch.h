// Host-callable wrappers around the HIP kernels (kernels.hip).  Each returns a hipError_t value as int.
#ifndef ECSPMV_LAUNCH_H
#define ECSPMV_LAUNCH_H

#include <stdint.h>

namespace ecs {

// One SpMV of a batched launch.  The table is passed to the kernel by value (kernel arguments) and read there with one
// 16-byte vector load per lane, so an item is three 16-byte pieces and the table starts on a 16-byte boundary.
struct EcsBatchItem {
    const uint8_t *image;     // device image of the matrix
    const uint16_t *x;        // device, n FP16
    uint16_t *y;              // device, m FP16
    uint32_t n, panel_stride, meta_stride, x_bytes;
    uint32_t block_end;       // workgroups [previous item's block_end, block_end) belong to this item
    uint32_t row_stride;      // several right-hand sides: elements from one row of X (and Y) to the next; 0 = packed
};
#define ECS_MAX_BATCH 16
struct EcsBatch {
    uint32_t count, pad_[3];
    EcsBatchItem item[ECS_MAX_BATCH];
};
static_assert(sizeof(EcsBatchItem) == 48 && sizeof(EcsBatch) == 16 + 48 * ECS_MAX_BATCH, "layout the kernel reads");

// Launches one kernel for all items (count <= ECS_MAX_BATCH, same workgroup size for all).
int launch_ecspmv(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, uint32_t type_mask, uint32_t delta_bits,
                  uint32_t value_bits, void *stream);
// One matrix, nb = 2, 4 or 8 right-hand sides (x: n rows of nb values, y: m rows of nb values); type_mask must not
// have the bit of the 16-grained set, nor that of the 8-grained set with FP32 values.
int launch_ecspmv_multi(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, uint32_t type_mask,
                        uint32_t delta_bits, uint32_t value_bits, uint32_t nb, void *stream);
int launch_csr(const void *d_rowptr, const void *d_col, const void *d_val, const void *d_x, void *d_y, uint32_t m,
               void *stream);
int launch_stream_read(const void *d_buf, uint64_t bytes, void *d_out, uint32_t num_wg, uint32_t threads, bool sliced,
                       void *stream);
int launch_empty(void *d_out, uint32_t num_wg, uint32_t threads, void *stream);
int copy_to_device(void *d_dst, const void *h_src, uint64_t bytes, void *stream);
int device_lds_limit(int *bytes);
int current_device(int *dev);
#ifdef ECS_TRACE
// Timeline stamps: each of the next `regions` launches stamps point `sel` into its own region of d_words (device;
// regions x wgs_per_region x 128 uint64).  d_words = null switches the stamps off.  Not thread-safe (a measurement aid).
int set_trace_buffer(void *d_words, uint32_t regions, uint32_t wgs_per_region, uint32_t sel);
#endif

}  // namespace ecs
#endif
