// Host-callable wrappers around the HIP kernels (kernels.hip).  Each returns a hipError_t value as int.
#ifndef ECSPMV_LAUNCH_H
#define ECSPMV_LAUNCH_H

#include <stdint.h>

namespace ecs {

int launch_ecspmv(const void *d_image, const void *d_x, void *d_y, uint32_t n, uint32_t num_panels, uint32_t threads,
                  uint32_t panel_stride, uint32_t meta_stride, uint32_t lds_bytes, void *stream);
int launch_csr(const void *d_rowptr, const void *d_col, const void *d_val, const void *d_x, void *d_y, uint32_t m,
               void *stream);
int launch_stream_read(const void *d_buf, uint64_t bytes, void *d_out, uint32_t num_wg, void *stream);
int copy_to_device(void *d_dst, const void *h_src, uint64_t bytes, void *stream);
int device_lds_limit(int *bytes);

}  // namespace ecs
#endif
