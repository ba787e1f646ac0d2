// Host-side data structures of the offline phase (see encoder.cpp).
#ifndef ECSPMV_ENCODER_H
#define ECSPMV_ENCODER_H

#include <cstdint>
#include <vector>

#include "../../include/ecspmv.h"
#include "ecspmv_format.h"

namespace ecs {

struct Csr {
    int64_t m = 0, n = 0;
    int value_bits = 16;                // 16: FP16 bit patterns, 32: FP32 bit patterns (both held in 32-bit containers)
    std::vector<int64_t> rowptr;
    std::vector<int32_t> col;
    std::vector<uint32_t> val;
};

struct BuildParams {
    int delta_bits = 8;
    int max_granularity = 8;
    int max_rounds = 64;
    int num_panels = 0;
    int num_threads = 0;
    int threads_per_wg = 0;
    bool global_matching = false;
    bool reorder = true;
    bool keep_small_sets = false;
    bool cluster_rows = false;          // bring similar rows into the same panel before the panels are cut
};

struct Image {
    std::vector<uint8_t> bytes;
    int64_t m = 0, n = 0, nnz = 0;
    int num_panels = 0, threads_per_wg = 1024, delta_bits = 8, value_bits = 16;
    uint32_t panel_stride = 0, meta_stride = 0, max_slots = 0, lds_bytes = 0;
    uint32_t type_mask = 0;   // bit t set: some panel holds units of granularity 2 << t
    ecspmv_stats_t stats;
};

struct Triples {
    std::vector<int32_t> rows, cols;
    std::vector<uint32_t> vals;         // FP16 or FP32 bit patterns
};

struct BlockSets {
    std::vector<int32_t> g, rows, cols;
};

int csr_from_dense(const uint16_t *W, int64_t m, int64_t n, int64_t ld, int threads, Csr &out);
int csr_from_csr(const int64_t *rowptr, const int32_t *col, const uint16_t *val, int64_t m, int64_t n, Csr &out);
int csr_from_dense_f32(const uint32_t *W, int64_t m, int64_t n, int64_t ld, int threads, Csr &out);
int csr_from_csr_f32(const int64_t *rowptr, const int32_t *col, const uint32_t *val, int64_t m, int64_t n, Csr &out);
int build_image(const Csr &A, const BuildParams &bp, Image &out);
int walk_image(const Image &im, Triples *tri, BlockSets *bs);

}  // namespace ecs
#endif
