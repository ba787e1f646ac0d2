// Device image layout of EC-CSR as this library stores it (shared by the host encoder and the HIP kernels).
//
// The paper's EC-CSR (Section 6.1) keeps, per block set, row_indices / block_indptr / base_indices /
// delta_indices / block_values.  The same information is laid out here for 64-wide wavefronts and
// 128-bit loads:
//
//   image  = [ImageHeader, 256 B] [panel 0] [panel 1] ... [panel P-1] [zeros]   each panel `panel_stride` bytes
//   panel  = [meta: PanelHeader + tables] [residual chunks] [deltas and values of each block set]
//
// A panel owns a set of output rows (a contiguous range, or rows brought together by similarity) and is processed by
// one workgroup, so y needs no atomics.
// Block sets inside a panel are kept apart by granularity (Section 6.1): g = 16, 8, 4, 2 and the 1-grained
// residual.  The unit of a g >= 2 set is 64 block columns (16 lanes x 4 columns): one 16-bit base column,
// 64 one-byte deltas (the first is 0, Section 6.2 worked example), 64*g FP16 values stored so that the k-th
// 128-bit load of lane j (j = 0..15) sits at byte k*256 + j*16 of the unit (the permutation of Section
// 6.3.2 for 16-byte vectors) and holds halfs [8k, 8k+8) of that lane's run values[(4j+c)*g + r].
// The unit of the residual set is a "lane unit": 16 consecutive elements of one row (16 delta bytes, 16 FP16
// values); 64 lane units form a chunk that one wavefront decodes with a prefix scan over lane totals.  Every lane
// unit leaves one FP32 partial sum in LDS; a row's lane units are consecutive, so the row's sum is a range of them.
//
// Value width: `value_bits` of the image header is 16 or 32 (the paper's two precisions).  With FP32 every value
// array is twice as long and a 128-bit load holds 4 values instead of 8: a unit has 256*g value bytes (the k-th load
// of lane j still at k*256 + j*16), a lane unit 64 (four loads per lane instead of two); x and y are FP32 as well.
//
// Delta width (Section 6.2, EC-CSR-8 / EC-CSR-4 of Section 8.2): `delta_bits` of the image header is 8 or 4.
// With 4 bits two deltas share a byte, the earlier one in the low nibble; a unit then has 32 delta bytes (2 per
// lane), a lane unit 8 and a residual chunk 512; the largest delta is 15 and everything else is unchanged.
// delta_bits = 16 switches index compression off (the first step of the paper's ablation, Section 8.3): every index is
// the 16-bit column itself, there are no gap fillers and no prefix scan; a unit has 128 index bytes (8 per lane), a lane
// unit 32 and a residual chunk 2048.
#ifndef ECSPMV_FORMAT_H
#define ECSPMV_FORMAT_H

#include <stdint.h>

#define ECS_MAGIC            0x52534345u /* "ECSR" */
#define ECS_VERSION          3u
#define ECS_IMAGE_HEADER     256u        /* bytes before panel 0 */
#define ECS_UNIT_COLS        64u         /* block columns per unit of a g >= 2 set */
#define ECS_LANE_ELEMS       16u         /* residual elements per lane unit */
#define ECS_CHUNK_LANES      64u         /* lane units per residual chunk */
#define ECS_MAX_DELTA(bits)  ((1u << (bits)) - 1u)   /* R_P - 1 (with 16 bits: no limit, columns are below 65536) */
#define ECS_UNIT_DBYTES(bits)  (8u * (bits))        /* delta bytes of a 64-column unit */
#define ECS_LANE_DBYTES(bits)  (2u * (bits))        /* delta bytes of a residual lane unit */
#define ECS_CHUNK_DBYTES(bits) (128u * (bits))      /* delta bytes of a full residual chunk */
#define ECS_NUM_BTYPES       4           /* t = 0..3  <->  g = 2, 4, 8, 16 */

/* Words (uint32) of the panel header, which occupies the first ECS_PANEL_HEADER bytes of a panel. */
#define ECS_PANEL_HEADER     128u
enum {
    PH_ROW0 = 0,        /* output row of the panel's first row (the rows of a panel are listed at PH_ROWIDX_OFF) */
    PH_NROWS = 1,       /* rows owned */
    PH_NSLOTS = 2,      /* FP32 partial-sum slots of the block sets, one per (unit, row); a row's slots are consecutive.
                           The residual set adds one partial sum per lane unit, kept after these in LDS. */
    PH_NRLANES = 3,     /* residual lane units */
    PH_NRENTRIES = 4,   /* residual row segments (one per row and chunk it appears in) */
    PH_ROWSLOT_OFF = 5, /* byte offset in panel: uint16 first slot of each row, nrows + 1 entries */
    PH_RCHUNK_OFF = 6,  /* byte offset in panel: EcsRChunk per residual chunk */
    PH_RENTRY_OFF = 7,  /* byte offset in panel: EcsREntry per residual row segment */
    PH_RD_OFF = 8,      /* byte offset in panel of residual chunk 0 */
    PH_RV_OFF = 9,      /* bytes from one residual chunk to the next: a chunk is the deltas of its 64 lane units (16, 8
                           or 32 B each) followed by their values, the k-th 128-bit load of lane l at k * 1024 + 16 * l.
                           A last chunk with nl < 64 lane units is stored tightly: nl delta runs (padded to 16 bytes), then
                           the k-th load of lane l at 16 * nl * k + 16 * l */
    PH_NUNITS = 10,     /* +t: units of granularity 2 << t */
    PH_UTAB_OFF = 14,   /* +t: byte offset in panel: per unit (1 + g) uint16 = base column, g slots */
    PH_BD_OFF = 18,     /* +t: byte offset in panel: 64 (8-bit) or 32 (4-bit) delta bytes per unit */
    PH_BV_OFF = 22,     /* +t: byte offset in panel: 128 * g value bytes per unit */
    PH_PANEL_BYTES = 26,
    PH_META_BYTES = 27,
    PH_ROWLU_OFF = 28,  /* byte offset in panel: uint32 first residual lane unit of each row, nrows + 1 entries */
    PH_ZERO_OFF = 29,   /* byte offset in panel of 16 zero bytes (what idle lanes of the last residual chunk load) */
    PH_ROWIDX_OFF = 30  /* byte offset in panel: uint32 output row of each of the panel's rows (the paper's row_indices,
                           Section 6.1): contiguous unless the rows were clustered before the panels were cut */
};

typedef struct EcsRChunk {
    uint64_t head_mask;  /* bit l set: lane unit l starts a row segment (bit 0 always set) */
    uint32_t entry0;     /* index of the first EcsREntry of this chunk */
    uint32_t nlanes;     /* lane units in this chunk (64 except the last) */
} EcsRChunk;

typedef struct EcsREntry {
    int32_t  c;          /* column before the segment's first element minus the sum of the deltas of all
                            earlier lanes of the chunk: col(l, k) = c + exclusive_scan(l) + local_prefix(k) */
    uint16_t reserved_;  /* 0 */
    uint16_t row_local;  /* row - PH_ROW0 (used by the host decoder only) */
} EcsREntry;

typedef struct EcsImageHeader {
    uint32_t magic, version;
    uint32_t m, n;
    uint32_t num_panels, threads_per_wg;
    uint32_t panel_stride, meta_stride;
    uint32_t max_slots, lds_bytes;
    uint64_t image_bytes, nnz;
    uint32_t delta_bits, value_bits;   /* value_bits: 16 (FP16 values, x, y) or 32 (FP32) */
} EcsImageHeader;

#endif
