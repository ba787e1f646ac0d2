// Online phase of EC-SpMV for CDNA4 (gfx950): y = W x over the EC-CSR image (paper Section 7), plus the
// plain CSR comparison kernel and a streaming-read kernel that measures the achievable HBM read rate.
//
// One workgroup per row panel.  The workgroup stages x and the panel's tables in LDS once, then its
// wavefronts stream the panel's delta and value arrays with 128-bit loads, rebuild absolute columns with
// cross-lane prefix scans (DPP), gather x from LDS and accumulate in FP32.  A block unit reduces its 16 lanes and
// leaves one FP32 partial per (unit, row) in an LDS slot; a residual lane unit (16 entries of one row) leaves its
// own partial sum.  After a barrier the slots and partial sums of each row are added in a fixed order and the
// row is stored.  No atomics, no pre-zeroed y, bit-reproducible results.
//
// One kernel template covers the variants: which block sets the image holds (TM), 8- or 4-bit deltas (DB),
// buffer depths for launches that carry several SpMVs (BATCH), loads per thread of the staging phase (K),
// 1, 2, 4 or 8 right-hand sides (NB), FP16 or FP32 values (VW).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "ecspmv_format.h"
#include "launch.h"

namespace {

// ---- timeline stamps (only in the library built with -DECS_TRACE, which the timeline script loads).  Reading the
// clock is a scalar memory operation, and many of them per wavefront change what they measure, so a launch takes ONE
// stamp per wavefront, at the point the launch's `sel` names, beside the clock at the wavefront's first and last
// instruction; the script launches once per point.  Words per wavefront: [0] start, [1] the selected point, [2] end,
// [3] constant-rate clock at start, [4] at end (8 words reserved).
#ifdef ECS_TRACE
struct TraceRegs {
    uint64_t sel_time = 0;
    uint32_t sel = 0xFFFFFFFFu;
};
#define ECS_STAMP(c, k)                                                                                              \
    do {                                                                                                             \
        if ((c).tr.sel == (uint32_t)(k)) (c).tr.sel_time = __builtin_amdgcn_s_memtime();                             \
    } while (0)
#define ECS_TRACE_DRAIN(c, k)                                                                                        \
    do {                                                                                                             \
        if ((c).tr.sel == (uint32_t)(k)) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                           \
    } while (0)
#else
#define ECS_STAMP(c, k) ((void)0)
#define ECS_TRACE_DRAIN(c, k) ((void)0)
#endif

// ---- cross-lane helpers (DPP).  With bound_ctrl = 0 a lane whose source lane does not exist keeps `old`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int dpp_i(int old, int src)
{
    return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xF, false);
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f(float old, float src)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(src), CTRL, ROW_MASK, 0xF, false));
}

#ifndef ECS_D4
#define ECS_D4 1
#define ECS_D2 2
#define ECS_DR 1
#endif
#ifndef ECS_DR0B
#define ECS_DR0B 2
#endif
// Register buffers per set (4-, 2- and 1-grained).  Measured on the box: one buffer for the 4-grained and residual
// sets and two for the 2-grained set; deeper buffering takes the kernel past the next step in registers (fewer
// wavefronts per SIMD) and is slower.  An image with no blocks at all (only the residual set) leaves room for two
// residual buffers at under 64 VGPRs: faster inside a batch, where many wavefronts share a compute unit and each
// must keep more bytes on the way, slower for a lone launch, whose wavefronts have one or two chunks each.
constexpr int D4 = ECS_D4, D2 = ECS_D2, DR = ECS_DR, DR0B = ECS_DR0B;

constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118;
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;
constexpr int DPP_QUAD_1032 = 0xB1, DPP_QUAD_2301 = 0x4E, DPP_ROW_HALF_MIRROR = 0x141, DPP_ROW_MIRROR = 0x140;

// inclusive prefix sum over the 16 lanes of a DPP row
__device__ __forceinline__ int row16_incl_scan(int v)
{
    v += dpp_i<DPP_ROW_SHR1>(0, v);
    v += dpp_i<DPP_ROW_SHR2>(0, v);
    v += dpp_i<DPP_ROW_SHR4>(0, v);
    v += dpp_i<DPP_ROW_SHR8>(0, v);
    return v;
}

// inclusive prefix sum over the 64 lanes of the wavefront
__device__ __forceinline__ int wave64_incl_scan(int v)
{
    v = row16_incl_scan(v);
    v += dpp_i<DPP_ROW_BCAST15, 0xA>(0, v);   // rows 1 and 3 take the total of rows 0 and 2
    v += dpp_i<DPP_ROW_BCAST31, 0xC>(0, v);   // rows 2 and 3 take the total of rows 0..1
    return v;
}

// sum over the 16 lanes of a DPP row, result in every lane
__device__ __forceinline__ float row16_allreduce(float a)
{
    a += dpp_f<DPP_QUAD_1032>(0.0f, a);
    a += dpp_f<DPP_QUAD_2301>(0.0f, a);
    a += dpp_f<DPP_ROW_HALF_MIRROR>(0.0f, a);
    a += dpp_f<DPP_ROW_MIRROR>(0.0f, a);
    return a;
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return __half2float(__ushort_as_half((unsigned short)h));
}

// acc += w * x with FP16 inputs taken exactly and FP32 accumulation
__device__ __forceinline__ float fma_h(uint32_t w_bits, float xf, float acc)
{
    return fmaf(half_bits_to_float(w_bits), xf, acc);
}

// the NB right-hand sides of one column sit side by side in LDS (x[col * NB + b]): one LDS read fetches them all
template <int NB, int VW>
__device__ __forceinline__ void gather_x(const uint16_t *xs, uint32_t col, float (&xv)[NB])
{
    if constexpr (VW == 4) {
        const float *xf = reinterpret_cast<const float *>(xs);
        if constexpr (NB == 1) {
            xv[0] = xf[col];
        } else if constexpr (NB == 2) {
            const float2 w = *reinterpret_cast<const float2 *>(xf + 2u * col);
            xv[0] = w.x, xv[1] = w.y;
        } else {
#pragma unroll
            for (int q = 0; q < NB / 4; ++q) {
                const float4 w = *reinterpret_cast<const float4 *>(xf + NB * col + 4 * q);
                xv[4 * q] = w.x, xv[4 * q + 1] = w.y, xv[4 * q + 2] = w.z, xv[4 * q + 3] = w.w;
            }
        }
    } else if constexpr (NB == 1) {
        xv[0] = half_bits_to_float(xs[col]);
    } else if constexpr (NB == 2) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(xs + 2u * col);
        xv[0] = half_bits_to_float(w & 0xFFFF), xv[1] = half_bits_to_float(w >> 16);
    } else if constexpr (NB == 4) {
        const uint2 w = *reinterpret_cast<const uint2 *>(xs + 4u * col);
        xv[0] = half_bits_to_float(w.x & 0xFFFF), xv[1] = half_bits_to_float(w.x >> 16);
        xv[2] = half_bits_to_float(w.y & 0xFFFF), xv[3] = half_bits_to_float(w.y >> 16);
    } else {
        const uint4 w = *reinterpret_cast<const uint4 *>(xs + 8u * col);
        xv[0] = half_bits_to_float(w.x & 0xFFFF), xv[1] = half_bits_to_float(w.x >> 16);
        xv[2] = half_bits_to_float(w.y & 0xFFFF), xv[3] = half_bits_to_float(w.y >> 16);
        xv[4] = half_bits_to_float(w.z & 0xFFFF), xv[5] = half_bits_to_float(w.z >> 16);
        xv[6] = half_bits_to_float(w.w & 0xFFFF), xv[7] = half_bits_to_float(w.w >> 16);
    }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 128-bit streaming load: every byte of the image is used once, so it is marked non-temporal
__device__ __forceinline__ uint4 load16(const uint8_t *p)
{
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ uint32_t load4(const uint8_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
}

__device__ __forceinline__ uint32_t load2(const uint8_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(p));
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 load8(const uint8_t *p)
{
    const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
    return make_uint2(t.x, t.y);
}

// A pointer put together from integers is one into global memory (the compiler would otherwise have to use the
// slower generic loads and stores for it)
template <class T>
__device__ __forceinline__ T *global_ptr(uint64_t bits)
{
    typedef T __attribute__((address_space(1))) * in_global;
    return (T *)(in_global)bits;
}

struct Ctx {
    const uint8_t *panel;      // global
    const uint16_t *xs;        // LDS: x as FP16 bits
    const uint8_t *meta;       // LDS copy of the panel's meta region
    float *slots;              // LDS partial sums
    uint32_t wave, lane, nwaves;
    uint32_t wshift;           // log2(nwaves) if the workgroup has a power-of-two number of wavefronts, else 32
    // quotient and remainder by the number of wavefronts: shifts in the usual case (a division by a run-time value is
    // some twenty instructions, and these sit on every wavefront's way to its first loads)
    __device__ __forceinline__ uint32_t div_nw(uint32_t a) const { return wshift < 32u ? a >> wshift : a / nwaves; }
    __device__ __forceinline__ uint32_t mod_nw(uint32_t a) const { return wshift < 32u ? a & (nwaves - 1u) : a % nwaves; }
#ifdef ECS_TRACE
    uint64_t *trace;           // this wavefront's 16 stamp words (null: no stamps)
    mutable TraceRegs tr;
#endif
};

// ---- g >= 2 block sets: a DPP row of 16 lanes takes one unit (64 columns), 4 columns per lane; a wavefront
// takes a chunk of 4 consecutive units.  DB = width of a delta index in bits (8 or 4).
// VW = bytes per value: 2 (FP16) or 4 (FP32)
template <int G, int VW>
struct UnitRegs {
    uint32_t d, d_hi;      // 4 indices: 4 delta bytes, or 4 nibbles in the low half, or (d, d_hi) = 4 16-bit columns
    uint4 v[G * VW / 4];   // 4 * G values of this lane
};

// Unconditional: DPP rows beyond the last unit of the set re-read that last unit (and ignore it), so that the
// number of loads in flight never depends on data and waits can name exact counts.
template <int G, int DB, int VW>
__device__ __forceinline__ void load_unit(const Ctx &c, uint32_t bd_off, uint32_t bv_off, uint32_t u, uint32_t nu,
                                          UnitRegs<G, VW> &r)
{
    const uint32_t j = c.lane & 15;
    const uint32_t uu = min(u, nu - 1u);
    // one 32-bit offset from the (wave-uniform) panel pointer per load: scalar base + vector offset addressing
    const uint32_t od = bd_off + (8u * DB) * uu + (DB / 2u) * j;
    const uint32_t ov = bv_off + (64u * VW * G) * uu + 16u * j;
    if constexpr (DB == 16) {
        const uint2 t = load8(c.panel + od);
        r.d = t.x, r.d_hi = t.y;
    } else if constexpr (DB == 8) {
        r.d = load4(c.panel + od);
    } else {
        r.d = load2(c.panel + od);
    }
#pragma unroll
    for (int k = 0; k < G * VW / 4; ++k) r.v[k] = load16(c.panel + (ov + 256u * k));
}

template <int G, int DB, int NB, int VW>
__device__ __forceinline__ void compute_unit(const Ctx &c, const uint16_t *utab, uint32_t u, uint32_t nu,
                                             const UnitRegs<G, VW> &r)
{
    const uint32_t j = c.lane & 15;
    const bool active = u < nu;
    const uint32_t uu = min(u, nu - 1u);
    // delta decode: local prefix over the lane's 4 columns, exclusive scan over the 16 lanes, unit base
    uint32_t rel[4], start;
    const uint16_t *ue = utab + uu * (1 + G);
    if constexpr (DB == 16) {                       // the indices are the columns: nothing to add up
        rel[0] = r.d & 0xFFFFu, rel[1] = r.d >> 16, rel[2] = r.d_hi & 0xFFFFu, rel[3] = r.d_hi >> 16;
        start = 0;
    } else {
        constexpr uint32_t DM = (1u << DB) - 1u;
        rel[0] = r.d & DM;
        rel[1] = rel[0] + ((r.d >> DB) & DM);
        rel[2] = rel[1] + ((r.d >> (2 * DB)) & DM);
        rel[3] = rel[2] + ((r.d >> (3 * DB)) & DM);
        const int incl = row16_incl_scan((int)rel[3]);
        start = (uint32_t)ue[0] + (uint32_t)incl - rel[3];
    }
    float xv[4][NB];
#pragma unroll
    for (int k = 0; k < 4; ++k) gather_x<NB, VW>(c.xs, start + rel[k], xv[k]);
    float acc[G][NB];
#pragma unroll
    for (int q = 0; q < G; ++q)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[q][b] = 0.0f;
#pragma unroll
    for (int f = 0; f < 4 * G; ++f) {                              // f = column * G + row
        if constexpr (VW == 2) {
            const uint4 q = r.v[f >> 3];
            const uint32_t word = ((f >> 1) & 3) == 0 ? q.x : ((f >> 1) & 3) == 1 ? q.y : ((f >> 1) & 3) == 2 ? q.z : q.w;
            const uint32_t hb = (f & 1) ? (word >> 16) : (word & 0xFFFF);
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[f % G][b] = fma_h(hb, xv[f / G][b], acc[f % G][b]);
        } else {
            const uint4 q = r.v[f >> 2];
            const uint32_t word = (f & 3) == 0 ? q.x : (f & 3) == 1 ? q.y : (f & 3) == 2 ? q.z : q.w;
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[f % G][b] = fmaf(__uint_as_float(word), xv[f / G][b], acc[f % G][b]);
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int q = 0; q < G; ++q) acc[q][b] = row16_allreduce(acc[q][b]);
        float out = acc[0][b];
#pragma unroll
        for (int q = 1; q < G; ++q) out = (j == (uint32_t)q) ? acc[q][b] : out;
        if (active && j < (uint32_t)G) c.slots[(uint32_t)ue[1 + j] * NB + b] = out;
    }
}

// A set's chunks c0, c0 + W, c0 + 2W, ... belong to this wavefront.  DEPTH register buffers take turns: all are
// requested before anything is computed, and each is refilled right after it has been consumed, so a wavefront
// always has its next DEPTH chunks on the way (the double buffering of Section 7, deeper and without copies).
// STRAIGHT: the chunks requested in the prologue are computed by run_first(), before any set issues further loads.
template <int G, int DB, int DEPTH, int NB, int VW, bool STRAIGHT = false>
struct BlockSet {
    UnitRegs<G, VW> buf[DEPTH];
    uint32_t nu, n, c0, bd_off, bv_off;
    const uint16_t *utab;

    __device__ __forceinline__ uint32_t unit_of(const Ctx &c, uint32_t i) const
    {
        return 4u * (c0 + i * c.nwaves) + (c.lane >> 4);
    }
    // `dealt`: chunks of the sets handled before this one.  The chunks of all sets are dealt to the wavefronts as one
    // round-robin sequence, so that the odd chunks of different sets go to different wavefronts.
    __device__ __forceinline__ void prologue(const Ctx &c, const uint32_t *hdr, int t, uint32_t &dealt)
    {
        nu = hdr[PH_NUNITS + t];
        bd_off = hdr[PH_BD_OFF + t];
        bv_off = hdr[PH_BV_OFF + t];
        utab = reinterpret_cast<const uint16_t *>(c.meta + hdr[PH_UTAB_OFF + t]);
        const uint32_t nch = (nu + 3u) >> 2;
        c0 = c.mod_nw(c.wave + c.nwaves - c.mod_nw(dealt));
        dealt += nch;
        n = nch > c0 ? c.div_nw(nch - c0 + c.nwaves - 1u) : 0u;
        // Every buffer is requested whether or not this wavefront has that many chunks (a missing chunk reads the
        // panel header instead): every wavefront then enters the loop below with the same loads in flight, which
        // keeps the wait counts exact.
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const bool have = (uint32_t)d < n;
            load_unit<G, DB, VW>(c, have ? bd_off : 0u, have ? bv_off : 0u, have ? unit_of(c, d) : 0u, have ? nu : 1u, buf[d]);
        }
    }
    // The chunks requested in the prologue are computed (run_first, every set in turn) before any set issues a
    // further load, so that every path to each of these computations has the same loads in flight.  Otherwise, where
    // paths with different loads in flight meet (a refill under a condition, a loop and its tail), the compiler takes
    // the stricter wait, and the wait for one set's data turns into a wait for younger loads of other sets as well: a
    // block chunk then waits for the residual chunk's whole round trip instead of being computed under it.
    __device__ __forceinline__ void run_first(const Ctx &c)
    {
        if constexpr (STRAIGHT) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                if ((uint32_t)d < n) compute_unit<G, DB, NB, VW>(c, utab, unit_of(c, d), nu, buf[d]);
        }
    }
    __device__ __forceinline__ void run(const Ctx &c)
    {
        uint32_t i = 0;
        if constexpr (STRAIGHT) {
            if (n <= (uint32_t)DEPTH) return;
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                if ((uint32_t)(DEPTH + d) < n) load_unit<G, DB, VW>(c, bd_off, bv_off, unit_of(c, DEPTH + d), nu, buf[d]);
            i = DEPTH;
        }
        for (; i + 2 * DEPTH - 1 < n; i += DEPTH) {    // chunks i + DEPTH ... i + 2 DEPTH - 1 exist: unconditional refills
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                compute_unit<G, DB, NB, VW>(c, utab, unit_of(c, i + d), nu, buf[d]);
                load_unit<G, DB, VW>(c, bd_off, bv_off, unit_of(c, i + DEPTH + d), nu, buf[d]);
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (i + d < n) {
                compute_unit<G, DB, NB, VW>(c, utab, unit_of(c, i + d), nu, buf[d]);
                if (i + DEPTH + d < n) load_unit<G, DB, VW>(c, bd_off, bv_off, unit_of(c, i + DEPTH + d), nu, buf[d]);
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (i + DEPTH + d < n) compute_unit<G, DB, NB, VW>(c, utab, unit_of(c, i + DEPTH + d), nu, buf[d]);
    }
};

// ---- residual (1-grained) set: a wavefront takes a chunk of 64 lane units, 16 elements per lane.
template <int DB, int VW>
struct ChunkRegs {
    uint32_t d[DB / 2]; // 16 indices: 16 delta bytes, 16 nibbles, or 16 16-bit columns
    uint4 v[VW];        // 16 values: two or four 128-bit loads
};

// Residual chunk `ch` of a panel sits at res_off + ch * (delta bytes + value bytes of a chunk): its deltas, then its
// values with the k-th 128-bit load of lane l at k * 1024 + 16 * l (a last chunk of nl < 64 lane units: nl delta runs
// padded to 16 bytes, then the k-th load of lane l at 16 * nl * k + 16 * l).
template <int DB, int VW>
__device__ __forceinline__ void issue_chunk_loads(const Ctx &c, uint32_t od, uint32_t ov, uint32_t step, ChunkRegs<DB, VW> &r)
{
    if constexpr (DB == 16) {
        const uint4 t = load16(c.panel + od), u = load16(c.panel + (od + (step ? 16u : 0u)));
        r.d[0] = t.x, r.d[1] = t.y, r.d[2] = t.z, r.d[3] = t.w, r.d[4] = u.x, r.d[5] = u.y, r.d[6] = u.z, r.d[7] = u.w;
    } else if constexpr (DB == 8) {
        const uint4 t = load16(c.panel + od);
        r.d[0] = t.x, r.d[1] = t.y, r.d[2] = t.z, r.d[3] = t.w;
    } else {
        const uint2 t = load8(c.panel + od);
        r.d[0] = t.x, r.d[1] = t.y;
    }
#pragma unroll
    for (int k = 0; k < VW; ++k) r.v[k] = load16(c.panel + (ov + step * k));
}

// Lanes beyond the end of the last chunk load 16 zero bytes the panel keeps for them (zero deltas, zero values), so
// that the arithmetic needs no masking.  Unconditional, like load_unit.
template <int DB, int VW>
__device__ __forceinline__ void load_chunk(const Ctx &c, uint32_t res_off, uint32_t zero_off, uint32_t ch, uint32_t nlanes,
                                           ChunkRegs<DB, VW> &r)
{
    const uint32_t nl = min(64u, nlanes - 64u * ch);
    const bool active = c.lane < nl;
    // a last chunk with fewer than 64 lane units is stored tightly
    const bool tight = nl < 64u;
    const uint32_t base = res_off + (128u * DB + 1024u * VW) * ch;
    const uint32_t od = active ? base + (2u * DB) * c.lane : zero_off;
    const uint32_t ov = active ? base + (tight ? ((2u * DB) * nl + 15u) / 16u * 16u : 128u * DB) + 16u * c.lane : zero_off;
    issue_chunk_loads<DB, VW>(c, od, ov, active ? (tight ? 16u * nl : 1024u) : 0u, r);
}

// One partial sum per lane unit goes to LDS (`part`, indexed by the lane unit's position in the residual stream); a
// row's lane units are consecutive, so the final pass adds a range of them.  No cross-lane reduction is needed here.
template <int DB, bool FENCE, int NB, int VW>
__device__ __forceinline__ void compute_chunk(const Ctx &c, const EcsRChunk *rch, const EcsREntry *ren, float *part,
                                              uint32_t ch, const ChunkRegs<DB, VW> &r)
{
    if constexpr (DB == 4 && NB == 1 && VW == 2) {
        // 4-bit deltas, FP16, one right-hand side: the 16 prefix sums of a lane are made eight at a time inside 32-bit
        // words, already doubled (they are byte offsets into the FP16 copy of x in LDS).  With lo / hi the even / odd
        // nibbles of a word spread to bytes (times two), T = bytewise running sum of lo + hi: byte k of T is the
        // prefix up to nibble 2k + 1, byte k of T - hi the prefix up to nibble 2k.  Eight deltas of at most 15 add
        // up to 120, doubled 240: a byte holds it.  Each gather address is then one add of a byte of such a word.
        constexpr uint32_t M2 = 0x1E1E1E1Eu;
        uint32_t pe[2], po[2];
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const uint32_t lo = (r.d[w] << 1) & M2, hi = (r.d[w] >> 3) & M2;
            uint32_t t = lo + hi;
            // t += t << 8; t += t << 16: written as two shift-adds (the compiler would make a 32-bit multiply by
            // 0x01010101 of it, which runs at a quarter of the rate)
            asm("v_lshl_add_u32 %0, %1, 8, %1" : "=v"(t) : "v"(t));
            asm("v_lshl_add_u32 %0, %1, 16, %1" : "=v"(t) : "v"(t));
            po[w] = t, pe[w] = t - hi;
        }
        const uint32_t tot0 = po[0] >> 24;                                 // twice the sum of the first eight deltas
        const int run = (int)((tot0 + (po[1] >> 24)) >> 1);
        const int incl = wave64_incl_scan(run);
        const uint64_t mask = rch[ch].head_mask;
        const uint64_t le = (c.lane == 63) ? ~0ull : ((2ull << c.lane) - 1ull);
        const int seg = __popcll(mask & le) - 1;
        const int start = ren[rch[ch].entry0 + seg].c + incl - run;
        const uint32_t base[2] = {2u * (uint32_t)start, 2u * (uint32_t)start + tot0};
        const uint8_t *xb = reinterpret_cast<const uint8_t *>(c.xs);
        float acc = 0.0f;
        const uint32_t vw[8] = {r.v[0].x, r.v[0].y, r.v[0].z, r.v[0].w, r.v[1].x, r.v[1].y, r.v[1].z, r.v[1].w};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t src = (i & 1) ? po[i >> 3] : pe[i >> 3];
            const uint32_t off = base[i >> 3] + ((src >> (8 * ((i & 7) >> 1))) & 0xFFu);
            const float xv = half_bits_to_float(*reinterpret_cast<const uint16_t *>(xb + off));
            const uint32_t word = vw[i >> 1];
            acc = fma_h((i & 1) ? (word >> 16) : (word & 0xFFFF), xv, acc);
        }
        part[64u * ch + c.lane] = acc;
        if constexpr (FENCE) __builtin_amdgcn_sched_barrier(0);
        return;
    }
    uint32_t rel[16];
    int start = 0;
    if constexpr (DB == 16) {                       // the indices are the columns: no prefix, no scan, no segment base
#pragma unroll
        for (int i = 0; i < 16; ++i) rel[i] = (r.d[i / 2] >> (16 * (i % 2))) & 0xFFFFu;
    } else {
        // lane-local inclusive prefix of the 16 deltas
        constexpr int PER = 32 / DB;                  // deltas per 32-bit word
        uint32_t run = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            run += (r.d[i / PER] >> (DB * (i % PER))) & ((1u << DB) - 1u);
            rel[i] = run;
        }
        // wave64 prefix scan of the lane totals; the segment's entry folds base column and earlier lanes
        const int incl = wave64_incl_scan((int)run);
        const uint64_t mask = rch[ch].head_mask;
        const uint64_t le = (c.lane == 63) ? ~0ull : ((2ull << c.lane) - 1ull);
        const int seg = __popcll(mask & le) - 1;
        start = ren[rch[ch].entry0 + seg].c + incl - (int)run;
    }
    float acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = 0.0f;
    uint32_t vw[4 * VW];
#pragma unroll
    for (int k = 0; k < VW; ++k) vw[4 * k] = r.v[k].x, vw[4 * k + 1] = r.v[k].y, vw[4 * k + 2] = r.v[k].z, vw[4 * k + 3] = r.v[k].w;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float xv[NB];
        gather_x<NB, VW>(c.xs, (uint32_t)(start + (int)rel[i]), xv);
        if constexpr (VW == 2) {
            const uint32_t word = vw[i >> 1];
            const uint32_t hb = (i & 1) ? (word >> 16) : (word & 0xFFFF);
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b] = fma_h(hb, xv[b], acc[b]);
        } else {
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b] = fmaf(__uint_as_float(vw[i]), xv[b], acc[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) part[(64u * ch + c.lane) * NB + b] = acc[b];
    // Nothing ties one chunk's arithmetic to the next: with two buffers the scheduler would interleave two chunks
    // and need 20 more registers, which costs a workgroup per compute unit where workgroups share one.
    if constexpr (FENCE) __builtin_amdgcn_sched_barrier(0);
}

template <int DB, int DEPTH, bool FENCE, int NB, int VW>
struct ResidualSet {
    ChunkRegs<DB, VW> buf[DEPTH];
    uint32_t nlanes, n, c0, res_off, zero_off;
    const EcsRChunk *rch;
    const EcsREntry *ren;
    float *part;

    __device__ __forceinline__ uint32_t chunk_of(const Ctx &c, uint32_t i) const { return c0 + i * c.nwaves; }
    __device__ __forceinline__ void prologue(const Ctx &c, const uint32_t *hdr, uint32_t dealt)
    {
        nlanes = hdr[PH_NRLANES];
        res_off = hdr[PH_RD_OFF];
        zero_off = hdr[PH_ZERO_OFF];
        part = c.slots + hdr[PH_NSLOTS] * NB;
        rch = reinterpret_cast<const EcsRChunk *>(c.meta + hdr[PH_RCHUNK_OFF]);
        ren = reinterpret_cast<const EcsREntry *>(c.meta + hdr[PH_RENTRY_OFF]);
        const uint32_t nch = (nlanes + 63u) >> 6;
        c0 = c.mod_nw(c.wave + c.nwaves - c.mod_nw(dealt));
        n = nch > c0 ? c.div_nw(nch - c0 + c.nwaves - 1u) : 0u;
        // unconditional, like the block sets: a missing chunk reads the panel header
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const bool have = (uint32_t)d < n;
            load_chunk<DB, VW>(c, have ? res_off : 0u, have ? zero_off : 0u, have ? chunk_of(c, d) : 0u,
                               have ? nlanes : 1u, buf[d]);
        }
    }
    // (stamps 5 + 2 k / 6 + 2 k: data of this wavefront's k-th chunk here / chunk done, k < 3)
    __device__ __forceinline__ void step(const Ctx &c, uint32_t k, int d)
    {
        if (k < 3) ECS_TRACE_DRAIN(c, 5 + 2 * k);
        if (k < 3) ECS_STAMP(c, 5 + 2 * k);
        compute_chunk<DB, FENCE, NB, VW>(c, rch, ren, part, chunk_of(c, k), buf[d]);
        if (k < 3) ECS_STAMP(c, 6 + 2 * k);
    }
    __device__ __forceinline__ void run(const Ctx &c)
    {
        uint32_t i = 0;
        for (; i + 2 * DEPTH - 1 < n; i += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                step(c, i + d, d);
                load_chunk<DB, VW>(c, res_off, zero_off, chunk_of(c, i + DEPTH + d), nlanes, buf[d]);
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (i + d < n) {
                step(c, i + d, d);
                if (i + DEPTH + d < n) load_chunk<DB, VW>(c, res_off, zero_off, chunk_of(c, i + DEPTH + d), nlanes, buf[d]);
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (i + DEPTH + d < n) step(c, i + DEPTH + d, d);
    }
};

// TM: bit t set = the image holds units of granularity 2 << t somewhere (the residual set is always handled);
// DB: width of the delta indices in bits; MODE: 0 = a launch that carries one SpMV (nothing of the batch table is
// compiled in: every instruction on the way to a wavefront's first loads counts, the scalar unit of a compute unit
// issues one instruction per cycle for all 16 wavefronts), 1 = several SpMVs, 2 = several SpMVs with the buffer
// depths that suit many workgroups per compute unit (residual-only images: deeper buffers; one block set: everything
// requested before the first barrier);
// K: 16-byte pieces of [tables | x] each thread brings to LDS before the generic loop takes the rest;
// NB: right-hand sides handled at once (x holds n rows of NB values, y m rows of NB values);
// VW: bytes per value of W, x and y (2 = FP16, 4 = FP32)
template <int TM, int DB, int MODE, int K, int NB, int VW>
__global__ __launch_bounds__(1024) void ecspmv_kernel(const uint32_t count, const uint32_t threads, const uint8_t *image0,
                                                      const uint16_t *x0, uint16_t *y0, const uint32_t n0,
                                                      const uint32_t panel_stride0, const uint32_t meta_stride0,
                                                      const uint32_t x_bytes0, const uint32_t block_end0,
                                                      const uint32_t row_stride0, const uint64_t trace_words,
                                                      const ecs::EcsBatch batch)
{
#ifdef ECS_TRACE
    const uint64_t t_start = __builtin_amdgcn_s_memtime(), t_start_real = __builtin_amdgcn_s_memrealtime();
#endif
    // which SpMV of the batch this workgroup works for (one item in the plain case)
    // What a lone launch needs (count, workgroup size, the first item) comes first in the kernel arguments, as
    // plain values the hardware can hand over in registers; the table behind them is read only by launches that
    // carry several SpMVs: one 16-byte vector load per lane fetches all of it (scalar loads by every wavefront of a
    // workgroup are served one wavefront after the other), and the item is then read out of the lanes.
    constexpr bool BATCH = MODE == 2, LONE = MODE == 0;
    ecs::EcsBatchItem it;
    it.image = image0, it.x = x0, it.y = y0, it.n = n0, it.panel_stride = panel_stride0, it.meta_stride = meta_stride0;
    it.x_bytes = x_bytes0, it.block_end = block_end0, it.row_stride = 0;
    uint32_t block0 = 0;
    if (!LONE && count > 1) {
        constexpr uint32_t kBatchOffset = 64, kPieces = (uint32_t)sizeof(ecs::EcsBatch) / 16u;   // 49
        static_assert(kBatchOffset % 16 == 0 && kPieces <= 64, "one 16-byte piece per lane");
        const uint8_t *ka = (const uint8_t *)__builtin_amdgcn_kernarg_segment_ptr();
        const uint32_t L = threadIdx.x & 63u;
        const uint4 t = reinterpret_cast<const uint4 *>(ka + kBatchOffset)[L < kPieces ? L : kPieces - 1u];
        // piece 3 j + 3 holds {meta_stride, x_bytes, block_end, row_stride} of item j
        const bool last_piece = L >= 3u && L % 3u == 0u && (L - 3u) / 3u + 1u < count;
        const uint32_t k = (uint32_t)__popcll(__ballot(last_piece && blockIdx.x >= t.z));
        auto rd = [&](uint32_t word, uint32_t lane) -> uint32_t { return (uint32_t)__builtin_amdgcn_readlane((int)word, (int)lane); };
        if (k) {
            block0 = rd(t.z, 3u * k);
            const uint32_t a = 3u * k + 1u;
            it.image = global_ptr<const uint8_t>((uint64_t)rd(t.x, a) | ((uint64_t)rd(t.y, a) << 32));
            it.x = global_ptr<const uint16_t>((uint64_t)rd(t.z, a) | ((uint64_t)rd(t.w, a) << 32));
            it.y = global_ptr<uint16_t>((uint64_t)rd(t.x, a + 1u) | ((uint64_t)rd(t.y, a + 1u) << 32));
            it.n = rd(t.z, a + 1u), it.panel_stride = rd(t.w, a + 1u);
            it.meta_stride = rd(t.x, a + 2u), it.x_bytes = rd(t.y, a + 2u), it.block_end = rd(t.z, a + 2u);
        }
    }
    const uint16_t *__restrict__ x = it.x;
    uint16_t *__restrict__ y = it.y;
    const uint32_t n = it.n * NB * (VW / 2), meta_stride = it.meta_stride, x_bytes = it.x_bytes;   // n: 2-byte units of x
    // several right-hand sides: elements from one row of X (and of Y) to the next.  NB when the launch handles all
    // columns of X; larger when X has more columns than this launch takes.
    uint32_t ld = NB;
    if constexpr (NB > 1) {
        const uint32_t given = row_stride0;
        if (given) ld = given;
    }

    extern __shared__ uint4 lds4[];
    uint8_t *lds = reinterpret_cast<uint8_t *>(lds4);
    uint16_t *xs = reinterpret_cast<uint16_t *>(lds);
    uint8_t *meta = lds + x_bytes;
    float *slots = reinterpret_cast<float *>(lds + x_bytes + meta_stride);

    const uint32_t tid = threadIdx.x, nt = threads;
    const uint8_t *panel = it.image + ECS_IMAGE_HEADER + (size_t)it.panel_stride * (blockIdx.x - block0);

    Ctx c;
    c.panel = panel;
    c.xs = xs;
    c.meta = meta;
    c.slots = slots;
    c.wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));      // wave-uniform: scalar arithmetic on it
    c.lane = tid & 63;
    c.nwaves = nt >> 6;
    c.wshift = (c.nwaves & (c.nwaves - 1u)) == 0u ? (uint32_t)__builtin_ctz(c.nwaves) : 32u;
#ifdef ECS_TRACE
    c.trace = (trace_words << 8) ? global_ptr<uint64_t>((trace_words << 8) >> 8) + ((size_t)blockIdx.x * 16u + c.wave) * 8u : nullptr;
    c.tr.sel = c.trace ? (uint32_t)(trace_words >> 56) : 0xFFFFFFFFu;      // the point to stamp rides in the top byte
#endif

    // Everything the workgroup needs first is requested at once: the panel header, and the panel's tables and x on
    // their way to LDS, as one list of 16-byte pieces [tables | x] with K pieces per thread.  These loads are
    // unconditional (indices clamped or folded), so none of them makes a later wait inexact; K is a template parameter,
    // the smallest that covers the list, because every wave-wide load costs issue time on the way to the first barrier
    // whether its lanes are needed or not.
    // The header travels through the vector memory path: lanes 0..7 of every wavefront load 16 bytes each (the other
    // lanes repeat them) and the words are then read out of the lanes into scalar registers.  Scalar loads of the same
    // 128 bytes by all wavefronts of a workgroup are served one wavefront after the other (measured: the last of 16
    // wavefronts has its header 1.4 us after the workgroup started, against 0.5 us this way).
    // (Measured and not kept: only the first four wavefronts staging all pieces.  The first barrier then passes 0.7 us
    // earlier, but those wavefronts request their chunks later, and when the chunks are requested is what decides.)
    // buffers per set: deeper where chunks are small and frequent, shallower where registers run out
    constexpr bool wide = (TM & 12) != 0;
    constexpr bool straight = !BATCH && NB == 1;
    BlockSet<16, DB, 1, NB, VW, straight> b16;
    BlockSet<8, DB, 1, NB, VW, straight> b8;
    BlockSet<4, DB, wide ? 1 : D4, NB, VW, straight> b4;
    BlockSet<2, DB, wide ? 2 : D2, NB, VW, straight> b2;
    ResidualSet<DB, wide ? 2 : (TM == 0 && BATCH ? DR0B : DR), TM == 0 && BATCH, NB, VW> rs;
    // A launch of an image with block sets that shares its compute units with few others requests the residual set's
    // first chunks only after the barrier: a wavefront cannot pass the barrier before its requests are out, with every
    // set requested up front the whole panel is on its way before anything is computed, and the block sets' first
    // chunks are computed while the residual chunk travels (run_first).  Measured: 3-5 % of a lone launch with one
    // block set, 2 % of a step (7 % of a 5120 x 5120 launch) with two, 6 % with three; with many workgroups per
    // compute unit (MODE 2) requesting everything first is the faster order.
    constexpr bool residual_late = TM != 0 && !BATCH && NB == 1 && VW == 2;
    const uint4 *p4 = reinterpret_cast<const uint4 *>(panel);
    const uint32_t nmeta = meta_stride / 16u;
    const uint32_t nvec = n / 8u;
    const bool x_fast = (reinterpret_cast<uintptr_t>(x) & 15) == 0 && nvec > 0 && ld == NB;
    const uint4 *xsrc = reinterpret_cast<const uint4 *>(x);
    const uint32_t ntot = nmeta + (x_fast ? nvec : 0u);         // nmeta >= 1
    uint4 *meta4 = reinterpret_cast<uint4 *>(meta);
    uint32_t hdr[ECS_PANEL_HEADER / 4];
    // Threads beyond the end of the list bring a piece a second time (same bytes to the same place): in a lone launch
    // all of them repeat the last piece (one cache line, few such threads); with several SpMVs in the launch there are
    // many such threads (K follows the widest x) and they are folded back onto the first 2^k <= ntot pieces, so that
    // the lanes of a wavefront write to different LDS addresses.  Both cost one or two instructions: this sits on
    // the way to the first loads of every wavefront.
    const bool wrap = !LONE && count > 1;
    const uint32_t fold = (1u << (31 - __builtin_clz(ntot))) - 1u;
    auto piece_index = [&](uint32_t k) -> uint32_t {
        const uint32_t idx = tid + k * nt;
        return idx < ntot ? idx : (wrap ? (idx & fold) : ntot - 1u);
    };
    auto piece = [&](uint32_t k) -> const uint4 * {
        const uint32_t idx = piece_index(k);
        return idx < nmeta ? p4 + idx : xsrc + (idx - nmeta);
    };
    ECS_STAMP(c, 22);           // just before the header request
    const uint4 hv = reinterpret_cast<const uint4 *>(panel)[c.lane & 7u];
    ECS_STAMP(c, 23);           // header requested
    uint4 s0 = *piece(0), s1 = s0, s2 = s0, s3 = s0;
    if constexpr (K > 1) s1 = *piece(1);
    if constexpr (K > 2) s2 = *piece(2), s3 = *piece(3);
    ECS_STAMP(c, 20);           // header and first pieces requested
    __builtin_amdgcn_sched_barrier(0);      // these loads do not wait for the header: keep them ahead of those that do
#pragma unroll
    for (int w = 0; w < (int)(ECS_PANEL_HEADER / 4); ++w) {
        const uint32_t part = (w & 3) == 0 ? hv.x : (w & 3) == 1 ? hv.y : (w & 3) == 2 ? hv.z : hv.w;
        hdr[w] = (uint32_t)__builtin_amdgcn_readlane((int)part, w >> 2);
    }

    // As soon as the header is here, the first chunks of every set are requested (one per register buffer), before
    // anything is computed and before the tables and x have even reached LDS.
    uint32_t dealt = 0;
    ECS_STAMP(c, 1);            // panel header here
    if constexpr ((TM & 8) != 0) b16.prologue(c, hdr, 3, dealt);
    if constexpr ((TM & 4) != 0) b8.prologue(c, hdr, 2, dealt);
    if constexpr ((TM & 2) != 0) b4.prologue(c, hdr, 1, dealt);
    if constexpr ((TM & 1) != 0) b2.prologue(c, hdr, 0, dealt);
    if constexpr (!residual_late) rs.prologue(c, hdr, dealt);
    ECS_STAMP(c, 2);            // first chunks of every set requested

#ifdef ECS_TRACE
    // (only meaningful for the residual-only kernel with one buffer: its three chunk loads stay in flight)
    if (c.tr.sel == 21u) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
#endif
    ECS_STAMP(c, 21);           // this wavefront's first piece here
    // tables and x into LDS
    // (no branches here either: with a store under a branch the compiler moves the load down to it and waits for
    // it there)
    auto place = [&](uint32_t k) -> uint4 * {
        const uint32_t idx = piece_index(k);
        return idx < nmeta ? meta4 + idx : lds4 + (idx - nmeta);
    };
    *place(0) = s0;
    if constexpr (K > 1) *place(1) = s1;
    if constexpr (K > 2) *place(2) = s2, *place(3) = s3;
    static_assert(K <= 4, "at most four pieces per thread are brought here");
    for (uint32_t idx = tid + (uint32_t)K * nt; idx < ntot; idx += nt) {
        if (idx < nmeta)
            meta4[idx] = p4[idx];
        else
            lds4[idx - nmeta] = xsrc[idx - nmeta];
    }
    // what 16-byte pieces do not cover: the last n % 8 entries of x, or all of x if it is not 16-byte aligned or its
    // rows are longer than the NB values this launch takes
    if (NB > 1 && ld != NB) {
        // one load of NB values per row of X where the alignment allows it (ld counts values of VW bytes)
        typedef uint16_t rowvec __attribute__((ext_vector_type(NB * VW / 2)));
        if ((reinterpret_cast<uintptr_t>(x) & (uint32_t)(VW * NB - 1)) == 0 && ld % NB == 0) {
            const rowvec *src = reinterpret_cast<const rowvec *>(x);
            rowvec *dst = reinterpret_cast<rowvec *>(xs);
            for (uint32_t i = tid; i < it.n; i += nt) dst[i] = src[i * (ld / NB)];
        } else if constexpr (VW == 2) {
            for (uint32_t i = tid; i < n; i += nt) xs[i] = x[(i / NB) * ld + (i % NB)];
        } else {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(x);
            uint32_t *dst = reinterpret_cast<uint32_t *>(xs);
            for (uint32_t i = tid; i < it.n * NB; i += nt) dst[i] = src[(i / NB) * ld + (i % NB)];
        }
    } else {
        for (uint32_t i = (x_fast ? nvec * 8u : 0u) + tid; i < n; i += nt) xs[i] = x[i];
    }
    ECS_STAMP(c, 3);            // this wavefront's pieces of the tables and x written to LDS
    __syncthreads();
    ECS_STAMP(c, 4);            // first barrier passed

    if constexpr (residual_late) rs.prologue(c, hdr, dealt);
    if constexpr ((TM & 8) != 0) b16.run_first(c);
    if constexpr ((TM & 4) != 0) b8.run_first(c);
    if constexpr ((TM & 2) != 0) b4.run_first(c);
    if constexpr ((TM & 1) != 0) b2.run_first(c);
    if constexpr ((TM & 8) != 0) b16.run(c);
    if constexpr ((TM & 4) != 0) b8.run(c);
    if constexpr ((TM & 2) != 0) b4.run(c);
    if constexpr ((TM & 1) != 0) b2.run(c);
    rs.run(c);
    ECS_STAMP(c, 11);           // all chunks of this wavefront done
    __syncthreads();
    ECS_STAMP(c, 12);           // second barrier passed

    // every row: add its slots and the partial sums of its lane units in a fixed order (16 lanes stride over them,
    // then a fixed tree), store FP16.  (Measured and not kept: a whole wavefront per row for long rows, 64 lanes
    // striding: 2 % slower on the decoder-layer shapes; four unconditional LDS reads issued ahead of the
    // additions, checked in the generated code: no difference, the final pass of one workgroup overlaps the chunks of
    // others.)
    const uint32_t nrows = hdr[PH_NROWS];
    const uint32_t *rowidx = reinterpret_cast<const uint32_t *>(meta + hdr[PH_ROWIDX_OFF]);   // the output row of each row
    const uint16_t *rowslot = reinterpret_cast<const uint16_t *>(meta + hdr[PH_ROWSLOT_OFF]);
    const uint32_t *rowlu = reinterpret_cast<const uint32_t *>(meta + hdr[PH_ROWLU_OFF]);
    const float *part = slots + hdr[PH_NSLOTS] * NB;
    const uint32_t j = tid & 15;
    for (uint32_t r = tid >> 4; r < nrows; r += nt >> 4) {
        float sum[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) sum[b] = 0.0f;
        if constexpr (TM != 0) {
            const uint32_t s0 = rowslot[r], s1 = rowslot[r + 1];
            for (uint32_t q = s0 + j; q < s1; q += 16)
#pragma unroll
                for (int b = 0; b < NB; ++b) sum[b] += slots[q * NB + b];
        }
        const uint32_t l0 = rowlu[r], l1 = rowlu[r + 1];
        for (uint32_t q = l0 + j; q < l1; q += 16)
#pragma unroll
            for (int b = 0; b < NB; ++b) sum[b] += part[q * NB + b];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float t = row16_allreduce(sum[b]);
            if constexpr (VW == 2) {
                if (j == 0) y[rowidx[r] * ld + b] = __half_as_ushort(__float2half_rn(t));
            } else {
                if (j == 0) reinterpret_cast<float *>(y)[rowidx[r] * ld + b] = t;
            }
        }
    }
#ifdef ECS_TRACE
    if (c.trace) {
        const uint64_t t_end = __builtin_amdgcn_s_memtime(), t_end_real = __builtin_amdgcn_s_memrealtime();
        if (c.lane == 0)
            c.trace[0] = t_start, c.trace[1] = c.tr.sel_time, c.trace[2] = t_end, c.trace[3] = t_start_real, c.trace[4] = t_end_real;
    }
#endif
}

// ---- plain CSR, one wavefront per row (comparison only)
__global__ __launch_bounds__(256) void csr_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                                                  const uint16_t *__restrict__ val, const uint16_t *__restrict__ x,
                                                  uint16_t *__restrict__ y, uint32_t m)
{
    const uint32_t row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    if (row >= m) return;
    const int32_t b = rowptr[row], e = rowptr[row + 1];
    float acc = 0.0f;
    for (int32_t p = b + (int32_t)lane; p < e; p += 64) acc = fma_h(val[p], half_bits_to_float(x[col[p]]), acc);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) y[row] = __half_as_ushort(__float2half_rn(acc));
}

// ---- streaming read: every byte once, non-temporal 128-bit loads as in the product kernel.  SLICED = false: grid-stride,
// four loads in flight per lane.  SLICED = true: every workgroup reads one contiguous slice of the buffer (as a
// workgroup of the product kernel reads its panel), two loads in flight per lane, which is the fastest way found to
// read 20-50 MB in a launch of its own.
template <bool SLICED>
__global__ __launch_bounds__(1024) void stream_read_kernel(const uint4 *__restrict__ buf, uint64_t nvec, uint32_t *__restrict__ out)
{
    uint32_t acc = 0;
    const uint8_t *bytes = reinterpret_cast<const uint8_t *>(buf);
    if (SLICED) {
        const uint64_t per_wg = (nvec + gridDim.x - 1) / gridDim.x;
        const uint64_t lo = per_wg * blockIdx.x, hi = lo + per_wg < nvec ? lo + per_wg : nvec;
        uint64_t i = lo + threadIdx.x;
        for (; i + blockDim.x < hi; i += 2 * blockDim.x) {
            const uint4 a = load16(bytes + 16 * i), b = load16(bytes + 16 * (i + blockDim.x));
            acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w;
        }
        if (i < hi) {
            const uint4 a = load16(bytes + 16 * i);
            acc ^= a.x ^ a.y ^ a.z ^ a.w;
        }
    } else {
        const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
        uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
        for (; i + 3 * stride < nvec; i += 4 * stride) {
            const uint4 a = load16(bytes + 16 * i), b = load16(bytes + 16 * (i + stride)), c = load16(bytes + 16 * (i + 2 * stride)),
                        d = load16(bytes + 16 * (i + 3 * stride));
            acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
        }
        for (; i < nvec; i += stride) {
            const uint4 a = load16(bytes + 16 * i);
            acc ^= a.x ^ a.y ^ a.z ^ a.w;
        }
    }
    __shared__ uint32_t red[16];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_down(acc, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = 0;
        for (uint32_t w = 0; w < (blockDim.x >> 6); ++w) r ^= red[w];
        out[blockIdx.x] = r;
    }
}

// ---- a launch that does nothing (one store per workgroup): what a launch of the product kernel's shape costs before
// any byte is read
__global__ __launch_bounds__(1024) void empty_kernel(uint32_t *__restrict__ out)
{
    if (threadIdx.x == 0) out[blockIdx.x] = blockIdx.x;
}

}  // namespace

namespace ecs {

#ifdef ECS_TRACE
// host-side cursor: every launch takes the next region (wgs_per_region x 256 words) until the buffer is used up
static uint64_t *g_trace_next = nullptr, *g_trace_end = nullptr;
static uint64_t g_region_words = 0, g_trace_sel = 0;
int set_trace_buffer(void *d_words, uint32_t regions, uint32_t wgs_per_region, uint32_t sel)
{
    g_trace_next = static_cast<uint64_t *>(d_words);
    g_trace_sel = sel & 0xFFu;
    g_region_words = (uint64_t)wgs_per_region * 128u;
    g_trace_end = g_trace_next ? g_trace_next + g_region_words * regions : nullptr;
    return 0;
}
static uint64_t next_trace_region(uint32_t grid)
{
    if (!g_trace_next || (uint64_t)grid * 128u > g_region_words || g_trace_next + g_region_words > g_trace_end) return 0;
    uint64_t *p = g_trace_next;
    g_trace_next += g_region_words;
    return reinterpret_cast<uint64_t>(p) | (g_trace_sel << 56);
}
#endif

template <int TM, int DB, int MODE, int K, int NB, int VW = 2>
static int launch_m(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, void *stream)
{
    static thread_local uint32_t attr_set_for = 0;
    if (lds_bytes > 65536 && lds_bytes > attr_set_for) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ecspmv_kernel<TM, DB, MODE, K, NB, VW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return (int)e;
        attr_set_for = lds_bytes;
    }
    const uint32_t grid = batch.item[batch.count - 1].block_end;
#ifdef ECS_TRACE
    const uint64_t trace_words = next_trace_region(grid);
#else
    const uint64_t trace_words = 0;
#endif
    hipLaunchKernelGGL((ecspmv_kernel<TM, DB, MODE, K, NB, VW>), dim3(grid), dim3(threads), lds_bytes, (hipStream_t)stream,
                       batch.count, threads, batch.item[0].image, batch.item[0].x, batch.item[0].y, batch.item[0].n,
                       batch.item[0].panel_stride, batch.item[0].meta_stride, batch.item[0].x_bytes, batch.item[0].block_end,
                       batch.item[0].row_stride, trace_words, batch);
    return (int)hipGetLastError();
}

// BATCH: the deeper-buffer variant for launches with many workgroups per compute unit; a launch that carries a single
// SpMV gets the variant with nothing of the batch table compiled in
template <int TM, int DB, bool BATCH, int K, int NB, int VW = 2>
static int launch_k(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, void *stream)
{
    if constexpr (BATCH) return launch_m<TM, DB, 2, K, NB, VW>(batch, threads, lds_bytes, stream);
    if (batch.count == 1) return launch_m<TM, DB, 0, K, NB, VW>(batch, threads, lds_bytes, stream);
    if constexpr (NB == 1) return launch_m<TM, DB, 1, K, NB, VW>(batch, threads, lds_bytes, stream);
    return (int)hipErrorInvalidValue;          // several right-hand sides: one matrix per launch
}

template <int TM, int DB, bool BATCH>
static int launch_b(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, void *stream)
{
    // staging pieces per thread: the largest [tables | x] list of the batch over the workgroup size
    uint32_t most = 1;
    for (uint32_t i = 0; i < batch.count; ++i) {
        const EcsBatchItem &it = batch.item[i];
        const bool aligned = (reinterpret_cast<uintptr_t>(it.x) & 15) == 0;
        const uint32_t pieces = it.meta_stride / 16u + (aligned ? it.n / 8u : 0u);
        most = pieces > most ? pieces : most;
    }
    const uint32_t per_thread = (most + threads - 1) / threads;
    if (per_thread <= 1) return launch_k<TM, DB, BATCH, 1, 1>(batch, threads, lds_bytes, stream);
    if (per_thread <= 2) return launch_k<TM, DB, BATCH, 2, 1>(batch, threads, lds_bytes, stream);
    return launch_k<TM, DB, BATCH, 4, 1>(batch, threads, lds_bytes, stream);
}

template <int TM>
static int launch_tm(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, uint32_t delta_bits, uint32_t value_bits,
                     void *stream)
{
    // FP32 values: one variant per set mask and delta width (widest staging, lone-launch buffer depths)
    if (value_bits == 32) {
        if (delta_bits == 16) return (int)hipErrorInvalidValue;
        return delta_bits == 4 ? launch_k<TM, 4, false, 4, 1, 4>(batch, threads, lds_bytes, stream)
                               : launch_k<TM, 8, false, 4, 1, 4>(batch, threads, lds_bytes, stream);
    }
    // index compression switched off (absolute 16-bit columns): the ablation point, one variant per set mask
    if (delta_bits == 16) return launch_k<TM, 16, false, 4, 1>(batch, threads, lds_bytes, stream);
    // Residual-only images and images with one block set have a second variant for launches that carry several
    // SpMVs.  The residual-only one (deeper buffers) pays once more than three 512-thread workgroups per compute
    // unit are launched (measured at 2, 3 and 7 per compute unit: slower, 1 % slower, faster).
    const uint32_t grid = batch.item[batch.count - 1].block_end;
    if ((TM == 0 && batch.count > 1 && grid > 768) || (TM == 1 && batch.count > 1))
        return delta_bits == 4 ? launch_b<TM, 4, TM <= 1>(batch, threads, lds_bytes, stream)
                               : launch_b<TM, 8, TM <= 1>(batch, threads, lds_bytes, stream);
    return delta_bits == 4 ? launch_b<TM, 4, false>(batch, threads, lds_bytes, stream)
                           : launch_b<TM, 8, false>(batch, threads, lds_bytes, stream);
}

// several right-hand sides: one matrix per launch, the widest staging variant, images with 8-grained sets at most
template <int TM, int DB, int VW = 2>
static int launch_nb(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, uint32_t nb, void *stream)
{
    switch (nb) {
    case 2: return launch_k<TM, DB, false, 4, 2, VW>(batch, threads, lds_bytes, stream);
    case 4: return launch_k<TM, DB, false, 4, 4, VW>(batch, threads, lds_bytes, stream);
    case 8: return launch_k<TM, DB, false, 4, 8, VW>(batch, threads, lds_bytes, stream);
    default: return (int)hipErrorInvalidValue;
    }
}

int launch_ecspmv_multi(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, uint32_t type_mask,
                        uint32_t delta_bits, uint32_t value_bits, uint32_t nb, void *stream)
{
    const int top = (type_mask & 4) ? 7 : (type_mask & 2) ? 3 : (type_mask & 1) ? 1 : 0;
    if (delta_bits == 16) return (int)hipErrorInvalidValue;          // the ablation point exists for one vector only
    if (value_bits == 32) {                          // FP32 values: images with 4-grained sets at most
        if (delta_bits == 4) {
            if (top == 3) return launch_nb<3, 4, 4>(batch, threads, lds_bytes, nb, stream);
            if (top == 1) return launch_nb<1, 4, 4>(batch, threads, lds_bytes, nb, stream);
            if (top == 0) return launch_nb<0, 4, 4>(batch, threads, lds_bytes, nb, stream);
            return (int)hipErrorInvalidValue;
        }
        if (top == 3) return launch_nb<3, 8, 4>(batch, threads, lds_bytes, nb, stream);
        if (top == 1) return launch_nb<1, 8, 4>(batch, threads, lds_bytes, nb, stream);
        if (top == 0) return launch_nb<0, 8, 4>(batch, threads, lds_bytes, nb, stream);
        return (int)hipErrorInvalidValue;
    }
    if (delta_bits == 4) {
        if (top == 7) return launch_nb<7, 4>(batch, threads, lds_bytes, nb, stream);
        if (top == 3) return launch_nb<3, 4>(batch, threads, lds_bytes, nb, stream);
        if (top == 1) return launch_nb<1, 4>(batch, threads, lds_bytes, nb, stream);
        return launch_nb<0, 4>(batch, threads, lds_bytes, nb, stream);
    }
    if (top == 7) return launch_nb<7, 8>(batch, threads, lds_bytes, nb, stream);
    if (top == 3) return launch_nb<3, 8>(batch, threads, lds_bytes, nb, stream);
    if (top == 1) return launch_nb<1, 8>(batch, threads, lds_bytes, nb, stream);
    return launch_nb<0, 8>(batch, threads, lds_bytes, nb, stream);
}

int launch_ecspmv(const EcsBatch &batch, uint32_t threads, uint32_t lds_bytes, uint32_t type_mask, uint32_t delta_bits,
                  uint32_t value_bits, void *stream)
{
    // one instantiation per highest granularity present: sets that do not occur cost no registers
    const int top = (type_mask & 8) ? 15 : (type_mask & 4) ? 7 : (type_mask & 2) ? 3 : (type_mask & 1) ? 1 : 0;
    switch (top) {
    case 15: return launch_tm<15>(batch, threads, lds_bytes, delta_bits, value_bits, stream);
    case 7: return launch_tm<7>(batch, threads, lds_bytes, delta_bits, value_bits, stream);
    case 3: return launch_tm<3>(batch, threads, lds_bytes, delta_bits, value_bits, stream);
    case 1: return launch_tm<1>(batch, threads, lds_bytes, delta_bits, value_bits, stream);
    default: return launch_tm<0>(batch, threads, lds_bytes, delta_bits, value_bits, stream);
    }
}

int launch_csr(const void *d_rowptr, const void *d_col, const void *d_val, const void *d_x, void *d_y, uint32_t m,
               void *stream)
{
    const uint32_t rows_per_wg = 4;
    hipLaunchKernelGGL(csr_kernel, dim3((m + rows_per_wg - 1) / rows_per_wg), dim3(64 * rows_per_wg), 0,
                       (hipStream_t)stream, (const int32_t *)d_rowptr, (const int32_t *)d_col, (const uint16_t *)d_val,
                       (const uint16_t *)d_x, (uint16_t *)d_y, m);
    return (int)hipGetLastError();
}

int launch_stream_read(const void *d_buf, uint64_t bytes, void *d_out, uint32_t num_wg, uint32_t threads, bool sliced,
                       void *stream)
{
    if (sliced)
        hipLaunchKernelGGL(stream_read_kernel<true>, dim3(num_wg), dim3(threads), 0, (hipStream_t)stream,
                           (const uint4 *)d_buf, bytes / 16, (uint32_t *)d_out);
    else
        hipLaunchKernelGGL(stream_read_kernel<false>, dim3(num_wg), dim3(threads), 0, (hipStream_t)stream,
                           (const uint4 *)d_buf, bytes / 16, (uint32_t *)d_out);
    return (int)hipGetLastError();
}

int launch_empty(void *d_out, uint32_t num_wg, uint32_t threads, void *stream)
{
    hipLaunchKernelGGL(empty_kernel, dim3(num_wg), dim3(threads), 0, (hipStream_t)stream, (uint32_t *)d_out);
    return (int)hipGetLastError();
}

int copy_to_device(void *d_dst, const void *h_src, uint64_t bytes, void *stream)
{
    hipError_t e = hipMemcpyAsync(d_dst, h_src, bytes, hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return (int)e;
    return (int)hipStreamSynchronize((hipStream_t)stream);
}

int current_device(int *dev) { return (int)hipGetDevice(dev); }

int device_lds_limit(int *bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    return (int)hipDeviceGetAttribute(bytes, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
}

}  // namespace ecs
