// Offline phase of EC-SpMV on the host: row panels, hierarchical block extraction (paper Section 4,
// Algorithms 1 and 2), clipping into fixed-size units and ordering (Section 5), EC-CSR encoding with 8-bit
// delta indices, padding and the load permutation (Section 6), plus the decoder used for round-trip checks.
#include "encoder.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <exception>
#include <mutex>
#include <system_error>
#include <thread>

namespace ecs {

// ------------------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------------------

template <class F>
static void parallel_for(int64_t count, int threads, F &&body)
{
    if (count <= 0) return;
    threads = (int)std::max<int64_t>(1, std::min<int64_t>(threads, count));
    if (threads == 1) {
        for (int64_t i = 0; i < count; ++i) body(i);
        return;
    }
    // An exception in a worker (out of memory) must not end the process: the first one is kept, the other workers
    // stop taking items, and it is thrown again in the caller once every worker has been joined.  If a worker cannot
    // be started the ones already running do all the work.
    std::atomic<int64_t> next(0);
    std::atomic<bool> failed(false);
    std::exception_ptr first;
    std::mutex first_lock;
    auto work = [&]() {
        try {
            for (;;) {
                const int64_t i = next.fetch_add(1);
                if (i >= count || failed.load(std::memory_order_relaxed)) break;
                body(i);
            }
        } catch (...) {
            std::lock_guard<std::mutex> g(first_lock);
            if (!first) first = std::current_exception();
            failed.store(true);
        }
    };
    std::vector<std::thread> pool;
    pool.reserve(threads);
    for (int t = 0; t + 1 < threads; ++t) {
        try {
            pool.emplace_back(work);
        } catch (const std::system_error &) {
            break;
        }
    }
    work();                                           // the calling thread is the last worker
    for (auto &th : pool) th.join();
    if (first) std::rethrow_exception(first);
}

static inline uint32_t align_up(uint32_t v, uint32_t a) { return (v + a - 1) / a * a; }

static int resolve_threads(int req)
{
    if (req > 0) return std::min(req, 64);
    unsigned hc = std::thread::hardware_concurrency();
    if (hc == 0) hc = 1;
    return (int)std::min<unsigned>(hc, 16);
}

// ------------------------------------------------------------------------------------------------------
// CSR input
// ------------------------------------------------------------------------------------------------------

namespace {

// an entry is stored iff it is neither +0 nor -0
inline bool stored16(uint16_t v) { return (v & 0x7FFFu) != 0; }
inline bool stored32(uint32_t v) { return (v & 0x7FFFFFFFu) != 0; }

template <typename T, typename Stored>
int csr_from_dense_t(const T *W, int64_t m, int64_t n, int64_t ld, int threads, int value_bits, Stored stored, Csr &out)
{
    out.m = m;
    out.n = n;
    out.value_bits = value_bits;
    out.rowptr.assign((size_t)m + 1, 0);
    std::vector<int64_t> cnt((size_t)m, 0);
    threads = resolve_threads(threads);
    parallel_for(m, threads, [&](int64_t i) {
        const T *row = W + i * ld;
        int64_t c = 0;
        for (int64_t j = 0; j < n; ++j) c += stored(row[j]);
        cnt[(size_t)i] = c;
    });
    for (int64_t i = 0; i < m; ++i) out.rowptr[(size_t)i + 1] = out.rowptr[(size_t)i] + cnt[(size_t)i];
    out.col.resize((size_t)out.rowptr[(size_t)m]);
    out.val.resize((size_t)out.rowptr[(size_t)m]);
    parallel_for(m, threads, [&](int64_t i) {
        const T *row = W + i * ld;
        int64_t p = out.rowptr[(size_t)i];
        for (int64_t j = 0; j < n; ++j)
            if (stored(row[j])) {
                out.col[(size_t)p] = (int32_t)j;
                out.val[(size_t)p] = row[j];
                ++p;
            }
    });
    return 0;
}

template <typename T, typename Stored>
int csr_from_csr_t(const int64_t *rowptr, const int32_t *col, const T *val, int64_t m, int64_t n, int value_bits,
                   Stored stored, Csr &out)
{
    if (rowptr[0] != 0) return -1;
    out.m = m;
    out.n = n;
    out.value_bits = value_bits;
    out.rowptr.assign((size_t)m + 1, 0);
    out.col.clear();
    out.val.clear();
    out.col.reserve((size_t)rowptr[m]);
    out.val.reserve((size_t)rowptr[m]);
    for (int64_t i = 0; i < m; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return -1;
        int64_t prev = -1;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t c = col[p];
            if (c < 0 || c >= n || c <= prev) return -1;
            prev = c;
            if (stored(val[p])) {
                out.col.push_back((int32_t)c);
                out.val.push_back(val[p]);
            }
        }
        out.rowptr[(size_t)i + 1] = (int64_t)out.col.size();
    }
    return 0;
}

}  // namespace

int csr_from_dense(const uint16_t *W, int64_t m, int64_t n, int64_t ld, int threads, Csr &out)
{
    return csr_from_dense_t(W, m, n, ld, threads, 16, stored16, out);
}
int csr_from_dense_f32(const uint32_t *W, int64_t m, int64_t n, int64_t ld, int threads, Csr &out)
{
    return csr_from_dense_t(W, m, n, ld, threads, 32, stored32, out);
}
int csr_from_csr(const int64_t *rowptr, const int32_t *col, const uint16_t *val, int64_t m, int64_t n, Csr &out)
{
    return csr_from_csr_t(rowptr, col, val, m, n, 16, stored16, out);
}
int csr_from_csr_f32(const int64_t *rowptr, const int32_t *col, const uint32_t *val, int64_t m, int64_t n, Csr &out)
{
    return csr_from_csr_t(rowptr, col, val, m, n, 32, stored32, out);
}

// ------------------------------------------------------------------------------------------------------
// hierarchical block extraction inside one panel
// ------------------------------------------------------------------------------------------------------

namespace {

// One row of a level matrix (Algorithm 1's A_E / A_R).  At level l a row stands for 2^l original rows
// (`members`) and a set bit at column c means all of them hold a stored entry at c (Section 4.2).
struct LRow {
    std::vector<uint64_t> bits;
    int cnt = 0;
    int child_a = -1, child_b = -1;   // the two rows of the level below this block was extracted from
    std::vector<int> members;         // panel-local original rows, size 2^level
};

struct PanelUnits {
    // extracted units per block type t (g = 2 << t): member rows (panel-local) and 64 sorted columns
    struct U {
        std::vector<int> rows;
        uint16_t cols[ECS_UNIT_COLS];
        int block_id;
        int block_len;
    };
    std::vector<U> units[ECS_NUM_BTYPES];
    std::vector<std::vector<int32_t>> resid;  // per panel-local row: sorted residual columns
};

inline int popcount_and(const uint64_t *a, const uint64_t *b, int nw)
{
    int s = 0;
    for (int w = 0; w < nw; ++w) s += __builtin_popcountll(a[w] & b[w]);
    return s;
}

// Columns of `bits` in increasing order.
inline void list_bits(const std::vector<uint64_t> &bits, std::vector<int32_t> &out)
{
    out.clear();
    for (size_t w = 0; w < bits.size(); ++w) {
        uint64_t v = bits[w];
        while (v) {
            int b = __builtin_ctzll(v);
            out.push_back((int32_t)(w * 64 + b));
            v &= v - 1;
        }
    }
}

// Cut a sorted column list into units of 64 columns whose successive gaps fit a delta index (Section 6.2: a
// block takes only columns that lie within the delta range of their neighbour; Section 6.3.1: block widths are
// whole multiples of the load quantum, here one unit).  Columns that end up in no unit go to `rest`.
void form_units(const std::vector<int32_t> &cols, int32_t max_delta, std::vector<int32_t> &taken,
                std::vector<int32_t> &rest)
{
    taken.clear();
    rest.clear();
    size_t start = 0;                 // start of the current candidate run inside cols
    for (size_t i = 0; i < cols.size(); ++i) {
        if (i > start && cols[i] - cols[i - 1] > max_delta) {
            for (size_t k = start; k < i; ++k) rest.push_back(cols[k]);
            start = i;
        }
        if (i + 1 - start == ECS_UNIT_COLS) {
            for (size_t k = start; k <= i; ++k) taken.push_back(cols[k]);
            start = i + 1;
        }
    }
    for (size_t k = start; k < cols.size(); ++k) rest.push_back(cols[k]);
}

// Greedy row matching (Algorithm 2).  Rows are popped in order of decreasing column count (ties: lower
// index first); the popped row takes the still unselected row with which it shares the most columns
// (ties: lower index).  A pair is kept only if the shared count reaches one unit, otherwise the popped
// row stays single this round.
void row_matching(const std::vector<LRow> &rows, int nw, std::vector<std::pair<int, int>> &pairs)
{
    pairs.clear();
    const int R = (int)rows.size();
    std::vector<int> order;
    order.reserve(R);
    for (int i = 0; i < R; ++i)
        if (rows[i].cnt >= (int)ECS_UNIT_COLS) order.push_back(i);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return rows[a].cnt > rows[b].cnt; });
    std::vector<char> unselected(R, 0);
    for (int i : order) unselected[i] = 1;
    for (int a : order) {
        if (!unselected[a]) continue;
        unselected[a] = 0;
        int best = -1, best_sim = 0;
        for (int b = 0; b < R; ++b) {
            if (!unselected[b]) continue;
            if (rows[b].cnt <= best_sim) continue;          // cannot beat the current best
            int sim = popcount_and(rows[a].bits.data(), rows[b].bits.data(), nw);
            if (sim > best_sim) {
                best_sim = sim;
                best = b;
            }
        }
        if (best >= 0 && best_sim >= (int)ECS_UNIT_COLS) {
            pairs.emplace_back(a, best);
            unselected[best] = 0;
        }
    }
}

void extract_panel(const Csr &A, const int32_t *prow, int nrows, int max_g, int max_rounds, int delta_bits, PanelUnits &out)
{
    const int32_t max_delta = (int32_t)ECS_MAX_DELTA(delta_bits);
    const int n = (int)A.n;
    const int nw = (n + 63) / 64;
    std::vector<std::vector<LRow>> levels(1);
    levels[0].resize(nrows);
    for (int r = 0; r < nrows; ++r) {
        LRow &L = levels[0][r];
        L.bits.assign(nw, 0);
        L.members.assign(1, r);
        for (int64_t p = A.rowptr[prow[r]]; p < A.rowptr[prow[r] + 1]; ++p) {
            int c = A.col[p];
            L.bits[c >> 6] |= 1ull << (c & 63);
        }
        L.cnt = (int)(A.rowptr[prow[r] + 1] - A.rowptr[prow[r]]);
    }

    std::vector<std::pair<int, int>> pairs;
    std::vector<uint64_t> common(nw);
    std::vector<int32_t> cols, taken, rest;

    // Algorithm 1: multi-level aggregation (outer), multi-round extraction (inner).
    for (int level = 0; (2 << level) <= max_g; ++level) {
        std::vector<LRow> next;                     // blocks extracted at this level = rows of the next A_E
        for (int round = 0; round < max_rounds; ++round) {
            std::vector<LRow> &AR = levels[level];
            row_matching(AR, nw, pairs);
            bool any = false;
            for (auto &pr : pairs) {
                LRow &a = AR[pr.first], &b = AR[pr.second];
                for (int w = 0; w < nw; ++w) common[w] = a.bits[w] & b.bits[w];
                list_bits(common, cols);
                form_units(cols, max_delta, taken, rest);
                if (taken.empty()) continue;
                any = true;
                LRow blk;
                blk.bits.assign(nw, 0);
                for (int32_t c : taken) {
                    uint64_t bit = 1ull << (c & 63);
                    blk.bits[c >> 6] |= bit;
                    a.bits[c >> 6] &= ~bit;         // extracted entries leave A_R
                    b.bits[c >> 6] &= ~bit;
                }
                blk.cnt = (int)taken.size();
                a.cnt -= blk.cnt;
                b.cnt -= blk.cnt;
                blk.child_a = pr.first;
                blk.child_b = pr.second;
                blk.members = a.members;
                blk.members.insert(blk.members.end(), b.members.begin(), b.members.end());
                next.push_back(std::move(blk));
            }
            if (!any) break;
        }
        if (next.empty()) break;
        levels.push_back(std::move(next));
    }

    // Decode what is left at every level into blocks of that level's granularity, coarsest first.  Columns
    // of a level >= 1 row that no longer form a valid unit (a neighbour was lifted to a coarser block and the
    // gap now exceeds the delta range) fall back to the two rows of the level below.
    out.resid.assign(nrows, {});
    int block_id = 0;
    for (int level = (int)levels.size() - 1; level >= 1; --level) {
        std::vector<LRow> &rows = levels[level];
        const int t = level - 1;
        for (LRow &L : rows) {
            list_bits(L.bits, cols);
            form_units(cols, max_delta, taken, rest);
            for (int32_t c : rest) {
                uint64_t bit = 1ull << (c & 63);
                LRow &ca = levels[level - 1][L.child_a], &cb = levels[level - 1][L.child_b];
                ca.bits[c >> 6] |= bit;
                cb.bits[c >> 6] |= bit;
                ++ca.cnt;
                ++cb.cnt;
            }
            const int nu = (int)(taken.size() / ECS_UNIT_COLS);
            for (int u = 0; u < nu; ++u) {
                PanelUnits::U unit;
                unit.rows = L.members;
                for (unsigned k = 0; k < ECS_UNIT_COLS; ++k) unit.cols[k] = (uint16_t)taken[u * ECS_UNIT_COLS + k];
                unit.block_id = block_id;
                unit.block_len = nu;
                out.units[t].push_back(std::move(unit));
            }
            if (nu) ++block_id;
        }
    }
    for (int r = 0; r < nrows; ++r) list_bits(levels[0][r].bits, out.resid[r]);
}

// value of W[row, col] (must be a stored entry)
inline uint32_t value_at(const Csr &A, int64_t row, int32_t col)
{
    const int32_t *b = A.col.data() + A.rowptr[row], *e = A.col.data() + A.rowptr[row + 1];
    const int32_t *p = std::lower_bound(b, e, col);
    return (p != e && *p == col) ? A.val[(size_t)(p - A.col.data())] : 0u;
}

struct PanelImage {
    std::vector<uint8_t> bytes;
    uint32_t meta_bytes = 0, nslots = 0, lds_slots = 0;
    int64_t value_bytes = 0, delta_bytes = 0, pad_elements = 0, gap_pads = 0;
    int64_t nnz_by_g[5] = {0, 0, 0, 0, 0};
    int64_t units_by_g[5] = {0, 0, 0, 0, 0};
    int64_t delta_hist[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    int err = 0;
};

inline int hist_bin(unsigned d)
{
    if (d == 0) return 0;
    int b = 1;
    while (d > 1 && b < 8) {
        d >>= 1;
        ++b;
    }
    return b;
}

// index k of an array of `bits`-wide indices: a delta with 8 or 4 bits (with 4 bits the earlier delta of a byte
// sits in its low nibble), the column itself with 16 bits (index compression switched off)
inline void put_delta(uint8_t *d, size_t k, int bits, uint32_t v)
{
    if (bits == 16)
        reinterpret_cast<uint16_t *>(d)[k] = (uint16_t)v;
    else if (bits == 8)
        d[k] = (uint8_t)v;
    else
        d[k >> 1] = (uint8_t)((k & 1) ? ((d[k >> 1] & 0x0F) | (v << 4)) : ((d[k >> 1] & 0xF0) | v));
}
inline uint32_t get_delta(const uint8_t *d, size_t k, int bits)
{
    if (bits == 16) return reinterpret_cast<const uint16_t *>(d)[k];
    return bits == 8 ? d[k] : ((d[k >> 1] >> (4 * (k & 1))) & 0xF);
}

void encode_panel(const Csr &A, const int32_t *prow, int nrows, PanelUnits &pu, bool reorder, int delta_bits, PanelImage &img)
{
    const int32_t max_delta = (int32_t)ECS_MAX_DELTA(delta_bits);
    const uint32_t unit_db = ECS_UNIT_DBYTES(delta_bits), lane_db = ECS_LANE_DBYTES(delta_bits);
    const uint32_t vw = (uint32_t)A.value_bits / 8u;      // bytes per value
    const uint32_t ep = 16u / vw;                         // values per 128-bit load
    auto put_val = [vw](uint8_t *base, size_t idx, uint32_t v) {
        if (vw == 2)
            reinterpret_cast<uint16_t *>(base)[idx] = (uint16_t)v;
        else
            reinterpret_cast<uint32_t *>(base)[idx] = v;
    };
    // ---- ordering (Section 5): sets by decreasing granularity (fixed by the layout); inside a set the
    // units of longer blocks first.
    if (reorder)
        for (int t = 0; t < ECS_NUM_BTYPES; ++t)
            std::stable_sort(pu.units[t].begin(), pu.units[t].end(),
                             [](const PanelUnits::U &a, const PanelUnits::U &b) { return a.block_len > b.block_len; });

    // ---- residual rows -> elements (delta, value) with gap fillers and tail padding -> lane units
    struct LaneUnit {
        uint16_t d[ECS_LANE_ELEMS];
        uint32_t v[ECS_LANE_ELEMS];
        int row;          // panel-local
        int32_t before;   // column "before" the first element: col0 for a row's first unit (its delta is 0)
        uint32_t total;   // sum of the 16 deltas
    };
    std::vector<LaneUnit> lanes;
    for (int r = 0; r < nrows; ++r) {
        const std::vector<int32_t> &cols = pu.resid[r];
        if (cols.empty()) continue;
        std::vector<uint16_t> ds;
        std::vector<uint32_t> vs;
        int32_t cur = cols[0];
        ds.push_back(0);
        vs.push_back(value_at(A, prow[r], cols[0]));
        for (size_t k = 1; k < cols.size(); ++k) {
            int32_t gap = cols[k] - cur;
            while (gap > max_delta) {                    // explicit zero every R_P - 1 columns (Section 6.2)
                ds.push_back((uint16_t)max_delta);
                vs.push_back(0);
                gap -= max_delta;
                ++img.gap_pads;
                ++img.pad_elements;
            }
            ds.push_back((uint16_t)gap);
            vs.push_back(value_at(A, prow[r], cols[k]));
            cur = cols[k];
            ++img.delta_hist[hist_bin((unsigned)gap)];
        }
        img.nnz_by_g[0] += (int64_t)cols.size();
        while (ds.size() % ECS_LANE_ELEMS) {             // tail alignment: zero-valued elements on the last column
            ds.push_back(0);
            vs.push_back(0);
            ++img.pad_elements;
        }
        int32_t before = cols[0];
        for (size_t e = 0; e < ds.size(); e += ECS_LANE_ELEMS) {
            LaneUnit lu;
            lu.row = r;
            lu.before = before;
            lu.total = 0;
            for (unsigned k = 0; k < ECS_LANE_ELEMS; ++k) {
                lu.d[k] = ds[e + k];
                lu.v[k] = vs[e + k];
                lu.total += ds[e + k];
            }
            before += (int32_t)lu.total;
            lanes.push_back(lu);
        }
    }
    const uint32_t nlanes = (uint32_t)lanes.size();
    const uint32_t nchunks = (nlanes + ECS_CHUNK_LANES - 1) / ECS_CHUNK_LANES;
    img.units_by_g[0] = nlanes;

    // ---- residual chunk tables
    std::vector<EcsRChunk> rchunks(nchunks);
    std::vector<EcsREntry> rentries;
    for (uint32_t c = 0; c < nchunks; ++c) {
        EcsRChunk &ch = rchunks[c];
        ch.head_mask = 0;
        ch.entry0 = (uint32_t)rentries.size();
        ch.nlanes = std::min<uint32_t>(ECS_CHUNK_LANES, nlanes - c * ECS_CHUNK_LANES);
        int64_t scan = 0;                                   // sum of totals of earlier lanes in this chunk
        for (uint32_t l = 0; l < ch.nlanes; ++l) {
            const LaneUnit &lu = lanes[c * ECS_CHUNK_LANES + l];
            bool head = (l == 0) || (lanes[c * ECS_CHUNK_LANES + l - 1].row != lu.row);
            if (head) {
                ch.head_mask |= 1ull << l;
                EcsREntry e;
                e.c = (int32_t)(lu.before - scan);
                e.reserved_ = 0;
                e.row_local = (uint16_t)lu.row;
                rentries.push_back(e);
            }
            scan += lu.total;
        }
    }

    // ---- slots: one per (unit, member row), a row's slots are consecutive; the residual set needs no table for
    // its partial sums (one per lane unit, in stream order) beyond the first lane unit of every row
    std::vector<uint32_t> per_row(nrows, 0);
    for (int t = 0; t < ECS_NUM_BTYPES; ++t)
        for (auto &u : pu.units[t])
            for (int r : u.rows) ++per_row[r];
    std::vector<uint32_t> rowlu(nrows + 1, 0);
    for (const LaneUnit &lu : lanes) ++rowlu[lu.row + 1];
    for (int r = 0; r < nrows; ++r) rowlu[r + 1] += rowlu[r];
    std::vector<uint32_t> rowslot(nrows + 1, 0);
    for (int r = 0; r < nrows; ++r) rowslot[r + 1] = rowslot[r] + per_row[r];
    img.nslots = rowslot[nrows];
    img.lds_slots = img.nslots + ECS_CHUNK_LANES * nchunks;
    if (img.nslots > 65535u || nrows > 65535) {
        img.err = -2;
        return;
    }
    std::vector<uint32_t> cursor(rowslot.begin(), rowslot.end() - 1);

    // ---- layout
    uint32_t off = ECS_PANEL_HEADER;
    uint32_t hdr[ECS_PANEL_HEADER / 4];
    std::memset(hdr, 0, sizeof(hdr));
    hdr[PH_ROW0] = (uint32_t)prow[0];
    hdr[PH_NROWS] = (uint32_t)nrows;
    hdr[PH_NSLOTS] = img.nslots;
    hdr[PH_NRLANES] = nlanes;
    hdr[PH_NRENTRIES] = (uint32_t)rentries.size();
    hdr[PH_ROWSLOT_OFF] = off;
    off = align_up(off + 2u * (uint32_t)(nrows + 1), 16);
    hdr[PH_ROWLU_OFF] = off;
    off = align_up(off + 4u * (uint32_t)(nrows + 1), 16);
    hdr[PH_ROWIDX_OFF] = off;
    off = align_up(off + 4u * (uint32_t)nrows, 16);
    for (int t = ECS_NUM_BTYPES - 1; t >= 0; --t) {
        const uint32_t g = 2u << t;
        hdr[PH_NUNITS + t] = (uint32_t)pu.units[t].size();
        hdr[PH_UTAB_OFF + t] = off;
        off = align_up(off + 2u * (1 + g) * (uint32_t)pu.units[t].size(), 16);
    }
    hdr[PH_RCHUNK_OFF] = off;
    off += (uint32_t)sizeof(EcsRChunk) * nchunks;
    hdr[PH_RENTRY_OFF] = off;
    off = align_up(off + (uint32_t)sizeof(EcsREntry) * (uint32_t)rentries.size(), 16);
    hdr[PH_ZERO_OFF] = off;
    off += 16;
    img.meta_bytes = off;
    hdr[PH_META_BYTES] = off;
    // Residual chunks first: a chunk = the deltas of its 64 lane units, then their values, the k-th 128-bit load of
    // lane l at k * 1024 + 16 * l; a last chunk of nl < 64 lane units is stored tightly (nl delta runs padded to 16
    // bytes, then the k-th load of lane l at 16 * nl * k + 16 * l).
    const uint32_t res_off = off;                                       // a multiple of 16
    const uint32_t chunk_bytes = ECS_CHUNK_DBYTES(delta_bits) + 1024u * vw;
    hdr[PH_RD_OFF] = res_off;
    hdr[PH_RV_OFF] = chunk_bytes;
    off = res_off + chunk_bytes * nchunks;
    {
        const uint32_t nl_last = nchunks ? nlanes - (nchunks - 1) * ECS_CHUNK_LANES : 0;
        if (nchunks && nl_last < ECS_CHUNK_LANES)
            off = res_off + chunk_bytes * (nchunks - 1) + align_up(lane_db * nl_last, 16) + 16u * vw * nl_last;
    }
    img.delta_bytes += (int64_t)lane_db * nlanes;
    img.value_bytes += 16ll * vw * nlanes;
    for (int t = ECS_NUM_BTYPES - 1; t >= 0; --t) {
        const uint32_t g = 2u << t;
        const uint32_t nu = (uint32_t)pu.units[t].size();
        hdr[PH_BD_OFF + t] = off;
        off += unit_db * nu;              // multiple of 16
        hdr[PH_BV_OFF + t] = off;
        off += 64u * vw * g * nu;
        img.delta_bytes += (int64_t)unit_db * nu;
        img.value_bytes += 64ll * vw * g * nu;
        img.units_by_g[t + 1] = nu;
        img.nnz_by_g[t + 1] = (int64_t)nu * ECS_UNIT_COLS * g;
    }
    off = align_up(off, 256);
    hdr[PH_PANEL_BYTES] = off;
    img.bytes.assign(off, 0);
    uint8_t *P = img.bytes.data();

    // ---- block sets
    for (int t = ECS_NUM_BTYPES - 1; t >= 0; --t) {
        const uint32_t g = 2u << t;
        uint16_t *utab = (uint16_t *)(P + hdr[PH_UTAB_OFF + t]);
        std::vector<uint32_t> flat(ECS_UNIT_COLS * g);
        for (size_t u = 0; u < pu.units[t].size(); ++u) {
            const PanelUnits::U &un = pu.units[t][u];
            uint16_t *ue = utab + u * (1 + g);
            ue[0] = un.cols[0];
            for (uint32_t r = 0; r < g; ++r) ue[1 + r] = (uint16_t)cursor[un.rows[r]]++;
            uint8_t *d = P + hdr[PH_BD_OFF + t] + unit_db * u;
            put_delta(d, 0, delta_bits, delta_bits == 16 ? un.cols[0] : 0u);
            for (unsigned k = 1; k < ECS_UNIT_COLS; ++k)
                put_delta(d, k, delta_bits, delta_bits == 16 ? un.cols[k] : (uint32_t)(un.cols[k] - un.cols[k - 1]));
            for (unsigned k = 0; k < ECS_UNIT_COLS; ++k)
                for (uint32_t r = 0; r < g; ++r) flat[k * g + r] = value_at(A, prow[un.rows[r]], un.cols[k]);
            // permutation: lane j owns flat[4*j*g, 4*(j+1)*g); its k-th 128-bit group (8 halfs or 4 floats) goes
            // to byte k*256 + 16*j of the unit
            uint8_t *v = P + hdr[PH_BV_OFF + t] + 64u * vw * g * u;
            for (uint32_t j = 0; j < 16; ++j)
                for (uint32_t k = 0; k < 4 * g / ep; ++k)
                    for (uint32_t i = 0; i < ep; ++i) put_val(v, k * 16 * ep + ep * j + i, flat[4 * j * g + ep * k + i]);
        }
    }

    // ---- residual set
    for (uint32_t c = 0; c < nchunks; ++c) {
        const uint32_t nl = rchunks[c].nlanes;
        const bool tight = nl < ECS_CHUNK_LANES;                                 // only ever the last chunk
        const uint32_t stride = tight ? nl : ECS_CHUNK_LANES;
        uint8_t *d = P + res_off + chunk_bytes * c;
        uint8_t *v = d + (tight ? align_up(lane_db * nl, 16) : ECS_CHUNK_DBYTES(delta_bits));
        for (uint32_t l = 0; l < nl; ++l) {
            const LaneUnit &lu = lanes[c * ECS_CHUNK_LANES + l];
            uint32_t col = (uint32_t)lu.before;                        // absolute columns where deltas are switched off
            for (uint32_t i = 0; i < ECS_LANE_ELEMS; ++i) {
                col += lu.d[i];
                put_delta(d + lane_db * l, i, delta_bits, delta_bits == 16 ? col : lu.d[i]);
            }
            for (uint32_t k = 0; k < ECS_LANE_ELEMS / ep; ++k)          // k-th 128-bit load of lane l
                for (uint32_t i = 0; i < ep; ++i) put_val(v, ep * stride * k + ep * l + i, lu.v[ep * k + i]);
        }
    }
    for (int r = 0; r < nrows; ++r)
        if (cursor[r] != rowslot[r + 1]) img.err = -100;

    std::memcpy(P, hdr, sizeof(hdr));
    uint16_t *rs = (uint16_t *)(P + hdr[PH_ROWSLOT_OFF]);
    for (int r = 0; r <= nrows; ++r) rs[r] = (uint16_t)rowslot[r];
    std::memcpy(P + hdr[PH_ROWLU_OFF], rowlu.data(), 4u * (size_t)(nrows + 1));
    std::memcpy(P + hdr[PH_ROWIDX_OFF], prow, 4u * (size_t)nrows);
    if (nchunks) std::memcpy(P + hdr[PH_RCHUNK_OFF], rchunks.data(), sizeof(EcsRChunk) * nchunks);
    if (!rentries.empty()) std::memcpy(P + hdr[PH_RENTRY_OFF], rentries.data(), sizeof(EcsREntry) * rentries.size());
}

}  // namespace

// ------------------------------------------------------------------------------------------------------
// row clustering: Algorithm 2 over ALL rows, level by level, to decide which rows share a panel
// ------------------------------------------------------------------------------------------------------

// The paper matches rows over the whole matrix (Section 4: the rows of a block need not be neighbours).  Here a
// panel owns its rows, so rows that belong together must first be brought into the same panel: the multi-level
// aggregation of Algorithm 1 is run once over all rows with one matching round per level (greedy row matching,
// Algorithm 2; a group stands for the columns all its members share), groups of up to `group` rows result, and the
// rows are listed group by group.  Panels are then cut from that list and extraction proper runs inside each panel.
// Returns the row order.
static void cluster_rows(const Csr &A, int group, int threads, std::vector<int32_t> &order)
{
    const int64_t m = A.m;
    const int nw = (int)((A.n + 63) / 64);
    struct Grp {
        std::vector<uint64_t> bits;
        int cnt;
        std::vector<int32_t> members;
    };
    std::vector<Grp> cur((size_t)m);
    parallel_for(m, threads, [&](int64_t i) {
        Grp &g = cur[(size_t)i];
        g.bits.assign(nw, 0);
        for (int64_t p = A.rowptr[i]; p < A.rowptr[i + 1]; ++p) g.bits[A.col[p] >> 6] |= 1ull << (A.col[p] & 63);
        g.cnt = (int)(A.rowptr[i + 1] - A.rowptr[i]);
        g.members.assign(1, (int32_t)i);
    });
    for (int size = 1; size < group && cur.size() > 1; size *= 2) {
        const int R = (int)cur.size();
        // every group's best partner over all others (ties: lower index), in parallel; the greedy pass below takes it
        // if it is still free and searches again among the free ones if not
        std::vector<int> best(R, -1), best_sim(R, 0);
        parallel_for(R, threads, [&](int64_t a) {
            int b_best = -1, s_best = 0;
            for (int b = 0; b < R; ++b) {
                if (b == a || cur[b].cnt <= s_best) continue;
                const int sim = popcount_and(cur[a].bits.data(), cur[b].bits.data(), nw);
                if (sim > s_best) s_best = sim, b_best = b;
            }
            best[a] = b_best, best_sim[a] = s_best;
        });
        std::vector<int> pop(R);
        for (int i = 0; i < R; ++i) pop[i] = i;
        std::stable_sort(pop.begin(), pop.end(), [&](int a, int b) { return cur[a].cnt > cur[b].cnt; });
        std::vector<char> free_(R, 1);
        std::vector<Grp> next;
        next.reserve((size_t)R / 2 + 1);
        std::vector<int> single;
        for (int a : pop) {
            if (!free_[a]) continue;
            free_[a] = 0;
            int b = best[a];
            if (b < 0 || !free_[b]) {
                b = -1;
                int s_best = 0;
                for (int c = 0; c < R; ++c) {
                    if (!free_[c] || cur[c].cnt <= s_best) continue;
                    const int sim = popcount_and(cur[a].bits.data(), cur[c].bits.data(), nw);
                    if (sim > s_best) s_best = sim, b = c;
                }
            }
            if (b < 0) {
                single.push_back(a);
                continue;
            }
            free_[b] = 0;
            Grp g;
            g.bits.resize(nw);
            int cnt = 0;
            for (int w = 0; w < nw; ++w) {
                g.bits[w] = cur[a].bits[w] & cur[b].bits[w];
                cnt += __builtin_popcountll(g.bits[w]);
            }
            g.cnt = cnt;
            g.members = cur[a].members;
            g.members.insert(g.members.end(), cur[b].members.begin(), cur[b].members.end());
            next.push_back(std::move(g));
        }
        for (int a : single) next.push_back(std::move(cur[a]));
        cur.swap(next);
    }
    order.clear();
    order.reserve((size_t)m);
    for (const Grp &g : cur) order.insert(order.end(), g.members.begin(), g.members.end());
}

// ------------------------------------------------------------------------------------------------------
// build
// ------------------------------------------------------------------------------------------------------

int build_image(const Csr &A, const BuildParams &bp, Image &out)
{
    auto t0 = std::chrono::steady_clock::now();
    const int64_t m = A.m, n = A.n;
    if (n > 65535 || m > 0x7fffffff) return -2;
    const int64_t nnz = A.rowptr[(size_t)m];
    int P = bp.num_panels;
    if (P <= 0) {
        P = (int)std::min<int64_t>(256, std::max<int64_t>(1, m / 16));
        // x and one FP32 partial sum per residual lane unit (16 entries) of a panel must fit the LDS of a compute
        // unit: where a panel of this size could not (few, long rows), more panels are made, down to one row each
        int64_t longest = 0;
        for (int64_t i = 0; i < m; ++i) longest = std::max(longest, A.rowptr[(size_t)i + 1] - A.rowptr[(size_t)i]);
        const int64_t x_bytes = n * (A.value_bits / 8), budget = 150 * 1024;
        while (P < m && x_bytes + 4 * ((nnz / P + longest) / 16 + m / P + 64) + 4096 > budget)
            P = (int)std::min<int64_t>(m, 2 * (int64_t)P);
    }
    if (bp.global_matching) P = 1;
    P = (int)std::min<int64_t>(P, m);

    // the order in which rows are dealt to panels: as they come, or brought together by similarity first
    const int threads = resolve_threads(bp.num_threads);
    std::vector<int32_t> order;
    if (bp.cluster_rows && P > 1 && bp.max_granularity > 1) {
        cluster_rows(A, std::max(2, bp.max_granularity), threads, order);
    } else {
        order.resize((size_t)m);
        for (int64_t i = 0; i < m; ++i) order[(size_t)i] = (int32_t)i;
    }
    std::vector<int64_t> pre((size_t)m + 1, 0);                                // stored entries before the k-th row dealt
    for (int64_t k = 0; k < m; ++k) pre[(size_t)k + 1] = pre[(size_t)k] + (A.rowptr[(size_t)order[(size_t)k] + 1] - A.rowptr[(size_t)order[(size_t)k]]);

    // nnz-balanced panels of consecutive rows of that order (Section 5: even work per processing unit): panel p ends
    // at the first row where the running nnz reaches (p + 1) / P of the total; ties in rows for empty matrices.
    std::vector<int64_t> bound(P + 1, 0);
    {
        int64_t r = 0;
        for (int p = 0; p < P; ++p) {
            bound[p] = r;
            const int64_t rows_left = m - r, panels_left = P - p;
            int64_t take;
            if (nnz == 0) {
                take = (rows_left + panels_left - 1) / panels_left;
            } else {
                const double target = (double)nnz * (p + 1) / P;
                int64_t e = r;
                while (e < m && (double)pre[(size_t)e + 1] <= target) ++e;
                // also take the row that crosses the target if that lands closer to it
                if (e < m && (double)pre[(size_t)e + 1] - target < target - (double)pre[(size_t)e]) ++e;
                take = e - r;
            }
            take = std::max<int64_t>(take, 1);                               // every panel owns at least one row
            take = std::min<int64_t>(take, rows_left - (panels_left - 1));   // and leaves one for each later panel
            r += take;
        }
        bound[P] = m;                                                        // the last panel ends at m
    }
    std::vector<PanelImage> imgs;
    // Every block set the image holds costs the SpMV launch a pipeline stage of its own, so a coarsest set that holds
    // next to nothing (under 1 % of the stored entries over the whole matrix) is not worth having: the granularity
    // cap is lowered and the matrix encoded again, until the coarsest set carries weight or no extraction is left.
    for (int max_g = bp.max_granularity;; max_g >>= 1) {
        imgs.assign(P, PanelImage());
        parallel_for(P, threads, [&](int64_t p) {
            const int64_t r0 = bound[p], r1 = (p + 1 == P) ? m : bound[p + 1];
            PanelUnits pu;
            extract_panel(A, order.data() + r0, (int)(r1 - r0), max_g, bp.max_rounds, bp.delta_bits, pu);
            encode_panel(A, order.data() + r0, (int)(r1 - r0), pu, bp.reorder, bp.delta_bits, imgs[p]);
        });
        if (bp.keep_small_sets || max_g == 1) break;
        int top = 0;                                                         // coarsest set present
        int64_t by_t[ECS_NUM_BTYPES + 1] = {0, 0, 0, 0, 0};
        for (auto &im : imgs)
            for (int t = 1; t <= ECS_NUM_BTYPES; ++t) by_t[t] += im.nnz_by_g[t];
        for (int t = 1; t <= ECS_NUM_BTYPES; ++t)
            if (by_t[t] > 0) top = t;
        if (top == 0 || by_t[top] * 100 >= nnz) break;
        max_g = 1 << top;                                                    // halved by the loop: drops set `top`
    }
    uint32_t stride = 256, meta = 16, slots = 1;
    for (auto &im : imgs) {
        if (im.err) return im.err;
        if (im.bytes.size() > 0xFFFFF000ull) return -2;                      // offsets inside a panel are 32-bit
        stride = std::max<uint32_t>(stride, (uint32_t)im.bytes.size());
        meta = std::max(meta, im.meta_bytes);
        slots = std::max(slots, im.lds_slots);
    }
    meta = align_up(meta, 16);
    // 4 KB of zeros after the last panel: loads that stand in for missing chunks may run past a short last panel
    const uint64_t total = ECS_IMAGE_HEADER + (uint64_t)stride * (uint64_t)P + 4096u;
    if (total > 0xFFFFFFFF00ull) return -2;
    out.bytes.assign((size_t)total, 0);
    out.m = m;
    out.n = n;
    out.nnz = nnz;
    out.num_panels = P;
    out.threads_per_wg = bp.threads_per_wg;
    out.delta_bits = bp.delta_bits;
    out.value_bits = A.value_bits;
    out.panel_stride = stride;
    out.meta_stride = meta;
    out.max_slots = slots;
    const uint32_t x_bytes = align_up((uint32_t)n * (uint32_t)(A.value_bits / 8), 16);
    out.lds_bytes = x_bytes + meta + align_up(slots * 4u, 16);

    ecspmv_stats_t &st = out.stats;
    std::memset(&st, 0, sizeof(st));
    st.struct_size = sizeof(st);
    st.m = m;
    st.n = n;
    st.nnz = nnz;
    st.image_bytes = (int64_t)total;
    st.csr32_bytes = (4 + A.value_bits / 8) * nnz + 4 * (m + 1);
    st.csr16_bytes = (2 + A.value_bits / 8) * nnz + 4 * (m + 1);
    st.value_bits = A.value_bits;
    st.num_panels = P;
    st.threads_per_wg = bp.threads_per_wg;
    st.delta_bits = bp.delta_bits;
    st.panel_stride = stride;
    st.meta_stride = meta;
    st.lds_bytes = out.lds_bytes;
    st.min_panel_bytes = INT64_MAX;
    for (int p = 0; p < P; ++p) {
        PanelImage &im = imgs[p];
        std::memcpy(out.bytes.data() + ECS_IMAGE_HEADER + (size_t)stride * p, im.bytes.data(), im.bytes.size());
        st.value_bytes += im.value_bytes;
        st.delta_bytes += im.delta_bytes;
        st.meta_bytes += im.meta_bytes;
        st.pad_elements += im.pad_elements;
        st.gap_pad_elements += im.gap_pads;
        st.max_panel_bytes = std::max<int64_t>(st.max_panel_bytes, (int64_t)im.bytes.size());
        st.min_panel_bytes = std::min<int64_t>(st.min_panel_bytes, (int64_t)im.bytes.size());
        for (int k = 0; k < 5; ++k) {
            st.nnz_by_g[k] += im.nnz_by_g[k];
            st.units_by_g[k] += im.units_by_g[k];
        }
        for (int k = 0; k < 9; ++k) st.delta_hist[k] += im.delta_hist[k];
    }
    out.type_mask = 0;
    for (int t = 0; t < ECS_NUM_BTYPES; ++t)
        if (st.units_by_g[t + 1] > 0) out.type_mask |= 1u << t;
    st.meta_bytes += ECS_IMAGE_HEADER;
    st.slack_bytes = st.image_bytes - st.value_bytes - st.delta_bytes - st.meta_bytes;
    for (int k = 0; k < 5; ++k) st.x_access_cost += (double)st.nnz_by_g[k] / (double)(1 << k);

    EcsImageHeader ih;
    std::memset(&ih, 0, sizeof(ih));
    ih.magic = ECS_MAGIC;
    ih.version = ECS_VERSION;
    ih.m = (uint32_t)m;
    ih.n = (uint32_t)n;
    ih.num_panels = (uint32_t)P;
    ih.threads_per_wg = (uint32_t)bp.threads_per_wg;
    ih.panel_stride = stride;
    ih.meta_stride = meta;
    ih.max_slots = slots;
    ih.lds_bytes = out.lds_bytes;
    ih.image_bytes = total;
    ih.nnz = (uint64_t)nnz;
    ih.delta_bits = (uint32_t)bp.delta_bits;
    ih.value_bits = (uint32_t)A.value_bits;
    std::memcpy(out.bytes.data(), &ih, sizeof(ih));
    st.build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return 0;
}

// ------------------------------------------------------------------------------------------------------
// decode: walk the image as the kernel does
// ------------------------------------------------------------------------------------------------------

namespace {

struct PanelView {
    const uint8_t *P;
    const uint32_t *hdr;
    const uint16_t *rowslot;
    uint32_t nrows;
    int row_of_slot(uint32_t s) const
    {
        // rowslot is non-decreasing; the owner of slot s is the last row whose first slot is <= s
        const uint16_t *e = std::upper_bound(rowslot, rowslot + nrows + 1, (uint16_t)s);
        return (int)(e - rowslot) - 1;
    }
};

}  // namespace

int walk_image(const Image &im, Triples *tri, BlockSets *bs)
{
    const uint8_t *base = im.bytes.data() + ECS_IMAGE_HEADER;
    const int bits = im.delta_bits;
    const uint32_t vw = (uint32_t)im.value_bits / 8u, ep = 16u / vw;
    auto get_val = [vw](const uint8_t *base, size_t idx) -> uint32_t {
        return vw == 2 ? (uint32_t)reinterpret_cast<const uint16_t *>(base)[idx]
                       : reinterpret_cast<const uint32_t *>(base)[idx];
    };
    const uint32_t absmask = vw == 2 ? 0x7FFFu : 0x7FFFFFFFu;
    for (int p = 0; p < im.num_panels; ++p) {
        PanelView pv;
        pv.P = base + (size_t)im.panel_stride * p;
        pv.hdr = (const uint32_t *)pv.P;
        pv.nrows = pv.hdr[PH_NROWS];
        pv.rowslot = (const uint16_t *)(pv.P + pv.hdr[PH_ROWSLOT_OFF]);
        const uint32_t *rowidx = (const uint32_t *)(pv.P + pv.hdr[PH_ROWIDX_OFF]);
        for (int t = ECS_NUM_BTYPES - 1; t >= 0; --t) {
            const uint32_t g = 2u << t, nu = pv.hdr[PH_NUNITS + t];
            const uint16_t *utab = (const uint16_t *)(pv.P + pv.hdr[PH_UTAB_OFF + t]);
            for (uint32_t u = 0; u < nu; ++u) {
                const uint16_t *ue = utab + u * (1 + g);
                const uint8_t *d = pv.P + pv.hdr[PH_BD_OFF + t] + ECS_UNIT_DBYTES(bits) * u;
                const uint8_t *v = pv.P + pv.hdr[PH_BV_OFF + t] + 64u * vw * g * u;
                int32_t cols[ECS_UNIT_COLS];
                // 16 lanes x 4 columns: local prefix inside a lane, exclusive scan over lanes, plus base
                uint32_t lane_excl = 0;
                for (uint32_t j = 0; j < 16; ++j) {
                    uint32_t rel = 0;
                    for (uint32_t c = 0; c < 4; ++c) {
                        rel += get_delta(d, 4 * j + c, bits);
                        cols[4 * j + c] = bits == 16 ? (int32_t)get_delta(d, 4 * j + c, bits) : (int32_t)(ue[0] + lane_excl + rel);
                    }
                    lane_excl += rel;
                }
                int rows[16];
                for (uint32_t r = 0; r < g; ++r) {
                    rows[r] = pv.row_of_slot(ue[1 + r]);
                    if (rows[r] < 0 || rows[r] >= (int)pv.nrows) return -100;
                }
                if (bs) {
                    bs->g.push_back((int32_t)g);
                    for (uint32_t r = 0; r < g; ++r) bs->rows.push_back((int32_t)rowidx[rows[r]]);
                    for (uint32_t k = 0; k < ECS_UNIT_COLS; ++k) bs->cols.push_back(cols[k]);
                }
                if (tri)
                    for (uint32_t j = 0; j < 16; ++j)
                        for (uint32_t k = 0; k < 4 * g / ep; ++k)
                            for (uint32_t i = 0; i < ep; ++i) {
                                const uint32_t f = ep * k + i;         // index in lane j's run
                                const uint32_t c = f / g, r = f % g;
                                const uint32_t val = get_val(v, k * 16 * ep + ep * j + i);
                                if ((val & absmask) == 0) continue;
                                tri->rows.push_back((int32_t)rowidx[rows[r]]);
                                tri->cols.push_back(cols[4 * j + c]);
                                tri->vals.push_back(val);
                            }
            }
        }
        if (!tri) continue;
        const uint32_t nlanes = pv.hdr[PH_NRLANES];
        const uint32_t nchunks = (nlanes + ECS_CHUNK_LANES - 1) / ECS_CHUNK_LANES;
        const EcsRChunk *rch = (const EcsRChunk *)(pv.P + pv.hdr[PH_RCHUNK_OFF]);
        const EcsREntry *ren = (const EcsREntry *)(pv.P + pv.hdr[PH_RENTRY_OFF]);
        for (uint32_t c = 0; c < nchunks; ++c) {
            const uint32_t nl = std::min<uint32_t>(ECS_CHUNK_LANES, nlanes - c * ECS_CHUNK_LANES);
            if (rch[c].nlanes != nl || !(rch[c].head_mask & 1)) return -101;
            const bool tight = nl < ECS_CHUNK_LANES;
            const uint32_t stride = tight ? nl : ECS_CHUNK_LANES;
            const uint8_t *d = pv.P + pv.hdr[PH_RD_OFF] + pv.hdr[PH_RV_OFF] * c;            // chunk c: deltas, then values
            const uint8_t *v = d + (tight ? align_up(ECS_LANE_DBYTES(bits) * nl, 16) : ECS_CHUNK_DBYTES(bits));
            int64_t excl = 0;
            for (uint32_t l = 0; l < nl; ++l) {
                const uint64_t below = rch[c].head_mask & ((l == 63) ? ~0ull : ((2ull << l) - 1));
                const EcsREntry &e = ren[rch[c].entry0 + (uint32_t)__builtin_popcountll(below) - 1];
                const int row = (int)e.row_local;
                const uint32_t *rowlu = (const uint32_t *)(pv.P + pv.hdr[PH_ROWLU_OFF]);
                const uint32_t L = c * ECS_CHUNK_LANES + l;
                if (row >= (int)pv.nrows || L < rowlu[row] || L >= rowlu[row + 1]) return -102;
                int64_t rel = 0;
                for (uint32_t k = 0; k < ECS_LANE_ELEMS; ++k) {
                    rel += get_delta(d + ECS_LANE_DBYTES(bits) * l, k, bits);
                    const uint32_t val = get_val(v, ep * stride * (k / ep) + ep * l + (k % ep));
                    if ((val & absmask) == 0) continue;
                    tri->rows.push_back((int32_t)rowidx[row]);
                    tri->cols.push_back(bits == 16 ? (int32_t)get_delta(d + ECS_LANE_DBYTES(bits) * l, k, bits)
                                                   : (int32_t)(e.c + excl + rel));
                    tri->vals.push_back(val);
                }
                excl += rel;
            }
        }
    }
    return 0;
}

}  // namespace ecs
