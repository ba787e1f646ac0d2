// C ABI of the library (see include/ecspmv.h): argument checks, option defaults, handle bookkeeping.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/ecspmv.h"
#include "encoder.h"
#include "launch.h"

struct ecspmv_matrix {
    ecs::Image image;
    void *d_image = nullptr;
};

struct ecspmv_csr {
    int64_t m = 0, n = 0, nnz = 0;
    std::vector<int32_t> rowptr, col;
    std::vector<uint16_t> val;
    size_t off_col = 0, off_val = 0, bytes = 0;
    uint8_t *d_buf = nullptr;
};

namespace {

thread_local int g_last_hip_error = 0;

int hip_status(int e)
{
    if (e == 0) return ECSPMV_OK;
    g_last_hip_error = e;
    return ECSPMV_ERR_HIP;
}

// LDS a workgroup may use on the current device, asked once per device and kept (the hot calls must not query the
// runtime on every launch)
int lds_limit(int *bytes)
{
    constexpr int kMaxDev = 64;
    static std::atomic<int> cached[kMaxDev];
    int dev = 0;
    int e = ecs::current_device(&dev);
    if (e) return e;
    if (dev >= 0 && dev < kMaxDev) {
        const int v = cached[dev].load(std::memory_order_relaxed);
        if (v > 0) {
            *bytes = v;
            return 0;
        }
    }
    e = ecs::device_lds_limit(bytes);
    if (e) return e;
    if (dev >= 0 && dev < kMaxDev) cached[dev].store(*bytes, std::memory_order_relaxed);
    return 0;
}

int map_build_error(int e)
{
    if (e == 0) return ECSPMV_OK;
    if (e == -2) return ECSPMV_ERR_UNSUPPORTED;
    return ECSPMV_ERR_INVALID;
}

int parse_opts(const ecspmv_build_opts *o, ecs::BuildParams &bp, int value_bits = 16)
{
    ecspmv_build_opts opts;
    std::memset(&opts, 0, sizeof(opts));
    if (o) {
        if (o->struct_size < sizeof(uint32_t)) return ECSPMV_ERR_INVALID;
        std::memcpy(&opts, o, o->struct_size < sizeof(opts) ? o->struct_size : sizeof(opts));
    }
    if (opts.delta_bits != 0 && opts.delta_bits != 8 && opts.delta_bits != 4 && opts.delta_bits != 16)
        return ECSPMV_ERR_UNSUPPORTED;
    if (opts.delta_bits == 16 && value_bits != 16) return ECSPMV_ERR_UNSUPPORTED;      // the ablation point exists for FP16 only
    bp.delta_bits = opts.delta_bits ? opts.delta_bits : 8;
    // default cap on g: 8, and 4 for FP32 values (an 8-grained FP32 unit holds 32 value registers per lane and the
    // kernel starts to spill; larger caps can still be asked for)
    const int g = opts.max_granularity ? opts.max_granularity : (value_bits == 32 ? 4 : 8);
    if (g != 1 && g != 2 && g != 4 && g != 8 && g != 16) return ECSPMV_ERR_UNSUPPORTED;
    bp.max_granularity = g;
    if (opts.max_rounds < 0 || opts.num_panels < 0 || opts.num_threads < 0) return ECSPMV_ERR_INVALID;
    bp.max_rounds = opts.max_rounds ? opts.max_rounds : 64;
    bp.num_panels = opts.num_panels;
    bp.num_threads = opts.num_threads;
    const int t = opts.threads_per_wg;
    if (t != 0 && (t < 64 || t > 1024 || t % 64)) return ECSPMV_ERR_INVALID;
    bp.threads_per_wg = t;
    bp.global_matching = (opts.flags & ECSPMV_FLAG_GLOBAL_MATCHING) != 0;
    bp.reorder = (opts.flags & ECSPMV_FLAG_NO_REORDER) == 0;
    bp.keep_small_sets = (opts.flags & ECSPMV_FLAG_KEEP_SMALL_SETS) != 0;
    bp.cluster_rows = (opts.flags & ECSPMV_FLAG_CLUSTER_ROWS) != 0;
    return ECSPMV_OK;
}

int finish_build(const ecs::Csr &A, const ecs::BuildParams &bp, ecspmv_matrix **out)
{
    ecspmv_matrix *h = new (std::nothrow) ecspmv_matrix;
    if (!h) return ECSPMV_ERR_NOMEM;
    int e = ecs::build_image(A, bp, h->image);
    if (e) {
        delete h;
        return map_build_error(e);
    }
    if (h->image.lds_bytes > 160u * 1024u) {
        delete h;
        return ECSPMV_ERR_UNSUPPORTED;
    }
    *out = h;
    return ECSPMV_OK;
}

// shared by ecspmv_decode (FP16 images, 16-bit values out) and ecspmv_decode_f32 (FP32 images, 32-bit values out)
template <typename T>
int decode_t(const ecspmv_matrix *A, int value_bits, int64_t *nnz, int32_t *rows, int32_t *cols, T *vals)
{
    if (!A || !nnz) return ECSPMV_ERR_INVALID;
    if (A->image.value_bits != value_bits) return ECSPMV_ERR_INVALID;
    try {
        ecs::Triples t;
        if (ecs::walk_image(A->image, &t, nullptr)) return ECSPMV_ERR_INVALID;
        const int64_t count = (int64_t)t.rows.size();
        if (!rows && !cols && !vals) {
            *nnz = count;
            return ECSPMV_OK;
        }
        if (!rows || !cols || !vals) return ECSPMV_ERR_INVALID;
        if (*nnz < count) return ECSPMV_ERR_TOO_SMALL;
        if (count) {
            std::memcpy(rows, t.rows.data(), sizeof(int32_t) * (size_t)count);
            std::memcpy(cols, t.cols.data(), sizeof(int32_t) * (size_t)count);
            for (int64_t i = 0; i < count; ++i) vals[i] = (T)t.vals[(size_t)i];
        }
        *nnz = count;
        return ECSPMV_OK;
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

}  // namespace

extern "C" {

int ecspmv_build_dense(const uint16_t *W, int64_t m, int64_t n, int64_t ld, const ecspmv_build_opts *opts,
                       ecspmv_matrix **out)
{
    if (!W || !out || m <= 0 || n <= 0 || ld < n) return ECSPMV_ERR_INVALID;
    if (n > 65535 || m > 0x7fffffff) return ECSPMV_ERR_UNSUPPORTED;
    ecs::BuildParams bp;
    int s = parse_opts(opts, bp);
    if (s) return s;
    try {
        ecs::Csr A;
        ecs::csr_from_dense(W, m, n, ld, bp.num_threads, A);
        return finish_build(A, bp, out);
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

int ecspmv_build_csr(const int64_t *rowptr, const int32_t *col, const uint16_t *val, int64_t m, int64_t n,
                     const ecspmv_build_opts *opts, ecspmv_matrix **out)
{
    if (!rowptr || !out || m <= 0 || n <= 0) return ECSPMV_ERR_INVALID;
    if (rowptr[m] < 0 || (rowptr[m] > 0 && (!col || !val))) return ECSPMV_ERR_INVALID;
    if (n > 65535 || m > 0x7fffffff) return ECSPMV_ERR_UNSUPPORTED;
    ecs::BuildParams bp;
    int s = parse_opts(opts, bp);
    if (s) return s;
    try {
        ecs::Csr A;
        if (ecs::csr_from_csr(rowptr, col, val, m, n, A)) return ECSPMV_ERR_INVALID;
        return finish_build(A, bp, out);
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

int ecspmv_build_dense_f32(const float *W, int64_t m, int64_t n, int64_t ld, const ecspmv_build_opts *opts,
                           ecspmv_matrix **out)
{
    if (!W || !out || m <= 0 || n <= 0 || ld < n) return ECSPMV_ERR_INVALID;
    if (n > 65535 || m > 0x7fffffff) return ECSPMV_ERR_UNSUPPORTED;
    ecs::BuildParams bp;
    int s = parse_opts(opts, bp, 32);
    if (s) return s;
    try {
        ecs::Csr A;
        ecs::csr_from_dense_f32(reinterpret_cast<const uint32_t *>(W), m, n, ld, bp.num_threads, A);
        return finish_build(A, bp, out);
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

int ecspmv_build_csr_f32(const int64_t *rowptr, const int32_t *col, const float *val, int64_t m, int64_t n,
                         const ecspmv_build_opts *opts, ecspmv_matrix **out)
{
    if (!rowptr || !out || m <= 0 || n <= 0) return ECSPMV_ERR_INVALID;
    if (rowptr[m] < 0 || (rowptr[m] > 0 && (!col || !val))) return ECSPMV_ERR_INVALID;
    if (n > 65535 || m > 0x7fffffff) return ECSPMV_ERR_UNSUPPORTED;
    ecs::BuildParams bp;
    int s = parse_opts(opts, bp, 32);
    if (s) return s;
    try {
        ecs::Csr A;
        if (ecs::csr_from_csr_f32(rowptr, col, reinterpret_cast<const uint32_t *>(val), m, n, A)) return ECSPMV_ERR_INVALID;
        return finish_build(A, bp, out);
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

void ecspmv_destroy(ecspmv_matrix *A) { delete A; }

int ecspmv_stats(const ecspmv_matrix *A, ecspmv_stats_t *st)
{
    if (!A || !st || st->struct_size < sizeof(uint32_t)) return ECSPMV_ERR_INVALID;
    const uint32_t want = st->struct_size < sizeof(ecspmv_stats_t) ? st->struct_size : (uint32_t)sizeof(ecspmv_stats_t);
    ecspmv_stats_t tmp = A->image.stats;
    tmp.struct_size = want;
    std::memcpy(st, &tmp, want);
    return ECSPMV_OK;
}

int ecspmv_decode(const ecspmv_matrix *A, int64_t *nnz, int32_t *rows, int32_t *cols, uint16_t *vals)
{
    return decode_t<uint16_t>(A, 16, nnz, rows, cols, vals);
}

int ecspmv_decode_f32(const ecspmv_matrix *A, int64_t *nnz, int32_t *rows, int32_t *cols, float *vals)
{
    return decode_t<uint32_t>(A, 32, nnz, rows, cols, reinterpret_cast<uint32_t *>(vals));
}

int ecspmv_block_sets(const ecspmv_matrix *A, int64_t *n_units, int64_t *n_rows, int32_t *g, int32_t *unit_rows,
                      int32_t *unit_cols)
{
    if (!A || !n_units || !n_rows) return ECSPMV_ERR_INVALID;
    try {
        ecs::BlockSets b;
        if (ecs::walk_image(A->image, nullptr, &b)) return ECSPMV_ERR_INVALID;
        const int64_t nu = (int64_t)b.g.size(), nr = (int64_t)b.rows.size();
        if (!g && !unit_rows && !unit_cols) {
            *n_units = nu;
            *n_rows = nr;
            return ECSPMV_OK;
        }
        if (!g || !unit_rows || !unit_cols) return ECSPMV_ERR_INVALID;
        if (*n_units < nu || *n_rows < nr) return ECSPMV_ERR_TOO_SMALL;
        if (nu) {
            std::memcpy(g, b.g.data(), sizeof(int32_t) * (size_t)nu);
            std::memcpy(unit_rows, b.rows.data(), sizeof(int32_t) * (size_t)nr);
            std::memcpy(unit_cols, b.cols.data(), sizeof(int32_t) * (size_t)nu * ECS_UNIT_COLS);
        }
        *n_units = nu;
        *n_rows = nr;
        return ECSPMV_OK;
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

int ecspmv_device_bytes(const ecspmv_matrix *A, size_t *bytes)
{
    if (!A || !bytes) return ECSPMV_ERR_INVALID;
    *bytes = A->image.bytes.size();
    return ECSPMV_OK;
}

int ecspmv_export_image(const ecspmv_matrix *A, void *host_dst, size_t bytes)
{
    if (!A || !host_dst) return ECSPMV_ERR_INVALID;
    if (bytes < A->image.bytes.size()) return ECSPMV_ERR_TOO_SMALL;
    std::memcpy(host_dst, A->image.bytes.data(), A->image.bytes.size());
    return ECSPMV_OK;
}

int ecspmv_upload(ecspmv_matrix *A, void *d_buf, size_t bytes, void *stream)
{
    if (!A || !d_buf || (reinterpret_cast<uintptr_t>(d_buf) & 255)) return ECSPMV_ERR_INVALID;
    if (bytes < A->image.bytes.size()) return ECSPMV_ERR_TOO_SMALL;
    int lim = 0;
    int e = lds_limit(&lim);
    if (e) return hip_status(e);
    if ((int64_t)A->image.lds_bytes > (int64_t)lim) return ECSPMV_ERR_UNSUPPORTED;
    e = ecs::copy_to_device(d_buf, A->image.bytes.data(), A->image.bytes.size(), stream);
    if (e) return hip_status(e);
    A->d_image = d_buf;
    return ECSPMV_OK;
}

int ecspmv_run_batch(const ecspmv_matrix *const *As, const void *const *d_xs, void *const *d_ys, int32_t count,
                     void *stream)
{
    if (!As || !d_xs || !d_ys || count <= 0) return ECSPMV_ERR_INVALID;
    for (int32_t i = 0; i < count; ++i) {
        if (!As[i] || !d_xs[i] || !d_ys[i]) return ECSPMV_ERR_INVALID;
        const uintptr_t align = (uintptr_t)(As[i]->image.value_bits / 8 - 1);       // x, y: 2- or 4-byte aligned
        if ((reinterpret_cast<uintptr_t>(d_xs[i]) & align) || (reinterpret_cast<uintptr_t>(d_ys[i]) & align))
            return ECSPMV_ERR_INVALID;
        if (!As[i]->d_image) return ECSPMV_ERR_NOT_UPLOADED;
    }
    // one launch per run of up to ECS_MAX_BATCH matrices with the same delta width and value width; nothing on
    // this path allocates or can throw
    for (int32_t base = 0, nb = 0; base < count; base += nb) {
        const int bits = As[base]->image.delta_bits;
        const int vbits = As[base]->image.value_bits;
        for (nb = 1; base + nb < count && nb < ECS_MAX_BATCH; ++nb) {
            const ecs::Image &nx = As[base + nb]->image;
            if (nx.delta_bits != bits || nx.value_bits != vbits) break;
        }
        ecs::EcsBatch b;
        std::memset(&b, 0, sizeof(b));
        b.count = (uint32_t)nb;
        uint32_t blocks = 0, lds = 0, mask = 0;
        for (int32_t i = 0; i < nb; ++i) {
            const int32_t src = base + i;
            const ecs::Image &im = As[src]->image;
            ecs::EcsBatchItem &it = b.item[i];
            it.image = static_cast<const uint8_t *>(As[src]->d_image);
            it.x = static_cast<const uint16_t *>(d_xs[src]);
            it.y = static_cast<uint16_t *>(d_ys[src]);
            it.n = (uint32_t)im.n;
            it.panel_stride = im.panel_stride;
            it.meta_stride = im.meta_stride;
            it.x_bytes = ((uint32_t)im.n * (uint32_t)(vbits / 8) + 15u) / 16u * 16u;
            blocks += (uint32_t)im.num_panels;
            it.block_end = blocks;
            lds = im.lds_bytes > lds ? im.lds_bytes : lds;
            mask |= im.type_mask;
        }
        // Workgroup size: a lone SpMV gets one 1024-thread workgroup per compute unit; in a batch, 512-thread
        // workgroups of neighbouring matrices share compute units and hide each other's start and end phases.
        uint32_t threads = nb > 1 ? 512u : 1024u;
        for (int32_t i = 0; i < nb; ++i) {
            const int t = As[base + i]->image.threads_per_wg;
            if (t) threads = (uint32_t)t;                      // a build-time choice overrides
        }
        int s = hip_status(ecs::launch_ecspmv(b, threads, lds, mask, (uint32_t)bits, (uint32_t)vbits, stream));
        if (s) return s;
    }
    return ECSPMV_OK;
}

int ecspmv_run(const ecspmv_matrix *A, const void *d_x, void *d_y, void *stream)
{
    return ecspmv_run_batch(&A, &d_x, &d_y, 1, stream);
}

int ecspmv_run_multi(const ecspmv_matrix *A, const void *d_X, void *d_Y, int32_t nb, void *stream)
{
    if (!A || !d_X || !d_Y) return ECSPMV_ERR_INVALID;
    if (nb == 1) return ecspmv_run(A, d_X, d_Y, stream);
    if (nb != 2 && nb != 4 && nb != 8) return ECSPMV_ERR_INVALID;
    const ecs::Image &im = A->image;
    const uint32_t vw = (uint32_t)im.value_bits / 8u;                 // bytes per value of W, X and Y
    if ((reinterpret_cast<uintptr_t>(d_X) & (vw - 1u)) || (reinterpret_cast<uintptr_t>(d_Y) & (vw - 1u)))
        return ECSPMV_ERR_INVALID;
    if (!A->d_image) return ECSPMV_ERR_NOT_UPLOADED;
    // registers run out with a 16-grained set, and with an 8-grained one if the values are FP32; absolute 16-bit
    // columns (index compression off) exist for one vector only
    if (im.type_mask & (vw == 4 ? ~3u : ~7u)) return ECSPMV_ERR_UNSUPPORTED;
    if (im.delta_bits == 16) return ECSPMV_ERR_UNSUPPORTED;
    int lim = 0;
    int e = lds_limit(&lim);
    if (e) return hip_status(e);
    // All nb right-hand sides in one launch if X and the partial sums fit LDS; otherwise several launches of nb / 2
    // or nb / 4 right-hand sides each, which read their columns of X and write their columns of Y with the row
    // stride nb (the image is then read once per launch).
    uint32_t per = (uint32_t)nb, x_bytes = 0;
    uint64_t lds = 0;
    for (;; per /= 2) {
        x_bytes = ((uint32_t)im.n * vw * per + 15u) / 16u * 16u;
        const uint32_t slot_bytes = (im.max_slots * 4u * per + 15u) / 16u * 16u;
        lds = (uint64_t)x_bytes + im.meta_stride + slot_bytes;
        if (lds <= (uint64_t)lim) break;
        if (per == 2) return ECSPMV_ERR_UNSUPPORTED;                  // not even two right-hand sides fit
    }
    const uint32_t threads = im.threads_per_wg ? (uint32_t)im.threads_per_wg : 1024u;
    for (uint32_t c0 = 0; c0 < (uint32_t)nb; c0 += per) {
        ecs::EcsBatch b;
        std::memset(&b, 0, sizeof(b));
        b.count = 1;
        ecs::EcsBatchItem &it = b.item[0];
        it.image = static_cast<const uint8_t *>(A->d_image);
        it.x = reinterpret_cast<const uint16_t *>(static_cast<const uint8_t *>(d_X) + (size_t)c0 * vw);
        it.y = reinterpret_cast<uint16_t *>(static_cast<uint8_t *>(d_Y) + (size_t)c0 * vw);
        it.n = (uint32_t)im.n;
        it.panel_stride = im.panel_stride;
        it.meta_stride = im.meta_stride;
        it.x_bytes = x_bytes;
        it.block_end = (uint32_t)im.num_panels;
        it.row_stride = (uint32_t)nb;                                 // of X and Y, in elements
        int s = hip_status(ecs::launch_ecspmv_multi(b, threads, (uint32_t)lds, im.type_mask, (uint32_t)im.delta_bits,
                                                    (uint32_t)im.value_bits, per, stream));
        if (s) return s;
    }
    return ECSPMV_OK;
}

int ecspmv_csr_build_dense(const uint16_t *W, int64_t m, int64_t n, int64_t ld, ecspmv_csr **out)
{
    if (!W || !out || m <= 0 || n <= 0 || ld < n) return ECSPMV_ERR_INVALID;
    try {
        ecs::Csr A;
        ecs::csr_from_dense(W, m, n, ld, 0, A);
        if (A.rowptr[(size_t)m] > 0x7fffffff || m > 0x7ffffffe) return ECSPMV_ERR_UNSUPPORTED;
        ecspmv_csr *c = new (std::nothrow) ecspmv_csr;
        if (!c) return ECSPMV_ERR_NOMEM;
        c->m = m;
        c->n = n;
        c->nnz = A.rowptr[(size_t)m];
        c->rowptr.resize((size_t)m + 1);
        for (int64_t i = 0; i <= m; ++i) c->rowptr[(size_t)i] = (int32_t)A.rowptr[(size_t)i];
        c->col.swap(A.col);
        c->val.assign(A.val.begin(), A.val.end());                 // FP16 bit patterns out of their 32-bit containers
        auto up = [](size_t v) { return (v + 255) / 256 * 256; };
        c->off_col = up(4 * ((size_t)m + 1));
        c->off_val = c->off_col + up(4 * (size_t)c->nnz);
        c->bytes = c->off_val + up(2 * (size_t)c->nnz) + 256;
        *out = c;
        return ECSPMV_OK;
    } catch (const std::bad_alloc &) {
        return ECSPMV_ERR_NOMEM;
    } catch (...) {                                  // nothing may leave through the C ABI (a worker thread that could
        return ECSPMV_ERR_INTERNAL;                  // not be started, for instance)
    }
}

void ecspmv_csr_destroy(ecspmv_csr *C) { delete C; }

int ecspmv_csr_device_bytes(const ecspmv_csr *C, size_t *bytes)
{
    if (!C || !bytes) return ECSPMV_ERR_INVALID;
    *bytes = C->bytes;
    return ECSPMV_OK;
}

int ecspmv_csr_upload(ecspmv_csr *C, void *d_buf, size_t bytes, void *stream)
{
    if (!C || !d_buf || (reinterpret_cast<uintptr_t>(d_buf) & 255)) return ECSPMV_ERR_INVALID;
    if (bytes < C->bytes) return ECSPMV_ERR_TOO_SMALL;
    uint8_t *d = static_cast<uint8_t *>(d_buf);
    int e = ecs::copy_to_device(d, C->rowptr.data(), 4 * C->rowptr.size(), stream);
    if (!e && C->nnz) e = ecs::copy_to_device(d + C->off_col, C->col.data(), 4 * C->col.size(), stream);
    if (!e && C->nnz) e = ecs::copy_to_device(d + C->off_val, C->val.data(), 2 * C->val.size(), stream);
    if (e) return hip_status(e);
    C->d_buf = d;
    return ECSPMV_OK;
}

int ecspmv_csr_run(const ecspmv_csr *C, const void *d_x, void *d_y, void *stream)
{
    if (!C || !d_x || !d_y) return ECSPMV_ERR_INVALID;
    if (!C->d_buf) return ECSPMV_ERR_NOT_UPLOADED;
    return hip_status(ecs::launch_csr(C->d_buf, C->d_buf + C->off_col, C->d_buf + C->off_val, d_x, d_y, (uint32_t)C->m,
                                      stream));
}

int ecspmv_stream_read(const void *d_buf, size_t bytes, void *d_out, int32_t num_wg, void *stream)
{
    if (!d_buf || !d_out || num_wg <= 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(d_buf) & 15))
        return ECSPMV_ERR_INVALID;
    return hip_status(ecs::launch_stream_read(d_buf, bytes, d_out, (uint32_t)num_wg, 1024u, false, stream));
}

int ecspmv_stream_read_sliced(const void *d_buf, size_t bytes, void *d_out, int32_t num_wg, int32_t threads_per_wg,
                              void *stream)
{
    if (!d_buf || !d_out || num_wg <= 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(d_buf) & 15))
        return ECSPMV_ERR_INVALID;
    if (threads_per_wg != 256 && threads_per_wg != 512 && threads_per_wg != 1024) return ECSPMV_ERR_INVALID;
    return hip_status(ecs::launch_stream_read(d_buf, bytes, d_out, (uint32_t)num_wg, (uint32_t)threads_per_wg, true,
                                              stream));
}

int ecspmv_empty_launch(void *d_out, int32_t num_wg, int32_t threads_per_wg, int32_t count, void *stream)
{
    if (!d_out || num_wg <= 0 || count <= 0 || threads_per_wg < 64 || threads_per_wg > 1024 || (threads_per_wg & 63))
        return ECSPMV_ERR_INVALID;
    for (int32_t i = 0; i < count; ++i) {
        int s = hip_status(ecs::launch_empty(d_out, (uint32_t)num_wg, (uint32_t)threads_per_wg, stream));
        if (s) return s;
    }
    return ECSPMV_OK;
}

#ifdef ECS_TRACE
// Only in the library built with -DECS_TRACE (libecspmv_trace.so, which the timeline script loads; the product library
// has no stamps compiled in).  Each of the next `regions` launches leaves, per wavefront, the clock at its first
// instruction, at point `sel` of the kernel and at its last instruction in its own region of d_words (device,
// regions x wgs_per_region x 128 uint64).  NULL switches the stamps off.
int ecspmv_trace_buffer(void *d_words, uint32_t regions, uint32_t wgs_per_region, uint32_t sel)
{
    return hip_status(ecs::set_trace_buffer(d_words, regions, wgs_per_region, sel));
}
#endif

const char *ecspmv_strerror(int status)
{
    switch (status) {
    case ECSPMV_OK: return "ok";
    case ECSPMV_ERR_INVALID: return "invalid argument";
    case ECSPMV_ERR_UNSUPPORTED: return "unsupported size or option";
    case ECSPMV_ERR_NOMEM: return "out of host memory";
    case ECSPMV_ERR_HIP: return "HIP call failed (see ecspmv_last_hip_error)";
    case ECSPMV_ERR_NOT_UPLOADED: return "matrix has no device image yet";
    case ECSPMV_ERR_TOO_SMALL: return "buffer too small";
    case ECSPMV_ERR_INTERNAL: return "unexpected failure inside the library";
    default: return "unknown status";
    }
}

int ecspmv_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
