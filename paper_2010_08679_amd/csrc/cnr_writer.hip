// Chunked encode with the device-to-host copy of one chunk overlapping the encode of the next
// (Sections 4.4 and 5.2: the optimized checkpoint is built chunk by chunk and every finished chunk
// is handed on while the next one is being quantized).
//
// Two device staging sets of chunk_rows rows take the encoder's output in turn; a copy stream of
// the writer's own (default priority) moves each finished chunk into the caller's host buffers.
// Events order the two streams: a chunk is copied after it is encoded, and a staging set is encoded
// into again only after its previous content has been copied out.
//
// The way back (Section 5.1, resume: baseline + incremental checkpoint; Section 6.2: de-quantize
// on load) runs through the same staging sets in the other direction: chunk c + 1 is copied from
// host memory while chunk c is de-quantized and scattered into the table.  When the host buffers are
// pinned there is a shorter way: the restore kernel reads them itself.  Its loads cross the host link
// while its stores go to the table, so the link is busy from the first wave to the last, no byte is
// written to device memory before it is used, and no copy engine, second stream or event is involved
// (measured 56-57 GB/s against 50 GB/s for the copies of the staged way).  The encode has the same
// short way, its stores crossing the link; it pays for rows of up to 64 elements, whose codes leave
// a wave as one contiguous block.
#include <new>

#include "cnr_common.h"

struct cnr_host_writer {
    cnr_ctx *ctx;
    uint32_t dim;
    int bits;
    uint64_t chunk_rows;
    size_t row_bytes;  // packed bytes per row
    uint32_t *ids[2];  // staging of the row ids (the way back only: the encoder reads the caller's list)
    float *scale[2], *bias[2];
    uint8_t *packed[2];
    hipStream_t copy;
    hipEvent_t encoded[2], drained[2];    // to host: chunk encoded (caller's stream), copied out (copy stream)
    hipEvent_t arrived[2], consumed[2];   // from host: chunk copied in (copy stream), restored (caller's stream)
    hipEvent_t fence;                     // "everything enqueued on the caller's stream so far"
    bool in_use[2];       // drained[b] has been recorded and not yet waited for
    bool consuming[2];    // consumed[b] has been recorded and not yet waited for
};

namespace {

// The address under which a kernel reaches pinned host memory, or nullptr (and *ok cleared) when p is
// not such memory.  A failed query leaves its error code with the runtime: it is taken out again, so
// that the next call of the caller does not report it.
template <typename T>
const T *device_view(const T *p, bool *ok) {
    if (!p) return nullptr;
    void *d = nullptr;
    if (hipHostGetDevicePointer(&d, const_cast<T *>(p), 0) != hipSuccess || !d) {
        (void)hipGetLastError();
        *ok = false;
        return nullptr;
    }
    return static_cast<const T *>(d);
}

void release(cnr_host_writer *w) {
    for (int b = 0; b < 2; ++b) {
        if (w->ids[b]) (void)hipFree(w->ids[b]);
        if (w->scale[b]) (void)hipFree(w->scale[b]);
        if (w->bias[b]) (void)hipFree(w->bias[b]);
        if (w->packed[b]) (void)hipFree(w->packed[b]);
        if (w->encoded[b]) (void)hipEventDestroy(w->encoded[b]);
        if (w->drained[b]) (void)hipEventDestroy(w->drained[b]);
        if (w->arrived[b]) (void)hipEventDestroy(w->arrived[b]);
        if (w->consumed[b]) (void)hipEventDestroy(w->consumed[b]);
    }
    if (w->fence) (void)hipEventDestroy(w->fence);
    if (w->copy) (void)hipStreamDestroy(w->copy);
    delete w;
}

}  // namespace

extern "C" {

size_t cnr_host_writer_device_bytes(uint32_t dim, int bits, uint64_t chunk_rows) {
    const size_t row_bytes = cnr_packed_row_bytes(dim, bits);
    if (row_bytes == 0) return 0;
    return (size_t)(2u * chunk_rows * (row_bytes + 12u));
}

cnr_status cnr_host_writer_create(cnr_ctx *ctx, uint32_t dim, int bits, uint64_t chunk_rows, cnr_host_writer **out) {
    if (!out) return CNR_E_INVALID;
    *out = nullptr;
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim % 4 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (chunk_rows == 0 || chunk_rows % 16) return CNR_E_INVALID;  // keeps every row-id slice 16-byte aligned
    cnr_host_writer *w = new (std::nothrow) cnr_host_writer();
    if (!w) return CNR_E_INVALID;
    *w = cnr_host_writer{};
    w->ctx = ctx;
    w->dim = dim;
    w->bits = bits;
    w->chunk_rows = chunk_rows;
    w->row_bytes = cnr_packed_row_bytes(dim, bits);
    hipError_t e = hipStreamCreateWithFlags(&w->copy, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&w->fence, hipEventDisableTiming);
    for (int b = 0; b < 2 && e == hipSuccess; ++b) {
        e = hipMalloc((void **)&w->ids[b], chunk_rows * sizeof(uint32_t));
        if (e == hipSuccess) e = hipMalloc((void **)&w->scale[b], chunk_rows * sizeof(float));
        if (e == hipSuccess) e = hipMalloc((void **)&w->bias[b], chunk_rows * sizeof(float));
        if (e == hipSuccess) e = hipMalloc((void **)&w->packed[b], chunk_rows * w->row_bytes);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&w->encoded[b], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&w->drained[b], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&w->arrived[b], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&w->consumed[b], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        release(w);
        return cnr_hip_status(ctx, e);
    }
    *out = w;
    return CNR_OK;
}

cnr_status cnr_host_writer_destroy(cnr_host_writer *w) {
    if (!w) return CNR_E_INVALID;
    cnr_status st = cnr_enter(w->ctx);
    if (st == CNR_OK) st = cnr_hip_status(w->ctx, hipStreamSynchronize(w->copy));
    release(w);
    return st;
}

cnr_status cnr_encode_to_host(cnr_host_writer *w, const float *table, uint64_t n_rows, const uint32_t *row_ids,
                              uint64_t n, cnr_range_mode mode, const cnr_greedy_params *greedy,
                              uint32_t *host_row_ids, float *host_scale, float *host_bias, uint8_t *host_packed,
                              int overlap, void *stream) {
    if (!w) return CNR_E_INVALID;
    cnr_ctx *ctx = w->ctx;
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (n == 0) return CNR_OK;
    if (!host_scale || !host_bias || !host_packed || (row_ids && !host_row_ids)) return CNR_E_INVALID;
    if (!row_ids && n > n_rows) return CNR_E_INVALID;  // without a row list the rows are 0 .. n-1 of the table
    if (overlap < CNR_HOST_SERIAL || overlap > CNR_HOST_DIRECT) return CNR_E_INVALID;
    hipStream_t main = as_stream(stream);
    hipError_t e = hipSuccess;
    if (overlap == CNR_HOST_DIRECT) {
        // The encode kernel stores scale, bias and codes into the pinned buffers itself; the id list,
        // which exists before the encode starts, is copied on the writer's stream meanwhile.
        bool pinned = true;
        float *scale = const_cast<float *>(device_view(host_scale, &pinned));
        float *bias = const_cast<float *>(device_view(host_bias, &pinned));
        uint8_t *packed = const_cast<uint8_t *>(device_view(host_packed, &pinned));
        if (row_ids) (void)device_view(host_row_ids, &pinned);
        if (!pinned) return CNR_E_HOST_MEMORY;
        if (row_ids) {
            e = hipEventRecord(w->fence, main);  // the list is complete once `stream` gets here
            if (e == hipSuccess) e = hipStreamWaitEvent(w->copy, w->fence, 0);
            if (e == hipSuccess) e = hipMemcpyAsync(host_row_ids, row_ids, n * sizeof(uint32_t), hipMemcpyDeviceToHost, w->copy);
            if (e != hipSuccess) return cnr_hip_status(ctx, e);
        }
        return cnr_quantize_rows(ctx, table, n_rows, w->dim, row_ids, nullptr, n, w->bits, mode, greedy, scale, bias,
                                 nullptr, nullptr, nullptr, packed, stream);
    }
    hipStream_t copier = overlap == CNR_HOST_OVERLAP ? w->copy : main;
    uint64_t c = 0;
    for (uint64_t k0 = 0; k0 < n && e == hipSuccess; k0 += w->chunk_rows, ++c) {
        const uint64_t m = n - k0 < w->chunk_rows ? n - k0 : w->chunk_rows;
        const int b = (int)(c & 1);
        w->consuming[b] = false;  // a restore that read this set is ahead of the encode on `stream`
        if (w->in_use[b]) {  // the staging set still holds a chunk that is being copied out
            e = hipStreamWaitEvent(main, w->drained[b], 0);
            if (e != hipSuccess) break;
            w->in_use[b] = false;
        }
        if (row_ids)
            st = cnr_quantize_rows(ctx, table, n_rows, w->dim, row_ids + k0, nullptr, m, w->bits, mode, greedy,
                                   w->scale[b], w->bias[b], nullptr, nullptr, nullptr, w->packed[b], stream);
        else  // rows k0 .. k0 + m - 1: the table from row k0 on, without a list
            st = cnr_quantize_rows(ctx, table + k0 * w->dim, n_rows - k0, w->dim, nullptr, nullptr, m, w->bits, mode,
                                   greedy, w->scale[b], w->bias[b], nullptr, nullptr, nullptr, w->packed[b], stream);
        if (st != CNR_OK) return st;
        if (copier != main) {
            e = hipEventRecord(w->encoded[b], main);
            if (e == hipSuccess) e = hipStreamWaitEvent(copier, w->encoded[b], 0);
            if (e != hipSuccess) break;
        }
        if (row_ids) e = hipMemcpyAsync(host_row_ids + k0, row_ids + k0, m * sizeof(uint32_t), hipMemcpyDeviceToHost, copier);
        if (e == hipSuccess) e = hipMemcpyAsync(host_scale + k0, w->scale[b], m * sizeof(float), hipMemcpyDeviceToHost, copier);
        if (e == hipSuccess) e = hipMemcpyAsync(host_bias + k0, w->bias[b], m * sizeof(float), hipMemcpyDeviceToHost, copier);
        if (e == hipSuccess)
            e = hipMemcpyAsync(host_packed + k0 * w->row_bytes, w->packed[b], m * w->row_bytes, hipMemcpyDeviceToHost, copier);
        if (e == hipSuccess && copier != main) {
            e = hipEventRecord(w->drained[b], copier);
            w->in_use[b] = e == hipSuccess;
        }
    }
    return cnr_hip_status(ctx, e);
}

cnr_status cnr_restore_from_host(cnr_host_writer *w, float *table, uint64_t n_rows, const uint32_t *host_row_ids,
                                 const float *host_scale, const float *host_bias, const uint8_t *host_packed,
                                 uint64_t n, int overlap, void *stream) {
    if (!w) return CNR_E_INVALID;
    cnr_ctx *ctx = w->ctx;
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (n == 0) return CNR_OK;
    if (!table || !host_scale || !host_bias || !host_packed || n_rows == 0) return CNR_E_INVALID;
    if (!host_row_ids && n > n_rows) return CNR_E_INVALID;  // without ids the rows are 0 .. n-1 of the table
    if (overlap < CNR_HOST_SERIAL || overlap > CNR_HOST_DIRECT) return CNR_E_INVALID;
    if (overlap == CNR_HOST_DIRECT) {
        bool pinned = true;
        const uint32_t *ids = device_view(host_row_ids, &pinned);
        const float *scale = device_view(host_scale, &pinned);
        const float *bias = device_view(host_bias, &pinned);
        const uint8_t *packed = device_view(host_packed, &pinned);
        if (!pinned) return CNR_E_HOST_MEMORY;
        return cnr_restore_rows(ctx, table, n_rows, w->dim, ids, nullptr, n, w->bits, packed, scale, bias, stream);
    }
    hipStream_t main = as_stream(stream);
    hipStream_t copier = overlap == CNR_HOST_OVERLAP ? w->copy : main;
    hipError_t e = hipSuccess;
    if (copier != main) {
        // whatever the caller's stream still does with the staging sets or the host buffers comes first
        e = hipEventRecord(w->fence, main);
        if (e == hipSuccess) e = hipStreamWaitEvent(copier, w->fence, 0);
        w->consuming[0] = w->consuming[1] = false;
    }
    uint64_t c = 0;
    for (uint64_t k0 = 0; k0 < n && e == hipSuccess; k0 += w->chunk_rows, ++c) {
        const uint64_t m = n - k0 < w->chunk_rows ? n - k0 : w->chunk_rows;
        const int b = (int)(c & 1);
        if (w->consuming[b]) {  // the chunk before last of this call is still being restored from this set
            e = hipStreamWaitEvent(copier, w->consumed[b], 0);
            if (e != hipSuccess) break;
            w->consuming[b] = false;
        }
        if (host_row_ids) e = hipMemcpyAsync(w->ids[b], host_row_ids + k0, m * sizeof(uint32_t), hipMemcpyHostToDevice, copier);
        if (e == hipSuccess) e = hipMemcpyAsync(w->scale[b], host_scale + k0, m * sizeof(float), hipMemcpyHostToDevice, copier);
        if (e == hipSuccess) e = hipMemcpyAsync(w->bias[b], host_bias + k0, m * sizeof(float), hipMemcpyHostToDevice, copier);
        if (e == hipSuccess)
            e = hipMemcpyAsync(w->packed[b], host_packed + k0 * w->row_bytes, m * w->row_bytes, hipMemcpyHostToDevice, copier);
        if (e == hipSuccess && copier != main) {
            e = hipEventRecord(w->arrived[b], copier);
            if (e == hipSuccess) e = hipStreamWaitEvent(main, w->arrived[b], 0);
        }
        if (e != hipSuccess) break;
        if (host_row_ids)
            st = cnr_restore_rows(ctx, table, n_rows, w->dim, w->ids[b], nullptr, m, w->bits, w->packed[b], w->scale[b],
                                  w->bias[b], stream);
        else
            st = cnr_restore_rows(ctx, table + k0 * w->dim, n_rows - k0, w->dim, nullptr, nullptr, m, w->bits,
                                  w->packed[b], w->scale[b], w->bias[b], stream);
        if (st != CNR_OK) return st;
        if (copier != main) {
            e = hipEventRecord(w->consumed[b], main);
            w->consuming[b] = e == hipSuccess;
        }
    }
    return cnr_hip_status(ctx, e);
}

cnr_status cnr_host_writer_wait(cnr_host_writer *w, void *stream) {
    if (!w) return CNR_E_INVALID;
    cnr_status st = cnr_enter(w->ctx);
    if (st != CNR_OK) return st;
    hipError_t e = hipStreamSynchronize(as_stream(stream));
    if (e == hipSuccess) e = hipStreamSynchronize(w->copy);
    w->in_use[0] = w->in_use[1] = false;
    w->consuming[0] = w->consuming[1] = false;
    return cnr_hip_status(w->ctx, e);
}

}  // extern "C"
