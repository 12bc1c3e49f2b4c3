// Data streaming (Section 3.2, "Asynchronous Data Streaming"): device memory holds an active and a
// swap buffer; while the kernels work on the chunk in the active buffer (compute stream) the next
// chunk is copied from pinned host memory into the swap buffer (copy stream); events hand the
// buffers over.  A chunk is a range of consecutive coordinates with its slices of idx and val;
// ptr, y, the model and the shared vector stay resident.
#include "common.h"

namespace snap {

int stream_alloc(snap_handle* h) {
    const size_t cap = (size_t)(h->max_chunk_nnz > 0 ? h->max_chunk_nnz : 1);
    for (int b = 0; b < 2; ++b) {
        SNAP_HIP(hipMalloc(&h->buf_idx[b], cap * sizeof(uint32_t)));
        SNAP_HIP(hipMalloc(&h->buf_val[b], cap * sizeof(float)));
        SNAP_HIP(hipEventCreateWithFlags(&h->ev_copied[b], hipEventDisableTiming));
        SNAP_HIP(hipEventCreateWithFlags(&h->ev_free[b], hipEventDisableTiming));
        h->buf_chunk[b] = -1;
        h->buf_folded[b] = false;
    }
    if (h->opt.profile) {
        h->ev_chunk = new (std::nothrow) hipEvent_t[(size_t)(4 * h->n_chunks)]();
        if (!h->ev_chunk) return SNAP_ENOMEM;
        for (int64_t i = 0; i < 4 * h->n_chunks; ++i) SNAP_HIP(hipEventCreate(&h->ev_chunk[i]));
    }
    return SNAP_OK;
}

void stream_free(snap_handle* h) {
    for (int b = 0; b < 2; ++b) {
        (void)hipFree(h->buf_idx[b]);
        (void)hipFree(h->buf_val[b]);
        if (h->ev_copied[b]) (void)hipEventDestroy(h->ev_copied[b]);
        if (h->ev_free[b]) (void)hipEventDestroy(h->ev_free[b]);
        h->buf_idx[b] = nullptr;
        h->buf_val[b] = nullptr;
        h->ev_copied[b] = h->ev_free[b] = nullptr;
    }
    if (h->ev_chunk) {
        for (int64_t i = 0; i < 4 * h->n_chunks; ++i)
            if (h->ev_chunk[i]) (void)hipEventDestroy(h->ev_chunk[i]);
        delete[] h->ev_chunk;
        h->ev_chunk = nullptr;
    }
}

// Enqueue the copy of chunk ch into buffer b on the copy stream, once the last user of b is done.
static int enqueue_copy(snap_handle* h, int64_t ch, int b, bool profile) {
    const snap_handle::Chunk& ck = h->chunks[ch];
    const size_t count = (size_t)(ck.nnz1 - ck.nnz0);
    SNAP_HIP(hipStreamWaitEvent(h->copy, h->ev_free[b], 0));
    if (profile) {
        SNAP_HIP(hipEventRecord(h->ev_chunk[4 * ch + 0], h->copy));
        h->chunk_copy_timed[(size_t)ch] = 1;
    }
    if (count > 0) {
        h->bytes_copied += (int64_t)(count * (h->stream_unit ? sizeof(uint32_t) : sizeof(uint32_t) + sizeof(float)));
        SNAP_HIP(hipMemcpyAsync(h->buf_idx[b], h->host_idx + ck.nnz0, count * sizeof(uint32_t), hipMemcpyHostToDevice,
                                h->copy));
        if (!h->stream_unit)       // (pattern-only data: the value buffers hold ones for good)
            SNAP_HIP(hipMemcpyAsync(h->buf_val[b], h->host_val + ck.nnz0, count * sizeof(float), hipMemcpyHostToDevice,
                                    h->copy));
    }
    if (profile) SNAP_HIP(hipEventRecord(h->ev_chunk[4 * ch + 1], h->copy));
    SNAP_HIP(hipEventRecord(h->ev_copied[b], h->copy));
    h->buf_chunk[b] = ch;
    h->buf_folded[b] = false;
    return SNAP_OK;
}

int for_each_chunk(snap_handle* h, ChunkFn fn, void* arg, bool fold, bool profile) {
    // the chunks to visit: all of them in order, or the caller's list (Section 3.2: a round may process
    // part of the data)
    const int64_t C = h->pass_list ? h->pass_count : h->n_chunks;
    if (C == 0) return SNAP_OK;
    if (!h->streaming) {
        ChunkView cv{h->ptr, h->idx, h->val, 0, 0, h->m};
        return fn(h, 0, cv, arg);
    }
    auto chunk_at = [&](int64_t i) { return h->pass_list ? h->pass_list[i] : i; };
    profile = profile && h->ev_chunk != nullptr && !h->pass_list;
    const int64_t first = chunk_at(0);
    // A profiled pass times the copies it enqueues, whichever pass they serve: the fetch of the first
    // chunk normally happens at the end of the pass before and is counted there.
    if (profile) h->chunk_copy_timed.assign((size_t)h->n_chunks, 0);
    int b = h->buf_chunk[0] == first ? 0 : (h->buf_chunk[1] == first ? 1 : -1);
    if (b < 0) {
        b = 0;
        SNAP_TRY(enqueue_copy(h, first, b, profile));
    }
    for (int64_t i = 0; i < C; ++i) {
        const int64_t ch = chunk_at(i);
        const int nb = 1 - b;
        const snap_handle::Chunk& ck = h->chunks[ch];
        // the next chunk (after the last one: the first again, for the next pass) goes to the other buffer
        // while this one is processed -- unless it still sits there from an earlier pass (a working
        // set of two chunks is copied once)
        const int64_t next = i + 1 < C ? chunk_at(i + 1) : first;
        if (next != ch && h->buf_chunk[nb] != next) SNAP_TRY(enqueue_copy(h, next, nb, profile));
        SNAP_HIP(hipStreamWaitEvent(h->compute, h->ev_copied[b], 0));
        if (profile) SNAP_HIP(hipEventRecord(h->ev_chunk[4 * ch + 2], h->compute));
        if (fold && h->kind == K_PRIMAL_LOGISTIC && !h->buf_folded[b]) {
            SNAP_TRY(fold_labels(h, h->buf_idx[b], ck.nnz1 - ck.nnz0, h->compute));
            h->buf_folded[b] = true;
        }
        ChunkView cv{h->ptr, h->buf_idx[b], h->buf_val[b], ck.nnz0, ck.c0, ck.c1};
        SNAP_TRY(fn(h, ch, cv, arg));
        if (profile) SNAP_HIP(hipEventRecord(h->ev_chunk[4 * ch + 3], h->compute));
        SNAP_HIP(hipEventRecord(h->ev_free[b], h->compute));
        b = nb;
    }
    if (profile) h->chunk_events_valid = true;
    else if (h->pass_list) h->chunk_events_valid = false;
    // The pass ends with the host waiting for the copy stream (by then only the fetch of chunk 0 for
    // the next pass is outstanding).  Measured: when the host instead runs a whole pass ahead of the
    // copy stream, the copy commands and the kernels stop overlapping (68 ms per chunk instead of 40
    // on the 200 M-row workload: each kernel then starts only when the next chunk's copy has ended).
    SNAP_HIP(hipStreamSynchronize(h->copy));
    return SNAP_OK;
}

}  // namespace snap
