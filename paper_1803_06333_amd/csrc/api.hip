// The C ABI of libsnap (see include/snap.h): argument checking, data placement, the epoch driver.
#include "common.h"
#include "perm_key.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <mutex>
#include <cmath>
#include <algorithm>
#include <new>
#include <vector>

namespace snap {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char* what, const char* file, int line) {
    set_error("HIP error %d (%s) in %s at %s:%d", (int)e, hipGetErrorString(e), what, file, line);
    return e == hipErrorOutOfMemory ? SNAP_ENOMEM : SNAP_EHIP;
}

__global__ void k_check_indices(const int32_t* __restrict__ idx, int64_t count, int64_t minor, uint32_t* flag) {
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < count; k += (int64_t)gridDim.x * blockDim.x)
        if (idx[k] < 0 || (int64_t)idx[k] >= minor) atomicOr(flag, 1u);
}

__global__ void k_check_labels(const float* __restrict__ y, int64_t n, uint32_t* flag) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        if (!(y[i] == 1.0f || y[i] == -1.0f)) atomicOr(flag, 2u);
}

// streaming: are all stored values 1.0 (pattern-only data, e.g. one-hot encodings)?  flag bit 2 says no
__global__ void k_check_unit_values(const float* __restrict__ val, int64_t count, uint32_t* flag) {
    bool other = false;
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < count; k += (int64_t)gridDim.x * blockDim.x)
        other |= val[k] != 1.0f;
    if (other) atomicOr(flag, 4u);
}

// the status word reaches the host through mapped pinned memory (a copy command could wait behind
// the chunk copies of a streamed pass)
__global__ void k_publish_status(const uint32_t* __restrict__ status, double* __restrict__ host_mapped) {
    if (threadIdx.x == 0) reinterpret_cast<uint32_t*>(host_mapped)[0] = *status;
}

__global__ void k_clear_status_bits(uint32_t* status, uint32_t mask) {
    if (threadIdx.x == 0) *status &= ~mask;
}

// The handle's status word as it stands once the work enqueued so far is done (synchronises).
int read_status(snap_handle* h, uint32_t* st) {
    hipLaunchKernelGGL(k_publish_status, dim3(1), dim3(WAVE), 0, h->compute, h->status, h->red.host_mapped + 7);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipStreamSynchronize(h->compute));
    *st = reinterpret_cast<const uint32_t*>(h->red.host + 7)[0];
    return SNAP_OK;
}

static int alloc_snapshots(snap_handle* h) {
    if (!h->x_snap) SNAP_HIP(hipMalloc(&h->x_snap, (size_t)(h->m ? h->m : 1) * sizeof(float)));
    if (!h->v_snap) SNAP_HIP(hipMalloc(&h->v_snap, (size_t)(h->vlen ? h->vlen : 1) * sizeof(float)));
    return SNAP_OK;
}

// Group sweeps of the ridge loss keep their sums in 64-bit fixed point with 2^39 of range; a term
// beyond 2^14 raises STATUS_RANGE.  The handle then leaves the group sweeps for good and goes on with
// the asynchronous engine, which has no such limit: the caller sees a slower epoch, not an error.
int leave_group_sweeps(snap_handle* h) {
    hipLaunchKernelGGL(k_clear_status_bits, dim3(1), dim3(WAVE), 0, h->compute, h->status, STATUS_RANGE);
    SNAP_HIP(hipGetLastError());
    h->grouped = false;
    h->group_fallback = true;
    h->perm_stale = false;
    (void)hipFree(h->share_bounds);                      // (the gap shares are per chunk from now on, not per group)
    (void)hipFree(h->share_out);
    h->share_bounds = nullptr;
    h->share_out = nullptr;
    h->adaptive = h->opt.adaptive != 2;                  // the asynchronous engine's default: accept check on
    if (h->adaptive) {
        SNAP_TRY(alloc_snapshots(h));
        if (h->opt.max_inflight_nnz <= 0) h->inflight_nnz = std::max<int64_t>(WAVE, (int64_t)(0.25 * (double)h->vlen));
    }
    h->monitor_valid = false;
    return SNAP_OK;
}

static int check_status(snap_handle* h) {
    hipLaunchKernelGGL(k_publish_status, dim3(1), dim3(WAVE), 0, h->compute, h->status, h->red.host_mapped + 7);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipStreamSynchronize(h->compute));
    const uint32_t st = reinterpret_cast<const uint32_t*>(h->red.host + 7)[0];
    if (st & STATUS_SPIN) {
        set_error("a scatter work item gave up waiting for its coordinate's step; the state is invalid");
        return SNAP_ESTATE;
    }
    if (st & STATUS_RANGE) {
        set_error("group sweeps: a term a (v - y) reached 2^14, beyond the range of the fixed-point sums; the state "
                  "is invalid (scale the data, or create the handle with auto_groups off and without group_bounds)");
        return SNAP_ESTATE;
    }
    return SNAP_OK;
}

static void destroy(snap_handle* h) {
    if (!h) return;
    if (h->compute) (void)hipStreamSynchronize(h->compute);
    if (h->copy) (void)hipStreamSynchronize(h->copy);
    (void)hipFree(h->ptr);
    (void)hipFree(h->idx);
    (void)hipFree(h->val);
    (void)hipFree(h->y);
    (void)hipFree(h->x);
    (void)hipFree(h->v);
    (void)hipFree(h->norms);
    (void)hipFree(h->cls);
    (void)hipFree(h->w_tmp);
    (void)hipFree(h->gdot);
    (void)hipFree(h->large_list);
    (void)hipFree(h->large_seg_off);
    (void)hipFree(h->seg_partial);
    (void)hipFree(h->keys);
    (void)hipFree(h->perm);
    (void)hipFree(h->order);
    (void)hipFree(h->lstate);
    (void)hipFree(h->item_start);
    (void)hipFree(h->ticket);
    (void)hipFree(h->status);
    (void)hipFree(h->x_snap);
    (void)hipFree(h->v_snap);
    (void)hipFree(h->share_bounds);
    (void)hipFree(h->share_out);
    stream_free(h);
    dense_tiles_free(h);
    grouped_free(h);
    for (auto& e : h->ev)
        if (e) (void)hipEventDestroy(e);
    sorter_free(h->sorter);
    host_keys_free(h);
    reducer_free(h->red);
    delete[] h->chunks;
    delete h;
}



// Creation pass over one chunk: indices in range, squared norms + size classes, access counts.
struct CreatePass {
    uint32_t* freq;
    int64_t minor;
    GroupSearch* search;       // streamed data: the search for groups rides on this pass (else null)
    const int64_t* hptr;
};

static int create_chunk(snap_handle* h, int64_t chunk, const ChunkView& cv, void* arg) {
    CreatePass* cp = (CreatePass*)arg;
    const snap_handle::Chunk& ck = h->chunks[chunk];
    const int64_t count = ck.nnz1 - ck.nnz0;
    if (!h->dense && count > 0)
        hipLaunchKernelGGL(k_check_indices, dim3(4096), dim3(256), 0, h->compute, (const int32_t*)cv.idx, count,
                           cp->minor, h->status);
    if (h->streaming && !h->stream_unit && count > 0)
        hipLaunchKernelGGL(k_check_unit_values, dim3(4096), dim3(256), 0, h->compute, cv.val, count, h->status);
    SNAP_HIP(hipGetLastError());
    if (!h->dense && cp->freq) SNAP_TRY(count_accesses_chunk(h, cv, count, cp->freq));
    SNAP_TRY(norms_and_classes_chunk(h, cv));
    if (cp->search) SNAP_TRY(group_search_advance(h, cp->search, cp->hptr, cv.idx, cv.nnz_base, cv.c1));
    return SNAP_OK;
}

// The library's own streams: one compute and one copy stream per device, created on first use and
// kept for the life of the process.  Handles come and go (a test suite makes hundreds of them) and
// all share these two: a stream may cost the runtime a hardware queue with its pinned host memory,
// and stream creation is not something to have fail in the middle of snap_create when pinned memory
// is short.
static int library_stream(int device, int which, hipStream_t* out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex lock;
    static hipStream_t streams[MAX_DEVICES][3] = {};
    if (device < 0 || device >= MAX_DEVICES) {
        set_error("device index %d out of range", device);
        return SNAP_EINVAL;
    }
    std::lock_guard<std::mutex> guard(lock);
    if (!streams[device][which]) SNAP_HIP(hipStreamCreateWithFlags(&streams[device][which], hipStreamNonBlocking));
    *out = streams[device][which];
    return SNAP_OK;
}

static int build(snap_handle* h, const snap_matrix* A, const float* y) {
    SNAP_HIP(hipGetDevice(&h->device));
    if (h->opt.compute_stream) h->compute = (hipStream_t)h->opt.compute_stream;
    else SNAP_TRY(library_stream(h->device, 0, &h->compute));
    if (h->opt.copy_stream) h->copy = (hipStream_t)h->opt.copy_stream;
    else SNAP_TRY(library_stream(h->device, 1, &h->copy));
    // host-made keys travel on a stream of their own: behind the copy of a whole chunk they would
    // hold up the sweep of the chunk they belong to
    if (h->opt.host_keys) SNAP_TRY(library_stream(h->device, 2, &h->hk_stream));
    for (auto& e : h->ev) SNAP_HIP(hipEventCreate(&e));
    SNAP_TRY(reducer_alloc(h->red));
    SNAP_HIP(hipMalloc(&h->status, sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->ticket, sizeof(uint32_t)));
    SNAP_TRY(fill_zero(h->status, 4, h->compute));
    SNAP_TRY(fill_zero(h->ticket, 4, h->compute));

    const int64_t m = h->m;
    if (const char* e = getenv("SNAP_SEG")) h->seg = std::max<int64_t>(256, atoll(e));          // tuning knobs
    if (const char* e = getenv("SNAP_SMALL_MAX")) h->small_max = std::max<int64_t>(0, atoll(e));

    // ---- offsets: host copy for planning, device copy for the kernels -------------------------------
    std::vector<int64_t> hptr;
    if (!h->dense) {
        hptr.resize((size_t)m + 1);
        SNAP_HIP(hipMemcpy(hptr.data(), A->ptr, (size_t)(m + 1) * sizeof(int64_t), hipMemcpyDefault));
        if (hptr[0] != 0 || hptr[(size_t)m] != h->nnz) {
            set_error("ptr[0] must be 0 and ptr[last] must equal nnz");
            return SNAP_EINVAL;
        }
        for (int64_t c = 0; c < m; ++c)
            if (hptr[(size_t)c + 1] < hptr[(size_t)c]) {
                set_error("ptr is not non-decreasing at %lld", (long long)c);
                return SNAP_EINVAL;
            }
        SNAP_HIP(hipMalloc(&h->ptr, (size_t)(m + 1) * sizeof(int64_t)));
        SNAP_HIP(hipMemcpyAsync(h->ptr, hptr.data(), (size_t)(m + 1) * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
    }
    auto len_of = [&](int64_t c) { return h->dense ? h->ld : hptr[(size_t)c + 1] - hptr[(size_t)c]; };

    // ---- chunks: one for resident data, else ranges of coordinates of at most chunk_bytes ------------
    h->streaming = !h->dense && h->opt.device_budget_bytes > 0 &&
                   (size_t)h->nnz * 8u > h->opt.device_budget_bytes;
    std::vector<snap_handle::Chunk> chunks;
    if (!h->streaming) {
        chunks.push_back({0, m, 0, h->nnz, 0, 0, 0, 0, 0});
    } else {
        if (A->mem != SNAP_MEM_HOST_PINNED) {
            set_error("streaming needs the matrix arrays in pinned host memory (SNAP_MEM_HOST_PINNED)");
            return SNAP_EINVAL;
        }
        const size_t chunk_bytes = h->opt.chunk_bytes ? h->opt.chunk_bytes : ((size_t)4 << 30);
        const int64_t chunk_nnz = std::max<int64_t>(1, (int64_t)(chunk_bytes / 8));
        int64_t c0 = 0;
        while (c0 < m) {
            int64_t c1 = c0 + 1;                       // at least one coordinate per chunk
            while (c1 < m && hptr[(size_t)c1 + 1] - hptr[(size_t)c0] <= chunk_nnz) ++c1;
            chunks.push_back({c0, c1, hptr[(size_t)c0], hptr[(size_t)c1], 0, 0, 0, 0, 0});
            c0 = c1;
        }
        if (chunks.empty()) chunks.push_back({0, 0, 0, 0, 0, 0, 0, 0, 0});
        h->host_ptr = A->ptr;
        h->host_idx = A->idx;
        h->host_val = A->val;
    }
    h->n_chunks = (int64_t)chunks.size();
    std::vector<int64_t> large, seg_off;
    seg_off.push_back(0);
    int64_t small_nnz = 0, n_small_total = 0;
    for (auto& ck : chunks) {
        ck.l0 = (int64_t)large.size();
        for (int64_t c = ck.c0; c < ck.c1; ++c) {
            const int64_t len = len_of(c);
            if (h->dense || len > h->small_max) {
                const int64_t ns = (len + h->seg - 1) / h->seg;
                ++ck.n_large;
                ck.n_items += 2 * ns;
                large.push_back(c);
                seg_off.push_back(seg_off.back() + ns);
            } else {
                ++ck.n_small;
                small_nnz += len;
                h->max_small_len = std::max(h->max_small_len, len);
            }
        }
        ck.l1 = (int64_t)large.size();
        n_small_total += ck.n_small;
        h->max_chunk_m = std::max(h->max_chunk_m, ck.c1 - ck.c0);
        h->max_large = std::max(h->max_large, ck.n_large);
        h->max_chunk_nnz = std::max(h->max_chunk_nnz, ck.nnz1 - ck.nnz0);
    }
    h->chunks = new (std::nothrow) snap_handle::Chunk[chunks.size()];
    if (!h->chunks) return SNAP_ENOMEM;
    std::copy(chunks.begin(), chunks.end(), h->chunks);
    h->n_large_total = (int64_t)large.size();
    h->n_seg_total = seg_off.back();
    h->avg_small_len = n_small_total > 0 ? std::max(1.0, (double)small_nnz / (double)n_small_total) : 1.0;
    h->nnz_small = small_nnz;
    h->nnz_large = h->nnz - small_nnz;

    // ---- device memory ---------------------------------------------------------------------------
    if (h->streaming) {
        SNAP_TRY(stream_alloc(h));
        if (!A->val) {
            // pattern-only data: the value buffers hold ones from the start and nothing but indices is copied
            for (int b = 0; b < 2; ++b) SNAP_TRY(fill_value(h->buf_val[b], 1.0f, h->max_chunk_nnz, h->compute));
            h->stream_unit = true;
        }
    } else if (!h->dense) {
        SNAP_HIP(hipMalloc(&h->idx, (size_t)(h->nnz ? h->nnz : 1) * sizeof(uint32_t)));
        SNAP_HIP(hipMalloc(&h->val, (size_t)(h->nnz ? h->nnz : 1) * sizeof(float)));
        SNAP_HIP(hipMemcpyAsync(h->idx, A->idx, (size_t)h->nnz * sizeof(uint32_t), hipMemcpyDefault, h->compute));
        if (A->val) SNAP_HIP(hipMemcpyAsync(h->val, A->val, (size_t)h->nnz * sizeof(float), hipMemcpyDefault, h->compute));
        else SNAP_TRY(fill_value(h->val, 1.0f, h->nnz, h->compute));
    } else {
        const size_t count = (size_t)h->n * (size_t)h->d;
        SNAP_HIP(hipMalloc(&h->val, (count ? count : 1) * sizeof(float)));
        SNAP_HIP(hipMemcpyAsync(h->val, A->val, count * sizeof(float), hipMemcpyDefault, h->compute));
    }
    SNAP_HIP(hipMalloc(&h->y, (size_t)(h->n ? h->n : 1) * sizeof(float)));
    SNAP_HIP(hipMemcpyAsync(h->y, y, (size_t)h->n * sizeof(float), hipMemcpyDefault, h->compute));
    SNAP_HIP(hipMalloc(&h->x, (size_t)(m ? m : 1) * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->v, (size_t)(h->vlen ? h->vlen : 1) * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->norms, (size_t)(m ? m : 1) * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->cls, (size_t)(m ? m : 1) + 4));
    SNAP_HIP(hipMalloc(&h->w_tmp, (size_t)(h->d ? h->d : 1) * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->gdot, (size_t)(m ? m : 1) * sizeof(double)));
    SNAP_HIP(hipMalloc(&h->keys, (size_t)(m ? m : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->perm, (size_t)(m ? m : 1) * sizeof(uint32_t)));
    SNAP_TRY(fill_zero(h->x, (size_t)m * sizeof(float), h->compute));
    SNAP_TRY(fill_zero(h->v, (size_t)h->vlen * sizeof(float), h->compute));
    SNAP_TRY(fill_zero(h->perm, (size_t)m * sizeof(uint32_t), h->compute));
    SNAP_TRY(fill_zero(h->keys, (size_t)m * sizeof(uint32_t), h->compute));
    SNAP_TRY(sorter_alloc(h->sorter, h->max_chunk_m));
    if (h->opt.host_keys) SNAP_TRY(host_keys_alloc(h, h->max_chunk_m));
    SNAP_HIP(hipMalloc(&h->order, (size_t)(h->max_chunk_m ? h->max_chunk_m : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->lstate, (size_t)(h->max_large + 1) * sizeof(LargeState)));
    SNAP_HIP(hipMalloc(&h->item_start, (size_t)(h->max_large + 2) * sizeof(int64_t)));
    SNAP_HIP(hipMalloc(&h->large_list, (large.size() + 1) * sizeof(int64_t)));
    SNAP_HIP(hipMalloc(&h->large_seg_off, seg_off.size() * sizeof(int64_t)));
    SNAP_HIP(hipMalloc(&h->seg_partial, (size_t)(h->n_seg_total + 1) * sizeof(double)));
    SNAP_HIP(hipMemcpyAsync(h->large_list, large.data(), large.size() * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
    SNAP_HIP(hipMemcpyAsync(h->large_seg_off, seg_off.data(), seg_off.size() * sizeof(int64_t), hipMemcpyHostToDevice,
                            h->compute));

    // ---- one pass over the data: validation, norms, classes, access counts --------------------------
    // default: on for the asynchronous epoch; off for group sweeps, which are exact (no asynchrony to guard)
    const bool use_tiles = h->opt.dense_tiles != 2 && h->opt.n_groups == 0 && dense_tiles_applicable(h);
    if (h->opt.dense_tiles == 1 && !use_tiles) {
        set_error("tile sweeps need dense column-major data, ridge loss, resident data and no groups");
        return SNAP_EUNSUPPORTED;
    }
    h->adaptive = h->opt.adaptive == 1 || (h->opt.adaptive == 0 && h->opt.n_groups == 0 && !use_tiles);
    h->damping = h->opt.damping > 0.0f ? h->opt.damping : 1.0f;
    h->inflight_floor = WAVE;
    const bool auto_cap = h->opt.max_inflight_nnz <= 0 && !h->dense && !h->adaptive;
    CreatePass cp{nullptr, h->form == SNAP_PRIMAL ? h->n : h->d, nullptr, hptr.data()};
    // streamed data: the search for groups is carried along by this pass, so that the data cross the host link once
    const bool search_streamed = h->streaming && h->opt.n_groups == 0 && h->opt.auto_groups != 2 && h->form == SNAP_PRIMAL &&
                                 m >= 2 && h->n >= 1 && h->nnz >= 1;
    if (auto_cap && h->vlen > 0) {
        SNAP_HIP(hipMalloc(&cp.freq, (size_t)h->vlen * sizeof(uint32_t)));
        const int rc = fill_zero(cp.freq, (size_t)h->vlen * sizeof(uint32_t), h->compute);
        if (rc != SNAP_OK) {
            (void)hipFree(cp.freq);
            return rc;
        }
    }
    if (h->loss != SNAP_RIDGE && h->n > 0)
        hipLaunchKernelGGL(k_check_labels, dim3(1024), dim3(256), 0, h->compute, h->y, h->n, h->status);
    int rc = search_streamed ? group_search_begin(h, &cp.search) : SNAP_OK;
    if (rc == SNAP_OK) rc = for_each_chunk(h, create_chunk, &cp, /*fold=*/false, /*profile=*/false);
    std::vector<int64_t> gbounds;
    if (rc == SNAP_OK && cp.search) rc = group_search_end(h, cp.search, hptr.data(), gbounds);
    uint32_t st = 0;
    if (rc == SNAP_OK) {
        hipError_t e = hipMemcpyAsync(&st, h->status, 4, hipMemcpyDeviceToHost, h->compute);
        if (e == hipSuccess) e = hipStreamSynchronize(h->compute);
        if (e != hipSuccess) rc = hip_fail(e, "creation pass", __FILE__, __LINE__);
    }
    double eff = (double)h->vlen;
    if (rc == SNAP_OK && cp.freq && !(st & 1u)) rc = access_moments(h, cp.freq, &eff);
    (void)hipStreamSynchronize(h->compute);
    (void)hipFree(cp.freq);
    group_search_free(cp.search);
    SNAP_TRY(rc);
    SNAP_TRY(fill_zero(h->status, 4, h->compute));
    if (st & 1u) {
        set_error("an index in idx is outside [0, %lld)", (long long)cp.minor);
        return SNAP_EINVAL;
    }
    if (st & 2u) {
        set_error("labels must be +1 or -1 for this loss");
        return SNAP_EINVAL;
    }
    if (h->streaming && !h->stream_unit && !(st & 4u) && h->nnz > 0) {
        // every stored value is 1.0: the value array never has to cross the host link again.  Both
        // value buffers are filled with ones once (after the prefetch that may still be writing one).
        SNAP_HIP(hipStreamSynchronize(h->copy));
        for (int b = 0; b < 2; ++b) SNAP_TRY(fill_value(h->buf_val[b], 1.0f, h->max_chunk_nnz, h->compute));
        h->stream_unit = true;
    }
    if (!h->streaming && h->kind == K_PRIMAL_LOGISTIC && !h->dense) SNAP_TRY(fold_labels(h, h->idx, h->nnz, h->compute));
    SNAP_HIP(hipStreamSynchronize(h->compute));   // host vectors above go out of scope

    // ---- groups of coordinates with disjoint supports: given by the caller, or looked for ------------
    if (h->opt.n_groups > 0) gbounds.assign(h->opt.group_bounds, h->opt.group_bounds + h->opt.n_groups + 1);
    else if (h->streaming) {
        if (!h->stream_unit) gbounds.clear();          // (streamed group sweeps take pattern-only data)
    } else if (h->opt.auto_groups != 2) SNAP_TRY(detect_groups(h, hptr.data(), gbounds));
    if (h->opt.auto_groups == 1 && gbounds.empty()) {
        set_error("no partition of the coordinates into few ranges with disjoint supports was found");
        return SNAP_EUNSUPPORTED;
    }
    if (!gbounds.empty() && h->opt.adaptive == 0) h->adaptive = false;   // group sweeps are exact: nothing to guard

    // ---- concurrency control ---------------------------------------------------------------------
    if (h->opt.max_inflight_nnz > 0) h->inflight_nnz = h->opt.max_inflight_nnz;
    else if (h->dense) h->inflight_nnz = 0;       // no cap; the adaptive check lowers it if needed
    else {
        // a quarter of the length of v; without the accept check to fall back on, a quarter of its
        // effective length (much smaller when a few entries of v take most of the accesses)
        const double len = h->adaptive ? (double)h->vlen : eff;
        h->inflight_nnz = std::max<int64_t>(WAVE, (int64_t)(0.25 * len));
    }
    if (h->adaptive) {
        SNAP_HIP(hipMalloc(&h->x_snap, (size_t)(m ? m : 1) * sizeof(float)));
        SNAP_HIP(hipMalloc(&h->v_snap, (size_t)(h->vlen ? h->vlen : 1) * sizeof(float)));
    }
    if (!gbounds.empty()) {
        SNAP_TRY(grouped_setup(h, hptr.data(), gbounds.data(), (int64_t)gbounds.size() - 1));
        if (!h->grouped) {
            // declined (the fixed-point sums would be too coarse for this lambda): the asynchronous engine runs
            if (h->opt.auto_groups == 1) {
                set_error("group sweeps were required (auto_groups = 1) but lambda * n_rows is too small for their "
                          "fixed-point sums");
                return SNAP_EUNSUPPORTED;
            }
            h->adaptive = h->opt.adaptive != 2;
            if (h->adaptive) {
                SNAP_TRY(alloc_snapshots(h));
                if (h->opt.max_inflight_nnz <= 0) h->inflight_nnz = std::max<int64_t>(WAVE, (int64_t)(0.25 * (double)h->vlen));
            }
        }
    }
    if (h->grouped && h->kind == K_PRIMAL_RIDGE) SNAP_TRY(alloc_snapshots(h));     // (see snap_epoch: the range guard)
    if (use_tiles) SNAP_TRY(dense_tiles_setup(h));
    if (h->form == SNAP_DUAL && h->loss == SNAP_LOGISTIC && m > 0) {
        // the entropy term of the logistic dual needs alpha inside (0,1): start at 1/2, v = A alpha
        SNAP_TRY(fill_value(h->x, 0.5f, m, h->compute));
        SNAP_TRY(recompute_shared(h));
    }
    return SNAP_OK;
}

// One chunk of an epoch: its permutation, then the SCD kernels.
static int epoch_chunk(snap_handle* h, int64_t chunk, const ChunkView& cv, void* arg) {
    const uint64_t seed = *(const uint64_t*)arg;
    const snap_handle::Chunk& ck = h->chunks[chunk];
    const int64_t mc = ck.c1 - ck.c0;
    if (mc == 0) return SNAP_OK;
    const bool prof = h->opt.profile != 0 && !h->streaming;
    SNAP_TRY(make_permutation(h, seed, (uint32_t)chunk, ck.c0, mc, h->keys + ck.c0, h->perm + ck.c0, h->order));
    if (prof) SNAP_HIP(hipEventRecord(h->ev[1], h->compute));
    return scd_run_chunk(h, cv, ck, h->order);
}

}  // namespace snap

using namespace snap;


extern "C" {

const char* snap_last_error(void) { return g_error; }

int snap_create(const snap_matrix* A, const float* y, int loss, double lambda, const snap_options* opt,
                snap_handle** out) {
    if (out) *out = nullptr;
    if (!A || !y || !out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    if (A->n_rows < 0 || A->n_cols < 0 || A->nnz < 0 || !(lambda > 0.0) || A->n_rows > 0x7FFFFFFFll ||
        A->n_cols > 0x7FFFFFFFll) {
        set_error("sizes must be non-negative and below 2^31 per dimension, lambda positive");
        return SNAP_EINVAL;
    }
    if (A->layout < SNAP_CSR || A->layout > SNAP_DENSE_COLMAJOR || A->mem < SNAP_MEM_HOST || A->mem > SNAP_MEM_DEVICE ||
        loss < SNAP_RIDGE || loss > SNAP_HINGE) {
        set_error("unknown layout, memory space or loss");
        return SNAP_EINVAL;
    }
    const bool dense = A->layout == SNAP_DENSE_ROWMAJOR || A->layout == SNAP_DENSE_COLMAJOR;
    if ((dense && !A->val) || (!dense && (!A->ptr || !A->idx))) {      // (val = NULL: pattern-only data)
        set_error("matrix arrays missing");
        return SNAP_EINVAL;
    }
    snap_options o{};
    if (opt) o = *opt;
    if (o.n_groups < 0 || (o.n_groups > 0 && !o.group_bounds)) {
        set_error("n_groups must be non-negative and come with group_bounds");
        return SNAP_EINVAL;
    }
    if (o.auto_groups < 0 || o.auto_groups > 2) {
        set_error("auto_groups must be 0, 1 or 2");
        return SNAP_EINVAL;
    }
    if (o.dense_tiles < 0 || o.dense_tiles > 2) {
        set_error("dense_tiles must be 0, 1 or 2");
        return SNAP_EINVAL;
    }
    if (!(o.lambda1 >= 0.0)) {
        set_error("lambda1 must be non-negative");
        return SNAP_EINVAL;
    }
    int form = o.form;
    const bool row_coords = A->layout == SNAP_CSR || A->layout == SNAP_DENSE_ROWMAJOR;
    if (form == SNAP_FORM_AUTO) form = row_coords ? SNAP_DUAL : SNAP_PRIMAL;
    if (form != SNAP_PRIMAL && form != SNAP_DUAL) {
        set_error("unknown form");
        return SNAP_EINVAL;
    }
    if ((form == SNAP_PRIMAL) == row_coords) {
        set_error("the primal form needs column access (CSC / dense column-major), the dual form row access");
        return SNAP_EUNSUPPORTED;
    }
    if ((form == SNAP_PRIMAL && loss == SNAP_HINGE) || (form == SNAP_DUAL && loss == SNAP_RIDGE)) {
        set_error("supported pairs: (ridge, primal), (logistic, primal), (logistic, dual), (hinge, dual)");
        return SNAP_EUNSUPPORTED;
    }
    if (form == SNAP_DUAL && o.lambda1 > 0.0) {
        set_error("the l1 term belongs to the primal forms");
        return SNAP_EUNSUPPORTED;
    }
    snap_handle* h = new (std::nothrow) snap_handle();
    if (!h) {
        set_error("out of host memory");
        return SNAP_ENOMEM;
    }
    h->layout = A->layout;
    h->loss = loss;
    h->form = form;
    h->kind = form == SNAP_DUAL ? K_DUAL : (loss == SNAP_RIDGE ? K_PRIMAL_RIDGE : K_PRIMAL_LOGISTIC);
    h->dense = dense;
    h->n = A->n_rows;
    h->d = A->n_cols;
    h->nnz = dense ? A->n_rows * A->n_cols : A->nnz;
    h->m = form == SNAP_PRIMAL ? h->d : h->n;
    h->vlen = form == SNAP_PRIMAL ? h->n : h->d;
    h->ld = dense ? h->vlen : 0;
    h->lambda = lambda;
    h->lambda1 = o.lambda1;
    h->opt = o;
    const int rc = build(h, A, y);
    if (rc != SNAP_OK) {
        destroy(h);
        return rc;
    }
    *out = h;
    return SNAP_OK;
}

void snap_destroy(snap_handle* h) { destroy(h); }

int snap_epoch(snap_handle* h, uint64_t perm_seed) {
    if (!h) {
        set_error("null handle");
        return SNAP_EINVAL;
    }
    if (h->m == 0) return SNAP_OK;
    const bool prof = h->opt.profile != 0;
    // group sweeps of the ridge loss can run out of the range of their fixed-point sums: the state before
    // the epoch is kept so that the epoch can be done again by the asynchronous engine
    const bool guard_range = h->grouped && h->kind == K_PRIMAL_RIDGE;
    // Group sweeps keep the state before the epoch for free (their first writing pass writes the shared
    // vector into the second array, and the two change roles at the end; only the model is copied) and sum
    // the loss in their last pass: the accept check then costs one small reduction (Section 3.1: the cost
    // of evaluating the objective is absorbed by the epoch's kernels).
    const bool keep_by_swap = h->grouped && (h->adaptive || guard_range);
    if (h->adaptive) {
        // value and state before the epoch, for the accept / discard decision
        if (!h->monitor_valid) {
            SNAP_TRY(monitor_value(h, &h->monitor_prev));
            h->monitor_valid = true;
        }
    }
    if (keep_by_swap) SNAP_TRY(copy_pair(h->x_snap, h->x, h->m, nullptr, nullptr, 0, h->compute));
    else if (h->adaptive) SNAP_TRY(copy_pair(h->x_snap, h->x, h->m, h->v_snap, h->v, h->vlen, h->compute));
    h->g_keep_old = keep_by_swap;
    h->g_want_loss = keep_by_swap && h->adaptive;
    h->g_swapped = false;
    auto restore = [&]() -> int {                    // back to the state before the epoch
        if (keep_by_swap) {
            if (h->g_swapped) std::swap(h->v, h->v_snap);
            h->g_swapped = false;
            return copy_pair(h->x, h->x_snap, h->m, nullptr, nullptr, 0, h->compute);
        }
        return copy_pair(h->x, h->x_snap, h->m, h->v, h->v_snap, h->vlen, h->compute);
    };
    if (prof) SNAP_HIP(hipEventRecord(h->ev[0], h->compute));
    if (h->grouped) {
        // exact group sweeps; the visiting order inside a group does not change the result and is
        // only generated when snap_get_perm asks for it
        if (prof) SNAP_HIP(hipEventRecord(h->ev[1], h->compute));
        h->last_seed = perm_seed;
        SNAP_TRY(grouped_epoch(h));
        if (prof) SNAP_HIP(hipEventRecord(h->ev[3], h->compute));
        h->perm_stale = true;
        if (guard_range) {
            uint32_t st = 0;
            SNAP_TRY(read_status(h, &st));
            if (st & STATUS_RANGE) {
                SNAP_TRY(restore());
                SNAP_TRY(leave_group_sweeps(h));
                h->pass_list = nullptr;                  // (a pass over part of the groups becomes a whole epoch)
                h->pass_count = 0;
                return snap_epoch(h, perm_seed);         // the same epoch, by the engine without the limit
            }
        }
    } else if (h->tiled) {
        if (h->pass_list) {
            set_error("a pass over part of the tiles is not supported by the dense tile sweeps");
            return SNAP_EUNSUPPORTED;
        }
        if (prof) SNAP_HIP(hipEventRecord(h->ev[1], h->compute));
        h->last_seed = perm_seed;
        SNAP_TRY(dense_tiles_epoch(h));
        if (prof) SNAP_HIP(hipEventRecord(h->ev[3], h->compute));
        h->perm_stale = true;
    } else {
        SNAP_TRY(for_each_chunk(h, epoch_chunk, &perm_seed, /*fold=*/true, /*profile=*/prof));
    }
    if (prof) {
        SNAP_HIP(hipEventRecord(h->ev[2], h->compute));
        h->stats_pending = true;
    }
    h->stats.inflight_nnz = h->inflight_nnz;
    h->stats.damping = h->damping;
    h->stats.rejected = 0;
    ++h->epochs_done;
    if (h->opt.refresh_v_every > 0 && h->epochs_done % h->opt.refresh_v_every == 0) SNAP_TRY(recompute_shared(h));
    if (h->adaptive) {
        double now = 0.0;
        const bool refreshed = h->opt.refresh_v_every > 0 && h->epochs_done % h->opt.refresh_v_every == 0;
        if (keep_by_swap && h->g_want_loss && !refreshed)  // (g_want_loss: now "the last pass has left its loss sums")
            SNAP_TRY(grouped_loss_value(h, &now));
        else
            SNAP_TRY(monitor_value(h, &now));
        const double slack = 1e-6 * std::max(std::fabs(h->monitor_prev), 1e-30);
        if (!(now <= h->monitor_prev + slack)) {          // worse (or not a number): discard the epoch
            SNAP_TRY(restore());
            h->stats.rejected = 1;
            // first fewer nonzeros in flight (down to one wavefront's worth), then smaller steps; group
            // sweeps have nothing in flight: smaller steps at once
            const int64_t cur = h->inflight_nnz > 0 ? h->inflight_nnz : (int64_t)256 * 8 * h->seg;
            if (cur > h->inflight_floor && !keep_by_swap)
                h->inflight_nnz = std::max<int64_t>(h->inflight_floor, cur / 2);
            else
                h->damping *= 0.5f;
        } else {
            h->monitor_prev = now;
        }
    }
    return SNAP_OK;
}

static int64_t chunk_count(const snap_handle* h) { return (h->grouped || h->tiled) ? h->n_groups : h->n_chunks; }

int snap_epoch_chunks(snap_handle* h, uint64_t perm_seed, const int64_t* chunks, int64_t count) {
    if (!h || count < 0 || (count > 0 && !chunks)) {
        set_error("snap_epoch_chunks: need a handle and a list of chunks");
        return SNAP_EINVAL;
    }
    const int64_t C = chunk_count(h);
    std::vector<char> seen((size_t)C, 0);
    for (int64_t i = 0; i < count; ++i) {
        if (chunks[i] < 0 || chunks[i] >= C || seen[(size_t)chunks[i]]) {
            set_error("snap_epoch_chunks: chunk numbers must lie in [0, n_chunks) and be distinct");
            return SNAP_EINVAL;
        }
        seen[(size_t)chunks[i]] = 1;
    }
    if (count == 0) return SNAP_OK;
    h->pass_list = chunks;
    h->pass_count = count;
    const int rc = snap_epoch(h, perm_seed);
    h->pass_list = nullptr;
    h->pass_count = 0;
    return rc;
}

int snap_chunk_gaps(snap_handle* h, double* shares_out, double* gap_out) {
    if (!h || !shares_out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    const int64_t C = chunk_count(h);
    SNAP_TRY(chunk_gap_shares(h, shares_out));
    if (gap_out) {
        double g = 0.0;
        for (int64_t c = 0; c < C; ++c) g += shares_out[c];
        *gap_out = g;
    }
    return SNAP_OK;
}

int snap_solve_selected(snap_handle* h, uint64_t seed0, int64_t max_passes, double gap_tol, int64_t refresh_every,
                        int64_t keep, int64_t* passes_out, int64_t* visits_out, double* gap_out) {
    if (!h || max_passes < 0 || refresh_every < 1 || keep < 0 || !(gap_tol >= 0.0)) {
        set_error("snap_solve_selected: need a handle, max_passes >= 0, refresh_every >= 1, keep >= 0, gap_tol >= 0");
        return SNAP_EINVAL;
    }
    const int64_t C = chunk_count(h);
    std::vector<double> shares((size_t)C, 0.0);
    std::vector<int64_t> chosen((size_t)C);
    for (int64_t c = 0; c < C; ++c) chosen[(size_t)c] = c;
    int64_t p = 0, visits = 0;
    double gap = INFINITY;
    while (p < max_passes) {
        const bool full = p % refresh_every == 0;
        if (full) {
            SNAP_TRY(snap_epoch(h, seed0 + (uint64_t)p));
            visits += C;
        } else {
            SNAP_TRY(snap_epoch_chunks(h, seed0 + (uint64_t)p, chosen.data(), (int64_t)chosen.size()));
            visits += (int64_t)chosen.size();
        }
        ++p;
        if (full) {
            SNAP_TRY(snap_chunk_gaps(h, shares.data(), &gap));
            if (gap <= gap_tol) break;
            // the `keep` chunks with the largest shares, largest first; equal shares in index order
            chosen.resize((size_t)C);
            for (int64_t c = 0; c < C; ++c) chosen[(size_t)c] = c;
            std::stable_sort(chosen.begin(), chosen.end(),
                             [&](int64_t a, int64_t b) { return shares[(size_t)a] > shares[(size_t)b]; });
            chosen.resize((size_t)std::min<int64_t>(keep, C));
        }
    }
    if (passes_out) *passes_out = p;
    if (visits_out) *visits_out = visits;
    if (gap_out) *gap_out = gap;
    return SNAP_OK;
}

int snap_get_bytes_copied(snap_handle* h, int64_t* total) {
    if (!h || !total) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    *total = h->bytes_copied;
    return SNAP_OK;
}

int snap_objective(snap_handle* h, double* primal, double* dual) {
    if (!h || !primal) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    SNAP_TRY(check_status(h));
    return objective(h, primal, dual, nullptr);
}

int snap_duality_gap(snap_handle* h, double* gap) {
    if (!h || !gap) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    SNAP_TRY(check_status(h));
    return objective(h, nullptr, nullptr, gap);
}

int snap_predict(snap_handle* h, const snap_matrix* X, float* out) {
    if (!h || !X || !out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    if (X->layout < SNAP_CSR || X->layout > SNAP_DENSE_COLMAJOR || X->mem < SNAP_MEM_HOST || X->mem > SNAP_MEM_DEVICE) {
        set_error("unknown layout or memory space");
        return SNAP_EINVAL;
    }
    const bool dense = X->layout >= SNAP_DENSE_ROWMAJOR;
    if (X->n_cols != h->d || X->n_rows < 0 || X->nnz < 0 || !X->val || (!dense && (!X->ptr || !X->idx))) {
        set_error("predict: the matrix must have the training number of columns and valid arrays");
        return SNAP_EINVAL;
    }
    SNAP_TRY(check_status(h));
    return predict(h, X, out);
}

int snap_predict_static(snap_handle* h, const snap_matrix* X, float* out) {
    if (!h || !X || !out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    if (X->layout < SNAP_CSR || X->layout > SNAP_DENSE_COLMAJOR || X->mem < SNAP_MEM_HOST || X->mem > SNAP_MEM_DEVICE) {
        set_error("unknown layout or memory space");
        return SNAP_EINVAL;
    }
    const bool dense = X->layout >= SNAP_DENSE_ROWMAJOR;
    if (X->n_cols != h->d || X->n_rows < 0 || X->nnz < 0 || !X->val || (!dense && (!X->ptr || !X->idx))) {
        set_error("predict: the matrix must have the training number of columns and valid arrays");
        return SNAP_EINVAL;
    }
    SNAP_TRY(check_status(h));
    return predict_static(h, X, out);
}

int snap_get_model(snap_handle* h, float* w_out, float* coord_out) {
    if (!h) {
        set_error("null handle");
        return SNAP_EINVAL;
    }
    SNAP_TRY(check_status(h));
    if (w_out) SNAP_TRY(weights_to_host(h, w_out));
    if (coord_out) {
        SNAP_HIP(hipMemcpyAsync(coord_out, h->x, (size_t)h->m * sizeof(float), hipMemcpyDeviceToHost, h->compute));
        SNAP_HIP(hipStreamSynchronize(h->compute));
    }
    return SNAP_OK;
}

int snap_set_model(snap_handle* h, const float* coord_in) {
    if (!h || !coord_in) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    SNAP_HIP(hipMemcpyAsync(h->x, coord_in, (size_t)h->m * sizeof(float), hipMemcpyHostToDevice, h->compute));
    if (h->form == SNAP_DUAL && h->loss == SNAP_LOGISTIC)       // the entropy term lives on (0,1)
        SNAP_TRY(clamp_range(h->x, (float)ALPHA_EPS, (float)(1.0 - ALPHA_EPS), h->m, h->compute));
    SNAP_TRY(recompute_shared(h));
    SNAP_HIP(hipStreamSynchronize(h->compute));
    h->monitor_valid = false;
    return SNAP_OK;
}

int snap_get_shared(snap_handle* h, float* v_out) {
    if (!h || !v_out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    SNAP_TRY(check_status(h));
    SNAP_HIP(hipMemcpyAsync(v_out, h->v, (size_t)h->vlen * sizeof(float), hipMemcpyDeviceToHost, h->compute));
    SNAP_HIP(hipStreamSynchronize(h->compute));
    return SNAP_OK;
}

int snap_recompute_shared(snap_handle* h) {
    if (!h) {
        set_error("null handle");
        return SNAP_EINVAL;
    }
    return recompute_shared(h);
}

int snap_get_perm(snap_handle* h, uint32_t* perm_out, uint32_t* keys_out) {
    if (!h || !perm_out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    const bool blocks = h->grouped || h->tiled;      // coordinates visited block by block (groups / tiles)
    if (blocks && h->perm_stale) {
        for (int64_t g = 0; g < h->n_groups; ++g) {
            const int64_t c0 = h->gbounds_host[g], sz = h->gbounds_host[g + 1] - c0;
            SNAP_TRY(make_permutation(h, h->last_seed, (uint32_t)g, c0, sz, h->keys + c0, h->perm + c0, nullptr));
        }
        h->perm_stale = false;
    }
    SNAP_HIP(hipMemcpyAsync(perm_out, h->perm, (size_t)h->m * sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
    if (keys_out)
        SNAP_HIP(hipMemcpyAsync(keys_out, h->keys, (size_t)h->m * sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
    SNAP_HIP(hipStreamSynchronize(h->compute));
    if (blocks) {
        // stored group by group; reported in visiting order: groups in the epoch's order, the
        // permutation of each group inside
        std::vector<uint32_t> tmp(perm_out, perm_out + h->m);
        int64_t pos = 0;
        for (int64_t g : group_order(h->last_seed, h->n_groups)) {
            const int64_t c0 = h->gbounds_host[g], c1 = h->gbounds_host[g + 1];
            for (int64_t c = c0; c < c1; ++c) perm_out[pos++] = tmp[(size_t)c] + (uint32_t)c0;
        }
        return SNAP_OK;
    }
    // The asynchronous epoch runs the split coordinates of a chunk first and the others after them,
    // each class in the order of the keys: that is the order reported.
    std::vector<uint8_t> cls((size_t)h->m);
    if (h->n_large_total > 0) {
        SNAP_HIP(hipMemcpyAsync(cls.data(), h->cls, (size_t)h->m, hipMemcpyDeviceToHost, h->compute));
        SNAP_HIP(hipStreamSynchronize(h->compute));
    }
    std::vector<uint32_t> rest;
    for (int64_t ch = 0; ch < h->n_chunks; ++ch) {
        const int64_t c0 = h->chunks[ch].c0, c1 = h->chunks[ch].c1;
        for (int64_t k = c0; k < c1; ++k) perm_out[k] += (uint32_t)c0;
        if (h->chunks[ch].n_large == 0) continue;
        rest.clear();
        int64_t pos = c0;
        for (int64_t k = c0; k < c1; ++k) {
            const uint32_t c = perm_out[k];
            if (cls[c]) perm_out[pos++] = c;
            else rest.push_back(c);
        }
        std::copy(rest.begin(), rest.end(), perm_out + pos);
    }
    return SNAP_OK;
}

int snap_get_epoch_stats(snap_handle* h, snap_epoch_stats* out) {
    if (!h || !out) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    if (h->stats_pending && h->gstream) {
        // group sweeps over streamed row maps: copies per visit on the copy stream, kernels per visit
        // (row pass + step kernel, measured from the moment the visit's map is there) on the compute stream
        SNAP_HIP(hipEventSynchronize(h->ev[2]));
        SNAP_HIP(hipStreamSynchronize(h->copy));
        float total = 0, copy = 0, scd = 0;
        SNAP_HIP(hipEventElapsedTime(&total, h->ev[0], h->ev[2]));
        if (h->gev_prof && h->gprof_valid && !h->gcopy_timed.empty())
            for (int64_t i = 0; i <= h->g_visits; ++i) {
                float a = 0, b = 0;
                if (i < h->g_visits && h->gcopy_timed[(size_t)i])
                    SNAP_HIP(hipEventElapsedTime(&a, h->gev_prof[4 * i + 0], h->gev_prof[4 * i + 1]));
                SNAP_HIP(hipEventElapsedTime(&b, h->gev_prof[4 * i + 2], h->gev_prof[4 * i + 3]));
                copy += a;
                scd += b;
            }
        h->stats.epoch_ms = total;
        h->stats.copy_ms = copy;
        h->stats.scd_ms = scd;
        h->stats.large_ms = h->stats.small_ms = h->stats.perm_ms = 0;
        h->stats_pending = false;
    }
    if (h->stats_pending && h->streaming) {
        SNAP_HIP(hipEventSynchronize(h->ev[2]));
        SNAP_HIP(hipStreamSynchronize(h->copy));
        float total = 0, copy = 0, scd = 0;
        SNAP_HIP(hipEventElapsedTime(&total, h->ev[0], h->ev[2]));
        if (h->chunk_events_valid)
            for (int64_t ch = 0; ch < h->n_chunks; ++ch) {
                float a = 0, b = 0;
                if (h->chunk_copy_timed[(size_t)ch])     // (a chunk that stayed in its buffer was not copied)
                    SNAP_HIP(hipEventElapsedTime(&a, h->ev_chunk[4 * ch + 0], h->ev_chunk[4 * ch + 1]));
                SNAP_HIP(hipEventElapsedTime(&b, h->ev_chunk[4 * ch + 2], h->ev_chunk[4 * ch + 3]));
                copy += a;
                scd += b;
            }
        h->stats.epoch_ms = total;
        h->stats.copy_ms = copy;
        h->stats.scd_ms = scd;
        h->stats.perm_ms = h->stats.large_ms = h->stats.small_ms = 0;
        h->stats_pending = false;
    }
    if (h->stats_pending && (h->grouped || h->tiled)) {
        SNAP_HIP(hipEventSynchronize(h->ev[2]));
        float total = 0, rows = 0;
        SNAP_HIP(hipEventElapsedTime(&total, h->ev[0], h->ev[2]));
        if (h->ev_group) {
            int timed = 0;
            for (int i = 0; i < h->n_row_passes; ++i) {
                if (!h->pass_timed[(size_t)i]) continue;
                float t = 0;
                SNAP_HIP(hipEventElapsedTime(&t, h->ev_group[2 * i], h->ev_group[2 * i + 1]));
                rows += t;
                ++timed;
            }
            // (profile = 2: the passes that were timed stand for the others)
            rows = timed > 0 ? rows * (float)h->n_row_passes / (float)timed : 0.0f;
        }
        h->stats.epoch_ms = h->stats.scd_ms = total;
        h->stats.large_ms = rows;              // the row passes
        h->stats.small_ms = total - rows;      // column-wise sums of the short coordinates + step kernels
        h->stats.perm_ms = h->stats.copy_ms = 0;
        h->stats_pending = false;
    }
    if (h->stats_pending) {
        SNAP_HIP(hipEventSynchronize(h->ev[2]));
        float total = 0, perm = 0, scd = 0, large = 0, small = 0;
        SNAP_HIP(hipEventElapsedTime(&large, h->ev[1], h->ev[3]));
        SNAP_HIP(hipEventElapsedTime(&small, h->ev[3], h->ev[2]));
        h->stats.large_ms = large;
        h->stats.small_ms = small;
        SNAP_HIP(hipEventElapsedTime(&total, h->ev[0], h->ev[2]));
        SNAP_HIP(hipEventElapsedTime(&perm, h->ev[0], h->ev[1]));
        SNAP_HIP(hipEventElapsedTime(&scd, h->ev[1], h->ev[2]));
        h->stats.epoch_ms = total;
        h->stats.perm_ms = perm;
        h->stats.scd_ms = scd;
        h->stats.copy_ms = 0;
        h->stats_pending = false;
    }
    h->stats.nnz_large = h->nnz_large;
    h->stats.nnz_small = h->nnz_small;
    h->stats.n_chunks = h->n_chunks;
    h->stats.n_small = h->stats.n_large = h->stats.n_items = 0;
    for (int64_t ch = 0; ch < h->n_chunks; ++ch) {
        h->stats.n_small += h->chunks[ch].n_small;
        h->stats.n_large += h->chunks[ch].n_large;
        h->stats.n_items += h->chunks[ch].n_items;
    }
    if (h->grouped || h->tiled) {   // group sweeps: "large" = hot ranks (row passes), "small" = the rest, items = row passes
        h->stats.n_chunks = h->n_groups;
        h->stats.n_large = h->g_hot_coords;
        h->stats.n_small = h->m - h->g_hot_coords;
        h->stats.nnz_large = h->g_hot_nnz;
        h->stats.nnz_small = h->nnz - h->g_hot_nnz;
        h->stats.n_items = h->n_row_passes;
    }
    h->stats.row_map_bytes = h->grouped ? (h->map16 ? 2 : 4) : 0;
    h->stats.byte_map_groups = h->grouped ? h->n_byte_maps : 0;
    h->stats.unit_values = (h->grouped ? h->unit_values : h->stream_unit) ? 1 : 0;
    *out = h->stats;
    return SNAP_OK;
}

int snap_get_chunks(snap_handle* h, int64_t* n_chunks, int64_t* bounds_out) {
    if (!h || !n_chunks) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    if (h->grouped || h->tiled) {
        *n_chunks = h->n_groups;
        if (bounds_out) std::copy(h->gbounds_host, h->gbounds_host + h->n_groups + 1, bounds_out);
        return SNAP_OK;
    }
    *n_chunks = h->n_chunks;
    if (bounds_out) {
        for (int64_t ch = 0; ch < h->n_chunks; ++ch) bounds_out[ch] = h->chunks[ch].c0;
        bounds_out[h->n_chunks] = h->m;
    }
    return SNAP_OK;
}

int snap_solve(snap_handle* h, uint64_t seed0, int64_t max_epochs, double gap_tol, int64_t check_every,
               int64_t* epochs_out, double* gap_out) {
    if (!h || max_epochs < 0 || check_every < 1 || !(gap_tol >= 0.0)) {
        set_error("snap_solve: need a handle, max_epochs >= 0, check_every >= 1, gap_tol >= 0");
        return SNAP_EINVAL;
    }
    int64_t e = 0;
    double gap = 0.0;
    bool fresh = false;
    for (; e < max_epochs; ++e) {
        SNAP_TRY(snap_epoch(h, seed0 + (uint64_t)e));
        fresh = false;
        if ((e + 1) % check_every == 0) {
            SNAP_TRY(snap_duality_gap(h, &gap));
            fresh = true;
            if (gap <= gap_tol) {
                ++e;
                break;
            }
        }
    }
    if (!fresh) SNAP_TRY(snap_duality_gap(h, &gap));
    if (epochs_out) *epochs_out = e;
    if (gap_out) *gap_out = gap;
    return SNAP_OK;
}

uint32_t snap_perm_key(uint64_t perm_seed, uint32_t chunk, uint32_t c) {
    return perm_key(perm_key_base(perm_seed, chunk), c);
}

int snap_block_order(uint64_t perm_seed, int64_t n_blocks, int64_t* order_out) {
    if (n_blocks < 0 || n_blocks > 0xFFFFFFFFll || (n_blocks > 0 && !order_out)) {
        set_error("snap_block_order: need 0 <= n_blocks < 2^32 and an output array");
        return SNAP_EINVAL;
    }
    const std::vector<int64_t> order = group_order(perm_seed, n_blocks);
    std::copy(order.begin(), order.end(), order_out);
    return SNAP_OK;
}

int snap_get_stream_bytes(snap_handle* h, int64_t* bytes_per_pass) {
    if (!h || !bytes_per_pass) {
        set_error("null argument");
        return SNAP_EINVAL;
    }
    if (h->gstream) *bytes_per_pass = h->gmap_bytes_per_pass;       // the row maps of the non-empty groups
    else *bytes_per_pass = h->streaming ? h->nnz * (int64_t)(h->stream_unit ? sizeof(uint32_t) : sizeof(uint32_t) + sizeof(float)) : 0;
    return SNAP_OK;
}

int snap_get_dims(snap_handle* h, int64_t* n_coords, int64_t* shared_len) {
    if (!h) {
        set_error("null handle");
        return SNAP_EINVAL;
    }
    if (n_coords) *n_coords = h->m;
    if (shared_len) *shared_len = h->vlen;
    return SNAP_OK;
}

}  // extern "C"
