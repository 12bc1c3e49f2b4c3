// The SCD epoch kernels (Section 3.1): per coordinate a gather-dot of its nonzeros with the shared
// vector v, a scalar step (closed form for ridge and for the clipped hinge dual, one Newton step
// for logistic regression), and an atomic scatter of delta * a_j into v.  Many coordinates are in
// flight at once and see each other's partial updates, as in the paper's asynchronous solver.
//
// The paper's solver gives every coordinate one thread block.  On a 256-CU part with click-log
// data (a few columns holding a fifth of all rows each, a million columns of a few hundred) that
// leaves the epoch waiting for a handful of blocks, so coordinates are handled in two classes:
//   small  (<= small_max = 4096 nonzeros): one 64-wide wavefront per coordinate, four per workgroup;
//   large  (longer): split into segments of seg = 16384 nonzeros.  Every segment is two
//          work items, "dot" and "scatter".  Workgroups draw items from one atomic ticket counter
//          in epoch order; the dot items of a coordinate add their partial sums into its state and
//          the last one to arrive takes the step and publishes delta; a scatter item waits for
//          that flag.  A waiting workgroup only ever waits for workgroups that drew an earlier
//          ticket and are therefore already running, so the wait always ends; it is bounded by
//          SPIN_LIMIT all the same and raises the handle's status word instead of hanging.
#include "scd_device.h"
#include <algorithm>

namespace snap {

// ---- small coordinates: one wavefront each ----------------------------------------------------
// A wavefront walks its share of the epoch order, and what a coordinate needs is a chain of dependent
// loads: its place in the order, its two ptr entries, its indices and values, the entries of v they
// name, its own x / norm / label.  With few coordinates in flight (the cap that keeps the asynchronous
// solver convergent: some hundred rows for the hinge dual on data with popular features) that chain,
// not bandwidth, sets the pace.  So the chain is taken apart over three visits: while the gather of
// coordinate i is under way, the nonzeros and scalars of i+1, the ptr entries of i+2 and the order
// entry of i+3 are requested too, all independent of each other; only the reads of v, which must be
// as late as possible, stay in the visit they belong to.  (x[c], the norms and the labels are not
// written by other coordinates' updates.)  Up to SMALL_ROUNDS nonzeros per lane travel this way and
// are scattered from registers; longer coordinates take the rest in plain loops.
// SMALL_ROUNDS is 1 when no small coordinate of the data is longer than a wavefront, else 4.
template <int SMALL_ROUNDS>
struct SmallCoord {
    int64_t c, s0, s1;            // coordinate, its range in the chunk's arrays
    uint32_t raw[SMALL_ROUNDS];   // index words of this lane: nonzeros s0 + j * 64 + lane
    float a[SMALL_ROUNDS];
    float xc, nc, yc;
};

template <int KIND, int SMALL_ROUNDS>
__global__ void __launch_bounds__(TPB)
k_scd_small(ChunkView cv, const uint32_t* __restrict__ order, int64_t n_small, const float* __restrict__ y,
            float* __restrict__ x, float* v, const float* __restrict__ norms, StepParams sp, int64_t n_waves) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wave0 = ((int64_t)blockIdx.x * TPB + threadIdx.x) / WAVE;
    if (wave0 >= n_waves) return;
    // n_waves wavefronts walk the epoch order round-robin: at most n_waves coordinates in flight.
    // What a visit requests for later coordinates is only touched in the next visit, arithmetic on
    // it included (the wait for a value sits before its first use: an addition right after the load
    // would put the wait there, and the requests would again be served one after the other).
    auto order_entry = [&](int64_t wid) -> uint32_t { return wid < n_small ? order[wid] : 0u; };
    auto ptr_pair = [&](int64_t c, int64_t& p0, int64_t& p1) {
        p0 = p1 = 0;
        if (c >= 0) {
            p0 = cv.ptr[c];
            p1 = cv.ptr[c + 1];
        }
    };
    auto fetch = [&](int64_t c, int64_t s0, int64_t s1) -> SmallCoord<SMALL_ROUNDS> {
        SmallCoord<SMALL_ROUNDS> q;
        q.c = c, q.s0 = s0, q.s1 = s1;
        q.xc = q.nc = q.yc = 0.0f;
#pragma unroll
        for (int j = 0; j < SMALL_ROUNDS; ++j) {
            const int64_t k = s0 + j * WAVE + lane;
            q.raw[j] = 0u;
            q.a[j] = 0.0f;
            if (k < s1) {
                q.raw[j] = cv.idx[k];
                q.a[j] = cv.val[k];
            }
        }
        if (c >= 0) {   // the same address in every lane: one request
            q.xc = x[c];
            q.nc = norms[c];
            if (KIND == K_DUAL) q.yc = y[c];
        }
        return q;
    };
    // fill the pipeline: three coordinates' order entries, two ptr pairs, one record
    auto coord_at = [&](int64_t wid, uint32_t entry) -> int64_t { return wid < n_small ? cv.c0 + (int64_t)entry : -1; };
    int64_t cB = coord_at(wave0 + n_waves, order_entry(wave0 + n_waves));   // its nonzeros are requested next
    uint32_t entryA = order_entry(wave0 + 2 * n_waves);                     // its ptr pair is read next
    int64_t p0B, p1B;
    SmallCoord<SMALL_ROUNDS> cur;
    {
        const int64_t c = coord_at(wave0, order_entry(wave0));
        int64_t p0, p1;
        ptr_pair(c, p0, p1);
        ptr_pair(cB, p0B, p1B);
        cur = fetch(c, p0 - cv.nnz_base, p1 - cv.nnz_base);
    }
    for (int64_t wid = wave0; wid < n_small; wid += n_waves) {
        // this visit's requests
        const int64_t c = cur.c, s0 = cur.s0, s1 = cur.s1;
        uint32_t r[SMALL_ROUNDS];
        float vv[SMALL_ROUNDS], yy[SMALL_ROUNDS];
        bool have[SMALL_ROUNDS];
#pragma unroll
        for (int j = 0; j < SMALL_ROUNDS; ++j) {
            have[j] = s0 + j * WAVE + lane < s1;
            r[j] = cur.raw[j] & (KIND == K_PRIMAL_LOGISTIC ? ~LABEL_BIT : 0xFFFFFFFFu);
            vv[j] = yy[j] = 0.0f;
            if (have[j]) {
                vv[j] = load_shared(v, r[j]);
                if (KIND == K_PRIMAL_RIDGE) yy[j] = y[r[j]];
                if (KIND == K_PRIMAL_LOGISTIC) yy[j] = (cur.raw[j] & LABEL_BIT) ? -1.0f : 1.0f;
            }
        }
        const SmallCoord<SMALL_ROUNDS> nxt = fetch(cB, p0B - cv.nnz_base, p1B - cv.nnz_base);
        const int64_t cA = coord_at(wid + 2 * n_waves, entryA);
        int64_t p0A, p1A;
        ptr_pair(cA, p0A, p1A);
        const uint32_t entry3 = order_entry(wid + 3 * n_waves);

        float g = 0.0f, h = 0.0f;
        // (these nonzeros stay in registers for the scatter pass)
#pragma unroll
        for (int j = 0; j < SMALL_ROUNDS; ++j)
            if (have[j]) accumulate<KIND>(cur.a[j], vv[j], yy[j], g, h);
        for (int64_t k = s0 + SMALL_ROUNDS * WAVE + lane; k < s1; k += WAVE) {
            uint32_t rr;
            float yk;
            decode<KIND>(cv.idx[k], rr, yk, y);
            accumulate<KIND>(cv.val[k], load_shared(v, rr), yk, g, h);
        }
        g = wave_sum(g);
        if (KIND == K_PRIMAL_LOGISTIC) h = wave_sum(h);
        float mult = 0.0f;
        if (lane == 0) x[c] = take_step<KIND>((double)g, (double)h, cur.xc, cur.nc, cur.yc, sp, mult);
        mult = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mult), 0));   // lane 0's, without an LDS round trip
        if (mult != 0.0f) {
#pragma unroll
            for (int j = 0; j < SMALL_ROUNDS; ++j)
                if (have[j]) unsafeAtomicAdd(v + r[j], mult * cur.a[j]);
            for (int64_t k = s0 + SMALL_ROUNDS * WAVE + lane; k < s1; k += WAVE) {
                const uint32_t rr = cv.idx[k] & (KIND == K_PRIMAL_LOGISTIC ? ~LABEL_BIT : 0xFFFFFFFFu);
                unsafeAtomicAdd(v + rr, mult * cv.val[k]);
            }
        }
        cur = nxt;
        cB = cA;
        p0B = p0A;
        p1B = p1A;
        entryA = entry3;
    }
}

// ---- large coordinates: segments, two phases, ticket order -------------------------------------
// Everything the workgroups of one coordinate exchange (partial sums, arrival count, the published
// step) goes through device-scope atomic operations, which are performed at the level of the
// memory system that all compute dies share.  Ordering between them therefore only needs the
// earlier operations to have completed, which a data dependence on their returned values gives; a
// device-scope fence would also write back and invalidate the L2 of the die on every work item,
// which costs far more than the item itself.
static_assert(sizeof(LargeState) == 32, "one coordinate's state is one 32-byte block (hipMalloc aligns the array)");

// One workgroup: prefix sums of the items of the large coordinates in epoch order, zeroed state,
// ticket counter back to zero.
__global__ void __launch_bounds__(1024)
k_large_prepare(const int64_t* __restrict__ ptr, int64_t c0, const uint32_t* __restrict__ order_large,
                int64_t n_large, int64_t dense_len, int64_t seg_len, int64_t* __restrict__ item_start,
                LargeState* __restrict__ st, uint32_t* __restrict__ ticket) {
    __shared__ int64_t part[1024];
    const int64_t per = (n_large + 1023) / 1024;
    const int64_t lo = min(n_large, (int64_t)threadIdx.x * per), hi = min(n_large, lo + per);
    int64_t s = 0;
    for (int64_t k = lo; k < hi; ++k) {
        const int64_t c = c0 + (int64_t)order_large[k];
        const int64_t len = dense_len > 0 ? dense_len : ptr[c + 1] - ptr[c];
        s += 2 * ((len + seg_len - 1) / seg_len);
        st[k] = LargeState{0.0, 0.0, 0ull, 0u, 0u};
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        int64_t t = threadIdx.x >= off ? part[threadIdx.x - off] : 0;
        __syncthreads();
        part[threadIdx.x] += t;
        __syncthreads();
    }
    int64_t run = part[threadIdx.x] - s;
    for (int64_t k = lo; k < hi; ++k) {
        const int64_t c = c0 + (int64_t)order_large[k];
        const int64_t len = dense_len > 0 ? dense_len : ptr[c + 1] - ptr[c];
        item_start[k] = run;
        run += 2 * ((len + seg_len - 1) / seg_len);
    }
    if (threadIdx.x == 1023) item_start[n_large] = part[1023];
    if (threadIdx.x == 0) *ticket = 0u;
}

#ifndef SNAP_UNROLL
#define SNAP_UNROLL 4
#endif
constexpr int UNROLL = SNAP_UNROLL;

// index / value streams are read once per pass: load them with the non-temporal hint so that they
// do not push the lines of v out of the caches
template <typename T>
__device__ __forceinline__ T stream_load(const T* p) {
#ifdef SNAP_NO_NT
    return *p;
#else
    return __builtin_nontemporal_load(p);
#endif
}

template <int KIND, bool DENSE>
__global__ void __launch_bounds__(TPB)
k_scd_large(ChunkView cv, const uint32_t* __restrict__ order_large, int64_t n_large,
            const int64_t* __restrict__ item_start, int64_t n_items, LargeState* st, uint32_t* ticket,
            uint32_t* status, const float* __restrict__ y, float* __restrict__ x, float* v,
            const float* __restrict__ norms, StepParams sp, int64_t dense_len, int64_t seg_len) {
    __shared__ uint32_t s_ticket;
    __shared__ float s_mult;
    __shared__ float s_part[2 * WAVES_PER_WG];
    // a fixed number of workgroups (the cap on work in flight) keeps drawing tickets
    for (;;) {
        __syncthreads();                                   // s_ticket / s_mult / s_part are reused
        if (threadIdx.x == 0) s_ticket = atomicAdd(ticket, 1u);
        __syncthreads();
        const int64_t t = (int64_t)s_ticket;
        if (t >= n_items) return;
        int64_t lo = 0, hi = n_large;                      // largest k with item_start[k] <= t
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (item_start[mid] <= t) lo = mid; else hi = mid;
        }
        const int64_t k = lo;
        const int64_t c = cv.c0 + (int64_t)order_large[k];
        int64_t b0, len;
        if (DENSE) {
            b0 = c * dense_len;
            len = dense_len;
        } else {
            b0 = cv.ptr[c] - cv.nnz_base;
            len = cv.ptr[c + 1] - cv.ptr[c];
        }
        const int64_t nseg = (len + seg_len - 1) / seg_len;
        const int64_t item = t - item_start[k];
        const bool dot_phase = item < nseg;
        const int64_t seg = dot_phase ? item : item - nseg;
        const int64_t e0 = seg * seg_len, e1 = min(len, e0 + seg_len);   // element range of the item
        const uint32_t* __restrict__ idxp = cv.idx + b0;
        const float* __restrict__ valp = cv.val + b0;

        if (dot_phase) {
            float g = 0.0f, h = 0.0f;
            int64_t e = e0 + threadIdx.x;
            // UNROLL independent index/value loads, then their gathers, then the arithmetic
            for (; e + (UNROLL - 1) * TPB < e1; e += UNROLL * TPB) {
                uint32_t r[UNROLL];
                float a[UNROLL], yy[UNROLL], vv[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const int64_t eu = e + u * TPB;
                    a[u] = stream_load(valp + eu);
                    if (DENSE) {
                        r[u] = (uint32_t)eu;
                        yy[u] = KIND == K_DUAL ? 0.0f : y[r[u]];
                    } else {
                        decode<KIND>(stream_load(idxp + eu), r[u], yy[u], y);
                    }
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) vv[u] = load_shared(v, r[u]);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) accumulate<KIND>(a[u], vv[u], yy[u], g, h);
            }
            for (; e < e1; e += TPB) {
                uint32_t r;
                float yy;
                if (DENSE) {
                    r = (uint32_t)e;
                    yy = KIND == K_DUAL ? 0.0f : y[r];
                } else {
                    decode<KIND>(idxp[e], r, yy, y);
                }
                accumulate<KIND>(valp[e], load_shared(v, r), yy, g, h);
            }
            g = wave_sum(g);
            h = wave_sum(h);
            const int w = threadIdx.x / WAVE;
            if ((threadIdx.x & (WAVE - 1)) == 0) {
                s_part[2 * w] = g;
                s_part[2 * w + 1] = h;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                double G = 0.0, H = 0.0;
#pragma unroll
                for (int ww = 0; ww < WAVES_PER_WG; ++ww) {
                    G += (double)s_part[2 * ww];
                    H += (double)s_part[2 * ww + 1];
                }
                // Both sums must have been performed before the count goes up.  The two additions return
                // the old values, and the increment is made to depend on them: a returning atomic
                // answers only once it has been performed where all compute dies see it, so no
                // fence (and no assumption about how one is lowered) is needed.
                const double g_seen = atomicAdd(&st[k].g, G);
                const double h_seen = atomicAdd(&st[k].h, H);
                uint32_t one = 1u;
                asm volatile("" : "+v"(one) : "v"(g_seen), "v"(h_seen));
                const uint32_t arrived = atomicAdd(&st[k].done, one);
                if (arrived == (uint32_t)nseg - 1u) {              // last dot item of this coordinate
                    const double Gt = atomicAdd(&st[k].g, 0.0);
                    const double Ht = atomicAdd(&st[k].h, 0.0);
                    const float xc = x[c];
                    const float yc = KIND == K_DUAL ? y[c] : 0.0f;
                    float mult;
                    x[c] = take_step<KIND>(Gt, Ht, xc, norms[c], yc, sp, mult);
                    const uint64_t word = (1ull << 32) | (uint64_t)__float_as_uint(mult);
                    __hip_atomic_store(&st[k].published, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            continue;
        }

        // scatter phase: wait (bounded) for the step of this coordinate
        if (threadIdx.x == 0) {
            uint32_t spins = 0;
            uint64_t word;
            while (((word = __hip_atomic_load(&st[k].published, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 32) == 0) {
                __builtin_amdgcn_s_sleep(16);
                if (++spins > SPIN_LIMIT) break;
            }
            if ((word >> 32) != 0) {
                s_mult = __uint_as_float((uint32_t)word);
            } else {
                s_mult = 0.0f;
                atomicOr(status, 1u);
            }
        }
        __syncthreads();
        const float mult = s_mult;
        if (mult == 0.0f) continue;
        int64_t e = e0 + threadIdx.x;
        for (; e + (UNROLL - 1) * TPB < e1; e += UNROLL * TPB) {
            uint32_t r[UNROLL];
            float a[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t eu = e + u * TPB;
                a[u] = stream_load(valp + eu);
                r[u] = DENSE ? (uint32_t)eu
                             : (stream_load(idxp + eu) & (KIND == K_PRIMAL_LOGISTIC ? ~LABEL_BIT : 0xFFFFFFFFu));
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) unsafeAtomicAdd(v + r[u], mult * a[u]);
        }
        for (; e < e1; e += TPB) {
            const uint32_t r = DENSE ? (uint32_t)e : (idxp[e] & (KIND == K_PRIMAL_LOGISTIC ? ~LABEL_BIT : 0xFFFFFFFFu));
            unsafeAtomicAdd(v + r, mult * valp[e]);
        }
    }
}

template <int KIND>
static int launch_kind(snap_handle* h, const ChunkView& cv, const snap_handle::Chunk& ck, const uint32_t* order,
                       const StepParams& sp) {
    const int64_t dense_len = h->dense ? h->ld : 0;
    if (ck.n_large > 0) {
        const uint32_t* order_large = order + ck.n_small;
        hipLaunchKernelGGL(k_large_prepare, dim3(1), dim3(1024), 0, h->compute, cv.ptr, cv.c0, order_large, ck.n_large,
                           dense_len, h->seg, h->item_start, h->lstate, h->ticket);
        int64_t wgs = ck.n_items;
        if (h->inflight_nnz > 0) wgs = std::min<int64_t>(wgs, std::max<int64_t>(1, h->inflight_nnz / h->seg));
        wgs = std::min<int64_t>(wgs, 256 * 8);          // no more than the device holds at once
        const dim3 grid((unsigned)wgs);
        if (h->dense)
            hipLaunchKernelGGL((k_scd_large<KIND, true>), grid, dim3(TPB), 0, h->compute, cv, order_large, ck.n_large,
                               h->item_start, ck.n_items, h->lstate, h->ticket, h->status, h->y, h->x, h->v, h->norms,
                               sp, dense_len, h->seg);
        else
            hipLaunchKernelGGL((k_scd_large<KIND, false>), grid, dim3(TPB), 0, h->compute, cv, order_large, ck.n_large,
                               h->item_start, ck.n_items, h->lstate, h->ticket, h->status, h->y, h->x, h->v, h->norms,
                               sp, dense_len, h->seg);
    }
    if (h->opt.profile && !h->streaming) SNAP_HIP(hipEventRecord(h->ev[3], h->compute));
    if (ck.n_small > 0) {
        int64_t waves = std::min<int64_t>(ck.n_small, 256 * 32);
        if (h->inflight_nnz > 0)
            waves = std::min<int64_t>(waves, std::max<int64_t>(1, (int64_t)((double)h->inflight_nnz / h->avg_small_len)));
        const dim3 grid((unsigned)((waves + WAVES_PER_WG - 1) / WAVES_PER_WG));
        if (h->max_small_len <= WAVE)
            hipLaunchKernelGGL((k_scd_small<KIND, 1>), grid, dim3(TPB), 0, h->compute, cv, order, ck.n_small, h->y, h->x,
                               h->v, h->norms, sp, waves);
        else
            hipLaunchKernelGGL((k_scd_small<KIND, 4>), grid, dim3(TPB), 0, h->compute, cv, order, ck.n_small, h->y, h->x,
                               h->v, h->norms, sp, waves);
    }
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

int scd_run_chunk(snap_handle* h, const ChunkView& cv, const snap_handle::Chunk& ck, const uint32_t* order) {
    const StepParams sp = make_step_params(h);
    if (ck.n_items > 0x7FFFFFFFll || ck.n_small / WAVES_PER_WG > 0x7FFFFFFFll) {
        set_error("chunk too large for one launch");
        return SNAP_EINVAL;
    }
    switch (h->kind) {
    case K_PRIMAL_RIDGE: return launch_kind<K_PRIMAL_RIDGE>(h, cv, ck, order, sp);
    case K_PRIMAL_LOGISTIC: return launch_kind<K_PRIMAL_LOGISTIC>(h, cv, ck, order, sp);
    case K_DUAL: return launch_kind<K_DUAL>(h, cv, ck, order, sp);
    }
    set_error("unknown solver kind");
    return SNAP_EINVAL;
}

}  // namespace snap
