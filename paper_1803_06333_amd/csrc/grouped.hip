// Exact group sweeps: an epoch for data whose coordinates come in groups with pairwise disjoint
// supports (the columns of one one-hot encoded field of click-log data, Section 4).  Coordinates of
// one group do not interact -- no row of v is touched by two of them -- so updating all of them at
// once IS the sequential coordinate-descent result for that group; groups are visited one after
// the other.  The epoch therefore equals sequential SCD (Section 3.1) in the order "group 0, group
// 1, ..." exactly (up to rounding), and needs neither atomics on v nor a cap on the work in flight.
//
// What makes it fast on this part is that both inner loops turn from random 4-byte accesses to the
// 183 MB vector v into coalesced streams over the rows:
//   - every group g has a row map: rowmap[g][r] = rank of the coordinate of g that contains row r
//     (ranks order the group's coordinates by decreasing length; bit 31 carries the label sign);
//   - one row pass reads v[r] once, applies the step of the previous group
//     (v[r] += delta[g-1][rank]), evaluates loss' and loss'' at the new v[r] and adds them into the
//     sums of group g's coordinate: hot ranks (the longest coordinates) accumulate in LDS, one
//     partial array per workgroup, summed afterwards in a fixed order;
//   - a second kernel sums the partials of the hot ranks, lets the remaining (short) coordinates of
//     the group take their sums column-wise, one wavefront per coordinate, and turns all sums into
//     the steps that the next row pass applies.
// Traffic per group and row: two map entries, read + write of v = 16 bytes (+ values unless all 1).
#include "scd_device.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <vector>

namespace snap {

constexpr uint32_t RANK_MASK = 0x7FFFFFFFu;
constexpr uint32_t RANK_NONE = 0x7FFFFFFFu;      // row not covered by the group
// The sums of the hot ranks are kept in LDS as 64-bit fixed-point integers: integer LDS atomics run
// more than twenty times faster here than ds_add_f32 (measured), the result does not depend on the
// order of the additions (the epoch is bit-reproducible), and with 40 fractional bits it is more
// accurate than fp32 accumulation.
constexpr int HOT_MAX = 8192;                    // ranks accumulated in LDS (two int64 each: 128 KB)
constexpr int ROW_TPB = 1024;
constexpr int ROW_WGS_DEFAULT = 256;             // one workgroup per compute unit
static int row_wgs() {
    static const int v = [] {
        const char* e = getenv("SNAP_ROW_WGS");      // tuning knob
        return e ? std::max(1, atoi(e)) : ROW_WGS_DEFAULT;
    }();
    return v;
}
static int hot_max() {
    static const int v = [] {
        const char* e = getenv("SNAP_HOT_MAX");      // tuning knob
        return e ? std::max(4, std::min(HOT_MAX, atoi(e))) : HOT_MAX;
    }();
    return v;
}

// ---- creation --------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, size_t count, uint32_t value) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        p[i] = value;
}

// For every nonzero: row map entry of its group <- rank of its coordinate.  A second writer of the
// same entry means two coordinates of one group share a row: flag it.
__global__ void __launch_bounds__(256)
k_build_rowmap(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, const float* __restrict__ val,
               int64_t m, int64_t nnz, const int64_t* __restrict__ gbounds, int64_t n_groups,
               const uint32_t* __restrict__ rank_of, int64_t n_pad, uint32_t* rowmap, float* rowval,
               uint32_t* flags) {
    const int64_t b0 = (int64_t)blockIdx.x * 4096, b1 = min(nnz, b0 + 4096);
    int64_t lo = 0, hi = m;                       // coordinate of the block's first nonzero
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr[mid] <= b0) lo = mid; else hi = mid;
    }
    const int64_t cstart = lo;
    for (int64_t k = b0 + threadIdx.x; k < b1; k += 256) {
        int64_t l = cstart, step = 1;
        while (l + step < m && ptr[l + step] <= k) { l += step; step <<= 1; }
        int64_t r = min(m, l + step);
        while (r - l > 1) {
            const int64_t mid = (l + r) >> 1;
            if (ptr[mid] <= k) l = mid; else r = mid;
        }
        int64_t glo = 0, ghi = n_groups;          // group of coordinate l
        while (ghi - glo > 1) {
            const int64_t mid = (glo + ghi) >> 1;
            if (gbounds[mid] <= l) glo = mid; else ghi = mid;
        }
        const size_t slot = (size_t)glo * (size_t)n_pad + (size_t)(idx[k] & ~LABEL_BIT);
        const uint32_t old = atomicCAS(rowmap + slot, RANK_NONE, rank_of[l]);
        if (old != RANK_NONE) atomicOr(flags, 1u);
        if (rowval) rowval[slot] = val[k];
        if (val[k] != 1.0f) atomicOr(flags, 2u);
        atomicMax(flags + 1, __float_as_uint(fabsf(val[k])));      // largest magnitude (bit order = value order)
    }
}

__global__ void k_rowmap_labels(uint32_t* __restrict__ rowmap, int64_t n_groups, int64_t n, int64_t n_pad,
                                const float* __restrict__ y) {
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t bit = y[r] < 0.0f ? LABEL_BIT : 0u;
        for (int64_t g = 0; g < n_groups; ++g) rowmap[(size_t)g * n_pad + r] |= bit;
    }
}

void grouped_free(snap_handle* h) {
    if (h->ev_group) {
        for (int64_t i = 0; i < 2 * (h->n_groups + 1); ++i)
            if (h->ev_group[i]) (void)hipEventDestroy(h->ev_group[i]);
        delete[] h->ev_group;
        h->ev_group = nullptr;
    }
    delete[] h->gbounds_host;
    delete[] h->ghot_host;
    h->gbounds_host = nullptr;
    h->ghot_host = nullptr;
    (void)hipFree(h->rowmap);
    (void)hipFree(h->rowval);
    (void)hipFree(h->rank_of);
    (void)hipFree(h->coord_of);
    (void)hipFree(h->gdelta);
    (void)hipFree(h->gpartial);
    h->rowmap = nullptr;
    h->rowval = nullptr;
    h->rank_of = h->coord_of = nullptr;
    h->gdelta = nullptr;
    h->gpartial = nullptr;
}

int grouped_setup(snap_handle* h, const int64_t* hptr) {
    const int64_t m = h->m, G = h->opt.n_groups, n = h->n;
    const int64_t* gb = h->opt.group_bounds;
    if (h->form != SNAP_PRIMAL || h->dense || h->streaming) {
        set_error("group sweeps need the primal form on resident sparse data");
        return SNAP_EUNSUPPORTED;
    }
    if (!gb || G < 1 || gb[0] != 0 || gb[G] != m) {
        set_error("group_bounds must run from 0 to the number of coordinates");
        return SNAP_EINVAL;
    }
    for (int64_t g = 0; g < G; ++g)
        if (gb[g + 1] < gb[g]) {
            set_error("group_bounds must be non-decreasing");
            return SNAP_EINVAL;
        }
    h->n_groups = G;
    h->n_pad = (n + 3) / 4 * 4;
    h->gbounds_host = new (std::nothrow) int64_t[(size_t)G + 1];
    h->ghot_host = new (std::nothrow) int[(size_t)G];
    if (!h->gbounds_host || !h->ghot_host) return SNAP_ENOMEM;
    std::copy(gb, gb + G + 1, h->gbounds_host);

    int lds_max = 0;
    SNAP_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device));
    const int hot_cap = std::max(4, std::min<int>(hot_max(), (lds_max - 1024) / 16));
    // ranks inside each group: coordinates by decreasing length (ties by index)
    std::vector<uint32_t> rank_of((size_t)m), coord_of((size_t)m);
    int max_hot = 1;
    for (int64_t g = 0; g < G; ++g) {
        const int64_t c0 = gb[g], sz = gb[g + 1] - gb[g];
        std::vector<int64_t> order((size_t)sz);
        std::iota(order.begin(), order.end(), c0);
        std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) {
            return hptr[a + 1] - hptr[a] > hptr[b + 1] - hptr[b];
        });
        for (int64_t r = 0; r < sz; ++r) {
            rank_of[(size_t)order[(size_t)r]] = (uint32_t)r;
            coord_of[(size_t)(c0 + r)] = (uint32_t)order[(size_t)r];
        }
        // hot ranks: accumulated in LDS by the row pass; a rank is worth a slot while its
        // coordinate is long enough to be hit by most workgroups
        int hot = 0;
        while (hot < sz && hot < hot_cap && hptr[order[(size_t)hot] + 1] - hptr[order[(size_t)hot]] >= ROW_WGS_DEFAULT / 2) ++hot;
        h->ghot_host[g] = hot;
        max_hot = std::max(max_hot, hot);
    }
    h->gpartial_stride = 2 * (int64_t)max_hot;

    int64_t* d_gb = nullptr;
    uint32_t* flags = nullptr;
    SNAP_HIP(hipMalloc(&h->rank_of, (size_t)(m ? m : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->coord_of, (size_t)(m ? m : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->gdelta, (size_t)(m ? m : 1) * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->gpartial, (size_t)row_wgs() * (size_t)h->gpartial_stride * sizeof(long long)));
    SNAP_HIP(hipMalloc(&h->rowmap, (size_t)G * (size_t)h->n_pad * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->rowval, (size_t)G * (size_t)h->n_pad * sizeof(float)));
    SNAP_HIP(hipMalloc(&d_gb, (size_t)(G + 1) * sizeof(int64_t)));
    SNAP_HIP(hipMalloc(&flags, 2 * sizeof(uint32_t)));
    auto fail = [&](int rc) {
        (void)hipFree(d_gb);
        (void)hipFree(flags);
        return rc;
    };
#define G_HIP(call)                                                                \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) return fail(hip_fail(e_, #call, __FILE__, __LINE__)); \
    } while (0)
    G_HIP(hipMemcpyAsync(h->rank_of, rank_of.data(), (size_t)m * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
    G_HIP(hipMemcpyAsync(h->coord_of, coord_of.data(), (size_t)m * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
    G_HIP(hipMemcpyAsync(d_gb, gb, (size_t)(G + 1) * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
    int rc = fill_zero(flags, 8, h->compute);
    if (rc == SNAP_OK) rc = fill_zero(h->rowval, (size_t)G * (size_t)h->n_pad * sizeof(float), h->compute);
    if (rc == SNAP_OK) rc = fill_zero(h->gdelta, (size_t)m * sizeof(float), h->compute);
    if (rc != SNAP_OK) return fail(rc);
    hipLaunchKernelGGL(k_fill_u32, dim3(8192), dim3(256), 0, h->compute, h->rowmap, (size_t)G * (size_t)h->n_pad, RANK_NONE);
    if (h->nnz > 0)
        hipLaunchKernelGGL(k_build_rowmap, dim3((unsigned)((h->nnz + 4095) / 4096)), dim3(256), 0, h->compute, h->ptr,
                           h->idx, h->val, m, h->nnz, d_gb, G, h->rank_of, h->n_pad, h->rowmap, h->rowval, flags);
    if (h->kind == K_PRIMAL_LOGISTIC && n > 0)
        hipLaunchKernelGGL(k_rowmap_labels, dim3(4096), dim3(256), 0, h->compute, h->rowmap, G, n, h->n_pad, h->y);
    G_HIP(hipGetLastError());
    uint32_t fl2[2] = {0, 0};
    G_HIP(hipMemcpyAsync(fl2, flags, 8, hipMemcpyDeviceToHost, h->compute));
    G_HIP(hipStreamSynchronize(h->compute));
    const uint32_t fl = fl2[0];
    {
        float amax;
        memcpy(&amax, &fl2[1], 4);
        int e = 0;
        if (amax > 0.0f) (void)frexpf(amax, &e);     // amax <= 2^e
        h->gscale_exp = e;
    }
#undef G_HIP
    (void)hipFree(d_gb);
    (void)hipFree(flags);
    if (fl & 1u) {
        set_error("two coordinates of one group share a row: the groups are not disjoint");
        return SNAP_EINVAL;
    }
    h->unit_values = !(fl & 2u);
    if (h->unit_values) {
        (void)hipFree(h->rowval);
        h->rowval = nullptr;
    }
    if (h->opt.profile) {
        h->ev_group = new (std::nothrow) hipEvent_t[(size_t)(2 * (G + 1))]();
        if (!h->ev_group) return SNAP_ENOMEM;
        for (int64_t i = 0; i < 2 * (G + 1); ++i) SNAP_HIP(hipEventCreate(&h->ev_group[i]));
    }
    // bookkeeping for the statistics: nonzeros and coordinates of the hot ranks
    h->g_hot_coords = h->g_hot_nnz = 0;
    for (int64_t g = 0; g < G; ++g) {
        h->g_hot_coords += h->ghot_host[g];
        for (int r = 0; r < h->ghot_host[g]; ++r) {
            const int64_t c = coord_of[(size_t)(gb[g] + r)];
            h->g_hot_nnz += hptr[c + 1] - hptr[c];
        }
    }
    h->grouped = true;
    return SNAP_OK;
}

// ---- the row pass ------------------------------------------------------------------------------------
// SCATTER: v[r] += delta_prev[rank] * a for the previous group.  HIST: sums of the current group's
// hot ranks.  Four consecutive rows per thread and iteration (128-bit loads and stores).
template <int KIND, bool UNIT, bool SCATTER, bool HIST>
__global__ void __launch_bounds__(ROW_TPB)
k_group_rows(const uint32_t* __restrict__ map_prev, const float* __restrict__ val_prev,
             const float* __restrict__ delta_prev, const uint32_t* __restrict__ map_cur,
             const float* __restrict__ val_cur, int hot, float* __restrict__ v, const float* __restrict__ y,
             int64_t n, long long* __restrict__ partial, int64_t partial_stride, float scale_g, float scale_h) {
    // fixed point: [0,hot): sum of a loss' * scale_g, [hot,2hot): sum of a^2 loss'' * scale_h
    extern __shared__ unsigned long long hist[];
    if (HIST) {
        for (int i = threadIdx.x; i < 2 * hot; i += ROW_TPB) hist[i] = 0ull;
        __syncthreads();
    }
    // the four longest coordinates of a group hold a third of its rows: their sums stay in
    // registers (one LDS update per wavefront at the end) instead of colliding in LDS
    float rg0 = 0.0f, rg1 = 0.0f, rg2 = 0.0f, rg3 = 0.0f, rh0 = 0.0f, rh1 = 0.0f, rh2 = 0.0f, rh3 = 0.0f;
    const int64_t quads = (n + 3) / 4;
    const int64_t per = (quads + gridDim.x - 1) / gridDim.x;
    const int64_t q0 = min(quads, (int64_t)blockIdx.x * per), q1 = min(quads, q0 + per);
    for (int64_t q = q0 + threadIdx.x; q < q1; q += ROW_TPB) {
        const int64_t r = 4 * q;
        float vv[4];
        uint32_t mp[4] = {RANK_NONE, RANK_NONE, RANK_NONE, RANK_NONE}, mc[4] = {RANK_NONE, RANK_NONE, RANK_NONE, RANK_NONE};
        float ap[4] = {1.0f, 1.0f, 1.0f, 1.0f}, ac[4] = {1.0f, 1.0f, 1.0f, 1.0f}, yy[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        const bool full = r + 3 < n;
        if (full) {
            const float4 t = *reinterpret_cast<const float4*>(v + r);
            vv[0] = t.x; vv[1] = t.y; vv[2] = t.z; vv[3] = t.w;
            if (SCATTER) {
                const uint4 u = *reinterpret_cast<const uint4*>(map_prev + r);
                mp[0] = u.x; mp[1] = u.y; mp[2] = u.z; mp[3] = u.w;
                if (!UNIT) {
                    const float4 a = *reinterpret_cast<const float4*>(val_prev + r);
                    ap[0] = a.x; ap[1] = a.y; ap[2] = a.z; ap[3] = a.w;
                }
            }
            if (HIST) {
                const uint4 u = *reinterpret_cast<const uint4*>(map_cur + r);
                mc[0] = u.x; mc[1] = u.y; mc[2] = u.z; mc[3] = u.w;
                if (!UNIT) {
                    const float4 a = *reinterpret_cast<const float4*>(val_cur + r);
                    ac[0] = a.x; ac[1] = a.y; ac[2] = a.z; ac[3] = a.w;
                }
                if (KIND == K_PRIMAL_RIDGE) {
                    const float4 t2 = *reinterpret_cast<const float4*>(y + r);
                    yy[0] = t2.x; yy[1] = t2.y; yy[2] = t2.z; yy[3] = t2.w;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = r + j < n;          // the maps are padded to a multiple of four rows
                vv[j] = in ? v[r + j] : 0.0f;
                if (SCATTER) {
                    mp[j] = in ? map_prev[r + j] : RANK_NONE;
                    if (!UNIT) ap[j] = in ? val_prev[r + j] : 0.0f;
                }
                if (HIST) {
                    mc[j] = in ? map_cur[r + j] : RANK_NONE;
                    if (!UNIT) ac[j] = in ? val_cur[r + j] : 0.0f;
                    if (KIND == K_PRIMAL_RIDGE) yy[j] = in ? y[r + j] : 0.0f;
                }
            }
        }
        if (SCATTER) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t rk = mp[j] & RANK_MASK;
                if (rk != RANK_NONE) vv[j] += delta_prev[rk] * ap[j];
            }
            if (full) {
                *reinterpret_cast<float4*>(v + r) = make_float4(vv[0], vv[1], vv[2], vv[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (r + j < n) v[r + j] = vv[j];
            }
        }
        if (HIST) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t rk = mc[j] & RANK_MASK;
                if (rk < (uint32_t)hot) {
                    if (KIND == K_PRIMAL_LOGISTIC) yy[j] = (mc[j] & LABEL_BIT) ? -1.0f : 1.0f;
                    float g = 0.0f, hh = 0.0f;
                    accumulate<KIND>(ac[j], vv[j], yy[j], g, hh);
                    if (rk < 4u) {
                        rg0 += rk == 0u ? g : 0.0f;
                        rg1 += rk == 1u ? g : 0.0f;
                        rg2 += rk == 2u ? g : 0.0f;
                        rg3 += rk == 3u ? g : 0.0f;
                        if (KIND == K_PRIMAL_LOGISTIC) {
                            rh0 += rk == 0u ? hh : 0.0f;
                            rh1 += rk == 1u ? hh : 0.0f;
                            rh2 += rk == 2u ? hh : 0.0f;
                            rh3 += rk == 3u ? hh : 0.0f;
                        }
                    } else {
                        atomicAdd(&hist[rk], (unsigned long long)__float2ll_rn(g * scale_g));
                        if (KIND == K_PRIMAL_LOGISTIC)
                            atomicAdd(&hist[hot + rk], (unsigned long long)__float2ll_rn(hh * scale_h));
                    }
                }
            }
        }
    }
    if (HIST) {
        rg0 = wave_sum(rg0); rg1 = wave_sum(rg1); rg2 = wave_sum(rg2); rg3 = wave_sum(rg3);
        if (KIND == K_PRIMAL_LOGISTIC) {
            rh0 = wave_sum(rh0); rh1 = wave_sum(rh1); rh2 = wave_sum(rh2); rh3 = wave_sum(rh3);
        }
        if ((threadIdx.x & (WAVE - 1)) == 0) {
            const float rg[4] = {rg0, rg1, rg2, rg3}, rh[4] = {rh0, rh1, rh2, rh3};
            for (int t = 0; t < 4 && t < hot; ++t) {
                atomicAdd(&hist[t], (unsigned long long)__float2ll_rn(rg[t] * scale_g));
                if (KIND == K_PRIMAL_LOGISTIC) atomicAdd(&hist[hot + t], (unsigned long long)__float2ll_rn(rh[t] * scale_h));
            }
        }
        __syncthreads();
        long long* out = partial + (size_t)blockIdx.x * (size_t)partial_stride;
        for (int i = threadIdx.x; i < 2 * hot; i += ROW_TPB) out[i] = (long long)hist[i];
    }
}

// ---- sums of the short coordinates and the steps of one group ------------------------------------------
// One launch, two kinds of workgroups.  The first n_hot_blocks handle the hot ranks: 32 ranks per
// workgroup, 8 threads per rank, each summing every 8th per-workgroup partial of the row pass (integer
// sums: exact and independent of the order), combined in LDS, then one thread takes the step.  The
// others handle the cold ranks: one wavefront per coordinate gathers its two sums column-wise (v is
// not written while this kernel runs) and takes the step right away.
constexpr int STEP_RANKS = 32, STEP_PARTS = 8;

template <int KIND>
__global__ void __launch_bounds__(STEP_RANKS * STEP_PARTS)
k_group_finish(const long long* __restrict__ partial, int64_t partial_stride, int n_wgs, int hot, int n_hot_blocks,
               double inv_scale_g, double inv_scale_h, const int64_t* __restrict__ ptr,
               const uint32_t* __restrict__ idx, const float* __restrict__ val, const float* __restrict__ v,
               const float* __restrict__ y, const uint32_t* __restrict__ coord_of, int64_t g0, int64_t group_size,
               float* __restrict__ x, const float* __restrict__ norms, float* __restrict__ delta, StepParams sp) {
    __shared__ long long sg[STEP_PARTS][STEP_RANKS], sh[STEP_PARTS][STEP_RANKS];
    if ((int)blockIdx.x >= n_hot_blocks) {
        const int lane = threadIdx.x & (WAVE - 1);
        const int64_t wave0 = ((int64_t)(blockIdx.x - n_hot_blocks) * blockDim.x + threadIdx.x) / WAVE;
        const int64_t nwaves = (int64_t)(gridDim.x - n_hot_blocks) * blockDim.x / WAVE;
        for (int64_t rk = hot + wave0; rk < group_size; rk += nwaves) {
            const int64_t c = coord_of[g0 + rk];
            float g = 0.0f, hh = 0.0f;
            for (int64_t k = ptr[c] + lane; k < ptr[c + 1]; k += WAVE) {
                uint32_t r;
                float yy;
                decode<KIND>(idx[k], r, yy, y);
                accumulate<KIND>(val[k], v[r], yy, g, hh);
            }
            g = wave_sum(g);
            hh = wave_sum(hh);
            if (lane == 0) {
                float mult;
                x[c] = take_step<KIND>((double)g, (double)hh, x[c], norms[c], 0.0f, sp, mult);
                delta[g0 + rk] = mult;
            }
        }
        return;
    }
    const int lr = threadIdx.x % STEP_RANKS, part = threadIdx.x / STEP_RANKS;
    const int64_t rk = (int64_t)blockIdx.x * STEP_RANKS + lr;
    long long Gi = 0, Hi = 0;
    if (rk < hot) {
        for (int w = part; w < n_wgs; w += STEP_PARTS) {
            Gi += partial[(size_t)w * partial_stride + rk];
            if (KIND == K_PRIMAL_LOGISTIC) Hi += partial[(size_t)w * partial_stride + hot + rk];
        }
    }
    sg[part][lr] = Gi;
    sh[part][lr] = Hi;
    __syncthreads();
    if (part != 0 || rk >= hot) return;
    Gi = 0;
    Hi = 0;
#pragma unroll
    for (int p = 0; p < STEP_PARTS; ++p) {
        Gi += sg[p][lr];
        Hi += sh[p][lr];
    }
    const int64_t c = coord_of[g0 + rk];
    float mult;
    x[c] = take_step<KIND>((double)Gi * inv_scale_g, (double)Hi * inv_scale_h, x[c], norms[c], 0.0f, sp, mult);
    delta[g0 + rk] = mult;
}

template <int KIND, bool UNIT>
static int grouped_epoch_kind(snap_handle* h) {
    const StepParams sp = make_step_params(h);
    const int64_t n = h->n, G = h->n_groups;
    long long* gpart = (long long*)h->gpartial;
    // power-of-two scales (exact in fp32): |a loss'| <= 2^e and a^2 loss'' <= 2^(2e) for the logistic loss,
    // at most 2^18 rows per workgroup, so the sums stay below 2^59; ridge terms are unbounded in
    // principle, 24 fractional bits leave 2^39 of range
    const float scale_g = KIND == K_PRIMAL_LOGISTIC ? ldexpf(1.0f, 40 - h->gscale_exp) : ldexpf(1.0f, 24);
    const float scale_h = ldexpf(1.0f, 40 - 2 * h->gscale_exp);
    int64_t prev = -1;                              // last non-empty group, whose steps are still to be applied
    const bool prof = h->opt.profile != 0 && h->ev_group != nullptr;
    int n_pass = 0;
    for (int64_t g = 0; g <= G; ++g) {
        const bool last = g == G;
        const int64_t g0 = last ? 0 : h->gbounds_host[g], sz = last ? 0 : h->gbounds_host[g + 1] - g0;
        if (!last && sz == 0) continue;
        const int hot = last ? 0 : h->ghot_host[g];
        const uint32_t* map_prev = prev >= 0 ? h->rowmap + (size_t)prev * h->n_pad : nullptr;
        const float* val_prev = (prev >= 0 && !UNIT) ? h->rowval + (size_t)prev * h->n_pad : nullptr;
        const float* delta_prev = prev >= 0 ? h->gdelta + h->gbounds_host[prev] : nullptr;
        const uint32_t* map_cur = last ? nullptr : h->rowmap + (size_t)g * h->n_pad;
        const float* val_cur = (last || UNIT) ? nullptr : h->rowval + (size_t)g * h->n_pad;
        const size_t lds = (size_t)2 * hot * sizeof(unsigned long long);
        const bool scatter = prev >= 0, histo = !last && hot > 0;
        if (n > 0 && (scatter || histo)) {
            if (prof) SNAP_HIP(hipEventRecord(h->ev_group[2 * n_pass], h->compute));
            if (scatter && histo)
                hipLaunchKernelGGL((k_group_rows<KIND, UNIT, true, true>), dim3(row_wgs()), dim3(ROW_TPB), lds, h->compute,
                                   map_prev, val_prev, delta_prev, map_cur, val_cur, hot, h->v, h->y, n, gpart,
                                   h->gpartial_stride, scale_g, scale_h);
            else if (scatter)
                hipLaunchKernelGGL((k_group_rows<KIND, UNIT, true, false>), dim3(row_wgs()), dim3(ROW_TPB), 0, h->compute,
                                   map_prev, val_prev, delta_prev, map_cur, val_cur, 0, h->v, h->y, n, gpart,
                                   h->gpartial_stride, scale_g, scale_h);
            else
                hipLaunchKernelGGL((k_group_rows<KIND, UNIT, false, true>), dim3(row_wgs()), dim3(ROW_TPB), lds, h->compute,
                                   map_prev, val_prev, delta_prev, map_cur, val_cur, hot, h->v, h->y, n, gpart,
                                   h->gpartial_stride, scale_g, scale_h);
            if (prof) SNAP_HIP(hipEventRecord(h->ev_group[2 * n_pass + 1], h->compute));
            ++n_pass;
        }
        if (last) break;
        const int n_hot_blocks = (hot + STEP_RANKS - 1) / STEP_RANKS;
        const int64_t cold = sz - hot;
        const int n_cold_blocks = (int)std::min<int64_t>((cold + 3) / 4, 16384);
        hipLaunchKernelGGL((k_group_finish<KIND>), dim3((unsigned)(n_hot_blocks + n_cold_blocks)),
                           dim3(STEP_RANKS * STEP_PARTS), 0, h->compute, gpart, h->gpartial_stride, row_wgs(), hot,
                           n_hot_blocks, 1.0 / (double)scale_g, 1.0 / (double)scale_h, h->ptr, h->idx, h->val, h->v,
                           h->y, h->coord_of, g0, sz, h->x, h->norms, h->gdelta, sp);
        prev = g;
    }
    h->n_row_passes = n_pass;
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

int grouped_epoch(snap_handle* h) {
    if (h->kind == K_PRIMAL_RIDGE)
        return h->unit_values ? grouped_epoch_kind<K_PRIMAL_RIDGE, true>(h) : grouped_epoch_kind<K_PRIMAL_RIDGE, false>(h);
    return h->unit_values ? grouped_epoch_kind<K_PRIMAL_LOGISTIC, true>(h)
                          : grouped_epoch_kind<K_PRIMAL_LOGISTIC, false>(h);
}

}  // namespace snap
