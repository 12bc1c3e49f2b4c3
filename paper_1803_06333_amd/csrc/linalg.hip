// Deterministic helper kernels around the SCD epoch: squared norms of the coordinates, label
// folding, v = A x (Algorithm 1: the shared vector is A alpha), the objective P(w) (eq. (1) with
// the 1/n scaling), the duality gap and decision values.  fp32 data, every sum in fp64 and in a
// fixed order (no atomics on the reduction paths, so repeated calls give identical bits; the
// only exception is the scatter product for compressed-column data, which uses atomics on v).
#include "scd_device.h"
#include <algorithm>
#include <mutex>

namespace snap {

constexpr int LTPB = 256;

__device__ __forceinline__ double wave_sum_d(double x) {
#pragma unroll
    for (int off = WAVE / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, WAVE);
    return x;
}

// sum over the workgroup, result valid in thread 0 (fixed order)
__device__ __forceinline__ double block_sum_d(double x, double* scratch /* >= LTPB/WAVE */) {
    x = wave_sum_d(x);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) scratch[threadIdx.x / WAVE] = x;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x / WAVE); ++w) s += scratch[w];
    return s;
}

__global__ void k_fill_zero(uint32_t* p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

__global__ void k_fill_value(float* p, float value, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = value;
}

int fill_value(float* p, float value, int64_t count, hipStream_t s) {
    if (count <= 0) return SNAP_OK;
    const int grid = (int)((count + 255) / 256 < 4096 ? (count + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_fill_value, dim3(grid), dim3(256), 0, s, p, value, count);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

__global__ void k_clamp(float* p, float lo, float hi, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = fminf(fmaxf(p[i], lo), hi);
}

int clamp_range(float* p, float lo, float hi, int64_t count, hipStream_t s) {
    if (count <= 0) return SNAP_OK;
    const int grid = (int)((count + 255) / 256 < 4096 ? (count + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_clamp, dim3(grid), dim3(256), 0, s, p, lo, hi, count);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

int fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return SNAP_OK;
    const size_t words = bytes / 4;   // all buffers here are multiples of 4 bytes
    int grid = (int)((words + 255) / 256 < 8192 ? (words + 255) / 256 : 8192);
    hipLaunchKernelGGL(k_fill_zero, dim3(grid), dim3(256), 0, s, (uint32_t*)p, words);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// Two copies in one launch (the state saved before an epoch that may be discarded): a copy command
// costs some tens of microseconds of queueing each, more than a short epoch's permutation.
__global__ void __launch_bounds__(256)
k_copy_pair(float* __restrict__ d0, const float* __restrict__ s0, int64_t n0, float* __restrict__ d1,
            const float* __restrict__ s1, int64_t n1) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    // hipMalloc'd arrays: 16-byte aligned, so whole float4s first, then the tail
    const int64_t q0 = n0 / 4, q1 = n1 / 4;
    for (int64_t i = first; i < q0; i += stride) ((float4*)d0)[i] = ((const float4*)s0)[i];
    for (int64_t i = 4 * q0 + first; i < n0; i += stride) d0[i] = s0[i];
    for (int64_t i = first; i < q1; i += stride) ((float4*)d1)[i] = ((const float4*)s1)[i];
    for (int64_t i = 4 * q1 + first; i < n1; i += stride) d1[i] = s1[i];
}

int copy_pair(float* d0, const float* s0, int64_t n0, float* d1, const float* s1, int64_t n1, hipStream_t s) {
    const int64_t quads = (n0 > n1 ? n0 : n1) / 4 + 1;
    const int grid = (int)((quads + 255) / 256 < 4096 ? (quads + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_copy_pair, dim3(grid), dim3(256), 0, s, d0, s0, n0, d1, s1, n1);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// ---- squared norms and size classes -------------------------------------------------------------
__global__ void __launch_bounds__(LTPB)
k_coord_norms(const int64_t* __restrict__ ptr, const float* __restrict__ val, int64_t nnz_base, int64_t c0,
              int64_t c1, int64_t dense_len, int64_t small_max, float* __restrict__ norms,
              uint8_t* __restrict__ cls) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const int64_t nwaves = (int64_t)gridDim.x * blockDim.x / WAVE;
    for (int64_t c = c0 + wave0; c < c1; c += nwaves) {
        const int64_t s0 = dense_len > 0 ? c * dense_len : ptr[c] - nnz_base;
        const int64_t s1 = dense_len > 0 ? s0 + dense_len : ptr[c + 1] - nnz_base;
        double acc = 0.0;
        for (int64_t k = s0 + lane; k < s1; k += WAVE) acc += (double)val[k] * (double)val[k];
        acc = wave_sum_d(acc);
        if (lane == 0) {
            norms[c] = (float)acc;
            cls[c] = (dense_len > 0 || s1 - s0 > small_max) ? 1 : 0;
        }
    }
}

int norms_and_classes_chunk(snap_handle* h, const ChunkView& cv) {
    const int64_t dense_len = h->dense ? h->ld : 0;
    const int64_t mc = cv.c1 - cv.c0;
    int grid = (int)((mc + 3) / 4 < 16384 ? (mc + 3) / 4 : 16384);
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(k_coord_norms, dim3(grid), dim3(LTPB), 0, h->compute, cv.ptr, cv.val, cv.nnz_base, cv.c0,
                       cv.c1, dense_len, h->small_max, h->norms, h->cls);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// Sign of the label folded into bit 31 of the row index (primal logistic regression).
__global__ void k_fold_labels(uint32_t* __restrict__ idx, int64_t count, const float* __restrict__ y) {
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < count; k += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t r = idx[k] & ~LABEL_BIT;
        idx[k] = r | (y[r] < 0.0f ? LABEL_BIT : 0u);
    }
}

int fold_labels(snap_handle* h, uint32_t* idx, int64_t count, hipStream_t s) {
    if (count == 0) return SNAP_OK;
    int grid = (int)((count + 255) / 256 < 16384 ? (count + 255) / 256 : 16384);
    hipLaunchKernelGGL(k_fold_labels, dim3(grid), dim3(256), 0, s, idx, count, h->y);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// ---- v = A x -------------------------------------------------------------------------------------
// compressed data: out[idx[k]] += mult(c) * val[k] for every nonzero k of every coordinate c in
// [c0, c1); mult(c) = x[c] (primal) or y[c] x[c] (dual).  Each workgroup takes a block of
// consecutive nonzeros and locates their coordinates by bisection of ptr.
// OUT = double: the sums are taken in fp64 (hardware atomics) and rounded to fp32 once at the end, so
// the result does not depend on the order of the additions beyond the last bit -- with fp32 sums a
// coordinate-by-coordinate order can lose four digits where large terms cancel (a trained dual
// model: partial sums of a frequent feature a few thousand times its final value).
constexpr int64_t AXPY_BLOCK = 4096;

template <typename OUT>
__global__ void __launch_bounds__(LTPB)
k_scatter_axpy(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, const float* __restrict__ val,
               int64_t nnz_base, int64_t c0, int64_t c1, int64_t k0, int64_t k1, const float* __restrict__ x,
               const float* __restrict__ ymul, uint32_t idx_mask, OUT* out) {
    const int64_t b0 = k0 + (int64_t)blockIdx.x * AXPY_BLOCK, b1 = min(k1, b0 + AXPY_BLOCK);
    // coordinate of the block's first nonzero: largest c in [c0, c1) with ptr[c] <= b0
    int64_t lo = c0, hi = c1;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr[mid] <= b0) lo = mid; else hi = mid;
    }
    const int64_t cstart = lo;
    for (int64_t k = b0 + threadIdx.x; k < b1; k += LTPB) {
        int64_t l = cstart, r = c1;                    // largest c >= cstart with ptr[c] <= k
        // gallop first: most blocks sit inside one or a few coordinates
        int64_t step = 1;
        while (l + step < c1 && ptr[l + step] <= k) { l += step; step <<= 1; }
        r = min(c1, l + step);
        while (r - l > 1) {
            const int64_t mid = (l + r) >> 1;
            if (ptr[mid] <= k) l = mid; else r = mid;
        }
        const float mult = ymul ? ymul[l] * x[l] : x[l];
        if (mult != 0.0f) unsafeAtomicAdd(out + (idx[k - nnz_base] & idx_mask), (OUT)mult * (OUT)val[k - nnz_base]);
    }
}

__global__ void k_round_to_float(const double* __restrict__ in, float* __restrict__ out, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        out[i] = (float)in[i];
}

// dense, coordinate-major (element e of coordinate c at A[c*len + e]): out[e] = sum_c mult(c) A[c*len+e]
__global__ void __launch_bounds__(LTPB)
k_dense_axpy_all(const float* __restrict__ A, int64_t m, int64_t len, const float* __restrict__ x,
                 const float* __restrict__ ymul, float* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= len) return;
    double acc = 0.0;
    for (int64_t c = 0; c < m; ++c) {
        const float mult = ymul ? ymul[c] * x[c] : x[c];
        acc += (double)mult * (double)A[c * len + e];
    }
    out[e] = (float)acc;
}

// user: fp64 accumulator of vlen entries, or null for sums straight into v
static int axpy_chunk(snap_handle* h, int64_t chunk, const ChunkView& cv, void* user) {
    const float* ymul = h->form == SNAP_DUAL ? h->y : nullptr;
    const snap_handle::Chunk& ck = h->chunks[chunk];
    if (ck.nnz1 == ck.nnz0) return SNAP_OK;
    const int64_t nb = (ck.nnz1 - ck.nnz0 + AXPY_BLOCK - 1) / AXPY_BLOCK;
    if (user)
        hipLaunchKernelGGL((k_scatter_axpy<double>), dim3((unsigned)nb), dim3(LTPB), 0, h->compute, cv.ptr, cv.idx,
                           cv.val, cv.nnz_base, cv.c0, cv.c1, ck.nnz0, ck.nnz1, h->x, ymul, ~LABEL_BIT, (double*)user);
    else
        hipLaunchKernelGGL((k_scatter_axpy<float>), dim3((unsigned)nb), dim3(LTPB), 0, h->compute, cv.ptr, cv.idx,
                           cv.val, cv.nnz_base, cv.c0, cv.c1, ck.nnz0, ck.nnz1, h->x, ymul, ~LABEL_BIT, h->v);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

int recompute_shared(snap_handle* h) {
    const float* ymul = h->form == SNAP_DUAL ? h->y : nullptr;
    if (h->dense) {
        hipLaunchKernelGGL(k_dense_axpy_all, dim3((unsigned)((h->ld + LTPB - 1) / LTPB)), dim3(LTPB), 0, h->compute,
                           h->val, h->m, h->ld, h->x, ymul, h->v);
        SNAP_HIP(hipGetLastError());
        return SNAP_OK;
    }
    // fp64 sums in a buffer held for this call only; if the device has no room for it, fp32 sums in v
    double* acc = nullptr;
    const size_t acc_bytes = (size_t)h->vlen * sizeof(double);
    if (h->vlen > 0 && hipMalloc(&acc, acc_bytes) != hipSuccess) {
        (void)hipGetLastError();
        acc = nullptr;
    }
    int rc = acc ? fill_zero(acc, acc_bytes, h->compute) : fill_zero(h->v, (size_t)h->vlen * sizeof(float), h->compute);
    if (rc == SNAP_OK) rc = for_each_chunk(h, axpy_chunk, acc, true, false);
    if (rc == SNAP_OK && acc) {
        const int64_t blocks = (h->vlen + 255) / 256;
        hipLaunchKernelGGL(k_round_to_float, dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, h->compute,
                           acc, h->v, h->vlen);
        if (hipGetLastError() != hipSuccess) rc = SNAP_EHIP;
    }
    if (acc) {
        (void)hipStreamSynchronize(h->compute);
        (void)hipFree(acc);
    }
    return rc;
}

// ---- per-coordinate dots with v (no update), fp64 ---------------------------------------------------
// primal: gdot[c] = sum_k a_k loss'(y_r, v_r); dual: gdot[c] = sum_k a_k v_r.
template <int KIND>
__device__ __forceinline__ double dot_term(float a, float vv, float yy) {
    if (KIND == K_PRIMAL_RIDGE) return (double)a * ((double)vv - (double)yy);
    if (KIND == K_PRIMAL_LOGISTIC) {
        const double t = (double)yy * (double)vv;            // p = sigmoid(-t), overflow safe
        const double p = t >= 0 ? exp(-t) / (1.0 + exp(-t)) : 1.0 / (1.0 + exp(t));
        return -(double)a * (double)yy * p;
    }
    return (double)a * (double)vv;
}

template <int KIND>
__device__ __forceinline__ double dot_range(const uint32_t* __restrict__ idx, const float* __restrict__ val,
                                            int64_t s0, int64_t s1, int64_t dense_e0, const float* __restrict__ v,
                                            const float* __restrict__ y, int first, int stride) {
    double acc = 0.0;
    for (int64_t k = s0 + first; k < s1; k += stride) {
        uint32_t r;
        float yy = 0.0f;
        if (idx) {
            const uint32_t raw = idx[k];
            if (KIND == K_PRIMAL_LOGISTIC) {
                r = raw & ~LABEL_BIT;
                yy = (raw & LABEL_BIT) ? -1.0f : 1.0f;
            } else {
                r = raw;
                if (KIND == K_PRIMAL_RIDGE) yy = y[r];
            }
        } else {
            r = (uint32_t)(dense_e0 + (k - s0));
            if (KIND != K_DUAL) yy = y[r];
        }
        acc += dot_term<KIND>(val[k], v[r], yy);
    }
    return acc;
}

// one wavefront per coordinate (all coordinates of class 0 in [c0,c1))
template <int KIND>
__global__ void __launch_bounds__(LTPB)
k_dots_small(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, const float* __restrict__ val,
             int64_t nnz_base, int64_t c0, int64_t c1, const uint8_t* __restrict__ cls, const float* __restrict__ v,
             const float* __restrict__ y, double* __restrict__ gdot) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const int64_t nwaves = (int64_t)gridDim.x * blockDim.x / WAVE;
    for (int64_t c = c0 + wave0; c < c1; c += nwaves) {
        if (cls[c]) continue;
        double acc = dot_range<KIND>(idx, val, ptr[c] - nnz_base, ptr[c + 1] - nnz_base, 0, v, y, lane, WAVE);
        acc = wave_sum_d(acc);
        if (lane == 0) gdot[c] = acc;
    }
}

// class-1 coordinates: one workgroup per segment of SEG elements writes a partial sum; the list
// (large_list, seg_off) is the static one built at creation
template <int KIND>
__global__ void __launch_bounds__(LTPB)
k_dots_large_partial(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, const float* __restrict__ val,
                     int64_t nnz_base, int64_t dense_len, const int64_t* __restrict__ large_list,
                     const int64_t* __restrict__ seg_off, int64_t l0, int64_t l1,
                     int64_t SEG, const float* __restrict__ v, const float* __restrict__ y, double* __restrict__ partial) {
    __shared__ double scratch[LTPB / WAVE];
    const int64_t s = seg_off[l0] + blockIdx.x;       // global segment number
    int64_t lo = l0, hi = l1;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (seg_off[mid] <= s) lo = mid; else hi = mid;
    }
    const int64_t c = large_list[lo];
    const int64_t seg = s - seg_off[lo];
    int64_t b0, len;
    if (dense_len > 0) { b0 = c * dense_len; len = dense_len; }
    else { b0 = ptr[c] - nnz_base; len = ptr[c + 1] - ptr[c]; }
    const int64_t e0 = seg * SEG, e1 = min(len, e0 + SEG);
    double acc = dot_range<KIND>(dense_len > 0 ? nullptr : idx, val, b0 + e0, b0 + e1, e0, v, y, threadIdx.x, LTPB);
    acc = block_sum_d(acc, scratch);
    if (threadIdx.x == 0) partial[s] = acc;
}

__global__ void k_dots_large_finish(const int64_t* __restrict__ large_list, const int64_t* __restrict__ seg_off,
                                    int64_t l0, int64_t l1, const double* __restrict__ partial,
                                    double* __restrict__ gdot) {
    const int64_t l = l0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= l1) return;
    double acc = 0.0;
    for (int64_t s = seg_off[l]; s < seg_off[l + 1]; ++s) acc += partial[s];
    gdot[large_list[l]] = acc;
}

template <int KIND>
static int coord_dots_chunk(snap_handle* h, int64_t chunk, const ChunkView& cv, void*) {
    const int64_t dense_len = h->dense ? h->ld : 0;
    const snap_handle::Chunk& ck = h->chunks[chunk];
    const int64_t mc = cv.c1 - cv.c0;
    if (!h->dense && mc > 0) {
        int grid = (int)((mc + 3) / 4 < 32768 ? (mc + 3) / 4 : 32768);
        hipLaunchKernelGGL((k_dots_small<KIND>), dim3(grid), dim3(LTPB), 0, h->compute, cv.ptr, cv.idx, cv.val,
                           cv.nnz_base, cv.c0, cv.c1, h->cls, h->v, h->y, h->gdot);
    }
    if (ck.l1 > ck.l0) {
        const int64_t nseg = ck.n_items / 2;
        hipLaunchKernelGGL((k_dots_large_partial<KIND>), dim3((unsigned)nseg), dim3(LTPB), 0, h->compute, cv.ptr,
                           cv.idx, cv.val, cv.nnz_base, dense_len, h->large_list, h->large_seg_off, ck.l0, ck.l1,
                           h->seg, h->v, h->y, h->seg_partial);
        hipLaunchKernelGGL(k_dots_large_finish, dim3((unsigned)((ck.l1 - ck.l0 + 255) / 256)), dim3(256), 0,
                           h->compute, h->large_list, h->large_seg_off, ck.l0, ck.l1, h->seg_partial, h->gdot);
    }
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

static int coord_dots(snap_handle* h) {
    switch (h->kind) {
    case K_PRIMAL_RIDGE: return for_each_chunk(h, coord_dots_chunk<K_PRIMAL_RIDGE>, nullptr, true, false);
    case K_PRIMAL_LOGISTIC: return for_each_chunk(h, coord_dots_chunk<K_PRIMAL_LOGISTIC>, nullptr, true, false);
    default: return for_each_chunk(h, coord_dots_chunk<K_DUAL>, nullptr, true, false);
    }
}

// ---- transform-reduce in fp64, fixed order ----------------------------------------------------------
enum ReduceMode {
    R_LOSS_RIDGE = 0,    // a = v, b = y      : 0.5 (v-y)^2
    R_LOSS_LOGISTIC = 1, // a = v, b = y      : log(1+exp(-y v))
    R_SQNORM = 2,        // a = x             : x^2
    R_SUM = 3,           // a = x             : x
    R_GRADSQ = 4,        // d = gdot, a = x   : (gdot*s0 + s1*x)^2
    R_HINGE = 5,         // d = gdot, b = y   : max(0, 1 - y gdot s0)
    R_LOSS_LOGISTIC_F32 = 6, // as R_LOSS_LOGISTIC with fp32 transcendentals (accept check of the epoch)
    R_ABSSUM = 7,        // a = x             : |x|
    R_CONJ_RIDGE = 8,    // a = v, b = y      : n f*(u) at u = (v-y)/n        = (v-y) y + (v-y)^2/2
    R_CONJ_LOGISTIC = 9, // a = v, b = y      : n f*(u) at u = -y p/n         = p ln p + (1-p) ln(1-p), p = sigmoid(-y v)
    R_CONJ_REG = 10,     // d = gdot          : max(|gdot s0| - s1, 0)^2      (2 lambda g*(a_j.u))
    R_LOGISTIC_MARGIN = 11, // d = gdot, b = y   : log(1 + exp(-y gdot s0))      (dual form: margins from the row dots)
    R_ENTROPY = 12       // a = alpha         : a ln a + (1-a) ln(1-a)        (0 ln 0 := 0)
};

struct ReduceArgs {
    const float* a;
    const float* b;
    const double* d;
    double s0, s1;
    int64_t count;
};

template <int MODE>
__device__ __forceinline__ double reduce_term(const ReduceArgs& r, int64_t i) {
    if (MODE == R_LOSS_RIDGE) {
        const double t = (double)r.a[i] - (double)r.b[i];
        return 0.5 * t * t;
    }
    if (MODE == R_LOSS_LOGISTIC) {
        const double t = -(double)r.b[i] * (double)r.a[i];
        return t > 0 ? t + log1p(exp(-t)) : log1p(exp(t));
    }
    if (MODE == R_LOSS_LOGISTIC_F32) return (double)logistic_loss_f32(-r.b[i] * r.a[i]);
    if (MODE == R_SQNORM) return (double)r.a[i] * (double)r.a[i];
    if (MODE == R_SUM) return (double)r.a[i];
    if (MODE == R_ABSSUM) return fabs((double)r.a[i]);
    if (MODE == R_CONJ_RIDGE) {
        const double t = (double)r.a[i] - (double)r.b[i];
        return t * (double)r.b[i] + 0.5 * t * t;
    }
    if (MODE == R_CONJ_LOGISTIC) {
        // ln p = -log(1+exp(t)), ln(1-p) = -log(1+exp(-t)), t = y v
        const double t = (double)r.b[i] * (double)r.a[i];
        const double lp = t > 0 ? t + log1p(exp(-t)) : log1p(exp(t));
        const double lq = t > 0 ? log1p(exp(-t)) : -t + log1p(exp(t));
        const double p = exp(-lp);
        return -(p * lp + (1.0 - p) * lq);
    }
    if (MODE == R_LOGISTIC_MARGIN) {
        const double t = -(double)r.b[i] * r.d[i] * r.s0;
        return t > 0 ? t + log1p(exp(-t)) : log1p(exp(t));
    }
    if (MODE == R_ENTROPY) {
        const double a = (double)r.a[i], b = 1.0 - a;
        return (a > 0.0 ? a * log(a) : 0.0) + (b > 0.0 ? b * log(b) : 0.0);
    }
    if (MODE == R_CONJ_REG) {
        const double t = fabs(r.d[i] * r.s0) - r.s1;
        return t > 0 ? t * t : 0.0;
    }
    if (MODE == R_GRADSQ) {
        const double t = r.d[i] * r.s0 + r.s1 * (double)r.a[i];
        return t * t;
    }
    const double t = 1.0 - (double)r.b[i] * r.d[i] * r.s0;
    return t > 0 ? t : 0.0;
}

template <int MODE>
__global__ void __launch_bounds__(LTPB) k_reduce_partial(ReduceArgs r, double* __restrict__ partial) {
    __shared__ double scratch[LTPB / WAVE];
    // contiguous slice per workgroup, strided inside it: the order of the additions is fixed
    const int64_t per = (r.count + gridDim.x - 1) / gridDim.x;
    const int64_t lo = min(r.count, (int64_t)blockIdx.x * per), hi = min(r.count, lo + per);
    double acc = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += LTPB) acc += reduce_term<MODE>(r, i);
    acc = block_sum_d(acc, scratch);
    if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

__global__ void __launch_bounds__(LTPB) k_reduce_final(const double* __restrict__ partial, int count,
                                                        double* __restrict__ out) {
    __shared__ double scratch[LTPB / WAVE];
    double acc = 0.0;
    for (int i = threadIdx.x; i < count; i += LTPB) acc += partial[i];
    acc = block_sum_d(acc, scratch);
    if (threadIdx.x == 0) *out = acc;
}

static int reduce_to(snap_handle* h, int mode, const ReduceArgs& r, int slot) {
    double* partial = h->red.partial;
    double* out = h->red.result + slot;
    const dim3 g(REDUCE_BLOCKS), b(LTPB);
    switch (mode) {
    case R_LOSS_RIDGE: hipLaunchKernelGGL((k_reduce_partial<R_LOSS_RIDGE>), g, b, 0, h->compute, r, partial); break;
    case R_LOSS_LOGISTIC: hipLaunchKernelGGL((k_reduce_partial<R_LOSS_LOGISTIC>), g, b, 0, h->compute, r, partial); break;
    case R_SQNORM: hipLaunchKernelGGL((k_reduce_partial<R_SQNORM>), g, b, 0, h->compute, r, partial); break;
    case R_SUM: hipLaunchKernelGGL((k_reduce_partial<R_SUM>), g, b, 0, h->compute, r, partial); break;
    case R_GRADSQ: hipLaunchKernelGGL((k_reduce_partial<R_GRADSQ>), g, b, 0, h->compute, r, partial); break;
    case R_LOSS_LOGISTIC_F32:
        hipLaunchKernelGGL((k_reduce_partial<R_LOSS_LOGISTIC_F32>), g, b, 0, h->compute, r, partial);
        break;
    case R_ABSSUM: hipLaunchKernelGGL((k_reduce_partial<R_ABSSUM>), g, b, 0, h->compute, r, partial); break;
    case R_CONJ_RIDGE: hipLaunchKernelGGL((k_reduce_partial<R_CONJ_RIDGE>), g, b, 0, h->compute, r, partial); break;
    case R_CONJ_LOGISTIC:
        hipLaunchKernelGGL((k_reduce_partial<R_CONJ_LOGISTIC>), g, b, 0, h->compute, r, partial);
        break;
    case R_CONJ_REG: hipLaunchKernelGGL((k_reduce_partial<R_CONJ_REG>), g, b, 0, h->compute, r, partial); break;
    case R_LOGISTIC_MARGIN:
        hipLaunchKernelGGL((k_reduce_partial<R_LOGISTIC_MARGIN>), g, b, 0, h->compute, r, partial);
        break;
    case R_ENTROPY: hipLaunchKernelGGL((k_reduce_partial<R_ENTROPY>), g, b, 0, h->compute, r, partial); break;
    default: hipLaunchKernelGGL((k_reduce_partial<R_HINGE>), g, b, 0, h->compute, r, partial); break;
    }
    hipLaunchKernelGGL(k_reduce_final, dim3(1), b, 0, h->compute, partial, REDUCE_BLOCKS, out);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// The eight result slots go to the host through mapped pinned memory, written by a kernel: a copy
// command, however small, can queue behind gigabytes of chunk copies on the copy engines.
__global__ void k_publish(const double* __restrict__ result, double* __restrict__ host_mapped, int count) {
    if ((int)threadIdx.x < count) host_mapped[threadIdx.x] = result[threadIdx.x];
}

static int fetch_results(snap_handle* h, int count) {
    hipLaunchKernelGGL(k_publish, dim3(1), dim3(WAVE), 0, h->compute, h->red.result, h->red.host_mapped, count);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipStreamSynchronize(h->compute));
    return SNAP_OK;
}

int reducer_alloc(Reducer& r) {
    SNAP_HIP(hipMalloc(&r.partial, 2 * REDUCE_BLOCKS * sizeof(double)));
    SNAP_HIP(hipMalloc(&r.result, 8 * sizeof(double)));
    SNAP_HIP(hipHostMalloc(&r.host, 8 * sizeof(double), hipHostMallocMapped));
    SNAP_HIP(hipHostGetDevicePointer((void**)&r.host_mapped, r.host, 0));
    return SNAP_OK;
}

void reducer_free(Reducer& r) {
    (void)hipFree(r.partial);
    (void)hipFree(r.result);
    (void)hipHostFree(r.host);
    r = Reducer{};
}

__global__ void k_scale(const float* __restrict__ in, float s, float* __restrict__ out, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        out[i] = in[i] * s;
}

// P, D and the gap.  Any of the outputs may be null; the gap (and D in primal form) needs one pass
// over the matrix, P in primal form only the vectors.
// Inner products of every coordinate with loss'(v): by the row passes of the group sweeps when the
// handle has them.  Ridge terms beyond the range of those passes' fixed-point sums make the handle leave
// the group sweeps, and the inner products are taken column by column instead.
static int gradient_dots(snap_handle* h) {
    if (!h->grouped) return coord_dots(h);
    SNAP_TRY(grouped_dots(h));
    if (h->kind != K_PRIMAL_RIDGE) return SNAP_OK;
    uint32_t st = 0;
    SNAP_TRY(read_status(h, &st));
    if (!(st & STATUS_RANGE)) return SNAP_OK;
    SNAP_TRY(leave_group_sweeps(h));
    return coord_dots(h);
}

int objective(snap_handle* h, double* primal, double* dual, double* gap) {
    const double n = (double)h->n, lam = h->lambda, lam1 = h->lambda1;
    double* res = h->red.host;
    if (h->form == SNAP_PRIMAL) {
        const bool need_gap = gap != nullptr || dual != nullptr;
        ReduceArgs r{h->v, h->y, nullptr, 0.0, 0.0, h->n};
        SNAP_TRY(reduce_to(h, h->loss == SNAP_RIDGE ? R_LOSS_RIDGE : R_LOSS_LOGISTIC, r, 0));
        ReduceArgs rx{h->x, nullptr, nullptr, 0.0, 0.0, h->m};
        SNAP_TRY(reduce_to(h, R_SQNORM, rx, 1));
        if (lam1 > 0.0) SNAP_TRY(reduce_to(h, R_ABSSUM, rx, 3));
        if (need_gap) {
            SNAP_TRY(gradient_dots(h));
            if (lam1 > 0.0) {
                // Fenchel form: P + f*(u) + sum_j g*(a_j.u), u = grad f(v); a_j.u = gdot_j / n
                ReduceArgs rg{nullptr, nullptr, h->gdot, 1.0 / n, lam1, h->m};
                SNAP_TRY(reduce_to(h, R_CONJ_REG, rg, 2));
                SNAP_TRY(reduce_to(h, h->loss == SNAP_RIDGE ? R_CONJ_RIDGE : R_CONJ_LOGISTIC, r, 4));
            } else {
                ReduceArgs rg{h->x, nullptr, h->gdot, 1.0 / n, lam, h->m};
                SNAP_TRY(reduce_to(h, R_GRADSQ, rg, 2));
            }
        }
        SNAP_TRY(fetch_results(h, 8));
        const double P = res[0] / n + 0.5 * lam * res[1] + (lam1 > 0.0 ? lam1 * res[3] : 0.0);
        double G = 0.0;
        if (need_gap) G = lam1 > 0.0 ? P + res[4] / n + res[2] / (2.0 * lam) : res[2] / (2.0 * lam);
        if (primal) *primal = P;
        if (gap) *gap = G;
        if (dual) *dual = P - G;
        return SNAP_OK;
    }
    // dual form: w = v/(lambda n); margins y_i x_i.w from the row dots with v;
    // D = (1/n) sum alpha - (lambda/2)||w||^2 (hinge), -(1/n) sum entropy terms - (lambda/2)||w||^2 (logistic)
    const bool logistic = h->loss == SNAP_LOGISTIC;
    SNAP_TRY(coord_dots(h));
    ReduceArgs rh{nullptr, h->y, h->gdot, 1.0 / (lam * n), 0.0, h->m};
    SNAP_TRY(reduce_to(h, logistic ? R_LOGISTIC_MARGIN : R_HINGE, rh, 0));
    ReduceArgs ra{h->x, nullptr, nullptr, 0.0, 0.0, h->m};
    SNAP_TRY(reduce_to(h, logistic ? R_ENTROPY : R_SUM, ra, 1));
    ReduceArgs rv{h->v, nullptr, nullptr, 0.0, 0.0, h->vlen};
    SNAP_TRY(reduce_to(h, R_SQNORM, rv, 2));
    SNAP_TRY(fetch_results(h, 8));
    const double ww = res[2] / (lam * n * lam * n);
    const double P = res[0] / n + 0.5 * lam * ww;
    const double D = (logistic ? -res[1] : res[1]) / n - 0.5 * lam * ww;
    if (primal) *primal = P;
    if (dual) *dual = D;
    if (gap) *gap = P - D;
    return SNAP_OK;
}

// Share of every chunk (or group) of coordinates in the duality gap, primal forms (Section 3.2: the
// importance measure for choosing what to process).  With u = grad f(v) the loss part of the Fenchel
// gap vanishes and the rest is a sum over the coordinates of
//     g(w_j) + g*(-z_j) + w_j z_j,   z_j = a_j . u,   g(w) = (lambda/2) w^2 + lambda1 |w|,
// which for lambda1 = 0 is (z_j + lambda w_j)^2 / (2 lambda).  Dual forms (MODE 1 hinge, 2 logistic):
// with w = v / (lambda n) the regulariser's part lambda ||w||^2 is (1/n) sum_i alpha_i m_i,
// m_i = y_i x_i . w, and the gap is the sum over the examples of
//     (1/n) [ l(m_i) + l*(-alpha_i) + alpha_i m_i ],
// l*(-a) = -a (hinge), a ln a + (1 - a) ln(1 - a) (logistic); inv_n then carries 1 / (lambda n).
// One workgroup per chunk, fixed order.
template <int MODE>
__global__ void __launch_bounds__(LTPB)
k_chunk_shares(const double* __restrict__ gdot, const float* __restrict__ x, const float* __restrict__ y,
               const int64_t* __restrict__ bounds, double inv_n, double lam, double lam1, double* __restrict__ out) {
    __shared__ double scratch[LTPB / WAVE];
    const int64_t c0 = bounds[blockIdx.x], c1 = bounds[blockIdx.x + 1];
    double acc = 0.0;
    for (int64_t j = c0 + threadIdx.x; j < c1; j += LTPB) {
        const double z = gdot[j] * inv_n, w = (double)x[j];
        if (MODE != 0) {
            const double mi = (double)y[j] * z;   // margin; w holds alpha_i
            double t;
            if (MODE == 1) t = fmax(0.0, 1.0 - mi) - w;
            else
                t = fmax(-mi, 0.0) + log1p(exp(-fabs(mi))) + (w > 0.0 ? w * log(w) : 0.0) +
                    (w < 1.0 ? (1.0 - w) * log1p(-w) : 0.0);
            acc += t + w * mi;
        } else if (lam1 == 0.0) {
            const double t = z + lam * w;
            acc += t * t / (2.0 * lam);
        } else {
            const double t = fmax(fabs(z) - lam1, 0.0);
            acc += 0.5 * lam * w * w + lam1 * fabs(w) + t * t / (2.0 * lam) + w * z;
        }
    }
    acc = block_sum_d(acc, scratch);
    if (MODE != 0) acc *= lam * inv_n;   // = 1/n
    if (threadIdx.x == 0) out[blockIdx.x] = acc;
}

int chunk_gap_shares(snap_handle* h, double* shares_out) {
    const bool by_group = h->grouped || h->tiled;
    const int64_t C = by_group ? h->n_groups : h->n_chunks;
    if (C <= 0) return SNAP_OK;
    if (!h->share_bounds) {
        std::vector<int64_t> b((size_t)C + 1);
        for (int64_t c = 0; c < C; ++c) b[(size_t)c] = by_group ? h->gbounds_host[c] : h->chunks[c].c0;
        b[(size_t)C] = h->m;
        SNAP_HIP(hipMalloc(&h->share_bounds, ((size_t)C + 1) * sizeof(int64_t)));
        SNAP_HIP(hipMalloc(&h->share_out, (size_t)C * sizeof(double)));
        SNAP_HIP(hipMemcpy(h->share_bounds, b.data(), ((size_t)C + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    }
    SNAP_TRY(gradient_dots(h));
    const dim3 grid((unsigned)C), block(LTPB);
    const double n = (double)h->n;
    if (h->form == SNAP_PRIMAL)
        hipLaunchKernelGGL((k_chunk_shares<0>), grid, block, 0, h->compute, h->gdot, h->x, h->y, h->share_bounds,
                           1.0 / n, h->lambda, h->lambda1, h->share_out);
    else if (h->loss == SNAP_LOGISTIC)
        hipLaunchKernelGGL((k_chunk_shares<2>), grid, block, 0, h->compute, h->gdot, h->x, h->y, h->share_bounds,
                           1.0 / (h->lambda * n), h->lambda, 0.0, h->share_out);
    else
        hipLaunchKernelGGL((k_chunk_shares<1>), grid, block, 0, h->compute, h->gdot, h->x, h->y, h->share_bounds,
                           1.0 / (h->lambda * n), h->lambda, 0.0, h->share_out);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipMemcpyAsync(shares_out, h->share_out, (size_t)C * sizeof(double), hipMemcpyDeviceToHost, h->compute));
    SNAP_HIP(hipStreamSynchronize(h->compute));
    return SNAP_OK;
}

int monitor_value(snap_handle* h, double* value) {
    const double n = (double)h->n, lam = h->lambda;
    double* res = h->red.host;
    if (h->form == SNAP_PRIMAL) {
        ReduceArgs r{h->v, h->y, nullptr, 0.0, 0.0, h->n};
        SNAP_TRY(reduce_to(h, h->loss == SNAP_RIDGE ? R_LOSS_RIDGE : R_LOSS_LOGISTIC_F32, r, 0));
        ReduceArgs rx{h->x, nullptr, nullptr, 0.0, 0.0, h->m};
        SNAP_TRY(reduce_to(h, R_SQNORM, rx, 1));
        if (h->lambda1 > 0.0) SNAP_TRY(reduce_to(h, R_ABSSUM, rx, 2));
    } else {
        ReduceArgs ra{h->x, nullptr, nullptr, 0.0, 0.0, h->m};
        SNAP_TRY(reduce_to(h, h->loss == SNAP_LOGISTIC ? R_ENTROPY : R_SUM, ra, 0));
        ReduceArgs rv{h->v, nullptr, nullptr, 0.0, 0.0, h->vlen};
        SNAP_TRY(reduce_to(h, R_SQNORM, rv, 1));
    }
    SNAP_TRY(fetch_results(h, 8));
    if (h->form == SNAP_PRIMAL) *value = res[0] / n + 0.5 * lam * res[1] + (h->lambda1 > 0.0 ? h->lambda1 * res[2] : 0.0);
    else *value = -((h->loss == SNAP_LOGISTIC ? -res[0] : res[0]) / n - 0.5 * res[1] / (lam * n * n));   // -D(alpha)
    return SNAP_OK;
}

// ---- effective length of v ------------------------------------------------------------------------
__global__ void k_count_accesses(const uint32_t* __restrict__ idx, int64_t count, uint32_t* __restrict__ freq) {
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < count; k += (int64_t)gridDim.x * blockDim.x)
        atomicAdd(freq + (idx[k] & ~LABEL_BIT), 1u);
}

__global__ void __launch_bounds__(LTPB)
k_freq_moments(const uint32_t* __restrict__ freq, int64_t count, double* __restrict__ partial) {
    __shared__ double scratch[LTPB / WAVE];
    const int64_t per = (count + gridDim.x - 1) / gridDim.x;
    const int64_t lo = min(count, (int64_t)blockIdx.x * per), hi = min(count, lo + per);
    double s1 = 0.0, s2 = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += LTPB) {
        const double f = (double)freq[i];
        s1 += f;
        s2 += f * f;
    }
    s1 = block_sum_d(s1, scratch);
    s2 = block_sum_d(s2, scratch);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = s1;
        partial[REDUCE_BLOCKS + blockIdx.x] = s2;
    }
}

int count_accesses_chunk(snap_handle* h, const ChunkView& cv, int64_t count, uint32_t* freq) {
    if (count > 0) hipLaunchKernelGGL(k_count_accesses, dim3(8192), dim3(256), 0, h->compute, cv.idx, count, freq);
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// How many entries of v the accesses are effectively spread over: (sum f)^2 / sum f^2 with f the
// number of nonzeros that touch each entry.  Uniform access gives the length of v; a few hot
// entries (popular columns in the dual form) give a much smaller number.
int access_moments(snap_handle* h, const uint32_t* freq, double* eff_len) {
    hipLaunchKernelGGL(k_freq_moments, dim3(REDUCE_BLOCKS), dim3(LTPB), 0, h->compute, freq, h->vlen, h->red.partial);
    hipLaunchKernelGGL(k_reduce_final, dim3(1), dim3(LTPB), 0, h->compute, h->red.partial, REDUCE_BLOCKS, h->red.result);
    hipLaunchKernelGGL(k_reduce_final, dim3(1), dim3(LTPB), 0, h->compute, h->red.partial + REDUCE_BLOCKS,
                       REDUCE_BLOCKS, h->red.result + 1);
    SNAP_TRY(fetch_results(h, 2));
    const double s1 = h->red.host[0], s2 = h->red.host[1];
    *eff_len = s2 > 0.0 ? s1 * s1 / s2 : (double)h->vlen;
    return SNAP_OK;
}

// ---- decision values -------------------------------------------------------------------------------
// L lanes per row (8 ... 64, chosen from the average row length): with the 39 entries of a click-log
// row a whole wavefront per row leaves a third of the lanes idle for one round of loads per row.
template <int L>
__global__ void __launch_bounds__(LTPB)
k_csr_rowdot(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx, const float* __restrict__ val,
             int64_t rows, const float* __restrict__ w, float* __restrict__ out) {
    const int sub = threadIdx.x & (L - 1);
    const int64_t g0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / L;
    const int64_t groups = (int64_t)gridDim.x * blockDim.x / L;
    for (int64_t i = g0; i < rows; i += groups) {
        double acc = 0.0;
        const int64_t s1 = ptr[i + 1];
        for (int64_t k = ptr[i] + sub; k < s1; k += L) acc += (double)val[k] * (double)w[idx[k]];
#pragma unroll
        for (int off = L / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, L);   // the row's L lanes are all here
        if (sub == 0) out[i] = (float)acc;
    }
}

// dense: out[i] = sum_j X(i,j) w[j]; element (i,j) at X[i*rs + j*cs]
__global__ void __launch_bounds__(LTPB)
k_dense_rowdot(const float* __restrict__ X, int64_t rows, int64_t cols, int64_t rs, int64_t cs,
               const float* __restrict__ w, float* __restrict__ out) {
    if (cs == 1) {      // row-major: one wavefront per row
        const int lane = threadIdx.x & (WAVE - 1);
        const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
        const int64_t nwaves = (int64_t)gridDim.x * blockDim.x / WAVE;
        for (int64_t i = wave0; i < rows; i += nwaves) {
            double acc = 0.0;
            for (int64_t j = lane; j < cols; j += WAVE) acc += (double)X[i * rs + j] * (double)w[j];
            acc = wave_sum_d(acc);
            if (lane == 0) out[i] = (float)acc;
        }
    } else {            // column-major: one thread per row, coalesced over rows
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < rows;
             i += (int64_t)gridDim.x * blockDim.x) {
            double acc = 0.0;
            for (int64_t j = 0; j < cols; ++j) acc += (double)X[i + j * cs] * (double)w[j];
            out[i] = (float)acc;
        }
    }
}

static int model_weights(snap_handle* h, const float** w) {
    if (h->form == SNAP_PRIMAL) {
        *w = h->x;
        return SNAP_OK;
    }
    int grid = (int)((h->d + 255) / 256 < 4096 ? (h->d + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_scale, dim3(grid), dim3(256), 0, h->compute, h->v, (float)(1.0 / (h->lambda * (double)h->n)),
                       h->w_tmp, h->d);
    SNAP_HIP(hipGetLastError());
    *w = h->w_tmp;
    return SNAP_OK;
}

int weights_to_host(snap_handle* h, float* w_out) {
    const float* w;
    SNAP_TRY(model_weights(h, &w));
    SNAP_HIP(hipMemcpyAsync(w_out, w, (size_t)h->d * sizeof(float), hipMemcpyDeviceToHost, h->compute));
    SNAP_HIP(hipStreamSynchronize(h->compute));
    return SNAP_OK;
}

// Compressed input of snap_predict: ptr[0] = 0, ptr non-decreasing, ptr[major] = nnz, 0 <= idx < minor.
// The row kernels follow ptr and idx without further checks, so a violation is reported here.
__global__ void k_check_compressed(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx, int64_t major,
                                   int64_t minor, int64_t nnz, uint32_t* flag) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    for (int64_t i = first; i <= major; i += stride) {
        const int64_t a = ptr[i];
        if (a < 0 || a > nnz || (i == 0 && a != 0) || (i == major && a != nnz) || (i < major && ptr[i + 1] < a)) bad = true;
    }
    for (int64_t k = first; k < nnz; k += stride)
        if (idx[k] < 0 || (int64_t)idx[k] >= minor) bad = true;
    if (bad) atomicOr(flag, 1u);
}

// the flag of k_check_compressed reaches the host through mapped pinned memory, like the status word
__global__ void k_publish_flag(const uint32_t* __restrict__ flag, double* __restrict__ host_mapped) {
    if (threadIdx.x == 0) reinterpret_cast<uint32_t*>(host_mapped)[0] = *flag;
}

// Checks ptr / idx of a compressed matrix in device memory; `flag` is one device word (cleared here).
static int check_compressed(snap_handle* h, int layout, const int64_t* dptr, const int32_t* didx, int64_t rows,
                            int64_t cols, int64_t count, uint32_t* flag) {
    const int64_t major = layout == SNAP_CSR ? rows : cols, minor = layout == SNAP_CSR ? cols : rows;
    const int64_t work = std::max<int64_t>(major + 1, count);
    SNAP_TRY(fill_zero(flag, sizeof(uint32_t), h->compute));
    hipLaunchKernelGGL(k_check_compressed, dim3((unsigned)std::min<int64_t>((work + 255) / 256, 16384)), dim3(256), 0,
                       h->compute, dptr, didx, major, minor, count, flag);
    hipLaunchKernelGGL(k_publish_flag, dim3(1), dim3(WAVE), 0, h->compute, flag, h->red.host_mapped + 6);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipStreamSynchronize(h->compute));
    if (reinterpret_cast<const uint32_t*>(h->red.host + 6)[0] != 0) {
        set_error("snap_predict: ptr must start at 0, not decrease and end at nnz; idx must lie in [0, %lld)",
                  (long long)minor);
        return SNAP_EINVAL;
    }
    return SNAP_OK;
}

// The row kernels for a matrix in device memory; acc: rows fp64 sums (CSC only, cleared here).
static int launch_rowdots(snap_handle* h, int layout, const int64_t* dptr, const int32_t* didx, const float* dval,
                          int64_t rows, int64_t cols, int64_t count, const float* w, float* dout, double* acc) {
    if (rows <= 0) return SNAP_OK;
    const int grid = (int)((rows + 3) / 4 < 32768 ? (rows + 3) / 4 : 32768);
    if (layout == SNAP_CSR) {
        const int64_t avg = count / rows;
        const int L = avg > 128 ? 64 : (avg > 64 ? 32 : (avg > 32 ? 16 : 8));   // about four to eight rounds per row
        const int64_t wgs = (rows + LTPB / L - 1) / (LTPB / L);
        const dim3 g((unsigned)std::min<int64_t>(wgs, 65536));
        if (L == 64) hipLaunchKernelGGL((k_csr_rowdot<64>), g, dim3(LTPB), 0, h->compute, dptr, didx, dval, rows, w, dout);
        else if (L == 32) hipLaunchKernelGGL((k_csr_rowdot<32>), g, dim3(LTPB), 0, h->compute, dptr, didx, dval, rows, w, dout);
        else if (L == 16) hipLaunchKernelGGL((k_csr_rowdot<16>), g, dim3(LTPB), 0, h->compute, dptr, didx, dval, rows, w, dout);
        else hipLaunchKernelGGL((k_csr_rowdot<8>), g, dim3(LTPB), 0, h->compute, dptr, didx, dval, rows, w, dout);
    } else if (layout == SNAP_CSC) {
        // column by column into fp64 sums (atomics), rounded once: the result does not depend on the
        // order of the additions beyond the last bit of the fp64 sum
        SNAP_TRY(fill_zero(acc, (size_t)rows * sizeof(double), h->compute));
        if (count > 0) {
            const int64_t nb = (count + AXPY_BLOCK - 1) / AXPY_BLOCK;
            hipLaunchKernelGGL((k_scatter_axpy<double>), dim3((unsigned)nb), dim3(LTPB), 0, h->compute, dptr,
                               (const uint32_t*)didx, dval, (int64_t)0, (int64_t)0, cols, (int64_t)0, count, w,
                               (const float*)nullptr, 0xFFFFFFFFu, acc);
        }
        const int64_t blocks = (rows + 255) / 256;
        hipLaunchKernelGGL(k_round_to_float, dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, h->compute,
                           acc, dout, rows);
    } else if (layout == SNAP_DENSE_ROWMAJOR) {
        hipLaunchKernelGGL(k_dense_rowdot, dim3(grid), dim3(LTPB), 0, h->compute, dval, rows, cols, cols, (int64_t)1, w, dout);
    } else {
        hipLaunchKernelGGL(k_dense_rowdot, dim3(grid), dim3(LTPB), 0, h->compute, dval, rows, cols, (int64_t)1, rows, w, dout);
    }
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

int predict(snap_handle* h, const snap_matrix* X, float* out) {
    const float* w;
    SNAP_TRY(model_weights(h, &w));
    const bool on_dev = X->mem == SNAP_MEM_DEVICE;
    const int64_t rows = X->n_rows, cols = X->n_cols;
    int64_t* dptr = nullptr;
    int32_t* didx = nullptr;
    float* dval = nullptr;
    float* dout = nullptr;
    uint32_t* flag = nullptr;
    double* acc = nullptr;
    int rc = SNAP_OK;
    const bool sparse = X->layout == SNAP_CSR || X->layout == SNAP_CSC;
    const int64_t major = X->layout == SNAP_CSR ? rows : cols;
    const int64_t count = sparse ? X->nnz : rows * cols;
    auto cleanup = [&]() {
        (void)hipFree(flag);
        (void)hipFree(acc);
        if (!on_dev) {
            (void)hipFree(dptr);
            (void)hipFree(didx);
            (void)hipFree(dval);
            (void)hipFree(dout);
        }
    };
#define PRED_HIP(call)                                              \
    do {                                                            \
        hipError_t e_ = (call);                                     \
        if (e_ != hipSuccess) {                                     \
            rc = hip_fail(e_, #call, __FILE__, __LINE__);           \
            cleanup();                                              \
            return rc;                                              \
        }                                                           \
    } while (0)
    if (on_dev) {
        dptr = const_cast<int64_t*>(X->ptr);
        didx = const_cast<int32_t*>(X->idx);
        dval = const_cast<float*>(X->val);
        dout = out;
    } else {
        if (sparse) {
            PRED_HIP(hipMalloc(&dptr, (size_t)(major + 1) * sizeof(int64_t)));
            PRED_HIP(hipMalloc(&didx, (size_t)(count ? count : 1) * sizeof(int32_t)));
            PRED_HIP(hipMemcpyAsync(dptr, X->ptr, (size_t)(major + 1) * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
            PRED_HIP(hipMemcpyAsync(didx, X->idx, (size_t)count * sizeof(int32_t), hipMemcpyHostToDevice, h->compute));
        }
        PRED_HIP(hipMalloc(&dval, (size_t)(count ? count : 1) * sizeof(float)));
        PRED_HIP(hipMemcpyAsync(dval, X->val, (size_t)count * sizeof(float), hipMemcpyHostToDevice, h->compute));
        PRED_HIP(hipMalloc(&dout, (size_t)(rows ? rows : 1) * sizeof(float)));
    }
    if (sparse) {
        PRED_HIP(hipMalloc(&flag, sizeof(uint32_t)));
        rc = check_compressed(h, X->layout, dptr, didx, rows, cols, count, flag);
        if (rc != SNAP_OK) {
            cleanup();
            return rc;
        }
    }
    if (X->layout == SNAP_CSC && rows > 0) PRED_HIP(hipMalloc(&acc, (size_t)rows * sizeof(double)));
    rc = launch_rowdots(h, X->layout, dptr, didx, dval, rows, cols, count, w, dout, acc);
    if (rc != SNAP_OK) {
        cleanup();
        return rc;
    }
    if (!on_dev) PRED_HIP(hipMemcpyAsync(out, dout, (size_t)rows * sizeof(float), hipMemcpyDeviceToHost, h->compute));
    PRED_HIP(hipStreamSynchronize(h->compute));
    cleanup();
#undef PRED_HIP
    return rc;
}

// ---- decision values for callers that cannot allocate -----------------------------------------------
// snap_predict allocates what it needs per call (the flag of the input check, the fp64 sums of a
// compressed-column matrix).  This variant keeps both in a file-scope device array instead: one
// copy per GPU, held until the process ends, shared by every call on that GPU (calls that overlap
// on one GPU would race on it).  Layout: [0, 256): the flag word; then STATIC_ROWS_MAX fp64 sums.
constexpr int64_t STATIC_ROWS_MAX = (int64_t)4 << 20;      // rows of a compressed-column matrix: 32 MiB of sums
constexpr size_t STATIC_HEAD = 256;
static __device__ __align__(256) unsigned char scratch[STATIC_HEAD + (size_t)STATIC_ROWS_MAX * sizeof(double)];

// The array's address on the current device (each GPU holds its own copy at its own address), looked
// up once per device.  The array's name is only a handle for this lookup in host code.
static int static_scratch(int device, unsigned char** out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex lock;
    static unsigned char* ptrs[MAX_DEVICES] = {};
    if (device < 0 || device >= MAX_DEVICES) {
        set_error("device index %d out of range", device);
        return SNAP_EINVAL;
    }
    std::lock_guard<std::mutex> guard(lock);
    if (!ptrs[device]) {
        void* p = nullptr;
        SNAP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) {
            set_error("the address of the static scratch array is null");
            return SNAP_EHIP;
        }
        ptrs[device] = static_cast<unsigned char*>(p);
    }
    *out = ptrs[device];
    return SNAP_OK;
}

int predict_static(snap_handle* h, const snap_matrix* X, float* out) {
    int device = -1;
    SNAP_HIP(hipGetDevice(&device));
    if (device != h->device) {
        set_error("snap_predict_static: the handle's device (%d) must be the current one (%d)", h->device, device);
        return SNAP_EINVAL;
    }
    if (X->mem != SNAP_MEM_DEVICE) {
        set_error("snap_predict_static: the matrix and the output must be in device memory (a host matrix would need a "
                  "device copy, which this call may not allocate)");
        return SNAP_EINVAL;
    }
    const int64_t rows = X->n_rows, cols = X->n_cols;
    const bool sparse = X->layout == SNAP_CSR || X->layout == SNAP_CSC;
    const int64_t count = sparse ? X->nnz : rows * cols;
    if (X->layout == SNAP_CSC && rows > STATIC_ROWS_MAX) {
        set_error("snap_predict_static: a compressed-column matrix may have at most %lld rows (the static buffer of fp64 "
                  "sums); use snap_predict or the row layouts", (long long)STATIC_ROWS_MAX);
        return SNAP_EINVAL;
    }
    unsigned char* base = nullptr;
    SNAP_TRY(static_scratch(device, &base));
    const float* w;
    SNAP_TRY(model_weights(h, &w));
    if (sparse) SNAP_TRY(check_compressed(h, X->layout, X->ptr, X->idx, rows, cols, count, reinterpret_cast<uint32_t*>(base)));
    SNAP_TRY(launch_rowdots(h, X->layout, X->ptr, X->idx, X->val, rows, cols, count, w, out,
                            reinterpret_cast<double*>(base + STATIC_HEAD)));
    SNAP_HIP(hipStreamSynchronize(h->compute));
    return SNAP_OK;
}

}  // namespace snap
