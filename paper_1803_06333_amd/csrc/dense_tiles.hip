// Exact tile sweeps for dense ridge regression (Section 3.1, dense data): the coordinates are cut
// into tiles of TILE_B consecutive columns.  For the quadratic loss the inner product that the step
// of coordinate b needs, a_b.(v - y), changes by  mult_a * (a_a.a_b)  when coordinate a of the same
// tile is updated first, so with the tile's TILE_B x TILE_B Gram block (constant, computed once at
// creation) the whole tile can be updated from ONE set of inner products taken at the tile's start:
// the result is that of visiting its coordinates one after the other, without any write to v in
// between.  An epoch is then a chain of fused passes over row blocks of the matrix,
//     v += A_prev * mult_prev   (plain stores: every workgroup owns its rows, no atomics)
//     partial sums of  A_cur^T (v - y)  for the next tile,
// with a one-workgroup kernel between two passes that finishes the sums and takes the TILE_B steps
// in the seeded order.  Tiles are visited in a seeded random order, the coordinates of a tile in the
// order of their keys under the tile's chunk id (the chunked permutation of Section 3.2).
#include <hip/hip_ext.h>
#include "common.h"
#include "perm_key.h"
#include "scd_device.h"
#include <type_traits>

#include <algorithm>
#include <cstdlib>
#include <new>
#include <vector>

namespace snap {

constexpr int TILE_B = 128;           // columns per tile
constexpr int CPL = TILE_B / WAVE;    // columns per lane of the wavefront that takes the steps
constexpr int PASS_TPB = 256;
constexpr int GRAM_ROWS = 8192;       // rows per workgroup of the Gram kernel

// ---- Gram blocks ------------------------------------------------------------------------------------
// gram64[t][a][b] += sum over the workgroup's rows of A[i, c0+a] * A[i, c0+b]; 256 threads, each a
// square block of the TILE_B x TILE_B outputs; fp32 inside the row slice, fp64 across slices.
__global__ void __launch_bounds__(256)
k_tile_gram(const float* __restrict__ A, int64_t ld, int64_t n, int64_t d, double* __restrict__ gram64) {
    constexpr int KB = 32, TT = TILE_B / 16;
    __shared__ float As[KB][TILE_B + 4];
    const int64_t c0 = (int64_t)blockIdx.x * TILE_B;
    const int nb = (int)min((int64_t)TILE_B, d - c0);
    const int64_t r0 = (int64_t)blockIdx.y * GRAM_ROWS, r1 = min(n, r0 + GRAM_ROWS);
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
    float acc[TT][TT] = {};
    for (int64_t k0 = r0; k0 < r1; k0 += KB) {
        // column c = e / KB, row k = e % KB: consecutive threads read consecutive rows of a column
        for (int e = threadIdx.x; e < KB * TILE_B; e += 256) {
            const int c = e / KB, k = e % KB;
            const int64_t r = k0 + k;
            As[k][c] = (c < nb && r < r1) ? A[(c0 + c) * ld + r] : 0.0f;
        }
        __syncthreads();
#pragma unroll 4
        for (int k = 0; k < KB; ++k) {
            float a[TT], b[TT];
#pragma unroll
            for (int i = 0; i < TT; ++i) {
                a[i] = As[k][ty * TT + i];
                b[i] = As[k][tx * TT + i];
            }
#pragma unroll
            for (int i = 0; i < TT; ++i)
#pragma unroll
                for (int j = 0; j < TT; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
    double* out = gram64 + (size_t)blockIdx.x * TILE_B * TILE_B;
#pragma unroll
    for (int i = 0; i < TT; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j) atomicAdd(out + (ty * TT + i) * TILE_B + tx * TT + j, (double)acc[i][j]);
}

__global__ void k_narrow_f64(const double* __restrict__ in, float* __restrict__ out, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        out[i] = (float)in[i];
}

// ---- the fused row pass -----------------------------------------------------------------------------
// Workgroup w owns rows [w * PASS_ROWS, ...): adds the previous tile's steps to its rows of v and
// takes its share of the next tile's inner products.  n_prev or n_cur may be 0 (first / last pass).
template <bool ALIGNED, int PASS_VEC>
__device__ __forceinline__ void load_rows(const float* __restrict__ col, int64_t i0, int live, float (&a)[PASS_VEC]) {
    if (ALIGNED && PASS_VEC == 4 && live == PASS_VEC) {
        const float4 t = *reinterpret_cast<const float4*>(col + i0);
        a[0] = t.x; a[1] = t.y; a[2] = t.z; a[3] = t.w;
    } else if (ALIGNED && PASS_VEC == 2 && live == PASS_VEC) {
        const float2 t = *reinterpret_cast<const float2*>(col + i0);
        a[0] = t.x; a[1] = t.y;
    } else {
#pragma unroll
        for (int k = 0; k < PASS_VEC; ++k) a[k] = k < live ? col[i0 + k] : 0.0f;
    }
}

template <bool ALIGNED, int PASS_VEC>
__global__ void __launch_bounds__(PASS_TPB)
k_tile_pass(const float* __restrict__ A, int64_t ld, int64_t n, int64_t prev_c0, int n_prev,
            const float* __restrict__ mult_prev, int64_t cur_c0, int n_cur, float* __restrict__ v,
            const float* __restrict__ y, float* __restrict__ partial) {
    constexpr int PASS_ROWS = PASS_TPB * PASS_VEC, NQ = PASS_TPB / WAVE;
    __shared__ float mult_s[TILE_B];
    __shared__ __align__(16) float r_s[PASS_ROWS];
    if (threadIdx.x < TILE_B) mult_s[threadIdx.x] = threadIdx.x < n_prev ? mult_prev[threadIdx.x] : 0.0f;
    __syncthreads();
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int64_t row0 = (int64_t)blockIdx.x * PASS_ROWS;
    // write-back of the previous tile: thread t owns rows row0 + t * PASS_VEC ...
    {
        const int64_t i0 = row0 + (int64_t)threadIdx.x * PASS_VEC;
        const int live = (int)max((int64_t)0, min((int64_t)PASS_VEC, n - i0));
        float acc[PASS_VEC];
        load_rows<ALIGNED, PASS_VEC>(v, i0, live, acc);
        if (n_prev > 0) {
            const float* col = A + prev_c0 * ld;
#pragma unroll 16
            for (int j = 0; j < n_prev; ++j) {
                float a[PASS_VEC];
                load_rows<ALIGNED, PASS_VEC>(col + (int64_t)j * ld, i0, live, a);
                const float mj = mult_s[j];
#pragma unroll
                for (int k = 0; k < PASS_VEC; ++k) acc[k] += mj * a[k];
            }
            if (ALIGNED && PASS_VEC == 4 && live == PASS_VEC) {
                *reinterpret_cast<float4*>(v + i0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            } else if (ALIGNED && PASS_VEC == 2 && live == PASS_VEC) {
                *reinterpret_cast<float2*>(v + i0) = make_float2(acc[0], acc[1]);
            } else {
#pragma unroll
                for (int k = 0; k < PASS_VEC; ++k)
                    if (k < live) v[i0 + k] = acc[k];
            }
        }
        if (n_cur == 0) return;
        float yy[PASS_VEC];
        load_rows<ALIGNED, PASS_VEC>(y, i0, live, yy);
#pragma unroll
        for (int k = 0; k < PASS_VEC; ++k) r_s[threadIdx.x * PASS_VEC + k] = k < live ? acc[k] - yy[k] : 0.0f;
    }
    __syncthreads();
    // inner products of the next tile: wavefront w takes columns w, w + 4, ... over ALL rows of the
    // workgroup (one reduction per column and workgroup); the residuals stay in registers
    float r[NQ][PASS_VEC];
    int64_t iq[NQ];
    int liveq[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int off = (q * WAVE + lane) * PASS_VEC;
        iq[q] = row0 + off;
        liveq[q] = (int)max((int64_t)0, min((int64_t)PASS_VEC, n - iq[q]));
#pragma unroll
        for (int k = 0; k < PASS_VEC; ++k) r[q][k] = r_s[off + k];
    }
    const float* col = A + cur_c0 * ld;
#pragma unroll 4
    for (int jj = 0; jj < TILE_B / NQ; ++jj) {
        const int j = w + jj * NQ;
        float s = 0.0f;
        if (j < n_cur) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                float a[PASS_VEC];
                load_rows<ALIGNED, PASS_VEC>(col + (int64_t)j * ld, iq[q], liveq[q], a);
#pragma unroll
                for (int k = 0; k < PASS_VEC; ++k) s += a[k] * r[q][k];
            }
        }
        s = wave_sum(s);
        if (lane == 0) partial[(size_t)blockIdx.x * TILE_B + j] = s;
    }
}

// ---- the steps of one tile ---------------------------------------------------------------------------
// One workgroup: finishes the tile's inner products from the per-workgroup partial sums (fp64, fixed
// order), then wavefront 0 takes the steps one after the other in the order of the keys, lane b
// holding coordinate c0 + b and correcting its inner product with the Gram entries after each step.
constexpr int SOLVE_TPB = 1024;
constexpr int SOLVE_PARTS = SOLVE_TPB / (TILE_B / 4);   // workgroup rows of partial sums read side by side

__global__ void __launch_bounds__(SOLVE_TPB)
k_tile_solve(const float* __restrict__ partial, int n_wg, int64_t c0, int nb, uint32_t tile, uint64_t seed,
             const float* __restrict__ gram, float* __restrict__ x, const float* __restrict__ norms,
             float* __restrict__ mult_out, StepParams sp) {
    // one LDS area, used twice: the partial sums of the reduction, then the Gram block (read by rows:
    // it is symmetric, and row a is contiguous over the lanes)
    __shared__ __align__(16) float lds[TILE_B * TILE_B];
    static_assert(sizeof(double) * SOLVE_PARTS * TILE_B <= sizeof(float) * TILE_B * TILE_B, "reduction fits");
    double* gs = reinterpret_cast<double*>(lds);
    // the Gram block is requested first (into registers): it arrives while the partial sums are reduced
    constexpr int GL = TILE_B * TILE_B / 4 / SOLVE_TPB;
    float4 mreg[GL];
#pragma unroll
    for (int i = 0; i < GL; ++i) mreg[i] = reinterpret_cast<const float4*>(gram)[threadIdx.x + i * SOLVE_TPB];
    {
        // thread: four consecutive columns cg * 4 .., every SOLVE_PARTS-th workgroup's partial sums
        constexpr int CG = TILE_B / 4;
        const int cg = threadIdx.x % CG, part = threadIdx.x / CG;
        const float4* p4 = reinterpret_cast<const float4*>(partial);
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        int wg = part;
        for (; wg + 3 * SOLVE_PARTS < n_wg; wg += 4 * SOLVE_PARTS) {      // four loads in flight (sixteen, predicated: slower)
            const float4 q0 = p4[(size_t)wg * CG + cg];
            const float4 q1 = p4[(size_t)(wg + SOLVE_PARTS) * CG + cg];
            const float4 q2 = p4[(size_t)(wg + 2 * SOLVE_PARTS) * CG + cg];
            const float4 q3 = p4[(size_t)(wg + 3 * SOLVE_PARTS) * CG + cg];
            acc[0] += ((double)q0.x + (double)q1.x) + ((double)q2.x + (double)q3.x);
            acc[1] += ((double)q0.y + (double)q1.y) + ((double)q2.y + (double)q3.y);
            acc[2] += ((double)q0.z + (double)q1.z) + ((double)q2.z + (double)q3.z);
            acc[3] += ((double)q0.w + (double)q1.w) + ((double)q2.w + (double)q3.w);
        }
        for (; wg < n_wg; wg += SOLVE_PARTS) {
            const float4 q0 = p4[(size_t)wg * CG + cg];
            acc[0] += (double)q0.x;
            acc[1] += (double)q0.y;
            acc[2] += (double)q0.z;
            acc[3] += (double)q0.w;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) gs[part * TILE_B + cg * 4 + k] = acc[k];
    }
    __syncthreads();
    // coordinate b of the tile: finished inner product and key (threads 0 .. TILE_B-1)
    double* gfin = gs + SOLVE_PARTS * TILE_B;
    uint32_t* keys = reinterpret_cast<uint32_t*>(gfin + TILE_B);
    int* seq_lds = reinterpret_cast<int*>(keys + TILE_B);
    static_assert(sizeof(double) * (SOLVE_PARTS + 1) * TILE_B + 8 * TILE_B <= sizeof(float) * TILE_B * TILE_B, "fits");
    uint32_t my_key = 0;
    if (threadIdx.x < TILE_B) {
        double acc = 0.0;
        for (int q = 0; q < SOLVE_PARTS; ++q) acc += gs[q * TILE_B + threadIdx.x];
        gfin[threadIdx.x] = acc;
        my_key = perm_key(perm_key_base(seed, tile), threadIdx.x);
        keys[threadIdx.x] = my_key;
    }
    __syncthreads();
    // position in the visiting order: rank of (key, index) among the tile's coordinates
    if ((int)threadIdx.x < nb) {
        int rank = 0;
        for (int o = 0; o < nb; ++o) {
            const uint32_t ko = keys[o];
            rank += (ko < my_key || (ko == my_key && o < (int)threadIdx.x)) ? 1 : 0;
        }
        seq_lds[rank] = threadIdx.x;
    }
    __syncthreads();
    const int lane = threadIdx.x & (WAVE - 1);
    const bool stepper = threadIdx.x < WAVE;             // wavefront 0 takes the steps
    // Lane l holds, in slot s, the coordinate that is visited (s * 64 + l)-th: then the step of the p-th visit
    // is taken from lane p % 64's own registers, slot p / 64, with no selection by coordinate, and only the
    // Gram row of the visited coordinate has to be read in that order (a gather from LDS).  u = (inner
    // product) / n is kept in fp64.
    double u[CPL];
    float Hf[CPL], rinv[CPL], xb[CPL], my_mult[CPL];
    int seq[CPL];                                         // the coordinate (0 .. nb-1 within the tile) of slot s
    if (stepper) {
#pragma unroll
        for (int s = 0; s < CPL; ++s) {
            const int pos = s * WAVE + lane;
            const bool live = pos < nb;
            const int b = live ? seq_lds[pos] : 0;
            seq[s] = b;
            u[s] = live ? gfin[b] * sp.inv_n : 0.0;
            xb[s] = live ? x[c0 + b] : 0.0f;
            const double hf = (double)(live ? norms[c0 + b] : 0.0f) * sp.inv_n;     // constant per coordinate
            Hf[s] = (float)hf;
            rinv[s] = (float)(1.0 / (hf + sp.lambda));
            my_mult[s] = 0.0f;
        }
    }
    __syncthreads();
    {
        const float inv_n = (float)sp.inv_n;             // the Gram block is stored divided by n, like u
#pragma unroll
        for (int i = 0; i < GL; ++i) {
            float4 t = mreg[i];
            t.x *= inv_n; t.y *= inv_n; t.z *= inv_n; t.w *= inv_n;
            reinterpret_cast<float4*>(lds)[threadIdx.x + i * SOLVE_TPB] = t;
        }
    }
    __syncthreads();
    if (!stepper) return;
    // Straight-line loop.  A single wavefront issues its instructions one after the other and fp64
    // instructions take several issue slots each, so only the running sums u stay in fp64; the step
    // itself is fp32 arithmetic (the result is an fp32 number anyway; the cancellation in u + lambda x
    // costs at most an ulp of x).  Every lane computes "its" step from its current sums at every visit; the one
    // whose turn it is publishes it.  The Gram rows of the next two visits are already on their way while a
    // step is computed; sums of coordinates that have had their turn are no longer kept up to date.
    const float lam = (float)sp.lambda, lam1 = (float)sp.lambda1, damp = (float)sp.damping;
    auto gram_row = [&](int pos, float (&m)[CPL]) {       // row of the coordinate visited pos-th, in visiting order
        int a = 0;
#pragma unroll
        for (int s = 0; s < CPL; ++s)
            if (pos / WAVE == s) a = __builtin_amdgcn_readlane(seq[s], pos & (WAVE - 1));
#pragma unroll
        for (int s = 0; s < CPL; ++s) m[s] = lds[a * TILE_B + seq[s]];
    };
    // A ring of four rows in registers, handed on by name (the loop is unrolled by four), not by moves: a move
    // at the end of a pass of the loop made every visit wait for the row it had just asked for.  Visit p works
    // with the row asked for three visits earlier and asks for the row of visit p + 3.
    float r0[CPL], r1[CPL], r2[CPL], r3[CPL];
    gram_row(0, r0);
    gram_row(nb > 1 ? 1 : 0, r1);
    gram_row(nb > 2 ? 2 : 0, r2);
    auto visit = [&](auto slot, int p, int p_end, const float (&row)[CPL], float (&ahead)[CPL]) {
        constexpr int sa = decltype(slot)::value;
        if (p >= p_end) return;                           // (uniform)
        gram_row(p + 3 < nb ? p + 3 : 0, ahead);
        const int la = p & (WAVE - 1);
        const float uf = (float)u[sa], xsel = xb[sa];
        float step;
        if (lam1 == 0.0f) {
            step = -(uf + lam * xsel) * rinv[sa];
        } else {
            const float t = Hf[sa] * xsel - uf;           // soft threshold, as in primal_step
            step = (t - fmaxf(-lam1, fminf(t, lam1))) * rinv[sa] - xsel;
        }
        const float xn = xsel + damp * step;
        const float m = xn - xsel;
        const float mult = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), la));
        const bool commit = lane == la;
        xb[sa] = commit ? xn : xb[sa];
        my_mult[sa] = commit ? m : my_mult[sa];
#pragma unroll
        for (int s = sa; s < CPL; ++s) u[s] += (double)(row[s] * mult);      // (earlier slots have had their turns)
    };
    auto half = [&](auto slot) {
        constexpr int sa = decltype(slot)::value;
        const int p_end = min(nb, (sa + 1) * WAVE);
        for (int p = sa * WAVE; p < p_end; p += 4) {      // (a slot starts at a multiple of four: the ring carries on)
            visit(slot, p, p_end, r0, r3);
            visit(slot, p + 1, p_end, r1, r0);
            visit(slot, p + 2, p_end, r2, r1);
            visit(slot, p + 3, p_end, r3, r2);
        }
    };
    static_assert(CPL == 2 && WAVE % 4 == 0, "two slots per lane");
    half(std::integral_constant<int, 0>{});
    half(std::integral_constant<int, 1>{});
#pragma unroll
    for (int s = 0; s < CPL; ++s) {
        if (s * WAVE + lane < nb) {
            x[c0 + seq[s]] = xb[s];
            mult_out[seq[s]] = my_mult[s];
        }
    }
}

// ---- host side -----------------------------------------------------------------------------------------
bool dense_tiles_applicable(const snap_handle* h) {
    return h->dense && h->layout == SNAP_DENSE_COLMAJOR && h->kind == K_PRIMAL_RIDGE && !h->streaming && h->n > 0 &&
           h->d > 0;
}

void dense_tiles_free(snap_handle* h) {
    (void)hipFree(h->tgram);
    (void)hipFree(h->tpartial);
    (void)hipFree(h->tmult);
    h->tgram = h->tpartial = h->tmult = nullptr;
}

int dense_tiles_setup(snap_handle* h) {
    const int64_t d = h->d, n = h->n;
    const int64_t T = (d + TILE_B - 1) / TILE_B;
    h->n_groups = T;
    h->gbounds_host = new (std::nothrow) int64_t[(size_t)T + 1];
    if (!h->gbounds_host) return SNAP_ENOMEM;
    for (int64_t t = 0; t <= T; ++t) h->gbounds_host[t] = std::min<int64_t>(d, t * TILE_B);
    h->tile_vec = 4;
    if (const char* e = getenv("SNAP_TILE_VEC")) {          // tuning knob: consecutive rows per thread
        const int vv = atoi(e);
        if (vv == 1 || vv == 2 || vv == 4) h->tile_vec = vv;
    }
    // vector loads need every column (stride ld) and the vectors v, y aligned to the vector size
    while (h->tile_vec > 1 && (h->ld % h->tile_vec != 0 || (uintptr_t)h->val % 16 != 0 || (uintptr_t)h->y % 16 != 0))
        h->tile_vec /= 2;
    h->tile_wgs = (n + PASS_TPB * h->tile_vec - 1) / (PASS_TPB * h->tile_vec);
    const size_t gcount = (size_t)T * TILE_B * TILE_B;
    double* gram64 = nullptr;
    SNAP_HIP(hipMalloc(&h->tgram, gcount * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->tpartial, (size_t)h->tile_wgs * TILE_B * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->tmult, 2 * TILE_B * sizeof(float)));
    SNAP_HIP(hipMalloc(&gram64, gcount * sizeof(double)));
    int rc = fill_zero(gram64, gcount * sizeof(double), h->compute);
    if (rc == SNAP_OK) {
        const dim3 grid((unsigned)T, (unsigned)((n + GRAM_ROWS - 1) / GRAM_ROWS));
        hipLaunchKernelGGL(k_tile_gram, grid, dim3(256), 0, h->compute, h->val, h->ld, n, d, gram64);
        hipLaunchKernelGGL(k_narrow_f64, dim3(1024), dim3(256), 0, h->compute, gram64, h->tgram, gcount);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = hipStreamSynchronize(h->compute);
        if (e != hipSuccess) rc = hip_fail(e, "Gram blocks of the tiles", __FILE__, __LINE__);
    }
    (void)hipFree(gram64);
    SNAP_TRY(rc);
    if (h->opt.profile) {
        h->ev_group = new (std::nothrow) hipEvent_t[(size_t)(2 * (T + 1))]();
        if (!h->ev_group) return SNAP_ENOMEM;
        for (int64_t i = 0; i < 2 * (T + 1); ++i) SNAP_HIP(hipEventCreate(&h->ev_group[i]));
        h->pass_timed.assign((size_t)(T + 1), 1);
    }
    h->g_hot_coords = h->m;             // statistics: every coordinate is handled by the row passes
    h->g_hot_nnz = h->nnz;
    h->tiled = true;
    return SNAP_OK;
}

int dense_tiles_epoch(snap_handle* h) {
    const StepParams sp = make_step_params(h);
    const int64_t n = h->n, T = h->n_groups;
    const bool prof = h->opt.profile != 0 && h->ev_group != nullptr;
    const std::vector<int64_t> order = group_order(h->last_seed, T);
    int64_t prev = -1;
    int n_pass = 0;
    for (int64_t ti = 0; ti <= T; ++ti) {
        const bool last = ti == T;
        const int64_t t = last ? T : order[(size_t)ti];
        const int64_t c0 = last ? 0 : h->gbounds_host[t];
        const int nb = last ? 0 : (int)(h->gbounds_host[t + 1] - c0);
        const int64_t p0 = prev >= 0 ? h->gbounds_host[prev] : 0;
        const int np = prev >= 0 ? (int)(h->gbounds_host[prev + 1] - p0) : 0;
        float* mult_prev = h->tmult + (size_t)((ti + 1) & 1) * TILE_B;
        float* mult_cur = h->tmult + (size_t)(ti & 1) * TILE_B;
        if (np == 0 && nb == 0) continue;
        // (profile: the two events take the kernel's own start and end times; events recorded between the
        // launches instead cost the chain of dependent kernels 3 us each)
        hipEvent_t ev_a = prof ? h->ev_group[2 * n_pass] : nullptr, ev_b = prof ? h->ev_group[2 * n_pass + 1] : nullptr;
#define SNAP_TILE_PASS(AL, VEC)                                                                                    \
    hipExtLaunchKernelGGL((k_tile_pass<AL, VEC>), dim3((unsigned)h->tile_wgs), dim3(PASS_TPB), 0, h->compute, ev_a, \
                          ev_b, 0, h->val, h->ld, n, p0, np, mult_prev, c0, nb, h->v, h->y, h->tpartial)
        if (h->tile_vec == 1) SNAP_TILE_PASS(false, 1);
        else if (h->tile_vec == 2) SNAP_TILE_PASS(true, 2);
        else SNAP_TILE_PASS(true, 4);
#undef SNAP_TILE_PASS
        ++n_pass;
        if (!last) {
            hipLaunchKernelGGL(k_tile_solve, dim3(1), dim3(SOLVE_TPB), 0, h->compute, h->tpartial, (int)h->tile_wgs, c0, nb,
                               (uint32_t)t, h->last_seed, h->tgram + (size_t)t * TILE_B * TILE_B, h->x, h->norms,
                               mult_cur, sp);
            prev = t;
        }
    }
    h->n_row_passes = n_pass;
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

}  // namespace snap
