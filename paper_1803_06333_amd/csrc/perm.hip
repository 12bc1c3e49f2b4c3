// Epoch order (Section 3.2, "Streaming Permutation Generation"): one 32-bit xorshift key per
// coordinate, then a sort of the keys that carries the coordinate indices.  The paper makes the
// keys on host threads and sorts them with a library radix sort; here the key is a counter-based
// function of (seed, chunk, coordinate), so it is produced directly on the device, and the sort is
// a least-significant-digit radix sort written for 64-wide wavefronts.  Equal keys keep the order
// of their indices (every pass is stable and the input is index-ascending), which makes the result
// unique and bit-comparable with any other correct sort.
#include "common.h"
#include "perm_key.h"

#include <algorithm>
#include <thread>
#include <vector>

namespace snap {

constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_TPB = 256;
constexpr int SORT_ROUNDS = 8;                                   // 64-element rounds per wavefront
constexpr int SORT_TILE = SORT_TPB * SORT_ROUNDS;                // 2048 elements per workgroup
constexpr int SORT_WAVES = SORT_TPB / WAVE;
static_assert(SORT_TPB == RADIX, "thread t of a sort workgroup owns digit t");

__global__ void k_make_keys(uint64_t seed, uint32_t chunk, uint32_t m, uint32_t* __restrict__ keys,
                            uint32_t* __restrict__ vals, uint32_t* __restrict__ keys_copy) {
    const uint64_t base = perm_key_base(seed, chunk);
    for (uint64_t c = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; c < m; c += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t k = perm_key(base, (uint32_t)c);
        keys[c] = k;
        vals[c] = (uint32_t)c;
        if (keys_copy) keys_copy[c] = k;
    }
}

// digit of element i: bits [shift, shift+8) of its key, or (cls != null) the class of its value
__device__ __forceinline__ uint32_t digit_of(uint32_t key, uint32_t val, int shift, const uint8_t* cls) {
    return cls ? (uint32_t)cls[val] : ((key >> shift) & (RADIX - 1));
}

// block_hist[digit * n_blocks + block] = number of elements of that digit in the block's tile
__global__ void __launch_bounds__(SORT_TPB)
k_radix_hist(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, uint32_t m, int shift,
             const uint8_t* __restrict__ cls, uint32_t* __restrict__ block_hist, uint32_t n_blocks) {
    __shared__ uint32_t hist[RADIX];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t base = blockIdx.x * SORT_TILE;
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        uint32_t i = base + r * SORT_TPB + threadIdx.x;
        if (i < m) atomicAdd(&hist[digit_of(keys[i], vals[i], shift, cls)], 1u);
    }
    __syncthreads();
    block_hist[(size_t)threadIdx.x * n_blocks + blockIdx.x] = hist[threadIdx.x];
}

// Offsets of the scatter in two levels.  Workgroup d turns the counts of digit d, one per block
// (block_hist[d * n_blocks ..]), into their exclusive prefix sums in place and writes the digit's
// total; the scatter kernel adds the prefix sum over the 256 totals itself.  (One workgroup
// scanning all 256 * n_blocks counts took four times as long as the rest of a pass.)
__global__ void __launch_bounds__(SORT_TPB)
k_digit_scan(uint32_t* __restrict__ block_hist, uint32_t n_blocks, uint32_t* __restrict__ totals) {
    __shared__ uint32_t wave_tot[SORT_WAVES];
    __shared__ uint32_t carry_s;
    uint32_t* a = block_hist + (size_t)blockIdx.x * n_blocks;
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint32_t base = 0; base < n_blocks; base += 4u * SORT_TPB) {
        const uint32_t i0 = base + 4u * threadIdx.x;
        uint32_t x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = i0 + j < n_blocks ? a[i0 + j] : 0u;
        const uint32_t mine = x[0] + x[1] + x[2] + x[3];
        uint32_t inc = mine;                               // inclusive scan across the wavefront
#pragma unroll
        for (int off = 1; off < WAVE; off <<= 1) {
            const uint32_t t = __shfl_up(inc, off, WAVE);
            if (lane >= off) inc += t;
        }
        if (lane == WAVE - 1) wave_tot[w] = inc;
        __syncthreads();
        uint32_t before = carry_s;
        for (int ww = 0; ww < w; ++ww) before += wave_tot[ww];
        uint32_t run = before + inc - mine;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i0 + j < n_blocks) a[i0 + j] = run;
            run += x[j];
        }
        __syncthreads();
        if (threadIdx.x == SORT_TPB - 1) carry_s = run;    // total so far
        __syncthreads();
    }
    if (threadIdx.x == 0) totals[blockIdx.x] = carry_s;
}

// The SORT_ROUNDS groups of 64 elements that one wavefront owns in a digit pass: the elements, their
// digits, and their ranks among the wavefront's elements of the same digit (inside a group from
// ballots, across groups from the wavefront's running counts cnt_w[digit]).
struct SortRounds {
    uint32_t key[SORT_ROUNDS], val[SORT_ROUNDS], dig[SORT_ROUNDS], rank[SORT_ROUNDS];
};

__device__ __forceinline__ void rank_rounds(const uint32_t* keys, const uint32_t* vals, uint32_t base, uint32_t m,
                                            int shift, const uint8_t* cls, uint32_t* cnt_w, SortRounds& q) {
    const int lane = threadIdx.x & (WAVE - 1);
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        const uint32_t i = base + r * WAVE + lane;
        const bool live = i < m;
        q.key[r] = live ? keys[i] : 0u;
        q.val[r] = live ? vals[i] : 0u;
        q.dig[r] = live ? digit_of(q.key[r], q.val[r], shift, cls) : 0u;
        uint64_t peers = __ballot(live);
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
            const bool bit = (q.dig[r] >> b) & 1u;
            const uint64_t bal = __ballot(bit && live);
            peers &= bit ? bal : ~bal;
        }
        if (!live) peers = 0;
        const uint32_t before = cnt_w[q.dig[r]];                 // all lanes read before any lane writes
        q.rank[r] = before + (uint32_t)__popcll(peers & lt);
        if (live && (peers & lt) == 0) cnt_w[q.dig[r]] = before + (uint32_t)__popcll(peers);
    }
}

// ... and their stable scatter once cnt_w[digit] holds the first position of the wavefront's elements
__device__ __forceinline__ void scatter_rounds(const SortRounds& q, uint32_t base, uint32_t m, const uint32_t* cnt_w,
                                               uint32_t* keys_out, uint32_t* vals_out) {
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        const uint32_t i = base + r * WAVE + lane;
        if (i < m) {
            const uint32_t pos = cnt_w[q.dig[r]] + q.rank[r];
            keys_out[pos] = q.key[r];
            vals_out[pos] = q.val[r];
        }
    }
}

// Stable scatter of one digit pass.  Wavefront w of the workgroup owns SORT_ROUNDS consecutive
// groups of 64 elements; inside a group the rank among equal digits comes from ballots, across
// groups from a per-wavefront running count in LDS, across wavefronts from a small prefix sum.
__global__ void __launch_bounds__(SORT_TPB)
k_radix_scatter(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals,
                uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out, uint32_t m, int shift,
                const uint8_t* __restrict__ cls, const uint32_t* __restrict__ block_off, uint32_t n_blocks,
                const uint32_t* __restrict__ totals) {
    __shared__ uint32_t cnt[SORT_WAVES][RADIX];
    __shared__ uint32_t digit_wave_tot[SORT_WAVES];
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    // first position of digit t = number of elements with a smaller digit: thread t holds digit t
    const uint32_t my_total = totals[threadIdx.x];
    uint32_t digit_base = my_total;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        const uint32_t t = __shfl_up(digit_base, off, WAVE);
        if (lane >= off) digit_base += t;
    }
    if (lane == WAVE - 1) digit_wave_tot[w] = digit_base;
    digit_base -= my_total;                                    // exclusive, within the wavefront
    for (int i = threadIdx.x; i < SORT_WAVES * RADIX; i += SORT_TPB) (&cnt[0][0])[i] = 0;
    __syncthreads();
    const uint32_t base = blockIdx.x * SORT_TILE + w * (SORT_ROUNDS * WAVE);
    SortRounds q;
    rank_rounds(keys, vals, base, m, shift, cls, cnt[w], q);
    __syncthreads();
    // exclusive prefix over the wavefronts, per digit; thread t handles digit t
    {
        for (int ww = 0; ww < w; ++ww) digit_base += digit_wave_tot[ww];
        uint32_t run = digit_base + block_off[(size_t)threadIdx.x * n_blocks + blockIdx.x];
#pragma unroll
        for (int ww = 0; ww < SORT_WAVES; ++ww) {
            uint32_t c = cnt[ww][threadIdx.x];
            cnt[ww][threadIdx.x] = run;
            run += c;
        }
    }
    __syncthreads();
    scatter_rounds(q, base, m, cnt[w], keys_out, vals_out);
}

// Up to SORT_TILE coordinates: the keys, the four digit passes and the class partition in one launch
// of one workgroup (a problem that small is bound by the sixteen launches of the general path, not by
// their work).  The passes go through the sorter's global buffers; the workgroup's barriers order them.
// Same keys, same stable passes: the same permutation.
__device__ __forceinline__ void one_block_pass(const uint32_t* keys, const uint32_t* vals, uint32_t* keys_out,
                                               uint32_t* vals_out, uint32_t m, int shift, const uint8_t* cls,
                                               uint32_t (*cnt)[RADIX], uint32_t* wave_tot) {
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    for (int i = threadIdx.x; i < SORT_WAVES * RADIX; i += SORT_TPB) (&cnt[0][0])[i] = 0;
    __syncthreads();
    const uint32_t base = w * (SORT_ROUNDS * WAVE);
    SortRounds q;
    rank_rounds(keys, vals, base, m, shift, cls, cnt[w], q);
    __syncthreads();
    // thread t holds digit t: elements with a smaller digit, then the wavefronts before this one
    uint32_t total = 0;
#pragma unroll
    for (int ww = 0; ww < SORT_WAVES; ++ww) total += cnt[ww][threadIdx.x];
    uint32_t run = total;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        const uint32_t t = __shfl_up(run, off, WAVE);
        if (lane >= off) run += t;
    }
    if (lane == WAVE - 1) wave_tot[w] = run;
    run -= total;
    __syncthreads();
    for (int ww = 0; ww < w; ++ww) run += wave_tot[ww];
#pragma unroll
    for (int ww = 0; ww < SORT_WAVES; ++ww) {
        const uint32_t c = cnt[ww][threadIdx.x];
        cnt[ww][threadIdx.x] = run;
        run += c;
    }
    __syncthreads();
    scatter_rounds(q, base, m, cnt[w], keys_out, vals_out);
    __syncthreads();   // the next pass reads what this one wrote, and reuses cnt
}

__global__ void __launch_bounds__(SORT_TPB)
k_sort_one_block(uint64_t seed, uint32_t chunk, uint32_t m, const uint8_t* __restrict__ cls, uint32_t* ka, uint32_t* va,
                 uint32_t* kb, uint32_t* vb, uint32_t* __restrict__ keys_out, uint32_t* __restrict__ order_out,
                 uint32_t* __restrict__ part_out) {
    __shared__ uint32_t cnt[SORT_WAVES][RADIX];
    __shared__ uint32_t wave_tot[SORT_WAVES];
    const uint64_t base = perm_key_base(seed, chunk);
    for (uint32_t c = threadIdx.x; c < m; c += SORT_TPB) {
        const uint32_t k = perm_key(base, c);
        ka[c] = k;
        va[c] = c;
        if (keys_out) keys_out[c] = k;
    }
    __syncthreads();
    for (int shift = 0; shift < 32; shift += RADIX_BITS) {
        one_block_pass(ka, va, kb, vb, m, shift, nullptr, cnt, wave_tot);
        uint32_t* t = ka; ka = kb; kb = t;
        t = va; va = vb; vb = t;
    }
    if (order_out)
        for (uint32_t c = threadIdx.x; c < m; c += SORT_TPB) order_out[c] = va[c];
    if (part_out) {
        one_block_pass(ka, va, kb, vb, m, 0, cls, cnt, wave_tot);
        for (uint32_t c = threadIdx.x; c < m; c += SORT_TPB) part_out[c] = vb[c];
    }
}

int sorter_alloc(Sorter& s, int64_t max_m) {
    s.max_m = max_m > 0 ? max_m : 1;
    s.n_blocks = (s.max_m + SORT_TILE - 1) / SORT_TILE;
    size_t bytes = (size_t)s.max_m * sizeof(uint32_t);
    SNAP_HIP(hipMalloc(&s.keys_a, bytes));
    SNAP_HIP(hipMalloc(&s.keys_b, bytes));
    SNAP_HIP(hipMalloc(&s.vals_a, bytes));
    SNAP_HIP(hipMalloc(&s.vals_b, bytes));
    // the counts per (digit, block), then the 256 totals per digit
    SNAP_HIP(hipMalloc(&s.block_hist, ((size_t)s.n_blocks + 1) * RADIX * sizeof(uint32_t)));
    return SNAP_OK;
}

void sorter_free(Sorter& s) {
    (void)hipFree(s.keys_a);
    (void)hipFree(s.keys_b);
    (void)hipFree(s.vals_a);
    (void)hipFree(s.vals_b);
    (void)hipFree(s.block_hist);
    s = Sorter{};
}

static int radix_pass(snap_handle* h, uint32_t*& ka, uint32_t*& va, uint32_t*& kb, uint32_t*& vb, uint32_t m,
                      int shift, const uint8_t* cls) {
    Sorter& s = h->sorter;
    const uint32_t nb = (m + SORT_TILE - 1) / SORT_TILE;
    hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(SORT_TPB), 0, h->compute, ka, va, m, shift, cls, s.block_hist, nb);
    uint32_t* totals = s.block_hist + (size_t)s.n_blocks * RADIX;
    hipLaunchKernelGGL(k_digit_scan, dim3(RADIX), dim3(SORT_TPB), 0, h->compute, s.block_hist, nb, totals);
    hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(SORT_TPB), 0, h->compute, ka, va, kb, vb, m, shift, cls,
                       s.block_hist, nb, totals);
    uint32_t* t = ka; ka = kb; kb = t;
    t = va; va = vb; vb = t;
    return SNAP_OK;
}

// ---- keys made on the host (options.host_keys): the third pipeline stage of Section 3.2 --------------
// Host threads fill a pinned buffer with the chunk's keys (the same counter-based generator as the
// device's, so the thread count does not matter), a stream of its own takes it to the device, and a small
// kernel hands the keys to the sorter.  Two buffers are used in turn: the host may prepare the keys of a
// chunk while the copy of the previous chunk's keys is still under way; since the calls that enqueue a
// chunk's work return long before the device gets to it, this overlaps with the device's sweep of the
// chunk before and with the copy engine's transfer of the one after.
__global__ void k_take_keys(const uint32_t* __restrict__ in, uint32_t m, uint32_t* __restrict__ keys,
                            uint32_t* __restrict__ vals, uint32_t* __restrict__ keys_copy) {
    for (uint64_t c = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; c < m; c += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t k = in[c];
        keys[c] = k;
        vals[c] = (uint32_t)c;
        if (keys_copy) keys_copy[c] = k;
    }
}

int host_keys_alloc(snap_handle* h, int64_t max_m) {
    const size_t bytes = (size_t)(max_m > 0 ? max_m : 1) * sizeof(uint32_t);
    for (int i = 0; i < 2; ++i) {
        SNAP_HIP(hipHostMalloc(&h->hk_host[i], bytes, hipHostMallocDefault));
        SNAP_HIP(hipMalloc(&h->hk_dev[i], bytes));
        SNAP_HIP(hipEventCreateWithFlags(&h->hk_copied[i], hipEventDisableTiming));
        SNAP_HIP(hipEventCreateWithFlags(&h->hk_taken[i], hipEventDisableTiming));
    }
    return SNAP_OK;
}

void host_keys_free(snap_handle* h) {
    for (int i = 0; i < 2; ++i) {
        if (h->hk_host[i]) (void)hipHostFree(h->hk_host[i]);
        (void)hipFree(h->hk_dev[i]);
        if (h->hk_copied[i]) (void)hipEventDestroy(h->hk_copied[i]);
        if (h->hk_taken[i]) (void)hipEventDestroy(h->hk_taken[i]);
        h->hk_host[i] = h->hk_dev[i] = nullptr;
        h->hk_copied[i] = h->hk_taken[i] = nullptr;
    }
}

static void host_fill_keys(uint32_t* out, uint64_t seed, uint32_t chunk, uint32_t m) {
    const uint64_t base = perm_key_base(seed, chunk);
    auto fill = [=](uint32_t lo, uint32_t hi) {
        for (uint32_t c = lo; c < hi; ++c) out[c] = perm_key(base, c);
    };
    const unsigned hw = std::max(1u, std::thread::hardware_concurrency());
    const unsigned threads = (unsigned)std::min<uint64_t>(std::min(16u, hw), std::max<uint64_t>(1, (uint64_t)m / 65536));
    if (threads <= 1) {
        fill(0, m);
        return;
    }
    std::vector<std::thread> pool;
    const uint32_t per = (m + threads - 1) / threads;
    for (unsigned t = 1; t < threads; ++t) pool.emplace_back(fill, std::min(m, t * per), std::min(m, (t + 1) * per));
    fill(0, std::min(m, per));
    for (auto& th : pool) th.join();
}

int make_permutation(snap_handle* h, uint64_t seed, uint32_t chunk, int64_t c0, int64_t m, uint32_t* keys_out,
                     uint32_t* order_out, uint32_t* part_out) {
    if (m <= 0) return SNAP_OK;
    Sorter& s = h->sorter;
    if (m > s.max_m || m > 0xFFFFFFFFll) {
        set_error("permutation of %lld coordinates exceeds the sorter capacity", (long long)m);
        return SNAP_EINVAL;
    }
    uint32_t *ka = s.keys_a, *va = s.vals_a, *kb = s.keys_b, *vb = s.vals_b;
    const uint32_t mm = (uint32_t)m;
    const int grid = (int)((m + 255) / 256 < 4096 ? (m + 255) / 256 : 4096);
    if (!h->hk_host[0] && m <= SORT_TILE) {
        hipLaunchKernelGGL(k_sort_one_block, dim3(1), dim3(SORT_TPB), 0, h->compute, seed, chunk, mm,
                           part_out ? h->cls + c0 : nullptr, ka, va, kb, vb, keys_out, order_out, part_out);
        SNAP_HIP(hipGetLastError());
        return SNAP_OK;
    }
    if (h->hk_host[0]) {
        const int sl = h->hk_slot;
        h->hk_slot ^= 1;
        SNAP_HIP(hipEventSynchronize(h->hk_copied[sl]));             // the last copy out of this host buffer is done
        host_fill_keys(h->hk_host[sl], seed, chunk, mm);
        SNAP_HIP(hipStreamWaitEvent(h->hk_stream, h->hk_taken[sl], 0));  // ... and the sorter has taken the device twin's last content
        SNAP_HIP(hipMemcpyAsync(h->hk_dev[sl], h->hk_host[sl], (size_t)m * sizeof(uint32_t), hipMemcpyHostToDevice,
                                h->hk_stream));
        SNAP_HIP(hipEventRecord(h->hk_copied[sl], h->hk_stream));
        SNAP_HIP(hipStreamWaitEvent(h->compute, h->hk_copied[sl], 0));
        hipLaunchKernelGGL(k_take_keys, dim3(grid), dim3(256), 0, h->compute, h->hk_dev[sl], mm, ka, va, keys_out);
        SNAP_HIP(hipEventRecord(h->hk_taken[sl], h->compute));
    } else {
        hipLaunchKernelGGL(k_make_keys, dim3(grid), dim3(256), 0, h->compute, seed, chunk, mm, ka, va, keys_out);
    }
    for (int shift = 0; shift < 32; shift += RADIX_BITS) SNAP_TRY(radix_pass(h, ka, va, kb, vb, mm, shift, nullptr));
    if (order_out)
        SNAP_HIP(hipMemcpyAsync(order_out, va, (size_t)m * sizeof(uint32_t), hipMemcpyDeviceToDevice, h->compute));
    if (part_out) {
        SNAP_TRY(radix_pass(h, ka, va, kb, vb, mm, 0, h->cls + c0));
        SNAP_HIP(hipMemcpyAsync(part_out, va, (size_t)m * sizeof(uint32_t), hipMemcpyDeviceToDevice, h->compute));
    }
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

}  // namespace snap
