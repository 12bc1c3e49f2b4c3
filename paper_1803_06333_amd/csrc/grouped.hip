// Exact group sweeps: an epoch for data whose coordinates come in groups with pairwise disjoint
// supports (the columns of one one-hot encoded field of click-log data, Section 4).  Coordinates of
// one group do not interact -- no row of v is touched by two of them -- so updating all of them at
// once IS the sequential coordinate-descent result for that group; groups are visited one after
// the other, in a seeded random order.  The epoch therefore equals sequential SCD (Section 3.1)
// in that order exactly (up to rounding), and needs neither atomics on v nor a cap on the work
// in flight.
//
// What makes it fast on this part is that both inner loops turn from random 4-byte accesses to the
// 183 MB vector v into coalesced streams over the rows:
//   - every group g has a row map: rowmap[g][r] = rank of the coordinate of g that contains row r
//     (ranks order the group's coordinates by decreasing length); 16 bits per entry when no group has
//     more than 65535 coordinates, else 32; the label signs sit in a bit array of their own;
//   - one row pass reads v[r] once, applies the step of the previous group
//     (v[r] += delta[g-1][rank]), evaluates loss' and loss'' at the new v[r] and adds them into the
//     sums of group g's coordinate: hot ranks (the longest coordinates) accumulate in LDS, one
//     partial array per workgroup, summed afterwards in a fixed order;
//   - a second kernel sums the partials of the hot ranks, lets the remaining (short) coordinates of
//     the group take their sums column-wise (from a dense buffer of their rows' entries of v that the
//     row pass fills on its way), and turns all sums into the steps that the next row pass applies.
// Traffic per group and row: two map entries (2 + 2 bytes), read + write of v (8 bytes), one label bit
// (+ values unless all 1).
#include "scd_device.h"
#include <hip/hip_ext.h>
#include "perm_key.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <type_traits>
#include <vector>

namespace snap {

constexpr uint32_t RANK_NONE = 0xFFFFFFFFu;      // row not covered by the group (all ones in either map width)
// The sums of the hot ranks are kept in LDS as 64-bit fixed-point integers: integer LDS atomics run
// more than twenty times faster here than ds_add_f32 (measured), and the result does not depend on
// the order of the additions (the epoch is bit-reproducible).  The terms of the logistic loss are
// bounded, so they are scaled to about 20 bits and turned into integers by the rounding of one
// floating-point addition (a float-to-int64 conversion costs a dozen instructions); the terms of the
// ridge loss are not and take that conversion, with 24 fractional bits.
//
// Packed ranks (logistic loss).  LDS capacity decides how many coordinates of a group are hot, and a
// row of a coordinate that is not costs several times a row of one that is (its entry of the shared
// vector takes a detour through a buffer to the finishing kernel, its step a gather in the next row
// pass).  Both sums of a rank
// whose coordinate has at most PACK_COUNT_MAX rows fit ONE 64-bit word -- the high half for the signed
// sum of a loss' (19 fractional bits relative to the largest |value|), the low half for the sum of
// a^2 loss'' (22 fractional bits), so that a word is put together from two 32-bit conversions without
// 64-bit arithmetic; the rounding of the terms averages out over the rows (relative error of a sum
// about 2e-6 / sqrt(rows)) -- so only the few hundred longest coordinates keep two words.  All ranks
// use these scales (one set of scales saves selects).  That halves the LDS per rank (and the LDS atomics
// per row) for the rest.
//
// One workgroup of 1024 threads per compute unit with all of its LDS: 12288 hot ranks (packed) and 12288
// steps of the previous group.  Two workgroups per unit with half the tables each used to run the pass
// 20 % faster while it was bound by instruction issue; since it no longer is, the pass runs as fast
// with 16 wavefronts per unit, and the larger tables take a tenth off the epoch (click-log workload:
// 5.84 -> 5.19 ms with 14336 ranks + 8192 steps; with the dense buffer for the short coordinates, which
// makes their rows cheaper, 12288 + 12288 is the better split: 4.92 against 4.95 ms).
constexpr int HOT_MAX = 16384;                   // most ranks accumulated in LDS (tuning knob's ceiling)
constexpr int HOT_DEFAULT = 12288;
constexpr int HOT_MIN_ROWS = 32;                 // a rank is worth an LDS slot while its coordinate has that many rows
constexpr int DELTA_LDS = 16384;                 // most steps of the previous group kept in LDS (tuning knob's ceiling)
constexpr int DELTA_DEFAULT = 12288;
constexpr int ROW_TPB = 1024;
constexpr int COLD_RING = 128;                   // entries per wavefront staged in LDS on their way to the short coordinates' buffer
constexpr int ROW_WGS_DEFAULT = 256;             // one workgroup per compute unit
constexpr int PACK_COUNT_MAX = 4095;             // rows of a coordinate whose two sums share one word
constexpr int PACK_H_BITS = 32;                  // a packed word: sum of a^2 loss'' in the low half, of a loss' in the high half
// Tuning knobs (environment variables), read when a handle is created.
static int row_wgs_knob() {
    const char* e = getenv("SNAP_ROW_WGS");
    return e ? std::max(1, atoi(e)) : 0;
}
static bool pack_knob() {
    const char* e = getenv("SNAP_PACK");             // 0 switches the packed ranks off
    return !(e && e[0] == '0');
}
static bool map8_knob() {
    const char* e = getenv("SNAP_MAP8");             // 0: no byte maps (resident: read by the row passes; streamed: on the host link)
    return !(e && e[0] == '0');
}
static bool pfx_knob() {
    const char* e = getenv("SNAP_PFX");              // 0: streamed row maps are never prefix-coded
    return !(e && e[0] == '0');
}
static bool compact_knob() {
    const char* e = getenv("SNAP_COMPACT");          // 0 switches the dense buffer of the short coordinates off
    return !(e && e[0] == '0');
}
static int hot_max() {
    const char* e = getenv("SNAP_HOT_MAX");
    return e ? std::max(4, std::min(HOT_MAX, atoi(e))) : HOT_DEFAULT;
}
static int hot_min_rows() {
    const char* e = getenv("SNAP_HOT_ROWS");
    return e ? std::max(1, atoi(e)) : HOT_MIN_ROWS;
}
static int wgs_per_cu() {
    const char* e = getenv("SNAP_WGS_PER_CU");       // 2 = two workgroups per compute unit, half the LDS each
    return (e && e[0] == '2') ? 2 : 1;
}

// ---- creation --------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, size_t count, uint32_t value) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        p[i] = value;
}

// Largest |value| (bit order = value order for non-negative floats) and whether every value is 1.
__global__ void k_value_stats(const float* __restrict__ val, int64_t nnz, uint32_t* flags) {
    uint32_t mx = 0, not_one = 0;
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < nnz; k += (int64_t)gridDim.x * blockDim.x) {
        const float a = val[k];
        mx = max(mx, __float_as_uint(fabsf(a)));
        not_one |= a != 1.0f ? 2u : 0u;
    }
    if (not_one) atomicOr(flags, 2u);
    atomicMax(flags + 1, mx);
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
    }
}

__global__ void k_narrow_map(const uint32_t* __restrict__ wide, uint16_t* __restrict__ narrow, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        narrow[i] = (uint16_t)wide[i];            // ranks are below 65535; "none" (all ones) stays all ones
}

// Row maps of groups with at most 255 coordinates as bytes ("none" = 0xFF) for the trip over the host
// link, and back to the 16-bit entries that the row pass reads; four entries per thread and step.
__global__ void k_map16_to_8(const uint16_t* __restrict__ in, uint8_t* __restrict__ out, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count / 4; i += (size_t)gridDim.x * blockDim.x) {
        const uint2 u = reinterpret_cast<const uint2*>(in)[i];
        reinterpret_cast<uint32_t*>(out)[i] = (u.x & 0xFFu) | ((u.x >> 16 & 0xFFu) << 8) | ((u.y & 0xFFu) << 16) | ((u.y >> 16 & 0xFFu) << 24);
    }
}
__global__ void k_map8_to_16(const uint8_t* __restrict__ in, uint16_t* __restrict__ out, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count / 4; i += (size_t)gridDim.x * blockDim.x) {
        const uint32_t u = reinterpret_cast<const uint32_t*>(in)[i];
        auto wide = [](uint32_t b) { return b == 0xFFu ? 0xFFFFu : b; };
        uint2 o;
        o.x = wide(u & 0xFFu) | (wide(u >> 8 & 0xFFu) << 16);
        o.y = wide(u >> 16 & 0xFFu) | (wide(u >> 24) << 16);
        reinterpret_cast<uint2*>(out)[i] = o;
    }
}

// Escape-coded byte maps: the ranks of a one-hot field with a Zipf-like popularity are concentrated
// (four of five rows of the click-log fields have a rank below 254), so a field of up to 65535 columns
// crosses the host link as one byte per row -- the rank, ESC8 for "rank >= 254", 0xFF for "none" -- plus
// the two-byte ranks of the escaped rows in row order.  Layout of a blob:
//   [ n_pad bytes ][ one uint32 per block of ESC_BLOCK rows: escaped rows before the block ][ uint16 ranks ]
// A workgroup of ESC_TPB threads handles one block, four consecutive rows per thread; the place of a
// thread's first escaped row is the block's offset plus an exclusive scan of the per-thread counts.
constexpr int ESC_TPB = 1024, ESC_BLOCK = 4 * ESC_TPB;
constexpr uint32_t ESC8 = 254u;

// exclusive prefix, over the workgroup, of a count 0 .. 4 per thread (three ballots per wavefront, one
// round through LDS for the wavefronts' totals); s_tot: ESC_TPB / WAVE + 1 words
__device__ __forceinline__ uint32_t esc_scan(uint32_t c, uint32_t* s_tot) {
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const unsigned long long m = __builtin_amdgcn_ballot_w64((c >> b) & 1u);
        before += (uint32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u)) << b;
        total += (uint32_t)__popcll(m) << b;
    }
    __syncthreads();                                   // (s_tot may still be read from an earlier use)
    if (lane == 0) s_tot[wave] = total;
    __syncthreads();
    uint32_t base = 0;
    for (int w = 0; w < wave; ++w) base += s_tot[w];
    return base + before;
}

__device__ __forceinline__ bool esc_row(uint32_t rank) { return rank >= ESC8 && rank != 0xFFFFu; }

// counts[block] <- escaped rows of the block
__global__ void __launch_bounds__(ESC_TPB)
k_esc_count(const uint16_t* __restrict__ map, uint32_t* __restrict__ counts) {
    __shared__ uint32_t s_tot[ESC_TPB / WAVE + 1];
    const uint2 u = reinterpret_cast<const uint2*>(map)[(size_t)blockIdx.x * ESC_TPB + threadIdx.x];
    const uint32_t c = esc_row(u.x & 0xFFFFu) + esc_row(u.x >> 16) + esc_row(u.y & 0xFFFFu) + esc_row(u.y >> 16);
    const uint32_t at = esc_scan(c, s_tot);
    if (threadIdx.x == ESC_TPB - 1) counts[blockIdx.x] = at + c;
}

// map (n_pad 16-bit entries, n_pad a multiple of ESC_BLOCK here: the staging map is padded with "none")
// -> bytes, and the escaped ranks at their places; offs[block] = escaped rows before the block
__global__ void __launch_bounds__(ESC_TPB)
k_esc_encode(const uint16_t* __restrict__ map, const uint32_t* __restrict__ offs, uint8_t* __restrict__ bytes,
             uint16_t* __restrict__ esc) {
    __shared__ uint32_t s_tot[ESC_TPB / WAVE + 1];
    const size_t t = (size_t)blockIdx.x * ESC_TPB + threadIdx.x;
    const uint2 u = reinterpret_cast<const uint2*>(map)[t];
    const uint32_t r[4] = {u.x & 0xFFFFu, u.x >> 16, u.y & 0xFFFFu, u.y >> 16};
    const uint32_t c = esc_row(r[0]) + esc_row(r[1]) + esc_row(r[2]) + esc_row(r[3]);
    uint32_t at = offs[blockIdx.x] + esc_scan(c, s_tot);
    uint32_t packed = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t b = r[j] == 0xFFFFu ? 0xFFu : r[j];
        if (esc_row(r[j])) {
            esc[at++] = (uint16_t)r[j];
            b = ESC8;
        }
        packed |= b << (8 * j);
    }
    reinterpret_cast<uint32_t*>(bytes)[t] = packed;
}

__global__ void __launch_bounds__(ESC_TPB)
k_esc_decode(const uint8_t* __restrict__ bytes, const uint32_t* __restrict__ offs, const uint16_t* __restrict__ esc,
             uint16_t* __restrict__ map) {
    __shared__ uint32_t s_tot[ESC_TPB / WAVE + 1];
    const size_t t = (size_t)blockIdx.x * ESC_TPB + threadIdx.x;
    const uint32_t u = reinterpret_cast<const uint32_t*>(bytes)[t];
    const uint32_t b[4] = {u & 0xFFu, u >> 8 & 0xFFu, u >> 16 & 0xFFu, u >> 24};
    const uint32_t c = (b[0] == ESC8) + (b[1] == ESC8) + (b[2] == ESC8) + (b[3] == ESC8);
    uint32_t at = offs[blockIdx.x] + esc_scan(c, s_tot);
    uint32_t r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = b[j] == ESC8 ? (uint32_t)esc[at++] : (b[j] == 0xFFu ? 0xFFFFu : b[j]);
    uint2 o;
    o.x = r[0] | (r[1] << 16);
    o.y = r[2] | (r[3] << 16);
    reinterpret_cast<uint2*>(map)[t] = o;
}

// Prefix-coded maps.  The ranks of a one-hot field carry far fewer bits than the one or two bytes of the
// codings above (the click-log fields: 7.7 bits of entropy per row for 38 430 columns with a Zipf(1.2)
// popularity, about 4 for the 64-bin fields), and what crosses the host link is what bounds a streamed
// epoch.  A rank is sent as the prefix code of its class followed by the class's extra bits:
//   groups of at most 62 coordinates: class = rank, no extra bits, "none" = class `size`;
//   larger groups: x = rank + 1 = 1 .. 65535 by quarter octaves -- x <= 7: class x - 1; else, with
//   b = floor(log2 x) >= 3, class 7 + 4 (b - 3) + (the two bits below the leading one), b - 2 extra
//   bits -- "none" = class 59.  (Within a quarter octave a Zipf-like popularity varies by a third, which
//   costs a tenth of a bit; whole octaves would cost 0.8.)
// The code of the classes is a Huffman code of the group's own class counts (known from the column lengths),
// limited to PFX_MAXLEN bits so that one table lookup decodes it; bits are written from the low end of
// 32-bit words.  A thread codes or decodes PFX_SUB consecutive rows; layout of a blob:
//   [ uint64 per block of PFX_BLOCK rows: bit offset of the block ][ the 32-bit words (+ 2 of padding) ]
//   [ uint16 per PFX_SUB rows: bit offset inside the block (at most 2048 x 25 bits) ]
// Per group the device holds a table: PFX_LUT entries (class << 4 | length) indexed by the next PFX_MAXLEN
// bits, then per class (rank of the class's first member | extra bits << 16), then per class (code | length << 16).
constexpr int PFX_SUB = 64, PFX_BLOCK = 2048, PFX_MAXLEN = 12, PFX_LUT = 1 << PFX_MAXLEN, PFX_CLASSES = 64;
constexpr int PFX_DIRECT_MAX = 62, PFX_NONE_CLASS = 59;
constexpr size_t PFX_TAB_BYTES = PFX_LUT * sizeof(uint16_t) + 2 * PFX_CLASSES * sizeof(uint32_t);

// class, extra bits and their count of a rank; direct_none: the class of "none" for a small group, -1 for a large one
__host__ __device__ __forceinline__ uint32_t pfx_class_of(uint32_t rank, int direct_none, uint32_t& extra, uint32_t& eb) {
    extra = 0;
    eb = 0;
    if (rank == 0xFFFFu) return direct_none >= 0 ? (uint32_t)direct_none : (uint32_t)PFX_NONE_CLASS;
    if (direct_none >= 0) return rank;
    const uint32_t x = rank + 1u;
    uint32_t b = 0;
#if defined(__HIP_DEVICE_COMPILE__)
    b = 31u - (uint32_t)__clz((int)x);
#else
    while ((x >> (b + 1)) != 0u) ++b;
#endif
    if (b <= 2u) return x - 1u;
    eb = b - 2u;
    extra = x & ((1u << eb) - 1u);
    return 7u + 4u * (b - 3u) + ((x >> eb) & 3u);
}

// sub_rel[t] <- bits of the rows before sub-block t in its block; block_bits[block] <- bits of the block
__global__ void __launch_bounds__(256)
k_pfx_count(const uint16_t* __restrict__ map, int64_t n_sub, const uint32_t* __restrict__ enc, int direct_none,
            uint16_t* __restrict__ sub_rel, uint32_t* __restrict__ block_bits) {
    __shared__ uint32_t s_enc[PFX_CLASSES];
    if (threadIdx.x < PFX_CLASSES) s_enc[threadIdx.x] = enc[threadIdx.x];
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t bits = 0;
    if (t < n_sub) {
        const uint4* src = reinterpret_cast<const uint4*>(map + (size_t)t * PFX_SUB);
        for (int q = 0; q < PFX_SUB / 8; ++q) {
            const uint4 u = src[q];
            const uint32_t r[8] = {u.x & 0xFFFFu, u.x >> 16, u.y & 0xFFFFu, u.y >> 16, u.z & 0xFFFFu, u.z >> 16, u.w & 0xFFFFu, u.w >> 16};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t extra, eb;
                const uint32_t c = pfx_class_of(r[j], direct_none, extra, eb);
                bits += (s_enc[c] >> 16) + eb;
            }
        }
    }
    // exclusive prefix over the 32 sub-blocks of a block: 32 consecutive lanes (n_sub is a multiple of 32)
    uint32_t incl = bits;
#pragma unroll
    for (int d = 1; d < PFX_BLOCK / PFX_SUB; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d, PFX_BLOCK / PFX_SUB);
        if ((int)(threadIdx.x & (PFX_BLOCK / PFX_SUB - 1)) >= d) incl += up;
    }
    if (t < n_sub) {
        sub_rel[t] = (uint16_t)(incl - bits);
        if ((t & (PFX_BLOCK / PFX_SUB - 1)) == PFX_BLOCK / PFX_SUB - 1) block_bits[t / (PFX_BLOCK / PFX_SUB)] = incl;
    }
}

// words must be zero before: neighbouring sub-blocks share their boundary words
__global__ void __launch_bounds__(256)
k_pfx_encode(const uint16_t* __restrict__ map, int64_t n_sub, const uint32_t* __restrict__ enc, int direct_none,
             const unsigned long long* __restrict__ block_off, const uint16_t* __restrict__ sub_rel, uint32_t* __restrict__ words) {
    __shared__ uint32_t s_enc[PFX_CLASSES];
    if (threadIdx.x < PFX_CLASSES) s_enc[threadIdx.x] = enc[threadIdx.x];
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_sub) return;
    const unsigned long long bitpos = block_off[t / (PFX_BLOCK / PFX_SUB)] + sub_rel[t];
    size_t wi = (size_t)(bitpos >> 5);
    uint32_t fill = (uint32_t)(bitpos & 31u);
    unsigned long long acc = 0;
    const uint4* src = reinterpret_cast<const uint4*>(map + (size_t)t * PFX_SUB);
    for (int q = 0; q < PFX_SUB / 8; ++q) {
        const uint4 u = src[q];
        const uint32_t r[8] = {u.x & 0xFFFFu, u.x >> 16, u.y & 0xFFFFu, u.y >> 16, u.z & 0xFFFFu, u.z >> 16, u.w & 0xFFFFu, u.w >> 16};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t extra, eb;
            const uint32_t c = pfx_class_of(r[j], direct_none, extra, eb);
            const uint32_t e = s_enc[c], len = e >> 16;
            acc |= (unsigned long long)((e & 0xFFFFu) | (extra << len)) << fill;       // at most 25 bits on top of at most 31
            fill += len + eb;
            if (fill >= 32u) {
                atomicOr(words + wi, (uint32_t)acc);
                ++wi;
                acc >>= 32;
                fill -= 32u;
            }
        }
    }
    if (fill > 0u) atomicOr(words + wi, (uint32_t)acc);
}

__global__ void __launch_bounds__(256)
k_pfx_decode(const unsigned long long* __restrict__ block_off, const uint32_t* __restrict__ words,
             const uint16_t* __restrict__ sub_rel, const uint8_t* __restrict__ tab, int64_t n_sub, uint16_t* __restrict__ map) {
    __shared__ uint16_t s_lut[PFX_LUT];
    __shared__ uint32_t s_cls[PFX_CLASSES];
    for (int i = threadIdx.x; i < PFX_LUT; i += 256) s_lut[i] = reinterpret_cast<const uint16_t*>(tab)[i];
    if (threadIdx.x < PFX_CLASSES) s_cls[threadIdx.x] = reinterpret_cast<const uint32_t*>(tab + PFX_LUT * sizeof(uint16_t))[threadIdx.x];
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_sub) return;
    const unsigned long long bitpos = block_off[t / (PFX_BLOCK / PFX_SUB)] + sub_rel[t];
    const uint32_t* wp = words + (size_t)(bitpos >> 5);
    const uint32_t shift = (uint32_t)(bitpos & 31u);
    // the low `have` bits of buf are the next bits of the stream (the words are padded: reading two past the end is fine)
    unsigned long long buf = ((unsigned long long)wp[0] | ((unsigned long long)wp[1] << 32)) >> shift;
    uint32_t have = 64u - shift;
    wp += 2;
    uint4* dst = reinterpret_cast<uint4*>(map + (size_t)t * PFX_SUB);
    for (int q = 0; q < PFX_SUB / 8; ++q) {
        uint32_t r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (have < 32u) {
                buf |= (unsigned long long)(*wp++) << have;
                have += 32u;
            }
            const uint32_t e = s_lut[(uint32_t)buf & (PFX_LUT - 1)];
            const uint32_t len = e & 15u, ce = s_cls[e >> 4], eb = ce >> 16;
            buf >>= len;
            r[j] = (ce & 0xFFFFu) + ((uint32_t)buf & ((1u << eb) - 1u));
            buf >>= eb;
            have -= len + eb;
        }
        dst[q] = make_uint4(r[0] | (r[1] << 16), r[2] | (r[3] << 16), r[4] | (r[5] << 16), r[6] | (r[7] << 16));
    }
}

// Code lengths of a Huffman code of the counts, limited to max_len bits (counts are flattened until the
// code fits: each round halves them, rounding up, which only shortens the longest codes).  Classes
// that do not occur get length 0.
static void pfx_code_lengths(const uint64_t (&count)[PFX_CLASSES], int max_len, int (&len)[PFX_CLASSES]) {
    uint64_t f[PFX_CLASSES];
    for (int i = 0; i < PFX_CLASSES; ++i) f[i] = count[i];
    for (;;) {
        struct Node {
            uint64_t w;
            int left, right;
        };
        std::vector<Node> nodes;
        std::vector<int> alive;
        for (int i = 0; i < PFX_CLASSES; ++i) {
            len[i] = 0;
            if (f[i] > 0) {
                nodes.push_back({f[i], -1 - i, 0});
                alive.push_back((int)nodes.size() - 1);
            }
        }
        if (alive.size() <= 1) {
            for (int i = 0; i < PFX_CLASSES; ++i) len[i] = f[i] > 0 ? 1 : 0;
            return;
        }
        while (alive.size() > 1) {          // (at most 64 leaves: a plain search for the two lightest will do)
            std::sort(alive.begin(), alive.end(), [&](int a, int b) { return nodes[a].w != nodes[b].w ? nodes[a].w > nodes[b].w : a > b; });
            const int a = alive.back();
            alive.pop_back();
            const int b = alive.back();
            alive.pop_back();
            nodes.push_back({nodes[a].w + nodes[b].w, a, b});
            alive.push_back((int)nodes.size() - 1);
        }
        int deepest = 0;
        std::vector<std::pair<int, int>> stack{{alive[0], 0}};
        while (!stack.empty()) {
            const auto [id, depth] = stack.back();
            stack.pop_back();
            if (nodes[id].left < 0) {
                len[-1 - nodes[id].left] = depth;
                deepest = std::max(deepest, depth);
            } else {
                stack.push_back({nodes[id].left, depth + 1});
                stack.push_back({nodes[id].right, depth + 1});
            }
        }
        if (deepest <= max_len) return;
        for (int i = 0; i < PFX_CLASSES; ++i)
            if (f[i] > 0) f[i] = (f[i] + 1) / 2;
    }
}

// The device table of a group (see above) from its code lengths: canonical codes, shorter first, reversed
// so that a code's first bit is the lowest.
static void pfx_make_table(const int (&len)[PFX_CLASSES], int direct_none, uint8_t* tab) {
    uint16_t* lut = reinterpret_cast<uint16_t*>(tab);
    uint32_t* cls = reinterpret_cast<uint32_t*>(tab + PFX_LUT * sizeof(uint16_t));
    uint32_t* enc = cls + PFX_CLASSES;
    memset(tab, 0, PFX_TAB_BYTES);
    uint32_t code = 0;
    for (int l = 1; l <= PFX_MAXLEN; ++l) {
        for (int c = 0; c < PFX_CLASSES; ++c) {
            if (len[c] != l) continue;
            uint32_t rev = 0;
            for (int b = 0; b < l; ++b) rev |= ((code >> b) & 1u) << (l - 1 - b);
            enc[c] = rev | ((uint32_t)l << 16);
            for (uint32_t hi = 0; hi < (1u << (PFX_MAXLEN - l)); ++hi) lut[rev | (hi << l)] = (uint16_t)((c << 4) | l);
            ++code;
        }
        code <<= 1;
    }
    for (int c = 0; c < PFX_CLASSES; ++c) {
        uint32_t base, eb = 0;
        if (direct_none >= 0) base = c == direct_none ? 0xFFFFu : (uint32_t)c;
        else if (c == PFX_NONE_CLASS) base = 0xFFFFu;
        else if (c < 7) base = (uint32_t)c;
        else {
            const uint32_t b = 3u + (uint32_t)(c - 7) / 4u, f = (uint32_t)(c - 7) % 4u;
            eb = b - 2u;
            base = ((4u + f) << eb) - 1u;
        }
        cls[c] = (base & 0xFFFFu) | (eb << 16);
    }
}

// bit (r & 7) of byte (r >> 3) = 1 when y[r] < 0
__global__ void k_label_bits(const float* __restrict__ y, int64_t n, uint8_t* __restrict__ bits, int64_t n_bytes) {
    for (int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; b < n_bytes; b += (int64_t)gridDim.x * blockDim.x) {
        uint32_t w = 0;
        for (int j = 0; j < 8; ++j) {
            const int64_t r = 8 * b + j;
            if (r < n && y[r] < 0.0f) w |= 1u << j;
        }
        bits[b] = (uint8_t)w;
    }
}

void grouped_free(snap_handle* h) {
    if (h->ev_group) {
        for (int64_t i = 0; i < 2 * (h->n_groups + 1); ++i)
            if (h->ev_group[i]) (void)hipEventDestroy(h->ev_group[i]);
        delete[] h->ev_group;
        h->ev_group = nullptr;
    }
    if (h->gev_prof) {
        for (int64_t i = 0; i < 4 * (h->n_groups + 1); ++i)
            if (h->gev_prof[i]) (void)hipEventDestroy(h->gev_prof[i]);
        delete[] h->gev_prof;
        h->gev_prof = nullptr;
    }
    for (int b = 0; b < 3; ++b) {
        (void)hipFree(h->gring[b]);
        (void)hipFree(h->gring8[b]);
        h->gring[b] = nullptr;
        h->gring8[b] = nullptr;
        if (h->gev_copied[b]) (void)hipEventDestroy(h->gev_copied[b]);
        if (h->gev_free[b]) (void)hipEventDestroy(h->gev_free[b]);
        h->gev_copied[b] = h->gev_free[b] = nullptr;
    }
    if (h->gmaps_host) (void)hipHostFree(h->gmaps_host);
    h->gmaps_host = nullptr;
    delete[] h->gmap8_host;
    delete[] h->gmap_off_host;
    delete[] h->gpfx_words_host;
    h->gmap8_host = nullptr;
    h->gmap_off_host = nullptr;
    h->gpfx_words_host = nullptr;
    (void)hipFree(h->gpfx_tab);
    h->gpfx_tab = nullptr;
    delete[] h->gbounds_host;
    delete[] h->ghot_host;
    delete[] h->gk64_host;
    delete[] h->gcompact_host;
    h->gcompact_host = nullptr;
    (void)hipFree(h->gwbase);
    (void)hipFree(h->gcidx);
    (void)hipFree(h->gcptr);
    (void)hipFree(h->gcbuf);
    h->gwbase = h->gcidx = nullptr;
    h->gcptr = nullptr;
    h->gcbuf = nullptr;
    h->gbounds_host = nullptr;
    h->ghot_host = nullptr;
    h->gk64_host = nullptr;
    (void)hipFree(h->rowmap);
    (void)hipFree(h->rowmap8);
    h->rowmap8 = nullptr;
    delete[] h->g8slot_host;
    h->g8slot_host = nullptr;
    h->n_byte_maps = 0;
    (void)hipFree(h->rowval);
    (void)hipFree(h->ybits);
    h->ybits = nullptr;
    (void)hipFree(h->rank_of);
    (void)hipFree(h->coord_of);
    (void)hipFree(h->gdelta);
    (void)hipFree(h->gpartial);
    (void)hipFree(h->gloss_partial);
    h->gloss_partial = nullptr;
    h->rowmap = nullptr;
    h->rowval = nullptr;
    h->rank_of = h->coord_of = nullptr;
    h->gdelta = nullptr;
    h->gpartial = nullptr;
}

// ---- finding the groups ---------------------------------------------------------------------------------
// Greedy cut of the coordinates into the fewest ranges of consecutive coordinates whose members share
// no row (for one-hot encoded data: the fields).  A range is grown by galloping: a candidate block of
// further coordinates is accepted when marking its rows with a fresh tag meets no row already
// marked by the range or by the block itself; after the first refusal the block size is halved
// until the exact end of the range is known.  Tags of refused blocks stay behind and are ignored
// (ok[] says which tags of the current range were accepted), so nothing is ever cleared and every
// nonzero is visited about twice.
__global__ void k_mark_rows(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, int64_t nnz_base, int64_t c0,
                            int64_t c1, int64_t n, uint32_t tag, uint32_t tag_lo, const uint8_t* __restrict__ ok,
                            uint32_t* __restrict__ tags, uint32_t* __restrict__ conflict) {
    // (idx holds the nonzeros from nnz_base on; an index outside [0, n) is skipped here: creation reports it)
    const int64_t k0 = ptr[c0], k1 = ptr[c1];
    bool bad = false;
    for (int64_t k = k0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < k1; k += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t r = idx[k - nnz_base] & ~LABEL_BIT;
        if ((int64_t)r >= n) continue;
        const uint32_t seen = tags[r];
        if (seen >= tag_lo && seen < tag && ok[seen - tag_lo]) {
            bad = true;                                   // the row belongs to the range already
        } else if (atomicExch(tags + r, tag) == tag) {
            bad = true;                                   // two coordinates of the block share the row
        }
    }
    if (bad) atomicOr(conflict, 1u);
}

// The search as a state that can be advanced piece by piece: resident data in one go, streamed data chunk by
// chunk as the chunks pass through the device during creation (a block of candidates never reaches beyond
// the chunk at hand; the end of a range, the first coordinate that shares a row with an earlier one of the
// range, does not depend on how the blocks were cut).
struct GroupSearch {
    static constexpr int MAX_TESTS = 128;                 // per range: 2 log2(range length) is needed
    uint32_t* tags = nullptr;
    uint32_t* conflict = nullptr;
    uint8_t* ok = nullptr;
    uint32_t* host_flag = nullptr;
    uint8_t ok_host[MAX_TESTS];
    uint32_t tag = 1, tag_lo = 1;                         // 0: never marked
    int tests = 0;
    int64_t start = 0, end = 0, step = 1;
    bool refused = false, gave_up = false;
    std::vector<int64_t> gb{0};
};

void group_search_free(GroupSearch* s) {
    if (!s) return;
    (void)hipFree(s->tags);
    (void)hipFree(s->conflict);
    (void)hipFree(s->ok);
    (void)hipHostFree(s->host_flag);
    delete s;
}

static int search_open_range(snap_handle* h, GroupSearch& s) {
    s.tag_lo = s.tag;
    s.tests = 0;
    memset(s.ok_host, 0, sizeof(s.ok_host));
    SNAP_HIP(hipMemsetAsync(s.ok, 0, GroupSearch::MAX_TESTS, h->compute));
    s.end = s.start;
    s.step = 1;
    s.refused = false;
    return SNAP_OK;
}

int group_search_begin(snap_handle* h, GroupSearch** out) {
    *out = nullptr;
    GroupSearch* s = new (std::nothrow) GroupSearch();
    if (!s) return SNAP_ENOMEM;
    *out = s;                                             // (freed by the caller, also after a failure below)
    SNAP_HIP(hipMalloc(&s->tags, (size_t)(h->n ? h->n : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&s->conflict, sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&s->ok, GroupSearch::MAX_TESTS));
    SNAP_HIP(hipHostMalloc(&s->host_flag, sizeof(uint32_t)));
    SNAP_TRY(fill_zero(s->tags, (size_t)h->n * sizeof(uint32_t), h->compute));
    return search_open_range(h, *s);
}

// The range under way is complete: note its end, apply the give-up rule, open the next one.
static int search_close_range(snap_handle* h, GroupSearch& s, const int64_t* hptr) {
    if (s.end == s.start) {                               // a coordinate with a repeated row: no structure to use
        s.gave_up = true;
        return SNAP_OK;
    }
    s.gb.push_back(s.end);
    s.start = s.end;
    // give up early on data without such structure: a range pays one pass over all rows, which is
    // only worth it when the range holds a good fraction of a nonzero per row
    const double covered = (double)hptr[s.end] / (double)h->n;
    if ((double)(s.gb.size() - 1) > 8.0 + 10.0 * covered) {
        s.gave_up = true;
        return SNAP_OK;
    }
    return search_open_range(h, s);
}

// Advance over the coordinates up to c_limit, whose nonzeros sit in idx (from nnz_base on).
int group_search_advance(snap_handle* h, GroupSearch* sp, const int64_t* hptr, const uint32_t* idx, int64_t nnz_base,
                         int64_t c_limit) {
    GroupSearch& s = *sp;
    while (!s.gave_up && s.end < c_limit) {
        if (s.step == 0 || s.tests >= GroupSearch::MAX_TESTS) {
            SNAP_TRY(search_close_range(h, s, hptr));
            continue;
        }
        const int64_t to = std::min(c_limit, s.end + s.step);
        bool good = true;
        if (hptr[to] > hptr[s.end]) {
            const int64_t cnt = hptr[to] - hptr[s.end];
            const int grid = (int)std::min<int64_t>((cnt + 255) / 256, 16384);
            SNAP_HIP(hipMemsetAsync(s.conflict, 0, sizeof(uint32_t), h->compute));
            hipLaunchKernelGGL(k_mark_rows, dim3(grid), dim3(256), 0, h->compute, h->ptr, idx, nnz_base, s.end, to, h->n, s.tag,
                               s.tag_lo, s.ok, s.tags, s.conflict);
            SNAP_HIP(hipMemcpyAsync(s.host_flag, s.conflict, sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
            SNAP_HIP(hipStreamSynchronize(h->compute));
            good = *s.host_flag == 0;
            if (good) {
                s.ok_host[s.tag - s.tag_lo] = 1;
                SNAP_HIP(hipMemcpyAsync(s.ok + (s.tag - s.tag_lo), s.ok_host + (s.tag - s.tag_lo), 1, hipMemcpyHostToDevice,
                                        h->compute));
            }
            ++s.tag;
            ++s.tests;
        }
        if (good) {
            s.end = to;
            s.step = s.refused ? s.step / 2 : s.step * 2;
        } else {
            s.refused = true;
            s.step /= 2;
        }
    }
    return SNAP_OK;
}

// After the last coordinate: the ranges found, or nothing when the search gave up.
int group_search_end(snap_handle* h, GroupSearch* sp, const int64_t* hptr, std::vector<int64_t>& bounds) {
    GroupSearch& s = *sp;
    bounds.clear();
    SNAP_HIP(hipStreamSynchronize(h->compute));
    if (!s.gave_up && s.gb.back() != h->m) {
        s.end = h->m;
        SNAP_TRY(search_close_range(h, s, hptr));
        SNAP_HIP(hipStreamSynchronize(h->compute));
    }
    if (!s.gave_up) bounds = s.gb;
    return SNAP_OK;
}

// bounds: empty when the data have no such structure worth using (see the give-up rule above).
int detect_groups(snap_handle* h, const int64_t* hptr, std::vector<int64_t>& bounds) {
    bounds.clear();
    const int64_t m = h->m, n = h->n;
    if (h->form != SNAP_PRIMAL || h->dense || h->streaming || m < 2 || n < 1 || h->nnz < 1) return SNAP_OK;
    GroupSearch* s = nullptr;
    int rc = group_search_begin(h, &s);
    if (rc == SNAP_OK) rc = group_search_advance(h, s, hptr, h->idx, 0, m);
    if (rc == SNAP_OK) rc = group_search_end(h, s, hptr, bounds);
    (void)hipStreamSynchronize(h->compute);
    group_search_free(s);
    SNAP_TRY(rc);
    if (bounds.empty()) return SNAP_OK;
    size_t free_b = 0, total_b = 0;
    SNAP_HIP(hipMemGetInfo(&free_b, &total_b));
    const size_t n_pad = (size_t)((n + 7) / 8 * 8);
    if ((bounds.size() - 1) * n_pad * 6 > free_b / 2) bounds.clear();      // the row maps would not fit comfortably
    return SNAP_OK;
}

static int cold_setup(snap_handle* h, const int64_t* hptr, const std::vector<uint32_t>& coord_of);
static int streamed_setup(snap_handle* h, const int64_t* hptr, const std::vector<uint32_t>& coord_of);

// The terms of the logistic loss enter the sums with a resolution of 2^-20 (loss') and 2^-23 (loss'') of
// the largest |value| a (squared for loss'').  That is far below fp32 rounding of the sums themselves unless
// the curvature sum of a coordinate is tiny and lambda n is tiny too (rows that the model separates
// perfectly: the step is g / (h + lambda n)): up to 4095 rounded terms are off by about 64 * 2^-24 a^2 in
// total, which stays below 1e-4 of the denominator when lambda n >= a^2 / 16.  Below that the group
// sweeps are declined and the handle runs the asynchronous engine.
static bool resolution_too_coarse(const snap_handle* h, int scale_exp) {
    // (the largest |value| lies in (2^(scale_exp - 1), 2^scale_exp])
    return h->kind == K_PRIMAL_LOGISTIC && h->lambda * (double)h->n < ldexp(1.0, 2 * scale_exp - 6);
}

int grouped_setup(snap_handle* h, const int64_t* hptr, const int64_t* gb, int64_t G) {
    const int64_t m = h->m, n = h->n;
    if (h->form != SNAP_PRIMAL || h->dense) {
        set_error("group sweeps need the primal form on sparse data");
        return SNAP_EUNSUPPORTED;
    }
    if (h->streaming && !h->stream_unit) {
        set_error("group sweeps on streamed data need all stored values to be 1 (pattern-only data)");
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
    h->gbounds_host = new (std::nothrow) int64_t[(size_t)G + 1];
    h->ghot_host = new (std::nothrow) int[(size_t)G];
    h->gk64_host = new (std::nothrow) int[(size_t)G];
    if (!h->gbounds_host || !h->ghot_host || !h->gk64_host) return SNAP_ENOMEM;
    std::copy(gb, gb + G + 1, h->gbounds_host);

    int lds_max = 0;
    SNAP_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device));
    // (the ridge loss has one sum per rank to begin with: 8 bytes each, nothing to pack)
    h->gpack = pack_knob();
    h->g_kd_max = DELTA_DEFAULT / wgs_per_cu();
    if (const char* e = getenv("SNAP_DELTA_LDS")) h->g_kd_max = std::max(1, std::min(DELTA_LDS, atoi(e)));   // tuning knob
    h->g_row_wgs = row_wgs_knob() > 0 ? row_wgs_knob() : wgs_per_cu() * ROW_WGS_DEFAULT;
    const int hot_cap = hot_max(), min_rows = hot_min_rows();
    const int ring_bytes = compact_knob() ? (ROW_TPB / WAVE) * COLD_RING * (int)sizeof(float) : 0;
    const int lds_budget = lds_max / wgs_per_cu() - 1024 - 4 * h->g_kd_max - ring_bytes;   // bytes for the sums
    // ranks inside each group: coordinates by decreasing length (ties by index)
    std::vector<uint32_t> rank_of((size_t)m), coord_of((size_t)m);
    int max_words = 2;
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
        // hot ranks: accumulated in LDS by the row pass; a rank is worth a slot (and its share of
        // every workgroup's partial array) while its coordinate has a few dozen rows
        // ... and of those, the first k64 keep two 64-bit words (too many rows for a packed word; ranks 0
        // and 1, which the row pass sums in registers, always do), the others one
        auto rows_of = [&](int r) { return hptr[order[(size_t)r] + 1] - hptr[order[(size_t)r]]; };
        int hot = 0, k64 = 0;
        while (hot < sz && hot < hot_cap && rows_of(hot) >= min_rows) {
            const bool two_words = h->kind == K_PRIMAL_LOGISTIC && (!h->gpack || hot < 2 || rows_of(hot) > PACK_COUNT_MAX);
            if (8 * (hot + 1 + k64 + (two_words ? 1 : 0)) > lds_budget) break;
            k64 += two_words ? 1 : 0;
            ++hot;
        }
        h->ghot_host[g] = hot;
        h->gk64_host[g] = k64;
        max_words = std::max(max_words, hot + k64);
    }
    h->gpartial_stride = (int64_t)max_words;

    h->map16 = true;
    for (int64_t g = 0; g < G; ++g)
        if (gb[g + 1] - gb[g] > 65535) h->map16 = false;
    h->n_pad = (n + 7) / 8 * 8;
    SNAP_HIP(hipMalloc(&h->rank_of, (size_t)(m ? m : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->coord_of, (size_t)(m ? m : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->gdelta, (size_t)(m ? m : 1) * sizeof(float)));
    SNAP_HIP(hipMalloc(&h->gpartial, (size_t)h->g_row_wgs * (size_t)h->gpartial_stride * sizeof(long long)));
    SNAP_HIP(hipMalloc(&h->gloss_partial, (size_t)h->g_row_wgs * 3 * sizeof(double)));
    SNAP_HIP(hipMalloc(&h->ybits, (size_t)(h->n_pad / 8 + 16)));
    SNAP_HIP(hipMemcpyAsync(h->rank_of, rank_of.data(), (size_t)m * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
    SNAP_HIP(hipMemcpyAsync(h->coord_of, coord_of.data(), (size_t)m * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
    SNAP_TRY(fill_zero(h->gdelta, (size_t)m * sizeof(float), h->compute));
    hipLaunchKernelGGL(k_label_bits, dim3(4096), dim3(256), 0, h->compute, h->y, n, h->ybits, h->n_pad / 8);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipStreamSynchronize(h->compute));     // (the host tables above are read by the copies)
    if (h->opt.profile) {
        h->ev_group = new (std::nothrow) hipEvent_t[(size_t)(2 * (G + 1))]();
        if (!h->ev_group) return SNAP_ENOMEM;
        for (int64_t i = 0; i < 2 * (G + 1); ++i) SNAP_HIP(hipEventCreate(&h->ev_group[i]));
        h->pass_timed.assign((size_t)(G + 1), 0);
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
    if (h->streaming) {
        if (resolution_too_coarse(h, 1)) {               // (pattern-only data: the largest value is 1 <= 2^1)
            grouped_free(h);
            h->n_groups = 0;
            return SNAP_OK;
        }
        const int rc = streamed_setup(h, hptr, coord_of);
        if (rc == SNAP_ENOMEM && h->gmaps_host == nullptr && h->gring[0] == nullptr) {   // no pinned memory for the maps
            grouped_free(h);
            h->n_groups = 0;
            h->gstream = false;
            return SNAP_OK;                              // declined: asynchronous engine on streamed column chunks
        }
        SNAP_TRY(rc);
        h->grouped = true;
        return SNAP_OK;
    }

    const size_t map_count = (size_t)G * (size_t)h->n_pad;
    int64_t* d_gb = nullptr;
    uint32_t* flags = nullptr;
    uint32_t* wide = nullptr;
    SNAP_HIP(hipMalloc(&d_gb, (size_t)(G + 1) * sizeof(int64_t)));
    SNAP_HIP(hipMalloc(&flags, 2 * sizeof(uint32_t)));
    auto fail = [&](int rc) {
        (void)hipFree(d_gb);
        (void)hipFree(flags);
        (void)hipFree(wide);
        return rc;
    };
#define G_HIP(call)                                                                \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) return fail(hip_fail(e_, #call, __FILE__, __LINE__)); \
    } while (0)
    G_HIP(hipMemcpyAsync(d_gb, gb, (size_t)(G + 1) * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
    int rc = fill_zero(flags, 8, h->compute);
    if (rc != SNAP_OK) return fail(rc);
    // values: all ones (no per-row value arrays) or not, and their largest magnitude
    uint32_t fl2[2] = {0, 0};
    if (h->nnz > 0) hipLaunchKernelGGL(k_value_stats, dim3(4096), dim3(256), 0, h->compute, h->val, h->nnz, flags);
    G_HIP(hipMemcpyAsync(fl2, flags, 8, hipMemcpyDeviceToHost, h->compute));
    G_HIP(hipStreamSynchronize(h->compute));
    h->unit_values = !(fl2[0] & 2u);
    {
        float amax;
        memcpy(&amax, &fl2[1], 4);
        int e = 0;
        if (amax > 0.0f) (void)frexpf(amax, &e);     // amax <= 2^e
        h->gscale_exp = e;
    }
    if (resolution_too_coarse(h, h->gscale_exp)) {
        (void)fail(SNAP_OK);
        grouped_free(h);
        h->n_groups = 0;
        return SNAP_OK;
    }
    if (!h->unit_values) {
        G_HIP(hipMalloc(&h->rowval, map_count * sizeof(float)));
        rc = fill_zero(h->rowval, map_count * sizeof(float), h->compute);
        if (rc != SNAP_OK) return fail(rc);
    }
    // 32-bit map first (compare-and-swap per nonzero), narrowed to 16 bits afterwards when possible
    G_HIP(hipMalloc(&wide, map_count * sizeof(uint32_t)));
    hipLaunchKernelGGL(k_fill_u32, dim3(8192), dim3(256), 0, h->compute, wide, map_count, RANK_NONE);
    if (h->nnz > 0)
        hipLaunchKernelGGL(k_build_rowmap, dim3((unsigned)((h->nnz + 4095) / 4096)), dim3(256), 0, h->compute, h->ptr,
                           h->idx, h->val, m, h->nnz, d_gb, G, h->rank_of, h->n_pad, wide, h->rowval, flags);
    if (h->map16) {
        G_HIP(hipMalloc(&h->rowmap, map_count * sizeof(uint16_t)));
        hipLaunchKernelGGL(k_narrow_map, dim3(8192), dim3(256), 0, h->compute, wide, (uint16_t*)h->rowmap, map_count);
    }
    G_HIP(hipGetLastError());
    G_HIP(hipMemcpyAsync(fl2, flags, 8, hipMemcpyDeviceToHost, h->compute));
    G_HIP(hipStreamSynchronize(h->compute));
#undef G_HIP
    (void)hipFree(d_gb);
    (void)hipFree(flags);
    if (h->map16) (void)hipFree(wide);
    else h->rowmap = wide;
    if (fl2[0] & 1u) {
        set_error("two coordinates of one group share a row: the groups are not disjoint");
        return SNAP_EINVAL;
    }
    // groups of at most 255 coordinates: the row passes read their maps as bytes (a byte less per row and map)
    h->g8slot_host = new (std::nothrow) int[(size_t)G];
    if (!h->g8slot_host) return SNAP_ENOMEM;
    for (int64_t g = 0; g < G; ++g) {
        const int64_t sz = gb[g + 1] - gb[g];
        h->g8slot_host[g] = (h->map16 && map8_knob() && sz > 0 && sz <= 255 && n > 0) ? h->n_byte_maps++ : -1;
    }
    if (h->n_byte_maps > 0) {
        SNAP_HIP(hipMalloc(&h->rowmap8, (size_t)h->n_byte_maps * (size_t)h->n_pad));
        for (int64_t g = 0; g < G; ++g)
            if (h->g8slot_host[g] >= 0)
                hipLaunchKernelGGL(k_map16_to_8, dim3(8192), dim3(256), 0, h->compute, (const uint16_t*)h->rowmap + (size_t)g * h->n_pad,
                                   h->rowmap8 + (size_t)h->g8slot_host[g] * h->n_pad, (size_t)h->n_pad);
        SNAP_HIP(hipGetLastError());
    }
    rc = cold_setup(h, hptr, coord_of);
    if (rc != SNAP_OK) return rc;
    h->grouped = true;
    return SNAP_OK;
}

// ---- the row pass ------------------------------------------------------------------------------------
// SCATTER: v[r] += delta_prev[rank] * a for the previous group.  HIST: sums of the current group's
// hot ranks.  Every thread takes one 128-bit load of each map per iteration: 8 consecutive rows with
// 16-bit maps, 4 with 32-bit maps.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <typename MAPT> struct MapTraits;
template <> struct MapTraits<uint8_t> { static constexpr int R = 8; static constexpr uint32_t NONE = 0xFFu; typedef u32x2 Raw; };
template <> struct MapTraits<uint16_t> { static constexpr int R = 8; static constexpr uint32_t NONE = 0xFFFFu; typedef u32x4 Raw; };
template <> struct MapTraits<uint32_t> { static constexpr int R = 4; static constexpr uint32_t NONE = 0xFFFFFFFFu; typedef u32x4 Raw; };

// Ridge terms a (v - y) have no a-priori bound and take the 64-bit conversion to fixed point.  With 24
// fractional bits the 64-bit sum of a ridge coordinate has 2^39 of range: every term must stay below 2^14
// for up to 2^25 rows; larger terms raise the handle's status word instead of overflowing silently.
constexpr float RIDGE_TERM_LIMIT = 16384.0f;

// One 128-bit load of map entries (non-temporal: the maps are read once per pass and should not push the
// shared vector out of the last-level cache; the shared vector itself is read with plain loads: with the
// hint on those too the pass was measured 12 % slower), and its unpacking into ranks.
__device__ __forceinline__ u32x4 load_map(const uint16_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
__device__ __forceinline__ u32x4 load_map(const uint32_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
__device__ __forceinline__ u32x2 load_map(const uint8_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)); }
__device__ __forceinline__ void unpack_ranks(const uint8_t*, u32x2 u, uint32_t (&out)[8]) {
    out[0] = u.x & 0xFFu; out[1] = u.x >> 8 & 0xFFu; out[2] = u.x >> 16 & 0xFFu; out[3] = u.x >> 24;
    out[4] = u.y & 0xFFu; out[5] = u.y >> 8 & 0xFFu; out[6] = u.y >> 16 & 0xFFu; out[7] = u.y >> 24;
}
__device__ __forceinline__ void unpack_ranks(const uint16_t*, u32x4 u, uint32_t (&out)[8]) {
    out[0] = u.x & 0xFFFFu; out[1] = u.x >> 16; out[2] = u.y & 0xFFFFu; out[3] = u.y >> 16;
    out[4] = u.z & 0xFFFFu; out[5] = u.z >> 16; out[6] = u.w & 0xFFFFu; out[7] = u.w >> 16;
}
__device__ __forceinline__ void unpack_ranks(const uint32_t*, u32x4 u, uint32_t (&out)[4]) {
    out[0] = u.x; out[1] = u.y; out[2] = u.z; out[3] = u.w;
}

template <int R>
__device__ __forceinline__ void load_floats(const float* p, float (&out)[R]) {
#pragma unroll
    for (int q = 0; q < R / 4; ++q) {
        const float4 t = *reinterpret_cast<const float4*>(p + 4 * q);
        out[4 * q] = t.x; out[4 * q + 1] = t.y; out[4 * q + 2] = t.z; out[4 * q + 3] = t.w;
    }
}

// ---- short coordinates: a dense buffer of their rows' shared-vector entries ------------------------------
// A coordinate too short for an LDS slot takes its sums column-wise in the finishing kernel.  Gathering
// its rows' entries straight from the shared vector fetches a whole cache line per nonzero (the rows of
// all short coordinates of a group are a few percent of the rows, about one per line).  Instead the row
// pass, which streams the shared vector anyway, writes the entries of these rows densely into a small
// buffer, in the order in which it visits them -- workgroup, wavefront, iteration, row of the thread's
// pack, lane -- and the finishing kernel gathers from that buffer (a few MB, served by the L2).  The
// order is fixed by the launch shape, so the buffer position of every row is found once, at creation, by
// two passes that mirror the row pass: one counts per wavefront, one (after a prefix sum on the host)
// numbers the rows.
__device__ __forceinline__ uint32_t cold_slot(bool cold, uint32_t& run) {
    const unsigned long long mask = __builtin_amdgcn_ballot_w64(cold);
    const uint32_t pos = run + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
    run += (uint32_t)__popcll(mask);
    return pos;
}

// WRITE = false: slots[wavefront] <- number of rows with a rank >= hot; WRITE = true: slots holds the
// first position of every wavefront and rowpos[row] <- position, for those rows.
template <typename MAPT, bool WRITE>
__global__ void __launch_bounds__(ROW_TPB)
k_cold_rows(const MAPT* __restrict__ map, int hot, int64_t n, uint32_t* __restrict__ slots, uint32_t* __restrict__ rowpos) {
    constexpr int R = MapTraits<MAPT>::R;
    constexpr uint32_t NONE = MapTraits<MAPT>::NONE;
    const int wave = (int)blockIdx.x * (ROW_TPB / WAVE) + (int)threadIdx.x / WAVE;
    uint32_t run = WRITE ? slots[wave] : 0u;
    const int64_t packs = (n + R - 1) / R;                     // (the same walk over the rows as in the row pass)
    for (int64_t q = (int64_t)blockIdx.x * ROW_TPB + threadIdx.x; q < packs; q += (int64_t)gridDim.x * ROW_TPB) {
        uint32_t mc[R];
        unpack_ranks(map, load_map(map + R * q), mc);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const bool cold = mc[j] >= (uint32_t)hot && mc[j] != NONE;
            const uint32_t pos = cold_slot(cold, run);
            if (WRITE && cold) rowpos[R * q + j] = pos;
        }
    }
    // (the first lane holds the wavefront's lowest pack: no lane runs more iterations)
    if (!WRITE && (threadIdx.x & (WAVE - 1)) == 0) slots[wave] = run;
}

// cidx[start of the rank + i] <- buffer position of the row of the coordinate's i-th nonzero (the label
// bit of the row index, when there is one, is carried along); one wavefront per coordinate.
__global__ void __launch_bounds__(256)
k_cold_index(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, int64_t nnz_base,
             const uint32_t* __restrict__ coord_of, const int64_t* __restrict__ cptr, int64_t g0, int hot,
             int64_t group_size, uint32_t label_mask, const uint32_t* __restrict__ rowpos, uint32_t* __restrict__ cidx) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const int64_t nwaves = (int64_t)gridDim.x * blockDim.x / WAVE;
    for (int64_t rk = hot + wave0; rk < group_size; rk += nwaves) {
        const int64_t c = coord_of[g0 + rk], p0 = ptr[c], len = ptr[c + 1] - p0, k0 = cptr[g0 + rk];
        for (int64_t i = lane; i < len; i += WAVE) {
            const uint32_t e = idx[p0 + i - nnz_base];       // (idx holds the nonzeros from nnz_base on)
            cidx[k0 + i] = rowpos[e & ~label_mask] | (e & label_mask);
        }
    }
}

template <typename MAPT>
static int cold_setup_maps(snap_handle* h, const std::vector<int64_t>& cold_rows, const std::vector<int64_t>& cptr, int64_t total) {
    const int64_t G = h->n_groups, m = h->m, n = h->n;
    const int nwaves = h->g_row_wgs * (ROW_TPB / WAVE);
    const MAPT* maps = (const MAPT*)h->rowmap;
    const int64_t most = *std::max_element(cold_rows.begin(), cold_rows.end());
    uint32_t* rowpos = nullptr;
    auto fail = [&](int rc) {
        (void)hipFree(rowpos);
        return rc;
    };
#define C_HIP(call)                                                                \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) return fail(hip_fail(e_, #call, __FILE__, __LINE__)); \
    } while (0)
    C_HIP(hipMalloc(&h->gwbase, (size_t)G * (size_t)nwaves * sizeof(uint32_t)));
    C_HIP(hipMalloc(&h->gcptr, (size_t)(m + 1) * sizeof(int64_t)));
    C_HIP(hipMalloc(&h->gcidx, (size_t)total * sizeof(uint32_t)));
    C_HIP(hipMalloc(&h->gcbuf, (size_t)most * sizeof(float)));
    C_HIP(hipMalloc(&rowpos, (size_t)h->n_pad * sizeof(uint32_t)));
    C_HIP(hipMemcpyAsync(h->gcptr, cptr.data(), (size_t)(m + 1) * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
    int rc = fill_zero(h->gwbase, (size_t)G * (size_t)nwaves * sizeof(uint32_t), h->compute);
    if (rc == SNAP_OK) rc = fill_zero(rowpos, (size_t)h->n_pad * sizeof(uint32_t), h->compute);   // (every entry a valid position)
    if (rc != SNAP_OK) return fail(rc);
    for (int64_t g = 0; g < G; ++g)
        if (h->gcompact_host[g])
            hipLaunchKernelGGL((k_cold_rows<MAPT, false>), dim3((unsigned)h->g_row_wgs), dim3(ROW_TPB), 0, h->compute,
                               maps + (size_t)g * h->n_pad, h->ghot_host[g], n, h->gwbase + (size_t)g * nwaves, (uint32_t*)nullptr);
    C_HIP(hipGetLastError());
    std::vector<uint32_t> slots((size_t)G * (size_t)nwaves);
    C_HIP(hipMemcpyAsync(slots.data(), h->gwbase, slots.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
    C_HIP(hipStreamSynchronize(h->compute));
    for (int64_t g = 0; g < G; ++g) {
        if (!h->gcompact_host[g]) continue;
        uint64_t sum = 0;
        for (int w = 0; w < nwaves; ++w) {
            uint32_t& sl = slots[(size_t)g * nwaves + w];
            const uint32_t count = sl;
            sl = (uint32_t)sum;
            sum += count;
        }
        if ((int64_t)sum != cold_rows[(size_t)g]) {          // the row maps and the column lengths disagree
            set_error("internal error: the rows of the short coordinates do not add up");
            return fail(SNAP_ESTATE);
        }
    }
    C_HIP(hipMemcpyAsync(h->gwbase, slots.data(), slots.size() * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
    const uint32_t label_mask = h->kind == K_PRIMAL_LOGISTIC ? LABEL_BIT : 0u;
    for (int64_t g = 0; g < G; ++g) {
        if (!h->gcompact_host[g]) continue;
        const int64_t g0 = h->gbounds_host[g], sz = h->gbounds_host[g + 1] - g0;
        const int hot = h->ghot_host[g];
        hipLaunchKernelGGL((k_cold_rows<MAPT, true>), dim3((unsigned)h->g_row_wgs), dim3(ROW_TPB), 0, h->compute,
                           maps + (size_t)g * h->n_pad, hot, n, h->gwbase + (size_t)g * nwaves, rowpos);
        const int blocks = (int)std::min<int64_t>((sz - hot + 3) / 4, 16384);
        hipLaunchKernelGGL(k_cold_index, dim3((unsigned)blocks), dim3(256), 0, h->compute, h->ptr, h->idx, (int64_t)0, h->coord_of,
                           h->gcptr, g0, hot, sz, label_mask, rowpos, h->gcidx);
    }
    C_HIP(hipGetLastError());
    C_HIP(hipStreamSynchronize(h->compute));
#undef C_HIP
    (void)hipFree(rowpos);
    return SNAP_OK;
}

static int cold_setup(snap_handle* h, const int64_t* hptr, const std::vector<uint32_t>& coord_of) {
    const int64_t G = h->n_groups, m = h->m;
    h->gcompact_host = new (std::nothrow) uint8_t[(size_t)G]();
    if (!h->gcompact_host) return SNAP_ENOMEM;
    if (!compact_knob() || h->n == 0) return SNAP_OK;
    // start in the index array of every (group start + rank); only the ranks behind the hot ones of a
    // group that has hot ranks (whose row pass computes sums at all) own a stretch of it
    std::vector<int64_t> cptr((size_t)m + 1, 0), cold_rows((size_t)G, 0);
    int64_t total = 0;
    for (int64_t g = 0; g < G; ++g) {
        const int64_t g0 = h->gbounds_host[g], sz = h->gbounds_host[g + 1] - g0;
        const int hot = h->ghot_host[g];
        for (int64_t r = 0; r < sz; ++r) {
            cptr[(size_t)(g0 + r)] = total;
            if (hot > 0 && r >= hot) {
                const int64_t c = coord_of[(size_t)(g0 + r)];
                total += hptr[c + 1] - hptr[c];
                cold_rows[(size_t)g] += hptr[c + 1] - hptr[c];
            }
        }
        h->gcompact_host[g] = cold_rows[(size_t)g] > 0;
    }
    cptr[(size_t)m] = total;
    if (total == 0) return SNAP_OK;
    size_t free_b = 0, total_b = 0;
    SNAP_HIP(hipMemGetInfo(&free_b, &total_b));
    if (((size_t)total + (size_t)h->n_pad) * 4 + (size_t)(m + 1) * 8 > free_b / 2) {      // not worth the squeeze
        std::fill(h->gcompact_host, h->gcompact_host + G, (uint8_t)0);
        return SNAP_OK;
    }
    return h->map16 ? cold_setup_maps<uint16_t>(h, cold_rows, cptr, total) : cold_setup_maps<uint32_t>(h, cold_rows, cptr, total);
}

// ---- streamed data: the row maps are built group by group into pinned host memory ------------------------
// The matrix stays in the caller's pinned host memory (Section 3.2).  What an epoch of group sweeps
// reads per nonzero is not its 4-byte row index but the 1-2-byte row-map entry, so the library keeps
// the maps -- in pinned host memory of its own, built once at creation -- and streams those: a group's
// nonzeros are copied to a staging buffer, turned into the group's row map on the device, and the map
// is copied back to the host.  The index lists of the short coordinates (a few percent of the
// nonzeros) stay on the device.
__global__ void __launch_bounds__(256)
k_build_rowmap_group(const int64_t* __restrict__ ptr, const uint32_t* __restrict__ idx, int64_t k_lo, int64_t k_hi,
                     int64_t c_lo, int64_t c_hi, const uint32_t* __restrict__ rank_of, uint32_t* __restrict__ wide,
                     uint32_t* __restrict__ flags) {
    // idx holds the nonzeros [k_lo, k_hi) of the coordinates [c_lo, c_hi); one block per 4096 of them
    const int64_t b0 = k_lo + (int64_t)blockIdx.x * 4096, b1 = min(k_hi, b0 + 4096);
    int64_t lo = c_lo, hi = c_hi;                 // coordinate of the block's first nonzero
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr[mid] <= b0) lo = mid; else hi = mid;
    }
    const int64_t cstart = lo;
    for (int64_t k = b0 + threadIdx.x; k < b1; k += 256) {
        int64_t l = cstart, step = 1;
        while (l + step < c_hi && ptr[l + step] <= k) { l += step; step <<= 1; }
        int64_t r = min(c_hi, l + step);
        while (r - l > 1) {
            const int64_t mid = (l + r) >> 1;
            if (ptr[mid] <= k) l = mid; else r = mid;
        }
        const uint32_t row = idx[k - k_lo] & ~LABEL_BIT;
        if (atomicCAS(wide + row, RANK_NONE, rank_of[l]) != RANK_NONE) atomicOr(flags, 1u);
    }
}

template <typename MAPT>
static int streamed_setup_maps(snap_handle* h, const int64_t* hptr) {
    const int64_t G = h->n_groups, m = h->m, n = h->n;
    const int nwaves = h->g_row_wgs * (ROW_TPB / WAVE);
    // host-side plan of the short coordinates' index lists (as for resident data)
    h->gcompact_host = new (std::nothrow) uint8_t[(size_t)G]();
    if (!h->gcompact_host) return SNAP_ENOMEM;
    std::vector<int64_t> cptr((size_t)m + 1, 0), cold_rows((size_t)G, 0);
    std::vector<uint32_t> coord_of((size_t)m);
    SNAP_HIP(hipMemcpy(coord_of.data(), h->coord_of, (size_t)m * sizeof(uint32_t), hipMemcpyDeviceToHost));
    int64_t total = 0, most = 0, max_group_nnz = 0;
    for (int64_t g = 0; g < G; ++g) {
        const int64_t g0 = h->gbounds_host[g], g1 = h->gbounds_host[g + 1];
        const int hot = h->ghot_host[g];
        for (int64_t r = 0; r < g1 - g0; ++r) {
            cptr[(size_t)(g0 + r)] = total;
            if (r >= hot) {           // (also in a group without hot ranks: the column indices are not on the device)
                const int64_t c = coord_of[(size_t)(g0 + r)];
                total += hptr[c + 1] - hptr[c];
                cold_rows[(size_t)g] += hptr[c + 1] - hptr[c];
            }
        }
        h->gcompact_host[g] = cold_rows[(size_t)g] > 0;
        most = std::max(most, cold_rows[(size_t)g]);
        max_group_nnz = std::max(max_group_nnz, hptr[g1] - hptr[g0]);
    }
    cptr[(size_t)m] = total;
    if (max_group_nnz > h->n_pad) {               // more nonzeros than rows: some row is in two coordinates
        set_error("two coordinates of one group share a row: the groups are not disjoint");
        return SNAP_EINVAL;
    }
    if (total > 0 && !compact_knob()) {
        set_error("group sweeps on streamed data need the dense buffer of the short coordinates (SNAP_COMPACT=0 is set)");
        return SNAP_EUNSUPPORTED;
    }
    // How every group's map crosses the host link: 0 = as it is read (2 or 4 bytes per row), 1 = one byte per
    // row (at most 255 coordinates), 2 = escape-coded bytes (see k_esc_encode) when that is at least a
    // tenth shorter than two bytes per row.  The device buffers are padded to whole blocks of ESC_BLOCK rows.
    const int64_t n_esc = (h->n_pad + ESC_BLOCK - 1) / ESC_BLOCK * ESC_BLOCK, n_blk = n_esc / ESC_BLOCK;
    const size_t map_bytes = (size_t)h->n_pad * sizeof(MAPT);
    // 3 = prefix-coded (see k_pfx_decode) when that is another tenth shorter.
    h->gmap8_host = new (std::nothrow) uint8_t[(size_t)G]();
    h->gmap_off_host = new (std::nothrow) int64_t[(size_t)G + 1]();
    h->gpfx_words_host = new (std::nothrow) int64_t[(size_t)G]();
    if (!h->gmap8_host || !h->gmap_off_host || !h->gpfx_words_host) return SNAP_ENOMEM;
    std::vector<int64_t> escaped((size_t)G, 0);     // rows of the group whose rank does not fit a byte
    std::vector<uint8_t> pfx_tabs;                   // tables of the prefix-coded groups (all groups' slots, to keep the indexing plain)
    std::vector<int64_t> pfx_bits((size_t)G, 0);
    const int64_t n_sub = n_esc / PFX_SUB, n_blk2 = n_esc / PFX_BLOCK;
    int64_t land_bytes = 0;                          // largest byte-coded map: size of the landing buffers
    for (int64_t g = 0; g < G; ++g) {
        const int64_t g0 = h->gbounds_host[g], sz = h->gbounds_host[g + 1] - g0;
        for (int64_t r = ESC8; r < sz; ++r) {
            const int64_t c = coord_of[(size_t)(g0 + r)];
            escaped[(size_t)g] += hptr[c + 1] - hptr[c];
        }
        const int64_t blob = (n_esc + 4 * n_blk + 2 * escaped[(size_t)g] + 7) / 8 * 8;
        int mode = 0;
        int64_t bytes = (int64_t)map_bytes;
        if (sizeof(MAPT) == 2 && map8_knob()) {
            if (sz <= 255) mode = 1, bytes = h->n_pad;                              // ranks 0 .. 254, 255 = none
            else if (10 * blob <= 9 * (int64_t)map_bytes) mode = 2, bytes = blob;
        }
        if (sizeof(MAPT) == 2 && map8_knob() && pfx_knob() && sz > 0) {
            // class counts from the column lengths (the maps are built from the same columns), code, size
            const int direct_none = sz <= PFX_DIRECT_MAX ? (int)sz : -1;
            uint64_t count[PFX_CLASSES] = {};
            int64_t covered = 0, extra_bits = 0;
            for (int64_t r = 0; r < sz; ++r) {
                const int64_t c = coord_of[(size_t)(g0 + r)], rows = hptr[c + 1] - hptr[c];
                uint32_t extra, eb;
                count[pfx_class_of((uint32_t)r, direct_none, extra, eb)] += (uint64_t)rows;
                extra_bits += rows * (int64_t)eb;
                covered += rows;
            }
            uint32_t extra, eb;
            count[pfx_class_of(0xFFFFu, direct_none, extra, eb)] += (uint64_t)(n_esc - covered);     // rows outside the group, padding
            int len[PFX_CLASSES];
            pfx_code_lengths(count, PFX_MAXLEN, len);
            int64_t bits = extra_bits;
            for (int c = 0; c < PFX_CLASSES; ++c) bits += (int64_t)count[c] * len[c];
            const int64_t words = (bits + 31) / 32 + 2;
            const int64_t pfx_blob = (8 * n_blk2 + 4 * words + 2 * n_sub + 7) / 8 * 8;
            if (covered <= n_esc && 10 * pfx_blob <= 9 * bytes) {
                mode = 3, bytes = pfx_blob;
                pfx_bits[(size_t)g] = bits;
                h->gpfx_words_host[g] = words;
                if (pfx_tabs.empty()) pfx_tabs.assign((size_t)G * PFX_TAB_BYTES, 0);
                pfx_make_table(len, direct_none, pfx_tabs.data() + (size_t)g * PFX_TAB_BYTES);
            }
        }
        h->gmap8_host[g] = (uint8_t)mode;
        if (mode != 0) land_bytes = std::max(land_bytes, bytes);
        h->gmap_off_host[g + 1] = h->gmap_off_host[g] + (sz == 0 ? 0 : bytes);
    }
    h->gmap_bytes_per_pass = h->gmap_off_host[G];
    const bool refuse = getenv("SNAP_NO_PINNED_MAPS") != nullptr;      // (test hook: behave as if the allocation had failed)
    if (refuse || hipHostMalloc(&h->gmaps_host, (size_t)std::max<int64_t>(h->gmap_off_host[G], 8), hipHostMallocDefault) != hipSuccess) {
        // pinned host memory is a limited resource (the caller's matrix sits in it too): without room for
        // the maps the group sweeps are declined and the handle streams column chunks instead
        (void)hipGetLastError();
        h->gmaps_host = nullptr;
        return SNAP_ENOMEM;
    }
    for (int b = 0; b < 3; ++b) {
        SNAP_HIP(hipMalloc(&h->gring[b], (size_t)n_esc * sizeof(MAPT)));
        if (land_bytes > 0) SNAP_HIP(hipMalloc(&h->gring8[b], (size_t)land_bytes));
        SNAP_HIP(hipEventCreateWithFlags(&h->gev_copied[b], hipEventDisableTiming));
        SNAP_HIP(hipEventCreateWithFlags(&h->gev_free[b], hipEventDisableTiming));
        h->gring_group[b] = -1;
    }
    if (!pfx_tabs.empty()) {
        SNAP_HIP(hipMalloc(&h->gpfx_tab, pfx_tabs.size()));
        SNAP_HIP(hipMemcpy(h->gpfx_tab, pfx_tabs.data(), pfx_tabs.size(), hipMemcpyHostToDevice));
    }
    SNAP_HIP(hipMalloc(&h->gwbase, (size_t)G * (size_t)nwaves * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->gcptr, (size_t)(m + 1) * sizeof(int64_t)));
    SNAP_HIP(hipMalloc(&h->gcidx, (size_t)(total ? total : 1) * sizeof(uint32_t)));
    SNAP_HIP(hipMalloc(&h->gcbuf, (size_t)(most ? most : 1) * sizeof(float)));
    SNAP_HIP(hipMemcpyAsync(h->gcptr, cptr.data(), (size_t)(m + 1) * sizeof(int64_t), hipMemcpyHostToDevice, h->compute));
    SNAP_TRY(fill_zero(h->gwbase, (size_t)G * (size_t)nwaves * sizeof(uint32_t), h->compute));
    uint32_t *stage = nullptr, *wide = nullptr, *rowpos = nullptr, *flags = nullptr;
    auto fail = [&](int rc) {
        (void)hipStreamSynchronize(h->compute);
        (void)hipFree(stage);
        (void)hipFree(wide);
        (void)hipFree(rowpos);
        (void)hipFree(flags);
        return rc;
    };
#define S_HIP(call)                                                                \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) return fail(hip_fail(e_, #call, __FILE__, __LINE__)); \
    } while (0)
#define S_TRY(call)                          \
    do {                                     \
        int rc_ = (call);                    \
        if (rc_ != SNAP_OK) return fail(rc_); \
    } while (0)
    S_HIP(hipMalloc(&stage, (size_t)(max_group_nnz ? max_group_nnz : 1) * sizeof(uint32_t)));
    S_HIP(hipMalloc(&wide, (size_t)n_esc * sizeof(uint32_t)));
    S_HIP(hipMalloc(&rowpos, (size_t)h->n_pad * sizeof(uint32_t)));
    std::vector<uint32_t> blk((size_t)n_blk);
    S_HIP(hipMalloc(&flags, sizeof(uint32_t)));
    S_TRY(fill_zero(flags, sizeof(uint32_t), h->compute));
    S_TRY(fill_zero(rowpos, (size_t)h->n_pad * sizeof(uint32_t), h->compute));   // (every entry a valid position)
    const uint32_t label_mask = h->kind == K_PRIMAL_LOGISTIC ? LABEL_BIT : 0u;
    std::vector<uint32_t> slots((size_t)nwaves);
    for (int64_t g = 0; g < G; ++g) {
        const int64_t g0 = h->gbounds_host[g], g1 = h->gbounds_host[g + 1], sz = g1 - g0;
        const int64_t k_lo = hptr[g0], k_hi = hptr[g1], cnt = k_hi - k_lo;
        const int hot = h->ghot_host[g];
        MAPT* narrow = (MAPT*)h->gring[0];        // (the ring is not in use yet)
        if (sz == 0) continue;
        hipLaunchKernelGGL(k_fill_u32, dim3(8192), dim3(256), 0, h->compute, wide, (size_t)n_esc, RANK_NONE);
        if (cnt > 0) {
            S_HIP(hipMemcpyAsync(stage, h->host_idx + k_lo, (size_t)cnt * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
            if (label_mask) S_TRY(fold_labels(h, stage, cnt, h->compute));
            hipLaunchKernelGGL(k_build_rowmap_group, dim3((unsigned)((cnt + 4095) / 4096)), dim3(256), 0, h->compute, h->ptr,
                               stage, k_lo, k_hi, g0, g1, h->rank_of, wide, flags);
        }
        if (sizeof(MAPT) == 2)
            hipLaunchKernelGGL(k_narrow_map, dim3(8192), dim3(256), 0, h->compute, wide, (uint16_t*)narrow, (size_t)n_esc);
        const MAPT* dev_map = sizeof(MAPT) == 2 ? narrow : (const MAPT*)wide;
        S_HIP(hipGetLastError());
        if (h->gmap8_host[g] == 1) {
            hipLaunchKernelGGL(k_map16_to_8, dim3(8192), dim3(256), 0, h->compute, (const uint16_t*)dev_map, h->gring8[0], (size_t)h->n_pad);
            S_HIP(hipGetLastError());
            S_HIP(hipMemcpyAsync((char*)h->gmaps_host + h->gmap_off_host[g], h->gring8[0], (size_t)h->n_pad, hipMemcpyDeviceToHost, h->compute));
        } else if (h->gmap8_host[g] == 3) {
            // prefix-coded: bits per sub-block and block, block offsets by a prefix sum on the host, then the bits
            uint8_t* blob = h->gring8[0];
            const int64_t words = h->gpfx_words_host[g];
            unsigned long long* block_off = reinterpret_cast<unsigned long long*>(blob);
            uint32_t* stream = reinterpret_cast<uint32_t*>(blob + 8 * n_blk2);
            uint16_t* sub_rel = reinterpret_cast<uint16_t*>(blob + 8 * n_blk2 + 4 * words);
            const uint8_t* tab = h->gpfx_tab + (size_t)g * PFX_TAB_BYTES;
            const uint32_t* enc = reinterpret_cast<const uint32_t*>(tab + PFX_LUT * sizeof(uint16_t)) + PFX_CLASSES;
            const int direct_none = sz <= PFX_DIRECT_MAX ? (int)sz : -1;
            uint32_t* block_bits = wide;              // (the 32-bit staging map has been narrowed: free)
            const unsigned sub_grid = (unsigned)((n_sub + 255) / 256);
            hipLaunchKernelGGL(k_pfx_count, dim3(sub_grid), dim3(256), 0, h->compute, (const uint16_t*)dev_map, n_sub, enc, direct_none,
                               sub_rel, block_bits);
            S_HIP(hipGetLastError());
            std::vector<uint32_t> bb((size_t)n_blk2);
            S_HIP(hipMemcpyAsync(bb.data(), block_bits, (size_t)n_blk2 * sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
            S_HIP(hipStreamSynchronize(h->compute));
            std::vector<unsigned long long> boff((size_t)n_blk2);
            unsigned long long run = 0;
            for (int64_t b = 0; b < n_blk2; ++b) {
                boff[(size_t)b] = run;
                run += bb[(size_t)b];
            }
            if ((int64_t)run != pfx_bits[(size_t)g]) {       // the row map and the column lengths disagree
                set_error("internal error: the bits of a prefix-coded row map do not add up");
                return fail(SNAP_ESTATE);
            }
            S_HIP(hipMemcpyAsync(block_off, boff.data(), (size_t)n_blk2 * sizeof(unsigned long long), hipMemcpyHostToDevice, h->compute));
            S_TRY(fill_zero(stream, (size_t)words * sizeof(uint32_t), h->compute));
            hipLaunchKernelGGL(k_pfx_encode, dim3(sub_grid), dim3(256), 0, h->compute, (const uint16_t*)dev_map, n_sub, enc, direct_none,
                               (const unsigned long long*)block_off, (const uint16_t*)sub_rel, stream);
            S_HIP(hipGetLastError());
            S_HIP(hipMemcpyAsync((char*)h->gmaps_host + h->gmap_off_host[g], blob,
                                 (size_t)(h->gmap_off_host[g + 1] - h->gmap_off_host[g]), hipMemcpyDeviceToHost, h->compute));
            S_HIP(hipStreamSynchronize(h->compute));     // (boff goes out of scope)
        } else if (h->gmap8_host[g] == 2) {
            // escape-coded: count per block, offsets by a prefix sum on the host, then bytes and escaped ranks
            uint8_t* blob = h->gring8[0];
            uint32_t* offs = reinterpret_cast<uint32_t*>(blob + n_esc);
            uint16_t* esc = reinterpret_cast<uint16_t*>(blob + n_esc + 4 * n_blk);
            hipLaunchKernelGGL(k_esc_count, dim3((unsigned)n_blk), dim3(ESC_TPB), 0, h->compute, (const uint16_t*)dev_map, offs);
            S_HIP(hipGetLastError());
            S_HIP(hipMemcpyAsync(blk.data(), offs, (size_t)n_blk * sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
            S_HIP(hipStreamSynchronize(h->compute));
            uint64_t run = 0;
            for (int64_t b = 0; b < n_blk; ++b) {
                const uint32_t cnt = blk[(size_t)b];
                blk[(size_t)b] = (uint32_t)run;
                run += cnt;
            }
            if ((int64_t)run != escaped[(size_t)g]) {      // the row map and the column lengths disagree
                set_error("internal error: the escaped rows of a row map do not add up");
                return fail(SNAP_ESTATE);
            }
            S_HIP(hipMemcpyAsync(offs, blk.data(), (size_t)n_blk * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
            hipLaunchKernelGGL(k_esc_encode, dim3((unsigned)n_blk), dim3(ESC_TPB), 0, h->compute, (const uint16_t*)dev_map, offs, blob, esc);
            S_HIP(hipGetLastError());
            S_HIP(hipMemcpyAsync((char*)h->gmaps_host + h->gmap_off_host[g], blob,
                                 (size_t)(h->gmap_off_host[g + 1] - h->gmap_off_host[g]), hipMemcpyDeviceToHost, h->compute));
        } else {
            S_HIP(hipMemcpyAsync((char*)h->gmaps_host + h->gmap_off_host[g], dev_map, map_bytes, hipMemcpyDeviceToHost, h->compute));
        }
        if (h->gcompact_host[g] && n > 0) {
            uint32_t* wb = h->gwbase + (size_t)g * nwaves;
            hipLaunchKernelGGL((k_cold_rows<MAPT, false>), dim3((unsigned)h->g_row_wgs), dim3(ROW_TPB), 0, h->compute, dev_map,
                               hot, n, wb, (uint32_t*)nullptr);
            S_HIP(hipGetLastError());
            S_HIP(hipMemcpyAsync(slots.data(), wb, slots.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, h->compute));
            S_HIP(hipStreamSynchronize(h->compute));
            uint64_t sum = 0;
            for (int w = 0; w < nwaves; ++w) {
                const uint32_t count = slots[(size_t)w];
                slots[(size_t)w] = (uint32_t)sum;
                sum += count;
            }
            if ((int64_t)sum != cold_rows[(size_t)g]) {      // the row map and the column lengths disagree
                set_error("internal error: the rows of the short coordinates do not add up");
                return fail(SNAP_ESTATE);
            }
            S_HIP(hipMemcpyAsync(wb, slots.data(), slots.size() * sizeof(uint32_t), hipMemcpyHostToDevice, h->compute));
            hipLaunchKernelGGL((k_cold_rows<MAPT, true>), dim3((unsigned)h->g_row_wgs), dim3(ROW_TPB), 0, h->compute, dev_map,
                               hot, n, wb, rowpos);
            const int blocks = (int)std::min<int64_t>((sz - hot + 3) / 4, 16384);
            hipLaunchKernelGGL(k_cold_index, dim3((unsigned)blocks), dim3(256), 0, h->compute, h->ptr, stage, k_lo, h->coord_of,
                               h->gcptr, g0, hot, sz, label_mask, rowpos, h->gcidx);
            S_HIP(hipGetLastError());
        }
        S_HIP(hipStreamSynchronize(h->compute));    // staging buffers and `slots` are reused by the next group
    }
    uint32_t fl = 0;
    S_HIP(hipMemcpy(&fl, flags, sizeof(uint32_t), hipMemcpyDeviceToHost));
#undef S_HIP
#undef S_TRY
    (void)fail(SNAP_OK);
    if (fl & 1u) {
        set_error("two coordinates of one group share a row: the groups are not disjoint");
        return SNAP_EINVAL;
    }
    if (h->opt.profile) {
        h->gev_prof = new (std::nothrow) hipEvent_t[(size_t)(4 * (G + 1))]();
        if (!h->gev_prof) return SNAP_ENOMEM;
        for (int64_t i = 0; i < 4 * (G + 1); ++i) SNAP_HIP(hipEventCreate(&h->gev_prof[i]));
    }
    return SNAP_OK;
}

static int streamed_setup(snap_handle* h, const int64_t* hptr, const std::vector<uint32_t>&) {
    h->unit_values = true;                 // (checked by the caller: streamed group sweeps take pattern-only data)
    h->gscale_exp = 1;                     // largest |value| = 1 <= 2^1, as frexp gives it for resident data
    h->gstream = true;
    return h->map16 ? streamed_setup_maps<uint16_t>(h, hptr) : streamed_setup_maps<uint32_t>(h, hptr);
}

// Scales of the sums (powers of two, exact in fp32).  Logistic: a loss' <= 2^e in magnitude gets 19 - e
// fractional bits (times at most 4095 rows: below 2^31), a^2 loss'' <= 2^(2e-2) gets 22 - 2e (below 2^32
// in total).  Ridge: 24 fractional bits for a (v - y); no second sum.
struct SumScales {
    float g, h;
};
static SumScales sum_scales(const snap_handle* h) {
    if (h->kind == K_PRIMAL_LOGISTIC) return SumScales{ldexpf(1.0f, 19 - h->gscale_exp), ldexpf(1.0f, 22 - 2 * h->gscale_exp)};
    return SumScales{ldexpf(1.0f, 24), 1.0f};
}
constexpr float FIX_MAGIC = 12582912.0f;         // 1.5 * 2^23
constexpr unsigned long long FIX_BIAS = 0x4B400000ull;   // its bit pattern

// The shared vector is read from vin and (SCATTER) written to vout: the same array, except in the first
// writing pass of an epoch whose earlier state must survive (the accept check of Section 3.1 may discard
// the epoch: the state before it then simply stays where it was, and the two arrays change roles).
// LOSS (the last pass of such an epoch): the loss of every row at its final value is summed on the way,
// per workgroup in a fixed order, so that the objective after the epoch costs one small reduction more.
// MAPP, MAPC: entry types of the previous and of the current group's map (one byte for groups of at most
// 255 coordinates; both take the same number of rows per thread and iteration).
template <int KIND, bool UNIT, bool SCATTER, bool HIST, typename MAPP, typename MAPC, bool LOSS = false>
__global__ void __launch_bounds__(ROW_TPB)
k_group_rows(const MAPP* __restrict__ map_prev, const float* __restrict__ val_prev,
             const float* __restrict__ delta_prev, const MAPC* __restrict__ map_cur,
             const float* __restrict__ val_cur, int hot, int k64, const float* vin, float* vout, const float* __restrict__ y,
             const uint8_t* __restrict__ ybits, int64_t n, long long* __restrict__ partial, int64_t partial_stride,
             SumScales scale, int kd, uint32_t* __restrict__ status,
             float* __restrict__ cbuf, const uint32_t* __restrict__ wbase, double* __restrict__ loss_partial = nullptr,
             const float* __restrict__ model = nullptr, int64_t m = 0) {
    constexpr int R = MapTraits<MAPC>::R;
    static_assert(MapTraits<MAPP>::R == R, "both maps must give a thread the same rows");
    constexpr uint32_t NONE_P = MapTraits<MAPP>::NONE, NONE_C = MapTraits<MAPC>::NONE;
    __shared__ double s_loss[LOSS ? 3 * (ROW_TPB / WAVE) : 1];
    double loss_acc = 0.0;
    // LDS: fixed-point sums.  Logistic: ranks below k64: [rank] sum of a loss' * scale.g, [k64 + rank]
    // sum of a^2 loss'' * scale.h; ranks k64 .. hot-1: one packed word at [k64 + rank] (k64 = hot: none).
    // Ridge: [rank] sum of a loss' * scale.g, k64 = 0.
    // Then the steps of the previous group's first kd ranks (a gather from global memory per row
    // costs a third of the pass; nearly every row hits one of these).
    extern __shared__ unsigned long long hist[];
    float* dl = reinterpret_cast<float*>(hist + hot + k64);
    // The workgroups walk the rows side by side: in iteration i workgroup b takes the ROW_TPB packs from
    // (i * gridDim.x + b) * ROW_TPB on, so that at any time the whole grid works on one contiguous window of
    // every array (measured with a bare kernel of the same byte mix: 5.65 TB/s, against 5.0 TB/s when every
    // workgroup streams a slab of its own).
    const int64_t packs = (n + R - 1) / R;
    const int64_t q_first = (int64_t)blockIdx.x * ROW_TPB + threadIdx.x, q_stride = (int64_t)gridDim.x * ROW_TPB;
    // All loads of an iteration are issued together, ahead of its first wait, and those of the first
    // iteration ahead of the set-up of the LDS tables (the loop below asks for the next pack's at its end.
    // Asking earlier was measured slower, with two packs per thread in turn by 3 % and with three, the
    // steps from beyond the LDS table gathered an iteration ahead too so that no wait is left inside the
    // arithmetic, by 4 %: the memory side delivers less when more of a wavefront's loads are under way,
    // as it does for a bare kernel that only moves the bytes).
    float vv[R], ap[R], ac[R], yy[R];
    typename MapTraits<MAPP>::Raw raw_prev = {};
    typename MapTraits<MAPC>::Raw raw_cur = {};
    uint32_t lab_byte = 0;
    auto request = [&](int64_t q) {
        const int64_t r = R * q;
        const bool full = r + R - 1 < n;           // maps, values and label bits are padded; v and y are not
        if (full) {
            load_floats<R>(vin + r, vv);
        } else {
#pragma unroll
            for (int j = 0; j < R; ++j) vv[j] = r + j < n ? vin[r + j] : 0.0f;
        }
        if (SCATTER) {
            raw_prev = load_map(map_prev + r);
            if (!UNIT) load_floats<R>(val_prev + r, ap);
        }
        if (HIST) {
            raw_cur = load_map(map_cur + r);
            if (!UNIT) load_floats<R>(val_cur + r, ac);
        }
        if (HIST || LOSS) {
            if (KIND == K_PRIMAL_LOGISTIC) {
                lab_byte = ybits[r >> 3];
            } else if (full) {
                load_floats<R>(y + r, yy);
            } else {
#pragma unroll
                for (int j = 0; j < R; ++j) yy[j] = r + j < n ? y[r + j] : 0.0f;
            }
        }
    };
    if (q_first < packs) request(q_first);
    if (HIST)
        for (int i = threadIdx.x; i < hot + k64; i += ROW_TPB) hist[i] = 0ull;
    if (SCATTER)
        for (int i = threadIdx.x; i <= kd; i += ROW_TPB) dl[i] = i < kd ? delta_prev[i] : 0.0f;   // [kd]: a zero for the rows without a step
    __syncthreads();
    // the two longest coordinates of a group hold a quarter of its rows: their sums stay in
    // registers (one LDS update per wavefront at the end) instead of colliding in LDS
    float rg0 = 0.0f, rg1 = 0.0f, rh0 = 0.0f, rh1 = 0.0f;
    // dense buffer of the short coordinates' rows (null: none): next position of this wavefront.  The
    // entries pass through a ring of 128 per wavefront in LDS and leave it 64 at a time, in one store
    // (written row by row they cost eight nearly empty stores per iteration).
    uint32_t crun = (HIST && cbuf) ? __builtin_amdgcn_readfirstlane(wbase[blockIdx.x * (ROW_TPB / WAVE) + threadIdx.x / WAVE]) : 0u;
    uint32_t cflushed = crun;
    float* stage = dl + kd + 1 + (threadIdx.x / WAVE) * COLD_RING;
    bool too_large = false;                    // ridge: a term outside the range the 64-bit sums are laid out for
    const uint32_t hot_lds = (uint32_t)max(hot, 2) - 2u;      // ranks 2 .. hot-1 take their sums in LDS: rank - 2 < hot_lds
    for (int64_t q = q_first; q < packs;) {
        const int64_t r = R * q;
        uint32_t mp[R], mc[R];
        const bool full = r + R - 1 < n;
        const uint32_t lab = lab_byte >> (r & 7);
        __builtin_amdgcn_sched_barrier(0);         // (nothing moves across: the requests stay ahead of the first wait;
                                                   // left to the compiler, the current group's map was fetched only
                                                   // after the store of the shared vector)
        if (SCATTER) {
            unpack_ranks(map_prev, raw_prev, mp);
            // straight-line per row (a wavefront's rows take every path anyway, and each divergent
            // region costs its exec-mask bookkeeping): the step comes from LDS with the index clamped
            // to kd, where a zero sits for the rows that the previous group does not cover; only the
            // rare rank beyond the LDS copy enters a region of its own
            float dv[R];
#pragma unroll
            for (int j = 0; j < R; ++j) dv[j] = dl[min(mp[j], (uint32_t)kd)];
#pragma unroll
            for (int j = 0; j < R; ++j) asm("" : "+v"(dv[j]));   // (keeps these LDS reads: merged with the global ones they turn into flat loads)
#pragma unroll
            for (int j = 0; j < R; ++j)
                if (mp[j] - (uint32_t)kd < NONE_P - (uint32_t)kd) dv[j] = delta_prev[mp[j]];   // kd <= rank < "none", in one comparison
#pragma unroll
            for (int j = 0; j < R; ++j) vv[j] += dv[j] * (UNIT ? 1.0f : ap[j]);
            if (full) {
#pragma unroll
                for (int qq = 0; qq < R / 4; ++qq)
                    *reinterpret_cast<float4*>(vout + r + 4 * qq) =
                        make_float4(vv[4 * qq], vv[4 * qq + 1], vv[4 * qq + 2], vv[4 * qq + 3]);
            } else {
#pragma unroll
                for (int j = 0; j < R; ++j)
                    if (r + j < n) vout[r + j] = vv[j];
            }
        }
        if (LOSS) {
            // loss of the rows at their value after the epoch (rows past the end count nothing)
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float l;
                if (KIND == K_PRIMAL_LOGISTIC) {
                    const uint32_t sgn = (lab << (31 - j)) & 0x80000000u;
                    l = logistic_loss_f32(-__uint_as_float(__float_as_uint(vv[j]) ^ sgn));       // log(1 + exp(-y v))
                } else {
                    const float t = vv[j] - yy[j];
                    l = 0.5f * t * t;
                }
                s += (full || r + j < n) ? l : 0.0f;
            }
            loss_acc += (double)s;
        }
        if (HIST) {
            unpack_ranks(map_cur, raw_cur, mc);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                // the terms are computed for every row (a row past the end has rank "none", which is
                // never hot, and v = 0); one region holds the LDS updates
                const uint32_t rk = mc[j];
                float g, hh = 0.0f;
                if (KIND == K_PRIMAL_LOGISTIC) {
                    // the label as a sign bit: y v by an xor, and the term is summed as y p = -loss'
                    // (p = sigmoid(-y v) >= 0 takes the sign by an or; the scale below is negative)
                    const uint32_t sgn = (lab << (31 - j)) & 0x80000000u;
                    const float p = __builtin_amdgcn_rcpf(1.0f + __expf(__uint_as_float(__float_as_uint(vv[j]) ^ sgn)));
                    g = __uint_as_float(__float_as_uint(p) | sgn);
                    hh = p - p * p;                                // loss'' = p (1 - p)
                    if (!UNIT) {
                        g *= ac[j];
                        hh *= ac[j] * ac[j];
                    }
                } else {
                    g = (UNIT ? 1.0f : ac[j]) * (vv[j] - yy[j]);
                }
                const bool in = rk < (uint32_t)hot;
                if (cbuf) {
                    // a row of a short coordinate: its entry goes to the buffer (ridge: minus the label,
                    // which the finishing kernel then need not gather either)
                    const bool cold = rk - (uint32_t)hot < NONE_C - (uint32_t)hot;      // hot <= rank < "none", in one comparison
                    const uint32_t pos = cold_slot(cold, crun);
                    if (cold) stage[pos & (COLD_RING - 1)] = KIND == K_PRIMAL_LOGISTIC ? vv[j] : vv[j] - yy[j];
                    if (crun - cflushed >= (uint32_t)WAVE) {      // (uniform; at most 64 entries arrive per row step)
                        // (the lanes still in the loop are the first ones of the wavefront)
                        const uint32_t lanes_on = (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(true));
                        for (uint32_t i = threadIdx.x & (WAVE - 1); i < (uint32_t)WAVE; i += lanes_on)
                            cbuf[cflushed + i] = stage[(cflushed + i) & (COLD_RING - 1)];
                        cflushed += WAVE;
                    }
                }
                if (KIND == K_PRIMAL_RIDGE) too_large |= in && !(fabsf(g) < RIDGE_TERM_LIMIT);
                // register ranks: indicator times term (two selects and an fma per sum instead of
                // a select and an add each; rank 1 is summed even when it is not hot, and then unused)
                const float m0 = rk == 0u ? 1.0f : 0.0f, m1 = rk == 1u ? 1.0f : 0.0f;
                rg0 = fmaf(m0, g, rg0);
                rg1 = fmaf(m1, g, rg1);
                if (KIND == K_PRIMAL_LOGISTIC) {
                    rh0 = fmaf(m0, hh, rh0);
                    rh1 = fmaf(m1, hh, rh1);
                    if (rk - 2u < hot_lds) {                       // 2 <= rank < hot
                        // fixed point by the rounding of an addition: the low mantissa bits of
                        // x + 1.5 * 2^23 hold round(x) for |x| < 2^22; the constant's bit pattern stays
                        // in every term and is taken out per coordinate, times its row count, by the
                        // finishing kernel.  Ranks below k64: sum of a^2 loss'' at [k64 + rank] and sum
                        // of a loss' at [rank]; the others: both in one word at [k64 + rank].
                        const uint32_t gb = __float_as_uint(fmaf(g, -scale.g, FIX_MAGIC));
                        const uint32_t hb = __float_as_uint(fmaf(hh, scale.h, FIX_MAGIC));
                        const bool two = rk < (uint32_t)k64;
                        atomicAdd(&hist[k64 + rk], (unsigned long long)hb | ((unsigned long long)(two ? 0u : gb) << PACK_H_BITS));
                        if (two) atomicAdd(&hist[rk], (unsigned long long)gb);
                    }
                } else if (rk - 2u < hot_lds) {
                    atomicAdd(&hist[rk], (unsigned long long)__float2ll_rn(g * scale.g));
                }
            }
        }
        q += q_stride;
        if (q < packs) request(q);
    }
    if (HIST) {
        if (cbuf) {
            // what is left in the ring; the counters are taken from the first lane, which holds the
            // wavefront's lowest pack and ran every iteration (a lane that left the loop earlier may
            // hold older ones)
            crun = __builtin_amdgcn_readfirstlane(crun);
            cflushed = __builtin_amdgcn_readfirstlane(cflushed);
            for (uint32_t i = cflushed + (threadIdx.x & (WAVE - 1)); i < crun; i += WAVE) cbuf[i] = stage[i & (COLD_RING - 1)];
        }
        if (KIND == K_PRIMAL_RIDGE && too_large) atomicOr(status, STATUS_RANGE);
        rg0 = wave_sum(rg0); rg1 = wave_sum(rg1);
        if (KIND == K_PRIMAL_LOGISTIC) {
            rh0 = wave_sum(rh0); rh1 = wave_sum(rh1);
        }
        if ((threadIdx.x & (WAVE - 1)) == 0) {
            const float rg[2] = {rg0, rg1}, rh[2] = {rh0, rh1};
            for (int t = 0; t < 2 && t < hot; ++t) {
                atomicAdd(&hist[t], (unsigned long long)__float2ll_rn(rg[t] * (KIND == K_PRIMAL_LOGISTIC ? -scale.g : scale.g)));
                if (KIND == K_PRIMAL_LOGISTIC) atomicAdd(&hist[k64 + t], (unsigned long long)__float2ll_rn(rh[t] * scale.h));
            }
        }
        __syncthreads();
        long long* out = partial + (size_t)blockIdx.x * (size_t)partial_stride;
        for (int i = threadIdx.x; i < hot + k64; i += ROW_TPB) out[i] = (long long)hist[i];
    }
    if (LOSS) {
        // the regulariser's sums over this workgroup's slice of the model (final by now: the last step kernel
        // of the epoch ran before this pass), so that the objective needs no pass of its own at all
        double sq = 0.0, ab = 0.0;
        const int64_t mper = (m + gridDim.x - 1) / gridDim.x;
        const int64_t m0 = min(m, (int64_t)blockIdx.x * mper), m1 = min(m, m0 + mper);
        for (int64_t i = m0 + threadIdx.x; i < m1; i += ROW_TPB) {
            const double xi = (double)model[i];
            sq += xi * xi;
            ab += fabs(xi);
        }
#pragma unroll
        for (int off = WAVE / 2; off > 0; off >>= 1) {
            loss_acc += __shfl_xor(loss_acc, off, WAVE);
            sq += __shfl_xor(sq, off, WAVE);
            ab += __shfl_xor(ab, off, WAVE);
        }
        if ((threadIdx.x & (WAVE - 1)) == 0) {
            s_loss[3 * (threadIdx.x / WAVE)] = loss_acc;
            s_loss[3 * (threadIdx.x / WAVE) + 1] = sq;
            s_loss[3 * (threadIdx.x / WAVE) + 2] = ab;
        }
        __syncthreads();
        if (threadIdx.x < 3) {
            double t = 0.0;
            for (int w = 0; w < ROW_TPB / WAVE; ++w) t += s_loss[3 * w + threadIdx.x];
            loss_partial[3 * blockIdx.x + threadIdx.x] = t;
        }
    }
}

// The three sums that the last row pass of an epoch leaves per workgroup (loss, ||x||^2, ||x||_1), added up
// in a fixed order and written straight into host memory mapped into the device's address space.
__global__ void __launch_bounds__(256)
k_group_loss_final(const double* __restrict__ partial, int n_wgs, double* __restrict__ host_mapped) {
    __shared__ double s[3][256];
    double t[3] = {0.0, 0.0, 0.0};
    for (int w = threadIdx.x; w < n_wgs; w += 256)
        for (int k = 0; k < 3; ++k) t[k] += partial[3 * w + k];
    for (int k = 0; k < 3; ++k) s[k][threadIdx.x] = t[k];
    __syncthreads();
    if (threadIdx.x < 3) {
        double acc = 0.0;
        for (int i = 0; i < 256; ++i) acc += s[threadIdx.x][i];
        host_mapped[threadIdx.x] = acc;
    }
}

// The objective after an epoch whose last pass has summed the loss (see g_want_loss); synchronises.
int grouped_loss_value(snap_handle* h, double* value) {
    hipLaunchKernelGGL(k_group_loss_final, dim3(1), dim3(256), 0, h->compute, h->gloss_partial, h->g_row_wgs, h->red.host_mapped);
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipStreamSynchronize(h->compute));
    const double* res = h->red.host;
    *value = res[0] / (double)h->n + 0.5 * h->lambda * res[1] + h->lambda1 * res[2];
    return SNAP_OK;
}

// ---- sums of the short coordinates and the steps of one group ------------------------------------------
// One launch, two kinds of workgroups.  The first n_hot_blocks handle the hot ranks: 32 ranks per
// workgroup, 32 threads per rank, each summing every 32nd per-workgroup partial of the row pass (integer
// sums: exact and independent of the order), combined in LDS, then one thread takes the step.  The
// others handle the cold ranks: 16 lanes per coordinate gather its two sums column-wise from the dense
// buffer of the row pass (or, where a group has none, one wavefront per coordinate from v itself, which is
// not written while this kernel runs) and take the step right away.
constexpr int STEP_RANKS = 32, STEP_PARTS = 32;

// DOTS: no step is taken; the first sum (the coordinate's inner product with loss'(v)) goes to gdot.
template <int KIND, bool DOTS>
__global__ void __launch_bounds__(STEP_RANKS * STEP_PARTS)
k_group_finish(const long long* __restrict__ partial, int64_t partial_stride, int n_wgs, int hot, int k64, int n_hot_blocks,
               double inv_scale_g, double inv_scale_h, const int64_t* __restrict__ ptr,
               const uint32_t* __restrict__ idx, const float* __restrict__ val, const float* __restrict__ v,
               const float* __restrict__ y, const uint32_t* __restrict__ coord_of, int64_t g0, int64_t group_size,
               float* __restrict__ x, const float* __restrict__ norms, float* __restrict__ delta, StepParams sp,
               double* __restrict__ gdot, const float* __restrict__ cbuf, const uint32_t* __restrict__ cidx,
               const int64_t* __restrict__ cptr, int unit) {
    __shared__ long long sg[STEP_PARTS][STEP_RANKS], sh[STEP_PARTS][STEP_RANKS];
    if ((int)blockIdx.x >= n_hot_blocks && cbuf) {
        // short coordinates, entries of their rows in the dense buffer: 16 lanes per coordinate (most have
        // a few dozen rows; four dependent chains per wavefront instead of one), index and value streams
        // contiguous per coordinate, four loads in flight per lane
        constexpr int SUB = 16, UNROLL = 4;
        const int sl = threadIdx.x & (SUB - 1);
        const int64_t sub0 = ((int64_t)(blockIdx.x - n_hot_blocks) * blockDim.x + threadIdx.x) / SUB;
        const int64_t nsubs = (int64_t)(gridDim.x - n_hot_blocks) * blockDim.x / SUB;
        for (int64_t rk = hot + sub0; rk < group_size; rk += nsubs) {
            const int64_t k0 = cptr[g0 + rk], k1 = cptr[g0 + rk + 1];
            const int64_t c = coord_of[g0 + rk];
            const float* vals = unit ? nullptr : val + ptr[c] - k0;      // value of the nonzero at index position k
            const float xc = DOTS ? 0.0f : x[c], nc = DOTS ? 0.0f : norms[c];   // (asked for early: off the chain of dependent loads)
            float g = 0.0f, hh = 0.0f;
            for (int64_t k = k0 + sl; k < k1; k += SUB * UNROLL) {
                uint32_t e[UNROLL];
                float a[UNROLL], vv[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const bool on = k + u * SUB < k1;
                    e[u] = on ? cidx[k + u * SUB] : 0u;
                    a[u] = !on ? 0.0f : unit ? 1.0f : vals[k + u * SUB];
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) vv[u] = cbuf[KIND == K_PRIMAL_LOGISTIC ? e[u] & ~LABEL_BIT : e[u]];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const float yy = KIND == K_PRIMAL_LOGISTIC ? ((e[u] & LABEL_BIT) ? -1.0f : 1.0f) : 0.0f;
                    accumulate<KIND>(a[u], vv[u], yy, g, hh);          // (a = 0 past the end: no contribution)
                }
            }
            g = row_sum(g);
            hh = row_sum(hh);
            if (sl == 0) {
                if (DOTS) {
                    gdot[c] = (double)g;
                } else {
                    float mult;
                    x[c] = take_step<KIND>((double)g, (double)hh, xc, nc, 0.0f, sp, mult);
                    delta[g0 + rk] = mult;
                }
            }
        }
        return;
    }
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
                if (DOTS) {
                    gdot[c] = (double)g;
                } else {
                    float mult;
                    x[c] = take_step<KIND>((double)g, (double)hh, x[c], norms[c], 0.0f, sp, mult);
                    delta[g0 + rk] = mult;
                }
            }
        }
        return;
    }
    const int lr = threadIdx.x % STEP_RANKS, part = threadIdx.x / STEP_RANKS;
    const int64_t rk = (int64_t)blockIdx.x * STEP_RANKS + lr;
    long long Gi = 0, Hi = 0;
    const bool packed = KIND == K_PRIMAL_LOGISTIC && rk >= k64;      // one word per workgroup holding both sums
    // what the thread that takes the step needs besides the sums is asked for first
    int64_t c = 0, rows = 0;
    float xc = 0.0f, nc = 0.0f;
    if (part == 0 && rk < hot) {
        c = coord_of[g0 + rk];
        rows = ptr[c + 1] - ptr[c];
        if (!DOTS) {
            xc = x[c];
            nc = norms[c];
        }
    }
    if (rk < hot) {
        if (!packed) {
#pragma unroll 8
            for (int w = part; w < n_wgs; w += STEP_PARTS) {
                Gi += partial[(size_t)w * partial_stride + rk];
                if (KIND == K_PRIMAL_LOGISTIC) Hi += partial[(size_t)w * partial_stride + k64 + rk];
            }
        } else {
#pragma unroll 8
            for (int w = part; w < n_wgs; w += STEP_PARTS) Gi += partial[(size_t)w * partial_stride + k64 + rk];   // whole words, modulo 2^64
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
    if (KIND == K_PRIMAL_LOGISTIC && rk >= 2) {
        // every term of these ranks carries the bit pattern of the rounding constant (the ranks 0 and 1
        // are summed in registers by the row pass and converted without it)
        const unsigned long long bias = (unsigned long long)rows * FIX_BIAS;
        if (packed) {
            const unsigned long long word = (unsigned long long)Gi - bias - (bias << PACK_H_BITS);
            Hi = (long long)(word & 0xFFFFFFFFull);                           // the low field is never negative
            Gi = (long long)(word - (unsigned long long)Hi) >> PACK_H_BITS;
        } else {
            Gi = (long long)((unsigned long long)Gi - bias);
            Hi = (long long)((unsigned long long)Hi - bias);
        }
    }
    const double gsum = (double)Gi * inv_scale_g;
    const double hsum = (double)Hi * inv_scale_h;
    if (DOTS) {
        gdot[c] = gsum;
        return;
    }
    float mult;
    x[c] = take_step<KIND>(gsum, hsum, xc, nc, 0.0f, sp, mult);
    delta[g0 + rk] = mult;
}

std::vector<int64_t> group_order(uint64_t seed, int64_t n_groups) {
    std::vector<uint64_t> comp((size_t)n_groups);
    const uint64_t base = perm_key_base(seed, GROUP_ORDER_CHUNK);
    for (int64_t g = 0; g < n_groups; ++g) comp[(size_t)g] = ((uint64_t)perm_key(base, (uint32_t)g) << 32) | (uint64_t)g;
    std::sort(comp.begin(), comp.end());
    std::vector<int64_t> order((size_t)n_groups);
    for (int64_t i = 0; i < n_groups; ++i) order[(size_t)i] = (int64_t)(comp[(size_t)i] & 0xFFFFFFFFull);
    return order;
}

// Streamed row maps: enqueue the copy of group g's map into ring slot `slot` on the copy stream, once
// the last pass that read the slot's earlier content is done.  A map that still sits in the slot is not
// copied again.  prof >= 0: the copy's start and end are recorded in that visit's pair of events.
static int enqueue_map_copy(snap_handle* h, int64_t g, int slot, int64_t prof) {
    if (prof >= 0) h->gcopy_timed[(size_t)prof] = 0;
    if (h->gring_group[slot] == g) return SNAP_OK;
    const size_t map_bytes = (size_t)(h->gmap_off_host[g + 1] - h->gmap_off_host[g]);
    const bool bytes8 = h->gmap8_host[g] != 0;          // byte-coded (plain or with escapes): lands in the byte buffer
    SNAP_HIP(hipStreamWaitEvent(h->copy, h->gev_free[slot], 0));
    if (prof >= 0) {
        SNAP_HIP(hipEventRecord(h->gev_prof[4 * prof + 0], h->copy));
        h->gcopy_timed[(size_t)prof] = 1;
    }
    SNAP_HIP(hipMemcpyAsync(bytes8 ? (void*)h->gring8[slot] : h->gring[slot], (const char*)h->gmaps_host + h->gmap_off_host[g],
                            map_bytes, hipMemcpyHostToDevice, h->copy));
    h->gring_widened[slot] = !bytes8;
    if (prof >= 0) SNAP_HIP(hipEventRecord(h->gev_prof[4 * prof + 1], h->copy));
    SNAP_HIP(hipEventRecord(h->gev_copied[slot], h->copy));
    h->gring_group[slot] = g;
    h->bytes_copied += (int64_t)map_bytes;
    return SNAP_OK;
}

// The compute stream takes over ring slot `slot`: wait for its copy and, for a byte-coded map, decode it.
// begin (may be null): an event to record once the copy is there, ahead of the decoding (profiling).
static int acquire_map(snap_handle* h, int slot, hipEvent_t begin) {
    SNAP_HIP(hipStreamWaitEvent(h->compute, h->gev_copied[slot], 0));
    if (begin) SNAP_HIP(hipEventRecord(begin, h->compute));
    if (!h->gring_widened[slot]) {
        const int64_t gg = h->gring_group[slot];
        if (h->gmap8_host[gg] == 3) {
            const int64_t n_esc = (h->n_pad + ESC_BLOCK - 1) / ESC_BLOCK * ESC_BLOCK, n_sub = n_esc / PFX_SUB, n_blk2 = n_esc / PFX_BLOCK;
            const uint8_t* blob = h->gring8[slot];
            hipLaunchKernelGGL(k_pfx_decode, dim3((unsigned)((n_sub + 255) / 256)), dim3(256), 0, h->compute,
                               reinterpret_cast<const unsigned long long*>(blob), reinterpret_cast<const uint32_t*>(blob + 8 * n_blk2),
                               reinterpret_cast<const uint16_t*>(blob + 8 * n_blk2 + 4 * h->gpfx_words_host[gg]),
                               (const uint8_t*)(h->gpfx_tab + (size_t)gg * PFX_TAB_BYTES), n_sub, (uint16_t*)h->gring[slot]);
        } else if (h->gmap8_host[gg] == 2) {
            const int64_t n_esc = (h->n_pad + ESC_BLOCK - 1) / ESC_BLOCK * ESC_BLOCK, n_blk = n_esc / ESC_BLOCK;
            const uint8_t* blob = h->gring8[slot];
            hipLaunchKernelGGL(k_esc_decode, dim3((unsigned)n_blk), dim3(ESC_TPB), 0, h->compute, blob,
                               reinterpret_cast<const uint32_t*>(blob + n_esc),
                               reinterpret_cast<const uint16_t*>(blob + n_esc + 4 * n_blk), (uint16_t*)h->gring[slot]);
        } else {
            hipLaunchKernelGGL(k_map8_to_16, dim3(4096), dim3(256), 0, h->compute, h->gring8[slot], (uint16_t*)h->gring[slot],
                               (size_t)h->n_pad);
        }
        SNAP_HIP(hipGetLastError());
        h->gring_widened[slot] = true;
    }
    return SNAP_OK;
}

template <int KIND, bool UNIT, typename MAPT>
static int grouped_epoch_kind(snap_handle* h) {
    const StepParams sp = make_step_params(h);
    const int64_t n = h->n, G = h->n_groups;
    long long* gpart = (long long*)h->gpartial;
    const SumScales scale = sum_scales(h);
    int64_t prev = -1;                              // last non-empty group, whose steps are still to be applied
    const bool prof = h->opt.profile != 0 && h->ev_group != nullptr;
    int n_pass = 0;
    // the groups are visited in a seeded random order (keys of the epoch's seed under a reserved
    // chunk id, sorted with the group index as tie-break): on the click-log workload a fresh order
    // every epoch reaches a given duality gap in a fifth of the epochs a fixed order needs
    // ... or, for a pass over part of the groups, the caller's list
    const std::vector<int64_t> gorder =
        h->pass_list ? std::vector<int64_t>(h->pass_list, h->pass_list + h->pass_count) : group_order(h->last_seed, G);
    std::vector<int64_t> visits;                    // the non-empty groups, in visiting order
    for (int64_t g : gorder)
        if (h->gbounds_host[g + 1] > h->gbounds_host[g]) visits.push_back(g);
    const int64_t n_visit = (int64_t)visits.size();
    // Streamed row maps (data in host memory, Section 3.2): visit i's map goes through ring slot i % 3.
    // Pass i reads the maps of visits i - 1 and i while the copy engine brings in the map of visit i + 1;
    // that copy is enqueued once pass i - 1, the last reader of the slot's earlier content, has been
    // launched, so copies run one pass ahead of the kernels and follow each other without a gap as long
    // as a pass is shorter than a copy.
    const bool streamed = h->gstream;
    const bool sprof = streamed && h->opt.profile != 0 && h->gev_prof != nullptr && !h->pass_list;
    // an epoch that may have to be undone leaves the state before it untouched: see g_keep_old
    const bool keep_old = h->g_keep_old && h->v_snap != nullptr;
    float* v_cur = h->v;
    bool swapped = false, loss_done = false;
    if (streamed) {
        h->gcopy_timed.assign((size_t)(G + 1), 0);
        for (int64_t i = 0; i < std::min<int64_t>(2, n_visit); ++i)
            SNAP_TRY(enqueue_map_copy(h, visits[(size_t)i], (int)(i % 3), sprof ? i : -1));
    }
    for (int64_t gi = 0; gi <= n_visit; ++gi) {
        const bool last = gi == n_visit;
        const int64_t g = last ? G : visits[(size_t)gi];
        const int64_t g0 = last ? 0 : h->gbounds_host[g], sz = last ? 0 : h->gbounds_host[g + 1] - g0;
        const int hot = last ? 0 : h->ghot_host[g], k64 = last ? 0 : h->gk64_host[g];
        const MAPT* maps = (const MAPT*)h->rowmap;
        const MAPT* map_prev = prev < 0 ? nullptr : streamed ? (const MAPT*)h->gring[(gi - 1) % 3] : maps + (size_t)prev * h->n_pad;
        const float* val_prev = (prev >= 0 && !UNIT) ? h->rowval + (size_t)prev * h->n_pad : nullptr;
        const float* delta_prev = prev >= 0 ? h->gdelta + h->gbounds_host[prev] : nullptr;
        const MAPT* map_cur = last ? nullptr : streamed ? (const MAPT*)h->gring[gi % 3] : maps + (size_t)g * h->n_pad;
        const float* val_cur = (last || UNIT) ? nullptr : h->rowval + (size_t)g * h->n_pad;
        const int kd = prev >= 0 ? (int)std::min<int64_t>(h->g_kd_max, h->gbounds_host[prev + 1] - h->gbounds_host[prev]) : 0;
        // short coordinates through the dense buffer (only with a row pass that computes sums)
        const bool compact = !last && h->gcompact_host[g] && n > 0;
        const size_t lds = (size_t)(hot + k64) * sizeof(unsigned long long) + (size_t)(kd + 1) * sizeof(float) +
                           (compact ? (size_t)(ROW_TPB / WAVE) * COLD_RING * sizeof(float) : 0);
        const dim3 row_grid((unsigned)h->g_row_wgs);
        const bool scatter = prev >= 0, histo = !last && (hot > 0 || compact);
        float* cbuf = compact ? h->gcbuf : nullptr;
        const uint32_t* wbase = compact ? h->gwbase + (size_t)g * (size_t)(h->g_row_wgs * (ROW_TPB / WAVE)) : nullptr;
        if (streamed && !last) SNAP_TRY(acquire_map(h, (int)(gi % 3), sprof ? h->gev_prof[4 * gi + 2] : nullptr));
        else if (sprof) SNAP_HIP(hipEventRecord(h->gev_prof[4 * gi + 2], h->compute));
        if (n > 0 && (scatter || histo)) {
            // (profile: the two events take the kernel's own start and end times; events recorded between
            // the launches instead cost the chain of dependent kernels 3 us each)
            // profile = 2 times one pass in four, a different one every epoch: even the attached events
            // hold the chain up a little (4.67 / 4.72 / 4.87 ms per epoch with none / a quarter / all timed)
            const bool timed = prof && (h->opt.profile != 2 || ((n_pass + h->epochs_done) & 3) == 0);
            if (prof) h->pass_timed[(size_t)n_pass] = timed ? 1 : 0;   // (sized with the events, at set-up)
            hipEvent_t ev_a = timed ? h->ev_group[2 * n_pass] : nullptr, ev_b = timed ? h->ev_group[2 * n_pass + 1] : nullptr;
            // the first writing pass of an epoch that may be undone writes into the other array
            const float* vin = v_cur;
            float* vout = (scatter && keep_old && !swapped) ? h->v_snap : v_cur;
            // byte maps where the group has one (resident 16-bit maps only); a pass that uses one map names its type twice
            const int slot_p = (prev >= 0 && !streamed && h->g8slot_host) ? h->g8slot_host[prev] : -1;
            const int slot_c = (!last && !streamed && h->g8slot_host) ? h->g8slot_host[g] : -1;
            auto launch = [&](auto tag_p, auto tag_c) {
                using MP = decltype(tag_p);
                using MC = decltype(tag_c);
                const MP* mp = std::is_same<MP, uint8_t>::value ? (const MP*)(h->rowmap8 + (size_t)std::max(slot_p, 0) * h->n_pad)
                                                                : (const MP*)map_prev;
                const MC* mc = std::is_same<MC, uint8_t>::value ? (const MC*)(h->rowmap8 + (size_t)std::max(slot_c, 0) * h->n_pad)
                                                                : (const MC*)map_cur;
                if (scatter && histo)
                    hipExtLaunchKernelGGL((k_group_rows<KIND, UNIT, true, true, MP, MC>), row_grid, dim3(ROW_TPB), lds, h->compute,
                                          ev_a, ev_b, 0, mp, val_prev, delta_prev, mc, val_cur, hot, k64, vin, vout, h->y,
                                          h->ybits, n, gpart, h->gpartial_stride, scale, kd, h->status, cbuf, wbase, (double*)nullptr,
                                          (const float*)nullptr, (int64_t)0);
                else if (scatter && last && h->g_want_loss) {
                    hipExtLaunchKernelGGL((k_group_rows<KIND, UNIT, true, false, MP, MP, true>), row_grid, dim3(ROW_TPB), lds, h->compute,
                                          ev_a, ev_b, 0, mp, val_prev, delta_prev, (const MP*)nullptr, val_cur, 0, 0, vin, vout, h->y,
                                          h->ybits, n, gpart, h->gpartial_stride, scale, kd, h->status, (float*)nullptr,
                                          (const uint32_t*)nullptr, h->gloss_partial, (const float*)h->x, h->m);
                    loss_done = true;
                } else if (scatter)
                    hipExtLaunchKernelGGL((k_group_rows<KIND, UNIT, true, false, MP, MP>), row_grid, dim3(ROW_TPB), lds, h->compute,
                                          ev_a, ev_b, 0, mp, val_prev, delta_prev, (const MP*)nullptr, val_cur, 0, 0, vin, vout, h->y,
                                          h->ybits, n, gpart, h->gpartial_stride, scale, kd, h->status, (float*)nullptr,
                                          (const uint32_t*)nullptr, (double*)nullptr, (const float*)nullptr, (int64_t)0);
                else
                    hipExtLaunchKernelGGL((k_group_rows<KIND, UNIT, false, true, MC, MC>), row_grid, dim3(ROW_TPB), lds, h->compute,
                                          ev_a, ev_b, 0, (const MC*)nullptr, val_prev, delta_prev, mc, val_cur, hot, k64, vin, vout, h->y,
                                          h->ybits, n, gpart, h->gpartial_stride, scale, kd, h->status, cbuf, wbase, (double*)nullptr,
                                          (const float*)nullptr, (int64_t)0);
            };
            if constexpr (std::is_same<MAPT, uint16_t>::value) {
                // (a pass with one map takes that map's type for both)
                const bool p8 = scatter ? slot_p >= 0 : slot_c >= 0, c8 = histo ? slot_c >= 0 : slot_p >= 0;
                if (p8 && c8) launch(uint8_t{}, uint8_t{});
                else if (p8) launch(uint8_t{}, uint16_t{});
                else if (c8) launch(uint16_t{}, uint8_t{});
                else launch(uint16_t{}, uint16_t{});
            } else {
                launch(MAPT{}, MAPT{});
            }
            if (vout != v_cur) {
                v_cur = vout;
                swapped = true;
            }
            ++n_pass;
        }
        if (streamed) {
            // the previous visit's map has had its last reader; the slot it frees takes the map of the
            // visit after next
            if (gi >= 1) SNAP_HIP(hipEventRecord(h->gev_free[(gi - 1) % 3], h->compute));
            if (gi + 2 < n_visit) SNAP_TRY(enqueue_map_copy(h, visits[(size_t)(gi + 2)], (int)((gi + 2) % 3), sprof ? gi + 2 : -1));
        }
        if (!last) {
            const int n_hot_blocks = (hot + STEP_RANKS - 1) / STEP_RANKS;
            const int64_t cold = sz - hot;
            const int waves_per_block = STEP_RANKS * STEP_PARTS / WAVE;
            const int per_block = compact ? STEP_RANKS * STEP_PARTS / 16 : waves_per_block;   // coordinates per pass of a workgroup
            const int n_cold_blocks = (int)std::min<int64_t>((cold + per_block - 1) / per_block, 8192);
            hipLaunchKernelGGL((k_group_finish<KIND, false>), dim3((unsigned)(n_hot_blocks + n_cold_blocks)),
                               dim3(STEP_RANKS * STEP_PARTS), 0, h->compute, gpart, h->gpartial_stride, h->g_row_wgs, hot, k64,
                               n_hot_blocks, 1.0 / (double)scale.g, 1.0 / (double)scale.h, h->ptr, h->idx, h->val, v_cur, h->y, h->coord_of, g0, sz, h->x, h->norms,
                               h->gdelta, sp, nullptr, cbuf, h->gcidx, h->gcptr, UNIT ? 1 : 0);
        }
        if (sprof) SNAP_HIP(hipEventRecord(h->gev_prof[4 * gi + 3], h->compute));
        if (last) break;
        prev = g;
    }
    if (streamed) {
        h->g_visits = n_visit;
        h->gprof_valid = sprof;                      // (a pass over listed groups is not timed)
        // the host does not run ahead of the copy stream by more than a pass (see for_each_chunk)
        SNAP_HIP(hipStreamSynchronize(h->copy));
    }
    if (swapped) std::swap(h->v, h->v_snap);       // v: the state after the epoch; v_snap: the one before it
    h->g_swapped = swapped;
    h->g_want_loss = loss_done;                    // (tells the caller whether the loss sums are there)
    h->n_row_passes = n_pass;
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

// Inner products of every coordinate with loss'(v) (the gradient of the loss term times n), for the
// objective / duality-gap pass: the same row passes as an epoch, sums only, nothing is stepped.
template <int KIND, bool UNIT, typename MAPT>
static int grouped_dots_kind(snap_handle* h) {
    const StepParams sp = make_step_params(h);
    const int64_t n = h->n, G = h->n_groups;
    long long* gpart = (long long*)h->gpartial;
    const SumScales scale = sum_scales(h);
    const MAPT* maps = (const MAPT*)h->rowmap;
    // streamed row maps: one map per pass through the ring of three, copies two passes ahead
    const bool streamed = h->gstream;
    std::vector<int64_t> visits;
    for (int64_t g = 0; g < G; ++g)
        if (h->gbounds_host[g + 1] > h->gbounds_host[g]) visits.push_back(g);
    const int64_t n_visit = (int64_t)visits.size();
    if (streamed)
        for (int64_t i = 0; i < std::min<int64_t>(3, n_visit); ++i) SNAP_TRY(enqueue_map_copy(h, visits[(size_t)i], (int)(i % 3), -1));
    for (int64_t gi = 0; gi < n_visit; ++gi) {
        const int64_t g = visits[(size_t)gi];
        const int64_t g0 = h->gbounds_host[g], sz = h->gbounds_host[g + 1] - g0;
        const int hot = h->ghot_host[g], k64 = h->gk64_host[g];
        const bool compact = h->gcompact_host[g] && n > 0;
        float* cbuf = compact ? h->gcbuf : nullptr;
        const uint32_t* wbase = compact ? h->gwbase + (size_t)g * (size_t)(h->g_row_wgs * (ROW_TPB / WAVE)) : nullptr;
        const MAPT* map_cur = streamed ? (const MAPT*)h->gring[gi % 3] : maps + (size_t)g * h->n_pad;
        if (streamed) SNAP_TRY(acquire_map(h, (int)(gi % 3), nullptr));
        if (n > 0 && (hot > 0 || compact)) {
            const size_t lds = (size_t)(hot + k64) * sizeof(unsigned long long) + sizeof(float) +
                               (compact ? (size_t)(ROW_TPB / WAVE) * COLD_RING * sizeof(float) : 0);
            const int slot_c = (!streamed && h->g8slot_host) ? h->g8slot_host[g] : -1;
            auto launch = [&](auto tag_c, const void* map) {
                using MC = decltype(tag_c);
                hipLaunchKernelGGL((k_group_rows<KIND, UNIT, false, true, MC, MC>), dim3((unsigned)h->g_row_wgs), dim3(ROW_TPB), lds,
                                   h->compute, (const MC*)nullptr, (const float*)nullptr, (const float*)nullptr,
                                   (const MC*)map, UNIT ? (const float*)nullptr : h->rowval + (size_t)g * h->n_pad, hot,
                                   k64, h->v, h->v, h->y, h->ybits, n, gpart, h->gpartial_stride, scale, 0, h->status, cbuf,
                                   wbase, (double*)nullptr, (const float*)nullptr, (int64_t)0);
            };
            if (slot_c >= 0) launch(uint8_t{}, h->rowmap8 + (size_t)slot_c * h->n_pad);
            else launch(MAPT{}, map_cur);
        }
        if (streamed) {
            SNAP_HIP(hipEventRecord(h->gev_free[gi % 3], h->compute));
            if (gi + 3 < n_visit) SNAP_TRY(enqueue_map_copy(h, visits[(size_t)(gi + 3)], (int)((gi + 3) % 3), -1));
        }
        const int n_hot_blocks = (hot + STEP_RANKS - 1) / STEP_RANKS;
        const int64_t cold = sz - hot;
        const int waves_per_block = STEP_RANKS * STEP_PARTS / WAVE;
        const int per_block = compact ? STEP_RANKS * STEP_PARTS / 16 : waves_per_block;
        const int n_cold_blocks = (int)std::min<int64_t>((cold + per_block - 1) / per_block, 8192);
        if (n_hot_blocks + n_cold_blocks > 0)
            hipLaunchKernelGGL((k_group_finish<KIND, true>), dim3((unsigned)(n_hot_blocks + n_cold_blocks)),
                               dim3(STEP_RANKS * STEP_PARTS), 0, h->compute, gpart, h->gpartial_stride, h->g_row_wgs, hot, k64,
                               n_hot_blocks, 1.0 / (double)scale.g, 1.0 / (double)scale.h, h->ptr, h->idx, h->val, h->v, h->y, h->coord_of, g0, sz, h->x, h->norms,
                               h->gdelta, sp, h->gdot, cbuf, h->gcidx, h->gcptr, UNIT ? 1 : 0);
    }
    if (streamed) SNAP_HIP(hipStreamSynchronize(h->copy));
    SNAP_HIP(hipGetLastError());
    return SNAP_OK;
}

template <int KIND>
static int grouped_dots_dispatch(snap_handle* h) {
    if (h->map16)
        return h->unit_values ? grouped_dots_kind<KIND, true, uint16_t>(h) : grouped_dots_kind<KIND, false, uint16_t>(h);
    return h->unit_values ? grouped_dots_kind<KIND, true, uint32_t>(h) : grouped_dots_kind<KIND, false, uint32_t>(h);
}

int grouped_dots(snap_handle* h) {
    return h->kind == K_PRIMAL_RIDGE ? grouped_dots_dispatch<K_PRIMAL_RIDGE>(h)
                                     : grouped_dots_dispatch<K_PRIMAL_LOGISTIC>(h);
}

template <int KIND>
static int grouped_epoch_dispatch(snap_handle* h) {
    if (h->map16)
        return h->unit_values ? grouped_epoch_kind<KIND, true, uint16_t>(h) : grouped_epoch_kind<KIND, false, uint16_t>(h);
    return h->unit_values ? grouped_epoch_kind<KIND, true, uint32_t>(h) : grouped_epoch_kind<KIND, false, uint32_t>(h);
}

int grouped_epoch(snap_handle* h) {
    return h->kind == K_PRIMAL_RIDGE ? grouped_epoch_dispatch<K_PRIMAL_RIDGE>(h)
                                     : grouped_epoch_dispatch<K_PRIMAL_LOGISTIC>(h);
}

}  // namespace snap
