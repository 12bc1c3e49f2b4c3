// Internal declarations shared by the HIP sources of libsnap (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstddef>
#include <vector>
#include "../../include/snap.h"

namespace snap {

// ---- error plumbing --------------------------------------------------------------------------
void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what, const char* file, int line);

#define SNAP_HIP(call)                                                         \
    do {                                                                       \
        hipError_t e_ = (call);                                                \
        if (e_ != hipSuccess) return ::snap::hip_fail(e_, #call, __FILE__, __LINE__); \
    } while (0)

#define SNAP_TRY(call)                 \
    do {                               \
        int rc_ = (call);              \
        if (rc_ != SNAP_OK) return rc_; \
    } while (0)

// ---- constants -------------------------------------------------------------------------------
constexpr int WAVE = 64;
constexpr int TPB = 256;                 // threads per workgroup of the epoch kernels (4 waves)
constexpr int WAVES_PER_WG = TPB / WAVE;
// A coordinate with more nonzeros than SMALL_MAX is split into segments of SEG nonzeros, one
// workgroup each (two phases: partial dots, then scatter).
constexpr int64_t SEG_DEFAULT = 16384;
constexpr int64_t SMALL_MAX_DEFAULT = 4096;
constexpr uint32_t LABEL_BIT = 0x80000000u;   // primal logistic: sign of y folded into the row index
constexpr uint32_t STATUS_SPIN = 1u;          // status word: a scatter item gave up waiting for its coordinate's step
constexpr uint32_t STATUS_RANGE = 8u;         // status word: a term too large for the fixed-point sums of a group sweep
constexpr uint32_t SPIN_LIMIT = 1u << 22;     // bounded wait of a scatter item for its coordinate's step

// K_DUAL: examples as coordinates (hinge or logistic loss: the kernels differ only in the scalar step)
enum Kind { K_PRIMAL_RIDGE = 0, K_PRIMAL_LOGISTIC = 1, K_DUAL = 2 };
constexpr double ALPHA_EPS = 1.0 / 1048576.0;   // logistic dual: the iterates stay in [2^-20, 1 - 2^-20]

// Per-epoch state of one split ("large") coordinate, indexed by its position in the epoch order.
struct LargeState {
    double g, h;          // accumulated partial sums of the dot phase
    uint64_t published;   // (1 << 32) | bits of the scatter multiplier, written once by one 64-bit store
    uint32_t done;        // dot items finished
    uint32_t pad;
};

// One chunk of coordinates [c0, c1) whose nonzeros [ptr[c0], ptr[c1]) sit in (idx, val).
struct ChunkView {
    const int64_t* ptr;       // device, absolute offsets, indexed by absolute coordinate
    const uint32_t* idx;      // device, element k of the matrix at idx[k - nnz_base]
    const float* val;
    int64_t nnz_base;
    int64_t c0, c1;
};

struct Sorter {              // scratch of the radix sort, sized for max_m coordinates
    uint32_t *keys_a = nullptr, *keys_b = nullptr, *vals_a = nullptr, *vals_b = nullptr;
    uint32_t* block_hist = nullptr;
    int64_t max_m = 0;
    int64_t n_blocks = 0;
};

struct Reducer {             // scratch for deterministic fp64 reductions
    double* partial = nullptr;   // [REDUCE_BLOCKS * 4]
    double* result = nullptr;    // [8] device
    double* host = nullptr;      // [8] pinned host, mapped into the device's address space
    double* host_mapped = nullptr;   // the device's pointer to the same memory
};
constexpr int REDUCE_BLOCKS = 1024;

}  // namespace snap

struct snap_handle {
    int layout = 0, loss = 0, form = 0, kind = 0;
    bool dense = false;
    int64_t n = 0, d = 0, nnz = 0;
    int64_t m = 0, vlen = 0;          // coordinates, length of v
    int64_t ld = 0;                   // dense: elements per coordinate (= n)
    int64_t seg = snap::SEG_DEFAULT;  // nonzeros per work item of a split coordinate
    int64_t small_max = snap::SMALL_MAX_DEFAULT;   // longest coordinate handled by one wavefront
    double lambda = 0, lambda1 = 0;
    snap_options opt{};
    int device = 0;

    // resident data (device)
    int64_t* ptr = nullptr;           // [m+1]
    uint32_t* idx = nullptr;          // [nnz] (label bit folded for primal logistic)
    float* val = nullptr;             // [nnz] or dense matrix, coordinate-major
    float* y = nullptr;               // [n]
    float* x = nullptr;               // [m]
    float* v = nullptr;               // [vlen]
    float* norms = nullptr;           // [m] squared norms of the coordinates
    uint8_t* cls = nullptr;           // [m] 0 = small, 1 = large
    float* w_tmp = nullptr;           // [d] scratch: w in dual form
    double* gdot = nullptr;           // [m] per-coordinate dots with v (objective / gap pass)

    // static list of the large coordinates (ascending) with their segment offsets
    int64_t* large_list = nullptr;    // [n_large_total]
    int64_t* large_seg_off = nullptr; // [n_large_total+1]
    double* seg_partial = nullptr;    // [n_seg_total]
    int64_t n_large_total = 0, n_seg_total = 0;

    // epoch order
    snap::Sorter sorter;
    uint32_t* keys = nullptr;         // [m] keys of the last epoch
    uint32_t* perm = nullptr;         // [m] visiting order of the last epoch
    uint32_t* order = nullptr;        // [max chunk m] order partitioned: small first, then large
    int64_t max_chunk_m = 0;

    // split-coordinate bookkeeping (per chunk, sized for the worst chunk)
    snap::LargeState* lstate = nullptr;
    int64_t* item_start = nullptr;    // [n_large+1] prefix sums of items in epoch order
    uint32_t* ticket = nullptr;       // work-item counter
    uint32_t* status = nullptr;       // device error flag
    int64_t max_large = 0;

    // chunks (resident: one chunk covering everything)
    struct Chunk { int64_t c0, c1, nnz0, nnz1, n_small, n_large, n_items, l0, l1; };   // [l0,l1): its range of large_list
    Chunk* chunks = nullptr;
    int64_t n_chunks = 0;
    bool streaming = false;
    bool stream_unit = false;            // streaming: all values are 1.0, only the indices are copied
    const int64_t* host_ptr = nullptr;   // streaming: borrowed pinned arrays
    const int32_t* host_idx = nullptr;
    const float* host_val = nullptr;
    uint32_t* buf_idx[2] = {nullptr, nullptr};
    float* buf_val[2] = {nullptr, nullptr};
    hipEvent_t ev_copied[2] = {nullptr, nullptr}, ev_free[2] = {nullptr, nullptr};
    int64_t buf_chunk[2] = {-1, -1};     // chunk held (or being loaded) by each buffer
    bool buf_folded[2] = {false, false}; // labels already folded into that copy
    int64_t max_chunk_nnz = 0;
    // keys of the epoch order made on the host (options.host_keys): two pinned host buffers and their
    // device twins, used in turn
    uint32_t* hk_host[2] = {nullptr, nullptr};
    uint32_t* hk_dev[2] = {nullptr, nullptr};
    hipEvent_t hk_copied[2] = {nullptr, nullptr}, hk_taken[2] = {nullptr, nullptr};
    int hk_slot = 0;
    hipStream_t hk_stream = nullptr;
    // a pass over part of the chunks (or groups): the list to visit, in order; null = all of them
    const int64_t* pass_list = nullptr;
    int64_t pass_count = 0;
    int64_t bytes_copied = 0;            // streaming: bytes of chunk copies enqueued since creation
    int64_t* share_bounds = nullptr;     // device [chunks + 1]: coordinate ranges for the gap shares
    double* share_out = nullptr;         // device [chunks]
    hipEvent_t* ev_chunk = nullptr;      // profile: 4 events per chunk (copy begin/end, compute begin/end)
    bool chunk_events_valid = false;
    std::vector<char> chunk_copy_timed;  // profile: the chunk's copy events were recorded during the last pass

    // exact group sweeps (coordinates of a group have disjoint supports)
    bool grouped = false;
    bool unit_values = false;         // every stored value is 1.0: no per-row value arrays
    int64_t n_groups = 0, n_pad = 0;  // n_pad: row stride of the per-group row maps (multiple of 8)
    int64_t* gbounds_host = nullptr;  // [n_groups+1]
    int* ghot_host = nullptr;         // [n_groups] number of hot (LDS-accumulated) ranks per group
    int* gk64_host = nullptr;         // [n_groups] of those, the leading ranks that keep two 64-bit sums (the rest: one packed word)
    bool gpack = false;               // packed ranks in use (logistic loss)
    int g_row_wgs = 0, g_kd_max = 0;  // workgroups of a row pass; steps of the previous group kept in LDS
    void* rowmap = nullptr;           // [n_groups][n_pad]: rank of the row's coordinate in the group (uint16 or uint32)
    bool map16 = true;
    uint8_t* rowmap8 = nullptr;       // resident 16-bit maps: byte copies of the maps of groups with at most 255 coordinates
    int* g8slot_host = nullptr;       // [n_groups] which of them (-1: the group has none)
    int n_byte_maps = 0;
    uint8_t* ybits = nullptr;         // bit r = 1 when y[r] < 0
    float* rowval = nullptr;          // [n_groups][n_pad] values (null when unit_values)
    uint32_t* rank_of = nullptr;      // [m] rank of a coordinate inside its group (by decreasing length)
    uint32_t* coord_of = nullptr;     // [m] coordinate at (group start + rank)
    float* gdelta = nullptr;          // [m] step of (group start + rank), read by the next row pass
    void* gpartial = nullptr;         // [row-pass workgroups][2*hot] per-workgroup partial sums (int64 fixed point)
    // short coordinates of a group: the row pass writes the shared-vector entries of their rows, densely,
    // in the order in which it visits them; the finishing kernel gathers from that small buffer
    uint8_t* gcompact_host = nullptr; // [n_groups] 1 when the group's short coordinates are handled that way
    uint32_t* gwbase = nullptr;       // [n_groups][row-pass wavefronts] first buffer position of the wavefront
    uint32_t* gcidx = nullptr;        // per nonzero of a short coordinate: buffer position of its row (| label bit)
    int64_t* gcptr = nullptr;         // [m+1] start in gcidx of (group start + rank); empty for the other ranks
    float* gcbuf = nullptr;           // [largest count over the groups] entries of the shared vector (ridge: minus label)
    int gscale_exp = 0;               // largest |value| <= 2^gscale_exp
    int64_t gpartial_stride = 0;
    hipEvent_t* ev_group = nullptr;   // profile: begin/end of every row pass
    int n_row_passes = 0;
    std::vector<char> pass_timed;        // profile: which row passes of the last epoch carry their two events
    int64_t g_hot_coords = 0, g_hot_nnz = 0;
    // an epoch of group sweeps that may have to be undone (accept check; ridge range guard): its first
    // writing pass reads v and writes v_snap, the later ones work in v_snap, and the two pointers are swapped
    // at the end -- the state before the epoch is then what v_snap holds, at no cost
    bool g_keep_old = false;          // set by snap_epoch for the epoch it is about to run
    bool g_want_loss = false;         // ... and: the last pass sums the loss into gloss_partial
    bool g_swapped = false;           // set by the epoch: v and v_snap have changed roles
    double* gloss_partial = nullptr;  // [row-pass workgroups]
    bool group_fallback = false;      // the group sweeps were left for the asynchronous engine (fixed-point range)
    bool perm_stale = false;          // grouped mode makes the visiting order only on request
    uint64_t last_seed = 0;
    // group sweeps over streamed data: the row maps live in pinned host memory of the library's own and
    // pass through a ring of three device buffers (previous group, current group, the one being copied)
    bool gstream = false;
    void* gmaps_host = nullptr;       // [n_groups][n_pad] row maps (uint16 or uint32), pinned
    void* gring[3] = {nullptr, nullptr, nullptr};                // device, [n_pad] map entries each
    int64_t gring_group[3] = {-1, -1, -1};                       // group whose map a slot holds or is being loaded with
    // a group of at most 255 coordinates crosses the host link as one byte per row and is widened to
    // the two-byte entries of the row pass on the device
    uint8_t* gmap8_host = nullptr;    // [n_groups] how the group's map crosses the host link: 0 as read, 1 bytes, 2 escape-coded bytes, 3 prefix-coded
    uint8_t* gpfx_tab = nullptr;      // device: per group the tables of its prefix code (groups coded that way)
    int64_t* gpfx_words_host = nullptr;   // [n_groups] 32-bit words of the group's prefix-coded stream, padding included
    int64_t* gmap_off_host = nullptr; // [n_groups + 1] byte offset of every group's map in gmaps_host
    uint8_t* gring8[3] = {nullptr, nullptr, nullptr};            // device, [n_pad] bytes each: landing place of a byte map
    bool gring_widened[3] = {false, false, false};               // the slot's byte map has been widened into gring
    hipEvent_t gev_copied[3] = {nullptr, nullptr, nullptr}, gev_free[3] = {nullptr, nullptr, nullptr};
    hipEvent_t* gev_prof = nullptr;   // profile: per visit copy begin / end (copy stream), kernels begin / end (compute stream)
    int64_t g_visits = 0;             // visits of the last pass (for the statistics)
    bool gprof_valid = false;         // the last pass recorded its per-visit events
    std::vector<char> gcopy_timed;    // profile: the visit's map was copied (not found in the ring) in the last pass
    int64_t gmap_bytes_per_pass = 0;  // bytes of row maps that a pass over all groups copies

    // exact tile sweeps (dense ridge): tiles of consecutive columns listed in gbounds_host / n_groups
    bool tiled = false;
    float* tgram = nullptr;           // [tiles][128][128] Gram blocks of the tiles
    float* tpartial = nullptr;        // [tile_wgs][128] per-workgroup partial inner products of the current tile
    float* tmult = nullptr;           // [2][128] steps of the previous / current tile
    int64_t tile_wgs = 0;
    int tile_vec = 4;                 // consecutive rows per thread of the row pass

    hipStream_t compute = nullptr, copy = nullptr;
    hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    // concurrency control and the adaptive safeguard
    int64_t inflight_nnz = 0;         // current cap on nonzeros in flight (<= 0: no cap)
    int64_t inflight_floor = 0;       // the cap is never halved below this
    float damping = 1.0f;
    bool adaptive = true;
    float* x_snap = nullptr;          // [m] state before the epoch (adaptive mode)
    float* v_snap = nullptr;          // [vlen]
    double monitor_prev = 0.0;        // objective before the epoch (minimised quantity)
    bool monitor_valid = false;
    double avg_small_len = 1.0;
    int64_t max_small_len = 0;   // longest coordinate handled by one wavefront
    int64_t nnz_small = 0, nnz_large = 0;
    snap_epoch_stats stats{};
    bool stats_pending = false;
    int64_t epochs_done = 0;
    snap::Reducer red;
};

namespace snap {

// perm.hip
int sorter_alloc(Sorter& s, int64_t max_m);
void sorter_free(Sorter& s);
// keys_out[c] = key(seed, chunk, c) for c in [0, m); order_out = coordinates sorted by (key, c);
// part_out = the same order stably partitioned by cls[c0 + c] (class 0 first); either may be null.
int host_keys_alloc(snap_handle* h, int64_t max_m);   // options.host_keys: pinned key buffers for make_permutation
void host_keys_free(snap_handle* h);
int make_permutation(snap_handle* h, uint64_t seed, uint32_t chunk, int64_t c0, int64_t m,
                     uint32_t* keys_out, uint32_t* order_out, uint32_t* part_out);

// scd.hip
int scd_run_chunk(snap_handle* h, const ChunkView& cv, const snap_handle::Chunk& ck, const uint32_t* order);

// stream.hip: run fn on every chunk in order (resident data: one chunk, no copies).  Streaming:
// double-buffered copies on the copy stream overlap fn's work on the compute stream.
using ChunkFn = int (*)(snap_handle* h, int64_t chunk, const ChunkView& cv, void* arg);
int for_each_chunk(snap_handle* h, ChunkFn fn, void* arg, bool fold, bool profile);
// api.hip: a ridge term beyond the range of the group sweeps' fixed-point sums was seen: clear the flag,
// switch the handle to the asynchronous engine for good
int leave_group_sweeps(snap_handle* h);
int read_status(snap_handle* h, uint32_t* st);      // the status word once the enqueued work is done (synchronises)
// grouped.hip
int grouped_setup(snap_handle* h, const int64_t* hptr, const int64_t* bounds, int64_t n_groups);
int detect_groups(snap_handle* h, const int64_t* hptr, std::vector<int64_t>& bounds);   // empty: nothing found
// the same search piece by piece, for streamed data (advanced as the chunks pass through the device at creation)
struct GroupSearch;
int group_search_begin(snap_handle* h, GroupSearch** out);
int group_search_advance(snap_handle* h, GroupSearch* s, const int64_t* hptr, const uint32_t* idx, int64_t nnz_base, int64_t c_limit);
int group_search_end(snap_handle* h, GroupSearch* s, const int64_t* hptr, std::vector<int64_t>& bounds);
void group_search_free(GroupSearch* s);
int grouped_epoch(snap_handle* h);
int grouped_dots(snap_handle* h);    // gdot[c] = inner product of coordinate c with loss'(v), by row passes
std::vector<int64_t> group_order(uint64_t seed, int64_t n_groups);   // visiting order of the groups for a seed
void grouped_free(snap_handle* h);

// dense_tiles.hip
bool dense_tiles_applicable(const snap_handle* h);
int dense_tiles_setup(snap_handle* h);
int dense_tiles_epoch(snap_handle* h);
void dense_tiles_free(snap_handle* h);

int stream_alloc(snap_handle* h);
void stream_free(snap_handle* h);

// linalg.hip
int norms_and_classes_chunk(snap_handle* h, const ChunkView& cv);
int count_accesses_chunk(snap_handle* h, const ChunkView& cv, int64_t count, uint32_t* freq);
int access_moments(snap_handle* h, const uint32_t* freq, double* eff_len);
int fold_labels(snap_handle* h, uint32_t* idx, int64_t count, hipStream_t s);
int recompute_shared(snap_handle* h);
int fill_value(float* p, float value, int64_t count, hipStream_t s);
int clamp_range(float* p, float lo, float hi, int64_t count, hipStream_t s);
int objective(snap_handle* h, double* primal, double* dual, double* gap);
// the quantity the solver decreases (P in primal form, -D in dual form), vectors only
int monitor_value(snap_handle* h, double* value);
int grouped_loss_value(snap_handle* h, double* value);   // grouped.hip: the same value from the sums the epoch's last row pass left
int chunk_gap_shares(snap_handle* h, double* shares_out);   // host array, one entry per chunk (or group)

int predict(snap_handle* h, const snap_matrix* X, float* out);
int predict_static(snap_handle* h, const snap_matrix* X, float* out);   // no allocation: scratch in a static device array
int weights_to_host(snap_handle* h, float* w_out);
int reducer_alloc(Reducer& r);
void reducer_free(Reducer& r);
int fill_zero(void* p, size_t bytes, hipStream_t s);
// d0[0..n0) = s0, d1[0..n1) = s1 in one launch (arrays from hipMalloc)
int copy_pair(float* d0, const float* s0, int64_t n0, float* d1, const float* s1, int64_t n1, hipStream_t s);

}  // namespace snap
