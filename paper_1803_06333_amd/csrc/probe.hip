// A measurement aid, not a step of the method: what bare streaming kernels reach on this device, to set
// the time of the group sweeps' row pass (Section 3.1's update of the shared vector, done for a whole
// one-hot field at once) beside something measured rather than beside the data sheet alone.
//   kind 0: read only (4 bytes per row)
//   kind 1: copy (read 4, write 4)
//   kind 2: the row pass's mix with two-byte row maps: read 4 + 2 + 2, write 4 bytes per row,
//           walking the rows the way the row pass walks them, the maps alternated as the sweeps alternate them
// The kernels do nothing else (an add per element so that the loads cannot be dropped).  The arrays hold
// a pattern, not zeros (all-zero data was measured 15 % faster than any other).
#include "common.h"
#include <algorithm>

namespace snap {

typedef float probe_f4 __attribute__((ext_vector_type(4)));
typedef unsigned probe_u2 __attribute__((ext_vector_type(2)));

__global__ void k_probe_fill(uint32_t* p, int64_t count, uint32_t base, uint32_t mask) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = base | ((uint32_t)i * 2654435761u & mask);
}

template <int TPB>
__global__ void __launch_bounds__(TPB) k_probe_read(const probe_f4* __restrict__ in, float* __restrict__ sink, int64_t packs) {
    float s = 0.0f;
    for (int64_t q = (int64_t)blockIdx.x * TPB + threadIdx.x; q < packs; q += (int64_t)gridDim.x * TPB) {
        const probe_f4 a = in[q];
        s += a.x + a.y + a.z + a.w;
    }
    if (s == 12345.678f) sink[0] = s;            // (practically never true; keeps the loads)
}

template <int TPB>
__global__ void __launch_bounds__(TPB) k_probe_copy(const probe_f4* __restrict__ in, probe_f4* __restrict__ out, int64_t packs) {
    for (int64_t q = (int64_t)blockIdx.x * TPB + threadIdx.x; q < packs; q += (int64_t)gridDim.x * TPB) out[q] = in[q];
}

// the workgroups walk the rows side by side, as the row pass does (in iteration i workgroup b takes the TPB
// packs from (i * gridDim.x + b) * TPB on), one pack of four rows per thread and iteration, the next
// pack's loads asked for before the work on the current one; vin may equal vout (the row pass updates the
// shared vector in place unless an epoch's earlier state must survive).  NTV / NTM: non-temporal loads of
// the vector / of the two maps.
template <bool NTV, bool NTM, int TPB>
__global__ void __launch_bounds__(TPB) k_probe_mix(const probe_f4* vin, probe_f4* vout, const probe_u2* __restrict__ ma,
                                                   const probe_u2* __restrict__ mb, int64_t packs) {
    const int64_t stride = (int64_t)gridDim.x * TPB;
    int64_t q = (int64_t)blockIdx.x * TPB + threadIdx.x;
    probe_f4 a = {};
    probe_u2 x = {}, y = {};
    auto request = [&](int64_t qq) {
        a = NTV ? __builtin_nontemporal_load(vin + qq) : vin[qq];
        x = NTM ? __builtin_nontemporal_load(ma + qq) : ma[qq];
        y = NTM ? __builtin_nontemporal_load(mb + qq) : mb[qq];
    };
    if (q < packs) request(q);
    while (q < packs) {
        probe_f4 t = a;
        const probe_u2 xx = x, yy = y;
        const int64_t qn = q + stride;
        if (qn < packs) request(qn);
        t.x += (float)(xx.x & 1u) + (float)(yy.x & 2u);
        t.y += (float)(xx.y & 1u);
        t.z += (float)(yy.y & 1u);
        vout[q] = t;
        q = qn;
    }
}

struct ProbeBuffers {
    float *a = nullptr, *b = nullptr;
    uint16_t* maps[4] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~ProbeBuffers() {
        (void)hipFree(a);
        (void)hipFree(b);
        for (auto m : maps) (void)hipFree(m);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

static int probe_run(int kind, int64_t rows, int passes, hipStream_t s, double* us_per_pass) {
    const int64_t n = (rows + 3) / 4 * 4, packs = n / 4;
    ProbeBuffers pb;
    SNAP_HIP(hipMalloc(&pb.a, (size_t)n * sizeof(float)));
    SNAP_HIP(hipMalloc(&pb.b, (size_t)n * sizeof(float)));
    // floats in [1, 2) and arbitrary map words
    hipLaunchKernelGGL(k_probe_fill, dim3(4096), dim3(256), 0, s, (uint32_t*)pb.a, n, 0x3F800000u, 0x007FFFFFu);
    hipLaunchKernelGGL(k_probe_fill, dim3(4096), dim3(256), 0, s, (uint32_t*)pb.b, n, 0x3F800000u, 0x007FFFFFu);
    if (kind == 2)
        for (auto& m : pb.maps) {
            SNAP_HIP(hipMalloc(&m, (size_t)n * sizeof(uint16_t)));
            hipLaunchKernelGGL(k_probe_fill, dim3(4096), dim3(256), 0, s, (uint32_t*)m, n / 2, 0u, 0xFFFFFFFFu);
        }
    SNAP_HIP(hipGetLastError());
    SNAP_HIP(hipEventCreate(&pb.e0));
    SNAP_HIP(hipEventCreate(&pb.e1));
    const int n_shapes = kind == 2 ? 3 : 2;
    double best = 0.0;
    for (int shape = 0; shape < n_shapes; ++shape) {
        for (int rep = 0; rep < 3; ++rep) {            // (the first repetition of a shape also warms it up)
            SNAP_HIP(hipEventRecord(pb.e0, s));
            for (int p = 0; p < passes; ++p) {
                const float* in = (p & 1) ? pb.b : pb.a;
                float* out = (p & 1) ? pb.a : pb.b;
                if (kind == 0) {
                    if (shape == 0) hipLaunchKernelGGL((k_probe_read<256>), dim3(2048), dim3(256), 0, s, (const probe_f4*)in, out, packs);
                    else hipLaunchKernelGGL((k_probe_read<1024>), dim3(256), dim3(1024), 0, s, (const probe_f4*)in, out, packs);
                } else if (kind == 1) {
                    if (shape == 0) hipLaunchKernelGGL((k_probe_copy<256>), dim3(4096), dim3(256), 0, s, (const probe_f4*)in, (probe_f4*)out, packs);
                    else hipLaunchKernelGGL((k_probe_copy<1024>), dim3(256), dim3(1024), 0, s, (const probe_f4*)in, (probe_f4*)out, packs);
                } else {
                    const probe_u2* ma = (const probe_u2*)pb.maps[p & 3];
                    const probe_u2* mb = (const probe_u2*)pb.maps[(p + 1) & 3];
                    // in place with the hint on the maps (what the row pass does), the same between two arrays,
                    // and between two arrays with the hint on every load
                    if (shape == 0)
                        hipLaunchKernelGGL((k_probe_mix<false, true, 1024>), dim3(256), dim3(1024), 0, s, (const probe_f4*)pb.a, (probe_f4*)pb.a, ma, mb, packs);
                    else if (shape == 1)
                        hipLaunchKernelGGL((k_probe_mix<false, true, 1024>), dim3(256), dim3(1024), 0, s, (const probe_f4*)in, (probe_f4*)out, ma, mb, packs);
                    else
                        hipLaunchKernelGGL((k_probe_mix<true, true, 1024>), dim3(256), dim3(1024), 0, s, (const probe_f4*)in, (probe_f4*)out, ma, mb, packs);
                }
            }
            SNAP_HIP(hipEventRecord(pb.e1, s));
            SNAP_HIP(hipEventSynchronize(pb.e1));
            SNAP_HIP(hipGetLastError());
            float ms = 0.0f;
            SNAP_HIP(hipEventElapsedTime(&ms, pb.e0, pb.e1));
            const double us = 1e3 * (double)ms / (double)passes;
            if (rep > 0 && (best == 0.0 || us < best)) best = us;
        }
    }
    *us_per_pass = best;
    return SNAP_OK;
}

}  // namespace snap

extern "C" int snap_stream_probe(int kind, int64_t rows, int passes, void* stream, double* us_per_pass) {
    using namespace snap;
    if (kind < 0 || kind > 2 || rows < 1 || rows > ((int64_t)1 << 32) || passes < 1 || passes > 1000 || !us_per_pass) {
        set_error("snap_stream_probe: kind in 0..2, rows in 1..2^32, passes in 1..1000, us_per_pass not NULL");
        return SNAP_EINVAL;
    }
    return probe_run(kind, rows, passes, (hipStream_t)stream, us_per_pass);
}
