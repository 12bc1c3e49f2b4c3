// A measurement aid, not a step of the method: what bare streaming kernels reach on this device, to set
// the time of the group sweeps' row pass (Section 3.1's update of the shared vector, done for a whole
// one-hot field at once) beside something measured rather than beside the data sheet alone.
//   kind 0: read only (4 bytes per row)
//   kind 1: copy (read 4, write 4)
//   kind 2: the row pass's mix with two-byte row maps: read 4 + 2 + 2, write 4 bytes per row,
//           from four arrays laid out and alternated the way the row pass alternates them
// The kernels do nothing else (an add per element so that the loads cannot be dropped).
#include "common.h"
#include <algorithm>

namespace snap {

typedef float probe_f4 __attribute__((ext_vector_type(4)));
typedef unsigned probe_u2 __attribute__((ext_vector_type(2)));

template <int TPB>
__global__ void __launch_bounds__(TPB) k_probe_read(const probe_f4* __restrict__ in, float* __restrict__ sink, int64_t packs) {
    float s = 0.0f;
    for (int64_t q = (int64_t)blockIdx.x * TPB + threadIdx.x; q < packs; q += (int64_t)gridDim.x * TPB) {
        const probe_f4 a = in[q];
        s += a.x + a.y + a.z + a.w;
    }
    if (s == 12345.678f) sink[0] = s;            // (never true for the zeros the probe reads; keeps the loads)
}

template <int TPB>
__global__ void __launch_bounds__(TPB) k_probe_copy(const probe_f4* __restrict__ in, probe_f4* __restrict__ out, int64_t packs) {
    for (int64_t q = (int64_t)blockIdx.x * TPB + threadIdx.x; q < packs; q += (int64_t)gridDim.x * TPB) out[q] = in[q];
}

// every workgroup takes one contiguous slab of the rows, as the row pass does; U packs of four rows per
// thread and iteration, all loads ahead of the first use
template <int U, bool NT, int TPB>
__global__ void __launch_bounds__(TPB) k_probe_mix(const probe_f4* __restrict__ vin, probe_f4* __restrict__ vout,
                                                   const probe_u2* __restrict__ ma, const probe_u2* __restrict__ mb, int64_t packs) {
    const int64_t per = (packs + gridDim.x - 1) / gridDim.x;
    const int64_t q0 = min(packs, (int64_t)blockIdx.x * per), q1 = min(packs, q0 + per);
    for (int64_t q = q0 + threadIdx.x; q < q1; q += (int64_t)U * TPB) {
        probe_f4 a[U];
        probe_u2 x[U], y[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t qq = q + (int64_t)u * TPB;
            if (qq < q1) {
                a[u] = NT ? __builtin_nontemporal_load(vin + qq) : vin[qq];
                x[u] = NT ? __builtin_nontemporal_load(ma + qq) : ma[qq];
                y[u] = NT ? __builtin_nontemporal_load(mb + qq) : mb[qq];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t qq = q + (int64_t)u * TPB;
            if (qq < q1) {
                a[u].x += (float)(x[u].x & 1u) + (float)(y[u].x & 2u);
                a[u].y += (float)(x[u].y & 1u);
                a[u].z += (float)(y[u].y & 1u);
                if (NT) __builtin_nontemporal_store(a[u], vout + qq);
                else vout[qq] = a[u];
            }
        }
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
    SNAP_TRY(fill_zero(pb.a, (size_t)n * sizeof(float), s));
    SNAP_TRY(fill_zero(pb.b, (size_t)n * sizeof(float), s));
    if (kind == 2)
        for (auto& m : pb.maps) {
            SNAP_HIP(hipMalloc(&m, (size_t)n * sizeof(uint16_t)));
            SNAP_TRY(fill_zero(m, (size_t)n * sizeof(uint16_t), s));
        }
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
                    if (shape == 0)
                        hipLaunchKernelGGL((k_probe_mix<4, true, 256>), dim3(4096), dim3(256), 0, s, (const probe_f4*)in, (probe_f4*)out, ma, mb, packs);
                    else if (shape == 1)
                        hipLaunchKernelGGL((k_probe_mix<1, false, 1024>), dim3(256), dim3(1024), 0, s, (const probe_f4*)in, (probe_f4*)out, ma, mb, packs);
                    else
                        hipLaunchKernelGGL((k_probe_mix<2, false, 512>), dim3(1024), dim3(512), 0, s, (const probe_f4*)in, (probe_f4*)out, ma, mb, packs);
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
