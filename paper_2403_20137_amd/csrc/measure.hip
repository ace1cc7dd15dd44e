// Measurement aid of libkvbfp: a read-only pass over exactly the cache bytes that decode attention
// streams (Sec. III run-time flow: the cached keys and values are read back once per decode step), with
// no arithmetic on them.  Its rate is the ceiling a kernel of that size and shape can reach on the
// machine, which is what the split pass of kvbfp_decode_attention is compared with.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kvbfp_internal.h"

using namespace kvbfp;

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct StreamArgs {
    const uint8_t* plane[4];
    int64_t unit_stride[4];     // bytes between the regions of consecutive (batch, kv-head) units
    int64_t unit_bytes[4];      // bytes read per unit
    uint32_t* sink;
};

// grid = (wgs per unit, units), block = 256.  Workgroup w of a unit takes the chunks w, w + n, ... of each
// plane's region, kUnroll loads of 16 bytes per lane in flight (chunks of kUnroll x 4 KB), so the workgroups of a
// unit sweep the region side by side.  How much a wavefront should keep in flight depends on the shape: with
// three workgroups per compute unit the 285 MB of the 32k-context workload take 45.0 / 46.0 / 46.9 / 47.5 us with
// 2 / 4 / 8 / 16 loads per lane (and 61 us with one), while shapes with fewer workgroups want more.  The
// measurement call therefore runs the forms with 2 and with 8 and reports the faster.
template <int kUnroll>
__global__ __launch_bounds__(256) void stream_read_kernel(StreamArgs a) {
    const int64_t unit = blockIdx.y;
    uint32_t acc = 0;
#pragma unroll 1
    for (int pl = 0; pl < 4; ++pl) {
        const uint8_t* p0 = a.plane[pl] + unit * a.unit_stride[pl];
        const uint8_t* p1 = p0 + a.unit_bytes[pl];
        // whole 16-byte words inside [p0, p1) (an exponent region may start and end off a 16-byte boundary)
        const u32x4* lo = (const u32x4*)(((uintptr_t)p0 + 15) & ~(uintptr_t)15);
        const u32x4* hi = (const u32x4*)((uintptr_t)p1 & ~(uintptr_t)15);
        const int64_t n_vec = hi > lo ? (int64_t)(hi - lo) : 0;
        const int64_t chunk = 256 * kUnroll;
        for (int64_t c0 = (int64_t)blockIdx.x * chunk; c0 < n_vec; c0 += (int64_t)gridDim.x * chunk) {
            u32x4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t i = c0 + u * 256 + threadIdx.x;
                v[u] = i < n_vec ? __builtin_nontemporal_load(lo + i) : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
        }
    }
    // keeps the loads alive; practically never taken
    if (acc == 0x9E3779B9u) a.sink[0] = acc;
}

}  // namespace

extern "C" int kvbfp_measure_stream_read(const kvbfp_layout* L, const kvbfp_cache* cache, int64_t n_tok,
                                         int32_t wgs_per_unit, void* sink, void* hip_stream, float* kernel_ms) {
    clear_error();
    if (int rc = check_device_layout(L)) return rc;
    if (int rc = check_cache(cache, true, true)) return rc;
    if (!sink || !kernel_ms) return fail(KVBFP_ERR_INVALID_ARG, "measure_stream_read: sink/kernel_ms is NULL");
    if (n_tok <= 0 || n_tok > L->max_seq)
        return fail(KVBFP_ERR_INVALID_ARG, "measure_stream_read: n_tok %lld outside (0, max_seq]", (long long)n_tok);
    const int64_t units = (int64_t)L->batch * L->n_kv_heads;
    if (units > 65535) return fail(KVBFP_ERR_UNSUPPORTED, "measure_stream_read: too many (batch, kv-head) units");
    if (wgs_per_unit <= 0) {      // about eight workgroups per compute unit
        wgs_per_unit = (int32_t)((2048 + units - 1) / units);
    }
    if (wgs_per_unit > 1024) wgs_per_unit = 1024;
    const int64_t row_m = (int64_t)L->head_dim * L->mant_bits / 8, row_e = L->head_dim / L->block;
    StreamArgs a{};
    a.plane[0] = cache->k_mant; a.plane[1] = cache->v_mant; a.plane[2] = cache->k_exp; a.plane[3] = cache->v_exp;
    for (int i = 0; i < 4; ++i) {
        const int64_t row = i < 2 ? row_m : row_e;
        a.unit_stride[i] = L->max_seq * row;
        a.unit_bytes[i] = n_tok * row;
    }
    a.sink = (uint32_t*)sink;
    hipStream_t s = (hipStream_t)hip_stream;
    hipEvent_t ev[2] = {nullptr, nullptr};
    if (hipEventCreate(&ev[0]) != hipSuccess) return fail(KVBFP_ERR_HIP, "measure_stream_read: hipEventCreate failed");
    if (hipEventCreate(&ev[1]) != hipSuccess) {
        (void)hipEventDestroy(ev[0]);
        return fail(KVBFP_ERR_HIP, "measure_stream_read: hipEventCreate failed");
    }
    hipError_t err = hipSuccess;
    float best = 0.f;
    const dim3 grid((unsigned)wgs_per_unit, (unsigned)units, 1);
    for (int form = 0; form < 2 && err == hipSuccess; ++form) {
        (void)hipEventRecord(ev[0], s);
        if (form == 0) stream_read_kernel<2><<<grid, 256, 0, s>>>(a);
        else stream_read_kernel<8><<<grid, 256, 0, s>>>(a);
        err = hipGetLastError();
        (void)hipEventRecord(ev[1], s);
        hipError_t e2 = hipEventSynchronize(ev[1]);
        float ms = 0.f;
        if (e2 == hipSuccess) e2 = hipEventElapsedTime(&ms, ev[0], ev[1]);
        if (err == hipSuccess) err = e2;
        if (form == 0 || ms < best) best = ms;
    }
    *kernel_ms = best;
    (void)hipEventDestroy(ev[0]);
    (void)hipEventDestroy(ev[1]);
    if (err != hipSuccess) return fail(KVBFP_ERR_HIP, "measure_stream_read: %s", hipGetErrorString(err));
    return KVBFP_OK;
}
