// Streaming read / copy bandwidth of the device, for reference against the decode kernel.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
template <int U>
__global__ __launch_bounds__(256) void read_nt_kernel(const u32x4_t* __restrict__ p, size_t nvec, uint32_t* sink) {
    size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x;
    size_t stride = (size_t)gridDim.x * 256 * U;
    uint32_t acc = 0;
    for (; i + (size_t)256 * (U - 1) < nvec; i += stride) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + i + (size_t)256 * u);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}
template <int U>
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ p, size_t nvec, uint32_t* sink) {
    size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x;
    size_t stride = (size_t)gridDim.x * 256 * U;
    uint32_t acc = 0;
    for (; i + (size_t)256 * (U - 1) < nvec; i += stride) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = p[i + (size_t)256 * u];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}
// The decode kernel's access pattern without its arithmetic: one workgroup per strip (a K part and a V part
// of `rows` rows of 256 bytes each), its four waves take tiles of U*4 rows round-robin, the next tile's loads
// are issued before the current one is consumed.
template <int U>
__global__ __launch_bounds__(256) void strip_read_kernel(const u32x4_t* __restrict__ p, int rows, size_t strip_vecs, uint32_t* sink) {
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const u32x4_t* k = p + (size_t)blockIdx.x * 2 * strip_vecs;
    const u32x4_t* v = k + strip_vecs;
    constexpr int TILE = U * 4;
    uint32_t acc = 0;
    u32x4_t kr[U], vr[U], kn[U], vn[U];
    int t0 = wave * TILE;
    if (t0 >= rows) return;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int r = min(t0 + u * 4 + lane / 16, rows - 1);
        kr[u] = __builtin_nontemporal_load(k + (size_t)r * 16 + lane % 16);
        vr[u] = __builtin_nontemporal_load(v + (size_t)r * 16 + lane % 16);
    }
    for (; t0 < rows; t0 += 4 * TILE) {
        const int tn = t0 + 4 * TILE;
        if (tn < rows) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = min(tn + u * 4 + lane / 16, rows - 1);
                kn[u] = __builtin_nontemporal_load(k + (size_t)r * 16 + lane % 16);
                vn[u] = __builtin_nontemporal_load(v + (size_t)r * 16 + lane % 16);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= kr[u].x ^ kr[u].w ^ vr[u].y ^ vr[u].z;
        if (tn < rows) {
#pragma unroll
            for (int u = 0; u < U; ++u) { kr[u] = kn[u]; vr[u] = vn[u]; }
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;
}
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ p, uint4* __restrict__ q, size_t nvec) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t stride = (size_t)gridDim.x * 256;
    for (; i < nvec; i += stride) q[i] = p[i];
}
int main() {
    size_t bytes = (size_t)1 << 30;
    uint4 *a, *b; uint32_t* sink;
    uint4* big;                                        // a and b are the two halves of one allocation
    CK(hipMalloc(&big, 2 * bytes)); CK(hipMalloc(&sink, 4));
    a = big; b = big + bytes / 16;
    CK(hipMemset(a, 1, bytes)); CK(hipMemset(b, 2, bytes));
    size_t nvec = bytes / 16;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    int grids[] = {256 * 4, 256 * 8, 256 * 16, 256 * 32, 256 * 64, (int)(nvec / 256 / 8)};
    for (int g : grids) {
        for (int rep = 0; rep < 2; ++rep) read_kernel<8><<<g, 256>>>(a, nvec, sink);
        hipEventRecord(e0);
        for (int rep = 0; rep < 10; ++rep) read_kernel<8><<<g, 256>>>(a, nvec, sink);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1);
        printf("read U=8 grid=%7d : %.1f GB/s\n", g, bytes * 10 / (ms * 1e-3) / 1e9);
    }
    for (int g : grids) {
        hipEventRecord(e0);
        for (int rep = 0; rep < 10; ++rep) read_kernel<4><<<g, 256>>>(a, nvec, sink);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1);
        printf("read U=4 grid=%7d : %.1f GB/s\n", g, bytes * 10 / (ms * 1e-3) / 1e9);
    }
    for (int g : grids) {
        hipEventRecord(e0);
        for (int rep = 0; rep < 10; ++rep) read_nt_kernel<8><<<g, 256>>>((const u32x4_t*)a, nvec, sink);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1);
        printf("read NT U=8 grid=%7d : %.1f GB/s\n", g, bytes * 10 / (ms * 1e-3) / 1e9);
    }
    // one decode launch streams 100-800 MB: the same amounts per launch, each launch on the next part of
    // the 2 GiB so that nothing is found in the 256 MB last-level cache, plain and non-temporal loads
    for (int nt = 0; nt < 2; ++nt)
        for (size_t mb : {50, 100, 200, 400, 800}) {
            size_t nv = mb * 1024 * 1024 / 16;
            int g = (int)(nv / 256 / 8);
            const int slots = (int)(2 * nvec / nv), reps = 20;
            for (int rep = 0; rep < 2; ++rep) read_kernel<8><<<g, 256>>>(big, nv, sink);
            hipEventRecord(e0);
            for (int rep = 0; rep < reps; ++rep) {
                const uint4* src = big + (size_t)(rep % slots) * nv;
                if (nt) read_nt_kernel<8><<<g, 256>>>((const u32x4_t*)src, nv, sink);
                else read_kernel<8><<<g, 256>>>(src, nv, sink);
            }
            hipEventRecord(e1); hipEventSynchronize(e1);
            float ms; hipEventElapsedTime(&ms, e0, e1);
            printf("read%s %zu MiB per launch, grid=%d : %.1f GB/s (%.1f us/launch)\n", nt ? " NT" : "", mb, g,
                   (double)nv * 16 * reps / (ms * 1e-3) / 1e9, ms * 1e3 / reps);
        }
    // the same bytes as one decode launch of the benchmark (1280 strips of 630 rows of K and V, 412 MB), read in
    // the decode kernel's pattern but without its arithmetic
    {
        const int strips = 1280, rows = 630;
        const size_t strip_vecs = (size_t)rows * 16;            // 256-byte rows
        const size_t launch_vecs = (size_t)strips * 2 * strip_vecs;
        const int slots = (int)(2 * nvec / launch_vecs), reps = 20;
        for (int which = 0; which < 3; ++which) {
            hipEventRecord(e0);
            for (int rep = 0; rep < reps; ++rep) {
                const u32x4_t* src = (const u32x4_t*)big + (size_t)(rep % slots) * launch_vecs;
                if (which == 0) strip_read_kernel<1><<<strips, 256>>>(src, rows, strip_vecs, sink);
                else if (which == 1) strip_read_kernel<4><<<strips, 256>>>(src, rows, strip_vecs, sink);
                else strip_read_kernel<8><<<strips, 256>>>(src, rows, strip_vecs, sink);
            }
            hipEventRecord(e1); hipEventSynchronize(e1);
            float ms; hipEventElapsedTime(&ms, e0, e1);
            printf("strip read, %d strips x 2 x %d rows (%.0f MB per launch), %d loads per tile : %.1f GB/s (%.1f us/launch)\n", strips, rows,
                   launch_vecs * 16 / 1e6, which == 0 ? 1 : which == 1 ? 4 : 8, (double)launch_vecs * 16 * reps / (ms * 1e-3) / 1e9, ms * 1e3 / reps);
        }
    }
    for (int g : {256 * 8, 256 * 32, (int)(nvec / 256)}) {
        hipEventRecord(e0);
        for (int rep = 0; rep < 10; ++rep) copy_kernel<<<g, 256>>>(a, b, nvec);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1);
        printf("copy grid=%7d : %.1f GB/s (read+write)\n", g, 2.0 * bytes * 10 / (ms * 1e-3) / 1e9);
    }
    hipEventRecord(e0);
    for (int rep = 0; rep < 10; ++rep) hipMemcpyAsync(b, a, bytes, hipMemcpyDeviceToDevice, 0);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    printf("hipMemcpy D2D : %.1f GB/s (read+write)\n", 2.0 * bytes * 10 / (ms * 1e-3) / 1e9);
    return 0;
}
