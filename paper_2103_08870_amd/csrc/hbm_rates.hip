// Stand-alone measurement (not part of liblgc): the HBM rates that plain streaming kernels reach on
// this GPU, to set beside the fused accumulate + candidate kernel, which moves the same 3 reads and
// 2 writes of 4 bytes per gradient element (Alg. 1 / Alg. 2: u <- m u + g, v <- v + u).
//   read   3 arrays summed, nothing written
//   copy   1 read + 1 write
//   3r+2w  g, u, v read; u, v written; no selection work at all
// Each with ordinary and with non-temporal loads and stores, one 256-thread block per 4096 elements,
// on arrays of the ResNet50-sized workload (4 x 25.6 M fp32 each), and the runtime's own
// device-to-device copy.  Prints a table, or one JSON object with --json.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>

typedef float f4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                              \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                      \
        }                                                                                  \
    } while (0)

template <bool NT> __device__ __forceinline__ f4 ld(const f4 *p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT> __device__ __forceinline__ void st(f4 *p, f4 x) {
    if (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

// a block handles the 1024 float4 groups that start at group 1024 * blockIdx.x: four per thread
template <bool NT>
__global__ __launch_bounds__(256) void k_read(const f4 *a, const f4 *b, const f4 *c, float *out, size_t n4) {
    const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    f4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const size_t j = i + r * 256;
        if (j < n4) s += ld<NT>(a + j) + ld<NT>(b + j) + ld<NT>(c + j);
    }
    if (s[0] + s[1] + s[2] + s[3] == 12345.678f) out[0] = 1.0f;   // keeps the loads alive; the arrays hold zeros
}

template <bool NT>
__global__ __launch_bounds__(256) void k_copy(const f4 *a, f4 *b, size_t n4) {
    const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    f4 x[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) if (i + r * 256 < n4) x[r] = ld<NT>(a + i + r * 256);
#pragma unroll
    for (int r = 0; r < 4; ++r) if (i + r * 256 < n4) st<NT>(b + i + r * 256, x[r]);
}

template <bool NT>
__global__ __launch_bounds__(256) void k_3r2w(const f4 *g, f4 *u, f4 *v, size_t n4, float m) {
    const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    f4 x[4], y[4], z[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const size_t j = i + r * 256;
        if (j < n4) { x[r] = ld<NT>(g + j); y[r] = ld<NT>(u + j); z[r] = ld<NT>(v + j); }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const size_t j = i + r * 256;
        if (j < n4) {
            y[r] = y[r] * m + x[r];
            z[r] = z[r] + y[r];
            st<NT>(u + j, y[r]);
            st<NT>(v + j, z[r]);
        }
    }
}

int main(int argc, char **argv) {
    const bool json = argc > 1 && strcmp(argv[1], "--json") == 0;
    const size_t n = 4ull * 25600000ull, n4 = n / 4;
    const unsigned grid = (unsigned)((n4 + 1023) / 1024);
    const int reps = 20;
    float *g, *u, *v, *o;
    CK(hipMalloc(&g, n * 4)); CK(hipMalloc(&u, n * 4)); CK(hipMalloc(&v, n * 4)); CK(hipMalloc(&o, 256));
    CK(hipMemset(g, 0, n * 4)); CK(hipMemset(u, 0, n * 4)); CK(hipMemset(v, 0, n * 4));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const f4 *cg = (const f4 *)g, *cu = (const f4 *)u, *cv = (const f4 *)v;
    f4 *mu = (f4 *)u, *mv = (f4 *)v;

    const char *names[7] = {"read", "read_nt", "copy", "copy_nt", "3r2w", "3r2w_nt", "hipMemcpyAsync_d2d"};
    const double bytes[7] = {12.0 * n, 12.0 * n, 8.0 * n, 8.0 * n, 20.0 * n, 20.0 * n, 8.0 * n};
    double gbps[7];
    for (int which = 0; which < 7; ++which) {
        auto launch = [&]() -> hipError_t {
            switch (which) {
                case 0: hipLaunchKernelGGL(k_read<false>, dim3(grid), dim3(256), 0, 0, cg, cu, cv, o, n4); break;
                case 1: hipLaunchKernelGGL(k_read<true>, dim3(grid), dim3(256), 0, 0, cg, cu, cv, o, n4); break;
                case 2: hipLaunchKernelGGL(k_copy<false>, dim3(grid), dim3(256), 0, 0, cg, mu, n4); break;
                case 3: hipLaunchKernelGGL(k_copy<true>, dim3(grid), dim3(256), 0, 0, cg, mu, n4); break;
                case 4: hipLaunchKernelGGL(k_3r2w<false>, dim3(grid), dim3(256), 0, 0, cg, mu, mv, n4, 0.9f); break;
                case 5: hipLaunchKernelGGL(k_3r2w<true>, dim3(grid), dim3(256), 0, 0, cg, mu, mv, n4, 0.9f); break;
                default: return hipMemcpyAsync(u, g, n * 4, hipMemcpyDeviceToDevice, 0);
            }
            return hipGetLastError();
        };
        for (int i = 0; i < 3; ++i) CK(launch());
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0, 0));
        for (int i = 0; i < reps; ++i) CK(launch());
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms = 0.f;
        CK(hipEventElapsedTime(&ms, e0, e1));
        gbps[which] = bytes[which] / (ms / reps * 1e-3) / 1e9;
        if (!json) printf("%-20s %8.1f us  %7.1f GB/s  %5.1f %% of 8 TB/s\n", names[which], ms / reps * 1e3, gbps[which], gbps[which] / 80.0);
    }
    if (json) {
        printf("{\"elements_per_array\": %zu", n);
        for (int which = 0; which < 7; ++which) printf(", \"%s_GBps\": %.1f", names[which], gbps[which]);
        printf("}\n");
    }
    CK(hipFree(g)); CK(hipFree(u)); CK(hipFree(v)); CK(hipFree(o));
    return 0;
}
