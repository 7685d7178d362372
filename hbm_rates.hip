// Stand-alone measurement (not part of liblgc): the HBM rates that plain streaming kernels reach on
// this GPU, to set beside the fused accumulate + candidate kernel, which moves the same 3 reads and
// 2 writes of 4 bytes per gradient element (Alg. 1 / Alg. 2: u <- m u + g, v <- v + u).
//   read   3 arrays summed, nothing written
//   copy   1 read + 1 write
//   3r+2w  g, u, v read; u, v written; no selection work at all
// Each with ordinary and with non-temporal loads and stores, one 256-thread block per 4096 elements,
// on arrays of the ResNet50-sized workload (4 x 25.6 M fp32 each), and the runtime's own
// device-to-device copy.  Prints a table, or one JSON object with --json.
// With --variants: other shapes of the same 3-reads-2-writes stream (how many loads a wavefront has in
// flight before its first store, the order of its stores, a persistent grid, separate output arrays,
// relative offsets of the arrays), each timed in the same run, to show which shape the memory system
// prefers; and what a launch with nothing to do costs.
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

// ---- variants of the 3-reads-2-writes stream (--variants) ----------------------------------------
// One wavefront per group of ROWS rows of 1024 elements, non-temporal throughout.
// ORDER 0: stores of u and v alternate per 256 elements (the library's shape); 1: all of u, then all of v.
// WAIT 0: a store goes out as soon as its own loads are back; 1: the wavefront first waits for all its
// loads; 2: the whole block does.  PERSIST: grid-stride over the groups.
template <int ROWS, int ORDER, int WAIT, bool PERSIST>
__global__ __launch_bounds__(256) void k_rows(const float *__restrict__ g, const float *__restrict__ u_in,
                                              const float *__restrict__ v_in, float *__restrict__ u, float *__restrict__ v,
                                              uint32_t ngroups, float m) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t grp = blockIdx.x * 4 + wave; grp < ngroups; grp += gridDim.x * 4) {
        const size_t base = (size_t)grp * ROWS * 1024 + lane * 4;
        f4 gg[ROWS * 4], uu[ROWS * 4], vv[ROWS * 4];
#pragma unroll
        for (int s = 0; s < ROWS * 4; ++s) {
            gg[s] = ld<true>((const f4 *)(g + base + s * 256));
            uu[s] = ld<true>((const f4 *)(u_in + base + s * 256));
            vv[s] = ld<true>((const f4 *)(v_in + base + s * 256));
        }
        if (WAIT >= 1) { __builtin_amdgcn_s_waitcnt(0x0F70); __builtin_amdgcn_sched_barrier(0); }
        if (WAIT == 2) __syncthreads();
#pragma unroll
        for (int s = 0; s < ROWS * 4; ++s) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { const float x = __fadd_rn(__fmul_rn(m, uu[s][j]), gg[s][j]); uu[s][j] = x; vv[s][j] = __fadd_rn(vv[s][j], x); }
            if (ORDER == 0) { st<true>((f4 *)(u + base + s * 256), uu[s]); st<true>((f4 *)(v + base + s * 256), vv[s]); }
        }
        if (ORDER == 1) {
#pragma unroll
            for (int s = 0; s < ROWS * 4; ++s) st<true>((f4 *)(u + base + s * 256), uu[s]);
#pragma unroll
            for (int s = 0; s < ROWS * 4; ++s) st<true>((f4 *)(v + base + s * 256), vv[s]);
        }
        if (!PERSIST) break;
    }
}

__global__ __launch_bounds__(256) void k_write2(float *u, float *v, uint32_t rows) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t r = blockIdx.x * 4 + wave;
    if (r >= rows) return;
    const size_t base = (size_t)r * 1024 + lane * 4;
    const f4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) { st<true>((f4 *)(u + base + s * 256), z); st<true>((f4 *)(v + base + s * 256), z); }
}

__global__ void k_nothing(const uint32_t *flag) { if (flag[0] == 0x12345u) ((uint32_t *)flag)[1] = 1u; }

static int run_variants() {
    const size_t n = 4ull * 25600000ull, slack = 1u << 20, per = n + slack;
    const uint32_t rows = (uint32_t)(n / 1024);
    float *pool;
    CK(hipMalloc(&pool, per * 5 * 4));
    CK(hipMemset(pool, 0, per * 5 * 4));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    auto arr = [&](int i, size_t off_bytes) { return pool + (size_t)i * per + off_bytes / 4; };
    float *g = arr(0, 0), *u = arr(1, 0), *v = arr(2, 0);
    const double B20 = 20.0 * n;
    auto timeit = [&](const char *name, double bytes, auto launch) -> int {
        for (int i = 0; i < 3; ++i) launch();
        CK(hipDeviceSynchronize());
        double best = 1e30, sum = 0.0;
        for (int b = 0; b < 5; ++b) {
            CK(hipEventRecord(e0, 0));
            for (int i = 0; i < 20; ++i) launch();
            CK(hipEventRecord(e1, 0));
            CK(hipEventSynchronize(e1));
            float ms = 0.f;
            CK(hipEventElapsedTime(&ms, e0, e1));
            best = ms / 20 < best ? ms / 20 : best;
            sum += ms / 20;
        }
        CK(hipGetLastError());
        if (bytes > 0) printf("| %-58s | %7.1f | %5.1f | %7.1f | %5.1f |\n", name, sum / 5 * 1e3, bytes / (sum / 5 * 1e-3) / 8e10, best * 1e3, bytes / (best * 1e-3) / 8e10);
        else printf("| %-58s | %7.1f |       | %7.1f |       |\n", name, sum / 5 * 1e3, best * 1e3);
        fflush(stdout);
        return 0;
    };
    printf("| variant (4 x 25.6 M elements per array, non-temporal)       | mean us | %% peak | best us | %% peak |\n|---|---:|---:|---:|---:|\n");
#define V(R, O, W, P, GRID, label) if (timeit(label, B20, [&] { hipLaunchKernelGGL((k_rows<R, O, W, P>), dim3(GRID), dim3(256), 0, 0, g, u, v, u, v, rows / R, 0.9f); })) return 1;
    V(1, 0, 0, false, rows / 4, "1 row per wavefront, stores alternate u, v (library)")
    V(1, 1, 0, false, rows / 4, "1 row, all stores of u, then all of v")
    V(1, 0, 1, false, rows / 4, "1 row, wavefront waits for all 12 loads before storing")
    V(1, 0, 2, false, rows / 4, "1 row, block waits for all 48 loads before storing")
    V(2, 0, 0, false, rows / 8, "2 rows per wavefront (24 loads, then 16 stores)")
    V(2, 1, 1, false, rows / 8, "2 rows, wavefront waits, u then v")
    V(4, 0, 1, false, rows / 16, "4 rows per wavefront (48 loads, then 32 stores), waits")
    V(1, 0, 0, true, 256, "persistent grid, 1 x 256 blocks")
    V(1, 0, 0, true, 1024, "persistent grid, 4 x 256 blocks")
    V(1, 0, 0, true, 4096, "persistent grid, 16 x 256 blocks")
    V(2, 1, 1, true, 2048, "persistent grid, 8 x 256 blocks, 2 rows, waits, u then v")
#undef V
    if (timeit("separate output arrays (reads g, u, v; writes u', v')", B20, [&] { hipLaunchKernelGGL((k_rows<1, 0, 0, false>), dim3(rows / 4), dim3(256), 0, 0, g, u, v, arr(3, 0), arr(4, 0), rows, 0.9f); })) return 1;
    const size_t offs[][2] = {{256, 512}, {4096, 8192}, {65536, 131072}, {1344, 2752}};
    for (auto &o : offs) {
        char nm[96];
        snprintf(nm, sizeof nm, "u shifted by %zu B, v by %zu B against g", o[0], o[1]);
        float *us = arr(1, o[0]), *vs = arr(2, o[1]);
        if (timeit(nm, B20, [&] { hipLaunchKernelGGL((k_rows<1, 0, 0, false>), dim3(rows / 4), dim3(256), 0, 0, g, us, vs, us, vs, rows, 0.9f); })) return 1;
    }
    if (timeit("reads only: g, u, v (12 B per element)", 12.0 * n, [&] { hipLaunchKernelGGL(k_read<true>, dim3((unsigned)((n / 4 + 1023) / 1024)), dim3(256), 0, 0, (const f4 *)g, (const f4 *)u, (const f4 *)v, arr(3, 0), n / 4); })) return 1;
    if (timeit("writes only: u, v (8 B per element)", 8.0 * n, [&] { hipLaunchKernelGGL(k_write2, dim3(rows / 4), dim3(256), 0, 0, u, v, rows); })) return 1;
    for (int blocks : {1, 256, 4096}) {
        char nm[96];
        snprintf(nm, sizeof nm, "a launch with nothing to do, %d blocks of 256 threads", blocks);
        if (timeit(nm, 0.0, [&] { hipLaunchKernelGGL(k_nothing, dim3(blocks), dim3(256), 0, 0, (const uint32_t *)pool); })) return 1;
    }
    CK(hipFree(pool));
    return 0;
}

int main(int argc, char **argv) {
    if (argc > 1 && strcmp(argv[1], "--variants") == 0) return run_variants();
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
