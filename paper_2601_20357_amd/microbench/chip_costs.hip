// Fixed costs of an MI355X that shaped the TABED kernels: launch-to-launch overhead, streaming reads of a
// cache-resident and of an HBM-sized buffer, dependent-load round trips, and what it costs to hand partial
// results from one workgroup to another (agent-scope fence vs. write-through stores that are waited for).
// Stand-alone: hipcc --offload-arch=gfx950 -O3 chip_costs.hip -o chip_costs ; ./chip_costs
#include <hip/hip_runtime.h>

#include <cstdio>
#include <vector>

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);      \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

__global__ void k_empty() {}

// `hops` dependent loads, one lane per workgroup matters: the time per hop is one memory round trip.
__global__ void k_chain(const int* __restrict__ next, int start, int hops, int* out) {
    int p = start;
    for (int i = 0; i < hops; ++i) p = next[p];
    if (threadIdx.x == 0) out[blockIdx.x] = p;
}

__global__ void k_read(const float4* __restrict__ a, float* out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float acc = 0.f;
    for (; i < n; i += stride) {
        const float4 v = a[i];
        acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 12345.678f) out[0] = acc;           // never true: keeps the loads alive
}

// Every workgroup streams the same small buffer `passes` times: what the L2s (one per XCD) deliver to the compute
// units once the buffer is resident in each of them.
__global__ void k_read_resident(const float4* __restrict__ a, float* out, size_t n, int passes) {
    float acc = 0.f;
    for (int p = 0; p < passes; ++p) {
        // rotate the starting point per workgroup so that the compute units do not walk the channels in step
        size_t i = ((size_t)blockIdx.x * 977 + threadIdx.x) % n;
        for (size_t k = 0; k < n / blockDim.x; ++k) {
            const float4 v = a[i];
            acc += v.x + v.y + v.z + v.w;
            i += blockDim.x;
            if (i >= n) i -= n;
        }
    }
    if (acc == 12345.678f) out[0] = acc;
}

// Back-to-back matrix instructions on independent accumulators, one wave per SIMD: the rate the matrix cores
// sustain when nothing else is in the way.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
// The operand walk of a GEMM whose operands are K-contiguous: a workgroup owns a tile of `rows` rows that are
// `stride` bytes apart and reads, step after step, the next 128 bytes of every row (8 lanes x 16 bytes per row).
__global__ __launch_bounds__(256) void k_walk(const unsigned char* __restrict__ base, size_t stride, int rows, int steps,
                                              size_t tile_stride, float* out) {
    const unsigned char* tile = base + (size_t)blockIdx.x * tile_stride;
    const int lane8 = threadIdx.x & 7, r0 = threadIdx.x >> 3;       // 32 rows per pass
    float acc = 0.f;
    for (int s = 0; s < steps; ++s)
        for (int r = r0; r < rows; r += 32) {
            const float4 v = *reinterpret_cast<const float4*>(tile + (size_t)r * stride + (size_t)s * 128 + lane8 * 16);
            acc += v.x + v.w;
        }
    if (acc == 1234.5f) out[0] = acc;
}

__global__ __launch_bounds__(256) void k_mfma_peak(int iters, float* out) {
    bf16x8_t a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(i * 0.5f); }
    f32x16_t acc[8];
    for (int j = 0; j < 8; ++j)
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float t = 0.f;
    for (int j = 0; j < 8; ++j) t += acc[j][0] + acc[j][5];
    if (t == 1234.5f) out[0] = t;
}

// Hand-over variants: every workgroup writes 256 floats, then one thread bumps a counter.
__global__ void k_handover_fence_all(int* counter, float* buf) {
    buf[blockIdx.x * 256 + threadIdx.x] = 1.f;
    __threadfence();
    if (threadIdx.x == 0) atomicAdd(counter, 1);
}
__global__ void k_handover_fence_one(int* counter, float* buf) {
    buf[blockIdx.x * 256 + threadIdx.x] = 1.f;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        atomicAdd(counter, 1);
    }
}
__global__ void k_handover_published(int* counter, float* buf) {
    __hip_atomic_store(&buf[blockIdx.x * 256 + threadIdx.x], 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__global__ void k_handover_nothing(int* counter, float* buf) {
    buf[blockIdx.x * 256 + threadIdx.x] = 1.f;
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

int main() {
    const size_t NI = 64u << 20;                    // 256 MB of ints: a 1 MB stride never revisits a line soon
    int* next;
    CK(hipMalloc(&next, NI * sizeof(int)));
    {
        std::vector<int> h(NI);
        const size_t stride = (1u << 20) / 4 + 16;
        for (size_t i = 0; i < NI; ++i) h[i] = (int)((i + stride) % NI);
        CK(hipMemcpy(next, h.data(), NI * sizeof(int), hipMemcpyHostToDevice));
    }
    int* out;
    CK(hipMalloc(&out, 1 << 20));
    CK(hipMemset(out, 0, 1 << 20));
    float4* a;
    const size_t NB = 1024u << 20;
    CK(hipMalloc(&a, NB));
    CK(hipMemset(a, 0, NB));
    float* small;
    CK(hipMalloc(&small, 4u << 20));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    auto time_us = [&](auto fn, int reps) {
        fn();
        (void)hipDeviceSynchronize();
        (void)hipEventRecord(e0, 0);
        for (int i = 0; i < reps; ++i) fn();
        (void)hipEventRecord(e1, 0);
        (void)hipEventSynchronize(e1);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        return (double)ms * 1e3 / reps;
    };
    printf("%-58s %9s\n", "measurement (back-to-back launches on one stream)", "us/launch");
    printf("%-58s %9.2f\n", "empty kernel, 1 workgroup x 64", time_us([&] { hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, 0); }, 500));
    printf("%-58s %9.2f\n", "empty kernel, 1024 workgroups x 256",
           time_us([&] { hipLaunchKernelGGL(k_empty, dim3(1024), dim3(256), 0, 0); }, 500));
    for (size_t mb : {8, 57, 512, 1024}) {
        const size_t n = mb * (1u << 20) / 16;
        const double us = time_us([&] { hipLaunchKernelGGL(k_read, dim3(2048), dim3(256), 0, 0, a, (float*)out, n); }, mb > 100 ? 20 : 100);
        char nm[96];
        snprintf(nm, sizeof nm, "read %zu MiB, same buffer every launch", mb);
        printf("%-58s %9.2f   %7.2f TB/s\n", nm, us, (double)mb * 1048576.0 / us * 1e-6);
    }
    for (size_t mb : {2, 4}) {
        const size_t n = mb * (1u << 20) / 16;
        const int passes = 16, wgs = 2048;
        const double us = time_us([&] { hipLaunchKernelGGL(k_read_resident, dim3(wgs), dim3(256), 0, 0, a, (float*)out, n, passes); }, 10);
        char nm[96];
        snprintf(nm, sizeof nm, "%d workgroups each read the same %zu MiB %d times", wgs, mb, passes);
        printf("%-58s %9.2f   %7.2f TB/s out of the L2s\n", nm, us, (double)wgs * passes * mb * 1048576.0 / us * 1e-6);
    }
    for (int same_tile : {1, 0}) {
        // 1008 workgroups x 256 rows x 32 steps of 128 bytes (k = 2048 in bf16, rows 4096 bytes apart): 1.06 GB
        const int wgs = 1008, rows = 256, steps = 32;
        const size_t stride = 4096, tile_stride = same_tile ? 0 : rows * stride;        // the last tile ends at 1008 MiB
        const double us = time_us([&] {
            hipLaunchKernelGGL(k_walk, dim3(wgs), dim3(256), 0, 0, (const unsigned char*)a, stride, rows, steps, tile_stride, (float*)out);
        }, 5);
        printf("%-58s %9.2f   %7.2f TB/s\n", same_tile ? "GEMM operand walk (256 rows x 4 KB), all the same tile" :
               "GEMM operand walk (256 rows x 4 KB), a tile per workgroup", us, (double)wgs * rows * steps * 128.0 / us * 1e-6);
    }
    {
        const int iters = 20000;
        const double us = time_us([&] { hipLaunchKernelGGL(k_mfma_peak, dim3(256), dim3(256), 0, 0, iters, (float*)out); }, 3);
        printf("%-58s %9.2f   %7.1f TFLOP/s\n", "v_mfma_f32_32x32x16_bf16 back to back, 1 wave per SIMD", us,
               256.0 * 4 * iters * 8 * 32768.0 / us * 1e-6);
    }
    int start = 0;
    double cold1 = 0, cold17 = 0;
    cold1 = time_us([&] { hipLaunchKernelGGL(k_chain, dim3(16), dim3(64), 0, 0, next, start, 1, out); start = (start + 4099) % (int)NI; }, 200);
    cold17 = time_us([&] { hipLaunchKernelGGL(k_chain, dim3(16), dim3(64), 0, 0, next, start, 17, out); start = (start + 4099) % (int)NI; }, 200);
    printf("%-58s %9.2f\n", "1 dependent load, never-seen address", cold1);
    printf("%-58s %9.2f   %7.2f us per extra hop\n", "17 dependent loads, never-seen addresses", cold17, (cold17 - cold1) / 16);
    const double warm1 = time_us([&] { hipLaunchKernelGGL(k_chain, dim3(16), dim3(64), 0, 0, next, 0, 1, out); }, 200);
    const double warm17 = time_us([&] { hipLaunchKernelGGL(k_chain, dim3(16), dim3(64), 0, 0, next, 0, 17, out); }, 200);
    printf("%-58s %9.2f   %7.2f us per extra hop\n", "17 dependent loads, same addresses every launch", warm17, (warm17 - warm1) / 16);
    for (int wgs : {128, 768}) {
        char nm[96];
        snprintf(nm, sizeof nm, "hand-over, %d workgroups: no ordering at all", wgs);
        printf("%-58s %9.2f\n", nm, time_us([&] { hipLaunchKernelGGL(k_handover_nothing, dim3(wgs), dim3(256), 0, 0, out, small); }, 200));
        snprintf(nm, sizeof nm, "hand-over, %d workgroups: published stores + wait", wgs);
        printf("%-58s %9.2f\n", nm, time_us([&] { hipLaunchKernelGGL(k_handover_published, dim3(wgs), dim3(256), 0, 0, out, small); }, 200));
        snprintf(nm, sizeof nm, "hand-over, %d workgroups: fence by one thread", wgs);
        printf("%-58s %9.2f\n", nm, time_us([&] { hipLaunchKernelGGL(k_handover_fence_one, dim3(wgs), dim3(256), 0, 0, out, small); }, 200));
        snprintf(nm, sizeof nm, "hand-over, %d workgroups: fence by every thread", wgs);
        printf("%-58s %9.2f\n", nm, time_us([&] { hipLaunchKernelGGL(k_handover_fence_all, dim3(wgs), dim3(256), 0, 0, out, small); }, 200));
    }
    return 0;
}
