// Machine ceilings of one MI355X, measured with register-resident loops and plain
// streaming kernels: the matrix-instruction rates (int8 32x32x32, FP4 32x32x64),
// LDS 16-byte reads, vector-L1 hits, and HBM read / write / copy.  These are the
// figures the kernels of libdsqconv are compared with, next to the published peaks.
// Stand-alone program:  hipcc --offload-arch=gfx950 -O3 ceilings.hip -o ceilings_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

// NACC independent accumulators, `iters` rounds: int8 form
template <int NACC>
__global__ __launch_bounds__(256) void mfma_i8(int iters, int *out)
{
    v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {3, 2, 1, (int)blockIdx.x};
    v16i acc[NACC];
    for (int i = 0; i < NACC; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < NACC; ++i) for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// the same with FP4 (e2m1) operands of the f8f6f4 form (K = 64 per instruction)
template <int NACC>
__global__ __launch_bounds__(256) void mfma_fp4(int iters, float *out)
{
    const int x = 0x11111111 * (int)(threadIdx.x & 3);           // small codes: sums stay finite
    v8i a = {x, x, x, x, 0, 0, 0, 0}, b = {0x22222222, x, 0x11111111, x, 0, 0, 0, 0};
    v16f acc[NACC];
    for (int i = 0; i < NACC; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 4, 4, 0, 0, 0, 0);
    }
    float s = 0;
    for (int i = 0; i < NACC; ++i) for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// The same two loops with operands that look like real code tensors: four different
// pseudo-random operand pairs per wave, used in turn (constant operands keep the
// datapath quiet; real data toggles it, which shows in the sustained clock).
__device__ __forceinline__ uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__global__ __launch_bounds__(256) void mfma_i8_data(int iters, int *out)
{
    v4i a[4], b[4];
    for (int k = 0; k < 4; ++k)
        for (int j = 0; j < 4; ++j) {
            a[k][j] = (int)(mix(threadIdx.x * 64 + blockIdx.x * 7919 + k * 8 + j) & 0x0F0F0F0Fu);       // 4-bit codes as int8
            b[k][j] = (int)(mix(threadIdx.x * 64 + blockIdx.x * 104729 + k * 8 + j + 4) & 0x0F0F0F0Fu);
        }
    v16i acc[4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[(i + it) & 3], acc[i], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
__global__ __launch_bounds__(256) void mfma_fp4_data(int iters, float *out)
{
    v8i a[4], b[4];
    for (int k = 0; k < 4; ++k) {
        for (int j = 0; j < 4; ++j) {
            a[k][j] = (int)(mix(threadIdx.x * 64 + blockIdx.x * 7919 + k * 8 + j) & 0x33333333u);       // 2-bit codes as FP4
            b[k][j] = (int)(mix(threadIdx.x * 64 + blockIdx.x * 104729 + k * 8 + j + 4) & 0x33333333u);
        }
        for (int j = 4; j < 8; ++j) { a[k][j] = 0; b[k][j] = 0; }
    }
    v16f acc[4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[(i + it) & 3], acc[i], 4, 4, 0, 0, 0, 0);
        if ((it & 1023) == 1023)                 // (keep the sums finite and exact: start again now and then)
            for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = acc[i][j] * 0.0f;
    }
    float s = 0;
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// FP6 (e2m3) operands, 32 random six-bit fields (24 bytes) per lane: the form a 3/4-bit
// layer could run on instead of int8 (a 4-bit code zero-extended to six bits is code/8).
__global__ __launch_bounds__(256) void mfma_fp6_data(int iters, float *out)
{
    v8i a[4], b[4];
    for (int k = 0; k < 4; ++k) {
        for (int j = 0; j < 6; ++j) {
            a[k][j] = (int)mix(threadIdx.x * 64 + blockIdx.x * 7919 + k * 8 + j);            // (e2m3 has no inf or NaN:
            b[k][j] = (int)mix(threadIdx.x * 64 + blockIdx.x * 104729 + k * 8 + j + 4);      //  every pattern is a number <= 7.5)
        }
        a[k][6] = a[k][7] = b[k][6] = b[k][7] = 0;
    }
    v16f acc[4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[(i + it) & 3], acc[i], 2, 2, 0, 0, 0, 0);
        if ((it & 255) == 255)
            for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = acc[i][j] * 0.0f;
    }
    float s = 0;
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// LDS: every lane reads 16 bytes per instruction, 32 pixels `stride` bytes apart per half wave
__global__ __launch_bounds__(256) void lds_read(int iters, int stride, int *out)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    for (int i = threadIdx.x; i < 16384; i += 256) ((int *)lds)[i] = i;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const unsigned off = (lane & 31) * stride + (lane >> 5) * 16;
    v4i s = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
        v4i v0, v1, v2, v3, v4, v5, v6, v7;
        asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:4096\n ds_read_b128 %2, %8 offset:8192\n"
                     "ds_read_b128 %3, %8 offset:12288\n ds_read_b128 %4, %8 offset:16384\n ds_read_b128 %5, %8 offset:20480\n"
                     "ds_read_b128 %6, %8 offset:24576\n ds_read_b128 %7, %8 offset:28672\n s_waitcnt lgkmcnt(0)\n"
                     : "=v"(v0), "=v"(v1), "=v"(v2), "=v"(v3), "=v"(v4), "=v"(v5), "=v"(v6), "=v"(v7) : "v"(off) : "memory");
        s += v0 + v1 + v2 + v3 + v4 + v5 + v6 + v7;
    }
    out[blockIdx.x * 256 + threadIdx.x] = s.x + s.y + s.z + s.w;
}

// vector L1 hits: each wave re-reads the same 8 KB with coalesced 16-byte loads
__global__ __launch_bounds__(256) void l1_read(int iters, const char *src, int *out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const v4i *p = reinterpret_cast<const v4i *>(src + (size_t)(blockIdx.x & 255) * 65536 + wave * 8192) + lane;
    v4i s = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) s += __builtin_nontemporal_load(p + k * 64 + (it & 1) * 0);
        asm volatile("" : "+v"(s));
    }
    out[blockIdx.x * 256 + threadIdx.x] = s.x + s.y + s.z + s.w;
}

// HBM streams: grid-stride over float4, 4 vectors in flight per thread
__global__ __launch_bounds__(256) void hbm_read(const v4f *src, size_t n4, float *out)
{
    v4f s = {0, 0, 0, 0};
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        const v4f a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        s += a + b + c + d;
    }
    for (; i < n4; i += stride) s += src[i];
    if (s.x + s.y + s.z + s.w == 12345.678f) out[0] = s.x;      // (never true: keeps the loads)
}
__global__ __launch_bounds__(256) void hbm_write(v4f *dst, size_t n4, float v)
{
    const size_t stride = (size_t)gridDim.x * 256;
    const v4f x = {v, v, v, v};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) __builtin_nontemporal_store(x, dst + i);
}
__global__ __launch_bounds__(256) void hbm_copy(const v4f *src, v4f *dst, size_t n4)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + stride < n4; i += 2 * stride) {
        const v4f a = src[i], b = src[i + stride];
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
    }
    for (; i < n4; i += stride) __builtin_nontemporal_store(src[i], dst + i);
}

int main()
{
    int *out; CK(hipMalloc(&out, 8192 * 256 * 4));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    auto timed = [&](auto launch, int reps) {
        launch(); CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int r = 0; r < reps; ++r) launch();
        CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        return (double)ms * 1e-3 / reps;
    };
    printf("| resource | measured | published peak | fraction |\n|---|---|---|---|\n");
    const int iters = 20000;
    for (int blocks : {256, 512, 1024}) {
        double t = timed([&] { mfma_i8<4><<<blocks, 256>>>(iters, out); }, 3);
        double tops = 4.0 * 4 * 2 * 32 * 32 * 32 * blocks * iters / t / 1e12;
        printf("| v_mfma_i32_32x32x32_i8, 4 accumulators, %d workgroups of 4 waves | %.0f TOP/s | 5000 | %.3f |\n", blocks, tops, tops / 5000);
    }
    for (int blocks : {256, 512, 1024}) {
        double t = timed([&] { mfma_fp4<4><<<blocks, 256>>>(iters, (float *)out); }, 3);
        double tops = 4.0 * 4 * 2 * 32 * 32 * 64 * blocks * iters / t / 1e12;
        printf("| v_mfma_f32_32x32x64_f8f6f4 (FP4 operands), 4 accumulators, %d workgroups | %.0f TOP/s | 10100 | %.3f |\n", blocks, tops, tops / 10100);
    }
    // sustained rates: the same loops ten times longer (tens of milliseconds: clocks settle under load)
    for (int blocks : {512, 768}) {
        double t = timed([&] { mfma_i8<4><<<blocks, 256>>>(10 * iters, out); }, 3);
        double tops = 4.0 * 4 * 2 * 32 * 32 * 32 * blocks * 10.0 * iters / t / 1e12;
        printf("| v_mfma_i32_32x32x32_i8 sustained (%.0f ms per launch), %d workgroups | %.0f TOP/s | 5000 | %.3f |\n", t * 1e3, blocks, tops, tops / 5000);
        t = timed([&] { mfma_fp4<4><<<blocks, 256>>>(10 * iters, (float *)out); }, 3);
        tops = 4.0 * 4 * 2 * 32 * 32 * 64 * blocks * 10.0 * iters / t / 1e12;
        printf("| v_mfma_f32_32x32x64_f8f6f4 (FP4) sustained (%.0f ms per launch), %d workgroups | %.0f TOP/s | 10100 | %.3f |\n", t * 1e3, blocks, tops, tops / 10100);
    }
    for (int blocks : {512, 768}) {
        double t = timed([&] { mfma_i8_data<<<blocks, 256>>>(10 * iters, out); }, 3);
        double tops = 4.0 * 4 * 2 * 32 * 32 * 32 * blocks * 10.0 * iters / t / 1e12;
        printf("| v_mfma_i32_32x32x32_i8 sustained on random 4-bit codes, %d workgroups | %.0f TOP/s | 5000 | %.3f |\n", blocks, tops, tops / 5000);
        t = timed([&] { mfma_fp4_data<<<blocks, 256>>>(10 * iters, (float *)out); }, 3);
        tops = 4.0 * 4 * 2 * 32 * 32 * 64 * blocks * 10.0 * iters / t / 1e12;
        printf("| v_mfma_f32_32x32x64_f8f6f4 (FP4) sustained on random 2-bit codes, %d workgroups | %.0f TOP/s | 10100 | %.3f |\n", blocks, tops, tops / 10100);
        t = timed([&] { mfma_fp6_data<<<blocks, 256>>>(10 * iters, (float *)out); }, 3);
        tops = 4.0 * 4 * 2 * 32 * 32 * 64 * blocks * 10.0 * iters / t / 1e12;
        printf("| v_mfma_f32_32x32x64_f8f6f4 (FP6) sustained on random bit patterns, %d workgroups | %.0f TOP/s | 10100 | %.3f |\n", blocks, tops, tops / 10100);
    }
    {
        double t = timed([&] { mfma_i8<1><<<512, 256>>>(iters, out); }, 3);
        printf("| v_mfma_i32_32x32x32_i8, one dependent chain per wave | %.0f TOP/s | 5000 | %.3f |\n",
               4.0 * 2 * 32 * 32 * 32 * 512 * iters / t / 1e12, 4.0 * 2 * 32 * 32 * 32 * 512 * iters / t / 1e12 / 5000);
    }
    CK(hipFuncSetAttribute((const void *)lds_read, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    for (int stride : {48, 64, 80}) {
        double t = timed([&] { lds_read<<<256, 256, 65536>>>(iters, stride, out); }, 3);
        const double bpc = 4.0 * 8 * 1024 * iters / t / 2.4e9;     // bytes per clock per CU at 2.4 GHz
        printf("| LDS ds_read_b128, pixel stride %d B | %.0f B/clk/CU (at 2.4 GHz) | 128 | %.3f |\n", stride, bpc, bpc / 128);
    }
    char *src; CK(hipMalloc(&src, 256 * 65536)); CK(hipMemset(src, 1, 256 * 65536));
    {
        double t = timed([&] { l1_read<<<256, 256>>>(2000, src, out); }, 3);
        const double bpc = 4.0 * 8 * 1024 * 2000 / t / 2.4e9;
        printf("| vector L1 hit, 16 B per lane | %.0f B/clk/CU (at 2.4 GHz) | 64 (one wave-wide load per 16 clk) | %.3f |\n", bpc, bpc / 64);
    }
    const size_t bytes = (size_t)2 << 30, n4 = bytes / 16;
    v4f *a, *b; CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 0, bytes)); CK(hipMemset(b, 0, bytes));
    for (int blocks : {2048, 8192, 32768}) {
        double tr = timed([&] { hbm_read<<<blocks, 256>>>(a, n4, (float *)out); }, 5);
        double tw = timed([&] { hbm_write<<<blocks, 256>>>(b, n4, 1.0f); }, 5);
        double tc = timed([&] { hbm_copy<<<blocks, 256>>>(a, b, n4); }, 5);
        printf("| HBM, 2 GiB, %d workgroups: read / write / copy (read + written bytes) | %.0f / %.0f / %.0f GB/s | 8000 | %.3f / %.3f / %.3f |\n",
               blocks, bytes / tr / 1e9, bytes / tw / 1e9, 2.0 * bytes / tc / 1e9, bytes / tr / 8e12, bytes / tw / 8e12, 2.0 * bytes / tc / 8e12);
    }
    return 0;
}
