// Microbenchmarks that put numbers behind the roofs this library is measured against on one MI355X (gfx950):
//   1. the int8 matrix cores in a register-only loop (v_mfma_i32_32x32x32_i8, the GEMM's instruction), with
//      operands that never change and with operands whose bits are refreshed every eight instructions,
//      at 1, 2 and 4 waves per SIMD;
//   2. LDS throughput of 16-byte reads in the GEMM's fragment pattern and of 16-byte writes in its staging
//      pattern, in bytes per clock and compute unit;
//   3. a plain streaming copy (16 bytes per lane), the practical HBM rate for read + write traffic.
// Standalone program: hipcc --offload-arch=gfx950 -O3 peaks.hip -o peaks && ./peaks
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define CK(x)                                                                             \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);         \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

// ---- 1. matrix cores -------------------------------------------------------------------------------
// Eight independent accumulators, 2 A x 4 B operand registers (the GEMM's wave tile).  REFRESH: a few
// cheap integer instructions change operand bits every eight MFMAs, as new tiles of real codes would.
template <bool REFRESH>
__global__ __launch_bounds__(256) void mfma_loop(int iters, int* sink) {
    v4i a[2], b[4];
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    auto rnd = [&]() { h ^= h << 13; h ^= h >> 17; h ^= h << 5; return (int)h; };
    for (int t = 0; t < 2; ++t) a[t] = (v4i){rnd(), rnd(), rnd(), rnd()};
    for (int t = 0; t < 4; ++t) b[t] = (v4i){rnd(), rnd(), rnd(), rnd()};
    v16i acc[8];
    for (int t = 0; t < 8; ++t)
        for (int v = 0; v < 16; ++v) acc[t][v] = 0;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t >> 2], b[t & 3], acc[t], 0, 0, 0);
        if (REFRESH) {
            a[0].x = rnd(); a[1].y = rnd(); b[0].z = rnd(); b[1].w = rnd(); b[2].x = rnd(); b[3].y = rnd();
            a[0].z ^= a[1].x; a[1].w ^= a[0].y; b[0].x ^= b[3].z; b[1].y ^= b[2].w; b[2].z ^= b[1].x; b[3].w ^= b[0].y;
        }
    }
    int s = 0;
    for (int t = 0; t < 8; ++t) s += acc[t][0];
    if (s == 0x7fffffff) sink[0] = s;
}

template <bool REFRESH>
static void run_mfma(int cus, int waves_per_simd, int* sink) {
    const int iters = 20000;
    const int blocks = cus * waves_per_simd;        // 256 threads = 4 waves = one wave per SIMD of a CU
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    hipLaunchKernelGGL(mfma_loop<REFRESH>, dim3(blocks), dim3(256), 0, 0, 200, sink);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(mfma_loop<REFRESH>, dim3(blocks), dim3(256), 0, 0, iters, sink);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double ops = (double)blocks * 4 * iters * 8 * (2.0 * 32 * 32 * 32);
    printf("mfma_i32_32x32x32_i8  operands %-9s  %d wave(s)/SIMD : %7.1f TOP/s\n", REFRESH ? "refreshed" : "constant",
           waves_per_simd, ops / (ms * 1e-3) / 1e12);
}

// ---- 2. LDS ----------------------------------------------------------------------------------------
// One workgroup of 512 threads per CU.  Reads: lane l of a wave reads 16 bytes at row (l % 32), byte offset
// 16 (l / 32) of an 80-byte-stride tile, the GEMM's operand fragment pattern.  Writes: thread t writes 16 bytes
// at row t / 4, offset 16 (t % 4), its staging pattern.
template <bool WRITE>
__global__ __launch_bounds__(512) void lds_loop(int iters, int* sink, long long* cycles) {
    __shared__ __align__(16) char tile[2 * 256 * 80];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 2 * 256 * 80 / 4; i += 512) reinterpret_cast<int*>(tile)[i] = i;
    __syncthreads();
    const long long t0 = clock64();
    v4i acc = {0, 0, 0, 0};
    // (an empty asm statement hides the offset from the optimizer each trip, so the accesses stay in the loop;
    // they are ordinary LDS accesses that the hardware may keep in flight together)
    if (WRITE) {
        int off = (tid >> 2) * 80 + (tid & 3) * 16;
        for (int i = 0; i < iters; ++i) {
            asm volatile("" : "+v"(off));
            acc.x += i;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                *reinterpret_cast<v4i*>(&tile[(u & 1) * 128 * 80 + off + (u >> 1) * 256 * 80]) = acc;      // < 40944
            asm volatile("" ::: "memory");
        }
    } else {
        int off = ((wave & 3) * 64 + (lane & 31)) * 80 + (lane >> 5) * 16;
        for (int i = 0; i < iters; ++i) {
            asm volatile("" : "+v"(off));
            v4i v[6];
#pragma unroll
            for (int u = 0; u < 6; ++u) v[u] = *reinterpret_cast<const v4i*>(&tile[off + u * 32 * 80]);      // < 33232
#pragma unroll
            for (int u = 0; u < 6; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
        }
    }
    __syncthreads();
    const long long t1 = clock64();
    if (tid == 0 && blockIdx.x == 0) cycles[0] = t1 - t0;
    if (acc.x == 0x7fffffff) sink[0] = acc.y + acc.z + acc.w + *reinterpret_cast<int*>(&tile[(tid * 4) % 1024]);
}

template <bool WRITE>
static void run_lds(int cus, int* sink, long long* cycles) {
    const int iters = 4000;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    hipLaunchKernelGGL(lds_loop<WRITE>, dim3(cus), dim3(512), 0, 0, 50, sink, cycles);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(lds_loop<WRITE>, dim3(cus), dim3(512), 0, 0, iters, sink, cycles);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    long long cyc = 0;
    CK(hipMemcpy(&cyc, cycles, sizeof(cyc), hipMemcpyDeviceToHost));
    const double bytes_per_cu = 512.0 * 16 * (WRITE ? 4 : 6) * iters;
    // clock64 counts at a fixed 100 MHz on this chip: the byte rate is quoted per nanosecond and CU as well
    printf("LDS 16-byte %-6s : %7.1f bytes/ns/CU  (%.3f ms for %.0f MB per CU)\n", WRITE ? "writes" : "reads",
           bytes_per_cu / (ms * 1e6), ms, bytes_per_cu / 1e6);
    (void)cyc;
}

// ---- 3. streaming copy -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy16(const float4* __restrict__ src, float4* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// read-only stream: every lane sums 16-byte loads, one value per workgroup leaves
__global__ __launch_bounds__(256) void read16(const float4* __restrict__ src, size_t n, float* __restrict__ out) {
    const size_t stride = (size_t)gridDim.x * 256;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const float4 v = src[i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.f) out[0] = 1.f;
}

int main() {
    int dev = 0;
    CK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, dev));
    const int cus = prop.multiProcessorCount;
    printf("%s, %d compute units, %d MHz\n", prop.gcnArchName, cus, prop.clockRate / 1000);
    int* sink;
    long long* cycles;
    CK(hipMalloc(&sink, 64));
    CK(hipMalloc(&cycles, 64));
    for (int w : {1, 2, 4}) run_mfma<false>(cus, w, sink);
    for (int w : {1, 2, 4}) run_mfma<true>(cus, w, sink);
    run_lds<false>(cus, sink, cycles);
    run_lds<true>(cus, sink, cycles);
    for (size_t mb : {64, 1024}) {
        const size_t n = mb * 1024 * 1024 / 16;
        float4 *a, *b;
        CK(hipMalloc(&a, n * 16));
        CK(hipMalloc(&b, n * 16));
        CK(hipMemset(a, 1, n * 16));
        hipEvent_t e0, e1;
        CK(hipEventCreate(&e0));
        CK(hipEventCreate(&e1));
        hipLaunchKernelGGL(copy16, dim3(cus * 8), dim3(256), 0, 0, a, b, n);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int r = 0; r < 10; ++r) hipLaunchKernelGGL(copy16, dim3(cus * 8), dim3(256), 0, 0, a, b, n);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms = 0.f;
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("copy %4zu MiB: %6.2f TB/s (read + write)\n", mb, 2.0 * n * 16 * 10 / (ms * 1e-3) / 1e12);
        CK(hipEventRecord(e0));
        for (int r = 0; r < 10; ++r) hipLaunchKernelGGL(read16, dim3(cus * 8), dim3(256), 0, 0, a, n, reinterpret_cast<float*>(sink));
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("read %4zu MiB: %6.2f TB/s\n", mb, 1.0 * n * 16 * 10 / (ms * 1e-3) / 1e12);
        CK(hipFree(a));
        CK(hipFree(b));
    }
    return 0;
}
