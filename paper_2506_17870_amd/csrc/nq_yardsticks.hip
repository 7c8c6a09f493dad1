// Hardware yardsticks for the roofline figures of this library: what the int8 matrix cores and the
// memory system of the GPU deliver to the simplest possible kernels.  Standalone program (built next
// to libnq.so as nq_yardsticks); prints one line per measurement.  Nothing of the paper's method is
// computed here.
//
//   nq_yardsticks            all measurements
//
// Matrix cores: streams of independent v_mfma_i32_32x32x32_i8 on registers, with one and with two
// waves per SIMD, with distinct operands per instruction, and with VALU instructions in between
// (which shows whether a wave's own VALU work hides behind its matrix-core work).
// Memory: copy, read-only and write-only kernels over 32 MiB, 256 MiB and 2 GiB, and a write of
// 25.7 MB (the output of the benchmark's convolution) in the store patterns of the epilogue.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
            exit(1);                                                                  \
        }                                                                             \
    } while (0)

// MODE 0: eight accumulators, all MFMAs share their operands.
// MODE 1: 4 x 2 distinct operand fragments (the shape of a wave tile), row-major order.
// MODE 2: as 1, four dependent VALU instructions after every pair of MFMAs.
// MODE 3: as 1, one VALU instruction after every MFMA.
template <int MODE, int OCC>
__global__ void __launch_bounds__(256, OCC) k_mfma(int iters, int *out, int seed)
{
    v4i a[4], b[2];
    for (int i = 0; i < 4; ++i) a[i] = v4i{seed + (int)threadIdx.x + i, 1 + i, 2, 3};
    for (int t = 0; t < 2; ++t) b[t] = v4i{3, 2 + t, 1, seed};
    v16i acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int t = 0; t < 2; ++t)
            for (int r = 0; r < 16; ++r) acc[i][t][r] = 0;
    int x0 = seed, x1 = seed + 1, x2 = seed + 2, x3 = seed + 3;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                acc[i][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[MODE ? i : 0], b[MODE ? t : 0], acc[i][t], 0, 0, 0);
                if constexpr (MODE == 3) {
                    x0 = x0 * 3 + x1;
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (MODE == 2) {
                __builtin_amdgcn_sched_barrier(0);
                x0 = x0 * 3 + 1;
                x1 = x1 * 5 + x0;
                x2 = x2 ^ x1;
                x3 = x3 + x2;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    int s = x0 + x1 + x2 + x3;
    for (int i = 0; i < 4; ++i)
        for (int t = 0; t < 2; ++t)
            for (int r = 0; r < 16; ++r) s += acc[i][t][r];
    if (s == 0x12345678) out[threadIdx.x] = s;   // keeps the work alive, practically never true
}

// NV independent one-cycle-per-lane VALU instructions (adds on eight separate chains) after every MFMA:
// how much vector work a wave can put in the shadow of its own matrix-core instructions.
template <int NV, int OCC>
__global__ void __launch_bounds__(256, OCC) k_mfma_valu(int iters, int *out, int seed)
{
    v4i a[4], b[2];
    for (int i = 0; i < 4; ++i) a[i] = v4i{seed + (int)threadIdx.x + i, 1 + i, 2, 3};
    for (int t = 0; t < 2; ++t) b[t] = v4i{3, 2 + t, 1, seed};
    v16i acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int t = 0; t < 2; ++t)
            for (int r = 0; r < 16; ++r) acc[i][t][r] = 0;
    int x[8];
    for (int j = 0; j < 8; ++j) x[j] = seed + j;
    const int y = seed * 7 + (int)threadIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                acc[i][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[t], acc[i][t], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < NV; ++j) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[(i * 2 + t + j) & 7]) : "v"(y));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    int s = 0;
    for (int j = 0; j < 8; ++j) s += x[j];
    for (int i = 0; i < 4; ++i)
        for (int t = 0; t < 2; ++t)
            for (int r = 0; r < 16; ++r) s += acc[i][t][r];
    if (s == 0x12345678) out[threadIdx.x] = s;
}

__global__ void k_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

// The same copy with the streaming (non-temporal) hint on loads and stores, four 16-byte pieces in flight per thread:
// the best copy known here, the practical ceiling for a kernel whose accesses are whole cache lines used once.
typedef unsigned y_u4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) k_copy_stream(const y_u4 *__restrict__ src, y_u4 *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 1024;
    for (; i + 768 < n; i += stride) {
        y_u4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + 256 * u);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + 256 * u);
    }
}

__global__ void k_read(const uint4 *__restrict__ src, int *out, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    uint4 s = make_uint4(0, 0, 0, 0);
    for (; i < n; i += stride) {
        const uint4 v = src[i];
        s.x ^= v.x; s.y ^= v.y; s.z ^= v.z; s.w ^= v.w;
    }
    if ((s.x ^ s.y ^ s.z ^ s.w) == 0x12345678) out[threadIdx.x] = 1;
}

__global__ void k_write(uint4 *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = make_uint4(1, 2, 3, 4);
}

// Output [M][64] fp32; each wave writes 32-row x 32-column tiles.  PAT 0: dword stores, lane =
// column, 16 stores per tile, each instruction two runs of 128 bytes (the fp32 epilogue).  PAT 1:
// 16-byte stores, eight rows x 128 bytes per instruction.  PAT 2: 16-byte stores, fully contiguous.
template <int PAT>
__global__ void __launch_bounds__(256) k_store(float *y, int tiles_per_wave, int total_tiles)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gw = blockIdx.x * 4 + wave;
    for (int t = 0; t < tiles_per_wave; ++t) {
        const int tile = gw + t * gridDim.x * 4;
        if (tile >= total_tiles) break;
        const int rb = tile >> 1, ch = tile & 1;
        float *base = y + (size_t)rb * 32 * 64 + ch * 32;
        if constexpr (PAT == 0) {
            const int col = lane & 31, rg = lane >> 5;
#pragma unroll
            for (int r = 0; r < 16; ++r) base[(8 * (r >> 2) + 4 * rg + (r & 3)) * 64 + col] = (float)(tile + r);
        } else if constexpr (PAT == 1) {
            const int r8 = lane >> 3, cg = lane & 7;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4 *>(base + (8 * q + r8) * 64 + 4 * cg) = make_float4(tile, q, lane, 1);
        } else {
            float *b2 = y + (size_t)tile * 1024;
#pragma unroll
            for (int q = 0; q < 4; ++q) *reinterpret_cast<float4 *>(b2 + q * 256 + 4 * lane) = make_float4(tile, q, lane, 1);
        }
    }
}

__global__ void k_empty(int *out)
{
    if (out == nullptr) return;
}

template <typename F>
static float time_ms(F f, int reps)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    f(0);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) f(i);
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipGetLastError());
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms / reps;
}

int main()
{
    int *out;
    CK(hipMalloc(&out, 4096));
    const int iters = 4000;
    printf("# int8 matrix cores: v_mfma_i32_32x32x32_i8, 8 accumulators per wave, %d x 8 MFMAs per wave\n", iters);
#define MFMA_RUN(MODE, OCC, BLOCKS, NAME)                                                                         \
    {                                                                                                             \
        const float ms = time_ms([&](int) { hipLaunchKernelGGL((k_mfma<MODE, OCC>), dim3(BLOCKS), dim3(256), 0, 0, \
                                                               iters, out, 1); }, 3);                             \
        printf("%-58s %8.1f TOPS\n", NAME, (double)BLOCKS * 4 * iters * 8 * 65536.0 / ms / 1e9);                   \
    }
    MFMA_RUN(0, 1, 256, "1 wave/SIMD, shared operands")
    MFMA_RUN(1, 1, 256, "1 wave/SIMD, 4 x 2 distinct operands")
    MFMA_RUN(2, 1, 256, "1 wave/SIMD, + 4 VALU per 2 MFMAs (serial sum = 80%)")
    MFMA_RUN(3, 1, 256, "1 wave/SIMD, + 1 VALU per MFMA (serial sum = 89%)")
    MFMA_RUN(1, 2, 512, "2 waves/SIMD, 4 x 2 distinct operands")
    MFMA_RUN(2, 2, 512, "2 waves/SIMD, + 4 VALU per 2 MFMAs")
    MFMA_RUN(3, 2, 512, "2 waves/SIMD, + 1 VALU per MFMA")
    printf("# the same MFMA stream with NV independent VALU adds after every MFMA (MFMA alone: 32 clocks; an add: 4 clocks of issue)\n");
#define MFMA_VALU_RUN(NV, OCC, BLOCKS)                                                                            \
    {                                                                                                             \
        const float ms = time_ms([&](int) { hipLaunchKernelGGL((k_mfma_valu<NV, OCC>), dim3(BLOCKS), dim3(256), 0, 0, \
                                                               iters, out, 1); }, 3);                             \
        printf(" %6.1f", (double)BLOCKS * 4 * iters * 8 * 65536.0 / ms / 1e9);                                     \
    }
    printf("NV =            0      1      2      3      4      5      6      7      8     10     12     16\n1 wave/SIMD ");
    MFMA_VALU_RUN(0, 1, 256) MFMA_VALU_RUN(1, 1, 256) MFMA_VALU_RUN(2, 1, 256) MFMA_VALU_RUN(3, 1, 256) MFMA_VALU_RUN(4, 1, 256)
    MFMA_VALU_RUN(5, 1, 256) MFMA_VALU_RUN(6, 1, 256) MFMA_VALU_RUN(7, 1, 256) MFMA_VALU_RUN(8, 1, 256) MFMA_VALU_RUN(10, 1, 256)
    MFMA_VALU_RUN(12, 1, 256) MFMA_VALU_RUN(16, 1, 256)
    printf(" TOPS\n2 waves/SIMD");
    MFMA_VALU_RUN(0, 2, 512) MFMA_VALU_RUN(1, 2, 512) MFMA_VALU_RUN(2, 2, 512) MFMA_VALU_RUN(3, 2, 512) MFMA_VALU_RUN(4, 2, 512)
    MFMA_VALU_RUN(5, 2, 512) MFMA_VALU_RUN(6, 2, 512) MFMA_VALU_RUN(7, 2, 512) MFMA_VALU_RUN(8, 2, 512) MFMA_VALU_RUN(10, 2, 512)
    MFMA_VALU_RUN(12, 2, 512) MFMA_VALU_RUN(16, 2, 512)
    printf(" TOPS\n");

    printf("# memory: 16-byte accesses, grid-stride kernels\n");
    for (size_t mb : {32, 256, 2048}) {
        const size_t bytes = mb << 20, n = bytes / 16;
        uint4 *s, *d;
        CK(hipMalloc(&s, bytes));
        CK(hipMalloc(&d, bytes));
        CK(hipMemset(s, 1, bytes));
        CK(hipMemset(d, 1, bytes));
        const int blocks = 4096;
        const float mc = time_ms([&](int) { hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, 0, s, d, n); }, 10);
        const float mr = time_ms([&](int) { hipLaunchKernelGGL(k_read, dim3(blocks), dim3(256), 0, 0, s, out, n); }, 10);
        const float mw = time_ms([&](int) { hipLaunchKernelGGL(k_write, dim3(blocks), dim3(256), 0, 0, d, n); }, 10);
        const float ms = time_ms([&](int) { hipLaunchKernelGGL(k_copy_stream, dim3(8192), dim3(256), 0, 0,
                                                               reinterpret_cast<const y_u4 *>(s), reinterpret_cast<y_u4 *>(d), n); }, 10);
        printf("%5zu MiB: copy %7.1f GB/s (read + write)   read %7.1f GB/s   write %7.1f GB/s   [copy %.1f us]   streaming copy "
               "%7.1f GB/s\n", mb, 2.0 * bytes / mc / 1e6, bytes / mr / 1e6, bytes / mw / 1e6, mc * 1000, 2.0 * bytes / ms / 1e6);
        CK(hipFree(s));
        CK(hipFree(d));
    }

    printf("# write of 100352 x 64 fp32 (25.7 MB), 8 buffers in turn, 512 blocks\n");
    {
        const size_t M = 100352;
        const int total_tiles = (int)(M / 32 * 2), sets = 8, blocks = 512;
        float *ys[sets];
        for (int i = 0; i < sets; ++i) {
            CK(hipMalloc(&ys[i], M * 64 * 4));
            CK(hipMemset(ys[i], 0, M * 64 * 4));
        }
        const int tpw = (total_tiles + blocks * 4 - 1) / (blocks * 4);
        const float a = time_ms([&](int i) { hipLaunchKernelGGL(k_store<0>, dim3(blocks), dim3(256), 0, 0, ys[i % sets], tpw, total_tiles); }, 40);
        const float b = time_ms([&](int i) { hipLaunchKernelGGL(k_store<1>, dim3(blocks), dim3(256), 0, 0, ys[i % sets], tpw, total_tiles); }, 40);
        const float c = time_ms([&](int i) { hipLaunchKernelGGL(k_store<2>, dim3(blocks), dim3(256), 0, 0, ys[i % sets], tpw, total_tiles); }, 40);
        printf("dword stores, 2 x 128 B per instruction %6.2f us | 16-byte stores, 8 x 128 B %6.2f us | 16-byte stores, contiguous %6.2f us\n",
               a * 1000, b * 1000, c * 1000);
        for (int i = 0; i < sets; ++i) CK(hipFree(ys[i]));
    }
    {
        const float e = time_ms([&](int) { hipLaunchKernelGGL(k_empty, dim3(512), dim3(256), 0, 0, out); }, 200);
        printf("# empty kernel, 512 blocks, back to back: %.2f us per launch\n", e * 1000);
    }
    CK(hipFree(out));
    return 0;
}
