// Ceilings of one MI355X (gfx950) as this build's kernels can reach them, measured with plain HIP:
// HBM copy rate, bf16 MFMA rate (constant and random operands, long and short kernels), fp32 FMA and
// bf16 dot2 vector rates, LDS ds_read_b128 rate.  The numbers set the denominators used when
// judging the diagonal-sparse kernels; nothing in the library depends on this program.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);      \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ void copy_kernel(const u32x4 *__restrict__ a, u32x4 *__restrict__ b, size_t n)
{
    size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x;
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    for (; i < n; i += stride) b[i] = a[i];
}

__global__ void fill_kernel(u32x4 *__restrict__ b, size_t n, unsigned word)
{
    size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x;
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    const u32x4 v = {word, word, word, word};
    for (; i < n; i += stride) b[i] = v;
}

// 2 x 5 accumulator tiles per wave and distinct operand registers, as in the product kernel
// stamps (or null): per workgroup the shader-clock counter and the 100 MHz wall clock at start and end, which
// together give the clock the chip sustained under this load
__global__ __launch_bounds__(256) void mfma_kernel(const bf16x8 *__restrict__ src, float *out, int iters,
                                                   unsigned long long *stamps)
{
    if (stamps && threadIdx.x == 0) {
        stamps[blockIdx.x * 4 + 0] = clock64();
        stamps[blockIdx.x * 4 + 1] = wall_clock64();
    }
    bf16x8 fa[2], fb[5];
    for (int i = 0; i < 2; ++i) fa[i] = src[threadIdx.x + 256 * i];
    for (int i = 0; i < 5; ++i) fb[i] = src[threadIdx.x + 256 * (2 + i)];
    f32x16 acc[2][5];
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 5; ++b)
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 5; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    float s = 0;
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 5; ++b)
            for (int i = 0; i < 16; ++i) s += acc[a][b][i];
    out[blockIdx.x * 256 + threadIdx.x] = s;
    if (stamps && threadIdx.x == 0) {
        stamps[blockIdx.x * 4 + 2] = clock64();
        stamps[blockIdx.x * 4 + 3] = wall_clock64();
    }
}

// Reads only: every workgroup walks tiles of `rows` rows of `row_bytes` bytes (a tile is contiguous in memory), either
// front to back or slice by slice -- bytes [s * slice_bytes, (s + 1) * slice_bytes) of every row, then the next s --
// which is how the product kernels take a block of token rows 64 contraction indices at a time.
__global__ __launch_bounds__(512) void read_kernel(const unsigned char *__restrict__ src, int rows, int row_bytes,
                                                   int slice_bytes, long tiles, unsigned *sink)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    const long tile_bytes = long(rows) * row_bytes;
    for (long tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const unsigned char *base = src + tile * tile_bytes;
        const int per_row = slice_bytes / 16, per_slice = rows * per_row, slices = row_bytes / slice_bytes;
        for (int s = 0; s < slices; ++s)
            for (int i = threadIdx.x; i < per_slice; i += 512 * 4) {
                u32x4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int j = i + u * 512, r = j / per_row, c = j % per_row;
                    v[u] = j < per_slice
                               ? *reinterpret_cast<const u32x4 *>(base + long(r) * row_bytes + s * slice_bytes + c * 16)
                               : u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc ^= v[u];
            }
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[0] = 1;  // keeps the loads alive
}

__global__ __launch_bounds__(256) void fma_kernel(float *out, int iters, float m)
{
    float a[8];
    for (int i = 0; i < 8; ++i) a[i] = threadIdx.x + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = fmaf(a[i], m, 1.0f);
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) s += a[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void dot2_kernel(float *out, int iters, unsigned seed)
{
    float a[8];
    for (int i = 0; i < 8; ++i) a[i] = threadIdx.x + i;
    bf16x2 x, y;
    x[0] = (__bf16)(seed * 0.5f);
    x[1] = (__bf16)1.0f;
    y[0] = (__bf16)0.5f;
    y[1] = (__bf16)(seed * 0.25f);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = __builtin_amdgcn_fdot2_f32_bf16(x, y, a[i], false);
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) s += a[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// eight independent ds_read_b128 per iteration, lane l at byte 16*l of a 1 KB row: conflict-free
__global__ __launch_bounds__(256) void lds_kernel(unsigned *out, int iters)
{
    extern __shared__ unsigned lds[];
    for (int i = threadIdx.x; i < 16384; i += 256) lds[i] = i;
    __syncthreads();
    const unsigned addr = (threadIdx.x & 63) * 16;
    u32x4 a0, a1, a2, a3, a4, a5, a6, a7;
    unsigned s = 0;
    for (int it = 0; it < iters; ++it) {
        asm volatile(
            "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:4096\n ds_read_b128 %2, %8 offset:8192\n"
            "ds_read_b128 %3, %8 offset:12288\n ds_read_b128 %4, %8 offset:16384\n ds_read_b128 %5, %8 offset:20480\n"
            "ds_read_b128 %6, %8 offset:24576\n ds_read_b128 %7, %8 offset:28672\n s_waitcnt lgkmcnt(0)"
            : "=v"(a0), "=v"(a1), "=v"(a2), "=v"(a3), "=v"(a4), "=v"(a5), "=v"(a6), "=v"(a7)
            : "v"(addr)
            : "memory");
        s ^= a0.x ^ a1.y ^ a2.z ^ a3.w ^ a4.x ^ a5.y ^ a6.z ^ a7.w;
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Cache read bandwidth: every workgroup streams again and again over a region small enough to stay in the
// L2 of its XCD (or, larger, in the memory-side cache); 16 bytes per lane, eight loads in flight per lane.
// to_lds = 1 moves the data straight into LDS (global_load_lds_dwordx4) instead of into registers.
template <int TO_LDS>
__global__ __launch_bounds__(256) void cache_read_kernel(const u32x4 *src, u32x4 *dst, int region_pieces, int iters)
{
    extern __shared__ __align__(16) unsigned char stage[];
    const int wave = threadIdx.x >> 6;
    const unsigned base = __builtin_amdgcn_readfirstlane(
        unsigned(reinterpret_cast<size_t>((__attribute__((address_space(3))) unsigned char *)stage)) + wave * 1024);
    u32x4 acc = {0, 0, 0, 0};
    int pos = int((size_t(blockIdx.x) * 977 * 256 + threadIdx.x) % size_t(region_pieces));
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (TO_LDS)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base + u * 4096),
                             "v"(src + pos)
                             : "memory", "m0");
            else
                acc ^= src[pos];
            pos += 256;
            pos = pos >= region_pieces ? pos - region_pieces : pos;
        }
        if (TO_LDS) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    }
    if (TO_LDS) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        acc = *reinterpret_cast<const u32x4 *>(stage + threadIdx.x * 16);
    }
    if (acc[0] == 0x12345678u) dst[threadIdx.x] = acc;
}

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    printf("device: %s, %d CUs, %d MHz shader clock, %zu B LDS per workgroup\n", prop.gcnArchName, cus,
           prop.clockRate / 1000, prop.sharedMemPerBlock);
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms;

    {  // HBM copy, 2 GiB in and 2 GiB out per pass
        const size_t bytes = size_t(2) << 30;
        u32x4 *a, *b;
        CK(hipMalloc(&a, bytes));
        CK(hipMalloc(&b, bytes));
        CK(hipMemset(a, 1, bytes));
        for (int blocks : {2048, 8192, 32768}) {
            copy_kernel<<<blocks, 256>>>(a, b, bytes / 16);
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0));
            for (int i = 0; i < 5; ++i) copy_kernel<<<blocks, 256>>>(a, b, bytes / 16);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
            printf("copy, %5d workgroups: %.0f GB/s (read + write)\n", blocks, 2.0 * bytes * 5 / ms / 1e6);
        }
        // writes only: 2 GiB per pass, and one pass over 113 MB (the dense operands of one shape of the ViT-Base stack)
        for (size_t fill_bytes : {bytes, size_t(113) << 20}) {
            fill_kernel<<<8192, 256>>>(b, fill_bytes / 16, 1u);
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0));
            for (int i = 0; i < 5; ++i) fill_kernel<<<8192, 256>>>(b, fill_bytes / 16, unsigned(i));
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
            printf("write, 8192 workgroups, %4zu MiB per pass: %.0f GB/s, %.1f us per pass\n", fill_bytes >> 20,
                   double(fill_bytes) * 5 / ms / 1e6, ms * 1e3 / 5);
        }
        // reads only, 160-row tiles of 1536-byte rows (a token block of the ViT-Base layers), 620 MB in all
        const int rows = 160, row_bytes = 1536;
        const long tiles = 316 * 8;
        for (int slice_bytes : {1536, 128, 64}) {
            for (int rep = 0; rep < 2; ++rep) {
                CK(hipEventRecord(e0));
                read_kernel<<<512, 512>>>((const unsigned char *)a, rows, row_bytes, slice_bytes, tiles, (unsigned *)b);
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
            }
            CK(hipEventElapsedTime(&ms, e0, e1));
            printf("read,  512 workgroups, %4d-byte pieces of each row at a time: %.0f GB/s\n", slice_bytes,
                   double(tiles) * rows * row_bytes / ms / 1e6);
        }
        CK(hipFree(a));
        CK(hipFree(b));
    }

    float *out;
    CK(hipMalloc(&out, size_t(cus) * 8 * 256 * 4));
    {  // MFMA, one workgroup of four waves per CU
        const size_t n = 256 * 7 * 8;
        std::vector<unsigned short> h(n);
        unsigned short *d;
        CK(hipMalloc(&d, n * 2));
        unsigned long long *stamps;
        CK(hipMalloc(&stamps, size_t(cus) * 4 * sizeof(unsigned long long)));
        std::vector<unsigned long long> hs(size_t(cus) * 4);
        for (int mode = 0; mode < 2; ++mode) {
            for (size_t i = 0; i < n; ++i) {
                const float f = mode == 0 ? 1.0f : ((rand() % 2000) - 1000) / 1000.0f;
                unsigned u;
                memcpy(&u, &f, 4);
                h[i] = (unsigned short)(u >> 16);
            }
            CK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
            for (int iters : {48, 480, 48000}) {
                mfma_kernel<<<cus, 256>>>((const bf16x8 *)d, out, iters, nullptr);
                CK(hipDeviceSynchronize());
                CK(hipEventRecord(e0));
                mfma_kernel<<<cus, 256>>>((const bf16x8 *)d, out, iters, stamps);
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
                CK(hipEventElapsedTime(&ms, e0, e1));
                CK(hipMemcpy(hs.data(), stamps, hs.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
                double ghz = 0;
                for (int w = 0; w < cus; ++w)
                    ghz += double(hs[w * 4 + 2] - hs[w * 4 + 0]) / (double(hs[w * 4 + 3] - hs[w * 4 + 1]) * 10.0);
                const double fl = double(cus) * 4 * iters * 10 * 2.0 * 32 * 32 * 16;
                printf("mfma_f32_32x32x16_bf16, %s operands, %5d MFMAs per wave: %8.3f ms, %.0f TFLOP/s, shader clock %.2f GHz\n",
                       mode ? "random  " : "constant", iters * 10, ms, fl / ms / 1e9, ghz / cus);
            }
        }
    }
    for (int wpc : {8, 32}) {  // vector ALU, wpc waves per CU
        const int blocks = cus * wpc / 4, iters = 20000;
        fma_kernel<<<blocks, 256>>>(out, 100, 1.0001f);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        fma_kernel<<<blocks, 256>>>(out, iters, 1.0001f);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("v_fma_f32, %2d waves per CU: %.1f TFLOP/s\n", wpc, double(blocks) * 256 * iters * 8 * 2.0 / ms / 1e9);
        CK(hipEventRecord(e0));
        dot2_kernel<<<blocks, 256>>>(out, iters, 3);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("v_dot2_f32_bf16, %2d waves per CU: %.1f TFLOP/s\n", wpc,
               double(blocks) * 256 * iters * 8 * 4.0 / ms / 1e9);
    }
    CK(hipFuncSetAttribute((const void *)lds_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    for (int wpc : {4, 8}) {
        const int blocks = cus * wpc / 4, iters = 20000;
        lds_kernel<<<blocks, 256, 65536>>>((unsigned *)out, 100);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        lds_kernel<<<blocks, 256, 65536>>>((unsigned *)out, iters);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        const double by = double(blocks) * 256 * iters * 8 * 16.0;
        printf("ds_read_b128, %d waves per CU: %.1f TB/s = %.0f B/clk/CU at 2.4 GHz\n", wpc, by / ms / 1e9,
               by / (ms * 1e-3) / cus / 2.4e9);
    }
    {  // reads served by the L2 (1 MB region per workgroup stream), by the memory-side cache (16 MB, 64 MB)
        const size_t bytes = size_t(64) << 20;
        u32x4 *src;
        CK(hipMalloc(&src, bytes));
        CK(hipMemset(src, 1, bytes));
        CK(hipFuncSetAttribute((const void *)cache_read_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 32768));
        const int iters = 400, wgs = 1024;
        for (int region_kb : {1024, 16384, 65536})
            for (int to_lds = 0; to_lds < 2; ++to_lds) {
                const int pieces = region_kb * 1024 / 16;
                for (int rep = 0; rep < 2; ++rep) {
                    CK(hipEventRecord(e0));
                    if (to_lds) cache_read_kernel<1><<<wgs, 256, 32768>>>(src, (u32x4 *)out, pieces, iters);
                    else cache_read_kernel<0><<<wgs, 256, 32768>>>(src, (u32x4 *)out, pieces, iters);
                    CK(hipEventRecord(e1));
                    CK(hipEventSynchronize(e1));
                }
                CK(hipEventElapsedTime(&ms, e0, e1));
                const double tb = double(wgs) * 256 * 16 * 8 * iters / 1e12;
                printf("cached reads, region %5d KB, into %s: %.1f TB/s = %.0f B/clk/CU at 2.4 GHz\n", region_kb,
                       to_lds ? "LDS      " : "registers", tb / (ms * 1e-3), tb * 1e12 / (ms * 1e-3) / cus / 2.4e9);
            }
        CK(hipFree(src));
    }
    return 0;
}
