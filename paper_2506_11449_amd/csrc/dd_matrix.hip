// Matrix-core path of the forward and backward-input products (bf16 storage, fp32 accumulate).
//
// On gfx950 one MFMA pipe retires 512 bf16 multiply-adds per clock against 16 fp32 FMAs on the
// vector ALU of the same SIMD, so down to a density K/D of a few percent it is faster to rebuild
// the K diagonals as a dense operand and run the product as a tiled contraction than to visit
// only the K*L stored weights on the vector ALUs.  HBM traffic is the same either way: X is read
// once, Y written once; the dense operand (<= a few MB) lives in L2.
//
// Step 1 (materialize_kernel): the operand Bt [NC x KD] (one row per output column, contraction
//   index contiguous) is written from (offsets, values) following Sec. 3.1 Eq. 1-3 / Appendix A.
// Step 2 (mm_kernel): C [T x NC] = A [T x KD] . Bt^T with v_mfma_f32_32x32x16_bf16.  A workgroup
//   of four waves owns a BM x BN tile of C; both operands are staged through LDS in 64-wide
//   k-slices, double buffered; 16-byte chunks are XOR-swizzled so that fragment reads are free of
//   bank conflicts.  The MFMA rows are output columns and the MFMA columns are tokens, which leaves
//   every lane with four consecutive output columns of one token, so the tile is transposed back
//   through LDS once and stored with full-width row segments.
#include "dd_common.h"
#include "dd_launch.h"

namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMmThreads = 256;
constexpr int kBK = 64;          // contraction extent of one LDS stage: 64 bf16 = 128 bytes per row
constexpr int kRowBytes = kBK * 2;
constexpr int kXcds = 8;

// position of 16-byte chunk `chunk` (0..7) inside its 128-byte row
__device__ __forceinline__ int swizzle(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// ---------------------------------------------------------------------------------------------
// Step 1: dense operand from the diagonals.
//   long_major = 1:  Bt[q][p] = sum_{k: (q - o_k) mod D = p < L} v_k[p]     rows q in [0, D), KD = L
//   long_major = 0:  Bt[p][q] = sum_{k: (p + o_k) mod D = q} v_k[p]         rows p in [0, L), KD = D
// One workgroup per row; the row is summed in fp32 in LDS (repeated offsets add, Eq. 3) and
// rounded to bf16 once.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void materialize_kernel(int D, int L, int K, int long_major,
                                                          const int *__restrict__ offsets,
                                                          const uint16_t *__restrict__ values,
                                                          uint16_t *__restrict__ Bt)
{
    extern __shared__ float row[];
    const int r = blockIdx.x;
    const int KD = long_major ? L : D;
    for (int c = threadIdx.x; c < KD; c += 256) row[c] = 0.f;
    __syncthreads();
    for (int k = threadIdx.x; k < K; k += 256) {
        const int o = canonical_offset(offsets[k], D);
        if (long_major) {
            int p = r - o;
            if (p < 0) p += D;
            if (p < L) atomicAdd(&row[p], bf16_to_f32(values[size_t(k) * L + p]));
        } else {
            int q = r + o;
            if (q >= D) q -= D;
            atomicAdd(&row[q], bf16_to_f32(values[size_t(k) * L + r]));
        }
    }
    __syncthreads();
    uint16_t *dst = Bt + size_t(r) * KD;
    for (int c = threadIdx.x; c < KD; c += 256) dst[c] = f32_to_bf16(row[c]);
}

// ---------------------------------------------------------------------------------------------
// Step 2: C [T x NC] = A [T x KD] . Bt[NC x KD]^T
// ---------------------------------------------------------------------------------------------
template <int BM, int BN>
struct MmTile {
    static constexpr int WN = BN / 4;              // output columns per wave
    static constexpr int FA = WN / 32;             // 32-row MFMA tiles along the output columns
    static constexpr int FB = BM / 32;             // 32-column MFMA tiles along the tokens
    static constexpr int X_CHUNKS = BM * 8 / kMmThreads;
    static constexpr int W_CHUNKS = BN * 8 / kMmThreads;
    static constexpr int X_BYTES = BM * kRowBytes;
    static constexpr int W_BYTES = BN * kRowBytes;
    static constexpr int STAGE = X_BYTES + W_BYTES;
    static constexpr int C_STRIDE = (BN + 8) * 2;  // bytes; the pad staggers rows over the banks
    static constexpr int C_BYTES = BM * C_STRIDE;
    static constexpr int LDS_BYTES = 2 * STAGE > C_BYTES ? 2 * STAGE : C_BYTES;
    static_assert(BM % 32 == 0 && BN % 128 == 0, "tile must split into 32x32 MFMA tiles over four waves");
};

template <int BM, int BN>
__global__ __launch_bounds__(kMmThreads) void mm_kernel(int T, int NC, int KD, int tiles_m, int tiles_n,
                                                        const uint16_t *__restrict__ A,
                                                        const uint16_t *__restrict__ Bt,
                                                        uint16_t *__restrict__ C)
{
    using Tl = MmTile<BM, BN>;
    extern __shared__ __align__(16) unsigned char smem[];

    // Workgroups are dealt round-robin to the eight XCDs, each with an L2 of its own.  Give every
    // XCD one contiguous run of tiles, column tiles innermost, so that the tiles sharing a token
    // block (and with it a slice of A) run on the same L2.
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const int lin = int(blockIdx.x % kXcds) * per_xcd + int(blockIdx.x / kXcds);
    if (lin >= n_tiles) return;
    const int tm = lin / tiles_n, tn = lin % tiles_n;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // global -> register -> LDS staging: thread handles chunk (row = idx / 8, chunk = idx % 8)
    const uint16_t *x_src[Tl::X_CHUNKS];
    int x_dst[Tl::X_CHUNKS];
#pragma unroll
    for (int n = 0; n < Tl::X_CHUNKS; ++n) {
        const int idx = tid + kMmThreads * n;
        const int row = idx >> 3, ch = idx & 7;
        int t = tm * BM + row;
        t = t < T ? t : T - 1;  // rows past the end re-read the last token; their results are not stored
        x_src[n] = A + size_t(t) * KD + ch * 8;
        x_dst[n] = row * kRowBytes + swizzle(row, ch) * 16;
    }
    const uint16_t *w_src[Tl::W_CHUNKS];
    int w_dst[Tl::W_CHUNKS];
#pragma unroll
    for (int n = 0; n < Tl::W_CHUNKS; ++n) {
        const int idx = tid + kMmThreads * n;
        const int row = idx >> 3, ch = idx & 7;
        w_src[n] = Bt + size_t(tn * BN + row) * KD + ch * 8;
        w_dst[n] = Tl::X_BYTES + row * kRowBytes + swizzle(row, ch) * 16;
    }

    f32x16 acc[Tl::FA][Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // fragment rows of this lane
    const int l32 = lane & 31, half = lane >> 5;
    int a_off[Tl::FA], a_sw[Tl::FA], b_off[Tl::FB], b_sw[Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a) {
        const int row = wave * Tl::WN + a * 32 + l32;
        a_off[a] = Tl::X_BYTES + row * kRowBytes;
        a_sw[a] = (row >> 1) & 7;
    }
#pragma unroll
    for (int b = 0; b < Tl::FB; ++b) {
        const int row = b * 32 + l32;
        b_off[b] = row * kRowBytes;
        b_sw[b] = (row >> 1) & 7;
    }

    // Software pipeline: the global loads of k-slice kt+1 are in flight while slice kt is multiplied
    // out of LDS; they are parked in LDS (other buffer) afterwards.  One barrier per slice.
    const int KT = KD / kBK;
    u32x4 x_reg[Tl::X_CHUNKS], w_reg[Tl::W_CHUNKS];
#define DD_LOAD_STAGE(kt_)                                                                              \
    _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n)                                            \
        x_reg[n] = *reinterpret_cast<const u32x4 *>(x_src[n] + (kt_) * kBK);                            \
    _Pragma("unroll") for (int n = 0; n < Tl::W_CHUNKS; ++n)                                            \
        w_reg[n] = *reinterpret_cast<const u32x4 *>(w_src[n] + (kt_) * kBK);
#define DD_STORE_STAGE(s_)                                                                              \
    _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n)                                            \
        *reinterpret_cast<u32x4 *>(smem + (s_) * Tl::STAGE + x_dst[n]) = x_reg[n];                      \
    _Pragma("unroll") for (int n = 0; n < Tl::W_CHUNKS; ++n)                                            \
        *reinterpret_cast<u32x4 *>(smem + (s_) * Tl::STAGE + w_dst[n]) = w_reg[n];
#define DD_COMPUTE_STAGE(s_)                                                                            \
    _Pragma("unroll") for (int ks = 0; ks < kBK / 16; ++ks) {                                           \
        const unsigned char *base = smem + (s_) * Tl::STAGE;                                            \
        const int ch = ks * 2 + half;                                                                   \
        bf16x8 fa[Tl::FA], fb[Tl::FB];                                                                  \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                              \
            fa[a] = *reinterpret_cast<const bf16x8 *>(base + a_off[a] + ((ch ^ a_sw[a]) << 4));         \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                              \
            fb[b] = *reinterpret_cast<const bf16x8 *>(base + b_off[b] + ((ch ^ b_sw[b]) << 4));         \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                              \
            _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                          \
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);  \
    }

    DD_LOAD_STAGE(0)
    DD_STORE_STAGE(0)
    __syncthreads();
    for (int kt = 0; kt + 1 < KT; ++kt) {
        DD_LOAD_STAGE(kt + 1)
        __builtin_amdgcn_sched_barrier(0);  // keep the loads ahead of the multiply, not behind it
        DD_COMPUTE_STAGE(kt & 1)
        __builtin_amdgcn_sched_barrier(0);
        DD_STORE_STAGE((kt + 1) & 1)
        __syncthreads();
    }
    DD_COMPUTE_STAGE((KT - 1) & 1)
    __syncthreads();
#undef DD_LOAD_STAGE
#undef DD_STORE_STAGE
#undef DD_COMPUTE_STAGE

    // Epilogue.  Accumulator i of lane l is output column 8*(i/4) + 4*(l/32) + i%4 of token l%32
    // inside its 32x32 tile: four consecutive columns per group, written as one 8-byte LDS store.
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                const bf16x4 h = __builtin_convertvector(v, bf16x4);
                const int t_local = b * 32 + l32;
                const int j_local = wave * Tl::WN + a * 32 + 8 * g + 4 * half;
                *reinterpret_cast<bf16x4 *>(smem + t_local * Tl::C_STRIDE + j_local * 2) = h;
            }
    __syncthreads();
    constexpr int ROW_CHUNKS = BN / 8;
    for (int idx = tid; idx < BM * ROW_CHUNKS; idx += kMmThreads) {
        const int row = idx / ROW_CHUNKS, ch = idx % ROW_CHUNKS;
        const int t = tm * BM + row;
        if (t < T)
            *reinterpret_cast<uint4 *>(C + size_t(t) * NC + tn * BN + ch * 8) =
                *reinterpret_cast<const uint4 *>(smem + row * Tl::C_STRIDE + ch * 16);
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
bool product_matrix_supported(int64_t T, int D, int L, bool bf16)
{
    return bf16 && T > 0 && T < (int64_t(1) << 31) && D % 128 == 0 && L % 128 == 0 && D <= 8192;
}

size_t product_matrix_ws_bytes(int D, int L) { return size_t(D) * size_t(L) * 2; }

template <int BM, int BN>
static hipError_t launch_mm(int T, int NC, int KD, const uint16_t *A, const uint16_t *Bt, uint16_t *C,
                            hipStream_t stream)
{
    using Tl = MmTile<BM, BN>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&mm_kernel<BM, BN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Tl::LDS_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int tiles_m = (T + BM - 1) / BM, tiles_n = NC / BN;
    const int per_xcd = (tiles_m * tiles_n + kXcds - 1) / kXcds;
    hipLaunchKernelGGL((mm_kernel<BM, BN>), dim3(per_xcd * kXcds), dim3(kMmThreads), Tl::LDS_BYTES, stream, T, NC, KD,
                       tiles_m, tiles_n, A, Bt, C);
    return hipGetLastError();
}

// Largest tile whose workgroup count fills the 256 CUs in the fewest, fullest rounds.
static int pick_tile(int64_t T, int NC)
{
    static const int bm[] = {192, 160, 128, 96, 64};
    int best = 0;
    double best_cost = 1e300;
    for (int i = 0; i < 5; ++i) {
        if (NC % 256) continue;
        const int64_t tiles = ((T + bm[i] - 1) / bm[i]) * (NC / 256);
        const int64_t rounds = (tiles + 255) / 256;
        // small tiles re-read more of both operands per multiply-add
        const double cost = double(rounds) * bm[i] * 256 * (1.0 + 24.0 / bm[i]);
        if (cost < best_cost) { best_cost = cost; best = bm[i]; }
    }
    return best;
}

hipError_t launch_product_matrix(const ProductArgs &a, hipStream_t stream)
{
    // masked gather: dst has D columns, contraction over the L columns of src  -> operand rows are long-side
    const int NC = a.masked ? a.D : a.L;
    const int KD = a.masked ? a.L : a.D;
    uint16_t *Bt = static_cast<uint16_t *>(a.ws);
    hipLaunchKernelGGL(materialize_kernel, dim3(NC), dim3(256), size_t(KD) * sizeof(float), stream, a.D, a.L, a.K,
                       a.masked ? 1 : 0, a.offsets, static_cast<const uint16_t *>(a.values), Bt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint16_t *A = static_cast<const uint16_t *>(a.src);
    uint16_t *C = static_cast<uint16_t *>(a.dst);
    const int T = int(a.T);
    if (NC % 256 == 0) {
        switch (pick_tile(a.T, NC)) {
        case 192: return launch_mm<192, 256>(T, NC, KD, A, Bt, C, stream);
        case 160: return launch_mm<160, 256>(T, NC, KD, A, Bt, C, stream);
        case 128: return launch_mm<128, 256>(T, NC, KD, A, Bt, C, stream);
        case 96: return launch_mm<96, 256>(T, NC, KD, A, Bt, C, stream);
        default: return launch_mm<64, 256>(T, NC, KD, A, Bt, C, stream);
        }
    }
    return launch_mm<128, 128>(T, NC, KD, A, Bt, C, stream);
}

}  // namespace dd
