// Products and weight gradient for a handful of diagonals (K <= 16): the regime of extreme sparsity (Sec. 4.4 trains
// down to a single active diagonal per layer), where the work T*K*L is so small that a product is bound by reading its
// input and writing its output once.  bf16 storage, fp32 accumulate, feature counts multiples of 128.
//
// The dense contraction of the matrix-core kernels costs the same at K = 1 as at K = D/10; these kernels visit only the
// K*L stored weights (Sec. 3.1 Eq. 3 applied diagonal by diagonal) and cost HBM traffic plus about 1.5 vector
// instructions per multiply-add:
//   * a tile of token rows is converted to fp32 once and laid out row-major in LDS, each row followed by a copy of its
//     first columns, so that a cyclically shifted read never wraps (and, for the masked gather, with zeros where the
//     source has no column);
//   * a lane owns the column pairs 2*lane + 128*i + {0, 1}, i < NI: for a fixed i the 64 lanes of a wave read 128
//     consecutive floats whatever the shift, which is free of bank conflicts at any offset, and store 256
//     consecutive bytes;
//   * the K x 2*NI weights a lane needs stay in registers for all rows of the tile, the K shifts in scalar registers.
#include "dd_common.h"
#include "dd_launch.h"

namespace dd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kLkMaxK = 16;
constexpr int kLkPieces = 4;              // 16-byte pieces of the next tile a thread holds in registers
constexpr int kLkResults = 8;             // packed results (column pairs x rows) of the current tile a lane holds
constexpr int kLkCUs = 256;
constexpr int kLkLdsPerCU = 160 * 1024;
constexpr int kLkLdsMax = 64 * 1024;      // per workgroup

// diagonals a kernel instance is unrolled for: exactly K up to 8, the next of 12 and 16 beyond (the spare
// diagonals carry zero weights)
constexpr int lowk_unroll(int K) { return K <= 8 ? K : (K <= 12 ? 12 : 16); }
// most waves of a workgroup: the 2 * ni * kc weights and kc read positions of a lane must fit the registers that many
// waves leave each other
constexpr int lowk_max_waves(int ni, int kc) { return (2 * ni + 1) * kc <= 40 ? 16 : 8; }

struct LkPlan {
    int ni;         // column pairs per lane: a slab is 128 * ni columns
    int slabs;      // slabs per destination row
    int groups;     // workgroups side by side along the row (blockIdx.y)
    int wg_slabs;   // slabs of one workgroup, one wave each ...
    int rowgroups;  // ... times this many waves per slab, which take every rowgroups-th row
    int threads;
    int wlds;       // floats per LDS row: D + slab width
    int rows_max;   // token rows per tile, at most
    bool ok;
};

// dst_cols: columns of the side the lanes own (the output of a product)
static LkPlan plan_lowk(int D, int dst_cols, int K)
{
    LkPlan pl{};
    if (D % 128 || dst_cols % 128 || D > 8192 || dst_cols < 128) return pl;
    const int units = dst_cols / 128;
    // fewest workgroups along the row first (each converts the whole tile of its own), then the narrowest slab
    // (its width is also the length of the wrapped copy every row carries)
    int best_groups = 1 << 30;
    for (int ni = 1; ni <= 4; ni *= 2) {
        if (units % ni) continue;
        const int slabs = units / ni, maxw = lowk_max_waves(ni, lowk_unroll(K));
        int groups = (slabs + maxw - 1) / maxw;
        while (slabs % groups) ++groups;
        if (groups < best_groups) { best_groups = groups; pl.ni = ni; pl.slabs = slabs; pl.groups = groups; }
    }
    pl.wg_slabs = pl.slabs / pl.groups;
    pl.rowgroups = pl.wg_slabs >= 4 ? 1 : 4 / pl.wg_slabs;
    pl.threads = 64 * pl.wg_slabs * pl.rowgroups;
    pl.wlds = D + 128 * pl.ni;
    // LDS: what a workgroup may take when as many workgroups as the wave slots allow share the CU
    int wgs = 32 / (pl.threads / 64);
    wgs = wgs < 1 ? 1 : (wgs > 8 ? 8 : wgs);
    int budget = kLkLdsPerCU / wgs - 512;
    if (budget > kLkLdsMax) budget = kLkLdsMax;
    const int by_lds = budget / (pl.wlds * 4);
    const int by_regs = kLkPieces * pl.threads / (pl.wlds / 8);
    pl.rows_max = by_lds < by_regs ? by_lds : by_regs;
    const int by_results = kLkResults / pl.ni * pl.rowgroups;
    if (pl.rows_max > by_results) pl.rows_max = by_results;
    pl.rows_max -= pl.rows_max % pl.rowgroups;
    pl.ok = pl.rows_max >= pl.rowgroups;
    return pl;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    return uint32_t(f32_to_bf16(a)) | (uint32_t(f32_to_bf16(b)) << 16);
}

// gather (MASKED = false):  dst[t, p] = sum_k src[t, (p + o_k) mod D] * v_k[p]            src [T x D], dst [T x L]
// masked gather:            dst[t, q] = sum_{k: c < L} src[t, c] * v_k[c], c = (q - o_k) mod D   src [T x L], dst [T x D]
// blockIdx.y: group of wg_slabs slabs, one per wave (times rowgroups waves that share the slab's rows);
// blockIdx.x walks the tiles of `rows` token rows with the grid's stride, so a wave loads its weights once.
// A tile is an LDS image of its rows in fp32: row r at r * wlds, logical column c (0 <= c < D) holds src[t0 + r][c]
// for c < src_cols and 0 beyond; columns D .. wlds repeat columns 0 .. wlds - D.  Rows past the last token are zero.
// While the waves work on a tile, the next one is on its way from memory into registers.
template <int NI, int KC, bool MASKED>
__global__ __launch_bounds__(64 * lowk_max_waves(NI, KC)) void lowk_product_kernel(
    int64_t T, int D, int L, int K, int wg_slabs, int rowgroups, int wlds, int rows, const uint16_t *__restrict__ src,
    const int *__restrict__ offsets, const uint16_t *__restrict__ values, uint16_t *__restrict__ dst)
{
    extern __shared__ __align__(16) float lk_lds[];
    __shared__ int s_off[kLkMaxK];
    const int src_cols = MASKED ? L : D, dst_cols = MASKED ? D : L;
    const int tid = threadIdx.x, lane = tid & 63, threads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    if (tid < KC) s_off[tid] = tid < K ? canonical_offset(offsets[tid], D) : 0;

    // the pieces of a tile this thread moves: 8 columns each, one 16-byte load, two 16-byte LDS stores
    const int ppr = wlds / 8, total = rows * ppr;
    int g_at[kLkPieces], l_at[kLkPieces], row_of[kLkPieces];
#pragma unroll
    for (int p = 0; p < kLkPieces; ++p) {
        const int idx = tid + p * threads;
        const int r = idx / ppr, c8 = (idx - r * ppr) * 8;
        const int c = c8 < D ? c8 : c8 - D;
        row_of[p] = r;
        l_at[p] = idx < total ? r * wlds + c8 : -1;
        g_at[p] = idx < total && c < src_cols ? r * src_cols + c : -1;
    }
    // Loads of the next tile: every thread issues all its loads (a piece without a source reads the first bytes of
    // src instead) and sorts out at the LDS store which of them count.
    u32x4 next[kLkPieces];
    unsigned live = 0;
    auto fetch = [&](int64_t t0) {
        live = 0;
#pragma unroll
        for (int p = 0; p < kLkPieces; ++p) {
            const bool there = g_at[p] >= 0 && t0 + row_of[p] < T;
            live |= unsigned(there) << p;
            next[p] = *reinterpret_cast<const u32x4 *>(there ? src + t0 * src_cols + g_at[p] : src);
        }
    };
    const int64_t n_tiles = (T + rows - 1) / rows;
    if (int64_t(blockIdx.x) >= n_tiles) return;  // (the grid is no larger than the number of tiles)
    fetch(int64_t(blockIdx.x) * rows);
#pragma unroll
    for (int p = 0; p < kLkPieces; ++p) {
        if (l_at[p] < 0) continue;
        u32x4 v = next[p];
        if (!(live >> p & 1)) v = u32x4{0u, 0u, 0u, 0u};
        float *at = lk_lds + l_at[p];
        *reinterpret_cast<f32x4 *>(at) = f32x4{__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xffff0000u),
                                               __uint_as_float(v[1] << 16), __uint_as_float(v[1] & 0xffff0000u)};
        *reinterpret_cast<f32x4 *>(at + 4) = f32x4{__uint_as_float(v[2] << 16), __uint_as_float(v[2] & 0xffff0000u),
                                                   __uint_as_float(v[3] << 16), __uint_as_float(v[3] & 0xffff0000u)};
    }
    __syncthreads();  // the offsets and the first tile are in LDS

    const int slab = int(blockIdx.y) * wg_slabs + wave % wg_slabs;
    const int first_row = wave / wg_slabs;
    const int j0 = slab * 128 * NI;
    // where in an LDS row this lane starts to read, and its weights, per diagonal
    int start[KC];
    float w[KC][NI][2];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const int o = s_off[k];
        int s = MASKED ? j0 - o : j0 + o;   // logical column the slab's first destination column reads
        s = s < 0 ? s + D : (s >= D ? s - D : s);
        start[k] = s + 2 * lane;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int j = j0 + 2 * lane + 128 * i + e;
                int c = j;
                if (MASKED) {
                    c = j - o;
                    c = c < 0 ? c + D : c;
                }
                const bool stored = k < K && c < L;
                const float v = bf16_to_f32(values[stored ? size_t(k) * L + c : 0]);
                w[k][i][e] = stored ? v : 0.f;
            }
    }

    // One round per tile: the next tile's loads go out first, the rows of the tile in LDS are worked into registers
    // while those loads fly, the loaded tile replaces the finished one in LDS, and only then are the results stored:
    // the wait for the loads so never waits for a store younger than one round.
    constexpr int RW = kLkResults / NI;  // rows of a tile a wave works, at most
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t t0 = tile * rows;
        if (tile + gridDim.x < n_tiles) fetch((tile + gridDim.x) * rows);
        uint32_t res[RW][NI];
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const int r = first_row + q * rowgroups;
            if (r >= rows) break;
            // (the row's place in LDS is worked out here, round by round: carried across the rounds, the addresses of
            // all rows and diagonals would take more registers than the weights)
            int row_at = r * wlds;
            asm volatile("" : "+s"(row_at));
            float a0[NI], a1[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) a0[i] = a1[i] = 0.f;
            // a batch of LDS reads, then their multiply-adds
            constexpr int KB = 8 / NI < KC ? 8 / NI : KC;
#pragma unroll
            for (int kb = 0; kb < KC; kb += KB) {
                float xv[KB][NI][2];
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    if (kb + k >= KC) break;
                    const float *x = lk_lds + row_at + start[kb + k];
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        xv[k][i][0] = x[128 * i];
                        xv[k][i][1] = x[128 * i + 1];
                    }
                }
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    if (kb + k >= KC) break;
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        a0[i] = fmaf(xv[k][i][0], w[kb + k][i][0], a0[i]);
                        a1[i] = fmaf(xv[k][i][1], w[kb + k][i][1], a1[i]);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < NI; ++i) res[q][i] = pack_bf16x2(a0[i], a1[i]);
        }
        // every load is waited for by every thread, whether or not its piece is kept
#pragma unroll
        for (int p = 0; p < kLkPieces; ++p)
            if (!(live >> p & 1)) next[p] = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();  // every wave is done with the tile in LDS
#pragma unroll
        for (int p = 0; p < kLkPieces; ++p) {
            if (l_at[p] < 0) continue;
            const u32x4 v = next[p];
            float *at = lk_lds + l_at[p];
            *reinterpret_cast<f32x4 *>(at) = f32x4{__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xffff0000u),
                                                   __uint_as_float(v[1] << 16), __uint_as_float(v[1] & 0xffff0000u)};
            *reinterpret_cast<f32x4 *>(at + 4) = f32x4{__uint_as_float(v[2] << 16), __uint_as_float(v[2] & 0xffff0000u),
                                                       __uint_as_float(v[3] << 16), __uint_as_float(v[3] & 0xffff0000u)};
        }
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const int r = first_row + q * rowgroups;
            if (r >= rows || t0 + r >= T) break;
            uint32_t *out = reinterpret_cast<uint32_t *>(dst + (t0 + r) * dst_cols + j0) + lane;
#pragma unroll
            for (int i = 0; i < NI; ++i) out[64 * i] = res[q][i];
        }
        __syncthreads();  // the next tile is in LDS
    }
}

// ---- weight gradient:  dV[k][p] = sum_t A[t, p] * B[t, (p + o_k) mod D],  A [T x L] the short side, B [T x D] ----
// The same tile image as the gather (rows of B in fp32, each followed by a copy of its first columns); a lane owns the
// positions p = j0 + 2*lane + 128*i + {0, 1} and keeps one accumulator per position and diagonal for all tokens of its
// workgroup.  Its own columns of A come straight from memory, four bytes per lane and row, one tile ahead.
// partial[chunk][k][p], chunk = blockIdx.x * rowgroups + (which of the waves that share a slab); lowk_reduce_kernel
// adds the chunks in index order.
constexpr int kLkMaxChunks = 512;
constexpr size_t kLkPartialBytes = size_t(16) << 20;  // partial sums of all chunks, at most (or 64 chunks' worth)

template <int NI, int KC>
__global__ __launch_bounds__(64 * lowk_max_waves(NI, KC)) void lowk_wgrad_kernel(
    int64_t T, int D, int L, int K, int wg_slabs, int rowgroups, int wlds, int rows, const uint16_t *__restrict__ A,
    const uint16_t *__restrict__ B, const int *__restrict__ offsets, float *__restrict__ partial)
{
    extern __shared__ __align__(16) float lk_lds[];
    __shared__ int s_off[kLkMaxK];
    const int tid = threadIdx.x, lane = tid & 63, threads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    if (tid < KC) s_off[tid] = tid < K ? canonical_offset(offsets[tid], D) : 0;

    const int ppr = wlds / 8, total = rows * ppr;
    int g_at[kLkPieces], l_at[kLkPieces], row_of[kLkPieces];
#pragma unroll
    for (int p = 0; p < kLkPieces; ++p) {
        const int idx = tid + p * threads;
        const int r = idx / ppr, c8 = (idx - r * ppr) * 8;
        const int c = c8 < D ? c8 : c8 - D;
        row_of[p] = r;
        l_at[p] = idx < total ? r * wlds + c8 : -1;
        g_at[p] = idx < total ? r * D + c : -1;
    }
    const int slab = int(blockIdx.y) * wg_slabs + wave % wg_slabs;
    const int first_row = wave / wg_slabs;
    const int j0 = slab * 128 * NI;
    constexpr int RW = kLkResults / NI;  // rows of a tile a wave works, at most

    u32x4 next[kLkPieces];
    uint32_t next_a[RW][NI];
    unsigned live = 0;
    auto fetch = [&](int64_t t0) {
        live = 0;
#pragma unroll
        for (int p = 0; p < kLkPieces; ++p) {
            const bool there = g_at[p] >= 0 && t0 + row_of[p] < T;
            live |= unsigned(there) << p;
            next[p] = *reinterpret_cast<const u32x4 *>(there ? B + t0 * D + g_at[p] : B);
        }
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const int r = first_row + q * rowgroups;
            const bool there = r < rows && t0 + r < T;
            const uint32_t *a = reinterpret_cast<const uint32_t *>(A + (there ? (t0 + r) * L + j0 : 0)) + lane;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const uint32_t v = a[64 * i];
                next_a[q][i] = there ? v : 0u;
            }
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int p = 0; p < kLkPieces; ++p) {
            if (l_at[p] < 0) continue;
            u32x4 v = next[p];
            if (!(live >> p & 1)) v = u32x4{0u, 0u, 0u, 0u};
            float *at = lk_lds + l_at[p];
            *reinterpret_cast<f32x4 *>(at) = f32x4{__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xffff0000u),
                                                   __uint_as_float(v[1] << 16), __uint_as_float(v[1] & 0xffff0000u)};
            *reinterpret_cast<f32x4 *>(at + 4) = f32x4{__uint_as_float(v[2] << 16), __uint_as_float(v[2] & 0xffff0000u),
                                                       __uint_as_float(v[3] << 16), __uint_as_float(v[3] & 0xffff0000u)};
        }
    };
    const int64_t n_tiles = (T + rows - 1) / rows;
    if (int64_t(blockIdx.x) >= n_tiles) return;  // (the grid is no larger than the number of tiles)
    fetch(int64_t(blockIdx.x) * rows);
    park();
    __syncthreads();  // the offsets and the first tile are in LDS

    int start[KC];
    float acc[KC][NI][2];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        int s = j0 + s_off[k];
        s = s >= D ? s - D : s;
        start[k] = s + 2 * lane;
#pragma unroll
        for (int i = 0; i < NI; ++i) acc[k][i][0] = acc[k][i][1] = 0.f;
    }

    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        uint32_t cur_a[RW][NI];
#pragma unroll
        for (int q = 0; q < RW; ++q)
#pragma unroll
            for (int i = 0; i < NI; ++i) cur_a[q][i] = next_a[q][i];
        const bool more = tile + gridDim.x < n_tiles;
        if (more) fetch((tile + gridDim.x) * rows);
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const int r = first_row + q * rowgroups;
            if (r >= rows) break;
            int row_at = r * wlds;
            asm volatile("" : "+s"(row_at));
            float a0[NI], a1[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                a0[i] = __uint_as_float(cur_a[q][i] << 16);
                a1[i] = __uint_as_float(cur_a[q][i] & 0xffff0000u);
            }
            constexpr int KB = 8 / NI < KC ? 8 / NI : KC;
#pragma unroll
            for (int kb = 0; kb < KC; kb += KB) {
                float xv[KB][NI][2];
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    if (kb + k >= KC) break;
                    const float *x = lk_lds + row_at + start[kb + k];
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        xv[k][i][0] = x[128 * i];
                        xv[k][i][1] = x[128 * i + 1];
                    }
                }
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    if (kb + k >= KC) break;
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        acc[kb + k][i][0] = fmaf(a0[i], xv[k][i][0], acc[kb + k][i][0]);
                        acc[kb + k][i][1] = fmaf(a1[i], xv[k][i][1], acc[kb + k][i][1]);
                    }
                }
            }
        }
        __syncthreads();  // every wave is done with the tile in LDS
        if (more) park();
        __syncthreads();  // the next tile is in LDS
    }

    const int chunk = int(blockIdx.x) * rowgroups + first_row;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        if (k >= K) break;
        float *out = partial + (size_t(chunk) * K + k) * L + j0 + 2 * lane;
#pragma unroll
        for (int i = 0; i < NI; ++i) *reinterpret_cast<float2 *>(out + 128 * i) = float2{acc[k][i][0], acc[k][i][1]};
    }
}

// dV[i..i+3] = partial[0][i..] + partial[1][i..] + ...: sixteen runs of consecutive chunks side by side, each summed in
// index order with up to eight loads in flight, then the sixteen sums in run order.  n4 = K * L / 4.
__global__ __launch_bounds__(1024) void lowk_reduce_kernel(int n4, int chunks, const float *__restrict__ partial,
                                                           float *__restrict__ dV)
{
    __shared__ f32x4 run_s[15][64];
    const int run = threadIdx.x >> 6, g = threadIdx.x & 63;
    const int i4 = blockIdx.x * 64 + g;
    const bool active = i4 < n4;
    const int per_run = (chunks + 15) / 16;
    const int s_begin = min(run * per_run, chunks), s_end = min(s_begin + per_run, chunks);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (active) {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(partial) + size_t(s_begin) * n4 + i4;
        int s = s_begin;
        for (; s + 8 <= s_end; s += 8) {
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[size_t(u) * n4];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
            src += size_t(8) * n4;
        }
        for (; s < s_end; ++s) {
            acc += *src;
            src += n4;
        }
    }
    if (run > 0) run_s[run - 1][g] = acc;
    __syncthreads();
    if (run == 0 && active) {
#pragma unroll
        for (int r = 0; r < 15; ++r) acc += run_s[r][g];
        reinterpret_cast<f32x4 *>(dV)[i4] = acc;
    }
}

bool product_lowk_supported(int64_t T, int D, int L, int K, bool bf16, bool masked)
{
    return bf16 && T > 0 && K >= 1 && K <= kLkMaxK && plan_lowk(D, masked ? D : L, K).ok;
}

// Rows per tile: between three quarters of the most and the most, whichever leaves the last round of tiles fullest.
static int lowk_rows(const LkPlan &pl, int64_t T, int64_t workers)
{
    int best = pl.rows_max;
    double best_fill = 0.0;
    const int lo = (3 * pl.rows_max + 3) / 4 > pl.rowgroups ? (3 * pl.rows_max + 3) / 4 : pl.rowgroups;
    for (int rows = pl.rows_max; rows >= lo; rows -= pl.rowgroups) {
        const int64_t tiles = (T + rows - 1) / rows, rounds = (tiles + workers - 1) / workers;
        const double fill = double(T) / (double(rounds) * double(workers) * rows);
        if (fill > best_fill + 1e-9) { best_fill = fill; best = rows; }
    }
    return best;
}

template <int NI, int KC, bool MASKED>
static hipError_t launch_lowk_product(const ProductArgs &a, const LkPlan &pl, hipStream_t stream)
{
    const void *kernel = reinterpret_cast<const void *>(&lowk_product_kernel<NI, KC, MASKED>);
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(kernel, kLkLdsMax, lds_allowed)) return e;
    const size_t lds_max = size_t(pl.rows_max) * pl.wlds * sizeof(float);
    // workgroups of this shape a CU holds (registers, LDS, wave slots): the last answer is remembered per block size
    static std::atomic<uint64_t> resident[17];  // LDS bytes << 16 | workgroups
    const uint64_t seen = resident[pl.threads / 64].load(std::memory_order_relaxed);
    int per_cu = int(seen & 0xffff);
    if (per_cu == 0 || (seen >> 16) != lds_max) {
        if (hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, pl.threads, lds_max)) return e;
        if (per_cu < 1) return hipErrorInvalidValue;
        resident[pl.threads / 64].store(uint64_t(lds_max) << 16 | uint64_t(per_cu), std::memory_order_relaxed);
    }
    int64_t workers = int64_t(kLkCUs) * per_cu / pl.groups;
    if (workers < 1) workers = 1;
    const int rows = lowk_rows(pl, a.T, workers);
    const int64_t n_tiles = (a.T + rows - 1) / rows;
    if (workers > n_tiles) workers = n_tiles;
    const dim3 grid{unsigned(workers), unsigned(pl.groups), 1u};
    hipLaunchKernelGGL((lowk_product_kernel<NI, KC, MASKED>), grid, dim3(pl.threads), lds_max, stream, a.T, a.D, a.L,
                       a.K, pl.wg_slabs, pl.rowgroups, pl.wlds, rows, static_cast<const uint16_t *>(a.src), a.offsets,
                       static_cast<const uint16_t *>(a.values), static_cast<uint16_t *>(a.dst));
    return hipGetLastError();
}

template <int NI, bool MASKED>
static hipError_t launch_lowk_product_k(const ProductArgs &a, const LkPlan &pl, hipStream_t stream)
{
    switch (lowk_unroll(a.K)) {
    case 1: return launch_lowk_product<NI, 1, MASKED>(a, pl, stream);
    case 2: return launch_lowk_product<NI, 2, MASKED>(a, pl, stream);
    case 3: return launch_lowk_product<NI, 3, MASKED>(a, pl, stream);
    case 4: return launch_lowk_product<NI, 4, MASKED>(a, pl, stream);
    case 5: return launch_lowk_product<NI, 5, MASKED>(a, pl, stream);
    case 6: return launch_lowk_product<NI, 6, MASKED>(a, pl, stream);
    case 7: return launch_lowk_product<NI, 7, MASKED>(a, pl, stream);
    case 8: return launch_lowk_product<NI, 8, MASKED>(a, pl, stream);
    case 12: return launch_lowk_product<NI, 12, MASKED>(a, pl, stream);
    default: return launch_lowk_product<NI, 16, MASKED>(a, pl, stream);
    }
}

template <int NI>
static hipError_t launch_lowk_product_m(const ProductArgs &a, const LkPlan &pl, hipStream_t stream)
{
    return a.masked ? launch_lowk_product_k<NI, true>(a, pl, stream) : launch_lowk_product_k<NI, false>(a, pl, stream);
}

hipError_t launch_product_lowk(const ProductArgs &a, hipStream_t stream)
{
    const LkPlan pl = plan_lowk(a.D, a.masked ? a.D : a.L, a.K);
    if (!pl.ok || a.K > kLkMaxK) return hipErrorInvalidValue;
    switch (pl.ni) {
    case 4: return launch_lowk_product_m<4>(a, pl, stream);
    case 2: return launch_lowk_product_m<2>(a, pl, stream);
    default: return launch_lowk_product_m<1>(a, pl, stream);
    }
}

// ---- weight gradient, host side ----

// most chunks of partial sums: bounded by number and by the bytes all of them take
static int lowk_wgrad_chunk_cap(const LkPlan &pl, int L, int K)
{
    int64_t cap = int64_t(kLkPartialBytes / (size_t(K) * L * sizeof(float)));
    if (cap < 64) cap = 64;
    if (cap > kLkMaxChunks) cap = kLkMaxChunks;
    cap -= cap % pl.rowgroups;
    return int(cap);
}

bool weight_grad_lowk_supported(int64_t T, int D, int L, int K, bool bf16)
{
    return bf16 && T > 0 && K >= 1 && K <= kLkMaxK && plan_lowk(D, L, K).ok;
}

size_t weight_grad_lowk_ws_bytes(int64_t T, int D, int L, int K)
{
    const LkPlan pl = plan_lowk(D, L, K);
    if (!pl.ok || K > kLkMaxK || T <= 0) return 0;
    return size_t(lowk_wgrad_chunk_cap(pl, L, K)) * K * L * sizeof(float);
}

template <int NI, int KC>
static hipError_t launch_lowk_wgrad(const WeightGradArgs &a, const LkPlan &pl, hipStream_t stream)
{
    const void *kernel = reinterpret_cast<const void *>(&lowk_wgrad_kernel<NI, KC>);
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(kernel, kLkLdsMax, lds_allowed)) return e;
    const size_t lds_max = size_t(pl.rows_max) * pl.wlds * sizeof(float);
    static std::atomic<uint64_t> resident[17];  // LDS bytes << 16 | workgroups
    const uint64_t seen = resident[pl.threads / 64].load(std::memory_order_relaxed);
    int per_cu = int(seen & 0xffff);
    if (per_cu == 0 || (seen >> 16) != lds_max) {
        if (hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, pl.threads, lds_max)) return e;
        if (per_cu < 1) return hipErrorInvalidValue;
        resident[pl.threads / 64].store(uint64_t(lds_max) << 16 | uint64_t(per_cu), std::memory_order_relaxed);
    }
    int64_t workers = int64_t(kLkCUs) * per_cu / pl.groups;
    const int64_t cap = lowk_wgrad_chunk_cap(pl, a.L, a.K) / pl.rowgroups;
    if (workers > cap) workers = cap;
    if (workers < 1) workers = 1;
    const int rows = lowk_rows(pl, a.T, workers);
    const int64_t n_tiles = (a.T + rows - 1) / rows;
    if (workers > n_tiles) workers = n_tiles;
    const dim3 grid{unsigned(workers), unsigned(pl.groups), 1u};
    float *partial = static_cast<float *>(a.ws);
    hipLaunchKernelGGL((lowk_wgrad_kernel<NI, KC>), grid, dim3(pl.threads), lds_max, stream, a.T, a.D, a.L, a.K,
                       pl.wg_slabs, pl.rowgroups, pl.wlds, rows, static_cast<const uint16_t *>(a.A),
                       static_cast<const uint16_t *>(a.B), a.offsets, partial);
    if (hipError_t e = hipGetLastError()) return e;
    const int n4 = a.K * a.L / 4, chunks = int(workers) * pl.rowgroups;
    hipLaunchKernelGGL(lowk_reduce_kernel, dim3((n4 + 63) / 64), dim3(1024), 0, stream, n4, chunks, partial, a.dValues);
    return hipGetLastError();
}

template <int NI>
static hipError_t launch_lowk_wgrad_k(const WeightGradArgs &a, const LkPlan &pl, hipStream_t stream)
{
    switch (lowk_unroll(a.K)) {
    case 1: return launch_lowk_wgrad<NI, 1>(a, pl, stream);
    case 2: return launch_lowk_wgrad<NI, 2>(a, pl, stream);
    case 3: return launch_lowk_wgrad<NI, 3>(a, pl, stream);
    case 4: return launch_lowk_wgrad<NI, 4>(a, pl, stream);
    case 5: return launch_lowk_wgrad<NI, 5>(a, pl, stream);
    case 6: return launch_lowk_wgrad<NI, 6>(a, pl, stream);
    case 7: return launch_lowk_wgrad<NI, 7>(a, pl, stream);
    case 8: return launch_lowk_wgrad<NI, 8>(a, pl, stream);
    case 12: return launch_lowk_wgrad<NI, 12>(a, pl, stream);
    default: return launch_lowk_wgrad<NI, 16>(a, pl, stream);
    }
}

hipError_t launch_weight_grad_lowk(const WeightGradArgs &a, hipStream_t stream)
{
    const LkPlan pl = plan_lowk(a.D, a.L, a.K);
    if (!pl.ok || a.K > kLkMaxK) return hipErrorInvalidValue;
    switch (pl.ni) {
    case 4: return launch_lowk_wgrad_k<4>(a, pl, stream);
    case 2: return launch_lowk_wgrad_k<2>(a, pl, stream);
    default: return launch_lowk_wgrad_k<1>(a, pl, stream);
    }
}

}  // namespace dd
