// Matrix-core path of the weight gradient (bf16 storage, fp32 accumulate), Fig. 3 h-i:
//   dV[k][p] = sum_t A[t, p] * B[t, (p + o_k) mod D],   A [T x L] the short side, B [T x D] the long side.
//
// The sum over tokens of the outer products A[t,:]^T B[t,:] is a contraction with the token index as the
// inner dimension, so it runs on the MFMA units tile by tile; of each finished 32x32 tile only the entries
// whose (column - row) mod D is an active offset are kept.  For the same reason as in the forward product
// (512 bf16 multiply-adds per clock per MFMA pipe against 16 on the vector ALU) this beats visiting only
// the K diagonals down to a density of a few percent, and it reads X and dY exactly as often.
//
//   tile:     128 short-side x 256 long-side entries of G per workgroup (four waves, 64 x 128 each),
//             over one chunk of tokens; chunks are summed afterwards in a fixed order (deterministic).
//   operands: both are stored token-major, the MFMA wants the contraction index contiguous per lane, so
//             token slices go to LDS as they are and come back through ds_read_b64_tr_b16, which hands
//             each lane four consecutive tokens of one feature.
//   select:   a table offset -> first diagonal with that offset (built by a one-workgroup kernel) picks
//             the entries of each accumulator tile; repeated offsets read the same partial sums.
#include "dd_common.h"
#include "dd_launch.h"

#include <limits.h>

namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWgT = 256;           // threads
constexpr int kTP = 128;            // tile extent along the short side (rows of the MFMA)
constexpr int kTQ = 256;            // tile extent along the long side (columns of the MFMA)
constexpr int kTS = 64;             // tokens per LDS stage
constexpr int kPad = 64;            // bytes added to every LDS row: rows of one transposing read fall on distinct banks
constexpr int kARow = kTP * 2 + kPad;
constexpr int kBRow = kTQ * 2 + kPad;
constexpr int kABytes = kTS * kARow;
constexpr int kBBytes = kTS * kBRow;
constexpr int kStageBytes = kABytes + kBBytes;
constexpr int kAChunks = kTS * (kTP / 8) / kWgT;   // 16-byte pieces per thread per stage
constexpr int kBChunks = kTS * (kTQ / 8) / kWgT;
constexpr int kNoDiagonal = INT_MAX;

// table[delta] = smallest k with canonical offset delta, or kNoDiagonal.  One workgroup.
__global__ __launch_bounds__(1024) void offset_table_kernel(int D, int K, const int *__restrict__ offsets,
                                                            int *__restrict__ table)
{
    for (int i = threadIdx.x; i < D; i += 1024) table[i] = kNoDiagonal;
    __syncthreads();
    for (int k = threadIdx.x; k < K; k += 1024) atomicMin(&table[canonical_offset(offsets[k], D)], k);
}

__device__ __forceinline__ bf16x8 read_transposed(const unsigned char *p0, const unsigned char *p1)
{
    // each call returns four consecutive tokens of this lane's feature; two make one MFMA operand
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// partial[split][k][p] for the representatives k of this tile's active offsets
__global__ __launch_bounds__(kWgT) void wgrad_mm_kernel(int T, int D, int L, int K, int tiles_p, int tiles_q,
                                                        int tokens_per_split, const uint16_t *__restrict__ A,
                                                        const uint16_t *__restrict__ B,
                                                        const int *__restrict__ table, float *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = blockIdx.x % (tiles_p * tiles_q);
    const int split = blockIdx.x / (tiles_p * tiles_q);
    const int p0 = (tile / tiles_q) * kTP, q0 = (tile % tiles_q) * kTQ;
    const int t_begin = split * tokens_per_split;
    const int t_end = min(t_begin + tokens_per_split, T);
    const int n_slices = (tokens_per_split + kTS - 1) / kTS;  // same for every split; tokens past t_end read as zero

    // global -> register -> LDS staging.  A piece is 8 features of one token.
    int a_row[kAChunks], a_col[kAChunks], b_row[kBChunks], b_col[kBChunks];
#pragma unroll
    for (int n = 0; n < kAChunks; ++n) {
        const int idx = tid + kWgT * n;
        a_row[n] = idx / (kTP / 8);
        a_col[n] = (idx % (kTP / 8)) * 8;
    }
#pragma unroll
    for (int n = 0; n < kBChunks; ++n) {
        const int idx = tid + kWgT * n;
        b_row[n] = idx / (kTQ / 8);
        b_col[n] = (idx % (kTQ / 8)) * 8;
    }
    u32x4 ag0[kAChunks], bg0[kBChunks];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
#define DD_WG_LOAD(ag_, bg_, s_)                                                                        \
    {                                                                                                   \
        const int tb = t_begin + (s_) * kTS;                                                            \
        _Pragma("unroll") for (int n = 0; n < kAChunks; ++n) {                                          \
            const int t = tb + a_row[n];                                                                \
            ag_[n] = t < t_end ? *reinterpret_cast<const u32x4 *>(A + size_t(t) * L + p0 + a_col[n]) : zero4; \
        }                                                                                               \
        _Pragma("unroll") for (int n = 0; n < kBChunks; ++n) {                                          \
            const int t = tb + b_row[n];                                                                \
            bg_[n] = t < t_end ? *reinterpret_cast<const u32x4 *>(B + size_t(t) * D + q0 + b_col[n]) : zero4; \
        }                                                                                               \
    }
#define DD_WG_STORE(ag_, bg_, buf_)                                                                     \
    {                                                                                                   \
        unsigned char *base = smem + (buf_) * kStageBytes;                                              \
        _Pragma("unroll") for (int n = 0; n < kAChunks; ++n)                                            \
            *reinterpret_cast<u32x4 *>(base + a_row[n] * kARow + a_col[n] * 2) = ag_[n];                \
        _Pragma("unroll") for (int n = 0; n < kBChunks; ++n)                                            \
            *reinterpret_cast<u32x4 *>(base + kABytes + b_row[n] * kBRow + b_col[n] * 2) = bg_[n];      \
    }

    // Fragment addressing.  In a group of 16 lanes, lane s supplies row s/4 (a token) and features
    // 4*(s%4)..+3; it receives feature s of the group for those four tokens.  Groups 0,1 cover features
    // 0-15 / 16-31 of the first 8 tokens of a k-step, groups 2,3 the same features of the last 8.
    const int s16 = lane & 15, grp = lane >> 4;
    const int frag_row = (grp >> 1) * 8 + (s16 >> 2);
    const int frag_col = (grp & 1) * 16 + (s16 & 3) * 4;
    const int wp = wave >> 1, wq = wave & 1;     // wave tile: rows wp*64.., columns wq*128..
    const int a_frag = frag_row * kARow + (wp * 64 + frag_col) * 2;
    const int b_frag = kABytes + frag_row * kBRow + (wq * 128 + frag_col) * 2;

    f32x16 acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

#define DD_WG_COMPUTE(buf_)                                                                             \
    _Pragma("unroll") for (int ks = 0; ks < kTS / 16; ++ks) {                                           \
        const unsigned char *base = smem + (buf_) * kStageBytes;                                        \
        bf16x8 fa[2], fb[4];                                                                            \
        _Pragma("unroll") for (int a = 0; a < 2; ++a) {                                                 \
            const unsigned char *p = base + a_frag + ks * 16 * kARow + a * 64;                          \
            fa[a] = read_transposed(p, p + 4 * kARow);                                                  \
        }                                                                                               \
        _Pragma("unroll") for (int b = 0; b < 4; ++b) {                                                 \
            const unsigned char *p = base + b_frag + ks * 16 * kBRow + b * 64;                          \
            fb[b] = read_transposed(p, p + 4 * kBRow);                                                  \
        }                                                                                               \
        _Pragma("unroll") for (int a = 0; a < 2; ++a)                                                   \
            _Pragma("unroll") for (int b = 0; b < 4; ++b)                                               \
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);  \
    }

    // one slice in flight in registers while the previous one is multiplied out of LDS; two LDS buffers,
    // one barrier per slice
    DD_WG_LOAD(ag0, bg0, 0)
    DD_WG_STORE(ag0, bg0, 0)
    __syncthreads();
    for (int s = 0; s < n_slices; ++s) {
        DD_WG_LOAD(ag0, bg0, s + 1)
        __builtin_amdgcn_sched_barrier(0);
        DD_WG_COMPUTE(s & 1)
        __builtin_amdgcn_sched_barrier(0);
        DD_WG_STORE(ag0, bg0, (s + 1) & 1)
        __syncthreads();
    }
#undef DD_WG_LOAD
#undef DD_WG_STORE
#undef DD_WG_COMPUTE

    // Keep the entries on active diagonals.  Accumulator i of lane l: row 8*(i/4) + 4*(l/32) + i%4,
    // column l%32 of its 32x32 tile.
    float *out = partial + size_t(split) * K * L;
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int q = q0 + wq * 128 + b * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int p = p0 + wp * 64 + a * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                int delta = q - p;
                if (delta < 0) delta += D;
                const int k = table[delta];
                if (k != kNoDiagonal) out[size_t(k) * L + p] = acc[a][b][i];
            }
        }
}

// dV[k][p] = sum over splits, in order, of partial[split][rep(k)][p], rep(k) = first diagonal with k's offset
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(int D, int L, int K, int splits,
                                                           const int *__restrict__ offsets,
                                                           const int *__restrict__ table,
                                                           const float *__restrict__ partial,
                                                           float *__restrict__ dV)
{
    const int k = blockIdx.y;
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= L) return;
    const int rep = table[canonical_offset(offsets[k], D)];
    float acc = 0.f;
    for (int s = 0; s < splits; ++s) acc += partial[(size_t(s) * K + rep) * L + p];
    dV[size_t(k) * L + p] = acc;
}

// ---- host side ----

struct WgradPlan {
    int tiles_p, tiles_q, splits, tokens_per_split;
};

static WgradPlan plan_wgrad(int64_t T, int D, int L)
{
    WgradPlan pl;
    pl.tiles_p = L / kTP;
    pl.tiles_q = D / kTQ;
    const int tiles = pl.tiles_p * pl.tiles_q;
    // as many token chunks as fit the 256 CUs in one round, each a whole number of 64-token slices
    int splits = 256 / tiles;
    const int64_t slices = (T + kTS - 1) / kTS;
    if (splits > slices) splits = int(slices);
    if (splits < 1) splits = 1;
    const int64_t per = ((slices + splits - 1) / splits) * kTS;
    pl.tokens_per_split = int(per);
    pl.splits = int((T + per - 1) / per);
    return pl;
}

bool weight_grad_matrix_supported(int64_t T, int D, int L, bool bf16)
{
    return bf16 && T > 0 && T < (int64_t(1) << 31) && L % kTP == 0 && D % kTQ == 0 && D <= 8192;
}

static size_t table_bytes(int D) { return (size_t(D) * sizeof(int) + 255) / 256 * 256; }

size_t weight_grad_matrix_ws_bytes(int64_t T, int D, int L, int K)
{
    const WgradPlan pl = plan_wgrad(T, D, L);
    return table_bytes(D) + size_t(pl.splits) * K * L * sizeof(float);
}

hipError_t launch_weight_grad_matrix(const WeightGradArgs &a, hipStream_t stream)
{
    const WgradPlan pl = plan_wgrad(a.T, a.D, a.L);
    int *table = static_cast<int *>(a.ws);
    float *partial = reinterpret_cast<float *>(static_cast<unsigned char *>(a.ws) + table_bytes(a.D));
    hipLaunchKernelGGL(offset_table_kernel, dim3(1), dim3(1024), 0, stream, a.D, a.K, a.offsets, table);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    static bool configured = false;
    if (!configured) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_mm_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStageBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int grid = pl.tiles_p * pl.tiles_q * pl.splits;
    hipLaunchKernelGGL(wgrad_mm_kernel, dim3(grid), dim3(kWgT), 2 * kStageBytes, stream, int(a.T), a.D, a.L, a.K,
                       pl.tiles_p, pl.tiles_q, pl.tokens_per_split, static_cast<const uint16_t *>(a.A),
                       static_cast<const uint16_t *>(a.B), table, partial);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((a.L + 255) / 256, a.K), dim3(256), 0, stream, a.D, a.L, a.K,
                       pl.splits, a.offsets, table, partial, a.dValues);
    return hipGetLastError();
}

}  // namespace dd
