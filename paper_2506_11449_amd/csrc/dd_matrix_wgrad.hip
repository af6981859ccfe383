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
//   select:   a table offset -> first diagonal with that offset (built in LDS by every workgroup while its
//             first token slices are in flight) picks the entries of each accumulator tile; repeated
//             offsets read the same partial sums.
#include "dd_common.h"
#include "dd_launch.h"

#include <limits.h>

namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWgT = 256;           // threads
constexpr int kTS = 64;             // tokens per LDS stage
constexpr int kPad = 64;            // bytes added to every LDS row: rows of one transposing read fall on distinct banks
constexpr int kNoDiagonal = INT_MAX;
constexpr int kWgXcds = 8;          // L2 caches (one per XCD); workgroups are dealt to them round-robin
constexpr int kCusPerXcd = 32;

// Tile of G per workgroup: TP short-side x TQ long-side entries, four waves in a 2 x 2 arrangement.
template <int TP, int TQ>
struct WgTile {
    static constexpr int FA = TP / 64;             // 32-row MFMA tiles per wave
    static constexpr int FB = TQ / 64;             // 32-column MFMA tiles per wave
    static constexpr int ARow = TP * 2 + kPad;
    static constexpr int BRow = TQ * 2 + kPad;
    static constexpr int ABytes = kTS * ARow;
    static constexpr int BBytes = kTS * BRow;
    static constexpr int StageBytes = ABytes + BBytes;
    static constexpr int AChunks = kTS * (TP / 8) / kWgT;   // 16-byte pieces per thread per stage
    static constexpr int BChunks = kTS * (TQ / 8) / kWgT;
    static_assert(TP % 64 == 0 && TQ % 64 == 0, "wave tiles are made of 32x32 MFMA tiles");
};

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
template <int TP, int TQ>
__global__ __launch_bounds__(kWgT) void wgrad_mm_kernel(int T, int D, int L, int K, int tiles_p, int tiles_q,
                                                        int splits, int slices,
                                                        const uint16_t *__restrict__ A,
                                                        const uint16_t *__restrict__ B,
                                                        const int *__restrict__ offsets, float *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using Tl = WgTile<TP, TQ>;
    constexpr int kARow = Tl::ARow, kBRow = Tl::BRow, kABytes = Tl::ABytes, kStageBytes = Tl::StageBytes;
    constexpr int kAChunks = Tl::AChunks, kBChunks = Tl::BChunks, kTP = TP, kTQ = TQ;
    int *table = reinterpret_cast<int *>(smem + 2 * kStageBytes);  // [D]: offset -> first diagonal, or kNoDiagonal
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Token chunks are dealt to the XCDs: every tile of one chunk runs on the same L2, so the chunk's
    // slices of X and dY come from HBM once and from that L2 for every other tile.
    const int tiles = tiles_p * tiles_q;
    const int xcd = blockIdx.x % kWgXcds, local = blockIdx.x / kWgXcds;
    const int split = (local / tiles) * kWgXcds + xcd;
    if (split >= splits) return;
    const int tile = local % tiles;
    const int p0 = (tile / tiles_q) * kTP, q0 = (tile % tiles_q) * kTQ;
    // chunk `split` owns the 64-token slices [split * slices / splits, (split + 1) * slices / splits)
    const int slice_begin = int(int64_t(split) * slices / splits), slice_end = int(int64_t(split + 1) * slices / splits);
    const int t_begin = slice_begin * kTS;
    const int t_end = min(slice_end * kTS, T);
    const int n_slices = slice_end - slice_begin;


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
    const uint16_t *a_base[kAChunks], *b_base[kBChunks];
#pragma unroll
    for (int n = 0; n < kAChunks; ++n) a_base[n] = A + p0 + a_col[n];
#pragma unroll
    for (int n = 0; n < kBChunks; ++n) b_base[n] = B + q0 + b_col[n];
    u32x4 ag0[kAChunks], bg0[kBChunks], ag1[kAChunks], bg1[kBChunks];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    // Rows past the end of the chunk must add nothing: their short-side piece is replaced by zeros (one
    // zero factor is enough); the loads themselves stay in bounds by re-reading the last token.
#define DD_WG_LOAD(ag_, bg_, s_)                                                                        \
    {                                                                                                   \
        const int tb = t_begin + (s_) * kTS;                                                            \
        _Pragma("unroll") for (int n = 0; n < kAChunks; ++n) {                                          \
            const int t = tb + a_row[n];                                                                \
            const u32x4 v = *reinterpret_cast<const u32x4 *>(a_base[n] + size_t(min(t, T - 1)) * L);    \
            ag_[n] = t < t_end ? v : zero4;                                                             \
        }                                                                                               \
        _Pragma("unroll") for (int n = 0; n < kBChunks; ++n) {                                          \
            const int t = min(tb + b_row[n], T - 1);                                                    \
            bg_[n] = *reinterpret_cast<const u32x4 *>(b_base[n] + size_t(t) * D);                       \
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
    const int wp = wave >> 1, wq = wave & 1;     // wave tile: rows wp*TP/2.., columns wq*TQ/2..
    const int a_frag = frag_row * kARow + (wp * (TP / 2) + frag_col) * 2;
    const int b_frag = kABytes + frag_row * kBRow + (wq * (TQ / 2) + frag_col) * 2;

    f32x16 acc[Tl::FA][Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

#define DD_WG_FRAGS(fa_, fb_, buf_, ks_)                                                                 \
    {                                                                                                   \
        const unsigned char *base = smem + (buf_) * kStageBytes;                                        \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a) {                                            \
            const unsigned char *p = base + a_frag + (ks_) * 16 * kARow + a * 64;                       \
            fa_[a] = read_transposed(p, p + 4 * kARow);                                                 \
        }                                                                                               \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b) {                                            \
            const unsigned char *p = base + b_frag + (ks_) * 16 * kBRow + b * 64;                       \
            fb_[b] = read_transposed(p, p + 4 * kBRow);                                                 \
        }                                                                                               \
    }
#define DD_WG_MFMA(fa_, fb_)                                                                            \
    _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                                  \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                              \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[a], fb_[b], acc[a][b], 0, 0, 0);
    // four k-steps of one slice; the fragments of the next k-step are fetched while the current one multiplies
#define DD_WG_COMPUTE(buf_)                                                                             \
    DD_WG_FRAGS(fa0, fb0, buf_, 0)                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_FRAGS(fa1, fb1, buf_, 1)                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_MFMA(fa0, fb0)                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_FRAGS(fa0, fb0, buf_, 2)                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_MFMA(fa1, fb1)                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_FRAGS(fa1, fb1, buf_, 3)                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_MFMA(fa0, fb0)                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    DD_WG_MFMA(fa1, fb1)
    bf16x8 fa0[Tl::FA], fb0[Tl::FB], fa1[Tl::FA], fb1[Tl::FB];

    // Two slices in flight in registers, two LDS buffers, one barrier per slice; slices are taken in pairs,
    // an odd last one on its own.  The offset table is filled in LDS while the first slices travel.
    DD_WG_LOAD(ag0, bg0, 0)
    DD_WG_LOAD(ag1, bg1, 1)
    for (int i = tid; i < D; i += kWgT) table[i] = kNoDiagonal;
    __syncthreads();
    for (int k = tid; k < K; k += kWgT) atomicMin(&table[canonical_offset(offsets[k], D)], k);
    DD_WG_STORE(ag0, bg0, 0)
    __syncthreads();
    for (int s = 0; s + 1 < n_slices; s += 2) {
        DD_WG_LOAD(ag0, bg0, s + 2)
        __builtin_amdgcn_sched_barrier(0);
        DD_WG_COMPUTE(0)
        __builtin_amdgcn_sched_barrier(0);
        DD_WG_STORE(ag1, bg1, 1)
        __syncthreads();
        DD_WG_LOAD(ag1, bg1, s + 3)
        __builtin_amdgcn_sched_barrier(0);
        DD_WG_COMPUTE(1)
        __builtin_amdgcn_sched_barrier(0);
        DD_WG_STORE(ag0, bg0, 0)
        __syncthreads();
    }
    if (n_slices & 1) {  // uniform over the workgroup; the last slice sits in buffer 0
        DD_WG_COMPUTE(0)
        __syncthreads();
    }
#undef DD_WG_LOAD
#undef DD_WG_STORE
#undef DD_WG_COMPUTE
#undef DD_WG_FRAGS
#undef DD_WG_MFMA

    // Keep the entries on active diagonals, one 32x32 accumulator tile at a time.  Accumulator i of lane l
    // is row 8*(i/4) + 4*(l/32) + i%4, column l%32 of the tile.  The tile is laid out column-major in a
    // small LDS buffer of the wave's own; the 63 offsets that cross it are looked up at once (one per
    // lane); every active one is then read back along the diagonal, lane = row, so that the partial sums
    // of one diagonal leave as one contiguous run.  (The loop's last barrier retired all stage reads.)
    constexpr int kTileStride = 36;  // floats per tile column: 16-byte aligned rows of four, odd diagonal stride
    float *tilebuf = reinterpret_cast<float *>(smem) + wave * (32 * kTileStride);
    float *out = partial + size_t(split) * K * L;
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b) {
            const int pb = p0 + wp * (TP / 2) + a * 32, qb = q0 + wq * (TQ / 2) + b * 32;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                *reinterpret_cast<f32x4 *>(tilebuf + l32 * kTileStride + 8 * g + 4 * half) = v;
            }
            // lane j < 63 looks up the diagonal with (column - row) = j - 31 inside this tile
            int delta = qb - pb + lane - 31;
            delta = delta < 0 ? delta + D : (delta >= D ? delta - D : delta);
            const int kj = lane < 63 ? table[delta] : kNoDiagonal;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            unsigned long long active = __ballot(kj != kNoDiagonal);
            // four diagonals per round, two per half-wave, so that their LDS reads overlap
            while (active) {
                int j[4], kk[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    j[u] = active ? __builtin_ctzll(active) : 63;  // lane 63 never holds a diagonal
                    active &= active - 1;                          // no-op once empty
                    kk[u] = __builtin_amdgcn_readlane(kj, j[u]);
                }
                float v[2];
                int kd[2];
                bool ok[2];
#pragma unroll
                for (int uu = 0; uu < 2; ++uu) {
                    const int jj = half ? j[2 * uu + 1] : j[2 * uu];
                    kd[uu] = half ? kk[2 * uu + 1] : kk[2 * uu];
                    const int col = l32 + jj - 31;  // column of this lane's row on that diagonal
                    ok[uu] = kd[uu] != kNoDiagonal && col >= 0 && col < 32;
                    v[uu] = ok[uu] ? tilebuf[col * kTileStride + l32] : 0.f;
                }
#pragma unroll
                for (int uu = 0; uu < 2; ++uu)
                    if (ok[uu]) out[unsigned(kd[uu]) * unsigned(L) + unsigned(pb + l32)] = v[uu];
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
}

// dV[k][p] = sum over splits, in order, of partial[split][rep(k)][p], rep(k) = first diagonal with k's offset
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(int D, int L, int K, int splits,
                                                           const int *__restrict__ offsets,
                                                           const float *__restrict__ partial,
                                                           float *__restrict__ dV)
{
    __shared__ int rep_s;
    const int k = blockIdx.y;
    if (threadIdx.x == 0) rep_s = k;
    __syncthreads();
    const int mine = canonical_offset(offsets[k], D);
    for (int j = threadIdx.x; j < k; j += 256)
        if (canonical_offset(offsets[j], D) == mine) atomicMin(&rep_s, j);
    __syncthreads();
    const int rep = rep_s;
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= L) return;
    float acc = 0.f;
    for (int s = 0; s < splits; ++s) acc += partial[(size_t(s) * K + rep) * L + p];
    dV[size_t(k) * L + p] = acc;
}

// ---- host side ----

struct WgradPlan {
    int tp, tq;            // tile
    int tiles_p, tiles_q;
    int splits;            // token chunks (a multiple of the XCD count unless T is tiny)
    int slices;            // T in units of 64 tokens
    int grid;
};

static WgradPlan plan_wgrad(int64_t T, int D, int L)
{
    WgradPlan pl;
    // 192 x 192 tiles keep the four waves square (96 x 96) and divide the ViT-Base widths; otherwise 128 x 256
    if (L % 192 == 0 && D % 192 == 0) { pl.tp = 192; pl.tq = 192; } else { pl.tp = 128; pl.tq = 256; }
    pl.tiles_p = L / pl.tp;
    pl.tiles_q = D / pl.tq;
    const int tiles = pl.tiles_p * pl.tiles_q;
    // chunks per XCD: as many as fill its 32 CUs in one round
    int per_xcd = kCusPerXcd / tiles;
    if (per_xcd < 1) per_xcd = 1;
    int64_t splits = int64_t(per_xcd) * kWgXcds;
    const int64_t slices = (T + kTS - 1) / kTS;
    if (splits > slices) splits = slices;
    pl.slices = int(slices);
    pl.splits = int(splits);
    const int rounds = (pl.splits + kWgXcds - 1) / kWgXcds;
    pl.grid = rounds * tiles * kWgXcds;
    return pl;
}

bool weight_grad_matrix_supported(int64_t T, int D, int L, bool bf16)
{
    if (!(bf16 && T > 0 && T < (int64_t(1) << 31) && D <= 8192)) return false;
    return (L % 192 == 0 && D % 192 == 0) || (L % 128 == 0 && D % 256 == 0);
}

size_t weight_grad_matrix_ws_bytes(int64_t T, int D, int L, int K)
{
    const WgradPlan pl = plan_wgrad(T, D, L);
    return size_t(pl.splits) * K * L * sizeof(float);
}

template <int TP, int TQ>
static hipError_t launch_wgrad_mm(const WeightGradArgs &a, const WgradPlan &pl, float *partial, hipStream_t stream)
{
    using Tl = WgTile<TP, TQ>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_mm_kernel<TP, TQ>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           2 * Tl::StageBytes + 8192 * int(sizeof(int)));
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int lds_bytes = 2 * Tl::StageBytes + a.D * int(sizeof(int));
    hipLaunchKernelGGL((wgrad_mm_kernel<TP, TQ>), dim3(pl.grid), dim3(kWgT), lds_bytes, stream, int(a.T), a.D, a.L,
                       a.K, pl.tiles_p, pl.tiles_q, pl.splits, pl.slices,
                       static_cast<const uint16_t *>(a.A), static_cast<const uint16_t *>(a.B), a.offsets, partial);
    return hipGetLastError();
}

hipError_t launch_weight_grad_matrix(const WeightGradArgs &a, hipStream_t stream)
{
    const WgradPlan pl = plan_wgrad(a.T, a.D, a.L);
    float *partial = static_cast<float *>(a.ws);
    hipError_t e = pl.tp == 192 ? launch_wgrad_mm<192, 192>(a, pl, partial, stream)
                                : launch_wgrad_mm<128, 256>(a, pl, partial, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((a.L + 255) / 256, a.K), dim3(256), 0, stream, a.D, a.L, a.K,
                       pl.splits, a.offsets, partial, a.dValues);
    return hipGetLastError();
}

}  // namespace dd
