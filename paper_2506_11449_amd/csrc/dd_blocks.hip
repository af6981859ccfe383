// Forward / backward-input product on the matrix cores that skips the blocks of the dense operand no diagonal
// crosses (bf16 storage, fp32 accumulate).
//
// Where the active offsets lie in runs of adjacent diagonals (the small-world structure learned masks show,
// Sec. 3.3 and the small-world appendix; the blocking of Appendix D relies on the same), most 32 x 16 blocks of
// W_K hold no entry at all: a block of output columns [j0, j0+32) and contraction indices [i0, i0+16) is crossed by
// the 47 offsets (long index - short index) that run through it and by no others.  With K offsets drawn uniformly
// nearly every block is crossed (density K/D per entry, but 47 K/D diagonals per block), so this kernel only pays
// for clustered offsets; it is chosen by the caller (DD_ALGO_BLOCKS), who knows where the offsets come from.
//
// Work split: a workgroup (four waves) owns 32*FB*NW tokens x 128 output columns, three workgroups share a CU.  Every wave owns 32*FB tokens and ALL 128 columns,
// so all waves meet the same blocks and skip the same blocks: skipping never leaves a wave waiting for another.
// (In mm_kernel the waves split the columns; there a wave whose blocks are empty would only wait at the next barrier.)
// Per 32-index k-slice that holds any crossed block, the token rows (32*FB*NW x 64 bytes) and the 8 operand blocks
// (1 KB each, fragment-major as materialize_kernel writes them; blocks that are not crossed are not fetched) travel
// from global memory straight into a three-deep ring of LDS stages; slices without a crossed block are not visited.
// With most blocks skipped a slice is multiplied in a few hundred clocks and a tile is a handful of slices: what
// bounds the kernel is latency (list, pipeline fill, copy-out), which the three workgroups of a CU hide for each other.
// Which blocks are crossed is worked out by every workgroup from the offsets (a bitmap of the D candidates in LDS).
#include "dd_common.h"
#include "dd_launch.h"
#include "dd_ring.h"

namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlkXcds = 8;
constexpr int kBlkBN = 128;            // output columns per workgroup: four 32-column blocks
constexpr int kBlkFA = kBlkBN / 32;
constexpr int kBlkSlice = 32;          // contraction indices per stage: 64 bytes per token row, two MFMA k-steps
constexpr int kBlkSteps = kBlkSlice / 16;
constexpr int kBlkRing = 3;            // LDS stages: one being multiplied, two on their way
constexpr int kBlkAhead = kBlkRing - 1;
constexpr int kBlkWBytes = kBlkFA * kBlkSteps * 1024;   // operand blocks of one slice
constexpr int kBlkMaxD = 8192;
constexpr int kBlkMaxSlices = kBlkMaxD / kBlkSlice;

__device__ __align__(16) const unsigned int blk_zero_piece[4] = {0u, 0u, 0u, 0u};

template <int FB, int NW>
struct BlkTile {
    static constexpr int THREADS = 64 * NW;
    static constexpr int BM = 32 * FB * NW;
    static constexpr int XBytes = BM * kBlkSlice * 2;
    static constexpr int StageBytes = XBytes + kBlkWBytes;
    static constexpr int XRounds = XBytes / 1024 / NW;        // 1 KB transfers per wave per stage, token rows
    static constexpr int WRounds = kBlkWBytes / 1024 / NW;    // operand blocks
    static constexpr int Rounds = XRounds + WRounds;
    static constexpr int CStride = kBlkBN * 2 + 16;           // bytes per token row of the result on its way out
    static constexpr int RingBytes = kBlkRing * StageBytes;
    static constexpr int LdsBytes = RingBytes + (kBlkMaxD / 32 + kBlkMaxSlices + 4) * 4;
    static_assert(XBytes % (1024 * NW) == 0 && kBlkWBytes % (1024 * NW) == 0, "a stage is moved in whole rounds of the workgroup");
    static_assert(32 * FB * CStride * NW <= RingBytes, "the result tile fits the ring on its way out");
    static_assert(3 * LdsBytes <= 160 * 1024, "three workgroups share a CU");
};

// 64-byte rows, four to a 256-byte line of LDS banks: the 16-byte pieces of row r are permuted by XOR with
// (r / 4) mod 4, so that 16 consecutive rows asked for the same piece fall on 16 different bank groups
__device__ __forceinline__ int blk_swizzle_key(int row) { return (row >> 2) & 3; }

// Is any of the 47 offsets lo, lo+1, ..., lo+46 (mod D) active?  bits: one bit per candidate, D a multiple of 128.
__device__ __forceinline__ bool blk_crossed(const unsigned *bits, int D, int lo)
{
    lo = lo % D;
    if (lo < 0) lo += D;
    const int words = D >> 5;
    int w = lo >> 5;
    const int s = lo & 31;
    const unsigned w0 = bits[w];
    w = w + 1 == words ? 0 : w + 1;
    const unsigned w1 = bits[w];
    w = w + 1 == words ? 0 : w + 1;
    const unsigned w2 = bits[w];
    unsigned long long window = (((unsigned long long)w1 << 32) | w0) >> s;  // 64 - s >= 33 bits
    if (s) window |= (unsigned long long)w2 << (64 - s);
    return (window & ((1ull << 47) - 1)) != 0;
}

// C [T x NC] = A [T x KD] . W, W fragment-major; long_cols: the output columns are the long side of the layer
// (masked gather), else the short side (gather).
template <int FB, int NW>
__global__ __launch_bounds__(64 * NW, 3) void mm_blocks_kernel(int T, int NC, int KD, int D, int K, int long_cols,
                                                                int tiles_m, int tiles_n,
                                                                const int *__restrict__ offsets,
                                                                const uint16_t *__restrict__ A,
                                                                const uint16_t *__restrict__ Wf,
                                                                uint16_t *__restrict__ C)
{
    using Tl = BlkTile<FB, NW>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned *bits = reinterpret_cast<unsigned *>(smem + Tl::RingBytes);  // [D / 32]
    unsigned *slice_list = bits + kBlkMaxD / 32;                           // [KD / 32]: slice | mask << 16
    int *n_list_p = reinterpret_cast<int *>(slice_list + kBlkMaxSlices);

    // Workgroups are dealt round-robin to the eight XCDs; every XCD gets one contiguous run of tiles, column tiles
    // innermost, so that the column tiles of a token block run on one L2 at about the same time.
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + kBlkXcds - 1) / kBlkXcds;
    const int lin = int(blockIdx.x % kBlkXcds) * per_xcd + int(blockIdx.x / kBlkXcds);
    if (lin >= n_tiles) return;
    const int tm = lin / tiles_n, tn = lin % tiles_n;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int n_slices = KD / kBlkSlice;

    // ---- which blocks of this column tile are crossed ----
    for (int i = tid; i < D / 32; i += Tl::THREADS) bits[i] = 0u;
    __syncthreads();
    for (int k = tid; k < K; k += Tl::THREADS) {
        const int o = canonical_offset(offsets[k], D);
        atomicOr(&bits[o >> 5], 1u << (o & 31));
    }
    __syncthreads();
    // slice g, block (a, ks): output columns j0 = 128 tn + 32 a .. +31, contraction indices i0 = 32 g + 16 ks .. +15;
    // long - short index runs over [j0 - i0 - 15, j0 - i0 + 31] (long columns) or [i0 - j0 - 31, i0 - j0 + 15].
    // Wave 0 ranks the slices that hold a crossed block, in order.
    if (wave == 0) {
        int base = 0;
        for (int g0 = 0; g0 < n_slices; g0 += 64) {
            const int g = g0 + lane;
            unsigned mask = 0;
            if (g < n_slices) {
#pragma unroll
                for (int a = 0; a < kBlkFA; ++a)
#pragma unroll
                    for (int ks = 0; ks < kBlkSteps; ++ks) {
                        const int j0 = tn * kBlkBN + a * 32, i0 = g * kBlkSlice + ks * 16;
                        const int lo = long_cols ? j0 - i0 - 15 : i0 - j0 - 31;
                        if (blk_crossed(bits, D, lo)) mask |= 1u << (a * kBlkSteps + ks);
                    }
            }
            const unsigned long long any = __ballot(mask != 0);
            const int rank = __builtin_amdgcn_mbcnt_hi(unsigned(any >> 32), __builtin_amdgcn_mbcnt_lo(unsigned(any), 0u));
            if (mask) slice_list[base + rank] = unsigned(g) | (mask << 16);
            base += __popcll(any);
        }
        if (lane == 0) *n_list_p = base;
    }
    __syncthreads();
    const int n_list = __builtin_amdgcn_readfirstlane(*n_list_p);

    // ---- transfers: memory -> LDS, 1 KB per wave and round ----
    // token rows: round i of wave w moves rows 16 (i NW + w) .. +15 of the tile; lane l lands at row 16j + l/4, 16-byte
    // position l%4, and asks for the piece that the swizzle puts there
    const uint16_t *x_src[Tl::XRounds];
#pragma unroll
    for (int i = 0; i < Tl::XRounds; ++i) {
        const int row = 16 * (i * NW + wave) + (lane >> 2);
        const int piece = (lane & 3) ^ blk_swizzle_key(row);
        int t = tm * Tl::BM + row;
        t = t < T ? t : T - 1;  // rows past the end repeat the last token; their results are not stored
        x_src[i] = A + size_t(t) * KD + piece * 8;
    }
    // operand blocks: round i of wave w moves block b = i NW + w = kBlkSteps a + ks of the slice
    const uint16_t *w_src[Tl::WRounds];
#pragma unroll
    for (int i = 0; i < Tl::WRounds; ++i) {
        const int b = i * NW + wave;
        w_src[i] = Wf + (size_t(tn * kBlkFA + b / kBlkSteps) * (KD / 16) + b % kBlkSteps) * 512 + lane * 8;
    }
    const unsigned lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(blk_zero_piece);
    // entry e_ of the list into stage st_; past the end of the list the same number of transfers is issued (from a
    // block of zeros into a stage nobody reads) so that the count in flight is the same in every iteration
#define DD_BLK_ISSUE(e_, st_)                                                                           \
    {                                                                                                   \
        const bool live = (e_) < n_list;                                                                \
        const unsigned entry = live ? slice_list[(e_)] : 0u;                                            \
        const int g = __builtin_amdgcn_readfirstlane(int(entry & 0xffffu));                             \
        const unsigned mask = __builtin_amdgcn_readfirstlane(entry >> 16);                              \
        _Pragma("unroll") for (int i = 0; i < Tl::XRounds; ++i)                                         \
            global_to_lds_16(live ? x_src[i] + g * kBlkSlice : zero,                                    \
                             lds0 + (st_) * Tl::StageBytes + (i * NW + wave) * 1024);                   \
        _Pragma("unroll") for (int i = 0; i < Tl::WRounds; ++i) {                                       \
            const int b = i * NW + wave;                                                                \
            global_to_lds_16(((mask >> b) & 1u) ? w_src[i] + size_t(g) * kBlkSteps * 512 : zero,        \
                             lds0 + (st_) * Tl::StageBytes + Tl::XBytes + b * 1024);                    \
        }                                                                                               \
    }
#define DD_BLK_ARRIVE(n_) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(n_) : "memory")

    f32x16 acc[kBlkFA][FB];
#pragma unroll
    for (int a = 0; a < kBlkFA; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    int x_frag[FB], x_key[FB];
#pragma unroll
    for (int b = 0; b < FB; ++b) {
        const int row = (wave * FB + b) * 32 + l32;
        x_frag[b] = row * (kBlkSlice * 2);
        x_key[b] = blk_swizzle_key(row);
    }

#pragma unroll
    for (int j = 0; j < kBlkAhead; ++j) DD_BLK_ISSUE(j, j)
    int stage = 0;
    for (int n = 0; n < n_list; ++n) {
        // entry n has landed for every wave (all but the transfers of the entries after it), and every wave is done
        // with entry n - 1, whose stage the next transfers go to
        DD_BLK_ARRIVE((kBlkAhead - 1) * Tl::Rounds);
        const int ahead = stage == 0 ? kBlkRing - 1 : stage - 1;
        DD_BLK_ISSUE(n + kBlkAhead, ahead)
        const unsigned mask = __builtin_amdgcn_readfirstlane(slice_list[n] >> 16);
        const unsigned char *base = smem + stage * Tl::StageBytes;
#pragma unroll
        for (int ks = 0; ks < kBlkSteps; ++ks) {
            if (((mask >> ks) & 0x55u) == 0) continue;
            bf16x8 xf[FB];
#pragma unroll
            for (int b = 0; b < FB; ++b)
                xf[b] = *reinterpret_cast<const bf16x8 *>(base + x_frag[b] + ((((ks << 1) | half) ^ x_key[b]) << 4));
#pragma unroll
            for (int a = 0; a < kBlkFA; ++a) {
                if (!((mask >> (a * kBlkSteps + ks)) & 1u)) continue;
                const bf16x8 wf = *reinterpret_cast<const bf16x8 *>(base + Tl::XBytes + (a * kBlkSteps + ks) * 1024 + lane * 16);
#pragma unroll
                for (int b = 0; b < FB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[b], acc[a][b], 0, 0, 0);
            }
        }
        stage = stage == kBlkRing - 1 ? 0 : stage + 1;
    }
    // the transfers past the end of the list have to land, and every wave has to be done with the stages,
    // before the ring becomes the result's way out
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
#undef DD_BLK_ISSUE
#undef DD_BLK_ARRIVE

    // Accumulator i of lane l is output column 8 (i/4) + 4 (l/32) + i%4 of token l%32 inside its 32 x 32 tile.  Each
    // wave lays its own 32 FB tokens x 128 columns out row by row and stores full-width row segments.
    unsigned char *out = smem + wave * (32 * FB * Tl::CStride);
#pragma unroll
    for (int a = 0; a < kBlkFA; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 v = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
                *reinterpret_cast<bf16x4 *>(out + (b * 32 + l32) * Tl::CStride + (a * 32 + 8 * q + 4 * half) * 2) =
                    __builtin_convertvector(v, bf16x4);
            }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    constexpr int kRowPieces = kBlkBN / 8;  // 16-byte pieces per row
#pragma unroll
    for (int i = 0; i < 32 * FB * kRowPieces / 64; ++i) {
        const int idx = i * 64 + lane;
        const int row = idx / kRowPieces, piece = idx % kRowPieces;
        const int t = tm * Tl::BM + wave * 32 * FB + row;
        if (t < T)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(out + row * Tl::CStride + piece * 16),
                                        reinterpret_cast<u32x4 *>(C + size_t(t) * NC + tn * kBlkBN + piece * 8));
    }
}

bool product_blocks_supported(int64_t T, int D, int L, bool bf16)
{
    return product_matrix_supported(T, D, L, bf16) && D <= kBlkMaxD;
}

template <int FB, int NW>
static hipError_t launch_blocks(const ProductArgs &a, hipStream_t stream)
{
    using Tl = BlkTile<FB, NW>;
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&mm_blocks_kernel<FB, NW>), Tl::LdsBytes, lds_allowed)) return e;
    const int NC = a.masked ? a.D : a.L, KD = a.masked ? a.L : a.D;
    const int T = int(a.T);
    const int tiles_m = (T + Tl::BM - 1) / Tl::BM, tiles_n = NC / kBlkBN;
    const int per_xcd = (tiles_m * tiles_n + kBlkXcds - 1) / kBlkXcds;
    hipLaunchKernelGGL((mm_blocks_kernel<FB, NW>), dim3(per_xcd * kBlkXcds), dim3(Tl::THREADS), Tl::LdsBytes, stream, T, NC,
                       KD, a.D, a.K, a.masked ? 1 : 0, tiles_m, tiles_n, a.offsets, static_cast<const uint16_t *>(a.src),
                       static_cast<const uint16_t *>(a.ws), static_cast<uint16_t *>(a.dst));
    return hipGetLastError();
}

hipError_t launch_product_blocks(const ProductArgs &a, hipStream_t stream)
{
    if (a.src_sets != 1 || a.dst_sets != 1 || !a.prepared || !a.offsets) return hipErrorInvalidValue;
    return launch_blocks<1, 4>(a, stream);
}

}  // namespace dd
