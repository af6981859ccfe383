// Matrix-core path of the weight gradient (bf16 storage, fp32 accumulate), Fig. 3 h-i:
//   dV[k][p] = sum_t A[t, p] * B[t, (p + o_k) mod D],   A [T x L] the short side, B [T x D] the long side.
//
// The sum over tokens of the outer products A[t,:]^T B[t,:] is a contraction with the token index as the
// inner dimension, so it runs on the MFMA units tile by tile; of each finished 32x32 tile only the entries
// whose (column - row) mod D is an active offset are kept.  For the same reason as in the forward product
// (512 bf16 multiply-adds per clock per MFMA pipe against 16 on the vector ALU) this beats visiting only
// the K diagonals down to a density of a few percent, and it reads X and dY exactly as often.
//
//   tile:     192 x 192 (or 128 short-side x 256 long-side) entries of G per workgroup, four waves in a 2 x 2
//             arrangement, over one chunk of tokens; two workgroups share a CU, so that one multiplies while
//             the other waits; chunks are summed afterwards in a fixed order (deterministic).
//   operands: both are stored token-major while the MFMA wants the contraction index contiguous per lane, so
//             16-token k-steps travel from global memory straight into a six-deep ring of LDS stages
//             (global_load_lds, five k-steps ahead, no registers in between) and come back through
//             ds_read_b64_tr_b16, which hands each lane four consecutive tokens of one feature.  Inside a
//             k-step the fragment reads of the next one and the new requests are dealt out between the MFMAs.
//   select:   a table (offset crossing this tile -> first diagonal with that offset) picks the entries of each
//             accumulator tile; repeated offsets read the same partial sums.
#include "dd_common.h"
#include "dd_launch.h"
#include "dd_ring.h"

#include <limits.h>

namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWgT = 256;           // threads
constexpr int kTS = 16;             // tokens per LDS stage: one MFMA k-step
constexpr int kSliceTokens = 32;    // token chunks are made of whole slices of two k-steps
constexpr int kWgRing = 6;          // LDS stages: one being read, up to four on their way, one just released
constexpr int kAhead = 5;           // a stage is requested this many k-steps before it is multiplied
constexpr int kNoDiagonal = INT_MAX;
constexpr int kWgXcds = 8;          // L2 caches (one per XCD); workgroups are dealt to them round-robin
constexpr int kCusPerXcd = 32;
constexpr int kWgPerCu = 2;         // two workgroups share a CU: one multiplies while the other waits for its slice

// What the transfers of short-side rows past the end of a chunk read instead: a zero factor adds nothing.
__device__ __align__(16) const unsigned int wg_zero_piece[4] = {0u, 0u, 0u, 0u};

// Tile of G per workgroup: TP short-side x TQ long-side entries, four waves in a 2 x 2 arrangement.
// A stage holds kTS tokens: first their TP short-side features (row = token), then their TQ long-side ones.
template <int TP, int TQ>
struct WgTile {
    static constexpr int FA = TP / 64;             // 32-row MFMA tiles per wave
    static constexpr int FB = TQ / 64;             // 32-column MFMA tiles per wave
    static constexpr int ARow = TP * 2;            // bytes
    static constexpr int BRow = TQ * 2;
    static constexpr int ABytes = kTS * ARow;
    static constexpr int BBytes = kTS * BRow;
    static constexpr int StageBytes = ABytes + BBytes;
    static constexpr int APieces = ABytes / 16;          // 16-byte pieces of a stage
    static constexpr int Rounds = StageBytes / 16 / kWgT;   // pieces per thread per stage
    static constexpr int Window = TP + TQ;         // offsets (column - row) that cross the tile: Window - 1 of them
    static constexpr int LdsBytes = kWgRing * StageBytes + Window * int(sizeof(int));
    static constexpr int NM = FA * FB;             // MFMAs per k-step
    static constexpr int NF = FA + FB;             // fragments per k-step
    static_assert(TP % 64 == 0 && TQ % 64 == 0, "wave tiles are made of 32x32 MFMA tiles");
    static_assert(StageBytes % (16 * kWgT) == 0, "a stage is moved in whole rounds of the workgroup");
};

// Rows are not padded; instead the 16-byte pieces of row r are permuted by XOR with 2 * (r mod 4), so that
// the four rows one transposing read touches fall on four different 32-byte bank groups.
__device__ __forceinline__ int wg_swizzle(int row) { return (row & 3) << 1; }

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
__global__ __launch_bounds__(kWgT, kWgPerCu) void wgrad_mm_kernel(int T, int D, int L, int K, int tiles_p,
                                                                  int tiles_q, int splits, int slices, int skew,
                                                                  const uint16_t *__restrict__ A,
                                                                  const uint16_t *__restrict__ B,
                                                                  const int *__restrict__ offsets,
                                                                  float *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using Tl = WgTile<TP, TQ>;
    constexpr int kARow = Tl::ARow, kBRow = Tl::BRow, kABytes = Tl::ABytes, kStageBytes = Tl::StageBytes;
    int *table = reinterpret_cast<int *>(smem + kWgRing * kStageBytes);  // [Window]: offset -> first diagonal
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Every kernel argument is brought into registers now: a scalar load still pending inside the main loop
    // would force each wait for LDS data to wait for everything outstanding.
    asm volatile("" ::"s"(partial), "s"(offsets), "s"(A), "s"(B), "s"(K), "s"(L));
    // Token chunks are dealt to the XCDs: every tile of one chunk runs on the same L2, so the chunk's
    // slices of X and dY come from HBM once and from that L2 for every other tile -- as long as the tiles that
    // share a slice walk the chunk together.  Of the two workgroups on a CU the one dispatched first gets ahead
    // of the other, so an XCD's first 32 workgroups and its next 32 drift apart by more tokens than the L2
    // holds.  Tiles are therefore numbered along the short side first: the tiles_p workgroups that share a
    // column tile of the long-side matrix (the bulk of the bytes) are neighbours, and only the short-side
    // matrix is fetched once per half (measured on 768 <-> 3072 at 50432 tokens: 476 MB from memory per launch
    // against 684 MB with the long side first; 388 MB is each byte once).
    const int tiles = tiles_p * tiles_q;
    const int xcd = blockIdx.x % kWgXcds, local = blockIdx.x / kWgXcds;
    const int split = (local / tiles) * kWgXcds + xcd;
    if (split >= splits) return;
    const int tile = local % tiles;
    // The two workgroups of a CU (an XCD's workgroup i and i + 32) take turns at the higher wave priority, k-step by
    // k-step.  Left alone the one dispatched first stays ahead and the two halves of the XCD drift apart by more
    // tokens than the L2 holds, so that what they share is fetched twice (768 <-> 3072 at 50432 tokens: 476 MB per
    // launch; taking turns: 388 MB, each byte once, and 1 % less time).  Only for the 192 x 192 tile: the 128 x 256
    // tile of the shapes that 192 does not divide fetches less this way too (1024 <-> 4096: 397 -> 310 MB) but
    // runs 3 % longer.
    constexpr bool kTakeTurns = TP == 192 && TQ == 192;
    const bool second = (local >> 5) & 1;
    const int p0 = (tile % tiles_p) * TP, q0 = (tile / tiles_p) * TQ;
    // Chunk `split` owns the 32-token slices [begin(split), begin(split + 1)), begin(s) = s * slices / splits
    // + skew * (2 min(s, splits / 2) - s): the chunks of the first half of the workgroups are `skew` slices longer
    // than an even share, those of the second half as much shorter (skew = 0: even shares).
    const int half_splits = splits / 2;
    const int slice_begin = int(int64_t(split) * slices / splits) + skew * (2 * min(split, half_splits) - split);
    const int slice_end =
        int(int64_t(split + 1) * slices / splits) + skew * (2 * min(split + 1, half_splits) - (split + 1));
    const int t_begin = slice_begin * kSliceTokens;
    const int t_end = min(slice_end * kSliceTokens, T);
    const int n_steps = (slice_end - slice_begin) * (kSliceTokens / kTS);  // even, at least 2

    // Memory -> LDS without passing through registers: in round i the workgroup moves pieces
    // [i * 256, i * 256 + 256) of the stage, each wave a contiguous kilobyte (lane l lands at +16 l).
    // Which piece of global memory a lane asks for is what realises the swizzle.
    const uint16_t *src_col[Tl::Rounds];  // column part of the address
    int src_row[Tl::Rounds];              // token of the piece in k-step 0
    int src_ld[Tl::Rounds];               // row pitch of the matrix the piece comes from
#pragma unroll
    for (int i = 0; i < Tl::Rounds; ++i) {
        const int piece_all = i * kWgT + tid;
        const bool is_a = piece_all < Tl::APieces;
        const int piece = is_a ? piece_all : piece_all - Tl::APieces;
        const int per_row = (is_a ? TP : TQ) / 8;
        const int row = piece / per_row, pos = piece % per_row;
        const int col = (pos ^ wg_swizzle(row)) * 8;
        src_col[i] = is_a ? A + p0 + col : B + q0 + col;
        src_row[i] = t_begin + row;
        src_ld[i] = is_a ? L : D;
    }
    const unsigned lds_stage0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * 1024);
    // Rows past the end of the chunk must add nothing: their pieces come from a block of zeros instead.  The
    // same holds for whole k-steps past the end, which are requested like any other so that the count of
    // transfers in flight is the same in every iteration.
#define DD_WG_ISSUE_PIECE(i_, s_, stage_)                                                                \
    {                                                                                                   \
        const int t = src_row[i_] + (s_) * kTS;                                                         \
        const uint16_t *g = src_col[i_] + size_t(t) * size_t(src_ld[i_]);                               \
        if (t >= t_end) g = reinterpret_cast<const uint16_t *>(wg_zero_piece);                          \
        global_to_lds_16(g, lds_stage0 + (stage_) * kStageBytes + (i_) * (kWgT * 16));                  \
    }
#define DD_WG_ISSUE(s_, stage_)                                                                          \
    _Pragma("unroll") for (int i = 0; i < Tl::Rounds; ++i) DD_WG_ISSUE_PIECE(i, s_, stage_)
    // The k-steps that lie wholly inside the chunk -- all but the last few -- need neither the row test nor the
    // multiplication: every piece comes 16 rows after the piece of the k-step before (run[] is where the next one starts).
    const uint16_t *run[Tl::Rounds];
#pragma unroll
    for (int i = 0; i < Tl::Rounds; ++i) run[i] = src_col[i] + size_t(src_row[i] + kAhead * kTS) * size_t(src_ld[i]);
#define DD_WG_ISSUE_PIECE_INSIDE(i_, s_, stage_)                                                         \
    {                                                                                                   \
        global_to_lds_16(run[i_], lds_stage0 + (stage_) * kStageBytes + (i_) * (kWgT * 16));            \
        run[i_] += size_t(kTS) * size_t(src_ld[i_]);                                                    \
    }
    // all but the newest `n_` of this wave's transfers have landed; then the same for the whole workgroup
#define DD_WG_ARRIVE(n_) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(n_) : "memory")
#define DD_WG_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

    // Fragment addressing.  In a group of 16 lanes, lane s supplies row s/4 (a token) and features
    // 4*(s%4)..+3; it receives feature s of the group for those four tokens.  Groups 0,1 cover features
    // 0-15 / 16-31 of the first 8 tokens of a k-step, groups 2,3 the same features of the last 8.
    const int s16 = lane & 15, grp = lane >> 4;
    const int frag_row = (grp >> 1) * 8 + (s16 >> 2);     // and frag_row + 4; both have row mod 4 = s16 / 4
    const int frag_col = (grp & 1) * 16 + (s16 & 3) * 4;
    const int wp = wave >> 1, wq = wave & 1;     // wave tile: rows wp*TP/2.., columns wq*TQ/2..
    int a_frag[Tl::FA], b_frag[Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a) {
        const int col = wp * (TP / 2) + a * 32 + frag_col;
        a_frag[a] = frag_row * kARow + (((col >> 3) ^ wg_swizzle(frag_row)) << 4) + (col & 7) * 2;
    }
#pragma unroll
    for (int b = 0; b < Tl::FB; ++b) {
        const int col = wq * (TQ / 2) + b * 32 + frag_col;
        b_frag[b] = kABytes + frag_row * kBRow + (((col >> 3) ^ wg_swizzle(frag_row)) << 4) + (col & 7) * 2;
    }

    f32x16 acc[Tl::FA][Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

#define DD_WG_FRAGS(fa_, fb_, base_)                                                                \
    {                                                                                                   \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a) {                                            \
            const unsigned char *p = (base_) + a_frag[a];                                               \
            fa_[a] = read_transposed(p, p + 4 * kARow);                                                 \
        }                                                                                               \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b) {                                            \
            const unsigned char *p = (base_) + b_frag[b];                                               \
            fb_[b] = read_transposed(p, p + 4 * kBRow);                                                 \
        }                                                                                               \
    }
#define DD_WG_MFMA(fa_, fb_)                                                                            \
    _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                                  \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                              \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[a], fb_[b], acc[a][b], 0, 0, 0);
    bf16x8 fa0[Tl::FA], fb0[Tl::FB], fa1[Tl::FA], fb1[Tl::FB];

    // The offsets are requested before the token slices and looked at after the main loop.
    const int window_base = q0 - p0 - TP + 1;
    constexpr int kMaxOwn = 4;
    int own[kMaxOwn];
#pragma unroll
    for (int j = 0; j < kMaxOwn; ++j) {
        const int k = tid + j * kWgT;
        own[j] = k < K ? offsets[k] : 0;
    }
    // k-step j_: wait until j_+1 has landed for every wave (every wave is then also done with j_-1, whose
    // stage is requested for j_+kAhead), and multiply the fragments of j_.  The fragment reads of j_+1 and
    // the new requests are dealt out one after each MFMA, so that they issue while the matrix pipe is busy.
#define DD_WG_STEP(j_, cur_a_, cur_b_, nxt_a_, nxt_b_, PIECE_)                                           \
    {                                                                                                   \
        const int next_stage = stage == kWgRing - 1 ? 0 : stage + 1;                                    \
        const int ahead = stage == 0 ? kWgRing - 1 : stage - 1; /* (stage + kAhead) mod kWgRing */      \
        DD_WG_STEP_BODY(j_, cur_a_, cur_b_, nxt_a_, nxt_b_, PIECE_)                                     \
        stage = next_stage;                                                                             \
    }
    // a k-step in stage STAGE_, a number the compiler knows: stage addresses become instruction offsets
#define DD_WG_STEP_FIXED(j_, cur_a_, cur_b_, nxt_a_, nxt_b_, STAGE_)                                     \
    {                                                                                                   \
        constexpr int next_stage = ((STAGE_) + 1) % kWgRing, ahead = ((STAGE_) + kAhead) % kWgRing;     \
        if constexpr (kTakeTurns) {                                                                     \
            if ((((STAGE_) & 1) != 0) == second) asm volatile("s_setprio 1"); else asm volatile("s_setprio 0"); \
        }                                                                                               \
        DD_WG_STEP_BODY(j_, cur_a_, cur_b_, nxt_a_, nxt_b_, DD_WG_ISSUE_PIECE_INSIDE)                    \
    }
#define DD_WG_STEP_BODY(j_, cur_a_, cur_b_, nxt_a_, nxt_b_, PIECE_)                                      \
    {                                                                                                   \
        DD_WG_ARRIVE((kAhead - 2) * Tl::Rounds);                                                        \
        const unsigned char *base = smem + next_stage * kStageBytes;                                    \
        _Pragma("unroll") for (int m = 0; m < Tl::NM; ++m) {                                            \
            const int a = kOrder.mfma_a[m], b = kOrder.mfma_b[m];                                       \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur_a_[a], cur_b_[b], acc[a][b], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0);                                                          \
            _Pragma("unroll") for (int k = 0; k < Tl::NF + Tl::Rounds; ++k) {                           \
                if ((k < Tl::NM ? k : Tl::NM - 1) != m) continue;                                       \
                if (k < Tl::NF) {                                                                       \
                    const int f = kOrder.frag_idx[k];                                                   \
                    if (kOrder.frag_is_a[k]) {                                                          \
                        const unsigned char *p = base + a_frag[f];                                      \
                        nxt_a_[f] = read_transposed(p, p + 4 * kARow);                                  \
                    } else {                                                                            \
                        const unsigned char *p = base + b_frag[f];                                      \
                        nxt_b_[f] = read_transposed(p, p + 4 * kBRow);                                  \
                    }                                                                                   \
                } else {                                                                                \
                    PIECE_(k - Tl::NF, (j_) + kAhead, ahead)                                            \
                }                                                                                       \
            }                                                                                           \
            __builtin_amdgcn_sched_barrier(0);                                                          \
        }                                                                                               \
    }
    static_assert(kAhead == kWgRing - 1, "the stage requested at k-step j is the one k-step j-1 has just left");
    static_assert(kWgRing == 6, "the loop over whole turns of the ring names its six stages");
    constexpr WgOrder<Tl::FA, Tl::FB> kOrder{};
#pragma unroll
    for (int j = 0; j < kAhead; ++j) DD_WG_ISSUE(j, j)
    for (int i = tid; i < Tl::Window; i += kWgT) table[i] = kNoDiagonal;  // filled in after the main loop
    DD_WG_ARRIVE((kAhead - 1) * Tl::Rounds);
    DD_WG_FRAGS(fa0, fb0, smem)
    int stage = 0;
    int j = 0;
    // k-steps whose requests (kAhead further on) lie wholly inside the chunk, two at a time
    const int inside = min((t_end - t_begin) / kTS - kAhead, n_steps - 2);
    for (; j + kWgRing <= inside; j += kWgRing) {  // one turn of the ring: `stage` is 0 before and after
        DD_WG_STEP_FIXED(j, fa0, fb0, fa1, fb1, 0)
        DD_WG_STEP_FIXED(j + 1, fa1, fb1, fa0, fb0, 1)
        DD_WG_STEP_FIXED(j + 2, fa0, fb0, fa1, fb1, 2)
        DD_WG_STEP_FIXED(j + 3, fa1, fb1, fa0, fb0, 3)
        DD_WG_STEP_FIXED(j + 4, fa0, fb0, fa1, fb1, 4)
        DD_WG_STEP_FIXED(j + 5, fa1, fb1, fa0, fb0, 5)
    }
    if constexpr (kTakeTurns) asm volatile("s_setprio 0");
    for (; j + 2 <= inside; j += 2) {
        DD_WG_STEP(j, fa0, fb0, fa1, fb1, DD_WG_ISSUE_PIECE_INSIDE)
        DD_WG_STEP(j + 1, fa1, fb1, fa0, fb0, DD_WG_ISSUE_PIECE_INSIDE)
    }
    for (; j < n_steps - 2; j += 2) {
        DD_WG_STEP(j, fa0, fb0, fa1, fb1, DD_WG_ISSUE_PIECE)
        DD_WG_STEP(j + 1, fa1, fb1, fa0, fb0, DD_WG_ISSUE_PIECE)
    }
    DD_WG_STEP(j, fa0, fb0, fa1, fb1, DD_WG_ISSUE_PIECE)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the requests past the end have to land before the stages are reused
    DD_WG_MFMA(fa1, fb1)
#undef DD_WG_STEP
#undef DD_WG_STEP_FIXED
#undef DD_WG_STEP_BODY
    // The table of the offsets that cross this tile: entry e stands for (column - row) = q0 - p0 - TP + 1 + e
    // (mod D) and holds the first diagonal with that offset.  (Cleared before the main loop; the barriers of
    // the loop lie between.)
#define DD_WG_ENTER(o_, k_)                                                                              \
    {                                                                                                   \
        int e = canonical_offset(o_, D) - window_base;                                                  \
        e = e < 0 ? e + D : (e >= D ? e - D : e);                                                       \
        if (e < Tl::Window - 1) atomicMin(&table[e], k_);                                               \
    }
#pragma unroll
    for (int j = 0; j < kMaxOwn; ++j)
        if (tid + j * kWgT < K) DD_WG_ENTER(own[j], tid + j * kWgT)
    for (int k = tid + kMaxOwn * kWgT; k < K; k += kWgT) DD_WG_ENTER(offsets[k], k)
#undef DD_WG_ENTER
    DD_WG_LDS_BARRIER();  // the table is complete and every wave is done with the stages: they become tile buffers
#undef DD_WG_ISSUE
#undef DD_WG_ISSUE_PIECE_INSIDE
#undef DD_WG_ARRIVE
#undef DD_WG_FRAGS
#undef DD_WG_MFMA

    // Keep the entries on active diagonals.  Accumulator i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column
    // l%32 of its 32x32 tile.  Tiles are handled three at a time to overlap their LDS round trips: each is
    // laid out column-major in a buffer of the wave's own; the 63 offsets that cross it were looked up in the
    // table (one per lane) and the active ones are compacted into a list; then eight diagonals are read back
    // at once along the diagonal -- lane = (list slot, row mod 8) -- and leave as 32-byte runs of partial sums.
    constexpr int kTileStride = 36;  // floats per tile column: 16-byte aligned rows of four, odd diagonal stride
    constexpr int kTileFloats = 32 * kTileStride;
    constexpr int kTilesPerWave = Tl::FA * Tl::FB;
    constexpr int kWaveBytes = kWgRing * kStageBytes / 4;
    constexpr int kRoom = (kWaveBytes - kTilesPerWave * 64 * 4) / (kTileFloats * 4);  // tile buffers beside the lists
    constexpr int kGroup = kRoom < 3 ? kRoom : 3;
    static_assert(kGroup >= 1, "at least one accumulator tile at a time");
    static_assert(kGroup * kTileFloats * 4 + kTilesPerWave * 64 * 4 <= kWaveBytes, "tile buffers and lists fit the wave's share of the stages");
    float *tilebuf = reinterpret_cast<float *>(smem + wave * kWaveBytes);                 // [kGroup][32 x 36]
    int *lists = reinterpret_cast<int *>(smem + wave * kWaveBytes) + kGroup * kTileFloats;  // [tiles][64]
    float *out = partial + size_t(split) * K * L;
    const int l32 = lane & 31, half = lane >> 5;
    const int slot = lane >> 3, rmod = lane & 7;
    // lane j < 63 of tile t: first diagonal with (column - row) = j - 31, if any; the active ones are ranked
    // and entered into the tile's list as (diagonal << 6 | j)
    int n_active[kTilesPerWave], kj[kTilesPerWave];
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const int pl = wp * (TP / 2) + (t / Tl::FB) * 32, ql = wq * (TQ / 2) + (t % Tl::FB) * 32;
        int e = ql - pl + lane - 31 + TP - 1;  // in [0, Window - 1]
        e = e >= D ? e - D : e;                // a window wider than D wraps onto itself
        kj[t] = table[e];
    }
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const bool mine = kj[t] != kNoDiagonal && lane < 63;
        const unsigned long long active = __ballot(mine);
        n_active[t] = __popcll(active);
        const int rank = __builtin_amdgcn_mbcnt_hi(unsigned(active >> 32), __builtin_amdgcn_mbcnt_lo(unsigned(active), 0u));
        lists[t * 64 + (mine ? rank : 63)] = (kj[t] << 6) | lane;  // at most 63 are active: slot 63 takes the rest
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int entry[kTilesPerWave];
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) entry[t] = lists[t * 64 + slot];
    // Values of list entry e_ of the tile in buffer g_ on rows rmod + 8 i.  col_ = row + (column - row) of the
    // entry, or something far outside the tile when the lane's list slot is empty; the read itself is always
    // in bounds (column clamped), the store is predicated on the column being inside the tile.
#define DD_WG_DIAG_LOAD(v_, col_, g_, e_, have_)                                                         \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                     \
        col_[i] = unsigned(rmod + 8 * i + ((have_) ? ((e_) & 63) - 31 : 64));                           \
        v_[i] = tilebuf[(g_) * kTileFloats + int(min(col_[i], 31u)) * kTileStride + rmod + 8 * i];      \
    }
#define DD_WG_DIAG_STORE(v_, col_, t_, e_)                                                               \
    {                                                                                                   \
        const unsigned byte0 = (unsigned((e_) >> 6) * unsigned(L) + unsigned(p0 + wp * (TP / 2) + ((t_) / Tl::FB) * 32 + rmod)) * 4u; \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                   \
            if (col_[i] < 32u)                                                         \
                *reinterpret_cast<float *>(reinterpret_cast<char *>(out) + (byte0 + 32u * i)) = v_[i];  \
    }
#pragma unroll
    for (int t0 = 0; t0 < kTilesPerWave; t0 += kGroup) {
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            const int t = t0 + g;
            if (t < kTilesPerWave) {
                const int a = t / Tl::FB, b = t % Tl::FB;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
                    *reinterpret_cast<f32x4 *>(tilebuf + g * kTileFloats + l32 * kTileStride + 8 * q + 4 * half) = v;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float v[kGroup][4];
        unsigned col[kGroup][4];
#pragma unroll
        for (int g = 0; g < kGroup; ++g)
            if (t0 + g < kTilesPerWave) DD_WG_DIAG_LOAD(v[g], col[g], g, entry[t0 + g], slot < n_active[t0 + g])
#pragma unroll
        for (int g = 0; g < kGroup; ++g)
            if (t0 + g < kTilesPerWave) DD_WG_DIAG_STORE(v[g], col[g], t0 + g, entry[t0 + g])
#pragma unroll
        for (int g = 0; g < kGroup; ++g)  // more than eight diagonals across one tile: rare at the paper's sparsities
            if (t0 + g < kTilesPerWave)
                for (int first = 8; first < n_active[t0 + g]; first += 8) {
                    const int e = lists[(t0 + g) * 64 + ((first + slot) & 63)];
                    DD_WG_DIAG_LOAD(v[g], col[g], g, e, first + slot < n_active[t0 + g])
                    DD_WG_DIAG_STORE(v[g], col[g], t0 + g, e)
                }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
#undef DD_WG_DIAG_LOAD
#undef DD_WG_DIAG_STORE
}

// dV[k][p] = sum over the chunks of partial[chunk][rep(k)][p], rep(k) = first diagonal with k's offset.  The
// chunks are cut into four runs that four groups of threads add up side by side, each in chunk order; the four
// sums are then added in run order: a fixed order, so the result is the same on every call.
// Repeated offsets are rare, so the first eight partial sums of diagonal k itself are requested before the search
// for rep(k) (whose loads and barriers they then overlap) and fetched again only if k turns out not to be first.
//
// SCALED: the adjoint of the scaling by the importance weights (Sec. 3.2 Eq. 4) as the epilogue: the sum g = dValues[k][p]
// leaves as alpha[o_k] * g, and <dValues[k], V[k]> is summed per workgroup into dots[k][blockIdx.x] (fixed order);
// wgrad_dalpha_kernel turns the dots into the gradient of the importance weights.
template <bool SCALED>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(int D, int L, int K, int splits,
                                                           const int *__restrict__ offsets,
                                                           const float *__restrict__ partial,
                                                           float *__restrict__ dV, const float *__restrict__ alpha,
                                                           const uint16_t *__restrict__ V, float *__restrict__ dots)
{
    __shared__ int rep_s;
    __shared__ f32x4 run_s[3][64];
    const int k = blockIdx.y;
    const int run = threadIdx.x >> 6, g = threadIdx.x & 63;
    const int p = blockIdx.x * 256 + g * 4;  // L is a multiple of 64
    const int per_run = (splits + 3) / 4;
    const int s_begin = min(run * per_run, splits), s_end = min(s_begin + per_run, splits);
    const size_t stride = size_t(K) * L;
    const bool active = p < L;
    const bool first_batch = active && s_begin + 8 <= s_end;
    f32x4 v[8];
    if (first_batch) {
        const float *src = partial + (size_t(s_begin) * K + k) * L + p;
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4 *>(src + u * stride);
    }

    if (threadIdx.x == 0) rep_s = k;
    __syncthreads();
    const int mine = canonical_offset(offsets[k], D);
    for (int j = threadIdx.x; j < k; j += 256)
        if (canonical_offset(offsets[j], D) == mine) atomicMin(&rep_s, j);
    __syncthreads();
    const int rep = rep_s;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (active) {
        const float *src = partial + (size_t(s_begin) * K + rep) * L + p;
        int s = s_begin;
        if (first_batch) {
            if (rep != k) {  // uniform over the workgroup
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4 *>(src + u * stride);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
            src += 8 * stride;
            s += 8;
        }
        for (; s + 8 <= s_end; s += 8) {  // eight loads in flight
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4 *>(src + u * stride);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
            src += 8 * stride;
        }
        for (; s < s_end; ++s) {
            acc += *reinterpret_cast<const f32x4 *>(src);
            src += stride;
        }
    }
    if (run > 0) run_s[run - 1][g] = acc;
    __syncthreads();
    if (run == 0 && active) acc = ((acc + run_s[0][g]) + run_s[1][g]) + run_s[2][g];
    if (!SCALED) {
        if (run == 0 && active) *reinterpret_cast<f32x4 *>(dV + size_t(k) * L + p) = acc;
        return;
    }
    if (run == 0) {  // exactly the first wave
        float dot = 0.f;
        if (active) {
            const uint16_t *v = V + size_t(k) * L + p;
            dot = fmaf(acc[3], bf16_to_f32(v[3]), fmaf(acc[2], bf16_to_f32(v[2]), fmaf(acc[1], bf16_to_f32(v[1]), acc[0] * bf16_to_f32(v[0]))));
            const float a = alpha[mine];
            const f32x4 scaled = {a * acc[0], a * acc[1], a * acc[2], a * acc[3]};
            *reinterpret_cast<f32x4 *>(dV + size_t(k) * L + p) = scaled;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) dot += __shfl_xor(dot, d, 64);
        if (g == 0) dots[size_t(k) * gridDim.x + blockIdx.x] = dot;
    }
}

// dalpha[i] = sum over the diagonals k with offset i of (dots[k][0] + dots[k][1] + ...), 0 for candidates without a
// diagonal.  One workgroup: the D sums are formed in LDS (one addition per diagonal; an offset given twice gets both
// dots -- a sum of two is the same in either order, only an offset given three times or more sees an unspecified order
// of fp32 additions) and written out once.
__global__ __launch_bounds__(256) void wgrad_dalpha_kernel(int D, int K, int per_k, const int *__restrict__ offsets,
                                                           const float *__restrict__ dots, float *__restrict__ dalpha)
{
    extern __shared__ float sums[];  // [D]
    for (int i = threadIdx.x; i < D; i += 256) sums[i] = 0.f;
    __syncthreads();
    for (int j = threadIdx.x; j < K; j += 256) {
        float sum = 0.f;
        for (int b = 0; b < per_k; ++b) sum += dots[size_t(j) * per_k + b];
        atomicAdd(&sums[canonical_offset(offsets[j], D)], sum);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < D; i += 256) dalpha[i] = sums[i];
}

// ---- host side ----

struct WgradPlan {
    int tp, tq;            // tile
    int tiles_p, tiles_q;
    int splits;            // token chunks (a multiple of the XCD count unless T is tiny)
    int slices;            // T in units of 32 tokens
    int skew;              // slices moved from each chunk of the second half of the workgroups to one of the first
    int grid;
};

static WgradPlan plan_wgrad(int64_t T, int D, int L)
{
    WgradPlan pl;
    // 192 x 192 tiles keep the four waves square (96 x 96) and divide the ViT-Base widths; otherwise 128 x 256,
    // and 128 x 128 where the long side is no multiple of 256
    if (L % 192 == 0 && D % 192 == 0) { pl.tp = 192; pl.tq = 192; }
    else if (D % 256 == 0) { pl.tp = 128; pl.tq = 256; }
    else { pl.tp = 128; pl.tq = 128; }
    pl.tiles_p = L / pl.tp;
    pl.tiles_q = D / pl.tq;
    const int tiles = pl.tiles_p * pl.tiles_q;
    // chunks per XCD: as many as fill its 32 CUs in one round
    int per_xcd = kCusPerXcd * kWgPerCu / tiles;
    if (per_xcd < 1) per_xcd = 1;
    int64_t splits = int64_t(per_xcd) * kWgXcds;
    const int64_t slices = (T + kSliceTokens - 1) / kSliceTokens;
    if (splits > slices) splits = slices;
    pl.slices = int(slices);
    pl.splits = int(splits);
    const int rounds = (pl.splits + kWgXcds - 1) / kWgXcds;
    pl.grid = rounds * tiles * kWgXcds;
    // When the grid is exactly the two workgroups per CU that fit, the second 256 get their first tokens about
    // 1.5 us after the first 256 (the burst of first requests is served in order) and would finish their main
    // loops as much later, alone on their CUs next to the first ones' epilogues.  Giving them two slices (four
    // k-steps) less and the first ones two more lets both loops end together (measured on the ViT-Base attention
    // layer: between 0.2 and 0.7 us of 22, box by box).  The split is a fixed function of the shape, so results stay reproducible.
    // (Workgroup b works on chunk (b / 8 / tiles) * 8 + b % 8: with an even number of chunks per XCD the first 256
    // workgroups are exactly the first half of the chunks.)
    pl.skew = (pl.grid == 256 * kWgPerCu && per_xcd % 2 == 0 && splits == int64_t(per_xcd) * kWgXcds &&
               slices / splits >= 8) ? 2 : 0;
    return pl;
}

bool weight_grad_matrix_supported(int64_t T, int D, int L, bool bf16)
{
    if (!(bf16 && T > 0 && T < (int64_t(1) << 31) && D <= 8192)) return false;
    return (L % 192 == 0 && D % 192 == 0) || (L % 128 == 0 && D % 128 == 0);
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
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&wgrad_mm_kernel<TP, TQ>), Tl::LdsBytes, lds_allowed)) return e;
    const int lds_bytes = Tl::LdsBytes;
    hipLaunchKernelGGL((wgrad_mm_kernel<TP, TQ>), dim3(pl.grid), dim3(kWgT), lds_bytes, stream, int(a.T), a.D, a.L,
                       a.K, pl.tiles_p, pl.tiles_q, pl.splits, pl.slices, pl.skew,
                       static_cast<const uint16_t *>(a.A), static_cast<const uint16_t *>(a.B), a.offsets, partial);
    return hipGetLastError();
}

static hipError_t launch_wgrad_mm_any(const WeightGradArgs &a, const WgradPlan &pl, float *partial, hipStream_t stream)
{
    return pl.tp == 192   ? launch_wgrad_mm<192, 192>(a, pl, partial, stream)
           : pl.tq == 256 ? launch_wgrad_mm<128, 256>(a, pl, partial, stream)
                          : launch_wgrad_mm<128, 128>(a, pl, partial, stream);
}

hipError_t launch_weight_grad_matrix(const WeightGradArgs &a, hipStream_t stream)
{
    const WgradPlan pl = plan_wgrad(a.T, a.D, a.L);
    float *partial = static_cast<float *>(a.ws);
    if (hipError_t e = launch_wgrad_mm_any(a, pl, partial, stream)) return e;
    hipLaunchKernelGGL(wgrad_reduce_kernel<false>, dim3((a.L + 255) / 256, a.K), dim3(256), 0, stream, a.D, a.L, a.K,
                       pl.splits, a.offsets, partial, a.dValues, static_cast<const float *>(nullptr),
                       static_cast<const uint16_t *>(nullptr), static_cast<float *>(nullptr));
    return hipGetLastError();
}

// tail: [K x ceil(L / 256)] dots
size_t weight_grad_scaled_tail_bytes(int L, int K)
{
    return (size_t(K) * ((L + 255) / 256) * sizeof(float) + 255) / 256 * 256;
}

hipError_t launch_weight_grad_matrix_scaled(const WeightGradArgs &a, const float *alpha, const void *V, float *dalpha,
                                            void *tail, hipStream_t stream)
{
    const WgradPlan pl = plan_wgrad(a.T, a.D, a.L);
    float *partial = static_cast<float *>(a.ws);
    float *dots = static_cast<float *>(tail);
    const int per_k = (a.L + 255) / 256;
    if (hipError_t e = launch_wgrad_mm_any(a, pl, partial, stream)) return e;
    hipLaunchKernelGGL(wgrad_reduce_kernel<true>, dim3(per_k, a.K), dim3(256), 0, stream, a.D, a.L, a.K, pl.splits,
                       a.offsets, partial, a.dValues, alpha, static_cast<const uint16_t *>(V), dots);
    if (hipError_t e = hipGetLastError()) return e;
    hipLaunchKernelGGL(wgrad_dalpha_kernel, dim3(1), dim3(256), size_t(a.D) * sizeof(float), stream, a.D, a.K, per_k,
                       a.offsets, dots, dalpha);
    return hipGetLastError();
}

}  // namespace dd
