// Matrix-core path of the forward and backward-input products (bf16 storage, fp32 accumulate).
//
// On gfx950 one MFMA pipe retires 512 bf16 multiply-adds per clock against 16 fp32 FMAs on the
// vector ALU of the same SIMD, so down to a density K/D of a few percent it is faster to rebuild
// the K diagonals as a dense operand and run the product as a tiled contraction than to visit
// only the K*L stored weights on the vector ALUs.  HBM traffic is the same either way: X is read
// once, Y written once; the dense operand (<= a few MB) lives in L2.
//
// Step 1 (materialize_kernel): the dense operand is written from (offsets, values) following
//   Sec. 3.1 Eq. 1-3 / Appendix A, directly in the register layout of the MFMA "A" operand:
//   a block of 32 output columns x 16 contraction indices is 1 KB, lane-major, so a wave fetches
//   a fragment with one fully coalesced 16-byte-per-lane load and the operand never touches LDS.
// Step 2 (mm_kernel): C [T x NC] = A [T x KD] . W with v_mfma_f32_32x32x16_bf16.  A workgroup of
//   NW waves (eight by default: two per SIMD, so that one wave's waits hide behind the other's
//   MFMAs) owns a BM x BN tile of C; each wave owns BN/NW output columns (its weight fragments
//   are private, loaded global -> registers one k-slice ahead) and all BM tokens.  All waves run in
//   step from barrier to barrier, so every other instruction of a k-slice (fragment reads, weight
//   loads, token pieces to LDS, new requests) is dealt out between the MFMAs instead of in phases.  The token
//   operand is shared by all waves and goes through a three-deep LDS ring in 64-wide k-slices,
//   XOR-swizzled in 16-byte chunks so that fragment reads are free of bank conflicts.
//   The MFMA rows are output columns and the MFMA columns are tokens, which leaves every lane
//   with four consecutive output columns of one token, so the tile is transposed back through
//   LDS once and stored with full-width row segments.
#include "dd_common.h"
#include "dd_launch.h"
#include "dd_select_block.h"

namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;           // contraction extent of one LDS stage: 64 bf16 = 128 bytes per row
constexpr int kChunksPerRow = kBK / 8;  // 16-byte chunks per LDS row
constexpr int kRowBytes = kBK * 2;
constexpr int kXcds = 8;
constexpr int kRing = 3;         // LDS stages of the token operand
constexpr int kFusedRows = 3;    // operand rows per workgroup of select_materialize_kernel

// position of 16-byte chunk `chunk` (0..7) inside its 128-byte row
__device__ __forceinline__ int swizzle_key(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swizzle(int row, int chunk) { return chunk ^ swizzle_key(row); }

// Fragment-major layout of the dense operand: element (output column j, contraction index i) of a
// matrix with KD contraction indices.  Block (j / 32, i / 16) holds 64 lanes x 8 elements; lane
// (j % 32) + 32 * ((i % 16) / 8) holds elements i % 8 -- the operand layout of the 32x32x16 MFMA.
__device__ __forceinline__ size_t fragment_index(int j, int i, int KD)
{
    return ((size_t(j >> 5) * (KD >> 4) + (i >> 4)) * 64 + (j & 31) + 32 * ((i >> 3) & 1)) * 8 + (i & 7);
}

// Eight floats rounded to bf16 (nearest even, the hardware's conversion) as one 16-byte piece.
__device__ __forceinline__ u32x4 pack_bf16x8(f32x4 lo, f32x4 hi)
{
    union {
        bf16x4 h[2];
        u32x4 w;
    } u;
    u.h[0] = __builtin_convertvector(lo, bf16x4);
    u.h[1] = __builtin_convertvector(hi, bf16x4);
    return u.w;
}

struct OperandPlace {
    int kd_total, col_step, k_step;
    size_t block_step;  // elements from one set's operand to the next where every set has an operand of its own
};

// ---------------------------------------------------------------------------------------------
// Step 1: dense operand from the diagonals.  Operand row r belongs to output column r of the product:
//   masked gather:  row r = q in [0, D), KD = L:  w[p] = sum_{k: (q - o_k) mod D = p < L} v_k[p]
//   gather:         row r = p in [0, L), KD = D:  w[q] = sum_{k: (p + o_k) mod D = q} v_k[p]
// A workgroup builds kMatRows = 32 consecutive rows over kMatRange consecutive contraction indices -- one run of
// whole fragments, contiguous in the fragment-major layout, so that it leaves in full 16-byte-per-lane stores
// (a workgroup per row would write its 16-byte pieces 512 bytes apart, every one a partial line).
// blockIdx.x numbers the (block of 32 rows, range of contraction indices) pairs, ranges innermost: first those of
// the `masked_blocks` blocks of the masked-gather operand, then those of the gather operand (either count may be
// zero).  Entries are summed in fp32 in LDS (repeated offsets add,
// Eq. 3) and rounded to bf16 once.  alpha (or null): importance weights of the D candidates (Sec. 3.2 Eq. 4);
// diagonal k then enters as alpha[o_k] * values[k], rounded to bf16 first -- exactly the values dd_scale_values
// would have stored.
// blockIdx.y numbers the sets of a group of layers of one shape whose operands are stacked into one matrix
// (set s uses offsets + s*K and values + s*K*L): an OperandPlace says where set s goes, s*col_step columns
// to the right (the sets' outputs side by side) or s*k_step contraction indices down (their results summed),
// inside a matrix of kd_total contraction indices; or, for layers that merely share a launch, set s has a whole
// operand of its own block_step elements further on.  D, L, col_step and k_step are multiples of 32.
// ---------------------------------------------------------------------------------------------
constexpr int kMatRows = 32;
constexpr int kMatRange = 256;
constexpr int kMatChunk = 512;             // diagonals looked at per pass
constexpr int kMatStride = kMatRange + 8;  // floats per row in LDS: the 32 rows of a fragment start 8 banks apart

__global__ __launch_bounds__(256) void materialize_kernel(int D, int L, int K, int masked_blocks,
                                                          const int *__restrict__ offsets,
                                                          const uint16_t *__restrict__ values,
                                                          uint16_t *__restrict__ Wf_masked,
                                                          uint16_t *__restrict__ Wf_gather, OperandPlace place_masked,
                                                          OperandPlace place_gather,
                                                          const float *__restrict__ alpha)
{
    __shared__ __attribute__((aligned(16))) float rows[kMatRows * kMatStride];
    __shared__ int hit_k[kMatChunk], hit_first[kMatChunk], hit_offset[kMatChunk], n_hits;
    const int ranges_masked = (L + kMatRange - 1) / kMatRange, ranges_gather = (D + kMatRange - 1) / kMatRange;
    const bool long_major = int(blockIdx.x) < masked_blocks * ranges_masked;
    const int job = long_major ? blockIdx.x : blockIdx.x - masked_blocks * ranges_masked;
    const int ranges = long_major ? ranges_masked : ranges_gather;
    const int r0 = job / ranges * kMatRows;
    const int KD = long_major ? L : D;
    const int i0 = job % ranges * kMatRange;
    const int extent = min(kMatRange, KD - i0);
    const int set = blockIdx.y;
    offsets += size_t(set) * K;
    values += size_t(set) * K * L;
    const OperandPlace place = long_major ? place_masked : place_gather;
    uint16_t *Wf = (long_major ? Wf_masked : Wf_gather) + size_t(set) * place.block_step;
    for (int c = threadIdx.x; c < kMatRows * kMatStride / 4; c += 256)
        reinterpret_cast<f32x4 *>(rows)[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    // A diagonal meets the block where the contraction indices of the 32 rows -- consecutive modulo D from `first`
    // on -- fall into this workgroup's range; most diagonals miss.  Up to kMatChunk diagonals at a time: every thread
    // looks at its share of the offsets (all loads first: one trip to memory) and lists the ones that meet the block;
    // then the (listed diagonal, row) pairs are dealt to all threads, rows innermost, so that a wave reads runs of
    // 32 consecutive values.
    for (int k0 = 0; k0 < K; k0 += kMatChunk) {
        if (threadIdx.x == 0) n_hits = 0;
        int o[kMatChunk / 256];
#pragma unroll
        for (int j = 0; j < kMatChunk / 256; ++j) {
            const int k = k0 + j * 256 + threadIdx.x;
            o[j] = k < K ? offsets[k] : 0;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kMatChunk / 256; ++j) {
            const int k = k0 + j * 256 + threadIdx.x;
            if (k >= K) continue;
            const int oc = canonical_offset(o[j], D);
            int first = long_major ? r0 - oc : r0 + oc;  // contraction index of row r0
            first += first < 0 ? D : 0;
            first -= first >= D ? D : 0;
            int d = first - i0;
            d += d < 0 ? D : 0;
            if (d >= extent && d + kMatRows <= D) continue;  // neither the first row inside nor a wrap into the range
            const int slot = atomicAdd(&n_hits, 1);
            hit_k[slot] = k;
            hit_first[slot] = first;
            hit_offset[slot] = oc;
        }
        __syncthreads();
        const int items = n_hits * kMatRows;
        for (int item = threadIdx.x; item < items; item += 256) {
            const int h = item / kMatRows, rr = item % kMatRows;
            const int i = hit_first[h] + rr >= D ? hit_first[h] + rr - D : hit_first[h] + rr;
            const int p = long_major ? i : r0 + rr;  // position along the diagonal
            if (unsigned(i - i0) >= unsigned(extent) || p >= L) continue;
            float v = bf16_to_f32(values[size_t(hit_k[h]) * L + p]);
            if (alpha) v = bf16_to_f32(f32_to_bf16(alpha[hit_offset[h]] * v));
            atomicAdd(&rows[rr * kMatStride + i - i0], v);
        }
        __syncthreads();  // the list may be overwritten; after the last pass: the rows are complete
    }
    // fragments (r0 / 32, i0 / 16 ...) lie one after the other: piece `pc` is lane pc % 64 of fragment pc / 64
    u32x4 *out = reinterpret_cast<u32x4 *>(Wf + fragment_index(r0 + set * place.col_step, i0 + set * place.k_step,
                                                                place.kd_total));
    for (int pc = threadIdx.x; pc < extent * 4; pc += 256) {
        const int lane = pc & 63;
        const float *src = rows + (lane & 31) * kMatStride + (pc >> 6) * 16 + 8 * (lane >> 5);
        out[pc] = pack_bf16x8(*reinterpret_cast<const f32x4 *>(src), *reinterpret_cast<const f32x4 *>(src + 4));
    }
}

// ---------------------------------------------------------------------------------------------
// Selection and step 1 in one launch, for layers small enough that the launches themselves are what the two
// steps cost: every workgroup repeats the selection of the K diagonals (Sec. 3.2 Eq. 4) for itself, keeps the
// chosen offsets in LDS, and then builds ROWS rows of the two operands from them; workgroup 0 also writes the
// offsets out.  Rows [0, D) are rows of the masked-gather operand, rows [D, D + L) rows of the gather operand.
// The selection never returns an offset twice, so no two diagonals meet in one entry and the operands come out
// bit for bit as materialize_kernel builds them.
// LDS: keys [D] | chosen offsets [K] | ROWS rows of D floats.
// ---------------------------------------------------------------------------------------------
template <int ROWS>
__global__ __launch_bounds__(kSelectThreads) void select_materialize_kernel(int D, int L, int K,
                                                                             const float *__restrict__ scores,
                                                                             const uint16_t *__restrict__ values,
                                                                             int *__restrict__ offsets_out,
                                                                             uint16_t *__restrict__ Wf_masked,
                                                                             uint16_t *__restrict__ Wf_gather)
{
    extern __shared__ uint32_t lds_words[];
    uint32_t *keys = lds_words;
    int *chosen = reinterpret_cast<int *>(lds_words + D);
    float *rows = reinterpret_cast<float *>(lds_words + D + K);
    for (int i = threadIdx.x; i < ROWS * D; i += kSelectThreads) rows[i] = 0.f;
    select_topk_block<true>(D, K, scores, keys, chosen);
    __syncthreads();
    if (blockIdx.x == 0)
        for (int k = threadIdx.x; k < K; k += kSelectThreads) offsets_out[k] = chosen[k];
    const int r0 = blockIdx.x * ROWS;
    for (int k = threadIdx.x; k < K; k += kSelectThreads) {
        const int o = chosen[k];  // already in [0, D)
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const int r = r0 + j;
            if (r < D) {  // masked gather, row q = r:  w[p] = v_k[p] where (q - o_k) mod D = p < L
                int pp = r - o;
                if (pp < 0) pp += D;
                if (pp < L) rows[j * D + pp] = bf16_to_f32(values[size_t(k) * L + pp]);
            } else if (r < D + L) {  // gather, row p = r - D:  w[q] = v_k[p] where q = (p + o_k) mod D
                int q = r - D + o;
                if (q >= D) q -= D;
                rows[j * D + q] = bf16_to_f32(values[size_t(k) * L + (r - D)]);
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const int r = r0 + j;
        if (r >= D + L) break;
        const bool long_major = r < D;
        const int KD = long_major ? L : D;
        uint16_t *Wf = long_major ? Wf_masked : Wf_gather;
        const int out_row = long_major ? r : r - D;
        for (int c8 = threadIdx.x; c8 < KD / 8; c8 += kSelectThreads) {
            const float *src = rows + j * D + c8 * 8;  // 4-byte aligned only: K words lie before the rows
            const u32x4 v = pack_bf16x8(f32x4{src[0], src[1], src[2], src[3]}, f32x4{src[4], src[5], src[6], src[7]});
            *reinterpret_cast<u32x4 *>(Wf + fragment_index(out_row, c8 * 8, KD)) = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Step 2: C [T x NC] = A [T x KD] . W,  W given fragment-major.
// A and C may each be a stack of equally shaped row-major matrices (a group of layers that share
// their input): A = KD / a_cols matrices [T x a_cols] one after the other, contraction index i in
// matrix i / a_cols, column i % a_cols; C = NC / c_cols matrices [T x c_cols] likewise.  a_cols is
// a multiple of the k-slice, c_cols of eight; a plain product has a_cols = KD and c_cols = NC.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int NW>
struct MmTile {
    static constexpr int THREADS = 64 * NW;
    static constexpr int WN = BN / NW;             // output columns per wave
    static constexpr int FA = WN / 32;             // 32-row MFMA tiles along the output columns
    static constexpr int FB = BM / 32;             // 32-column MFMA tiles along the tokens
    static constexpr int X_CHUNKS = (BM * kChunksPerRow + THREADS - 1) / THREADS;  // 16-byte pieces per thread per stage
    static constexpr int X_BYTES = BM * kRowBytes;
    static constexpr int C_STRIDE = (BN + 8) * 2;  // bytes; the pad staggers rows over the banks
    static constexpr int C_BYTES = BM * C_STRIDE;
    static constexpr int LDS_BYTES = kRing * X_BYTES > C_BYTES ? kRing * X_BYTES : C_BYTES;
    static_assert(BM % 32 == 0 && BN % (32 * NW) == 0, "tile must split into 32x32 MFMA tiles over the waves");
    static_assert((BM * 8) % 64 == 0, "a stage is filled by whole waves");
};

// Result tile (tm, tn), held row by row in LDS, to the stack of [T x c_cols] matrices C: 16-byte pieces, full-width
// row segments.  A tile of BN <= 256 columns reaches into at most three matrices of 128 or more columns.
// One 16-byte piece per thread: piece number idx of the tile whose first column is column first_col of matrix
// first_matrix of the stack.
template <int BM, int BN>
__device__ __forceinline__ void store_tile_piece(uint16_t *__restrict__ C, const unsigned char *tile, int tile_stride,
                                                 int tm, int first_matrix, int first_col, int T, int c_cols, int idx)
{
    constexpr int ROW_CHUNKS = BN / 8;
    const int row = idx / ROW_CHUNKS, ch = idx % ROW_CHUNKS;
    const int t = tm * BM + row;
    int matrix = first_matrix, col = first_col + ch * 8;
#pragma unroll
    for (int hop = 0; hop < 2; ++hop)
        if (col >= c_cols) {
            col -= c_cols;
            ++matrix;
        }
    // The result is not read again by this kernel: a streaming store keeps it from piling up dirty in the L2, which
    // would otherwise be written back in one piece when the kernel ends (measured: 2 us of a 22 us product).
    if (row < BM && t < T)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(tile + row * tile_stride + ch * 16),
                                    reinterpret_cast<u32x4 *>(C + (size_t(matrix) * T + t) * c_cols + col));
}

template <int BM, int BN, int THREADS>
__device__ __forceinline__ void store_tile(uint16_t *__restrict__ C, const unsigned char *tile, int tile_stride, int tm,
                                           int tn, int T, int c_cols, int tid)
{
    const int first_matrix = (tn * BN) / c_cols;
    const int first_col = tn * BN - first_matrix * c_cols;
    for (int idx = tid; idx < BM * (BN / 8); idx += THREADS)
        store_tile_piece<BM, BN>(C, tile, tile_stride, tm, first_matrix, first_col, T, c_cols, idx);
}

template <int BM, int BN, int NW>
__global__ __launch_bounds__(64 * NW) void mm_kernel(int T, int NC, int KD, int a_cols, int c_cols, int tiles_m,
                                                        int tiles_n, int group_n, const uint16_t *__restrict__ A,
                                                        const uint16_t *__restrict__ Wf,
                                                        uint16_t *__restrict__ C)
{
    using Tl = MmTile<BM, BN, NW>;
    constexpr int kMmThreads = Tl::THREADS;
    extern __shared__ __align__(16) unsigned char smem[];

    // Workgroups are dealt round-robin to the eight XCDs, each with an L2 of its own.  Give every
    // XCD one contiguous run of tiles, column tiles innermost, so that the tiles sharing a token
    // block (and with it a slice of A) run on the same L2.
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const int lin = int(blockIdx.x % kXcds) * per_xcd + int(blockIdx.x / kXcds);
    if (lin >= n_tiles) return;
    // (column tiles in groups of group_n, see tile_group: all token blocks of one group before the next group)
    const int vrow = lin / group_n, group = vrow / tiles_m;
    const int tm = vrow - group * tiles_m, tn = group * group_n + lin % group_n;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int KT = KD / kBK;  // even: feature counts are multiples of 128

    // token operand, global -> registers -> LDS: thread handles chunk (row = idx / 8, chunk = idx % 8)
    const uint16_t *x_src[Tl::X_CHUNKS];
    int x_dst[Tl::X_CHUNKS];
#pragma unroll
    for (int n = 0; n < Tl::X_CHUNKS; ++n) {
        const int idx = min(tid + kMmThreads * n, BM * kChunksPerRow - 1);  // a last partial round repeats the final piece
        const int row = idx / kChunksPerRow, ch = idx % kChunksPerRow;
        int t = tm * BM + row;
        t = t < T ? t : T - 1;  // rows past the end re-read the last token; their results are not stored
        x_src[n] = A + size_t(t) * a_cols + ch * 8;
        x_dst[n] = row * kRowBytes + swizzle(row, ch) * 16;
    }
    // Where the next k-slice to request starts, relative to a row's first element: 64 columns further on, or in
    // the next matrix of the stack.  Past the last slice the cursor stays put (the loop then re-reads that slice).
    size_t x_off = 0;
    int x_in = 0, x_slice = 0;
    const size_t x_jump = size_t(T - 1) * a_cols;
#define DD_X_ADVANCE                                                                                    \
    if (x_slice < KT - 1) {                                                                             \
        ++x_slice;                                                                                      \
        x_off += kBK;                                                                                   \
        x_in += kBK;                                                                                    \
        if (x_in == a_cols) {                                                                           \
            x_in = 0;                                                                                   \
            x_off += x_jump;                                                                            \
        }                                                                                               \
    }
    // weight fragments of this wave: block row (tn*BN + wave*WN)/32 + a, 1 KB per k-step, 16 bytes per lane
    const uint16_t *w_src[Tl::FA];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
        w_src[a] = Wf + (size_t((tn * BN + wave * Tl::WN) / 32 + a) * (KD / 16) * 64 + lane) * 8;
    // token fragments of this lane
    int b_off[Tl::FB], b_sw[Tl::FB];
#pragma unroll
    for (int b = 0; b < Tl::FB; ++b) {
        const int row = b * 32 + l32;
        b_off[b] = row * kRowBytes;
        b_sw[b] = swizzle_key(row);
    }

    f32x16 acc[Tl::FA][Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    u32x4 xg0[Tl::X_CHUNKS], xg1[Tl::X_CHUNKS];       // token slices in flight from global memory
    bf16x8 wf0[4][Tl::FA], wf1[4][Tl::FA];             // weight fragments of the current / next k-slice
    bf16x8 xf0[Tl::FB], xf1[Tl::FB];                   // token fragments of the current / next k-step

#define DD_LOAD_X(xg_) /* the slice under the cursor; the cursor moves on */                           \
    {                                                                                                   \
        _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n)                                        \
            xg_[n] = *reinterpret_cast<const u32x4 *>(x_src[n] + x_off);                                \
        DD_X_ADVANCE                                                                                    \
    }
#define DD_STORE_X(xg_, kt_)                                                                            \
    {                                                                                                   \
        unsigned char *dstb = smem + ((kt_) % kRing) * Tl::X_BYTES;                                     \
        _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n)                                        \
            *reinterpret_cast<u32x4 *>(dstb + x_dst[n]) = xg_[n];                                       \
    }
#define DD_LOAD_W(wf_, g_) /* g_ counts groups of four k-steps (64 contraction indices) */            \
    {                                                                                                   \
        const int gmax = KD / 64 - 1;                                                                   \
        const size_t kk = size_t((g_) < gmax ? (g_) : gmax) * 4 * 512;                                  \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                \
            _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                          \
                wf_[ks][a] = *reinterpret_cast<const bf16x8 *>(w_src[a] + kk + ks * 512);               \
    }
    // The ring of token slices: byte offsets of the stage being multiplied, the next one and the one being filled;
    // they change places after every slice.
    int ring_cur = 0, ring_next = Tl::X_BYTES, ring_fill = 2 * Tl::X_BYTES;
#define DD_LOAD_XF(xf_, ring_, ks_)                                                                     \
    {                                                                                                   \
        const unsigned char *srcb = smem + (ring_);                                                     \
        const int ch = (ks_) * 2 + half;                                                                \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                              \
            xf_[b] = *reinterpret_cast<const bf16x8 *>(srcb + b_off[b] + ((ch ^ b_sw[b]) << 4));        \
    }
#define DD_MFMA(wf_, ks_, xf_)                                                                          \
    _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                                  \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                              \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf_[ks_][a], xf_[b], acc[a][b], 0, 0, 0);
    // One k-slice: four k-steps; the token fragments of the next k-step are fetched from LDS while
    // the current one is multiplied; then the slice two ahead is parked in LDS and a new one requested.
    // one k-step: after each MFMA the token fragment of the following k-step for the same token tile, and one
    // piece of the slice's other traffic (weight fragments of the next slice, token pieces into LDS, new requests)
#define DD_XF_ONE(xf_, ring_, ks_, b_)                                                                  \
    xf_[b_] = *reinterpret_cast<const bf16x8 *>(smem + (ring_) + b_off[b_] + ((((ks_) * 2 + half) ^ b_sw[b_]) << 4));
#define DD_STEP(wf_cur_, ks_, xf_cur_, xf_nxt_, ring_nxt_, ks_nxt_, extra_)                               \
    _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b) {                                                \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                              \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf_cur_[ks_][a], xf_cur_[b], acc[a][b], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        DD_XF_ONE(xf_nxt_, ring_nxt_, ks_nxt_, b)                                                       \
        extra_                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
#define DD_SLICE(kt_, wf_cur_, wf_next_, xg_)                                                           \
    {                                                                                                   \
        const int gmax = KD / 64 - 1;                                                                   \
        const size_t w_kk = size_t(((kt_) + 1) < gmax ? ((kt_) + 1) : gmax) * 4 * 512;                  \
        const size_t x_kk = x_off; /* slice kt_ + 4 */                                                 \
        DD_X_ADVANCE                                                                                    \
        unsigned char *x_dstb = smem + ring_fill;                                                       \
        DD_STEP(wf_cur_, 0, xf0, xf1, ring_cur, 1,                                                      \
                if (b < 2) { _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a) {                       \
                    wf_next_[2 * b][a] = *reinterpret_cast<const bf16x8 *>(w_src[a] + w_kk + (2 * b) * 512); \
                    wf_next_[2 * b + 1][a] = *reinterpret_cast<const bf16x8 *>(w_src[a] + w_kk + (2 * b + 1) * 512); } }) \
        DD_STEP(wf_cur_, 1, xf1, xf0, ring_cur, 2, )                                                    \
        DD_STEP(wf_cur_, 2, xf0, xf1, ring_cur, 3,                                                      \
                if (b < Tl::X_CHUNKS) { *reinterpret_cast<u32x4 *>(x_dstb + x_dst[b]) = xg_[b];         \
                                        xg_[b] = *reinterpret_cast<const u32x4 *>(x_src[b] + x_kk); })  \
        DD_STEP(wf_cur_, 3, xf1, xf0, ring_next, 0, )                                                   \
        {                                                                                               \
            const int t = ring_cur;                                                                     \
            ring_cur = ring_next;                                                                       \
            ring_next = ring_fill;                                                                      \
            ring_fill = t;                                                                              \
        }                                                                                               \
        __syncthreads();                                                                                \
    }
    static_assert(Tl::X_CHUNKS <= Tl::FB && Tl::FB >= 2, "one extra piece of work per MFMA");

    // prologue: slices 0 and 1 in LDS, slices 2 and 3 in flight, weight fragments of slice 0 loaded
    DD_LOAD_X(xg0)
    DD_LOAD_X(xg1)
    DD_LOAD_W(wf0, 0)
    DD_STORE_X(xg0, 0)
    DD_STORE_X(xg1, 1)
    DD_LOAD_X(xg0)
    DD_LOAD_X(xg1)
    __syncthreads();
    DD_LOAD_XF(xf0, ring_cur, 0)
    for (int kt = 0; kt < KT; kt += 2) {
        DD_SLICE(kt, wf0, wf1, xg0)
        DD_SLICE(kt + 1, wf1, wf0, xg1)
    }
#undef DD_LOAD_X
#undef DD_X_ADVANCE
#undef DD_STORE_X
#undef DD_LOAD_W
#undef DD_LOAD_XF
#undef DD_MFMA
#undef DD_SLICE
#undef DD_STEP
#undef DD_XF_ONE

    // Epilogue.  Accumulator i of lane l is output column 8*(i/4) + 4*(l/32) + i%4 of token l%32
    // inside its 32x32 tile: four consecutive columns per group, written as one 8-byte LDS store.
    // (The last barrier of the loop has retired every read of the ring.)
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
    store_tile<BM, BN, kMmThreads>(C, smem, Tl::C_STRIDE, tm, tn, T, c_cols, tid);
}

// ---------------------------------------------------------------------------------------------
// Step 2 for products with more tiles than CUs: one workgroup per CU walks a list of tiles, and the
// software pipeline of mm_kernel runs through from tile to tile: while the last k-slices of a tile are
// multiplied, the first slices of the next tile are already on their way (where mm_kernel re-reads the
// last slice to keep its loop uniform), so a tile costs its main loop, not another fill of the pipeline.  The
// copy-out of a tile's result is dealt out between the MFMAs of the next tile's first two slices: at the end of
// a tile the accumulators are rounded into registers and cleared, during the next slice those registers go to an
// LDS buffer of the result's own beside the ring, and during the slice after that the buffer leaves for memory
// in full-width row segments.  Only the last tile of a workgroup is copied out with nothing to hide behind.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int NW>
__global__ __launch_bounds__(64 * NW) void mm_persistent_kernel(int T, int NC, int KD, int a_cols, int c_cols,
                                                                  int tiles_m, int tiles_n, int group_n,
                                                                  unsigned tiles_m_magic,
                                                                  const uint16_t *__restrict__ A,
                                                                  const uint16_t *__restrict__ Wf,
                                                                  uint16_t *__restrict__ C)
{
    using Tl = MmTile<BM, BN, NW>;
    constexpr int kMmThreads = Tl::THREADS;
    constexpr int kSlots = 256 / kXcds;  // workgroups per XCD: one per CU
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *c_buf = smem + kRing * Tl::X_BYTES;

    // The tiles are cut into one contiguous run per XCD (column tiles innermost, so that tiles sharing a
    // token block run on the same L2); workgroup `slot` of an XCD takes every kSlots-th tile of its run.
    // The order of the tiles is that of a matrix of group_n column tiles and tiles_m * (tiles_n / group_n) rows:
    // row v of it is token block v mod tiles_m of column group v / tiles_m (see tile_group).  The cursors below walk
    // that matrix; the token block and column tile a position stands for are kept beside it (one multiply-high by
    // tiles_m_magic = ceil(2^32 / tiles_m) per move, on the scalar unit).
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int run_begin = xcd * per_xcd, run_end = min(run_begin + per_xcd, n_tiles);
    const int first = run_begin + slot;
    if (first >= run_end) return;
    const int n_mine = (run_end - first + kSlots - 1) / kSlots;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int KT = KD / kBK;  // even: feature counts are multiples of 128

    int x_row[Tl::X_CHUNKS], x_col[Tl::X_CHUNKS], x_dst[Tl::X_CHUNKS];
#pragma unroll
    for (int n = 0; n < Tl::X_CHUNKS; ++n) {
        const int idx = min(tid + kMmThreads * n, BM * kChunksPerRow - 1);  // a last partial round repeats the final piece
        x_row[n] = idx / kChunksPerRow;
        x_col[n] = (idx % kChunksPerRow) * 8;
        x_dst[n] = x_row[n] * kRowBytes + swizzle(x_row[n], idx % kChunksPerRow) * 16;
    }
    int b_off[Tl::FB], b_sw[Tl::FB];
#pragma unroll
    for (int b = 0; b < Tl::FB; ++b) {
        const int row = b * 32 + l32;
        b_off[b] = row * kRowBytes;
        b_sw[b] = swizzle_key(row);
    }

    f32x16 acc[Tl::FA][Tl::FB];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a)
#pragma unroll
        for (int b = 0; b < Tl::FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    u32x4 xg0[Tl::X_CHUNKS], xg1[Tl::X_CHUNKS];
    bf16x8 wf0[4][Tl::FA], wf1[4][Tl::FA];
    bf16x8 xf0[Tl::FB], xf1[Tl::FB];

    // Two cursors walk the k-slices of this workgroup's tiles in order, one for the weight fragments (one slice
    // ahead of the multiplication) and one for the token slices (four ahead).  Inside a tile a cursor only counts and
    // the request addresses move on by a constant; the tile's place, its token block and its column tile are worked out
    // once per tile, behind a branch every wave takes together.  After the last slice of the last tile a cursor walks
    // that tile again: the requests past the end only have to name valid addresses, what they fetch is never
    // multiplied.
    struct Cursor {
        int tiles_left;  // my tiles after this one
        int kt;          // k-slice inside the tile
        int tm, tn;      // the tile's place in the grouped order: row and column of the matrix described above
        int in;          // first contraction index of the slice inside its matrix of the stack A
    };
    const int hop_m = kSlots / group_n, hop_n = kSlots % group_n;  // from one of my tiles to the next
#define DD_REAL_M(v_) (int(v_) - int(__umulhi(unsigned(v_), tiles_m_magic)) * tiles_m)
#define DD_REAL_N(v_, c_) (int(__umulhi(unsigned(v_), tiles_m_magic)) * group_n + (c_))
    Cursor wc = {n_mine - 1, 0, first / group_n, first % group_n, 0};
    Cursor xc = wc;
    int out_tm = wc.tm, out_tn = wc.tn;  // the tile being multiplied (place in the grouped order)
    // a cursor that has walked its tile's last slice: on to my next tile, if there is one
#define DD_NEXT_TILE(c_)                                                                                \
    {                                                                                                   \
        c_.kt = 0;                                                                                      \
        c_.in = 0;                                                                                      \
        if (c_.tiles_left > 0) {                                                                        \
            --c_.tiles_left;                                                                            \
            const int carry = c_.tn + hop_n >= group_n ? 1 : 0;                                         \
            c_.tn += hop_n - carry * group_n;                                                           \
            c_.tm += hop_m + carry;                                                                     \
        }                                                                                               \
    }
    size_t w_lane[Tl::FA];
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a) w_lane[a] = (size_t(wave * (Tl::WN / 32) + a) * (KD / 16) * 64 + lane) * 8;
    const size_t w_tile_step = size_t(BN / 32) * (KD / 16) * 512;  // from one column tile to the next
    const size_t a_matrix = size_t(T) * a_cols;                    // from one matrix of the stack to the next
    const uint16_t *x_ptr[Tl::X_CHUNKS];  // where the next token slice to request starts, piece by piece
    const uint16_t *w_ptr[Tl::FA];        // where the next weight fragments to request start
    // first slice of the tile under the cursor: piece n_ of this thread (rows past the end re-read the last token),
    // fragment row a_ of this wave
#define DD_X_TILE(n_)                                                                                   \
    (A + x_col[n_] + size_t(unsigned(min(DD_REAL_M(xc.tm) * BM + x_row[n_], T - 1))) * unsigned(a_cols))
#define DD_W_TILE(a_) (Wf + size_t(DD_REAL_N(wc.tm, wc.tn)) * w_tile_step + w_lane[a_])
    // the token cursor and its addresses move on by one slice: 64 columns further on, or into the next matrix of the
    // stack, or to the next tile
#define DD_X_ADVANCE                                                                                    \
    {                                                                                                   \
        ++xc.kt;                                                                                        \
        xc.in += kBK;                                                                                   \
        size_t step = kBK;                                                                              \
        if (xc.in == a_cols) {                                                                          \
            xc.in = 0;                                                                                  \
            step += a_matrix - size_t(a_cols);                                                          \
        }                                                                                               \
        if (__builtin_expect(xc.kt == KT, 0)) {                                                         \
            DD_NEXT_TILE(xc)                                                                            \
            _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n) x_ptr[n] = DD_X_TILE(n);           \
        } else {                                                                                        \
            _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n) x_ptr[n] += step;                  \
        }                                                                                               \
    }
#define DD_W_ADVANCE                                                                                    \
    {                                                                                                   \
        ++wc.kt;                                                                                        \
        if (__builtin_expect(wc.kt == KT, 0)) {                                                         \
            DD_NEXT_TILE(wc)                                                                            \
            _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a) w_ptr[a] = DD_W_TILE(a);                 \
        } else {                                                                                        \
            _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a) w_ptr[a] += 4 * 512;                     \
        }                                                                                               \
    }
#define DD_LOAD_X(xg_) /* the slice under the cursor; the cursor moves on */                           \
    {                                                                                                   \
        _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n)                                        \
            xg_[n] = *reinterpret_cast<const u32x4 *>(x_ptr[n]);                                        \
        DD_X_ADVANCE                                                                                    \
    }
#define DD_STORE_X(xg_, slot_)                                                                          \
    {                                                                                                   \
        unsigned char *dstb = smem + (slot_) * Tl::X_BYTES;                                             \
        _Pragma("unroll") for (int n = 0; n < Tl::X_CHUNKS; ++n)                                        \
            *reinterpret_cast<u32x4 *>(dstb + x_dst[n]) = xg_[n];                                       \
    }
#define DD_LOAD_W(wf_)                                                                                  \
    {                                                                                                   \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                              \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                            \
                wf_[ks][a] = *reinterpret_cast<const bf16x8 *>(w_ptr[a] + ks * 512);                    \
        DD_W_ADVANCE                                                                                    \
    }
    // The ring of token slices: byte offsets of the stage being multiplied, the next one and the one being filled;
    // they change places after every slice.
    int ring_cur = 0, ring_next = Tl::X_BYTES, ring_fill = 2 * Tl::X_BYTES;
#define DD_RING_TURN                                                                                    \
    {                                                                                                   \
        const int t = ring_cur;                                                                         \
        ring_cur = ring_next;                                                                           \
        ring_next = ring_fill;                                                                          \
        ring_fill = t;                                                                                  \
    }
#define DD_LOAD_XF(xf_, ring_, ks_)                                                                     \
    {                                                                                                   \
        const unsigned char *srcb = smem + (ring_);                                                     \
        const int ch = (ks_) * 2 + half;                                                                \
        _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                              \
            xf_[b] = *reinterpret_cast<const bf16x8 *>(srcb + b_off[b] + ((ch ^ b_sw[b]) << 4));        \
    }
#define DD_XF_ONE(xf_, ring_, ks_, b_)                                                                  \
    xf_[b_] = *reinterpret_cast<const bf16x8 *>(smem + (ring_) + b_off[b_] + ((((ks_) * 2 + half) ^ b_sw[b_]) << 4));
    // one k-step: after each MFMA the token fragment of the following k-step for the same token tile, and one
    // piece of the slice's other traffic
#define DD_STEP(wf_cur_, ks_, xf_cur_, xf_nxt_, ring_nxt_, ks_nxt_, extra_)                             \
    _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b) {                                                \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                              \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf_cur_[ks_][a], xf_cur_[b], acc[a][b], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        DD_XF_ONE(xf_nxt_, ring_nxt_, ks_nxt_, b)                                                       \
        extra_                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
    // One k-slice.  Its requests (weight fragments of the slice after it, the token slice four on) go to addresses that
    // were settled at the end of the slice before; the cursors move on behind the last MFMA, so that the branch of a
    // tile change does not cut through the k-steps, whose instructions are dealt out by hand.
#define DD_SLICE_X(wf_cur_, wf_next_, xg_, e0_, e1_, e2_, e3_)                                           \
    {                                                                                                   \
        unsigned char *x_dstb = smem + ring_fill;                                                       \
        DD_STEP(wf_cur_, 0, xf0, xf1, ring_cur, 1,                                                      \
                if (b < 2) { _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a) {                       \
                    wf_next_[2 * b][a] = *reinterpret_cast<const bf16x8 *>(w_ptr[a] + (2 * b) * 512);   \
                    wf_next_[2 * b + 1][a] = *reinterpret_cast<const bf16x8 *>(w_ptr[a] + (2 * b + 1) * 512); } } \
                e0_)                                                                                    \
        DD_STEP(wf_cur_, 1, xf1, xf0, ring_cur, 2, e1_)                                                 \
        DD_STEP(wf_cur_, 2, xf0, xf1, ring_cur, 3,                                                      \
                if (b < Tl::X_CHUNKS) { *reinterpret_cast<u32x4 *>(x_dstb + x_dst[b]) = xg_[b];         \
                                        xg_[b] = *reinterpret_cast<const u32x4 *>(x_ptr[b]); }          \
                e2_)                                                                                    \
        DD_STEP(wf_cur_, 3, xf1, xf0, ring_next, 0, e3_)                                                \
        asm volatile("" ::: "memory"); /* no request sinks out of the k-steps into the branches below */ \
        DD_W_ADVANCE                                                                                    \
        DD_X_ADVANCE                                                                                    \
        DD_RING_TURN                                                                                    \
        __syncthreads();                                                                                \
    }
#define DD_SLICE(wf_cur_, wf_next_, xg_) DD_SLICE_X(wf_cur_, wf_next_, xg_, , , , )
    static_assert(Tl::X_CHUNKS <= Tl::FB && Tl::FB >= 2, "one extra piece of work per MFMA");

    // The result on its way out.  Accumulator i of lane l is output column 8*(i/4) + 4*(l/32) + i%4 of token l%32
    // inside its 32x32 tile: four consecutive columns per group, one 8-byte LDS store.
    // In the copy-out thread `tid` moves the 16-byte piece tid % 32 of rows tid / 32 + 16 i, i = 0..9; rows past
    // the last token repeat the last valid row (same bytes to the same place), so no piece needs a predicate.
    bf16x4 parked[Tl::FA][Tl::FB][4];
    uint16_t *parked_dst = C;  // row 0 of the parked tile, this thread's piece
    int parked_rows = 1;       // valid token rows of the parked tile
    const int out_row0 = tid / (BN / 8), out_piece = tid % (BN / 8);
#define DD_PARK /* the tile is complete */                                                              \
    {                                                                                                   \
        _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                              \
            _Pragma("unroll") for (int b = 0; b < Tl::FB; ++b)                                          \
                _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                         \
                    f32x4 v = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]}; \
                    parked[a][b][q] = __builtin_convertvector(v, bf16x4);                               \
                    _Pragma("unroll") for (int i = 0; i < 4; ++i) acc[a][b][4 * q + i] = 0.f;           \
                }                                                                                       \
        {                                                                                               \
            const int real_tm = DD_REAL_M(out_tm), real_tn = DD_REAL_N(out_tm, out_tn);                 \
            int matrix = (real_tn * BN) / c_cols;                                                       \
            int col = real_tn * BN - matrix * c_cols + out_piece * 8;                                   \
            _Pragma("unroll") for (int hop = 0; hop < 2; ++hop)                                         \
                if (col >= c_cols) {                                                                    \
                    col -= c_cols;                                                                      \
                    ++matrix;                                                                           \
                }                                                                                       \
            parked_dst = C + (size_t(matrix) * T + size_t(real_tm) * BM) * c_cols + col;                \
            parked_rows = min(BM, T - real_tm * BM);                                                    \
        }                                                                                               \
        const bool carry = out_tn + hop_n >= group_n;                                                   \
        out_tn += hop_n - (carry ? group_n : 0);                                                        \
        out_tm += hop_m + (carry ? 1 : 0);                                                              \
    }
    // token tile b_ of the parked result -> LDS
#define DD_C_WRITE(b_)                                                                                  \
    _Pragma("unroll") for (int a = 0; a < Tl::FA; ++a)                                                  \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                                   \
            *reinterpret_cast<bf16x4 *>(c_buf + ((b_) * 32 + l32) * Tl::C_STRIDE +                      \
                                        (wave * Tl::WN + a * 32 + 8 * q + 4 * half) * 2) = parked[a][b_][q];
    // piece i_ of this thread's share of the copy-out, LDS -> memory
#define DD_C_OUT(i_)                                                                                    \
    {                                                                                                   \
        const int r = min(out_row0 + (kMmThreads / (BN / 8)) * (i_), parked_rows - 1);                  \
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(c_buf + r * Tl::C_STRIDE + out_piece * 16), \
                                    reinterpret_cast<u32x4 *>(parked_dst + size_t(unsigned(r)) * unsigned(c_cols))); \
    }
    constexpr int kOutPieces = (BM * BN / 8 + kMmThreads - 1) / kMmThreads;
    static_assert(Tl::FB == 5 && kOutPieces % 10 == 0, "the copy-out is dealt over ten free places of a slice of five token tiles per k-step");
    constexpr int kPiecesPerPlace = kOutPieces / 10;
#define DD_C_OUT_PLACE(s_) _Pragma("unroll") for (int u = 0; u < kPiecesPerPlace; ++u) { DD_C_OUT((s_) * kPiecesPerPlace + u) }

#pragma unroll
    for (int n = 0; n < Tl::X_CHUNKS; ++n) x_ptr[n] = DD_X_TILE(n);
#pragma unroll
    for (int a = 0; a < Tl::FA; ++a) w_ptr[a] = DD_W_TILE(a);
    DD_LOAD_X(xg0)
    DD_LOAD_X(xg1)
    DD_LOAD_W(wf0)
    DD_STORE_X(xg0, 0)
    DD_STORE_X(xg1, 1)
    DD_LOAD_X(xg0)
    DD_LOAD_X(xg1)
    __syncthreads();
    DD_LOAD_XF(xf0, ring_cur, 0)
    for (int kt = 0; kt < KT; kt += 2) {  // the first tile
        DD_SLICE(wf0, wf1, xg0)
        DD_SLICE(wf1, wf0, xg1)
    }
    DD_PARK
    for (int tile = 1; tile < n_mine; ++tile) {
        // first slice: the parked result goes to LDS (token tiles 0-2, then 3-4); second slice, after the barrier
        // between the two: the pieces leave for memory
        DD_SLICE_X(wf0, wf1, xg0, if (b >= 2) { DD_C_WRITE(b - 2) }, if (b == 2 || b == 3) { DD_C_WRITE(b + 1) }, , )
        DD_SLICE_X(wf1, wf0, xg1, if (b >= 2) { DD_C_OUT_PLACE(b - 2) }, if (b >= 2) { DD_C_OUT_PLACE(b + 1) },
                   if (b >= 3) { DD_C_OUT_PLACE(b + 3) }, if (b == 4) { DD_C_OUT_PLACE(8) DD_C_OUT_PLACE(9) })
        for (int kt = 2; kt < KT; kt += 2) {
            DD_SLICE(wf0, wf1, xg0)
            DD_SLICE(wf1, wf0, xg1)
        }
        DD_PARK
    }
    // the last tile: nothing left to hide its copy-out behind
#pragma unroll
    for (int b = 0; b < Tl::FB; ++b) { DD_C_WRITE(b) }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kOutPieces; ++i) { DD_C_OUT(i) }
#undef DD_PARK
#undef DD_C_WRITE
#undef DD_C_OUT
#undef DD_C_OUT_PLACE
#undef DD_SLICE_X
#undef DD_STEP
#undef DD_XF_ONE
#undef DD_NEXT_TILE
#undef DD_X_ADVANCE
#undef DD_W_ADVANCE
#undef DD_RING_TURN
#undef DD_REAL_M
#undef DD_REAL_N
#undef DD_X_TILE
#undef DD_W_TILE
#undef DD_LOAD_X
#undef DD_STORE_X
#undef DD_LOAD_W
#undef DD_LOAD_XF
#undef DD_MFMA
#undef DD_SLICE
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
bool product_matrix_supported(int64_t T, int D, int L, bool bf16)
{
    return bf16 && T > 0 && T < (int64_t(1) << 31) && D % 128 == 0 && L % 128 == 0 && D <= 8192;
}

size_t product_matrix_ws_bytes(int D, int L) { return size_t(D) * size_t(L) * 2; }

// Order of the result tiles.  A workgroup's column tile needs BN columns of the dense operand over the whole
// contraction; the column tiles that run side by side on one XCD should find theirs in its 4 MB L2 together with
// the token rows in flight.  Where the whole operand is too large for that (ViT MLP layers: 4.7 MB), the column
// tiles are taken in groups whose operand slice fits, every token block of one group before the next group: the
// token matrix is then fetched once per group instead of the operand once per round of tiles.  Returns the
// number of column tiles per group (a divisor of tiles_n; tiles_n itself = plain order), by the fetches either
// order costs.
static int tile_group(int64_t tiles_m, int tiles_n, int BN, int KD)
{
    const double col_tile = double(BN) * KD * 2;               // operand bytes of one column tile
    const double fits = 1.75 * 1024 * 1024;                    // what stays resident beside the streams
    const double a_bytes = double(tiles_m) * 160 * KD * 2;     // token matrix (160-token blocks)
    const double rounds = double(tiles_m) * tiles_n / (kXcds * 32);  // per XCD: every round streams what does not fit
    int best = tiles_n;
    double best_cost = a_bytes + kXcds * col_tile * tiles_n * (col_tile * tiles_n <= fits ? 1.0 : (rounds > 1 ? rounds : 1.0));
    for (int g = tiles_n - 1; g >= 1; --g) {
        if (tiles_n % g || col_tile * g > fits) continue;
        const double cost = a_bytes * (tiles_n / g) + kXcds * col_tile * tiles_n;
        if (cost < best_cost) { best_cost = cost; best = g; }
    }
    return best;
}

template <int BM, int BN, int NW>
static hipError_t launch_mm(int T, int NC, int KD, int a_cols, int c_cols, const uint16_t *A, const uint16_t *Wf,
                            uint16_t *C, hipStream_t stream)
{
    using Tl = MmTile<BM, BN, NW>;
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&mm_kernel<BM, BN, NW>), Tl::LDS_BYTES, lds_allowed)) return e;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = NC / BN;
    const int per_xcd = (tiles_m * tiles_n + kXcds - 1) / kXcds;
    hipLaunchKernelGGL((mm_kernel<BM, BN, NW>), dim3(per_xcd * kXcds), dim3(Tl::THREADS), Tl::LDS_BYTES, stream, T, NC, KD,
                       a_cols, c_cols, tiles_m, tiles_n, tiles_n, A, Wf, C);  // every tile is resident at once: plain order
    return hipGetLastError();
}

// workgroups of materialize_kernel: every (block of rows, range of contraction indices) pair of the two operands x sets
static dim3 materialize_grid(int D, int L, int masked_rows, int gather_rows, int sets)
{
    const int ranges_masked = (L + kMatRange - 1) / kMatRange, ranges_gather = (D + kMatRange - 1) / kMatRange;
    return dim3(masked_rows / kMatRows * ranges_masked + gather_rows / kMatRows * ranges_gather, sets);
}

hipError_t launch_prepare_matrix(int D, int L, int K, int sets, bool expanding, const int32_t *offsets,
                                 const void *values, void *forward_operand, void *backward_operand, hipStream_t stream,
                                 const float *alpha)
{
    // The forward product is the masked gather when the layer expands (M <= N), else the plain gather.  The sets'
    // forward operands stand side by side (every set has outputs of its own), their backward-input operands on top
    // of each other (the sets' contributions to the one input gradient add up in the contraction).
    const OperandPlace side_by_side = {expanding ? L : D, expanding ? D : L, 0, 0};
    const OperandPlace stacked = {sets * (expanding ? D : L), 0, expanding ? D : L, 0};
    hipLaunchKernelGGL(materialize_kernel, materialize_grid(D, L, D, L, sets), dim3(256), 0, stream, D, L, K, D / kMatRows,
                       offsets, static_cast<const uint16_t *>(values),
                       static_cast<uint16_t *>(expanding ? forward_operand : backward_operand),
                       static_cast<uint16_t *>(expanding ? backward_operand : forward_operand),
                       expanding ? side_by_side : stacked, expanding ? stacked : side_by_side, alpha);
    return hipGetLastError();
}

hipError_t launch_prepare_matrix_batched(int D, int L, int K, int layers, bool expanding, const int32_t *offsets,
                                         const void *values, void *prepared, hipStream_t stream)
{
    // layer i: forward operand at block i, backward-input operand D*L elements behind it, as launch_prepare_matrix
    // lays out one layer
    const size_t operand = size_t(D) * L;
    const OperandPlace masked = {L, 0, 0, 2 * operand}, gather = {D, 0, 0, 2 * operand};
    uint16_t *first = static_cast<uint16_t *>(prepared);
    hipLaunchKernelGGL(materialize_kernel, materialize_grid(D, L, D, L, layers), dim3(256), 0, stream, D, L, K, D / kMatRows,
                       offsets, static_cast<const uint16_t *>(values), expanding ? first : first + operand,
                       expanding ? first + operand : first, masked, gather, static_cast<const float *>(nullptr));
    return hipGetLastError();
}

bool select_prepare_fused(int D, int L, int K)
{
    // pays while a handful of resident workgroups per CU cover all rows at once; beyond that the repeated
    // selections cost more than the launch they save
    return D <= 1024 && size_t(D + K + kFusedRows * D) * 4 <= 48 * 1024;
}

hipError_t launch_select_prepare(int D, int L, int K, bool expanding, const float *scores, const void *values,
                                 int32_t *offsets_out, void *forward_operand, void *backward_operand,
                                 hipStream_t stream)
{
    const size_t lds = size_t(D + K + kFusedRows * D) * 4;
    hipLaunchKernelGGL(select_materialize_kernel<kFusedRows>, dim3((D + L + kFusedRows - 1) / kFusedRows),
                       dim3(kSelectThreads), lds, stream, D, L, K, scores, static_cast<const uint16_t *>(values),
                       offsets_out, static_cast<uint16_t *>(expanding ? forward_operand : backward_operand),
                       static_cast<uint16_t *>(expanding ? backward_operand : forward_operand));
    return hipGetLastError();
}

template <int BM, int BN, int NW>
static hipError_t launch_mm_persistent(int T, int NC, int KD, int a_cols, int c_cols, const uint16_t *A,
                                       const uint16_t *Wf, uint16_t *C, hipStream_t stream)
{
    using Tl = MmTile<BM, BN, NW>;
    constexpr int kLds = kRing * Tl::X_BYTES + Tl::C_BYTES;
    static_assert(kLds <= 160 * 1024, "ring and result tile fit the LDS of a CU");
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&mm_persistent_kernel<BM, BN, NW>), kLds, lds_allowed)) return e;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = NC / BN;
    int group_n = tile_group(tiles_m, tiles_n, BN, KD);
    // rows of the grouped order are divided by tiles_m with one multiply-high: exact while rows * tiles_m < 2^32;
    // in the plain order the quotient is always 0, which a multiplier of 0 gives for any size
    if (uint64_t(tiles_m) * tiles_m * (tiles_n / group_n) >= (uint64_t(1) << 32)) group_n = tiles_n;
    const unsigned magic = group_n == tiles_n ? 0u : unsigned(((uint64_t(1) << 32) + tiles_m - 1) / tiles_m);
    hipLaunchKernelGGL((mm_persistent_kernel<BM, BN, NW>), dim3(256), dim3(Tl::THREADS), kLds, stream, T, NC, KD,
                       a_cols, c_cols, tiles_m, tiles_n, group_n, magic, A, Wf, C);
    return hipGetLastError();
}

constexpr int kMmWaves = 8;  // two waves per SIMD: one wave's waits hide behind the other's MFMAs

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
    const int c_cols = a.masked ? a.D : a.L;
    const int a_cols = a.masked ? a.L : a.D;
    // a group of layers sharing their input: the sets' results side by side, or their contributions summed
    const int NC = c_cols * a.dst_sets;
    const int KD = a_cols * a.src_sets;
    uint16_t *Wf = static_cast<uint16_t *>(a.ws);
    if (!a.prepared) {
        if (a.src_sets != 1 || a.dst_sets != 1) return hipErrorInvalidValue;  // groups come prepared
        const OperandPlace place = {KD, 0, 0, 0};
        hipLaunchKernelGGL(materialize_kernel, materialize_grid(a.D, a.L, a.masked ? NC : 0, a.masked ? 0 : NC, 1), dim3(256), 0, stream, a.D, a.L, a.K,
                           a.masked ? NC / kMatRows : 0, a.offsets, static_cast<const uint16_t *>(a.values), Wf, Wf, place, place,
                           static_cast<const float *>(nullptr));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const uint16_t *A = static_cast<const uint16_t *>(a.src);
    uint16_t *C = static_cast<uint16_t *>(a.dst);
    const int T = int(a.T);
    const int64_t tiles160 = ((a.T + 159) / 160) * ((NC + 255) / 256);
    if (NC % 256 == 0) {
        // more tiles than CUs: one workgroup per CU walks its tiles with the pipeline kept running
        if (tiles160 > 256) return launch_mm_persistent<160, 256, kMmWaves>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
        switch (pick_tile(a.T, NC)) {
        case 192: return launch_mm<192, 256, kMmWaves>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
        case 160: return launch_mm<160, 256, kMmWaves>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
        case 128: return launch_mm<128, 256, kMmWaves>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
        case 96: return launch_mm<96, 256, kMmWaves>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
        default: return launch_mm<64, 256, kMmWaves>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
        }
    }
    return launch_mm<128, 128, 4>(T, NC, KD, a_cols, c_cols, A, Wf, C, stream);
}

}  // namespace dd
