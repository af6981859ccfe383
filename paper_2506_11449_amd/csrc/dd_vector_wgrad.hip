// Weight gradient on the vector ALUs with packed bf16 dot products (bf16 storage, fp32 accumulate),
// Fig. 3 h-i:  dV[k][p] = sum_t A[t, p] * B[t, (p + o_k) mod D],  A [T x L] the short side, B [T x D] the long.
//
// Only the K stored diagonals are visited: a lane owns one position p and keeps one fp32 accumulator per
// diagonal of its block of diagonals; v_dot2_f32_bf16 adds two tokens per instruction.  Tokens are
// processed in tiles of 8*NT; both operands are transposed on their way into LDS (8 x 8 register
// transposes) so that the eight tokens of one (column, octet) pair are one 16-byte LDS word: a lane then
// needs exactly one ds_read_b128 per diagonal and octet, at an address fixed for the whole kernel, and
// neighbouring lanes read neighbouring words (a one-word pad per column keeps them on distinct banks).
// The tile is double buffered; the next tile's global loads are in flight while the current one is used.
//
// Workgroup = 256 positions x one block of <= 32 diagonals x one chunk of tokens.  Chunks are dealt to
// the XCDs so that all workgroups of a chunk share an L2; they are summed afterwards in index order.
#include "dd_common.h"
#include "dd_launch.h"

namespace dd {

typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kVwThreads = 256;
constexpr int kVwKBlock = 32;     // accumulators (diagonals) per lane
constexpr int kVwXcds = 8;
constexpr int kVwCusPerXcd = 32;

__device__ __forceinline__ float dot2(unsigned a, unsigned b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, a), __builtin_bit_cast(bf16x2v, b), c, false);
}

template <int NT, int MAXB>
__global__ __launch_bounds__(kVwThreads) void wgrad_dot2_kernel(int T, int D, int L, int K, int p_blocks, int k_blocks,
                                                                int chunks, const uint16_t *__restrict__ A,
                                                                const uint16_t *__restrict__ B,
                                                                const int *__restrict__ offsets,
                                                                float *__restrict__ partial)
{
    constexpr int STRIDE = (NT + 1) * 16;   // bytes per column: NT octets of eight tokens + one pad word
    constexpr int TILE = 8 * NT;            // tokens per tile
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int buf_bytes = (D + kVwThreads) * STRIDE;

    const int per_chunk = p_blocks * k_blocks;
    const int xcd = blockIdx.x % kVwXcds, local = blockIdx.x / kVwXcds;
    const int chunk = (local / per_chunk) * kVwXcds + xcd;
    if (chunk >= chunks) return;
    const int sub = local % per_chunk;
    const int p0 = (sub / k_blocks) * kVwThreads;
    const int kb = sub % k_blocks;
    const int k_begin = int(int64_t(kb) * K / k_blocks), k_end = int(int64_t(kb + 1) * K / k_blocks);
    const int nk = k_end - k_begin;  // <= kVwKBlock

    const int tiles_total = (T + TILE - 1) / TILE;
    const int tile_begin = int(int64_t(chunk) * tiles_total / chunks);
    const int tile_end = int(int64_t(chunk + 1) * tiles_total / chunks);
    const int n_tiles = tile_end - tile_begin;
    const int t_end = min(tile_end * TILE, T);

    const int p = p0 + tid;
    const bool active = p < L;

    // LDS byte address of every diagonal's column for this lane (fixed for the whole kernel)
    int qa[kVwKBlock];
#pragma unroll
    for (int kk = 0; kk < kVwKBlock; ++kk) {
        int q = 0;
        if (active && kk < nk) {
            q = p + canonical_offset(offsets[k_begin + kk], D);
            if (q >= D) q -= D;
        }
        qa[kk] = q * STRIDE;
    }
    const int a_addr = (D + tid) * STRIDE;

    // staging: a block is 8 tokens x 8 columns, MAXB blocks per thread and tile
    const int cg_b = D / 8;                  // column groups of B; A adds up to 32 more
    const int n_blocks = NT * (cg_b + kVwThreads / 8);
    const uint16_t *blk_src[MAXB];
    int blk_stride[MAXB], blk_dst[MAXB], blk_oct[MAXB];
    bool blk_is_a[MAXB], blk_ok[MAXB];
#pragma unroll
    for (int n = 0; n < MAXB; ++n) {
        const int b = tid + kVwThreads * n;
        const int oct = b / (cg_b + kVwThreads / 8), cg = b % (cg_b + kVwThreads / 8);
        const bool is_a = cg >= cg_b;
        const int col = is_a ? p0 + (cg - cg_b) * 8 : cg * 8;
        blk_is_a[n] = is_a;
        blk_ok[n] = b < n_blocks && (!is_a || col < L);
        blk_src[n] = (is_a ? A : B) + (blk_ok[n] ? col : 0);
        blk_stride[n] = is_a ? L : D;
        blk_oct[n] = oct;
        blk_dst[n] = (is_a ? D + (cg - cg_b) * 8 : cg * 8) * STRIDE + oct * 16;
    }
    u32x4 rows0[MAXB][8];
    // Tokens past the chunk (and whole tiles past its end) must add nothing: one zero factor, the short
    // side, is enough; it is masked rather than branched on so that the loads stay in flight together.
#define DD_VW_LOAD(rows, tile_)                                                                         \
    {                                                                                                   \
        const int tb = (tile_begin + min((tile_), n_tiles - 1)) * TILE;                                 \
        const bool past = (tile_) >= n_tiles;                                                           \
        _Pragma("unroll") for (int n = 0; n < MAXB; ++n)                                                \
            _Pragma("unroll") for (int r = 0; r < 8; ++r) {                                             \
                const int t = tb + blk_oct[n] * 8 + r;                                                  \
                const u32x4 v = *reinterpret_cast<const u32x4 *>(blk_src[n] + size_t(min(t, T - 1)) * blk_stride[n]); \
                const unsigned keep = 0u - unsigned(!(blk_is_a[n] && (past || t >= t_end)));            \
                rows[n][r] = v & keep;                                                                  \
            }                                                                                           \
    }
    // rows r (tokens) x 8 columns  ->  columns c x 8 tokens, one 16-byte word per column
#define DD_VW_STORE(rows, buf_)                                                                             \
    _Pragma("unroll") for (int n = 0; n < MAXB; ++n) if (blk_ok[n]) {                                   \
        unsigned char *dst = smem + (buf_) * buf_bytes + blk_dst[n];                                    \
        _Pragma("unroll") for (int w = 0; w < 4; ++w) {                                                 \
            u32x4 even, odd;                                                                            \
            _Pragma("unroll") for (int a = 0; a < 4; ++a) {                                             \
                const unsigned lo = rows[n][2 * a][w], hi = rows[n][2 * a + 1][w];                      \
                even[a] = (lo & 0xffffu) | (hi << 16);                                                  \
                odd[a] = (lo >> 16) | (hi & 0xffff0000u);                                               \
            }                                                                                           \
            *reinterpret_cast<u32x4 *>(dst + (2 * w) * STRIDE) = even;                                  \
            *reinterpret_cast<u32x4 *>(dst + (2 * w + 1) * STRIDE) = odd;                               \
        }                                                                                               \
    }

    float acc[kVwKBlock];
#pragma unroll
    for (int kk = 0; kk < kVwKBlock; ++kk) acc[kk] = 0.f;

    // one tile: NT octets x kVwKBlock diagonals
#define DD_VW_COMPUTE(buf_)                                                                             \
    {                                                                                                   \
        const unsigned char *cur = smem + (buf_) * buf_bytes;                                           \
        _Pragma("unroll") for (int oct = 0; oct < NT; ++oct) {                                          \
            const u32x4 a4 = *reinterpret_cast<const u32x4 *>(cur + a_addr + oct * 16);                 \
            /* slots past the block's last diagonal read column 0 and are dropped: no branch, so that */ \
            /* the LDS reads of an octet stay in flight together */                                     \
            _Pragma("unroll") for (int kk = 0; kk < kVwKBlock; ++kk) {                                  \
                const u32x4 b4 = *reinterpret_cast<const u32x4 *>(cur + qa[kk] + oct * 16);             \
                float s = acc[kk];                                                                      \
                s = dot2(a4[0], b4[0], s);                                                              \
                s = dot2(a4[1], b4[1], s);                                                              \
                s = dot2(a4[2], b4[2], s);                                                              \
                s = dot2(a4[3], b4[3], s);                                                              \
                acc[kk] = s;                                                                            \
            }                                                                                           \
        }                                                                                               \
    }

    // the next tile's global loads are in flight while the current one is used; two LDS buffers, one
    // barrier per tile
    DD_VW_LOAD(rows0, 0)
    DD_VW_STORE(rows0, 0)
    __syncthreads();
    for (int i = 0; i < n_tiles; ++i) {
        DD_VW_LOAD(rows0, i + 1)
        __builtin_amdgcn_sched_barrier(0);
        DD_VW_COMPUTE(i & 1)
        __builtin_amdgcn_sched_barrier(0);
        DD_VW_STORE(rows0, (i + 1) & 1)
        __syncthreads();
    }
#undef DD_VW_COMPUTE
#undef DD_VW_LOAD
#undef DD_VW_STORE

    if (active) {
        float *out = partial + (size_t(chunk) * K + k_begin) * L + p;
#pragma unroll
        for (int kk = 0; kk < kVwKBlock; ++kk)
            if (kk < nk) out[size_t(kk) * L] = acc[kk];
    }
}

// ---- host side ----

struct VwPlan {
    bool ok;
    int nt, maxb, p_blocks, k_blocks, chunks, grid;
    size_t lds;
};

static VwPlan plan_vw(int64_t T, int D, int L, int K)
{
    VwPlan pl = {};
    if (T <= 0 || T >= (int64_t(1) << 31) || D % 8 || L % 8) return pl;
    const size_t lds_limit = 160 * 1024;
    for (int nt = 2; nt >= 1; --nt) {
        const size_t lds = 2 * size_t(D + kVwThreads) * (nt + 1) * 16;
        const int blocks = nt * (D / 8 + kVwThreads / 8);
        if (lds <= lds_limit && blocks <= 2 * kVwThreads) {
            pl.nt = nt;
            pl.maxb = (blocks + kVwThreads - 1) / kVwThreads;
            pl.lds = lds;
            pl.ok = true;
            break;
        }
    }
    if (!pl.ok) return pl;
    pl.p_blocks = (L + kVwThreads - 1) / kVwThreads;
    pl.k_blocks = (K + kVwKBlock - 1) / kVwKBlock;
    const int per_chunk = pl.p_blocks * pl.k_blocks;
    int per_xcd = kVwCusPerXcd / per_chunk;  // chunks whose workgroups fill an XCD's 32 CUs in one round
    if (per_xcd < 1) per_xcd = 1;
    int64_t chunks = int64_t(per_xcd) * kVwXcds;
    const int64_t tiles = (T + 8 * pl.nt - 1) / (8 * pl.nt);
    if (chunks > tiles) chunks = tiles;
    pl.chunks = int(chunks);
    pl.grid = int((chunks + kVwXcds - 1) / kVwXcds) * per_chunk * kVwXcds;
    return pl;
}

bool weight_grad_dot2_supported(int64_t T, int D, int L, int K) { return plan_vw(T, D, L, K).ok; }

size_t weight_grad_dot2_ws_bytes(int64_t T, int D, int L, int K)
{
    const VwPlan pl = plan_vw(T, D, L, K);
    return size_t(pl.chunks) * K * L * sizeof(float);
}

int weight_grad_dot2_chunks(int64_t T, int D, int L, int K) { return plan_vw(T, D, L, K).chunks; }

template <int NT, int MAXB>
static hipError_t launch_vw(const WeightGradArgs &a, const VwPlan &pl, hipStream_t stream)
{
    static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&wgrad_dot2_kernel<NT, MAXB>), 160 * 1024, lds_allowed)) return e;
    hipLaunchKernelGGL((wgrad_dot2_kernel<NT, MAXB>), dim3(pl.grid), dim3(kVwThreads), pl.lds, stream, int(a.T), a.D,
                       a.L, a.K, pl.p_blocks, pl.k_blocks, pl.chunks, static_cast<const uint16_t *>(a.A),
                       static_cast<const uint16_t *>(a.B), a.offsets, static_cast<float *>(a.ws));
    return hipGetLastError();
}

// partial sums only; the caller adds the chunks in order
hipError_t launch_weight_grad_dot2_partials(const WeightGradArgs &a, hipStream_t stream)
{
    const VwPlan pl = plan_vw(a.T, a.D, a.L, a.K);
    if (pl.nt == 2) return pl.maxb == 1 ? launch_vw<2, 1>(a, pl, stream) : launch_vw<2, 2>(a, pl, stream);
    return pl.maxb == 1 ? launch_vw<1, 1>(a, pl, stream) : launch_vw<1, 2>(a, pl, stream);
}

}  // namespace dd
