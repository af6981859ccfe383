// The hard TopK selection (Sec. 3.2, Eq. 4) as a workgroup-level routine, shared by the selection kernel and by
// kernels that select and go on with the result.
//
// Method: scores are mapped to 32-bit keys whose unsigned order is the required total order
// (NaN lowest, -0 == +0) and parked in LDS.  A four-pass byte-wise radix search finds the K-th
// largest key tau and how many of the keys equal to tau still belong to the selection (the
// lowest-indexed ones); each pass is one LDS histogram plus a suffix scan done by a single wave
// with lane shuffles.  A last pass walks the indices in ascending order and compacts the chosen
// ones with a workgroup prefix sum, which also yields them already sorted by index.
#pragma once
#include "dd_common.h"

namespace dd {

constexpr int kSelectThreads = 256;
constexpr int kSelectLdsKeys = 16384;  // score vectors up to this length keep their keys in LDS

__device__ __forceinline__ uint32_t score_key(float s)
{
    if (s != s) return 0u;             // NaN: below every number
    uint32_t u = __float_as_uint(s + 0.0f);  // -0 + 0 = +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the 64 lanes of a wave, without a trip through LDS: four shift-and-add steps inside
// each row of 16 lanes (DPP row_shr, lanes shifted in from outside the row read 0), then the totals of the rows
// before a lane's own row, read from lanes 15, 31 and 47.
__device__ __forceinline__ unsigned wave_inclusive_scan(unsigned v, int lane)
{
#define DD_ROW_SHR(n_) unsigned(__builtin_amdgcn_update_dpp(0, int(v), 0x110 + (n_), 0xf, 0xf, true))
    v += DD_ROW_SHR(1);
    v += DD_ROW_SHR(2);
    v += DD_ROW_SHR(4);
    v += DD_ROW_SHR(8);
#undef DD_ROW_SHR
    const unsigned r0 = unsigned(__builtin_amdgcn_readlane(int(v), 15));
    const unsigned r1 = unsigned(__builtin_amdgcn_readlane(int(v), 31));
    const unsigned r2 = unsigned(__builtin_amdgcn_readlane(int(v), 47));
    const int row = lane >> 4;
    return v + (row >= 1 ? r0 : 0u) + (row >= 2 ? r1 : 0u) + (row >= 3 ? r2 : 0u);
}

// The selection for one score vector `row` by one workgroup of kSelectThreads threads: the K chosen indices go to
// `dst` (global or LDS), ascending.  s_keys: D words of LDS when KEYS_IN_LDS.  Ends without a barrier.
template <bool KEYS_IN_LDS>
__device__ __forceinline__ void select_topk_block(int D, int K, const float *__restrict__ row, uint32_t *s_keys,
                                                  int *dst)
{
    __shared__ unsigned hist[256];
    __shared__ unsigned s_prefix, s_remaining;
    __shared__ unsigned wave_gt[4], wave_eq[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto key_at = [&](int i) -> uint32_t { return KEYS_IN_LDS ? s_keys[i] : score_key(row[i]); };

    if (KEYS_IN_LDS)
        for (int i = tid; i < D; i += kSelectThreads) s_keys[i] = score_key(row[i]);
    if (tid == 0) { s_prefix = 0u; s_remaining = unsigned(K); }
    unsigned mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0u;
        __syncthreads();
        const unsigned prefix = s_prefix, remaining = s_remaining;
        for (int i = tid; i < D; i += kSelectThreads) {
            const uint32_t key = key_at(i);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns bins 255-4l .. 252-4l (descending); find the bin where the running count of
            // larger-or-equal keys first reaches `remaining`
            unsigned h[4], mine = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) { h[j] = hist[255 - 4 * lane - j]; mine += h[j]; }
            const unsigned incl = wave_inclusive_scan(mine, lane);
            unsigned above = incl - mine;  // keys in bins larger than this lane's
            if (above < remaining && incl >= remaining) {  // exactly one lane
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (above + h[j] >= remaining) {
                        s_remaining = remaining - above;  // still to take inside the chosen bin
                        s_prefix = prefix | (unsigned(255 - 4 * lane - j) << shift);
                        break;
                    }
                    above += h[j];
                }
            }
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t tau = s_prefix;          // the K-th largest key
    const unsigned take_eq = s_remaining;   // how many keys equal to tau are selected (>= 1)

    // contiguous chunk of indices per thread, so that a prefix sum keeps ascending order
    const int chunk = (D + kSelectThreads - 1) / kSelectThreads;
    const int lo = min(tid * chunk, D), hi = min(lo + chunk, D);
    unsigned n_gt = 0u, n_eq = 0u;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = key_at(i);
        n_gt += key > tau;
        n_eq += key == tau;
    }
    const unsigned incl_gt = wave_inclusive_scan(n_gt, lane), incl_eq = wave_inclusive_scan(n_eq, lane);
    if (lane == 63) { wave_gt[wave] = incl_gt; wave_eq[wave] = incl_eq; }
    __syncthreads();
    unsigned base_gt = 0u, base_eq = 0u;
    for (int w = 0; w < wave; ++w) { base_gt += wave_gt[w]; base_eq += wave_eq[w]; }
    unsigned eq_rank = base_eq + incl_eq - n_eq;                       // equal keys before this chunk
    unsigned pos = (base_gt + incl_gt - n_gt) + min(eq_rank, take_eq);  // selected before this chunk
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = key_at(i);
        if (key > tau) {
            dst[pos++] = i;
        } else if (key == tau) {
            if (eq_rank < take_eq) dst[pos++] = i;
            ++eq_rank;
        }
    }
}

}  // namespace dd
