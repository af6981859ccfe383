// Pieces shared by the kernels that stream their operands from global memory straight into a ring of LDS
// stages (weight gradient, products with many tiles): the transfer itself and the order of work in a k-step.
#pragma once
#include <stdint.h>

namespace dd {

// Sixteen bytes per lane from global memory straight into LDS: lane l of the wave lands at lds_base + 16 l.
// lds_base is a byte address inside LDS and must be the same in every lane.  Written as assembly so that
// the compiler does not serialise every later LDS read behind the transfer; completion is tracked by hand
// with the vector-memory counter (transfers finish in issue order).
__device__ __forceinline__ void global_to_lds_16(const void *g, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(g) : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_address(const void *p)
{
    return unsigned(reinterpret_cast<size_t>((__attribute__((address_space(3))) const char *)(p)));
}

// Order of work inside a k-step.  Fragments are fetched A0, B0, A1, B1, ... and the MFMAs are taken in the
// order in which their fragments arrive: by max(a, b).
template <int FA, int FB>
struct WgOrder {
    int mfma_a[FA * FB], mfma_b[FA * FB];
    int frag_is_a[FA + FB], frag_idx[FA + FB];
    constexpr WgOrder() : mfma_a(), mfma_b(), frag_is_a(), frag_idx()
    {
        int n = 0;
        for (int level = 0; level < (FA > FB ? FA : FB); ++level)
            for (int a = 0; a < FA; ++a)
                for (int b = 0; b < FB; ++b)
                    if ((a > b ? a : b) == level) { mfma_a[n] = a; mfma_b[n] = b; ++n; }
        int k = 0;
        for (int i = 0; i < (FA > FB ? FA : FB); ++i) {
            if (i < FA) { frag_is_a[k] = 1; frag_idx[k] = i; ++k; }
            if (i < FB) { frag_is_a[k] = 0; frag_idx[k] = i; ++k; }
        }
    }
};

}  // namespace dd
