// One instantiation unit: compile with -DWT_IN=<0|1> -DWT_OUT=<0|1> -DWT_LIST=<0|1|2>.
// Expands the matching list of configs.def into kernels and a table of their entry points.
#include "gemm_kernel.hpp"
#include "registry.hpp"

#if WT_IN == 0
#if WT_LIST == 0
#define WT_LIST_LARGE_BF16
#elif WT_LIST == 1
#define WT_LIST_MEDIUM_BF16
#else
#define WT_LIST_SMALL_BF16
#endif
#else
#if WT_LIST == 0
#define WT_LIST_LARGE_FP8
#elif WT_LIST == 1
#define WT_LIST_MEDIUM_FP8
#else
#define WT_LIST_SMALL_FP8
#endif
#endif

#define WT_CAT2(a, b) a##b
#define WT_CAT(a, b) WT_CAT2(a, b)
#define WT_FN_NAME WT_CAT(WT_CAT(WT_CAT(WT_CAT(WT_CAT(wt_kernels_in, WT_IN), _out), WT_OUT), _list), WT_LIST)

namespace wt {

#define WT_CFGX(BM, BN, BK, WM, WN, WK, ST, MIF)                                                       \
    {BM, BN, BK, WM, WN, WK, ST, GemmTraits<BM, BN, BK, WM, WN, ST, WT_IN, WT_OUT, WK, MIF>::LDS_BYTES,  \
     GemmTraits<BM, BN, BK, WM, WN, ST, WT_IN, WT_OUT, WK, MIF>::LDS_BYTES_PERSISTENT,                   \
     reinterpret_cast<const void*>(&gemm_kernel<BM, BN, BK, WM, WN, ST, WT_IN, WT_OUT, WK, MIF>),        \
     reinterpret_cast<const void*>(&gemm_kernel_persistent<BM, BN, BK, WM, WN, ST, WT_IN, WT_OUT, WK, MIF>)},
#define WT_CFGK(BM, BN, BK, WM, WN, WK, ST) WT_CFGX(BM, BN, BK, WM, WN, WK, ST, 0)
#define WT_CFG(BM, BN, BK, WM, WN, ST) WT_CFGX(BM, BN, BK, WM, WN, 1, ST, 0)
// the same key computed with 16x16 MFMA tiles although its sub-tile would allow 32x32
#define WT_CFG16(BM, BN, BK, WM, WN, ST) WT_CFGX(BM, BN, BK, WM, WN, 1, ST, 16)
static const KernelEntry kEntries[] = {
#include "configs.def"
};
#undef WT_CFG
#undef WT_CFG16
#undef WT_CFGK
#undef WT_CFGX

const KernelEntry* WT_FN_NAME(int* n) {
    *n = static_cast<int>(sizeof(kEntries) / sizeof(kEntries[0]));
    return kEntries;
}

}  // namespace wt
