// Instantiation unit of the attention kernels: expands the WT_ATTN list of configs.def into kernels and a table
// of their entry points (structural key <T_Q, 1, T_KV, wavefronts>: bm = T_Q, bn = 1, bk = T_KV).
#include "attn_kernel.hpp"
#include "registry.hpp"

namespace wt {

#define WT_ATTN(TQ, TKV, NW)                                                \
    {TQ, 1, TKV, NW, 1, 1, 1, AttnTraits<TQ, TKV, NW>::LDS_BYTES, 0,        \
     reinterpret_cast<const void*>(&attn_kernel<TQ, TKV, NW>), nullptr},
static const KernelEntry kAttnEntries[] = {
#define WT_LIST_ATTN
#include "configs.def"
#undef WT_LIST_ATTN
};
#undef WT_ATTN

const KernelEntry* wt_kernels_attn(int* n) {
    *n = static_cast<int>(sizeof(kAttnEntries) / sizeof(kAttnEntries[0]));
    return kAttnEntries;
}

}  // namespace wt
