// Internal: compiled-kernel table entries shared by the instantiation units and the C ABI.
#pragma once
#include <stdint.h>

namespace wt {

struct KernelEntry {
    int bm, bn, bk, wm, wn, wk, st;  // wk: wavefronts sharing a sub-tile along k (nwave = wm*wn*wk)
    int lds_bytes;
    int lds_bytes_persistent;  // dynamic LDS of the persistent kernel (stages + C staging + hand-over slot)
    const void* fn;  // __global__ function taking GemmArgs by value (NULL in a host-only build)
    const void* fn_persistent;  // the same configuration as a persistent kernel
};

// list: 0 = large, 1 = medium, 2 = small.  in: 0 bf16, 1 fp8.  out: 0 f32, 1 bf16.
// Returns the entries of that translation unit (count in *n), or NULL if the pair is not built.
const KernelEntry* kernel_list(int in, int out, int list, int* n);

}  // namespace wt
