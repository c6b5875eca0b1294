// Per-kernel resource table: what the compiler reported for every projection-kernel instantiation when this
// library was built (kernel_resources.inc is written by the build from hipcc's kernel-resource-usage remarks).
// The cost model's W(c) (wave capacity, "SM" of Eq. 6) is derived from it instead of a register-count guess.
#include <cstring>

#include "ramp_internal.h"

namespace ramp {

static const KernelResources kResources[] = {
#include "kernel_resources.inc"
    {nullptr, 0, {0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0, 0},
};

const KernelResources *find_resources(const char *family, const int *targs, int n_targs)
{
    for (const KernelResources *r = kResources; r->family; ++r) {
        if (r->n_targs != n_targs || std::strcmp(r->family, family) != 0) continue;
        bool same = true;
        for (int i = 0; i < n_targs; ++i) same = same && r->targs[i] == targs[i];
        if (same) return r;
    }
    return nullptr;
}

}  // namespace ramp
