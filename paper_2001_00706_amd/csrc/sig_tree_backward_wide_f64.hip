// fp64 instantiation of the prefix-tree gradient kernels for d = 9..16 (see sig_tree_backward_impl.h).
#include "sig_tree_backward_impl.h"

namespace sig {

hipError_t launch_tree_backward_wide(const Shape &sh, const double *path, const double *sig, const double *gout,
                                     double *gpath, double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    return launch_tb<double, true>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

}  // namespace sig
