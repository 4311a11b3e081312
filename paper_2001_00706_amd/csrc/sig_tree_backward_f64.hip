// fp64 instantiation of the prefix-tree gradient kernels (see sig_tree_backward_impl.h).
#include "sig_tree_backward_impl.h"

namespace sig {

hipError_t launch_tree_backward_f64(const Shape &sh, const double *path, const double *sig, const double *gout,
                                    double *gpath, double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    return launch_tb<double, false>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

}  // namespace sig
