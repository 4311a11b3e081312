// fp32 instantiation of the prefix-tree gradient kernels (see sig_tree_backward_impl.h).
#include "sig_tree_backward_impl.h"

namespace sig {

bool tree_backward_supported(const Shape &sh) { return tb_workspace_bytes(sh, 4) >= 0; }

int64_t tree_backward_workspace_bytes(const Shape &sh, sig_dtype dtype)
{
    return tb_workspace_bytes(sh, dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double)));
}

hipError_t launch_tree_backward_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    return launch_tb<float, false>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

}  // namespace sig
