// Prefix-tree kernel family, d = 9..16 (see sig_tree_impl.h): one level of d scalars per thread below its word.
#include "sig_tree_impl.h"

namespace sig {

template <typename T>
static hipError_t launch_tree_wide_t(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    switch (sh.d) {
        case 9: return launch_tree_d<T, 9>(sh, path, out, st);
        case 10: return launch_tree_d<T, 10>(sh, path, out, st);
        case 11: return launch_tree_d<T, 11>(sh, path, out, st);
        case 12: return launch_tree_d<T, 12>(sh, path, out, st);
        case 13: return launch_tree_d<T, 13>(sh, path, out, st);
        case 14: return launch_tree_d<T, 14>(sh, path, out, st);
        case 15: return launch_tree_d<T, 15>(sh, path, out, st);
        case 16: return launch_tree_d<T, 16>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

hipError_t launch_tree_wide(const Shape &sh, const float *path, float *out, hipStream_t st) { return launch_tree_wide_t<float>(sh, path, out, st); }
hipError_t launch_tree_wide(const Shape &sh, const double *path, double *out, hipStream_t st) { return launch_tree_wide_t<double>(sh, path, out, st); }

}  // namespace sig
