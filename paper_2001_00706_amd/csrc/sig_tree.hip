// Prefix-tree kernel family, d = 2..8 (see sig_tree_impl.h); d = 9..16 is instantiated in sig_tree_wide.hip.
#include "sig_tree_impl.h"

namespace sig {

bool tree_supported(const Shape &sh)
{
    if (sh.S >= (int64_t(1) << 31) || sh.N < 2) return false;
    return (sh.d >= 2 && sh.d <= 8 && sh.N <= kTreeMaxDepth) || (sh.d >= 9 && sh.d <= 16 && sh.N <= kTreeWideMaxDepth);
}

template <typename T>
hipError_t launch_tree_t(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    if (!tree_supported(sh)) return hipErrorNotSupported;
    if (sh.d > 8) return launch_tree_wide(sh, path, out, st);
    switch (sh.d) {
        case 2: return launch_tree_d<T, 2>(sh, path, out, st);
        case 3: return launch_tree_d<T, 3>(sh, path, out, st);
        case 4: return launch_tree_d<T, 4>(sh, path, out, st);
        case 5: return launch_tree_d<T, 5>(sh, path, out, st);
        case 6: return launch_tree_d<T, 6>(sh, path, out, st);
        case 7: return launch_tree_d<T, 7>(sh, path, out, st);
        case 8: return launch_tree_d<T, 8>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

hipError_t launch_tree_f32(const Shape &sh, const float *path, float *out, hipStream_t st) { return launch_tree_t<float>(sh, path, out, st); }
hipError_t launch_tree_f64(const Shape &sh, const double *path, double *out, hipStream_t st) { return launch_tree_t<double>(sh, path, out, st); }

}  // namespace sig
