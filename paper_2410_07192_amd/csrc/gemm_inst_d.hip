// Explicit instantiations of the tiled bf16 GEMM for some epilogue combinations (compiled in parallel with the others).
#include "gemm_tile.h"

namespace pf {
namespace gemm {

template hipError_t launch_fast<bf16_t, E_BIAS | E_RESID>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
template hipError_t launch_fast<bf16_t, E_BIAS | E_GELU | E_PRE>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);

}  // namespace gemm
}  // namespace pf
