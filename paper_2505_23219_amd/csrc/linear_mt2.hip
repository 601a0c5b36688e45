// Instantiations of the skinny linear kernel for up to 32 rows of x.
#include "linear_impl.h"

namespace ghd {

ghd_status launch_linear_mt2(const FusedArgs& a, hipStream_t st) { return launch_linear_mt<2>(a, st); }

}  // namespace ghd
