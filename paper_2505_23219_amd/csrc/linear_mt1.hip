// Instantiations of the skinny linear kernel for up to 16 rows of x.
#include "linear_impl.h"

namespace ghd {

ghd_status launch_linear_mt1(const FusedArgs& a, hipStream_t st) { return launch_linear_mt<1>(a, st); }

}  // namespace ghd
