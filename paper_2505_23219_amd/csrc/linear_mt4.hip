// Instantiations of the skinny linear kernel for up to 64 rows of x.
#include "linear_impl.h"

namespace ghd {

ghd_status launch_linear_mt4(const FusedArgs& a, hipStream_t st) { return launch_linear_mt<4>(a, st); }

}  // namespace ghd
