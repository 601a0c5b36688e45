// Instantiations of the fused QKV + attention kernel for up to 32 rows of x.
#include "qkv_attn_impl.h"

namespace ghd {

ghd_status launch_qkv_attn_mt2(const FusedArgs& a, hipStream_t st) { return launch_qkv_attn_mt<2>(a, st); }

}  // namespace ghd
