// Instantiations of the fused QKV + attention kernel for up to 16 rows of x.
#include "qkv_attn_impl.h"

namespace ghd {

ghd_status launch_qkv_attn_mt1(const FusedArgs& a, hipStream_t st) { return launch_qkv_attn_mt<1>(a, st); }

}  // namespace ghd
