// Instantiations of the fused QKV + attention kernel for up to 64 rows of x.
#include "qkv_attn_impl.h"

namespace ghd {

ghd_status launch_qkv_attn_mt4(const FusedArgs& a, hipStream_t st) { return launch_qkv_attn_mt<4>(a, st); }

}  // namespace ghd
