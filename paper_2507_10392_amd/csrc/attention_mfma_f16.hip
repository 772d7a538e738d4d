// The fp16 build of the matrix-core attention kernels: the same source with IEEE half as element type.
#define ZS_ATTN_F16 1
#include "attention_mfma.hip"
