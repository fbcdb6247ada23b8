// Reuse-layer gather kernels for head_dim 128 (see reuse_attn_impl.h).
#define HYLRA_BUILD_D 128
#include "reuse_attn_impl.h"
