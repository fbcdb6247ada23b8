// Reuse-layer gather kernels for head_dim 64 (see reuse_attn_impl.h).
#define HYLRA_BUILD_D 64
#include "reuse_attn_impl.h"
