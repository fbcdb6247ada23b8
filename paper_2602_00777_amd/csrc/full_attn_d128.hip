// Full-layer streaming kernels for head_dim 128 (see full_attn_impl.h).
#define HYLRA_BUILD_D 128
#include "full_attn_impl.h"
