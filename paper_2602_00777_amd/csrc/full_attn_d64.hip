// Full-layer streaming kernels for head_dim 64 (see full_attn_impl.h).
#define HYLRA_BUILD_D 64
#include "full_attn_impl.h"
