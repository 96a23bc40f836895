// The 16-bit GEMM kernels built for fp16 storage (the paper's precision): the same source as for bf16.
#define KFKB_H16_IS_F16 1
#include "gemm_bf16.hip"
