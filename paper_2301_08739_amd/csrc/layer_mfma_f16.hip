// IEEE half (fp16) instantiation of the fused group attention layer: the kernels of layer_mfma.hip
// with 16-bit storage and matrix-core operands in half precision (v_mfma_f32_16x16x32_f16), the
// precision the paper runs its model in (Sec. 5.1 'Training and inference'); accumulation,
// statistics, softmax and GELU stay fp32 exactly as in the bfloat16 build.
#define FF_LAYER_F16 1
#include "layer_mfma.hip"
