#define V16_DT DT_BF16
#define V16_PRE "bf16"
#define V16_FN variants_bf16_nn
#include "variants_16nn.inc"
