#define V16_DT DT_F16
#define V16_PRE "f16"
#define V16_FN variants_f16_nn
#include "variants_16nn.inc"
