#define V16_DT DT_BF16
#define V16_PRE "bf16"
#define V16_FN variants_bf16_nt
#include "variants_16nt.inc"
