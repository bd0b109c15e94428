// The fp16 instance of kernels_bf16_convert.hip: same source, element type fp16 (v_mfma_*_f16, fp16 conversions), namespace f16.
#define HX_ELEM_F16 1
#include "kernels_bf16_convert.hip"
