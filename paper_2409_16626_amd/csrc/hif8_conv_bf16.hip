// Conversion kernels and launchers of libhif8 for bf16 tensors (see hif8_conv.hpp).
#include "hif8_conv.hpp"

HIF8_INSTANTIATE_CONV(hif8dev::kSrcBF16)
