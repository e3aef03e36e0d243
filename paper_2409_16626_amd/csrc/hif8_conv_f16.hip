// Conversion kernels and launchers of libhif8 for f16 tensors (see hif8_conv.hpp).
#include "hif8_conv.hpp"

HIF8_INSTANTIATE_CONV(hif8dev::kSrcF16)
