// Implicit-GEMM instantiations that read weights pre-packed by hgc_conv2d_pack_weights.
#define HGC_IGEMM_PACKED 1
#define HGC_IGEMM_ACCESSOR igemm_variants_packed
#include "igemm_kernel.h"
