// Implicit-GEMM instantiations that read weights pre-packed by hgc_conv2d_pack_weights: part 0 of the table.
#define HGC_IGEMM_PACKED 1
#define HGC_IGEMM_PART 0
#define HGC_IGEMM_ACCESSOR igemm_variants_packed_0
#include "igemm_kernel.h"
