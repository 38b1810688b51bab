// 2-D image kernels for images with 128 rows (first-axis length N1 = 128).
#define TFNO_N1 128
#include "fused2d_images.inc"
