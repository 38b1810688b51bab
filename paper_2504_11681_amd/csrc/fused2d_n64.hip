// 2-D image kernels for images with 64 rows (first-axis length N1 = 64).
#define TFNO_N1 64
#include "fused2d_images.inc"
