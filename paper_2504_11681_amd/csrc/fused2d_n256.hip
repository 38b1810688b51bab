// 2-D image kernels for images with 256 rows (first-axis length N1 = 256).
#define TFNO_N1 256
#include "fused2d_images.inc"
