// 2-D image kernels of the real-field FNO layer for images with 64 rows.
#define TFNO_N1 64
#define TFNO_FNO 1
#include "fused2d_images.inc"
