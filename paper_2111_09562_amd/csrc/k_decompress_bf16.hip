// Decompression kernels with bfloat16 output (COMET Sec. 3.4): see k_decompress_body.h.
#define COMET_DEC_OUT 2
#include "k_decompress_body.h"
