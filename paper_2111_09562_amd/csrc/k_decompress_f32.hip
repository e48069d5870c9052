// Decompression kernels with fp32 output (COMET Sec. 3.4): see k_decompress_body.h.
#define COMET_DEC_OUT 0
#include "k_decompress_body.h"
