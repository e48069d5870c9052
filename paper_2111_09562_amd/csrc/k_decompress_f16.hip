// Decompression kernels with IEEE half output (COMET Sec. 3.4): see k_decompress_body.h.
#define COMET_DEC_OUT 1
#include "k_decompress_body.h"
