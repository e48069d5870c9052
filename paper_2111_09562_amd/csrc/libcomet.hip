// Single translation unit of libcomet: the kernels and the C ABI are compiled
// together so that no relocatable device code is needed.
#include "k_quantize.hip"
#include "k_quantize_rows.hip"
#include "k_codebook.hip"
#include "k_encode.hip"
#include "k_reconstruct.hip"
#include "k_decompress.hip"
#include "k_stats.hip"
#include "comet_api.hip"
