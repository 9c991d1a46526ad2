// The kernels of ggnn_search_reg.hip for vector arrays of 4 GiB and more (64-bit row offsets).
#define GGNN_WIDE_OFFSETS 1
#include "ggnn_search_reg.hip"
