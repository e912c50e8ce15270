// The single-sweep kernel for ComplEx: same source, own translation unit (compiles in parallel).
#define LEGEND_FAST_SCORE 2
#include "kernels_chunk_fast.hip"
