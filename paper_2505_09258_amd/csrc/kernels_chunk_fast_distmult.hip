// The single-sweep kernel for DistMult: same source, own translation unit (compiles in parallel).
#define LEGEND_FAST_SCORE 1
#include "kernels_chunk_fast.hip"
