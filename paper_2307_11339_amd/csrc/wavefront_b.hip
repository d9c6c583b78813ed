// The variants of wavefront.hip with the optional peephole and clipping terms in the gate phase.
#define RNN_CELL_EXT 1
#include "wavefront.hip"
