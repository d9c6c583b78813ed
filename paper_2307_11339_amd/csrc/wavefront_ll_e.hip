// Variants of wavefront_ll.hip, part 1, with the optional peephole and clipping terms in the gate phase.
#define RNN_LL_PART 1
#define RNN_CELL_EXT 1
#include "wavefront_ll.hip"
