// Variants of wavefront_ll.hip, part 0, with the optional peephole and clipping terms in the gate phase.
#define RNN_LL_PART 0
#define RNN_CELL_EXT 1
#include "wavefront_ll.hip"
