// Third translation unit of the tag-in-data kernel: bf16 layers whose width is not 128 times a power
// of two, and layers of 2048 units (see wavefront_ll.hip).
#define RNN_LL_PART 2
#include "wavefront_ll.hip"
