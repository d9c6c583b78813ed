// Second translation unit of the tag-in-data kernel: the fp32 variants (see wavefront_ll.hip).
#define RNN_LL_PART 1
#include "wavefront_ll.hip"
