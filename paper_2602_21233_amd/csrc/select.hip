// Top-k + static merge on caller-supplied scores, and the dispatcher of the score/top-k kernels
// (pattern computation, steps 2-4; Sec. 4.1.1).  The implementation is select_impl.hpp.
#include "select_impl.hpp"
