// Score / top-k kernels of the select stage for head_dim 64 (pattern computation, steps 1-4 for the
// queries, 2-4 overall; Sec. 4.1.1).  The implementation is select_impl.hpp.
#define SPA_SELECT_D 64
#include "select_impl.hpp"
