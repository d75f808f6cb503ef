// Search kernels for a dataset stored as fp32 (see search_kernels_impl.h).
#define CAGRA_ELEM 0
#define CAGRA_ELEM_NAME f32
#include "search_kernels_impl.h"
