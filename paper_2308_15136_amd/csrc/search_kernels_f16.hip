// Search kernels for a dataset stored as fp16 (see search_kernels_impl.h).
#define CAGRA_ELEM 1
#define CAGRA_ELEM_NAME f16
#include "search_kernels_impl.h"
