// Search kernels for a dataset stored as uint8 (see search_kernels_impl.h).
#define CAGRA_ELEM 2
#define CAGRA_ELEM_NAME u8
#include "search_kernels_impl.h"
