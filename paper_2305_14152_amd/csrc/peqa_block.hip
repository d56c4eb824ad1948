// Placeholder: the block-level entry points are added below in this file.
#include "peqa_kernels.h"
