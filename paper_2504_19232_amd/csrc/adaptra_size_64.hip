// The scenario-lanes and candidate-lanes recurrence kernels at 64 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 64
#include "adaptra_size.inc"
