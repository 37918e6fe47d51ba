// The scenario-lanes and candidate-lanes recurrence kernels at 32 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 32
#include "adaptra_size.inc"
