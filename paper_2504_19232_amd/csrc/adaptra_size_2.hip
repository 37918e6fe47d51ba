// The scenario-lanes and candidate-lanes recurrence kernels at 2 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 2
#include "adaptra_size.inc"
