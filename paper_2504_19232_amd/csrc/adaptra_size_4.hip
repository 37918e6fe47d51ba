// The scenario-lanes and candidate-lanes recurrence kernels at 4 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 4
#include "adaptra_size.inc"
