// The scenario-lanes and candidate-lanes recurrence kernels at 12 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 12
#include "adaptra_size.inc"
