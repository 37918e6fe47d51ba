// The scenario-lanes and candidate-lanes recurrence kernels at 8 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 8
#include "adaptra_size.inc"
