// The scenario-lanes and candidate-lanes recurrence kernels at 24 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 24
#include "adaptra_size.inc"
