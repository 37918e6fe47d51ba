// The scenario-lanes and candidate-lanes recurrence kernels at 16 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 16
#include "adaptra_size.inc"
