// The scenario-lanes and candidate-lanes recurrence kernels at 48 stages (see adaptra_size.inc).
#define ADAPTRA_SIZE 48
#include "adaptra_size.inc"
