#define OCTOPUS_PART 1
#include "octopus_plans_sweep.inc"
