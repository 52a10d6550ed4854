#define OCTOPUS_PART 3
#include "octopus_plans_sweep.inc"
