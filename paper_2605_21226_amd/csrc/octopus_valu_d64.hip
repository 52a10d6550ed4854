#define OCTOPUS_D 64
#define OCTOPUS_PART 2
#include "octopus_plans.inc"
