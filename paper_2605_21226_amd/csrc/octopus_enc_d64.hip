#define OCTOPUS_D 64
#define OCTOPUS_PART 3
#include "octopus_plans.inc"
