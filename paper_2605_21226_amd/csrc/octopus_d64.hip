#define OCTOPUS_D 64
#define OCTOPUS_PART 1
#include "octopus_plans.inc"
