#define OCTOPUS_D 64
#define OCTOPUS_PART 4
#include "octopus_plans.inc"
