#define OCTOPUS_D 128
#define OCTOPUS_PART 3
#include "octopus_plans.inc"
