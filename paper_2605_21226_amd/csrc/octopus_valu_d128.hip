#define OCTOPUS_D 128
#define OCTOPUS_PART 2
#include "octopus_plans.inc"
