#define OCTOPUS_D 128
#define OCTOPUS_PART 4
#include "octopus_plans.inc"
