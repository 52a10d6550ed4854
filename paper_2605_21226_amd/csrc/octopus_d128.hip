#define OCTOPUS_D 128
#define OCTOPUS_PART 1
#include "octopus_plans.inc"
