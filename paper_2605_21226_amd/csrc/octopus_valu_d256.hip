#define OCTOPUS_D 256
#define OCTOPUS_PART 2
#include "octopus_plans.inc"
