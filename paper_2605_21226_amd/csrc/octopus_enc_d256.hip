#define OCTOPUS_D 256
#define OCTOPUS_PART 3
#include "octopus_plans.inc"
