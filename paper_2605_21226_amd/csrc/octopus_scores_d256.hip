#define OCTOPUS_D 256
#define OCTOPUS_PART 4
#include "octopus_plans.inc"
