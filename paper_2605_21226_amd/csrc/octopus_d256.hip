#define OCTOPUS_D 256
#define OCTOPUS_PART 1
#include "octopus_plans.inc"
