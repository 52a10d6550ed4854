#define OCTOPUS_D 64
#define OCTOPUS_VB 3
#include "octopus_plans_vqm.inc"
