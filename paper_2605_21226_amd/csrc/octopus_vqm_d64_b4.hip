#define OCTOPUS_D 64
#define OCTOPUS_VB 4
#include "octopus_plans_vqm.inc"
