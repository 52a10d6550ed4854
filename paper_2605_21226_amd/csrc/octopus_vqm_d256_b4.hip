#define OCTOPUS_D 256
#define OCTOPUS_VB 4
#include "octopus_plans_vqm.inc"
