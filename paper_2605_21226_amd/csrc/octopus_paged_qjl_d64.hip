#define OCTOPUS_D 64
#include "octopus_plans_paged_qjl.inc"
