#define OCTOPUS_D 128
#include "octopus_plans_paged_qjl.inc"
