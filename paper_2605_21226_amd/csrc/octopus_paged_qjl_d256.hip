#define OCTOPUS_D 256
#include "octopus_plans_paged_qjl.inc"
