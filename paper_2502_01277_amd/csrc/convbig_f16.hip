// The wide 3x3 kernel's instances for one storage type (see the end of convbig.hip).
#define OCTO_BIG_ONLY_F16
#include "convbig.hip"
