// The wide 3x3 kernel's instances for one storage type (see the end of convbig.hip).
#define OCTO_BIG_ONLY_BF16
#include "convbig.hip"
