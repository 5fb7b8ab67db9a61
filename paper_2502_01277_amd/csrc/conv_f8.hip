// The general convolution kernel's instances for one storage type (see the end of conv.hip).
#define OCTO_CONV_ONLY_F8
#include "conv.hip"
