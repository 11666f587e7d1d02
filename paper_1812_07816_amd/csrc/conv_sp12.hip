// The plane-streaming convolution of conv_sp.hip with 12-row patches (3 rows per wave), for output planes that
// 16-row patches cover badly; see the note at the top of that file.
#define SP_TH 12
#define SP_RH 3
#define SP_NS th12
#include "conv_sp.hip"
