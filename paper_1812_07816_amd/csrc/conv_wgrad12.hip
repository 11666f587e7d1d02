// The weight-gradient kernel of conv_wgrad.hip with 12-row patches, for dy planes that 16-row patches cover badly; see
// the note at the top of that file.
#define WG_TH 12
#define WG_NS th12
#include "conv_wgrad.hip"
