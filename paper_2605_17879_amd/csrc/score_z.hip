// The scoring launches that write the optional z output: the same source as score.hip,
// compiled as a translation unit of its own so that the two halves build side by side.
#define GD_SCORE_WANT_Z 1
#include "score.hip"
