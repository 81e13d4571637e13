// The LDS-staged forward kernels once more, for spline degrees 4 and 5 (window of six rows).  kan_lds.hip is
// written against kMaxK; this translation unit compiles it with kMaxK = 6 in the namespace of the other six-row
// builds (kan_generic_k5.hip calls forward_lds_plan / launch_forward_lds of that namespace).
#define KAN_MAXK 6
#define KAN_NS kan_k5
#include "kan_lds.hip"
