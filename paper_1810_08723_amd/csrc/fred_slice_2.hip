// Slice 2 of the fused elementwise+reduce kernels (see fred_inst.inl).
#define OCN_SLICE 2
#define OCN_NSLICES 4
#include "fred_inst.inl"
