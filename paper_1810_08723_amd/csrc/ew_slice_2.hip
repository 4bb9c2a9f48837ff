#define OCN_SLICE 2
#define OCN_NSLICES 8
#include "ew_inst.inl"
