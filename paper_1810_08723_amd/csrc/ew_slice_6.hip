#define OCN_SLICE 6
#define OCN_NSLICES 8
#include "ew_inst.inl"
