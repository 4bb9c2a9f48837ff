#define OCN_SLICE 1
#define OCN_NSLICES 8
#include "ew_inst.inl"
