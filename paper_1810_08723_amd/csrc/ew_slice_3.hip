#define OCN_SLICE 3
#define OCN_NSLICES 8
#include "ew_inst.inl"
