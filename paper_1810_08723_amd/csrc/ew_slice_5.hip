#define OCN_SLICE 5
#define OCN_NSLICES 8
#include "ew_inst.inl"
