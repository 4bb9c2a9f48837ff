#define OCN_SLICE 7
#define OCN_NSLICES 8
#include "ew_inst.inl"
