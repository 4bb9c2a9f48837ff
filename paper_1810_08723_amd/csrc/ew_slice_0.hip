#define OCN_SLICE 0
#define OCN_NSLICES 8
#include "ew_inst.inl"
