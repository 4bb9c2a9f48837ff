#define OCN_SLICE 4
#define OCN_NSLICES 8
#include "ew_inst.inl"
