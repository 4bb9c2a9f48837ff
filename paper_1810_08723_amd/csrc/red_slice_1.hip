#define OCN_SLICE 1
#define OCN_NSLICES 4
#include "red_inst.inl"
