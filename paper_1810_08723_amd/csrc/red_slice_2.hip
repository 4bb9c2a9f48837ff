#define OCN_SLICE 2
#define OCN_NSLICES 4
#include "red_inst.inl"
