#define OCN_SLICE 3
#define OCN_NSLICES 4
#include "red_inst.inl"
