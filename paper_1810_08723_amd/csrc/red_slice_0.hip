#define OCN_SLICE 0
#define OCN_NSLICES 4
#include "red_inst.inl"
