// One translation unit per (tile configuration, input type): compiled with -DHIDET_TU=<config index>
// and -DHIDET_TYPE=<0 f32 | 1 f16 | 2 bf16>.  Exports hidet_register_<index>_<type>(Registry*).
#include "registry.hpp"

#ifndef HIDET_TU
#error "compile with -DHIDET_TU=<config index> -DHIDET_TYPE=<type index>"
#endif

#define HIDET_CAT2(a, b, c, d) a##b##c##d
#define HIDET_CAT(a, b, c, d) HIDET_CAT2(a, b, c, d)

#if HIDET_TYPE == 0
using ElemT = float;
#define X16(...)
#define X32(idx, BM, BN, BK, WM, WN, MI, TA, SC)                                              \
  extern "C" void HIDET_CAT(hidet_register_, idx, _, HIDET_TYPE)(hidet::Registry * r) {   \
    hidet::register_config<ElemT, BM, BN, BK, WM, WN, MI, TA, SC>(*r, idx, HIDET_TYPE);       \
  }
#else
#if HIDET_TYPE == 1
using ElemT = hidet::f16;
#else
using ElemT = hidet::bf16;
#endif
#define X32(...)
#define X16(idx, BM, BN, BK, WM, WN, MI, TA, SC)                                              \
  extern "C" void HIDET_CAT(hidet_register_, idx, _, HIDET_TYPE)(hidet::Registry * r) {   \
    hidet::register_config<ElemT, BM, BN, BK, WM, WN, MI, TA, SC>(*r, idx, HIDET_TYPE);       \
  }
#endif

#include "configs.def"
