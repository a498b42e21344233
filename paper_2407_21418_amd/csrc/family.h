// The compiled uKernel family: every (reg_tile, wave grid) the generator can emit has a body.
// X(code, WM, WN, GM, GN); TK = 64 for all.  reg_tile = WM x WN per wave, smem_tile =
// (GM*WM) x (GN*WN) x 64.  Rows of 16 use v_mfma_f32_16x16x32, all others v_mfma_f32_32x32x16.
#pragma once
#include <stdint.h>
#define FT_FAMILY(X)                                                                     \
    X(0, 16, 16, 1, 4)   X(1, 16, 16, 2, 2)   X(2, 16, 16, 4, 1)                         \
    X(3, 16, 32, 1, 4)   X(4, 16, 32, 2, 2)   X(5, 16, 32, 4, 1)                         \
    X(6, 16, 64, 1, 4)   X(7, 16, 64, 2, 2)   X(8, 16, 64, 4, 1)                         \
    X(9, 32, 32, 1, 4)   X(10, 32, 32, 2, 2)  X(11, 32, 32, 4, 1)                        \
    X(12, 32, 64, 1, 4)  X(13, 32, 64, 2, 2)  X(14, 32, 64, 4, 1)                        \
    X(15, 64, 32, 1, 4)  X(16, 64, 32, 2, 2)  X(17, 64, 32, 4, 1)                        \
    X(18, 64, 64, 1, 4)  X(19, 64, 64, 2, 2)  X(20, 64, 64, 4, 1)                        \
    X(21, 64, 128, 1, 4) X(22, 64, 128, 2, 2) X(23, 64, 128, 4, 1)                       \
    X(24, 128, 64, 1, 4) X(25, 128, 64, 2, 2) X(26, 128, 64, 4, 1)                       \
    X(27, 128, 128, 1, 4) X(28, 128, 128, 2, 2) X(29, 128, 128, 4, 1)

// Split-k wave grid (1 x 1 x 4): X(code, TM, TN, twin) -- every wave owns the whole TM x TN tile and
// a quarter of the reduce axis.  twin = code of the standard-grid body with the same tile, used by
// the general (unaligned / convolution) path, which has no split-k variant.
#define FT_FAMILY_SPLITK(X)                                                              \
    X(30, 16, 64, 0) X(31, 32, 32, 1) X(32, 32, 64, 4) X(33, 64, 32, 5) X(34, 64, 64, 10)   \
    X(35, 16, 32, 37) X(36, 16, 16, 38)

// Tiles smaller than four MFMA blocks have no four-wave standard grid; their twins for the general
// path use fewer computing waves (the idle ones still help with the copies):
// X(code, WM, WN, GM, GN) with GM*GN < 4.  Compiled into the general dispatcher only.
#define FT_FAMILY_PARTIAL(X) X(37, 16, 16, 1, 2) X(38, 16, 16, 1, 1)

// Eight-wave grids (2 x 4 or 4 x 2 waves, two per SIMD, all on the same k-tile): X(code, WM, WN, GM, GN,
// twin) with twin = the four-wave body of the same tile, which the general path runs instead.
#define FT_FAMILY_W8(X)                                                                  \
    X(40, 128, 64, 2, 4, 28) X(41, 64, 128, 4, 2, 28) X(42, 64, 64, 2, 4, 22) X(43, 64, 64, 4, 2, 25)
#define FT_W8_ACC_MAX 128

// Two-team ("ping-pong") workgroups of eight waves run the standard-grid bodies above, gk = 2: both
// teams' rings of at least two stages must fit the LDS and each wave keeps at most 64 accumulator
// registers (two waves per SIMD in a 256-register kernel; class 0: <= 32 in 128 registers).
#define FT_PP_STAGE_MAX 40960
#define FT_PP_ACC_MAX 64
#define FT_TK 64
#define FT_NUM_CLASSES 3
// bodies with more accumulator registers per lane than this cannot take part in a reduce-axis
// split over workgroups (no registers left for the exchange of the partial tiles)
#define FT_KPART_ACC_MAX 128
// register class of a body: accumulator registers per lane -> launch-bounds budget
//   class 0: acc <= 32  (kernel compiled for 4 waves/SIMD, <= 128 registers)
//   class 1: acc <= 128 (2 waves/SIMD, <= 256 registers)
//   class 2: acc <= 256 (1 wave/SIMD,  <= 512 registers)
static inline int ft_class_of_acc(int acc_regs) { return acc_regs <= 32 ? 0 : (acc_regs <= 128 ? 1 : 2); }
static inline int ft_body_code(int wm, int wn, int gm, int gn, int gk) {
    if (gk == 2 && ((gm * wm + gn * wn) * FT_TK * 2 > FT_PP_STAGE_MAX || wm * wn / 64 > FT_PP_ACC_MAX)) return -1;
    if (gk == 1 && gm * gn == 8) {
#define FT_X(code, WM, WN, GM, GN, TWIN) if (wm == WM && wn == WN && gm == GM && gn == GN) return code;
        FT_FAMILY_W8(FT_X)
#undef FT_X
        return -1;
    }
    if (gk == 1 || gk == 2) {            // two teams (gk = 2) run the standard-grid body of the same code
#define FT_X(code, WM, WN, GM, GN) if (wm == WM && wn == WN && gm == GM && gn == GN) return code;
        FT_FAMILY(FT_X)
#undef FT_X
    } else if (gk == 4 && gm == 1 && gn == 1) {
#define FT_X(code, TM, TN, TWIN) if (wm == TM && wn == TN) return code;
        FT_FAMILY_SPLITK(FT_X)
#undef FT_X
    }
    return -1;
}
// LDS bytes of one stage (A tile + B tile, tk = 64, 16-bit elements) of the body with this code
static inline uint32_t ft_stage_bytes_of_code(int code) {
#define FT_X(c, WM, WN, GM, GN, TWIN) if (code == c) return (uint32_t)(((GM) * (WM) + (GN) * (WN)) * FT_TK * 2);
    FT_FAMILY_W8(FT_X)
#undef FT_X
#define FT_X(c, WM, WN, GM, GN) if (code == c) return (uint32_t)(((GM) * (WM) + (GN) * (WN)) * FT_TK * 2);
    FT_FAMILY(FT_X)
    FT_FAMILY_PARTIAL(FT_X)
#undef FT_X
#define FT_X(c, TM, TN, TWIN) if (code == c) return (uint32_t)(((TM) + (TN)) * FT_TK * 2);
    FT_FAMILY_SPLITK(FT_X)
#undef FT_X
    return 0;
}
// accumulator registers per lane of the body with this code
static inline int ft_acc_of_code(int code) {
#define FT_X(c, WM, WN, GM, GN, TWIN) if (code == c) return (WM) * (WN) / 64;
    FT_FAMILY_W8(FT_X)
#undef FT_X
#define FT_X(c, WM, WN, GM, GN) if (code == c) return (WM) * (WN) / 64;
    FT_FAMILY(FT_X)
    FT_FAMILY_PARTIAL(FT_X)
#undef FT_X
#define FT_X(c, TM, TN, TWIN) if (code == c) return (TM) * (TN) / 64;
    FT_FAMILY_SPLITK(FT_X)
#undef FT_X
    return 1 << 30;
}
// bodies that exist in the general dispatcher only
static inline int ft_is_partial_code(int code) {
#define FT_X(c, WM, WN, GM, GN) if (code == c) return 1;
    FT_FAMILY_PARTIAL(FT_X)
#undef FT_X
    return 0;
}
// an eight-wave grid body
static inline int ft_is_w8_code(int code) {
#define FT_X(c, WM, WN, GM, GN, TWIN) if (code == c) return 1;
    FT_FAMILY_W8(FT_X)
#undef FT_X
    return 0;
}
// body the general path runs for a given code (split-k codes map to their standard-grid twin)
static inline int ft_general_code(int code) {
#define FT_X(c, WM, WN, GM, GN, TWIN) if (code == c) return TWIN;
    FT_FAMILY_W8(FT_X)
#undef FT_X
#define FT_X(c, TM, TN, TWIN) if (code == c) return TWIN;
    FT_FAMILY_SPLITK(FT_X)
#undef FT_X
    return code;
}
// body a launch with ragged rows (K or N not a multiple of 8) runs for a given code on the LDS-DMA path:
// a split-k uKernel goes to its standard-grid twin, except the two narrowest tiles, whose twins exist
// among the general bodies only and whose split-k bodies handle ragged rows themselves
static inline int ft_ragged_code(int code) {
    const int twin = ft_general_code(code);
    return ft_is_partial_code(twin) ? code : twin;
}
