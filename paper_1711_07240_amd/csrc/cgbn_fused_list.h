// The (bytes per load, register slots per plane) combinations the NCHW single-launch
// kernels are built for; slots per plane 0 = large planes cut into tiles.  With R the
// register slots per tensor (forward: 32 for 16-byte loads, 64 for 8-byte, 128 for 4-byte;
// backward: half of that) the slot counts offered lie between R/16 and R (plus one beyond R, see below).  4-byte loads
// serve small planes whose byte size is not a multiple of 8.  Slots per plane -2: two planes of up to half a
// tile each per workgroup.  X(LB, LPPC).
#pragma once

#define CGBN_FUSED_COMMON_WIDE(X)                                                             \
    X(16, 0) X(8, 0) X(16, -2)                                                                \
    X(16, 2) X(16, 3) X(16, 4) X(16, 5) X(16, 6) X(16, 8) X(16, 10) X(16, 12) X(16, 16)       \
    X(8, 4) X(8, 5) X(8, 6) X(8, 8) X(8, 10) X(8, 12) X(8, 16) X(8, 24) X(8, 32)
#define CGBN_FUSED_COMMON_NARROW(X) X(4, 8) X(4, 10) X(4, 12) X(4, 16) X(4, 24) X(4, 32) X(4, 64)
#define CGBN_FUSED_COMMON(X) CGBN_FUSED_COMMON_WIDE(X) CGBN_FUSED_COMMON_NARROW(X)
// The last two of each line: planes up to 6 KiB (forward) / 3 KiB (backward, per tensor) longer than a wavefront's
// share of the registers: one plane per wavefront, the slots beyond the registers in LDS.
#define CGBN_FUSED_FORWARD_ONLY(X) X(16, 24) X(16, 32) X(8, 64) X(4, 128) X(16, 38) X(8, 76)
#define CGBN_FUSED_BACKWARD_ONLY_WIDE(X) X(8, 2) X(8, 3) X(16, 19) X(8, 38)
#define CGBN_FUSED_BACKWARD_ONLY_NARROW(X) X(4, 4) X(4, 5) X(4, 6)
#define CGBN_FUSED_BACKWARD_ONLY(X) CGBN_FUSED_BACKWARD_ONLY_WIDE(X) CGBN_FUSED_BACKWARD_ONLY_NARROW(X)

// Slots per plane -N: N whole planes of one channel (consecutive images) per workgroup, in workgroup-wide slots of
// 256 lanes x 16 bytes, a row each.  -2 is built for both LDS splits (it is in the common list); 3 and 4 planes per
// workgroup only for the split that keeps more unit data in LDS (few rows and shards to stage).  They serve planes
// too long for a wavefront and much shorter than half a tile (forward 38-56 KiB, backward 19-28 KiB per tensor),
// which two to a workgroup fill 45-65 % of what it can hold.  (Measured and not built: 5 to 8 planes per workgroup
// in place of one plane per wavefront for planes of 9-32 KiB.  The units are fuller, 75-90 % against 40-56 %, and
// no faster: fp32 50x84 planes forward 244 -> 251 us, fp32 50x50 backward 439 -> 462 us; the two barriers per plane
// and pass cost what the fuller units gain.)
#define CGBN_FUSED_WGP_FORWARD(X) X(16, -3) X(16, -4)
#define CGBN_FUSED_WGP_BACKWARD(X) X(16, -3) X(16, -4)

// Small planes with few rows and shards to stage (BIG == 2): further whole planes per wavefront in LDS.
// Only slot counts for which at least one plane fits the LDS share of either direction.
#define CGBN_FUSED_BIG_SMALL_WIDE(X) X(8, 4) X(8, 5) X(8, 6) X(8, 8) X(8, 10) X(16, 2) X(16, 3) X(16, 4) X(16, 5)
#define CGBN_FUSED_BIG_SMALL_NARROW(X) X(4, 8) X(4, 10) X(4, 12) X(4, 16)
#define CGBN_FUSED_BIG_SMALL(X) CGBN_FUSED_BIG_SMALL_WIDE(X) CGBN_FUSED_BIG_SMALL_NARROW(X)

// The ReLU backward of float tensors is not built with 4-byte accesses, one slot count excepted: next to the stored
// output's extra round of loads those variants do not fit a wavefront's register budget (65 to 104 registers go
// to scratch memory) and run slower than the multi-sweep kernels (measured, 64 x 1024 channels: planes of 255
// to 4095 floats 1.3 to 1.6 times slower; the 24-slot variant, planes of 1075 to 1535 floats, 1.5 times faster).
// Such shapes take the multi-sweep kernels for that call.
#define CGBN_FUSED_RELU_BWD_F32_NARROW(X) X(4, 24)

// The slot counts the host may choose for small planes, ascending: for a plane of LPP slots it takes the smallest
// count >= LPP that leaves at most 16 planes per wavefront (count * 16 >= R, R the register slots per tensor) and
// fits the registers (count <= R).  Hence a variant built for `lppc` slots only ever sees planes longer than the
// next smaller admissible count: that many leading slots of every plane are full in every shape the variant
// serves, and its kernels check neither the plane's length nor the lanes there.  A plane longer than the
// registers (lppc > R: the last slots live in LDS) fills all R register slots.
constexpr int kCgbnSlotCounts[] = {2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32, 64, 128};
constexpr int cgbn_full_slots(int lppc, int R)
{
    if (lppc > R) return R;
    int prev = 0;
    for (int c : kCgbnSlotCounts) {
        if (c >= lppc) break;
        prev = c;
    }
    return prev * 16 >= R ? prev : 0;
}
