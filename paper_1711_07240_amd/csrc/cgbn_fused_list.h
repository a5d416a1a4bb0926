// The (bytes per load, register slots per plane) combinations the NCHW single-launch
// kernels are built for; slots per plane 0 = large planes cut into tiles.  With R the
// register slots per tensor (forward: 32 for 16-byte loads, 64 for 8-byte, 128 for 4-byte;
// backward: half of that) the slot counts offered lie between R/16 and R (plus one beyond R, see below).  4-byte loads
// serve small planes whose byte size is not a multiple of 8.  Slots per plane -2: two planes of up to half a
// tile each per workgroup.  X(LB, LPPC).
#pragma once

#define CGBN_FUSED_COMMON(X)                                                                  \
    X(16, 0) X(8, 0) X(16, -2)                                                                \
    X(16, 2) X(16, 3) X(16, 4) X(16, 5) X(16, 6) X(16, 8) X(16, 10) X(16, 12) X(16, 16)       \
    X(8, 4) X(8, 5) X(8, 6) X(8, 8) X(8, 10) X(8, 12) X(8, 16) X(8, 24) X(8, 32)                \
    X(4, 8) X(4, 10) X(4, 12) X(4, 16) X(4, 24) X(4, 32) X(4, 64)
// The last two of each line: planes up to 6 KiB (forward) / 3 KiB (backward, per tensor) longer than a wavefront's
// share of the registers: one plane per wavefront, the slots beyond the registers in LDS.
#define CGBN_FUSED_FORWARD_ONLY(X) X(16, 24) X(16, 32) X(8, 64) X(4, 128) X(16, 38) X(8, 76)
#define CGBN_FUSED_BACKWARD_ONLY(X) X(8, 2) X(8, 3) X(4, 4) X(4, 5) X(4, 6) X(16, 19) X(8, 38)

// Small planes with few rows and shards to stage (BIG == 2): further whole planes per wavefront in LDS.
// Only slot counts for which at least one plane fits the LDS share of either direction.
#define CGBN_FUSED_BIG_SMALL(X)                                                               \
    X(4, 8) X(4, 10) X(4, 12) X(4, 16) X(8, 4) X(8, 5) X(8, 6) X(8, 8) X(8, 10) X(16, 2) X(16, 3) X(16, 4) X(16, 5)
