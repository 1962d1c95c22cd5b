// gfx950 (MI355X) kernels for the ODC hot path: gather, scatter-accumulate, reset.
//
// Nothing here is a contraction, so there is no MFMA: every kernel is a pure HBM stream
// (0 or 0.1 flop per byte) and is shaped for that -- 64-lane wavefronts issuing 128-bit
// loads/stores that are contiguous across the wave, several independent vectors in flight
// per lane, non-temporal hints on data that is touched once, and thousands of workgroups so
// that all 256 CUs in the 8 XCDs stay busy.  Rank base pointers travel in the kernel
// arguments; blockIdx.y selects the owner rank, so the flat kernels do no division at all.
//
// What is computed (paper Section 3, Section 3.1, Appendix B, Section 2.1 with w_m = 1):
//   gather:      full[r*S + i]  = shard_r[i]                       i < valid_r
//   accumulate:  acc_r[i]       = fl32(acc_r[i] + widen(g[r*S+i])) i < valid_r
//   reset:       acc_r[i]       = +0.0f                            i < valid_r
// with S = ceil(N / R) and valid_r = clamp(N - r*S, 0, S).  Padding is never touched.
//
// Misalignment: shard boundaries r*S fall on any 2-byte boundary.  The side that is written
// is always accessed with naturally aligned 16-byte vectors (head and tail elements are
// peeled); the read-only side uses byte-unaligned wide loads, which global memory on this
// target supports in hardware, so no LDS staging is needed for the shift.
//
// The kernels live in one header per family; this one includes them all.
#pragma once

#include "odc_dev_common.h"
#include "odc_dev_flat.h"
#include "odc_dev_batched.h"
#include "odc_dev_fused.h"
#include "odc_dev_staging.h"
#include "odc_dev_retrieve.h"
#include "odc_dev_wide.h"
#include "odc_dev_hybrid.h"
