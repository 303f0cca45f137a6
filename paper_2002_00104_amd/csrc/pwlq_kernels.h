// libpwlq kernels for gfx950.  Pipeline of one search call:
//
//   k_tile_absmax  max|w| of every tile                         (HBM read)
//   k_prep         group absmax; magnitudes rescaled to "candidate units"
//                  u = |w|/m * n and partitioned into one bucket per block of
//                  64 candidates                                (HBM read+write)
//   k_search       the hot loop: lane = candidate, elements arrive as
//                  wave-uniform scalar loads; binary32 squared error of every
//                  (element, candidate) pair                    (VALU bound)
//   k_flag         per group: candidates whose binary32 SSE is within the
//                  rounding slack of the minimum
//   k_exact        flagged candidates re-evaluated with the canonical binary32
//                  code and binary64 error; argmin for single-tile groups
//   k_final        argmin for groups spread over several tiles
//
// A call too small to fill the chip (at most kSmallCallTiles single-tile groups
// of at most 1024 elements, at most 1024 candidates and kSmallCallEvals
// evaluations in all) runs k_small instead: all of the above for one group
// inside one workgroup, one launch.
//
// and of one quantize call:  k_emit (HBM bound).
//
// The analytic selectors run k_stats (per-tile max, sum of squares, sum of
// magnitudes) and k_select (one thread per group solves for p); the error at a
// given (m, p) runs k_mse_tile and k_mse_final.
#pragma once

#include "pwlq_prep.h"
#include "pwlq_search.h"
#include "pwlq_refine.h"
#include "pwlq_emit.h"
#include "pwlq_select.h"
#include "pwlq_fast.h"
#include "pwlq_linear.h"
#include "pwlq_small.h"
