// Device kernels of the LIEC-SGD compressed step for gfx950 (CDNA4, wave64).
//
// Element ownership in the streaming kernels: a wave walks "wave tiles" of 1024 consecutive
// columns (4 chunks of 256); in chunk u, lane l owns columns 256u + 4l .. 256u + 4l + 3 (one
// 128-bit access per lane, 1 KiB contiguous per wave and instruction).  A block of 256 threads
// (4 waves) covers 4096 consecutive columns per iteration.  All fp32 arithmetic that reaches the
// outputs is written as single IEEE operations (__fadd_rn / __fsub_rn / __fmaf_rn) so that the
// result does not depend on compiler contraction.  Streams that are read or written once are
// accessed with non-temporal hints.
//
// kernels/common.hpp     constants, row descriptor, random-k generator, accessors, reductions
// kernels/sign.hpp       scaled sign and blockwise scaled sign: L1 norms and sign bits
// kernels/select.hpp     threshold search of top-k and random-k
// kernels/step.hpp       aggregation (server compensation) and update (recompression, error, models)
// kernels/sync.hpp       averaging iteration
// kernels/wire.hpp       wire forms of the messages
// kernels/telemetry.hpp  l2 norm, copy probe
#pragma once
#include "kernels/common.hpp"
#include "kernels/select.hpp"
#include "kernels/sign.hpp"
#include "kernels/step.hpp"
#include "kernels/sync.hpp"
#include "kernels/telemetry.hpp"
#include "kernels/wire.hpp"
