// Phase stamps: a profiling build of libsentencekv (compiled with -DSKV_PHASE_STAMPS into libsentencekv_stamps.so) records
// the constant 100 MHz wall clock at marked places of the decode kernels, one row of slots per block, and exports
// skv_stamps_read() to copy the table out.  In the ordinary build SKV_T(k) expands to nothing and the table does not exist.
#pragma once

#ifdef SKV_PHASE_STAMPS
#include <hip/hip_runtime.h>
namespace skv {
constexpr int kStampBlocks = 4096, kStampSlots = 16;
extern __device__ unsigned long long g_stamps[kStampBlocks * kStampSlots];
}  // namespace skv
// thread 0 of a block stores the clock into slot k of the block's row (blocks are numbered x-fastest)
#define SKV_T(k)                                                                                       \
    do {                                                                                               \
        if (threadIdx.x == 0) {                                                                        \
            const unsigned skv_blk = blockIdx.y * gridDim.x + blockIdx.x;                              \
            if (skv_blk < skv::kStampBlocks) skv::g_stamps[skv_blk * skv::kStampSlots + (k)] = wall_clock64(); \
        }                                                                                              \
    } while (0)
#else
#define SKV_T(k)
#endif
