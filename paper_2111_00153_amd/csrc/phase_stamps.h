// Per-wave phase timestamps for tuning builds (-DRMSMP_PHASE_TIMING); without that define every
// macro here is empty and PHASE_LDS_BYTES is 0, so the kernels carry no trace of them.
// RMSMP_PHASE: a stamp is one clock read parked in the first KiB of dynamic LDS (16 slots per
// wave); the kernel copies the slots to g_phase_buf when it ends, so a stamp costs no memory
// round trip where it is taken.  RMSMP_REG_STAMP: the same with eight slots held in registers,
// for kernels whose LDS layout leaves no room (the weight-stream kernel).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace rmsmp {

#ifdef RMSMP_PHASE_TIMING
__device__ unsigned long long* g_phase_buf = nullptr;
constexpr int PHASE_LDS_BYTES = 1024;
extern __shared__ __attribute__((aligned(16))) uint8_t phase_smem[];
#define RMSMP_PHASE(id)                                                                                  \
  do {                                                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    if ((threadIdx.x & 63) == 0) ((unsigned long long*)phase_smem)[(threadIdx.x >> 6) * 16 + (id)] = clock64(); \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
  } while (0)
#define RMSMP_PHASE_FLUSH()                                                                              \
  do {                                                                                                   \
    if (g_phase_buf && (threadIdx.x & 63) == 0)                                                          \
      for (int i_ = 0; i_ < 16; ++i_)                                                                    \
        g_phase_buf[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + i_] =                                  \
            ((unsigned long long*)phase_smem)[(threadIdx.x >> 6) * 16 + i_];                             \
  } while (0)
#define RMSMP_REG_STAMPS_DECLARE() unsigned long long reg_stamps_[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define RMSMP_REG_STAMP(id)                \
  do {                                     \
    __builtin_amdgcn_sched_barrier(0);     \
    reg_stamps_[id] = clock64();           \
    __builtin_amdgcn_sched_barrier(0);     \
  } while (0)
#define RMSMP_REG_STAMPS_FLUSH()                                                               \
  do {                                                                                         \
    if (g_phase_buf && (threadIdx.x & 63) == 0)                                                \
      for (int i_ = 0; i_ < 8; ++i_)                                                           \
        g_phase_buf[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + i_] = reg_stamps_[i_];        \
  } while (0)
#else
constexpr int PHASE_LDS_BYTES = 0;
#define RMSMP_REG_STAMPS_DECLARE() \
  do {                             \
  } while (0)
#define RMSMP_REG_STAMP(id) \
  do {                      \
  } while (0)
#define RMSMP_REG_STAMPS_FLUSH() \
  do {                           \
  } while (0)
#define RMSMP_PHASE(id) \
  do {                  \
  } while (0)
#define RMSMP_PHASE_FLUSH() \
  do {                      \
  } while (0)
#endif

}  // namespace rmsmp
