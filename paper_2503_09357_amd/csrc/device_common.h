// Shared device-side definitions of the dagsched kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dagsched.h"

namespace dagsched_dev {

constexpr int kWave = 64;

// bits collected per candidate while it is being evaluated; turned into one DAGSCHED_FLAG_* at the end
constexpr int kBitCyclic = 1, kBitBadPlacement = 2, kBitBadRank = 4, kBitInternal = 8, kBitOverMemory = 16;

__device__ __forceinline__ int flag_from_bits(int bits) {
  return (bits & kBitBadPlacement) ? DAGSCHED_FLAG_BAD_PLACEMENT
       : (bits & kBitBadRank)      ? DAGSCHED_FLAG_BAD_RANK
       : (bits & kBitInternal)     ? DAGSCHED_FLAG_INTERNAL
       : (bits & kBitCyclic)       ? DAGSCHED_FLAG_CYCLIC
       : (bits & kBitOverMemory)   ? DAGSCHED_FLAG_OVER_MEMORY
                                   : DAGSCHED_FLAG_OK;
}

// Loads/stores that must observe data written earlier in the same kernel by other lanes go to L2
// (agent scope) so that a stale line in the per-CU vector cache can never be returned.
__device__ __forceinline__ int32_t ld_agent(const int32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int32_t *p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS pointers with an explicit address space: volatile accesses through generic pointers would be
// compiled to flat loads, these compile to ds_read/ds_write.
#define DAGSCHED_LDS __attribute__((address_space(3)))
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef DAGSCHED_LDS unsigned char lds_byte_t;
typedef DAGSCHED_LDS volatile uint32_t lds_vu32_t;
typedef DAGSCHED_LDS volatile uint64_t lds_vu64_t;
typedef DAGSCHED_LDS volatile uint16_t lds_vu16_t;
typedef DAGSCHED_LDS volatile int32_t lds_vi32_t;
typedef DAGSCHED_LDS const uint8_t lds_cu8_t;
typedef DAGSCHED_LDS volatile u32x4_t lds_vu32x4_t;

// Where the outputs of one evaluate call go.
struct OutPtrs {
  int32_t *makespan;
  int64_t *bubble;
  int64_t *peak_mem;
  int32_t *flags;
  int64_t peak_stride_c, peak_stride_j;   // peak_mem[c*peak_stride_c + j*peak_stride_j]
};

}  // namespace dagsched_dev
