// Internal helpers shared by the device entry points (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include "../../include/aurora_moe.h"

#define MOE_MAX_E 256
#define MOE_MAX_G 64
#define MOE_MAX_K 16
#define MOE_MAX_LOCAL 64
#define MOE_SLOTS_PER_BLOCK 1024   // counting-scan granularity: 4 waves x 4 rounds x 64 lanes

int moe_set_error(int status, const char* fmt, ...);
int moe_check_shape(const moe_shape* s);   // the checks of moe_ctx_create

#define MOE_HIP(call)                                                                     \
    do {                                                                                  \
        hipError_t e__ = (call);                                                          \
        if (e__ != hipSuccess)                                                            \
            return moe_set_error(MOE_EHIP, "%s: %s", #call, hipGetErrorString(e__));      \
    } while (0)

#define MOE_LAUNCH_CHECK(name)                                                            \
    do {                                                                                  \
        hipError_t e__ = hipGetLastError();                                               \
        if (e__ != hipSuccess)                                                            \
            return moe_set_error(MOE_EHIP, "launch %s: %s", name, hipGetErrorString(e__)); \
    } while (0)

struct moe_ctx {
    moe_shape s;
    int32_t n_slots;      // T * k
    int32_t n_blocks;     // ceil(n_slots / MOE_SLOTS_PER_BLOCK)
    int32_t* block_hist;  // device [n_blocks][E]: slots per expert in each block, later its exclusive prefix
    int32_t* raw_count;   // device [E]: slots per expert before the capacity rule
    int32_t* slot_rank;   // device [n_slots]: rank of a slot among the slots of its expert (-1: index out of range)
    const void* rank_src; // host: the topk_idx pointer the LAST call on this context (a moe_traffic) ranked, else NULL
    bool reuse_ranks;     // host: moe_ctx_set_rank_reuse; off unless the caller asks
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte load/store unit

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline int elem_size(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }

// bf16 <-> fp32 on the device (round to nearest even; inputs are finite in this library)
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
