// Shared host/device helpers of libvmoba (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "vmoba.h"

#define VMOBA_MAX_BLOCKS 512
#define VMOBA_MAX_MASK_WORDS (VMOBA_MAX_BLOCKS / 32)

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Kernel-side view of a vmoba_tensor whose D channels are contiguous.
struct TensorView {
    char* ptr;
    int64_t stride_b, stride_s, stride_h;  // in elements
};

static inline TensorView make_view(const vmoba_tensor* t) {
    TensorView v;
    v.ptr = (char*)t->ptr;
    v.stride_b = t->stride_b;
    v.stride_s = t->stride_s;
    v.stride_h = t->stride_h;
    return v;
}

static inline int dtype_size(int dt) { return dt == VMOBA_BF16 ? 2 : 4; }

static inline bool tensor_ok(const vmoba_tensor* t) {
    if (!t || !t->ptr) return false;
    if (t->dtype != VMOBA_F32 && t->dtype != VMOBA_BF16) return false;
    if (((uintptr_t)t->ptr) & 15) return false;
    int64_t per16 = 16 / dtype_size(t->dtype);
    if (t->stride_b % per16 || t->stride_s % per16 || t->stride_h % per16) return false;
    return true;
}

#define VMOBA_CHECK_LAUNCH()                                   \
    do {                                                       \
        if (hipGetLastError() != hipSuccess) return VMOBA_ERR_HIP; \
    } while (0)

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// pack two floats to two bf16 (round to nearest even), low half = a
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t w = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<uint32_t*>(&w);
}

// Optional event pairs recorded around single kernel launches (see vmoba_profile_events).
struct ProfileSlot { hipEvent_t start, stop; };
extern ProfileSlot g_profile[4];
#define VMOBA_PROFILE_BEGIN(slot, st) do { if (g_profile[slot].start) (void)hipEventRecord(g_profile[slot].start, st); } while (0)
#define VMOBA_PROFILE_END(slot, st) do { if (g_profile[slot].stop) (void)hipEventRecord(g_profile[slot].stop, st); } while (0)
