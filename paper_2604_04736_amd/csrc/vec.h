// Device helpers shared by the libhot translation units (gfx950 only).
#ifndef HOT_VEC_H
#define HOT_VEC_H

#include <hip/hip_runtime.h>

#include <cstdint>

// hipError_t of the last failed HIP call made by this thread through a plan-less entry point
// (defined in hot.hip; hot_last_hip_error(NULL) returns it).
namespace hot_detail {
__attribute__((visibility("hidden"))) int note_hip(hipError_t e);   // records e if it is an error; returns HOT_OK or HOT_EHIP
}

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));   // same vector, only dword-aligned in memory

// 16-byte load / store of four consecutive floats.  ALIGNED = false still issues one
// dwordx4 access; the address then only has to be a multiple of 4 bytes.
template <bool ALIGNED, bool NT>
__device__ __forceinline__ f4 load4(const float *p)
{
    if constexpr (ALIGNED) {
        const f4 *q = reinterpret_cast<const f4 *>(p);
        if constexpr (NT) return __builtin_nontemporal_load(q);
        else return *q;
    } else {
        const f4u *q = reinterpret_cast<const f4u *>(p);
        if constexpr (NT) return __builtin_nontemporal_load(q);
        else return *q;
    }
}

template <bool ALIGNED, bool NT>
__device__ __forceinline__ void store4(float *p, f4 v)
{
    if constexpr (ALIGNED) {
        f4 *q = reinterpret_cast<f4 *>(p);
        if constexpr (NT) __builtin_nontemporal_store(v, q);
        else *q = v;
    } else {
        f4u *q = reinterpret_cast<f4u *>(p);
        if constexpr (NT) __builtin_nontemporal_store(v, q);
        else *q = v;
    }
}

// Range-checked 16-byte accesses for column tiles narrower than their threads' reach: a window of `bytes` bytes at
// p (uniform over the wave), addressed by byte offsets.  The hardware's buffer addressing returns zeros for a load
// beyond the window and drops a store beyond it, so no thread branches around its accesses: a branch would make
// the compiler wait for ALL outstanding memory operations before every store behind it (it cannot count them
// across the join), which serialises a workgroup's stores.  Windows and offsets here are multiples of 16 bytes
// (of 4 for the base address), so a quad is inside or outside as a whole.
typedef int i4 __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t window_t;

__device__ __forceinline__ window_t window(const float *p, unsigned bytes)
{
    // (stride 0, `bytes` records, 32-bit data format: the raw-buffer descriptor of gfx9-family chips)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p), 0, (int)bytes, 0x00020000);
}

template <bool NT>
__device__ __forceinline__ f4 window_load4(window_t win, unsigned byte_offset)
{
    return __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(win, (int)byte_offset, 0, NT ? 2 : 0));
}

template <bool NT>
__device__ __forceinline__ void window_store4(window_t win, unsigned byte_offset, f4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i4, v), win, (int)byte_offset, 0, NT ? 2 : 0);
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    return v;   // complete in lane 0
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

}  // namespace

#endif  // HOT_VEC_H
