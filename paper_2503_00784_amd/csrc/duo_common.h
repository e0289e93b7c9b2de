// Shared device-side types and helpers (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Every kernel launch of the library goes through DUO_LAUNCH.  When the per-kernel profiler is armed
// (see duo_profile_enable) the launch carries a start and a stop event that take the dispatch's own
// begin and end timestamps, the same clock a kernel trace reads; otherwise it is a plain launch.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
    char* name = nullptr;  // armed: 128 bytes where the launch helper may leave the kernel's name with its template arguments
};
static LaunchEvents g_launch_events;
// The kernel about to be launched, spelled as a kernel trace prints it (e.g. "gemm_wide_kernel<4, 2, 3, 1, 8, 4, EpiSwiGLU, false>"),
// so that a timing taken here can be matched with counter summaries taken by a profiler.  No effect unless the timer is armed.
#define DUO_KERNEL_NAME(...)                                                               \
    do {                                                                                   \
        if (g_launch_events.name) snprintf(g_launch_events.name, 128, __VA_ARGS__);        \
    } while (0)
#define DUO_LAUNCH(kernel, grid, block, stream, ...)                                                            \
    do {                                                                                                        \
        if (g_launch_events.start) {                                                                            \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, g_launch_events.start, g_launch_events.stop, \
                                  0, __VA_ARGS__);                                                              \
            g_launch_events = LaunchEvents{};                                                                   \
        } else {                                                                                                \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                                    \
        }                                                                                                       \
    } while (0)

// The 16-bit element type of the weights, the KV cache and the operand buffers.  The library is built twice from
// the same sources: bf16 (the default; every comment that says "bf16" describes this build) and, with DUO_FP16
// defined, IEEE fp16, the format the paper ran its target model in (Sec. 4.1).  Everything type-dependent is in
// this block: conversions (round to nearest even), the two-element pack, and the MFMA.  Buffers are uint16_t
// bit patterns of whichever type the build uses; inputs here are finite.
#ifdef DUO_FP16
typedef _Float16 elem_t;
__device__ __forceinline__ float elem_to_f32(u16 b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ u16 f32_to_elem(float f) { return __builtin_bit_cast(u16, (_Float16)f); }
#else
typedef __bf16 elem_t;
__device__ __forceinline__ float elem_to_f32(u16 b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ u16 f32_to_elem(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (u16)(u >> 16);
}
#endif
typedef elem_t elem8 __attribute__((ext_vector_type(8)));
typedef elem_t elem2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two floats -> two elements (round to nearest even) in one register, a in the low half: the hardware conversion.
__device__ __forceinline__ uint32_t pack_elem2(float a, float b) {
    const elem2 v = __builtin_convertvector(f32x2{a, b}, elem2);
    return __builtin_bit_cast(uint32_t, v);
}
// the two halves of such a register back as floats
__device__ __forceinline__ float elem2_lo_f32(uint32_t p) { return elem_to_f32((u16)(p & 0xffffu)); }
__device__ __forceinline__ float elem2_hi_f32(uint32_t p) { return elem_to_f32((u16)(p >> 16)); }
// x[0..7] -> hi = elem(x), lo = elem(x - hi), as MFMA operand registers
__device__ __forceinline__ void split_elem8(const float (&x)[8], u32x4& hi, u32x4& lo) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t h = pack_elem2(x[2 * j], x[2 * j + 1]);
        hi[j] = h;
        lo[j] = pack_elem2(x[2 * j] - elem2_lo_f32(h), x[2 * j + 1] - elem2_hi_f32(h));
    }
}

union Frag8 {  // eight bf16 values = one 16-byte load = one MFMA operand
    elem8 v;
    u32x4 q;
    u16 h[8];
};

__device__ __forceinline__ elem8 load_frag(const u16* p) {
    Frag8 f;
    f.q = *reinterpret_cast<const u32x4*>(p);
    return f.v;
}
// The same load with the non-temporal hint: for data that is read exactly once (the weight stream, the prefix keys and
// values), so that it does not displace what is re-read from the caches (the activation operand every workgroup
// pulls through its L2).  Measured on the gate/up projection at 8 rows: 29.2 against 31.7 us (6.2 against 5.7 TB/s).
__device__ __forceinline__ elem8 load_frag_stream(const u16* p) {
    Frag8 f;
    f.q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return f.v;
}
__device__ __forceinline__ f32x4 mfma16(elem8 a, elem8 b, f32x4 c) {
    // D[16x16] += A[16x32] * B[32x16]; lane l supplies A[l%16][8*(l/16) .. +8] and
    // B[8*(l/16) .. +8][l%16]; it receives D[4*(l/16) .. +4][l%16].
#ifdef DUO_FP16
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
#endif
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}

// KV-cache layout inside one (layer, kv head) plane of max_seq * D elements.  Both caches are stored as the
// 1 KiB MFMA operand tiles the attention kernels consume, 32 slots (one key block) at a time, so that a wave
// fetches a tile with one fully coalesced load (lane l reads bytes 16*l .. 16*l+15) instead of sixteen half
// cache lines.
//   K: block B = slot / 32 holds 2 * D/32 tiles, tile (t, ks) = 16 keys x 32 channels.  Lane (c = l % 16,
//      g = l / 16) holds key 8*(c/4) + 4*t + c%4 of the block, channels 32*ks + 8*g .. +8: the key order
//      that lets the score accumulator of a lane be the softmax-weight operand of the same lane.
//   V: block B holds D/16 tiles, tile dt = 16 channels x 32 keys.  Lane (c, g) holds channel 16*dt + c,
//      keys 8*g .. 8*g+7 of the block (V transposed: the P*V product contracts over keys).
__host__ __device__ __forceinline__ size_t k_cache_offset(int D, int slot, int d) {
    const int B = slot >> 5, w = slot & 31, q = w >> 3, t = (w >> 2) & 1, r = w & 3;
    const int ks = d >> 5, g = (d >> 3) & 3, j = d & 7;
    return ((((size_t)B * 2 + t) * (D >> 5) + ks) * 64 + g * 16 + q * 4 + r) * 8 + j;
}
__host__ __device__ __forceinline__ size_t v_cache_offset(int D, int slot, int d) {
    const int B = slot >> 5, w = slot & 31, g = w >> 3, j = w & 7;
    const int dt = d >> 4, c = d & 15;
    return (((size_t)B * (D >> 4) + dt) * 64 + g * 16 + c) * 8 + j;
}

// Row bookkeeping of one pass: row m -> (sequence, index in sequence, position, slot).
struct RowPlan {
    int P;       // prefix length
    int R;       // 1 if row 0 is the shared root token
    int n, k;    // n sequences of k tokens
    int M;       // R + n*k
    __device__ __forceinline__ int pos(int m) const { return m < R ? P : P + R + (m - R) % k; }
    __device__ __forceinline__ int slot(int m) const { return P + m; }
};
