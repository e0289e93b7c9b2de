// One-time repacking of row-major bf16 matrices into the MFMA-tile streaming layout of duo_gemm.h:
// band b (16 rows), K step ks, lane l  ->  eight values row(b, l % 16), columns 32*ks + 8*(l/16) .. +8,
// stored at element ((b * K/32 + ks) * 64 + l) * 8.  Which source rows make up band b is the packer's
// choice: plain order, Q/K/V channels next to their rotary partners, gate/up bands interleaved.
#pragma once
#include "duo_common.h"

struct PlainRows {  // band b = rows 16b .. 16b+15; rows beyond N are zero
    const u16* src;
    int N, K;
    __device__ __forceinline__ const u16* row(int band, int c) const {
        const int r = band * 16 + c;
        return r < N ? src + (size_t)r * K : nullptr;
    }
};

struct QKVRows {  // band (head, j): rows 0..7 are channels 8j .. 8j+7 of that head, rows 8..15 their rotary partners D/2 + 8j ..
    const u16* wq;
    const u16* wk;
    const u16* wv;
    int Hq, Hkv, D, half, bph, K;  // bph = D/16 bands per head
    __device__ __forceinline__ const u16* row(int band, int c) const {
        int head = band / bph;
        const int r = (band - head * bph) * 8 + (c & 7) + (c >= 8 ? half : 0);
        if (head < Hq) return wq + (size_t)(head * D + r) * K;
        head -= Hq;
        if (head < Hkv) return wk + (size_t)(head * D + r) * K;
        head -= Hkv;
        return wv + (size_t)(head * D + r) * K;
    }
};

struct GateUpRows {  // band 2*w = gate rows 16w.., band 2*w+1 = up rows 16w..
    const u16* wg;
    const u16* wu;
    int F, K;
    __device__ __forceinline__ const u16* row(int band, int c) const {
        const int r = (band >> 1) * 16 + c;
        if (r >= F) return nullptr;
        return ((band & 1) ? wu : wg) + (size_t)r * K;
    }
};

template <class Rows>
__global__ __launch_bounds__(256) void pack_bands_kernel(Rows rows, int steps, u16* __restrict__ dst) {
    const int band = blockIdx.x, lane = threadIdx.x & 63;
    const u16* src = rows.row(band, lane & 15);
    for (int ks = threadIdx.x >> 6; ks < steps; ks += 4) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (src) v = *reinterpret_cast<const u32x4*>(src + ks * 32 + (lane >> 4) * 8);
        *reinterpret_cast<u32x4*>(dst + (((size_t)band * steps + ks) * 64 + lane) * 8) = v;
    }
}

// Plain activation rows [rows][K] -> operand layout [K/32][tiles][64][8]; rows beyond `rows` are zero.
__global__ __launch_bounds__(256) void pack_operand_kernel(const u16* __restrict__ src, int rows, int K, int tiles,
                                                            u16* __restrict__ dst) {
    const int ks = blockIdx.x, lane = threadIdx.x & 63;
    for (int mt = threadIdx.x >> 6; mt < tiles; mt += 4) {
        const int r = mt * 16 + (lane & 15);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r < rows) v = *reinterpret_cast<const u32x4*>(src + (size_t)r * K + ks * 32 + (lane >> 4) * 8);
        *reinterpret_cast<u32x4*>(dst + (((size_t)ks * tiles + mt) * 64 + lane) * 8) = v;
    }
}
