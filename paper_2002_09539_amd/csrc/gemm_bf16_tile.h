// Operand tiles of the bf16 matrix-core kernels (v_mfma_f32_32x32x16_bf16, gfx950): global -> registers -> LDS copies
// in the operand's own memory order with 16-byte vectors, and the per-lane fragments the MFMA takes (8 consecutive
// contraction indices of one row).
//   * TileKC: the operand is contiguous along the contraction index (memory [rows][K]); LDS [ROWS][BK + 8]; a fragment
//     is one 16-byte LDS read.
//   * TileRC: the operand's rows are contiguous (memory [K][rows]); LDS [BK][ROWS + 32]; a fragment is two LDS transpose
//     reads (ds_read_b64_tr_b16): within each block of 16 lanes, lane j passes the address of an 8-byte piece and lane i
//     receives element i % 4 of the pieces of lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4.  With lane j pointing at
//     row k0 + j / 4, columns n0 + 4 (j % 4) .., lane i receives column n0 + i of rows k0 .. k0 + 3.
// Row paddings keep both read patterns free of bank conflicts.  Used by the grouped GEMMs of the MLP and by the
// convolutions (forward / backward of the models whose gradients are the g_i of Section 2, arXiv 2002.09539).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ols {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f2v __attribute__((ext_vector_type(2)));
typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kTileThreads = 256;   // lanes that copy a tile together

// Buffer addressing: a descriptor of [base, base + bytes) and 32-bit byte offsets.  The hardware checks the lane's offset
// against the range: a load outside returns zeros and a store outside is dropped, so tiles that hang over either end of
// a tensor (the strip's halo, the last tile's rows) need no per-lane predicates or 64-bit address arithmetic.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);   // raw buffer, 32-bit data format
}
__device__ __forceinline__ u4 buf_load(rsrc_t r, unsigned lane_off, unsigned uniform_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)uniform_off, 0);
}
__device__ __forceinline__ void buf_store(u4 v, rsrc_t r, unsigned lane_off) { __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)lane_off, 0, 0); }


// K-contiguous operand tile: memory [rows][K]; LDS [ROWS][BK + 8].
template <int ROWS, int BK, int THREADS = kTileThreads>
struct TileKC {
    static constexpr int kPitch = BK + 8;                 // bf16 elements; 16-byte aligned rows
    static constexpr int kVecPerLine = BK / 8;
    static constexpr int kVecs = ROWS * kVecPerLine;
    static constexpr int kPerThread = (kVecs + THREADS - 1) / THREADS;
    static constexpr int kElems = ROWS * kPitch;
    // Every lane ALWAYS issues its loads (out-of-range lanes re-read the operand's first vector) and the
    // zero fill is applied when the registers are written to LDS: no branch around the loads, so a later
    // slice's loads stay in flight while an earlier slice is stored.
    __device__ static unsigned load(u4 (&r)[kPerThread], const uint16_t* __restrict__ base, int ld, int row0, int k0,
                                    int rows, int klen) {
        unsigned okmask = 0;
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * THREADS;
            const int row = row0 + v / kVecPerLine, k = k0 + (v % kVecPerLine) * 8;
            const bool ok = (kVecs % THREADS == 0 || v < kVecs) && row < rows && k < klen;
            r[t] = *(const u4*)(base + (ok ? (int64_t)row * ld + k : 0));
            okmask |= ok ? (1u << t) : 0u;
        }
        return okmask;
    }
    __device__ static void store(uint16_t* lds, const u4 (&r)[kPerThread], unsigned okmask) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * THREADS;
            if (kVecs % THREADS == 0 || v < kVecs) {
                const u4 zero = {0u, 0u, 0u, 0u};
                *(u4*)(lds + (v / kVecPerLine) * kPitch + (v % kVecPerLine) * 8) = (okmask >> t) & 1u ? r[t] : zero;
            }
        }
    }
    // rows r0 .. r0 + 31, k-step s (16 contraction indices): lane holds k = 16 s + 8 (lane / 32) + 0..7 of row lane % 32
    __device__ static bf16x8 frag(const uint16_t* lds, int r0, int s, int lane) {
        return __builtin_bit_cast(bf16x8, *(const u4*)(lds + (r0 + lane % 32) * kPitch + 16 * s + 8 * (lane / 32)));
    }
    // Full tiles (no bounds): vector t of a lane is kLineStep lines below vector 0, so one 32-bit lane offset
    // plus wave-uniform bases address all of them and the loop carries no per-lane address arithmetic.
    static constexpr int kLineStep = THREADS / kVecPerLine;
    __device__ static unsigned lane_offset_bytes(int ld) {
        return 2u * ((threadIdx.x / kVecPerLine) * (unsigned)ld + (threadIdx.x % kVecPerLine) * 8u);
    }
    __device__ static int64_t line_step_bytes(int ld) { return 2 * (int64_t)kLineStep * ld; }
    __device__ static int64_t slice_step_bytes(int ld) { return 2 * (int64_t)BK; }
    __device__ static uint16_t* lane_lds(uint16_t* lds) {
        return lds + (threadIdx.x / kVecPerLine) * kPitch + (threadIdx.x % kVecPerLine) * 8;
    }
    static constexpr int kLdsLineStep = kLineStep * kPitch;
};

// Row-contiguous operand tile: memory [K][rows]; LDS [BK][ROWS + 32], read with the transpose load.
template <int ROWS, int BK, int THREADS = kTileThreads>
struct TileRC {
    static constexpr int kPitch = ROWS + 32;              // pitch = 64 bytes mod 256: the 4 k-rows of a read hit distinct banks
    static constexpr int kVecPerLine = ROWS / 8;
    static constexpr int kVecs = BK * kVecPerLine;
    static constexpr int kPerThread = (kVecs + THREADS - 1) / THREADS;
    static constexpr int kElems = BK * kPitch;
    __device__ static unsigned load(u4 (&r)[kPerThread], const uint16_t* __restrict__ base, int ld, int row0, int k0,
                                    int rows, int klen) {
        unsigned okmask = 0;
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * THREADS;
            const int k = k0 + v / kVecPerLine, row = row0 + (v % kVecPerLine) * 8;
            const bool ok = (kVecs % THREADS == 0 || v < kVecs) && row < rows && k < klen;
            r[t] = *(const u4*)(base + (ok ? (int64_t)k * ld + row : 0));
            okmask |= ok ? (1u << t) : 0u;
        }
        return okmask;
    }
    __device__ static void store(uint16_t* lds, const u4 (&r)[kPerThread], unsigned okmask) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * THREADS;
            if (kVecs % THREADS == 0 || v < kVecs) {
                const u4 zero = {0u, 0u, 0u, 0u};
                *(u4*)(lds + (v / kVecPerLine) * kPitch + (v % kVecPerLine) * 8) = (okmask >> t) & 1u ? r[t] : zero;
            }
        }
    }
    __device__ static bf16x8 frag(const uint16_t* lds, int r0, int s, int lane) {
        const int blk = lane / 16, j = lane % 16;
        const uint16_t* p = lds + (16 * s + 8 * (blk / 2) + j / 4) * kPitch + r0 + 16 * (blk % 2) + 4 * (j % 4);
        typedef s4v __attribute__((address_space(3))) * lds_s4_ptr;
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)p);
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(p + 4 * kPitch));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
    static constexpr int kLineStep = THREADS / kVecPerLine;   // k-rows between consecutive vectors of a lane
    __device__ static unsigned lane_offset_bytes(int ld) {
        return 2u * ((threadIdx.x / kVecPerLine) * (unsigned)ld + (threadIdx.x % kVecPerLine) * 8u);
    }
    __device__ static int64_t line_step_bytes(int ld) { return 2 * (int64_t)kLineStep * ld; }
    __device__ static int64_t slice_step_bytes(int ld) { return 2 * (int64_t)BK * ld; }
    __device__ static uint16_t* lane_lds(uint16_t* lds) {
        return lds + (threadIdx.x / kVecPerLine) * kPitch + (threadIdx.x % kVecPerLine) * 8;
    }
    static constexpr int kLdsLineStep = kLineStep * kPitch;
};

}  // namespace ols
