// Operand tiles of the fp32 MFMA GEMM kernels (v_mfma_f32_32x32x2_f32): how a ROWS x BK slice of an operand is copied
// global -> registers -> LDS in its own memory order with 16-byte vectors, and how a wavefront reads its MFMA
// fragments back.  Shared by the grouped GEMMs of the MLPs and the implicit-GEMM convolution kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ols {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;   // four wavefronts per workgroup

// One operand tile of ROWS x BK in LDS.  KC: stored [ROWS][BK + 4]; RC: stored [BK][ROWS + 4].
template <int ROWS, int BK, bool KC>
struct Tile {
    static constexpr int kPitch = KC ? BK + 4 : ROWS + 4;
    static constexpr int kLines = KC ? ROWS : BK;         // lines of contiguous memory
    static constexpr int kLineLen = KC ? BK : ROWS;       // elements per line
    static constexpr int kVecPerLine = kLineLen / 4;
    static constexpr int kVecs = kLines * kVecPerLine;
    static constexpr int kPerThread = (kVecs + kGemmThreads - 1) / kGemmThreads;
    static constexpr int kFloats = kLines * kPitch;

    // Global -> registers.  `base` points at the operand of this group; (row0, k0) is the tile origin;
    // rows / klen bound the valid region.  Row and k extents are multiples of 4.
    // Every lane ALWAYS issues its load (out-of-range lanes re-read the operand's first vector) and the
    // zero fill is applied only when the registers are written to LDS: with no branch around the loads
    // and no use of their result in between, the compiler can count outstanding loads and let a later
    // slice's loads stay in flight while an earlier slice is stored.
    __device__ static unsigned load(f4 (&r)[kPerThread], const float* __restrict__ base, int ld, int row0, int k0,
                                    int rows, int klen) {
        unsigned okmask = 0;
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * kGemmThreads;
            const int line = v / kVecPerLine, off = (v % kVecPerLine) * 4;
            const int row = KC ? row0 + line : row0 + off;
            const int k = KC ? k0 + off : k0 + line;
            const bool ok = (kVecs % kGemmThreads == 0 || v < kVecs) && row < rows && k < klen;
            const int64_t idx = KC ? (int64_t)row * ld + k : (int64_t)k * ld + row;
            r[t] = *(const f4*)(base + (ok ? idx : 0));
            okmask |= ok ? (1u << t) : 0u;
        }
        return okmask;
    }
    __device__ static void store(float* lds, const f4 (&r)[kPerThread], unsigned okmask) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * kGemmThreads;
            if (kVecs % kGemmThreads == 0 || v < kVecs) {
                const int line = v / kVecPerLine, off = (v % kVecPerLine) * 4;
                const f4 zero = {0.f, 0.f, 0.f, 0.f};
                *(f4*)(lds + line * kPitch + off) = (okmask >> t) & 1u ? r[t] : zero;
            }
        }
    }
    // Full tiles (no bounds to check): the lane's vectors of a slice sit at fixed 32-bit byte offsets from a
    // uniform base that advances by a uniform amount per slice, so a K loop iteration spends no vector
    // instructions on addresses or on zero-fill selects.
    __device__ static void lane_offsets(unsigned (&off)[kPerThread], int ld) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * kGemmThreads;
            const int line = v / kVecPerLine, o = (v % kVecPerLine) * 4;
            off[t] = 4u * (unsigned)(line * ld + o);
        }
    }
    // elements between the tile origins of consecutive slices
    __device__ static int64_t slice_step(int ld) { return KC ? (int64_t)BK : (int64_t)BK * ld; }
    __device__ static void load_full(f4 (&r)[kPerThread], const char* base, const unsigned (&off)[kPerThread]) {
        static_assert(kVecs % kGemmThreads == 0, "full tiles need a whole number of vectors per lane");
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) r[t] = *(const f4*)(base + off[t]);
    }
    __device__ static void store_full(float* lds, const f4 (&r)[kPerThread]) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * kGemmThreads;
            *(f4*)(lds + (v / kVecPerLine) * kPitch + (v % kVecPerLine) * 4) = r[t];
        }
    }
    // Fragment of the 32-row block starting at `r0` for k-octet q: four values, one per MFMA step e,
    // value e belonging to k = 8 q + 4 half + e.
    __device__ static f4 frag(const float* lds, int r0, int q, int lane32, int half) {
        if (KC) return *(const f4*)(lds + (r0 + lane32) * kPitch + 8 * q + 4 * half);
        f4 v;
        const float* p = lds + (8 * q + 4 * half) * kPitch + r0 + lane32;
        v.x = p[0];
        v.y = p[kPitch];
        v.z = p[2 * kPitch];
        v.w = p[3 * kPitch];
        return v;
    }
};

}  // namespace ols
