// Pieces shared by the matrix-core kernels of the recurrent gate (Eq. 3): operand types, the gate
// nonlinearities, the workgroup geometry that fixes the packed weight layouts, and the power-of-two scale of W_hh.
#pragma once
#include "common.hpp"

namespace kvev {

typedef _Float16 f16_t;
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

// Gate nonlinearities through the hardware exp2 and reciprocal (about 1 ulp
// each).  Their absolute error stays below ~2e-7 everywhere, which is what the
// cell update needs (it consumes the values, not their logarithms): the
// relative error of exp(x) grows like |x| * 2^-24, but it is multiplied by
// s(1-s), which decays exponentially.
__device__ __forceinline__ float sigmoid_hw(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * -1.4426950408889634f));
}
__device__ __forceinline__ float tanh_hw(float x)
{
    return fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * 2.8853900817779268f)), 1.0f);
}

// Hardware workgroup ids go round-robin over the 8 XCDs.  Give each XCD a
// contiguous run of sequence groups, i.e. a few layers at a time, so that the
// layer weights a workgroup streams every step stay in that XCD's 4 MB L2
// instead of all layers cycling through all eight of them.
__device__ __forceinline__ int xcd_order(int block, int nblocks)
{
    return nblocks % 8 == 0 ? (block % 8) * (nblocks / 8) + block / 8 : block;
}

// Geometry shared by the three kernels: unit tiles per wave, waves per workgroup,
// and the order in which a wave walks its ITEMS = UT*KS weight items per step (an
// item = the 4 gate fragments of one unit tile at one k-step, 4 KiB per wave): one
// unit tile after the other, so that only 4 accumulators are live and the cell
// update of a finished tile overlaps with the other waves' MFMAs.
template <int DG> struct Geo {
    static constexpr int UT = DG == 512 ? 4 : 2;   // keeps the workgroup at 8 waves (256 registers per lane)
    static constexpr int NW = DG / (16 * UT);
    static constexpr int KS = DG / 32;
    static constexpr int THREADS = NW * 64;
    static constexpr int ITEMS = UT * KS;
    static constexpr int ut_of(int i) { return i / KS; }
    static constexpr int ks_of(int i) { return i % KS; }
};

// Scratch layout of the input projections: 1 KiB blocks of 64 lanes x 4 floats, one per
// (group of 16 sequences, step of the block, wave, unit tile, gate).
template <int DG>
__device__ __forceinline__ size_t xp_block(int group, int tb, int tt, int wave, int ut, int q)
{
    return ((((size_t)group * tb + tt) * Geo<DG>::NW + wave) * Geo<DG>::UT + ut) * 4 + q;
}

__device__ __forceinline__ void lds_barrier()
{
    // LDS traffic of this wave done, then the barrier: unlike __syncthreads() this does not wait for the global
    // stores in flight (a publication to other workgroups), which nobody in the workgroup reads
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

constexpr int kScaleBlocks = 32;   // partial maxima of |W_hh| per layer (one per preparation workgroup)

// The power of two s that lifts max |W_hh| of a layer into [2^14, 2^15), from the
// bit pattern of that maximum (s = 1 for an all-zero matrix).
__device__ __forceinline__ int whh_scale_exp(uint32_t max_bits)
{
    const float m = __uint_as_float(max_bits);
    int k = m > 0.f ? 14 - ilogbf(m) : 0;
    return k > 100 ? 100 : k < -100 ? -100 : k;
}

// max |W_hh| of a layer from the kScaleBlocks partial maxima
__device__ __forceinline__ uint32_t whh_layer_max(const uint32_t *max_bits, int l)
{
    uint32_t m = 0;
#pragma unroll 8
    for (int p = 0; p < kScaleBlocks; ++p) m = max(m, max_bits[l * kScaleBlocks + p]);
    return m;
}

}  // namespace kvev
