// Small device helpers: bf16 <-> fp32, 8-element loads, wave reductions, MFMA types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rnnlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two floats to two bfloat16 (round to nearest even, one v_cvt_pk_bf16_f32), `lo` in the
// low half.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// x = x1 + x2 + x3 with bf16 terms (round to nearest even each time): the three-way split that
// puts an fp32 operand on the bf16 matrix cores.
__device__ __forceinline__ void split3_bf16(float x, uint16_t &x1, uint16_t &x2, uint16_t &x3) {
    const uint32_t p1 = pack_bf16x2(x, 0.f);
    const float r1 = x - __uint_as_float(p1 << 16);
    const uint32_t p2 = pack_bf16x2(r1, 0.f);
    const float r2 = r1 - __uint_as_float(p2 << 16);
    const uint32_t p3 = pack_bf16x2(r2, 0.f);
    x1 = (uint16_t)p1; x2 = (uint16_t)p2; x3 = (uint16_t)p3;
}

// Eight consecutive weights starting at element index `at` (a multiple of 8) as floats.
__device__ __forceinline__ void load8_weights(const uint16_t *p, size_t at, float (&out)[8]) {
    u32x4 v = *reinterpret_cast<const u32x4 *>(p + at);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(v[i] << 16);
        out[2 * i + 1] = __uint_as_float(v[i] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void load8_weights(const float *p, size_t at, float (&out)[8]) {
    f32x4 a = *reinterpret_cast<const f32x4 *>(p + at);
    f32x4 b = *reinterpret_cast<const f32x4 *>(p + at + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { out[i] = a[i]; out[4 + i] = b[i]; }
}

// Eight consecutive floats row[k0 .. k0+7] of a caller-owned row of length H (not padded);
// elements at or beyond H read as `fill`.  Vector loads when the row allows them.
__device__ __forceinline__ void load8_row(const float *row, int k0, int H, bool vec_ok, float fill,
                                          float (&out)[8]) {
    if (vec_ok && k0 + 8 <= H) {
        f32x4 a = *reinterpret_cast<const f32x4 *>(row + k0);
        f32x4 b = *reinterpret_cast<const f32x4 *>(row + k0 + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) { out[i] = a[i]; out[4 + i] = b[i]; }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = (k0 + i < H) ? row[k0 + i] : fill;
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// 2^x with the hardware instruction (x = -inf gives 0).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Merge two (max, sum) pairs of a base-2 log-sum-exp: value = 2^m * s.
__device__ __forceinline__ void lse2_merge(float &m, float &s, float m2, float s2) {
    float mm = fmaxf(m, m2);
    if (mm == -INFINITY) { m = mm; s = 0.f; return; }
    s = s * fast_exp2(m - mm) + s2 * fast_exp2(m2 - mm);
    m = mm;
}

// Fold sixteen base-2 logits of one row into the (max, sum) pair.
template <bool FIXED>
__device__ __forceinline__ void lse2_fold16(const float (&x)[16], float &mrun, float &srun) {
    if (FIXED) {
#pragma unroll
        for (int i = 0; i < 16; ++i) srun += fast_exp2(x[i]);          // offset already inside x
    } else {
        float mx = x[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, x[i]);
        const float mn = fmaxf(mrun, mx);
        if (mn != -INFINITY) {
            float tsum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) tsum += fast_exp2(x[i] - mn);
            srun = srun * fast_exp2(mrun - mn) + tsum;
            mrun = mn;
        }
    }
}

// Direct global->LDS load of 16 bytes per lane: lane i of the wave writes LDS bytes
// [lds_base + 16 i, lds_base + 16 i + 16) with the 16 bytes at sbase + voff (its own voff).
// sbase and lds_base must be the same in all lanes (they travel in SGPRs / M0).  Written as
// inline assembly on purpose: when the compiler knows of a pending LDS-DMA it makes every
// later LDS read wait for ALL outstanding LDS reads (lgkmcnt(0)) instead of just its own,
// which stalls the MFMA pipeline; completion is awaited explicitly with vmcnt before the
// workgroup barrier that publishes the data.  M0 is an input operand, so the compiler writes it
// and knows that it is in use; the s_nop is the wait state between that write and the load.
__device__ __forceinline__ void lds_dma_16(const void *sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "{m0}"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}

// The same with a full 64-bit address per lane (rows gathered from anywhere in a buffer).
__device__ __forceinline__ void lds_dma_16_ptr(const void *lane_ptr, uint32_t lds_base) {
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "{m0}"(lds_base), "v"(lane_ptr)
                 : "memory");
}

// The same as lds_dma_16 by lane 0 alone (16 bytes to lds_base), without a branch around it: the
// execution mask is narrowed to lane 0 for the one instruction and put back.  Counts as one
// vector-memory operation of the wave like any other load.
__device__ __forceinline__ void lds_dma_16_lane0(const void *sbase, uint32_t voff, uint32_t lds_base) {
    uint64_t saved_exec;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 1\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved_exec)
                 : "{m0}"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)reinterpret_cast<uintptr_t>(p);         // LDS offsets are the low 32 bits
}

// Wait until at most N of this wave's vector-memory operations are outstanding (vmcnt is a
// 6-bit field on gfx9: bits 3:0 and 15:14 of the immediate; lgkmcnt and expcnt left alone).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// 64-bit key -> 32 well-mixed bits (hash tables of history ids).
__device__ __forceinline__ uint32_t mix64(uint64_t k) {
    // splitmix64 finaliser
    k ^= k >> 30; k *= 0xBF58476D1CE4E5B9ull;
    k ^= k >> 27; k *= 0x94D049BB133111EBull;
    k ^= k >> 31;
    return (uint32_t)k;
}

// The same finaliser with all 64 bits kept.
__device__ __forceinline__ uint64_t mix64_full(uint64_t k) {
    k ^= k >> 30; k *= 0xBF58476D1CE4E5B9ull;
    k ^= k >> 27; k *= 0x94D049BB133111EBull;
    k ^= k >> 31;
    return k;
}

// Block-wide exclusive prefix sum of one int per thread; returns the exclusive prefix and,
// through `total`, the block sum.  `wsum` is LDS scratch of blockDim.x/64 + 1 ints.
__device__ __forceinline__ int block_exclusive_scan(int v, int *wsum, int &total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        int w = (lane < nwaves) ? wsum[lane] : 0;
        int wi = w;
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            int t = __shfl_up(wi, off, 64);
            if (lane >= off) wi += t;
        }
        if (lane < nwaves) wsum[lane] = wi - w;       // exclusive prefix of the wave sums
        if (lane == nwaves - 1) wsum[nwaves] = wi;    // block total
    }
    __syncthreads();
    int excl = wsum[wave] + incl - v;
    total = wsum[nwaves];
    __syncthreads();                                  // wsum may be reused by the caller
    return excl;
}

// Natural-log normaliser of one row from its `splits` per-split (max, sum) partials of the
// base-2 log-sum-exp, merged in a fixed order by one whole wave (every lane gets the result).
__device__ __forceinline__ float lse_from_partials(const float2 *part_row, int splits, int lane) {
    float pm = -INFINITY, ps = 0.f;
    for (int s = lane; s < splits; s += 64) {
        float2 p = part_row[s];
        lse2_merge(pm, ps, p.x, p.y);
    }
    const float mm = wave_max(pm);
    const float ss = wave_sum(mm == -INFINITY ? 0.f : ps * fast_exp2(pm - mm));
    return (mm + fast_log2(ss)) * 0.6931471805599453f;
}

// Batches of eight dot products per wave (query gather, hierarchical output layer): value u
// of a batch is finished by the lanes whose bits (5, 4, 3) spell u.
__device__ __forceinline__ int batch_slot_of_lane(int lane) {
    return ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
}
constexpr int lane_of_batch_slot(int u) { return 32 * ((u >> 2) & 1) + 16 * ((u >> 1) & 1) + 8 * (u & 1); }

// Sums over the wave of eight per-lane values at once: the same xor butterfly (32, 16, ...,
// 1) as wave_sum, but in the first three levels a lane passes on the half of the values it
// will not finish, so 10 exchanges do the work of 48.  Returns the sum of value
// batch_slot_of_lane(lane); bit-identical to wave_sum of that value.
__device__ __forceinline__ float wave_sum8(const float (&acc)[8], int lane) {
    float v4[4], v2[2];
    const bool up5 = (lane & 32) != 0, up4 = (lane & 16) != 0, up3 = (lane & 8) != 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) v4[i] = (up5 ? acc[4 + i] : acc[i]) + __shfl_xor(up5 ? acc[i] : acc[4 + i], 32, 64);
#pragma unroll
    for (int i = 0; i < 2; ++i) v2[i] = (up4 ? v4[2 + i] : v4[i]) + __shfl_xor(up4 ? v4[i] : v4[2 + i], 16, 64);
    float v = (up3 ? v2[1] : v2[0]) + __shfl_xor(up3 ? v2[0] : v2[1], 8, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 1, 64);
    return v;
}

__device__ __forceinline__ float quiet_nan() { return __uint_as_float(0x7FC00000u); }

}  // namespace rnnlm
