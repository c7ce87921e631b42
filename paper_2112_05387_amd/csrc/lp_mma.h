// MFMA micro-tile wrappers for gfx950 (wave64).
//
// All kernels keep both GEMM operands in LDS as [row][k] with k contiguous and read them as 16-byte
// fragments: lane l of a wave reads row (l % MT) of a micro-tile and the 16-byte k-chunk (l / MT).
// One "k-step" therefore covers KSTEP = (64/MT) * (16/sizeof(T)) reduction elements:
//   bf16, MT=16: v_mfma_f32_16x16x32_bf16 (one instruction, 32 k)
//   bf16, MT=32: v_mfma_f32_32x32x16_bf16 (one instruction, 16 k)
//   f32,  MT=16: 4 x v_mfma_f32_16x16x4_f32 (element e of each lane's chunk feeds instruction e; the
//                hardware's k slot (l/16) then stands for k = 4*(l/16)+e, identically for A and B)
//   f32,  MT=32: 4 x v_mfma_f32_32x32x2_f32
// Accumulator layout (both dtypes): column = l % MT; MT=16: rows 4*(l/16)+r, r<4;
// MT=32: rows 8*(r/4) + 4*(l/32) + r%4, r<16.
#pragma once
#include <hip/hip_runtime.h>

namespace lp {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct bf16_t { unsigned short v; };   // storage-only bfloat16

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((unsigned)x.v) << 16); }
__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {   // round to nearest even
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);   // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
// two floats -> packed bf16 pair (low half = a), round to nearest even in hardware (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b) {
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
template <typename T> __device__ __forceinline__ T from_float(float f);
template <> __device__ __forceinline__ float from_float<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float f) { bf16_t r; r.v = float_to_bf16_bits(f); return r; }

template <int MT> struct AccT;
template <> struct AccT<16> { typedef f32x4 type; static constexpr int N = 4; };
template <> struct AccT<32> { typedef f32x16 type; static constexpr int N = 16; };

// row of accumulator register r inside the micro-tile
template <int MT> __device__ __forceinline__ int acc_row(int r, int lane) {
    if constexpr (MT == 16) return 4 * (lane >> 4) + r;
    else return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

template <typename T, int MT> struct Mma;

template <> struct Mma<bf16_t, 16> {
    __device__ static __forceinline__ void run(const u32x4& a, const u32x4& b, f32x4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<bf16_t, 32> {
    __device__ static __forceinline__ void run(const u32x4& a, const u32x4& b, f32x16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float, 16> {
    __device__ static __forceinline__ void run(const u32x4& a, const u32x4& b, f32x4& c) {
        f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[0], bf[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[1], bf[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[2], bf[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[3], bf[3], c, 0, 0, 0);
    }
};
template <> struct Mma<float, 32> {
    __device__ static __forceinline__ void run(const u32x4& a, const u32x4& b, f32x16& c) {
        f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[0], bf[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[1], bf[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[2], bf[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[3], bf[3], c, 0, 0, 0);
    }
};

// One k-tile of a wave's FM x FN micro-tiles from LDS operands laid out [row][PITCH] (k contiguous).
template <typename T, int MT, int FM, int FN, int BK, int PITCH>
__device__ __forceinline__ void mma_ktile(const T* __restrict__ As, const T* __restrict__ Bs,
                                          int a_row0, int b_row0, int lane,
                                          typename AccT<MT>::type (&acc)[FM][FN]) {
    constexpr int EPV = 16 / (int)sizeof(T);
    constexpr int KSTEP = (64 / MT) * EPV;
    const int lr = lane % MT, lk = (lane / MT) * EPV;
#pragma unroll
    for (int ks = 0; ks < BK / KSTEP; ++ks) {
        u32x4 af[FM], bfr[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i)
            af[i] = *reinterpret_cast<const u32x4*>(As + (a_row0 + i * MT + lr) * PITCH + ks * KSTEP + lk);
#pragma unroll
        for (int j = 0; j < FN; ++j)
            bfr[j] = *reinterpret_cast<const u32x4*>(Bs + (b_row0 + j * MT + lr) * PITCH + ks * KSTEP + lk);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) Mma<T, MT>::run(af[i], bfr[j], acc[i][j]);
    }
}

}  // namespace lp
