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

// Parameter update of a finished gradient tile by one workgroup of NT threads (epilogues of the filter-gradient
// kernels):  g' = dW + wd * W;  v <- momentum * v + g';  W <- W - lr * (v or g')  -- the arithmetic of the parameter-update
// kernel, element by element.  The tile is `nrows` runs of `ncols` consecutive elements; run q starts at element
// row_start(q) of the filter / gradient / velocity / master tensors (all in the filter's [Cout][R][S][Cin] order).
// Runs whose start and length are multiples of four go as 16-byte vectors (8 bytes of a bf16 filter), U vectors per
// thread in flight: all loads of a trip first, then the arithmetic, then the stores.
struct SgdCoef { float lr, momentum, wd; bool lowp; };

// The gradient was accumulated by device-scope atomics of workgroups on other XCDs, i.e. at the memory side, past the
// L2 of this XCD, which may still hold the line as the clearing kernel left it: read it at device scope as well.
__device__ __forceinline__ float load_agent(const float* p) {
    return __hip_atomic_load(const_cast<float*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float sgd_step(float& v, float w, float grad, bool has_v, const SgdCoef& c) {
    float d = fmaf(c.wd, w, grad);
    if (has_v) { d = fmaf(c.momentum, v, d); v = d; }
    return fmaf(-c.lr, d, w);
}

template <int NT, int U, typename RowStart>
__device__ __forceinline__ void sgd_update_tile(void* __restrict__ w, float* __restrict__ vel, float* __restrict__ master,
                                                const float* __restrict__ dw, int nrows, int ncols, bool vec4, RowStart row_start,
                                                const SgdCoef& c, int tid) {
    unsigned short* wl = reinterpret_cast<unsigned short*>(w);
    float* wf = reinterpret_cast<float*>(w);
    if (vec4) {
        const int vpr = ncols >> 2, nvec = nrows * vpr;
        for (int v0 = tid; v0 < nvec; v0 += NT * U) {
            size_t idx[U]; bool ok[U];
            f32x4 gr[U], x[U], vv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v = v0 + u * NT;
                ok[u] = v < nvec;
                const int q = ok[u] ? v / vpr : 0, cv = ok[u] ? v - q * vpr : 0;
                idx[u] = row_start(q) + 4 * (size_t)cv;
#pragma unroll
                for (int e = 0; e < 4; ++e) gr[u][e] = load_agent(dw + idx[u] + e);
                if (master) x[u] = *reinterpret_cast<const f32x4*>(master + idx[u]);
                else if (c.lowp) {
                    const u32x2 r = *reinterpret_cast<const u32x2*>(wl + idx[u]);
                    x[u][0] = __uint_as_float(r[0] << 16); x[u][1] = __uint_as_float(r[0] & 0xffff0000u);
                    x[u][2] = __uint_as_float(r[1] << 16); x[u][3] = __uint_as_float(r[1] & 0xffff0000u);
                } else x[u] = *reinterpret_cast<const f32x4*>(wf + idx[u]);
                if (vel) vv[u] = *reinterpret_cast<const f32x4*>(vel + idx[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!ok[u]) continue;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float ve = vel ? vv[u][e] : 0.f;
                    x[u][e] = sgd_step(ve, x[u][e], gr[u][e], vel != nullptr, c);
                    vv[u][e] = ve;
                }
                if (vel) *reinterpret_cast<f32x4*>(vel + idx[u]) = vv[u];
                if (master) *reinterpret_cast<f32x4*>(master + idx[u]) = x[u];
                if (c.lowp) {
                    u32x2 r; r[0] = pack_bf16x2(x[u][0], x[u][1]); r[1] = pack_bf16x2(x[u][2], x[u][3]);
                    *reinterpret_cast<u32x2*>(wl + idx[u]) = r;
                } else *reinterpret_cast<f32x4*>(wf + idx[u]) = x[u];
            }
        }
    } else {
        const int n = nrows * ncols;
        for (int i = tid; i < n; i += NT) {
            const int q = i / ncols;
            const size_t id = row_start(q) + (size_t)(i - q * ncols);
            float x = master ? master[id] : (c.lowp ? bf16_bits_to_float(wl[id]) : wf[id]);
            float ve = vel ? vel[id] : 0.f;
            x = sgd_step(ve, x, load_agent(dw + id), vel != nullptr, c);
            if (vel) vel[id] = ve;
            if (master) master[id] = x;
            if (c.lowp) wl[id] = float_to_bf16_bits(x);
            else wf[id] = x;
        }
    }
}

}  // namespace lp
