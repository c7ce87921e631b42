// Grouped HBM-bound kernels of the local step: batch-norm apply (+ReLU, +skip), batch-norm backward
// (reduce / apply), the local penalty / augmented-Lagrangian loss and terminal adjoint, the multiplier
// update, the classification head, max pooling and buffer clears.  NHWC, 16-byte accesses with the
// channel index fastest, fp32 arithmetic, wavefront/LDS reductions, one atomic per channel per workgroup.
#include "lp_kernels.h"
#include "lp_mma.h"

namespace lp {

namespace {

template <typename T> struct Vec {
    static constexpr int N = 16 / (int)sizeof(T);
    __device__ static __forceinline__ void load(const T* p, float (&f)[N]) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(p);
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(v[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                f[2 * e] = __uint_as_float(v[e] << 16);
                f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
            }
        }
    }
    // the 16 bytes as loaded, and their conversion: kernels that want many loads in flight issue all load_raw first
    __device__ static __forceinline__ u32x4 load_raw(const T* p) { return *reinterpret_cast<const u32x4*>(p); }
    __device__ static __forceinline__ void unpack(const u32x4& v, float (&f)[N]) {
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(v[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                f[2 * e] = __uint_as_float(v[e] << 16);
                f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
            }
        }
    }
    __device__ static __forceinline__ void store(T* p, const float (&f)[N]) {
        u32x4 v;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(f[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[e] = pack_bf16x2(f[2 * e], f[2 * e + 1]);
        }
        *reinterpret_cast<u32x4*>(p) = v;
    }
};

__device__ __forceinline__ void bn_coeffs(const double* stats, const float* gamma, const float* beta, int c, int C,
                                          int M, float eps, float& sc, float& sh, float& mean, float& invstd) {
    const double inv_m = 1.0 / (double)M;          // the same for every channel: the compiler hoists it out of loops
    double s1 = 0.0, s2 = 0.0;
    const int ns = stat_stripes(C);
    for (int st = 0; st < ns; ++st) { s1 += stats[st * 2 * C + c]; s2 += stats[st * 2 * C + C + c]; }
    const double mu = s1 * inv_m;
    double var = s2 * inv_m - mu * mu;
    if (var < 0.0) var = 0.0;
    mean = (float)mu;
    invstd = rsqrtf((float)var + eps);
    sc = gamma[c] * invstd;
    sh = beta[c] - mean * sc;
}

template <typename G> __device__ __forceinline__ int find_problem(const G& g, int bid) {
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if (bid >= g.p[i].block_start) pi = i;
    return pi;
}

constexpr int kMaxC = 2048;

// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum(float v, float* s_tmp);

// FUSE: the pass also evaluates the local loss and terminal adjoint of the interface tensor it writes (exactly the
// arithmetic of loss_kernel, on the value as stored, vector by vector in the same order)
template <typename T, bool FUSE>
__global__ __launch_bounds__(kElemBlock) void bn_apply_kernel(const BnApplyGroup g) {
    constexpr int EPV = Vec<T>::N;
    // per-channel coefficients: 4 arrays of g.cmax floats (sized by the launch: the LDS footprint limits occupancy)
    extern __shared__ __attribute__((aligned(16))) float s_coef[];
    const int cm = 4 * (g.cmax >> 2);      // written as a multiple of 4 so that the arrays are visibly 16-byte aligned
    float* s_sc = s_coef;
    float* s_sh = s_coef + cm;
    float* s_ssc = s_coef + 2 * cm;
    float* s_ssh = s_coef + 3 * cm;
    const BnApplyProb& P = g.p[find_problem(g, blockIdx.x)];
    const int C = P.C, M = P.M;
    for (int c = threadIdx.x; c < C; c += kElemBlock) {
        float sc, sh, mu, is;
        bn_coeffs(P.stats, P.gamma, P.beta, c, C, M, g.eps, sc, sh, mu, is);
        s_sc[c] = sc; s_sh[c] = sh;
        if (P.skip_mode == 2) {
            bn_coeffs(P.sstats, P.sgamma, P.sbeta, c, C, M, g.eps, sc, sh, mu, is);
            s_ssc[c] = sc; s_ssh[c] = sh;
        }
    }
    __syncthreads();
    const T* __restrict__ y = reinterpret_cast<const T*>(P.y);
    const T* __restrict__ skip = reinterpret_cast<const T*>(P.skip);
    T* __restrict__ out = reinterpret_cast<T*>(P.out);
    const size_t nvec = (size_t)M * C / EPV;
    const int cv = C / EPV;
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    // four vectors per trip, loads first: up to eight independent 16-byte loads in flight per thread
    constexpr int U = 4;
    // channel vector of this thread's first vector; it advances by kElemBlock (mod cv) from vector to vector, which
    // avoids a 64-bit remainder per vector
    const unsigned cstep = (unsigned)kElemBlock % (unsigned)cv;
    unsigned cidx = (unsigned)((base + threadIdx.x) % (size_t)cv);
    const T* __restrict__ xn = reinterpret_cast<const T*>(P.xn);
    const T* lam = reinterpret_cast<const T*>(P.lam);
    T* lam_out = reinterpret_cast<T*>(P.lam_out);          // may alias lam: every vector is read before it is written
    T* __restrict__ dyp = reinterpret_cast<T*>(P.dy);
    float lacc = 0.f, racc = 0.f;
    for (int i0 = threadIdx.x; i0 < kElemVecsPerBlock; i0 += U * kElemBlock) {
        // Unconditional loads (a vector beyond the end re-reads the last one and is dropped): behind a per-lane branch
        // the compiler waits for each pair of loads before it issues the next.
        u32x4 fraw[U], skraw[U], xnraw[FUSE ? U : 1], lmraw[FUSE ? U : 1];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t v = base + i0 + u * kElemBlock;
            ok[u] = v < nvec;
            const size_t vc = ok[u] ? v : nvec - 1;
            fraw[u] = Vec<T>::load_raw(y + vc * EPV);
            if (P.skip_mode) skraw[u] = Vec<T>::load_raw(skip + vc * EPV);
            if constexpr (FUSE) {
                xnraw[u] = Vec<T>::load_raw(xn + vc * EPV);
                if (lam) lmraw[u] = Vec<T>::load_raw(lam + vc * EPV);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c0 = (int)cidx * EPV;
            cidx += cstep;
            if (cidx >= (unsigned)cv) cidx -= (unsigned)cv;
            if (!ok[u]) continue;
            const size_t v = base + i0 + u * kElemBlock;
            float f[1][EPV], sk[1][EPV], o[EPV];
            Vec<T>::unpack(fraw[u], f[0]);
            if (P.skip_mode) Vec<T>::unpack(skraw[u], sk[0]);
#pragma unroll
            for (int e = 0; e < EPV; ++e) o[e] = fmaf(s_sc[c0 + e], f[0][e], s_sh[c0 + e]);
            if (P.skip_mode == 2) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) o[e] += fmaf(s_ssc[c0 + e], sk[0][e], s_ssh[c0 + e]);
            } else if (P.skip_mode == 1) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) o[e] += sk[0][e];
            }
            if (P.relu) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) o[e] = fmaxf(o[e], 0.f);
            }
            Vec<T>::store(out + v * EPV, o);
            if constexpr (FUSE) {
                if constexpr (sizeof(T) == 2) {             // the loss is defined on F_k(x_k) as stored
#pragma unroll
                    for (int e = 0; e < EPV; e += 2) {
                        const unsigned pk = pack_bf16x2(o[e], o[e + 1]);
                        o[e] = __uint_as_float(pk << 16); o[e + 1] = __uint_as_float(pk & 0xffff0000u);
                    }
                }
                float b[EPV], l[EPV], d[EPV];
                Vec<T>::unpack(xnraw[u], b);
                if (lam) Vec<T>::unpack(lmraw[u], l);
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const float r = o[e] - b[e];
                    const float lm = lam ? l[e] : 0.f;
                    lacc += 0.5f * g.rho * r * r + lm * r;
                    racc += r * r;
                    d[e] = g.scale * (g.rho * r + lm);
                }
                Vec<T>::store(dyp + v * EPV, d);
                if (lam && lam_out) {
#pragma unroll
                    for (int e = 0; e < EPV; ++e) l[e] = fmaf(g.step, o[e] - b[e], l[e]);
                    Vec<T>::store(lam_out + v * EPV, l);
                }
            }
        }
    }
    if constexpr (FUSE) {
        __shared__ float s_tmp[kElemBlock / 64];
        const float tot = block_sum(lacc, s_tmp);
        if (threadIdx.x == 0 && tot != 0.f) atomicAdd(P.loss, g.scale * tot);
        if (P.r2) {
            const float rt = block_sum(racc, s_tmp);
            if (threadIdx.x == 0 && rt != 0.f) atomicAdd(P.r2, rt);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// red[c] += sum g', red[C+c] += sum g'*yhat over this workgroup's rows.
// C / EPV <= NT channel vectors (C <= 2048): thread t owns channel vector t % cv and is row lane t / cv.  A trip is
// four rows per row lane, i.e. eight independent 16-byte loads per thread.  The trips of the blocks are interleaved
// (block b takes trips b, b + nblocks, ...), so that at any time the blocks together read one contiguous, moving window
// of the two tensors instead of nblocks distant streams.  The first trip is requested before the coefficient prologue
// (it does not depend on it) and every further trip before the previous one is consumed.
template <typename T, int NT>
__global__ __launch_bounds__(NT) void bn_bwd_reduce_kernel(const BnBwdGroup g) {
    constexpr int EPV = Vec<T>::N;
    __shared__ float s_red[NT * EPV * 2];
    // per-channel coefficients, computed once per workgroup (4 arrays of g.cmax floats, sized by the launch)
    extern __shared__ __attribute__((aligned(16))) float s_coef[];
    const int cm = 4 * (g.cmax >> 2);
    float* s_sc = s_coef;
    float* s_sh = s_coef + cm;
    float* s_mu = s_coef + 2 * cm;
    float* s_is = s_coef + 3 * cm;
    const BnBwdProb& P = g.p[find_problem(g, blockIdx.x)];
    const int C = P.C, M = P.M, cv = C / EPV;
    const int b = blockIdx.x - P.block_start;
    const T* __restrict__ gp = reinterpret_cast<const T*>(P.g);
    const T* __restrict__ y = reinterpret_cast<const T*>(P.y);
    const int rl = NT / cv;                      // row lanes
    const int tcv = threadIdx.x % cv, trl = threadIdx.x / cv;
    const bool active = trl < rl;
    const int c0 = tcv * EPV;
    const int rows_trip = 4 * rl, stride = P.nblocks * rows_trip;
    // a trip as loaded (32 registers); rows past the end read the last row and count as zero when consumed
    auto request = [&](u32x4 (&graw)[4], u32x4 (&yraw)[4], int r0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = min(r0 + trl + u * rl, M - 1);
            graw[u] = Vec<T>::load_raw(gp + (size_t)r * C + c0);
            yraw[u] = Vec<T>::load_raw(y + (size_t)r * C + c0);
        }
    };
    u32x4 ga[4], ya[4], gb[4], yb[4];
    int r0 = b * rows_trip;
    if (active && r0 < M) request(ga, ya, r0);
    for (int c = threadIdx.x; c < C; c += NT) {
        float sc, sh, mu, is;
        bn_coeffs(P.stats, P.gamma, P.beta, c, C, M, g.eps, sc, sh, mu, is);
        s_sc[c] = sc; s_sh[c] = sh; s_mu[c] = mu; s_is[c] = is;
    }
    __syncthreads();
    float a1[EPV], a2[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) { a1[e] = 0.f; a2[e] = 0.f; }
    if (active) {
        float sc[EPV], sh[EPV], mu[EPV], is[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) { sc[e] = s_sc[c0 + e]; sh[e] = s_sh[c0 + e]; mu[e] = s_mu[c0 + e]; is[e] = s_is[c0 + e]; }
        auto consume = [&](const u32x4 (&graw)[4], const u32x4 (&yraw)[4], int rbase) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float gv[EPV], yv[EPV];
                Vec<T>::unpack(graw[u], gv);
                Vec<T>::unpack(yraw[u], yv);
                const bool in = rbase + trl + u * rl < M;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    float gg = in ? gv[e] : 0.f;
                    if (P.relu && !(fmaf(sc[e], yv[e], sh[e]) > 0.f)) gg = 0.f;
                    a1[e] += gg;
                    a2[e] += gg * ((yv[e] - mu[e]) * is[e]);
                }
            }
        };
        while (r0 < M) {
            int rn = r0 + stride;
            if (rn < M) request(gb, yb, rn);
            __builtin_amdgcn_sched_barrier(0);
            consume(ga, ya, r0);
            if (rn >= M) break;
            r0 = rn; rn = r0 + stride;
            if (rn < M) request(ga, ya, rn);
            __builtin_amdgcn_sched_barrier(0);
            consume(gb, yb, r0);
            r0 = rn;
        }
    }
    if (active) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            s_red[((trl * cv + tcv) * EPV + e) * 2] = a1[e];
            s_red[((trl * cv + tcv) * EPV + e) * 2 + 1] = a2[e];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cv * EPV; i += NT) {
        float s1 = 0.f, s2 = 0.f;
        for (int l = 0; l < rl; ++l) { s1 += s_red[((l * cv * EPV) + i) * 2]; s2 += s_red[((l * cv * EPV) + i) * 2 + 1]; }
        double* red = P.red + (size_t)(blockIdx.x % stat_stripes(C)) * 2 * C;
        atomicAdd(&red[i], (double)s1);
        atomicAdd(&red[C + i], (double)s2);
    }
}

// red[c] += sum y, red[C+c] += sum y^2 over this workgroup's rows (batch statistics of a tensor no convolution
// of this module produced: a module input in the pre-activation order)
template <typename T>
__global__ __launch_bounds__(kElemBlock) void bn_stats_kernel(const BnBwdGroup g) {
    constexpr int EPV = Vec<T>::N;
    __shared__ float s_red[kElemBlock * EPV * 2];
    const BnBwdProb& P = g.p[find_problem(g, blockIdx.x)];
    const int C = P.C, M = P.M, cv = C / EPV;
    const int b = blockIdx.x - P.block_start;
    const int rows_pb = (M + P.nblocks - 1) / P.nblocks;
    const int row0 = b * rows_pb, row1 = min(M, row0 + rows_pb);
    const T* __restrict__ y = reinterpret_cast<const T*>(P.y);
    for (int cbase = 0; cbase < cv; cbase += kElemBlock) {
        const int ncv = min(cv - cbase, kElemBlock);
        const int rl = kElemBlock / ncv;
        const int tcv = threadIdx.x % ncv, trl = threadIdx.x / ncv;
        float a1[EPV], a2[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) { a1[e] = 0.f; a2[e] = 0.f; }
        if (trl < rl) {
            const int c0 = (cbase + tcv) * EPV;
            int r = row0 + trl;
            for (; r + 3 * rl < row1; r += 4 * rl) {
                float yv[4][EPV];
#pragma unroll
                for (int u = 0; u < 4; ++u) Vec<T>::load(y + (size_t)(r + u * rl) * C + c0, yv[u]);
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int e = 0; e < EPV; ++e) { a1[e] += yv[u][e]; a2[e] += yv[u][e] * yv[u][e]; }
            }
            for (; r < row1; r += rl) {
                float yv[EPV];
                Vec<T>::load(y + (size_t)r * C + c0, yv);
#pragma unroll
                for (int e = 0; e < EPV; ++e) { a1[e] += yv[e]; a2[e] += yv[e] * yv[e]; }
            }
        }
        __syncthreads();
        if (trl < rl) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                s_red[((trl * ncv + tcv) * EPV + e) * 2] = a1[e];
                s_red[((trl * ncv + tcv) * EPV + e) * 2 + 1] = a2[e];
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < ncv * EPV; i += kElemBlock) {
            float s1 = 0.f, s2 = 0.f;
            for (int l = 0; l < rl; ++l) { s1 += s_red[((l * ncv * EPV) + i) * 2]; s2 += s_red[((l * ncv * EPV) + i) * 2 + 1]; }
            const int c = cbase * EPV + i;
            double* red = P.red + (size_t)(blockIdx.x % stat_stripes(C)) * 2 * C;
            atomicAdd(&red[c], (double)s1);
            atomicAdd(&red[C + c], (double)s2);
        }
    }
}

// dy = gamma*invstd*(g' - red0/M - yhat*red1/M)
template <typename T>
__global__ __launch_bounds__(kElemBlock) void bn_bwd_apply_kernel(const BnBwdGroup g) {
    constexpr int EPV = Vec<T>::N;
    // per-channel coefficients: 5 arrays of g.cmax floats (sized by the launch: the LDS footprint limits occupancy)
    extern __shared__ __attribute__((aligned(16))) float s_coef[];
    const int cm = 4 * (g.cmax >> 2);      // written as a multiple of 4 so that the arrays are visibly 16-byte aligned
    float* s_sc = s_coef;
    float* s_sh = s_coef + cm;
    float* s_k1 = s_coef + 2 * cm;
    float* s_k2 = s_coef + 3 * cm;
    float* s_k3 = s_coef + 4 * cm;
    const BnBwdProb& P = g.p[find_problem(g, blockIdx.x)];
    const int C = P.C, M = P.M;
    const bool first = (int)blockIdx.x == P.block_start;
    for (int c = threadIdx.x; c < C; c += kElemBlock) {
        float sc, sh, mu, is;
        bn_coeffs(P.stats, P.gamma, P.beta, c, C, M, g.eps, sc, sh, mu, is);
        const double inv_m = 1.0 / (double)M;
        double rs0 = 0.0, rs1 = 0.0;
        for (int st = 0; st < stat_stripes(C); ++st) { rs0 += P.red[st * 2 * C + c]; rs1 += P.red[st * 2 * C + C + c]; }
        const float r0 = (float)(rs0 * inv_m), r1 = (float)(rs1 * inv_m);
        const float k1 = P.gamma[c] * is;
        const float k2 = k1 * is * r1;
        s_sc[c] = sc; s_sh[c] = sh;
        s_k1[c] = k1; s_k2[c] = k2; s_k3[c] = k2 * mu - k1 * r0;
        if (first) {
            P.dgamma[c] = (float)rs1;
            P.dbeta[c] = (float)rs0;
        }
    }
    __syncthreads();
    const T* __restrict__ gp = reinterpret_cast<const T*>(P.g);
    const T* __restrict__ y = reinterpret_cast<const T*>(P.y);
    T* __restrict__ dy = reinterpret_cast<T*>(P.dy);
    const size_t nvec = (size_t)M * C / EPV;
    const int cv = C / EPV;
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    const unsigned cstep = (unsigned)kElemBlock % (unsigned)cv;     // channel vector advances by kElemBlock (mod cv)
    unsigned cidx = (unsigned)((base + threadIdx.x) % (size_t)cv);
    for (int i = threadIdx.x; i < kElemVecsPerBlock; i += kElemBlock) {
        const size_t v = base + i;
        if (v >= nvec) break;
        const int c0 = (int)cidx * EPV;
        cidx += cstep;
        if (cidx >= (unsigned)cv) cidx -= (unsigned)cv;
        float gv[EPV], yv[EPV], o[EPV];
        Vec<T>::load(gp + v * EPV, gv);
        Vec<T>::load(y + v * EPV, yv);
        // the five coefficient vectors of these EPV channels, as 16-byte LDS reads
        float sc[EPV], sh[EPV], k1[EPV], k2[EPV], k3[EPV];
#pragma unroll
        for (int q4 = 0; q4 < EPV / 4; ++q4) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(s_sc + c0 + 4 * q4), b = *reinterpret_cast<const f32x4*>(s_sh + c0 + 4 * q4);
            const f32x4 c = *reinterpret_cast<const f32x4*>(s_k1 + c0 + 4 * q4), d = *reinterpret_cast<const f32x4*>(s_k2 + c0 + 4 * q4);
            const f32x4 f = *reinterpret_cast<const f32x4*>(s_k3 + c0 + 4 * q4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { sc[4 * q4 + e] = a[e]; sh[4 * q4 + e] = b[e]; k1[4 * q4 + e] = c[e]; k2[4 * q4 + e] = d[e]; k3[4 * q4 + e] = f[e]; }
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            float gg = gv[e];
            if (P.relu && !(fmaf(sc[e], yv[e], sh[e]) > 0.f)) gg = 0.f;
            o[e] = k1[e] * gg - k2[e] * yv[e] + k3[e];
        }
        if (P.add) {
            float av[EPV];
            Vec<T>::load(reinterpret_cast<const T*>(P.add) + v * EPV, av);
#pragma unroll
            for (int e = 0; e < EPV; ++e) o[e] += av[e];
        }
        Vec<T>::store(dy + v * EPV, o);
    }
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kElemBlock) void fill_kernel(const FillGroup g) {
    const FillProb& P = g.p[find_problem(g, blockIdx.x)];
    const size_t nvec = P.bytes / 16;
    u32x4* p = reinterpret_cast<u32x4*>(P.ptr);
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int i = threadIdx.x; i < kElemVecsPerBlock; i += kElemBlock) {
        const size_t v = base + i;
        if (v >= nvec) break;
        p[v] = z;
    }
}

__device__ __forceinline__ float block_sum(float v, float* s_tmp) {
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) v += __shfl_xor(v, sh, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) s_tmp[wave] = v;
    __syncthreads();
    float r = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) r += s_tmp[w];
    return r;
}

// local penalty / augmented-Lagrangian term and terminal adjoint
template <typename T>
__global__ __launch_bounds__(kElemBlock) void loss_kernel(const LossGroup g) {
    constexpr int EPV = Vec<T>::N;
    __shared__ float s_tmp[kElemBlock / 64];
    const LossProb& P = g.p[find_problem(g, blockIdx.x)];
    const T* __restrict__ y = reinterpret_cast<const T*>(P.y);
    const T* __restrict__ xn = reinterpret_cast<const T*>(P.xn);
    const T* lam = reinterpret_cast<const T*>(P.lam);
    T* lam_out = reinterpret_cast<T*>(P.lam_out);          // may alias lam: every vector is read before it is written
    T* __restrict__ dy = reinterpret_cast<T*>(P.dy);
    const size_t nvec = P.numel / EPV;
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    float acc = 0.f, racc = 0.f;
    for (int i = threadIdx.x; i < kElemVecsPerBlock; i += kElemBlock) {
        const size_t v = base + i;
        if (v >= nvec) break;
        float a[EPV], b[EPV], l[EPV], o[EPV];
        Vec<T>::load(y + v * EPV, a);
        Vec<T>::load(xn + v * EPV, b);
        if (lam) Vec<T>::load(lam + v * EPV, l);
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float r = a[e] - b[e];
            const float lm = lam ? l[e] : 0.f;
            acc += 0.5f * g.rho * r * r + lm * r;
            racc += r * r;
            o[e] = g.scale * (g.rho * r + lm);
        }
        Vec<T>::store(dy + v * EPV, o);
        if (lam && lam_out) {       // multiplier update of the same interface, from the same y - x_next
#pragma unroll
            for (int e = 0; e < EPV; ++e) l[e] = fmaf(g.step, a[e] - b[e], l[e]);
            Vec<T>::store(lam_out + v * EPV, l);
        }
    }
    const float tot = block_sum(acc, s_tmp);
    if (threadIdx.x == 0 && tot != 0.f) atomicAdd(P.loss, g.scale * tot);
    if (P.r2) {
        const float rt = block_sum(racc, s_tmp);
        if (threadIdx.x == 0 && rt != 0.f) atomicAdd(P.r2, rt);
    }
}

// gradient through the ReLU behind a residual sum: gm = g where the stored block output is positive, else 0
template <typename T>
__global__ __launch_bounds__(kElemBlock) void relu_mask_kernel(const MaskGroup g) {
    constexpr int EPV = Vec<T>::N;
    const MaskProb& P = g.p[find_problem(g, blockIdx.x)];
    const T* __restrict__ gp = reinterpret_cast<const T*>(P.g);
    const T* __restrict__ out = reinterpret_cast<const T*>(P.out);
    T* __restrict__ gm = reinterpret_cast<T*>(P.gm);
    const size_t nvec = P.numel / EPV;
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    for (int i = threadIdx.x; i < kElemVecsPerBlock; i += kElemBlock) {
        const size_t v = base + i;
        if (v >= nvec) break;
        float a[EPV], o[EPV];
        Vec<T>::load(gp + v * EPV, a);
        Vec<T>::load(out + v * EPV, o);
#pragma unroll
        for (int e = 0; e < EPV; ++e) a[e] = o[e] > 0.f ? a[e] : 0.f;
        Vec<T>::store(gm + v * EPV, a);
    }
}

template <typename T>
__global__ __launch_bounds__(kElemBlock) void mult_kernel(const MultGroup g) {
    constexpr int EPV = Vec<T>::N;
    const MultProb& P = g.p[find_problem(g, blockIdx.x)];
    T* __restrict__ lam = reinterpret_cast<T*>(P.lam);
    const T* __restrict__ y = reinterpret_cast<const T*>(P.y);
    const T* __restrict__ xn = reinterpret_cast<const T*>(P.xn);
    const size_t nvec = P.numel / EPV;
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    for (int i = threadIdx.x; i < kElemVecsPerBlock; i += kElemBlock) {
        const size_t v = base + i;
        if (v >= nvec) break;
        float a[EPV], b[EPV], l[EPV];
        Vec<T>::load(y + v * EPV, a);
        Vec<T>::load(xn + v * EPV, b);
        Vec<T>::load(lam + v * EPV, l);
#pragma unroll
        for (int e = 0; e < EPV; ++e) l[e] = fmaf(g.step, a[e] - b[e], l[e]);
        Vec<T>::store(lam + v * EPV, l);
    }
}

// parameter update, one tensor per problem (bf16 or fp32 parameter, fp32 gradient / velocity / master copy).
// Every tensor starts on a 16-byte boundary of its buffer: four elements per lane and access, scalar tail.
__device__ __forceinline__ float sgd_elem(const SgdGroup& g, float w, float grad, float* v) {
    float d = fmaf(g.wd, w, grad);
    if (v) { d = fmaf(g.momentum, *v, d); *v = d; }
    return fmaf(-g.lr, d, w);
}
__global__ __launch_bounds__(kElemBlock) void sgd_kernel(const SgdGroup g) {
    const SgdProb& P = g.p[find_problem(g, blockIdx.x)];
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kSgdElemsPerBlock;
    unsigned short* pl = reinterpret_cast<unsigned short*>(P.p);
    float* pf = reinterpret_cast<float*>(P.p);
#pragma unroll
    for (int i = 0; i < kSgdElemsPerBlock / (4 * kElemBlock); ++i) {
        const size_t e = base + 4 * ((size_t)i * kElemBlock + threadIdx.x);
        if (e + 4 <= P.numel) {
            f32x4 w;
            if (P.master) w = *reinterpret_cast<const f32x4*>(P.master + e);
            else if (P.lowp) {
                const u32x2 r = *reinterpret_cast<const u32x2*>(pl + e);
                w[0] = __uint_as_float(r[0] << 16); w[1] = __uint_as_float(r[0] & 0xffff0000u);
                w[2] = __uint_as_float(r[1] << 16); w[3] = __uint_as_float(r[1] & 0xffff0000u);
            } else w = *reinterpret_cast<const f32x4*>(pf + e);
            const f32x4 gr = *reinterpret_cast<const f32x4*>(P.g + e);
            f32x4 v;
            if (P.v) v = *reinterpret_cast<const f32x4*>(P.v + e);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float vq = P.v ? v[q] : 0.f;
                w[q] = sgd_elem(g, w[q], gr[q], P.v ? &vq : nullptr);
                v[q] = vq;
            }
            if (P.v) *reinterpret_cast<f32x4*>(P.v + e) = v;
            if (P.master) *reinterpret_cast<f32x4*>(P.master + e) = w;
            if (P.lowp) {
                u32x2 r; r[0] = pack_bf16x2(w[0], w[1]); r[1] = pack_bf16x2(w[2], w[3]);
                *reinterpret_cast<u32x2*>(pl + e) = r;
            } else *reinterpret_cast<f32x4*>(pf + e) = w;
        } else {
            for (size_t t = e; t < P.numel; ++t) {
                float w = P.master ? P.master[t] : (P.lowp ? bf16_bits_to_float(pl[t]) : pf[t]);
                w = sgd_elem(g, w, P.g[t], P.v ? P.v + t : nullptr);
                if (P.master) P.master[t] = w;
                if (P.lowp) pl[t] = float_to_bf16_bits(w);
                else pf[t] = w;
            }
        }
    }
}

// correction of the auxiliary variables: one gradient step of the relaxed objective with respect to x_k
template <typename T>
__global__ __launch_bounds__(kElemBlock) void auxvar_kernel(const AuxVarGroup g) {
    constexpr int EPV = Vec<T>::N;
    const AuxVarProb& P = g.p[find_problem(g, blockIdx.x)];
    T* __restrict__ x = reinterpret_cast<T*>(P.x);
    const T* __restrict__ yp = reinterpret_cast<const T*>(P.yprev);
    const T* __restrict__ dx = reinterpret_cast<const T*>(P.dx);
    const T* __restrict__ lam = reinterpret_cast<const T*>(P.lam);
    T* __restrict__ gout = reinterpret_cast<T*>(P.gout);
    const size_t nvec = P.numel / EPV;
    const size_t base = (size_t)(blockIdx.x - P.block_start) * kElemVecsPerBlock;
    for (int i = threadIdx.x; i < kElemVecsPerBlock; i += kElemBlock) {
        const size_t v = base + i;
        if (v >= nvec) break;
        float a[EPV], b[EPV], d[EPV], l[EPV];
        Vec<T>::load(x + v * EPV, a);
        Vec<T>::load(yp + v * EPV, b);
        Vec<T>::load(dx + v * EPV, d);
        if (lam) Vec<T>::load(lam + v * EPV, l);
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float gr = g.scale * (g.rho * (a[e] - b[e]) - (lam ? l[e] : 0.f)) + d[e];
            a[e] = gout ? gr : a[e] - g.eta * gr;
        }
        Vec<T>::store((gout ? gout : x) + v * EPV, a);
    }
}

// ------------------------------------------------------------------------------------------------
// max pooling (first maximum in row-major window order wins); one thread per pixel and 16-byte channel vector
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const PoolProb P) {
    constexpr int EPV = Vec<T>::N;
    const int cv = P.C / EPV;
    const size_t total = (size_t)P.N * P.Ho * P.Wo * cv;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const T* __restrict__ x = reinterpret_cast<const T*>(P.x);
    const int c0 = (int)(i % cv) * EPV;
    unsigned r = (unsigned)(i / cv);
    const int wo = (int)(r % (unsigned)P.Wo); r /= (unsigned)P.Wo;
    const int ho = (int)(r % (unsigned)P.Ho);
    const int n = (int)(r / (unsigned)P.Ho);
    float best[EPV];
    int bi[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) { best[e] = 0.f; bi[e] = -1; }
    for (int a = 0; a < P.R; ++a) {
        const int hi = ho * P.stride - P.pad + a;
        if (hi < 0 || hi >= P.H) continue;
        for (int b = 0; b < P.R; ++b) {
            const int wi = wo * P.stride - P.pad + b;
            if (wi < 0 || wi >= P.W) continue;
            float v[EPV];
            Vec<T>::load(x + ((size_t)(n * P.H + hi) * P.W + wi) * P.C + c0, v);
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                if (bi[e] < 0 || v[e] > best[e]) { best[e] = v[e]; bi[e] = a * P.R + b; }
        }
    }
    const size_t o = (size_t)(i / cv) * P.C + c0;
    Vec<T>::store(reinterpret_cast<T*>(P.y) + o, best);
    uint8_t arg[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) arg[e] = (uint8_t)bi[e];
    if constexpr (EPV == 8) *reinterpret_cast<uint2*>(P.arg + o) = *reinterpret_cast<const uint2*>(arg);
    else *reinterpret_cast<unsigned*>(P.arg + o) = *reinterpret_cast<const unsigned*>(arg);
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const PoolProb P) {
    constexpr int EPV = Vec<T>::N;
    const int cv = P.C / EPV;
    const size_t total = (size_t)P.N * P.H * P.W * cv;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const T* __restrict__ dy = reinterpret_cast<const T*>(P.dy);
    const int c0 = (int)(i % cv) * EPV;
    unsigned r = (unsigned)(i / cv);
    const int wi = (int)(r % (unsigned)P.W); r /= (unsigned)P.W;
    const int hi = (int)(r % (unsigned)P.H);
    const int n = (int)(r / (unsigned)P.H);
    float acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
    // windows (ho, wo) that contain (hi, wi): ho*stride - pad + a = hi
    for (int a = 0; a < P.R; ++a) {
        const int th = hi + P.pad - a;
        if (th < 0 || th % P.stride) continue;
        const int ho = th / P.stride;
        if (ho >= P.Ho) continue;
        for (int b = 0; b < P.R; ++b) {
            const int tw = wi + P.pad - b;
            if (tw < 0 || tw % P.stride) continue;
            const int wo = tw / P.stride;
            if (wo >= P.Wo) continue;
            const size_t o = ((size_t)(n * P.Ho + ho) * P.Wo + wo) * P.C + c0;
            float g[EPV];
            Vec<T>::load(dy + o, g);
            uint8_t arg[EPV];
            if constexpr (EPV == 8) *reinterpret_cast<uint2*>(arg) = *reinterpret_cast<const uint2*>(P.arg + o);
            else *reinterpret_cast<unsigned*>(arg) = *reinterpret_cast<const unsigned*>(P.arg + o);
            const uint8_t me = (uint8_t)(a * P.R + b);
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                if (arg[e] == me) acc[e] += g[e];
        }
    }
    Vec<T>::store(reinterpret_cast<T*>(P.dx) + (size_t)(i / cv) * P.C + c0, acc);
}

// ------------------------------------------------------------------------------------------------
// head: pooled[n,c] = mean_{hw} feat;  logits = pooled W^T + b
template <typename T>
__global__ void avgpool_kernel(const HeadProb P) {           // one thread per (n, 16-byte channel vector)
    constexpr int EPV = Vec<T>::N;
    const int cv = P.C / EPV;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P.N * cv) return;
    const int n = i / cv, c0 = (i % cv) * EPV;
    const T* __restrict__ f = reinterpret_cast<const T*>(P.feat) + (size_t)n * P.HW * P.C + c0;
    float s[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) s[e] = 0.f;
    int p = 0;
    for (; p + 4 <= P.HW; p += 4) {                      // four independent loads in flight
        float v[4][EPV];
#pragma unroll
        for (int u = 0; u < 4; ++u) Vec<T>::load(f + (size_t)(p + u) * P.C, v[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < EPV; ++e) s[e] += v[u][e];
    }
    for (; p < P.HW; ++p) {
        float v[EPV];
        Vec<T>::load(f + (size_t)p * P.C, v);
#pragma unroll
        for (int e = 0; e < EPV; ++e) s[e] += v[e];
    }
#pragma unroll
    for (int e = 0; e < EPV; ++e) P.pooled[n * P.C + c0 + e] = s[e] / (float)P.HW;
}
__global__ void fc_fwd_kernel(const HeadProb P) {          // one wave per (n, class)
    const int o = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (o >= P.N * P.classes) return;
    const int n = o / P.classes, j = o % P.classes, lane = threadIdx.x & 63;
    float s = 0.f;
    for (int c = lane; c < P.C; c += 64) s += P.pooled[n * P.C + c] * P.w[(size_t)j * P.C + c];
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) s += __shfl_xor(s, sh, 64);
    if (lane == 0) P.logits[o] = s + P.b[j];
}
// dW[j,c] = sum_n dz[n,j]*pooled[n,c]; db[j] = sum_n dz[n,j]: one thread per element, the samples in order (no
// partial sums to combine: pooled and dz stay in cache, the whole pass reads 2*N values per thread)
__global__ void fc_bwd_w_kernel(const HeadProb P) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P.classes * P.C) return;
    const int j = i / P.C, c = i % P.C;
    float s = 0.f, sb = 0.f;
#pragma unroll 8
    for (int n = 0; n < P.N; ++n) {
        const float d = P.dlogits[n * P.classes + j];
        s += d * P.pooled[n * P.C + c];
        sb += d;
    }
    P.dw[i] = s;
    if (c == 0) P.db[j] = sb;
}
// dfeat[n,p,c] = (sum_j dz[n,j]*W[j,c]) / HW
template <typename T>
__global__ __launch_bounds__(256) void fc_bwd_x_kernel(const HeadProb P) {
    // One block per sample and chunk of 256 channels: d pooled[c] = sum_j dlogits[j] * w[j][c] (lanes along c: coalesced
    // rows of w, summed in the order of the classes), then the block broadcasts it, divided by the number of pixels, to
    // every pixel of the sample with 16-byte stores.
    constexpr int EPV = Vec<T>::N;
    extern __shared__ float s_dp[];      // 256 floats, then the sample's `classes` logit gradients
    const int n = blockIdx.x, cbase = blockIdx.y * 256, C = P.C, classes = P.classes;
    const int nc = min(256, C - cbase);
    const float inv = 1.f / (float)P.HW;
    float* s_dl = s_dp + 256;
    for (int j = threadIdx.x; j < classes; j += 256) s_dl[j] = P.dlogits[(size_t)n * classes + j];
    __syncthreads();
    if ((int)threadIdx.x < nc) {
        const int c = cbase + threadIdx.x;
        float acc = 0.f;
        int j = 0;
        for (; j + 7 < classes; j += 8) {       // eight rows of w in flight
            float w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = P.w[(size_t)(j + u) * C + c];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += s_dl[j + u] * w[u];
        }
        for (; j < classes; ++j) acc += s_dl[j] * P.w[(size_t)j * C + c];
        s_dp[threadIdx.x] = acc * inv;
    }
    __syncthreads();
    T* __restrict__ d = reinterpret_cast<T*>(P.dfeat) + (size_t)n * P.HW * C + cbase;
    const int cvn = nc / EPV;
    for (int i = threadIdx.x; i < P.HW * cvn; i += 256) {
        const int p = i / cvn, v = i - p * cvn;
        float o[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) o[e] = s_dp[v * EPV + e];
        Vec<T>::store(d + (size_t)p * C + v * EPV, o);
    }
}

// softmax cross-entropy, mini-batch mean; one workgroup per sample
__global__ __launch_bounds__(kElemBlock) void ce_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                        float* loss, float* __restrict__ dlogits, int N, int classes) {
    __shared__ float s_tmp[kElemBlock / 64];
    __shared__ float s_max[kElemBlock / 64];
    const int n = blockIdx.x;
    const float* z = logits + (size_t)n * classes;
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < classes; j += kElemBlock) mx = fmaxf(mx, z[j]);
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) mx = fmaxf(mx, __shfl_xor(mx, sh, 64));
    if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = s_max[0];
    for (int w = 1; w < kElemBlock / 64; ++w) mx = fmaxf(mx, s_max[w]);
    float se = 0.f;
    for (int j = threadIdx.x; j < classes; j += kElemBlock) se += __expf(z[j] - mx);
    se = block_sum(se, s_tmp);
    const int lab = labels[n];
    const float inv = 1.f / se, invN = 1.f / (float)N;
    for (int j = threadIdx.x; j < classes; j += kElemBlock) {
        float p = __expf(z[j] - mx) * inv;
        if (j == lab) p -= 1.f;
        dlogits[(size_t)n * classes + j] = p * invN;
    }
    if (threadIdx.x == 0) atomicAdd(loss, (logf(se) + mx - z[lab]) * invN);
}

__global__ void zero_selected_kernel(float* v, uint32_t mask, int n) {
    const int i = threadIdx.x;
    if (i < n && ((mask >> i) & 1u)) v[i] = 0.f;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
#define LP_DISPATCH_T(dtype, KERNEL, grid, block, stream, ...)                                   \
    do {                                                                                         \
        if ((dtype) == 1) hipLaunchKernelGGL(KERNEL<bf16_t>, grid, block, 0, stream, __VA_ARGS__); \
        else hipLaunchKernelGGL(KERNEL<float>, grid, block, 0, stream, __VA_ARGS__);             \
    } while (0)

hipError_t launch_bn_apply(const BnApplyGroup& g, int dtype, bool fused_loss, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    const size_t lds = (size_t)4 * g.cmax * sizeof(float);
    const dim3 grid(g.total_blocks), block(kElemBlock);
    if (dtype == 1) {
        if (fused_loss) hipLaunchKernelGGL((bn_apply_kernel<bf16_t, true>), grid, block, lds, s, g);
        else hipLaunchKernelGGL((bn_apply_kernel<bf16_t, false>), grid, block, lds, s, g);
    } else {
        if (fused_loss) hipLaunchKernelGGL((bn_apply_kernel<float, true>), grid, block, lds, s, g);
        else hipLaunchKernelGGL((bn_apply_kernel<float, false>), grid, block, lds, s, g);
    }
    return hipGetLastError();
}
hipError_t launch_bn_bwd_reduce(const BnBwdGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    const size_t lds = (size_t)4 * g.cmax * sizeof(float);
    // narrow tensors (at most 64 channels): 256-thread workgroups -- with 512 threads half of the 256 workgroups of a
    // 32 x 32 x 16 tensor have no trip at all and the others' final sum over the row lanes is twice as long
    if (bn_reduce_threads(g.cmax) == 256) {
        if (dtype == 1) hipLaunchKernelGGL((bn_bwd_reduce_kernel<bf16_t, 256>), dim3(g.total_blocks), dim3(256), lds, s, g);
        else hipLaunchKernelGGL((bn_bwd_reduce_kernel<float, 256>), dim3(g.total_blocks), dim3(256), lds, s, g);
        return hipGetLastError();
    }
    if (dtype == 1) hipLaunchKernelGGL((bn_bwd_reduce_kernel<bf16_t, kBnReduceBlock>), dim3(g.total_blocks), dim3(kBnReduceBlock), lds, s, g);
    else hipLaunchKernelGGL((bn_bwd_reduce_kernel<float, kBnReduceBlock>), dim3(g.total_blocks), dim3(kBnReduceBlock), lds, s, g);
    return hipGetLastError();
}
hipError_t launch_bn_stats(const BnBwdGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    LP_DISPATCH_T(dtype, bn_stats_kernel, dim3(g.total_blocks), dim3(kElemBlock), s, g);
    return hipGetLastError();
}
hipError_t launch_bn_bwd_apply(const BnBwdGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    const size_t lds = (size_t)5 * g.cmax * sizeof(float);
    if (dtype == 1) hipLaunchKernelGGL(bn_bwd_apply_kernel<bf16_t>, dim3(g.total_blocks), dim3(kElemBlock), lds, s, g);
    else hipLaunchKernelGGL(bn_bwd_apply_kernel<float>, dim3(g.total_blocks), dim3(kElemBlock), lds, s, g);
    return hipGetLastError();
}
hipError_t launch_fill(const FillGroup& g, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_kernel, dim3(g.total_blocks), dim3(kElemBlock), 0, s, g);
    return hipGetLastError();
}
hipError_t launch_relu_mask(const MaskGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    LP_DISPATCH_T(dtype, relu_mask_kernel, dim3(g.total_blocks), dim3(kElemBlock), s, g);
    return hipGetLastError();
}
hipError_t launch_loss(const LossGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    LP_DISPATCH_T(dtype, loss_kernel, dim3(g.total_blocks), dim3(kElemBlock), s, g);
    return hipGetLastError();
}
hipError_t launch_sgd(const SgdGroup& g, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(sgd_kernel, dim3(g.total_blocks), dim3(kElemBlock), 0, s, g);
    return hipGetLastError();
}
hipError_t launch_auxvar(const AuxVarGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    LP_DISPATCH_T(dtype, auxvar_kernel, dim3(g.total_blocks), dim3(kElemBlock), s, g);
    return hipGetLastError();
}
hipError_t launch_mult(const MultGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    LP_DISPATCH_T(dtype, mult_kernel, dim3(g.total_blocks), dim3(kElemBlock), s, g);
    return hipGetLastError();
}
hipError_t launch_maxpool_fwd(const PoolProb& p, int dtype, hipStream_t s) {
    const size_t total = (size_t)p.N * p.Ho * p.Wo * (p.C / (dtype == 1 ? 8 : 4));
    LP_DISPATCH_T(dtype, maxpool_fwd_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), s, p);
    return hipGetLastError();
}
hipError_t launch_maxpool_bwd(const PoolProb& p, int dtype, hipStream_t s) {
    const size_t total = (size_t)p.N * p.H * p.W * (p.C / (dtype == 1 ? 8 : 4));
    LP_DISPATCH_T(dtype, maxpool_bwd_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), s, p);
    return hipGetLastError();
}
hipError_t launch_head_fwd(const HeadProb& p, int dtype, hipStream_t s) {
    const int epv = dtype == 1 ? 8 : 4;
    LP_DISPATCH_T(dtype, avgpool_kernel, dim3((p.N * (p.C / epv) + 63) / 64), dim3(64), s, p);
    hipLaunchKernelGGL(fc_fwd_kernel, dim3((p.N * p.classes + 3) / 4), dim3(256), 0, s, p);
    return hipGetLastError();
}
hipError_t launch_head_bwd(const HeadProb& p, int dtype, hipStream_t s) {
    hipLaunchKernelGGL(fc_bwd_w_kernel, dim3((p.classes * p.C + 255) / 256), dim3(256), 0, s, p);
    const size_t lds = (size_t)(256 + p.classes) * sizeof(float);
    const dim3 grid(p.N, (p.C + 255) / 256);
    if (dtype == 1) hipLaunchKernelGGL(fc_bwd_x_kernel<bf16_t>, grid, dim3(256), lds, s, p);
    else hipLaunchKernelGGL(fc_bwd_x_kernel<float>, grid, dim3(256), lds, s, p);
    return hipGetLastError();
}
hipError_t launch_zero_selected(float* v, uint32_t mask, int n, hipStream_t s) {
    hipLaunchKernelGGL(zero_selected_kernel, dim3(1), dim3(64), 0, s, v, mask, n);
    return hipGetLastError();
}
hipError_t launch_ce(const float* logits, const int32_t* labels, float* loss, float* dlogits, int N, int classes,
                     hipStream_t s) {
    hipLaunchKernelGGL(ce_kernel, dim3(N), dim3(kElemBlock), 0, s, logits, labels, loss, dlogits, N, classes);
    return hipGetLastError();
}

}  // namespace lp
