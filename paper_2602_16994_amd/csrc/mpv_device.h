// Device-side building blocks for the verification kernels (gfx950, wave64).
//
// Arithmetic convention used by every kernel in this library
// ---------------------------------------------------------
// k32  = float(log2(e) / T)                       one rounded constant per call
// A    = log2( sum_v 2^(z_v * k32) )              the row's log-partition (base 2), kept in double
// p_v  = 2^(z_v * k32 - A)                        softmax(z / T)   (Sec. 3: next-token distribution)
// Every V-wide term is evaluated as v_exp_f32( fma(z, k32, -A_hi) ) with A split
// into a float A_hi and a tiny double remainder that is applied to the reduced
// scalar, so the rounding of A never scales a whole row.  Sums are accumulated in
// several independent float partials per lane and reduced across lanes and waves
// in double, in a fixed order (bitwise reproducible).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpv {

constexpr int kWave = 64;

// ---------------------------------------------------------------- element types

struct ElemF32 {
    using T = float;
    static constexpr int VEC = 4;                       // elements per 16-byte load
    __device__ static __forceinline__ float load_one(const T* p) { return *p; }
    __device__ static __forceinline__ void unpack(const uint4& r, float (&o)[VEC]) {
        o[0] = __uint_as_float(r.x); o[1] = __uint_as_float(r.y);
        o[2] = __uint_as_float(r.z); o[3] = __uint_as_float(r.w);
    }
    __device__ static __forceinline__ void load_vec(const T* p, float (&o)[VEC]) {
        unpack(*reinterpret_cast<const uint4*>(p), o);
    }
};

struct ElemBF16 {
    using T = uint16_t;
    static constexpr int VEC = 8;
    __device__ static __forceinline__ float load_one(const T* p) {
        return __uint_as_float(static_cast<uint32_t>(*p) << 16);
    }
    __device__ static __forceinline__ void unpack(const uint4& r, float (&o)[VEC]) {
        o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
        o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
        o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
        o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    __device__ static __forceinline__ void load_vec(const T* p, float (&o)[VEC]) {
        unpack(*reinterpret_cast<const uint4*>(p), o);
    }
};

// 16 aligned bytes of a row, still packed
template <class T>
__device__ __forceinline__ uint4 load_raw(const T* p) { return *reinterpret_cast<const uint4*>(p); }

// 2^x on the hardware transcendental unit (results below 2^-126 flush to zero,
// which is what every caller wants for a vanishing probability).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------- reductions

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Inclusive prefix sum across the 64 lanes of a wave.
__device__ __forceinline__ double wave_inclusive_scan(double v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const double t = __shfl_up(v, o, kWave);
        if (lane >= o) v += t;
    }
    return v;
}

// Block-wide reductions of two values at once; every thread gets the result.
// `scratch` must hold 2 * (BLOCK / 64) doubles and may be reused after return.
template <int BLOCK>
__device__ __forceinline__ void block_max2(float& a, float& b, double* scratch) {
    constexpr int NW = BLOCK / kWave;
    float* s = reinterpret_cast<float*>(scratch);
    a = wave_max(a);
    b = wave_max(b);
    const int w = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    __syncthreads();
    if (lane == 0) { s[2 * w] = a; s[2 * w + 1] = b; }
    __syncthreads();
    float ra = s[0], rb = s[1];
#pragma unroll
    for (int i = 1; i < NW; ++i) { ra = fmaxf(ra, s[2 * i]); rb = fmaxf(rb, s[2 * i + 1]); }
    a = ra; b = rb;
}

template <int BLOCK>
__device__ __forceinline__ void block_sum2(double& a, double& b, double* scratch) {
    constexpr int NW = BLOCK / kWave;
    a = wave_sum(a);
    b = wave_sum(b);
    const int w = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    __syncthreads();
    if (lane == 0) { scratch[2 * w] = a; scratch[2 * w + 1] = b; }
    __syncthreads();
    double ra = scratch[0], rb = scratch[1];
#pragma unroll
    for (int i = 1; i < NW; ++i) { ra += scratch[2 * i]; rb += scratch[2 * i + 1]; }
    a = ra; b = rb;
}

template <int BLOCK>
__device__ __forceinline__ double block_sum(double a, double* scratch) {
    double b = 0.0;
    block_sum2<BLOCK>(a, b, scratch);
    return a;
}

// ---------------------------------------------------------------- row sweeps
//
// A sweep visits every element of one row, or of a (target, draft) row pair, once.
// Rows start at element-aligned addresses; the two rows of a pair have the same
// offset modulo 16 bytes (both base pointers are 16-byte aligned and the rows
// have the same index).  Elements before the first and after the last aligned
// 16-byte vector are handled one by one, the rest with 16-byte loads, UNROLL of
// them in flight per lane.

template <class E, int BLOCK, int UNROLL, class F>
__device__ __forceinline__ void sweep_pair(const typename E::T* __restrict__ zt,
                                           const typename E::T* __restrict__ zd,
                                           int V, F& f) {
    using T = typename E::T;
    constexpr int VEC = E::VEC;
    const int tid = threadIdx.x;
    const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(zt) & 15u) / sizeof(T));
    const int head = mis ? min(VEC - mis, V) : 0;
    const int nvec = (V - head) / VEC;
    const int tail0 = head + nvec * VEC;
    if (tid < head) f.one(E::load_one(zt + tid), E::load_one(zd + tid));
    if (tail0 + tid < V) f.one(E::load_one(zt + tail0 + tid), E::load_one(zd + tail0 + tid));
    const T* bt = zt + head;
    const T* bd = zd + head;
    for (int i = tid; i < nvec; i += BLOCK * UNROLL) {
        float a[UNROLL][VEC], d[UNROLL][VEC];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = i + u * BLOCK;
            if (idx < nvec) {
                E::load_vec(bt + static_cast<size_t>(idx) * VEC, a[u]);
                E::load_vec(bd + static_cast<size_t>(idx) * VEC, d[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = i + u * BLOCK;
            if (idx < nvec) f.vec(a[u], d[u]);
        }
    }
}

template <class E, int BLOCK, int UNROLL, class F>
__device__ __forceinline__ void sweep_row(const typename E::T* __restrict__ z, int V, F& f) {
    using T = typename E::T;
    constexpr int VEC = E::VEC;
    const int tid = threadIdx.x;
    const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(z) & 15u) / sizeof(T));
    const int head = mis ? min(VEC - mis, V) : 0;
    const int nvec = (V - head) / VEC;
    const int tail0 = head + nvec * VEC;
    if (tid < head) f.one(E::load_one(z + tid));
    if (tail0 + tid < V) f.one(E::load_one(z + tail0 + tid));
    const T* bz = z + head;
    for (int i = tid; i < nvec; i += BLOCK * UNROLL) {
        float a[UNROLL][VEC];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = i + u * BLOCK;
            if (idx < nvec) E::load_vec(bz + static_cast<size_t>(idx) * VEC, a[u]);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = i + u * BLOCK;
            if (idx < nvec) f.vec(a[u]);
        }
    }
}

// ---------------------------------------------------------------- softmax statistics
//
// Per-lane online accumulation of sum_v 2^(z_v*k32 - mk) against a running
// reference mk = fl(m * k32), m the running maximum.  Because mk is an exactly
// known float, lane partials combine exactly as s * 2^(mk - MK).

struct OnlineLse {
    float m, mk, s;
    __device__ __forceinline__ void init() { m = -INFINITY; mk = -INFINITY; s = 0.f; }
    __device__ __forceinline__ void raise(float lm, float k32) {
        if (lm > m) {
            const float nmk = lm * k32;
            s *= fast_exp2(mk - nmk);        // first time: 2^-inf = 0, s stays 0
            m = lm;
            mk = nmk;
        }
    }
    __device__ __forceinline__ void one(float z, float k32) {
        raise(z, k32);
        if (z > -INFINITY) s += fast_exp2(fmaf(z, k32, -mk));
    }
    template <int VEC>
    __device__ __forceinline__ void vec(const float (&z)[VEC], float k32) {
        float lm = z[0];
#pragma unroll
        for (int i = 1; i < VEC; ++i) lm = fmaxf(lm, z[i]);
        raise(lm, k32);
        if (m > -INFINITY) {
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) t += fast_exp2(fmaf(z[i], k32, -mk));
            s += t;
        }
    }
};

// Result of the statistics of one row.
struct RowStat {
    float m;      // max_v z_v  (-inf for a row of -inf)
    double A;     // log2 sum_v 2^(z_v k32)
};

// Combine the lanes' OnlineLse states of two rows into their RowStats.
template <int BLOCK>
__device__ __forceinline__ void finish_stats2(const OnlineLse& t, const OnlineLse& d,
                                              RowStat& rt, RowStat& rd, double* scratch) {
    float Mt = t.mk, Md = d.mk;
    block_max2<BLOCK>(Mt, Md, scratch);
    float mt = t.m, md = d.m;
    block_max2<BLOCK>(mt, md, scratch);
    double st = (t.s > 0.f) ? static_cast<double>(t.s * fast_exp2(t.mk - Mt)) : 0.0;
    double sd = (d.s > 0.f) ? static_cast<double>(d.s * fast_exp2(d.mk - Md)) : 0.0;
    block_sum2<BLOCK>(st, sd, scratch);
    rt.m = mt; rt.A = static_cast<double>(Mt) + log2(st);
    rd.m = md; rd.A = static_cast<double>(Md) + log2(sd);
}

template <class E, int BLOCK, int UNROLL>
struct PairStatsF {
    OnlineLse t, d;
    float k32;
    __device__ __forceinline__ void one(float a, float b) { t.one(a, k32); d.one(b, k32); }
    __device__ __forceinline__ void vec(const float (&a)[E::VEC], const float (&b)[E::VEC]) {
        t.vec(a, k32);
        d.vec(b, k32);
    }
};

template <class E>
struct RowStatsF {
    OnlineLse t;
    float k32;
    __device__ __forceinline__ void one(float a) { t.one(a, k32); }
    __device__ __forceinline__ void vec(const float (&a)[E::VEC]) { t.vec(a, k32); }
};

// ---------------------------------------------------------------- residual mass
//
// W(c) = sum_v (p_v - c q_v)_+   (the normaliser of App. B Alg. 4's p <- norm (p-q)_+
// after any number of rounds, and of the Traversal update (a P - q)_+).
// Lanes accumulate  sum (e_t - rho e_d)_+  with e_t = 2^(zt k32 - At_hi),
// e_d = 2^(zd k32 - Ad_hi); the caller multiplies by 2^-At_lo.

template <class E>
struct ResidualMassF {
    float k32, nAt, nAd, rho;       // nAt = -At_hi, nAd = -(Ad - log2 c)_hi
    float acc0, acc1;
    __device__ __forceinline__ void init() { acc0 = 0.f; acc1 = 0.f; }
    __device__ __forceinline__ float term(float a, float b) const {
        const float et = fast_exp2(fmaf(a, k32, nAt));
        const float ed = fast_exp2(fmaf(b, k32, nAd));
        return fmaxf(fmaf(-rho, ed, et), 0.f);
    }
    __device__ __forceinline__ void one(float a, float b) { acc0 += term(a, b); }
    __device__ __forceinline__ void vec(const float (&a)[E::VEC], const float (&b)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) {
            acc0 += term(a[i], b[i]);
            acc1 += term(a[i + 1], b[i + 1]);
        }
    }
};

// Scalars that turn (row statistics, c) into the constants of ResidualMassF.
struct ResidualConsts {
    float nAt, nAd, rho;
    double scale;                   // 2^-At_lo : W = scale * sum
};

__device__ __forceinline__ ResidualConsts residual_consts(double At, double Ad, double c) {
    ResidualConsts r;
    const float At_hi = static_cast<float>(At);
    const double At_lo = At - static_cast<double>(At_hi);
    const double Adc = Ad - log2(c);                 // c > 0
    const float Ad_hi = static_cast<float>(Adc);
    const double Ad_lo = isfinite(Adc) ? Adc - static_cast<double>(Ad_hi) : 0.0;   // c = inf: every term vanishes
    r.nAt = -At_hi;
    r.nAd = -Ad_hi;
    r.rho = static_cast<float>(exp2(At_lo - Ad_lo));
    r.scale = exp2(-At_lo);
    return r;
}

// ---------------------------------------------------------------- a row pair kept on chip
//
// A node task sweeps the same (target, draft) row pair 1 + (number of children)
// times.  The first sweep keeps as much of the pair as the compute unit can hold:
// R 16-byte vectors per lane and row in registers, L more in LDS; later sweeps
// replay those and re-read only the rest ("streamed" part) from memory.  The
// streamed part is the last thing the first sweep loads and the first thing a
// replay reads, so that it is still in the L2 cache.
//
// Vector i of a row belongs to lane i % BLOCK, slot i / BLOCK: slots [0,R) live in
// registers, [R,R+L) in LDS (lds[slot-R][lane]), the rest is streamed.

template <class E, int BLOCK, int R, int L, int CH, bool FULL>
struct RetainedPair {
    // FULL: the caller guarantees nvec >= (R + L) * BLOCK, so every register and
    // LDS slot of every lane is in range and those parts run without a branch.
    using T = typename E::T;
    static constexpr int VEC = E::VEC;
    uint4 rt[R > 0 ? R : 1], rd[R > 0 ? R : 1];
    const T* zt;
    const T* zd;
    const T* bt;
    const T* bd;
    uint4* lt;
    uint4* ld;
    int V, head, nvec, tail0;

    __device__ __forceinline__ void setup(const T* zt_, const T* zd_, int V_, uint4* lds_t, uint4* lds_d) {
        zt = zt_; zd = zd_; V = V_; lt = lds_t; ld = lds_d;
        const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(zt) & 15u) / sizeof(T));
        head = mis ? min(VEC - mis, V) : 0;
        nvec = (V - head) / VEC;
        tail0 = head + nvec * VEC;
        bt = zt + head;
        bd = zd + head;
    }

    __device__ __forceinline__ bool in_range(int idx) const { return FULL || idx < nvec; }

    template <class F>
    __device__ __forceinline__ void edges(F& f) const {
        const int tid = threadIdx.x;
        if (tid < head) f.one(E::load_one(zt + tid), E::load_one(zd + tid));
        if (tail0 + tid < V) f.one(E::load_one(zt + tail0 + tid), E::load_one(zd + tail0 + tid));
    }

    template <class F>
    __device__ __forceinline__ void streamed(F& f) const {
        const int tid = threadIdx.x;
        for (int i = tid + (R + L) * BLOCK; i < nvec; i += BLOCK * CH) {
            uint4 a[CH], d[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int idx = min(i + u * BLOCK, nvec - 1);      // clamped: always a valid load
                a[u] = load_raw(bt + static_cast<size_t>(idx) * VEC);
                d[u] = load_raw(bd + static_cast<size_t>(idx) * VEC);
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (i + u * BLOCK < nvec) f.vec(a[u], d[u]);
            }
        }
    }

    // First sweep: load everything once, keep what fits, feed f.
    template <class F>
    __device__ __forceinline__ void first_pass(F& f) {
        const int tid = threadIdx.x;
        if (!FULL && nvec == 0) { edges(f); return; }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int idx = FULL ? tid + j * BLOCK : min(tid + j * BLOCK, nvec - 1);
            rt[j] = load_raw(bt + static_cast<size_t>(idx) * VEC);
            rd[j] = load_raw(bd + static_cast<size_t>(idx) * VEC);
        }
        edges(f);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (in_range(tid + j * BLOCK)) f.vec(rt[j], rd[j]);
        }
#pragma unroll
        for (int j0 = 0; j0 < L; j0 += CH) {
            uint4 a[CH], d[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (j0 + u < L) {
                    const int idx = FULL ? tid + (R + j0 + u) * BLOCK : min(tid + (R + j0 + u) * BLOCK, nvec - 1);
                    a[u] = load_raw(bt + static_cast<size_t>(idx) * VEC);
                    d[u] = load_raw(bd + static_cast<size_t>(idx) * VEC);
                }
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (j0 + u < L) {
                    lt[(j0 + u) * BLOCK + tid] = a[u];
                    ld[(j0 + u) * BLOCK + tid] = d[u];
                    if (in_range(tid + (R + j0 + u) * BLOCK)) f.vec(a[u], d[u]);
                }
            }
        }
        streamed(f);
    }

    // Later sweeps: streamed part (from L2 / memory), then LDS, then registers.
    // The empty asm marks each kept register as "possibly changed", so that the
    // compiler does not hoist the unpacked form of the whole pair out of the
    // caller's loop over children (which would double the register footprint).
    template <class F>
    __device__ __forceinline__ void replay(F& f) {
        const int tid = threadIdx.x;
        if (!FULL && nvec == 0) { edges(f); return; }
        streamed(f);
        edges(f);
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (in_range(tid + (R + j) * BLOCK)) f.vec(lt[j * BLOCK + tid], ld[j * BLOCK + tid]);
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            asm volatile("" : "+v"(rt[j].x), "+v"(rt[j].y), "+v"(rt[j].z), "+v"(rt[j].w));
            asm volatile("" : "+v"(rd[j].x), "+v"(rd[j].y), "+v"(rd[j].z), "+v"(rd[j].w));
            if (in_range(tid + j * BLOCK)) f.vec(rt[j], rd[j]);
        }
    }
};

template <class E>
struct PairStatsRawF {
    OnlineLse t, d;
    float k32;
    __device__ __forceinline__ void one(float a, float b) { t.one(a, k32); d.one(b, k32); }
    __device__ __forceinline__ void vec(const uint4& ra, const uint4& rb) {
        float a[E::VEC], b[E::VEC];
        E::unpack(ra, a);
        E::unpack(rb, b);
        t.vec(a, k32);
        d.vec(b, k32);
    }
};

template <class E>
struct ResidualMassRawF : ResidualMassF<E> {
    __device__ __forceinline__ void vec(const uint4& ra, const uint4& rb) {
        float a[E::VEC], b[E::VEC];
        E::unpack(ra, a);
        E::unpack(rb, b);
        ResidualMassF<E>::vec(a, b);
    }
    using ResidualMassF<E>::one;
};

}  // namespace mpv
