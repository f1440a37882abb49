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

// Every pointer the kernels follow points into device memory.  Where the compiler cannot see
// that (a pointer read from a table in LDS, or handed to a function that is not inlined) it
// would use the generic "flat" instructions, whose completion is counted together with LDS
// traffic: every wait for an LDS read would then also wait for every row load in flight.
// as_global() states the address space.
#define MPV_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ MPV_GLOBAL T* as_global(T* p) { return (MPV_GLOBAL T*)p; }

// 16 bytes from device memory
__device__ __forceinline__ uint4 load_global_16B(const void* p) {
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u t = *as_global(reinterpret_cast<const v4u*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// ---------------------------------------------------------------- element types

// What a node task keeps on chip is the row as stored, except for bf16 rows: those are kept as
// IEEE half precision, to which the statistics sweep converts them while it has them unpacked
// anyway.  Every bf16 logit of ordinary size is a half-precision number too (8 significant bits
// against 11; exponents from 2^-14 to 2^15, below that down to 2^-24 with the bits that are left,
// which moves an exponent argument by less than 2^-24), and the multiply-add that forms the
// exponent argument reads a half-precision operand directly (v_fma_mix_f32): the later sweeps
// save the two instructions per element pair that unpacking bf16 costs.
struct ElemF32 {
    using T = float;
    static constexpr int VEC = 4;                       // elements per 16-byte load
    static constexpr bool KEPT_AS_HALF = false;
    __device__ static __forceinline__ void unpack_kept(const uint4& r, float (&o)[VEC]) { unpack(r, o); }
    __device__ static __forceinline__ uint4 pack_kept(const float (&o)[VEC]) {
        return make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3]));
    }
    __device__ static __forceinline__ float load_one(const T* p) { return *p; }
    __device__ static __forceinline__ float load_one_global(const T* p) { return *as_global(p); }
    __device__ static __forceinline__ void unpack(const uint4& r, float (&o)[VEC]) {
        o[0] = __uint_as_float(r.x); o[1] = __uint_as_float(r.y);
        o[2] = __uint_as_float(r.z); o[3] = __uint_as_float(r.w);
    }
    __device__ static __forceinline__ void load_vec(const T* p, float (&o)[VEC]) {
        unpack(load_global_16B(p), o);
    }
};

typedef _Float16 mpv_half2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_half2(float lo, float hi) {
    // (round toward zero: the values are exact in half precision wherever that matters)
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
__device__ __forceinline__ float half_lo(unsigned w) { return static_cast<float>(__builtin_bit_cast(mpv_half2, w).x); }
__device__ __forceinline__ float half_hi(unsigned w) { return static_cast<float>(__builtin_bit_cast(mpv_half2, w).y); }

struct ElemBF16 {
    using T = uint16_t;
    static constexpr int VEC = 8;
    static constexpr bool KEPT_AS_HALF = true;
    __device__ static __forceinline__ void unpack_kept(const uint4& r, float (&o)[VEC]) {
        o[0] = half_lo(r.x); o[1] = half_hi(r.x); o[2] = half_lo(r.y); o[3] = half_hi(r.y);
        o[4] = half_lo(r.z); o[5] = half_hi(r.z); o[6] = half_lo(r.w); o[7] = half_hi(r.w);
    }
    __device__ static __forceinline__ uint4 pack_kept(const float (&o)[VEC]) {
        return make_uint4(pack_half2(o[0], o[1]), pack_half2(o[2], o[3]), pack_half2(o[4], o[5]), pack_half2(o[6], o[7]));
    }
    __device__ static __forceinline__ float load_one(const T* p) {
        return __uint_as_float(static_cast<uint32_t>(*p) << 16);
    }
    __device__ static __forceinline__ float load_one_global(const T* p) {
        return __uint_as_float(static_cast<uint32_t>(*as_global(p)) << 16);
    }
    __device__ static __forceinline__ void unpack(const uint4& r, float (&o)[VEC]) {
        o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
        o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
        o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
        o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    __device__ static __forceinline__ void load_vec(const T* p, float (&o)[VEC]) {
        unpack(load_global_16B(p), o);
    }
};

// 16 aligned bytes of a row, still packed
template <class T>
__device__ __forceinline__ uint4 load_raw(const T* p) { return load_global_16B(p); }
// vector number `vec` (16-byte units) after a wave-uniform base: 32-bit offset arithmetic
template <class T>
__device__ __forceinline__ uint4 load_raw_at(const T* base, int vec) {
    return load_global_16B(reinterpret_cast<const char*>(base) + (static_cast<unsigned>(vec) << 4));
}
// the same, marked non-temporal: data that will not be read from memory again (it is kept on
// chip) should not push re-read data out of the L2 cache
template <class T>
__device__ __forceinline__ uint4 load_raw_at_nt(const T* base, int vec) {
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u t = __builtin_nontemporal_load(
        as_global(reinterpret_cast<const v4u*>(reinterpret_cast<const char*>(base) + (static_cast<unsigned>(vec) << 4))));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// 2^x on the hardware transcendental unit (results below 2^-126 flush to zero,
// which is what every caller wants for a vanishing probability).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Tell the compiler a value is the same in every lane (it then lives in scalar
// registers instead of occupying a vector register per lane).
__device__ __forceinline__ float uniform_f32(float x) {
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
}
__device__ __forceinline__ double uniform_f64(double x) {
    const int lo = __builtin_amdgcn_readfirstlane(__double2loint(x));
    const int hi = __builtin_amdgcn_readfirstlane(__double2hiint(x));
    return __hiloint2double(hi, lo);
}

// ---------------------------------------------------------------- reductions

// Cross-lane moves inside a row of 16 lanes with DPP (data-parallel primitives: a few
// cycles each, no LDS crossbar), then the 4 row results through scalar registers.
//   0xB1 quad_perm [1,0,3,2]   0x4E quad_perm [2,3,0,1]   0x124 row_ror:4   0x128 row_ror:8
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ float lane_f32(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ double lane_f64(double v, int lane) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}

// All-lanes reductions; the result is the same in every lane (fixed order: reproducible).
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));
    v = fmaxf(v, dpp_f32<0x4E>(v));
    v = fmaxf(v, dpp_f32<0x124>(v));
    v = fmaxf(v, dpp_f32<0x128>(v));
    return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}

__device__ __forceinline__ float wave_sum_f32(float v) {
    v += dpp_f32<0xB1>(v);
    v += dpp_f32<0x4E>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x128>(v);
    return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}

__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_f64<0xB1>(v);
    v += dpp_f64<0x4E>(v);
    v += dpp_f64<0x124>(v);
    v += dpp_f64<0x128>(v);
    return (lane_f64(v, 0) + lane_f64(v, 16)) + (lane_f64(v, 32) + lane_f64(v, 48));
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

__device__ __forceinline__ int wave_inclusive_scan_i32(int v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int t = __shfl_up(v, o, kWave);
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
    if (tid < head) f.one(E::load_one_global(zt + tid), E::load_one_global(zd + tid));
    if (tail0 + tid < V) f.one(E::load_one_global(zt + tail0 + tid), E::load_one_global(zd + tail0 + tid));
    const T* bt = zt + head;
    const T* bd = zd + head;
    for (int i = tid; i < nvec; i += BLOCK * UNROLL) {
        uint4 ra[UNROLL], rd[UNROLL];             // kept packed until they are used
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = min(i + u * BLOCK, nvec - 1);       // clamped: always a valid load
            ra[u] = load_raw_at(bt, idx);
            rd[u] = load_raw_at(bd, idx);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (i + u * BLOCK < nvec) {
                float a[VEC], d[VEC];
                E::unpack(ra[u], a);
                E::unpack(rd[u], d);
                f.vec(a, d);
            }
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
    if (tid < head) f.one(E::load_one_global(z + tid));
    if (tail0 + tid < V) f.one(E::load_one_global(z + tail0 + tid));
    const T* bz = z + head;
    for (int i = tid; i < nvec; i += BLOCK * UNROLL) {
        uint4 ra[UNROLL];                         // kept packed until they are used
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) ra[u] = load_raw_at(bz, min(i + u * BLOCK, nvec - 1));   // clamped: always a valid load
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (i + u * BLOCK < nvec) {
                float a[VEC];
                E::unpack(ra[u], a);
                f.vec(a);
            }
        }
    }
}

// ---------------------------------------------------------------- softmax statistics
//
// Per-lane online accumulation of sum_v 2^(z_v*k32 - mk) against a running
// reference mk = fl(m * k32), m the running maximum.  Because mk is an exactly
// known float, lane partials combine exactly as s * 2^(mk - MK).

struct OnlineLse {
    // The reference starts at a huge negative but finite value, so that a row (or a
    // vector) of -inf logits needs no special case: fma(-inf, k, big) = -inf -> 2^-inf = 0.
    static constexpr float kFloor = -1e30f;
    float m, mk, s;
    __device__ __forceinline__ void init() { m = -INFINITY; mk = kFloor; s = 0.f; }
    // The reference follows the running maximum only in steps: it is moved when the
    // new maximum lies more than kSlack binary orders above it.  Terms then reach at most
    // 2^kSlack (their exponent argument is still exact to 2^-22), and after the first few
    // vectors of a row no lane of a wave moves its reference any more, so the whole
    // block below is skipped by a wave-level branch.
    static constexpr float kSlack = 4.f;
    __device__ __forceinline__ void raise(float lm, float k32) {
        m = fmaxf(m, lm);                    // dead code unless the caller asks for the maximum
        const float nmk = lm * k32;
        if (nmk > mk + kSlack) {
            asm volatile("" ::: "memory");   // keep this a branch: if-converted, it would run for every vector
            s *= fast_exp2(mk - nmk);        // first time: 2^-huge = 0, s stays 0
            mk = nmk;
        }
    }
    __device__ __forceinline__ void one(float z, float k32) {
        raise(z, k32);
        s += fast_exp2(fmaf(z, k32, -mk));
    }
    template <int VEC>
    __device__ __forceinline__ void vec(const float (&z)[VEC], float k32) {
        float lm = fmaxf(z[0], z[1]);
#pragma unroll
        for (int i = 2; i < VEC; ++i) lm = fmaxf(lm, z[i]);
        raise(lm, k32);
        float t0 = 0.f, t1 = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; i += 2) {
            t0 += fast_exp2(fmaf(z[i], k32, -mk));
            t1 += fast_exp2(fmaf(z[i + 1], k32, -mk));
        }
        s += t0 + t1;
    }
};

// The same sum for code that every lane of a wave runs together (the node task's sweep over the
// part it keeps on chip): the reference is one per wave.  It starts as the wave's maximum of the
// first vector it sees and is moved only when some lane meets a vector whose terms add up to
// more than 2^kSlack (found by one comparison per vector instead of a running maximum per
// element; the first vector, measured against the huge negative start value, always does).
// Exponent arguments therefore stay below kSlack and exact to 2^-21.  The fields are those of
// OnlineLse (mk the same in every lane of the wave), so lane states combine the same way.
struct WaveLse : OnlineLse {
    static constexpr float kSlack = 6.f;
    template <int COUNT>
    __device__ __forceinline__ float terms(const float (&z)[COUNT], float k32) const {
        if (COUNT == 1) return fast_exp2(fmaf(z[0], k32, -mk));
        float t0 = fast_exp2(fmaf(z[0], k32, -mk));            // (started with the first terms: no 0 + x)
        float t1 = fast_exp2(fmaf(z[COUNT > 1 ? 1 : 0], k32, -mk));
#pragma unroll
        for (int i = 2; i + 1 < COUNT; i += 2) {
            t0 += fast_exp2(fmaf(z[i], k32, -mk));
            t1 += fast_exp2(fmaf(z[i + 1], k32, -mk));
        }
        if (COUNT > 1 && (COUNT & 1)) t0 += fast_exp2(fmaf(z[COUNT - 1], k32, -mk));
        return t0 + t1;
    }
    // every lane of the wave must call this together
    template <int COUNT>
    __device__ __forceinline__ void add(const float (&z)[COUNT], float k32) {
        float v = terms(z, k32);
        if (__builtin_amdgcn_ballot_w64(!(v <= 0x1p6f)) != 0ull) {     // (also true for inf)
            float lm = z[0];
#pragma unroll
            for (int i = 1; i < COUNT; ++i) lm = fmaxf(lm, z[i]);
            const float nmk = wave_max(lm) * k32;
            if (nmk > mk) {                      // the same in every lane; -inf (nothing but masked entries) moves nothing
                s *= fast_exp2(mk - nmk);        // first time: 2^-huge = 0, s stays 0
                mk = nmk;
                v = terms(z, k32);
            }
        }
        s += v;
    }
    template <int VEC>
    __device__ __forceinline__ void vec(const float (&z)[VEC], float k32) { add(z, k32); }
    __device__ __forceinline__ void one(float z, float k32) {
        const float zz[1] = {z};
        add(zz, k32);
    }
};

// Result of the statistics of one row.
struct RowStat {
    float m;      // max_v z_v  (-inf for a row of -inf)
    double A;     // log2 sum_v 2^(z_v k32)
};

// Combine the lanes' OnlineLse states of two rows into their RowStats (the row
// maxima only if WANT_MAX; the path itself needs A alone).
template <int BLOCK, bool WANT_MAX = true>
__device__ __forceinline__ void finish_stats2(const OnlineLse& t, const OnlineLse& d,
                                              RowStat& rt, RowStat& rd, double* scratch) {
    float Mt = t.mk, Md = d.mk;
    block_max2<BLOCK>(Mt, Md, scratch);
    float mt = t.m, md = d.m;
    if (WANT_MAX) block_max2<BLOCK>(mt, md, scratch);
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
    const double ln2 = 0.6931471805599453;
    if (c < 0x1p40) {
        // c of ordinary size multiplies q as a factor: no logarithm.  (For a huge c the product
        // c q_v can be of ordinary size where q_v itself is below float range: then c goes into
        // the exponent, below.)
        const float Ad_hi = static_cast<float>(Ad);
        const double Ad_lo = Ad - static_cast<double>(Ad_hi);
        const double x = (At_lo - Ad_lo) * ln2, y = -At_lo * ln2;
        r.nAt = -At_hi;
        r.nAd = -Ad_hi;
        r.rho = static_cast<float>(c * (1.0 + x + 0.5 * x * x));
        r.scale = 1.0 + y + 0.5 * y * y;
        return r;
    }
    const double Adc = Ad - log2(c);                 // c > 0
    const float Ad_hi = static_cast<float>(Adc);
    const double Ad_lo = isfinite(Adc) ? Adc - static_cast<double>(Ad_hi) : 0.0;   // c = inf: every term vanishes
    r.nAt = -At_hi;
    r.nAd = -Ad_hi;
    // 2^x for |x| < 2^-17 (the float rounding remainders): two terms of the series are exact to 1e-16
    const double x = (At_lo - Ad_lo) * ln2, y = -At_lo * ln2;
    r.rho = static_cast<float>(1.0 + x + 0.5 * x * x);
    r.scale = 1.0 + y + 0.5 * y * y;
    return r;
}

// ---------------------------------------------------------------- a part of a row pair kept on chip
//
// A node task sweeps the same (target, draft) row pair 1 + (number of children) times.  The pair
// is split by vocabulary range among the G workgroups of a team (G chosen so that a part fits):
// each keeps its part on chip for the whole task, R 16-byte vectors per lane and row in
// registers and up to L more in LDS, loaded once, and every sweep runs over those.  If a part is
// larger than that (vocabularies beyond G_max parts), the rest is read again in every sweep.
//
// Vector i of the part (i counted from the part's first vector) belongs to lane i % BLOCK,
// slot i / BLOCK: slots [0,R) live in registers, [R,R+L) in LDS (lds[slot-R][lane]), the rest is
// streamed.  Lanes past the end of the part hold -inf logits (probability zero in every sweep).

// 16 bytes per lane from global memory straight into LDS (no register in between):
// the wave's 64 lanes fill 1 KB starting at the wave-uniform address `lds_wave_base`.
__device__ __forceinline__ void load_to_lds_16B(const void* gptr, uint4* lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                     (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

template <class E> struct NegInfVec;
template <> struct NegInfVec<ElemF32> { static __device__ __forceinline__ uint4 v() { return make_uint4(0xff800000u, 0xff800000u, 0xff800000u, 0xff800000u); } };
template <> struct NegInfVec<ElemBF16> { static __device__ __forceinline__ uint4 v() { return make_uint4(0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u); } };

template <class E, int BLOCK, int R, int L>
struct RetainedPart {
    using T = typename E::T;
    static constexpr int VEC = E::VEC;
    uint4 rt[R], rd[R];
    const T* zt;                // the rows themselves (element 0)
    const T* zd;
    const T* bt;                // first 16-byte aligned vector of the rows
    const T* bd;
    uint4* lt;                  // LDS, [L][BLOCK] each
    uint4* ld;
    int V, head, nvec, tail0;   // row geometry: `head` elements, nvec vectors, then elements from tail0
    int v0, nv, nslots;         // this part: vectors [v0, v0 + nv) of the row, ceil(nv / BLOCK) slots
    int tid;
    bool first_part, last_part; // who looks after the elements before / after the aligned vectors

    // per: vectors per part (a multiple of 64: the bonus sampler's wave tiles never straddle parts)
    __device__ __forceinline__ void setup(const T* zt_, const T* zd_, int V_, uint4* lds_t, uint4* lds_d, int tid_,
                                          int member, int team_size, int per) {
        zt = zt_; zd = zd_; V = V_; lt = lds_t; ld = lds_d; tid = tid_;
        const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(zt) & 15u) / sizeof(T));
        head = mis ? min(VEC - mis, V) : 0;
        nvec = (V - head) / VEC;
        tail0 = head + nvec * VEC;
        bt = zt + head;
        bd = zd + head;
        v0 = min(member * per, nvec);
        nv = min(per, nvec - v0);
        nslots = (nv + BLOCK - 1) / BLOCK;
        first_part = member == 0;
        last_part = member == team_size - 1;
    }

    // the elements before and after the aligned vectors: every lane calls the functor, with
    // -inf logits (probability zero in every sweep) where it has no such element
    template <class F>
    __device__ __forceinline__ void edges(F& f) const {
        if (first_part && head > 0) {                       // (the same in every lane)
            float a = -INFINITY, b = -INFINITY;
            if (tid < head) { a = E::load_one_global(zt + tid); b = E::load_one_global(zd + tid); }
            f.one(a, b);
        }
        if (last_part && tail0 < V) {
            float a = -INFINITY, b = -INFINITY;
            if (tail0 + tid < V) { a = E::load_one_global(zt + tail0 + tid); b = E::load_one_global(zd + tail0 + tid); }
            f.one(a, b);
        }
    }

    // slot s of this lane: its vector number in the row (clamped into the part: always a valid
    // address when the part is not empty) and whether it lies inside the part
    __device__ __forceinline__ int vec_of(int s) const { return v0 + min(s * BLOCK + tid, nv - 1); }
    __device__ __forceinline__ bool inside(int s) const { return s * BLOCK + tid < nv; }
    // every lane of the workgroup owns a vector in slot s (the same in every lane: a branch, so
    // that full slots do not pay for the padding of the last one)
    __device__ __forceinline__ bool full_slot(int s) const { return (s + 1) * BLOCK <= nv; }

    // Put every load of the kept slots in flight (registers first: they are consumed first).
    // An empty part (nv = 0) loads nothing.
    __device__ __forceinline__ void issue_loads() {
        if (nv <= 0) return;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            rt[j] = load_raw_at_nt(bt, vec_of(j));
            rd[j] = load_raw_at_nt(bd, vec_of(j));
        }
        const int wave0 = (tid / kWave) * kWave;
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (R + j < nslots) {
                load_to_lds_16B(bt + static_cast<size_t>(vec_of(R + j)) * VEC, lt + j * BLOCK + wave0);
                load_to_lds_16B(bd + static_cast<size_t>(vec_of(R + j)) * VEC, ld + j * BLOCK + wave0);
            }
        }
    }

    // slots beyond what is kept: read from memory, CH loads in flight
    template <class F>
    __device__ __forceinline__ void streamed(F& f) const {
        constexpr int CH = 2;
        for (int s = R + L + 1; s < nslots; s += CH) {
            uint4 a[CH], d[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                a[u] = load_raw_at(bt, vec_of(s + u));
                d[u] = load_raw_at(bd, vec_of(s + u));
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (s + u >= nslots) break;               // (the same in every lane)
                if (!inside(s + u)) { a[u] = NegInfVec<E>::v(); d[u] = NegInfVec<E>::v(); }
                f.vec(a[u], d[u]);                        // every lane, together
            }
        }
    }

    // First sweep: consumes the loads of issue_loads() in the order they were issued, pads the
    // lanes past the end of the part with -inf (kept that way for the later sweeps).
    // One slot beyond the kept ones (a part slightly too large) is asked for when a sweep starts
    // and used when it ends: its memory latency hides behind the kept slots.  More than that is
    // streamed two slots at a time (streamed()).
    __device__ __forceinline__ bool has_overflow() const { return nslots > R + L; }      // (the same in every lane)
    __device__ __forceinline__ void ask_overflow(uint4& a, uint4& d) const {
        a = load_raw_at(bt, vec_of(R + L));
        d = load_raw_at(bd, vec_of(R + L));
    }
    template <class F>
    __device__ __forceinline__ void use_overflow(F& f, uint4 a, uint4 d) const {
        if (!inside(R + L)) { a = NegInfVec<E>::v(); d = NegInfVec<E>::v(); }
        f.vec(a, d);
    }

    template <class F>
    __device__ __forceinline__ void first_pass(F& f) {
        edges(f);
        if (nv <= 0) return;
        uint4 oa, od;
        const bool overflow = has_overflow();
        if (overflow) ask_overflow(oa, od);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (j < nslots) {
                if (!full_slot(j)) {
                    if (!inside(j)) { rt[j] = NegInfVec<E>::v(); rd[j] = NegInfVec<E>::v(); }
                }
                if (E::KEPT_AS_HALF) {              // swept as stored, then kept in the form the later sweeps read
                    float a[VEC], d[VEC];
                    E::unpack(rt[j], a);
                    E::unpack(rd[j], d);
                    f.vecf(a, d);
                    rt[j] = E::pack_kept(a);
                    rd[j] = E::pack_kept(d);
                } else {
                    f.vec(rt[j], rd[j]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (R + j < nslots) {
                uint4 a = lt[j * BLOCK + tid], d = ld[j * BLOCK + tid];
                bool padded = false;
                if (!full_slot(R + j)) {
                    if (!inside(R + j)) { a = NegInfVec<E>::v(); d = NegInfVec<E>::v(); padded = true; }
                }
                if (E::KEPT_AS_HALF) {
                    float fa[VEC], fd[VEC];
                    E::unpack(a, fa);
                    E::unpack(d, fd);
                    f.vecf(fa, fd);
                    lt[j * BLOCK + tid] = E::pack_kept(fa);                  // the lane's own entry
                    ld[j * BLOCK + tid] = E::pack_kept(fd);
                } else {
                    if (padded) { lt[j * BLOCK + tid] = a; ld[j * BLOCK + tid] = d; }
                    f.vec(a, d);
                }
            }
        }
        if (overflow) use_overflow(f, oa, od);
        streamed(f);
    }

    // Later sweeps.  The empty asm marks each kept register as "possibly changed", so that the
    // compiler does not hoist the unpacked form of the whole part out of the caller's loop over
    // children (which would double the register footprint).
    template <class F>
    __device__ __forceinline__ void replay(F& f) {
        edges(f);
        if (nv <= 0) return;
        uint4 oa, od;
        const bool overflow = has_overflow();
        if (overflow) ask_overflow(oa, od);
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (R + j < nslots) f.vec_kept(lt[j * BLOCK + tid], ld[j * BLOCK + tid]);
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (j < nslots) {
                asm volatile("" : "+v"(rt[j].x), "+v"(rt[j].y), "+v"(rt[j].z), "+v"(rt[j].w));
                asm volatile("" : "+v"(rd[j].x), "+v"(rd[j].y), "+v"(rd[j].z), "+v"(rd[j].w));
                f.vec_kept(rt[j], rd[j]);
            }
        }
        if (overflow) use_overflow(f, oa, od);
        streamed(f);
    }
};

template <class E>
struct PairStatsRawF {
    WaveLse t, d;               // (every lane of a wave calls one() and vec() together)
    float k32;
    __device__ __forceinline__ void one(float a, float b) { t.one(a, k32); d.one(b, k32); }
    __device__ __forceinline__ void vecf(const float (&a)[E::VEC], const float (&b)[E::VEC]) {
        t.vec(a, k32);
        d.vec(b, k32);
    }
    __device__ __forceinline__ void vec(const uint4& ra, const uint4& rb) {
        float a[E::VEC], b[E::VEC];
        E::unpack(ra, a);
        E::unpack(rb, b);
        vecf(a, b);
    }
};

// W(c) = sum_v (p_v - c q_v)_+ together with  sum_{p_v > c q_v} c q_v  (so that dW/dc = -that / c):
// value and slope from one sweep, for SpecTr's root search.
template <class E>
struct ResidualMassSlopeRawF {
    float k32, nAt, nAd, rho;
    float acc0, acc1, q0, q1;
    __device__ __forceinline__ void init() { acc0 = 0.f; acc1 = 0.f; q0 = 0.f; q1 = 0.f; }
    __device__ __forceinline__ void term(float a, float b, float& acc, float& q) const {
        const float et = fast_exp2(fmaf(a, k32, nAt));
        const float ed = rho * fast_exp2(fmaf(b, k32, nAd));
        const float diff = et - ed;
        acc += fmaxf(diff, 0.f);
        q += diff > 0.f ? ed : 0.f;
    }
    __device__ __forceinline__ void one(float a, float b) { term(a, b, acc0, q0); }
    __device__ __forceinline__ void vecf(const float (&a)[E::VEC], const float (&b)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) {
            term(a[i], b[i], acc0, q0);
            term(a[i + 1], b[i + 1], acc1, q1);
        }
    }
    __device__ __forceinline__ void vec(const uint4& ra, const uint4& rb) {          // a vector as stored
        float a[E::VEC], b[E::VEC];
        E::unpack(ra, a);
        E::unpack(rb, b);
        vecf(a, b);
    }
    __device__ __forceinline__ void vec_kept(const uint4& ra, const uint4& rb) {     // a vector as kept on chip
        float a[E::VEC], b[E::VEC];
        E::unpack_kept(ra, a);
        E::unpack_kept(rb, b);
        vecf(a, b);
    }
};

// ---------------------------------------------------------------- acceptance rates (App. C)
//
// 1 - (1 - q)^m, the chance that one of m tokens drawn from q is a given token of probability q.
// Small q: three terms of the binomial series (1 - q itself would round q away); else directly.
__device__ __forceinline__ float hit_probability(float q, float m, float c2, float c3) {
    const float series = q * (m - q * (c2 - q * c3));
    const float direct = 1.f - fast_exp2(m * __builtin_amdgcn_logf(fmaxf(1.f - q, 0.f)));     // q = 1: 2^-inf = 0
    return q < 0x1p-12f ? series : direct;
}

// NSS:   sum_t p (1 - (1-q)^m)                                  (m = k)
// Naive: sum_t min(p,q) + sum_t (p-q)_+ (1 - (1-q)^m)           (m = k - 1)
// p = 2^(zt k32 + nAt) sp and q = 2^(zd k32 + nAd) sq are the normalised probabilities themselves.
template <class E>
struct AcceptanceF {
    float k32, nAt, nAd, sp, sq, m, c2, c3;
    bool naive;
    float acc0, acc1;
    __device__ __forceinline__ void init(float k, float nat, float nad, float sp_, float sq_, int m_, bool naive_) {
        k32 = k; nAt = nat; nAd = nad; sp = sp_; sq = sq_; naive = naive_;
        m = static_cast<float>(m_);
        c2 = 0.5f * m * (m - 1.f);
        c3 = c2 * (m - 2.f) * (1.f / 3.f);
        acc0 = 0.f; acc1 = 0.f;
    }
    __device__ __forceinline__ float term(float a, float b) const {
        const float p = fast_exp2(fmaf(a, k32, nAt)) * sp;
        const float q = fast_exp2(fmaf(b, k32, nAd)) * sq;
        const float hit = (m > 0.f) ? hit_probability(q, m, c2, c3) : 0.f;
        return naive ? fminf(p, q) + fmaxf(p - q, 0.f) * hit : p * hit;
    }
    __device__ __forceinline__ void one(float a, float b) { acc0 += term(a, b); }
    __device__ __forceinline__ void vec(const float (&a)[E::VEC], const float (&b)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) {
            acc0 += term(a[i], b[i]);
            acc1 += term(a[i + 1], b[i + 1]);
        }
    }
    __device__ __forceinline__ void vec(const uint4& ra, const uint4& rb) {
        float a[E::VEC], b[E::VEC];
        E::unpack(ra, a);
        E::unpack(rb, b);
        vec(a, b);
    }
    __device__ __forceinline__ void vec_kept(const uint4& ra, const uint4& rb) {     // a vector as kept on chip
        float a[E::VEC], b[E::VEC];
        E::unpack_kept(ra, a);
        E::unpack_kept(rb, b);
        vec(a, b);
    }
};

// The node task's form of it.  Both exponents are lowered by one, so that every term is below
// 1 and "(x)_+" can be the clamp to [0, 1] that the multiply-add applies to its own result (one
// instruction less per element); total() undoes the halving.
template <class E>
struct ResidualMassRawF {
    float k32, nAt, nAd, rho;
    float acc0, acc1;
    __device__ __forceinline__ void init(float k, float nat, float nad, float r) {
        k32 = k; nAt = nat - 1.f; nAd = nad - 1.f; rho = r; acc0 = 0.f; acc1 = 0.f;
    }
    __device__ __forceinline__ float term(float a, float b) const {
        const float et = fast_exp2(fmaf(a, k32, nAt));
        const float ed = fast_exp2(fmaf(b, k32, nAd));
        return __builtin_amdgcn_fmed3f(fmaf(-rho, ed, et), 0.f, 1.f);
    }
    __device__ __forceinline__ void one(float a, float b) { acc0 += term(a, b); }
    __device__ __forceinline__ void vecf(const float (&a)[E::VEC], const float (&b)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) {
            acc0 += term(a[i], b[i]);
            acc1 += term(a[i + 1], b[i + 1]);
        }
    }
    __device__ __forceinline__ void vec(const uint4& ra, const uint4& rb) {          // a vector as stored
        float a[E::VEC], b[E::VEC];
        E::unpack(ra, a);
        E::unpack(rb, b);
        vecf(a, b);
    }
    __device__ __forceinline__ void vec_kept(const uint4& ra, const uint4& rb) {     // a vector as kept on chip
        float a[E::VEC], b[E::VEC];
        E::unpack_kept(ra, a);
        E::unpack_kept(rb, b);
        vecf(a, b);
    }
    __device__ __forceinline__ double total() const { return 2.0 * (static_cast<double>(acc0) + static_cast<double>(acc1)); }
};

}  // namespace mpv
