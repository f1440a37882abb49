// Nucleus (top-p) transform of logit rows: device code (included by mpv.hip).
//
// Sec. 4.1 names the setting (nucleus sampling with top-p 0.9 and 0.99); the definition taken
// is the usual one.  With p = softmax(z / T): keep the smallest set {v : z_v >= tau}, tau one
// of the row's values, whose mass reaches top_p; every other token gets the logit -inf, so that
// whatever reads the row afterwards sees the renormalised truncated distribution.  Tokens with
// equal logits are kept or dropped together.
//
// One workgroup per row:
//   1. the row's maximum m (the one read from memory that computes next to nothing);
//   2. tau by bisection over the order-preserving integer keys of float values.  One probe per
//      step: the mass of {z >= cut} together with the nearest row values on either side of the
//      cut, to which the bracket then snaps, so a step never lands between two row values
//      twice (at most 33 steps for float rows, 18 for bfloat16 rows).  A first sweep adds up the
//      whole row (masses are 2^((z - m) log2(e)/T): the largest is 1) and copies the tokens whose
//      probability is within 2^-12 of the largest into LDS; if they reach top_p and fit, the
//      probes run over that copy, else over the row itself (which stays in the caches);
//   3. the row is written out, masked.
// The masses are float sums in a fixed order (bitwise reproducible); "reaches top_p" is decided
// against the sum of the whole row computed the same way, by the same sweep.

#pragma once

#include "mpv_device.h"

namespace mpv {

constexpr int kNucleusBlock = 512;
constexpr int kNucleusUnroll = 4;     // 16-byte loads in flight per lane

// ascending unsigned key of a float (no NaN): negative values reversed, sign bit flipped
__device__ __forceinline__ uint32_t float_key(float f) {
    const uint32_t b = __float_as_uint(f + 0.0f);            // -0 -> +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

template <class E>
struct NucleusProbeF {
    float k32, nA;          // p_v = 2^(z_v k32 + nA), up to a factor common to the row
    float cut;
    float acc0, acc1;       // mass of {z >= cut}
    float below, above;     // largest z < cut, smallest z >= cut
    int count;              // |{z >= cut}|
    __device__ __forceinline__ void init(float k, float na, float c) {
        k32 = k; nA = na; cut = c; acc0 = 0.f; acc1 = 0.f; below = -INFINITY; above = INFINITY; count = 0;
    }
    __device__ __forceinline__ void item(float z, float& acc) {
        const float e = fast_exp2(fmaf(z, k32, nA));
        const bool in = z >= cut;
        acc += in ? e : 0.f;
        below = in ? below : fmaxf(below, z);
        above = in ? fminf(above, z) : above;
        count += in ? 1 : 0;
    }
    __device__ __forceinline__ void one(float z) { item(z, acc0); }
    __device__ __forceinline__ void vec(const float (&z)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) { item(z[i], acc0); item(z[i + 1], acc1); }
    }
};

struct NucleusProbeResult { double mass; float below, above; int count; double whole; };

// One value per workgroup of each of the numbers of a probe (`whole`: a second sum that goes along,
// scratch has room for both); the same values in every lane.
__device__ __forceinline__ NucleusProbeResult nucleus_reduce(double mass, float below, float above, int count,
                                                             double* scratch, float* fscratch, int* iscratch,
                                                             double whole = 0.0) {
    constexpr int NW = kNucleusBlock / kWave;
    const int w = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    const double m = wave_sum(mass);
    const double wh = wave_sum(whole);
    const float lo = wave_max(below);
    const float hi = -wave_max(-above);
    const int c = wave_inclusive_scan_i32(count);            // lane 63 holds the wave's total
    __syncthreads();                                          // the previous probe's results have been read
    if (lane == kWave - 1) { scratch[w] = m; scratch[NW + w] = wh; fscratch[2 * w] = lo; fscratch[2 * w + 1] = hi; iscratch[w] = c; }
    __syncthreads();
    NucleusProbeResult r;
    r.mass = scratch[0]; r.whole = scratch[NW]; r.below = fscratch[0]; r.above = fscratch[1]; r.count = iscratch[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
        r.mass += scratch[i];
        r.whole += scratch[NW + i];
        r.below = fmaxf(r.below, fscratch[2 * i]);
        r.above = fminf(r.above, fscratch[2 * i + 1]);
        r.count += iscratch[i];
    }
    return r;
}

// the largest value of a row
template <class E>
struct RowMaxF {
    float m0, m1;
    __device__ __forceinline__ void init() { m0 = -INFINITY; m1 = -INFINITY; }
    __device__ __forceinline__ void one(float z) { m0 = fmaxf(m0, z); }
    __device__ __forceinline__ void vec(const float (&z)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) { m0 = fmaxf(m0, z[i]); m1 = fmaxf(m1, z[i + 1]); }
    }
};

// Probe over the whole row in memory.
template <class E>
__device__ __forceinline__ NucleusProbeResult nucleus_probe(const typename E::T* z, int V, float k32, float nA, float cut,
                                                            double* scratch, float* fscratch, int* iscratch) {
    NucleusProbeF<E> f;
    f.init(k32, nA, cut);
    sweep_row<E, kNucleusBlock, kNucleusUnroll>(z, V, f);
    return nucleus_reduce(static_cast<double>(f.acc0) + static_cast<double>(f.acc1), f.below, f.above, f.count,
                          scratch, fscratch, iscratch);
}

// The tokens that can matter are usually few: those whose probability is within 2^-kNucleusSpan of
// the largest.  One sweep copies them (value and mass) into LDS; if they hold enough mass and fit,
// tau is found among them without touching the row again.
constexpr int kNucleusCap = 8192;
constexpr float kNucleusSpan = 12.f;
// candidate masses are added as integers (units of 2^-40, exact in a double): the order in which
// the waves append their candidates does not change any sum
constexpr double kNucleusUnit = 1099511627776.0;

template <class E>
struct NucleusCollectF {
    float k32, nA, cut;
    float* cand_z;
    float* cand_e;
    int* cand_n;
    float acc0, acc1, below, above;
    float all0, all1;       // the mass of the whole row
    int count;
    __device__ __forceinline__ void init(float k, float na, float c, float* cz, float* ce, int* cn) {
        k32 = k; nA = na; cut = c; cand_z = cz; cand_e = ce; cand_n = cn;
        acc0 = 0.f; acc1 = 0.f; all0 = 0.f; all1 = 0.f; below = -INFINITY; above = INFINITY; count = 0;
    }
    __device__ __forceinline__ void item(float z, float& acc, float& all) {
        const float e = fast_exp2(fmaf(z, k32, nA));
        const bool in = z >= cut;
        all += e;
        acc += in ? e : 0.f;
        below = in ? below : fmaxf(below, z);
        above = in ? fminf(above, z) : above;
        count += in ? 1 : 0;
        const unsigned long long m = __ballot(in);            // lanes of this wave that are here and have one
        if (m) {
            const int lane = threadIdx.x & (kWave - 1);
            const int leader = __ffsll(static_cast<long long>(m)) - 1;
            int base = 0;
            if (lane == leader) base = atomicAdd(cand_n, __popcll(m));
            base = __shfl(base, leader, kWave);
            const int idx = base + __popcll(m & ((1ull << lane) - 1ull));
            if (in && idx < kNucleusCap) { cand_z[idx] = z; cand_e[idx] = e; }
        }
    }
    __device__ __forceinline__ void one(float z) { item(z, acc0, all0); }
    __device__ __forceinline__ void vec(const float (&z)[E::VEC]) {
#pragma unroll
        for (int i = 0; i < E::VEC; i += 2) { item(z[i], acc0, all0); item(z[i + 1], acc1, all1); }
    }
};

// Probe over the n candidates in LDS; masses in units of 2^-40.
__device__ __forceinline__ NucleusProbeResult nucleus_probe_candidates(const float* cand_z, const float* cand_e, int n, float cut,
                                                                       double* scratch, float* fscratch, int* iscratch) {
    double mass = 0.0;
    float below = -INFINITY, above = INFINITY;
    int count = 0;
    for (int i = threadIdx.x; i < n; i += kNucleusBlock) {
        const float z = cand_z[i];
        const bool in = z >= cut;
        mass += in ? floor(static_cast<double>(cand_e[i]) * kNucleusUnit) : 0.0;
        below = in ? below : fmaxf(below, z);
        above = in ? fminf(above, z) : above;
        count += in ? 1 : 0;
    }
    return nucleus_reduce(mass, below, above, count, scratch, fscratch, iscratch);
}

template <class E> struct MaskedStore;
template <> struct MaskedStore<ElemF32> {
    __device__ static __forceinline__ float one(float z, float tau) { return z >= tau ? z : -INFINITY; }
    __device__ static __forceinline__ uint4 vec(const uint4& r, float tau) {
        uint4 o;
        o.x = __float_as_uint(one(__uint_as_float(r.x), tau)); o.y = __float_as_uint(one(__uint_as_float(r.y), tau));
        o.z = __float_as_uint(one(__uint_as_float(r.z), tau)); o.w = __float_as_uint(one(__uint_as_float(r.w), tau));
        return o;
    }
    __device__ static __forceinline__ float to_elem(float v) { return v; }
};
template <> struct MaskedStore<ElemBF16> {
    static constexpr uint32_t kNegInf = 0xff80u;
    __device__ static __forceinline__ uint32_t word(uint32_t w, float tau) {
        const uint32_t lo = (__uint_as_float(w << 16) >= tau) ? (w & 0xffffu) : kNegInf;
        const uint32_t hi = (__uint_as_float(w & 0xffff0000u) >= tau) ? (w & 0xffff0000u) : (kNegInf << 16);
        return hi | lo;
    }
    __device__ static __forceinline__ uint4 vec(const uint4& r, float tau) {
        uint4 o;
        o.x = word(r.x, tau); o.y = word(r.y, tau); o.z = word(r.z, tau); o.w = word(r.w, tau);
        return o;
    }
    __device__ static __forceinline__ uint16_t to_elem(float v) { return static_cast<uint16_t>(__float_as_uint(v) >> 16); }
};

// top_p in (0, 1): see the file header; keep_all: top_p = 1, nothing is dropped (tau = the row's
// minimum).  threshold_out / kept_out may be null.
template <class E>
__global__ __launch_bounds__(kNucleusBlock) void nucleus_kernel(const typename E::T* in, typename E::T* out, int64_t rows,
                                                                int V, float k32, float top_p, int keep_all,
                                                                float* threshold_out, int32_t* kept_out) {
    using T = typename E::T;
    constexpr int NW = kNucleusBlock / kWave;
    __shared__ double scratch[2 * NW];
    __shared__ float fscratch[2 * NW];
    __shared__ int iscratch[NW];
    __shared__ float cand_z[kNucleusCap], cand_e[kNucleusCap];
    __shared__ int cand_n;
    const int64_t r = blockIdx.x;
    const T* z = in + r * V;
    T* o = out + r * V;

    float tau = -INFINITY;                                    // so far: everything is kept
    int kept = V;
    // 1. the maximum (the same value in every lane)
    float row_max = -INFINITY;
    if (!keep_all) {
        RowMaxF<E> mf;
        mf.init();
        sweep_row<E, kNucleusBlock, kNucleusUnroll>(z, V, mf);
        const NucleusProbeResult top = nucleus_reduce(0.0, fmaxf(mf.m0, mf.m1), INFINITY, 0, scratch, fscratch, iscratch);
        row_max = top.below;
    }
    // 2. tau.  The masses a probe adds up are 2^(z k32 + nA) = 2^((z - m) k32); over the whole row
    //    they add up to S.  (A row of -inf only has nothing to drop.)
    if (!keep_all && row_max > -INFINITY) {
        const float nA = -row_max * k32;
        if (threadIdx.x == 0) cand_n = 0;
        __syncthreads();
        const float cut0 = row_max - kNucleusSpan / k32;
        NucleusCollectF<E> cf;
        cf.init(k32, nA, cut0, cand_z, cand_e, &cand_n);
        sweep_row<E, kNucleusBlock, kNucleusUnroll>(z, V, cf);
        const NucleusProbeResult first = nucleus_reduce(static_cast<double>(cf.acc0) + static_cast<double>(cf.acc1),
                                                        cf.below, cf.above, cf.count, scratch, fscratch, iscratch,
                                                        static_cast<double>(cf.all0) + static_cast<double>(cf.all1));
        const double want = static_cast<double>(top_p) * first.whole;
        uint32_t lo_key, hi_key = float_key(row_max) + 1u;    // cuts from hi_key on leave nothing above them
        bool in_lds = false;
        if (first.mass >= want) {                             // tau >= cut0
            tau = first.above;                                // the upper set of cut0, named by its smallest value
            kept = first.count;
            lo_key = float_key(tau);
            in_lds = first.count <= kNucleusCap;
        } else {                                              // tau < cut0: the candidates are not enough
            lo_key = float_key(-INFINITY);
            hi_key = float_key(first.below) + 1u;
        }
        if (in_lds) {
            const int n = first.count;
            const double want_units = want * kNucleusUnit;
            // everything at or above cut0 is in LDS; is it still enough counted in units?
            const NucleusProbeResult c0 = nucleus_probe_candidates(cand_z, cand_e, n, cut0, scratch, fscratch, iscratch);
            if (c0.mass >= want_units) {
                for (int step = 0; step < 40 && hi_key - lo_key > 1u; ++step) {
                    const float cut = key_float(lo_key + (hi_key - lo_key) / 2u);      // tau < cut <= maximum
                    const NucleusProbeResult p = nucleus_probe_candidates(cand_z, cand_e, n, cut, scratch, fscratch, iscratch);
                    if (p.mass >= want_units) {
                        tau = p.above;                        // the same upper set, named by its smallest value
                        kept = p.count;
                        lo_key = float_key(tau);
                    } else {
                        hi_key = float_key(p.below) + 1u;     // every cut above `below` has this upper set or less
                    }
                }
                hi_key = lo_key;                              // done
            } else {                                          // within rounding of top_p at cut0: decide in memory
                tau = -INFINITY;
                kept = V;
                lo_key = float_key(-INFINITY);
                hi_key = float_key(row_max) + 1u;
            }
        }
        for (int step = 0; step < 40 && hi_key - lo_key > 1u; ++step) {
            const float cut = key_float(lo_key + (hi_key - lo_key) / 2u);
            const NucleusProbeResult p = nucleus_probe<E>(z, V, k32, nA, cut, scratch, fscratch, iscratch);
            if (p.mass >= want) {
                tau = p.above;
                kept = p.count;
                lo_key = float_key(tau);
            } else {
                hi_key = float_key(p.below) + 1u;
            }
        }
    }

    // 3. masked copy (in place if out == in: every element is read and written by the same lane)
    const int tid = threadIdx.x;
    const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(z) & 15u) / sizeof(T));
    const int head = mis ? min(E::VEC - mis, V) : 0;
    const int nvec = (V - head) / E::VEC;
    const int tail0 = head + nvec * E::VEC;
    if (tid < head) o[tid] = MaskedStore<E>::to_elem(MaskedStore<ElemF32>::one(E::load_one(z + tid), tau));
    if (tail0 + tid < V) o[tail0 + tid] = MaskedStore<E>::to_elem(MaskedStore<ElemF32>::one(E::load_one(z + tail0 + tid), tau));
    const uint4* zv = reinterpret_cast<const uint4*>(z + head);
    uint4* ov = reinterpret_cast<uint4*>(o + head);
    int i = tid;
    for (; i + 3 * kNucleusBlock < nvec; i += 4 * kNucleusBlock) {       // four loads in flight per lane
        const uint4 a0 = zv[i], a1 = zv[i + kNucleusBlock], a2 = zv[i + 2 * kNucleusBlock], a3 = zv[i + 3 * kNucleusBlock];
        ov[i] = MaskedStore<E>::vec(a0, tau);
        ov[i + kNucleusBlock] = MaskedStore<E>::vec(a1, tau);
        ov[i + 2 * kNucleusBlock] = MaskedStore<E>::vec(a2, tau);
        ov[i + 3 * kNucleusBlock] = MaskedStore<E>::vec(a3, tau);
    }
    for (; i < nvec; i += kNucleusBlock) ov[i] = MaskedStore<E>::vec(zv[i], tau);
    if (tid == 0) {
        if (threshold_out) threshold_out[r] = tau;
        if (kept_out) kept_out[r] = kept;
    }
}

}  // namespace mpv
