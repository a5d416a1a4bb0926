// Device code of libcgbn for gfx950 (wave64): the sweeps over the activation
// tensors and the small cross-shard reductions.  No MFMA anywhere: every kernel
// here is a streaming reduction or a streaming elementwise map, bound by HBM.
//
// Sweeps (one launch each):
//   reduce  OP_SUM    sum x                       Algorithm 1 steps 1-3
//   reduce  OP_SQDEV  sum (x - mean)^2            Algorithm 1 steps 6-8
//   reduce  OP_BWD    sum dy, sum dy*xhat         backward device sums
//   map     EL_NORM   y  = gamma*(x-mean)*invstd + beta            step 11
//   map     EL_DX     dx = gamma*invstd*(dy - dbeta/M - xhat*dgamma/M)
//   reduce  OP_BWD_RELU       sum dz, sum dz*xhat with dz = dy where y > 0 (y: the stored output), else 0
//   map     EL_NORM_RELU      y  = max(0, step 11)
//   map     EL_NORM_ADD_RELU  y  = max(0, step 11 + shortcut)
//   map     EL_DX_RELU        dx from dz; optionally writes dz, the shortcut's gradient
//   map     EL_FROZEN         y  = gamma*(x-m)/sqrt(s2+eps) + beta with fixed statistics m, s2 (sections 3.1, 3.3)
//   map     EL_SCALE          dx = dy*gamma/sqrt(s2+eps), the backward of the fixed-statistics layer
//   reduce  OP_MOMENTS        per row, sum (x - p) about the channel's pivot p and M2, the squared deviations from the
//                             row's OWN mean: steps 1-3 and the raw material of steps 6-8 in one sweep over x
// A reduce sweep leaves one float per (channel, row) in `part`, where the rows
// of a channel are ordered shard by shard; combine_rows then adds the rows of a
// shard (the device sum of Algorithm 1) and the shards (its reduce step) in
// double precision in a fixed order.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cgbn {

constexpr int kThreads = 256;   // 4 wavefronts per workgroup
constexpr int kWave = 64;

enum { OP_SUM = 0, OP_SQDEV = 1, OP_BWD = 2, OP_BWD_RELU = 3, OP_MOMENTS = 4 };
enum { EL_NORM = 0, EL_DX = 1, EL_FROZEN = 2, EL_SCALE = 3, EL_NORM_RELU = 4, EL_NORM_ADD_RELU = 5, EL_DX_RELU = 6 };
// which tensors a sweep reads besides x: `dy` (the second input: dy, or the shortcut) and
// `aux` (the third: the stored output y, whose sign is the ReLU's mask)
constexpr bool op_has_dy(int op) { return op == OP_BWD || op == OP_BWD_RELU; }
constexpr bool op_has_y(int op) { return op == OP_BWD_RELU; }
constexpr int op_sums(int op) { return (op_has_dy(op) || op == OP_MOMENTS) ? 2 : 1; }   // row partials per workgroup
constexpr bool el_has_2(int el) { return el == EL_DX || el == EL_NORM_ADD_RELU || el == EL_DX_RELU; }
constexpr bool el_has_3(int el) { return el == EL_DX_RELU; }
constexpr bool el_is_norm(int el) { return el == EL_NORM || el == EL_NORM_RELU || el == EL_NORM_ADD_RELU; }
enum { CM_MEAN = 0, CM_INVSTD = 1, CM_BWD = 2, CM_SHARDS1 = 3, CM_SHARDS2 = 4, CM_MOMENTS = 5 };

struct bf16_t { uint16_t bits; };

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct SweepArgs {
    const void* x;
    const void* dy;
    const void* aux;          // stored output y (ReLU variants of the backward)
    void* out;
    void* out2;               // dz, the shortcut's gradient (EL_DX_RELU; may be null)
    const float* mean;
    const float* mean_lo;     // may be null
    const float* invstd;
    const float* gamma;
    const float* beta;
    const float* dgamma;
    const float* dbeta;
    float* part0;             // row partials: NCHW [C][rows], NHWC [rows][C] (a workgroup's channels side by side)
    float* part1;
    long long S;              // elements in the tensor
    int N, C, HW, rows;
    // NCHW
    int L, sp;                // chunk elements, chunks per plane
    int tg;                   // tiny planes: planes per workgroup (a power of two, 8 ... 256)
    // NHWC
    int cv, TW, ctiles, rpp, PL, pps;
    long long spix;           // pixels per shard
    long long pivot_stride;   // elements between the first values of consecutive channels
    float inv_M;
    float eps;                // fixed-statistics maps: `invstd` then points at variances
    int reverse;              // walk the grid backwards
    int nt;                   // non-temporal stores
};

// --------------------------------------------------------------------------
// element access
// --------------------------------------------------------------------------

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Two floats to two bfloat16 in one register (the first in the low half): gfx950's own
// conversion instruction, round to nearest even, NaN stays a quiet NaN.
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    f32x2_hw v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw));
}
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return f32x2_to_bf16x2(f, 0.f) & 0xffffu; }

template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ float load1(const float* p) { return *p; }
    static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
    static __device__ __forceinline__ void loadv(const float* p, float (&f)[4])
    {
        f32x4 v = *reinterpret_cast<const f32x4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    typedef f32x4 Raw;       // 16 bytes as they are stored
    static __device__ __forceinline__ Raw load_raw(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
    static __device__ __forceinline__ void storev(float* p, const float (&f)[4], int nt)
    {
        f32x4 v = {f[0], f[1], f[2], f[3]};
        if (nt) __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
        else *reinterpret_cast<f32x4*>(p) = v;
    }
};

template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float load1(const bf16_t* p) { return bf16_to_f32(p->bits); }
    static __device__ __forceinline__ void store1(bf16_t* p, float v) { p->bits = (uint16_t)f32_to_bf16(v); }
    static __device__ __forceinline__ void loadv(const bf16_t* p, float (&f)[8])
    {
        u32x4 v = *reinterpret_cast<const u32x4*>(p);
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    typedef u32x4 Raw;
    static __device__ __forceinline__ Raw load_raw(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
    static __device__ __forceinline__ void storev(bf16_t* p, const float (&f)[8], int nt)
    {
        u32x4 v;
        v.x = f32x2_to_bf16x2(f[0], f[1]);
        v.y = f32x2_to_bf16x2(f[2], f[3]);
        v.z = f32x2_to_bf16x2(f[4], f[5]);
        v.w = f32x2_to_bf16x2(f[6], f[7]);
        if (nt) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
        else *reinterpret_cast<u32x4*>(p) = v;
    }
};

// VEC-wide access for the channels-last kernels (V == Elem<T>::VEC or 1)
template <typename T, int V> struct Access {
    static __device__ __forceinline__ void load(const T* p, float (&f)[V]) { Elem<T>::loadv(p, f); }
    static __device__ __forceinline__ void store(T* p, const float (&f)[V], int nt) { Elem<T>::storev(p, f, nt); }
};
template <typename T> struct Access<T, 1> {
    static __device__ __forceinline__ void load(const T* p, float (&f)[1]) { f[0] = Elem<T>::load1(p); }
    static __device__ __forceinline__ void store(T* p, const float (&f)[1], int) { Elem<T>::store1(p, f[0]); }
};

// --------------------------------------------------------------------------
// wavefront and workgroup sums (fixed order, so results are reproducible)
// --------------------------------------------------------------------------

template <int CTRL> __device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Sum over the 64 lanes of a wavefront; every lane must be active.  Four DPP
// steps fold each row of 16 lanes (swap neighbours, swap pairs, mirror the
// half-row, mirror the row), then the four row totals are read out.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror
    float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

template <int V> __device__ __forceinline__ float fold(const float (&a)[V])
{
    if constexpr (V == 8) return ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
    else if constexpr (V == 4) return (a[0] + a[1]) + (a[2] + a[3]);
    else return a[0];
}

// --------------------------------------------------------------------------
// one-sweep statistics: running summaries (count, sum, M2)
// --------------------------------------------------------------------------

// A summary of a set of values taken about the channel's pivot: how many, their sum, and M2, the sum of their
// squared deviations from the set's OWN mean.  Values arrive in small chunks whose sum and M2 are formed exactly
// as written (sum, mean, deviations from that mean: everything is in registers); a chunk is merged into the
// running summary by the pairwise update
//     M2 <- M2 + M2_chunk + (mean_chunk - mean)^2 * n * c / (n + c)
// so nothing is ever formed as a difference of large sums, wherever the pivot lies.
struct Run {
    float n, S, M2;
};
// merge of two summaries (a to the left of b: the order is part of the result's bits)
__device__ __forceinline__ Run run_join(const Run& a, const Run& b)
{
    const float n = a.n + b.n;
    const float ma = a.n > 0.f ? a.S * __builtin_amdgcn_rcpf(a.n) : 0.f;
    const float mb = b.n > 0.f ? b.S * __builtin_amdgcn_rcpf(b.n) : 0.f;
    const float w = n > 0.f ? a.n * b.n * __builtin_amdgcn_rcpf(n) : 0.f;
    const float d = mb - ma;
    Run r;
    r.n = n;
    r.S = a.S + b.S;
    r.M2 = (a.M2 + b.M2) + (d * d) * w;
    return r;
}
// a chunk of C values v[] (already taken about the pivot) joins the summary
template <int C> __device__ __forceinline__ void run_feed(Run& r, const float (&v)[C])
{
    float cs = 0.f;
#pragma unroll
    for (int i = 0; i < C; ++i) cs += v[i];
    const float cm = cs * (1.0f / (float)C);
    float cq = 0.f;
#pragma unroll
    for (int i = 0; i < C; ++i) {
        const float d = v[i] - cm;
        cq += d * d;
    }
    Run c = {(float)C, cs, cq};
    r = run_join(r, c);
}
// all 64 lanes' summaries joined in a fixed tree (the lower lane always on the left); every lane gets the result
__device__ __forceinline__ Run run_wave_join(Run mine, int lane)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        Run other;
        other.n = __shfl_xor(mine.n, off);
        other.S = __shfl_xor(mine.S, off);
        other.M2 = __shfl_xor(mine.M2, off);
        mine = (lane & off) ? run_join(other, mine) : run_join(mine, other);
    }
    return mine;
}

// --------------------------------------------------------------------------
// walking one contiguous run of elements with 16-byte vector accesses
// --------------------------------------------------------------------------

// Thread `t` of `STRIDE` cooperating threads visits its share of the elements
// [seg0, seg0 + len): up to VEC-1 leading and trailing elements one by one (so
// that the body starts on a 16-byte boundary of a 16-byte aligned tensor) and
// the body as whole vectors, four at a time while that many remain.
template <int STRIDE, int VEC, class F>
__device__ __forceinline__ void walk_segment(long long seg0, int len, int t, long long S, F& f)
{
    if (seg0 < 0 || len <= 0 || seg0 + len > S) return;   // never touch memory outside the tensor
    int mis = (int)(seg0 & (long long)(VEC - 1));
    int head = mis ? min(VEC - mis, len) : 0;
    int body = len - head;
    int nvec = body / VEC;
    int tail = body - nvec * VEC;
    long long v0 = seg0 + head;
    if (t < head) f.one(seg0 + t);
    int i = t;
    for (; i + 3 * STRIDE < nvec; i += 4 * STRIDE)
        f.four(v0 + (long long)i * VEC, (long long)STRIDE * VEC);
    for (; i < nvec; i += STRIDE) f.vec(v0 + (long long)i * VEC);
    if (t < tail) f.one(v0 + (long long)nvec * VEC + t);
}

// per-channel constants of a sweep
struct ChanConst {
    float mu, mulo, istd, g, b, c2;
};

// The plain sum is taken about a pivot, the channel's first stored value, and the
// pivot is added back in double precision by the combine step: the float
// accumulators then hold numbers of the size of the channel's spread, not of its
// offset, so the pooled mean keeps its accuracy when |mean| >> sigma.
template <typename T, int OP> __device__ __forceinline__ ChanConst reduce_consts(const SweepArgs& A, int c)
{
    ChanConst k = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (OP == OP_SUM || OP == OP_MOMENTS) {
        k.mu = Elem<T>::load1(static_cast<const T*>(A.x) + (long long)c * A.pivot_stride);
    } else {
        k.mu = A.mean[c];
        k.mulo = A.mean_lo ? A.mean_lo[c] : 0.f;
    }
    if (op_has_dy(OP)) k.istd = A.invstd[c];
    return k;
}

template <int EL> __device__ __forceinline__ ChanConst map_consts(const SweepArgs& A, int c)
{
    ChanConst k;
    if (EL == EL_FROZEN || EL == EL_SCALE) {
        // fixed statistics: `invstd` points at the variances; the root and the division are
        // correctly rounded float operations, once per thread and channel
        k.istd = 1.0f / sqrtf(A.invstd[c] + A.eps);
        k.g = A.gamma[c] * k.istd;
        k.mu = EL == EL_FROZEN ? A.mean[c] : 0.f;
        k.b = EL == EL_FROZEN ? A.beta[c] : 0.f;
        k.mulo = 0.f;
        k.c2 = 0.f;
        return k;
    }
    k.mu = A.mean[c];
    k.mulo = A.mean_lo ? A.mean_lo[c] : 0.f;
    k.istd = A.invstd[c];
    k.g = A.gamma[c] * k.istd;
    if (el_is_norm(EL)) {
        k.b = A.beta[c];
        k.c2 = 0.f;
    } else {
        k.b = A.dbeta[c] * A.inv_M;
        k.c2 = A.dgamma[c] * A.inv_M;
    }
    return k;
}

template <int OP> __device__ __forceinline__ void accumulate(const ChanConst& k, float xv, float dyv, float yv, float& a0, float& a1)
{
    if (op_has_y(OP)) dyv = yv > 0.f ? dyv : 0.f;
    if (OP == OP_SUM) {
        a0 += xv - k.mu;
    } else if (OP == OP_SQDEV) {
        float d = (xv - k.mu) - k.mulo;
        a0 += d * d;
    } else {
        float xh = ((xv - k.mu) - k.mulo) * k.istd;
        a0 += dyv;
        a1 += dyv * xh;
    }
}

// `v2`: dy or the shortcut; `v3`: the stored output; `dz`: the masked dy (EL_DX_RELU)
template <int EL> __device__ __forceinline__ float map_value(const ChanConst& k, float xv, float v2, float v3, float& dz)
{
    if (EL == EL_SCALE) return xv * k.g;
    if (EL == EL_FROZEN) return (xv - k.mu) * k.g + k.b;
    float d = (xv - k.mu) - k.mulo;
    if (EL == EL_NORM) return d * k.g + k.b;
    if (EL == EL_NORM_RELU || EL == EL_NORM_ADD_RELU) {
        float z = d * k.g + k.b;
        if (EL == EL_NORM_ADD_RELU) z += v2;
        return z < 0.f ? 0.f : z;                  // NaN stays NaN
    }
    float dyv = v2;
    if (EL == EL_DX_RELU) {
        dyv = v3 > 0.f ? v2 : 0.f;
        dz = dyv;
    }
    return k.g * ((dyv - k.b) - (d * k.istd) * k.c2);
}

// --------------------------------------------------------------------------
// NCHW: a plane of H*W contiguous elements belongs to one channel
// --------------------------------------------------------------------------

template <typename T, int OP> struct PlaneReduce {
    static constexpr int VEC = Elem<T>::VEC;
    static constexpr bool DY = op_has_dy(OP), Y = op_has_y(OP);
    const T* x;
    const T* dy;
    const T* aux;
    ChanConst k;
    float a0[VEC], a1[VEC];
    Run run;                       // OP_MOMENTS: this lane's summary

    __device__ __forceinline__ void one(long long off)
    {
        if constexpr (OP == OP_MOMENTS) {
            float v[1] = {Elem<T>::load1(x + off) - k.mu};
            run_feed<1>(run, v);
            return;
        }
        float xv = Elem<T>::load1(x + off);
        float dv = DY ? Elem<T>::load1(dy + off) : 0.f;
        float yv = Y ? Elem<T>::load1(aux + off) : 0.f;
        accumulate<OP>(k, xv, dv, yv, a0[0], a1[0]);
    }
    __device__ __forceinline__ void vec(long long off)
    {
        float xv[VEC], dv[VEC], yv[VEC];
        Elem<T>::loadv(x + off, xv);
        if constexpr (OP == OP_MOMENTS) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) xv[e] -= k.mu;
            run_feed<VEC>(run, xv);
            return;
        }
        if (DY) Elem<T>::loadv(dy + off, dv);
        if (Y) Elem<T>::loadv(aux + off, yv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) accumulate<OP>(k, xv[e], DY ? dv[e] : 0.f, Y ? yv[e] : 0.f, a0[e], a1[e]);
    }
    __device__ __forceinline__ void four(long long off, long long step)
    {
        float xv[4][VEC], dv[4][VEC], yv[4][VEC];
#pragma unroll
        for (int u = 0; u < 4; ++u) Elem<T>::loadv(x + off + u * step, xv[u]);
        if constexpr (OP == OP_MOMENTS) {
            float v[4 * VEC];              // one chunk: all of them are values of this plane
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[u * VEC + e] = xv[u][e] - k.mu;
            run_feed<4 * VEC>(run, v);
            return;
        }
        if (DY) {
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<T>::loadv(dy + off + u * step, dv[u]);
        }
        if (Y) {
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<T>::loadv(aux + off + u * step, yv[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                accumulate<OP>(k, xv[u][e], DY ? dv[u][e] : 0.f, Y ? yv[u][e] : 0.f, a0[e], a1[e]);
    }
};

template <typename T, int EL> struct PlaneMap {
    static constexpr int VEC = Elem<T>::VEC;
    static constexpr bool IN2 = el_has_2(EL), IN3 = el_has_3(EL);
    const T* x;
    const T* dy;
    const T* aux;
    T* out;
    T* out2;       // may be null
    ChanConst k;
    int nt;

    __device__ __forceinline__ void one(long long off)
    {
        float xv = Elem<T>::load1(x + off);
        float v2 = IN2 ? Elem<T>::load1(dy + off) : 0.f;
        float v3 = IN3 ? Elem<T>::load1(aux + off) : 0.f;
        float dz = 0.f;
        Elem<T>::store1(out + off, map_value<EL>(k, xv, v2, v3, dz));
        if (IN3 && out2) Elem<T>::store1(out2 + off, dz);
    }
    __device__ __forceinline__ void vec(long long off)
    {
        float xv[VEC], v2[VEC], v3[VEC], r[VEC], dz[VEC];
        Elem<T>::loadv(x + off, xv);
        if (IN2) Elem<T>::loadv(dy + off, v2);
        if (IN3) Elem<T>::loadv(aux + off, v3);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            dz[e] = 0.f;
            r[e] = map_value<EL>(k, xv[e], IN2 ? v2[e] : 0.f, IN3 ? v3[e] : 0.f, dz[e]);
        }
        Elem<T>::storev(out + off, r, nt);
        if (IN3 && out2) Elem<T>::storev(out2 + off, dz, nt);
    }
    __device__ __forceinline__ void four(long long off, long long step)
    {
        float xv[4][VEC], v2[4][VEC], v3[4][VEC];
#pragma unroll
        for (int u = 0; u < 4; ++u) Elem<T>::loadv(x + off + u * step, xv[u]);
        if (IN2) {
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<T>::loadv(dy + off + u * step, v2[u]);
        }
        if (IN3) {
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<T>::loadv(aux + off + u * step, v3[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float r[VEC], dz[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                dz[e] = 0.f;
                r[e] = map_value<EL>(k, xv[u][e], IN2 ? v2[u][e] : 0.f, IN3 ? v3[u][e] : 0.f, dz[e]);
            }
            Elem<T>::storev(out + off + u * step, r, nt);
            if (IN3 && out2) Elem<T>::storev(out2 + off + u * step, dz, nt);
        }
    }
};

// One workgroup per (plane, chunk): grid = N*C*sp.
template <typename T, int OP>
__global__ __launch_bounds__(kThreads) void nchw_reduce_block(SweepArgs A)
{
    constexpr int VEC = Elem<T>::VEC;
    constexpr int Q = op_sums(OP);
    __shared__ float sm[2 * 4];
    long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    int j = (int)(b % A.sp);
    long long plane = b / A.sp;
    int c = (int)(plane % A.C);
    int n = (int)(plane / A.C);
    int beg = j * A.L;
    int len = min(A.L, A.HW - beg);

    PlaneReduce<T, OP> f;
    f.x = static_cast<const T*>(A.x);
    f.dy = static_cast<const T*>(A.dy);
    f.aux = static_cast<const T*>(A.aux);
    f.k = reduce_consts<T, OP>(A, c);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { f.a0[e] = 0.f; f.a1[e] = 0.f; }
    f.run = Run{0.f, 0.f, 0.f};
    walk_segment<kThreads, VEC>(plane * A.HW + beg, len, (int)threadIdx.x, A.S, f);

    int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    if constexpr (OP == OP_MOMENTS) {
        // the lanes' summaries, then the four wavefronts', joined in a fixed order: the row is (sum, M2)
        __shared__ Run wr[4];
        const Run r = run_wave_join(f.run, lane);
        if (lane == 0) wr[w] = r;
        __syncthreads();
        if (threadIdx.x == 0) {
            const Run t = run_join(run_join(wr[0], wr[1]), run_join(wr[2], wr[3]));
            size_t o = (size_t)c * A.rows + (size_t)n * A.sp + j;
            A.part0[o] = t.S;
            A.part1[o] = t.M2;
        }
        return;
    }
    float v[2] = {wave_sum(fold<VEC>(f.a0)), Q == 2 ? wave_sum(fold<VEC>(f.a1)) : 0.f};
    if (lane == 0) { sm[w] = v[0]; sm[4 + w] = v[1]; }
    __syncthreads();
    if (threadIdx.x == 0) {
        size_t o = (size_t)c * A.rows + (size_t)n * A.sp + j;
        A.part0[o] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
        if (Q == 2) A.part1[o] = (sm[4] + sm[5]) + (sm[6] + sm[7]);
    }
}

// One wavefront per plane (small planes): grid = ceil(N*C / 4).
template <typename T, int OP>
__global__ __launch_bounds__(kThreads) void nchw_reduce_wave(SweepArgs A)
{
    constexpr int VEC = Elem<T>::VEC;
    constexpr int Q = op_sums(OP);
    long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    long long plane = b * 4 + w;
    if (plane >= (long long)A.N * A.C) return;         // whole wavefronts leave together
    int c = (int)(plane % A.C);
    int n = (int)(plane / A.C);

    PlaneReduce<T, OP> f;
    f.x = static_cast<const T*>(A.x);
    f.dy = static_cast<const T*>(A.dy);
    f.aux = static_cast<const T*>(A.aux);
    f.k = reduce_consts<T, OP>(A, c);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { f.a0[e] = 0.f; f.a1[e] = 0.f; }
    f.run = Run{0.f, 0.f, 0.f};
    walk_segment<kWave, VEC>(plane * A.HW, A.HW, lane, A.S, f);

    if constexpr (OP == OP_MOMENTS) {
        const Run r = run_wave_join(f.run, lane);
        if (lane == 0) {
            size_t o = (size_t)c * A.rows + n;
            A.part0[o] = r.S;
            A.part1[o] = r.M2;
        }
        return;
    }
    float v0 = wave_sum(fold<VEC>(f.a0));
    float v1 = Q == 2 ? wave_sum(fold<VEC>(f.a1)) : 0.f;
    if (lane == 0) {
        size_t o = (size_t)c * A.rows + n;
        A.part0[o] = v0;
        if (Q == 2) A.part1[o] = v1;
    }
}

template <typename T, int EL>
__global__ __launch_bounds__(kThreads) void nchw_map_block(SweepArgs A)
{
    constexpr int VEC = Elem<T>::VEC;
    long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    int j = (int)(b % A.sp);
    long long plane = b / A.sp;
    int c = (int)(plane % A.C);
    int beg = j * A.L;
    int len = min(A.L, A.HW - beg);
    PlaneMap<T, EL> f;
    f.x = static_cast<const T*>(A.x);
    f.dy = static_cast<const T*>(A.dy);
    f.aux = static_cast<const T*>(A.aux);
    f.out = static_cast<T*>(A.out);
    f.out2 = static_cast<T*>(A.out2);
    f.k = map_consts<EL>(A, c);
    f.nt = A.nt;
    walk_segment<kThreads, VEC>(plane * A.HW + beg, len, (int)threadIdx.x, A.S, f);
}

template <typename T, int EL>
__global__ __launch_bounds__(kThreads) void nchw_map_wave(SweepArgs A)
{
    constexpr int VEC = Elem<T>::VEC;
    long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    long long plane = b * 4 + w;
    if (plane >= (long long)A.N * A.C) return;
    int c = (int)(plane % A.C);
    PlaneMap<T, EL> f;
    f.x = static_cast<const T*>(A.x);
    f.dy = static_cast<const T*>(A.dy);
    f.aux = static_cast<const T*>(A.aux);
    f.out = static_cast<T*>(A.out);
    f.out2 = static_cast<T*>(A.out2);
    f.k = map_consts<EL>(A, c);
    f.nt = A.nt;
    walk_segment<kWave, VEC>(plane * A.HW, A.HW, lane, A.S, f);
}

// --------------------------------------------------------------------------
// NCHW, tiny planes (at most kTinyPlaneBytes each, C a multiple of 8)
// --------------------------------------------------------------------------
// A wavefront per plane wastes most of its lanes on a plane of a few dozen values, and a launch of
// N * C / 4 workgroups that each fetch a hundred bytes is bound by dispatch, not by memory.  Here a
// workgroup takes `tg` planes of consecutive channels of one image: one contiguous, 16-byte aligned run of
// memory (8 planes of any size are a multiple of 16 bytes, and so is an image when C is a multiple of 8).
// Reductions stage the run in LDS with 16-byte loads, then 256 / tg neighbouring threads share a plane;
// the elementwise sweeps walk the run in vectors and look the channel of every element up.

constexpr int kTinyPlaneBytes = 2048;
constexpr int kTinyStageBytes = 16384;       // LDS per staged tensor: tg * plane bytes never exceeds it

// `tp` neighbouring lanes (a power of two <= 64, aligned) add their values in a fixed tree; all get the sum
__device__ __forceinline__ float group_sum(float v, int tp)
{
    for (int off = 1; off < tp; off <<= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ Run group_run_join(Run mine, int tp, int lane)
{
    for (int off = 1; off < tp; off <<= 1) {
        Run other;
        other.n = __shfl_xor(mine.n, off);
        other.S = __shfl_xor(mine.S, off);
        other.M2 = __shfl_xor(mine.M2, off);
        mine = (lane & off) ? run_join(other, mine) : run_join(mine, other);
    }
    return mine;
}

template <typename T, int OP>
__global__ __launch_bounds__(kThreads) void nchw_reduce_tiny(SweepArgs A)
{
    constexpr int VEC = Elem<T>::VEC;
    constexpr int Q = op_sums(OP);
    constexpr bool DY = op_has_dy(OP), Y = op_has_y(OP);
    using Raw = typename Elem<T>::Raw;
    __shared__ Raw sx[kTinyStageBytes / 16];
    __shared__ Raw sd[DY ? kTinyStageBytes / 16 : 1];
    __shared__ Raw sy[Y ? kTinyStageBytes / 16 : 1];
    const long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    const int groups = (A.C + A.tg - 1) / A.tg;
    const int n = (int)(b / groups), c0 = (int)(b % groups) * A.tg;
    const int gc = min(A.tg, A.C - c0);                       // planes of this workgroup (a multiple of 8)
    const long long e0 = ((long long)n * A.C + c0) * A.HW;    // its first element
    const int nvec = gc * A.HW / VEC;
    const int t = threadIdx.x;
    if (n >= A.N || e0 < 0 || e0 + (long long)gc * A.HW > A.S) return;     // never outside the tensor
    for (int v = t; v < nvec; v += kThreads) {
        sx[v] = Elem<T>::load_raw(static_cast<const T*>(A.x) + e0 + (long long)v * VEC);
        if (DY) sd[v] = Elem<T>::load_raw(static_cast<const T*>(A.dy) + e0 + (long long)v * VEC);
        if (Y) sy[v] = Elem<T>::load_raw(static_cast<const T*>(A.aux) + e0 + (long long)v * VEC);
    }
    __syncthreads();
    const int tp = kThreads / A.tg;                           // threads per plane (1 ... 32)
    const int pl = t / tp, sub = t % tp;
    const bool live = pl < gc;
    const int c = c0 + (live ? pl : 0);
    const ChanConst k = reduce_consts<T, OP>(A, c);
    const T* px = reinterpret_cast<const T*>(sx) + pl * A.HW;
    const T* pd = reinterpret_cast<const T*>(sd) + pl * A.HW;
    const T* py = reinterpret_cast<const T*>(sy) + pl * A.HW;
    float a0 = 0.f, a1 = 0.f;
    Run run = {0.f, 0.f, 0.f};
    if (live) {
        for (int j = sub; j < A.HW; j += tp) {
            const float xv = Elem<T>::load1(px + j);
            if constexpr (OP == OP_MOMENTS) {
                float v[1] = {xv - k.mu};
                run_feed<1>(run, v);
            } else {
                accumulate<OP>(k, xv, DY ? Elem<T>::load1(pd + j) : 0.f, Y ? Elem<T>::load1(py + j) : 0.f, a0, a1);
            }
        }
    }
    // (a plane's threads are neighbouring lanes of one wavefront: tp divides 64)
    const size_t o = (size_t)c * A.rows + n;
    if constexpr (OP == OP_MOMENTS) {
        run = group_run_join(run, tp, t & (kWave - 1));
        if (live && sub == 0) { A.part0[o] = run.S; A.part1[o] = run.M2; }
    } else {
        a0 = group_sum(a0, tp);
        if (Q == 2) a1 = group_sum(a1, tp);
        if (live && sub == 0) {
            A.part0[o] = a0;
            if (Q == 2) A.part1[o] = a1;
        }
    }
}

template <typename T, int EL>
__global__ __launch_bounds__(kThreads) void nchw_map_tiny(SweepArgs A)
{
    constexpr int VEC = Elem<T>::VEC;
    constexpr bool IN2 = el_has_2(EL), IN3 = el_has_3(EL);
    __shared__ ChanConst sk[256];
    const long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    const int groups = (A.C + A.tg - 1) / A.tg;
    const int n = (int)(b / groups), c0 = (int)(b % groups) * A.tg;
    const int gc = min(A.tg, A.C - c0);
    const long long e0 = ((long long)n * A.C + c0) * A.HW;
    const int nvec = gc * A.HW / VEC;
    const int t = threadIdx.x;
    if (n >= A.N || e0 < 0 || e0 + (long long)gc * A.HW > A.S) return;
    if (t < gc) sk[t] = map_consts<EL>(A, c0 + t);
    __syncthreads();
    const T* x = static_cast<const T*>(A.x) + e0;
    const T* v2p = static_cast<const T*>(A.dy) + e0;
    const T* v3p = static_cast<const T*>(A.aux) + e0;
    T* out = static_cast<T*>(A.out) + e0;
    T* out2 = A.out2 ? static_cast<T*>(A.out2) + e0 : nullptr;
    const float inv_hw = 1.0f / (float)A.HW;
    for (int v = t; v < nvec; v += kThreads) {
        float xv[VEC], v2[VEC], v3[VEC], r[VEC], dz[VEC];
        Elem<T>::loadv(x + (long long)v * VEC, xv);
        if (IN2) Elem<T>::loadv(v2p + (long long)v * VEC, v2);
        if (IN3) Elem<T>::loadv(v3p + (long long)v * VEC, v3);
        // plane of the vector's first element: the float quotient is exact to within one for indices below
        // 2^23, the two corrections settle it
        const int i0 = v * VEC;
        int pl = (int)((float)i0 * inv_hw);
        int rem = i0 - pl * A.HW;
        if (rem < 0) { rem += A.HW; --pl; }
        if (rem >= A.HW) { rem -= A.HW; ++pl; }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            while (rem >= A.HW) { rem -= A.HW; ++pl; }        // (planes may be shorter than a vector)
            dz[e] = 0.f;
            r[e] = map_value<EL>(sk[pl], xv[e], IN2 ? v2[e] : 0.f, IN3 ? v3[e] : 0.f, dz[e]);
            ++rem;
        }
        Elem<T>::storev(out + (long long)v * VEC, r, A.nt);
        if (IN3 && out2) Elem<T>::storev(out2 + (long long)v * VEC, dz, A.nt);
    }
}

// --------------------------------------------------------------------------
// NHWC: the C channels of a pixel are contiguous; a thread owns V channels
// --------------------------------------------------------------------------

// Workgroup = (row, column tile).  A row is a run of up to PL pixels of one
// shard; a column tile is TW vectors of V channels.  Thread t works on vector
// column t % TW of pixels t / TW, t / TW + rpp, ...
template <typename T, int V, int OP>
__global__ __launch_bounds__(kThreads) void nhwc_reduce(SweepArgs A)
{
    constexpr int Q = op_sums(OP);
    __shared__ float sm[Q * kThreads * V];
    long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    int ct = (int)(b % A.ctiles);
    int row = (int)(b / A.ctiles);
    int k = row / A.pps, pj = row % A.pps;
    long long pix0 = (long long)k * A.spix + (long long)pj * A.PL;
    long long left = A.spix - (long long)pj * A.PL;
    int npix = (int)(left < A.PL ? left : A.PL);
    if (pix0 < 0 || (pix0 + npix) * A.C > A.S) npix = 0;    // never outside the tensor
    int t = threadIdx.x;
    int col = t % A.TW, r = t / A.TW;
    int vc = ct * A.TW + col;
    bool active = r < A.rpp && vc < A.cv;
    int cb = vc * V;

    float a0[V], a1[V];
    float cnt = 0.f;                 // OP_MOMENTS: values per channel this thread has taken in so far
#pragma unroll
    for (int e = 0; e < V; ++e) { a0[e] = 0.f; a1[e] = 0.f; }
    if (active) {
        ChanConst kc[V];
#pragma unroll
        for (int e = 0; e < V; ++e) kc[e] = reduce_consts<T, OP>(A, cb + e);
        const T* px = static_cast<const T*>(A.x) + pix0 * A.C + cb;
        const T* pd = static_cast<const T*>(A.dy) + pix0 * A.C + cb;
        const T* py = static_cast<const T*>(A.aux) + pix0 * A.C + cb;
        const long long C = A.C;
        const int rpp = A.rpp;
        int i = r;
        constexpr bool DY = op_has_dy(OP), Y = op_has_y(OP);
        constexpr int UNR = DY ? 4 : 8;        // loads in flight per lane and tensor
        for (; i + (UNR - 1) * rpp < npix; i += UNR * rpp) {
            float xv[UNR][V], dv[UNR][V], yv[UNR][V];
#pragma unroll
            for (int u = 0; u < UNR; ++u) Access<T, V>::load(px + (long long)(i + u * rpp) * C, xv[u]);
            if (DY) {
#pragma unroll
                for (int u = 0; u < UNR; ++u) Access<T, V>::load(pd + (long long)(i + u * rpp) * C, dv[u]);
            }
            if (Y) {
#pragma unroll
                for (int u = 0; u < UNR; ++u) Access<T, V>::load(py + (long long)(i + u * rpp) * C, yv[u]);
            }
            if constexpr (OP == OP_MOMENTS) {
                // a chunk of UNR pixels joins this thread's summaries (a0: sum, a1: M2); the count and the
                // weights of the join are the same for all of the thread's channels
                const float rn = cnt > 0.f ? __builtin_amdgcn_rcpf(cnt) : 0.f;
                const float wj = cnt * (float)UNR * __builtin_amdgcn_rcpf(cnt + (float)UNR);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    float cs = 0.f, cq = 0.f;
#pragma unroll
                    for (int u = 0; u < UNR; ++u) {
                        xv[u][e] -= kc[e].mu;
                        cs += xv[u][e];
                    }
                    const float cm = cs * (1.0f / (float)UNR);
#pragma unroll
                    for (int u = 0; u < UNR; ++u) {
                        const float d = xv[u][e] - cm;
                        cq += d * d;
                    }
                    const float d = cm - a0[e] * rn;
                    a1[e] += cq + (d * d) * wj;
                    a0[e] += cs;
                }
                cnt += (float)UNR;
                continue;
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    accumulate<OP>(kc[e], xv[u][e], DY ? dv[u][e] : 0.f, Y ? yv[u][e] : 0.f, a0[e], a1[e]);
        }
        for (; i < npix; i += rpp) {
            float xv[V], dv[V], yv[V];
            Access<T, V>::load(px + (long long)i * C, xv);
            if constexpr (OP == OP_MOMENTS) {
                const float rn = cnt > 0.f ? __builtin_amdgcn_rcpf(cnt) : 0.f;
                const float wj = cnt * __builtin_amdgcn_rcpf(cnt + 1.f);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float v = xv[e] - kc[e].mu;
                    const float d = v - a0[e] * rn;
                    a1[e] += (d * d) * wj;
                    a0[e] += v;
                }
                cnt += 1.f;
                continue;
            }
            if (DY) Access<T, V>::load(pd + (long long)i * C, dv);
            if (Y) Access<T, V>::load(py + (long long)i * C, yv);
#pragma unroll
            for (int e = 0; e < V; ++e) accumulate<OP>(kc[e], xv[e], DY ? dv[e] : 0.f, Y ? yv[e] : 0.f, a0[e], a1[e]);
        }
    }
    // fold the rpp pixel rows of the workgroup, in a fixed order
    const int nout = A.TW * V;
    if (r < A.rpp) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            sm[(0 * A.rpp + r) * nout + col * V + e] = a0[e];
            if (Q == 2) sm[(1 * A.rpp + r) * nout + col * V + e] = a1[e];
        }
    }
    __syncthreads();
    for (int o = t; o < nout; o += kThreads) {
        int ch = ct * nout + o;
        if (ch >= A.C) continue;
        float s0 = 0.f, s1 = 0.f;
        if constexpr (OP == OP_MOMENTS) {
            // the pixel rows' summaries joined in row order; row rr took pixels rr, rr + rpp, ... of the piece
            Run acc = {0.f, 0.f, 0.f};
            for (int rr = 0; rr < A.rpp; ++rr) {
                const int n_rr = rr < npix ? (npix - rr + A.rpp - 1) / A.rpp : 0;
                Run part = {(float)n_rr, sm[(0 * A.rpp + rr) * nout + o], sm[(1 * A.rpp + rr) * nout + o]};
                acc = run_join(acc, part);
            }
            s0 = acc.S;
            s1 = acc.M2;
        } else {
            for (int rr = 0; rr < A.rpp; ++rr) {
                s0 += sm[(0 * A.rpp + rr) * nout + o];
                if (Q == 2) s1 += sm[(1 * A.rpp + rr) * nout + o];
            }
        }
        size_t po = (size_t)row * A.C + ch;          // consecutive threads, consecutive floats: whole lines per store
        A.part0[po] = s0;
        if (Q == 2) A.part1[po] = s1;
    }
}

template <typename T, int V, int EL>
__global__ __launch_bounds__(kThreads) void nhwc_map(SweepArgs A)
{
    long long b = A.reverse ? (long long)gridDim.x - 1 - blockIdx.x : (long long)blockIdx.x;
    int ct = (int)(b % A.ctiles);
    int row = (int)(b / A.ctiles);
    int k = row / A.pps, pj = row % A.pps;
    long long pix0 = (long long)k * A.spix + (long long)pj * A.PL;
    long long left = A.spix - (long long)pj * A.PL;
    int npix = (int)(left < A.PL ? left : A.PL);
    if (pix0 < 0 || (pix0 + npix) * A.C > A.S) npix = 0;
    int t = threadIdx.x;
    int col = t % A.TW, r = t / A.TW;
    int vc = ct * A.TW + col;
    if (!(r < A.rpp && vc < A.cv)) return;
    int cb = vc * V;
    ChanConst kc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) kc[e] = map_consts<EL>(A, cb + e);
    const T* px = static_cast<const T*>(A.x) + pix0 * A.C + cb;
    const T* pd = static_cast<const T*>(A.dy) + pix0 * A.C + cb;
    const T* py = static_cast<const T*>(A.aux) + pix0 * A.C + cb;
    T* po = static_cast<T*>(A.out) + pix0 * A.C + cb;
    T* po2 = A.out2 ? static_cast<T*>(A.out2) + pix0 * A.C + cb : nullptr;
    constexpr bool IN2 = el_has_2(EL), IN3 = el_has_3(EL);
    const long long C = A.C;
    const int rpp = A.rpp;
    int i = r;
    // loads in flight per lane and tensor: as many as the registers allow next to the other operands (measured on
    // 64 x 50 x 84 x 512 bf16, normalise / dx: 4 each 110 / 166 us, 16 / 8 99 / 160)
    constexpr int UNR = IN3 ? 4 : IN2 ? 8 : 16;
    for (; i + (UNR - 1) * rpp < npix; i += UNR * rpp) {
        float xv[UNR][V], v2[UNR][V], v3[UNR][V];
#pragma unroll
        for (int u = 0; u < UNR; ++u) Access<T, V>::load(px + (long long)(i + u * rpp) * C, xv[u]);
        if (IN2) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) Access<T, V>::load(pd + (long long)(i + u * rpp) * C, v2[u]);
        }
        if (IN3) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) Access<T, V>::load(py + (long long)(i + u * rpp) * C, v3[u]);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float o[V], dz[V];
#pragma unroll
            for (int e = 0; e < V; ++e) {
                dz[e] = 0.f;
                o[e] = map_value<EL>(kc[e], xv[u][e], IN2 ? v2[u][e] : 0.f, IN3 ? v3[u][e] : 0.f, dz[e]);
            }
            Access<T, V>::store(po + (long long)(i + u * rpp) * C, o, A.nt);
            if (IN3 && po2) Access<T, V>::store(po2 + (long long)(i + u * rpp) * C, dz, A.nt);
        }
    }
    for (; i < npix; i += rpp) {
        float xv[V], v2[V], v3[V], o[V], dz[V];
        Access<T, V>::load(px + (long long)i * C, xv);
        if (IN2) Access<T, V>::load(pd + (long long)i * C, v2);
        if (IN3) Access<T, V>::load(py + (long long)i * C, v3);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            dz[e] = 0.f;
            o[e] = map_value<EL>(kc[e], xv[e], IN2 ? v2[e] : 0.f, IN3 ? v3[e] : 0.f, dz[e]);
        }
        Access<T, V>::store(po + (long long)i * C, o, A.nt);
        if (IN3 && po2) Access<T, V>::store(po2 + (long long)i * C, dz, A.nt);
    }
}

// --------------------------------------------------------------------------
// cross-shard reductions (tiny: [C][rows] floats or [K][C] doubles)
// --------------------------------------------------------------------------

struct CombineArgs {
    const float* part0;   // row r of channel c at c * cs + r * rs
    const float* part1;   // the same (CM_BWD, CM_SHARDS2 only)
    long long cs, rs;
    double* sh0;          // [K][C] shard sums out, may be null
    double* sh1;
    float* out0;          // mean | invstd | dbeta
    float* out1;          // mean_lo (workspace) | - | dgamma
    float* out2;          // mean_lo (caller, may be null)
    float* out3;          // invstd (CM_MOMENTS)
    double M;
    double eps;
    double shard_count;   // values per shard and channel
    const void* x;        // pivots are read from here when pivot_stride > 0
    long long pivot_stride;
    int is_bf16;
    int C, rows, K, rps, G; // G lanes share one shard, a power of two <= 64
    long long row_mod, row_full, row_total;   // CM_MOMENTS: values per row (see merge_shard_moments)
    unsigned* clear_word;   // set to zero if not null (the workspace's error word)
};

__device__ __forceinline__ double pivot_of(const CombineArgs& A, int c)
{
    if (A.pivot_stride <= 0) return 0.0;
    long long o = (long long)c * A.pivot_stride;
    if (A.is_bf16) return (double)bf16_to_f32(static_cast<const bf16_t*>(A.x)[o].bits);
    return (double)static_cast<const float*>(A.x)[o];
}

// One wavefront per channel.  Level 1: groups of G lanes add the rows of one
// shard (the device sum of Algorithm 1).  Level 2: the shard sums are added
// (its reduce step).  Double precision, fixed order.
__device__ __forceinline__ double shard_then_total(const float* pr, double* sh, int c, const CombineArgs& A, int lane,
                                                   double shard_offset)
{
    const int G = A.G;
    const int gl = lane & (G - 1), gi = lane / G, spp = kWave / G;
    constexpr int B = 8;                 // passes whose first loads are issued together
    double tot = 0.0;
    for (int k0 = 0; k0 < A.K; k0 += B * spp) {
        double acc[B];
        // the first row of every pass: independent loads, one memory round trip for all B passes
#pragma unroll
        for (int u = 0; u < B; ++u) {
            int k = k0 + u * spp + gi;
            bool have = k < A.K && gl < A.rps;
            float v = pr[have ? ((size_t)k * A.rps + gl) * A.rs : 0];
            acc[u] = have ? (double)v : 0.0;
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
            int k = k0 + u * spp + gi;
            if (k < A.K)
                for (int r = gl + G; r < A.rps; r += G) acc[u] += (double)pr[((size_t)k * A.rps + r) * A.rs];
            for (int off = G >> 1; off >= 1; off >>= 1) acc[u] += __shfl_xor(acc[u], off);
            if (k < A.K) {
                if (sh && gl == 0) sh[(size_t)k * A.C + c] = acc[u] + shard_offset;
                tot += acc[u];
            }
        }
    }
    for (int off = kWave >> 1; off >= G; off >>= 1) tot += __shfl_xor(tot, off);
    return tot;
}

// One-sweep statistics: a summary (count, mean, M2) of a set of values, M2 the sum of
// squared deviations from the set's own mean, and the pairwise merge of two summaries.
struct Moments {
    double n, mean, m2;
};
// 1/v in double precision without the division sequence: the hardware's float reciprocal, two Newton steps
// (1e-7 -> 1e-14 -> rounding).  For counts, which are positive and far inside float range.
__device__ __forceinline__ double rcp_count(double v)
{
    double y = (double)__builtin_amdgcn_rcpf((float)v);
    y = y * (2.0 - v * y);
    y = y * (2.0 - v * y);
    return y;
}
__device__ __forceinline__ Moments merge_moments(const Moments& a, const Moments& b)
{
    Moments r;
    r.n = a.n + b.n;
    if (r.n == 0.0) return a;
    const double rn = rcp_count(r.n);
    const double d = b.mean - a.mean;
    r.mean = a.mean + d * (b.n * rn);
    r.m2 = a.m2 + b.m2 + d * d * (a.n * b.n * rn);
    return r;
}

// Rows of (sum(x - p), M2 about the row's own mean) -> one summary per shard (its mean taken
// about the pivot p) -> all shards merged.  Shards are dealt to lane groups as in
// shard_then_total; the lanes of a group merge their rows of the shard in order and then among
// themselves, a lane merges its shards in order, then the 64 lanes merge in a fixed tree (the
// lower lane always on the left).  Double precision throughout; every M2 that enters is a sum
// of squares about its own set's mean, so nothing is formed as a difference of large numbers.
// Row r of a channel holds min(row_full, row_total - (r % row_mod) * row_full) values.
__device__ __forceinline__ Moments merge_shard_moments(const float* p1, const float* p2, const CombineArgs& A, int lane)
{
    const int G = A.G;
    const int gl = lane & (G - 1), gi = lane / G, spp = kWave / G;
    Moments mine = {0.0, 0.0, 0.0};
    for (int k0 = 0; k0 < A.K; k0 += spp) {
        const int k = k0 + gi;
        Moments sk = {0.0, 0.0, 0.0};
        if (k < A.K)
            for (int r = gl; r < A.rps; r += G) {
                const long long row = (long long)k * A.rps + r;
                const long long left = A.row_total - (row % A.row_mod) * A.row_full;
                Moments m;
                m.n = (double)(left < A.row_full ? left : A.row_full);
                m.mean = (double)p1[(size_t)row * A.rs] / m.n;             // about the pivot
                m.m2 = (double)p2[(size_t)row * A.rs];
                sk = merge_moments(sk, m);
            }
        for (int off = 1; off < G; off <<= 1) {       // the group's lanes, the lower lane on the left
            Moments other;
            other.n = __shfl_xor(sk.n, off);
            other.mean = __shfl_xor(sk.mean, off);
            other.m2 = __shfl_xor(sk.m2, off);
            sk = (gl & off) ? merge_moments(other, sk) : merge_moments(sk, other);
        }
        if (k < A.K && gl == 0) mine = merge_moments(mine, sk);
    }
    for (int off = 1; off < kWave; off <<= 1) {
        Moments other;
        other.n = __shfl_xor(mine.n, off);
        other.mean = __shfl_xor(mine.mean, off);
        other.m2 = __shfl_xor(mine.m2, off);
        mine = (lane & off) ? merge_moments(other, mine) : merge_moments(mine, other);
    }
    return mine;
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void combine_rows(CombineArgs A)
{
    int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    int c = blockIdx.x * 4 + w;
    if (A.clear_word && blockIdx.x == 0 && threadIdx.x == 0) *A.clear_word = 0u;
    if (c >= A.C) return;
    const double pivot = pivot_of(A, c);      // zero unless the rows hold sums about a pivot
    if (MODE == CM_MOMENTS) {
        Moments m = merge_shard_moments(A.part0 + (size_t)c * A.cs, A.part1 + (size_t)c * A.cs, A, lane);
        if (lane != 0) return;
        double mean = pivot + m.mean;
        float hi = (float)mean;
        float lo = (float)(mean - (double)hi);
        float istd = (float)(1.0 / sqrt(m.m2 / A.M + A.eps));
        A.out0[c] = hi;
        A.out1[c] = lo;
        if (A.out2) A.out2[c] = lo;
        A.out3[c] = istd;
        return;
    }
    double t0 = shard_then_total(A.part0 + (size_t)c * A.cs, A.sh0, c, A, lane, pivot * A.shard_count);
    double t1 = 0.0;
    if (MODE == CM_BWD || MODE == CM_SHARDS2)
        t1 = shard_then_total(A.part1 + (size_t)c * A.cs, A.sh1, c, A, lane, 0.0);
    if (lane != 0) return;
    if (MODE == CM_MEAN) {
        double m = pivot + t0 / A.M;
        float hi = (float)m;
        float lo = (float)(m - (double)hi);
        A.out0[c] = hi;
        A.out1[c] = lo;
        if (A.out2) A.out2[c] = lo;
    } else if (MODE == CM_INVSTD) {
        A.out0[c] = (float)(1.0 / sqrt(t0 / A.M + A.eps));
    } else if (MODE == CM_BWD) {
        A.out0[c] = (float)t0;
        A.out1[c] = (float)t1;
    }
}

constexpr int kCombineChannels = 16;
// The same for channels-last row partials ([rows][C]: a row's channels side by side).  There one wavefront per
// channel would fetch every row from a different cache line; here a workgroup takes CL = 16 neighbouring channels and
// its 256 threads are CL channels x RL = 16 "row lanes".  A.G row lanes (a power of two) share one shard: each
// adds every G-th row of the shard in order, the G partial sums are added in lane order (the device sum of
// Algorithm 1, stored to the shard-sum arrays if wanted), and the group's first lane keeps the running total of the
// shards the group takes in turn (k, k + RL / G, ...); the totals of a channel are then added in lane order (the
// reduce step).  Double precision, fixed order.  CM_MOMENTS: summaries merged pairwise instead of sums added, in
// the same order.  The host picks G as large as the shard count and the rows per shard allow, so that a lane walks
// few rows one after the other (8 or 4 channels per workgroup, for more workgroups, measured the same).
template <int MODE>
__global__ __launch_bounds__(kThreads) void combine_rows_cl(CombineArgs A)
{
    constexpr int Q = (MODE == CM_BWD || MODE == CM_SHARDS2 || MODE == CM_MOMENTS) ? 2 : 1;
    constexpr int CL = kCombineChannels, RL = kThreads / CL;   // channels, row lanes
    __shared__ double tot[3][RL][CL];           // [what][row lane][channel]
    const int t = threadIdx.x, cl = t % CL, rl = t / CL;
    const int G = A.G, gl = rl & (G - 1), gi = rl / G, spp = RL / G;
    const int c = blockIdx.x * CL + cl;
    if (A.clear_word && blockIdx.x == 0 && t == 0) *A.clear_word = 0u;
    const bool live = c < A.C;
    const double pivot = live ? pivot_of(A, c) : 0.0;
    double t0 = 0.0, t1 = 0.0;
    Moments mine = {0.0, 0.0, 0.0};
    // CM_MOMENTS: a row holds row_full values, the last row of a run what is left
    const double n_last = (double)(A.row_total - (A.row_mod - 1) * A.row_full);
    const double r_full = MODE == CM_MOMENTS ? rcp_count((double)A.row_full) : 0.0;
    const double r_last = MODE == CM_MOMENTS ? rcp_count(n_last) : 0.0;
    const float* p0 = A.part0 + (live ? c : 0);
    const float* p1 = A.part1 + (live ? c : 0);
    for (int k0 = 0; k0 < A.K; k0 += spp) {      // the same trip count for every thread: barriers inside
        const int k = k0 + gi;
        const bool work = live && k < A.K;
        double a0 = 0.0, a1 = 0.0;
        Moments sk = {0.0, 0.0, 0.0};
        constexpr int B = 8;                     // rows fetched together
        if (work)
            for (int r0 = gl; r0 < A.rps; r0 += B * G) {
                float v0[B], v1[B];
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    const bool have = r0 + u * G < A.rps;
                    const size_t o = have ? ((size_t)k * A.rps + r0 + u * G) * (size_t)A.C : 0;
                    v0[u] = p0[o];
                    v1[u] = Q == 2 ? p1[o] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    if (r0 + u * G < A.rps) {
                        if (MODE == CM_MOMENTS) {
                            const long long row = (long long)k * A.rps + r0 + u * G;
                            const bool last = row % A.row_mod == A.row_mod - 1;
                            Moments m;
                            m.n = last ? n_last : (double)A.row_full;
                            m.mean = (double)v0[u] * (last ? r_last : r_full);        // about the pivot
                            m.m2 = (double)v1[u];
                            sk = merge_moments(sk, m);
                        } else {
                            a0 += (double)v0[u];
                            a1 += (double)v1[u];
                        }
                    }
                }
            }
        if (G > 1) {                             // the group's partial results, added by its first lane in lane order
            if (MODE == CM_MOMENTS) {
                tot[0][rl][cl] = sk.n;
                tot[1][rl][cl] = sk.mean;
                tot[2][rl][cl] = sk.m2;
            } else {
                tot[0][rl][cl] = a0;
                tot[1][rl][cl] = a1;
            }
            __syncthreads();
            if (gl == 0)
                for (int j = 1; j < G; ++j) {
                    if (MODE == CM_MOMENTS) {
                        Moments o = {tot[0][rl + j][cl], tot[1][rl + j][cl], tot[2][rl + j][cl]};
                        sk = merge_moments(sk, o);
                    } else {
                        a0 += tot[0][rl + j][cl];
                        a1 += tot[1][rl + j][cl];
                    }
                }
            __syncthreads();
        }
        if (work && gl == 0) {
            if (MODE == CM_MOMENTS) {
                mine = merge_moments(mine, sk);
            } else {
                if (A.sh0) A.sh0[(size_t)k * A.C + c] = a0 + pivot * A.shard_count;
                if (Q == 2 && A.sh1) A.sh1[(size_t)k * A.C + c] = a1;
                t0 += a0;
                t1 += a1;
            }
        }
    }
    if (MODE == CM_MOMENTS) {
        tot[0][rl][cl] = mine.n;
        tot[1][rl][cl] = mine.mean;
        tot[2][rl][cl] = mine.m2;
    } else {
        tot[0][rl][cl] = t0;
        tot[1][rl][cl] = t1;
    }
    __syncthreads();
    if (rl != 0 || !live) return;
    if (MODE == CM_MOMENTS) {
        Moments m = {tot[0][0][cl], tot[1][0][cl], tot[2][0][cl]};
        for (int j = G; j < RL; j += G) {
            Moments o = {tot[0][j][cl], tot[1][j][cl], tot[2][j][cl]};
            m = merge_moments(m, o);
        }
        double mean = pivot + m.mean;
        float hi = (float)mean;
        float lo = (float)(mean - (double)hi);
        A.out0[c] = hi;
        A.out1[c] = lo;
        if (A.out2) A.out2[c] = lo;
        A.out3[c] = (float)(1.0 / sqrt(m.m2 / A.M + A.eps));
        return;
    }
    double s0 = 0.0, s1 = 0.0;
    for (int j = 0; j < RL; j += G) {
        s0 += tot[0][j][cl];
        s1 += tot[1][j][cl];
    }
    if (MODE == CM_MEAN) {
        double m = pivot + s0 / A.M;
        float hi = (float)m;
        float lo = (float)(m - (double)hi);
        A.out0[c] = hi;
        A.out1[c] = lo;
        if (A.out2) A.out2[c] = lo;
    } else if (MODE == CM_INVSTD) {
        A.out0[c] = (float)(1.0 / sqrt(s0 / A.M + A.eps));
    } else if (MODE == CM_BWD) {
        A.out0[c] = (float)s0;
        A.out1[c] = (float)s1;
    }
}

// Reduce step alone, from caller-held shard sums: one thread per channel.
template <int MODE>
__global__ __launch_bounds__(kThreads) void combine_shards(const double* s0, const double* s1, int K, int C,
                                                           double M, double eps, float* out0, float* out1)
{
    int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= C) return;
    double t0 = 0.0, t1 = 0.0;
    for (int k = 0; k < K; ++k) {
        t0 += s0[(size_t)k * C + c];
        if (MODE == CM_BWD) t1 += s1[(size_t)k * C + c];
    }
    if (MODE == CM_MEAN) {
        double m = t0 / M;
        float hi = (float)m;
        out0[c] = hi;
        if (out1) out1[c] = (float)(m - (double)hi);
    } else if (MODE == CM_INVSTD) {
        out0[c] = (float)(1.0 / sqrt(t0 / M + eps));
    } else {
        out0[c] = (float)t0;
        out1[c] = (float)t1;
    }
}

// Exponential moving average of the pooled statistics (one thread per channel, float64).
// The biased batch variance is recovered from invstd: var = 1/invstd^2 - eps.
static __global__ __launch_bounds__(kThreads) void running_update(const float* mean, const float* mean_lo, const float* invstd,
                                                           double eps, double unbias, double momentum,
                                                           float* running_mean, float* running_var, int C)
{
    int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= C) return;
    double mu = (double)mean[c] + (mean_lo ? (double)mean_lo[c] : 0.0);
    double is = (double)invstd[c];
    double var = 1.0 / (is * is) - eps;
    if (var < 0.0) var = 0.0;                       // rounding of invstd when var << eps; NaN stays NaN
    double keep = 1.0 - momentum;
    running_mean[c] = (float)(keep * (double)running_mean[c] + momentum * mu);
    running_var[c] = (float)(keep * (double)running_var[c] + momentum * (var * unbias));
}

// Plain copy of `nvec` 16-byte vectors, 8 per thread: reads and writes a known
// number of bytes, for calibrating hardware traffic counters.
static __global__ __launch_bounds__(kThreads) void calibration_copy(const u32x4* src, u32x4* dst, size_t nvec)
{
    size_t i = (size_t)blockIdx.x * (kThreads * 8) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 8; ++u, i += kThreads)
        if (i < nvec) dst[i] = src[i];
}

}  // namespace cgbn
