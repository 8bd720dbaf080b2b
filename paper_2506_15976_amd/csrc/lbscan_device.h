// Device-side helpers shared by the lbscan HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lbscan {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// 2^v through the hardware transcendental (v_exp_f32), without the range
// fix-ups of the library exp2f: arguments here are <= ~30 and results that
// underflow may flush to zero.
__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float fast_log2(float v) { return __builtin_amdgcn_logf(v); }
__device__ __forceinline__ float fast_rcp(float v) { return __builtin_amdgcn_rcpf(v); }

// softplus(v) = log(1 + exp(v)), v > 20 -> v (Algorithm 1's Delta line), and its
// derivative sigma(v) = e / (1 + e) (1 above 20).  The time step multiplies every
// state update, so it is kept to a few ulp, in one branch-free form for all v:
// with e = exp(v) and w = fl(1 + e),
//     log(1 + e) = log(w) + (e - (w - 1)) / w        (up to O(ulp^2)),
// where the second term restores the bits lost when 1 + e was rounded (it is all
// of the result for e < 2^-24).  v_log_f32 is accurate to ~1e-7 of its result
// also for arguments next to 1 (measured on MI355X: 1.1e-7 over w - 1 in
// [1e-7, 1]), so no series is needed there.  For v > 88 e overflows to inf and
// the sum becomes NaN; the selects below discard it.
__device__ __forceinline__ float softplus_f32(float v, float& dsoftplus)
{
    const float e = fast_exp2(v * kLog2e);
    const float w = 1.0f + e;
    const float rw = fast_rcp(w);
    const float r = fmaf(fast_log2(w), kLn2, (e - (w - 1.0f)) * rw);
    const bool lin = v > 20.0f;
    dsoftplus = lin ? 1.0f : e * rw;
    return lin ? v : r;
}
__device__ __forceinline__ float softplus_f32(float v)
{
    float unused;
    return softplus_f32(v, unused);
}

__device__ __forceinline__ float sigmoid_f32(float v)
{
    return fast_rcp(1.0f + fast_exp2(-v * kLog2e));
}

// ---- scan order ------------------------------------------------------------
// The order in which a row's tokens are scanned: index t of the scanned sequence ->
// index of the token as stored.  kind 0: the tokens as stored.  kind 1: the tokens
// [prefix, prefix + H W) are an H x W grid stored row by row and are scanned column
// by column, top to bottom (the vertical scans of the multi-direction models of
// Sec. 4.5 / Appendix D); tokens before and after the grid (class tokens) keep
// their places.  Set by the host; H > 0 also for kind 0.
struct TokenOrder {
    int kind, prefix, H, W, HW;
    float rH;          // 1 / H
    __device__ __forceinline__ int operator()(int t) const
    {
        if (kind == 0) return t;
        const int k = t - prefix;
        if (k < 0 || k >= HW) return t;
        // column c = k / H: the float quotient is off by at most one for k < 2^24
        int c = (int)((float)k * rH);
        int r = k - c * H;
        if (r < 0) { r += H; --c; }
        if (r >= H) { r -= H; ++c; }
        return prefix + r * W + c;
    }
};

// ---- storage types -------------------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
// round to nearest even; NaN stays NaN (gfx950 converts in hardware, two values per
// v_cvt_pk_bf16_f32 where the compiler can pair them)
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v)
{
    bf16_t o;
    o.bits = __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
    return o;
}

// Four consecutive elements.  Global memory on gfx950 serves multi-dword
// accesses at dword alignment, so the fp32 quad only promises 4-byte alignment
// (rows of odd length start at any dword); the bf16 quad promises 4 bytes too:
// where a row can start at an odd element callers use quad_raw_unaligned /
// quad_store_unaligned inside the row and element accesses at its ragged end.
template <typename T> struct Quad;
template <> struct __attribute__((packed, aligned(4))) Quad<float> { float v[4]; };
template <> struct __attribute__((packed, aligned(4))) Quad<bf16_t> { bf16_t v[4]; };

// One quad of a (rows, L) tensor.  `base` is uniform, `off` the element offset of
// quad element 0 and `ph` its token index.  The fast form is one unconditional
// quad load.  The checked form zeroes elements whose token index ph + e is outside
// [0, L); it loads from a clamped (always valid) address and selects afterwards,
// so that no load sits behind a divergent branch: a load that is conditionally
// re-issued into the same registers would force the compiler to wait for the
// first one and serialise the prefetch.
template <typename T>
__device__ __forceinline__ void quad_load_fast(const T* __restrict__ base, long off, float out[4])
{
    const Quad<T> q = *reinterpret_cast<const Quad<T>*>(base + off);
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = to_f32(q.v[e]);
}

template <typename T>
__device__ __forceinline__ void quad_load_checked(const T* __restrict__ base, long off, int ph,
                                                  int L, float out[4])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int t = ph + e;
        const int tc = t < 0 ? 0 : (t >= L ? L - 1 : t);
        const float v = to_f32(base[off + (tc - ph)]);
        out[e] = (t == tc) ? v : 0.0f;
    }
}

// The same two loads, returning the raw quad (storage type) for later conversion.
template <typename T>
__device__ __forceinline__ Quad<T> quad_raw_fast(const T* __restrict__ base, long off)
{
    return *reinterpret_cast<const Quad<T>*>(base + off);
}

// Four consecutive 2-byte elements at ANY element address (rows of odd length start at
// odd elements every other row, where a 4-byte access is not allowed): the three
// aligned dwords around them are loaded and shifted by 16 bits where the address is
// odd.  Branch-free, so lanes of either parity share the instructions.  The load
// covers the 12 bytes from the address rounded down to 4: the caller guarantees that
// they lie inside the tensor (one element before an odd address always does; up to
// two elements after the quad must).
__device__ __forceinline__ Quad<bf16_t> quad_raw_unaligned(const bf16_t* __restrict__ p)
{
    struct __attribute__((packed, aligned(4))) Words3 { uint32_t v[3]; };
    const uintptr_t u = reinterpret_cast<uintptr_t>(p);
    const Words3 w = *reinterpret_cast<const Words3*>(u & ~static_cast<uintptr_t>(3));
    const uint32_t sh = (static_cast<uint32_t>(u) & 2u) * 8u;           // 0 or 16
    const uint32_t lo = __builtin_amdgcn_alignbit(w.v[1], w.v[0], sh);
    const uint32_t hi = __builtin_amdgcn_alignbit(w.v[2], w.v[1], sh);
    Quad<bf16_t> q;
    q.v[0].bits = (uint16_t)lo; q.v[1].bits = (uint16_t)(lo >> 16);
    q.v[2].bits = (uint16_t)hi; q.v[3].bits = (uint16_t)(hi >> 16);
    return q;
}
// (fp32 rows need no such path; the overload keeps templates uniform)
__device__ __forceinline__ Quad<float> quad_raw_unaligned(const float* __restrict__ p)
{
    return *reinterpret_cast<const Quad<float>*>(p);
}
// The matching store: 2 + 4 + 2 bytes at an odd element address, 8 bytes at an even one.
__device__ __forceinline__ void quad_store_unaligned(bf16_t* __restrict__ p, const float in[4])
{
    bf16_t e[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) e[k] = from_f32<bf16_t>(in[k]);
    if (reinterpret_cast<uintptr_t>(p) & 2u) {
        p[0] = e[0];
        *reinterpret_cast<uint32_t*>(p + 1) = (uint32_t)e[1].bits | ((uint32_t)e[2].bits << 16);
        p[3] = e[3];
    } else {
        Quad<bf16_t> q;
#pragma unroll
        for (int k = 0; k < 4; ++k) q.v[k] = e[k];
        *reinterpret_cast<Quad<bf16_t>*>(p) = q;
    }
}
__device__ __forceinline__ void quad_store_unaligned(float* __restrict__ p, const float in[4])
{
    Quad<float> q;
#pragma unroll
    for (int k = 0; k < 4; ++k) q.v[k] = in[k];
    *reinterpret_cast<Quad<float>*>(p) = q;
}

template <typename T> __device__ __forceinline__ T zero_elem();
template <> __device__ __forceinline__ float zero_elem<float>() { return 0.0f; }
template <> __device__ __forceinline__ bf16_t zero_elem<bf16_t>() { bf16_t z; z.bits = 0; return z; }

template <typename T>
__device__ __forceinline__ Quad<T> quad_raw_checked(const T* __restrict__ base, long off, int ph, int L)
{
    Quad<T> q;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int t = ph + e;
        const int tc = t < 0 ? 0 : (t >= L ? L - 1 : t);
        const T v = base[off + (tc - ph)];
        q.v[e] = (t == tc) ? v : zero_elem<T>();
    }
    return q;
}
// The same for a scan order: element e is the token ord(ph + e) of the row that
// starts at base + off - ph.
template <typename T>
__device__ __forceinline__ Quad<T> quad_raw_checked(const T* __restrict__ base, long off, int ph, int L,
                                                    const TokenOrder& ord)
{
    if (ord.kind == 0) return quad_raw_checked<T>(base, off, ph, L);
    Quad<T> q;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int t = ph + e;
        const int tc = t < 0 ? 0 : (t >= L ? L - 1 : t);
        const T v = base[(off - ph) + ord(tc)];
        q.v[e] = (t == tc) ? v : zero_elem<T>();
    }
    return q;
}

// The same result as quad_raw_checked with ONE quad load, for rows of at least four
// tokens that allow quad loads: the quad is loaded from the nearest position that
// lies inside the row (ph clamped to [0, L-4]) and its elements are moved to where
// they belong; elements whose token ph + e is outside [0, L) become zero.  Element
// loads cost the texture-address unit one pass per element (a wave's 64 dwords sit
// in up to 64 different sectors), which made the ragged last tile of a row as
// expensive as a full one.
// Two steps, so that the load can stay in flight: quad_raw_clamped issues it,
// quad_rearrange (when the data is needed) moves the elements.
template <typename T>
__device__ __forceinline__ Quad<T> quad_raw_clamped(const T* __restrict__ base, long off, int ph, int L)
{
    const int phc = ph < 0 ? 0 : (ph > L - 4 ? L - 4 : ph);
    return *reinterpret_cast<const Quad<T>*>(base + (off + (phc - ph)));
}
template <typename T>
__device__ __forceinline__ Quad<T> quad_rearrange(const Quad<T>& q, int ph, int L)
{
    const int phc = ph < 0 ? 0 : (ph > L - 4 ? L - 4 : ph);
    const int s = ph - phc;                       // wanted element e is loaded element e + s
    Quad<T> r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int k = e + s;
        T v = zero_elem<T>();
#pragma unroll
        for (int j = 0; j < 4; ++j) v = (k == j) ? q.v[j] : v;
        r.v[e] = v;
    }
    return r;
}
template <typename T>
__device__ __forceinline__ Quad<T> quad_raw_ragged(const T* __restrict__ base, long off, int ph, int L)
{
    const int phc = ph < 0 ? 0 : (ph > L - 4 ? L - 4 : ph);
    const Quad<T> q = *reinterpret_cast<const Quad<T>*>(base + (off + (phc - ph)));
    const int s = ph - phc;                       // wanted element e is loaded element e + s
    Quad<T> r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int k = e + s;
        T v = zero_elem<T>();
#pragma unroll
        for (int j = 0; j < 4; ++j) v = (k == j) ? q.v[j] : v;
        r.v[e] = v;
    }
    return r;
}

template <typename T>
__device__ __forceinline__ void quad_store(T* __restrict__ base, long off, bool fast,
                                           int ph, int L, const float in[4])
{
    if (fast) {
        Quad<T> q;
#pragma unroll
        for (int e = 0; e < 4; ++e) q.v[e] = from_f32<T>(in[e]);
        *reinterpret_cast<Quad<T>*>(base + off) = q;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (ph + e >= 0 && ph + e < L) base[off + e] = from_f32<T>(in[e]);
    }
}
// The same for a scan order (never fast then: the four tokens are not neighbours).
template <typename T>
__device__ __forceinline__ void quad_store(T* __restrict__ base, long off, bool fast,
                                           int ph, int L, const float in[4], const TokenOrder& ord)
{
    if (ord.kind == 0) { quad_store<T>(base, off, fast, ph, L, in); return; }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (ph + e >= 0 && ph + e < L) base[(off - ph) + ord(ph + e)] = from_f32<T>(in[e]);
}

}  // namespace lbscan
