// Forward kernel, "chunk per lane" mapping, for rows of about a thousand tokens and
// more when there are rows enough to give each a wave.
//
// One wave owns one (batch, channel) row; each lane owns kP = 16 consecutive tokens
// of a 1024-token chunk and keeps them in registers.  Per state n the lane scans
// its tokens from a zero state (Eq. 1, Sec. 3.1), the wave combines the lanes'
// results with a prefix scan of affine maps c -> P c + e (P: product of the lane's
// abar, e: the state it reaches from zero), every lane restarts from the state
// that enters its tokens, and the local backward recurrence of each window
// (Sec. 3.2, Eq. 7) runs on the same registers right after; Eq. 8, the skip term
// and the gate of Algorithm 1 follow.  The window length divides the lane's 16
// tokens, so no window leaves a lane.  This is the organisation the paper
// describes for its own kernel (Sec. 3.4: a tile of tokens per thread, partial
// results exchanged between threads, a second traversal), with the exchange done
// by DPP inside a wave and the state that leaves a chunk carried to the next
// through one LDS word per state.  Against the row-per-lane kernel it reads every tensor once
// and needs no summary pass for long rows, at the price of the second traversal
// and the prefix scan (about 2 more issue slots per state update) and of Bm / Cm
// reads per lane instead of per wave; it wins where rows are long and many
// (4096-token images), and loses where a row is much shorter than a chunk.
// REV scans the reversed sequence: logical token t is the stored token L-1-t.
//
// Bm[b,n,:] and Cm[b,n,:] of the chunk are shared by the kR rows (waves) of a
// block: they are staged once per state in LDS (double buffered, one barrier per
// state) in the layout the lanes read them back in.  Row tensors are loaded with
// coalesced quad loads and turned through a wave-private LDS buffer so that each
// lane ends up with its own 16 tokens; y goes back the same way.
#include <type_traits>

#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

constexpr int kP = 16;                 // tokens per lane
constexpr int kChunk = 64 * kP;        // tokens per wave and chunk
#ifndef LBSCAN_CHUNK_ROWS
#define LBSCAN_CHUNK_ROWS 4
#endif
#ifndef LBSCAN_CHUNK_MINBLOCKS
#define LBSCAN_CHUNK_MINBLOCKS 3
#endif
constexpr int kR = LBSCAN_CHUNK_ROWS;  // rows (waves) per block
constexpr int kPitch = kP + 4;         // LDS pitch of a lane's tokens (16-byte reads, see lbscan_bwd_rowlane.inc)
constexpr int kBuf = 64 * kPitch;      // floats of one staged chunk

__device__ __forceinline__ void lds_get4(const float* a, int o, float (&v)[4])
{
    const float4 q = *reinterpret_cast<const float4*>(a + o);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
}

__device__ __forceinline__ void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// v of the lane that the DPP control names; `old` in lanes that have no such lane or
// that the row mask leaves out.
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_or(float old, float v)
{
    return __uint_as_float(__builtin_amdgcn_update_dpp(__float_as_uint(old), __float_as_uint(v), CTRL, ROWS, 0xF, false));
}
// Inclusive prefix scan over the 64 lanes of the affine maps c -> P c + e (the map of
// the lane to the left is applied first): P <- P_left P, e <- P e_left + e.  Four
// steps inside rows of 16 lanes (row_shr), then the last lane of a row into the
// rows to its right (row_bcast).  The partner's value is read through DPP by the
// multiply itself; lanes without a partner, or outside the row mask, are not
// written and keep their value, which is what the scan wants.  The s_nop cover the
// two wait states a DPP read needs after a VALU write of the same register (the
// compiler does not look into the asm block).
__device__ __forceinline__ void wave_scan_affine(float& P, float& e)
{
#define LBSCAN_SCAN_STEP(ctrl) \
    "v_fmac_f32_dpp %0, %0, %1 " ctrl " bank_mask:0xf\n\t" \
    "v_mul_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"
    asm volatile(
        "s_nop 1\n\t"
        LBSCAN_SCAN_STEP("row_shr:1 row_mask:0xf") "s_nop 0\n\t"
        LBSCAN_SCAN_STEP("row_shr:2 row_mask:0xf") "s_nop 0\n\t"
        LBSCAN_SCAN_STEP("row_shr:4 row_mask:0xf") "s_nop 0\n\t"
        LBSCAN_SCAN_STEP("row_shr:8 row_mask:0xf") "s_nop 0\n\t"
        LBSCAN_SCAN_STEP("row_bcast:15 row_mask:0xa") "s_nop 0\n\t"
        LBSCAN_SCAN_STEP("row_bcast:31 row_mask:0xc")
        : "+v"(e), "+v"(P));
#undef LBSCAN_SCAN_STEP
}

// Quad q (tokens 4q .. 4q+3 of the chunk) lands where lane q / 4 reads its tokens from.
__device__ __forceinline__ int quad_slot(int q) { return (q >> 2) * kPitch + 4 * (q & 3); }

// Four quads of a row tensor of element type U, as loaded (lane l: quads l, l+64, ...).
template <typename U> struct RowQuads { Quad<U> q[4]; };

// TY: element type of y (the storage type, or float for the first pass of the two-pass
// global bi-directional scan, which leaves its ungated result in fp32).
template <typename T, int M, bool REV, typename TY>
__global__ void __launch_bounds__(64 * kR, LBSCAN_CHUNK_MINBLOCKS)
chunk_fwd_kernel(const FwdParams p)
{
    static_assert(kP % M == 0, "windows stay inside a lane's tokens");
    __shared__ __attribute__((aligned(16))) float sBC[2][2][kBuf];   // [buffer][Bm | Cm]
    __shared__ __attribute__((aligned(16))) float swave[kR][kBuf];   // per wave: turning row tensors
    __shared__ float scar[kR][16];          // per wave: state entering the chunk
    __shared__ float sA2[kR][16];           // per wave: A[d, :] log2(e) (read from LDS per state: a
                                            // global load in the state loop would make its wait
                                            // cover the Bm / Cm prefetch issued just before it)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = p.seqlen, D = p.dim, N = p.dstate;
    const int nbx = (D + kR - 1) / kR;
    const int b = blockIdx.x / nbx, d0 = (blockIdx.x % nbx) * kR;
    const int d = d0 + wv;
    const bool row_ok = d < D;                       // uniform per wave
    const int dc = row_ok ? d : D - 1;
    const long rowoff = ((long)b * D + dc) * L;
    const T* __restrict__ xg = static_cast<const T*>(p.x) + rowoff;
    const T* __restrict__ dg = static_cast<const T*>(p.delta) + rowoff;
    const T* __restrict__ zg = p.z ? static_cast<const T*>(p.z) + rowoff : nullptr;
    TY* __restrict__ yg = static_cast<TY*>(p.y) + rowoff;
    const float* __restrict__ yprevg = p.yprev ? p.yprev + rowoff : nullptr;   // added to y before the gate
    const T* __restrict__ Bg = static_cast<const T*>(p.Bm) + (long)b * N * L;
    const T* __restrict__ Cg = static_cast<const T*>(p.Cm) + (long)b * N * L;
    const float bias = p.bias ? p.bias[dc] : 0.0f;
    const float skip = p.Dskip ? p.Dskip[dc] : 0.0f;
    float* wbuf = swave[wv];

    if (lane < N) {
        scar[wv][lane] = (p.h0 && row_ok) ? p.h0[((long)b * D + d) * N + lane] : 0.0f;
        sA2[wv][lane] = p.A[(long)dc * N + lane] * kLog2e;
    }

    const int nchunks = (L + kChunk - 1) / kChunk;
    // Bm / Cm staging: the 256 quads of each are spread over the block's threads
    constexpr int kBCQ = 256 / (64 * kR) > 0 ? 256 / (64 * kR) : 1;   // quads per thread and tensor
    static_assert(64 * kR * kBCQ == 256, "one block stages a chunk of Bm and Cm");
    struct BCQuads { Quad<T> q[2][kBCQ]; };
    // (whether a chunk lies inside the row is decided once per chunk, for all lanes:
    // per-quad checks would put every load behind a branch of its own)
    auto chunk_is_whole = [&](int chunk) { return (chunk + 1) * kChunk <= L; };
    // The quad of logical tokens t0 .. t0+3 of a row tensor.  REV: logical token t is the
    // stored token L-1-t (the scan runs over the reversed sequence), i.e. the stored
    // quad that ends at L-t0, its elements in opposite order.
    auto fetch_quad = [&](const auto* src, int t0, bool whole) {
        using U = std::remove_cv_t<std::remove_pointer_t<decltype(src)>>;
        const int ph = REV ? L - 4 - t0 : t0;
        Quad<U> q;
        if (whole) q = quad_raw_fast<U>(src, ph);
        else q = quad_raw_checked<U>(src, ph, ph, L);
        if (REV) {
            const U a = q.v[0], b2 = q.v[1];
            q.v[0] = q.v[3]; q.v[1] = q.v[2]; q.v[2] = b2; q.v[3] = a;
        }
        return q;
    };
    auto load_bc = [&](int chunk, int n) {
        BCQuads r;
        const bool whole = chunk_is_whole(chunk);
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const T* src = (w ? Cg : Bg) + (long)n * L;
#pragma unroll
            for (int j = 0; j < kBCQ; ++j) {
                const int t0 = chunk * kChunk + 4 * (tid + 64 * kR * j);
                r.q[w][j] = fetch_quad(src, t0, whole);
            }
        }
        return r;
    };
    auto put_bc = [&](int buf, const BCQuads& r) {
#pragma unroll
        for (int w = 0; w < 2; ++w)
#pragma unroll
            for (int j = 0; j < kBCQ; ++j) {
                const Quad<T>& q = r.q[w][j];
                *reinterpret_cast<float4*>(&sBC[buf][w][quad_slot(tid + 64 * kR * j)]) =
                    make_float4(to_f32(q.v[0]), to_f32(q.v[1]), to_f32(q.v[2]), to_f32(q.v[3]));
            }
    };
    // one row tensor of the chunk: coalesced quads (issue_row), turned through the
    // wave's LDS buffer into this lane's 16 tokens (turn_row) when they are needed
    auto issue_row = [&](const auto* src, int chunk) {
        using U = std::remove_cv_t<std::remove_pointer_t<decltype(src)>>;
        RowQuads<U> r;
        const bool whole = chunk_is_whole(chunk);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t0 = chunk * kChunk + 4 * (lane + 64 * j);
            r.q[j] = fetch_quad(src, t0, whole);
        }
        return r;
    };
    auto turn_row = [&](const auto& r, float (&out)[kP]) {
        wave_sync_lds();                              // earlier readers of wbuf are done
#pragma unroll
        for (int j = 0; j < 4; ++j)
            *reinterpret_cast<float4*>(&wbuf[quad_slot(lane + 64 * j)]) =
                make_float4(to_f32(r.q[j].v[0]), to_f32(r.q[j].v[1]), to_f32(r.q[j].v[2]), to_f32(r.q[j].v[3]));
        wave_sync_lds();
#pragma unroll
        for (int g = 0; g < kP / 4; ++g) {
            float v[4];
            lds_get4(wbuf, lane * kPitch + 4 * g, v);
#pragma unroll
            for (int k = 0; k < 4; ++k) out[4 * g + k] = v[k];
        }
    };

    // first (chunk, state) staged before the loop
    put_bc(0, load_bc(0, 0));
    __syncthreads();

    // the time steps of a chunk are fetched during the last state of the chunk before
    // and its x while that chunk's result is stored; z during the chunk's own last state
    // (fp32 quads are twice the registers: there the time steps wait for the store phase too)
    constexpr bool kEarlyDt = sizeof(T) == 2;
    RowQuads<T> qd = issue_row(dg, 0), qx = issue_row(xg, 0), qz;
    for (int chunk = 0; chunk < nchunks; ++chunk) {
        const int t_lane = chunk * kChunk + lane * kP;          // this lane's first token
        float dt[kP], dx[kP], y[kP];
        {
            float xv[kP];
            turn_row(qd, dt);
#pragma unroll
            for (int k = 0; k < kP; ++k) dt[k] += bias;
            if (p.softplus) {
#pragma unroll
                for (int k = 0; k < kP; ++k) dt[k] = softplus_f32(dt[k]);
            }
            turn_row(qx, xv);
            // tokens past the end of the row: identity steps (abar = 1, u = 0)
            if (!chunk_is_whole(chunk)) {
#pragma unroll
                for (int k = 0; k < kP; ++k) { if (t_lane + k >= L) { dt[k] = 0.0f; xv[k] = 0.0f; } }
            }
#pragma unroll
            for (int k = 0; k < kP; ++k) { dx[k] = dt[k] * xv[k]; y[k] = skip * xv[k]; }
        }
        float dsum = 0.0f;                                       // sum of the lane's time steps
#pragma unroll
        for (int k = 0; k < kP; ++k) dsum += dt[k];

        // one state of the chunk; LAST: also fetch the row tensors needed next
        auto state_step = [&](int n, auto last_tag) {
            constexpr bool LAST = decltype(last_tag)::value;
            const int buf = (chunk * N + n) & 1;
            // the next (chunk, state) of Bm / Cm is fetched while this one is used
            const bool more = n + 1 < N || chunk + 1 < nchunks;
            BCQuads nxt;
            if (more) nxt = n + 1 < N ? load_bc(chunk, n + 1) : load_bc(chunk + 1, 0);
            if constexpr (LAST) {
                if (zg) qz = issue_row(zg, chunk);
                if constexpr (kEarlyDt) { if (chunk + 1 < nchunks) qd = issue_row(dg, chunk + 1); }
            }

            if (row_ok) {
                const float A2 = sA2[wv][n];                                     // uniform
                float a[kP], u[kP];
                // first traversal: the state the lane's tokens reach from zero
                float e = 0.0f;
#pragma unroll
                for (int g = 0; g < kP / 4; ++g) {
                    float Bv[4];
                    lds_get4(sBC[buf][0], lane * kPitch + 4 * g, Bv);
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        a[4 * g + k] = fast_exp2(dt[4 * g + k] * A2);
                        u[4 * g + k] = dx[4 * g + k] * Bv[k];
                        e = fmaf(a[4 * g + k], e, u[4 * g + k]);
                    }
                }
                float P = fast_exp2(dsum * A2);          // product of the lane's abar
                // inclusive prefix scan over the lanes of the affine maps c -> P c + e
                wave_scan_affine(P, e);
                // the state after each lane's tokens; shifted by one lane it is the state
                // entering the next lane's tokens; lane 63 holds the state leaving the chunk
                const float car = scar[wv][n];
                const float after = fmaf(P, car, e);
                float f = dpp_or<0x138, 0xF>(car, after);          // wave_shr:1, lane 0 keeps car
                if (lane == 63) scar[wv][n] = after;
                // second traversal, window by window: the forward states, then right to
                // left S = g + u of the step to the right and h = f + abar S (Eq. 7-8)
                constexpr int WG = M < 4 ? 4 : M;                  // tokens handled together
#pragma unroll
                for (int w0 = 0; w0 < kP; w0 += WG) {
                    float Cv[WG];
#pragma unroll
                    for (int g = 0; g < WG / 4; ++g) {
                        float c4[4];
                        lds_get4(sBC[buf][1], lane * kPitch + w0 + 4 * g, c4);
#pragma unroll
                        for (int k = 0; k < 4; ++k) Cv[4 * g + k] = c4[k];
                    }
#pragma unroll
                    for (int v0 = 0; v0 < WG; v0 += M) {
                        float ft[M];
#pragma unroll
                        for (int t = 0; t < M; ++t) {
                            f = fmaf(a[w0 + v0 + t], f, u[w0 + v0 + t]);
                            ft[t] = f;
                        }
                        const int tl = w0 + v0 + M - 1;             // the window's last token: g = 0
                        y[tl] = fmaf(Cv[v0 + M - 1], ft[M - 1], y[tl]);
                        float S = u[tl];
#pragma unroll
                        for (int t = M - 2; t >= 0; --t) {
                            const int tk = w0 + v0 + t;
                            const float h = fmaf(a[tk], S, ft[t]);
                            y[tk] = fmaf(Cv[v0 + t], h, y[tk]);
                            if (t > 0) S = fmaf(a[tk], S, u[tk]);
                        }
                    }
                }
            }
            if (more) put_bc(buf ^ 1, nxt);
            __syncthreads();
        };
#pragma unroll 1
        for (int n = 0; n < N - 1; ++n) state_step(n, std::false_type{});
        state_step(N - 1, std::true_type{});

        // the result of an earlier pass (two-pass scan), gate, store
        if (yprevg) {
            float pv[kP];
            turn_row(issue_row(yprevg, chunk), pv);
#pragma unroll
            for (int k = 0; k < kP; ++k) y[k] += pv[k];
        }
        if (zg) {
            float zv[kP];
            turn_row(qz, zv);
#pragma unroll
            for (int k = 0; k < kP; ++k) y[k] *= zv[k] * sigmoid_f32(zv[k]);
        }
        wave_sync_lds();
#pragma unroll
        for (int g = 0; g < kP / 4; ++g)
            *reinterpret_cast<float4*>(&wbuf[lane * kPitch + 4 * g]) =
                make_float4(y[4 * g], y[4 * g + 1], y[4 * g + 2], y[4 * g + 3]);
        wave_sync_lds();
        if (chunk + 1 < nchunks) {
            if constexpr (!kEarlyDt) qd = issue_row(dg, chunk + 1);
            qx = issue_row(xg, chunk + 1);
        }
        if (row_ok) {
            const bool whole = chunk_is_whole(chunk);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int q = lane + 64 * j;
                const int t0 = chunk * kChunk + 4 * q;
                float v[4];
                lds_get4(wbuf, quad_slot(q), v);
                if (REV) {
                    const float a = v[0], b2 = v[1];
                    v[0] = v[3]; v[1] = v[2]; v[2] = b2; v[3] = a;
                }
                const int ph = REV ? L - 4 - t0 : t0;
                quad_store<TY>(yg, ph, whole, ph, L, v);
            }
        }
    }
    if (p.hT && row_ok) {
        wave_sync_lds();
        if (lane < N) p.hT[((long)b * D + d) * N + lane] = scar[wv][lane];
    }
}

template <typename T>
hipError_t launch_chunk_t(const FwdParams& p, hipStream_t s)
{
    const long nblocks = (long)((p.dim + kR - 1) / kR) * p.batch;
    if (nblocks > 0x7fffffffL) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)nblocks), block(64 * kR);
#define LBSCAN_LAUNCH_CHUNK(M)                                                                 \
    if (p.reverse) hipLaunchKernelGGL((chunk_fwd_kernel<T, M, true, T>), grid, block, 0, s, p);   \
    else hipLaunchKernelGGL((chunk_fwd_kernel<T, M, false, T>), grid, block, 0, s, p)
    if (p.y_is_f32 && p.dtype != 0) {
        // fp32 result from bf16 inputs: the plain scan only (first pass of the two-pass scan)
        if (p.window != 1) return hipErrorInvalidValue;
        if (p.reverse) hipLaunchKernelGGL((chunk_fwd_kernel<T, 1, true, float>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((chunk_fwd_kernel<T, 1, false, float>), grid, block, 0, s, p);
        return hipGetLastError();
    }
    switch (p.window) {
        case 1:  LBSCAN_LAUNCH_CHUNK(1); break;
        case 2:  LBSCAN_LAUNCH_CHUNK(2); break;
        case 4:  LBSCAN_LAUNCH_CHUNK(4); break;
        case 8:  LBSCAN_LAUNCH_CHUNK(8); break;
        case 16: LBSCAN_LAUNCH_CHUNK(16); break;
        default: return hipErrorInvalidValue;
    }
#undef LBSCAN_LAUNCH_CHUNK
    return hipGetLastError();
}

}  // namespace

bool fwd_chunk_supported(const FwdParams& p)
{
    // stored order (either direction), rows that allow quad accesses, nothing that
    // only the row-per-lane kernels produce (checkpoints, first-pass partials)
    if (!window_supported(p.window) || p.order.kind != 0) return false;
    if (p.ckpt || p.summary_only || p.generic_window) return false;
    if (p.y_is_f32 && p.dtype != 0 && p.window != 1) return false;
    if (p.dtype != 0 && (p.seqlen & 1)) return false;
    return p.dstate >= 1 && p.dstate <= 16;
}

hipError_t launch_fwd_chunk(const FwdParams& p, hipStream_t stream)
{
    return p.dtype == 0 ? launch_chunk_t<float>(p, stream) : launch_chunk_t<bf16_t>(p, stream);
}

}  // namespace lbscan
