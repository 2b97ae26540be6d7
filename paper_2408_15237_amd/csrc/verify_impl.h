// The fused multi-step verification kernel (Section 4.2 MultiStep, fused as in Section 4.3 of
// arXiv 2408.15237): replay of the pending tokens, snapshot h_j, k draft steps with outputs,
// snapshot h_k and the stash of this round's tokens, in one launch.
//
// Work decomposition (gfx950, wave64):
//   * A state row is the N fp32 values h[row][0..N).  LPR = min(16, N/4) lanes share a row, each
//     holding EPL = N/LPR values as V = EPL/4 float4 strips, so one global_load_dwordx4 of a wave
//     covers RPI = 64/LPR consecutive rows (N*4*RPI = 1 KiB contiguous at N = 64): every
//     state access is a full-width coalesced 16-byte access.
//   * A lane keeps R rows (interleaved: row = base + r*RPI + lane/LPR) in VGPRs for the whole
//     pend+k steps; the state is read once and written once per snapshot.
//   * A workgroup of `waves` waves owns rows_wg = waves*RPI*R rows of ONE (sequence, head)
//     (scalar-A mode) or of one sequence's channels (diagonal-A mode), so the replay trip count
//     pend[b] is uniform over the workgroup.
//   * The pend+k tokens' B, C, decay, dt*x and D*x are staged once in LDS as fp32.
//   * y_t[row] = sum_n C_t[n] h[row][n] is EPL FMAs in-lane, then a reduction over the LPR lanes
//     of the row with DPP row operations (no LDS, no atomics).
#pragma once

#include "ssmv_internal.h"

namespace ssmv {

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// sum over the LPR (<=16, power of two) adjacent lanes that share a row; every lane gets the total
template <int LPR>
__device__ __forceinline__ float row_sum(float v)
{
    if constexpr (LPR >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    if constexpr (LPR >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) v += dpp_move<0x141>(v);   // row_half_mirror
    if constexpr (LPR >= 16) v += dpp_move<0x140>(v);  // row_mirror
    return v;
}

// LDS plan (floats).  T = lds_tokens.
//   sB   [T][N]        B of every token (pending first, then drafts)
//   sC   [k][N]        C of the drafts
//   sDec [T]           scalar mode: exp(dt*A) per token
//   sDt  [T][rows_wg]  diag mode: dt per (token,row)
//   sDtx [T][rows_wg]  dt*x per (token,row)
//   sY   [k][rows_wg]  D*x per (draft,row), turned into y in place
template <bool DIAG>
__host__ __device__ inline size_t verify_lds_floats(int T, int k, int N, int rows_wg)
{
    size_t n = (size_t)T * N + (size_t)k * N + (size_t)T * rows_wg + (size_t)k * rows_wg;
    n += DIAG ? (size_t)T * rows_wg : (size_t)((T + 3) & ~3);
    return n;
}

template <int N, int R, bool DIAG>
__global__ __launch_bounds__(256) void verify_kernel(const VerifyParams p)
{
    constexpr int LPR = lanes_per_row(N);
    constexpr int EPL = N / LPR;
    constexpr int V = EPL / 4;
    constexpr int RPI = 64 / LPR;
    constexpr float LOG2E = 1.4426950408889634f;

    extern __shared__ float4 lds_raw[];
    float *lds = reinterpret_cast<float *>(lds_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int sub = lane % LPR;          // which strip of the row
    const int rsel = lane / LPR;         // which of the RPI rows of a load instruction
    const int rows_wg = p.rows_wg;
    const int k = p.k;
    const bool materialize = p.h_out != nullptr;

    // ---- which (sequence, head, tile) -------------------------------------------------------
    int b, hd, tile;
    {
        int w = blockIdx.x;
        tile = w % p.tiles;
        w /= p.tiles;
        if (DIAG) {
            b = w;
            hd = 0;
        } else {
            hd = w % p.H;
            b = w / p.H;
        }
    }
    const int rows_dom = DIAG ? p.H : p.P;              // rows of the tiled domain
    const int row0 = tile * rows_wg;                    // first row of this workgroup in the domain
    const size_t grow0 = DIAG ? (size_t)b * p.H : ((size_t)b * p.H + hd) * p.P;   // global row of domain row 0

    // bookkeeping written by the commit kernel; clamped so that a corrupted cache cannot index out of bounds
    const int cur = (int)((unsigned)p.cur_slot[b] % 3u);
    const int pd = min(max(p.pend[b], 0), p.kmax - 1);
    const int par = p.win_par[0] & 1;
    const int T = pd + k;

    // ---- issue the state loads first: they are the long-latency part ------------------------------
    float4 h[R][V];
    int lrow[R];                                        // row inside the workgroup
    bool rvalid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        lrow[r] = wave * (RPI * R) + r * RPI + rsel;
        rvalid[r] = (row0 + lrow[r]) < rows_dom;
        const float *src = p.state + (size_t)cur * p.slot_stride + (grow0 + row0 + lrow[r]) * N + sub * 4;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            h[r][v] = rvalid[r] ? *reinterpret_cast<const float4 *>(src + v * (LPR * 4)) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }

    // diag mode: the lane's A strips, pre-multiplied by log2(e) so the decay is one exp2
    float4 a2[DIAG ? R : 1][DIAG ? V : 1];
    if constexpr (DIAG) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                if (rvalid[r]) t = *reinterpret_cast<const float4 *>(p.A + (size_t)(row0 + lrow[r]) * N + v * (LPR * 4) + sub * 4);
                a2[r][v] = make_float4(t.x * LOG2E, t.y * LOG2E, t.z * LOG2E, t.w * LOG2E);
            }
    }

    // ---- stage the tokens in LDS --------------------------------------------------------------------
    const int TL = p.lds_tokens;
    float *sB = lds;
    float *sC = sB + (size_t)TL * N;
    float *sDec = sC + (size_t)k * N;                                  // scalar: [T]; diag: sDt [T][rows_wg]
    float *sDtx = sDec + (DIAG ? (size_t)TL * rows_wg : (size_t)((TL + 3) & ~3));
    float *sY = sDtx + (size_t)TL * rows_wg;

    const int HP = p.H * p.P;
    const int nthreads = blockDim.x;
    const int g = DIAG ? 0 : (int)(((long)hd * p.G) / p.H);
    const int heads_per_group = p.H / p.G;
    const bool first_tile = tile == 0;
    const bool writes_B = !materialize && first_tile && (DIAG || (hd % heads_per_group) == 0);
    const void *winB = p.win_B[par];
    void *winB_out = p.win_B[par ^ 1];
    const void *winX = p.win_xc[par];
    void *winX_out = p.win_xc[par ^ 1];
    const void *winDt = p.win_dt[par];
    void *winDt_out = p.win_dt[par ^ 1];

    for (int idx = tid; idx < T * N; idx += nthreads) {
        const int tt = idx / N, n = idx - tt * N;
        float v;
        if (tt < pd) {
            v = load_io(winB, (((size_t)b * p.kmax + tt) * p.G + g) * N + n, p.io);
        } else {
            const int t = tt - pd;
            v = load_io(p.Bm, (((size_t)b * k + t) * p.G + g) * N + n, p.io);
            if (writes_B) store_io(winB_out, (((size_t)b * p.kmax + t) * p.G + g) * N + n, v, p.io);
            sC[(size_t)t * N + n] = load_io(p.Cm, (((size_t)b * k + t) * p.G + g) * N + n, p.io);
        }
        sB[(size_t)tt * N + n] = v;
    }

    if constexpr (!DIAG) {
        const float A_h = p.A[hd];
        for (int tt = tid; tt < T; tt += nthreads) {
            float dtv;
            if (tt < pd) {
                dtv = load_io(winDt, ((size_t)b * p.kmax + tt) * p.H + hd, p.io);
            } else {
                dtv = load_io(p.dt, ((size_t)b * k + (tt - pd)) * p.H + hd, p.io);
                if (first_tile && !materialize) store_io(winDt_out, ((size_t)b * p.kmax + (tt - pd)) * p.H + hd, dtv, p.io);
            }
            sDec[tt] = expf(dtv * A_h);
        }
    }

    {
        const float D_h = DIAG ? 0.f : p.D[hd];
        for (int idx = tid; idx < T * rows_wg; idx += nthreads) {
            const int tt = idx / rows_wg, i = idx - tt * rows_wg;
            const int row = row0 + i;
            float xv = 0.f, dtv = 0.f, Dv = D_h;
            if (row < rows_dom) {
                const int ch = DIAG ? row : hd * p.P + row;            // conv channel == x channel
                const int dth = DIAG ? row : hd;
                if (tt < pd) {
                    xv = load_io(winX, ((size_t)b * p.kmax + tt) * HP + ch, p.io);
                    dtv = load_io(winDt, ((size_t)b * p.kmax + tt) * p.H + dth, p.io);
                } else {
                    const int t = tt - pd;
                    xv = load_io(p.xc, ((size_t)b * k + t) * HP + ch, p.io);
                    dtv = load_io(p.dt, ((size_t)b * k + t) * p.H + dth, p.io);
                    if (!materialize) {
                        store_io(winX_out, ((size_t)b * p.kmax + t) * HP + ch, xv, p.io);
                        if (DIAG) store_io(winDt_out, ((size_t)b * p.kmax + t) * p.H + dth, dtv, p.io);
                    }
                }
                if (DIAG) Dv = p.D[row];
            }
            sDtx[(size_t)tt * rows_wg + i] = dtv * xv;
            if (DIAG) sDec[(size_t)tt * rows_wg + i] = dtv;      // A carries the log2(e) factor
            if (tt >= pd) sY[(size_t)(tt - pd) * rows_wg + i] = Dv * xv;
        }
    }
    if (!materialize && first_tile && hd == 0 && tid == 0) p.last_k[b] = k;
    __syncthreads();

    // one recurrence step on the lane's strips: h <- decay*h + (dt*x) * B
    auto step = [&](int tt, float4 (&Bv)[V]) {
#pragma unroll
        for (int v = 0; v < V; ++v) Bv[v] = *reinterpret_cast<const float4 *>(sB + (size_t)tt * N + v * (LPR * 4) + sub * 4);
        float dec = 0.f;
        if constexpr (!DIAG) dec = sDec[tt];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float dtx = sDtx[(size_t)tt * rows_wg + lrow[r]];
            float dt2 = 0.f;
            if constexpr (DIAG) dt2 = sDec[(size_t)tt * rows_wg + lrow[r]];
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float4 d4;
                if constexpr (DIAG) {
                    d4.x = __builtin_amdgcn_exp2f(dt2 * a2[r][v].x);
                    d4.y = __builtin_amdgcn_exp2f(dt2 * a2[r][v].y);
                    d4.z = __builtin_amdgcn_exp2f(dt2 * a2[r][v].z);
                    d4.w = __builtin_amdgcn_exp2f(dt2 * a2[r][v].w);
                } else {
                    d4 = make_float4(dec, dec, dec, dec);
                }
                h[r][v].x = fmaf(d4.x, h[r][v].x, dtx * Bv[v].x);
                h[r][v].y = fmaf(d4.y, h[r][v].y, dtx * Bv[v].y);
                h[r][v].z = fmaf(d4.z, h[r][v].z, dtx * Bv[v].z);
                h[r][v].w = fmaf(d4.w, h[r][v].w, dtx * Bv[v].w);
            }
        }
    };

    auto store_state = [&](float *dst_base) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!rvalid[r]) continue;
            float *dst = dst_base + (grow0 + row0 + lrow[r]) * N + sub * 4;
#pragma unroll
            for (int v = 0; v < V; ++v) *reinterpret_cast<float4 *>(dst + v * (LPR * 4)) = h[r][v];
        }
    };

    // ---- (i) replay the pending tokens: no outputs ------------------------------------------------
    for (int s = 0; s < pd; ++s) {
        float4 Bv[V];
        step(s, Bv);
    }
    if (materialize) {
        store_state(p.h_out);
        return;
    }
    // ---- (ii) snapshot h_j --------------------------------------------------------------------------
    if (pd > 0) store_state(p.state + (size_t)((cur + 1) % 3) * p.slot_stride);

    // ---- (iii) the k draft tokens -------------------------------------------------------------------
    for (int t = 0; t < k; ++t) {
        float4 Bv[V];
        step(pd + t, Bv);
        float4 Cv[V];
#pragma unroll
        for (int v = 0; v < V; ++v) Cv[v] = *reinterpret_cast<const float4 *>(sC + (size_t)t * N + v * (LPR * 4) + sub * 4);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                acc = fmaf(Cv[v].x, h[r][v].x, acc);
                acc = fmaf(Cv[v].y, h[r][v].y, acc);
                acc = fmaf(Cv[v].z, h[r][v].z, acc);
                acc = fmaf(Cv[v].w, h[r][v].w, acc);
            }
            acc = row_sum<LPR>(acc);
            if (sub == 0) sY[(size_t)t * rows_wg + lrow[r]] += acc;
        }
    }
    // ---- (iv) snapshot h_k ---------------------------------------------------------------------------
    store_state(p.state + (size_t)((cur + 2) % 3) * p.slot_stride);

    __syncthreads();
    for (int idx = tid; idx < k * rows_wg; idx += nthreads) {
        const int t = idx / rows_wg, i = idx - t * rows_wg;
        const int row = row0 + i;
        if (row < rows_dom) {
            const int ch = DIAG ? row : hd * p.P + row;
            store_io(p.y, ((size_t)b * k + t) * HP + ch, sY[idx], p.io);
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------

template <int N, int R, bool DIAG>
static int launch_one(const VerifyParams &p, int waves, size_t lds_bytes, hipStream_t stream)
{
    const long groups = (long)p.batch * (DIAG ? 1 : p.H) * p.tiles;
    hipLaunchKernelGGL((verify_kernel<N, R, DIAG>), dim3((unsigned)groups), dim3(64 * waves), lds_bytes, stream, p);
    return (int)hipGetLastError();
}

template <int N, bool DIAG>
static int launch_n(const VerifyParams &p, VerifyShape s, size_t lds_bytes, hipStream_t stream)
{
    constexpr int V = (N / lanes_per_row(N)) / 4;
    constexpr int MAXRV = DIAG ? 4 : 8;      // registers: R*V float4 of state (+ as many of A in diag mode)
    switch (s.rows_per_lane) {
        case 1: return launch_one<N, 1, DIAG>(p, s.waves, lds_bytes, stream);
        case 2: if constexpr (2 * V <= MAXRV) return launch_one<N, 2, DIAG>(p, s.waves, lds_bytes, stream); break;
        case 4: if constexpr (4 * V <= MAXRV) return launch_one<N, 4, DIAG>(p, s.waves, lds_bytes, stream); break;
        case 8: if constexpr (8 * V <= MAXRV) return launch_one<N, 8, DIAG>(p, s.waves, lds_bytes, stream); break;
        default: break;
    }
    return (int)hipErrorInvalidConfiguration;
}

template <bool DIAG>
static int launch_verify_any(const VerifyParams &p, VerifyShape s, hipStream_t stream)
{
    const size_t lds_bytes = verify_lds_floats<DIAG>(p.lds_tokens, p.k, p.N, p.rows_wg) * sizeof(float);
    switch (p.N) {
        case 16: return launch_n<16, DIAG>(p, s, lds_bytes, stream);
        case 32: return launch_n<32, DIAG>(p, s, lds_bytes, stream);
        case 64: return launch_n<64, DIAG>(p, s, lds_bytes, stream);
        case 128: return launch_n<128, DIAG>(p, s, lds_bytes, stream);
        case 256: return launch_n<256, DIAG>(p, s, lds_bytes, stream);
        default: break;
    }
    return (int)hipErrorInvalidConfiguration;
}

}  // namespace ssmv
