// The fused multi-step verification kernel (Section 4.2 MultiStep, fused as in Section 4.3 of
// arXiv 2408.15237): replay of the pending tokens, snapshot h_j, k draft steps with outputs,
// snapshot h_k and the stash of this round's tokens, in one launch; optionally with the conv
// roll over the circular buffer (Section 4.3 footnote) folded into the token staging.
//
// Work decomposition (gfx950, wave64):
//   * A state row is the N fp32 values h[row][0..N).  LPR = min(16, N/4) lanes share a row, each
//     holding EPL = N/LPR values as V = EPL/4 float4 strips, so one global_load_dwordx4 of a wave
//     covers RPI = 64/LPR consecutive rows (N*4*RPI = 1 KiB contiguous at N = 64): every
//     state access is a full-width coalesced 16-byte access.
//   * A lane keeps R adjacent rows (row = base + (lane/LPR)*R + r) in VGPRs for the whole pend+k steps, so
//     one load instruction of a wave covers RPI pieces of N*4 contiguous bytes, R rows apart; the state
//     is read once and written once per snapshot.
//   * A workgroup of `waves` waves owns rows_wg = waves*RPI*R rows of ONE (sequence, head)
//     (scalar-A mode) or of one sequence's channels (diagonal-A mode), so the replay trip count
//     pend[b] is uniform over the workgroup.
//   * The kernel is latency-bound before it is bandwidth-bound (one verify moves a few tens of
//     MB), so the prologue is kept short: the state loads are issued first, from a uniform base
//     pointer plus 32-bit lane offsets; then every thread issues ALL its token loads (raw bits)
//     before the first wait, and decodes them into LDS afterwards.
//   * The pend+k tokens' B, C, decay, dt*x and D*x are staged once in LDS as fp32.
//   * y_t[row] = sum_n C_t[n] h[row][n] is EPL FMAs in-lane, then a reduction over the LPR lanes
//     of the row with DPP row operations; the row's first lane adds it to D*x in LDS with a
//     no-return LDS add, and the workgroup writes y with 16-byte stores at the end.
//   * The state is read and the snapshots are written with non-temporal accesses: each byte is touched
//     once per round and a decoder streams the model's weights through the caches before the next one.
//     (Mixing a temporal and a non-temporal access to one address under an `if` lets the optimiser merge
//     them and drop the hint - keep them unconditional.)
#pragma once

#include "ssmv_internal.h"

namespace ssmv {

typedef float v4f __attribute__((ext_vector_type(4)));

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

// the same for R independent values, stage by stage
template <int LPR, int R>
__device__ __forceinline__ void row_sum_all(float (&v)[R])
{
    if constexpr (LPR >= 2) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] += dpp_move<0xB1>(v[r]);
    }
    if constexpr (LPR >= 4) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] += dpp_move<0x4E>(v[r]);
    }
    if constexpr (LPR >= 8) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] += dpp_move<0x141>(v[r]);
    }
    if constexpr (LPR >= 16) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] += dpp_move<0x140>(v[r]);
    }
}

__host__ __device__ constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }

// LDS plan (floats).  T = lds_tokens.
//   sB   [T][N]        B of every token (pending first, then drafts)
//   sC   [k][N]        C of the drafts
//   sDec               scalar mode: dt per token [T]; diag mode: dt per (token,row) [T][rows_wg]
//   sDt  [T][rows_wg]  diag mode: dt per (token,row)
//   sDtx [T][rows_wg]  diag mode: dt*x per (token,row); scalar mode: x (dt is one number per token and is
//                      folded into B in the step instead, so the x items never wait for or touch dt)
//   sY   [k][rows_wg]  D*x per (draft,row), turned into y in place
//   sG   [k][rows_wg]  with a gate: z*sigmoid(z) per (draft,row)
template <bool DIAG>
__host__ __device__ inline size_t verify_lds_floats(int T, int k, int N, int rows_wg, bool gated)
{
    size_t n = (size_t)T * N + (size_t)k * N + (size_t)T * rows_wg + (size_t)k * rows_wg;
    n += DIAG ? (size_t)T * rows_wg : (size_t)((T + 3) & ~3);
    if (gated) n += (size_t)k * rows_wg;
    return n;
}

// At least 4 waves per SIMD (<= 128 VGPRs): a second generation of workgroups costs far more than a few moves.
// EXTRA: the optional pieces (step-size transform, gate, rounds fed by several calls) are compiled in; the plain
// verification launch carries none of their instructions.
template <int N, int R, bool DIAG, int IO, bool CONV, bool EXTRA>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void verify_kernel(const VerifyParams p)
{
    constexpr int LPR = lanes_per_row(N);
    constexpr int EPL = N / LPR;
    constexpr int V = EPL / 4;
    constexpr int RPI = 64 / LPR;
    constexpr int LOG2N = ilog2(N);
    constexpr float LOG2E = 1.4426950408889634f;
    using Vec = IoVec<IO>;
    constexpr int EV = Vec::EV;
    constexpr int VN = N / EV;                           // 16-byte vectors per token of B or C
    constexpr int LOG2VN = ilog2(VN);
    constexpr int W = SSMV_CONV_WIDTH;

    extern __shared__ float4 lds_raw[];
    float *lds = reinterpret_cast<float *>(lds_raw);

    const unsigned tid = threadIdx.x;
    const unsigned lane = tid & 63u;
    const unsigned wave = tid >> 6;
    const unsigned sub = lane % LPR;         // which strip of the row
    const unsigned rsel = lane / LPR;        // which of the RPI rows of a load instruction
    const int rows_wg = p.rows_wg;
    const int k = p.k;
    const bool materialize = p.h_out != nullptr;

    // ---- which (sequence, head, tile): all uniform ------------------------------------------------
    // grid = (tiles, heads, batch) in scalar mode, (tiles, batch) in diag mode: no integer division needed
    const int tile = blockIdx.x;
    const int hd = DIAG ? 0 : blockIdx.y;
    const int b = DIAG ? blockIdx.y : blockIdx.z;
    const int rows_dom = DIAG ? p.H : p.P;              // rows of the tiled domain
    const int row0 = tile * rows_wg;                    // first row of this workgroup in the domain
    const size_t grow = (DIAG ? (size_t)b * p.H : ((size_t)b * p.H + hd) * p.P) + row0;   // its global row

    // bookkeeping written by the commit kernel; clamped so that a corrupted cache cannot index out of bounds
    // tok0 > 0: a later call of a round that was begun by an earlier call (draft side, Section 4.3: the draft
    // model produces its tokens one call at a time).  It continues from the state the earlier call left in the
    // h_k slot, updates that slot in place (each workgroup has read its rows before it writes them), replays
    // nothing, and appends its tokens to the round's stash and conv ring behind the tok0 earlier ones.
    const int t0 = EXTRA ? p.tok0 : 0;
    const int cur = (int)((unsigned)p.cur_slot[b] % 3u);
    // branch-free on purpose (pend_mask = 0 and src_add = 2 for a later call, else ~0 and 0): a select here becomes a
    // branch around the load of pend[b], and that serialises two scalar-load round trips ahead of the state loads
    const int pd = min(max(p.pend[b], 0), p.pend_max) & (EXTRA ? p.pend_mask : ~0);
    const int src_slot = EXTRA ? (cur + p.src_add) % 3 : cur;
    const int par = p.win_par[0] & 1;
    // deferred advance: the window is a ring per sequence, token q of the sequence at entry q % 16, the first pending one
    // is token pos[b]; h_j is stored only when more than pend_hi tokens are pending (pend_hi = 0 otherwise)
    const int wp = (int)p.pos[b] & (SSMV_WINDOW - 1);
    const bool wring = p.win_ring != 0;
    auto slot_in = [&](int tt) { return wring ? (wp + tt) & (SSMV_WINDOW - 1) : tt; };               // pending token tt
    auto slot_out = [&](int t) { return wring ? (wp + pd + t) & (SSMV_WINDOW - 1) : t0 + t; };       // token t of this call

    // ---- state loads first: uniform base pointer + 32-bit lane offsets -------------------------------
    v4f h[R][V];
    v4f a2[DIAG ? R : 1][DIAG ? V : 1];                 // diag mode: A strips times log2(e): the decay is one exp2
    // a lane's R rows are adjacent (their per-row scalars are one LDS vector, their addresses one base register plus
    // immediates): row r is lrow0 + r inside the workgroup, its first strip at element loff0 + r*N, valid iff r < nvalid
    const unsigned lrow0 = wave * (RPI * R) + rsel * R;
    const unsigned loff0 = (lrow0 << LOG2N) + sub * 4;
    const int nvalid = rows_dom - (int)(row0 + lrow0);
    // element offset, inside a slot, of strip v of the lane's row r.  Row-major slots: the lane's rows are N apart.  Tiled
    // slots (scalar mode, state_off4): 16-byte pieces scattered over the tiles - this kernel then only serves the calls
    // the matrix-core kernel does not take (materialize, an explicitly chosen launch shape).
    const bool tiled = !DIAG && p.tiled;
    // uniform base of the workgroup inside a slot plus a 32-bit lane offset
    const size_t slot_base = tiled ? ((size_t)b * p.H + hd) * p.P * N : (grow << LOG2N);
    auto state_elem = [&](int r, int v) -> unsigned {
        if (tiled) return (unsigned)state_off4(true, (int)(row0 + lrow0) + r, (int)(sub * 4 + v * (LPR * 4)), N);
        return loff0 + r * N + v * (LPR * 4);
    };
    {
        const float *src = p.state + (size_t)src_slot * p.slot_stride + slot_base;
        const float *srcA = p.A + ((size_t)row0 << LOG2N);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int rr = r < nvalid ? r : -(int)lrow0;   // clamp to the workgroup's row 0: unconditional in-bounds load
#pragma unroll
            // streamed once per round: non-temporal, so that 100 MB per launch do not churn the caches
            for (int v = 0; v < V; ++v) h[r][v] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(src + state_elem(rr, v)));
            if constexpr (DIAG) {
                const unsigned o = r < nvalid ? loff0 + r * N : sub * 4;
#pragma unroll
                for (int v = 0; v < V; ++v) a2[r][v] = *reinterpret_cast<const v4f *>(srcA + o + v * (LPR * 4)) * LOG2E;
            }
        }
    }

    // (after the state loads have been issued: nothing they need depends on it)
    // ragged drafts: sequence b takes only the first k_seq[b] of the k tokens given (the arrays keep the stride k)
    int kb = k;
    if constexpr (EXTRA) if (p.k_seq) kb = min(max(p.k_seq[b], 1), k);
    const int T = pd + kb;

    // ---- LDS carve-up -------------------------------------------------------------------------------
    const int TL = p.lds_tokens;
    float *sB = lds;
    float *sC = sB + TL * N;
    float *sDec = sC + k * N;                                          // scalar: [T]; diag: sDt [T][rows_wg]
    float *sDtF = sDec;                                                // scalar: dt [T]
    float *sDtx = sDec + (DIAG ? TL * rows_wg : ((TL + 3) & ~3));
    float *sY = sDtx + TL * rows_wg;
    float *sG = sY + k * rows_wg;                                      // only with a gate

    // ---- token staging: uniform bases (element units of the I/O type), 32-bit offsets -----------------
    const int H = p.H, HP = p.H * p.P, GN = p.G * N;
    const int nthreads = blockDim.x;
    int g = 0;                                           // B/C group of this head
    bool first_head_of_group = true;
    if (!DIAG && p.G > 1) {
        const int hpg = p.H / p.G;
        g = hd / hpg;
        first_head_of_group = hd - g * hpg == 0;
    }
    const bool first_tile = tile == 0;
    const bool writes_B = !materialize && first_tile && first_head_of_group;
    const int ch0 = DIAG ? row0 : hd * p.P + row0;       // first x / conv channel of this workgroup
    const int dth0 = DIAG ? row0 : hd;                   // first dt entry of this workgroup
    const size_t tok_in = (size_t)b * k, tok_win = (size_t)b * p.win_tokens;   // first token row of this sequence
    // pending window (read: half `par`; written: the other half) and this round's inputs
    const void *winB = p.win_B[par];
    void *winB_out = p.win_B[par ^ 1];
    const void *winX = p.win_xc[par];
    void *winX_out = p.win_xc[par ^ 1];
    const void *winDt = p.win_dt[par];
    void *winDt_out = p.win_dt[par ^ 1];
    const size_t oB_win = tok_win * GN + (size_t)g * N, oB_in = tok_in * GN + (size_t)g * N;
    const size_t oX_win = tok_win * HP + ch0, oX_in = tok_in * HP + ch0;
    const size_t oDt_win = tok_win * H + dth0, oDt_in = tok_in * H + dth0;
    // Lane-varying strides are multiplied with the 24-bit multiplier (full rate; the 32-bit one runs at a quarter):
    // token indices are < 32 and the host refuses row lengths of 2^22 elements or more.
    auto m24 = [](int a, int b_) { return __mul24(a, b_); };
    const size_t ring_b = (size_t)b * p.ring_len * HP + ch0;            // this sequence's ring rows, this workgroup's channels
    const int ring_mask = p.ring_len - 1;
    // optional softplus(dt + dt_bias) ahead of the discretisation (Section 2.2: dt is the positive step)
    const float dtb_h = (EXTRA && !DIAG && p.dt_bias) ? p.dt_bias[hd] : 0.f;
    auto dt_fix = [&](float d, float bias) {
        if constexpr (EXTRA) {
            d += bias;
            if (p.dt_softplus) d = softplus_fast(d);
        }
        return d;
    };
    const bool gated = EXTRA && p.z != nullptr;
    auto silu = [&](float zv) { return silu_fast(zv); };
    auto dt_bias_of = [&](int row) { return (EXTRA && p.dt_bias) ? p.dt_bias[row] : 0.f; };   // diag mode: per channel
    const float D_h = DIAG ? 0.f : p.D[hd];
    const float A_h = DIAG ? 0.f : p.A[hd];
    // x (and dt) items: XW adjacent rows of one token.  Without the conv a 16-byte vector; with it only 4 bytes
    // (2 bf16 / 1 fp32), so that the conv arithmetic spreads over all lanes and waves instead of 64 lanes of
    // one wave (a workgroup's waves run on different SIMDs).  Odd shapes fall back to one element at a time.
    constexpr int XW = CONV ? (IO == SSMV_BF16 ? 2 : 1) : EV;
    using XV = XVec<IO, XW>;
    using XRawT = typename XV::Raw;
    const bool vec_rows = (rows_dom % XW) == 0 && (rows_wg % XW) == 0 && (DIAG || (p.P % XW) == 0);
    const int log2VR = p.log2_rows_wg - ilog2(XW);       // rows_wg is a power of two
    const int nXv = vec_rows ? (T << log2VR) : 0;        // x items to stage
    int conv_head = 0;
    if constexpr (CONV) conv_head = (p.conv_head[b] + t0) & (p.ring_len - 1);   // newest raw input fed so far

    struct BReq { int tt, n; bool on; };
    struct XReq { int tt, i; bool on, inb; };
    auto b_req = [&](int idx, int count) {
        BReq q;
        q.on = idx < count;
        const int c = q.on ? idx : 0;
        q.tt = c >> LOG2VN;
        q.n = (c & (VN - 1)) * EV;
        return q;
    };
    auto x_req = [&](int idx) {
        XReq q;
        q.on = idx < nXv;
        const int c = q.on ? idx : 0;
        q.tt = c >> log2VR;
        q.i = (c - (q.tt << log2VR)) * XW;
        q.inb = row0 + q.i < rows_dom;
        if (!q.inb) q.i = 0;                             // clamp: loads stay in bounds, results are not used
        return q;
    };
    // Loads return raw bits; decoding to fp32 happens in the *_use step, after everything is in flight.
    // Lanes with nothing to fetch issue no request.
    auto b_load = [&](const BReq &q) {                   // B of token tt (pending window or this round's input)
        uint4 r = make_uint4(0, 0, 0, 0);
        const bool old = q.tt < pd;
        if (q.on) r = Vec::load_raw(old ? winB : p.Bm, (old ? oB_win + m24(slot_in(q.tt), GN) : oB_in + m24(q.tt - pd, GN)) + q.n);
        return r;
    };
    auto c_load = [&](const BReq &q) {
        uint4 r = make_uint4(0, 0, 0, 0);
        if (q.on) r = Vec::load_raw(p.Cm, oB_in + m24(q.tt, GN) + q.n);
        return r;
    };
    // (scalar mode: the x items carry no dt - it is one number per token, handled by dec_load/dec_use below)
    struct XRaw { XRawT x, dt, bias, z; XRawT tap[CONV ? W - 1 : 1]; uint4 wv; };
    auto x_load = [&](const XReq &q) {
        XRaw r;
        r.x = XV::zero();
        r.dt = XV::zero();
        const bool old = q.tt < pd;
        const int t = q.tt - pd;
        if (!q.on) return r;                             // idle lane: no request at all
        // one x load whatever the source (window, conv output, or raw input = newest tap): x_raw and xc share
        // the [batch][k][channels] layout.  Two exclusive branches with a load each would share registers and
        // make the second wait for the first.
        const bool fresh = CONV && !old;
        r.x = XV::load(fresh ? p.x_raw : (old ? winX : p.xc), (old ? oX_win + m24(slot_in(q.tt), HP) : oX_in + m24(t, HP)) + q.i);
        if (fresh) {
            // older taps from earlier inputs of the round or the ring
#pragma unroll
            for (int w = 0; w < W - 1; ++w) {
                const int j = t - (W - 1) + w;           // position relative to the round's first token
                const bool from_ring = j < 0;
                r.tap[w] = XV::load(from_ring ? p.ring : p.x_raw,
                                    (from_ring ? ring_b + m24((conv_head + 1 + j) & ring_mask, HP) : oX_in + m24(j, HP)) + q.i);
            }
            r.wv = Vec::load_raw(p.wgt, (size_t)(ch0 + q.i) * W);           // XW channels x W taps = 16 bytes
            r.bias = p.bias ? XV::load(p.bias, ch0 + q.i) : XV::zero();
        }
        if constexpr (DIAG) r.dt = XV::load(old ? winDt : p.dt, (old ? oDt_win + m24(slot_in(q.tt), H) : oDt_in + m24(t, H)) + q.i);
        if (gated && !old) r.z = XV::load(p.z, oX_in + m24(t, HP) + q.i);
        return r;
    };
    auto b_use = [&](const BReq &q, uint4 raw) {
        if (!q.on) return;
        if (q.tt >= pd && writes_B) Vec::store_raw(winB_out, oB_win + m24(slot_out(q.tt - pd), GN) + q.n, raw);
        float v[EV];
        Vec::decode(raw, v);
#pragma unroll
        for (int e = 0; e < EV; ++e) sB[q.tt * N + q.n + e] = v[e];
    };
    auto c_use = [&](const BReq &q, uint4 raw) {
        if (!q.on) return;
        float v[EV];
        Vec::decode(raw, v);
#pragma unroll
        for (int e = 0; e < EV; ++e) sC[q.tt * N + q.n + e] = v[e];
    };
    auto x_use = [&](const XReq &q, const XRaw &r) {
        if (!q.on || !q.inb) return;                     // rows past the domain are never read back
        const int t = q.tt - pd;
        float xv[XW], dtv[XW], Dv[XW];
        XRawT xbits = r.x;
        XV::decode(r.x, xv);
        if (CONV && t >= 0) {
            // width-4 causal depthwise conv, fp32 accumulate in tap order, rounded to the I/O type
            float tap[W - 1][XW], wv[EV], bias[XW];
#pragma unroll
            for (int w = 0; w < W - 1; ++w) XV::decode(r.tap[w], tap[w]);
            Vec::decode(r.wv, wv);                       // wgt[channel c][tap] sits at [c*W + tap]
            XV::decode(r.bias, bias);
            XV::store(p.ring, ring_b + m24((conv_head + 1 + t) & ring_mask, HP) + q.i, r.x);
#pragma unroll
            for (int e = 0; e < XW; ++e) {
                float s = bias[e];
                s = fmaf(wv[e * W + 0], tap[0][e], s);
                s = fmaf(wv[e * W + 1], tap[1][e], s);
                s = fmaf(wv[e * W + 2], tap[2][e], s);
                s = fmaf(wv[e * W + 3], xv[e], s);
                if (p.conv_act == SSMV_ACT_SILU) s = s / (1.f + expf(-s));
                xv[e] = s;
            }
            xbits = XV::encode(xv);
            XV::decode(xbits, xv);                       // what is fed on is what is stored
        }
        if constexpr (DIAG) {
            XV::decode(r.dt, dtv);
#pragma unroll
            for (int e = 0; e < XW; ++e) dtv[e] = dt_fix(dtv[e], dt_bias_of(row0 + q.i + e));
        } else {
#pragma unroll
            for (int e = 0; e < XW; ++e) dtv[e] = 1.f;   // the step scales B by dt instead
        }
        if (gated && t >= 0) {
            float zv[XW];
            XV::decode(r.z, zv);
#pragma unroll
            for (int e = 0; e < XW; ++e) sG[(t << p.log2_rows_wg) + q.i + e] = silu(zv[e]);
        }
#pragma unroll
        for (int e = 0; e < XW; ++e) Dv[e] = DIAG ? p.D[row0 + q.i + e] : D_h;
        if (t >= 0 && !materialize) {
            XV::store(winX_out, oX_win + m24(slot_out(t), HP) + q.i, xbits);
            if (DIAG) XV::store(winDt_out, oDt_win + m24(slot_out(t), H) + q.i, r.dt);      // the raw dt: replay applies dt_fix again
        }
#pragma unroll
        for (int e = 0; e < XW; ++e) {
            sDtx[(q.tt << p.log2_rows_wg) + q.i + e] = dtv[e] * xv[e];
            if (DIAG) sDec[(q.tt << p.log2_rows_wg) + q.i + e] = dtv[e];             // A carries the log2(e) factor
            if (t >= 0) sY[(t << p.log2_rows_wg) + q.i + e] = Dv[e] * xv[e];
        }
    };
    auto dec_load = [&](int tt) {                        // scalar mode: dt of token tt for the decay factor
        const bool old = tt < pd || T == 0;
        return Vec::load_raw1(old ? winDt : p.dt, old ? oDt_win + m24(slot_in(tt), H) : oDt_in + m24(tt - pd, H));
    };
    auto dec_use = [&](int tt, uint32_t raw) {
        if (tt >= pd && first_tile && !materialize) Vec::store_raw1(winDt_out, oDt_win + m24(slot_out(tt - pd), H), raw);
        const float d = dt_fix(Vec::decode1(raw), dtb_h);
        sDtF[tt] = d;
    };

    // first pass: every thread issues its B, C, x (and dt) loads, then consumes them
    const int nB = T << LOG2VN, nC = kb << LOG2VN;
    const BReq qB = b_req(tid, nB), qC = b_req(tid, nC);
    const XReq qX = x_req(tid), qX2 = x_req(tid + nthreads);           // two x items per thread before any wait
    const uint4 fB = b_load(qB);
    const uint4 fC = c_load(qC);
    const XRaw fX = x_load(qX);
    const XRaw fX2 = x_load(qX2);
    const bool vec_y = (rows_dom % EV) == 0 && (rows_wg % EV) == 0 && (DIAG || (p.P % EV) == 0);
    const int log2VY = p.log2_rows_wg - ilog2(EV);
    uint32_t fDec = 0;
    if constexpr (!DIAG) fDec = dec_load((int)tid < T ? tid : 0);      // unconditional (idle lanes read token 0), like dt above
    __builtin_amdgcn_sched_barrier(0);
    b_use(qB, fB);
    c_use(qC, fC);
    x_use(qX, fX);
    x_use(qX2, fX2);
    if (!DIAG && (int)tid < T) dec_use(tid, fDec);
    // whatever one pass did not cover (large k, small workgroups)
    for (int idx = tid + nthreads; idx < nB; idx += nthreads) {
        const BReq q = b_req(idx, nB);
        b_use(q, b_load(q));
    }
    for (int idx = tid + nthreads; idx < nC; idx += nthreads) {
        const BReq q = b_req(idx, nC);
        c_use(q, c_load(q));
    }
    for (int idx = tid + 2 * nthreads; idx < nXv; idx += nthreads) {
        const XReq q = x_req(idx);
        x_use(q, x_load(q));
    }
    if constexpr (!DIAG) {
        for (int tt = tid + nthreads; tt < T; tt += nthreads) dec_use(tt, dec_load(tt));
    }
    if (!vec_rows) {
        // odd shapes: one (token,row) element at a time
        for (int idx = tid; idx < T * rows_wg; idx += nthreads) {
            const int tt = idx / rows_wg, i = idx - tt * rows_wg;
            const int t = tt - pd;
            float xv = 0.f, dtv = 0.f, Dv = D_h;
            if (row0 + i < rows_dom) {
                const size_t dti = DIAG ? i : 0;
                if (t < 0) {
                    xv = load_io(winX, oX_win + slot_in(tt) * HP + i, IO);
                    dtv = load_io(winDt, oDt_win + slot_in(tt) * H + dti, IO);
                } else {
                    if constexpr (CONV) {
                        float s = p.bias ? load_io(p.bias, ch0 + i, IO) : 0.f;
#pragma unroll
                        for (int w = 0; w < W; ++w) {
                            const int j = t - (W - 1) + w;
                            const size_t ring_row = (size_t)b * p.ring_len + ((conv_head + 1 + j) & (p.ring_len - 1));
                            const float tapv = j < 0 ? load_io(p.ring, ring_row * HP + ch0 + i, IO) : load_io(p.x_raw, oX_in + j * HP + i, IO);
                            s = fmaf(load_io(p.wgt, (size_t)(ch0 + i) * W + w, IO), tapv, s);
                            if (w == W - 1)
                                store_io(p.ring, ((size_t)b * p.ring_len + ((conv_head + 1 + t) & (p.ring_len - 1))) * HP + ch0 + i, tapv, IO);
                        }
                        if (p.conv_act == SSMV_ACT_SILU) s = s / (1.f + expf(-s));
                        xv = IO == SSMV_BF16 ? bf16_bits_to_f32(f32_to_bf16_bits(s)) : s;
                    } else {
                        xv = load_io(p.xc, oX_in + t * HP + i, IO);
                    }
                    dtv = load_io(p.dt, oDt_in + t * H + dti, IO);
                    if (!materialize) {
                        store_io(winX_out, oX_win + slot_out(t) * HP + i, xv, IO);
                        if (DIAG) store_io(winDt_out, oDt_win + slot_out(t) * H + dti, dtv, IO);
                    }
                }
                dtv = DIAG ? dt_fix(dtv, dt_bias_of(row0 + i)) : 1.f;
                if (DIAG) Dv = p.D[row0 + i];
                if (gated && t >= 0) sG[t * rows_wg + i] = silu(load_io(p.z, oX_in + t * HP + i, IO));
            }
            sDtx[tt * rows_wg + i] = dtv * xv;
            if (DIAG) sDec[tt * rows_wg + i] = dtv;                        // A carries the log2(e) factor
            if (t >= 0) sY[t * rows_wg + i] = Dv * xv;
        }
    }
    if (!materialize && first_tile && hd == 0 && tid == 0) p.last_k[b] = t0 + kb;
    __syncthreads();

    // the per-row values of the lane's R adjacent rows out of a [rows_wg] LDS array (16-byte reads where R allows)
    auto lane_rows = [&](const float *arr, float (&out)[R]) {
        if constexpr (R % 4 == 0) {
#pragma unroll
            for (int j = 0; j < R / 4; ++j) {
                const v4f t = *reinterpret_cast<const v4f *>(arr + lrow0 + 4 * j);
                out[4 * j] = t.x; out[4 * j + 1] = t.y; out[4 * j + 2] = t.z; out[4 * j + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) out[r] = arr[lrow0 + r];
        }
    };
    // one recurrence step on the lane's strips: h <- decay*h + (dt*x) * B
    auto step = [&](int tt) {
        v4f Bv[V];
#pragma unroll
        for (int v = 0; v < V; ++v) Bv[v] = *reinterpret_cast<const v4f *>(sB + tt * N + v * (LPR * 4) + sub * 4);
        float dec = 0.f;
        if constexpr (!DIAG) {
            dec = expf(sDtF[tt] * A_h);                  // only the rare plain step of scalar mode gets here
            const float dts = sDtF[tt];
#pragma unroll
            for (int v = 0; v < V; ++v) Bv[v] *= dts;
        }
        float xr[R], dr[DIAG ? R : 1];
        lane_rows(sDtx + tt * rows_wg, xr);
        if constexpr (DIAG) lane_rows(sDec + tt * rows_wg, dr);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float dtx = xr[r];
            float dt2 = 0.f;
            if constexpr (DIAG) dt2 = dr[r];
#pragma unroll
            for (int v = 0; v < V; ++v) {
                v4f d4;
                if constexpr (DIAG) {
                    d4.x = __builtin_amdgcn_exp2f(dt2 * a2[r][v].x);
                    d4.y = __builtin_amdgcn_exp2f(dt2 * a2[r][v].y);
                    d4.z = __builtin_amdgcn_exp2f(dt2 * a2[r][v].z);
                    d4.w = __builtin_amdgcn_exp2f(dt2 * a2[r][v].w);
                } else {
                    d4 = v4f{dec, dec, dec, dec};
                }
                // decay in place, then one fma: no temporaries (the other order keeps 4*R*V products alive)
                h[r][v] *= d4;
                h[r][v].x = fmaf(dtx, Bv[v].x, h[r][v].x);
                h[r][v].y = fmaf(dtx, Bv[v].y, h[r][v].y);
                h[r][v].z = fmaf(dtx, Bv[v].z, h[r][v].z);
                h[r][v].w = fmaf(dtx, Bv[v].w, h[r][v].w);
            }
        }
    };
    // Scaled form (scalar mode).  With alpha_t = exp(A * (dt_b + .. + dt_t)) accumulated from some base token b and
    // g_t = h_t / alpha_t, the recurrence of Section 2.1 becomes g_t = g_(t-1) + (dt_t / alpha_t) x_t (x) B_t: ONE
    // fma per state element and token instead of a multiply and an fma; y_t = alpha_t (C_t . g_t) and a snapshot is
    // alpha_t g_t.  alpha_t / alpha_s <= 1 for s <= t, so a rounding error made at token s only shrinks.  So that
    // 1/alpha cannot overflow, alpha is folded into the registers (and the base moved) before it would fall below
    // 2^-64, and a single token that decays by more than that takes the plain two-operation step.
    constexpr bool SC = !DIAG;
    float L2 = 0.f;                                     // log2 alpha of the last token taken (0 in diag mode)
    const float A2 = A_h * LOG2E;
    auto fold_scale = [&]() {
        const float al = __builtin_amdgcn_exp2f(L2);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v) h[r][v] *= al;
        L2 = 0.f;
    };
    auto advance = [&](int tt) {
        if constexpr (!SC) {
            step(tt);
        } else {
            const float dts = sDtF[tt];
            const float dl = dts * A2;
            if (!(fabsf(L2 + dl) <= 64.f)) {            // rare; also taken for a NaN
                fold_scale();
                if (!(fabsf(dl) <= 64.f)) {
                    step(tt);
                    return;
                }
            }
            L2 += dl;
            const float sc = dts * __builtin_amdgcn_exp2f(-L2);
            v4f Bv[V];
#pragma unroll
            for (int v = 0; v < V; ++v) Bv[v] = *reinterpret_cast<const v4f *>(sB + tt * N + v * (LPR * 4) + sub * 4) * sc;
            float xr[R];
            lane_rows(sDtx + tt * rows_wg, xr);
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    h[r][v].x = fmaf(xr[r], Bv[v].x, h[r][v].x);
                    h[r][v].y = fmaf(xr[r], Bv[v].y, h[r][v].y);
                    h[r][v].z = fmaf(xr[r], Bv[v].z, h[r][v].z);
                    h[r][v].w = fmaf(xr[r], Bv[v].w, h[r][v].w);
                }
            }
        }
    };
    auto store_state = [&](float *dst_base, bool slot_layout) {    // into a slot, or row-major into the caller's h_out
        float *dst = dst_base + (slot_layout ? slot_base : (grow << LOG2N));
        const float al = SC ? __builtin_amdgcn_exp2f(L2) : 1.f;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r >= nvalid) continue;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const unsigned o = slot_layout ? state_elem(r, v) : loff0 + r * N + v * (LPR * 4);
                __builtin_nontemporal_store(SC ? h[r][v] * al : h[r][v], reinterpret_cast<v4f *>(dst + o));
            }
        }
    };
    // (i) replay the pending tokens: no outputs
    for (int s_ = 0; s_ < pd; ++s_) advance(s_);
    if (materialize) {
        store_state(p.h_out, false);
        return;
    }
    // (ii) snapshot h_j
    if (pd > p.pend_hi) store_state(p.state + (size_t)((cur + 1) % 3) * p.slot_stride, true);
    // (iii) the k draft tokens
    for (int t = 0; t < kb; ++t) {
        advance(pd + t);
        const float al = SC ? __builtin_amdgcn_exp2f(L2) : 1.f;
        v4f Cv[V];
#pragma unroll
        for (int v = 0; v < V; ++v) Cv[v] = *reinterpret_cast<const v4f *>(sC + t * N + v * (LPR * 4) + sub * 4);
        float acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r] = 0.f;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                acc[r] = fmaf(Cv[v].x, h[r][v].x, acc[r]);
                acc[r] = fmaf(Cv[v].y, h[r][v].y, acc[r]);
                acc[r] = fmaf(Cv[v].z, h[r][v].z, acc[r]);
                acc[r] = fmaf(Cv[v].w, h[r][v].w, acc[r]);
            }
        }
        // the reduction over the row's lanes, one stage for all R rows at a time: a DPP operand must not have been
        // written by the instruction just before it, and R independent chains fill those slots
        row_sum_all<LPR, R>(acc);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if constexpr (SC) acc[r] *= al;
            // y = D*x + C.h : no-return LDS add by the row's first lane, nothing waits on it
            if (sub == 0) __hip_atomic_fetch_add(&sY[t * rows_wg + lrow0 + r], acc[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    // (iv) snapshot h_k (Algorithm 2), unless every accepted token is to stay pending
    if (p.write_hk) store_state(p.state + (size_t)((cur + 2) % 3) * p.slot_stride, true);

    __syncthreads();
    // y <- y * z * sigmoid(z) when a gate is given (the SiLU gate of a Mamba block), in fp32 before the rounding
    if (vec_y) {
        for (int idx = tid; idx < (k << log2VY); idx += nthreads) {
            const int t = idx >> log2VY, i = (idx - (t << log2VY)) * EV;
            if (row0 + i < rows_dom) {
                float yv[EV];
#pragma unroll
                for (int e = 0; e < EV; ++e) yv[e] = t < kb ? sY[t * rows_wg + i + e] : 0.f;    // tokens not taken: zeros
                if (gated && t < kb) {
#pragma unroll
                    for (int e = 0; e < EV; ++e) yv[e] *= sG[t * rows_wg + i + e];
                }
                Vec::store_raw(p.y, oX_in + m24(t, HP) + i, Vec::encode(yv));
            }
        }
    } else {
        for (int idx = tid; idx < k * rows_wg; idx += nthreads) {
            const int t = idx / rows_wg, i = idx - t * rows_wg;
            if (row0 + i < rows_dom) {
                float yv = t < kb ? sY[idx] : 0.f;
                if (gated && t < kb) yv *= sG[idx];
                store_io(p.y, oX_in + t * HP + i, yv, IO);
            }
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------

template <int N, int R, bool DIAG>
static int launch_io(const VerifyParams &p, int waves, size_t lds_bytes, hipStream_t stream)
{
    const dim3 grid = DIAG ? dim3(p.tiles, p.batch, 1) : dim3(p.tiles, p.H, p.batch);
    const dim3 block(64 * waves);
    const bool conv = p.x_raw != nullptr;
    const bool extra = p.tok0 > 0 || p.dt_softplus || p.dt_bias || p.z || p.k_seq;
    const int sel = (p.io == SSMV_BF16 ? 4 : 0) + (conv ? 2 : 0) + (extra ? 1 : 0);
    switch (sel) {
        case 0: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_F32, false, false>), grid, block, lds_bytes, stream, p); break;
        case 1: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_F32, false, true>), grid, block, lds_bytes, stream, p); break;
        case 2: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_F32, true, false>), grid, block, lds_bytes, stream, p); break;
        case 3: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_F32, true, true>), grid, block, lds_bytes, stream, p); break;
        case 4: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_BF16, false, false>), grid, block, lds_bytes, stream, p); break;
        case 5: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_BF16, false, true>), grid, block, lds_bytes, stream, p); break;
        case 6: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_BF16, true, false>), grid, block, lds_bytes, stream, p); break;
        default: hipLaunchKernelGGL((verify_kernel<N, R, DIAG, SSMV_BF16, true, true>), grid, block, lds_bytes, stream, p); break;
    }
    return (int)hipGetLastError();
}

template <int N, bool DIAG>
static int launch_n(const VerifyParams &p, VerifyShape s, size_t lds_bytes, hipStream_t stream)
{
    constexpr int V = (N / lanes_per_row(N)) / 4;
    constexpr int MAXRV = DIAG ? 4 : 8;      // registers: R*V float4 of state (+ as many of A in diag mode)
    switch (s.rows_per_lane) {
        case 1: return launch_io<N, 1, DIAG>(p, s.waves, lds_bytes, stream);
        case 2: if constexpr (2 * V <= MAXRV) return launch_io<N, 2, DIAG>(p, s.waves, lds_bytes, stream); break;
        case 4: if constexpr (4 * V <= MAXRV) return launch_io<N, 4, DIAG>(p, s.waves, lds_bytes, stream); break;
        case 8: if constexpr (8 * V <= MAXRV) return launch_io<N, 8, DIAG>(p, s.waves, lds_bytes, stream); break;
        default: break;
    }
    return (int)hipErrorInvalidConfiguration;
}

template <bool DIAG>
static int launch_verify_any(const VerifyParams &p, VerifyShape s, hipStream_t stream)
{
    const size_t lds_bytes = verify_lds_floats<DIAG>(p.lds_tokens, p.k, p.N, p.rows_wg, p.z != nullptr) * sizeof(float);
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
