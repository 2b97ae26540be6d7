// The fused multi-step verification kernel (Section 4.2 MultiStep, fused as in Section 4.3 of arXiv 2408.15237) with its
// arithmetic on the matrix cores: scalar-A mode, bf16 tokens, fp32 state kept in 16x16 tiles (state_off4), at most 16 tokens
// (pending + drafts) per launch.
//
// Eq. 1 unrolled over the T = pend + k tokens of a launch, with cum_t = A * (dt_0 + .. + dt_t) (in log2 units) and h_0 the
// live state:
//   h_j  = 2^cum_(pend-1) h_0 + sum_{s <  pend} w^j_s x_s (x) B_s ,   w^j_s = dt_s 2^(cum_(pend-1) - cum_s)
//   h_k  = beta h_j           + sum_{s >= pend} w^k_s x_s (x) B_s ,   w^k_s = dt_s 2^(cum_(T-1) - cum_s),  beta = 2^(cum_(T-1) - cum_(pend-1))
//   y_t  = 2^cum_t C_t . h_0  + sum_{s <= t} M_ts x_s ,               M_ts = (C_t . B_s) dt_s 2^(cum_t - cum_s)  (+ D at s = t)
// Every exponent is <= 0, so nothing overflows however strong the decay.  The three sums and C . h_0 are products of 16 x 16
// tiles with a contraction over the tokens (padded to 16) or over n, on v_mfma_f32_16x16x32_bf16; x, B and C ARE bf16 and
// enter exactly; every fp32 operand (h_0, the weighted rows w_s B_s, M) enters as a bf16 head plus a bf16 tail
// (v = hi + lo + O(2^-17 |v|)), the two stacked along the 32-deep contraction of one instruction against the other operand
// repeated; accumulation is fp32, and the decay of the state itself (2^cum h_0, beta h_j) is an fp32 multiply.
//
// Layout (gfx950, wave64; lane l = 16 g + li):
//   * one workgroup of 4 waves owns 64 NT rows (channels) of ONE (sequence, head); wave w owns NT tiles of 16 rows.  A tile
//     of the state (16 rows x 16 n) is 1 KiB contiguous in memory and ONE 16-byte access per lane: lane l holds the floats
//     n = 16 q + 4 g .. + 3 of row li.  Those four registers are at once (a) the accumulator layout of U = (w B)^T X with rows
//     n and columns p, so the snapshots are produced in place and stored as they were loaded, and (b) after conversion, four
//     k-slots of the first operand of Y1^T = h_0 C^T (rows p, contraction over n).
//   * The tokens are fetched BEFORE the state, and turned into the LDS operands (the conv roll, the transposed and weighted B
//     rows, G = B C^T and M on the matrix core of wave 0) while the 33 MB of state of the launch are still under way: the wait
//     that staging needs covers the token loads only (loads return in order).  After the barrier a wave needs, per tile of
//     16 x 64 state values, 4 + 4 + 4 + 1 matrix instructions and about 100 vector instructions.
//   * x and the weighted B sit in LDS as [row][16 tokens] bf16 with rows padded to 48 bytes: the 16-byte operand reads of 8
//     lanes then fall into 8 different bank groups.
#include "ssmv_internal.h"

namespace ssmv {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf8 as_bf8(u4v v) { return __builtin_bit_cast(bf8, v); }
__device__ __forceinline__ v4f mfma16(bf8 a, bf8 b, v4f c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }

template <int CTRL>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// inclusive prefix sum over the 16 lanes of a row (row_shr 1, 2, 4, 8; lanes shifted in from outside read 0)
__device__ __forceinline__ float prefix16(float v)
{
    v += dpp_or_zero<0x111>(v);
    v += dpp_or_zero<0x112>(v);
    v += dpp_or_zero<0x114>(v);
    v += dpp_or_zero<0x118>(v);
    return v;
}
__device__ __forceinline__ float lane_get(float v, int lane)     // the value lane `lane` of this wave holds
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute(lane << 2, __float_as_int(v)));
}
__device__ __forceinline__ float uniform_lane(float v, int lane)  // the same for a wave-uniform lane number
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// two fp32 values -> packed bf16 heads and packed bf16 tails (first value in the low half)
__device__ __forceinline__ void split2(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = pack_bf16x2(a, b);
    lo = pack_bf16x2(a - bf16lo(hi), b - bf16hi(hi));
}

// Keeps the optimiser from moving the decode of a loaded value up to its load (where it would need a wait for every load
// issued before it): the value is opaque from here on.
__device__ __forceinline__ void pin(uint32_t &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin(u2v &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin(u4v &v) { asm volatile("" : "+v"(v)); }

#ifdef SSMV_TRACE
// Profiling builds only: 8 wall-clock stamps per workgroup (100 MHz), written by thread 0.
__device__ long long *trace_buf_ = nullptr;
#define SSMV_TP(i) do { if (trace_ && threadIdx.x == 0) trace_[i] = wall_clock64(); } while (0)
#else
#define SSMV_TP(i) do { } while (0)
#endif

template <int N, int NT, bool CONV, bool EXTRA>
// The seven pointers that the first scalar loads go through are kernel arguments of their own, ahead of the parameter
// block: this file is compiled with kernel-argument preload, which hands the first arguments to a wave in scalar registers
// when it starts, so those loads leave at once instead of behind a first round trip for the parameter block (where the
// firmware does not preload, the compiler's own prologue loads them, as before).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4)))
void verify_mfma_kernel(const int32_t *a_cur, const int32_t *a_pend, const int32_t *a_par, const int32_t *a_pos, const int32_t *a_head,
                        const float *a_A, const float *a_D, const VerifyParams p)
{
    constexpr int NQ = N / 16;                           // 16-wide tiles along n
    constexpr int NH = N / 32;                           // 32-deep steps of a contraction over n
    constexpr int RW = 64 * NT;                          // rows (channels) of the workgroup
    constexpr int XS = 20;                               // LDS row stride (bf16) of a [.][16 tokens] operand row: 40 bytes
    constexpr int CS = N + 8;                            // LDS row stride of a B or C row
    constexpr int XRS = RW + 8;                          // LDS row stride of a raw x row
    constexpr int CX = RW / 8, CB = N / 8;               // 16-byte pieces of an x row, of a B or C row
    constexpr int W = SSMV_CONV_WIDTH;
    constexpr int BT0 = 256 - 2 * N > 0 ? 256 - 2 * N : 0;   // first thread that builds the weighted B rows
    constexpr int XIT = (3 + 16 + 64 / CX - 1) / (64 / CX);  // load rounds of wave 0 over the raw x rows
    constexpr int BIT = (16 + 64 / CB - 1) / (64 / CB);      // load rounds of waves 1 and 2 over the B and C rows
    static_assert(W == 4, "the conv below is written for four taps");

    __shared__ __attribute__((aligned(16))) uint16_t sXr[19 * XRS];        // raw x: 3 rows of history, then row 3 + token
    __shared__ __attribute__((aligned(16))) uint16_t sBr[16 * CS];         // B       [token][n]
    __shared__ __attribute__((aligned(16))) uint16_t sC[16 * CS];          // C       [draft][n]
    __shared__ __attribute__((aligned(16))) uint16_t sWgt[RW * W];         // conv taps [row][4]
    __shared__ __attribute__((aligned(16))) uint16_t sBias[RW];
    __shared__ __attribute__((aligned(16))) uint16_t sX[RW * XS];          // x           [row][token]
    __shared__ __attribute__((aligned(16))) uint16_t sWj[2 * N * XS];      // w^j_s B_s   [head|tail][n][token]
    __shared__ __attribute__((aligned(16))) uint16_t sWk[2 * N * XS];      // w^k_s B_s
    __shared__ __attribute__((aligned(16))) uint16_t sM[2 * 16 * XS];      // M           [head|tail][draft][token]
    __shared__ uint16_t sDtRaw[16];                                        // dt of the launch's tokens, raw

    const unsigned tid = threadIdx.x, l = tid & 63u, w = __builtin_amdgcn_readfirstlane(tid >> 6), li = l & 15u, g = l >> 4;
    const int tile = blockIdx.x, hd = blockIdx.y, b = blockIdx.z;
#ifdef SSMV_TRACE
    long long *trace_ = trace_buf_ ? trace_buf_ + 8 * ((size_t)blockIdx.x + gridDim.x * (blockIdx.y + (size_t)gridDim.y * blockIdx.z)) : nullptr;
#endif
    SSMV_TP(0);
    const int k = p.k, H = p.H, P = p.P, HP = H * P, GN = p.G * N;

    // ---- bookkeeping written by the commit kernel (clamped: a corrupted cache cannot index out of bounds) ---------------
    // tok0 > 0: a later call of a round that an earlier call began (draft side, Section 4.3): continue from the h_k slot,
    // in place, replay nothing, append to the round's stash and ring behind the tok0 earlier tokens.
    const int t0 = EXTRA ? p.tok0 : 0;
    // every data-dependent scalar is requested here, ahead of the first use of any of them: scalar loads return out of
    // order, so the first use waits for all that have been issued - left to itself the compiler issues some of them behind
    // that wait, and each such level is one more round trip to memory at the head of the launch
    // (readfirstlane: free for a value that already sits in a scalar register, and it keeps the constraint below legal in
    // builds where a store ahead of these loads turns them into vector loads)
    auto uni = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    int cur_raw = uni(a_cur[b]), pd_raw = uni(a_pend[b]), par_raw = uni(a_par[0]);
    int pos_raw = uni(a_pos[2 * b]);                                      // the low half: only pos % 16 is needed
    int A_bits = uni(__float_as_int(a_A[hd])), D_bits = uni(__float_as_int(a_D[hd]));
    int ch_raw = 0, ks_raw = k, dtb_bits = 0;
    if constexpr (CONV) ch_raw = uni(a_head[b]);
    if constexpr (EXTRA) {
        if (p.k_seq) ks_raw = uni(p.k_seq[b]);
        if (p.dt_bias) dtb_bits = uni(__float_as_int(p.dt_bias[hd]));
    }
    asm volatile("" : "+s"(cur_raw), "+s"(pd_raw), "+s"(par_raw), "+s"(pos_raw), "+s"(A_bits), "+s"(D_bits), "+s"(ch_raw), "+s"(ks_raw), "+s"(dtb_bits));
    const float A_raw = __int_as_float(A_bits), D_h = __int_as_float(D_bits), dtb_h = __int_as_float(dtb_bits);
    const int cur = (int)((unsigned)cur_raw % 3u);
    const int pd = min(max(pd_raw, 0), p.pend_max) & (EXTRA ? p.pend_mask : ~0);
    const int src_slot = EXTRA ? (cur + p.src_add) % 3 : cur;
    const int par = par_raw & 1;
    // deferred advance: the window is a ring per sequence, token q of the sequence at entry q % 16, the first pending one
    // is token pos[b]; h_j is stored only when more than pend_hi tokens are pending (pend_hi = 0 otherwise)
    const int wp = pos_raw & (SSMV_WINDOW - 1);
    const bool adv = pd > p.pend_hi;
    const int kb = min(max(ks_raw, 1), k);
    // replayed round (Section 4.3, the draft model's recomputation): the pe tokens that earlier calls fed to this round are
    // taken again out of the round's own half of the window, behind the pending ones and ahead of this call's
    const int pe = EXTRA ? p.replay_tok : 0;
    const int pq = pd + pe;                              // tokens that come out of the stash
    const int T = pq + kb;                               // <= 16: the host launches this kernel only if pend_max + kmax <= 16
    const float A2 = A_raw * 1.4426950408889634f;
    const int conv_head = (ch_raw + t0) & (p.ring_len - 1);      // newest raw input fed so far

    int grp = 0;
    bool first_head_of_group = true;
    if (p.G > 1) {
        const int hpg = H / p.G;
        grp = hd / hpg;
        first_head_of_group = hd - grp * hpg == 0;
    }
    const bool first_tile = tile == 0;
    const bool writes_B = first_tile && first_head_of_group;
    const int ch0 = hd * P + tile * RW;                  // first channel of this workgroup
    const size_t tok_in = (size_t)b * k, tok_win = (size_t)b * p.win_tokens;
    // both halves of the window are kernel arguments; a select, not an indexed load that would wait for `par`
    auto half = [&](void *const (&w2)[2], int which) { return static_cast<uint16_t *>(which ? w2[1] : w2[0]); };
    const uint16_t *winB = half(p.win_B, par), *winX = half(p.win_xc, par), *winDt = half(p.win_dt, par);
    uint16_t *winB_out = half(p.win_B, par ^ 1), *winX_out = half(p.win_xc, par ^ 1), *winDt_out = half(p.win_dt, par ^ 1);
    // token tt < pd: pending, half `par`, entry tt; pd <= tt < pq: fed earlier to this round, the other half, entry tt - pd
    // (ring: both halves are the one ring, entry (wp + tt) % 16)
    auto stashed = [&](const uint16_t *cur_half, const uint16_t *round_half, size_t o_win, int tt, int stride) {
        const int e = p.win_ring ? (wp + tt) & (SSMV_WINDOW - 1) : (tt < pd ? tt : tt - pd);
        return (tt < pd ? cur_half : round_half) + o_win + (size_t)e * stride;
    };
    // window entry that token j of this call goes to
    auto out_entry = [&](int j) { return p.win_ring ? (wp + pq + j) & (SSMV_WINDOW - 1) : t0 + j; };
    const uint16_t *Bmp = static_cast<const uint16_t *>(p.Bm), *Cmp = static_cast<const uint16_t *>(p.Cm);
    const uint16_t *dtp = static_cast<const uint16_t *>(p.dt);
    const uint16_t *xin = static_cast<const uint16_t *>(CONV ? p.x_raw : p.xc);
    uint16_t *ring = static_cast<uint16_t *>(p.ring);
    const size_t oB_win = tok_win * GN + (size_t)grp * N, oB_in = tok_in * GN + (size_t)grp * N;
    const size_t oX_win = tok_win * HP + ch0, oX_in = tok_in * HP + ch0;
    const size_t oDt_win = tok_win * H + hd, oDt_in = tok_in * H + hd;
    const size_t ring_b = (size_t)b * p.ring_len * HP + ch0;
    const int ring_mask = p.ring_len - 1;

    // ---- token loads: whole rows in 16-byte pieces, a few instructions per wave, all issued before the state loads -------
    // wave 0: the raw x rows (history out of the ring, pending tokens out of the stash, this call's tokens); wave 1: the B
    // rows; wave 2: the C rows; wave 3: conv taps and bias, and dt of token li in lane li.
    // Loads are unconditional inside a role (rows past the last one read the last one again and are dropped at the use):
    // a load under a lane mask, or one merged with a constant, makes the compiler wait for it on the spot.
    u4v xk[XIT], bk[BIT], ck[3];                         // one set per role: no value is merged across the roles
    if (w == 0) {
        constexpr int RPI = 64 / CX;                     // rows per load instruction
        const int rfirst = CONV ? 0 : 3, nrow = 3 + T - rfirst;
#pragma unroll
        for (int it = 0; it < XIT; ++it) {
            if (it * RPI < nrow) {
                const int r = min(rfirst + it * RPI + (int)(l / CX), 2 + T);       // row of sXr
                const int tt = r - 3;
                const uint16_t *src = r < 3 ? ring + ring_b + (size_t)((conv_head - 2 + r) & ring_mask) * HP
                                     : tt < pq ? stashed(winX, winX_out, oX_win, tt, HP) : xin + oX_in + (size_t)(tt - pq) * HP;
                xk[it] = *reinterpret_cast<const u4v *>(src + 8 * (l % CX));
            }
        }
    } else if (w == 1 || w == 2) {
        constexpr int RPI = 64 / CB;
        const int nrow = w == 1 ? T : kb;
#pragma unroll
        for (int it = 0; it < BIT; ++it) {
            if (it * RPI < nrow) {
                const int r = min(it * RPI + (int)(l / CB), nrow - 1);
                const uint16_t *src = w == 2 ? Cmp + oB_in + (size_t)r * GN : r < pq ? stashed(winB, winB_out, oB_win, r, GN) : Bmp + oB_in + (size_t)(r - pq) * GN;
                bk[it] = *reinterpret_cast<const u4v *>(src + 8 * (l % CB));
            }
        }
    } else if (CONV) {
        // taps [row][4] bf16: RW/2 pieces; bias: RW/8 pieces (no bias: the taps are read once more and dropped)
        const u4v *wsrc = reinterpret_cast<const u4v *>(static_cast<const uint16_t *>(p.wgt) + (size_t)ch0 * W);
        ck[0] = wsrc[min(l, (unsigned)(RW / 2 - 1))];
        if constexpr (RW / 2 > 64) ck[1] = wsrc[64 + l];
        ck[2] = (p.bias ? reinterpret_cast<const u4v *>(static_cast<const uint16_t *>(p.bias) + ch0) : wsrc)[l % CX];
    }
    // dt of token li in lane li (lanes past the last token read the last one).  One wave fetches it for the workgroup (it
    // goes round through LDS with the rows): sixteen 2-byte reads out of sixteen cache lines per wave were half of the
    // line requests of the token phase when every wave made them
    uint32_t dt_raw = 0;
    if (w == 3) {
        const int tt = min((int)li, T - 1);
        dt_raw = tt < pq ? *stashed(winDt, winDt_out, oDt_win, tt, H) : (dtp + oDt_in)[(tt - pq) * H];
    }
    __builtin_amdgcn_sched_barrier(0);
    SSMV_TP(1);

    // ---- state loads: NT tiles of 16 rows per wave, NQ accesses of 1 KiB per tile (streamed once per round: non-temporal) ---
    v4f st[NT][NQ];
    const size_t head_base = ((size_t)b * H + hd) * P * N;
    const unsigned pt0 = tile * (RW / 16) + w * NT;     // this wave's first row tile inside the head
    const unsigned st_off = ((pt0 * NQ) << 8) + l * 4;  // its first access inside the head's block
    {
        const float *src = p.state + (size_t)src_slot * p.slot_stride + head_base + st_off;
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int q = 0; q < NQ; ++q) st[i][q] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(src + ((i * NQ + q) << 8)));
    }
    const bool gated = EXTRA && p.z != nullptr;
    u2v zraw[NT];
    if constexpr (EXTRA) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            zraw[i] = u2v{0u, 0u};
            if (gated && (int)li < kb)
                zraw[i] = *reinterpret_cast<const u2v *>(static_cast<const uint16_t *>(p.z) + oX_in + (size_t)li * HP + (w * NT + i) * 16 + 4 * g);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    SSMV_TP(2);

    // ---- the token rows into LDS as they are (the wait this needs covers the token loads only: loads return in order); the
    // ring append and the stash of B straight from the registers ---------------------------------------------------------
    pin(dt_raw);
    if (w == 0) {
        constexpr int RPI = 64 / CX;
        const int rfirst = CONV ? 0 : 3, nrow = 3 + T - rfirst;
#pragma unroll
        for (int it = 0; it < XIT; ++it) {
            if (it * RPI < nrow) {
                pin(xk[it]);
                const int r = rfirst + it * RPI + (int)(l / CX);
                const int j = r - 3 - pq;                // >= 0: a token of this call
                if (r < 3 + T) {
                    *reinterpret_cast<u4v *>(sXr + r * XRS + 8 * (l % CX)) = xk[it];
                    if (CONV && j >= 0)
                        *reinterpret_cast<u4v *>(ring + ring_b + (size_t)((conv_head + 1 + j) & ring_mask) * HP + 8 * (l % CX)) = xk[it];
                }
            }
        }
    } else if (w == 1 || w == 2) {
        constexpr int RPI = 64 / CB;
        const int nrow = w == 1 ? T : kb;
        uint16_t *dst = w == 1 ? sBr : sC;
#pragma unroll
        for (int it = 0; it < BIT; ++it) {
            if (it * RPI < nrow) {
                pin(bk[it]);
                const int r = it * RPI + (int)(l / CB);
                if (r < nrow) {
                    *reinterpret_cast<u4v *>(dst + r * CS + 8 * (l % CB)) = bk[it];
                    if (w == 1 && writes_B && r >= pq)
                        *reinterpret_cast<u4v *>(winB_out + oB_win + (size_t)out_entry(r - pq) * GN + 8 * (l % CB)) = bk[it];
                }
            }
        }
    } else if (CONV) {
        pin(ck[0]);
        if ((int)l < RW / 2) reinterpret_cast<u4v *>(sWgt)[l] = ck[0];
        if constexpr (RW / 2 > 64) {
            pin(ck[1]);
            reinterpret_cast<u4v *>(sWgt)[64 + l] = ck[1];
        }
        pin(ck[2]);
        if ((int)l < CX) reinterpret_cast<u4v *>(sBias)[l] = p.bias ? ck[2] : u4v{0u, 0u, 0u, 0u};
    }
    SSMV_TP(3);
    if (w == 3 && l < 16) sDtRaw[l] = (uint16_t)dt_raw;
    __syncthreads();
    dt_raw = sDtRaw[li];

    // ---- decay factors and weights: every wave, lane li = token li ---------------------------------------------------------
    float dtv = bf16lo(dt_raw);
    if constexpr (EXTRA) {                               // optional softplus(dt + dt_bias) ahead of the discretisation (Section 2.2)
        dtv += dtb_h;
        if (p.dt_softplus) dtv = softplus_fast(dtv);
    }
    if ((int)li >= T) dtv = 0.f;
    const float cum = prefix16(dtv * A2);                // log2 of the decay over tokens 0..li
    const float cumJ = pd > 0 ? uniform_lane(cum, pd - 1) : 0.f;
    const float cumK = uniform_lane(cum, T - 1);
    const float wj = (int)li < pd ? dtv * __builtin_amdgcn_exp2f(cumJ - cum) : 0.f;
    const float wk = ((int)li >= pd && (int)li < T) ? dtv * __builtin_amdgcn_exp2f(cumK - cum) : 0.f;
    const float alphaJ = __builtin_amdgcn_exp2f(cumJ), beta = __builtin_amdgcn_exp2f(cumK - cumJ);
    const float cy = lane_get(cum, min(pq + (int)li, 15));   // draft li is token pq + li
    const float alphaY = __builtin_amdgcn_exp2f(cy);
    if (w == 0 && first_tile) {
        if (g == 0 && (int)li >= pq && (int)li < T) winDt_out[oDt_win + (size_t)out_entry(li - pq) * H] = (uint16_t)dt_raw;   // the raw dt: replay transforms it again
        if (hd == 0 && tid == 0) p.last_k[b] = t0 + kb;
    }

    // ---- x: conv roll, stash, and the [row][token] operand.  An item is two adjacent channels x two adjacent token slots ----
    {
        constexpr int XI = RW * 4 / 256;                 // items per thread
        const uint32_t *sXr32 = reinterpret_cast<const uint32_t *>(sXr);
        uint32_t *sX32 = reinterpret_cast<uint32_t *>(sX);
#pragma unroll
        for (int it = 0; it < XI; ++it) {
            const unsigned idx = tid + 256 * it, cp = idx % (RW / 2), u = idx / (RW / 2);
            uint32_t outA = 0, outB = 0;                 // channel 2 cp and channel 2 cp + 1: slots 2 u, 2 u + 1
            if ((int)(2 * u) < T) {
                float wf[2][4], bias_f[2] = {0.f, 0.f};
                if constexpr (CONV) {
                    const u4v wv = reinterpret_cast<const u4v *>(sWgt)[cp];
                    wf[0][0] = bf16lo(wv.x); wf[0][1] = bf16hi(wv.x); wf[0][2] = bf16lo(wv.y); wf[0][3] = bf16hi(wv.y);
                    wf[1][0] = bf16lo(wv.z); wf[1][1] = bf16hi(wv.z); wf[1][2] = bf16lo(wv.w); wf[1][3] = bf16hi(wv.w);
                    const uint32_t bv = reinterpret_cast<const uint32_t *>(sBias)[cp];
                    bias_f[0] = bf16lo(bv); bias_f[1] = bf16hi(bv);
                }
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int tt = 2 * (int)u + e, j = tt - pq;
                    if (tt < T) {
                        uint32_t bits = sXr32[(3 + tt) * (XRS / 2) + cp];
                        if (CONV && j >= 0) {
                            // width-4 causal depthwise conv, fp32 accumulate in tap order, rounded to the I/O type; the
                            // three inputs before token j: earlier tokens of this call, else the ring's history rows
                            float s0 = bias_f[0], s1 = bias_f[1];
#pragma unroll
                            for (int i = 0; i < 3; ++i) {
                                const uint32_t tap = sXr32[(j + i < 3 ? j + i : tt + i) * (XRS / 2) + cp];
                                s0 = fmaf(wf[0][i], bf16lo(tap), s0);
                                s1 = fmaf(wf[1][i], bf16hi(tap), s1);
                            }
                            s0 = fmaf(wf[0][3], bf16lo(bits), s0);
                            s1 = fmaf(wf[1][3], bf16hi(bits), s1);
                            if (p.conv_act == SSMV_ACT_SILU) {
                                s0 = s0 / (1.f + expf(-s0));
                                s1 = s1 / (1.f + expf(-s1));
                            }
                            bits = pack_bf16x2(s0, s1);
                        }
                        if (j >= 0) reinterpret_cast<uint32_t *>(winX_out + oX_win + (size_t)out_entry(j) * HP)[cp] = bits;
                        outA |= (bits & 0xffffu) << (16 * e);
                        outB |= (bits >> 16) << (16 * e);
                    }
                }
            }
            sX32[(2 * cp) * (XS / 2) + u] = outA;
            sX32[(2 * cp + 1) * (XS / 2) + u] = outB;
        }
    }

    // ---- weighted, transposed B rows: head and tail, for the snapshot h_j (pending tokens) and for h_k (drafts).  Only if
    // this launch forms a snapshot for this sequence: with a deferred advance, and in a call of a replayed round that is not
    // its last, most launches form none ---------------------------------------------------------------------------------
    const bool forms_state = (!EXTRA || p.store_state) && (adv || p.write_hk);
    if (forms_state && (int)tid >= BT0) {
        const unsigned bi = tid - BT0, bn = bi % N;
        // the eight tokens of this thread's unit: the same for the whole wave when a wave covers one n range (N >= 64), and
        // then a weight comes out of its lane with a scalar read instead of a trip through the LDS crossbar
        const unsigned bt0 = N >= 64 ? 8 * __builtin_amdgcn_readfirstlane(bi / N) : 8 * (bi / N);
        auto weight = [&](float v, int lane) { return N >= 64 ? uniform_lane(v, lane) : lane_get(v, lane); };
        uint32_t hj[4], lj[4], hk[4], lk[4];
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            const int ta = bt0 + 2 * ii;
            // rows past the last token hold whatever LDS held: select, do not multiply
            const float b0 = ta < T ? bf16lo(sBr[ta * CS + bn]) : 0.f, b1 = ta + 1 < T ? bf16lo(sBr[(ta + 1) * CS + bn]) : 0.f;
            split2(weight(wk, ta) * b0, weight(wk, ta + 1) * b1, hk[ii], lk[ii]);
            split2(weight(wj, ta) * b0, weight(wj, ta + 1) * b1, hj[ii], lj[ii]);
        }
        u2v *dk = reinterpret_cast<u2v *>(sWk + bn * XS + bt0), *dkl = reinterpret_cast<u2v *>(sWk + (N + bn) * XS + bt0);
        dk[0] = u2v{hk[0], hk[1]}; dk[1] = u2v{hk[2], hk[3]};
        dkl[0] = u2v{lk[0], lk[1]}; dkl[1] = u2v{lk[2], lk[3]};
        if (pd > 0) {
            u2v *dj = reinterpret_cast<u2v *>(sWj + bn * XS + bt0), *djl = reinterpret_cast<u2v *>(sWj + (N + bn) * XS + bt0);
            dj[0] = u2v{hj[0], hj[1]}; dj[1] = u2v{hj[2], hj[3]};
            djl[0] = u2v{lj[0], lj[1]}; djl[1] = u2v{lj[2], lj[3]};
        }
    }

    // ---- wave 0: G^T = B C^T on the matrix core, M^T from it ---------------------------------------------------------------
    if (w == 0) {
        v4f G = {0.f, 0.f, 0.f, 0.f};                    // lane: draft t = li, tokens s = 4 g + r
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            u4v bs = *reinterpret_cast<const u4v *>(sBr + li * CS + 8 * g + 32 * h), cs_ = *reinterpret_cast<const u4v *>(sC + li * CS + 8 * g + 32 * h);
            if ((int)li >= T) bs = u4v{0u, 0u, 0u, 0u};
            if ((int)li >= kb) cs_ = u4v{0u, 0u, 0u, 0u};
            G = mfma16(as_bf8(bs), as_bf8(cs_), G);
        }
        const int tty = pq + (int)li;                    // draft li as a token of the launch
        float m[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int s = 4 * g + r;
            const float cs = lane_get(cum, s), ds = lane_get(dtv, s);
            float mv = G[r] * __builtin_amdgcn_exp2f(cy - cs) * ds;
            if (s == tty) mv += D_h;                     // the skip term D x_t
            m[r] = ((int)li < kb && s <= tty) ? mv : 0.f;
        }
        uint32_t h0, h1, l0, l1;
        split2(m[0], m[1], h0, l0);
        split2(m[2], m[3], h1, l1);
        *reinterpret_cast<u2v *>(sM + li * XS + 4 * g) = u2v{h0, h1};
        *reinterpret_cast<u2v *>(sM + (16 + li) * XS + 4 * g) = u2v{l0, l1};
    }
    __syncthreads();
    SSMV_TP(4);
    // Every wave of the workgroup has its whole share of the state before any of them starts to store: a wave that stores
    // its first tile while the loads of its second one (or of its neighbours) are still under way makes the launch 1-2 %
    // slower (measured; reads and writes mixed finely are served worse than a read phase followed by a write phase).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    SSMV_TP(5);
    __builtin_amdgcn_s_barrier();

    // ---- the products: the outputs of every tile of the wave, then h_j of every tile, then h_k of every tile.  The order of
    // the stores is worth 3 % of the launch: the outputs (32-byte pieces that the L2 puts together into lines) leave ahead of
    // the state stores, not between or behind them (small cached stores as the last thing a wave does cost a microsecond),
    // and a wave writes its 8 KB of one snapshot in one run instead of changing slots every 4 KB -----------------------------
    float *dstJ = p.state + (size_t)((cur + 1) % 3) * p.slot_stride + head_base + st_off;
    float *dstK = p.state + (size_t)((cur + 2) % 3) * p.slot_stride + head_base + st_off;
    uint16_t *yp = static_cast<uint16_t *>(p.y);
    // a [.][16 tokens] operand row: 16 bytes at an 8-byte aligned address
    auto row16 = [](const uint16_t *row) {
        const u2v a = reinterpret_cast<const u2v *>(row)[0], c = reinterpret_cast<const u2v *>(row)[1];
        return as_bf8(u4v{a.x, a.y, c.x, c.y});
    };
    bf8 Xop[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const unsigned ptl = w * NT + i;                 // row tile inside the workgroup
        Xop[i] = row16(sX + (ptl * 16 + li) * XS + 8 * (g & 1));
        // Y1^T = h_0 C^T : rows p, columns t, contraction over n; head and tail of h_0 stacked along the contraction
        v4f Y1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const v4f hv = st[i][q];
            uint32_t a0, a1, a2, a3;
            split2(hv.x, hv.y, a0, a2);
            split2(hv.z, hv.w, a1, a3);
            const u4v a = {a0, a1, a2, a3};
            const u2v c2 = *reinterpret_cast<const u2v *>(sC + li * CS + 16 * q + 4 * g);
            Y1 = mfma16(as_bf8(a), as_bf8(u4v{c2.x, c2.y, c2.x, c2.y}), Y1);
        }
        // Y2^T = X^T M^T : the drafts' outputs from the tokens of this launch (D x_t on the diagonal of M)
        const bf8 Mop = row16(sM + ((g >> 1) * 16 + li) * XS + 8 * (g & 1));
        const v4f Y2 = mfma16(Xop[i], Mop, v4f{0.f, 0.f, 0.f, 0.f});
        // lane: draft t = li, channels ptl*16 + 4 g .. + 3
        if ((int)li < k) {
            float yv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) yv[r] = (int)li < kb ? fmaf(Y1[r], alphaY, Y2[r]) : 0.f;    // tokens not taken: zeros
            if constexpr (EXTRA) {
                if (gated) {                             // y <- y * z * sigmoid(z), in fp32 before the rounding
                    yv[0] *= silu_fast(bf16lo(zraw[i].x)); yv[1] *= silu_fast(bf16hi(zraw[i].x));
                    yv[2] *= silu_fast(bf16lo(zraw[i].y)); yv[3] *= silu_fast(bf16hi(zraw[i].y));
                }
            }
            *reinterpret_cast<u2v *>(yp + oX_in + (size_t)li * HP + ptl * 16 + 4 * g) = u2v{pack_bf16x2(yv[0], yv[1]), pack_bf16x2(yv[2], yv[3])};
        }
    }
    // (a call of a replayed round that is not its last needs the outputs only: no snapshot is formed)
    if (forms_state) {
        // (i) + (ii): fold the pending tokens in and store the snapshot h_j (a deferred advance stores it only when the
        // window is about to fill up; until then it is needed, unstored, as the start of h_k or not at all)
        if (adv || (pd > 0 && p.write_hk)) {
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const bf8 Aw = row16(sWj + ((g >> 1) * N + 16 * q + li) * XS + 8 * (g & 1));
                    st[i][q] = mfma16(Aw, Xop[i], st[i][q] * alphaJ);
                    if (adv) __builtin_nontemporal_store(st[i][q], reinterpret_cast<v4f *>(dstJ + ((i * NQ + q) << 8)));
                }
        }
        // (iii) + (iv): the drafts, and the snapshot h_k (Algorithm 2), unless every accepted token is to stay pending
        if (p.write_hk) {
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const bf8 Aw = row16(sWk + ((g >> 1) * N + 16 * q + li) * XS + 8 * (g & 1));
                    st[i][q] = mfma16(Aw, Xop[i], st[i][q] * beta);
                    __builtin_nontemporal_store(st[i][q], reinterpret_cast<v4f *>(dstK + ((i * NQ + q) << 8)));
                }
        }
    }
    SSMV_TP(6);
#ifdef SSMV_TRACE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's stores have been acknowledged
    SSMV_TP(7);
#endif
}

template <int N, int NT, bool CONV, bool EXTRA>
void launch_one(const VerifyParams &p, hipStream_t stream)
{
    const dim3 grid(p.P / (64 * NT), p.H, p.batch), block(256);
    // the pointers of the first scalar loads ahead of the parameter block (kernel-argument preload)
    hipLaunchKernelGGL((verify_mfma_kernel<N, NT, CONV, EXTRA>), grid, block, 0, stream, p.cur_slot, p.pend, p.win_par,
                       reinterpret_cast<const int32_t *>(p.pos), p.conv_head, p.A, p.D, p);
}

template <int N, int NT>
int launch_shape(const VerifyParams &p, hipStream_t stream)
{
    const bool conv = p.x_raw != nullptr;
    const bool extra = p.tok0 > 0 || p.dt_softplus || p.dt_bias || p.z || p.k_seq || !p.store_state;
    if (conv) {
        if (extra) launch_one<N, NT, true, true>(p, stream);
        else launch_one<N, NT, true, false>(p, stream);
    } else {
        if (extra) launch_one<N, NT, false, true>(p, stream);
        else launch_one<N, NT, false, false>(p, stream);
    }
    return (int)hipGetLastError();
}

}  // namespace

#ifdef SSMV_TRACE
int set_trace_mfma(long long *buf) { return (int)hipMemcpyToSymbol(HIP_SYMBOL(trace_buf_), &buf, sizeof(buf)); }
#endif

bool verify_mfma_supported(int N, int P) { return (N == 32 || N == 64 || N == 128) && P >= 64 && P % 64 == 0; }

int launch_verify_mfma(const VerifyParams &p, hipStream_t stream)
{
    if (!verify_mfma_supported(p.N, p.P) || p.io != SSMV_BF16 || !p.tiled || p.h_out || p.lds_tokens > 16)
        return (int)hipErrorInvalidConfiguration;
    // two row tiles per wave while that still leaves four workgroups per compute unit, else one
    const bool two = p.N <= 64 && p.P % 128 == 0 && (long)p.batch * p.H * (p.P / 128) >= 1024;
    switch (p.N) {
        case 32: return two ? launch_shape<32, 2>(p, stream) : launch_shape<32, 1>(p, stream);
        case 64: return two ? launch_shape<64, 2>(p, stream) : launch_shape<64, 1>(p, stream);
        default: return launch_shape<128, 1>(p, stream);
    }
}

}  // namespace ssmv
