// Chunked prefill for bf16 tensors on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, 16 times the fp32 MFMA rate).
// Same evaluation of Section 2.1 Eq. 1 (discretisation of Section 2.2) as prefill.hip, chunk by chunk:
//   G = C B^T,  M_ts = G_ts exp(cum_t - cum_s) dt_s (s <= t) + [s = t] D,
//   Y = M X + diag(exp(cum_t)) C h^T,   h <- exp(cum_Q) h + X^T diag(w) B,   w_s = exp(cum_Q - cum_s) dt_s,
// with the operands arranged so that fp32 accuracy survives the 8-bit mantissa of the multiplier inputs:
//   * B, C and the conv output X ARE bf16 (the tensors' storage type; the conv output is rounded to it by
//     definition), so they enter exactly;
//   * the fp32 operand of the product that UPDATES THE STATE (the weighted rows w_s B_s) is split into a bf16 head and a
//     bf16 tail, v = hi + lo + O(2^-17 |v|), and contributes two products into the same fp32 accumulator: the state
//     carries over the whole prompt and stays at fp32 accuracy;
//   * the fp32 operands of the two products that end in OUTPUTS only (the state h in h C^T, the masked matrix M in M X)
//     enter as their bf16 head alone: a relative 2^-9 per term, the size of the rounding the outputs get anyway when
//     they are stored as bf16, and nothing of it feeds back into the state.  (Their tails cost a fifth of the kernel's
//     vector and matrix instructions: 0.41 -> 0.36 ms for 32 x 2048 tokens of a 32 x 128 x 64 layer; the largest output
//     error against the fp64 scan went from 0.0058 to 0.0075 of the largest output.)
// One workgroup owns one (sequence, head); wave w owns the 32 channels [32 w, 32 w + 32).  The state lives in the
// accumulator registers for the whole prompt, TRANSPOSED (tile rows = state index n, columns = channel p): in that
// shape the registers of a lane (its channel, 16 of the 32 n of a tile) are directly the k-slots of the A operand of
// h C^T, so the state never visits LDS; the result tile comes out as [channel][token], a lane holding runs of four
// adjacent channels of its token (the wave turns the tile through a patch of LDS of its own into 64-byte rows for the
// stores).  G^T (32 x 32) is computed by every wave (four products, the matrix pipe has slack); each wave finishes a
// quarter of its registers into M^T (mask, decay, dt_s, D on the diagonal, head and tail) and shares it through LDS.
// Operand layout (checked on the hardware): A[i = lane%32][k = 8 (lane/32) + j], B[k = 8 (lane/32) + j][col = lane%32],
// j = 0..7 the elements of the lane's 16-byte operand; result register v of a lane is row 8 (v/4) + 4 (lane/32) + v%4,
// column lane%32.  Registers 8 st .. 8 st + 7 of a result tile, used as the operand of step st of a following
// product, are therefore rows 16 st + 8 (j/4) + 4 (lane/32) + j%4.  Rows of the state tiles (the index n) are stored
// under the permutation "swap bits 2 and 3" of the row index: then those eight registers hold the CONSECUTIVE indices
// 16 st + 8 (lane/32) + j, and the other operand of h C^T is one 16-byte LDS read, the same read that G^T needs
// anyway; likewise X serves M X and the update with one read.
// The chunk's raw x, B and C rows travel from global memory straight into LDS (no registers, 1 KB per wave and
// instruction), one chunk ahead: they are requested right after the barrier that ends the staging of chunk c, land
// during its arithmetic, and the barrier at its end publishes them.
// LDS rows that the kernel writes itself are padded by 16 bytes: a row stride that is an odd multiple of 16 bytes
// spreads 16-byte reads of consecutive rows over all banks; the rows of B and C, which the direct loads fill without
// gaps, have their 16-byte pieces XOR-swizzled instead (by the choice of the global address each lane fetches).
#include "ssmv_internal.h"

namespace ssmv {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kQ = 32;      // tokens per chunk
constexpr float kLog2e = 1.4426950408889634f;

// waves per 32-channel tile: a large state under a narrow head is split over n
__host__ __device__ constexpr int prefill_nsplit(int P, int N) { return (N >= 128 && P <= 64) ? 2 : 1; }

template <int P, int N>
struct PfLds {              // byte offsets of the LDS arrays (bf16 unless said)
    static constexpr int XS = kQ * 2 + 16;                 // row stride of the arrays indexed [..][token]
    static constexpr int NP = P / 32;                      // 32-channel tiles of the head
    static constexpr int NSPL = prefill_nsplit(P, N);
    static constexpr int NW = NP * NSPL;                   // waves
    static constexpr int oX = 0;                           // [P][Q]  conv output x_s
    static constexpr int oBh = oX + P * XS;                // [N][Q]  head of w_s B_s, transposed
    static constexpr int oBl = oBh + N * XS;               // [N][Q]  tail of w_s B_s, transposed
    static constexpr int oMh = oBl + N * XS;               // [Q][Q]  M^T, rows t (rounded to bf16: it only feeds outputs)
    static constexpr int YS = 32 * 2 + 16;                 // row stride of a wave's output tile [token][32 channels]
    static constexpr int oY = oMh + kQ * XS;               // [NP][Q][32]  the output tiles, for stores of whole 64-byte rows
    // filled by loads that go from global memory straight into LDS (1 KB per wave and instruction, lane l at byte 16 l):
    static constexpr int oZ = oY + NP * kQ * YS;           // fp32 [NP][16][64]  h C^T over the second half of n, for the tile's first wave
    static constexpr int oXraw = oZ + (NSPL - 1) * NP * 4096;        // [Q][P]  raw conv inputs of the chunk, rows of 2 P bytes
    static constexpr int BCS = kQ * N * 2;                 // one copy of B or C: [Q][N], rows of 2 N bytes, 16-byte pieces swizzled
    // Two copies of B and C (chunks alternate; the next chunk's are requested at the start of this one's arithmetic) where
    // that does not cost a workgroup per CU; else one copy, and the next chunk's B and C are requested only once this
    // chunk's have been read (after the barrier in the middle): narrow heads (few waves per workgroup: 48 KB -> 40 KB
    // is a fourth workgroup per CU) and N = 128 (90 KB -> 74 KB is a second one).
    static constexpr int BCC = (P >= 128 && N < 128) ? 2 : 1;
    static constexpr int oB = oXraw + kQ * P * 2;
    static constexpr int oC = oB + BCC * BCS;
    static constexpr int oCar = oC + BCC * BCS;              // fp32 [2][3][P]  the last three raw inputs of a chunk, for the next one's conv
    static constexpr int oCum = oCar + 2 * 3 * P * 4;      // fp32 [NW][Q]  log2 e times the inclusive prefix of dt*A (a copy per wave)
    static constexpr int oDt = oCum + NW * kQ * 4;         // fp32 [NW][Q]  dt
    static constexpr int oW = oDt + NW * kQ * 4;           // fp32 [NW][Q]  exp(cum_Q - cum_s) dt_s
    static constexpr int total = oW + NW * kQ * 4;
    // Rows of B and C are 2 N bytes with no padding (the direct loads fill LDS contiguously), so the 16-byte pieces of row r
    // sit at piece index (logical index ^ swz(r)): 16 consecutive rows then spread a 16-byte column read over all banks.
    static constexpr int PIECES = N / 8;
    static __host__ __device__ constexpr int swz(int r) { return PIECES == 16 ? (r & 15) : PIECES == 8 ? ((r ^ (r >> 3)) & 7) : ((r >> 2) & 3); }
};

typedef __attribute__((address_space(3))) char lds_char_t;

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at LDS address `dst` + 16 l (dst is the
// same in all lanes and travels in M0).  Issued from assembly, so that the compiler does not count these loads: it would
// otherwise wait for them before the next LDS read that it cannot prove to be disjoint from their target, and at every
// workgroup barrier.  The kernel waits for them itself (wait_direct_loads) ahead of the barrier that publishes the data.
__device__ __forceinline__ void load_to_lds16(const void *src, const char *dst)
{
    const unsigned lds_addr = (unsigned)(size_t)(lds_char_t *)dst;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void wait_direct_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// two fp32 values -> packed bf16 heads and packed bf16 tails (first value in the low half)
__device__ __forceinline__ void split2(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = pack_bf16x2(a, b);
    lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

__device__ __forceinline__ bf8 as_bf8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    const uint4 u = make_uint4(a, b, c, d);
    return __builtin_bit_cast(bf8, u);
}
__device__ __forceinline__ bf8 as_bf8(uint4 u) { return __builtin_bit_cast(bf8, u); }

__device__ __forceinline__ f16v mfma(bf8 a, bf8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }

// inclusive prefix sums over lanes 0..31 and, separately, over lanes 32..63 (rows of 16 lanes: shifts inside a row,
// then the first row's total into the second); a lane shifted in from outside its row contributes 0
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROWS, 0xf, false));
}
__device__ __forceinline__ float prefix32(float v)
{
    v += dpp_or_zero<0x111, 0xf>(v);     // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);     // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);     // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);     // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);     // row_bcast:15 into rows 1 and 3
    return v;
}

__device__ __forceinline__ int swap23(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

#ifdef SSMV_TRACE
// Profiling builds only: per workgroup, the shader-clock and the 100 MHz wall-clock ticks the kernel took.
__device__ long long *pf_trace_buf_ = nullptr;
#endif

}  // namespace

// Two waves per SIMD (256 registers each, and then the compiler keeps the accumulators in ordinary registers: no copies
// between the two register files around every use); a tile's state of N = 128 in one wave (64 registers per lane) does
// not fit that.
// A state of N = 128 under a narrow head (P <= 64) is split over two waves per 32-channel tile, each with half of n: the
// second adds its share of h C^T through LDS, both update their own half of the state, and the workgroup has twice the
// threads for the staging.
template <int P, int N>
__global__ __launch_bounds__(2 * P * prefill_nsplit(P, N)) __attribute__((amdgpu_waves_per_eu((N >= 128 && prefill_nsplit(P, N) == 1) ? 1 : 2)))
void prefill_bf16_kernel(const PrefillParams p)
{
    using Ld = PfLds<P, N>;
    constexpr int Q = kQ;
    constexpr int W = SSMV_CONV_WIDTH;
    constexpr int NSPL = Ld::NSPL;
    constexpr int NT = 2 * P * NSPL;     // threads: one wave per 32 channels (and per half of n where the state is split)
    constexpr int TN = N / 32;
    constexpr int TNL = TN / NSPL;       // state tiles of a wave
    constexpr int QS = Q * P / NT;       // consecutive tokens one thread convolves per chunk (NT / P threads per channel)
    constexpr int XS = Ld::XS, PIECES = Ld::PIECES;
    using Vec = IoVec<SSMV_BF16>;
    constexpr int EV = Vec::EV;
    static_assert(P % 32 == 0 && P <= 128 && N % 32 == 0 && W == 4, "tile shapes");

    extern __shared__ float4 lds_raw[];
    char *lds = reinterpret_cast<char *>(lds_raw);
    char *sX = lds + Ld::oX, *sBh = lds + Ld::oBh, *sBl = lds + Ld::oBl, *sMh = lds + Ld::oMh, *sXraw = lds + Ld::oXraw;
    uint32_t *sCar = reinterpret_cast<uint32_t *>(lds + Ld::oCar);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#ifdef SSMV_TRACE
    const long long tr_c0 = clock64(), tr_w0 = wall_clock64();
#endif
    const int li = lane & 31, lh = lane >> 5;           // MFMA: row/column index and k half of this lane
    const int lperm = swap23(li);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int pt = Ld::NSPL == 1 ? wave_u : wave_u % Ld::NP;   // the wave's 32-channel tile
    const int nh = Ld::NSPL == 1 ? 0 : wave_u / Ld::NP;        // and its half of n (0 unless the state is split)
    char *sY = lds + Ld::oY + pt * (Q * Ld::YS);
    float *sCum = reinterpret_cast<float *>(lds + Ld::oCum) + wave * Q;
    float *sDt = reinterpret_cast<float *>(lds + Ld::oDt) + wave * Q;
    float *sW = reinterpret_cast<float *>(lds + Ld::oW) + wave * Q;
    const int H = p.H, G = p.G;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);       // the heads of a sequence on one XCD: B and C come out of its L2
    const int hd = item % H, b = item / H;
    const int Ls = p.L;                                 // token stride of the arrays
    const int L = p.seq_len ? min(max(p.seq_len[b], 0), Ls) : Ls;     // this sequence's prompt length
    if (L == 0) return;                                 // nothing to feed: state, ring and outputs stay as they are
    const int HP = H * P, GN = G * N;
    const int g = hd / (H / G);
    const int cur = (int)((unsigned)p.cur_slot[b] % 3u);
    const int mask = p.ring_len - 1;
    const int conv_head = p.conv_head[b] & mask;
    const float A2_h = p.A[hd] * kLog2e, D_h = p.D[hd];
    const float dtb_h = p.dt_bias ? p.dt_bias[hd] : 0.f;
    const bool gated = p.z != nullptr, silu = p.conv_act == SSMV_ACT_SILU;
    float *state = p.state + (size_t)cur * p.slot_stride + ((size_t)b * H + hd) * P * N;

    // state -> accumulator registers, transposed tiles [n][p]: register 4 q + e of tile tn holds
    // h[p = 32 pt + li][n = 32 (TNL nh + tn) + 16 (q/2) + 8 lh + 4 (q%2) + e]
    f16v hacc[TNL];
    // (row, first column) of the lane's float4 number q of tile tn; the slot is row-major or tiled (state_off4)
    const int srow_ = pt * 32 + li, scol0 = 32 * TNL * nh + 8 * lh;
    auto state_at = [&](int tn, int q) { return state + state_off4(p.tiled, srow_, scol0 + 32 * tn + 16 * (q / 2) + 4 * (q % 2), N); };
#pragma unroll
    for (int tn = 0; tn < TNL; ++tn)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = *reinterpret_cast<const float4 *>(state_at(tn, q));
            hacc[tn][4 * q + 0] = v.x; hacc[tn][4 * q + 1] = v.y; hacc[tn][4 * q + 2] = v.z; hacc[tn][4 * q + 3] = v.w;
        }
    // Every wave computes G^T whole (rows s, columns t = li) and finishes the 16 / (waves) of its registers that are its
    // share of M^T: register 4 q + e is token s = 8 q + 4 lh + e.  The causal mask, and the skip term D on the diagonal:
    constexpr int RW = 4 / Ld::NW;                       // register quads per wave
    float dadd[4 * RW];
    bool keep[4 * RW];
#pragma unroll
    for (int r = 0; r < 4 * RW; ++r) {
        const int s = 8 * (RW * wave + r / 4) + 4 * lh + r % 4;
        keep[r] = s <= li;
        dadd[r] = s == li ? D_h : 0.f;
    }
    // this thread's conv channel: weights and bias stay in registers for the whole prompt
    const int pc = tid % P;
    const int sg = P >= 64 ? __builtin_amdgcn_readfirstlane(tid / P) : tid / P;      // uniform over a wave when P >= 64
    const unsigned ch = hd * P + pc;
    // the four taps as two packed pairs (they are bf16 in memory): the conv is two bf16 dot products per token
    const uint2 wraw = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(p.wgt) + (size_t)ch * W);
    const bf2 w01 = __builtin_bit_cast(bf2, wraw.x), w23 = __builtin_bit_cast(bf2, wraw.y);
    const float cbias = p.bias ? load_io(p.bias, ch, SSMV_BF16) : 0.f;
    // One base pointer per tensor that is uniform over the workgroup plus an element offset; tokens are clamped into
    // the prompt, so every load is unconditional: a token before the prompt is replaced by the ring history, tokens past
    // its end carry dt = 0 and thereby weight 0 everywhere (their rows of X, B, C are the last token's: finite).
    const uint16_t *x_b = reinterpret_cast<const uint16_t *>(p.x_raw) + (size_t)b * Ls * HP;
    const char *z_b = reinterpret_cast<const char *>(p.z) + (size_t)b * Ls * HP * 2;
    char *y_b = reinterpret_cast<char *>(p.y) + (size_t)b * Ls * HP * 2;
    const uint16_t *B_b = reinterpret_cast<const uint16_t *>(p.Bm) + (size_t)b * Ls * GN + (size_t)g * N;
    const uint16_t *C_b = reinterpret_cast<const uint16_t *>(p.Cm) + (size_t)b * Ls * GN + (size_t)g * N;
    const uint16_t *dt_b = reinterpret_cast<const uint16_t *>(p.dt) + (size_t)b * Ls * H + hd;
    auto off = [](int token, int stride, int rest) { return (size_t)(unsigned)(__umul24(token, stride) + rest); };
    auto clampL = [&](int tg) { return tg < 0 ? 0 : (tg < L ? tg : L - 1); };
    auto raw_bits = [&](int tg) { return (uint32_t)(x_b + (size_t)clampL(tg) * HP)[ch]; };    // uniform row pointer, 32-bit lane offset
    // the W-1 raw inputs ahead of the prompt (newest last)
    uint32_t hist[W - 1];                               // as bits
#pragma unroll
    for (int j = 0; j < W - 1; ++j)
        hist[j] = reinterpret_cast<const uint16_t *>(p.ring)[((size_t)b * p.ring_len + ((conv_head + 1 - (W - 1) + j) & mask)) * HP + ch];

    constexpr int UI = (4 * N + NT - 1) / NT;           // (n, eight tokens) units of the transposed B per thread and chunk
    // The chunk's raw x, B and C rows go from global memory straight into LDS, 1 KB per wave and instruction (lane l's 16
    // bytes land at byte 16 l of the destination): no registers hold them while they are under way, and a chunk costs a
    // wave 4 to 6 load instructions instead of 30.  dt (one value per lane) takes the ordinary way.
    auto issue_x_loads = [&](int c, uint32_t &dt_bits) {
        const int t0 = c * Q;
        auto tok = [&](int row) { return min(t0 + row, L - 1); };
        constexpr int LR = P / 8;                       // lanes per row of x, 64 / LR rows per instruction, P / 16 instructions
        constexpr int XPW = 2 / NSPL;                   // of them per wave
#pragma unroll
        for (int k = 0; k < XPW; ++k) {
            const int idx = XPW * wave_u + k;
            const int row = idx * (64 / LR) + lane / LR, piece = lane % LR;
            load_to_lds16(x_b + off(tok(row), HP, hd * P + piece * 8), sXraw + idx * 1024);
        }
        dt_bits = dt_b[off(tok(li), H, 0)];
    };
    auto issue_bc_loads = [&](int c) {
        const int t0 = c * Q;
        auto tok = [&](int row) { return min(t0 + row, L - 1); };
        char *dB = lds + Ld::oB + (c & (Ld::BCC - 1)) * Ld::BCS, *dC = lds + Ld::oC + (c & (Ld::BCC - 1)) * Ld::BCS;
#pragma unroll
        for (int k = 0; k < (PIECES / 2 + Ld::NW - 1) / Ld::NW; ++k) {
            const int idx = wave_u + k * Ld::NW;        // PIECES / 2 instructions cover the 32 rows
            if (idx < PIECES / 2) {
                const int row = idx * (64 / PIECES) + lane / PIECES, pp = lane % PIECES;
                const size_t o = off(tok(row), GN, (pp ^ Ld::swz(row)) * 8);
                load_to_lds16(B_b + o, dB + idx * 1024);
                load_to_lds16(C_b + o, dC + idx * 1024);
            }
        }
    };
    // Per chunk, of this lane's token t = li: log2 e * cum_t and exp(cum_t); and exp(cum_Q) (the same in every lane).
    float cum_t, at_t, aq;
    auto consume = [&](int c, uint32_t dt_bits) {
        const int t0 = c * Q, s0 = sg * QS;
        const char *sB = lds + Ld::oB + (c & (Ld::BCC - 1)) * Ld::BCS;
        // ---- dt, its prefix sums and the decay factors: every wave for itself (32 tokens, both halves alike) ----
        {
            float d = Vec::decode1(dt_bits) + dtb_h;
            if (p.dt_softplus) d = softplus_fast(d);
            if (t0 + li >= L) d = 0.f;                  // padding: no decay, no input
            float v = d * A2_h;
            v = prefix32(v);
            const float cq = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), Q - 1));
            cum_t = v;
            at_t = __builtin_amdgcn_exp2f(v);
            aq = __builtin_amdgcn_exp2f(cq);
            if (lh == 0) {
                sCum[li] = v;
                sDt[li] = d;
                sW[li] = __builtin_amdgcn_exp2f(cq - v) * d;
            }
            __builtin_amdgcn_wave_barrier();            // the wave's own LDS traffic stays in program order
        }
        // ---- conv of this thread's QS tokens, rows [p][token] ----
        {
            // raw inputs: [token][channel] in LDS; the three ahead of this thread's tokens are the ring history (first chunk),
            // what the other half's threads left of the previous chunk, or simply earlier rows of this one
            const uint16_t *xin = reinterpret_cast<const uint16_t *>(sXraw) + pc;
            uint32_t xb[QS + W - 1];                    // the raw inputs of tokens s0 - 3 .. s0 + QS - 1, as bits
            if (s0 != 0) {
#pragma unroll
                for (int j = 0; j < W - 1; ++j) xb[j] = xin[(s0 - (W - 1) + j) * P];
            } else if (c == 0) {
#pragma unroll
                for (int j = 0; j < W - 1; ++j) xb[j] = hist[j];
            } else {
#pragma unroll
                for (int j = 0; j < W - 1; ++j) xb[j] = sCar[(((c - 1) & 1) * 3 + j) * P + pc];
            }
#pragma unroll
            for (int j = 0; j < QS; ++j) xb[j + W - 1] = xin[(s0 + j) * P];
            // x_t = bias + (w0, w1).(r_(t-3), r_(t-2)) + (w2, w3).(r_(t-1), r_t): bf16 products are exact in fp32, the sums
            // are fp32 (v_dot2c_f32_bf16); adjacent raw inputs are packed once and serve two tokens
            bf2 pk[QS + 2];
#pragma unroll
            for (int i = 0; i < QS + 2; ++i) pk[i] = __builtin_bit_cast(bf2, xb[i] | (xb[i + 1] << 16));
            float xv[QS];
#pragma unroll
            for (int j = 0; j < QS; ++j)
                xv[j] = __builtin_amdgcn_fdot2_f32_bf16(w23, pk[j + 2], __builtin_amdgcn_fdot2_f32_bf16(w01, pk[j], cbias, false), false);
            if (s0 + QS == Q) {                         // the chunk's last three raw inputs, for the next chunk
#pragma unroll
                for (int j = 0; j < W - 1; ++j) sCar[((c & 1) * 3 + j) * P + pc] = xb[QS + j];
            }
            if (silu) {
#pragma unroll
                for (int j = 0; j < QS; ++j) xv[j] = xv[j] / (1.f + expf(-xv[j]));
            }
            uint32_t xr[QS / 2];
#pragma unroll
            for (int j2 = 0; j2 < QS / 2; ++j2) xr[j2] = pack_bf16x2(xv[2 * j2], xv[2 * j2 + 1]);     // the rounding to the storage type
            const int o = pc * XS + s0 * 2;
#pragma unroll
            for (int v = 0; v < QS / 8; ++v)
                *reinterpret_cast<uint4 *>(sX + o + 16 * v) = make_uint4(xr[4 * v], xr[4 * v + 1], xr[4 * v + 2], xr[4 * v + 3]);
        }
        // ---- w_s B_s transposed, head and tail: eight tokens of one n per unit ----
#pragma unroll
        for (int i = 0; i < UI; ++i) {
            const int u = tid + i * NT;
            if (u < 4 * N) {
                const int n = u % N;
                const int oct = N >= 64 ? __builtin_amdgcn_readfirstlane(u / N) : u / N;
                const float4 w0 = *reinterpret_cast<const float4 *>(sW + 8 * oct), w1 = *reinterpret_cast<const float4 *>(sW + 8 * oct + 4);
                const float wv[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
                uint32_t bh[4], bl[4];
                // B[token 8 oct + j][n] out of the swizzled rows: the piece index of n, XORed with the row's key (the same
                // in all lanes), plus what does not depend on j - one instruction per element
                const int piece16 = (n >> 3) * 16, rest = (n & 7) * 2 + oct * (8 * N * 2);
                auto b_at = [&](int j) {
                    const int key16 = Ld::swz(8 * oct + j) * 16;
                    return Vec::decode1(*reinterpret_cast<const uint16_t *>(sB + ((piece16 ^ key16) + rest) + j * (N * 2)));
                };
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) split2(wv[2 * j2] * b_at(2 * j2), wv[2 * j2 + 1] * b_at(2 * j2 + 1), bh[j2], bl[j2]);
                *reinterpret_cast<uint4 *>(sBh + n * XS + oct * 16) = make_uint4(bh[0], bh[1], bh[2], bh[3]);
                *reinterpret_cast<uint4 *>(sBl + n * XS + oct * 16) = make_uint4(bl[0], bl[1], bl[2], bl[3]);
            }
        }
    };

    // The output tile [token][32 channels] of a chunk goes into the wave's own LDS patch and leaves as 64-byte rows or wider
    // (four lanes a row: a store instruction then touches 16 cache lines, not 32 with 16 bytes in each), one chunk LATE, next
    // to the issue of the following chunk's loads: loads and stores share one counter and complete in no fixed order
    // among each other, so the wait for the loads at the top of a chunk also waits for every store issued before it -
    // which by then is a whole chunk old instead of a few cycles.
    auto flush_outputs = [&](int c) {
        const int t0 = c * Q;
        // By then every wave's tile of that chunk is complete (the barrier at the chunk's end lies in between), so the rows are
        // dealt out again: a wave stores whole rows of the head (all its 32-channel tiles side by side: whole cache lines
        // from one instruction instead of 64-byte halves from two waves at different times) for its share of the tokens.
        // 4 to 8 % on the 64- and 128-channel heads (3 % slower with the 128 x 128 tile, which keeps the wave's own rows).
        if constexpr (NSPL == 1 && Ld::NP > 1 && !(P >= 128 && N >= 128)) {
            constexpr int LPT = 4 * Ld::NP, TPI = 64 / LPT;      // lanes per token row of the head, tokens per instruction
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int tt = (2 * wave_u + r) * TPI + lane / LPT, piece = lane % LPT;
                const uint4 v = *reinterpret_cast<const uint4 *>(lds + Ld::oY + (piece >> 2) * (Q * Ld::YS) + tt * Ld::YS + (piece & 3) * 16);
                if (t0 + tt < L) Vec::store_raw(y_b, off(t0 + tt, HP, hd * P + piece * 8), v);
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int tt = 16 * r + (lane >> 2), piece = lane & 3;
            const uint4 v = *reinterpret_cast<const uint4 *>(sY + tt * Ld::YS + piece * 16);
            if (t0 + tt < L) Vec::store_raw(y_b, off(t0 + tt, HP, hd * P + pt * 32 + piece * 8), v);
        }
    };
    const int n_chunks = (L + Q - 1) / Q;
    const int prow = pt * 32 + li;                      // this lane's channel (inside the head) as an operand row
    float *sZ = reinterpret_cast<float *>(lds + Ld::oZ) + pt * 1024;
    uint32_t dt_bits;
    issue_x_loads(0, dt_bits);
    issue_bc_loads(0);
    wait_direct_loads();
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        const int t0 = c * Q;
        const char *sB = lds + Ld::oB + (c & (Ld::BCC - 1)) * Ld::BCS, *sC = lds + Ld::oC + (c & (Ld::BCC - 1)) * Ld::BCS;
        consume(c, dt_bits);
        __syncthreads();
        // the stores ahead of the loads on the wide tiles (2 % there; the other way round on the narrow ones)
        constexpr bool kStoresFirst = P >= 128 && N >= 64;
        if (kStoresFirst && c > 0 && nh == 0) {
            flush_outputs(c - 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (c + 1 < n_chunks) {                         // under way for the whole chunk
            issue_x_loads(c + 1, dt_bits);
            if (Ld::BCC == 2) issue_bc_loads(c + 1);
        }
        if (!kStoresFirst && c > 0 && nh == 0) flush_outputs(c - 1);
        __builtin_amdgcn_sched_barrier(0);              // the loads and stores stay here, a chunk of arithmetic ahead of the next wait

        const int t = li;                               // this lane's token within the chunk
        const bool live = t0 + t < L;
        using QV = XVec<SSMV_BF16, 4>;                  // four adjacent channels
        typename QV::Raw zraw[4];
        if (gated && nh == 0) {                         // requested ahead of the matrix products
            const int tc = live ? t0 + t : L - 1;
#pragma unroll
            for (int q = 0; q < 4; ++q) zraw[q] = QV::load(z_b, off(tc, HP, hd * P + pt * 32 + 8 * q + 4 * lh));
        }
        // C of this lane's token, all of it: the B operand of G^T and of h C^T
        uint4 cop[N / 16];
#pragma unroll
        for (int st = 0; st < N / 16; ++st) cop[st] = *reinterpret_cast<const uint4 *>(sC + t * (N * 2) + (((2 * st + lh) ^ Ld::swz(t)) * 16));
        // ---- G^T = B C^T, then this wave's share of M^T: masked, decayed, scaled, D on the diagonal; to LDS ----
        {
            f16v gacc = {0};
#pragma unroll
            for (int st = 0; st < N / 16; ++st)
                gacc = mfma(as_bf8(*reinterpret_cast<const uint4 *>(sB + li * (N * 2) + (((2 * st + lh) ^ Ld::swz(li)) * 16))), as_bf8(cop[st]), gacc);
            // registers 4 q .. 4 q + 3 of G^T -> M^T for tokens s = 8 q + 4 lh + [0, 4); r = the quad's index within the wave's share
            auto finish = [&](int q, int r, float g0, float g1, float g2, float g3) {
                const int s0 = 8 * q + 4 * lh;
                const float4 cs = *reinterpret_cast<const float4 *>(sCum + s0), ds = *reinterpret_cast<const float4 *>(sDt + s0);
                const float csv[4] = {cs.x, cs.y, cs.z, cs.w}, dsv[4] = {ds.x, ds.y, ds.z, ds.w}, g4[4] = {g0, g1, g2, g3};
                float m[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float dec = __builtin_amdgcn_exp2f(cum_t - csv[e]) * dsv[e];      // may overflow where s > t: selected away
                    m[e] = keep[4 * r + e] ? fmaf(g4[e], dec, dadd[4 * r + e]) : 0.f;
                }
                *reinterpret_cast<uint2 *>(sMh + t * XS + s0 * 2) = make_uint2(pack_bf16x2(m[0], m[1]), pack_bf16x2(m[2], m[3]));
            };
            // the wave's quads: a uniform branch, so that no register is indexed by a variable
            if constexpr (RW == 4) {
#pragma unroll
                for (int r = 0; r < 4; ++r) finish(r, r, gacc[4 * r], gacc[4 * r + 1], gacc[4 * r + 2], gacc[4 * r + 3]);
            } else if constexpr (RW == 2) {
                if (wave_u == 0) {
                    finish(0, 0, gacc[0], gacc[1], gacc[2], gacc[3]);
                    finish(1, 1, gacc[4], gacc[5], gacc[6], gacc[7]);
                } else {
                    finish(2, 0, gacc[8], gacc[9], gacc[10], gacc[11]);
                    finish(3, 1, gacc[12], gacc[13], gacc[14], gacc[15]);
                }
            } else {
                switch (wave_u) {
                    case 0: finish(0, 0, gacc[0], gacc[1], gacc[2], gacc[3]); break;
                    case 1: finish(1, 0, gacc[4], gacc[5], gacc[6], gacc[7]); break;
                    case 2: finish(2, 0, gacc[8], gacc[9], gacc[10], gacc[11]); break;
                    default: finish(3, 0, gacc[12], gacc[13], gacc[14], gacc[15]); break;
                }
            }
        }
        // ---- Y^T = h C^T, scaled by exp(cum_t): the state registers are the A operand ----
        f16v yacc = {0};
#pragma unroll
        for (int tn = 0; tn < TNL; ++tn)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                uint32_t ah[4];                          // heads only: these products end in outputs, not in the state
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    ah[d] = pack_bf16x2(hacc[tn][8 * st + 2 * d], hacc[tn][8 * st + 2 * d + 1]);
                }
                // C for the wave's own tiles: with a split state read again at the wave's offset (a choice between
                // registers by a variable would put the array into scratch memory)
                uint4 c4;
                if constexpr (NSPL == 2) c4 = *reinterpret_cast<const uint4 *>(sC + t * (N * 2) + (((2 * (2 * (TNL * nh + tn) + st) + lh) ^ Ld::swz(t)) * 16));
                else c4 = cop[2 * tn + st];
                const bf8 cb = as_bf8(c4);
                yacc = mfma(as_bf8(ah[0], ah[1], ah[2], ah[3]), cb, yacc);
            }
        if constexpr (NSPL == 2) {
            if (nh == 1) {                              // the second half of n: hand the sum to the tile's first wave
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4 *>(sZ + q * 256 + lane * 4) = make_float4(yacc[4 * q], yacc[4 * q + 1], yacc[4 * q + 2], yacc[4 * q + 3]);
            }
        }
        // ---- Y^T += X^T M^T;  h^T <- exp(cum_Q) h^T + (diag(w) B)^T X: X is the A operand of one, the B operand of the other ----
        uint4 xop[2];
#pragma unroll
        for (int st = 0; st < 2; ++st) xop[st] = *reinterpret_cast<const uint4 *>(sX + prow * XS + (16 * st + 8 * lh) * 2);
        __syncthreads();     // M^T is complete; nobody reads this chunk's B and C rows any more
        if (Ld::BCC == 1 && c + 1 < n_chunks) issue_bc_loads(c + 1);
        if (nh == 0) {
            if constexpr (NSPL == 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 z4 = *reinterpret_cast<const float4 *>(sZ + q * 256 + lane * 4);
                    yacc[4 * q] += z4.x; yacc[4 * q + 1] += z4.y; yacc[4 * q + 2] += z4.z; yacc[4 * q + 3] += z4.w;
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) yacc[v] *= at_t;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const int o = t * XS + (16 * st + 8 * lh) * 2;
                yacc = mfma(as_bf8(xop[st]), as_bf8(*reinterpret_cast<const uint4 *>(sMh + o)), yacc);
            }
        }
#pragma unroll
        for (int tn = 0; tn < TNL; ++tn) {
#pragma unroll
            for (int v = 0; v < 16; ++v) hacc[tn][v] *= aq;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const int o = (32 * (TNL * nh + tn) + lperm) * XS + (16 * st + 8 * lh) * 2;
                hacc[tn] = mfma(as_bf8(*reinterpret_cast<const uint4 *>(sBh + o)), as_bf8(xop[st]), hacc[tn]);
                hacc[tn] = mfma(as_bf8(*reinterpret_cast<const uint4 *>(sBl + o)), as_bf8(xop[st]), hacc[tn]);
            }
        }
        // ---- gate, store ----
        if (nh == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float yv[4] = {yacc[4 * q + 0], yacc[4 * q + 1], yacc[4 * q + 2], yacc[4 * q + 3]};
            if (gated) {
                float zf[4];
                QV::decode(zraw[q], zf);
#pragma unroll
                for (int e = 0; e < 4; ++e) yv[e] *= silu_fast(zf[e]);
            }
            *reinterpret_cast<uint2 *>(sY + t * Ld::YS + (8 * q + 4 * lh) * 2) = QV::encode(yv);
        }
        }
        __builtin_amdgcn_wave_barrier();                // the tile waits in the wave's LDS patch: flush_outputs
        wait_direct_loads();                            // this wave's share of the next chunk's inputs has landed ...
        __syncthreads();     // ... and so has everybody's; the next chunk overwrites X, B^T, M
    }

    if (nh == 0) flush_outputs(n_chunks - 1);
    // ---- state back in place; the newest W-1 raw inputs into the ring behind conv_head -----------------------
#pragma unroll
    for (int tn = 0; tn < TNL; ++tn)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4 *>(state_at(tn, q)) =
                make_float4(hacc[tn][4 * q + 0], hacc[tn][4 * q + 1], hacc[tn][4 * q + 2], hacc[tn][4 * q + 3]);
    if (tid < P) {
        for (int tg = (L - (W - 1) > 0 ? L - (W - 1) : 0); tg < L; ++tg)
            Vec::store_raw1(p.ring, ((size_t)b * p.ring_len + ((conv_head + 1 + tg) & mask)) * HP + ch, raw_bits(tg));
    }
#ifdef SSMV_TRACE
    if (pf_trace_buf_ && tid == 0) {
        pf_trace_buf_[2 * blockIdx.x] = clock64() - tr_c0;
        pf_trace_buf_[2 * blockIdx.x + 1] = wall_clock64() - tr_w0;
    }
#endif
}

template <int P, int N>
static int launch_pn(const PrefillParams &p, hipStream_t stream)
{
    const size_t lds = PfLds<P, N>::total;
    const dim3 grid(p.H * p.batch), block(2 * P * PfLds<P, N>::NSPL);
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_bf16_kernel<P, N>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return (int)e;
    hipLaunchKernelGGL((prefill_bf16_kernel<P, N>), grid, block, lds, stream, p);
    return (int)hipGetLastError();
}

template <int P>
static int launch_p(const PrefillParams &p, hipStream_t stream)
{
    switch (p.N) {
        case 32: return launch_pn<P, 32>(p, stream);
        case 64: return launch_pn<P, 64>(p, stream);
        case 128: return launch_pn<P, 128>(p, stream);
        default: return (int)hipErrorInvalidConfiguration;
    }
}

#ifdef SSMV_TRACE
int set_trace_prefill(long long *buf) { return (int)hipMemcpyToSymbol(HIP_SYMBOL(pf_trace_buf_), &buf, sizeof(buf)); }
#endif

// the main kernel only; the caller appends the bookkeeping launch
int launch_prefill_bf16(const PrefillParams &p, hipStream_t stream)
{
    switch (p.P) {
        case 32: return launch_p<32>(p, stream);
        case 64: return launch_p<64>(p, stream);
        case 128: return launch_p<128>(p, stream);
        default: return (int)hipErrorInvalidConfiguration;
    }
}

}  // namespace ssmv
