// Chunked prefill of a scalar-decay (Mamba-2 style) layer with fp32 tensors (bf16 tensors: prefill_bf16.hip, same
// evaluation on the bf16 matrix cores): all L prompt tokens through the recurrence of
// Section 2.1 Eq. 1 (with the discretisation of Section 2.2), producing every y_t and leaving the cached state and
// the conv ring as if the L tokens had been verified and accepted.  This is where the path has a dense
// contraction, so it runs on the matrix cores (fp32 MFMA: the state and the outputs keep fp32 accuracy).
//
// Per chunk of Q = 32 tokens, with cum_t = A * (dt_0 + .. + dt_t) inside the chunk and h the state before it:
//   G      = C B^T                                            [Q x Q]   contraction over N
//   M_ts   = G_ts exp(cum_t - cum_s) dt_s   for s <= t, else 0
//   Y      = M X  +  diag(exp(cum_t)) C h^T  +  D X           [Q x P]   contractions over Q and over N
//   h     <- exp(cum_Q) h  +  (diag(w) X)^T B,  w_s = exp(cum_Q - cum_s) dt_s      [P x N]   contraction over Q
// which is Eq. 1 unrolled over the chunk and regrouped (the "chunked" or "state-space dual" evaluation of the
// scan; the paper's own prefill uses the hardware-aware scan of its reference [Mamba]).  One workgroup of four
// waves owns one (sequence, head); the state stays in LDS across the chunks, the chunk's X, B, C in LDS as fp32.
// v_mfma_f32_32x32x2_f32 operands: A[i = lane%32][k = lane/32], B[k = lane/32][j = lane%32]; result register v of
// a lane is D[8*(v/4) + 4*(lane/32) + v%4][lane%32]; v_mfma_f32_16x16x4_f32 (used for the Q x Q product, one
// quadrant per wave): A[i = lane%16][k = lane/16], B[k = lane/16][j = lane%16], D[4*(lane/16) + v][lane%16].  Rows of
// the LDS arrays that are read with the lane as the ROW index are padded by one float, so that the lanes hit
// different banks.
// The global loads of chunk c+1 are issued (as raw bits, unconditionally, from clamped addresses) right after the
// barrier that ends the staging of chunk c and are decoded into LDS after chunk c's arithmetic: one chunk of
// latency hiding for a kernel that would otherwise wait for memory once per chunk.
#include "ssmv_internal.h"

namespace ssmv {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef float v4f_t __attribute__((ext_vector_type(4)));

constexpr int kQ = 32;     // tokens per chunk

template <int P, int N>
__host__ __device__ constexpr size_t prefill_lds_floats()
{
    return (size_t)P * (N + 1) + (size_t)kQ * P + 2 * (size_t)kQ * (N + 1) + (size_t)kQ * (kQ + 1) + 4 * kQ;
}

template <int P, int N, int IO>
__global__ __launch_bounds__(256) void prefill_kernel(const PrefillParams p)
{
    constexpr int Q = kQ;
    constexpr int W = SSMV_CONV_WIDTH;
    constexpr int NP = N + 1, QP = Q + 1;
    constexpr int TP = P / 32, TN = N / 32;
    constexpr int XG = 256 / P;          // thread groups along the tokens of a chunk
    constexpr int QS = Q / XG;           // consecutive tokens one thread convolves per chunk
    using Vec = IoVec<IO>;
    constexpr int EV = Vec::EV;
    static_assert(P % 32 == 0 && P <= 128 && N % 32 == 0, "tile shapes");

    extern __shared__ float4 lds_raw[];
    float *sH = reinterpret_cast<float *>(lds_raw);     // [P][N+1]  state
    float *sX = sH + P * NP;                            // [Q][P]    conv output of the chunk (rounded to the I/O type)
    float *sB = sX + Q * P;                             // [Q][N+1]
    float *sC = sB + Q * NP;                            // [Q][N+1]
    float *sM = sC + Q * NP;                            // [Q][Q+1]
    float *sDt = sM + Q * QP;                           // [Q]
    float *sCum = sDt + Q;                              // [Q]  inclusive prefix of dt*A
    float *sAt = sCum + Q;                              // [Q]  exp(cum_t): decay from the chunk's start to after token t
    float *sW = sAt + Q;                                // [Q]  exp(cum_Q - cum_s) dt_s: weight of token s in the chunk's state update

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lk = lane >> 5;           // MFMA: row/column index and k index of this lane
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
    const float A_h = p.A[hd], D_h = p.D[hd];
    const float dtb_h = p.dt_bias ? p.dt_bias[hd] : 0.f;
    const bool gated = p.z != nullptr;
    float *state = p.state + (size_t)cur * p.slot_stride + ((size_t)b * H + hd) * P * N;

    // state -> LDS
    for (int idx = tid; idx < P * N / 4; idx += 256) {
        const int row = (idx * 4) / N, col = (idx * 4) % N;
        const float4 v = *reinterpret_cast<const float4 *>(state + state_off4(p.tiled, row, col, N));
        float *d = sH + row * NP + col;
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    }
    // this thread's conv channel: weights and bias stay in registers for the whole prompt
    const int pc = tid % P, sg = tid / P;
    const int ch = hd * P + pc;
    float wgt[W];
#pragma unroll
    for (int w = 0; w < W; ++w) wgt[w] = load_io(p.wgt, (size_t)ch * W + w, IO);
    const float cbias = p.bias ? load_io(p.bias, ch, IO) : 0.f;
    // raw conv input of prompt token tg for this channel (bits), from a clamped address: a token before the prompt is
    // replaced by the ring history below, one past the end is zeroed when it is used.  (One base pointer only: a
    // select between two gets compiled into two loads and a select of their results, with a wait on the spot.)
    // Addresses: a base pointer per sequence that is uniform over the workgroup plus a 32-bit element offset from the
    // 24-bit multiplier (the host refuses prompts whose tensors would not fit), so that no load needs 64-bit or
    // quarter-rate integer arithmetic.
    constexpr size_t ES = IO == SSMV_BF16 ? 2 : 4;
    const char *x_b = reinterpret_cast<const char *>(p.x_raw) + (size_t)b * Ls * HP * ES;
    const char *z_b = reinterpret_cast<const char *>(p.z) + (size_t)b * Ls * HP * ES;
    char *y_b = reinterpret_cast<char *>(p.y) + (size_t)b * Ls * HP * ES;
    const char *B_b = reinterpret_cast<const char *>(p.Bm) + ((size_t)b * Ls * GN + (size_t)g * N) * ES;
    const char *C_b = reinterpret_cast<const char *>(p.Cm) + ((size_t)b * Ls * GN + (size_t)g * N) * ES;
    const char *dt_b = reinterpret_cast<const char *>(p.dt) + ((size_t)b * Ls * H + hd) * ES;
    auto off = [](int token, int stride, int rest) { return (size_t)(unsigned)(__umul24(token, stride) + rest); };
    auto raw_bits = [&](int tg) {
        const int tc = tg < 0 ? 0 : (tg < L ? tg : L - 1);
        return Vec::load_raw1(x_b, off(tc, HP, ch));
    };
    // the W-1 raw inputs ahead of the prompt (newest last)
    float hist[W - 1];
#pragma unroll
    for (int j = 0; j < W - 1; ++j)
        hist[j] = load_io(p.ring, ((size_t)b * p.ring_len + ((conv_head + 1 - (W - 1) + j) & mask)) * HP + ch, IO);
    constexpr int BI = (Q * (N / EV) + 255) / 256;      // 16-byte B (and C) vectors per thread and chunk
    struct Fetch { uint32_t x[QS + W - 1]; uint4 bv[BI], cv[BI]; uint32_t dt; };
    auto prefetch = [&](int c, Fetch &f) {
        const int t0 = c * Q, s0 = sg * QS;
#pragma unroll
        for (int j = 0; j < QS + W - 1; ++j) f.x[j] = raw_bits(t0 + s0 - (W - 1) + j);
#pragma unroll
        for (int i = 0; i < BI; ++i) {
            const int item = tid + i * 256;
            const int s_ = item / (N / EV), n = (item % (N / EV)) * EV;
            const int tg = t0 + (s_ < Q ? s_ : Q - 1);
            const size_t o = off(tg < L ? tg : L - 1, GN, n);
            f.bv[i] = Vec::load_raw(B_b, o);
            f.cv[i] = Vec::load_raw(C_b, o);
        }
        const int tq = t0 + (tid & (Q - 1));
        f.dt = Vec::load_raw1(dt_b, off(tq < L ? tq : L - 1, H, 0));
    };
    auto consume = [&](int c, const Fetch &f) {
        const int t0 = c * Q, s0 = sg * QS;
        float tap[W - 1];
#pragma unroll
        for (int j = 0; j < W - 1; ++j) {
            const int tg = t0 + s0 - (W - 1) + j;       // < 0 only in the first chunk: -(W-1)+j, i.e. hist[j]
            tap[j] = tg < 0 ? hist[j] : Vec::decode1(f.x[j]);
        }
        float t1 = tap[0], t2 = tap[1], t3 = tap[2];
#pragma unroll
        for (int j = 0; j < QS; ++j) {
            const int tg = t0 + s0 + j;
            const float r = Vec::decode1(f.x[j + W - 1]);
            // same fp32 order and rounding as conv1d_state_update
            float acc = cbias;
            acc = fmaf(wgt[0], t1, acc);
            acc = fmaf(wgt[1], t2, acc);
            acc = fmaf(wgt[2], t3, acc);
            acc = fmaf(wgt[3], r, acc);
            if (p.conv_act == SSMV_ACT_SILU) acc = acc / (1.f + expf(-acc));
            if (IO == SSMV_BF16) acc = bf16_bits_to_f32(f32_to_bf16_bits(acc));
            sX[(s0 + j) * P + pc] = tg < L ? acc : 0.f;
            t1 = t2; t2 = t3; t3 = r;
        }
#pragma unroll
        for (int i = 0; i < BI; ++i) {
            const int item = tid + i * 256;
            if (item < Q * (N / EV)) {
                const int s_ = item / (N / EV), n = (item % (N / EV)) * EV;
                const bool live = t0 + s_ < L;
                float bv[EV], cv[EV];
                Vec::decode(f.bv[i], bv);
                Vec::decode(f.cv[i], cv);
#pragma unroll
                for (int e = 0; e < EV; ++e) {
                    sB[s_ * NP + n + e] = live ? bv[e] : 0.f;
                    sC[s_ * NP + n + e] = live ? cv[e] : 0.f;
                }
            }
        }
        if (tid < Q) {
            float d = Vec::decode1(f.dt) + dtb_h;
            if (p.dt_softplus) d = softplus_fast(d);
            if (t0 + tid >= L) d = 0.f;                                                      // padding: no decay, no input
            float v = d * A_h;
#pragma unroll
            for (int off = 1; off < Q; off <<= 1) {
                const float u = __shfl_up(v, off, 64);
                if (tid >= off) v += u;
            }
            const float cq = __shfl(v, Q - 1, 64);
            sDt[tid] = d;
            sCum[tid] = v;
            sAt[tid] = expf(v);
            sW[tid] = expf(cq - v) * d;
        }
    };

    const int n_chunks = (L + Q - 1) / Q;
    Fetch fetch;
    prefetch(0, fetch);
    for (int c = 0; c < n_chunks; ++c) {
        const int t0 = c * Q;
        consume(c, fetch);
        __syncthreads();
        if (c + 1 < n_chunks) prefetch(c + 1, fetch);
        __builtin_amdgcn_sched_barrier(0);              // the loads stay here, a whole chunk of arithmetic ahead of their use

        // ---- G = C B^T, one 16x16 quadrant per wave, masked and scaled into M; Y <- diag(exp(cum)) C h^T -----------
        {
            const int qi = wave >> 1, qj = wave & 1;        // rows t in [16 qi, +16), columns s in [16 qj, +16)
            const int l16 = lane & 15, k4 = lane >> 4;
            const int srow = qj * 16 + l16;
            if (qj <= qi) {                                 // the upper-right quadrant is all s > t
                f4v gacc = {0};
#pragma unroll
                for (int kk = 0; kk < N / 4; ++kk) {
                    const int n = 4 * kk + k4;
                    gacc = __builtin_amdgcn_mfma_f32_16x16x4f32(sC[(qi * 16 + l16) * NP + n], sB[srow * NP + n], gacc, 0, 0, 0);
                }
                const float cs = sCum[srow], ds = sDt[srow];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int t = qi * 16 + 4 * k4 + v;
                    const bool keep = srow <= t;
                    const float dec = expf(keep ? sCum[t] - cs : 0.f);
                    sM[t * QP + srow] = keep ? gacc[v] * dec * ds : 0.f;
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) sM[(qi * 16 + 4 * k4 + v) * QP + srow] = 0.f;
            }
        }
        // The output tile is accumulated TRANSPOSED (rows = the wave's 32 channels, columns = the chunk's tokens): a lane
        // then holds, for its token, runs of four adjacent channels, which leave as 8- or 16-byte stores and meet the
        // gate inputs and the skip term in the same shape, with no trip through LDS.
        f16v yacc = {0};
        if (wave < TP) {
            const float at = sAt[li];
            const float *hrow = sH + (wave * 32 + li) * NP;
#pragma unroll
            for (int kk = 0; kk < N / 2; ++kk) {
                const int n = 2 * kk + lk;
                yacc = __builtin_amdgcn_mfma_f32_32x32x2f32(hrow[n], sC[li * NP + n] * at, yacc, 0, 0, 0);
            }
        }
        __syncthreads();     // M is complete; nobody reads the old state any more

        // ---- Y^T += X^T M^T, + D X, gate, store ---------------------------------------------------------
        if (wave < TP) {
            const int t = li;                                   // this lane's token within the chunk
            const bool live = t0 + t < L;
            const int tc = live ? t0 + t : L - 1;
            using QV = XVec<IO, 4>;                             // four adjacent channels in the I/O type
            typename QV::Raw zraw[4];
            if (gated) {                                        // requested ahead of the matrix products
#pragma unroll
                for (int q = 0; q < 4; ++q) zraw[q] = QV::load(z_b, off(tc, HP, hd * P + wave * 32 + 8 * q + 4 * lk));
            }
#pragma unroll
            for (int kk = 0; kk < Q / 2; ++kk) {
                const int s_ = 2 * kk + lk;
                yacc = __builtin_amdgcn_mfma_f32_32x32x2f32(sX[s_ * P + wave * 32 + li], sM[li * QP + s_], yacc, 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int pl = wave * 32 + 8 * q + 4 * lk;      // first of the four channels (inside the head)
                const v4f_t xs = *reinterpret_cast<const v4f_t *>(sX + t * P + pl);
                float yv[4] = {fmaf(D_h, xs.x, yacc[4 * q + 0]), fmaf(D_h, xs.y, yacc[4 * q + 1]), fmaf(D_h, xs.z, yacc[4 * q + 2]),
                               fmaf(D_h, xs.w, yacc[4 * q + 3])};
                if (gated) {
                    float zf[4];
                    QV::decode(zraw[q], zf);
#pragma unroll
                    for (int e = 0; e < 4; ++e) yv[e] *= silu_fast(zf[e]);
                }
                if (live) QV::store(y_b, off(t0 + t, HP, hd * P + pl), QV::encode(yv));
            }
        }
        // ---- h <- exp(cum_Q) h + (diag(w) X)^T B, tile by tile ---------------------------------------------
        {
            const float aq = sAt[Q - 1];
            for (int tile = wave; tile < TP * TN; tile += 4) {
                const int tp = tile / TN, tn = tile % TN;
                f16v sacc = {0};
#pragma unroll
                for (int kk = 0; kk < Q / 2; ++kk) {
                    const int s = 2 * kk + lk;
                    const float ws = sW[s];
                    sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(sX[s * P + tp * 32 + li] * ws, sB[s * NP + tn * 32 + li], sacc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float *d = sH + (tp * 32 + 8 * (v / 4) + 4 * lk + (v % 4)) * NP + tn * 32 + li;
                    *d = fmaf(aq, *d, sacc[v]);
                }
            }
        }
        __syncthreads();     // the next chunk overwrites X, B, C, M and reads the new state
    }

    // ---- state back in place; the newest W-1 raw inputs into the ring behind conv_head -----------------------
    for (int idx = tid; idx < P * N / 4; idx += 256) {
        const int row = (idx * 4) / N, col = (idx * 4) % N;
        const float *s = sH + row * NP + col;
        *reinterpret_cast<float4 *>(state + state_off4(p.tiled, row, col, N)) = make_float4(s[0], s[1], s[2], s[3]);
    }
    if (tid < P) {
        for (int tg = (L - (W - 1) > 0 ? L - (W - 1) : 0); tg < L; ++tg)
            Vec::store_raw1(p.ring, ((size_t)b * p.ring_len + ((conv_head + 1 + tg) & mask)) * HP + ch, raw_bits(tg));
    }
}

// pos += L, conv_head += L; a prefill on a cache with pending tokens or an uncommitted verify is a sequencing error
__global__ void prefill_finish_kernel(int batch, int Ls, const int32_t *seq_len, int ring_len, int64_t *pos, int32_t *conv_head,
                                      const int32_t *pend, const int32_t *last_k, int32_t *err_flag)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int L = seq_len ? min(max(seq_len[b], 0), Ls) : Ls;
    if (pend[b] != 0 || last_k[b] != 0) *err_flag = 1;
    pos[b] += L;
    conv_head[b] = (conv_head[b] + L) & (ring_len - 1);
}

template <int P, int N>
static int launch_pn(const PrefillParams &p, hipStream_t stream)
{
    const size_t lds = prefill_lds_floats<P, N>() * sizeof(float);
    const dim3 grid(p.H * p.batch), block(256);
    // fp32 tensors only: bf16 tensors take the bf16 matrix cores (prefill_bf16.hip)
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_kernel<P, N, SSMV_F32>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return (int)e;
    hipLaunchKernelGGL((prefill_kernel<P, N, SSMV_F32>), grid, block, lds, stream, p);
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

bool prefill_shape_supported(int P, int N)
{
    return (P == 32 || P == 64 || P == 128) && (N == 32 || N == 64 || N == 128);
}

int launch_prefill(const PrefillParams &p, hipStream_t stream)
{
    int rc;
    if (p.io == SSMV_BF16) {
        rc = launch_prefill_bf16(p, stream);
    } else {
        switch (p.P) {
            case 32: rc = launch_p<32>(p, stream); break;
            case 64: rc = launch_p<64>(p, stream); break;
            case 128: rc = launch_p<128>(p, stream); break;
            default: return (int)hipErrorInvalidConfiguration;
        }
    }
    if (rc != 0) return rc;
    hipLaunchKernelGGL(prefill_finish_kernel, dim3((p.batch + 63) / 64), dim3(64), 0, stream, p.batch, p.L, p.seq_len, p.ring_len, p.pos,
                       p.conv_head_rw, p.pend, p.last_k, p.err_flag);
    return (int)hipGetLastError();
}

}  // namespace ssmv
