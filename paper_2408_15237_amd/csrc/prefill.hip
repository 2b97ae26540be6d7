// Chunked prefill of a scalar-decay (Mamba-2 style) layer: all L prompt tokens through the recurrence of
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
// a lane is D[8*(v/4) + 4*(lane/32) + v%4][lane%32].  Rows of the LDS arrays that are read with the lane as the
// ROW index are padded by one float, so that the 32 lanes hit 32 banks.
#include "ssmv_internal.h"

namespace ssmv {

typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kQ = 32;     // tokens per chunk

template <int P, int N>
__host__ __device__ constexpr size_t prefill_lds_floats()
{
    return (size_t)P * (N + 1) + (size_t)kQ * P + 2 * (size_t)kQ * (N + 1) + (size_t)kQ * (kQ + 1) + 2 * kQ;
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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lk = lane >> 5;           // MFMA: row/column index and k index of this lane
    const int hd = blockIdx.x, b = blockIdx.y;
    const int H = p.H, G = p.G, L = p.L;
    const int HP = H * P, GN = G * N;
    const int g = hd / (H / G);
    const int cur = (int)((unsigned)p.cur_slot[b] % 3u);
    const int mask = p.ring_len - 1;
    const int conv_head = p.conv_head[b] & mask;
    const float A_h = p.A[hd], D_h = p.D[hd];
    float *state = p.state + (size_t)cur * p.slot_stride + ((size_t)b * H + hd) * P * N;

    // state -> LDS
    for (int idx = tid; idx < P * N / 4; idx += 256) {
        const float4 v = *reinterpret_cast<const float4 *>(state + idx * 4);
        const int row = (idx * 4) / N, col = (idx * 4) % N;
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
    // raw conv input of global token tg for this channel: the ring for tokens before the prompt, zero past its end
    auto raw_at = [&](int tg) {
        if (tg >= L) return 0.f;
        if (tg < 0) return load_io(p.ring, ((size_t)b * p.ring_len + ((conv_head + 1 + tg) & mask)) * HP + ch, IO);
        return load_io(p.x_raw, ((size_t)b * L + tg) * HP + ch, IO);
    };

    const int n_chunks = (L + Q - 1) / Q;
    for (int c = 0; c < n_chunks; ++c) {
        const int t0 = c * Q;
        // ---- staging ------------------------------------------------------------------------------
        {
            const int s0 = sg * QS;
            float t1 = raw_at(t0 + s0 - 3), t2 = raw_at(t0 + s0 - 2), t3 = raw_at(t0 + s0 - 1);
#pragma unroll
            for (int j = 0; j < QS; ++j) {
                const int tg = t0 + s0 + j;
                const float r = raw_at(tg);
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
        }
        for (int item = tid; item < Q * (N / EV); item += 256) {
            const int s = item / (N / EV), n = (item % (N / EV)) * EV;
            const int tg = t0 + s;
            float bv[EV], cv[EV];
            if (tg < L) {
                const size_t o = ((size_t)b * L + tg) * GN + (size_t)g * N + n;
                Vec::load(p.Bm, o, bv);
                Vec::load(p.Cm, o, cv);
            } else {
#pragma unroll
                for (int e = 0; e < EV; ++e) bv[e] = cv[e] = 0.f;
            }
#pragma unroll
            for (int e = 0; e < EV; ++e) {
                sB[s * NP + n + e] = bv[e];
                sC[s * NP + n + e] = cv[e];
            }
        }
        if (tid < Q) {
            const int tg = t0 + tid;
            const float d = tg < L ? load_io(p.dt, ((size_t)b * L + tg) * H + hd, IO) : 0.f;   // padding: no decay, no input
            float v = d * A_h;
#pragma unroll
            for (int off = 1; off < Q; off <<= 1) {
                const float u = __shfl_up(v, off, 64);
                if (tid >= off) v += u;
            }
            sDt[tid] = d;
            sCum[tid] = v;
        }
        __syncthreads();

        // ---- G = C B^T, masked and scaled into M (wave 0); Y <- diag(exp(cum)) C h^T (every wave its tile) ----
        if (wave == 0) {
            f16v gacc = {0};
            for (int kk = 0; kk < N / 2; ++kk) {
                const int n = 2 * kk + lk;
                gacc = __builtin_amdgcn_mfma_f32_32x32x2f32(sC[li * NP + n], sB[li * NP + n], gacc, 0, 0, 0);
            }
            const float cs = sCum[li], ds = sDt[li];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = 8 * (v / 4) + 4 * lk + (v % 4);
                const bool keep = li <= t;
                const float dec = expf(keep ? sCum[t] - cs : 0.f);
                sM[t * QP + li] = keep ? gacc[v] * dec * ds : 0.f;
            }
        }
        f16v yacc = {0};
        if (wave < TP) {
            const float at = expf(sCum[li]);
            const float *hrow = sH + (wave * 32 + li) * NP;
            for (int kk = 0; kk < N / 2; ++kk) {
                const int n = 2 * kk + lk;
                yacc = __builtin_amdgcn_mfma_f32_32x32x2f32(sC[li * NP + n] * at, hrow[n], yacc, 0, 0, 0);
            }
        }
        __syncthreads();     // M is complete; nobody reads the old state any more

        // ---- Y += M X, + D X, store ------------------------------------------------------------------
        if (wave < TP) {
            const int pcol = wave * 32 + li;
            for (int kk = 0; kk < Q / 2; ++kk) {
                const int s = 2 * kk + lk;
                yacc = __builtin_amdgcn_mfma_f32_32x32x2f32(sM[li * QP + s], sX[s * P + pcol], yacc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = 8 * (v / 4) + 4 * lk + (v % 4);
                if (t0 + t < L) store_io(p.y, ((size_t)b * L + t0 + t) * HP + hd * P + pcol, fmaf(D_h, sX[t * P + pcol], yacc[v]), IO);
            }
        }
        // ---- h <- exp(cum_Q) h + (diag(w) X)^T B, tile by tile ---------------------------------------------
        {
            const float cq = sCum[Q - 1];
            const float aq = expf(cq);
            for (int tile = wave; tile < TP * TN; tile += 4) {
                const int tp = tile / TN, tn = tile % TN;
                f16v sacc = {0};
                for (int kk = 0; kk < Q / 2; ++kk) {
                    const int s = 2 * kk + lk;
                    const float ws = expf(cq - sCum[s]) * sDt[s];
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
        *reinterpret_cast<float4 *>(state + idx * 4) = make_float4(s[0], s[1], s[2], s[3]);
    }
    if (tid < P) {
        for (int tg = (L - (W - 1) > 0 ? L - (W - 1) : 0); tg < L; ++tg)
            store_io(p.ring, ((size_t)b * p.ring_len + ((conv_head + 1 + tg) & mask)) * HP + ch, raw_at(tg), IO);
    }
}

// pos += L, conv_head += L; a prefill on a cache with pending tokens or an uncommitted verify is a sequencing error
__global__ void prefill_finish_kernel(int batch, int L, int ring_len, int64_t *pos, int32_t *conv_head, const int32_t *pend,
                                      const int32_t *last_k, int32_t *err_flag)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    if (pend[b] != 0 || last_k[b] != 0) *err_flag = 1;
    pos[b] += L;
    conv_head[b] = (conv_head[b] + L) & (ring_len - 1);
}

template <int P, int N>
static int launch_pn(const PrefillParams &p, hipStream_t stream)
{
    const size_t lds = prefill_lds_floats<P, N>() * sizeof(float);
    const dim3 grid(p.H, p.batch), block(256);
    hipError_t e;
    if (p.io == SSMV_BF16) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_kernel<P, N, SSMV_BF16>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        hipLaunchKernelGGL((prefill_kernel<P, N, SSMV_BF16>), grid, block, lds, stream, p);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_kernel<P, N, SSMV_F32>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        hipLaunchKernelGGL((prefill_kernel<P, N, SSMV_F32>), grid, block, lds, stream, p);
    }
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
    switch (p.P) {
        case 32: rc = launch_p<32>(p, stream); break;
        case 64: rc = launch_p<64>(p, stream); break;
        case 128: rc = launch_p<128>(p, stream); break;
        default: return (int)hipErrorInvalidConfiguration;
    }
    if (rc != 0) return rc;
    hipLaunchKernelGGL(prefill_finish_kernel, dim3((p.batch + 63) / 64), dim3(64), 0, stream, p.batch, p.L, p.ring_len, p.pos,
                       p.conv_head_rw, p.pend, p.last_k, p.err_flag);
    return (int)hipGetLastError();
}

}  // namespace ssmv
