// Internal declarations shared by the translation units of libssmv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ssmv.h"

namespace ssmv {

// ---- kernel parameter blocks (passed by value as kernel arguments) ---------------------------

struct VerifyParams {
    // shapes
    int batch, H, P, N, G, kmax, k;
    int io;              // SSMV_F32 | SSMV_BF16
    int rows_wg;         // state rows one workgroup owns
    int tiles;           // scalar mode: tiles per head; diag mode: tiles per sequence
    int lds_tokens;      // tokens the dynamic LDS was sized for (pend_max + k)
    int pend_max;        // largest legal pend: kmax-1, kmax when h_k is never stored, SSMV_WINDOW-kmax with a deferred advance
    int pend_hi;         // h_j is stored (and the commit moves the live slot there) iff pend > pend_hi; 0 unless SSMV_SNAP_DEFER
    int write_hk;        // 1: SSMV_SNAP_BOTH
    int win_ring;        // 1 (SSMV_SNAP_DEFER): the window is ONE ring of SSMV_WINDOW entries per sequence (both "halves" point
                         // to it), token q of the sequence at entry q % SSMV_WINDOW; 0: two halves of kmax entries
    int win_tokens;      // window entries per sequence and array: SSMV_WINDOW or kmax
    int tok0;            // tokens earlier calls have already fed to this round (0: first call)
    int pend_mask;       // tok0 > 0 ? 0 : ~0  (a later call replays nothing)
    int src_add;         // tok0 > 0 ? 2 : 0   (a later call continues in the h_k slot)
    int replay_tok;      // tokens of this round that the call replays out of the round's own stash (0, or tok0)
    int store_state;     // 0: a call of a replayed round that is not its last stores no snapshot
    int dt_softplus;     // 1: dt <- softplus(dt + dt_bias) before use
    const float *dt_bias;  // [nheads] or null
    const void *z;       // gate input [batch][k][channels] or null
    const int *k_seq;    // per-sequence draft counts [batch] or null
    int log2_rows_wg;    // rows_wg is a power of two
    int tiled;           // 1: the state slots are kept in 16x16 tiles (state_off4), scalar mode only
    // fused conv roll (x_raw != nullptr): ring append + width-4 conv computed while staging
    int ring_len, conv_act;
    void *ring;
    const int32_t *conv_head;
    const void *x_raw, *wgt, *bias;
    // cache
    float *state;        // [3][batch][H][P][N]
    size_t slot_stride;  // elements per slot
    void *win_xc[2];
    void *win_dt[2];
    void *win_B[2];
    const int32_t *cur_slot;
    const int32_t *pend;
    int32_t *last_k;
    const int32_t *win_par;
    const int64_t *pos;  // read with win_ring only
    // round inputs / outputs
    const void *xc, *dt, *Bm, *Cm;
    const float *A, *D;
    void *y;
    float *h_out;        // non-null: materialize mode (replay only, write here, touch nothing else)
};

struct ConvParams {
    int batch, Cx, k, R, io, act;
    void *ring;              // [batch][R][Cx]
    const int32_t *conv_head;
    const void *x_raw, *wgt, *bias;
    void *xc;
};

struct PrefillParams {
    int batch, H, P, N, G, L, io, ring_len, conv_act;   // L: token stride of the arrays = longest prompt
    int dt_softplus;         // 1: dt <- softplus(dt + dt_bias)
    int tiled;               // 1: the state slots are kept in 16x16 tiles (state_off4)
    const float *dt_bias;    // [H] or null
    const void *z;           // gate input [batch][L][H*P] or null
    const int32_t *seq_len;  // [batch] or null: prompt length per sequence (<= L)
    float *state;            // [3][batch][H][P][N]; the live slot is advanced in place
    size_t slot_stride;
    void *ring;
    const int32_t *cur_slot, *conv_head;
    const void *x_raw, *wgt, *bias, *dt, *Bm, *Cm;
    const float *A, *D;
    void *y;
    // bookkeeping advanced by the follow-up launch
    int64_t *pos;
    int32_t *conv_head_rw;
    const int32_t *pend, *last_k;
    int32_t *err_flag;
};

struct CacheInts {
    int32_t *cur_slot, *pend, *conv_head, *last_k, *win_par, *err_flag;
    int64_t *pos;
};

constexpr int kCommitMaxCaches = 32;     // caches one commit launch covers (kernel argument space)

struct CommitParams {
    int batch, R, n_caches;
    int mode;                // SSMV_SNAP_*
    int pend_hi;             // SSMV_SNAP_DEFER: the live slot moves iff pend > pend_hi
    const int32_t *accepted;
    CacheInts c[kCommitMaxCaches];
};

struct ResetParams {
    int batch, Cx, R, W, io;
    int P, N, tiled;         // rows and columns of one (sequence, head) block of the state, and its layout
    size_t state_elems;      // batch*H*P*N (slot 0 only)
    float *state;
    const float *h0;
    void *ring;
    const void *conv_init;
    int32_t *cur_slot, *pend, *conv_head, *last_k, *win_par, *err_flag;
    int64_t *pos;
};

// ---- launch shape -------------------------------------------------------------------------------

struct VerifyShape {
    int rows_per_lane;   // R
    int waves;           // waves per workgroup
};

// lanes that share one state row, and rows one wave covers per 16-byte load instruction
__host__ __device__ constexpr int lanes_per_row(int N) { return (N / 4 < 16) ? N / 4 : 16; }
__host__ __device__ constexpr int rows_per_instr(int N) { return 64 / lanes_per_row(N); }

// ---- layout of a state slot ---------------------------------------------------------------------
// A slot holds batch*H blocks of P rows x N fp32, one per (sequence, head).  Inside a block the layout is either plain
// row-major (element (p, n) at p*N + n) or TILED: 16x16 tiles in the register order of a 16x16 matrix-core accumulator.
// Tile (p/16, n/16) is 256 consecutive floats; inside it the four floats n%16 in [4g, 4g+4) of row p%16 are the float4
// number 16 g + p%16.  Lane l = 16 g + p%16 of a wave then holds, after ONE 16-byte access per lane that covers 1 KiB of
// contiguous memory, exactly its share of the tile as accumulator (rows n, columns p) - and the same registers are the
// k-slots of the other operand of a product that contracts over n.  Row-major memory would make that access 16 rows x 64
// bytes per instruction, which the memory system serves an eighth (loads) to a third (stores) slower.
// Tiled needs P and N to be multiples of 16; n is a multiple of 4 here.
__host__ __device__ inline size_t state_off4(bool tiled, int p, int n, int N)
{
    return tiled ? (((size_t)(p >> 4) * (N >> 4) + (n >> 4)) << 8) + ((((n & 15) >> 2) << 4) + (p & 15)) * 4 : (size_t)p * N + n;
}

// launchers implemented in verify_scalar.hip / verify_diag.hip; return hipError_t as int
int launch_verify_scalar(const VerifyParams &p, VerifyShape shape, hipStream_t stream);
int launch_verify_diag(const VerifyParams &p, VerifyShape shape, hipStream_t stream);
size_t verify_lds_bytes(const VerifyParams &p, bool diag);
// the matrix-core form of the scalar-mode kernel (verify_mfma.hip): bf16 I/O, tiled state, at most 16 tokens per launch
int launch_verify_mfma(const VerifyParams &p, hipStream_t stream);
bool verify_mfma_supported(int N, int P);
bool verify_shape_supported(int N, int R, bool diag);

int launch_conv(const ConvParams &p, hipStream_t stream);
int launch_prefill(const PrefillParams &p, hipStream_t stream);
int launch_prefill_bf16(const PrefillParams &p, hipStream_t stream);      // bf16 tensors: the main kernel only
bool prefill_shape_supported(int P, int N);
int launch_commit(const CommitParams &p, hipStream_t stream);
int launch_reset(const ResetParams &p, hipStream_t stream);
int launch_first_conflict(const int32_t *draft, const int32_t *target, int batch, int k, int32_t *accepted,
                          hipStream_t stream);
int launch_copy_probe(const void *src, void *dst0, void *dst1, size_t n_bytes, hipStream_t stream);
int launch_stream_probe(int mode, const void *src, void *dst0, void *dst1, size_t n_bytes, int piece_kib, int grid, hipStream_t stream);
int launch_gated_rmsnorm(const void *y, const void *z, const float *weight, int rows, int channels, int group, float eps, int io,
                         void *out, hipStream_t stream);

// Workgroups are dealt to the 8 XCDs (each with its own L2) round robin by their linear index.  This maps the linear
// index to a work item so that every XCD gets one contiguous range of items: the workgroups that share inputs (the
// heads of one sequence read the same B and C rows) then share an L2.  Identity when the count is no multiple of 8.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned wg, unsigned total)
{
    constexpr unsigned kXcds = 8;
    return total % kXcds == 0 ? (wg % kXcds) * (total / kXcds) + wg / kXcds : wg;
}

// ---- storage-type helpers (device) ----------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

// round-to-nearest-even; NaN stays NaN.  One v_cvt_pk_bf16_f32 on gfx950.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    const __bf16 r = static_cast<__bf16>(f);
    return __builtin_bit_cast(uint16_t, r);
}

// two values into one 32-bit word (first in the low half): one instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 b2_t __attribute__((ext_vector_type(2)));
    const f2_t v = {lo, hi};
    const b2_t r = __builtin_convertvector(v, b2_t);
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float load_io(const void *base, size_t idx, int io)
{
    if (io == SSMV_BF16) return bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(base)[idx]);
    return reinterpret_cast<const float *>(base)[idx];
}

__device__ __forceinline__ void store_io(void *base, size_t idx, float v, int io)
{
    if (io == SSMV_BF16)
        reinterpret_cast<uint16_t *>(base)[idx] = f32_to_bf16_bits(v);
    else
        reinterpret_cast<float *>(base)[idx] = v;
}

// softplus and SiLU on the hardware exp2/log2/rcp (about 1 ulp each); log(1+t) by its series where 1+t would lose the
// low bits of t
__device__ __forceinline__ float softplus_fast(float d)
{
    if (d > 20.f) return d;
    const float t = __builtin_amdgcn_exp2f(d * 1.4426950408889634f);
    const float series = t * (1.f - t * (0.5f - t * (0.33333334f - t * (0.25f - t * 0.2f))));
    return t < 0.0625f ? series : __builtin_amdgcn_logf(1.f + t) * 0.6931471805599453f;
}

__device__ __forceinline__ float silu_fast(float z)
{
    return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-z * 1.4426950408889634f));
}

// ---- 16-byte vector access in the I/O storage type -------------------------------------------------

template <int IO>
struct IoVec;

template <>
struct IoVec<SSMV_F32> {
    static constexpr int EV = 4;
    // raw 16-byte vector / raw scalar: load now, decode at the point of use
    static __device__ __forceinline__ uint4 load_raw(const void *base, size_t idx)
    {
        return *reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(base) + idx);
    }
    static __device__ __forceinline__ void store_raw(void *base, size_t idx, uint4 r)
    {
        *reinterpret_cast<uint4 *>(reinterpret_cast<float *>(base) + idx) = r;
    }
    static __device__ __forceinline__ void decode(uint4 r, float (&v)[4])
    {
        v[0] = __uint_as_float(r.x); v[1] = __uint_as_float(r.y); v[2] = __uint_as_float(r.z); v[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ uint4 encode(const float (&v)[4])
    {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    }
    static __device__ __forceinline__ uint32_t load_raw1(const void *base, size_t idx) { return reinterpret_cast<const uint32_t *>(base)[idx]; }
    static __device__ __forceinline__ void store_raw1(void *base, size_t idx, uint32_t r) { reinterpret_cast<uint32_t *>(base)[idx] = r; }
    static __device__ __forceinline__ float decode1(uint32_t r) { return __uint_as_float(r); }
    static __device__ __forceinline__ void load(const void *base, size_t idx, float (&v)[4])
    {
        const float4 t = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(base) + idx);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    static __device__ __forceinline__ void store(void *base, size_t idx, const float (&v)[4])
    {
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(base) + idx) = make_float4(v[0], v[1], v[2], v[3]);
    }
};

template <>
struct IoVec<SSMV_BF16> {
    static constexpr int EV = 8;
    static __device__ __forceinline__ uint4 load_raw(const void *base, size_t idx)
    {
        return *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(base) + idx);
    }
    static __device__ __forceinline__ void store_raw(void *base, size_t idx, uint4 r)
    {
        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(base) + idx) = r;
    }
    static __device__ __forceinline__ void decode(uint4 r, float (&v)[8])
    {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uint4 encode(const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
    static __device__ __forceinline__ uint32_t load_raw1(const void *base, size_t idx) { return reinterpret_cast<const uint16_t *>(base)[idx]; }
    static __device__ __forceinline__ void store_raw1(void *base, size_t idx, uint32_t r) { reinterpret_cast<uint16_t *>(base)[idx] = (uint16_t)r; }
    static __device__ __forceinline__ float decode1(uint32_t r) { return __uint_as_float(r << 16); }
    static __device__ __forceinline__ void load(const void *base, size_t idx, float (&v)[8])
    {
        const uint4 t = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(base) + idx);
        const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(void *base, size_t idx, const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(base) + idx) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// XW elements of the I/O type as one access: 16 bytes (XW == IoVec::EV) or 4 bytes (2 bf16 / 1 fp32)
template <int IO, int XW>
struct XVec {
    static_assert(XW == IoVec<IO>::EV, "16-byte case");
    using Raw = uint4;
    static __device__ __forceinline__ Raw zero() { return make_uint4(0, 0, 0, 0); }
    static __device__ __forceinline__ Raw load(const void *base, size_t idx) { return IoVec<IO>::load_raw(base, idx); }
    static __device__ __forceinline__ void store(void *base, size_t idx, Raw r) { IoVec<IO>::store_raw(base, idx, r); }
    static __device__ __forceinline__ void decode(Raw r, float (&v)[XW]) { IoVec<IO>::decode(r, v); }
    static __device__ __forceinline__ Raw encode(const float (&v)[XW]) { return IoVec<IO>::encode(v); }
};

template <>
struct XVec<SSMV_BF16, 2> {
    using Raw = uint32_t;
    static __device__ __forceinline__ Raw zero() { return 0u; }
    static __device__ __forceinline__ Raw load(const void *base, size_t idx)
    {
        return *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint16_t *>(base) + idx);
    }
    static __device__ __forceinline__ void store(void *base, size_t idx, Raw r)
    {
        *reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(base) + idx) = r;
    }
    static __device__ __forceinline__ void decode(Raw r, float (&v)[2])
    {
        v[0] = __uint_as_float(r << 16);
        v[1] = __uint_as_float(r & 0xffff0000u);
    }
    static __device__ __forceinline__ Raw encode(const float (&v)[2])
    {
        return pack_bf16x2(v[0], v[1]);
    }
};

template <>
struct XVec<SSMV_BF16, 4> {                                 // four bf16 values: 8 bytes
    using Raw = uint2;
    static __device__ __forceinline__ Raw zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ Raw load(const void *base, size_t idx)
    {
        return *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(base) + idx);
    }
    static __device__ __forceinline__ void store(void *base, size_t idx, Raw r)
    {
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(base) + idx) = r;
    }
    static __device__ __forceinline__ void decode(Raw r, float (&v)[4])
    {
        v[0] = __uint_as_float(r.x << 16);
        v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16);
        v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
    static __device__ __forceinline__ Raw encode(const float (&v)[4])
    {
        return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    }
};

template <>
struct XVec<SSMV_F32, 1> {
    using Raw = uint32_t;
    static __device__ __forceinline__ Raw zero() { return 0u; }
    static __device__ __forceinline__ Raw load(const void *base, size_t idx) { return reinterpret_cast<const uint32_t *>(base)[idx]; }
    static __device__ __forceinline__ void store(void *base, size_t idx, Raw r) { reinterpret_cast<uint32_t *>(base)[idx] = r; }
    static __device__ __forceinline__ void decode(Raw r, float (&v)[1]) { v[0] = __uint_as_float(r); }
    static __device__ __forceinline__ Raw encode(const float (&v)[1]) { return __float_as_uint(v[0]); }
};

}  // namespace ssmv
