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
    int lds_tokens;      // tokens the dynamic LDS was sized for (kmax-1+k)
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

struct CommitParams {
    int batch, R;
    int32_t *cur_slot, *pend, *conv_head, *last_k, *win_par, *err_flag;
    int64_t *pos;
    const int32_t *accepted;
};

struct ResetParams {
    int batch, Cx, R, W, io;
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

// launchers implemented in verify_scalar.hip / verify_diag.hip; return hipError_t as int
int launch_verify_scalar(const VerifyParams &p, VerifyShape shape, hipStream_t stream);
int launch_verify_diag(const VerifyParams &p, VerifyShape shape, hipStream_t stream);
size_t verify_lds_bytes(const VerifyParams &p, bool diag);
bool verify_shape_supported(int N, int R, bool diag);

int launch_conv(const ConvParams &p, hipStream_t stream);
int launch_commit(const CommitParams &p, hipStream_t stream);
int launch_reset(const ResetParams &p, hipStream_t stream);
int launch_first_conflict(const int32_t *draft, const int32_t *target, int batch, int k, int32_t *accepted,
                          hipStream_t stream);
int launch_copy_probe(const void *src, void *dst0, void *dst1, size_t n_bytes, hipStream_t stream);

// ---- storage-type helpers (device) ----------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
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

}  // namespace ssmv
