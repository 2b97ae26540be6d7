// Small kernels around the fused verification kernel: the conv roll over the circular buffer
// (Section 4.3 footnote of arXiv 2408.15237), the integer commit/rollback of Algorithm 2,
// FirstConflict, cache reset, and a plain copy kernel for bandwidth calibration.
#include "ssmv_internal.h"

namespace ssmv {

// one element at a time, for channel counts that are no multiple of the 16-byte vector
template <int IO>
struct IoOne {
    static constexpr int EV = 1;
    static __device__ __forceinline__ void load(const void *base, size_t idx, float (&v)[1]) { v[0] = load_io(base, idx, IO); }
    static __device__ __forceinline__ void store(void *base, size_t idx, const float (&v)[1]) { store_io(base, idx, v[0], IO); }
};

// ---- conv roll -----------------------------------------------------------------------------------
// One thread owns VEC adjacent channels of one sequence for all k tokens: it reads the W-1 newest
// committed ring entries, then per new token appends the raw input to the ring and emits the
// width-4 causal dot product.  Ring slots written are head+1..head+k, slots read are
// head-2..head, disjoint because R >= W-1+kmax.
template <int IO, typename VT>
__global__ __launch_bounds__(256) void conv_kernel(const ConvParams p)
{
    constexpr int W = SSMV_CONV_WIDTH;
    constexpr int VEC = VT::EV;
    const int chunks = p.Cx / VEC;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (long)p.batch * chunks) return;
    const int b = (int)(gid / chunks);
    const int c0 = (int)(gid - (long)b * chunks) * VEC;
    const int head = p.conv_head[b];
    const int mask = p.R - 1;

    float hist[W - 1][VEC];
#pragma unroll
    for (int i = 0; i < W - 1; ++i)
        VT::load(p.ring, ((size_t)b * p.R + ((head - (W - 2) + i) & mask)) * p.Cx + c0, hist[i]);

    float w[VEC][W];
#pragma unroll
    for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int i = 0; i < W; ++i) w[c][i] = load_io(p.wgt, (size_t)(c0 + c) * W + i, IO);
    float bias[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) bias[c] = p.bias ? load_io(p.bias, c0 + c, IO) : 0.f;

    for (int t = 0; t < p.k; ++t) {
        float x[VEC], out[VEC];
        VT::load(p.x_raw, ((size_t)b * p.k + t) * p.Cx + c0, x);
        VT::store(p.ring, ((size_t)b * p.R + ((head + 1 + t) & mask)) * p.Cx + c0, x);
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float s = bias[c];
            s = fmaf(w[c][0], hist[0][c], s);
            s = fmaf(w[c][1], hist[1][c], s);
            s = fmaf(w[c][2], hist[2][c], s);
            s = fmaf(w[c][3], x[c], s);
            if (p.act == SSMV_ACT_SILU) s = s / (1.f + expf(-s));
            out[c] = s;
            hist[0][c] = hist[1][c];
            hist[1][c] = hist[2][c];
            hist[2][c] = x[c];
        }
        VT::store(p.xc, ((size_t)b * p.k + t) * p.Cx + c0, out);
    }
}

int launch_conv(const ConvParams &p, hipStream_t stream)
{
    const int vec = p.io == SSMV_BF16 ? 8 : 4;
    const bool vec_ok = (p.Cx % vec) == 0;
    const long threads = (long)p.batch * (vec_ok ? p.Cx / vec : p.Cx);
    const int block = 256;
    const unsigned grid = (unsigned)((threads + block - 1) / block);
    if (p.io == SSMV_BF16) {
        if (vec_ok) hipLaunchKernelGGL((conv_kernel<SSMV_BF16, IoVec<SSMV_BF16>>), dim3(grid), dim3(block), 0, stream, p);
        else hipLaunchKernelGGL((conv_kernel<SSMV_BF16, IoOne<SSMV_BF16>>), dim3(grid), dim3(block), 0, stream, p);
    } else {
        if (vec_ok) hipLaunchKernelGGL((conv_kernel<SSMV_F32, IoVec<SSMV_F32>>), dim3(grid), dim3(block), 0, stream, p);
        else hipLaunchKernelGGL((conv_kernel<SSMV_F32, IoOne<SSMV_F32>>), dim3(grid), dim3(block), 0, stream, p);
    }
    return (int)hipGetLastError();
}

// ---- commit / rollback (Algorithm 2: "return h_k if k'=k else h_j", lazily advanced cache) -----------
// grid.y = cache (layer), one thread per sequence.  Every load is issued before the first use:
// the kernel is a chain of memory latencies and nothing else.
__global__ __launch_bounds__(256) void commit_kernel(const CommitParams p)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= p.batch) return;
    const CacheInts &c = p.c[blockIdx.y];
    const int lk = c.last_k[b];
    int a = p.accepted[b];
    const int cur = c.cur_slot[b];
    const int pd = c.pend[b];
    const int head = c.conv_head[b];
    const int64_t pos = c.pos[b];
    const int par = b == 0 ? *c.win_par : 0;
    if (lk == 0) {                       // nothing was verified: leave everything, flag it
        *c.err_flag = 1;
        return;
    }
    if (a < 0 || a > lk) {
        *c.err_flag = 1;
        a = a < 0 ? 0 : lk;
    }
    if (p.mode == SSMV_SNAP_DEFER) {     // deferred advance: the live slot moves only when the verify stored h_j
        if (pd > p.pend_hi) {
            c.cur_slot[b] = (cur + 1) % 3;
            c.pos[b] = pos + pd;
            c.pend[b] = a;
        } else {
            c.pend[b] = pd + a;
        }
    } else if (a == lk && p.mode == SSMV_SNAP_BOTH) {   // every draft accepted: h_k becomes the live state
        c.cur_slot[b] = (cur + 2) % 3;
        c.pos[b] = pos + pd + a;
        c.pend[b] = 0;
    } else if (pd > 0) {                 // rejection: fall back to h_j, the accepted prefix stays pending
        c.cur_slot[b] = (cur + 1) % 3;
        c.pos[b] = pos + pd;
        c.pend[b] = a;
    } else {                             // rejection with nothing pending: the live slot already is h_j
        c.pend[b] = a;
    }
    c.conv_head[b] = (head + a) & (p.R - 1);
    c.last_k[b] = 0;
    if (b == 0) *c.win_par = par ^ 1;
}

int launch_commit(const CommitParams &p, hipStream_t stream)
{
    const int block = 256;
    hipLaunchKernelGGL(commit_kernel, dim3((p.batch + block - 1) / block, p.n_caches), dim3(block), 0, stream, p);
    return (int)hipGetLastError();
}

// ---- FirstConflict ----------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void first_conflict_kernel(const int32_t *draft, const int32_t *target, int batch, int k,
                                                             int32_t *accepted)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    int n = 0;
    while (n < k && draft[(size_t)b * k + n] == target[(size_t)b * k + n]) ++n;
    accepted[b] = n;
}

int launch_first_conflict(const int32_t *draft, const int32_t *target, int batch, int k, int32_t *accepted, hipStream_t stream)
{
    const int block = 256;
    hipLaunchKernelGGL(first_conflict_kernel, dim3((batch + block - 1) / block), dim3(block), 0, stream, draft, target, batch, k,
                       accepted);
    return (int)hipGetLastError();
}

// ---- reset (fill kernels, so that a caller may capture it in a graph) -----------------------------------
__global__ __launch_bounds__(256) void reset_state_kernel(const ResetParams p)
{
    const size_t n4 = p.state_elems / 4;       // N is a multiple of 4, so is the slot size
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p.h0) v = reinterpret_cast<const float4 *>(p.h0)[i];
        size_t o = i * 4;
        if (p.tiled) {                         // h0 is row-major; the slot keeps each (sequence, head) block in tiles
            const size_t blk = (size_t)p.P * p.N, head = o / blk, e = o - head * blk;
            o = head * blk + state_off4(true, (int)(e / p.N), (int)(e % p.N), p.N);
        }
        *reinterpret_cast<float4 *>(p.state + o) = v;
    }
}

__global__ __launch_bounds__(256) void reset_ring_kernel(const ResetParams p)
{
    const size_t n = (size_t)p.batch * p.R * p.Cx;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int c = (int)(i % p.Cx);
        const size_t br = i / p.Cx;
        const int slot = (int)(br % p.R);
        const int b = (int)(br / p.R);
        float v = 0.f;
        if (p.conv_init && slot < p.W - 1) v = load_io(p.conv_init, ((size_t)b * (p.W - 1) + slot) * p.Cx + c, p.io);
        store_io(p.ring, i, v, p.io);
    }
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (size_t b = gid; b < (size_t)p.batch; b += stride) {
        p.cur_slot[b] = 0;
        p.pend[b] = 0;
        p.pos[b] = 0;
        p.conv_head[b] = p.W - 2;
        p.last_k[b] = 0;
    }
    if (gid == 0) {
        *p.win_par = 0;
        *p.err_flag = 0;
    }
}

int launch_reset(const ResetParams &p, hipStream_t stream)
{
    const int block = 256;
    size_t n4 = p.state_elems / 4;
    unsigned g1 = (unsigned)((n4 + block - 1) / block);
    if (g1 > 8192) g1 = 8192;
    if (g1 == 0) g1 = 1;
    hipLaunchKernelGGL(reset_state_kernel, dim3(g1), dim3(block), 0, stream, p);
    size_t n = (size_t)p.batch * p.R * p.Cx;
    unsigned g2 = (unsigned)((n + block - 1) / block);
    if (g2 > 8192) g2 = 8192;
    if (g2 == 0) g2 = 1;
    hipLaunchKernelGGL(reset_ring_kernel, dim3(g2), dim3(block), 0, stream, p);
    return (int)hipGetLastError();
}

// ---- plain copy: read n bytes, write them once or twice ----------------------------------------------
typedef float copy_v4f __attribute__((ext_vector_type(4)));

// A workgroup copies contiguous tiles of 8 x 256 float4 (32 KiB): eight loads in flight per thread, then the
// stores - the verify kernel's shape - with the same streaming hints as its state traffic.
__global__ __launch_bounds__(256) void copy_probe_kernel(const copy_v4f *__restrict__ src, copy_v4f *__restrict__ dst0,
                                                         copy_v4f *__restrict__ dst1, size_t n16)
{
    constexpr int U = 8;
    const size_t tiles = (n16 + U * 256 - 1) / (U * 256);
    for (size_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const size_t base = tile * (U * 256) + threadIdx.x;
        copy_v4f v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = base + u * 256;
            v[u] = __builtin_nontemporal_load(src + (i < n16 ? i : n16 - 1));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = base + u * 256;
            if (i < n16) {
                __builtin_nontemporal_store(v[u], dst0 + i);
                if (dst1) __builtin_nontemporal_store(v[u], dst1 + i);
            }
        }
    }
}

// Gated RMS norm of a Mamba-2 block: g = y * z * sigmoid(z) (or y without z); out = g * rsqrt(mean_group(g^2) + eps) * w.
// `gt` threads (a multiple of 64, at least the group's 16-byte vectors up to 256) per (token row, group), 256 / gt groups of
// a row per workgroup; a thread takes 16-byte vectors of its group, the sum of squares goes through wave shuffles and
// one LDS slot per wave, and a second pass runs over the values kept in registers.
template <int IO>
__global__ __launch_bounds__(256) void gated_rmsnorm_kernel(const void *y, const void *z, const float *weight, int channels,
                                                            int group, int gt, float eps, void *out)
{
    using Vec = IoVec<IO>;
    constexpr int EV = Vec::EV;
    constexpr int MAXV = 4;                              // vectors per thread: groups of up to 256*4*EV channels
    __shared__ float partial[4];
    const int row = blockIdx.x, sub = threadIdx.x / gt, tid = threadIdx.x % gt;
    const int grp = blockIdx.y * (256 / gt) + sub;
    const bool have = grp < channels / group;            // the last workgroup of a row may hold fewer groups
    const size_t base = (size_t)row * channels + (size_t)(have ? grp : 0) * group;
    const int nvec = have ? group / EV : 0;
    float g[MAXV][EV];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int v = tid + i * gt;
        if (v < nvec) {
            Vec::load(y, base + (size_t)v * EV, g[i]);
            if (z) {
                float zv[EV];
                Vec::load(z, base + (size_t)v * EV, zv);
#pragma unroll
                for (int e = 0; e < EV; ++e) g[i][e] *= silu_fast(zv[e]);
            }
#pragma unroll
            for (int e = 0; e < EV; ++e) ss = fmaf(g[i][e], g[i][e], ss);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((threadIdx.x & 63) == 0) partial[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < gt / 64; ++w) tot += partial[sub * (gt / 64) + w];
    const float scale = rsqrtf(tot / (float)group + eps);
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int v = tid + i * gt;
        if (v < nvec) {
            float o[EV];
#pragma unroll
            for (int e = 0; e < EV; ++e) o[e] = g[i][e] * scale * weight[(size_t)grp * group + (size_t)v * EV + e];
            Vec::store(out, base + (size_t)v * EV, o);
        }
    }
}

int launch_gated_rmsnorm(const void *y, const void *z, const float *weight, int rows, int channels, int group, float eps, int io,
                         void *out, hipStream_t stream)
{
    const int nvec = group / (io == SSMV_BF16 ? 8 : 4);
    const int gt = nvec > 128 ? 256 : (nvec > 64 ? 128 : 64);       // threads per group
    const int gpb = 256 / gt, ngroups = channels / group;
    const dim3 grid(rows, (ngroups + gpb - 1) / gpb), block(256);
    if (io == SSMV_BF16) hipLaunchKernelGGL(gated_rmsnorm_kernel<SSMV_BF16>, grid, block, 0, stream, y, z, weight, channels, group, gt, eps, out);
    else hipLaunchKernelGGL(gated_rmsnorm_kernel<SSMV_F32>, grid, block, 0, stream, y, z, weight, channels, group, gt, eps, out);
    return (int)hipGetLastError();
}

// ---- bandwidth probe: what the memory system gives a plain stream of a given direction and shape --------------------------
// MODE 0 read only, 1 write only, 2 read 1 / write 1, 3 read 1 / write 2, 4 nothing (the floor of a launch).  A workgroup of
// 256 threads takes contiguous pieces of U x 4 KiB (a wave instruction = 1 KiB), non-temporal as the verify kernel's state.
template <int MODE, int U>
__global__ __launch_bounds__(256) void stream_probe_kernel(const copy_v4f *__restrict__ src, copy_v4f *__restrict__ dst0,
                                                           copy_v4f *__restrict__ dst1, size_t n16)
{
    if (MODE == 4) return;
    const size_t tiles = n16 / (U * 256);
    for (size_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const size_t base = tile * (U * 256) + threadIdx.x;
        copy_v4f v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = MODE == 1 ? copy_v4f{(float)tile, 1.f, 2.f, 3.f} : __builtin_nontemporal_load(src + base + u * 256);
        if (MODE == 0) {
            float a = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) a += v[u].x + v[u].y + v[u].z + v[u].w;
            if (a == 123.456f) dst0[base] = v[0];            // keeps the loads alive; practically never taken
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                __builtin_nontemporal_store(v[u], dst0 + base + u * 256);
                if (MODE == 3) __builtin_nontemporal_store(v[u], dst1 + base + u * 256);
            }
        }
    }
}

template <int MODE>
static void launch_probe_u(int u, unsigned grid, const copy_v4f *s, copy_v4f *d0, copy_v4f *d1, size_t n16, hipStream_t stream)
{
    if (u == 1) hipLaunchKernelGGL((stream_probe_kernel<MODE, 1>), dim3(grid), dim3(256), 0, stream, s, d0, d1, n16);
    else if (u == 2) hipLaunchKernelGGL((stream_probe_kernel<MODE, 2>), dim3(grid), dim3(256), 0, stream, s, d0, d1, n16);
    else hipLaunchKernelGGL((stream_probe_kernel<MODE, 8>), dim3(grid), dim3(256), 0, stream, s, d0, d1, n16);
}

int launch_stream_probe(int mode, const void *src, void *dst0, void *dst1, size_t n_bytes, int piece_kib, int grid, hipStream_t stream)
{
    const size_t n16 = n_bytes / 16;
    const int u = piece_kib / 4;
    const size_t tiles = n16 / ((size_t)u * 256);
    const unsigned g = grid > 0 ? (unsigned)grid : (unsigned)(tiles > 0x7fffffff ? 0x7fffffff : tiles);
    const copy_v4f *s = reinterpret_cast<const copy_v4f *>(src);
    copy_v4f *d0 = reinterpret_cast<copy_v4f *>(dst0), *d1 = reinterpret_cast<copy_v4f *>(dst1);
    switch (mode) {
        case 0: launch_probe_u<0>(u, g, s, d0, d1, n16, stream); break;
        case 1: launch_probe_u<1>(u, g, s, d0, d1, n16, stream); break;
        case 2: launch_probe_u<2>(u, g, s, d0, d1, n16, stream); break;
        case 3: launch_probe_u<3>(u, g, s, d0, d1, n16, stream); break;
        default: launch_probe_u<4>(u, g, s, d0, d1, n16, stream); break;
    }
    return (int)hipGetLastError();
}

int launch_copy_probe(const void *src, void *dst0, void *dst1, size_t n_bytes, hipStream_t stream)
{
    const size_t n16 = n_bytes / 16;
    const size_t tiles = (n16 + 8 * 256 - 1) / (8 * 256);
    const unsigned grid = (unsigned)(tiles > 65536 ? 65536 : tiles);
    hipLaunchKernelGGL(copy_probe_kernel, dim3(grid), dim3(256), 0, stream, reinterpret_cast<const copy_v4f *>(src),
                       reinterpret_cast<copy_v4f *>(dst0), reinterpret_cast<copy_v4f *>(dst1), n16);
    return (int)hipGetLastError();
}

}  // namespace ssmv
