// The C ABI of libssmv: argument validation on the host (before any HIP call, so the error
// paths run without a GPU), choice of the launch shape, and kernel launches.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "ssmv_internal.h"

using namespace ssmv;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(int hip_code, const char *what)
{
    return fail(SSMV_EHIP, "%s: %s", what, hipGetErrorString((hipError_t)hip_code));
}

std::atomic<int> g_tune_rows{0};
std::atomic<int> g_tune_waves{0};

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
size_t io_bytes(int io) { return io == SSMV_BF16 ? 2 : 4; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_dims(const ssmv_dims *d)
{
    if (!d) return fail(SSMV_EINVAL, "dims is NULL");
    if (d->batch < 1 || d->nheads < 1 || d->headdim < 1 || d->dstate < 1 || d->ngroups < 1)
        return fail(SSMV_EINVAL, "batch/nheads/headdim/dstate/ngroups must be >= 1");
    if (d->io_dtype != SSMV_F32 && d->io_dtype != SSMV_BF16) return fail(SSMV_EINVAL, "io_dtype %d unknown", d->io_dtype);
    if (d->a_mode != SSMV_A_SCALAR && d->a_mode != SSMV_A_DIAG) return fail(SSMV_EINVAL, "a_mode %d unknown", d->a_mode);
    if (d->conv_act != SSMV_ACT_NONE && d->conv_act != SSMV_ACT_SILU) return fail(SSMV_EINVAL, "conv_act %d unknown", d->conv_act);
    if (d->snapshot_mode != SSMV_SNAP_BOTH && d->snapshot_mode != SSMV_SNAP_HJ_ONLY && d->snapshot_mode != SSMV_SNAP_DEFER)
        return fail(SSMV_EINVAL, "snapshot_mode %d unknown", d->snapshot_mode);
    if (d->snapshot_mode == SSMV_SNAP_DEFER && 2 * d->kmax > SSMV_WINDOW)
        return fail(SSMV_EUNSUPPORTED, "SSMV_SNAP_DEFER keeps two rounds in a window of %d tokens: kmax %d > %d", SSMV_WINDOW, d->kmax,
                    SSMV_WINDOW / 2);
    if (d->engine != SSMV_ENGINE_AUTO && d->engine != SSMV_ENGINE_VECTOR) return fail(SSMV_EINVAL, "engine %d unknown", d->engine);
    if (d->nheads % d->ngroups != 0) return fail(SSMV_EINVAL, "nheads %d not a multiple of ngroups %d", d->nheads, d->ngroups);
    if ((long)d->conv_channels != (long)d->nheads * d->headdim)
        return fail(SSMV_EINVAL, "conv_channels %d != nheads*headdim %ld", d->conv_channels, (long)d->nheads * d->headdim);
    if (d->kmax < 1) return fail(SSMV_EINVAL, "kmax %d < 1", d->kmax);
    if (d->kmax > SSMV_KMAX_LIMIT) return fail(SSMV_EUNSUPPORTED, "kmax %d > %d", d->kmax, SSMV_KMAX_LIMIT);
    if (d->conv_width != SSMV_CONV_WIDTH) return fail(SSMV_EUNSUPPORTED, "conv_width %d (only %d)", d->conv_width, SSMV_CONV_WIDTH);
    if (!is_pow2(d->ring_len) || d->ring_len < d->conv_width - 1 + d->kmax)
        return fail(SSMV_EINVAL, "ring_len %d must be a power of two >= conv_width-1+kmax = %d", d->ring_len,
                    d->conv_width - 1 + d->kmax);
    if (d->dstate != 16 && d->dstate != 32 && d->dstate != 64 && d->dstate != 128 && d->dstate != 256)
        return fail(SSMV_EUNSUPPORTED, "dstate %d (supported: 16, 32, 64, 128, 256)", d->dstate);
    if (d->a_mode == SSMV_A_DIAG) {
        if (d->headdim != 1) return fail(SSMV_EINVAL, "diag mode needs headdim 1 (got %d)", d->headdim);
        if (d->ngroups != 1) return fail(SSMV_EUNSUPPORTED, "diag mode needs ngroups 1 (got %d)", d->ngroups);
        if (d->dstate > 64) return fail(SSMV_EUNSUPPORTED, "diag mode supports dstate <= 64 (got %d)", d->dstate);
    }
    if (d->batch > 65535) return fail(SSMV_EUNSUPPORTED, "batch %d > 65535", d->batch);
    // the kernels multiply token indices with these row lengths on the 24-bit multiplier
    if (d->conv_channels >= (1 << 22) || (long)d->ngroups * d->dstate >= (1 << 22) || d->nheads >= (1 << 22))
        return fail(SSMV_EUNSUPPORTED, "a token row of 2^22 elements or more (channels %d, groups*dstate %ld, heads %d)",
                    d->conv_channels, (long)d->ngroups * d->dstate, d->nheads);
    if (d->a_mode == SSMV_A_SCALAR && d->nheads > 65535) return fail(SSMV_EUNSUPPORTED, "nheads %d > 65535 in scalar mode", d->nheads);
    if ((double)d->batch * d->kmax * d->nheads * d->headdim >= 2.0e9 || (double)d->batch * d->ring_len * d->nheads * d->headdim >= 2.0e9)
        return fail(SSMV_EUNSUPPORTED, "token tensors beyond 2^31 elements");
    const double slot = (double)d->batch * d->nheads * d->headdim * d->dstate;
    if (slot * 3 > 2.0e10) return fail(SSMV_EUNSUPPORTED, "state of %.3g elements is beyond what one cache may hold", slot * 3);
    if ((double)d->batch * d->nheads * d->headdim > 2.0e9) return fail(SSMV_EUNSUPPORTED, "too many state rows");
    return SSMV_OK;
}

// Largest number of pending tokens a verify may meet.
int pend_max_of(const ssmv_dims *d)
{
    if (d->snapshot_mode == SSMV_SNAP_DEFER) return SSMV_WINDOW - d->kmax;
    return d->snapshot_mode == SSMV_SNAP_HJ_ONLY ? d->kmax : d->kmax - 1;
}
// A verify stores h_j, and its commit moves the live slot there, iff it meets more pending tokens than this.  With a
// deferred advance: as long as pend + (accepted <= kmax) + (next k <= kmax) still fits the window, nothing is stored.
int pend_hi_of(const ssmv_dims *d) { return d->snapshot_mode == SSMV_SNAP_DEFER ? SSMV_WINDOW - 2 * d->kmax : 0; }

// Whether the caches of these dimensions keep their state slots in 16x16 tiles (state_off4) and their verify launches run
// on the matrix cores: scalar-A mode, bf16 tokens, a shape that kernel is built for, and never more than 16 tokens
// (pending + drafts) in one launch.  A property of the dimensions, so every call on a cache agrees on it.
bool state_tiled(const ssmv_dims *d)
{
    return d->engine == SSMV_ENGINE_AUTO && d->a_mode == SSMV_A_SCALAR && d->io_dtype == SSMV_BF16 &&
           verify_mfma_supported(d->dstate, d->headdim) && pend_max_of(d) + d->kmax <= 16;
}

int check_ptr(const void *p, const char *name)
{
    if (!p) return fail(SSMV_EINVAL, "%s is NULL", name);
    if (!aligned16(p)) return fail(SSMV_EALIGN, "%s (%p) is not 16-byte aligned", name, p);
    return SSMV_OK;
}

int check_cache(const ssmv_cache *c)
{
    if (!c) return fail(SSMV_EINVAL, "cache is NULL");
    int rc;
#define CK(field) if ((rc = check_ptr(c->field, "cache." #field)) != SSMV_OK) return rc
    CK(state); CK(conv_ring);
    CK(win_xc[0]); CK(win_xc[1]); CK(win_dt[0]); CK(win_dt[1]); CK(win_B[0]); CK(win_B[1]);
    CK(cur_slot); CK(pend); CK(pos); CK(conv_head); CK(last_k); CK(win_par); CK(err_flag);
#undef CK
    return SSMV_OK;
}

int check_k(const ssmv_dims *d, int k)
{
    if (k < 1 || k > d->kmax) return fail(SSMV_EINVAL, "k %d outside [1, kmax=%d]", k, d->kmax);
    return SSMV_OK;
}

// rows per lane and waves per workgroup for the verify kernel
int choose_shape(const ssmv_dims *d, int lds_tokens, int k, bool gated, VerifyShape *out, int *rows_wg, int *tiles)
{
    const bool diag = d->a_mode == SSMV_A_DIAG;
    const int N = d->dstate;
    const int rpi = rows_per_instr(N);
    const int dom = diag ? d->nheads : d->headdim;          // rows of the tiled domain
    const long domains = diag ? d->batch : (long)d->batch * d->nheads;
    int R = g_tune_rows.load(), waves = g_tune_waves.load();
    if (R != 0 && !verify_shape_supported(N, R, diag)) return fail(SSMV_EUNSUPPORTED, "rows_per_lane %d not built for dstate %d", R, N);
    const bool autoR = R == 0, autoW = waves == 0;
    auto fits = [&](int r, int w) {
        VerifyParams q{};
        q.lds_tokens = lds_tokens; q.k = k; q.N = N; q.rows_wg = w * rpi * r;
        q.z = gated ? static_cast<const void *>(&q) : nullptr;      // only tested against null: LDS for the gate factors
        return verify_lds_bytes(q, diag) <= 64 * 1024;
    };
    if (autoR || autoW) {
        // Largest tile that still leaves >= 1024 workgroups (4 per compute unit) and does not
        // exceed the domain; otherwise the smallest tile, to spread a small problem over the chip.
        int bestR = -1, bestW = -1;
        long best_rows = -1;
        for (int r = 8; r >= 1; r /= 2) {
            if (!autoR && r != R) continue;
            if (!verify_shape_supported(N, r, diag)) continue;
            for (int w = 4; w >= 1; w /= 2) {
                if (!autoW && w != waves) continue;
                if (!fits(r, w)) continue;
                const int rw = w * rpi * r;
                const long t = (dom + rw - 1) / rw;
                const long groups = domains * t;
                const bool wasteful = rw > dom && rw > rpi;     // tile larger than the domain
                long score;                                                    // ties: more waves, fewer rows per lane
                if (groups >= 1024 && !wasteful) score = 1000000L + 16L * rw + w;   // big tiles first
                else score = wasteful ? -16L * rw + w : 500000L - 16L * rw + w;     // else the more groups the better
                if (score > best_rows) { best_rows = score; bestR = r; bestW = w; }
            }
        }
        if (bestR < 0) return fail(SSMV_EUNSUPPORTED, "no launch shape fits (dstate %d, tokens %d)", N, lds_tokens);
        R = bestR; waves = bestW;
    } else if (!fits(R, waves)) {
        return fail(SSMV_EUNSUPPORTED, "LDS need of the requested shape exceeds 64 KiB");
    }
    if (waves != 1 && waves != 2 && waves != 4) return fail(SSMV_EINVAL, "waves_per_group %d not in {1,2,4}", waves);
    out->rows_per_lane = R;
    out->waves = waves;
    *rows_wg = waves * rpi * R;
    *tiles = (dom + *rows_wg - 1) / *rows_wg;
    if (*tiles > 65535 * 32) return fail(SSMV_EUNSUPPORTED, "too many row tiles (%d)", *tiles);
    return SSMV_OK;
}

int ilog2_host(int v) { int l = 0; while ((1 << (l + 1)) <= v) ++l; return l; }

void fill_verify(VerifyParams &p, const ssmv_dims *d, const ssmv_cache *c)
{
    p.batch = d->batch; p.H = d->nheads; p.P = d->headdim; p.N = d->dstate; p.G = d->ngroups; p.kmax = d->kmax;
    p.io = d->io_dtype;
    p.state = c->state;
    p.slot_stride = (size_t)d->batch * d->nheads * d->headdim * d->dstate;
    p.win_ring = d->snapshot_mode == SSMV_SNAP_DEFER;
    p.win_tokens = p.win_ring ? SSMV_WINDOW : d->kmax;
    // (the ring is the first array of each pair; the kernels pick "the half" by the window parity and find the same array)
    for (int i = 0; i < 2; ++i) {
        const int j = p.win_ring ? 0 : i;
        p.win_xc[i] = c->win_xc[j]; p.win_dt[i] = c->win_dt[j]; p.win_B[i] = c->win_B[j];
    }
    p.pend_max = pend_max_of(d);
    p.pend_hi = pend_hi_of(d);
    p.cur_slot = c->cur_slot; p.pend = c->pend; p.last_k = c->last_k; p.win_par = c->win_par; p.pos = c->pos;
    p.ring = c->conv_ring; p.conv_head = c->conv_head; p.ring_len = d->ring_len; p.conv_act = d->conv_act;
    p.tiled = state_tiled(d);
}

}  // namespace

#ifdef SSMV_TRACE
// Profiling builds (-DSSMV_TRACE) only, no part of the library's interface: a device buffer of 8 wall-clock stamps per
// workgroup of the matrix-core verify kernel.
namespace ssmv { int set_trace_mfma(long long *buf); int set_trace_prefill(long long *buf); }
extern "C" int ssmv_debug_set_trace(long long *buf) { return ssmv::set_trace_mfma(buf); }
extern "C" int ssmv_debug_set_trace_prefill(long long *buf) { return ssmv::set_trace_prefill(buf); }
#endif

extern "C" {

const char *ssmv_last_error(void) { return g_err; }
const char *ssmv_version(void) { return "ssmv 0.1 (gfx950)"; }

int ssmv_set_tuning(int32_t rows_per_lane, int32_t waves_per_group)
{
    if (rows_per_lane != 0 && rows_per_lane != 1 && rows_per_lane != 2 && rows_per_lane != 4 && rows_per_lane != 8)
        return fail(SSMV_EINVAL, "rows_per_lane %d not in {0,1,2,4,8}", rows_per_lane);
    if (waves_per_group != 0 && waves_per_group != 1 && waves_per_group != 2 && waves_per_group != 4)
        return fail(SSMV_EINVAL, "waves_per_group %d not in {0,1,2,4}", waves_per_group);
    g_tune_rows.store(rows_per_lane);
    g_tune_waves.store(waves_per_group);
    return SSMV_OK;
}

int ssmv_engine_of(const ssmv_dims *d)
{
    const int rc = check_dims(d);
    if (rc != SSMV_OK) return rc;
    return state_tiled(d) ? 1 : 0;
}

int ssmv_cache_sizes(const ssmv_dims *d, size_t out_bytes[SSMV_CACHE_NPTR])
{
    int rc = check_dims(d);
    if (rc != SSMV_OK) return rc;
    if (!out_bytes) return fail(SSMV_EINVAL, "out_bytes is NULL");
    const size_t e = io_bytes(d->io_dtype);
    const size_t B = d->batch, H = d->nheads, P = d->headdim, N = d->dstate, G = d->ngroups, K = d->kmax, Cx = d->conv_channels;
    size_t *o = out_bytes;
    o[0] = 3 * B * H * P * N * sizeof(float);
    o[1] = B * d->ring_len * Cx * e;
    if (d->snapshot_mode == SSMV_SNAP_DEFER) {   // one ring of SSMV_WINDOW entries per sequence; the second arrays are not used
        o[2] = B * SSMV_WINDOW * Cx * e;
        o[4] = B * SSMV_WINDOW * H * e;
        o[6] = B * SSMV_WINDOW * G * N * e;
        o[3] = o[5] = o[7] = 256;
    } else {
        o[2] = o[3] = B * K * Cx * e;
        o[4] = o[5] = B * K * H * e;
        o[6] = o[7] = B * K * G * N * e;
    }
    o[8] = B * sizeof(int32_t);   // cur_slot
    o[9] = B * sizeof(int32_t);   // pend
    o[10] = B * sizeof(int64_t);  // pos
    o[11] = B * sizeof(int32_t);  // conv_head
    o[12] = B * sizeof(int32_t);  // last_k
    o[13] = sizeof(int32_t);      // win_par
    o[14] = sizeof(int32_t);      // err_flag
    for (int i = 0; i < SSMV_CACHE_NPTR; ++i) o[i] = (o[i] + 255) / 256 * 256;   // whole 256-byte granules
    return SSMV_OK;
}

int ssmv_cache_reset(const ssmv_dims *d, const ssmv_cache *c, const float *h0, const void *conv_init, void *hip_stream)
{
    int rc;
    if ((rc = check_dims(d)) != SSMV_OK) return rc;
    if ((rc = check_cache(c)) != SSMV_OK) return rc;
    if (h0 && !aligned16(h0)) return fail(SSMV_EALIGN, "h0 is not 16-byte aligned");
    if (conv_init && !aligned16(conv_init)) return fail(SSMV_EALIGN, "conv_init is not 16-byte aligned");
    ResetParams p{};
    p.batch = d->batch; p.Cx = d->conv_channels; p.R = d->ring_len; p.W = d->conv_width; p.io = d->io_dtype;
    p.state_elems = (size_t)d->batch * d->nheads * d->headdim * d->dstate;
    p.P = d->headdim; p.N = d->dstate; p.tiled = state_tiled(d);
    p.state = c->state; p.h0 = h0; p.ring = c->conv_ring; p.conv_init = conv_init;
    p.cur_slot = c->cur_slot; p.pend = c->pend; p.conv_head = c->conv_head; p.last_k = c->last_k;
    p.win_par = c->win_par; p.err_flag = c->err_flag; p.pos = c->pos;
    const int hc = launch_reset(p, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssmv_cache_reset");
}

int conv1d_state_update(const ssmv_dims *d, const ssmv_cache *c, const void *x_raw, const void *wgt, const void *bias,
                        int32_t k, void *xc_out, void *hip_stream)
{
    int rc;
    if ((rc = check_dims(d)) != SSMV_OK) return rc;
    if ((rc = check_cache(c)) != SSMV_OK) return rc;
    if ((rc = check_k(d, k)) != SSMV_OK) return rc;
    if ((rc = check_ptr(x_raw, "x_raw")) != SSMV_OK) return rc;
    if ((rc = check_ptr(wgt, "wgt")) != SSMV_OK) return rc;
    if ((rc = check_ptr(xc_out, "xc_out")) != SSMV_OK) return rc;
    if (bias && !aligned16(bias)) return fail(SSMV_EALIGN, "bias is not 16-byte aligned");
    ConvParams p{};
    p.batch = d->batch; p.Cx = d->conv_channels; p.k = k; p.R = d->ring_len; p.io = d->io_dtype; p.act = d->conv_act;
    p.ring = c->conv_ring; p.conv_head = c->conv_head; p.x_raw = x_raw; p.wgt = wgt; p.bias = bias; p.xc = xc_out;
    const int hc = launch_conv(p, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "conv1d_state_update");
}

static int verify_common(const ssmv_dims *d, const ssmv_cache *c, const ssmv_step_args *a, void *hip_stream, const char *what)
{
    int rc;
    if ((rc = check_dims(d)) != SSMV_OK) return rc;
    if ((rc = check_cache(c)) != SSMV_OK) return rc;
    if (!a) return fail(SSMV_EINVAL, "args is NULL");
    const int k = a->k;
    if ((rc = check_k(d, k)) != SSMV_OK) return rc;
    if (a->tok0 < 0 || a->tok0 + k > d->kmax) return fail(SSMV_EINVAL, "tok0 %d + k %d outside [0, kmax=%d]", a->tok0, k, d->kmax);
    if ((a->replay_round != 0 && a->replay_round != 1) || (a->last_call != 0 && a->last_call != 1))
        return fail(SSMV_EINVAL, "replay_round %d and last_call %d must be 0 or 1", a->replay_round, a->last_call);
    if (a->last_call && !a->replay_round) return fail(SSMV_EINVAL, "last_call is a flag of replay_round = 1");
    const bool replay = a->replay_round == 1;
    if (replay && (!state_tiled(d) || g_tune_rows.load() != 0 || g_tune_waves.load() != 0))
        return fail(SSMV_EUNSUPPORTED, "replay_round needs the matrix-core engine (see ssmv_engine_of) and no forced launch shape");
    if (a->tok0 > 0 && !replay && d->snapshot_mode != SSMV_SNAP_BOTH)
        return fail(SSMV_EUNSUPPORTED, "a round fed by several calls needs the h_k slot (SSMV_SNAP_BOTH) unless replay_round = 1");
    if (a->tok0 > 0 && a->k_seq)
        return fail(SSMV_EUNSUPPORTED, "ragged draft counts in a round fed by several calls (a sequence's window entries would not be contiguous)");
    if (a->dt_softplus != 0 && a->dt_softplus != 1) return fail(SSMV_EINVAL, "dt_softplus %d not in {0,1}", a->dt_softplus);
    if ((a->x_raw != nullptr) == (a->xc != nullptr)) return fail(SSMV_EINVAL, "exactly one of x_raw and xc must be given");
    if (a->xc && a->tok0 > 0)
        return fail(SSMV_EUNSUPPORTED, "a later call of a round (tok0 %d > 0) must pass x_raw: conv1d_state_update cannot append behind "
                                       "the round's earlier tokens", a->tok0);
    if (a->x_raw) {
        if ((rc = check_ptr(a->x_raw, "x_raw")) != SSMV_OK) return rc;
        if ((rc = check_ptr(a->conv_wgt, "wgt")) != SSMV_OK) return rc;
        if (a->conv_bias && !aligned16(a->conv_bias)) return fail(SSMV_EALIGN, "bias is not 16-byte aligned");
    } else {
        if ((rc = check_ptr(a->xc, "xc")) != SSMV_OK) return rc;
    }
    if ((rc = check_ptr(a->dt, "dt")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->Bm, "Bm")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->Cm, "Cm")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->A, "A")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->D, "D")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->y_out, "y_out")) != SSMV_OK) return rc;
    if (a->z && !aligned16(a->z)) return fail(SSMV_EALIGN, "z is not 16-byte aligned");
    if (a->k_seq && ((uintptr_t)a->k_seq & 3)) return fail(SSMV_EALIGN, "k_seq is not 4-byte aligned");
    if (a->dt_bias && ((uintptr_t)a->dt_bias & 3)) return fail(SSMV_EALIGN, "dt_bias is not 4-byte aligned");
    VerifyParams p{};
    fill_verify(p, d, c);
    p.k = k;
    p.tok0 = a->tok0;
    p.pend_mask = (a->tok0 > 0 && !replay) ? 0 : ~0;
    p.src_add = (a->tok0 > 0 && !replay) ? 2 : 0;
    p.replay_tok = replay ? a->tok0 : 0;
    p.store_state = (replay && !a->last_call) ? 0 : 1;
    p.dt_softplus = a->dt_softplus;
    p.dt_bias = a->dt_bias;
    p.z = a->z;
    p.k_seq = a->k_seq;
    p.write_hk = d->snapshot_mode == SSMV_SNAP_BOTH;
    p.lds_tokens = ((a->tok0 > 0 && !replay) ? 0 : p.pend_max) + p.replay_tok + k;
    p.xc = a->xc; p.dt = a->dt; p.Bm = a->Bm; p.Cm = a->Cm; p.A = a->A; p.D = a->D; p.y = a->y_out; p.h_out = nullptr;
    p.x_raw = a->x_raw; p.wgt = a->conv_wgt; p.bias = a->conv_bias;
    // tiled caches: the matrix-core kernel, unless a launch shape of the vector kernel was asked for explicitly
    if (p.tiled && g_tune_rows.load() == 0 && g_tune_waves.load() == 0) {
        const int hm = launch_verify_mfma(p, (hipStream_t)hip_stream);
        return hm == 0 ? SSMV_OK : hip_fail(hm, what);
    }
    VerifyShape shape;
    if ((rc = choose_shape(d, p.lds_tokens, k, p.z != nullptr, &shape, &p.rows_wg, &p.tiles)) != SSMV_OK) return rc;
    p.log2_rows_wg = ilog2_host(p.rows_wg);
    const int hc = d->a_mode == SSMV_A_DIAG ? launch_verify_diag(p, shape, (hipStream_t)hip_stream)
                                             : launch_verify_scalar(p, shape, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, what);
}

int ssm_verify_multistep(const ssmv_dims *d, const ssmv_cache *c, const void *xc, const void *dt, const void *Bm,
                         const void *Cm, const float *A, const float *D, int32_t k, void *y_out, void *hip_stream)
{
    if (!xc) return fail(SSMV_EINVAL, "xc is NULL");
    ssmv_step_args a{};
    a.xc = xc; a.dt = dt; a.Bm = Bm; a.Cm = Cm; a.A = A; a.D = D; a.k = k; a.y_out = y_out;
    return verify_common(d, c, &a, hip_stream, "ssm_verify_multistep");
}

int ssm_conv_verify_multistep(const ssmv_dims *d, const ssmv_cache *c, const void *x_raw, const void *wgt, const void *bias,
                              const void *dt, const void *Bm, const void *Cm, const float *A, const float *D, int32_t k,
                              void *y_out, void *hip_stream)
{
    if (!x_raw) return fail(SSMV_EINVAL, "x_raw is NULL");
    ssmv_step_args a{};
    a.x_raw = x_raw; a.conv_wgt = wgt; a.conv_bias = bias; a.dt = dt; a.Bm = Bm; a.Cm = Cm; a.A = A; a.D = D; a.k = k; a.y_out = y_out;
    return verify_common(d, c, &a, hip_stream, "ssm_conv_verify_multistep");
}

int ssm_block_multistep(const ssmv_dims *d, const ssmv_cache *c, const ssmv_step_args *args, void *hip_stream)
{
    return verify_common(d, c, args, hip_stream, "ssm_block_multistep");
}

int ssmv_materialize_block(const ssmv_dims *d, const ssmv_cache *c, const float *A, const float *dt_bias, int32_t dt_softplus,
                           float *h_out, void *hip_stream)
{
    int rc;
    if ((rc = check_dims(d)) != SSMV_OK) return rc;
    if ((rc = check_cache(c)) != SSMV_OK) return rc;
    if ((rc = check_ptr(A, "A")) != SSMV_OK) return rc;
    if ((rc = check_ptr(h_out, "h_out")) != SSMV_OK) return rc;
    if (dt_softplus != 0 && dt_softplus != 1) return fail(SSMV_EINVAL, "dt_softplus %d not in {0,1}", dt_softplus);
    VerifyParams p{};
    fill_verify(p, d, c);
    p.k = 0;
    p.pend_mask = ~0;
    p.dt_softplus = dt_softplus;
    p.dt_bias = dt_bias;
    p.write_hk = 0;
    p.lds_tokens = p.pend_max > 0 ? p.pend_max : 1;
    p.A = A; p.D = A;   // D is not read when k == 0
    p.h_out = h_out;
    VerifyShape shape;
    if ((rc = choose_shape(d, p.lds_tokens, 0, false, &shape, &p.rows_wg, &p.tiles)) != SSMV_OK) return rc;
    p.log2_rows_wg = ilog2_host(p.rows_wg);
    const int hc = d->a_mode == SSMV_A_DIAG ? launch_verify_diag(p, shape, (hipStream_t)hip_stream)
                                             : launch_verify_scalar(p, shape, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssmv_materialize");
}

int ssmv_materialize(const ssmv_dims *d, const ssmv_cache *c, const float *A, float *h_out, void *hip_stream)
{
    return ssmv_materialize_block(d, c, A, nullptr, 0, h_out, hip_stream);
}

int ssm_prefill_block(const ssmv_dims *d, const ssmv_cache *c, const ssmv_prefill_args *a, void *hip_stream)
{
    int rc;
    if ((rc = check_dims(d)) != SSMV_OK) return rc;
    if ((rc = check_cache(c)) != SSMV_OK) return rc;
    if (!a) return fail(SSMV_EINVAL, "args is NULL");
    if (a->L < 1) return fail(SSMV_EINVAL, "prompt length %d < 1", a->L);
    if (a->dt_softplus != 0 && a->dt_softplus != 1) return fail(SSMV_EINVAL, "dt_softplus %d not in {0,1}", a->dt_softplus);
    if (d->a_mode != SSMV_A_SCALAR) return fail(SSMV_EUNSUPPORTED, "the chunked prefill needs one decay per head (a_mode scalar)");
    if (!prefill_shape_supported(d->headdim, d->dstate))
        return fail(SSMV_EUNSUPPORTED, "chunked prefill is built for headdim in {32,64,128} and dstate in {32,64,128}, not %d x %d",
                    d->headdim, d->dstate);
    // the kernel addresses a sequence's tokens with 32-bit element offsets formed on the 24-bit multiplier
    // (x and y rows are conv_channels long, B and C rows ngroups*dstate, dt rows nheads)
    const double widest = (double)(d->conv_channels > d->ngroups * d->dstate ? d->conv_channels : d->ngroups * d->dstate);
    if (a->L >= (1 << 24) || (double)a->L * widest >= 2147483648.0)
        return fail(SSMV_EUNSUPPORTED, "a prompt of %d tokens x %.0f elements per token row does not fit 32-bit offsets: feed it in pieces",
                    a->L, widest);
    if ((rc = check_ptr(a->x_raw, "x_raw")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->conv_wgt, "wgt")) != SSMV_OK) return rc;
    if (a->conv_bias && !aligned16(a->conv_bias)) return fail(SSMV_EALIGN, "bias is not 16-byte aligned");
    if ((rc = check_ptr(a->dt, "dt")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->Bm, "Bm")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->Cm, "Cm")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->A, "A")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->D, "D")) != SSMV_OK) return rc;
    if ((rc = check_ptr(a->y_out, "y_out")) != SSMV_OK) return rc;
    if (a->z && !aligned16(a->z)) return fail(SSMV_EALIGN, "z is not 16-byte aligned");
    if (a->dt_bias && ((uintptr_t)a->dt_bias & 3)) return fail(SSMV_EALIGN, "dt_bias is not 4-byte aligned");
    if (a->seq_len && ((uintptr_t)a->seq_len & 3)) return fail(SSMV_EALIGN, "seq_len is not 4-byte aligned");
    PrefillParams p{};
    p.batch = d->batch; p.H = d->nheads; p.P = d->headdim; p.N = d->dstate; p.G = d->ngroups; p.L = a->L; p.io = d->io_dtype;
    p.ring_len = d->ring_len; p.conv_act = d->conv_act;
    p.dt_softplus = a->dt_softplus; p.dt_bias = a->dt_bias; p.z = a->z; p.seq_len = a->seq_len;
    p.tiled = state_tiled(d);
    p.state = c->state;
    p.slot_stride = (size_t)d->batch * d->nheads * d->headdim * d->dstate;
    p.ring = c->conv_ring; p.cur_slot = c->cur_slot; p.conv_head = c->conv_head;
    p.x_raw = a->x_raw; p.wgt = a->conv_wgt; p.bias = a->conv_bias; p.dt = a->dt; p.Bm = a->Bm; p.Cm = a->Cm; p.A = a->A; p.D = a->D;
    p.y = a->y_out;
    p.pos = c->pos; p.conv_head_rw = c->conv_head; p.pend = c->pend; p.last_k = c->last_k; p.err_flag = c->err_flag;
    const int hc = launch_prefill(p, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssm_prefill_block");
}

int ssm_prefill_chunked(const ssmv_dims *d, const ssmv_cache *c, const void *x_raw, const void *wgt, const void *bias,
                        const void *dt, const void *Bm, const void *Cm, const float *A, const float *D, int32_t L,
                        void *y_out, void *hip_stream)
{
    ssmv_prefill_args a{};
    a.x_raw = x_raw; a.conv_wgt = wgt; a.conv_bias = bias; a.dt = dt; a.Bm = Bm; a.Cm = Cm; a.A = A; a.D = D; a.L = L; a.y_out = y_out;
    return ssm_prefill_block(d, c, &a, hip_stream);
}

int ssm_commit_rollback_multi(const ssmv_dims *d, const ssmv_cache *caches, int32_t n_caches, const int32_t *accepted,
                              void *hip_stream)
{
    int rc;
    if ((rc = check_dims(d)) != SSMV_OK) return rc;
    if (!caches) return fail(SSMV_EINVAL, "caches is NULL");
    if (n_caches < 1) return fail(SSMV_EINVAL, "n_caches %d < 1", n_caches);
    for (int i = 0; i < n_caches; ++i)
        if ((rc = check_cache(&caches[i])) != SSMV_OK) return rc;
    if (!accepted) return fail(SSMV_EINVAL, "accepted is NULL");
    if ((reinterpret_cast<uintptr_t>(accepted) & 3u) != 0) return fail(SSMV_EALIGN, "accepted is not 4-byte aligned");
    for (int first = 0; first < n_caches; first += kCommitMaxCaches) {
        CommitParams p{};
        p.batch = d->batch; p.R = d->ring_len; p.accepted = accepted;
        p.mode = d->snapshot_mode;
        p.pend_hi = pend_hi_of(d);
        p.n_caches = n_caches - first < kCommitMaxCaches ? n_caches - first : kCommitMaxCaches;
        for (int i = 0; i < p.n_caches; ++i) {
            const ssmv_cache &c = caches[first + i];
            p.c[i] = CacheInts{c.cur_slot, c.pend, c.conv_head, c.last_k, c.win_par, c.err_flag, c.pos};
        }
        const int hc = launch_commit(p, (hipStream_t)hip_stream);
        if (hc != 0) return hip_fail(hc, "ssm_commit_rollback");
    }
    return SSMV_OK;
}

int ssm_commit_rollback(const ssmv_dims *d, const ssmv_cache *c, const int32_t *accepted, void *hip_stream)
{
    if (!c) return fail(SSMV_EINVAL, "cache is NULL");
    return ssm_commit_rollback_multi(d, c, 1, accepted, hip_stream);
}

int ssmv_first_conflict(const int32_t *draft, const int32_t *target, int32_t batch, int32_t k, int32_t *accepted,
                        void *hip_stream)
{
    if (!draft || !target || !accepted) return fail(SSMV_EINVAL, "draft/target/accepted is NULL");
    if (batch < 1 || k < 1) return fail(SSMV_EINVAL, "batch %d and k %d must be >= 1", batch, k);
    const int hc = launch_first_conflict(draft, target, batch, k, accepted, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssmv_first_conflict");
}

int ssmv_check(const ssmv_cache *c, void *hip_stream)
{
    if (!c || !c->err_flag) return fail(SSMV_EINVAL, "cache or cache.err_flag is NULL");
    int32_t flag = 0;
    hipError_t e = hipMemcpyAsync(&flag, c->err_flag, sizeof(flag), hipMemcpyDeviceToHost, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail((int)e, "ssmv_check copy");
    e = hipStreamSynchronize((hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail((int)e, "ssmv_check sync");
    if (flag != 0) return fail(SSMV_ESEQUENCE, "device flagged a bad accepted[] value or a commit without a verify");
    return SSMV_OK;
}

int ssmv_gated_rmsnorm(const void *y, const void *z, const float *weight, int32_t rows, int32_t channels, int32_t group_size,
                       float eps, int32_t io_dtype, void *out, void *hip_stream)
{
    int rc;
    if (io_dtype != SSMV_F32 && io_dtype != SSMV_BF16) return fail(SSMV_EINVAL, "io_dtype %d", io_dtype);
    const int ev = io_dtype == SSMV_BF16 ? 8 : 4;
    if (rows < 1 || rows > 65535 * 32 || channels < 1 || group_size < 1 || channels % group_size != 0)
        return fail(SSMV_EINVAL, "rows %d, channels %d, group_size %d", rows, channels, group_size);
    if (channels / group_size > 65535) return fail(SSMV_EUNSUPPORTED, "more than 65535 groups");
    if (group_size % ev != 0 || group_size > 256 * 4 * ev)
        return fail(SSMV_EUNSUPPORTED, "group_size %d must be a multiple of %d and at most %d", group_size, ev, 256 * 4 * ev);
    if (!(eps >= 0.f)) return fail(SSMV_EINVAL, "eps must be >= 0");
    if ((rc = check_ptr(y, "y")) != SSMV_OK) return rc;
    if (z && !aligned16(z)) return fail(SSMV_EALIGN, "z is not 16-byte aligned");
    if ((rc = check_ptr(weight, "weight")) != SSMV_OK) return rc;
    if ((rc = check_ptr(out, "out")) != SSMV_OK) return rc;
    const int hc = launch_gated_rmsnorm(y, z, weight, rows, channels, group_size, eps, io_dtype, out, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssmv_gated_rmsnorm");
}

int ssmv_stream_probe(int32_t mode, const void *src, void *dst0, void *dst1, size_t n_bytes, int32_t piece_kib, int32_t grid,
                      void *hip_stream)
{
    int rc;
    if (mode < SSMV_PROBE_READ || mode > SSMV_PROBE_EMPTY) return fail(SSMV_EINVAL, "mode %d unknown", mode);
    if (piece_kib != 4 && piece_kib != 8 && piece_kib != 32) return fail(SSMV_EINVAL, "piece_kib %d not in {4, 8, 32}", piece_kib);
    if (grid < 0) return fail(SSMV_EINVAL, "grid %d < 0", grid);
    if (n_bytes == 0 || n_bytes % ((size_t)piece_kib * 1024) != 0)
        return fail(SSMV_EINVAL, "n_bytes %zu must be a positive multiple of the piece size", n_bytes);
    if (mode != SSMV_PROBE_WRITE && mode != SSMV_PROBE_EMPTY && (rc = check_ptr(src, "src")) != SSMV_OK) return rc;
    if ((rc = check_ptr(dst0, "dst0")) != SSMV_OK) return rc;
    if (mode == SSMV_PROBE_R1W2 && (rc = check_ptr(dst1, "dst1")) != SSMV_OK) return rc;
    const int hc = launch_stream_probe(mode, src, dst0, dst1, n_bytes, piece_kib, grid, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssmv_stream_probe");
}

int ssmv_copy_probe(const void *src, void *dst0, void *dst1, size_t n_bytes, void *hip_stream)
{
    int rc;
    if ((rc = check_ptr(src, "src")) != SSMV_OK) return rc;
    if ((rc = check_ptr(dst0, "dst0")) != SSMV_OK) return rc;
    if (dst1 && !aligned16(dst1)) return fail(SSMV_EALIGN, "dst1 is not 16-byte aligned");
    if (n_bytes == 0 || (n_bytes & 15u) != 0) return fail(SSMV_EINVAL, "n_bytes %zu must be a positive multiple of 16", n_bytes);
    const int hc = launch_copy_probe(src, dst0, dst1, n_bytes, (hipStream_t)hip_stream);
    return hc == 0 ? SSMV_OK : hip_fail(hc, "ssmv_copy_probe");
}

}  // extern "C"
