// Host side of the bf16 MFMA kernel families: support check, workspace layout and the launch
// sequences of the forward and backward passes.  Two sets of kernels: the chunked form for p = 2,
// d = v = 64, and the attention form (chunk == T, no state) for p in {2, 3, 4}, d = v in {32, 64, 128}.
#include "mfma_common.hpp"

namespace pa {
namespace {

using namespace mfma;

struct Layout {
    int cs, nstate;
    bool keep;
    size_t off_kt, off_vt, off_gam, off_sc;                      // forward
    size_t off_qt, off_gh, off_ght, off_gz, off_omg, off_rc;     // backward only
    size_t off_kts, off_qts;                                     // gated: copies of K, Q scaled for the scans
    size_t total;
};

// One layout serves both passes: the forward part comes first and the backward part is appended,
// so a forward pass that keeps its states leaves them where the backward pass looks for them.
Layout make_layout(const pa_problem& pr, bool backward) {
    Layout L{};
    L.cs = pr.chunk;
    L.nstate = pr.T / L.cs;
    L.keep = pr.keep_state != 0;
    const size_t BH = (size_t)pr.B * pr.H;
    const size_t tok = BH * pr.T * DH * 2;
    const size_t st = BH * L.nstate * (size_t)STATE_ELEMS * 2;
    const size_t gm = BH * L.nstate * (size_t)DH * DH * 2;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    L.off_kt = take(tok);
    L.off_vt = take(tok);
    L.off_gam = take(gm);
    L.off_sc = take(st);
    L.off_kts = pr.gated ? take(tok) : L.off_kt;
    L.off_qts = 0;
    if (backward || L.keep) {
        L.off_qt = take(tok);
        L.off_gh = take(tok);
        L.off_ght = take(tok);
        L.off_gz = take(BH * pr.T * sizeof(float));
        L.off_omg = take(gm);
        L.off_rc = take(st);
        L.off_qts = pr.gated ? take(tok) : L.off_qt;
    }
    L.total = off;
    return L;
}

// resident-state kernels: workspace of the forward pass (the backward part is appended)
struct ResLayout {
    ResidentPlan pl;
    size_t off_kt, off_vt, off_gam, off_gram, off_tot, off_part, off_zpart;
    size_t off_qt, off_ght, off_gh, off_gz, off_omg, off_totr, off_pdq, off_pdk;   // backward only
    size_t total;
};
ResLayout make_res_layout(const pa_problem& pr, bool backward) {
    ResLayout L{};
    const int BH = pr.B * pr.H;
    L.pl = resident_plan(pr.d, BH, pr.T, pr.chunk);
    const size_t tok = (size_t)BH * pr.T * pr.d * 2;
    const size_t gm = (size_t)BH * (pr.T / pr.chunk) * pr.d * pr.d * 2;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    L.off_kt = take(tok);
    L.off_vt = take(tok);
    L.off_gam = take(gm);
    L.off_gram = take(L.pl.gram_bytes);
    L.off_tot = take(L.pl.tot_bytes);
    L.off_part = take(L.pl.part_bytes);
    L.off_zpart = take((size_t)BH * pr.T * sizeof(float));
    if (backward || pr.keep_state) {
        const size_t slab = (size_t)BH * pr.T * pr.d * sizeof(float);
        L.off_qt = take(tok);
        L.off_ght = take(tok);
        L.off_gh = take(tok);
        L.off_gz = take((size_t)BH * pr.T * sizeof(float));
        L.off_omg = take(gm);
        L.off_totr = take(L.pl.tot_bytes);
        L.off_pdq = take((L.pl.nslab + 1) * slab);     // the last slab is the normaliser's share
        L.off_pdk = take((L.pl.nslab + 1) * slab);
    }
    L.total = off;
    return L;
}
bool resident_ok(const pa_problem& pr) {
    return pr.dtype == PA_DTYPE_BF16 && pr.p == 2 && (pr.d == 64 || pr.d == 128) && pr.v == pr.d && pr.chunk > 0 &&
           pr.chunk % QBLK == 0 && pr.T % pr.chunk == 0 && !pr.gated && (size_t)pr.B * pr.H <= 65535u;
}
bool chunked_ok(const pa_problem& pr) {
    return pr.dtype == PA_DTYPE_BF16 && pr.p == 2 && pr.d == DH && pr.v == DH && pr.chunk % QBLK == 0 &&
           (size_t)pr.B * pr.H <= 65535u;
}
// gated: the boundary sums of the gate gradient are kept per block of keys of the dK / dV kernel
bool attn_ok(const pa_problem& pr) {
    return pr.dtype == PA_DTYPE_BF16 && pr.d == pr.v && attn_shape_ok(pr.p, pr.d) && pr.chunk == pr.T &&
           (!pr.gated || pr.T % attn_gate_block(pr.d) == 0) && (size_t)pr.B * pr.H <= 65535u;
}
// One chunk: the attention-form kernels.  (The chunked kernels can run p = 2, d = 64 as one chunk
// too; that path remains for gated sequences that are a multiple of 128 but not of the block.)
bool use_attn(const pa_problem& pr) { return attn_ok(pr) && pr.impl != PA_IMPL_RESIDENT && pr.impl != PA_IMPL_TILED; }
bool use_tiled(const pa_problem& pr);
// The resident-state kernels run when asked for by name, and wherever they are the only matrix-core kernels
// for the chunked form
bool use_resident(const pa_problem& pr) {
    if (pr.impl == PA_IMPL_TILED || !resident_ok(pr)) return false;
    return pr.impl == PA_IMPL_RESIDENT || (!chunked_ok(pr) && !attn_ok(pr) && !use_tiled(pr));
}

// tiled kernels (any degree and tile width, chunk states in memory): workspace of the forward pass, the backward
// part appended
struct TiledLayout {
    TiledPlan pl;
    size_t off_tab, off_vp, off_sc, off_part, off_zpart;
    size_t off_gh, off_gz, off_gp, off_rc, off_pdq, off_pdk;   // backward only
    size_t total;
};
int tiled_dt(const pa_problem& pr) { return pr.d_tile > 0 ? pr.d_tile : tiled_default_dt(pr.p); }
TiledLayout make_tiled_layout(const pa_problem& pr, bool backward) {
    TiledLayout L{};
    const size_t BH = (size_t)pr.B * pr.H;
    L.pl = tiled_plan(pr.p, pr.d, tiled_dt(pr));
    const size_t rows = BH * pr.T;
    const size_t st = BH * (pr.T / pr.chunk) * L.pl.state_elems * 2;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    L.off_tab = take((size_t)L.pl.nentry * sizeof(TileDesc));
    L.off_vp = take(rows * L.pl.vp * 2);
    L.off_sc = take(st);
    L.off_part = take(rows * pr.d * sizeof(float));
    L.off_zpart = take(rows * sizeof(float));
    if (backward || pr.keep_state) {
        L.off_gh = take(rows * pr.d * 2);
        L.off_gz = take(rows * sizeof(float));
        L.off_gp = take(rows * L.pl.vp * 2);
        L.off_rc = take(st);
        L.off_pdq = take(rows * pr.d * sizeof(float));
        L.off_pdk = take(rows * pr.d * sizeof(float));
    }
    L.total = off;
    return L;
}
bool tiled_ok(const pa_problem& pr) {
    return pr.dtype == PA_DTYPE_BF16 && pr.d == pr.v && pr.chunk > 0 && pr.chunk % QBLK == 0 && pr.T % pr.chunk == 0 &&
           pr.chunk < pr.T && !pr.gated && tiled_shape_ok(pr.p, pr.d, tiled_dt(pr)) && (size_t)pr.B * pr.H <= 65535u;
}

// attention form, backward: ghat (bf16) and gz (float32) per token
struct AttnLayout {
    size_t off_gh, off_gz, off_wsum, total;
};
AttnLayout make_attn_layout(const pa_problem& pr, bool backward) {
    AttnLayout L{};
    if (!backward) return L;
    const size_t rows = (size_t)pr.B * pr.H * pr.T;
    L.off_gh = 0;
    L.off_gz = align_up(rows * pr.d * 2, 256);
    L.off_wsum = L.off_gz + align_up(rows * sizeof(float), 256);
    L.total = L.off_wsum;
    if (pr.gated) {
        const size_t nblk = (size_t)(pr.T / attn_gate_block(pr.d));
        L.total += align_up((size_t)pr.B * pr.H * nblk * nblk * 4 * sizeof(float), 256);
    }
    return L;
}

// The tiled kernels run when asked for by name or for a tile width, and wherever no other matrix-core kernel takes the
// chunked form of the problem (degrees 3 and 4, d = 32) or they are the faster ones (d = 128: measured against the
// resident-state walk, which has to cut the state into slabs there)
bool use_tiled(const pa_problem& pr) {
    if (!tiled_ok(pr)) return false;
    if (pr.impl == PA_IMPL_TILED) return true;
    if (pr.impl == PA_IMPL_RESIDENT) return false;
    return pr.d_tile > 0 || (!chunked_ok(pr) && !attn_ok(pr));
}

}  // namespace

int mfma_gate_fin_chunk(const pa_problem& pr) { return use_attn(pr) ? attn_gate_block(pr.d) : pr.chunk; }

pa_status mfma_supported(const pa_problem& pr, bool backward) {
    if (pr.impl == PA_IMPL_RESIDENT) return resident_ok(pr) ? PA_OK : PA_ERR_UNSUPPORTED;
    if (pr.impl == PA_IMPL_TILED || pr.d_tile > 0) return tiled_ok(pr) ? PA_OK : PA_ERR_UNSUPPORTED;
    return chunked_ok(pr) || attn_ok(pr) || resident_ok(pr) || tiled_ok(pr) ? PA_OK : PA_ERR_UNSUPPORTED;
}

long long mfma_state_rows(const pa_problem& pr) {
    if (use_tiled(pr)) {
        const TiledPlan pl = tiled_plan(pr.p, pr.d, tiled_dt(pr));
        return (long long)pl.ntile * pl.rows_per_tile;
    }
    if (use_resident(pr)) return (long long)(pr.d / 8) * (pr.d / 8 + 1) / 2 * 64;
    return use_attn(pr) ? 0 : (long long)NTILES * 64;
}

size_t mfma_workspace_bytes(const pa_problem& pr, bool backward) {
    if (use_tiled(pr)) return make_tiled_layout(pr, backward).total;
    if (use_resident(pr)) return make_res_layout(pr, backward).total;
    return use_attn(pr) ? make_attn_layout(pr, backward).total : make_layout(pr, backward).total;
}

#define PA_TRY(CALL) \
    if (!(CALL)) return PA_ERR_HIP;

// Gated problems (c.gate non-null): the scans read copies of K (Q in the backward pass) scaled by
// the square root of the per-token decay, and multiply the running sum by the per-chunk decay;
// the per-chunk kernels apply the remaining factors (see the chunk kernels).
pa_status mfma_fwd(const Ctx& c, const void* Q, const void* K, const void* V, void* O, float* Z) {
    const pa_problem& pr = c.prob;
    const int BH = pr.B * pr.H;
    if (use_attn(pr)) {
        PA_TRY(launch_attn_fwd(c.stream, pr.p, pr.d, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (bf16_t*)O, Z, BH, pr.T,
                               pr.scale, pr.normalize, c.gate.bl))
        return PA_OK;
    }
    if (use_tiled(pr)) {
        // tile table, values extended by the normaliser's one, state scan, read-out; the in-chunk part and the
        // division on the chunk-local attention kernel
        const TiledLayout L = make_tiled_layout(pr, pr.keep_state != 0);
        TileDesc* tab = (TileDesc*)(c.ws + L.off_tab);
        bf16_t* Vp = (bf16_t*)(c.ws + L.off_vp);
        bf16_t* Sc = (bf16_t*)(c.ws + L.off_sc);
        float* part = (float*)(c.ws + L.off_part);
        float* zpart = (float*)(c.ws + L.off_zpart);
        PA_TRY(launch_tiled_table(c.stream, L.pl, tab))
        PA_TRY(launch_tiled_pack(c.stream, pr.d, (const bf16_t*)V, nullptr, Vp, (long long)BH * pr.T))
        PA_TRY(launch_tiled_scan("tiled_state_scan", c.stream, L.pl, false, (const bf16_t*)K, Vp, tab, Sc, BH, pr.T, pr.chunk, 1.0f))
        PA_TRY(launch_tiled_readout("tiled_query_state", c.stream, L.pl, (const bf16_t*)Q, tab, Sc, part, zpart, BH, pr.T, pr.chunk,
                                    pr.scale))
        PA_TRY(launch_chunk_fwd(c.stream, pr.p, pr.d, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (bf16_t*)O, Z, BH, pr.T,
                                pr.chunk, pr.scale, pr.normalize, part, 1, zpart))
        return PA_OK;
    }
    if (use_resident(pr)) {
        const ResLayout R = make_res_layout(pr, pr.keep_state != 0);
        bf16_t* Kt = (bf16_t*)(c.ws + R.off_kt);
        bf16_t* Vt = (bf16_t*)(c.ws + R.off_vt);
        bf16_t* Gam = (bf16_t*)(c.ws + R.off_gam);
        float* gram = (float*)(c.ws + R.off_gram);
        float* tot = (float*)(c.ws + R.off_tot);
        float* part = (float*)(c.ws + R.off_part);
        float* zpart = (float*)(c.ws + R.off_zpart);
        PA_TRY(launch_transpose_hd(c.stream, pr.d, (const bf16_t*)K, Kt, BH, pr.T))
        PA_TRY(launch_transpose_hd(c.stream, pr.d, (const bf16_t*)V, Vt, BH, pr.T))
        PA_TRY(launch_gram(c.stream, pr.d, Kt, nullptr, gram, Gam, BH, pr.T, pr.chunk, false, 1.0f))
        if (R.pl.nseg > 1)
            PA_TRY(launch_res_walk("res_state_totals", c.stream, pr.d, false, 0, Kt, Vt, nullptr, nullptr, tot, nullptr, BH, pr.T,
                                   pr.chunk, R.pl, 1.0f))
        PA_TRY(launch_res_walk("res_state_walk", c.stream, pr.d, false, 1, Kt, Vt, (const bf16_t*)Q, nullptr, tot, part, BH, pr.T,
                               pr.chunk, R.pl, pr.scale * pr.scale))
        if (pr.d == DH) {
            PA_TRY(launch_fwd_chunk(c.stream, (const bf16_t*)Q, (const bf16_t*)K, Vt, nullptr, Gam, (bf16_t*)O, Z, BH, pr.T,
                                    pr.chunk, pr.scale, pr.normalize, nullptr, nullptr, part, R.pl.nslab))
        } else {
            // the normaliser's share of the denominator, then the in-chunk part on the attention-form kernel
            PA_TRY(launch_gram_apply(c.stream, pr.d, (const bf16_t*)Q, Gam, nullptr, nullptr, zpart, BH, pr.T, pr.chunk, 0.f,
                                     pr.scale * pr.scale))
            PA_TRY(launch_chunk_fwd(c.stream, pr.p, pr.d, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (bf16_t*)O, Z, BH,
                                    pr.T, pr.chunk, pr.scale, pr.normalize, part, R.pl.nslab, zpart))
        }
        return PA_OK;
    }
    const Layout L = make_layout(pr, false);
    const GateBuf& gt = c.gate;
    bf16_t* Kt = (bf16_t*)(c.ws + L.off_kt);
    bf16_t* Kts = (bf16_t*)(c.ws + L.off_kts);
    bf16_t* Vt = (bf16_t*)(c.ws + L.off_vt);
    bf16_t* Sc = (bf16_t*)(c.ws + L.off_sc);
    bf16_t* Gam = (bf16_t*)(c.ws + L.off_gam);
    if (!pr.gated || L.keep)   // the plain copy of K serves the scan (un-gated) and the backward pass's dQ
        PA_TRY(launch_transpose(c.stream, (const bf16_t*)K, Kt, BH, pr.T))
    if (pr.gated) PA_TRY(launch_transpose(c.stream, (const bf16_t*)K, Kts, BH, pr.T, gt.kfac))
    PA_TRY(launch_transpose(c.stream, (const bf16_t*)V, Vt, BH, pr.T))
    PA_TRY(launch_scan("mfma_state_scan", c.stream, false, Kts, Vt, nullptr, Sc, Gam, BH, pr.T, L.cs, 1.0f, gt.lam))
    PA_TRY(launch_fwd_chunk(c.stream, (const bf16_t*)Q, (const bf16_t*)K, Vt, Sc, Gam, (bf16_t*)O, Z, BH, pr.T, L.cs,
                            pr.scale, pr.normalize, gt.bl, gt.qfac))
    return PA_OK;
}

// The backward pass has two independent strands that meet only at the end: dQ needs the forward
// state S, while dK / dV need the state gradient R, whose scan is a long chain of small steps
// that leaves most of each CU idle.  The R strand therefore runs on a second stream (created
// once, default priority) so that dQ's workgroups fill the CUs under the scan.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, scanned = nullptr;
    bool ok = false;
    int device = -1;
};
// One side stream per host thread (so that calls from several threads never share one), bound to the
// device of the thread's first backward call; a call on any other device simply runs both strands on the
// caller's stream.  power_attn_release_thread() destroys it.
static thread_local SideStream t_side;
static SideStream side_stream() {
    SideStream& s = t_side;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SideStream{};
    if (s.device < 0) {
        s.device = dev;
        s.ok = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess &&
               hipEventCreateWithFlags(&s.fork, hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&s.join, hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&s.scanned, hipEventDisableTiming) == hipSuccess;
    }
    return s.device == dev ? s : SideStream{};
}

void mfma_release_side_stream() {
    SideStream& s = t_side;
    if (s.stream != nullptr) (void)hipStreamDestroy(s.stream);
    if (s.fork != nullptr) (void)hipEventDestroy(s.fork);
    if (s.join != nullptr) (void)hipEventDestroy(s.join);
    if (s.scanned != nullptr) (void)hipEventDestroy(s.scanned);
    s = SideStream{};
}

pa_status mfma_bwd(const Ctx& c, const void* Q, const void* K, const void* V, const void* O, const float* Z,
                   const void* dO, void* dQ, void* dK, void* dV) {
    const pa_problem& pr = c.prob;
    const int BH = pr.B * pr.H;
    if (use_attn(pr)) {
        const AttnLayout A = make_attn_layout(pr, true);
        AttnGate ag;
        if (pr.gated) {
            ag.bl = c.gate.bl;       // with chunk == T: running sums from the start of the sequence
            ag.qdq = c.gate.db;
            ag.kdk = c.gate.db2;
            ag.xb = c.gate.xb;
            ag.wsum = (float*)(c.ws + A.off_wsum);
        }
        PA_TRY(launch_attn_bwd(c.stream, pr.p, pr.d, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)O, Z,
                               (const bf16_t*)dO, (bf16_t*)(c.ws + A.off_gh), (float*)(c.ws + A.off_gz), (bf16_t*)dQ, (bf16_t*)dK,
                               (bf16_t*)dV, BH, pr.T, pr.scale, pr.normalize, ag))
        return PA_OK;
    }
    if (use_tiled(pr)) {
        // dQ's state part from S and [ghat, gz]; the state gradient R from phi(q) [ghat, gz]^T, read out with phi(k) for
        // dV and contracted with [v, 1] for dK; one kernel then adds the in-chunk gradients
        const TiledLayout L = make_tiled_layout(pr, true);
        TileDesc* tab = (TileDesc*)(c.ws + L.off_tab);
        bf16_t* Vp = (bf16_t*)(c.ws + L.off_vp);
        bf16_t* Sc = (bf16_t*)(c.ws + L.off_sc);
        bf16_t* Gh = (bf16_t*)(c.ws + L.off_gh);
        float* gz = (float*)(c.ws + L.off_gz);
        bf16_t* Gp = (bf16_t*)(c.ws + L.off_gp);
        bf16_t* Rc = (bf16_t*)(c.ws + L.off_rc);
        float* pdv = (float*)(c.ws + L.off_part);
        float* pdq = (float*)(c.ws + L.off_pdq);
        float* pdk = (float*)(c.ws + L.off_pdk);
        const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V;
        const long long rows = (long long)BH * pr.T;
        hipStream_t st = c.stream;
        PA_TRY(launch_attn_prep(st, pr.d, (const bf16_t*)dO, (const bf16_t*)O, Z, Gh, gz, rows, pr.normalize))
        PA_TRY(launch_tiled_pack(st, pr.d, Gh, gz, Gp, rows))
        if (!pr.keep_state) {
            PA_TRY(launch_tiled_table(st, L.pl, tab))
            PA_TRY(launch_tiled_pack(st, pr.d, v, nullptr, Vp, rows))
            PA_TRY(launch_tiled_scan("tiled_state_scan_bwd", st, L.pl, false, k, Vp, tab, Sc, BH, pr.T, pr.chunk, 1.0f))
        }
        PA_TRY(launch_tiled_dphi("tiled_dq", st, L.pl, q, Gp, tab, Sc, pdq, BH, pr.T, pr.chunk, pr.scale, pr.scale))
        PA_TRY(launch_tiled_scan("tiled_state_grad_scan", st, L.pl, true, q, Gp, tab, Rc, BH, pr.T, pr.chunk, pr.scale))
        PA_TRY(launch_tiled_readout("tiled_dv", st, L.pl, k, tab, Rc, pdv, nullptr, BH, pr.T, pr.chunk, 1.0f))
        PA_TRY(launch_tiled_dphi("tiled_dk", st, L.pl, k, Vp, tab, Rc, pdk, BH, pr.T, pr.chunk, 1.0f, 1.0f))
        PA_TRY(launch_chunk_bwd(st, pr.p, pr.d, q, k, v, Gh, gz, (bf16_t*)dQ, (bf16_t*)dK, (bf16_t*)dV, BH, pr.T, pr.chunk, pr.scale,
                                pdq, 1, pdk, 1, pdv, 1))
        return PA_OK;
    }
    if (use_resident(pr)) {
        // Every part that goes through a state is left per slab in float32 by a walk that keeps that state in
        // registers: J_phi(q)^T (S ghat) for dQ from a forward walk, R^T phi(k) for dV and J_phi(k)^T (R v) for dK
        // from two backward walks over R (the two contractions want the accumulators in different orientations);
        // the normaliser's shares come from the d x d states; one kernel then adds the in-chunk gradients.
        const ResLayout R = make_res_layout(pr, true);
        const float s2 = pr.scale * pr.scale;
        const size_t slab = (size_t)BH * pr.T * pr.d;   // floats
        bf16_t* Kt = (bf16_t*)(c.ws + R.off_kt);
        bf16_t* Vt = (bf16_t*)(c.ws + R.off_vt);
        bf16_t* Qt = (bf16_t*)(c.ws + R.off_qt);
        bf16_t* Ght = (bf16_t*)(c.ws + R.off_ght);
        bf16_t* Gh = (bf16_t*)(c.ws + R.off_gh);
        float* gz = (float*)(c.ws + R.off_gz);
        bf16_t* Gam = (bf16_t*)(c.ws + R.off_gam);
        bf16_t* Omg = (bf16_t*)(c.ws + R.off_omg);
        float* gram = (float*)(c.ws + R.off_gram);
        float* totS = (float*)(c.ws + R.off_tot);
        float* totR = (float*)(c.ws + R.off_totr);
        float* pdv = (float*)(c.ws + R.off_part);
        float* pdq = (float*)(c.ws + R.off_pdq);
        float* pdk = (float*)(c.ws + R.off_pdk);
        const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V;
        hipStream_t st = c.stream;
        PA_TRY(launch_attn_prep(st, pr.d, (const bf16_t*)dO, (const bf16_t*)O, Z, Gh, gz, (long long)BH * pr.T, pr.normalize))
        PA_TRY(launch_transpose_hd(st, pr.d, q, Qt, BH, pr.T))
        PA_TRY(launch_transpose_hd(st, pr.d, Gh, Ght, BH, pr.T))
        if (!pr.keep_state) {
            PA_TRY(launch_transpose_hd(st, pr.d, k, Kt, BH, pr.T))
            PA_TRY(launch_transpose_hd(st, pr.d, v, Vt, BH, pr.T))
            PA_TRY(launch_gram(st, pr.d, Kt, nullptr, gram, Gam, BH, pr.T, pr.chunk, false, 1.0f))
            if (R.pl.nseg > 1)
                PA_TRY(launch_res_walk("res_state_totals", st, pr.d, false, 0, Kt, Vt, nullptr, nullptr, totS, nullptr, BH, pr.T,
                                       pr.chunk, R.pl, 1.0f))
        }
        PA_TRY(launch_gram(st, pr.d, Qt, gz, gram, Omg, BH, pr.T, pr.chunk, true, s2))
        PA_TRY(launch_gram_apply(st, pr.d, q, Gam, gz, pdq + R.pl.nslab * slab, nullptr, BH, pr.T, pr.chunk, 2.f * s2, 0.f))
        PA_TRY(launch_gram_apply(st, pr.d, k, Omg, nullptr, pdk + R.pl.nslab * slab, nullptr, BH, pr.T, pr.chunk, 2.f, 0.f))
        PA_TRY(launch_res_walk("res_dq_walk", st, pr.d, false, 2, Kt, Vt, q, Gh, totS, pdq, BH, pr.T, pr.chunk, R.pl, s2))
        if (R.pl.nseg > 1)
            PA_TRY(launch_res_walk("res_grad_totals", st, pr.d, true, 0, Qt, Ght, nullptr, nullptr, totR, nullptr, BH, pr.T,
                                   pr.chunk, R.pl, 1.0f))
        PA_TRY(launch_res_walk("res_dv_walk", st, pr.d, true, 1, Qt, Ght, k, nullptr, totR, pdv, BH, pr.T, pr.chunk, R.pl, s2))
        PA_TRY(launch_res_walk("res_dk_walk", st, pr.d, true, 2, Qt, Ght, k, v, totR, pdk, BH, pr.T, pr.chunk, R.pl, s2))
        PA_TRY(launch_chunk_bwd(st, pr.p, pr.d, q, k, v, Gh, gz, (bf16_t*)dQ, (bf16_t*)dK, (bf16_t*)dV, BH, pr.T, pr.chunk, pr.scale,
                                pdq, R.pl.nslab + 1, pdk, R.pl.nslab + 1, pdv, R.pl.nslab))
        return PA_OK;
    }
    const Layout L = make_layout(pr, true);
    const GateBuf& gt = c.gate;
    bf16_t* Kt = (bf16_t*)(c.ws + L.off_kt);
    bf16_t* Kts = (bf16_t*)(c.ws + L.off_kts);
    bf16_t* Vt = (bf16_t*)(c.ws + L.off_vt);
    bf16_t* Qt = (bf16_t*)(c.ws + L.off_qt);
    bf16_t* Qts = (bf16_t*)(c.ws + L.off_qts);
    bf16_t* Gh = (bf16_t*)(c.ws + L.off_gh);
    bf16_t* Ght = (bf16_t*)(c.ws + L.off_ght);
    float* gz = (float*)(c.ws + L.off_gz);
    bf16_t* Gam = (bf16_t*)(c.ws + L.off_gam);
    bf16_t* Omg = (bf16_t*)(c.ws + L.off_omg);
    bf16_t* Sc = (bf16_t*)(c.ws + L.off_sc);
    bf16_t* Rc = (bf16_t*)(c.ws + L.off_rc);
    const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V;
    const float s2 = pr.scale * pr.scale;
    SideStream side = side_stream();
    if (profile_enabled()) side.ok = false;   // timed kernel by kernel: no overlap
    hipStream_t s_main = c.stream, s_side = side.ok ? side.stream : c.stream;

    PA_TRY(launch_bwd_prep(s_main, (const bf16_t*)dO, (const bf16_t*)O, Z, Gh, gz, (long long)BH * pr.T, pr.normalize))
    PA_TRY(launch_transpose(s_main, q, Qt, BH, pr.T))
    if (pr.gated) PA_TRY(launch_transpose(s_main, q, Qts, BH, pr.T, gt.qfac))
    PA_TRY(launch_transpose(s_main, Gh, Ght, BH, pr.T))
    // The fork sits here, not right after the preparation kernel that dQ depends on: the scan's
    // workgroups need most of a CU's LDS and must be placed before dQ's fill the CUs.
    if (side.ok) {
        if (hipEventRecord(side.fork, s_main) != hipSuccess || hipStreamWaitEvent(s_side, side.fork, 0) != hipSuccess)
            return PA_ERR_HIP;
    }
    // strand R (caller's stream, so that its workgroups are placed first): state-gradient scan
    PA_TRY(launch_scan("mfma_state_grad_scan", s_main, true, Qts, Ght, gz, Rc, Omg, BH, pr.T, L.cs, s2, gt.lam))
    if (pr.gated && side.ok && hipEventRecord(side.scanned, s_main) != hipSuccess) return PA_ERR_HIP;
    // strand S (side stream): dQ from the forward state
    if (!L.keep) {
        // nothing but O and Z was saved: rebuild the chunk states
        PA_TRY(launch_transpose(s_side, k, Kt, BH, pr.T))
        if (pr.gated) PA_TRY(launch_transpose(s_side, k, Kts, BH, pr.T, gt.kfac))
        PA_TRY(launch_transpose(s_side, v, Vt, BH, pr.T))
        PA_TRY(launch_scan("mfma_state_scan_bwd", s_side, false, Kts, Vt, nullptr, Sc, Gam, BH, pr.T, L.cs, 1.0f, gt.lam))
    }
    PA_TRY(launch_bwd_dq(s_side, q, k, v, Gh, gz, Kt, Sc, Gam, (bf16_t*)dQ, BH, pr.T, L.cs, pr.scale, gt.bl, gt.qfac, gt.db))
    PA_TRY(launch_bwd_dkdv(s_main, q, k, v, Gh, gz, Qt, Ght, Rc, Omg, (bf16_t*)dK, (bf16_t*)dV, BH, pr.T, L.cs, pr.scale,
                           gt.bl, gt.kfac, gt.db2))
    if (pr.gated) {
        // the pairs that straddle the chunk boundaries, from both sets of states: behind dQ on the side
        // strand (S is complete there), once the scan on the caller's stream has produced R
        if (side.ok && hipStreamWaitEvent(s_side, side.scanned, 0) != hipSuccess) return PA_ERR_HIP;
        PA_TRY(launch_gate_boundary(s_side, Sc, Rc, Gam, Omg, gt.xb, BH, L.nstate))
    }
    if (side.ok) {
        if (hipEventRecord(side.join, s_side) != hipSuccess || hipStreamWaitEvent(s_main, side.join, 0) != hipSuccess)
            return PA_ERR_HIP;
    }
    return PA_OK;
}

// ---- a prompt into a decode state, through the state scan ----------------------------------------------
// The sum the decode state needs is what the forward scan accumulates.  The prompt is scanned as the first
// of two chunks of its own length (the second is never read): the state "before chunk 1" is the sum over
// the whole prompt, written once, in bf16 tiles.  A small kernel then adds it, in the decode step's basis
// (monomials x_i x_j, i <= j, multiplicity on the state), to the float32 decode state: off-diagonal tiles
// map one to one, a diagonal tile holds (a, b) and (b, a) of one monomial.  Gates: keys scaled by the square
// root of their decay to the end of the prompt (one chunk, so no per-chunk decay), the old state by the
// decay across the whole prompt.
namespace {

struct AbsorbLayout {
    size_t off_kt, off_vt, off_sc, off_gam, off_gate, total;
};
AbsorbLayout make_absorb_layout(const pa_problem& pr) {
    AbsorbLayout L{};
    const size_t BH = (size_t)pr.B * pr.H;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    L.off_kt = take(BH * 2 * pr.T * DH * 2);
    L.off_vt = take(BH * 2 * pr.T * DH * 2);
    L.off_sc = take(BH * 2 * (size_t)STATE_ELEMS * 2);
    L.off_gam = take(BH * 2 * (size_t)DH * DH * 2);
    L.off_gate = off;
    pa_problem gp = pr;
    gp.chunk = pr.T;
    L.total = off + gate_workspace_bytes(gp, false);
    return L;
}

__global__ __launch_bounds__(256) void k_absorb_convert(const bf16_t* __restrict__ StC, const bf16_t* __restrict__ Gam,
                                                        const float* __restrict__ lam, float* __restrict__ S,
                                                        float* __restrict__ gamd, int D) {
    const int bh = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x;          // (row r, column c), c == DH: the normaliser column
    if (idx >= D * (DH + 1)) return;
    const int r = idx / (DH + 1), c = idx % (DH + 1);
    int i = 0, rem = r;
    while (rem >= DH - i) {
        rem -= DH - i;
        ++i;
    }
    const int j = i + rem;
    const float decay = lam != nullptr ? lam[bh] : 1.f;
    if (c == DH) {
        const float g = bf16_to_f32(Gam[((size_t)bh * 2 + 1) * DH * DH + (size_t)j * DH + i]);
        float* dst = gamd + (size_t)bh * D + r;
        *dst = decay * *dst + (i == j ? g : 2.f * g);
        return;
    }
    const int ti = i >> 3, a = i & 7, tj = j >> 3, b = j & 7;
    const bf16_t* tile = StC + (((size_t)bh * 2 + 1) * NTILES + (tj * (tj + 1) / 2 + ti)) * TILE_ELEMS;
    float x = bf16_to_f32(tile[(a * DH + c) * 8 + b]);
    if (ti == tj && a != b) x += bf16_to_f32(tile[(b * DH + c) * 8 + a]);
    float* dst = S + ((size_t)bh * D + r) * DH + c;
    *dst = decay * *dst + x;
}

}  // namespace

bool mfma_absorb_supported(const pa_problem& pr) {
    return pr.dtype == PA_DTYPE_BF16 && pr.p == 2 && pr.d == DH && pr.v == DH && pr.T % QBLK == 0 &&
           (size_t)pr.B * pr.H <= 65535u;
}
size_t mfma_absorb_workspace_bytes(const pa_problem& pr) { return mfma_absorb_supported(pr) ? make_absorb_layout(pr).total : 0; }

pa_status mfma_absorb(const pa_problem& pr, const void* K, const void* V, const float* log_g, char* ws, hipStream_t s, float* S,
                      float* gamd, int D) {
    const AbsorbLayout L = make_absorb_layout(pr);
    const int BH = pr.B * pr.H;
    bf16_t* Kt = (bf16_t*)(ws + L.off_kt);
    bf16_t* Vt = (bf16_t*)(ws + L.off_vt);
    bf16_t* Sc = (bf16_t*)(ws + L.off_sc);
    bf16_t* Gam = (bf16_t*)(ws + L.off_gam);
    const float *kfac = nullptr, *lam = nullptr;
    if (log_g != nullptr) {
        pa_problem gp = pr;
        gp.chunk = pr.T;
        gp.gated = 1;
        Ctx c{gp, s, ws, L.total, gate_buffers(gp, false, ws + L.off_gate)};
        pa_status st = gate_prepare(c, log_g);
        if (st != PA_OK) return st;
        kfac = c.gate.kfac;
        lam = c.gate.lam;
    }
    PA_TRY(launch_transpose(s, (const bf16_t*)K, Kt, BH, pr.T, kfac, 2 * pr.T))
    PA_TRY(launch_transpose(s, (const bf16_t*)V, Vt, BH, pr.T, nullptr, 2 * pr.T))
    PA_TRY(launch_scan("decode_absorb_scan", s, false, Kt, Vt, nullptr, Sc, Gam, BH, 2 * pr.T, pr.T, 1.0f, nullptr))
    LaunchScope ls("decode_absorb_convert", s);
    hipLaunchKernelGGL(k_absorb_convert, dim3((D * (DH + 1) + 255) / 256, BH), dim3(256), 0, s, (const bf16_t*)Sc,
                       (const bf16_t*)Gam, lam, S, gamd, D);
    return launch_ok() ? PA_OK : PA_ERR_HIP;
}

}  // namespace pa
