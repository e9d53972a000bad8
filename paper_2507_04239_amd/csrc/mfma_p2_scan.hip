// State scan of the bf16 MFMA family (p = 2): feature-major copies of the inputs, and the fused
// update-state + cumulative sum over chunks.  See mfma_common.hpp for the embedding and layouts.
#include "mfma_common.hpp"

namespace pa {
namespace mfma {
namespace {

// ---- token-major -> feature-major in blocks of 64 tokens -----------------------------------
// [BH][T][DH] -> [BH][T/64][DH][64] (bf16).  Each block is 8 KB contiguous, so the readers'
// accesses stay dense (rows of a plain [DH][T] transpose would sit a power of two apart and
// pile onto the same memory channel).

// `fac` (gating, may be null): token t is multiplied by sqrt(fac[t]) on the way.  For p = 2 a
// weight w on phi(x) is the same as sqrt(w) on x, so the scans of a gated problem read copies
// scaled this way and need no per-token weights of their own.
__global__ __launch_bounds__(256) void k_transpose(const bf16_t* __restrict__ in, bf16_t* __restrict__ out, int T,
                                                   const float* __restrict__ fac, int out_blocks) {
    __shared__ bf16_t tile[TBLK][DH + 2];
    const int bh = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const bf16_t* src = in + ((size_t)bh * T + (size_t)blk * TBLK) * DH;
    if (fac == nullptr) {
        for (int e = tid; e < TBLK * DH; e += 256) tile[e / DH][e % DH] = src[e];
    } else {
        const float* f = fac + (size_t)bh * T + (size_t)blk * TBLK;
        for (int e = tid; e < TBLK * DH; e += 256) tile[e / DH][e % DH] = f32_to_bf16(bf16_to_f32(src[e]) * sqrtf(f[e / DH]));
    }
    __syncthreads();
    bf16_t* dst = out + ((size_t)bh * out_blocks + blk) * DH * TBLK;
    for (int e = tid; e < TBLK * DH; e += 256) dst[e] = tile[e % TBLK][e / TBLK];
}

// ---- state scan ----------------------------------------------------------------------------
// Fused update-state + cumulative sum over chunks (App. E.2 + E.3, no gating), used for
//   the forward state     S_n = sum_{j <  n cs}     phi(k_j) v_j^T        (X = K, Y = V)
//   the state gradient    R_m = sum_{i >= (m+1) cs} phi(q_i) ghat_i^T     (X = Q, Y = dO/Z, REV)
// One workgroup of 256 threads per (tile pair, head).  Workgroup `pair` owns two 64 x DH state tiles of
// one tile row, (ti, tj0) and (ti, tj1) (a tile row with an odd number of tiles ends in a "pair" of
// one tile taken twice: both halves then compute and store the same values); wave w owns the rows
// a = 2 w, 2 w + 1 of both.  A 16-row MFMA block is one a and the 8 + 8 values b of the two tiles, so
// the factor x[8 ti + a] of its 16 rows is the same for all of them: a lane reads ONE float of it per
// k-step (token 8 g + (r16 & 7) of row a = 2 w + (r16 >> 3)) and the multiply fetches the token it
// needs from that lane of its 16-lane row by DPP (row_newbcast), instead of reading the 8 tokens per
// lane and row block from LDS (64 of 160 bytes per lane and k-step).  A tile pair stages only the
// 24 feature rows of X it multiplies.  (Measured on the headline shape: 11 % off the scan at 256 or
// more tokens per state; at 128 the scan is bound by its 1.86 GB of state writes - with the MFMAs
// taken out it is no faster, with the stores taken out it is.)
// Workgroup NPAIR owns the normaliser in its d x d form: Gamma = sum k k^T, or
// Omega = sum gz_i q_i q_i^T for the gradient (same code: the A operand is x itself, times the
// weight, and the B operand comes from X instead of Y; only waves 0 and 1 have rows).
// The state is written every `cs` tokens, before the tokens of that stretch are added.
//
// Each workgroup walks the sequence in stages of 128 tokens.  A stage's X (as float32) and Y
// (bf16) are staged in LDS, feature-major, and shared by the four waves; the global loads of
// SCAN_PF further stages are in flight in registers.
//
constexpr int NPAIR = 20;                      // 4 + 4 + 3 + 3 + 2 + 2 + 1 + 1 pairs in the tile rows ti = 0 .. 7
constexpr int SCAN_TOK = 128;                  // tokens per stage
constexpr int SCAN_PF = 3;                     // stages in flight in registers
constexpr int XS_PITCH = SCAN_TOK + 4;         // floats; pitch = 4 mod 64 banks
constexpr int YS_PITCH = SCAN_TOK + 8;         // bf16;   pitch = 4 mod 64 banks (in dwords)
static_assert(NTILES == 36 && DH == 64, "the pair table below is written for 8 x 8 tiles of 64 rows");

// The reverse scan (state gradient) runs side by side with the dQ kernel, whose workgroups need
// LDS of their own on the same CU: there Y is single-buffered (ys[1] is not allocated), at the
// price of a second barrier per stage.
struct ScanSmem {
    float xs[2][DH][XS_PITCH];
    float ws[2][SCAN_TOK];
    bf16_t ys[2][DH][YS_PITCH];
};
template <bool REV>
constexpr size_t scan_smem_bytes() {
    return REV ? sizeof(ScanSmem) - sizeof(bf16_t) * DH * YS_PITCH : sizeof(ScanSmem);
}

// One 128-token stage of one wave: acc[rbk][cb] += phi-rows(32) x Y(64 columns), four k-steps of
// 32 tokens.  Written as an explicit software pipeline, because a workgroup of this kernel is
// alone on its CU (one wave per SIMD): the LDS operands of k-step s+1 are read and its A
// operands expanded while the MFMAs of k-step s run.
struct ScanOps {          // LDS operands of one k-step for one lane
    float4 xal[2], xah[2];   // normaliser only: x[fa(rbk)][8 tokens]
    float xa1;               // tiles: x[8 ti + 2 w + (r16 >> 3)][token 8 g + (r16 & 7)], shared along the 16-lane row
    float4 xbl, xbh;         // x[fb][8 tokens]  (or the weights / ones for the normaliser)
    uint4 b[4];              // Y^T fragments, 4 column blocks
};

// the value of lane L of this lane's 16-lane row
template <int L>
__device__ __forceinline__ float row_lane(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + L, 0xf, 0xf, false));
}

template <bool GAMMA, bool REV>
__device__ __forceinline__ void scan_load_ops(ScanOps& o, const ScanSmem& sm, int buf, int s, int fa0, int fa_step,
                                              int fb, int r16, int g) {
    const int t0 = 32 * s + 8 * g;
    if (GAMMA) {
#pragma unroll
        for (int rbk = 0; rbk < 2; ++rbk) {
            const float* xa = &sm.xs[buf][fa0 + fa_step * rbk][t0];
            o.xal[rbk] = *(const float4*)xa;
            o.xah[rbk] = *(const float4*)(xa + 4);
        }
    } else {
        o.xa1 = sm.xs[buf][fa0][t0 + (r16 & 7)];
    }
    if (!GAMMA) {
        o.xbl = *(const float4*)&sm.xs[buf][fb][t0];
        o.xbh = *(const float4*)&sm.xs[buf][fb][t0 + 4];
    } else if (REV) {
        o.xbl = *(const float4*)&sm.ws[buf][t0];
        o.xbh = *(const float4*)&sm.ws[buf][t0 + 4];
    } else {
        o.xbl = make_float4(1.f, 1.f, 1.f, 1.f);
        o.xbh = o.xbl;
    }
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) o.b[cb] = *(const uint4*)&sm.ys[REV ? 0 : buf][16 * cb + r16][t0];
}

template <bool GAMMA>
__device__ __forceinline__ void scan_expand(Frag (&af)[2], const ScanOps& o) {
    if (!GAMMA) {
        // row block rbk: a = 2 w + rbk, whose 8 tokens sit in lanes 8 rbk .. 8 rbk + 7 of the row
        af[0].v[0] = (__bf16)(row_lane<0>(o.xa1) * o.xbl.x); af[0].v[1] = (__bf16)(row_lane<1>(o.xa1) * o.xbl.y);
        af[0].v[2] = (__bf16)(row_lane<2>(o.xa1) * o.xbl.z); af[0].v[3] = (__bf16)(row_lane<3>(o.xa1) * o.xbl.w);
        af[0].v[4] = (__bf16)(row_lane<4>(o.xa1) * o.xbh.x); af[0].v[5] = (__bf16)(row_lane<5>(o.xa1) * o.xbh.y);
        af[0].v[6] = (__bf16)(row_lane<6>(o.xa1) * o.xbh.z); af[0].v[7] = (__bf16)(row_lane<7>(o.xa1) * o.xbh.w);
        af[1].v[0] = (__bf16)(row_lane<8>(o.xa1) * o.xbl.x); af[1].v[1] = (__bf16)(row_lane<9>(o.xa1) * o.xbl.y);
        af[1].v[2] = (__bf16)(row_lane<10>(o.xa1) * o.xbl.z); af[1].v[3] = (__bf16)(row_lane<11>(o.xa1) * o.xbl.w);
        af[1].v[4] = (__bf16)(row_lane<12>(o.xa1) * o.xbh.x); af[1].v[5] = (__bf16)(row_lane<13>(o.xa1) * o.xbh.y);
        af[1].v[6] = (__bf16)(row_lane<14>(o.xa1) * o.xbh.z); af[1].v[7] = (__bf16)(row_lane<15>(o.xa1) * o.xbh.w);
        return;
    }
#pragma unroll
    for (int rbk = 0; rbk < 2; ++rbk) {
        af[rbk].v[0] = (__bf16)(o.xal[rbk].x * o.xbl.x); af[rbk].v[1] = (__bf16)(o.xal[rbk].y * o.xbl.y);
        af[rbk].v[2] = (__bf16)(o.xal[rbk].z * o.xbl.z); af[rbk].v[3] = (__bf16)(o.xal[rbk].w * o.xbl.w);
        af[rbk].v[4] = (__bf16)(o.xah[rbk].x * o.xbh.x); af[rbk].v[5] = (__bf16)(o.xah[rbk].y * o.xbh.y);
        af[rbk].v[6] = (__bf16)(o.xah[rbk].z * o.xbh.z); af[rbk].v[7] = (__bf16)(o.xah[rbk].w * o.xbh.w);
    }
}

__device__ __forceinline__ void scan_mma(f32x4 (&acc)[2][4], const Frag (&af)[2], const ScanOps& o) {
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        Frag bf;
        bf.u = o.b[cb];
        acc[0][cb] = mfma16(af[0].v, bf.v, acc[0][cb]);
        acc[1][cb] = mfma16(af[1].v, bf.v, acc[1][cb]);
    }
}

// 8 MFMAs with 3 vector-ALU instructions after each: the expansion of the next k-step rides in
// the shadow of the matrix pipe
__device__ __forceinline__ void scan_interleave_hint() {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
    }
}

// x, y: two dwords each.  Lanes of an even 16-lane row r receive (x of row r, x of row r + 1),
// lanes of an odd row r receive (y of row r - 1, y of row r), as (.x, .z) and (.y, .w) for the
// two dwords: 8 consecutive bf16 when a lane's dwords hold 4.
__device__ __forceinline__ uint4 pair_rows(uint2 x, uint2 y) {
    const auto d0 = __builtin_amdgcn_permlane16_swap(x.x, y.x, false, false);
    const auto d1 = __builtin_amdgcn_permlane16_swap(x.y, y.y, false, false);
    return make_uint4(d0[0], d1[0], d0[1], d1[1]);
}

// A state leaving the chip: four 16-byte runs per lane, at dst + run_offset(k)
struct StateOut {
    uint4 run[4];
    bf16_t* dst;
};
template <bool GAMMA>
__device__ __forceinline__ void store_run(const StateOut& so, int k) {
    // state tile [a][v][b]: run k = (row block k >> 1 = a, column-block pair k & 1); Gamma: column block k
    const int off = GAMMA ? 16 * DH * k : (k >> 1) * (DH * 8) + (k & 1) * (32 * 8);
    __builtin_nontemporal_store((u32x4){so.run[k].x, so.run[k].y, so.run[k].z, so.run[k].w}, (u32x4*)(so.dst + off));
}

// PACED: one run of `so` is stored after each k-step.  A CU drains stores slowly (about 10 bytes
// per clock were measured); issued back to back the four waves' 16 KB stall every wave for the
// length of the whole compute phase, spread over it they cost nothing.
template <bool GAMMA, bool REV, bool PACED>
__device__ __forceinline__ void scan_stage(f32x4 (&acc)[2][4], const ScanSmem& sm, int buf, int fa0, int fa_step,
                                           int fb, int r16, int g, const StateOut& so) {
    ScanOps o0, o1;
    Frag af0[2], af1[2];
    scan_load_ops<GAMMA, REV>(o0, sm, buf, 0, fa0, fa_step, fb, r16, g);
    scan_load_ops<GAMMA, REV>(o1, sm, buf, 1, fa0, fa_step, fb, r16, g);
    scan_expand<GAMMA>(af0, o0);
    __builtin_amdgcn_sched_barrier(0);
    scan_mma(acc, af0, o0);          // k-step 0
    scan_expand<GAMMA>(af1, o1);
    scan_interleave_hint();
    if (PACED) store_run<GAMMA>(so, 0);
    __builtin_amdgcn_sched_barrier(0);
    scan_load_ops<GAMMA, REV>(o0, sm, buf, 2, fa0, fa_step, fb, r16, g);
    scan_mma(acc, af1, o1);          // k-step 1
    scan_expand<GAMMA>(af0, o0);
    scan_interleave_hint();
    if (PACED) store_run<GAMMA>(so, 1);
    __builtin_amdgcn_sched_barrier(0);
    scan_load_ops<GAMMA, REV>(o1, sm, buf, 3, fa0, fa_step, fb, r16, g);
    scan_mma(acc, af0, o0);          // k-step 2
    scan_expand<GAMMA>(af1, o1);
    scan_interleave_hint();
    if (PACED) store_run<GAMMA>(so, 2);
    __builtin_amdgcn_sched_barrier(0);
    scan_mma(acc, af1, o1);          // k-step 3
    if (PACED) store_run<GAMMA>(so, 3);
}

// EVERY: cs == SCAN_TOK, a state is written at every stage.  The stores are then unconditional,
// and the compiler knows how many vector-memory operations separate a stage's loads from their
// use; behind a branch it has to assume none, and waits for all but the newest loads, i.e. also
// for the previous stage's stores.
template <bool GAMMA, bool REV, bool EVERY, bool GATED>
__device__ __forceinline__ void scan_body(const bf16_t* __restrict__ Xt, const bf16_t* __restrict__ Yt,
                                          const float* __restrict__ wgt, bf16_t* __restrict__ StC,
                                          bf16_t* __restrict__ Gam, int T, int cs,
                                          float out_scale, const float* __restrict__ lam, ScanSmem& sm, int pair, int bh) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int nstate = T / cs;
    // pair -> tile row ti and the two tiles (ti, tj0), (ti, tj1) of it: row ti has 8 - ti tiles
    int ti = 0, tj0 = 0;
    if (!GAMMA) {
        int left = pair;
        while (left >= (9 - ti) / 2) {
            left -= (9 - ti) / 2;
            ++ti;
        }
        tj0 = ti + 2 * left;
    }
    const int tj1 = min(tj0 + 1, DH / 8 - 1);
    // As an A operand, lane r16 is row (tile r16 >> 3, b = r16 & 7) of the row block; as an accumulator,
    // lane (r16, g) holds rows 4 g + r: tile g >> 1, b = 4 (g & 1) + r.
    const int tj_c = (g >> 1) ? tj1 : tj0;
    const int tile = GAMMA ? 0 : tj_c * (tj_c + 1) / 2 + ti;   // storage order of the tiles: by columns tj
    const float mult = GAMMA ? out_scale : ((ti == tj_c) ? 1.f : 2.f) * out_scale;
    // tiles: the shared factor's feature (lanes 0-7 of a row: a = 2 w, lanes 8-15: a = 2 w + 1), and this
    // lane's own;   Gamma: feature 32 w + 16 rbk + r16
    const int fa0 = GAMMA ? (32 * (w & 1) + r16) : 8 * ti + 2 * w + (r16 >> 3);
    const int fa_step = GAMMA ? 16 : 0;
    const int fb = 8 * ((r16 >> 3) ? tj1 : tj0) + (r16 & 7);
    const bool has_rows = !GAMMA || w < 2;

    // global -> LDS staging: thread t moves pieces t, t + 256, t + 512, t + 768 of the stage; a
    // piece is 8 tokens of one feature (16 bytes of bf16) of X and of Y
    const bf16_t* Xh = Xt + (size_t)bh * DH * T;
    const bf16_t* Yh = (GAMMA ? Xt : Yt) + (size_t)bh * DH * T;
    const float* Wh = (GAMMA && REV) ? wgt + (size_t)bh * T : nullptr;
    int p_feat[4], p_tok[4], p_off[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int id = tid + 256 * q;
        p_feat[q] = id >> 4;
        p_tok[q] = 8 * (id & 15);                                        // token inside the stage
        p_off[q] = (p_tok[q] >> 6) * (DH * TBLK) + p_feat[q] * TBLK + (p_tok[q] & 63);
    }
    // X: a tile pair multiplies only the 3 x 8 features of ti, tj0 and tj1, 384 pieces: threads 0 .. 127
    // move two, the others one (and repeat the last piece: same bytes to the same place).  The
    // normaliser needs all 64 rows, pieces as for Y.
    int x_feat[4], x_tok[4], x_off[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (GAMMA) {
            x_feat[q] = p_feat[q];
            x_tok[q] = p_tok[q];
            x_off[q] = p_off[q];
        } else {
            const int id = min(tid + 256 * (q & 1), 24 * 16 - 1);
            const int grp = id >> 7;
            x_feat[q] = 8 * (grp == 0 ? ti : (grp == 1 ? tj0 : tj1)) + ((id >> 4) & 7);
            x_tok[q] = 8 * (id & 15);
            x_off[q] = (x_tok[q] >> 6) * (DH * TBLK) + x_feat[q] * TBLK + (x_tok[q] & 63);
        }
    }

    f32x4 acc[2][4];
#pragma unroll
    for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[rbk][cb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // Both stores below hand every lane 16 contiguous bytes: a lane's 4 accumulator rows are half
    // of an 8-row run whose other half sits 16 lanes away, so two lanes swap halves of two
    // column blocks (or row blocks) and each stores one complete run.
    // gated: right after a state has been packed the running sum decays by `decay`, the factor of
    // the chunk that is about to be added.  One pass over the accumulators does both: a second
    // pass costs registers, and the reverse scan has to stay within 288 so that a wave of the dQ
    // kernel (224) fits beside it on the SIMD.
    auto pack = [&](f32x4& c, float decay) {
        union {
            bf16x4 v;
            uint2 u;
        } o;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            o.v[r] = (__bf16)(c[r] * mult);
            if (GATED) c[r] *= decay;
        }
        return o.u;
    };
    // the state as it stands, packed for storing as state n
    auto pack_state = [&](StateOut& so, int n, float decay) {
        if (!GAMMA) {
            // layout [a][v][b]: accumulator rows are b = 4 (g & 1) + r of tile (ti, tj0 / tj1 by g >> 1),
            // row block rbk is a = 2 w + rbk
            so.dst = StC + ((size_t)(bh * nstate + n) * NTILES + tile) * TILE_ELEMS + (2 * w * DH + 16 * (g & 1) + r16) * 8;
#pragma unroll
            for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
                for (int cp = 0; cp < 2; ++cp) {  // g even: column block 2 cp; g odd: 2 cp + 1
                    const uint2 lo = pack(acc[rbk][2 * cp], decay), hi = pack(acc[rbk][2 * cp + 1], decay);
                    so.run[2 * rbk + cp] = pair_rows(lo, hi);
                }
        } else {
            // Gamma / Omega are symmetric: element (row, col) is stored at [col][row], where the
            // accumulator rows 32 w + 16 rbk + 4 g + r are contiguous
            so.dst = Gam + (size_t)(bh * nstate + n) * DH * DH + r16 * DH + 32 * (w & 1) + 16 * (g & 1) + 8 * (g >> 1);
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {     // g even: row block 0; g odd: row block 1
                const uint2 lo = pack(acc[0][cb], decay), hi = pack(acc[1][cb], decay);
                so.run[cb] = pair_rows(lo, hi);
            }
        }
    };
    auto write_state = [&](int n, float decay) {
        StateOut so;
        pack_state(so, n, decay);
        if (has_rows) {
#pragma unroll
            for (int k = 0; k < 4; ++k) store_run<GAMMA>(so, k);
        }
    };

    // Stretches at the far end never feed a state that is written, so the walk stops early.
    const int nstage = (T - cs) / SCAN_TOK;
    const int nstage_all = T / SCAN_TOK;
    if (nstage > 0) {
        // Register ring: slot J holds the global data of stage (st0 + J).  Every load is
        // unconditional (indices are clamped instead of branching) so that the compiler can
        // count the loads in flight instead of waiting for all of them.  Separately named
        // registers and macros instead of arrays and lambdas: the slot has to be a
        // compile-time name or the ring is demoted to scratch memory.
#define PA_SLOT(J) uint4 x0_##J, x1_##J, x2_##J, x3_##J, y0_##J, y1_##J, y2_##J, y3_##J; float wv_##J;
        PA_SLOT(0) PA_SLOT(1) PA_SLOT(2)
#undef PA_SLOT
        static_assert(SCAN_PF == 3, "the ring below is written out for 3 slots");
#define PA_LOAD_STAGE(J, ST)                                                              \
    {                                                                                     \
        const int sc_ = min((ST), nstage - 1);                                            \
        const int sidx_ = REV ? nstage_all - 1 - sc_ : sc_;                               \
        const size_t so_ = (size_t)sidx_ * (2 * DH * TBLK);                               \
        x0_##J = *(const uint4*)(Xh + so_ + x_off[0]);                                    \
        x1_##J = *(const uint4*)(Xh + so_ + x_off[1]);                                    \
        if (GAMMA) {                                                                      \
            x2_##J = *(const uint4*)(Xh + so_ + x_off[2]);                                \
            x3_##J = *(const uint4*)(Xh + so_ + x_off[3]);                                \
        }                                                                                 \
        y0_##J = *(const uint4*)(Yh + so_ + p_off[0]);                                    \
        y1_##J = *(const uint4*)(Yh + so_ + p_off[1]);                                    \
        y2_##J = *(const uint4*)(Yh + so_ + p_off[2]);                                    \
        y3_##J = *(const uint4*)(Yh + so_ + p_off[3]);                                    \
        if (GAMMA && REV) wv_##J = Wh[(size_t)sidx_ * SCAN_TOK + (tid & (SCAN_TOK - 1))]; \
    }
#define PA_FILL_X(BUF, Q, XR)                                                             \
    {                                                                                     \
        float* d_ = &sm.xs[BUF][x_feat[Q]][x_tok[Q]];                                     \
        *(float4*)d_ = make_float4(bf_lo(XR.x), bf_hi(XR.x), bf_lo(XR.y), bf_hi(XR.y));   \
        *(float4*)(d_ + 4) = make_float4(bf_lo(XR.z), bf_hi(XR.z), bf_lo(XR.w), bf_hi(XR.w)); \
    }
#define PA_CONSUME(J, ST, BUF)                                                                \
    if ((ST) < nstage) { /* uniform; no global loads inside this branch */                    \
        const int edge_ = REV ? T - (ST) * SCAN_TOK : (ST) * SCAN_TOK;                        \
        StateOut so_;                                                                         \
        if (EVERY || edge_ % cs == 0) {                                                       \
            const int n_ = REV ? edge_ / cs - 1 : edge_ / cs;                                 \
            const float l_ = GATED ? lam[(size_t)bh * nstate + n_] : 1.f;                     \
            if (EVERY) pack_state(so_, n_, l_);                                               \
            else write_state(n_, l_);                                                         \
        }                                                                                     \
        PA_FILL_X(BUF, 0, x0_##J) PA_FILL_X(BUF, 1, x1_##J)                                   \
        if (GAMMA) {                                                                          \
            PA_FILL_X(BUF, 2, x2_##J) PA_FILL_X(BUF, 3, x3_##J)                               \
        }                                                                                     \
        if (GAMMA && REV && tid < SCAN_TOK) sm.ws[BUF][tid] = wv_##J;                         \
        if (REV) lds_barrier(); /* every wave is done with the Y of the stage before */       \
        *(uint4*)&sm.ys[REV ? 0 : BUF][p_feat[0]][p_tok[0]] = y0_##J;                         \
        *(uint4*)&sm.ys[REV ? 0 : BUF][p_feat[1]][p_tok[1]] = y1_##J;                         \
        *(uint4*)&sm.ys[REV ? 0 : BUF][p_feat[2]][p_tok[2]] = y2_##J;                         \
        *(uint4*)&sm.ys[REV ? 0 : BUF][p_feat[3]][p_tok[3]] = y3_##J;                         \
        lds_barrier();                                                                        \
        if (has_rows) scan_stage<GAMMA, REV, EVERY>(acc, sm, BUF, fa0, fa_step, fb, r16, g, so_); \
    }
        // The LDS buffer alternates with the stage parity; 2 * SCAN_PF stages per trip keep both
        // the ring slot and the buffer compile-time constants.
        PA_LOAD_STAGE(0, 0) PA_LOAD_STAGE(1, 1) PA_LOAD_STAGE(2, 2)
        for (int st0 = 0; st0 < nstage; st0 += 2 * SCAN_PF) {
            PA_CONSUME(0, st0 + 0, 0) PA_LOAD_STAGE(0, st0 + 3)
            PA_CONSUME(1, st0 + 1, 1) PA_LOAD_STAGE(1, st0 + 4)
            PA_CONSUME(2, st0 + 2, 0) PA_LOAD_STAGE(2, st0 + 5)
            PA_CONSUME(0, st0 + 3, 1) PA_LOAD_STAGE(0, st0 + 6)
            PA_CONSUME(1, st0 + 4, 0) PA_LOAD_STAGE(1, st0 + 7)
            PA_CONSUME(2, st0 + 5, 1) PA_LOAD_STAGE(2, st0 + 8)
        }
#undef PA_CONSUME
#undef PA_FILL_X
#undef PA_LOAD_STAGE
    }
    write_state(REV ? 0 : nstate - 1, 1.f);
}

template <bool REV, bool EVERY, bool GATED>
__global__ __launch_bounds__(256) void k_mfma_scan(const bf16_t* __restrict__ Xt, const bf16_t* __restrict__ Yt,
                                                   const float* __restrict__ wgt, bf16_t* __restrict__ StC,
                                                   bf16_t* __restrict__ Gam, int T, int cs, float out_scale,
                                                   int nheads, const float* __restrict__ lam) {
    extern __shared__ __attribute__((aligned(16))) unsigned char scan_smem_raw[];
    ScanSmem& sm = *reinterpret_cast<ScanSmem*>(scan_smem_raw);
    // A scan workgroup is a long chain of dependent steps and the critical path of its pass; waves
    // of other kernels that share the SIMD (dQ runs side by side with the reverse scan) yield to it.
    __builtin_amdgcn_s_setprio(3);
    // Workgroups are dealt to the 8 XCDs round-robin by their linear id.  The NPAIR + 1 workgroups
    // of one head read the same K / V stream, so the logical work items (head-major) are laid out
    // in contiguous runs per XCD: a head's stream is then pulled into one or two L2s, not eight.
    const int total = (NPAIR + 1) * nheads;
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int base_cnt = total / 8, extra = total % 8;          // XCDs 0 .. extra-1 take one more
    const int cnt = base_cnt + (xcd < extra ? 1 : 0);
    if (q >= cnt) return;
    const int item = xcd * base_cnt + min(xcd, extra) + q;
    const int bh = item / (NPAIR + 1), pair = item % (NPAIR + 1);
    if (pair == NPAIR)
        scan_body<true, REV, EVERY, GATED>(Xt, Yt, wgt, StC, Gam, T, cs, out_scale, lam, sm, pair, bh);
    else
        scan_body<false, REV, EVERY, GATED>(Xt, Yt, wgt, StC, Gam, T, cs, out_scale, lam, sm, pair, bh);
}

}  // namespace

// LDS beyond the default per-kernel limit has to be requested once per kernel
template <typename F>
static bool allow_smem(F* fn, size_t bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) note_hip_error(e, "hipFuncSetAttribute(max dynamic LDS)");
    return e == hipSuccess;
}

bool launch_transpose(hipStream_t s, const bf16_t* in, bf16_t* out, int BH, int T, const float* fac, int out_T) {
    LaunchScope ls("mfma_transpose", s);
    hipLaunchKernelGGL(k_transpose, dim3(T / TBLK, BH), dim3(256), 0, s, in, out, T, fac, (out_T > 0 ? out_T : T) / TBLK);
    return launch_ok();
}

template <bool REV, bool EVERY, bool GATED>
static bool launch_scan_t(const char* name, hipStream_t s, const bf16_t* Xt, const bf16_t* Yt, const float* wgt,
                          bf16_t* stC, bf16_t* gam, int BH, int T, int cs, float out_scale, const float* lam) {
    if (!allow_smem(k_mfma_scan<REV, EVERY, GATED>, scan_smem_bytes<REV>())) return false;
    LaunchScope ls(name, s);
    const int total = (NPAIR + 1) * BH;
    hipLaunchKernelGGL((k_mfma_scan<REV, EVERY, GATED>), dim3(8 * ((total + 7) / 8)), dim3(256), scan_smem_bytes<REV>(), s, Xt, Yt, wgt,
                       stC, gam, T, cs, out_scale, BH, lam);
    return launch_ok();
}

bool launch_scan(const char* name, hipStream_t s, bool rev, const bf16_t* Xt, const bf16_t* Yt, const float* wgt, bf16_t* stC,
                 bf16_t* gam, int BH, int T, int cs, float out_scale, const float* lam) {
    const bool every = cs == SCAN_TOK;
#define PA_GO(R, E, G) return launch_scan_t<R, E, G>(name, s, Xt, Yt, wgt, stC, gam, BH, T, cs, out_scale, lam);
    if (lam == nullptr) {
        if (!rev) {
            if (every) PA_GO(false, true, false)
            PA_GO(false, false, false)
        }
        if (every) PA_GO(true, true, false)
        PA_GO(true, false, false)
    }
    if (!rev) {
        if (every) PA_GO(false, true, true)
        PA_GO(false, false, true)
    }
    if (every) PA_GO(true, true, true)
    PA_GO(true, false, true)
#undef PA_GO
}

}  // namespace mfma
}  // namespace pa
