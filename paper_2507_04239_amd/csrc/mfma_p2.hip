// bf16 MFMA kernel family for degree p = 2 (gfx950, 64-wide wavefronts).
//
// Chunked form of arXiv 2507.04239 (Sec. 2 "Chunked form", App. E) with the tiled
// symmetric-power embedding of Sec. 4.1.1 at d_tile = 8:  the expanded row (ti, tj, a, b),
// ti <= tj, of phi(x) is x[8 ti + a] * x[8 tj + b]; tiles off the diagonal carry the
// multiplicity 2, which is applied once, to the state (instead of sqrt(2) on both sides).
// Expanded operands are built in registers in MFMA operand order and never stored.
//
//   state scan   (App. E.2 + E.3): S_n = sum_{j < n*cs} phi(k_j) v_j^T as bf16 tiles, written
//                in the exact order the read-out kernel's MFMA operand wants them, plus the
//                normaliser state (sum of expanded keys, gamma of App. E.2) kept in its
//                un-symmetrised d x d form Gamma_n = sum_j k_j k_j^T.
//   chunk kernel (App. E.1 + E.4): attention form inside the chunk, phi(Q) S read-out,
//                phi(Q).gamma = q^T Gamma q, combination and normalisation.
//
// MFMA used: v_mfma_f32_16x16x32_bf16.  Operand layout (lane l, r16 = l % 16, g = l / 16):
//   A: row r16,   k-slots 8g..8g+7        B: column r16, k-slots 8g..8g+7
//   C: column r16, rows 4g..4g+3 (4 floats)
// Only the pairing of A and B k-slots matters, so k-slots are assigned to whatever order
// the data is already in (no shuffles between the two MFMAs of the attention form).
#include "common.hpp"

namespace pa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int DH = 64;                         // head size (d = v)
constexpr int NTB = DH / 8;                    // 8-wide feature blocks
constexpr int NTILES = NTB * (NTB + 1) / 2;    // 36 tiles of 64 expanded rows
constexpr int TILE_ELEMS = 8 * DH * 8;         // [a][v][b]
constexpr int QBLK = 128;                      // query rows per workgroup of the chunk kernel
constexpr int RO_PF = 8;                       // read-out steps kept in flight (72 % RO_PF == 0, even)

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

union Frag {
    bf16x8 v;
    uint4 u;
    uint2 h[2];
};

// ---- token-major -> feature-major in blocks of 64 tokens -----------------------------------
// [BH][T][DH] -> [BH][T/64][DH][64] (bf16).  Each block is 8 KB contiguous, so the readers'
// accesses stay dense (rows of a plain [DH][T] transpose would sit a power of two apart and
// pile onto the same memory channel).
constexpr int TBLK = 64;

__global__ __launch_bounds__(256) void k_transpose(const bf16_t* __restrict__ in, bf16_t* __restrict__ out, int T) {
    __shared__ bf16_t tile[TBLK][DH + 2];
    const int bh = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const bf16_t* src = in + ((size_t)bh * T + (size_t)blk * TBLK) * DH;
    for (int e = tid; e < TBLK * DH; e += 256) tile[e / DH][e % DH] = src[e];
    __syncthreads();
    bf16_t* dst = out + ((size_t)bh * (T / TBLK) + blk) * DH * TBLK;
    for (int e = tid; e < TBLK * DH; e += 256) dst[e] = tile[e % TBLK][e / TBLK];
}

// ---- state scan ----------------------------------------------------------------------------
// Fused update-state + cumulative sum over chunks (App. E.2 + E.3, no gating), used for
//   the forward state     S_n = sum_{j <  n cs}     phi(k_j) v_j^T        (X = K, Y = V)
//   the state gradient    R_m = sum_{i >= (m+1) cs} phi(q_i) ghat_i^T     (X = Q, Y = dO/Z, REV)
// grid (NPAIR + 1, BH), 256 threads.  Workgroup `pair` owns the two 64 x DH state tiles
// 2 pair, 2 pair + 1; wave w owns 32 rows (a in 4(w&1) .. +3) of tile 2 pair + (w >> 1).
// Workgroup NPAIR owns the normaliser in its d x d form: Gamma = sum k k^T, or
// Omega = sum gz_i q_i q_i^T for the gradient (same code: the A operand is x itself, times the
// weight, and the B operand comes from X instead of Y; only waves 0 and 1 have rows).
// The state is written every `cs` tokens, before the tokens of that stretch are added.
//
// Each workgroup walks the sequence in stages of 128 tokens.  A stage's X (as float32) and Y
// (bf16) are staged in LDS, feature-major, and shared by the four waves; the global loads of
// SCAN_PF further stages are in flight in registers.
//
// Two layouts of a 64-row tile (bf16), chosen by which contraction the reader does:
//   "C" [a][v][b]   8 expanded rows contiguous: operand of a contraction over rows (read-out)
//   "R" [row][v]    8 value columns contiguous: operand of a contraction over v (d phi)
constexpr int NPAIR = NTILES / 2;
constexpr int SCAN_TOK = 128;                  // tokens per stage
constexpr int SCAN_PF = 3;                     // stages in flight in registers
constexpr int XS_PITCH = SCAN_TOK + 4;         // floats; pitch = 4 mod 64 banks
constexpr int YS_PITCH = SCAN_TOK + 8;         // bf16;   pitch = 4 mod 64 banks (in dwords)
constexpr int TR_PITCH = DH + 8;               // bf16
static_assert(NTILES % 2 == 0, "tiles are handled in pairs");

struct ScanSmem {
    float xs[2][DH][XS_PITCH];
    bf16_t ys[2][DH][YS_PITCH];
    float ws[2][SCAN_TOK];
    bf16_t tr[4][32][TR_PITCH];
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory,
// i.e. waits for every outstanding global load, which would drain the register ring below.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <bool GAMMA, bool REV, bool WC, bool WR>
__device__ __forceinline__ void scan_body(const bf16_t* __restrict__ Xt, const bf16_t* __restrict__ Yt,
                                          const float* __restrict__ wgt, bf16_t* __restrict__ StC,
                                          bf16_t* __restrict__ StR, bf16_t* __restrict__ Gam, int T, int cs,
                                          float out_scale, ScanSmem& sm) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    const int nstate = T / cs;
    const int tile = GAMMA ? 0 : 2 * (int)blockIdx.x + (w >> 1);
    int ti = 0, tj = 0;
    for (int l = 0; l < tile; ++l) {
        if (++ti > tj) {
            ++tj;
            ti = 0;
        }
    }
    const float mult = GAMMA ? out_scale : ((ti == tj) ? 1.f : 2.f) * out_scale;
    // feature rows this lane expands: row block rbk in {0,1} covers tile rows 32 (w&1) + 16 rbk + r16
    //   tiles: a = 4 (w&1) + 2 rbk + (r16 >> 3), b = r16 & 7;   Gamma: feature 32 w + 16 rbk + r16
    const int fa0 = GAMMA ? (32 * (w & 1) + r16) : 8 * ti + 4 * (w & 1) + (r16 >> 3);
    const int fa_step = GAMMA ? 16 : 2;
    const int fb = 8 * tj + (r16 & 7);
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

    f32x4 acc[2][4];
#pragma unroll
    for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[rbk][cb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    auto write_state = [&](int n) {
        if (!GAMMA) {
            const size_t tbase = ((size_t)(bh * nstate + n) * NTILES + tile) * TILE_ELEMS;
            if (WC) {
                bf16_t* dst = StC + tbase;
#pragma unroll
                for (int rbk = 0; rbk < 2; ++rbk) {
                    const int a = 4 * (w & 1) + 2 * rbk + (g >> 1), b0 = 4 * (g & 1);
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) {
                        bf16x4 o;
#pragma unroll
                        for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[rbk][cb][r] * mult);
                        *(bf16x4*)(dst + ((a * DH + 16 * cb + r16) * 8 + b0)) = o;
                    }
                }
            }
            if (WR) {
                // transpose the wave's 32 x 64 block through its private LDS patch, then store rows
#pragma unroll
                for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            sm.tr[w][16 * rbk + 4 * g + r][16 * cb + r16] = f32_to_bf16(acc[rbk][cb][r] * mult);
                bf16_t* dst = StR + tbase + (size_t)32 * (w & 1) * DH;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int unit = lane + 64 * q;          // 32 rows x 8 units of 16 bytes
                    const uint4 val = *(const uint4*)&sm.tr[w][unit >> 3][8 * (unit & 7)];
                    *(uint4*)(dst + (unit >> 3) * DH + 8 * (unit & 7)) = val;
                }
            }
        } else if (has_rows) {
            bf16_t* dst = Gam + (size_t)(bh * nstate + n) * DH * DH;
#pragma unroll
            for (int rbk = 0; rbk < 2; ++rbk)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        dst[(32 * w + 16 * rbk + 4 * g + r) * DH + 16 * cb + r16] = f32_to_bf16(acc[rbk][cb][r] * mult);
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
        x0_##J = *(const uint4*)(Xh + so_ + p_off[0]);                                    \
        x1_##J = *(const uint4*)(Xh + so_ + p_off[1]);                                    \
        x2_##J = *(const uint4*)(Xh + so_ + p_off[2]);                                    \
        x3_##J = *(const uint4*)(Xh + so_ + p_off[3]);                                    \
        y0_##J = *(const uint4*)(Yh + so_ + p_off[0]);                                    \
        y1_##J = *(const uint4*)(Yh + so_ + p_off[1]);                                    \
        y2_##J = *(const uint4*)(Yh + so_ + p_off[2]);                                    \
        y3_##J = *(const uint4*)(Yh + so_ + p_off[3]);                                    \
        if (GAMMA && REV) wv_##J = Wh[(size_t)sidx_ * SCAN_TOK + (tid & (SCAN_TOK - 1))]; \
    }
#define PA_FILL_X(BUF, Q, XR)                                                             \
    {                                                                                     \
        float* d_ = &sm.xs[BUF][p_feat[Q]][p_tok[Q]];                                     \
        *(float4*)d_ = make_float4(bf_lo(XR.x), bf_hi(XR.x), bf_lo(XR.y), bf_hi(XR.y));   \
        *(float4*)(d_ + 4) = make_float4(bf_lo(XR.z), bf_hi(XR.z), bf_lo(XR.w), bf_hi(XR.w)); \
    }
#define PA_CONSUME(J, ST, BUF)                                                                \
    if ((ST) < nstage) { /* uniform; no global loads inside this branch */                    \
        const int edge_ = REV ? T - (ST) * SCAN_TOK : (ST) * SCAN_TOK;                        \
        if (edge_ % cs == 0) write_state(REV ? edge_ / cs - 1 : edge_ / cs);                  \
        PA_FILL_X(BUF, 0, x0_##J) PA_FILL_X(BUF, 1, x1_##J)                                   \
        PA_FILL_X(BUF, 2, x2_##J) PA_FILL_X(BUF, 3, x3_##J)                                   \
        *(uint4*)&sm.ys[BUF][p_feat[0]][p_tok[0]] = y0_##J;                                   \
        *(uint4*)&sm.ys[BUF][p_feat[1]][p_tok[1]] = y1_##J;                                   \
        *(uint4*)&sm.ys[BUF][p_feat[2]][p_tok[2]] = y2_##J;                                   \
        *(uint4*)&sm.ys[BUF][p_feat[3]][p_tok[3]] = y3_##J;                                   \
        if (GAMMA && REV && tid < SCAN_TOK) sm.ws[BUF][tid] = wv_##J;                         \
        lds_barrier();                                                                        \
        if (has_rows) {                                                                       \
            _Pragma("unroll") for (int s_ = 0; s_ < SCAN_TOK / 32; ++s_) {                    \
                const int t0_ = 32 * s_ + 8 * g;                                              \
                float xb_[8];                                                                 \
                if (!GAMMA) {                                                                 \
                    const float4 l_ = *(const float4*)&sm.xs[BUF][fb][t0_];                   \
                    const float4 h_ = *(const float4*)&sm.xs[BUF][fb][t0_ + 4];               \
                    xb_[0] = l_.x; xb_[1] = l_.y; xb_[2] = l_.z; xb_[3] = l_.w;               \
                    xb_[4] = h_.x; xb_[5] = h_.y; xb_[6] = h_.z; xb_[7] = h_.w;               \
                } else if (REV) {                                                             \
                    const float4 l_ = *(const float4*)&sm.ws[BUF][t0_];                       \
                    const float4 h_ = *(const float4*)&sm.ws[BUF][t0_ + 4];                   \
                    xb_[0] = l_.x; xb_[1] = l_.y; xb_[2] = l_.z; xb_[3] = l_.w;               \
                    xb_[4] = h_.x; xb_[5] = h_.y; xb_[6] = h_.z; xb_[7] = h_.w;               \
                } else {                                                                      \
                    _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) xb_[i_] = 1.f;           \
                }                                                                             \
                Frag af_[2];                                                                  \
                _Pragma("unroll") for (int rbk_ = 0; rbk_ < 2; ++rbk_) {                      \
                    const float* xa_ = &sm.xs[BUF][fa0 + fa_step * rbk_][t0_];                \
                    const float4 l_ = *(const float4*)xa_;                                    \
                    const float4 h_ = *(const float4*)(xa_ + 4);                              \
                    af_[rbk_].v[0] = (__bf16)(l_.x * xb_[0]); af_[rbk_].v[1] = (__bf16)(l_.y * xb_[1]); \
                    af_[rbk_].v[2] = (__bf16)(l_.z * xb_[2]); af_[rbk_].v[3] = (__bf16)(l_.w * xb_[3]); \
                    af_[rbk_].v[4] = (__bf16)(h_.x * xb_[4]); af_[rbk_].v[5] = (__bf16)(h_.y * xb_[5]); \
                    af_[rbk_].v[6] = (__bf16)(h_.z * xb_[6]); af_[rbk_].v[7] = (__bf16)(h_.w * xb_[7]); \
                }                                                                             \
                _Pragma("unroll") for (int cb_ = 0; cb_ < 4; ++cb_) {                         \
                    Frag bf_;                                                                 \
                    bf_.u = *(const uint4*)&sm.ys[BUF][16 * cb_ + r16][t0_];                  \
                    acc[0][cb_] = mfma16(af_[0].v, bf_.v, acc[0][cb_]);                       \
                    acc[1][cb_] = mfma16(af_[1].v, bf_.v, acc[1][cb_]);                       \
                }                                                                             \
            }                                                                                 \
        }                                                                                     \
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
    write_state(REV ? 0 : nstate - 1);
}

template <bool REV, bool WC, bool WR>
__global__ __launch_bounds__(256) void k_mfma_scan(const bf16_t* __restrict__ Xt, const bf16_t* __restrict__ Yt,
                                                   const float* __restrict__ wgt, bf16_t* __restrict__ StC,
                                                   bf16_t* __restrict__ StR, bf16_t* __restrict__ Gam, int T, int cs,
                                                   float out_scale) {
    extern __shared__ __attribute__((aligned(16))) unsigned char scan_smem_raw[];
    ScanSmem& sm = *reinterpret_cast<ScanSmem*>(scan_smem_raw);
    if (blockIdx.x == NPAIR)
        scan_body<true, REV, WC, WR>(Xt, Yt, wgt, StC, StR, Gam, T, cs, out_scale, sm);
    else
        scan_body<false, REV, WC, WR>(Xt, Yt, wgt, StC, StR, Gam, T, cs, out_scale, sm);
}

// ---- read-out: contraction over the expanded rows (query-state, App. E.4) -----------------------
// acc[vb][ib] (+)= S^T phi(x)^T for the 64 tokens of wave wv: 16 value columns x 16 tokens per
// block.  `Sn` is one state in layout "C"; `Xs` holds the block's 128 rows of x (float32, already
// scaled).  The state is one linear stream (step u = 2 tile + s holds rows a = 4s + g of the
// tile); RO_PF steps are kept in flight in registers, loads unconditional and clamped.
__device__ __forceinline__ void readout(f32x4 (&acc)[4][4], const bf16_t* __restrict__ Sn,
                                        const float (*Xs)[DH + 4], int wv, int r16, int g) {
    Sn += (size_t)g * DH * 8 + r16 * 8;
    constexpr int STEP_ELEMS = 4 * DH * 8;
    Frag sf[RO_PF][4];
#pragma unroll
    for (int j = 0; j < RO_PF; ++j)
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) sf[j][vb].u = *(const uint4*)(Sn + (size_t)j * STEP_ELEMS + 16 * vb * 8);
    int ti = 0, tj = 0;
    float xbv[4][8];
    for (int u0 = 0; u0 < 2 * NTILES; u0 += RO_PF) {
#pragma unroll
        for (int j = 0; j < RO_PF; ++j) {
            const int u = u0 + j;
            const int s = j & 1;
            if (s == 0) {
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    const float4 lo = *(const float4*)&Xs[64 * wv + 16 * ib + r16][8 * tj];
                    const float4 hi = *(const float4*)&Xs[64 * wv + 16 * ib + r16][8 * tj + 4];
                    xbv[ib][0] = lo.x; xbv[ib][1] = lo.y; xbv[ib][2] = lo.z; xbv[ib][3] = lo.w;
                    xbv[ib][4] = hi.x; xbv[ib][5] = hi.y; xbv[ib][6] = hi.z; xbv[ib][7] = hi.w;
                }
            }
            Frag pf[4];
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const float xa = Xs[64 * wv + 16 * ib + r16][8 * ti + 4 * s + g];
#pragma unroll
                for (int i = 0; i < 8; ++i) pf[ib].v[i] = (__bf16)(xa * xbv[ib][i]);
            }
#pragma unroll
            for (int vb = 0; vb < 4; ++vb)
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = mfma16(sf[j][vb].v, pf[ib].v, acc[vb][ib]);
            {
                const int un = min(u + RO_PF, 2 * NTILES - 1);
#pragma unroll
                for (int vb = 0; vb < 4; ++vb)
                    sf[j][vb].u = *(const uint4*)(Sn + (size_t)un * STEP_ELEMS + 16 * vb * 8);
            }
            if (s == 1) {
                if (++ti > tj) {
                    ++tj;
                    ti = 0;
                }
            }
        }
    }
}

// ---- d phi: contraction over the value columns, then the Jacobian of phi ----------------------
// For the 64 tokens of wave wv and a state `Sn` in layout "R":
//     A[row, token] = sum_v S[row, v] y[token, v]                      (MFMA)
//     Dacc[token][8 ti + a] += sum_b A[(a,b)] x[8 tj + b]
//     Dacc[token][8 tj + b] += sum_a A[(a,b)] x[8 ti + a]              (vector ALU)
// i.e. Dacc += J_phi(x)^T (S y) for phi(x)_(ti,tj,a,b) = x[8ti+a] x[8tj+b] (the multiplicity of
// the tile is already in S).  yf[ib][ks] are the B operands y^T (k-slots = v 32 ks + 8 g ..).
// Dacc rows of this wave's tokens are touched by this wave only.
__device__ __forceinline__ void dphi_contract(float (*Dacc)[DH + 4], const bf16_t* __restrict__ Sn,
                                              const Frag (&yf)[4][2], const float (*Xs)[DH + 4], int wv, int r16,
                                              int g) {
    const bf16_t* Sl = Sn + (size_t)r16 * DH + 8 * g;
    int ti = 0, tj = 0;
    for (int tile = 0; tile < NTILES; ++tile) {
        float u2[4][4];
#pragma unroll
        for (int ib = 0; ib < 4; ++ib)
#pragma unroll
            for (int r = 0; r < 4; ++r) u2[ib][r] = 0.f;
        Frag sf[4][2];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                sf[rb][ks].u = *(const uint4*)(Sl + ((size_t)tile * 64 + 16 * rb) * DH + 32 * ks);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int a = 2 * rb + (g >> 1);
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                c = mfma16(sf[rb][0].v, yf[ib][0].v, c);
                c = mfma16(sf[rb][1].v, yf[ib][1].v, c);
                const int tok = 64 * wv + 16 * ib + r16;
                const float4 xb = *(const float4*)&Xs[tok][8 * tj + 4 * (g & 1)];
                const float xa = Xs[tok][8 * ti + a];
                float t1 = c[0] * xb.x + c[1] * xb.y + c[2] * xb.z + c[3] * xb.w;
                t1 += __shfl_xor(t1, 16);
                if ((g & 1) == 0) Dacc[tok][8 * ti + a] += t1;
#pragma unroll
                for (int r = 0; r < 4; ++r) u2[ib][r] += c[r] * xa;
            }
        }
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) {
            const int tok = 64 * wv + 16 * ib + r16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float u = u2[ib][r];
                u += __shfl_xor(u, 32);
                if ((g >> 1) == 0) Dacc[tok][8 * tj + 4 * (g & 1) + r] += u;
            }
        }
        if (++ti > tj) {
            ++tj;
            ti = 0;
        }
    }
}

// stage `scale * X` rows [row0, row0 + 128) as float32 in LDS
__device__ __forceinline__ void stage_rows_f32(float (*Xs)[DH + 4], const bf16_t* __restrict__ X, size_t row0,
                                               float scale, int tid) {
    for (int e = tid; e < QBLK * DH / 8; e += 128) {
        const int row = e / (DH / 8), c8 = e % (DH / 8);
        const uint4 raw = *(const uint4*)(X + (row0 + row) * DH + 8 * c8);
        const uint32_t* pr = (const uint32_t*)&raw;
        float* dst = &Xs[row][8 * c8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dst[2 * i] = scale * bf_lo(pr[i]);
            dst[2 * i + 1] = scale * bf_hi(pr[i]);
        }
    }
}

// ---- chunk kernel: attention form + read-out + normalise --------------------------------------
// grid (T / 128, BH), 128 threads; wave wv owns query rows [64 wv, 64 wv + 64) of the block.
// Accumulators hold O^T: acc[vb][ib] = 16 value columns x 16 queries.
__global__ __launch_bounds__(128) void k_mfma_fwd_chunk(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                        const bf16_t* __restrict__ Vt, const bf16_t* __restrict__ St,
                                                        const bf16_t* __restrict__ Gam, bf16_t* __restrict__ O,
                                                        float* __restrict__ Z, int T, int cs, float scale,
                                                        int normalize) {
    __shared__ __attribute__((aligned(16))) float Qs[QBLK][DH + 4];   // scale * q, float32
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int qb = blockIdx.x, bh = blockIdx.y;
    const int i0 = qb * QBLK;                 // first query row of the block
    const int n = i0 / cs;                    // state entering the stretch this block lies in
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;

    // stage scale * Q as float32
    for (int e = tid; e < QBLK * DH / 8; e += 128) {
        const int row = e / (DH / 8), c8 = e % (DH / 8);
        const uint4 raw = *(const uint4*)(Q + (head_tok + i0 + row) * DH + 8 * c8);
        const uint32_t* pr = (const uint32_t*)&raw;
        float* dst = &Qs[row][8 * c8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dst[2 * i] = scale * bf_lo(pr[i]);
            dst[2 * i + 1] = scale * bf_hi(pr[i]);
        }
    }
    // Q^T as MFMA B operand: qf[ib][ks] = features 32 ks + 8 g .. +7 of query 64 wv + 16 ib + r16
    Frag qf[4][2];
#pragma unroll
    for (int ib = 0; ib < 4; ++ib)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            qf[ib][ks].u = *(const uint4*)(Q + (head_tok + i0 + 64 * wv + 16 * ib + r16) * DH + 32 * ks + 8 * g);

    f32x4 acc[4][4];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float zsum[4] = {0.f, 0.f, 0.f, 0.f};     // per query block ib: partial sum of scores (this lane's k-slots)
    __syncthreads();

    // ---- attention form over the keys of the stretch, up to the diagonal -----------------------
    const int key_lo = n * cs;
    for (int kb0 = key_lo; kb0 <= i0; kb0 += QBLK) {
        const bool diag = kb0 == i0;
        const int nsteps = diag ? 2 * (wv + 1) : 4;     // 32-key steps this wave needs
        for (int s = 0; s < nsteps; ++s) {
            const int key0 = kb0 + 32 * s;
            // S^T blocks: keys (2 blocks of 16) x queries (4 blocks of 16)
            f32x4 sc[2][4];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                Frag kf[2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    kf[ks].u = *(const uint4*)(K + (head_tok + key0 + 16 * jb + r16) * DH + 32 * ks + 8 * g);
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                    c = mfma16(kf[0].v, qf[ib][0].v, c);
                    c = mfma16(kf[1].v, qf[ib][1].v, c);
                    sc[jb][ib] = c;
                }
            }
            // p = 2: square, mask, row sums; pack as B operand (k-slots: keys 4g+r of block 2s, then of 2s+1)
            Frag pf[4];
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const int qrow = i0 + 64 * wv + 16 * ib + r16;
#pragma unroll
                for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float sv = scale * sc[jb][ib][r];
                        float pv = sv * sv;
                        if (diag && key0 + 16 * jb + 4 * g + r > qrow) pv = 0.f;
                        zsum[ib] += pv;
                        pf[ib].v[4 * jb + r] = (__bf16)pv;
                    }
            }
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) {
                Frag vf;
                const bf16_t* vp = Vt + (size_t)bh * DH * T + (size_t)(key0 / TBLK) * (DH * TBLK) +
                                   (16 * vb + r16) * TBLK + (key0 % TBLK) + 4 * g;
                vf.h[0] = *(const uint2*)vp;
                vf.h[1] = *(const uint2*)(vp + 16);
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = mfma16(vf.v, pf[ib].v, acc[vb][ib]);
            }
        }
    }

    if (n > 0) {
        // ---- phi(q) . gamma = (scale q)^T Gamma (scale q) ----------------------------------------
        const bf16_t* Gn = Gam + (size_t)(bh * nstate + n) * DH * DH;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
            Frag gf[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) gf[ks].u = *(const uint4*)(Gn + (16 * ab + r16) * DH + 32 * ks + 8 * g);
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                c = mfma16(gf[0].v, qf[ib][0].v, c);
                c = mfma16(gf[1].v, qf[ib][1].v, c);
                const float4 qv = *(const float4*)&Qs[64 * wv + 16 * ib + r16][16 * ab + 4 * g];
                zsum[ib] += scale * (c[0] * qv.x + c[1] * qv.y + c[2] * qv.z + c[3] * qv.w);
            }
        }
        readout(acc, St + (size_t)(bh * nstate + n) * NTILES * TILE_ELEMS, Qs, wv, r16, g);
    }

    // ---- normalise and store ------------------------------------------------------------------
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        float z = zsum[ib];
        z += __shfl_xor(z, 16);
        z += __shfl_xor(z, 32);
        const float inv = normalize ? (z != 0.f ? 1.f / z : 0.f) : 1.f;
        const size_t row = head_tok + i0 + 64 * wv + 16 * ib + r16;
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[vb][ib][r] * inv);
            *(bf16x4*)(O + row * DH + 16 * vb + 4 * g) = o;
        }
        if (Z != nullptr && g == 0) Z[row] = z;
    }
}

// ---- backward: preparation -----------------------------------------------------------------------
// ghat = dO / Z (bf16, [BH][T][DH]) and gz = -(ghat . O) (float32, [BH][T]); un-normalised:
// ghat = dO, gz = 0.  Rows with Z == 0 give zeros.  One 16-lane group per row.
__global__ __launch_bounds__(256) void k_mfma_bwd_prep(const bf16_t* __restrict__ dO, const bf16_t* __restrict__ O,
                                                       const float* __restrict__ Z, bf16_t* __restrict__ Gh,
                                                       float* __restrict__ gz, long long rows, int normalize) {
    const long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int c4 = threadIdx.x & 15;
    if (row >= rows) return;
    const uint2 graw = *(const uint2*)(dO + row * DH + 4 * c4);
    const float gv[4] = {bf_lo(graw.x), bf_hi(graw.x), bf_lo(graw.y), bf_hi(graw.y)};
    float inv = 1.f;
    if (normalize) {
        const float z = Z[row];
        inv = z != 0.f ? 1.f / z : 0.f;
    }
    bf16x4 o;
    float gr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[i] = (__bf16)(gv[i] * inv);
        gr[i] = (float)o[i];
    }
    *(bf16x4*)(Gh + row * DH + 4 * c4) = o;
    // gz is formed from the ROUNDED ghat, so that ghat . v_j + gz = ghat . (v_j - O_i) keeps its
    // exact cancellations (a row that attends to one key only gets a zero gradient, as it must)
    float delta = 0.f;
    if (normalize) {
        const uint2 oraw = *(const uint2*)(O + row * DH + 4 * c4);
        delta = gr[0] * bf_lo(oraw.x) + gr[1] * bf_hi(oraw.x) + gr[2] * bf_lo(oraw.y) + gr[3] * bf_hi(oraw.y);
        delta += __shfl_xor(delta, 1);
        delta += __shfl_xor(delta, 2);
        delta += __shfl_xor(delta, 4);
        delta += __shfl_xor(delta, 8);
    }
    if (c4 == 0) gz[row] = -delta;
}

// ---- backward, queries: dQ ------------------------------------------------------------------------
// grid (T / 128, BH), 128 threads; wave wv owns query rows [64 wv, 64 wv + 64) of the block.
//   dq_i = scale * [ sum_{j<=i, same stretch} t_ij k_j + 2 gz_i Gamma q~_i + J_phi(q~_i)^T (S_n ghat_i) ]
//   q~ = scale q,  s_ij = q~_i . k_j,  t_ij = 2 s_ij (ghat_i . v_j + gz_i)
// acc[fb][ib] holds the attention-form part transposed (16 features x 16 queries); the state part
// is accumulated in LDS (Dacc).
__global__ __launch_bounds__(128) void k_mfma_bwd_dq(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                     const bf16_t* __restrict__ V, const bf16_t* __restrict__ Gh,
                                                     const float* __restrict__ gz, const bf16_t* __restrict__ Kt,
                                                     const bf16_t* __restrict__ StR, const bf16_t* __restrict__ Gam,
                                                     bf16_t* __restrict__ dQ, int T, int cs, float scale) {
    __shared__ __attribute__((aligned(16))) float Qs[QBLK][DH + 4];
    __shared__ __attribute__((aligned(16))) float Dacc[QBLK][DH + 4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int qb = blockIdx.x, bh = blockIdx.y;
    const int i0 = qb * QBLK;
    const int n = i0 / cs;
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;

    stage_rows_f32(Qs, Q, head_tok + i0, scale, tid);
    for (int e = tid; e < QBLK * (DH + 4); e += 128) (&Dacc[0][0])[e] = 0.f;
    Frag qf[4][2], gf[4][2];
    float gzq[4];
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        const size_t row = head_tok + i0 + 64 * wv + 16 * ib + r16;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            qf[ib][ks].u = *(const uint4*)(Q + row * DH + 32 * ks + 8 * g);
            gf[ib][ks].u = *(const uint4*)(Gh + row * DH + 32 * ks + 8 * g);
        }
        gzq[ib] = gz[row];
    }
    f32x4 acc[4][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) acc[fb][ib] = (f32x4){0.f, 0.f, 0.f, 0.f};
    __syncthreads();

    const int key_lo = n * cs;
    for (int kb0 = key_lo; kb0 <= i0; kb0 += QBLK) {
        const bool diag = kb0 == i0;
        const int nsteps = diag ? 2 * (wv + 1) : 4;
        for (int s = 0; s < nsteps; ++s) {
            const int key0 = kb0 + 32 * s;
            f32x4 sc[2][4], ec[2][4];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                Frag kf[2], vf[2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    kf[ks].u = *(const uint4*)(K + (head_tok + key0 + 16 * jb + r16) * DH + 32 * ks + 8 * g);
                    vf[ks].u = *(const uint4*)(V + (head_tok + key0 + 16 * jb + r16) * DH + 32 * ks + 8 * g);
                }
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                    c = mfma16(kf[0].v, qf[ib][0].v, c);
                    c = mfma16(kf[1].v, qf[ib][1].v, c);
                    sc[jb][ib] = c;
                    f32x4 e = (f32x4){0.f, 0.f, 0.f, 0.f};
                    e = mfma16(vf[0].v, gf[ib][0].v, e);
                    e = mfma16(vf[1].v, gf[ib][1].v, e);
                    ec[jb][ib] = e;
                }
            }
            Frag tf[4];
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const int qrow = i0 + 64 * wv + 16 * ib + r16;
#pragma unroll
                for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float tv = 2.f * scale * sc[jb][ib][r] * (ec[jb][ib][r] + gzq[ib]);
                        if (diag && key0 + 16 * jb + 4 * g + r > qrow) tv = 0.f;
                        tf[ib].v[4 * jb + r] = (__bf16)tv;
                    }
            }
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) {
                Frag ktf;
                const bf16_t* kp = Kt + (size_t)bh * DH * T + (size_t)(key0 / TBLK) * (DH * TBLK) +
                                   (16 * fb + r16) * TBLK + (key0 % TBLK) + 4 * g;
                ktf.h[0] = *(const uint2*)kp;
                ktf.h[1] = *(const uint2*)(kp + 16);
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) acc[fb][ib] = mfma16(ktf.v, tf[ib].v, acc[fb][ib]);
            }
        }
    }

    if (n > 0) {
        // normaliser: d/dq~ of gz q~^T Gamma q~ = 2 gz Gamma q~
        const bf16_t* Gn = Gam + (size_t)(bh * nstate + n) * DH * DH;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
            Frag gm[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) gm[ks].u = *(const uint4*)(Gn + (16 * ab + r16) * DH + 32 * ks + 8 * g);
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                c = mfma16(gm[0].v, qf[ib][0].v, c);
                c = mfma16(gm[1].v, qf[ib][1].v, c);
                const int tok = 64 * wv + 16 * ib + r16;
                const float f = 2.f * gzq[ib] * scale;
#pragma unroll
                for (int r = 0; r < 4; ++r) Dacc[tok][16 * ab + 4 * g + r] += f * c[r];
            }
        }
        dphi_contract(Dacc, StR + (size_t)(bh * nstate + n) * NTILES * TILE_ELEMS, gf, Qs, wv, r16, g);
    }
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int ib = 0; ib < 4; ++ib)
#pragma unroll
            for (int r = 0; r < 4; ++r) Dacc[64 * wv + 16 * ib + r16][16 * fb + 4 * g + r] += acc[fb][ib][r];
    __syncthreads();
    for (int e = tid; e < QBLK * DH / 4; e += 128) {
        const int row = e / (DH / 4), c4 = e % (DH / 4);
        const float4 v4 = *(const float4*)&Dacc[row][4 * c4];
        bf16x4 o;
        o[0] = (__bf16)(scale * v4.x); o[1] = (__bf16)(scale * v4.y);
        o[2] = (__bf16)(scale * v4.z); o[3] = (__bf16)(scale * v4.w);
        *(bf16x4*)(dQ + (head_tok + i0 + row) * DH + 4 * c4) = o;
    }
}

// ---- backward, keys / values: dK, dV ----------------------------------------------------------------
// grid (T / 128, BH), 128 threads; wave wv owns key rows [64 wv, 64 wv + 64) of the block.
//   dv_j = sum_{i>=j, same stretch} s_ij^2 ghat_i + R_m^T phi(k_j)
//   dk_j = scale * sum_i t_ij q_i + 2 Omega_m k_j + J_phi(k_j)^T (R_m v_j)
// (R and Omega already carry scale^2).  accK / accV hold the attention-form parts transposed
// (16 features x 16 keys); the d phi part of dK is accumulated in LDS (Dacc).
__global__ __launch_bounds__(128) void k_mfma_bwd_dkdv(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                       const bf16_t* __restrict__ V, const bf16_t* __restrict__ Gh,
                                                       const float* __restrict__ gz, const bf16_t* __restrict__ Qt,
                                                       const bf16_t* __restrict__ Ght, const bf16_t* __restrict__ RtC,
                                                       const bf16_t* __restrict__ RtR, const bf16_t* __restrict__ Omg,
                                                       bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, int T, int cs,
                                                       float scale) {
    __shared__ __attribute__((aligned(16))) float Ks[QBLK][DH + 4];
    __shared__ __attribute__((aligned(16))) float Dacc[QBLK][DH + 4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int kb = blockIdx.x, bh = blockIdx.y;
    const int j0 = kb * QBLK;
    const int m = j0 / cs;
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;

    stage_rows_f32(Ks, K, head_tok + j0, 1.f, tid);
    for (int e = tid; e < QBLK * (DH + 4); e += 128) (&Dacc[0][0])[e] = 0.f;
    Frag kf[4][2], vf[4][2];   // K^T and V^T of this wave's keys as B operands
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        const size_t row = head_tok + j0 + 64 * wv + 16 * jb + r16;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            kf[jb][ks].u = *(const uint4*)(K + row * DH + 32 * ks + 8 * g);
            vf[jb][ks].u = *(const uint4*)(V + row * DH + 32 * ks + 8 * g);
        }
    }
    f32x4 accK[4][4], accV[4][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            accK[fb][jb] = (f32x4){0.f, 0.f, 0.f, 0.f};
            accV[fb][jb] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    __syncthreads();

    const int q_hi = (m + 1) * cs;   // queries of the same stretch, from the diagonal block on
    for (int qb0 = j0; qb0 < q_hi; qb0 += QBLK) {
        const bool diag = qb0 == j0;
        const int s_lo = diag ? 2 * wv : 0;    // queries before this wave's first key are masked
        for (int s = s_lo; s < 4; ++s) {
            const int q0 = qb0 + 32 * s;
            f32x4 sc[2][4], ec[2][4];
            float gzr[2][4];
#pragma unroll
            for (int ibq = 0; ibq < 2; ++ibq) {
                Frag qa[2], ga[2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    qa[ks].u = *(const uint4*)(Q + (head_tok + q0 + 16 * ibq + r16) * DH + 32 * ks + 8 * g);
                    ga[ks].u = *(const uint4*)(Gh + (head_tok + q0 + 16 * ibq + r16) * DH + 32 * ks + 8 * g);
                }
                const float4 gz4 = *(const float4*)(gz + head_tok + q0 + 16 * ibq + 4 * g);
                gzr[ibq][0] = gz4.x; gzr[ibq][1] = gz4.y; gzr[ibq][2] = gz4.z; gzr[ibq][3] = gz4.w;
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) {
                    f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                    c = mfma16(qa[0].v, kf[jb][0].v, c);
                    c = mfma16(qa[1].v, kf[jb][1].v, c);
                    sc[ibq][jb] = c;
                    f32x4 e = (f32x4){0.f, 0.f, 0.f, 0.f};
                    e = mfma16(ga[0].v, vf[jb][0].v, e);
                    e = mfma16(ga[1].v, vf[jb][1].v, e);
                    ec[ibq][jb] = e;
                }
            }
            Frag tf[4], af[4];
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                const int krow = j0 + 64 * wv + 16 * jb + r16;
#pragma unroll
                for (int ibq = 0; ibq < 2; ++ibq)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float sv = scale * sc[ibq][jb][r];
                        float tv = 2.f * sv * (ec[ibq][jb][r] + gzr[ibq][r]);
                        float av = sv * sv;
                        if (diag && q0 + 16 * ibq + 4 * g + r < krow) {
                            tv = 0.f;
                            av = 0.f;
                        }
                        tf[jb].v[4 * ibq + r] = (__bf16)tv;
                        af[jb].v[4 * ibq + r] = (__bf16)av;
                    }
            }
            const size_t blk_off = (size_t)bh * DH * T + (size_t)(q0 / TBLK) * (DH * TBLK) + (q0 % TBLK) + 4 * g;
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) {
                Frag qtf, gtf;
                const bf16_t* qp = Qt + blk_off + (16 * fb + r16) * TBLK;
                const bf16_t* gp = Ght + blk_off + (16 * fb + r16) * TBLK;
                qtf.h[0] = *(const uint2*)qp;
                qtf.h[1] = *(const uint2*)(qp + 16);
                gtf.h[0] = *(const uint2*)gp;
                gtf.h[1] = *(const uint2*)(gp + 16);
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) {
                    accK[fb][jb] = mfma16(qtf.v, tf[jb].v, accK[fb][jb]);
                    accV[fb][jb] = mfma16(gtf.v, af[jb].v, accV[fb][jb]);
                }
            }
        }
    }
    // attention-form part of dK carries one more factor scale (d s / d k = scale q)
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int jb = 0; jb < 4; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) accK[fb][jb][r] *= scale;

    if (m < nstate - 1) {
        const bf16_t* Om = Omg + (size_t)(bh * nstate + m) * DH * DH;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
            Frag gm[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) gm[ks].u = *(const uint4*)(Om + (16 * ab + r16) * DH + 32 * ks + 8 * g);
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                f32x4 c = (f32x4){0.f, 0.f, 0.f, 0.f};
                c = mfma16(gm[0].v, kf[jb][0].v, c);
                c = mfma16(gm[1].v, kf[jb][1].v, c);
#pragma unroll
                for (int r = 0; r < 4; ++r) accK[ab][jb][r] += 2.f * c[r];
            }
        }
        readout(accV, RtC + (size_t)(bh * nstate + m) * NTILES * TILE_ELEMS, Ks, wv, r16, g);
        dphi_contract(Dacc, RtR + (size_t)(bh * nstate + m) * NTILES * TILE_ELEMS, vf, Ks, wv, r16, g);
    }
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            const size_t row = head_tok + j0 + 64 * wv + 16 * jb + r16;
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                Dacc[64 * wv + 16 * jb + r16][16 * fb + 4 * g + r] += accK[fb][jb][r];
                o[r] = (__bf16)accV[fb][jb][r];
            }
            *(bf16x4*)(dV + row * DH + 16 * fb + 4 * g) = o;
        }
    __syncthreads();
    for (int e = tid; e < QBLK * DH / 4; e += 128) {
        const int row = e / (DH / 4), c4 = e % (DH / 4);
        const float4 v4 = *(const float4*)&Dacc[row][4 * c4];
        bf16x4 o;
        o[0] = (__bf16)v4.x; o[1] = (__bf16)v4.y; o[2] = (__bf16)v4.z; o[3] = (__bf16)v4.w;
        *(bf16x4*)(dK + (head_tok + j0 + row) * DH + 4 * c4) = o;
    }
}

struct Layout {
    int cs, nstate;
    size_t off_kt, off_vt, off_sc, off_gam;                              // forward
    size_t off_qt, off_gh, off_ght, off_gz, off_sr, off_rc, off_rr, off_omg;  // backward only
    size_t total;
};

Layout make_layout(const pa_problem& pr, bool backward) {
    Layout L{};
    L.cs = pr.chunk;
    L.nstate = pr.T / L.cs;
    const size_t BH = (size_t)pr.B * pr.H;
    const size_t tok = BH * pr.T * DH * 2;
    const size_t st = BH * L.nstate * (size_t)NTILES * TILE_ELEMS * 2;
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
    if (!backward) {
        L.off_sc = take(st);
    } else {
        L.off_qt = take(tok);
        L.off_gh = take(tok);
        L.off_ght = take(tok);
        L.off_gz = take(BH * pr.T * sizeof(float));
        L.off_omg = take(gm);
        L.off_sr = take(st);
        L.off_rc = take(st);
        L.off_rr = take(st);
    }
    L.total = off;
    return L;
}

// LDS beyond the default per-kernel limit has to be requested once per kernel
template <typename F>
bool allow_smem(F* fn, size_t bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) note_hip_error(e, "hipFuncSetAttribute(max dynamic LDS)");
    return e == hipSuccess;
}

#define PA_LAUNCH(NAME, ...)                   \
    {                                          \
        LaunchScope ls_(NAME, c.stream);       \
        hipLaunchKernelGGL(__VA_ARGS__);       \
    }                                          \
    if (!launch_ok()) return PA_ERR_HIP;

}  // namespace

pa_status mfma_supported(const pa_problem& pr, bool backward) {
    (void)backward;
    if (pr.dtype != PA_DTYPE_BF16 || pr.p != 2) return PA_ERR_UNSUPPORTED;
    if (pr.d != DH || pr.v != DH) return PA_ERR_UNSUPPORTED;
    if (pr.chunk % QBLK != 0) return PA_ERR_UNSUPPORTED;
    if ((size_t)pr.B * pr.H > 65535u) return PA_ERR_UNSUPPORTED;
    return PA_OK;
}

long long mfma_state_rows(const pa_problem&) { return (long long)NTILES * 64; }

size_t mfma_workspace_bytes(const pa_problem& pr, bool backward) { return make_layout(pr, backward).total; }

pa_status mfma_fwd(const Ctx& c, const void* Q, const void* K, const void* V, void* O, float* Z) {
    const pa_problem& pr = c.prob;
    const Layout L = make_layout(pr, false);
    const unsigned BH = (unsigned)(pr.B * pr.H);
    bf16_t* Kt = (bf16_t*)(c.ws + L.off_kt);
    bf16_t* Vt = (bf16_t*)(c.ws + L.off_vt);
    bf16_t* Sc = (bf16_t*)(c.ws + L.off_sc);
    bf16_t* Gam = (bf16_t*)(c.ws + L.off_gam);
    const dim3 tgrid(pr.T / TBLK, BH);
    PA_LAUNCH("mfma_transpose", k_transpose, tgrid, dim3(256), 0, c.stream, (const bf16_t*)K, Kt, pr.T)
    PA_LAUNCH("mfma_transpose", k_transpose, tgrid, dim3(256), 0, c.stream, (const bf16_t*)V, Vt, pr.T)
    if (!allow_smem(k_mfma_scan<false, true, false>, sizeof(ScanSmem))) return PA_ERR_HIP;
    PA_LAUNCH("mfma_state_scan", (k_mfma_scan<false, true, false>), dim3(NPAIR + 1, BH), dim3(256), sizeof(ScanSmem), c.stream, Kt, Vt,
              (const float*)nullptr, Sc, (bf16_t*)nullptr, Gam, pr.T, L.cs, 1.0f)
    PA_LAUNCH("mfma_fwd_chunk", k_mfma_fwd_chunk, dim3(pr.T / QBLK, BH), dim3(128), 0, c.stream, (const bf16_t*)Q,
              (const bf16_t*)K, Vt, Sc, Gam, (bf16_t*)O, Z, pr.T, L.cs, pr.scale, pr.normalize)
    return PA_OK;
}

pa_status mfma_bwd(const Ctx& c, const void* Q, const void* K, const void* V, const void* O, const float* Z,
                   const void* dO, void* dQ, void* dK, void* dV) {
    const pa_problem& pr = c.prob;
    const Layout L = make_layout(pr, true);
    const unsigned BH = (unsigned)(pr.B * pr.H);
    bf16_t* Kt = (bf16_t*)(c.ws + L.off_kt);
    bf16_t* Vt = (bf16_t*)(c.ws + L.off_vt);
    bf16_t* Qt = (bf16_t*)(c.ws + L.off_qt);
    bf16_t* Gh = (bf16_t*)(c.ws + L.off_gh);
    bf16_t* Ght = (bf16_t*)(c.ws + L.off_ght);
    float* gz = (float*)(c.ws + L.off_gz);
    bf16_t* Gam = (bf16_t*)(c.ws + L.off_gam);
    bf16_t* Omg = (bf16_t*)(c.ws + L.off_omg);
    bf16_t* Sr = (bf16_t*)(c.ws + L.off_sr);
    bf16_t* Rc = (bf16_t*)(c.ws + L.off_rc);
    bf16_t* Rr = (bf16_t*)(c.ws + L.off_rr);
    const long long rows = (long long)BH * pr.T;
    const dim3 tgrid(pr.T / TBLK, BH);
    const float s2 = pr.scale * pr.scale;
    PA_LAUNCH("mfma_bwd_prep", k_mfma_bwd_prep, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, c.stream,
              (const bf16_t*)dO, (const bf16_t*)O, Z, Gh, gz, rows, pr.normalize)
    PA_LAUNCH("mfma_transpose", k_transpose, tgrid, dim3(256), 0, c.stream, (const bf16_t*)K, Kt, pr.T)
    PA_LAUNCH("mfma_transpose", k_transpose, tgrid, dim3(256), 0, c.stream, (const bf16_t*)V, Vt, pr.T)
    PA_LAUNCH("mfma_transpose", k_transpose, tgrid, dim3(256), 0, c.stream, (const bf16_t*)Q, Qt, pr.T)
    PA_LAUNCH("mfma_transpose", k_transpose, tgrid, dim3(256), 0, c.stream, (const bf16_t*)Gh, Ght, pr.T)
    // chunk states are recomputed (nothing but O and Z is saved by the forward pass), in the
    // layout the d phi contraction reads
    if (!allow_smem(k_mfma_scan<false, false, true>, sizeof(ScanSmem)) ||
        !allow_smem(k_mfma_scan<true, true, true>, sizeof(ScanSmem)))
        return PA_ERR_HIP;
    PA_LAUNCH("mfma_state_scan_bwd", (k_mfma_scan<false, false, true>), dim3(NPAIR + 1, BH), dim3(256), sizeof(ScanSmem), c.stream, Kt,
              Vt, (const float*)nullptr, (bf16_t*)nullptr, Sr, Gam, pr.T, L.cs, 1.0f)
    PA_LAUNCH("mfma_state_grad_scan", (k_mfma_scan<true, true, true>), dim3(NPAIR + 1, BH), dim3(256), sizeof(ScanSmem), c.stream, Qt,
              Ght, (const float*)gz, Rc, Rr, Omg, pr.T, L.cs, s2)
    PA_LAUNCH("mfma_bwd_dq", k_mfma_bwd_dq, dim3(pr.T / QBLK, BH), dim3(128), 0, c.stream, (const bf16_t*)Q,
              (const bf16_t*)K, (const bf16_t*)V, Gh, gz, Kt, Sr, Gam, (bf16_t*)dQ, pr.T, L.cs, pr.scale)
    PA_LAUNCH("mfma_bwd_dkdv", k_mfma_bwd_dkdv, dim3(pr.T / QBLK, BH), dim3(128), 0, c.stream, (const bf16_t*)Q,
              (const bf16_t*)K, (const bf16_t*)V, Gh, gz, Qt, Ght, Rc, Rr, Omg, (bf16_t*)dK, (bf16_t*)dV, pr.T, L.cs,
              pr.scale)
    return PA_OK;
}

}  // namespace pa
