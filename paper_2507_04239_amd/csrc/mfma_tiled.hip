// Chunked form on the matrix cores for any degree and tile width: the tiled symmetric-power embedding of
// arXiv 2507.04239 Sec. 4.1.1 (TSPOW) with the degree p and the tile width d_tile as template parameters,
// update-state + cumulative sum (App. E.2, E.3), query-state (App. E.4) and the state parts of the backward
// pass (derived from the forward definition; the paper gives none).
//
// Embedding.  The d features are cut into d / d_tile blocks; a tile is a non-decreasing multi-index
// (t_1 <= ... <= t_p) of blocks and holds the d_tile^p products x[d_tile t_1 + a_1] ... x[d_tile t_p + a_p].
// Its multiplicity p! / prod(run lengths)! is an integer and is put on the state (once) instead of its
// square root on both sides.  A row is written as (alpha, beta): alpha runs over the first p / 2 positions
// ("left", NL = d_tile^(p/2) values), beta over the others ("right", NR values), row = alpha NR + beta, so
// that phi[row] = uL[alpha] uR[beta] and the Jacobian factors the same way (dL/duL[alpha] = sum_beta A uR,
// dL/duR[beta] = sum_alpha A uL, then the chain rule through the one or two features of each side).
//
// Work is cut into units of 64 state rows: a 64-row slice of a tile (all beta for 64 / NR values of alpha)
// when a tile has 64 rows or more, else 64 / rows whole tiles.  phi is formed by one thread per token from
// that token's features (all digit loops are compile-time, no lane holds a lane-dependent digit), rounded to
// bf16 once and laid down in LDS as a [token][row] tile, from which the MFMA operands are read - plainly for
// a contraction over the rows, through the transposing LDS read for a contraction over the tokens.  The
// gradient with respect to phi takes the same road back: MFMA results go to LDS as [token][row] float32 and
// the thread that owns the token applies the Jacobian and adds into that token's d accumulators (LDS,
// [feature][token], touched by their owner only: plain read-add-write).
//
// States: per (head, chunk) `nunit` units of 64 rows x VP = d + 16 value columns, bf16, row-major; column d
// carries the normaliser (the values are extended by a one, App. E.4's l), the remaining 15 are zero.  In
// memory a row keeps only its first SP = d + 4 columns; the columns beyond exist in the read-out's LDS tile
// only, as zeros.  The read-out (contraction over the rows) passes a unit through LDS for the transposing read;
// d phi (contraction over the columns) takes its operand fragments, runs of 8 columns of one row, straight
// from memory.
// MFMA: v_mfma_f32_16x16x32_bf16 throughout; where the contraction runs over the value columns, the columns
// beyond d fill part of a k = 32 step, the rest is zero.  Operand layouts as in mfma_common.hpp.
#include <cmath>
#include <type_traits>

#include "mfma_common.hpp"

namespace pa {
namespace mfma {
namespace {

constexpr int ipowc(int b, int e) { return e == 0 ? 1 : b * ipowc(b, e - 1); }

template <int P, int DT>
struct Emb {
    static constexpr int PL = P / 2, PR = P - PL;
    static constexpr int NL = ipowc(DT, PL), NR = ipowc(DT, PR), R = NL * NR;
    static constexpr int TPU = R >= 64 ? 1 : 64 / R;    // tiles per unit
    static constexpr int UPT = R >= 64 ? R / 64 : 1;    // units per tile
    static constexpr int NA = R >= 64 ? 64 / NR : NL;   // left indices per unit (per tile when a unit holds whole tiles)
    static_assert(R % 16 == 0 && (R >= 64 ? 64 % NR == 0 : 64 % R == 0), "tile shape");
};

// 64 rows x W columns of bf16 in LDS.  What decides the pitch is the transposing read: each of 16 rows is read by 4
// lanes, 8 dwords in a row; with 64 banks and 32 lanes at a time that is free of conflicts when the pitch is an odd
// multiple of 8 dwords, which the widths of the state and value tiles (48, 80, 144) are as they stand (measured
// against 8 columns of padding: bank-conflict cycles of the scan 21 -> 11 %, of the read-out 31 -> 26 %, times
// unchanged).  The phi tile (64) is also written 16 bytes per token and read row-wise, and does best on all
// three with 8 columns of padding.
template <int W>
struct Tile64 {
    static constexpr int PITCH = W == 64 ? W + 8 : W;
    static_assert(W == 64 || (W / 2) % 16 == 8, "pitch: an odd multiple of 8 dwords");
    bf16_t r[64][PITCH];
};

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// Operand of a contraction over the tile's 64 rows: k-slots = rows 32 s + 8g .. + 7 (so that the other operand,
// read row-wise, is one 16-byte read per lane), lane r16 = column c0 + r16 % 4 of the four columns its pointer
// lane r16 / 4 names.  (The transposing read
// hands lane n of a 16-lane group column n of the 4 x 16 block whose row j the lanes 4j .. 4j+3 point at.)
template <int W>
__device__ __forceinline__ bf16x8 col_frag_at(const Tile64<W>& t, int s, int col4, int r16, int g) {
    const bf16_t* p = &t.r[32 * s + 8 * g + (r16 >> 2)][col4];
    union {
        bf16x8 v;
        bf16x4 h[2];
    } f;
    f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p);
    f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * Tile64<W>::PITCH));
    return f.v;
}
// columns 16 cb .. 16 cb + 15 in order
template <int W>
__device__ __forceinline__ bf16x8 col_frag(const Tile64<W>& t, int s, int cb, int r16, int g) {
    return col_frag_at<W>(t, s, 16 * cb + 4 * (r16 & 3), r16, g);
}

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
// A contraction over 16 columns, lane (r16, g) holding columns 4g .. 4g + 3 of its row: a k = 32 step whose slots
// 8g + 4 .. 8g + 7 are zero on both sides.  (Not v_mfma_f32_16x16x16_bf16: chained behind 16x16x32 steps with its
// result in other registers than its addend it read that addend too early - wrong values in 16 lanes, run to
// run, that wait states between the two kinds made go away.)
__device__ __forceinline__ f32x4 mfma16k16(uint2 a, uint2 b, f32x4 c) {
    Frag fa, fb;
    fa.u = make_uint4(a.x, a.y, 0u, 0u);
    fb.u = make_uint4(b.x, b.y, 0u, 0u);
    return mfma16(fa.v, fb.v, c);
}

// LDS traffic of one wave is ordered; this keeps the compiler from moving accesses across the hand-over
// between the lanes of a wave
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- the embedding, one thread per token ----------------------------------------------------------------
// A token's features as they wait in LDS for the thread that owns the token.
struct RowBF16 {
    const bf16_t* p;
    __device__ __forceinline__ float operator[](int i) const { return bf16_to_f32(p[i]); }
};
// A token's features in LDS: bf16 as they come (rows of float32 were tried where LDS has the room: slower, they
// cost a workgroup per CU at d = 32)
template <int HD>
struct XStore {
    typedef bf16_t elem;
    typedef RowBF16 row;
    static constexpr int PITCH = HD + 2;   // an odd number of dwords: the lanes' rows start in different banks
};

// x: the token's features.  td: the tile (uniform over the wave).
template <int P, int DT, typename X>
__device__ __forceinline__ void right_feats(const X x, const TileDesc& td, float (&uR)[Emb<P, DT>::NR]) {
    using E = Emb<P, DT>;
    if constexpr (E::PR == 1) {
#pragma unroll
        for (int b = 0; b < DT; ++b) uR[b] = x[DT * td.t[E::PL] + b];
    } else {
        float xc[DT], xd[DT];
#pragma unroll
        for (int i = 0; i < DT; ++i) {
            xc[i] = x[DT * td.t[E::PL] + i];
            xd[i] = x[DT * td.t[E::PL + 1] + i];
        }
#pragma unroll
        for (int c = 0; c < DT; ++c)
#pragma unroll
            for (int d = 0; d < DT; ++d) uR[c * DT + d] = xc[c] * xd[d];
    }
}
// alpha may be a run-time value (uniform over the wave): features are fetched from LDS by address
template <int P, int DT, typename X>
__device__ __forceinline__ float left_feat(const X x, const TileDesc& td, int alpha) {
    using E = Emb<P, DT>;
    if constexpr (E::PL == 1) return x[DT * td.t[0] + alpha];
    else return x[DT * td.t[0] + alpha / DT] * x[DT * td.t[1] + alpha % DT];
}

template <int P, int DT, typename X>
__device__ __forceinline__ void unit_phi(const X x, const TileDesc* __restrict__ tab, int unit, float (&phi)[64]) {
    using E = Emb<P, DT>;
    if constexpr (E::R >= 64) {
        const TileDesc td = tab[unit / E::UPT];
        const int a0 = (unit % E::UPT) * E::NA;
        float uR[E::NR];
        right_feats<P, DT>(x, td, uR);
#pragma unroll
        for (int ai = 0; ai < E::NA; ++ai) {
            const float ul = left_feat<P, DT>(x, td, a0 + ai);
#pragma unroll
            for (int b = 0; b < E::NR; ++b) phi[ai * E::NR + b] = ul * uR[b];
        }
    } else {
#pragma unroll
        for (int tt = 0; tt < E::TPU; ++tt) {
            const TileDesc td = tab[unit * E::TPU + tt];
            float uR[E::NR];
            right_feats<P, DT>(x, td, uR);
#pragma unroll
            for (int a = 0; a < E::NL; ++a) {
                const float ul = left_feat<P, DT>(x, td, a);
#pragma unroll
                for (int b = 0; b < E::NR; ++b) phi[tt * E::R + a * E::NR + b] = ul * uR[b];
            }
        }
    }
}

// Where a token's d accumulators of d phi live; add(f, v): dx[f] += v, f uniform over the wave.
// LDS: [feature][token], the token's column (stride 64 floats between features), touched by its owner only.
struct DxLds {
    float* col;
    __device__ __forceinline__ void add(int f, float v) { col[64 * f] += v; }
};
// Registers, indexed relative to a scalar (a vector type keeps a dynamically indexed array out of scratch memory):
// all 32 features of a token.
typedef float f32x32 __attribute__((ext_vector_type(32)));
struct DxRegs32 {
    f32x32 v;
    __device__ __forceinline__ void clear() { v = 0.f; }
    __device__ __forceinline__ void add(int f, float x) { v[f] += x; }
};
template <typename DX>
__device__ __forceinline__ void dx_add(DX& dx, int f, float v) { dx.add(f, v); }

// chain rule through one side: du[i] = dL/du for the N = DT^PS values of the side whose first position is
// `pos`; alpha0: index of du[0] within the side (non-zero only for a slice of the left side)
template <int DT, int PS, int N, typename X, typename DX>
__device__ __forceinline__ void side_chain(const X x, const TileDesc& td, int pos, int alpha0, const float (&du)[N], DX& dx) {
    if constexpr (PS == 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) dx_add(dx, DT * td.t[pos] + alpha0 + i, du[i]);
    } else if constexpr (N == DT * DT) {
        float xc[DT], xd[DT];
#pragma unroll
        for (int i = 0; i < DT; ++i) {
            xc[i] = x[DT * td.t[pos] + i];
            xd[i] = x[DT * td.t[pos + 1] + i];
        }
#pragma unroll
        for (int c = 0; c < DT; ++c) {
            float s = 0.f;
#pragma unroll
            for (int d = 0; d < DT; ++d) s += du[c * DT + d] * xd[d];
            dx_add(dx, DT * td.t[pos] + c, s);
        }
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            float s = 0.f;
#pragma unroll
            for (int c = 0; c < DT; ++c) s += du[c * DT + d] * xc[c];
            dx_add(dx, DT * td.t[pos + 1] + d, s);
        }
    } else {
        // a slice of a two-position side: N consecutive values starting at alpha0 (run-time, uniform)
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = (alpha0 + i) / DT, d = (alpha0 + i) % DT;
            dx_add(dx, DT * td.t[pos] + c, du[i] * x[DT * td.t[pos + 1] + d]);
            dx_add(dx, DT * td.t[pos + 1] + d, du[i] * x[DT * td.t[pos] + c]);
        }
    }
}

// The Jacobian of a unit, one block of 16 rows at a time (block nb = rows 16 nb .. 16 nb + 15 of the unit), for one
// token: A[i] = dL/dphi of the block's rows.  The right side's sums run over the whole unit (units of whole tiles:
// over the block's tile) and are landed by finish().
template <int P, int DT>
struct UnitJacobian {
    using E = Emb<P, DT>;
    static constexpr bool SLICE = E::R >= 64;                  // the unit is a slice of one tile
    static constexpr int APB = SLICE ? 16 / E::NR : E::NL;      // left indices per block
    static_assert(!SLICE || (E::NR <= 16 && 16 % E::NR == 0), "a block of 16 rows holds whole left indices");
    static_assert(SLICE || E::R == 16, "a block of 16 rows is one tile");
    float uR[E::NR], dR[E::NR];
    TileDesc td;
    int a0;

    template <typename X>
    __device__ __forceinline__ void begin(const X x, const TileDesc* __restrict__ tab, int unit) {
        if constexpr (SLICE) {
            td = tab[unit / E::UPT];
            a0 = (unit % E::UPT) * E::NA;
            right_feats<P, DT>(x, td, uR);
#pragma unroll
            for (int b = 0; b < E::NR; ++b) dR[b] = 0.f;
        }
    }
    template <typename X, typename DX>
    __device__ __forceinline__ void block(const X x, const TileDesc* __restrict__ tab, int unit, int nb, const float (&A)[16],
                                          DX& dx) {
        if constexpr (!SLICE) {
            td = tab[unit * E::TPU + nb];
            a0 = 0;
            right_feats<P, DT>(x, td, uR);
#pragma unroll
            for (int b = 0; b < E::NR; ++b) dR[b] = 0.f;
        }
        float dL[APB];
#pragma unroll
        for (int aa = 0; aa < APB; ++aa) {
            const float ul = left_feat<P, DT>(x, td, a0 + (SLICE ? nb * APB : 0) + aa);
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < E::NR; ++b) {
                s += A[aa * E::NR + b] * uR[b];
                dR[b] += A[aa * E::NR + b] * ul;
            }
            dL[aa] = s;
        }
        side_chain<DT, E::PL, APB>(x, td, 0, a0 + (SLICE ? nb * APB : 0), dL, dx);
        if constexpr (!SLICE) side_chain<DT, E::PR, E::NR>(x, td, E::PL, 0, dR, dx);
    }
    template <typename X, typename DX>
    __device__ __forceinline__ void finish(const X x, DX& dx) {
        if constexpr (SLICE) side_chain<DT, E::PR, E::NR>(x, td, E::PL, 0, dR, dx);
    }
};

// ntok token rows of X (bf16, [.][HD]) -> xs[token][.]
template <int HD, int NT>
__device__ __forceinline__ void stage_x(bf16_t (*xs)[XStore<HD>::PITCH], const bf16_t* __restrict__ Xrows, int ntok, int tid) {
    for (int id = tid; id < ntok * (HD / 8); id += NT) {
        const int row = id / (HD / 8), c8 = id % (HD / 8);
        const uint4 u = *(const uint4*)(Xrows + (size_t)row * HD + 8 * c8);
        uint32_t* dst = (uint32_t*)&xs[row][8 * c8];   // rows start on a dword, not on 16 bytes
        dst[0] = u.x; dst[1] = u.y; dst[2] = u.z; dst[3] = u.w;
    }
}

// phi[64] (its 8-row pieces I0 .. I1 - 1) -> one row of a [token][row] tile, rounded to bf16
template <int I0 = 0, int I1 = 8>
__device__ __forceinline__ void put_phi(Tile64<64>& t, int token, const float (&phi)[64]) {
#pragma unroll
    for (int i = I0; i < I1; ++i) {
        Frag f;
#pragma unroll
        for (int j = 0; j < 8; ++j) f.v[j] = (__bf16)phi[8 * i + j];
        *(uint4*)&t.r[token][8 * i] = f.u;
    }
}

// ---- tile table ------------------------------------------------------------------------------------------
__device__ __forceinline__ int binom(int n, int k) {
    if (k < 0 || k > n) return 0;
    int r = 1;
    for (int i = 1; i <= k; ++i) r = r * (n - k + i) / i;
    return r;
}
// entry i: the i-th non-decreasing multi-index of length p over nb blocks (lexicographic) and its
// multiplicity; entries from ntile on are padding (multiplicity 0: their state rows stay zero)
__global__ __launch_bounds__(256) void k_tile_table(TileDesc* __restrict__ tab, int p, int nb, int ntile, int nentry) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= nentry) return;
    TileDesc td;
    td.t[0] = td.t[1] = td.t[2] = td.t[3] = 0;
    td.mult = 0.f;
    if (i < ntile) {
        int rem = i, lo = 0;
        for (int pos = 0; pos < p; ++pos) {
            const int left = p - pos - 1;   // positions after this one
            for (int f = lo; f < nb; ++f) {
                const int cnt = binom(nb - f + left - 1, left);   // non-decreasing tails over blocks f .. nb - 1
                if (rem < cnt) {
                    td.t[pos] = (unsigned char)f;
                    lo = f;
                    break;
                }
                rem -= cnt;
            }
        }
        float m = 1.f;
        int run = 1;
        for (int pos = 0; pos < p; ++pos) {
            m *= (float)(pos + 1);
            if (pos > 0 && td.t[pos] == td.t[pos - 1]) ++run; else run = 1;
            m /= (float)run;
        }
        td.mult = m;
    }
    tab[i] = td;
}

// Yp[row][0 .. HD-1] = Y[row], Yp[row][HD] = col[row] (1 when col is null), zeros up to HD + 15
template <int HD>
__global__ __launch_bounds__(256) void k_tiled_pack(const bf16_t* __restrict__ Y, const float* __restrict__ col,
                                                    bf16_t* __restrict__ Yp, long long rows) {
    constexpr int VP = HD + 16, PPR = VP / 8;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= rows * PPR) return;
    const long long row = id / PPR;
    const int c8 = (int)(id % PPR);
    uint4 u = make_uint4(0, 0, 0, 0);
    if (c8 < HD / 8) u = *(const uint4*)(Y + row * HD + 8 * c8);
    else if (c8 == HD / 8) u.x = f32_to_bf16(col != nullptr ? col[row] : 1.f);
    *(uint4*)(Yp + row * VP + 8 * c8) = u;
}

// ---- update-state and cumulative sum ----------------------------------------------------------------------
// One workgroup walks a group of four units (256 state rows; eight at d = 128) of one head over the whole sequence;
// wave w owns unit w of the group as float32 accumulators, transposed (value column x state row, so that a lane ends up
// with VP / 4 consecutive value columns of one state row).  Before the tokens of chunk c are added, the
// running sum - the state entering chunk c - is stored (REV: the walk runs from the last chunk down and the
// stored sum is the state gradient of the chunks after c).  X: the rows phi is formed from (K; REV: Q, times
// oscale, which goes onto the stored state), Yp: the extended value rows ([V, 1]; REV: [ghat, gz]).
template <int HD>
constexpr int scan_units() { return HD >= 128 ? 8 : 4; }   // units (waves) per workgroup: each re-reads the head's token rows

template <int P, int DT, int HD, bool REV>
__global__ __launch_bounds__(64 * scan_units<HD>(), 2) void k_tiled_scan(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Yp,
                                                    const TileDesc* __restrict__ tab, bf16_t* __restrict__ st, int T, int cs,
                                                    int nunit, float oscale) {
    using E = Emb<P, DT>;
    constexpr int UPW = scan_units<HD>(), NT = 64 * UPW, VP = HD + 16, NVB = VP / 16, SP = HD + 4;
    typedef XStore<HD> XS;
    __shared__ __attribute__((aligned(16))) typename XS::elem xs[64][XS::PITCH];
    __shared__ __attribute__((aligned(16))) Tile64<VP> yt;
    __shared__ __attribute__((aligned(16))) Tile64<64> phis[UPW];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), r16 = lane & 15, g = lane >> 4;
    // Every workgroup of a head streams that head's token rows.  Workgroups are dealt to the 8 XCDs round-robin
    // by their linear id; with a multiple of 8 heads the ids are re-read so that a head's workgroups all sit on one
    // XCD and its rows come out of that XCD's L2 (otherwise each L2 fetches every head, and falls behind).
    int ugrp = blockIdx.x, bh = blockIdx.y;
    if (gridDim.y % 8 == 0) {
        const int lin = blockIdx.x + gridDim.x * blockIdx.y, slot = lin / 8;
        bh = (slot / gridDim.x) * 8 + lin % 8;
        ugrp = slot % gridDim.x;
    }
    const int unit = ugrp * UPW + w, nchunk = T / cs;
    const size_t head = (size_t)bh * T;

    float mult[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) mult[nb] = oscale * tab[E::R >= 64 ? unit / E::UPT : unit * E::TPU + (16 * nb) / E::R].mult;
    f32x4 acc[NVB][4];
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[vb][nb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // the token rows of a step wait in registers while the step before them is being worked on
    constexpr int XP = (64 * (HD / 8) + NT - 1) / NT, YP = (64 * (VP / 8) + NT - 1) / NT;
    u32x4 xr[XP], yr[YP];   // (a true vector type: copies of HIP's uint4 struct become memcpy calls that keep the array in scratch)
    const int spc = cs / 64, nstep = (nchunk - 1) * spc;    // the last chunk walked is never added
#define PA_STEP_FETCH(SL)                                                                                        \
    {                                                                                                            \
        const int ci_ = (SL) / spc, c_ = REV ? nchunk - 1 - ci_ : ci_;                                           \
        const size_t tok0_ = head + (size_t)c_ * cs + 64 * ((SL) % spc);                                         \
        _Pragma("unroll") for (int q_ = 0; q_ < XP; ++q_) {                                                      \
            const int id_ = min(tid + NT * q_, 64 * (HD / 8) - 1);                                              \
            xr[q_] = *(const u32x4*)(X + tok0_ * HD + (size_t)id_ * 8);                                          \
        }                                                                                                        \
        _Pragma("unroll") for (int q_ = 0; q_ < YP; ++q_) {                                                      \
            const int id_ = min(tid + NT * q_, 64 * (VP / 8) - 1);                                              \
            yr[q_] = *(const u32x4*)(Yp + tok0_ * VP + (size_t)id_ * 8);                                         \
        }                                                                                                        \
    }
    PA_STEP_FETCH(0)   // (a sequence of one chunk never gets here: the launchers ask for at least two)
    for (int sl = 0; sl <= nstep; ++sl) {
        if (sl % spc == 0) {
            // the running sum is the state entering this chunk (REV: the state gradient of the chunks after it).
            // A lane holds 8-byte runs of 16 different rows; written as they are, every store instruction would
            // touch 64 cache lines in part.  The unit's 64 x SP block is contiguous in memory, so it goes through
            // the wave's phi tile (free between two steps) and leaves as whole 16-byte pieces, 1 KB per instruction.
            const int ci = sl / spc, c = REV ? nchunk - 1 - ci : ci;
            bf16_t* dst = st + (((size_t)bh * nchunk + c) * nunit + unit) * 64 * SP;
            constexpr int PASSES = 64 * SP * 2 > (int)sizeof(Tile64<64>) ? 2 : 1, NBP = 4 / PASSES;   // blocks of 16 rows per pass
            constexpr int PIECES = NBP * 16 * SP / 8;                                                  // of 16 bytes
            static_assert(NBP * 16 * SP * 2 <= (int)sizeof(Tile64<64>) && (NBP * 16 * SP) % 8 == 0, "a pass fits the phi tile");
            bf16_t* stage = (bf16_t*)&phis[w];
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
#pragma unroll
                for (int nl = 0; nl < NBP; ++nl) {
                    const int nb = ps * NBP + nl;
#pragma unroll
                    for (int vb = 0; vb < NVB; ++vb) {
                        bf16x4 o;
#pragma unroll
                        for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[vb][nb][r] * mult[nb]);
                        const int col = g * (VP / 4) + 4 * vb;
                        if (col < SP) *(bf16x4*)(stage + (16 * nl + r16) * SP + col) = o;
                    }
                }
                wave_sync();
#pragma unroll
                for (int k = 0; k < (PIECES + 63) / 64; ++k) {
                    const int idx = lane + 64 * k;
                    // (streaming stores: a state is not read again by this kernel, and left to age in L2 like other
                    // lines it pushes out the token rows that the head's other workgroups are about to ask for)
                    if (idx < PIECES)
                        __builtin_nontemporal_store(*(const u32x4*)(stage + 8 * idx), (u32x4*)(dst + (size_t)ps * (NBP * 16 * SP) + 8 * idx));
                }
                wave_sync();
            }
        }
        if (sl == nstep) break;
        __syncthreads();
        // (threads past the last piece repeat it: same data to the same place)
#pragma unroll
        for (int q = 0; q < XP; ++q) {
            const int id = min(tid + NT * q, 64 * (HD / 8) - 1);
            const u32x4 u = xr[q];
            uint32_t* dst = (uint32_t*)&xs[id / (HD / 8)][8 * (id % (HD / 8))];
            dst[0] = u[0]; dst[1] = u[1]; dst[2] = u[2]; dst[3] = u[3];
        }
#pragma unroll
        for (int q = 0; q < YP; ++q) {
            const int id = min(tid + NT * q, 64 * (VP / 8) - 1);
            *(u32x4*)&yt.r[id / (VP / 8)][8 * (id % (VP / 8))] = yr[q];
        }
        __syncthreads();
        PA_STEP_FETCH(min(sl + 1, nstep - 1))
        {
            float phi[64];
            unit_phi<P, DT>(typename XS::row{&xs[lane][0]}, tab, unit, phi);
            put_phi(phis[w], lane, phi);
        }
        wave_sync();
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 pf[4];
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) pf[nb] = col_frag<64>(phis[w], s, nb, r16, g);
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb) {
                // A row 4 g' + r of block vb is value column g' VP / 4 + 4 vb + r
                const bf16x8 yf = col_frag_at<VP>(yt, s, (r16 & 3) * (VP / 4) + 4 * vb, r16, g);
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) acc[vb][nb] = mfma16(yf, pf[nb], acc[vb][nb]);
            }
        }
        wave_sync();
    }
#undef PA_STEP_FETCH
}

// ---- query-state: part[t][:] = S_chunk(t)^T phi(x_t) -------------------------------------------------------
// A workgroup takes 128 tokens of one chunk (two waves of 64 tokens, O^T accumulators in registers; two waves
// per 64 tokens at d = 128, see below) and streams that chunk's state, unit by unit: NPF units are on their way
// from memory in registers while one is being worked on from LDS (two slots taken in turn, one from d = 128 on).  zpart (may be null) receives the normaliser column's share.
// Also serves dV: the state gradient read out with phi(k).
// Workgroups are dealt to the 8 XCDs round-robin by their linear id, each XCD with an L2 of its own.  The m
// 128-token blocks of one chunk stream the same state, so they are given ids 8 apart: same XCD, about the
// same time.  (Identity when the grid is not a multiple of 8 m blocks.)
__device__ __forceinline__ int token_block(int bx, int nblk, int m) {
    if (m <= 1 || nblk % (8 * m) != 0) return bx;
    const int base = bx - bx % (8 * m), r = bx % (8 * m);
    return (base / m + r % 8) * m + r / 8;
}

template <int HD>
constexpr int units_in_flight() { return 4; }   // per workgroup, in registers

// unit u (64 rows x SP bf16, contiguous) of the state at sbase -> registers; PPT pieces of 8 bytes per thread
// (loads are unconditional, on clamped indices: an array that is assigned under a condition is kept in scratch
// memory by the compiler, and the load then waits to be stored there; threads past the last piece repeat it)
#define PA_UNIT_LOAD(REGS, U)                                                                                    \
    _Pragma("unroll") for (int q_ = 0; q_ < PPT; ++q_) {                                                         \
        const int id_ = min(tid + NT * q_, PIECES - 1);                                                         \
        REGS[q_] = *(const u32x2*)(sbase + ((size_t)min((U), nunit_real - 1) * PIECES + id_) * 4);               \
    }
#define PA_UNIT_STORE(DST, REGS)                                                                                 \
    _Pragma("unroll") for (int q_ = 0; q_ < PPT; ++q_) {                                                         \
        const int id_ = min(tid + NT * q_, PIECES - 1);                                                         \
        *(u32x2*)&DST.r[id_ / (SP / 4)][4 * (id_ % (SP / 4))] = REGS[q_];                                        \
    }
// columns SP .. VP - 1 of an LDS state tile are zero and never written again
#define PA_UNIT_ZERO_PAD(DST)                                                                                    \
    for (int id_ = tid; id_ < 64 * ((VP - SP) / 4); id_ += NT)                                                  \
        *(u32x2*)&DST.r[id_ / ((VP - SP) / 4)][SP + 4 * (id_ % ((VP - SP) / 4))] = (u32x2){0u, 0u};

// At d = 128 two waves share a group of 64 tokens (LDS leaves room for two workgroups per CU, and two waves each
// would leave every SIMD with a single wave, nothing to run under its MFMAs): each forms half of the rows of
// phi and takes half of the value columns' accumulators.
template <int HD>
constexpr int readout_waves_per_group() { return HD >= 128 ? 2 : 1; }

template <int P, int DT, int HD>
__global__ __launch_bounds__(128 * readout_waves_per_group<HD>(), 2) void k_tiled_readout(
    const bf16_t* __restrict__ X, const TileDesc* __restrict__ tab, const bf16_t* __restrict__ st, float* __restrict__ part,
    float* __restrict__ zpart, int T, int cs, int nunit, int nunit_real, float oscale) {
    constexpr int WPG = readout_waves_per_group<HD>(), NT = 128 * WPG;
    constexpr int VP = HD + 16, NVB = VP / 16, NVW = (NVB + WPG - 1) / WPG, SP = HD + 4, PIECES = 64 * (SP / 4), PPT = (PIECES + NT - 1) / NT;
    constexpr int NPF = units_in_flight<HD>();
    typedef XStore<HD> XS;
    __shared__ __attribute__((aligned(16))) typename XS::elem xs[128][XS::PITCH];
    constexpr int SLOTS = HD >= 128 ? 1 : 2;   // LDS decides how many workgroups share a CU: one slot costs a second barrier per unit
    static_assert(WPG == 1 || SLOTS == 1, "waves that share phi meet at the second barrier of a unit");
    __shared__ __attribute__((aligned(16))) Tile64<VP> stt[SLOTS];
    __shared__ __attribute__((aligned(16))) Tile64<64> phis[2];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), r16 = lane & 15, g = lane >> 4;
    const int grp = w / WPG, part_w = w % WPG, vb0 = part_w * NVW;   // token group; first block of value columns of this wave
    const int bh = blockIdx.y, tok0 = token_block(blockIdx.x, gridDim.x, cs / 128) * 128, nchunk = T / cs, chunk = tok0 / cs;
    const size_t head = (size_t)bh * T;
    const bf16_t* sbase = st + ((size_t)bh * nchunk + chunk) * nunit * 64 * SP;

    u32x2 pre[NPF][PPT];
#pragma unroll
    for (int j = 0; j < NPF - 1; ++j) PA_UNIT_LOAD(pre[j], j)
    PA_UNIT_ZERO_PAD(stt[0])
    if (SLOTS > 1) PA_UNIT_ZERO_PAD(stt[SLOTS - 1])
    stage_x<HD, NT>(xs, X + (head + tok0) * HD, 128, tid);
    f32x4 acc[NVW][4];
#pragma unroll
    for (int vb = 0; vb < NVW; ++vb)
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = (f32x4){0.f, 0.f, 0.f, 0.f};

    for (int u0 = 0; u0 < nunit_real; u0 += NPF) {
#pragma unroll
        for (int j = 0; j < NPF; ++j) {
            const int u = u0 + j;
            PA_UNIT_LOAD(pre[(j + NPF - 1) % NPF], u + NPF - 1)
            if (u >= nunit_real) continue;
            Tile64<VP>& cur = stt[j & (SLOTS - 1)];
            if (SLOTS == 1) __syncthreads();
            PA_UNIT_STORE(cur, pre[j])
            if constexpr (WPG == 1) {
                __syncthreads();
                float phi[64];
                unit_phi<P, DT>(typename XS::row{&xs[64 * grp + lane][0]}, tab, u, phi);
                put_phi(phis[grp], lane, phi);
                wave_sync();
            } else {
                // (each branch uses half of phi; what it does not store is never computed)
                if (part_w == 0) {
                    float phi[64];
                    unit_phi<P, DT>(typename XS::row{&xs[64 * grp + lane][0]}, tab, u, phi);
                    put_phi<0, 4>(phis[grp], lane, phi);
                } else {
                    float phi[64];
                    unit_phi<P, DT>(typename XS::row{&xs[64 * grp + lane][0]}, tab, u, phi);
                    put_phi<4, 8>(phis[grp], lane, phi);
                }
                __syncthreads();
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                Frag qf[4];
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    qf[ib].u = *(const uint4*)&phis[grp].r[16 * ib + r16][32 * s + 8 * g];
                }
#pragma unroll
                for (int vb = 0; vb < NVW; ++vb) {
                    if (WPG > 1 && vb0 + vb >= NVB) continue;   // (uniform: the last wave of a group has a block less)
                    const bf16x8 sf = col_frag<VP>(cur, s, vb0 + vb, r16, g);
#pragma unroll
                    for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = mfma16(sf, qf[ib].v, acc[vb][ib]);
                }
            }
            if constexpr (WPG == 1) wave_sync();
        }
    }
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        const size_t row = head + tok0 + 64 * grp + 16 * ib + r16;
#pragma unroll
        for (int vb = 0; vb < NVW; ++vb) {
            const int cb = vb0 + vb;   // block of 16 value columns; block HD / 16 holds the normaliser's column
            if (cb < HD / 16)
                *(float4*)(part + row * HD + 16 * cb + 4 * g) = make_float4(oscale * acc[vb][ib][0], oscale * acc[vb][ib][1],
                                                                            oscale * acc[vb][ib][2], oscale * acc[vb][ib][3]);
            else if (cb == HD / 16 && zpart != nullptr && g == 0)
                zpart[row] = oscale * acc[vb][ib][0];
        }
    }
}

// ---- d phi and the Jacobian: part[t][:] = oscale J_phi(x_t)^T (S_chunk(t) y'_t) ----------------------------
// A workgroup takes 128 tokens of one chunk.  Per block of 16 state rows: A = S y'^T on the matrix cores
// (contraction over the VP value columns; y' = [ghat, gz] for dQ, [v, 1] for dK, held as operand fragments in
// registers), laid down in LDS as [token][row], then the Jacobian by a thread that owns the token.
// The state's operand fragments are rows of the stored state (lane (r16, g): row r16 of the block, 8 columns
// from 8g), so every wave loads them straight from memory, NPF units ahead, and no state passes through LDS:
// the waves of a workgroup read the same bytes (from L2 the second time) and do not wait for each other.
// At d = 128 (p = 2, d_tile 8) two waves share a group of 64 tokens: the float32 accumulators of 128 tokens
// (64 KB) leave room for one workgroup per CU, and two waves would keep only two of its four SIMDs busy.  Wave
// h of a pair takes the unit's rows with left index alpha in [4h, 4h + 4) and lands the sums whose feature
// index within the tile is in that same range, on either side: the two waves then never touch the same
// accumulator.  The right side's sums run over all alpha, so each wave passes the half it does not land to its
// partner through LDS (two buffers taken in turn, one barrier per unit) and adds what it receives one unit late.
template <int HD>
constexpr int dphi_waves_per_group() { return HD >= 128 ? 2 : 1; }

typedef u32x4 __attribute__((aligned(4))) u32x4_dword_aligned;   // rows of SP = d + 4 columns start on 8 bytes

template <int NBW, int NK>
struct StateFrags {
    u32x4 sf[NBW][NK];
    u32x2 tail[NBW];
};
// unit u of the state at sbase, the blocks nb0 .. nb0 + NBW - 1: this lane's operand fragments
template <int NBW, int NK, int HD>
__device__ __forceinline__ void load_frags(StateFrags<NBW, NK>& f, const bf16_t* __restrict__ sbase, int u, int nb0, int r16, int g) {
    constexpr int SP = HD + 4;
#pragma unroll
    for (int k = 0; k < NBW; ++k) {
        const bf16_t* row = sbase + ((size_t)u * 64 + 16 * (nb0 + k) + r16) * SP;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) f.sf[k][ks] = *(const u32x4_dword_aligned*)(row + 32 * ks + 8 * g);
        f.tail[k] = *(const u32x2*)(row + HD);   // columns d .. d + 3; what lies beyond them in a k-step is zero
    }
}

template <int P, int DT, int HD>
__global__ __launch_bounds__(128 * dphi_waves_per_group<HD>()) void k_tiled_dphi(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ Yp, const TileDesc* __restrict__ tab, const bf16_t* __restrict__ st,
    float* __restrict__ part, int T, int cs, int nunit, int nunit_real, float oscale) {
    constexpr int WPG = dphi_waves_per_group<HD>(), NT = 128 * WPG, NBW = 4 / WPG;
    constexpr int VP = HD + 16, NK = HD / 32, SP = HD + 4, AP = 16 + 4;
    constexpr int NPF = 3;   // units on their way from memory, per wave
    typedef XStore<HD> XS;
    __shared__ __attribute__((aligned(16))) typename XS::elem xs[128][XS::PITCH];
    __shared__ __attribute__((aligned(16))) float dph[2 * WPG][64][AP];
    // the accumulators: registers at d = 32 (all features of the thread's token), LDS beyond (64 more registers do
    // not fit beside the operands at d = 64; at d = 128, with the half of the features that a wave lands in
    // registers, LDS would allow two workgroups per CU but the kernel ran at 32 ms instead of 22)
    constexpr bool DXREG = HD == 32;
    typedef typename std::conditional<DXREG, DxRegs32, DxLds>::type DX;
    __shared__ float dxs[DXREG ? 1 : 2][DXREG ? 1 : HD][64];
    __shared__ float handed[WPG > 1 ? 2 : 1][WPG > 1 ? 4 : 1][4][64];   // [unit parity][wave that wrote it][i][token]
    static_assert(WPG == 1 || (P == 2 && DT == 8), "the split of a unit between two waves is laid out for one 8 x 8 tile per unit");
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), r16 = lane & 15, g = lane >> 4;
    const int grp = w / WPG, part_w = w % WPG;   // token group of the wave, and which blocks of a unit it takes
    const int bh = blockIdx.y, tok0 = token_block(blockIdx.x, gridDim.x, cs / 128) * 128, nchunk = T / cs, chunk = tok0 / cs;
    const size_t head = (size_t)bh * T;
    const bf16_t* sbase = st + ((size_t)bh * nchunk + chunk) * nunit * 64 * SP;

    StateFrags<NBW, NK> fr[NPF];
#pragma unroll
    for (int j = 0; j < NPF - 1; ++j) load_frags<NBW, NK, HD>(fr[j], sbase, min(j, nunit_real - 1), part_w * NBW, r16, g);
    stage_x<HD, NT>(xs, X + (head + tok0) * HD, 128, tid);
    DX dx;
    if constexpr (DXREG) {
        dx.clear();
    } else {
        dx.col = &dxs[grp][0][lane];
#pragma unroll
        for (int f = 0; f < HD / WPG; ++f) dxs[grp][part_w * (HD / WPG) + f][lane] = 0.f;
    }
    Frag yf[4][NK];
    uint2 ytail[4];
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        const bf16_t* yrow = Yp + (head + tok0 + 64 * grp + 16 * ib + r16) * VP;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) yf[ib][ks].u = *(const uint4*)(yrow + 32 * ks + 8 * g);
        ytail[ib] = *(const uint2*)(yrow + HD);   // pairs with the state's tail: columns d .. d + 3 in the first four k-slots
    }
    const typename XS::row xrow{&xs[64 * grp + lane][0]};
    float kept[4] = {0.f, 0.f, 0.f, 0.f};   // WPG > 1: the right side's sums of the last unit that this wave lands
    int kept_f = -1;                        // their first feature (-1: none yet)
    __syncthreads();                        // token rows and cleared accumulators in place

    for (int u0 = 0; u0 < nunit_real; u0 += NPF) {
#pragma unroll
        for (int j = 0; j < NPF; ++j) {
            const int u = u0 + j;
            load_frags<NBW, NK, HD>(fr[(j + NPF - 1) % NPF], sbase, min(u + NPF - 1, nunit_real - 1), part_w * NBW, r16, g);
            if (u >= nunit_real) continue;
            const StateFrags<NBW, NK>& cur = fr[j];
            if constexpr (WPG > 1) {
                if (kept_f >= 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) dx_add(dx, kept_f + i, kept[i] + handed[(u - 1) & 1][w ^ 1][i][lane]);
                }
            }
            UnitJacobian<P, DT> jac;
            jac.begin(xrow, tab, u);
#pragma unroll
            for (int k = 0; k < NBW; ++k) {
                const int nb = part_w * NBW + k;
                // only the lanes g = 0 carry the tail's four columns; the other k-slots of that step are zero
                const uint2 stail = g == 0 ? make_uint2(cur.tail[k][0], cur.tail[k][1]) : make_uint2(0u, 0u);
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    f32x4 c = {0.f, 0.f, 0.f, 0.f};   // rows 16 nb + 4g + r, token 16 ib + r16
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) {
                        Frag sfk;
                        sfk.q = cur.sf[k][ks];
                        c = mfma16(sfk.v, yf[ib][ks].v, c);
                    }
                    c = mfma16k16(stail, ytail[ib], c);
                    *(float4*)&dph[w][16 * ib + r16][4 * g] = make_float4(c[0], c[1], c[2], c[3]);
                }
                wave_sync();
                float A[16];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 a4 = *(const float4*)&dph[w][lane][4 * i];
                    A[4 * i] = a4.x; A[4 * i + 1] = a4.y; A[4 * i + 2] = a4.z; A[4 * i + 3] = a4.w;
                }
                wave_sync();
                jac.block(xrow, tab, u, nb, A, dx);
            }
            if constexpr (WPG > 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    kept[i] = part_w ? jac.dR[4 + i] : jac.dR[i];
                    handed[u & 1][w][i][lane] = part_w ? jac.dR[i] : jac.dR[4 + i];
                }
                kept_f = DT * jac.td.t[1] + 4 * part_w;
                __syncthreads();   // the partner's half of this unit is in place; the buffer is written again two units on
            } else {
                jac.finish(xrow, dx);
            }
        }
    }
    if constexpr (WPG > 1) {
        if (kept_f >= 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) dx_add(dx, kept_f + i, kept[i] + handed[(nunit_real - 1) & 1][w ^ 1][i][lane]);
        }
        __syncthreads();
    } else {
        wave_sync();
    }
    if constexpr (DXREG) {
        float* out = part + (head + tok0 + 64 * grp + lane) * HD;
#pragma unroll
        for (int f4 = 0; f4 < HD / 4; ++f4)
            *(float4*)(out + 4 * f4) = make_float4(oscale * dx.v[4 * f4], oscale * dx.v[4 * f4 + 1], oscale * dx.v[4 * f4 + 2], oscale * dx.v[4 * f4 + 3]);
    } else {
        float* out = part + (head + tok0 + 64 * grp + lane) * HD + part_w * (HD / WPG);
        const float* mine = &dxs[grp][part_w * (HD / WPG)][lane];
#pragma unroll
        for (int f4 = 0; f4 < HD / WPG / 4; ++f4)
            *(float4*)(out + 4 * f4) = make_float4(oscale * mine[64 * (4 * f4)], oscale * mine[64 * (4 * f4 + 1)],
                                                   oscale * mine[64 * (4 * f4 + 2)], oscale * mine[64 * (4 * f4 + 3)]);
    }
}
#undef PA_UNIT_LOAD
#undef PA_UNIT_STORE
#undef PA_UNIT_ZERO_PAD

template <int P, int DT, int HD>
bool scan_t(const char* name, hipStream_t s, const TiledPlan& pl, bool rev, const bf16_t* X, const bf16_t* Yp, const TileDesc* tab,
            bf16_t* st, int BH, int T, int cs, float xscale) {
    LaunchScope ls(name, s);
    constexpr int UPW = scan_units<HD>();
    const dim3 grid(pl.nunit / UPW, BH);
    const float oscale = powf(xscale, (float)P);   // phi(s x) = s^p phi(x)
    if (rev) hipLaunchKernelGGL((k_tiled_scan<P, DT, HD, true>), grid, dim3(64 * UPW), 0, s, X, Yp, tab, st, T, cs, pl.nunit, oscale);
    else hipLaunchKernelGGL((k_tiled_scan<P, DT, HD, false>), grid, dim3(64 * UPW), 0, s, X, Yp, tab, st, T, cs, pl.nunit, oscale);
    return launch_ok();
}
template <int P, int DT, int HD>
bool readout_t(const char* name, hipStream_t s, const TiledPlan& pl, const bf16_t* X, const TileDesc* tab, const bf16_t* st,
               float* part, float* zpart, int BH, int T, int cs, float xscale) {
    LaunchScope ls(name, s);
    hipLaunchKernelGGL((k_tiled_readout<P, DT, HD>), dim3(T / 128, BH), dim3(128 * readout_waves_per_group<HD>()), 0, s, X, tab, st, part, zpart, T, cs, pl.nunit,
                       pl.nunit_real, powf(xscale, (float)P));
    return launch_ok();
}
template <int P, int DT, int HD>
bool dphi_t(const char* name, hipStream_t s, const TiledPlan& pl, const bf16_t* X, const bf16_t* Yp, const TileDesc* tab,
            const bf16_t* st, float* part, int BH, int T, int cs, float xscale, float outscale) {
    LaunchScope ls(name, s);
    hipLaunchKernelGGL((k_tiled_dphi<P, DT, HD>), dim3(T / 128, BH), dim3(128 * dphi_waves_per_group<HD>()), 0, s, X, Yp, tab, st, part, T, cs, pl.nunit,
                       pl.nunit_real, outscale * powf(xscale, (float)(P - 1)));   // J_phi(s x) = s^(p-1) J_phi(x)
    return launch_ok();
}

}  // namespace

// every (degree, tile width, head size) the kernels are built for
#define PA_TILED_SHAPES(X) \
    X(2, 4, 32) X(2, 8, 32) X(2, 16, 32) X(3, 4, 32) X(4, 2, 32) X(4, 4, 32) \
    X(2, 4, 64) X(2, 8, 64) X(2, 16, 64) X(3, 4, 64) \
    X(2, 8, 128)

bool tiled_shape_ok(int p, int d, int dt) {
#define PA_X(PP, DD, HH) \
    if (p == PP && dt == DD && d == HH) return true;
    PA_TILED_SHAPES(PA_X)
#undef PA_X
    return false;
}

// 8 for p = 2 and 4 for p = 3 (the widths Sec. 4.1.1 names); p = 4 at d = 32: 2 (62016 state rows against 84480 with 4:
// measured 24 against 28 ms per step on B2 H8 T16384)
int tiled_default_dt(int p) { return p == 2 ? 8 : p == 3 ? 4 : 2; }

TiledPlan tiled_plan(int p, int d, int dt) {
    TiledPlan pl{};
    pl.p = p;
    pl.dt = dt;
    pl.hd = d;
    pl.vp = d + 16;
    const int nb = d / dt;
    long long nt = 1;   // C(nb + p - 1, p)
    for (int i = 1; i <= p; ++i) nt = nt * (nb + p - i) / i;
    pl.ntile = (int)nt;
    int rows = 1;
    for (int i = 0; i < p; ++i) rows *= dt;
    pl.rows_per_tile = rows;
    pl.nunit_real = rows >= 64 ? pl.ntile * (rows / 64) : (pl.ntile + 64 / rows - 1) / (64 / rows);
    const int upw = d >= 128 ? 8 : 4;   // units per workgroup of the scan
    pl.nunit = (pl.nunit_real + upw - 1) / upw * upw;
    pl.nentry = rows >= 64 ? (pl.nunit + rows / 64 - 1) / (rows / 64) : pl.nunit * (64 / rows);
    pl.state_elems = (size_t)pl.nunit * 64 * (d + 4);   // rows are stored without their zero columns
    return pl;
}

bool launch_tiled_table(hipStream_t s, const TiledPlan& pl, TileDesc* tab) {
    LaunchScope ls("tiled_table", s);
    hipLaunchKernelGGL(k_tile_table, dim3((pl.nentry + 255) / 256), dim3(256), 0, s, tab, pl.p, pl.hd / pl.dt, pl.ntile, pl.nentry);
    return launch_ok();
}

bool launch_tiled_pack(hipStream_t s, int hd, const bf16_t* Y, const float* col, bf16_t* Yp, long long rows) {
    LaunchScope ls("tiled_pack", s);
    const long long n = rows * ((hd + 16) / 8);
    if (hd == 32) hipLaunchKernelGGL((k_tiled_pack<32>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, Y, col, Yp, rows);
    else if (hd == 64) hipLaunchKernelGGL((k_tiled_pack<64>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, Y, col, Yp, rows);
    else if (hd == 128) hipLaunchKernelGGL((k_tiled_pack<128>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, Y, col, Yp, rows);
    else return false;
    return launch_ok();
}

bool launch_tiled_scan(const char* name, hipStream_t s, const TiledPlan& pl, bool rev, const bf16_t* X, const bf16_t* Yp,
                       const TileDesc* tab, bf16_t* st, int BH, int T, int cs, float xscale) {
    if (cs % 128 != 0 || T % cs != 0) return false;
#define PA_X(PP, DD, HH) \
    if (pl.p == PP && pl.dt == DD && pl.hd == HH) return scan_t<PP, DD, HH>(name, s, pl, rev, X, Yp, tab, st, BH, T, cs, xscale);
    PA_TILED_SHAPES(PA_X)
#undef PA_X
    return false;
}

bool launch_tiled_readout(const char* name, hipStream_t s, const TiledPlan& pl, const bf16_t* X, const TileDesc* tab, const bf16_t* st,
                          float* part, float* zpart, int BH, int T, int cs, float xscale) {
    if (cs % 128 != 0 || T % cs != 0) return false;
#define PA_X(PP, DD, HH) \
    if (pl.p == PP && pl.dt == DD && pl.hd == HH) return readout_t<PP, DD, HH>(name, s, pl, X, tab, st, part, zpart, BH, T, cs, xscale);
    PA_TILED_SHAPES(PA_X)
#undef PA_X
    return false;
}

bool launch_tiled_dphi(const char* name, hipStream_t s, const TiledPlan& pl, const bf16_t* X, const bf16_t* Yp, const TileDesc* tab,
                       const bf16_t* st, float* part, int BH, int T, int cs, float xscale, float outscale) {
    if (cs % 128 != 0 || T % cs != 0) return false;
#define PA_X(PP, DD, HH)                           \
    if (pl.p == PP && pl.dt == DD && pl.hd == HH) \
        return dphi_t<PP, DD, HH>(name, s, pl, X, Yp, tab, st, part, BH, T, cs, xscale, outscale);
    PA_TILED_SHAPES(PA_X)
#undef PA_X
    return false;
}

}  // namespace mfma
}  // namespace pa
