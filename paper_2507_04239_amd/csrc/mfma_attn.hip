// bf16 MFMA kernels for the attention form of power attention (arXiv 2507.04239, Sec. 2 Eq. 5 with
// the kernel of Sec. 4 Eq. 7): the whole sequence is one chunk, no state is built,
//     O_i = sum_{j <= i} a_ij v_j / Z_i,   a_ij = (scale q_i . k_j)^p,   Z_i = sum_{j <= i} a_ij,
// for degrees p in {2, 3, 4}, head sizes d = v in {32, 64, 128} and any sequence length.  The paper switches to this form where
// it is the cheaper one (Sec. 4.1.2, the throughput comparison); here it is also what runs the degrees and
// head sizes the chunked MFMA family (p = 2, d = 64) does not cover.
//
// Backward pass (the paper gives none; derived from the definition): with ghat_i = dO_i / Z_i and
// gz_i = -ghat_i . O_i (normalised; ghat = dO, gz = 0 otherwise),
//     e_ij = ghat_i . v_j + gz_i                       dL / d a_ij
//     t_ij = e_ij p scale (scale q_i . k_j)^(p-1)      dL / d (q_i . k_j)
//     dQ_i = sum_{j <= i} t_ij k_j,   dK_j = sum_{i >= j} t_ij q_i,   dV_j = sum_{i >= j} a_ij ghat_i.
//
// All three kernels have one shape: a workgroup of 4 waves owns a block of rows (queries for the
// forward pass and dQ, keys for dK / dV), each wave OWN of them with its operands and accumulators
// in registers, and walks over the other side's rows in tiles of 64 that are staged row-major in
// LDS (double-buffered, one barrier per tile).  Operands that are needed transposed (V^T, K^T, Q^T,
// ghat^T as the MFMA's A operand) come from the same row-major tile through the transposing LDS
// read, so no transposed copy exists anywhere.  MFMA operand layouts as in mfma_common.hpp; the
// 8 k-slots of the second contraction are rows 4g..4g+3 of two 16-row blocks, which is how the
// first contraction's accumulators already hold them.
#include <type_traits>

#include "mfma_common.hpp"

namespace pa {
namespace mfma {
namespace {

constexpr int AT = 64;   // rows per streamed tile

template <int HD>
struct AttnTile {
    bf16_t r[AT][HD + 8];   // pitch (HD + 8) / 2 dwords = 4 (mod 8): the 16 rows of a fragment read hit distinct banks
};

template <int P>
__device__ __forceinline__ float ipow(float x) {
    float r = 1.f;
#pragma unroll
    for (int i = 0; i < P; ++i) r *= x;
    return r;
}
template <>
__device__ __forceinline__ float ipow<4>(float x) {
    const float x2 = x * x;
    return x2 * x2;
}

// Staging of a 64-row tile of a row-major [.][HD] array: HD / 32 pieces of 16 bytes per thread,
// piece id = tid + 256 q is row id / (HD / 8), features 8 (id % (HD / 8)) .. + 7.  The pieces wait
// in registers while the tile before them is being used (plain arrays and unrolled loops in the
// kernels: wrapped in a struct they end up in scratch memory).
// T need not be a multiple of the tile: rows past the end are read as row T - 1 (keys and queries
// there are masked out by causality, or never stored) or, with ZERO, as zeros (ghat, whose rows
// past the end must not contribute to dK, dV).
template <int HD, bool ZERO>
__device__ __forceinline__ uint4 piece_load(const bf16_t* __restrict__ head_base, int row0, int id, int T) {
    const int row = row0 + id / (HD / 8);
    const uint4 u = *(const uint4*)(head_base + (size_t)min(row, T - 1) * HD + 8 * (id % (HD / 8)));
    return ZERO && row >= T ? make_uint4(0, 0, 0, 0) : u;
}
template <int HD>
__device__ __forceinline__ void piece_store(AttnTile<HD>& dst, int id, uint4 u) {
    *(uint4*)&dst.r[id / (HD / 8)][8 * (id % (HD / 8))] = u;
}
#define PA_TILE_LOAD(REGS, BASE, ROW0, ZERO)        \
    _Pragma("unroll") for (int q_ = 0; q_ < HD / 32; ++q_) REGS[q_] = piece_load<HD, ZERO>(BASE, ROW0, tid + 256 * q_, T);
#define PA_TILE_STORE(DST, REGS)                    \
    _Pragma("unroll") for (int q_ = 0; q_ < HD / 32; ++q_) piece_store<HD>(DST, tid + 256 * q_, REGS[q_]);

// rows 16 blk + r16, features 32 ks + 8 g .. + 7: A operand (rows x features) or B operand
// (features x rows) of a contraction over the features
template <int HD>
__device__ __forceinline__ bf16x8 row_frag(const AttnTile<HD>& t, int blk, int ks, int r16, int g) {
    Frag f;
    f.u = *(const uint4*)&t.r[16 * blk + r16][32 * ks + 8 * g];
    return f.v;
}
template <int HD>
__device__ __forceinline__ bf16x8 row_frag_global(const bf16_t* __restrict__ X, size_t row, int ks, int g) {
    Frag f;
    f.u = *(const uint4*)(X + row * HD + 32 * ks + 8 * g);
    return f.v;
}

// A operand of a contraction over the tile's rows: column 16 cb + r16, k-slots = rows
// 32 s + 4g .. + 3 and 32 s + 16 + 4g .. + 3.  The transposing read hands lane n of a 16-lane
// group column n of the 4 x 16 block whose row j the lanes 4j .. 4j+3 point at (4 columns each).
template <int HD>
__device__ __forceinline__ bf16x8 col_frag(const AttnTile<HD>& t, int s, int cb, int r16, int g) {
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    const bf16_t* p = &t.r[32 * s + 4 * g + (r16 >> 2)][16 * cb + 4 * (r16 & 3)];
    union {
        bf16x8 v;
        bf16x4 h[2];
    } f;
    f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p);
    f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 16 * (HD + 8)));
    return f.v;
}

// Gating (Sec. 2 "Gating"): the pair (i, j) carries exp(b_i - b_j), b the running sum of the log-gates.
// For a tile whose every pair is below the diagonal the factor is split at a reference m inside the
// gap between the two sides, exp(b_i - m) exp(m - b_j), both <= 1: one of them is staged with the tile
// (GateTile::f, per streamed row), the other is formed once per tile for the rows a lane owns.  Tiles
// on the diagonal use the difference itself (GateTile::b), where a split could overflow.
struct GateTile {
    float b[AT], f[AT];
};
// streamed rows row0 .. row0 + 63 of one head; m_row: the row whose b is the reference;
// sign = +1: f = exp(m - b) (streamed keys), -1: f = exp(b - m) (streamed queries)
__device__ __forceinline__ void gate_tile_load(float& b, float& f, const float* __restrict__ bl_head, int row0, int m_row,
                                               float sign, int tid, int T) {
    if (tid < AT) {
        b = bl_head[min(row0 + tid, T - 1)];
        f = __expf(sign * (bl_head[min(m_row, T - 1)] - b));
    }
}
__device__ __forceinline__ void gate_tile_store(GateTile& t, float b, float f, int tid) {
    if (tid < AT) {
        t.b[tid] = b;
        t.f[tid] = f;
    }
}

// Workgroups are numbered so that the ones with the longest walk start first.
__device__ __forceinline__ int heavy_first(int nblocks, bool longest_is_last) {
    return longest_is_last ? nblocks - 1 - (int)blockIdx.x : (int)blockIdx.x;
}

// ---- forward ----------------------------------------------------------------------------------------
// acc[vb][ib] = O^T: value columns 16 vb + 4g + r, query 16 ib + r16 of the wave's OWN queries.
// WPE: waves per SIMD the register budget is set for.  With 2 (at most 256 registers) the MFMAs
// write plain vector registers; with 1 the compiler moves every score through the accumulation
// registers and back, which costs more vector-ALU instructions than the arithmetic itself.
// CHUNKED (the in-chunk part of the chunked form, App. E.1, for any degree and head size): a query sees the
// keys of its own chunk of `cs` tokens only (cs a multiple of the 64-key tile), and the part that comes
// through the state has been left by other kernels: part[slab][bh][t][v] (float32, `nslab` slabs, summed
// here) joins the numerator and zpart[bh][t] the denominator before the division.
struct ChunkedIn {
    int cs = 0, nslab = 0, nslab2 = 0;
    const float* part = nullptr;     // forward: numerator; dQ kernel: dQ; dK / dV kernel: dK
    const float* part2 = nullptr;    // dK / dV kernel: dV (nslab2 slabs)
    const float* zpart = nullptr;    // forward: denominator
};
template <int P, int HD, int OWN, int WPE, bool GATED, bool CHUNKED = false>
__global__ __launch_bounds__(256, WPE) void k_attn_fwd(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                       const bf16_t* __restrict__ V, bf16_t* __restrict__ O,
                                                       float* __restrict__ Z, int T, float scale, int normalize,
                                                       const float* __restrict__ bl, ChunkedIn ck) {
    constexpr int NI = OWN / 16, NK = HD / 32, NV = HD / 16, WG = 4 * OWN;
    extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
    AttnTile<HD>* kt = reinterpret_cast<AttnTile<HD>*>(attn_smem);      // [2]
    AttnTile<HD>* vt = kt + 2;                                          // [2]
    GateTile* gtile = reinterpret_cast<GateTile*>(vt + 2);              // [2]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r16 = lane & 15, g = lane >> 4;
    const int nblk = (T + WG - 1) / WG;
    const int i0 = heavy_first(nblk, true) * WG;
    const int q0 = i0 + OWN * w;                    // the wave's first query
    const bool active = q0 < T;
    const size_t head = (size_t)blockIdx.y * T;
    const bf16_t* Kh = K + head * HD;
    const bf16_t* Vh = V + head * HD;

    bf16x8 qf[NI][NK];
    f32x4 acc[NV][NI];
    // Z rides on the matrix cores too: a row of ones as the A operand sums the rounded weights of
    // a step's 32 keys for every query (all four accumulator rows of a lane hold the same sum)
    f32x4 zacc[NI];
    Frag ones;
    ones.u = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
        zacc[ib] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NK; ++ks)
            qf[ib][ks] = row_frag_global<HD>(Q, head + min(q0 + 16 * ib + r16, T - 1), ks, g);
#pragma unroll
        for (int vb = 0; vb < NV; ++vb) acc[vb][ib] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    const float* bl_head = GATED ? bl + head : nullptr;
    float bq[NI];
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) bq[ib] = GATED ? bl_head[min(q0 + 16 * ib + r16, T - 1)] : 0.f;

    // one 64-key tile; DIAG: some pair of the tile lies above the diagonal and has to be masked
    auto tile = [&](auto diag_c, int buf, int key0) {
        constexpr bool DIAG = decltype(diag_c)::value;
        float fq[NI];
        if (GATED && !DIAG) {
            const float m = gtile[buf].b[AT - 1];          // the tile's last key
#pragma unroll
            for (int ib = 0; ib < NI; ++ib) fq[ib] = __expf(bq[ib] - m);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            Frag pf[NI];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                const int kb = 2 * s + jb;
                bf16x8 kf[NK];
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) kf[ks] = row_frag<HD>(kt[buf], kb, ks, r16, g);
                float4 gk = make_float4(0.f, 0.f, 0.f, 0.f);
                if (GATED) gk = *(const float4*)(DIAG ? &gtile[buf].b[16 * kb + 4 * g] : &gtile[buf].f[16 * kb + 4 * g]);
                const float gkr[4] = {gk.x, gk.y, gk.z, gk.w};
#pragma unroll
                for (int ib = 0; ib < NI; ++ib) {
                    f32x4 c = {0.f, 0.f, 0.f, 0.f};    // S^T: key 16 kb + 4g + r, query 16 ib + r16
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) c = mfma16(kf[ks], qf[ib][ks], c);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float a = ipow<P>(scale * c[r]);
                        if (GATED) a *= DIAG ? __expf(bq[ib] - gkr[r]) : fq[ib] * gkr[r];
                        if (DIAG && key0 + 16 * kb + 4 * g + r > q0 + 16 * ib + r16) a = 0.f;
                        pf[ib].v[4 * jb + r] = (__bf16)a;
                    }
                }
            }
            // the denominator sums the rounded weights, the ones the numerator uses: the output is
            // then an exact convex combination of the values
#pragma unroll
            for (int ib = 0; ib < NI; ++ib) zacc[ib] = mfma16(ones.v, pf[ib].v, zacc[ib]);
#pragma unroll
            for (int vb = 0; vb < NV; ++vb) {
                const bf16x8 vf = col_frag<HD>(vt[buf], s, vb, r16, g);
#pragma unroll
                for (int ib = 0; ib < NI; ++ib) acc[vb][ib] = mfma16(vf, pf[ib].v, acc[vb][ib]);
            }
        }
    };

    const int ntile = (min(i0 + WG, T) + AT - 1) / AT;   // key tiles 0 .. ntile - 1 reach the block's last query
    // chunked: the walk starts at the chunk of the block's first query, and a wave skips the tiles before its own chunk
    const int t_lo = CHUNKED ? (i0 / ck.cs) * ck.cs / AT : 0;
    const int k_lo = CHUNKED ? (q0 / ck.cs) * ck.cs : 0;
    uint4 kr[HD / 32], vr[HD / 32];
    float gb = 0.f, gf = 0.f;
    PA_TILE_LOAD(kr, Kh, t_lo * AT, false)
    PA_TILE_LOAD(vr, Vh, t_lo * AT, false)
    if (GATED) gate_tile_load(gb, gf, bl_head, 0, AT - 1, 1.f, tid, T);
    PA_TILE_STORE(kt[0], kr)
    PA_TILE_STORE(vt[0], vr)
    if (GATED) gate_tile_store(gtile[0], gb, gf, tid);
    __syncthreads();
    for (int t = t_lo; t < ntile; ++t) {
        const int buf = (t - t_lo) & 1, key0 = t * AT;
        if (t + 1 < ntile) {
            PA_TILE_LOAD(kr, Kh, key0 + AT, false)
            PA_TILE_LOAD(vr, Vh, key0 + AT, false)
            if (GATED) gate_tile_load(gb, gf, bl_head, key0 + AT, key0 + 2 * AT - 1, 1.f, tid, T);
        }
        if (active && key0 <= q0 + OWN - 1 && key0 >= k_lo) {
            if (key0 + AT - 1 > q0) tile(std::true_type{}, buf, key0);
            else tile(std::false_type{}, buf, key0);
        }
        if (t + 1 < ntile) {
            PA_TILE_STORE(kt[buf ^ 1], kr)
            PA_TILE_STORE(vt[buf ^ 1], vr)
            if (GATED) gate_tile_store(gtile[buf ^ 1], gb, gf, tid);
        }
        __syncthreads();
    }

    if (!active) return;
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
        if (q0 + 16 * ib + r16 >= T) continue;      // past the end of a sequence that is not a multiple of the block
        const size_t row = head + q0 + 16 * ib + r16;
        float z = zacc[ib][0];
        if (CHUNKED) {
            z += ck.zpart[row];
            const size_t slab_stride = (size_t)gridDim.y * T * HD;
            for (int sl = 0; sl < ck.nslab; ++sl)
#pragma unroll
                for (int vb = 0; vb < NV; ++vb) {
                    const float4 pv = *(const float4*)(ck.part + sl * slab_stride + row * HD + 16 * vb + 4 * g);
                    acc[vb][ib][0] += pv.x; acc[vb][ib][1] += pv.y; acc[vb][ib][2] += pv.z; acc[vb][ib][3] += pv.w;
                }
        }
        const float inv = normalize ? (z != 0.f ? 1.f / z : 0.f) : 1.f;
#pragma unroll
        for (int vb = 0; vb < NV; ++vb) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[vb][ib][r] * inv);
            *(bf16x4*)(O + row * HD + 16 * vb + 4 * g) = o;
        }
        if (Z != nullptr && g == 0) Z[row] = z;
    }
}

// ---- backward: preparation -------------------------------------------------------------------------
// ghat = dO / Z (bf16) and gz = -(ghat . O) (float32); un-normalised: ghat = dO, gz = 0.  Rows with
// Z == 0 give zeros.  HD / 4 lanes per row.  gz is formed from the rounded ghat, so that
// ghat . v_j + gz = ghat . (v_j - O_i) keeps its exact cancellations.
template <int HD>
__global__ __launch_bounds__(256) void k_attn_prep(const bf16_t* __restrict__ dO, const bf16_t* __restrict__ O,
                                                   const float* __restrict__ Z, bf16_t* __restrict__ Gh,
                                                   float* __restrict__ gz, long long rows, int normalize) {
    constexpr int LPR = HD / 4;
    const long long row = (long long)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
    const int c4 = threadIdx.x % LPR;
    if (row >= rows) return;
    const uint2 graw = *(const uint2*)(dO + row * HD + 4 * c4);
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
    *(bf16x4*)(Gh + row * HD + 4 * c4) = o;
    float delta = 0.f;
    if (normalize) {
        const uint2 oraw = *(const uint2*)(O + row * HD + 4 * c4);
        delta = gr[0] * bf_lo(oraw.x) + gr[1] * bf_hi(oraw.x) + gr[2] * bf_lo(oraw.y) + gr[3] * bf_hi(oraw.y);
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) delta += __shfl_xor(delta, off);
    }
    if (c4 == 0) gz[row] = -delta;
}

// ---- backward: dQ -----------------------------------------------------------------------------------
// acc[fb][ib] = dQ^T: feature 16 fb + 4g + r, query 16 ib + r16.
template <int P, int HD, int OWN, int WPE, bool GATED, bool CHUNKED = false>
__global__ __launch_bounds__(256, WPE) void k_attn_dq(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                 const bf16_t* __restrict__ V, const bf16_t* __restrict__ Gh,
                                                 const float* __restrict__ gz, bf16_t* __restrict__ dQ, int T,
                                                 float scale, const float* __restrict__ bl, float* __restrict__ qdq,
                                                 ChunkedIn ck) {
    constexpr int NI = OWN / 16, NK = HD / 32, NF = HD / 16, WG = 4 * OWN;
    extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
    AttnTile<HD>* kt = reinterpret_cast<AttnTile<HD>*>(attn_smem);      // [2]
    AttnTile<HD>* vt = kt + 2;                                          // [2]
    GateTile* gtile = reinterpret_cast<GateTile*>(vt + 2);              // [2]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r16 = lane & 15, g = lane >> 4;
    const int nblk = (T + WG - 1) / WG;
    const int i0 = heavy_first(nblk, true) * WG;
    const int q0 = i0 + OWN * w;
    const bool active = q0 < T;
    const size_t head = (size_t)blockIdx.y * T;
    const bf16_t* Kh = K + head * HD;
    const bf16_t* Vh = V + head * HD;
    const float pscale = (float)P * scale;

    bf16x8 qf[NI][NK], gf[NI][NK];
    f32x4 acc[NF][NI];
    float gzq[NI];
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
        const size_t row = head + min(q0 + 16 * ib + r16, T - 1);
        gzq[ib] = gz[row];
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            qf[ib][ks] = row_frag_global<HD>(Q, row, ks, g);
            gf[ib][ks] = row_frag_global<HD>(Gh, row, ks, g);
        }
#pragma unroll
        for (int fb = 0; fb < NF; ++fb) acc[fb][ib] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    const float* bl_head = GATED ? bl + head : nullptr;
    // gated: rsum = sum_j t_ij (q_i . k_j) = q_i . dq_i, the row's share of the gate gradient, summed
    // here from the unrounded t (the dot product of the stored dq with q carries bf16 noise that a
    // sum over a block of tokens amplifies)
    float bq[NI], rsum[NI];
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
        bq[ib] = GATED ? bl_head[min(q0 + 16 * ib + r16, T - 1)] : 0.f;
        rsum[ib] = 0.f;
    }

    auto tile = [&](auto diag_c, int buf, int key0) {
        constexpr bool DIAG = decltype(diag_c)::value;
        float fq[NI];
        if (GATED && !DIAG) {
            const float m = gtile[buf].b[AT - 1];          // the tile's last key
#pragma unroll
            for (int ib = 0; ib < NI; ++ib) fq[ib] = __expf(bq[ib] - m);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            Frag tf[NI];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                const int kb = 2 * s + jb;
                bf16x8 kf[NK], vf[NK];
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) {
                    kf[ks] = row_frag<HD>(kt[buf], kb, ks, r16, g);
                    vf[ks] = row_frag<HD>(vt[buf], kb, ks, r16, g);
                }
                float4 gk = make_float4(0.f, 0.f, 0.f, 0.f);
                if (GATED) gk = *(const float4*)(DIAG ? &gtile[buf].b[16 * kb + 4 * g] : &gtile[buf].f[16 * kb + 4 * g]);
                const float gkr[4] = {gk.x, gk.y, gk.z, gk.w};
#pragma unroll
                for (int ib = 0; ib < NI; ++ib) {
                    f32x4 c = {0.f, 0.f, 0.f, 0.f}, e = {gzq[ib], gzq[ib], gzq[ib], gzq[ib]};
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) {
                        c = mfma16(kf[ks], qf[ib][ks], c);    // S^T
                        e = mfma16(vf[ks], gf[ib][ks], e);    // E^T = V ghat^T + gz
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float tv = e[r] * pscale * ipow<P - 1>(scale * c[r]);
                        if (GATED) tv *= DIAG ? __expf(bq[ib] - gkr[r]) : fq[ib] * gkr[r];
                        if (DIAG && key0 + 16 * kb + 4 * g + r > q0 + 16 * ib + r16) tv = 0.f;
                        if (GATED) rsum[ib] += tv * c[r];
                        tf[ib].v[4 * jb + r] = (__bf16)tv;
                    }
                }
            }
#pragma unroll
            for (int fb = 0; fb < NF; ++fb) {
                const bf16x8 kc = col_frag<HD>(kt[buf], s, fb, r16, g);   // K^T
#pragma unroll
                for (int ib = 0; ib < NI; ++ib) acc[fb][ib] = mfma16(kc, tf[ib].v, acc[fb][ib]);
            }
        }
    };

    const int ntile = (min(i0 + WG, T) + AT - 1) / AT;
    const int t_lo = CHUNKED ? (i0 / ck.cs) * ck.cs / AT : 0;     // chunked: keys of the query's own chunk only
    const int k_lo = CHUNKED ? (q0 / ck.cs) * ck.cs : 0;
    uint4 kr[HD / 32], vr[HD / 32];
    float gb = 0.f, gf2 = 0.f;
    PA_TILE_LOAD(kr, Kh, t_lo * AT, false)
    PA_TILE_LOAD(vr, Vh, t_lo * AT, false)
    if (GATED) gate_tile_load(gb, gf2, bl_head, 0, AT - 1, 1.f, tid, T);
    PA_TILE_STORE(kt[0], kr)
    PA_TILE_STORE(vt[0], vr)
    if (GATED) gate_tile_store(gtile[0], gb, gf2, tid);
    __syncthreads();
    for (int t = t_lo; t < ntile; ++t) {
        const int buf = (t - t_lo) & 1, key0 = t * AT;
        if (t + 1 < ntile) {
            PA_TILE_LOAD(kr, Kh, key0 + AT, false)
            PA_TILE_LOAD(vr, Vh, key0 + AT, false)
            if (GATED) gate_tile_load(gb, gf2, bl_head, key0 + AT, key0 + 2 * AT - 1, 1.f, tid, T);
        }
        if (active && key0 <= q0 + OWN - 1 && key0 >= k_lo) {
            if (key0 + AT - 1 > q0) tile(std::true_type{}, buf, key0);
            else tile(std::false_type{}, buf, key0);
        }
        if (t + 1 < ntile) {
            PA_TILE_STORE(kt[buf ^ 1], kr)
            PA_TILE_STORE(vt[buf ^ 1], vr)
            if (GATED) gate_tile_store(gtile[buf ^ 1], gb, gf2, tid);
        }
        __syncthreads();
    }

    if (!active) return;
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
        const bool in = q0 + 16 * ib + r16 < T;
        const size_t row = head + min(q0 + 16 * ib + r16, T - 1);
        if (CHUNKED) {   // what came through the state (and the normaliser), per slab
            const size_t slab_stride = (size_t)gridDim.y * T * HD;
            for (int sl = 0; sl < ck.nslab; ++sl)
#pragma unroll
                for (int fb = 0; fb < NF; ++fb) {
                    const float4 pv = *(const float4*)(ck.part + sl * slab_stride + row * HD + 16 * fb + 4 * g);
                    acc[fb][ib][0] += pv.x; acc[fb][ib][1] += pv.y; acc[fb][ib][2] += pv.z; acc[fb][ib][3] += pv.w;
                }
        }
#pragma unroll
        for (int fb = 0; fb < NF; ++fb) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (__bf16)acc[fb][ib][r];
            if (in) *(bf16x4*)(dQ + row * HD + 16 * fb + 4 * g) = o;
        }
        if (GATED) {
            float dot = rsum[ib];
            dot += __shfl_xor(dot, 16);
            dot += __shfl_xor(dot, 32);
            if (in && g == 0) qdq[row] = dot;
        }
    }
}

// ---- backward: dK, dV ---------------------------------------------------------------------------------
// dk[fb][kb] = dK^T: feature 16 fb + 4g + r, key 16 kb + r16 of the wave's OWN keys; dv likewise.
// S and E are formed queries x keys here, so that their accumulators are the B operand (k-slots =
// queries) of the two contractions over the queries.
template <int P, int HD, int OWN, int WPE, bool GATED, bool CHUNKED = false>
__global__ __launch_bounds__(256, WPE) void k_attn_dkdv(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                   const bf16_t* __restrict__ V, const bf16_t* __restrict__ Gh,
                                                   const float* __restrict__ gz, bf16_t* __restrict__ dK,
                                                   bf16_t* __restrict__ dV, int T, float scale,
                                                   const float* __restrict__ bl, float* __restrict__ kdk,
                                                   float* __restrict__ wsum, ChunkedIn ck) {
    constexpr int NJ = OWN / 16, NK = HD / 32, NF = HD / 16, WG = 4 * OWN;
    extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
    AttnTile<HD>* qt = reinterpret_cast<AttnTile<HD>*>(attn_smem);      // [2]
    AttnTile<HD>* gt = qt + 2;                                          // [2]
    float(*gzt)[AT] = reinterpret_cast<float(*)[AT]>(gt + 2);           // [2][AT]
    GateTile* gtile = reinterpret_cast<GateTile*>(gzt + 2);             // [2]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r16 = lane & 15, g = lane >> 4;
    const int j0 = heavy_first((T + WG - 1) / WG, false) * WG;
    const int k0 = j0 + OWN * w;                    // the wave's first key
    const bool active = k0 < T;
    const size_t head = (size_t)blockIdx.y * T;
    const bf16_t* Qh = Q + head * HD;
    const bf16_t* Gh_h = Gh + head * HD;
    const float* gzh = gz + head;
    const float pscale = (float)P * scale;

    bf16x8 kf[NJ][NK], vf[NJ][NK];
    f32x4 dk[NF][NJ], dv[NF][NJ];
#pragma unroll
    for (int kb = 0; kb < NJ; ++kb) {
        const size_t row = head + min(k0 + 16 * kb + r16, T - 1);
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            kf[kb][ks] = row_frag_global<HD>(K, row, ks, g);
            vf[kb][ks] = row_frag_global<HD>(V, row, ks, g);
        }
#pragma unroll
        for (int fb = 0; fb < NF; ++fb) {
            dk[fb][kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
            dv[fb][kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    }

    const float* bl_head = GATED ? bl + head : nullptr;
    // gated: csum = sum_i e_ij a_ij = k_j . dk_j / p, the key's share of the gate gradient, from the
    // unrounded weights
    float bk[NJ], csum[NJ];
#pragma unroll
    for (int kb = 0; kb < NJ; ++kb) {
        bk[kb] = GATED ? bl_head[min(k0 + 16 * kb + r16, T - 1)] : 0.f;
        csum[kb] = 0.f;
    }

    float wprev = 0.f;   // the wave's total of csum at the end of the last complete block of queries
    auto tile = [&](auto diag_c, int buf, int q0) {
        constexpr bool DIAG = decltype(diag_c)::value;
        float fk[NJ];
        if (GATED && !DIAG) {
            const float m = gtile[buf].b[0];               // the tile's first query
#pragma unroll
            for (int kb = 0; kb < NJ; ++kb) fk[kb] = __expf(m - bk[kb]);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            Frag tf[NJ], pf[NJ];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                const int qb = 2 * s + jb;
                bf16x8 qa[NK], ga[NK];
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) {
                    qa[ks] = row_frag<HD>(qt[buf], qb, ks, r16, g);
                    ga[ks] = row_frag<HD>(gt[buf], qb, ks, r16, g);
                }
                const float4 gz4 = *(const float4*)&gzt[buf][16 * qb + 4 * g];
                const f32x4 e0 = {gz4.x, gz4.y, gz4.z, gz4.w};
                float4 gq = make_float4(0.f, 0.f, 0.f, 0.f);
                if (GATED) gq = *(const float4*)(DIAG ? &gtile[buf].b[16 * qb + 4 * g] : &gtile[buf].f[16 * qb + 4 * g]);
                const float gqr[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
                for (int kb = 0; kb < NJ; ++kb) {
                    f32x4 c = {0.f, 0.f, 0.f, 0.f}, e = e0;   // query 16 qb + 4g + r, key 16 kb + r16
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) {
                        c = mfma16(qa[ks], kf[kb][ks], c);    // S
                        e = mfma16(ga[ks], vf[kb][ks], e);    // E = ghat V^T + gz
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float sc = scale * c[r];
                        const float pw = ipow<P - 1>(sc);
                        float a = pw * sc, tv = e[r] * pscale * pw;
                        if (GATED) {
                            const float gg = DIAG ? __expf(gqr[r] - bk[kb]) : gqr[r] * fk[kb];
                            a *= gg;
                            tv *= gg;
                        }
                        if (DIAG && q0 + 16 * qb + 4 * g + r < k0 + 16 * kb + r16) {
                            a = 0.f;
                            tv = 0.f;
                        }
                        if (GATED) csum[kb] += e[r] * a;
                        pf[kb].v[4 * jb + r] = (__bf16)a;
                        tf[kb].v[4 * jb + r] = (__bf16)tv;
                    }
                }
            }
#pragma unroll
            for (int fb = 0; fb < NF; ++fb) {
                const bf16x8 qc = col_frag<HD>(qt[buf], s, fb, r16, g);   // Q^T
                const bf16x8 gc = col_frag<HD>(gt[buf], s, fb, r16, g);   // ghat^T
#pragma unroll
                for (int kb = 0; kb < NJ; ++kb) {
                    dk[fb][kb] = mfma16(qc, tf[kb].v, dk[fb][kb]);
                    dv[fb][kb] = mfma16(gc, pf[kb].v, dv[fb][kb]);
                }
            }
        }
    };

    // query tiles t_first .. ntile - 1 reach the block's first key; chunked: up to the end of the chunk of the block's
    // last key, and a wave stops at the end of its own keys' chunk
    const int t_first = j0 / AT;
    const int ntile = CHUNKED ? min(((j0 + WG - 1) / ck.cs + 1) * ck.cs, T) / AT : (T + AT - 1) / AT;
    const int q_hi = CHUNKED ? (k0 / ck.cs + 1) * ck.cs : T + AT;
    uint4 qr[HD / 32], gr[HD / 32];
    float gzr = 0.f, gb = 0.f, gf2 = 0.f;
    PA_TILE_LOAD(qr, Qh, t_first * AT, false)
    PA_TILE_LOAD(gr, Gh_h, t_first * AT, true)
    if (tid < AT) gzr = t_first * AT + tid < T ? gzh[t_first * AT + tid] : 0.f;
    if (GATED) gate_tile_load(gb, gf2, bl_head, t_first * AT, t_first * AT, -1.f, tid, T);
    PA_TILE_STORE(qt[0], qr)
    PA_TILE_STORE(gt[0], gr)
    if (tid < AT) gzt[0][tid] = gzr;
    if (GATED) gate_tile_store(gtile[0], gb, gf2, tid);
    __syncthreads();
    for (int t = t_first; t < ntile; ++t) {
        const int buf = (t - t_first) & 1, q0 = t * AT;
        if (t + 1 < ntile) {
            PA_TILE_LOAD(qr, Qh, q0 + AT, false)
            PA_TILE_LOAD(gr, Gh_h, q0 + AT, true)
            if (tid < AT) gzr = q0 + AT + tid < T ? gzh[q0 + AT + tid] : 0.f;
            if (GATED) gate_tile_load(gb, gf2, bl_head, q0 + AT, q0 + AT, -1.f, tid, T);
        }
        if (active && q0 + AT - 1 >= k0 && q0 < q_hi) {
            if (q0 < k0 + OWN - 1) tile(std::true_type{}, buf, q0);   // some pair of this tile lies above the diagonal
            else tile(std::false_type{}, buf, q0);
        }
        if (GATED && active && (q0 + AT) % WG == 0) {
            // a block of queries is complete: the wave's sum goes to wsum[head][key block][query block][wave]
            // (the key block's own query block is not a boundary sum: its pairs are summed per token)
            // = what the block added to the wave's running column sums
            const int jblk = j0 / WG, iblk = q0 / WG, nblk = T / WG;
            float v = 0.f;
#pragma unroll
            for (int kb = 0; kb < NJ; ++kb) v += csum[kb];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
            if (iblk > jblk && lane == 0) wsum[(((size_t)blockIdx.y * nblk + jblk) * nblk + iblk) * 4 + w] = v - wprev;
            wprev = v;
        }
        if (t + 1 < ntile) {
            PA_TILE_STORE(qt[buf ^ 1], qr)
            PA_TILE_STORE(gt[buf ^ 1], gr)
            if (tid < AT) gzt[buf ^ 1][tid] = gzr;
            if (GATED) gate_tile_store(gtile[buf ^ 1], gb, gf2, tid);
        }
        __syncthreads();
    }

    if (!active) return;
#pragma unroll
    for (int kb = 0; kb < NJ; ++kb) {
        const bool in = k0 + 16 * kb + r16 < T;
        const size_t row = head + min(k0 + 16 * kb + r16, T - 1);
        if (CHUNKED) {
            const size_t slab_stride = (size_t)gridDim.y * T * HD;
            for (int sl = 0; sl < ck.nslab; ++sl)
#pragma unroll
                for (int fb = 0; fb < NF; ++fb) {
                    const float4 pv = *(const float4*)(ck.part + sl * slab_stride + row * HD + 16 * fb + 4 * g);
                    dk[fb][kb][0] += pv.x; dk[fb][kb][1] += pv.y; dk[fb][kb][2] += pv.z; dk[fb][kb][3] += pv.w;
                }
            for (int sl = 0; sl < ck.nslab2; ++sl)
#pragma unroll
                for (int fb = 0; fb < NF; ++fb) {
                    const float4 pv = *(const float4*)(ck.part2 + sl * slab_stride + row * HD + 16 * fb + 4 * g);
                    dv[fb][kb][0] += pv.x; dv[fb][kb][1] += pv.y; dv[fb][kb][2] += pv.z; dv[fb][kb][3] += pv.w;
                }
        }
#pragma unroll
        for (int fb = 0; fb < NF; ++fb) {
            bf16x4 a, b;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                a[r] = (__bf16)dk[fb][kb][r];
                b[r] = (__bf16)dv[fb][kb][r];
            }
            if (in) {
                *(bf16x4*)(dK + row * HD + 16 * fb + 4 * g) = a;
                *(bf16x4*)(dV + row * HD + 16 * fb + 4 * g) = b;
            }
        }
        if (GATED) {
            float dot = csum[kb];
            dot += __shfl_xor(dot, 16);
            dot += __shfl_xor(dot, 32);
            if (in && g == 0) kdk[row] = (float)P * dot;
        }
    }
}

template <int HD>
constexpr size_t attn_smem_bytes() {
    return 4 * sizeof(AttnTile<HD>) + 2 * AT * sizeof(float) + 2 * sizeof(GateTile);
}
// LDS beyond the default per-kernel limit has to be requested once per kernel
template <typename F>
bool allow_smem(F* fn, size_t bytes) {
    if (bytes <= 64 * 1024) return true;
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) note_hip_error(e, "hipFuncSetAttribute(max dynamic LDS)");
    return e == hipSuccess;
}

// Gate gradient, the part that crosses block boundaries: xb[head][m] = sum of e_ij a_ij over the pairs
// with key block <= m < query block, from wsum[head][key block][query block][wave].
// First along the query blocks: wsum[J][m][0] <- sum over I > m (one thread per key block J) ...
__global__ __launch_bounds__(64) void k_attn_gate_rows(float* __restrict__ wsum, int nblk) {
    const int jb = blockIdx.x * 64 + threadIdx.x, bh = blockIdx.y;
    if (jb >= nblk) return;
    float* rowp = wsum + ((size_t)bh * nblk + jb) * nblk * 4;
    float run = 0.f;
    for (int i = nblk - 1; i >= jb; --i) {
        const float here = i > jb ? rowp[4 * i] + rowp[4 * i + 1] + rowp[4 * i + 2] + rowp[4 * i + 3] : 0.f;
        rowp[4 * i] = run;
        run += here;
    }
}
// ... then down the key blocks: xb[m] = sum over J <= m (one thread per boundary m)
__global__ __launch_bounds__(64) void k_attn_gate_cols(const float* __restrict__ wsum, float* __restrict__ xb, int nblk) {
    const int m = blockIdx.x * 64 + threadIdx.x, bh = blockIdx.y;
    if (m >= nblk) return;
    float acc = 0.f;
    for (int jb = 0; jb <= m; ++jb) acc += wsum[(((size_t)bh * nblk + jb) * nblk + m) * 4];
    xb[(size_t)bh * nblk + m] = acc;
}

// Rows of the block one wave owns and the waves per SIMD the kernel is compiled for.  Two waves
// per SIMD (at most 256 registers) let one wave's vector-ALU work run under the other's MFMAs
// and are worth more than the larger block: measured, dK / dV at d = 64 take 1.05 ms with 32 keys
// per wave and two waves against 1.58 ms with 64 keys and one.  Only dK / dV at d = 128 (192
// registers of operands and accumulators per wave) cannot fit two.
template <int HD>
struct Shape {
    static constexpr int FWD_OWN = HD == 128 ? 32 : 64, FWD_WPE = 2;
    static constexpr int DQ_OWN = HD == 128 ? 32 : 64, DQ_WPE = 2;
    static constexpr int DKDV_OWN = HD == 32 ? 64 : 32, DKDV_WPE = HD == 128 ? 1 : 2;
};

template <int P, int HD, bool GATED, bool CHUNKED = false>
bool fwd_t(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* V, bf16_t* O, float* Z, int BH, int T, float scale,
           int normalize, const float* bl, ChunkedIn ck = ChunkedIn()) {
    constexpr int WG = 4 * Shape<HD>::FWD_OWN;
    auto kern = k_attn_fwd<P, HD, Shape<HD>::FWD_OWN, Shape<HD>::FWD_WPE, GATED, CHUNKED>;
    if (!allow_smem(kern, attn_smem_bytes<HD>())) return false;
    LaunchScope ls(CHUNKED ? "chunk_fwd" : "attn_fwd", s);
    hipLaunchKernelGGL(kern, dim3((T + WG - 1) / WG, BH), dim3(256), attn_smem_bytes<HD>(), s, Q, K, V, O, Z, T, scale, normalize,
                       bl, ck);
    return launch_ok();
}

template <int P, int HD, bool GATED, bool CHUNKED = false>
bool bwd_t(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* O, const float* Z, const bf16_t* dO,
           bf16_t* Gh, float* gz, bf16_t* dQ, bf16_t* dK, bf16_t* dV, int BH, int T, float scale, int normalize,
           const AttnGate& gate, ChunkedIn ckq = ChunkedIn(), ChunkedIn ckk = ChunkedIn()) {
    const float* bl = gate.bl;
    const long long rows = (long long)BH * T;
    if (!CHUNKED) {
        constexpr int RPB = 256 / (HD / 4);
        LaunchScope ls("attn_bwd_prep", s);
        hipLaunchKernelGGL((k_attn_prep<HD>), dim3((unsigned)((rows + RPB - 1) / RPB)), dim3(256), 0, s, dO, O, Z, Gh, gz, rows,
                           normalize);
        if (!launch_ok()) return false;
    }
    {
        constexpr int WG = 4 * Shape<HD>::DKDV_OWN;
        auto kern = k_attn_dkdv<P, HD, Shape<HD>::DKDV_OWN, Shape<HD>::DKDV_WPE, GATED, CHUNKED>;
        if (!allow_smem(kern, attn_smem_bytes<HD>())) return false;
        LaunchScope ls(CHUNKED ? "chunk_bwd_dkdv" : "attn_bwd_dkdv", s);
        hipLaunchKernelGGL(kern, dim3((T + WG - 1) / WG, BH), dim3(256), attn_smem_bytes<HD>(), s, Q, K, V, Gh, gz, dK, dV, T,
                           scale, bl, gate.kdk, gate.wsum, ckk);
        if (!launch_ok()) return false;
        if (GATED) {
            const int nblk = T / WG;
            LaunchScope ls2("attn_gate_boundary", s);
            hipLaunchKernelGGL(k_attn_gate_rows, dim3((nblk + 63) / 64, BH), dim3(64), 0, s, gate.wsum, nblk);
            hipLaunchKernelGGL(k_attn_gate_cols, dim3((nblk + 63) / 64, BH), dim3(64), 0, s, gate.wsum, gate.xb, nblk);
            if (!launch_ok()) return false;
        }
    }
    {
        constexpr int WG = 4 * Shape<HD>::DQ_OWN;
        auto kern = k_attn_dq<P, HD, Shape<HD>::DQ_OWN, Shape<HD>::DQ_WPE, GATED, CHUNKED>;
        if (!allow_smem(kern, attn_smem_bytes<HD>())) return false;
        LaunchScope ls(CHUNKED ? "chunk_bwd_dq" : "attn_bwd_dq", s);
        hipLaunchKernelGGL(kern, dim3((T + WG - 1) / WG, BH), dim3(256), attn_smem_bytes<HD>(), s, Q, K, V, Gh, gz, dQ, T, scale,
                           bl, gate.qdq, ckq);
        if (!launch_ok()) return false;
    }
    return true;
}

}  // namespace

int attn_gate_block(int d) { return 4 * (d == 128 ? Shape<128>::DKDV_OWN : d == 64 ? Shape<64>::DKDV_OWN : Shape<32>::DKDV_OWN); }

bool attn_shape_ok(int p, int d) { return (p == 2 || p == 3 || p == 4) && (d == 32 || d == 64 || d == 128); }

bool launch_attn_fwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, bf16_t* O, float* Z, int BH,
                     int T, float scale, int normalize, const float* bl) {
#define PA_CASE(PP, DD)                                                                                      \
    if (p == PP && d == DD)                                                                                  \
        return bl != nullptr ? fwd_t<PP, DD, true>(s, Q, K, V, O, Z, BH, T, scale, normalize, bl)            \
                             : fwd_t<PP, DD, false>(s, Q, K, V, O, Z, BH, T, scale, normalize, bl);
    PA_CASE(2, 32) PA_CASE(2, 64) PA_CASE(2, 128)
    PA_CASE(3, 32) PA_CASE(3, 64) PA_CASE(3, 128)
    PA_CASE(4, 32) PA_CASE(4, 64) PA_CASE(4, 128)
#undef PA_CASE
    return false;
}

bool launch_chunk_fwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, bf16_t* O, float* Z, int BH,
                      int T, int cs, float scale, int normalize, const float* part, int nslab, const float* zpart) {
    ChunkedIn ck;
    ck.cs = cs;
    ck.nslab = nslab;
    ck.part = part;
    ck.zpart = zpart;
    if (cs % AT != 0 || T % cs != 0) return false;
#define PA_CASE(PP, DD) \
    if (p == PP && d == DD) return fwd_t<PP, DD, false, true>(s, Q, K, V, O, Z, BH, T, scale, normalize, nullptr, ck);
    PA_CASE(2, 32) PA_CASE(2, 64) PA_CASE(2, 128)
    PA_CASE(3, 32) PA_CASE(3, 64)
    PA_CASE(4, 32)
#undef PA_CASE
    return false;
}

bool launch_attn_prep(hipStream_t s, int d, const bf16_t* dO, const bf16_t* O, const float* Z, bf16_t* Gh, float* gz, long long rows,
                      int normalize) {
    LaunchScope ls("attn_bwd_prep", s);
    if (d == 32)
        hipLaunchKernelGGL((k_attn_prep<32>), dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, s, dO, O, Z, Gh, gz, rows, normalize);
    else if (d == 64)
        hipLaunchKernelGGL((k_attn_prep<64>), dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, s, dO, O, Z, Gh, gz, rows, normalize);
    else if (d == 128)
        hipLaunchKernelGGL((k_attn_prep<128>), dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, s, dO, O, Z, Gh, gz, rows, normalize);
    else
        return false;
    return launch_ok();
}

bool launch_chunk_bwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* Gh,
                      const float* gz, bf16_t* dQ, bf16_t* dK, bf16_t* dV, int BH, int T, int cs, float scale, const float* part_dq,
                      int nslab_dq, const float* part_dk, int nslab_dk, const float* part_dv, int nslab_dv) {
    ChunkedIn ckq, ckk;
    ckq.cs = ckk.cs = cs;
    ckq.part = part_dq;
    ckq.nslab = nslab_dq;
    ckk.part = part_dk;
    ckk.nslab = nslab_dk;
    ckk.part2 = part_dv;
    ckk.nslab2 = nslab_dv;
    if (cs % AT != 0 || T % cs != 0) return false;
#define PA_CASE(PP, DD)     \
    if (p == PP && d == DD) \
        return bwd_t<PP, DD, false, true>(s, Q, K, V, nullptr, nullptr, nullptr, const_cast<bf16_t*>(Gh), const_cast<float*>(gz), dQ, dK, dV, BH, T, scale, 1, AttnGate(), ckq, ckk);
    PA_CASE(2, 32) PA_CASE(2, 64) PA_CASE(2, 128)
    PA_CASE(3, 32) PA_CASE(3, 64)
    PA_CASE(4, 32)
#undef PA_CASE
    return false;
}

bool launch_attn_bwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* O,
                     const float* Z, const bf16_t* dO, bf16_t* Gh, float* gz, bf16_t* dQ, bf16_t* dK, bf16_t* dV, int BH, int T,
                     float scale, int normalize, const AttnGate& gate) {
#define PA_CASE(PP, DD)                                                                                                          \
    if (p == PP && d == DD)                                                                                                      \
        return gate.bl != nullptr ? bwd_t<PP, DD, true>(s, Q, K, V, O, Z, dO, Gh, gz, dQ, dK, dV, BH, T, scale, normalize, gate) \
                                  : bwd_t<PP, DD, false>(s, Q, K, V, O, Z, dO, Gh, gz, dQ, dK, dV, BH, T, scale, normalize, gate);
    PA_CASE(2, 32) PA_CASE(2, 64) PA_CASE(2, 128)
    PA_CASE(3, 32) PA_CASE(3, 64) PA_CASE(3, 128)
    PA_CASE(4, 32) PA_CASE(4, 64) PA_CASE(4, 128)
#undef PA_CASE
    return false;
}

}  // namespace mfma
}  // namespace pa
