// Per-chunk kernels of the bf16 MFMA family (p = 2): forward (attention form inside the chunk +
// query-state read-out + normalisation, App. E.1 / E.4 of arXiv 2507.04239) and the three
// backward kernels (dQ, dK, dV).  See mfma_common.hpp for the embedding and the state layouts.
//
// All four share one shape: grid (T / 128, B*H), 128 threads; wave wv owns token rows
// [64 wv, 64 wv + 64) of the block as four 16-token MFMA column blocks `ib`.  The block's own
// rows (Q or K) sit in LDS as bf16; accumulators are transposed, acc[fb][ib] = 16 features (or
// value columns) x 16 tokens.  Register use is kept under 256 so that two waves share a SIMD
// and one wave's vector-ALU work (building phi, the Jacobian of phi) overlaps the other's MFMAs.
#include "mfma_common.hpp"

namespace pa {
namespace mfma {
namespace {

constexpr int XB_PITCH = DH + 8;   // bf16 elements; 36 dwords, so 16 rows hit 16 distinct bank groups

typedef bf16_t XbRow[XB_PITCH];

__device__ __forceinline__ float lds_bf(const bf16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }

__device__ __forceinline__ void stage_rows(XbRow* Xb, const bf16_t* __restrict__ X, size_t row0, int tid, int nthreads = 128) {
    for (int e = tid; e < QBLK * DH / 8; e += nthreads) {
        const int row = e >> 3, c8 = e & 7;
        *(uint4*)&Xb[row][8 * c8] = *(const uint4*)(X + (row0 + row) * DH + 8 * c8);
    }
}

// B (or A) operand of a 16-row block of the staged rows: features 32 ks + 8 g .. + 7 of row `row`
__device__ __forceinline__ bf16x8 lds_frag(const XbRow* Xb, int row, int ks, int g) {
    Frag f;
    f.u = *(const uint4*)&Xb[row][32 * ks + 8 * g];
    return f.v;
}

__device__ __forceinline__ bf16x8 glb_frag(const bf16_t* __restrict__ X, size_t row, int ks, int g) {
    Frag f;
    f.u = *(const uint4*)(X + row * DH + 32 * ks + 8 * g);
    return f.v;
}

// A operand whose k-slots are the 8 tokens {t0 + 4g + r, t0 + 16 + 4g + r : r < 4} of feature row
// `feat` of a feature-major copy (the k-slot order of a C-layout block fed back as a B operand)
__device__ __forceinline__ bf16x8 tmajor_frag(const bf16_t* __restrict__ Xt_head, int feat, int t0, int g) {
    const bf16_t* p = Xt_head + (size_t)(t0 / TBLK) * (DH * TBLK) + feat * TBLK + (t0 % TBLK) + 4 * g;
    Frag f;
    f.h[0] = *(const uint2*)p;
    f.h[1] = *(const uint2*)(p + 16);
    return f.v;
}

constexpr f32x4 ZERO4 = {0.f, 0.f, 0.f, 0.f};

// The 128-token block this workgroup works on.  With cs > 128 the cs / 128 blocks of one stretch
// stream the same state.  Workgroups are dealt to the 8 XCDs round-robin by their linear id, each XCD
// with an L2 of its own, so the blocks of a stretch are given ids 8 apart: same XCD, dispatched
// almost together, and part of the state traffic stays in that L2 (measured at cs = 256: the dK / dV
// kernel fetches 1.9 GB instead of 2.5 GB).
__device__ __forceinline__ int stretch_block(int cs) {
    const int nb = cs / QBLK, per = 8 * nb, x = blockIdx.x;
    if (nb == 1 || gridDim.x % per != 0) return x;
    const int r = x % per;
    return (8 * (x / per) + (r & 7)) * nb + (r >> 3);
}

// ---- state streaming: global -> LDS ring of 8 KB tiles, without passing through registers ------
// A workgroup streams one chunk state (36 tiles of 8 KB) per kernel.  The two waves would
// otherwise both load every byte (twice the L1 / L2 traffic, and measurably less HBM bandwidth).
// Instead each wave issues half of a tile's eight 1 KB `global_load_lds` copies (64 lanes x 16
// bytes land contiguously at the LDS address held in M0), RING_TILES - 1 tiles ahead, and both
// read their MFMA fragments from LDS.  One barrier per tile keeps the waves in step: after it,
// tile t is complete and the slot of tile t - 1 is free.  The fragment reads go through inline
// assembly on purpose: the compiler cannot tell the ring reads from the copies in flight and
// would wait for ALL of them before every read.
constexpr int TILE_U4 = TILE_ELEMS / 8;   // 16-byte units per tile
constexpr int RING_RO = 4;                // ring depth of the read-out kernels (bound by HBM)
constexpr int RING_DP = 2;                // ring depth of the d phi kernels (bound by the vector ALUs:
                                          // a smaller ring lets a fourth workgroup share the CU)

template <int RING_TILES>
struct ChunkSmem {
    bf16_t xb[QBLK][XB_PITCH];
    uint4 ring[RING_TILES][TILE_U4];
};

__device__ __forceinline__ uint4 lds_read16(uint32_t addr) {
    uint4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}

// Transposing LDS read (ds_read_b64_tr_b16).  Inside each group of 16 lanes, lane 4 j + m points
// at 4 consecutive 16-bit elements: row j, columns 4 m .. 4 m + 3 of a 4 x 16 block.  Lane n
// receives column n of the block, i.e. element n % 4 of the lanes n / 4 + 4 j, j = 0 .. 3.
template <int OFF>
__device__ __forceinline__ uint2 lds_read_tr(uint32_t addr) {
    uint2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}

// Wait for this wave's LDS reads.  The eight fragments they fill pass through the statement as
// in/out registers, so that no use of them can be scheduled ahead of the wait.
__device__ __forceinline__ void lds_read_wait(Frag& f0, Frag& f1, Frag& f2, Frag& f3, Frag& f4, Frag& f5, Frag& f6, Frag& f7) {
    u32x4 u0 = f0.q, u1 = f1.q, u2 = f2.q, u3 = f3.q, u4 = f4.q, u5 = f5.q, u6 = f6.q, u7 = f7.q;
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(u0), "+v"(u1), "+v"(u2), "+v"(u3), "+v"(u4), "+v"(u5), "+v"(u6), "+v"(u7)
                 :
                 : "memory");
    f0.q = u0;
    f1.q = u1;
    f2.q = u2;
    f3.q = u3;
    f4.q = u4;
    f5.q = u5;
    f6.q = u6;
    f7.q = u7;
}

// Copy tile `tile` of the state `Sn` (layout [a][v][b], 16-byte units (a, v)) into ring slot
// `slot`.  SWIZZLE = false: straight copy, for the read-out, whose fragment order is the storage
// order.  SWIZZLE = true, for the transposing reads of d phi: unit (a, v) is stored at
// (a, v ^ 4 (a & 1)), which puts the two rows a of one transposing read on different banks.
// NW waves share the ring; wave `wr` of them issues 8 / NW of a tile's eight copies.
template <bool SWIZZLE, int NW, int RING_TILES>
__device__ __forceinline__ void ring_issue(ChunkSmem<RING_TILES>& sm, int slot, const bf16_t* __restrict__ Sn, int tile, int wr,
                                           int lane) {
    const bf16_t* src = Sn + (size_t)tile * TILE_ELEMS;
#pragma unroll
    for (int q = 0; q < 8 / NW; ++q) {
        const int instr = (8 / NW) * wr + q;
        const int unit = instr * 64 + (SWIZZLE ? (lane ^ ((instr & 1) << 2)) : lane);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + unit * 8),
                                         (__attribute__((address_space(3))) void*)&sm.ring[slot][instr * 64], 16, 0, 2);   // (aux 2: streaming, each state byte is read once)
    }
}

// Traversal order of the 36 tiles for the d phi contraction: by blocks of 2 x 2 tiles
// (fbi, fbj) = (ti >> 1, tj >> 1), fbj outermost, so that inside one block the accumulator rows
// both terms add to, acc[fbi] and acc[fbj], are compile-time names.  Entry = ti | tj << 8 |
// tile index << 16; one sentinel at the end repeats the last tile.
struct DphiOrder {
    int v[NTILES + 1];
};
constexpr DphiOrder make_dphi_order() {
    DphiOrder t{};
    int k = 0;
    for (int fbj = 0; fbj < 4; ++fbj)
        for (int fbi = 0; fbi <= fbj; ++fbi)
            for (int tj = 2 * fbj; tj < 2 * fbj + 2; ++tj)
                for (int ti = 2 * fbi; ti < 2 * fbi + 2; ++ti)
                    if (ti <= tj) t.v[k++] = ti | (tj << 8) | ((tj * (tj + 1) / 2 + ti) << 16);
    t.v[k] = t.v[k - 1];
    return t;
}
__constant__ DphiOrder DPHI_ORDER = make_dphi_order();
constexpr int dphi_block_begin(int fbi, int fbj) {
    int k = 0;
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i <= j; ++i) {
            if (i == fbi && j == fbj) return k;
            k += (i == j) ? 3 : 4;
        }
    return k;
}

// ---- read-out: contraction over the expanded rows (query-state, App. E.4) -----------------------
// acc[vb][ib] += S^T phi(xscale^(1/2) x)^T for the 64 tokens of wave wv.  `Sn` is one state in
// layout "C": tile (ti, tj) = two steps of 32 expanded rows, step s holding rows a = 4s + g.
// Must be called by both waves of the workgroup (it contains barriers).
// DORDER = false: tiles in storage order from a plain ring.  DORDER = true: tiles in the order
// of the d phi contraction from a swizzled ring, for a workgroup whose other waves do that
// contraction on the same ring.  `wv`: which 64 tokens; `wr`: this wave's index among the NW
// waves that share the ring.
// GATED: the contribution of token column ib is multiplied by colf[ib] (folded into x[8 tj ..]).
template <int RING_TILES, int NW, bool DORDER, bool GATED = false>
__device__ __forceinline__ void readout(f32x4 (&acc)[4][4], const bf16_t* __restrict__ Sn, ChunkSmem<RING_TILES>& sm,
                                        float xscale, int wv, int wr, int lane, const float* colf = nullptr) {
    const int r16 = lane & 15, g = lane >> 4;
    const XbRow* Xb = sm.xb;
    // fragment (s, vb) of a tile: unit (a = 4 s + g, v = 16 vb + r16); swizzled: v ^ 4 (a & 1)
    const uint32_t ring0 = lds_addr(&sm.ring[0][0]) + (uint32_t)(g * 64 + (DORDER ? (r16 ^ ((g & 1) << 2)) : r16)) * 16u;
    auto tile_of = [&](int k) { return DORDER ? (DPHI_ORDER.v[min(k, NTILES)] >> 16) : min(k, NTILES - 1); };
#pragma unroll
    for (int t = 0; t < RING_TILES - 1; ++t) ring_issue<DORDER, NW>(sm, t, Sn, tile_of(t), wr, lane);
    int ti = 0, tj = 0, tj_loaded = -1;
    float xbv[4][8];
    for (int k = 0; k < NTILES; ++k) {
        if (DORDER) {
            const int code = DPHI_ORDER.v[k];
            ti = code & 255;
            tj = (code >> 8) & 255;
        }
        vm_wait<(8 / NW) * (RING_TILES - 2)>();
        __builtin_amdgcn_s_barrier();
        ring_issue<DORDER, NW>(sm, (k + RING_TILES - 1) % RING_TILES, Sn, tile_of(k + RING_TILES - 1), wr, lane);
        const uint32_t slot = ring0 + (uint32_t)(k % RING_TILES) * (TILE_U4 * 16u);
        Frag sf[2][4];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) sf[s][vb].u = lds_read16(slot + (uint32_t)(s * 256 + vb * 16) * 16u);
        if (tj != tj_loaded) {   // a new column block tj: x[8 tj .. 8 tj + 7] of each token
            tj_loaded = tj;
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const uint4 raw = *(const uint4*)&Xb[64 * wv + 16 * ib + r16][8 * tj];
                xbv[ib][0] = bf_lo(raw.x); xbv[ib][1] = bf_hi(raw.x);
                xbv[ib][2] = bf_lo(raw.y); xbv[ib][3] = bf_hi(raw.y);
                xbv[ib][4] = bf_lo(raw.z); xbv[ib][5] = bf_hi(raw.z);
                xbv[ib][6] = bf_lo(raw.w); xbv[ib][7] = bf_hi(raw.w);
                if (GATED) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) xbv[ib][i] *= colf[ib];
                }
            }
        }
        lds_read_wait(sf[0][0], sf[0][1], sf[0][2], sf[0][3], sf[1][0], sf[1][1], sf[1][2], sf[1][3]);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            Frag pf[4];
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const float xa = xscale * lds_bf(&Xb[64 * wv + 16 * ib + r16][8 * ti + 4 * s + g]);
#pragma unroll
                for (int i = 0; i < 8; ++i) pf[ib].v[i] = (__bf16)(xa * xbv[ib][i]);
            }
#pragma unroll
            for (int vb = 0; vb < 4; ++vb)
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = mfma16(sf[s][vb].v, pf[ib].v, acc[vb][ib]);
        }
        if (!DORDER && ++ti > tj) {
            ++tj;
            ti = 0;
        }
    }
    vm_wait<0>();
}

// ---- d phi: contraction over the value columns, then the Jacobian of phi ----------------------
// For the 64 tokens of wave wv, x~ = xscale * x, and a state `Sn` (layout [a][v][b], the same
// copy the read-out uses; the operand of this contraction needs 8 value columns per lane, which
// the transposing LDS read gathers from 8 units):
//     A[(a,b), token] = sum_v S[(ti,tj,a,b), v] y[token, v]                       (MFMA)
//     acc[8 ti + a][token] += sum_b A[(a,b)] x~[8 tj + b]        (term 1)
//     acc[8 tj + b][token] += sum_a A[(a,b)] x~[8 ti + a]        (term 2)        (vector ALU)
// i.e. acc += J_phi(x~)^T (S y), phi(x)_(ti,tj,a,b) = x[8ti+a] x[8tj+b] (tile multiplicity is in
// S).  yf[ib][ks] are the B operands y^T (k-slots = value columns 32 ks + 8 g ..).
//
// The MFMA result block (rb, ib) holds, in lane (token r16, g), rows a = 2 rb + (g >> 1),
// b = 4 (g & 1) + r.  Both terms are finished in registers: term 2 is summed over the tiles of a
// column block tj and lands once per visit; term 1 is summed across the lane pair, exchanged
// across the half-waves and added by the lane that owns feature 8 ti + a in the accumulator
// layout (feature 16 fb + 4 g' + r').
template <int FBI, int FBJ, int RING_TILES, int NW, bool GATED>
__device__ __forceinline__ void dphi_block(f32x4 (&acc)[4][4], const bf16_t* __restrict__ Sn, ChunkSmem<RING_TILES>& sm,
                                           const Frag (&yf)[4][2], float xscale, int wv, int wr, int lane,
                                           const float* colf) {
    constexpr int K0 = dphi_block_begin(FBI, FBJ), K1 = K0 + (FBI == FBJ ? 3 : 4);
    const int r16 = lane & 15, g = lane >> 4;
    const XbRow* Xb = sm.xb;
    // Fragment (rb, ks) of a tile in the ring = state rows 16 rb + r16 (a = 2 rb + (r16 >> 3),
    // b = r16 & 7), value columns 32 ks + 8 g .. + 7, from two transposing reads (columns
    // + 0..3, + 4..7).  As a source lane of those reads, lane (r16 = 4 j + m, g) points at the
    // four b = 4 (m & 1) .. + 3 of unit (a = 2 rb + (m >> 1), v = 32 ks + 8 g + 4 h + j).
    const int sj = r16 >> 2, sm1 = (r16 >> 1) & 1, sm0 = r16 & 1;
    const uint32_t lane_lo = (uint32_t)(16 * (64 * sm1 + 8 * g + (4 * sm1) + sj) + 8 * sm0);   // h = 0, swizzled
    const uint32_t ring_lo = lds_addr(&sm.ring[0][0]) + lane_lo;
    const uint32_t ring_hi = lds_addr(&sm.ring[0][0]) + (lane_lo ^ 64u);                       // h = 1
    float xb[4][4], u2[4][4];
#pragma unroll 1
    for (int k = K0; k < K1; ++k) {
        const int code = DPHI_ORDER.v[k];
        const int ti = code & 255, tj = (code >> 8) & 255;
        vm_wait<(8 / NW) * (RING_TILES - 2)>();
        __builtin_amdgcn_s_barrier();
        ring_issue<true, NW>(sm, (k + RING_TILES - 1) % RING_TILES, Sn, DPHI_ORDER.v[min(k + RING_TILES - 1, NTILES)] >> 16, wr, lane);
        const uint32_t slot_lo = ring_lo + (uint32_t)(k % RING_TILES) * (TILE_U4 * 16u);
        const uint32_t slot_hi = ring_hi + (uint32_t)(k % RING_TILES) * (TILE_U4 * 16u);
        Frag sf[4][2];
#define PA_TR(RB, KS)                                                       \
    sf[RB][KS].h[0] = lds_read_tr<2048 * (RB) + 512 * (KS)>(slot_lo);       \
    sf[RB][KS].h[1] = lds_read_tr<2048 * (RB) + 512 * (KS)>(slot_hi);
        PA_TR(0, 0) PA_TR(0, 1) PA_TR(1, 0) PA_TR(1, 1) PA_TR(2, 0) PA_TR(2, 1) PA_TR(3, 0) PA_TR(3, 1)
#undef PA_TR
        if (ti == 2 * FBI) {   // first tile of a column block: x~[8 tj + 4 (g&1) + r]; restart term 2
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const uint2 raw = *(const uint2*)&Xb[64 * wv + 16 * ib + r16][8 * tj + 4 * (g & 1)];
                xb[ib][0] = xscale * bf_lo(raw.x); xb[ib][1] = xscale * bf_hi(raw.x);
                xb[ib][2] = xscale * bf_lo(raw.y); xb[ib][3] = xscale * bf_hi(raw.y);
#pragma unroll
                for (int r = 0; r < 4; ++r) u2[ib][r] = 0.f;
            }
        }
        // Row blocks rb and rb + 2 go through the cross-lane steps together.  After the 16-lane
        // swap and one add, the 16-lane rows hold the term-1 sums over all b for
        // a = 2 rb, 2 rb + 4, 2 rb + 1, 2 rb + 5; the 32-lane swap brings a and a + 1 together in
        // the lanes g with (g & 1) = a >> 2, and the two lanes g >> 1 = ti & 1 own those features.
        const float own_mask = ((g >> 1) == (ti & 1)) ? 1.f : 0.f;
        lds_read_wait(sf[0][0], sf[0][1], sf[1][0], sf[1][1], sf[2][0], sf[2][1], sf[3][0], sf[3][1]);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                f32x4 ca = mfma16(sf[rb][0].v, yf[ib][0].v, ZERO4);
                ca = mfma16(sf[rb][1].v, yf[ib][1].v, ca);
                f32x4 cb = mfma16(sf[rb + 2][0].v, yf[ib][0].v, ZERO4);
                cb = mfma16(sf[rb + 2][1].v, yf[ib][1].v, cb);
                const bf16_t* xrow = &Xb[64 * wv + 16 * ib + r16][8 * ti + 2 * rb + (g >> 1)];
                const float xa_a = lds_bf(xrow), xa_b = lds_bf(xrow + 4);   // unscaled: xscale is applied on landing
                const float own_a = ca[0] * xb[ib][0] + ca[1] * xb[ib][1] + ca[2] * xb[ib][2] + ca[3] * xb[ib][3];
                const float own_b = cb[0] * xb[ib][0] + cb[1] * xb[ib][1] + cb[2] * xb[ib][2] + cb[3] * xb[ib][3];
                const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(own_a), __float_as_uint(own_b), false, false);
                float lo, hi;
                halves(__uint_as_float(sw[0]) + __uint_as_float(sw[1]), lo, hi);
                const float om = GATED ? own_mask * colf[ib] : own_mask;
                acc[FBI][ib][2 * rb] += om * lo;
                acc[FBI][ib][2 * rb + 1] += om * hi;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    u2[ib][r] += ca[r] * xa_a;
                    u2[ib][r] += cb[r] * xa_b;
                }
            }
        }
        if (ti == min(tj, 2 * FBI + 1)) {   // last tile of the column block here: land term 2
            const float mk = ((g >> 1) == (tj & 1)) ? xscale : 0.f;
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const float mkc = GATED ? mk * colf[ib] : mk;
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[FBJ][ib][r] += mkc * xor32_sum(u2[ib][r]);
            }
        }
    }
}

// Must be called by all NW waves that share the ring (it contains barriers), or run side by side
// with waves that execute readout<.., NW, true> on the same ring.
// GATED: the contribution of token column ib is multiplied by colf[ib] (folded into the masks).
template <int RING_TILES, int NW, bool GATED = false>
__device__ __forceinline__ void dphi(f32x4 (&acc)[4][4], const bf16_t* __restrict__ Sn, ChunkSmem<RING_TILES>& sm,
                                     const Frag (&yf)[4][2], float xscale, int wv, int wr, int lane,
                                     const float* colf = nullptr) {
#pragma unroll
    for (int k = 0; k < RING_TILES - 1; ++k) ring_issue<true, NW>(sm, k, Sn, DPHI_ORDER.v[k] >> 16, wr, lane);
#define PA_BLOCK(I, J) dphi_block<I, J, RING_TILES, NW, GATED>(acc, Sn, sm, yf, xscale, wv, wr, lane, colf);
    PA_BLOCK(0, 0) PA_BLOCK(0, 1) PA_BLOCK(1, 1) PA_BLOCK(0, 2) PA_BLOCK(1, 2) PA_BLOCK(2, 2)
    PA_BLOCK(0, 3) PA_BLOCK(1, 3) PA_BLOCK(2, 3) PA_BLOCK(3, 3)
#undef PA_BLOCK
    vm_wait<0>();
}

// ---- gating ------------------------------------------------------------------------------------
// Gated kernels (template flag GATED; Sec. 2 "Gating", App. E.2 / E.3) take two per-token arrays:
// bl, the sum of the log-gates from the start of the token's chunk, and fac, the decay that goes
// with the state term: exp(bl_i) for a query (the state is seen from the chunk's start), or
// exp(bl_end - bl_j) for a key (its contribution to R is seen from the chunk's end).  The state
// term's routines fold fac into values they already multiply by; a pair inside the chunk carries
// exp(bl_i - bl_j).  Masked pairs are zeroed by selection, so an overflowing factor of a masked
// pair is harmless.

// x_t . (the accumulator column of token t) for the wave's tokens, from the float32 accumulators
// acc[fb][ib] (16 features x 16 tokens; lane (r16, g) holds features 16 fb + 4 g + r of token r16)
// and the bf16 rows x in LDS; written by the lanes g == 0.  These dot products give the gradient
// of the log-gates: a_ij is homogeneous of degree p in q_i and in k_j.
__device__ __forceinline__ void store_row_dots(float* __restrict__ out, size_t row0, const f32x4 (&acc)[4][4],
                                               const XbRow* Xb, int xrow0, float mul, int r16, int g) {
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        float s = 0.f;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            const uint2 raw = *(const uint2*)&Xb[xrow0 + 16 * ib + r16][16 * fb + 4 * g];
            s += acc[fb][ib][0] * bf_lo(raw.x) + acc[fb][ib][1] * bf_hi(raw.x) + acc[fb][ib][2] * bf_lo(raw.y) +
                 acc[fb][ib][3] * bf_hi(raw.y);
        }
        s = xor32_sum(xor16_sum(s));
        if (g == 0) out[row0 + 16 * ib + r16] = mul * s;
    }
}

// per-lane values of a per-token array for the wave's four 16-token column blocks
__device__ __forceinline__ void load_cols(float (&out)[4], const float* __restrict__ arr, size_t row0, int r16) {
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) out[ib] = arr[row0 + 16 * ib + r16];
}

// ---- forward chunk kernel -------------------------------------------------------------------------
// acc[vb][ib] = O^T: 16 value columns x 16 queries.
// PARTIAL: the state's read-out has already been taken (resident-state walk); its per-slab partial
// sums part[slab][bh][t][v] (float32, already scaled) are added instead of streaming the state.
template <bool GATED, bool PARTIAL = false>
__global__ __launch_bounds__(128, 2) void k_mfma_fwd_chunk(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                           const bf16_t* __restrict__ Vt, const bf16_t* __restrict__ StC,
                                                           const bf16_t* __restrict__ Gam, bf16_t* __restrict__ O,
                                                           float* __restrict__ Z, int T, int cs, float scale,
                                                           int normalize, const float* __restrict__ bl,
                                                           const float* __restrict__ qfac,
                                                           const float* __restrict__ part, int nslab) {
    __shared__ __attribute__((aligned(16))) ChunkSmem<RING_RO> sm;
    XbRow* Xb = sm.xb;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    const int i0 = stretch_block(cs) * QBLK;         // first query row of the block
    const int n = i0 / cs;                    // state entering the stretch this block lies in
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;
    const bf16_t* Vt_head = Vt + (size_t)bh * DH * T;
    const float s2 = scale * scale;

    stage_rows(Xb, Q, head_tok + i0, tid);
    f32x4 acc[4][4];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = ZERO4;
    float zsum[4] = {0.f, 0.f, 0.f, 0.f};     // per query block: partial sum of scores (this lane's k-slots)
    __syncthreads();

    float blq[4] = {0.f, 0.f, 0.f, 0.f};
    if (GATED) load_cols(blq, bl, head_tok + i0 + 64 * wv, r16);

    // attention form over the keys of the stretch, up to the diagonal
    for (int kb0 = n * cs; kb0 <= i0; kb0 += QBLK) {
        const bool diag = kb0 == i0;
        const int nsteps = diag ? 2 * (wv + 1) : 4;     // 32-key steps this wave needs
        for (int s = 0; s < nsteps; ++s) {
            const int key0 = kb0 + 32 * s;
            Frag pf[4];   // P^T as B operand; k-slots: keys 4g+r of block 0, then of block 1
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                const size_t krow = head_tok + key0 + 16 * jb + r16;
                const bf16x8 kf0 = glb_frag(K, krow, 0, g), kf1 = glb_frag(K, krow, 1, g);
                float blk[4] = {0.f, 0.f, 0.f, 0.f};
                if (GATED) {
                    const float4 b4 = *(const float4*)(bl + head_tok + key0 + 16 * jb + 4 * g);
                    blk[0] = b4.x; blk[1] = b4.y; blk[2] = b4.z; blk[3] = b4.w;
                }
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    const int qrow = 64 * wv + 16 * ib + r16;
                    f32x4 c = mfma16(kf0, lds_frag(Xb, qrow, 0, g), ZERO4);
                    c = mfma16(kf1, lds_frag(Xb, qrow, 1, g), c);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float pv = s2 * c[r] * c[r];
                        if (GATED) pv *= __expf(blq[ib] - blk[r]);
                        if (diag && key0 + 16 * jb + 4 * g + r > i0 + qrow) pv = 0.f;
                        // the denominator sums the ROUNDED weights, the ones the numerator uses: the
                        // output is then an exact convex combination (a row that sees one key returns
                        // that value bit for bit, which the backward pass's cancellations rely on)
                        const __bf16 pb = (__bf16)pv;
                        zsum[ib] += (float)pb;
                        pf[ib].v[4 * jb + r] = pb;
                    }
                }
            }
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) {
                const bf16x8 vf = tmajor_frag(Vt_head, 16 * vb + r16, key0, g);
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = mfma16(vf, pf[ib].v, acc[vb][ib]);
            }
        }
    }

    if (n > 0) {
        float qf[4] = {1.f, 1.f, 1.f, 1.f};
        if (GATED) load_cols(qf, qfac, head_tok + i0 + 64 * wv, r16);
        // phi(q~) . gamma = q~^T Gamma q~
        const bf16_t* Gn = Gam + (size_t)(bh * nstate + n) * DH * DH;
#pragma unroll 1
        for (int ab = 0; ab < 4; ++ab) {
            const bf16x8 gm0 = glb_frag(Gn, 16 * ab + r16, 0, g), gm1 = glb_frag(Gn, 16 * ab + r16, 1, g);
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const int qrow = 64 * wv + 16 * ib + r16;
                f32x4 c = mfma16(gm0, lds_frag(Xb, qrow, 0, g), ZERO4);
                c = mfma16(gm1, lds_frag(Xb, qrow, 1, g), c);
                const uint2 raw = *(const uint2*)&Xb[qrow][16 * ab + 4 * g];
                const float zs = s2 * (c[0] * bf_lo(raw.x) + c[1] * bf_hi(raw.x) + c[2] * bf_lo(raw.y) + c[3] * bf_hi(raw.y));
                zsum[ib] += GATED ? qf[ib] * zs : zs;
            }
        }
        if (PARTIAL) {
            const size_t slab_stride = (size_t)gridDim.y * T * DH;
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const float* prow = part + (head_tok + i0 + 64 * wv + 16 * ib + r16) * DH + 4 * g;
                for (int sl = 0; sl < nslab; ++sl)
#pragma unroll
                    for (int vb = 0; vb < 4; ++vb) {
                        const float4 pv = *(const float4*)(prow + sl * slab_stride + 16 * vb);
                        acc[vb][ib][0] += pv.x; acc[vb][ib][1] += pv.y; acc[vb][ib][2] += pv.z; acc[vb][ib][3] += pv.w;
                    }
            }
        } else {
            readout<RING_RO, 2, false, GATED>(acc, StC + (size_t)(bh * nstate + n) * STATE_ELEMS, sm, s2, wv, wv, lane, qf);
        }
    }

#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        float z = zsum[ib];
        z = xor32_sum(xor16_sum(z));
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
//   dq_i = scale * [ sum_{j<=i, same stretch} t_ij k_j + 2 gz_i Gamma q~_i + J_phi(q~_i)^T (S_n ghat_i) ]
//   q~ = scale q,  s_ij = q~_i . k_j,  t_ij = 2 s_ij (ghat_i . v_j + gz_i)
// acc[fb][ib] = (the bracket)^T: 16 features x 16 queries.
template <bool GATED>
__global__ __launch_bounds__(128, 2) void k_mfma_bwd_dq(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                        const bf16_t* __restrict__ V, const bf16_t* __restrict__ Gh,
                                                        const float* __restrict__ gz, const bf16_t* __restrict__ Kt,
                                                        const bf16_t* __restrict__ StC, const bf16_t* __restrict__ Gam,
                                                        bf16_t* __restrict__ dQ, int T, int cs, float scale,
                                                        const float* __restrict__ bl, const float* __restrict__ qfac,
                                                        float* __restrict__ qdq) {
    __shared__ __attribute__((aligned(16))) ChunkSmem<RING_DP> sm;
    XbRow* Xb = sm.xb;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    const int i0 = stretch_block(cs) * QBLK;
    const int n = i0 / cs;
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;
    const bf16_t* Kt_head = Kt + (size_t)bh * DH * T;

    stage_rows(Xb, Q, head_tok + i0, tid);
    Frag gf[4][2];   // ghat^T of this wave's queries as B operands
    float gzq[4];
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        const size_t row = head_tok + i0 + 64 * wv + 16 * ib + r16;
        gf[ib][0].v = glb_frag(Gh, row, 0, g);
        gf[ib][1].v = glb_frag(Gh, row, 1, g);
        gzq[ib] = gz[row];
    }
    f32x4 acc[4][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) acc[fb][ib] = ZERO4;
    __syncthreads();

    float blq[4] = {0.f, 0.f, 0.f, 0.f};
    if (GATED) load_cols(blq, bl, head_tok + i0 + 64 * wv, r16);

    for (int kb0 = n * cs; kb0 <= i0; kb0 += QBLK) {
        const bool diag = kb0 == i0;
        const int nsteps = diag ? 2 * (wv + 1) : 4;
        for (int s = 0; s < nsteps; ++s) {
            const int key0 = kb0 + 32 * s;
            Frag tf[4];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                const size_t krow = head_tok + key0 + 16 * jb + r16;
                const bf16x8 kf0 = glb_frag(K, krow, 0, g), kf1 = glb_frag(K, krow, 1, g);
                const bf16x8 vf0 = glb_frag(V, krow, 0, g), vf1 = glb_frag(V, krow, 1, g);
                float blk[4] = {0.f, 0.f, 0.f, 0.f};
                if (GATED) {
                    const float4 b4 = *(const float4*)(bl + head_tok + key0 + 16 * jb + 4 * g);
                    blk[0] = b4.x; blk[1] = b4.y; blk[2] = b4.z; blk[3] = b4.w;
                }
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    const int qrow = 64 * wv + 16 * ib + r16;
                    f32x4 c = mfma16(kf0, lds_frag(Xb, qrow, 0, g), ZERO4);
                    c = mfma16(kf1, lds_frag(Xb, qrow, 1, g), c);
                    f32x4 e = mfma16(vf0, gf[ib][0].v, ZERO4);
                    e = mfma16(vf1, gf[ib][1].v, e);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float tv = 2.f * scale * c[r] * (e[r] + gzq[ib]);
                        if (GATED) tv *= __expf(blq[ib] - blk[r]);
                        if (diag && key0 + 16 * jb + 4 * g + r > i0 + qrow) tv = 0.f;
                        tf[ib].v[4 * jb + r] = (__bf16)tv;
                    }
                }
            }
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) {
                const bf16x8 ktf = tmajor_frag(Kt_head, 16 * fb + r16, key0, g);
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) acc[fb][ib] = mfma16(ktf, tf[ib].v, acc[fb][ib]);
            }
        }
    }
    if (n > 0) {
        float qf[4] = {1.f, 1.f, 1.f, 1.f};
        if (GATED) load_cols(qf, qfac, head_tok + i0 + 64 * wv, r16);
        // normaliser: d/dq~ of gz q~^T Gamma q~ = 2 gz Gamma q~
        const bf16_t* Gn = Gam + (size_t)(bh * nstate + n) * DH * DH;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
            const bf16x8 gm0 = glb_frag(Gn, 16 * ab + r16, 0, g), gm1 = glb_frag(Gn, 16 * ab + r16, 1, g);
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                const int qrow = 64 * wv + 16 * ib + r16;
                f32x4 c = mfma16(gm0, lds_frag(Xb, qrow, 0, g), ZERO4);
                c = mfma16(gm1, lds_frag(Xb, qrow, 1, g), c);
                const float f = 2.f * gzq[ib] * scale * (GATED ? qf[ib] : 1.f);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[ab][ib][r] += f * c[r];
            }
        }
        dphi<RING_DP, 2, GATED>(acc, StC + (size_t)(bh * nstate + n) * STATE_ELEMS, sm, gf, scale, wv, wv, lane, qf);
    }
    if (GATED) store_row_dots(qdq, head_tok + i0 + 64 * wv, acc, Xb, 64 * wv, scale, r16, g);
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        const size_t row = head_tok + i0 + 64 * wv + 16 * ib + r16;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (__bf16)(scale * acc[fb][ib][r]);
            *(bf16x4*)(dQ + row * DH + 16 * fb + 4 * g) = o;
        }
    }
}

// ---- backward, keys: dK ---------------------------------------------------------------------------
//   dk_j = scale * sum_{i>=j, same stretch} t_ij q_i + 2 Omega_m k_j + J_phi(k_j)^T (R_m v_j)
// (R and Omega already carry scale^2).  acc[fb][jb] = dK^T: 16 features x 16 keys.
// Body for the 64 keys of token half `wv`; the block's K rows are already staged in sm.xb.
template <int RING_TILES, int NW, bool GATED>
__device__ __forceinline__ void dk_body(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                                        const bf16_t* __restrict__ Gh, const float* __restrict__ gz,
                                        const bf16_t* __restrict__ Qt, const bf16_t* __restrict__ RtC,
                                        const bf16_t* __restrict__ Omg, bf16_t* __restrict__ dK, int T, int cs, float scale,
                                        const float* __restrict__ bl, const float* __restrict__ kfac,
                                        float* __restrict__ kdk, ChunkSmem<RING_TILES>& sm, int wv, int wr, int lane) {
    const XbRow* Xb = sm.xb;
    const int r16 = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    const int j0 = stretch_block(cs) * QBLK;
    const int m = j0 / cs;
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;
    const bf16_t* Qt_head = Qt + (size_t)bh * DH * T;

    Frag vf[4][2];   // V^T of this wave's keys as B operands
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        const size_t row = head_tok + j0 + 64 * wv + 16 * jb + r16;
        vf[jb][0].v = glb_frag(V, row, 0, g);
        vf[jb][1].v = glb_frag(V, row, 1, g);
    }
    f32x4 acc[4][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) acc[fb][jb] = ZERO4;

    float blk[4] = {0.f, 0.f, 0.f, 0.f};
    if (GATED) load_cols(blk, bl, head_tok + j0 + 64 * wv, r16);

    // The state part comes first: the workgroups that stream the same state then start on it together
    // (the pairs inside the stretch, whose number differs from block to block, follow).  Measured 3 %
    // faster than the other order here - and 5 to 10 % slower in the forward and dQ kernels, which keep it.
    if (m < nstate - 1) {
        float kf[4] = {1.f, 1.f, 1.f, 1.f};
        if (GATED) load_cols(kf, kfac, head_tok + j0 + 64 * wv, r16);
        const bf16_t* Om = Omg + (size_t)(bh * nstate + m) * DH * DH;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
            const bf16x8 gm0 = glb_frag(Om, 16 * ab + r16, 0, g), gm1 = glb_frag(Om, 16 * ab + r16, 1, g);
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                const int krow = 64 * wv + 16 * jb + r16;
                f32x4 c = mfma16(gm0, lds_frag(Xb, krow, 0, g), ZERO4);
                c = mfma16(gm1, lds_frag(Xb, krow, 1, g), c);
                const float f = GATED ? 2.f * kf[jb] : 2.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[ab][jb][r] += f * c[r];
            }
        }
        dphi<RING_TILES, NW, GATED>(acc, RtC + (size_t)(bh * nstate + m) * STATE_ELEMS, sm, vf, 1.f, wv, wr, lane, kf);
    }
    const float ts = 2.f * scale * scale;   // d s / d k = scale q; t carries 2 scale
    const int q_hi = (m + 1) * cs;          // queries of the same stretch, from the diagonal block on
    for (int qb0 = j0; qb0 < q_hi; qb0 += QBLK) {
        const bool diag = qb0 == j0;
        for (int s = diag ? 2 * wv : 0; s < 4; ++s) {   // queries before this wave's first key are masked
            const int q0 = qb0 + 32 * s;
            Frag tf[4];
#pragma unroll
            for (int ibq = 0; ibq < 2; ++ibq) {
                const size_t qrow = head_tok + q0 + 16 * ibq + r16;
                const bf16x8 qa0 = glb_frag(Q, qrow, 0, g), qa1 = glb_frag(Q, qrow, 1, g);
                const bf16x8 ga0 = glb_frag(Gh, qrow, 0, g), ga1 = glb_frag(Gh, qrow, 1, g);
                const float4 gz4 = *(const float4*)(gz + head_tok + q0 + 16 * ibq + 4 * g);
                const float gzr[4] = {gz4.x, gz4.y, gz4.z, gz4.w};
                float blq[4] = {0.f, 0.f, 0.f, 0.f};
                if (GATED) {
                    const float4 b4 = *(const float4*)(bl + head_tok + q0 + 16 * ibq + 4 * g);
                    blq[0] = b4.x; blq[1] = b4.y; blq[2] = b4.z; blq[3] = b4.w;
                }
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) {
                    const int krow = 64 * wv + 16 * jb + r16;
                    f32x4 c = mfma16(qa0, lds_frag(Xb, krow, 0, g), ZERO4);
                    c = mfma16(qa1, lds_frag(Xb, krow, 1, g), c);
                    f32x4 e = mfma16(ga0, vf[jb][0].v, ZERO4);
                    e = mfma16(ga1, vf[jb][1].v, e);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float tv = ts * c[r] * (e[r] + gzr[r]);
                        if (GATED) tv *= __expf(blq[r] - blk[jb]);
                        if (diag && q0 + 16 * ibq + 4 * g + r < j0 + krow) tv = 0.f;
                        tf[jb].v[4 * ibq + r] = (__bf16)tv;
                    }
                }
            }
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) {
                const bf16x8 qtf = tmajor_frag(Qt_head, 16 * fb + r16, q0, g);
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) acc[fb][jb] = mfma16(qtf, tf[jb].v, acc[fb][jb]);
            }
        }
    }
    if (GATED) store_row_dots(kdk, head_tok + j0 + 64 * wv, acc, Xb, 64 * wv, 1.f, r16, g);
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        const size_t row = head_tok + j0 + 64 * wv + 16 * jb + r16;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (__bf16)acc[fb][jb][r];
            *(bf16x4*)(dK + row * DH + 16 * fb + 4 * g) = o;
        }
    }
}

// ---- backward, values: dV ---------------------------------------------------------------------------
//   dv_j = sum_{i>=j, same stretch} s_ij^2 ghat_i + R_m^T phi(k_j)
// acc[vb][jb] = dV^T: 16 value columns x 16 keys.
// Body for the 64 keys of token half `wv`; the block's K rows are already staged in sm.xb.
template <int RING_TILES, int NW, bool DORDER, bool GATED>
__device__ __forceinline__ void dv_body(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                        const bf16_t* __restrict__ Ght, const bf16_t* __restrict__ RtC,
                                        bf16_t* __restrict__ dV, int T, int cs, float scale, const float* __restrict__ bl,
                                        const float* __restrict__ kfac, ChunkSmem<RING_TILES>& sm, int wv, int wr, int lane) {
    const XbRow* Xb = sm.xb;
    const int r16 = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    const int j0 = stretch_block(cs) * QBLK;
    const int m = j0 / cs;
    const int nstate = T / cs;
    const size_t head_tok = (size_t)bh * T;
    const bf16_t* Ght_head = Ght + (size_t)bh * DH * T;
    const float s2 = scale * scale;

    f32x4 acc[4][4];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) acc[vb][jb] = ZERO4;

    float blk[4] = {0.f, 0.f, 0.f, 0.f};
    if (GATED) load_cols(blk, bl, head_tok + j0 + 64 * wv, r16);

    // state part first, as in dk_body (the two run side by side and meet at the ring's barriers)
    if (m < nstate - 1) {
        float kf[4] = {1.f, 1.f, 1.f, 1.f};
        if (GATED) load_cols(kf, kfac, head_tok + j0 + 64 * wv, r16);
        readout<RING_TILES, NW, DORDER, GATED>(acc, RtC + (size_t)(bh * nstate + m) * STATE_ELEMS, sm, 1.f, wv, wr, lane, kf);
    }
    const int q_hi = (m + 1) * cs;
    for (int qb0 = j0; qb0 < q_hi; qb0 += QBLK) {
        const bool diag = qb0 == j0;
        for (int s = diag ? 2 * wv : 0; s < 4; ++s) {
            const int q0 = qb0 + 32 * s;
            Frag af[4];
#pragma unroll
            for (int ibq = 0; ibq < 2; ++ibq) {
                const size_t qrow = head_tok + q0 + 16 * ibq + r16;
                const bf16x8 qa0 = glb_frag(Q, qrow, 0, g), qa1 = glb_frag(Q, qrow, 1, g);
                float blq[4] = {0.f, 0.f, 0.f, 0.f};
                if (GATED) {
                    const float4 b4 = *(const float4*)(bl + head_tok + q0 + 16 * ibq + 4 * g);
                    blq[0] = b4.x; blq[1] = b4.y; blq[2] = b4.z; blq[3] = b4.w;
                }
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) {
                    const int krow = 64 * wv + 16 * jb + r16;
                    f32x4 c = mfma16(qa0, lds_frag(Xb, krow, 0, g), ZERO4);
                    c = mfma16(qa1, lds_frag(Xb, krow, 1, g), c);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float av = s2 * c[r] * c[r];
                        if (GATED) av *= __expf(blq[r] - blk[jb]);
                        if (diag && q0 + 16 * ibq + 4 * g + r < j0 + krow) av = 0.f;
                        af[jb].v[4 * ibq + r] = (__bf16)av;
                    }
                }
            }
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) {
                const bf16x8 gtf = tmajor_frag(Ght_head, 16 * vb + r16, q0, g);
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) acc[vb][jb] = mfma16(gtf, af[jb].v, acc[vb][jb]);
            }
        }
    }
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        const size_t row = head_tok + j0 + 64 * wv + 16 * jb + r16;
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (__bf16)acc[vb][jb][r];
            *(bf16x4*)(dV + row * DH + 16 * vb + 4 * g) = o;
        }
    }
}

// ---- backward, keys and values in one pass over R ------------------------------------------------
// dK and dV both stream the state gradient R_m of their chunk.  Here one workgroup of four waves
// streams it once: waves 0, 1 run the dK body and waves 2, 3 the dV body for the same 128 keys,
// all four feeding and reading one LDS ring (swizzled for the transposing reads of d phi, tiles
// in the d phi order; the read-out does not care about either).  The two bodies execute the same
// number of barriers.
constexpr int RING_KV = 4;
template <bool GATED>
__global__ __launch_bounds__(256, 2) void k_mfma_bwd_dkdv(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                          const bf16_t* __restrict__ V, const bf16_t* __restrict__ Gh,
                                                          const float* __restrict__ gz, const bf16_t* __restrict__ Qt,
                                                          const bf16_t* __restrict__ Ght, const bf16_t* __restrict__ RtC,
                                                          const bf16_t* __restrict__ Omg, bf16_t* __restrict__ dK,
                                                          bf16_t* __restrict__ dV, int T, int cs, float scale,
                                                          const float* __restrict__ bl, const float* __restrict__ kfac,
                                                          float* __restrict__ kdk) {
    __shared__ __attribute__((aligned(16))) ChunkSmem<RING_KV> sm;
    const int tid = threadIdx.x, lane = tid & 63, w4 = tid >> 6;
    stage_rows(sm.xb, K, (size_t)blockIdx.y * T + stretch_block(cs) * QBLK, tid, 256);
    __syncthreads();
    if (w4 < 2)
        dk_body<RING_KV, 4, GATED>(Q, K, V, Gh, gz, Qt, RtC, Omg, dK, T, cs, scale, bl, kfac, kdk, sm, w4, w4, lane);
    else
        dv_body<RING_KV, 4, true, GATED>(Q, K, Ght, RtC, dV, T, cs, scale, bl, kfac, sm, w4 - 2, w4, lane);
}

// ---- gating: the pairs that straddle a chunk boundary -------------------------------------------
// xb[bh][n] = < R_n , S_{n+1} > + < Omega_n , Gamma_{n+1} >: the sum of e_ij a_ij over the pairs
// j <= end of chunk n < i (0 for the last chunk), which the gradient of the log-gates needs per
// boundary.  Both stored states carry the tile multiplicity; the inner product of the expanded
// vectors carries it once, hence the 1/2 on the off-diagonal tiles.
__device__ __forceinline__ float dot8(uint4 a, uint4 b) {
    return bf_lo(a.x) * bf_lo(b.x) + bf_hi(a.x) * bf_hi(b.x) + bf_lo(a.y) * bf_lo(b.y) + bf_hi(a.y) * bf_hi(b.y) +
           bf_lo(a.z) * bf_lo(b.z) + bf_hi(a.z) * bf_hi(b.z) + bf_lo(a.w) * bf_lo(b.w) + bf_hi(a.w) * bf_hi(b.w);
}
__global__ __launch_bounds__(256) void k_mfma_gate_boundary(const bf16_t* __restrict__ StC, const bf16_t* __restrict__ RtC,
                                                            const bf16_t* __restrict__ Gam, const bf16_t* __restrict__ Omg,
                                                            float* __restrict__ xb, int nstate) {
    __shared__ float red[4];
    const int n = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    float acc = 0.f;
    if (n < nstate - 1) {
        const uint4* S = (const uint4*)(StC + (size_t)(bh * nstate + n + 1) * STATE_ELEMS);
        const uint4* R = (const uint4*)(RtC + (size_t)(bh * nstate + n) * STATE_ELEMS);
        int ti = 0, tj = 0;
        for (int tile = 0; tile < NTILES; ++tile) {
            float part = 0.f;
            for (int u = tid; u < TILE_U4; u += 256) part += dot8(S[tile * TILE_U4 + u], R[tile * TILE_U4 + u]);
            acc += ti == tj ? part : 0.5f * part;
            if (++ti > tj) {
                ++tj;
                ti = 0;
            }
        }
        const uint4* G = (const uint4*)(Gam + (size_t)(bh * nstate + n + 1) * DH * DH);
        const uint4* W = (const uint4*)(Omg + (size_t)(bh * nstate + n) * DH * DH);
        for (int u = tid; u < DH * DH / 8; u += 256) acc += dot8(G[u], W[u]);
    }
    acc = xor32_sum(xor16_sum(acc));
    for (int off = 8; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) xb[(size_t)bh * nstate + n] = red[0] + red[1] + red[2] + red[3];
}

}  // namespace

bool launch_gate_boundary(hipStream_t s, const bf16_t* stC, const bf16_t* rtC, const bf16_t* gam, const bf16_t* omg, float* xb,
                          int BH, int nstate) {
    LaunchScope ls("mfma_gate_boundary", s);
    hipLaunchKernelGGL(k_mfma_gate_boundary, dim3(nstate, BH), dim3(256), 0, s, stC, rtC, gam, omg, xb, nstate);
    return launch_ok();
}

// `gate`: bl and the state-term decay (qfac for the query-side kernels, kfac for the key-side one),
// both null when the problem is not gated
bool launch_fwd_chunk(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* Vt, const bf16_t* stC,
                      const bf16_t* gam, bf16_t* O, float* Z, int BH, int T, int cs, float scale, int normalize,
                      const float* bl, const float* qfac, const float* part, int nslab) {
    LaunchScope ls(part != nullptr ? "mfma_fwd_chunk_partial" : "mfma_fwd_chunk", s);
    if (part != nullptr)
        hipLaunchKernelGGL((k_mfma_fwd_chunk<false, true>), dim3(T / QBLK, BH), dim3(128), 0, s, Q, K, Vt, stC, gam, O, Z, T, cs,
                           scale, normalize, bl, qfac, part, nslab);
    else if (bl != nullptr)
        hipLaunchKernelGGL((k_mfma_fwd_chunk<true>), dim3(T / QBLK, BH), dim3(128), 0, s, Q, K, Vt, stC, gam, O, Z, T, cs, scale,
                           normalize, bl, qfac, part, nslab);
    else
        hipLaunchKernelGGL((k_mfma_fwd_chunk<false>), dim3(T / QBLK, BH), dim3(128), 0, s, Q, K, Vt, stC, gam, O, Z, T, cs, scale,
                           normalize, bl, qfac, part, nslab);
    return launch_ok();
}

bool launch_bwd_prep(hipStream_t s, const bf16_t* dO, const bf16_t* O, const float* Z, bf16_t* Gh, float* gz,
                     long long rows, int normalize) {
    LaunchScope ls("mfma_bwd_prep", s);
    hipLaunchKernelGGL(k_mfma_bwd_prep, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, s, dO, O, Z, Gh, gz, rows,
                       normalize);
    return launch_ok();
}

bool launch_bwd_dq(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* Gh,
                   const float* gz, const bf16_t* Kt, const bf16_t* stC, const bf16_t* gam, bf16_t* dQ, int BH, int T,
                   int cs, float scale, const float* bl, const float* qfac, float* qdq) {
    LaunchScope ls("mfma_bwd_dq", s);
    if (bl != nullptr)
        hipLaunchKernelGGL(k_mfma_bwd_dq<true>, dim3(T / QBLK, BH), dim3(128), 0, s, Q, K, V, Gh, gz, Kt, stC, gam, dQ, T, cs,
                           scale, bl, qfac, qdq);
    else
        hipLaunchKernelGGL(k_mfma_bwd_dq<false>, dim3(T / QBLK, BH), dim3(128), 0, s, Q, K, V, Gh, gz, Kt, stC, gam, dQ, T, cs,
                           scale, bl, qfac, qdq);
    return launch_ok();
}

bool launch_bwd_dkdv(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* Gh, const float* gz,
                     const bf16_t* Qt, const bf16_t* Ght, const bf16_t* rtC, const bf16_t* omg, bf16_t* dK, bf16_t* dV, int BH,
                     int T, int cs, float scale, const float* bl, const float* kfac, float* kdk) {
    LaunchScope ls("mfma_bwd_dkdv", s);
    if (bl != nullptr)
        hipLaunchKernelGGL(k_mfma_bwd_dkdv<true>, dim3(T / QBLK, BH), dim3(256), 0, s, Q, K, V, Gh, gz, Qt, Ght, rtC, omg, dK,
                           dV, T, cs, scale, bl, kfac, kdk);
    else
        hipLaunchKernelGGL(k_mfma_bwd_dkdv<false>, dim3(T / QBLK, BH), dim3(256), 0, s, Q, K, V, Gh, gz, Qt, Ght, rtC, omg, dK,
                           dV, T, cs, scale, bl, kfac, kdk);
    return launch_ok();
}

}  // namespace mfma
}  // namespace pa
