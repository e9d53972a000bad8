// Resident-state kernels of the bf16 MFMA family (p = 2): the chunk states of the chunked form
// (arXiv 2507.04239, Sec. 2 "Chunked form", App. E.2 - E.4) are never written to memory.  A workgroup
// owns a slab of the state S (a set of rows of the tiled symmetric-power embedding of Sec. 4.1.1, all
// value columns) as float32 MFMA accumulators, walks the chunks of its stretch of the sequence in order
// and, per chunk, first reads the state out for the chunk's queries (query-state, App. E.4) and then
// adds the chunk's keys (update-state, App. E.2; the cumulative sum of App. E.3 is the accumulator
// itself).  What leaves the chip is the read-out's partial result per slab, token and value column,
// which the per-chunk kernel adds to its in-chunk part.
//
// Embedding and ownership.  phi(x) rows are (a, b) -> x[8 I + a] x[8 J + b] over unordered pairs of
// 8-wide feature blocks {I, J}, multiplicity 2 when I != J (applied to the state, once).  Two such
// tiles with the same a-block form a "pair": 8 values a times 16 b-slots (8 of block J0, 8 of block J1),
// so that a 16-row MFMA block is one a and 16 b-slots.  The factor x[8 I + a] is then the same for the
// 16 rows of a block, a lane reads ONE float of it per k-step, and the multiply fetches the token it
// needs from its 16-lane row by DPP (row_newbcast).  Rows with an odd number of tiles hand one tile over,
// transposed, to another such row, so the tiles pair up without waste (18 pairs at d = 64, 68 at 128).
// A workgroup of 4 waves holds 2 NHP pairs: wave w has the a-half w & 1 (4 values a) of the NHP pairs
// of group w >> 1, i.e. NHP x 4 blocks x (v / 16) column blocks of accumulators (192 registers at d = 64).
//
// The state's accumulator block C[b-slot][v] (lane (r16, g): column v = r16, b-slots 4 g .. 4 g + 3) is,
// rounded to bf16, directly the A operand of the read-out O^T[v][token] += S^T phi(q)^T: its 8 k-slots
// are the b-slots 4 g .. 4 g + 3 of two blocks a, a + 1, and phi(q) is built in exactly that order.
//
// With few heads the sequence is cut into segments (one workgroup per slab, head and segment): a first
// launch adds up every segment's own keys (update only), the second starts each segment from the sum of
// the totals before it.
#include "mfma_common.hpp"

namespace pa {
namespace mfma {
namespace {

// ---- pairs of tiles ---------------------------------------------------------------------------------
// code = a-block | b-block 0 << 8 | b-block 1 << 16 | multiplicity 0 << 24 | multiplicity 1 << 28
template <int NB>
struct PairCodes {
    int n;
    uint32_t v[NB * (NB + 1) / 4];
};
template <int NB>
constexpr PairCodes<NB> make_pair_codes() {
    PairCodes<NB> t{};
    int cnt[NB] = {};
    int tl[NB][NB + 1] = {};
    for (int i = 0; i < NB; ++i)
        for (int j = i; j < NB; ++j) tl[i][cnt[i]++] = j;
    for (int i = 0; i < NB; ++i) {
        if (cnt[i] % 2 == 0) continue;
        for (int j = i + 1; j < NB; ++j) {   // tile {i, j} moves to row j, where i plays the b-block
            if (cnt[j] % 2 == 0) continue;
            int k = 0;
            while (tl[i][k] != j) ++k;
            for (; k + 1 < cnt[i]; ++k) tl[i][k] = tl[i][k + 1];
            --cnt[i];
            tl[j][cnt[j]++] = i;
            break;
        }
    }
    int n = 0;
    for (int i = 0; i < NB; ++i)
        for (int k = 0; k + 1 < cnt[i]; k += 2) {
            const int j0 = tl[i][k], j1 = tl[i][k + 1];
            t.v[n++] = (uint32_t)i | ((uint32_t)j0 << 8) | ((uint32_t)j1 << 16) | ((j0 == i ? 1u : 2u) << 24) |
                       ((j1 == i ? 1u : 2u) << 28);
        }
    t.n = n;
    return t;
}
__constant__ PairCodes<8> PAIRS_64 = make_pair_codes<8>();
__constant__ PairCodes<16> PAIRS_128 = make_pair_codes<16>();
static_assert(make_pair_codes<8>().n == 18 && make_pair_codes<16>().n == 68, "every tile belongs to exactly one pair");

template <int HD>
__device__ __forceinline__ uint32_t pair_code(int i) {
    if (HD == 64) return PAIRS_64.v[min(i, 17)];
    return PAIRS_128.v[min(i, 67)];
}

template <int HD, int NHP>
struct ResShape {
    static constexpr int NVB = HD / 16;                       // value column blocks
    static constexpr int NPAIR = (HD / 8) * (HD / 8 + 1) / 4;
    static constexpr int NSLAB = (NPAIR + 2 * NHP - 1) / (2 * NHP);
    static constexpr int ACC_FLOATS = NHP * 4 * NVB * 256;    // per wave: blocks of 16 x 16 floats
};

// x of lane L of this lane's 16-lane row, times y: one DPP multiply (the compiler's own DPP folding
// leaves most of these as a move plus a multiply).  x must come straight from a load, not from a
// vector-ALU instruction (a DPP read right after such a write needs wait states the assembler does not add).
template <int L>
__device__ __forceinline__ float row_lane_mul(float x, float y) {
    float r;
    asm("v_mul_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x), "v"(y), "n"(L));
    return r;
}

// LDS of the walk.  A read-out phase uses qs and ob, an update phase xs and ys; the two never overlap
// in time, so their inputs share storage.
template <int HD, int GRP, int OBT, int MODE>
struct WalkSmem {
    union {
        struct {
            float qs[MODE != 0 ? GRP : 1][HD + 4];       // read-out side rows (queries), token-major
            bf16_t gs[MODE == 2 ? GRP : 1][HD + 8];      // d phi: the rows the state is contracted with (ghat), token-major
        } rd;
        struct {
            float xs[HD][GRP + 4];               // update side (keys), feature-major
            bf16_t ys[HD][GRP + 8];              // values, feature-major
        } kv;
    } in;
    float ob[MODE != 0 ? 2 : 1][4][MODE != 0 ? OBT : 1][HD + 4];   // each wave's partial result for OBT tokens, double-buffered
};

// one dword of an expanded operand: two products, rounded to bf16
__device__ __forceinline__ uint32_t pk_bf16(float lo, float hi) {
    union {
        __attribute__((ext_vector_type(2))) __bf16 v;
        uint32_t u;
    } o;
    o.v[0] = (__bf16)lo;
    o.v[1] = (__bf16)hi;
    return o.u;
}

// ---- the walk ----------------------------------------------------------------------------------------
// Xt, Yt: feature-major copies [BH][T / 64][HD][64] (bf16) of the update side's rows and values.
// Qr: token-major rows [BH][T][HD] of the read-out side.  tot: per-segment totals, float32,
// [segment][BH][NSLAB][wave][half-pair][a][column block][b-slot][column].  part: [NSLAB][BH][T][HD] float32.
// The sequence is walked chunk by chunk, forwards (REV = false: the state holds the chunks before the
// current one) or backwards (REV = true: the chunks after it), in phases of GRP tokens: per chunk first
// the read-out phases of its token groups (READOUT only; the state entering the chunk is rounded to bf16
// once, times its multiplicity and snap_scale, and held as the read-out's A operands), then the update
// phases.  Keeping the two apart keeps the register need of either below 256 beside the accumulators:
// the rounded state is dead during an update, the update's operands during a read-out.  The next phase's
// input is in flight in registers while a phase computes.
// READOUT = false: a segment's own total is written to tot[segment] (segments 0 .. nseg - 2 are launched).
// READOUT = true: the segment starts from the sum of tot[0 .. segment - 1]; every read-out goes to `part`.
//
// MODE 2 (d phi, the backward pass's gradient through the embedding): the accumulators are kept transposed,
// C[v][b-slot], so that, rounded to bf16, they are the A operand of the contraction over the value columns,
//     A[b-slot][token] = sum_v S[(a, b-slot), v] y_token[v]          (y = Gr: ghat for dQ, v for dK),
// whose result block holds, in lane (token r16, g), the b-slots 4 g .. 4 g + 3 of one a.  The Jacobian of phi
// follows on the vector ALUs, in registers: x[8 J + b] A[b] summed over b goes to feature 8 I + a, and
// x[8 I + a] A[b] summed over a to feature 8 J + b; per 16 tokens the sums land in the wave's LDS buffer.
// `part` then receives J_phi(x_t)^T (S y_t) * snap_scale per slab, token and feature.
template <int HD, int NHP, int GRP, int OBT, bool REV, int MODE>
__global__ __launch_bounds__(256, 1) void k_res_walk(const bf16_t* __restrict__ Xt, const bf16_t* __restrict__ Yt,
                                                     const bf16_t* __restrict__ Qr, const bf16_t* __restrict__ Gr,
                                                     float* __restrict__ tot,
                                                     float* __restrict__ part, int T, int cs, int nheads, int nseg,
                                                     int seg_chunks, float snap_scale) {
    typedef ResShape<HD, NHP> SH;
    constexpr int NVB = SH::NVB, NSLAB = SH::NSLAB;
    constexpr bool READOUT = MODE != 0, DPHI = MODE == 2;
    static_assert(HD * GRP / 8 / 256 == 4, "four 16-byte pieces per thread and staged array");
    static_assert(GRP % OBT == 0 && OBT % 16 == 0 && OBT * HD / 4 / 256 == 2, "read-out buffer shape");
    static_assert(GRP % 64 == 0, "a group is whole 64-token blocks of the feature-major copies");
    extern __shared__ __attribute__((aligned(16))) unsigned char res_smem_raw[];
    WalkSmem<HD, GRP, OBT, MODE>& sm = *reinterpret_cast<WalkSmem<HD, GRP, OBT, MODE>*>(res_smem_raw);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r16 = lane & 15, g = lane >> 4;

    // Workgroups are dealt to the 8 XCDs round-robin by their linear id; the slabs of one head and segment
    // read the same streams, so the work items (segment, head, slab; slab fastest) are laid out in contiguous
    // runs per XCD.
    const int nseg_run = READOUT ? nseg : nseg - 1;
    const int total = nseg_run * nheads * NSLAB;
    const int xcd = blockIdx.x & 7, qi = blockIdx.x >> 3;
    const int base_cnt = total / 8, extra = total % 8;
    if (qi >= base_cnt + (xcd < extra ? 1 : 0)) return;
    const int item = xcd * base_cnt + min(xcd, extra) + qi;
    const int slab = item % NSLAB, bh = (item / NSLAB) % nheads, seg = item / (NSLAB * nheads);

    const int nchunk = T / cs, gpc = cs / GRP, ngrp_all = T / GRP;
    const int c_lo = seg * seg_chunks, c_hi = min(c_lo + seg_chunks, nchunk);
    if (c_lo >= c_hi) return;
    const int ppc = READOUT ? 2 * gpc : gpc;          // phases per chunk
    const int nph = (c_hi - c_lo) * ppc;

    // this wave's half-pairs
    const int pg = w >> 1, ah = w & 1;
    int fa[NHP], fb[NHP], qa_col[NHP], qb_col[NHP];
    float ml[NHP];
#pragma unroll
    for (int h = 0; h < NHP; ++h) {
        const int pi = slab * 2 * NHP + NHP * pg + h;
        const uint32_t code = pair_code<HD>(pi);
        const int ia = code & 255, jb0 = (code >> 8) & 255, jb1 = (code >> 16) & 255;
        const float m0 = (float)((code >> 24) & 15), m1 = (float)(code >> 28);
        fa[h] = 8 * ia + 4 * ah + (r16 >> 3);                // + 2 a2: the feature whose token (r16 & 7) this lane reads
        fb[h] = 8 * (r16 < 8 ? jb0 : jb1) + (r16 & 7);
        qa_col[h] = 8 * ia + 4 * ah;
        qb_col[h] = 8 * (g < 2 ? jb0 : jb1) + 4 * (g & 1);
        // multiplicity of the tile this lane's accumulator rows belong to (b-slots 4 g .. : g; transposed: r16)
        ml[h] = (pi < SH::NPAIR ? ((DPHI ? r16 < 8 : g < 2) ? m0 : m1) : 0.f) * snap_scale;
    }

    f32x4 acc[NHP][4][NVB];
    float* tot_w = tot + (((size_t)bh * NSLAB + slab) * 4 + w) * SH::ACC_FLOATS;
    const size_t tot_seg = (size_t)nheads * NSLAB * 4 * SH::ACC_FLOATS;
#pragma unroll
    for (int h = 0; h < NHP; ++h)
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb) acc[h][a][vb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (READOUT) {
        for (int s0 = 0; s0 < seg; ++s0) {
            const float* src = tot_w + (size_t)s0 * tot_seg;
#pragma unroll
            for (int h = 0; h < NHP; ++h)
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            acc[h][a][vb][r] += DPHI ? src[(((h * 4 + a) * NVB + vb) * 16 + r16) * 16 + 4 * g + r]
                                                     : src[(((h * 4 + a) * NVB + vb) * 16 + 4 * g + r) * 16 + r16];
        }
        // the waves' result buffers start from zero (the d phi sums are added into them)
        for (int e = tid; e < (int)(sizeof(sm.ob) / sizeof(float)); e += 256) (&sm.ob[0][0][0][0])[e] = 0.f;
    }

    const bf16_t* Xh = Xt + (size_t)bh * HD * T;
    const bf16_t* Yh = Yt + (size_t)bh * HD * T;
    const bf16_t* Qh = READOUT ? Qr + (size_t)bh * T * HD : nullptr;
    const bf16_t* Gh = DPHI ? Gr + (size_t)bh * T * HD : nullptr;
    // Phase ph of the segment: chunk c_lo + ph / ppc (walk order); of its ppc phases the first gpc read out
    // (READOUT), the others update; token group (walk order) gw, tokens [tok0, tok0 + GRP).
#define PA_PH_IS_R(PH) (READOUT && ((PH) % ppc) < gpc)
#define PA_PH_TOK0(PH)                                                     \
    ({                                                                     \
        const int gw_ = (c_lo + (PH) / ppc) * gpc + ((PH) % ppc) % gpc;    \
        (REV ? ngrp_all - 1 - gw_ : gw_) * GRP;                            \
    })
    // Staging: piece id = tid + 256 q, q < 4, 8 elements each.  Separately named registers and macros: as
    // arrays, or behind a lambda, the prefetch registers end up in scratch memory.
    uint4 p0, p1, p2, p3, p4, p5, p6, p7;
    p0 = p1 = p2 = p3 = p4 = p5 = p6 = p7 = make_uint4(0, 0, 0, 0);
    // K / V piece: 64-token block id / (8 HD), feature (id / 8) % HD, tokens 8 (id % 8) .. + 7 of the block
#define PA_KV_SRC(Q_) ((size_t)(((tid + 256 * (Q_)) / (8 * HD)) * (HD * TBLK) + (((tid + 256 * (Q_)) >> 3) % HD) * TBLK + ((tid + 256 * (Q_)) & 7) * 8))
#define PA_KV_FEAT(Q_) (((tid + 256 * (Q_)) >> 3) % HD)
#define PA_KV_TOK(Q_) (((tid + 256 * (Q_)) / (8 * HD)) * TBLK + ((tid + 256 * (Q_)) & 7) * 8)
#define PA_LOAD_PHASE(PH)                                                                  \
    {                                                                                      \
        const int ph_ = min((PH), nph - 1);                                                \
        const int tok0_ = PA_PH_TOK0(ph_);                                                 \
        if (PA_PH_IS_R(ph_)) {                                                             \
            const bf16_t* src_ = Qh + (size_t)tok0_ * HD + (size_t)tid * 8;                \
            p0 = *(const uint4*)(src_);                                                    \
            p1 = *(const uint4*)(src_ + 2048);                                             \
            p2 = *(const uint4*)(src_ + 4096);                                             \
            p3 = *(const uint4*)(src_ + 6144);                                             \
            if (DPHI) {                                                                    \
                const bf16_t* gsrc_ = Gh + (size_t)tok0_ * HD + (size_t)tid * 8;           \
                p4 = *(const uint4*)(gsrc_);                                               \
                p5 = *(const uint4*)(gsrc_ + 2048);                                        \
                p6 = *(const uint4*)(gsrc_ + 4096);                                        \
                p7 = *(const uint4*)(gsrc_ + 6144);                                        \
            }                                                                              \
        } else {                                                                           \
            const size_t blk_ = (size_t)(tok0_ / TBLK) * (HD * TBLK);                      \
            p0 = *(const uint4*)(Xh + blk_ + PA_KV_SRC(0));                                \
            p1 = *(const uint4*)(Xh + blk_ + PA_KV_SRC(1));                                \
            p2 = *(const uint4*)(Xh + blk_ + PA_KV_SRC(2));                                \
            p3 = *(const uint4*)(Xh + blk_ + PA_KV_SRC(3));                                \
            p4 = *(const uint4*)(Yh + blk_ + PA_KV_SRC(0));                                \
            p5 = *(const uint4*)(Yh + blk_ + PA_KV_SRC(1));                                \
            p6 = *(const uint4*)(Yh + blk_ + PA_KV_SRC(2));                                \
            p7 = *(const uint4*)(Yh + blk_ + PA_KV_SRC(3));                                \
        }                                                                                  \
    }
#define PA_UNPACK8(D, U)                                                                   \
    {                                                                                      \
        *(float4*)(D) = make_float4(bf_lo(U.x), bf_hi(U.x), bf_lo(U.y), bf_hi(U.y));       \
        *(float4*)((D) + 4) = make_float4(bf_lo(U.z), bf_hi(U.z), bf_lo(U.w), bf_hi(U.w)); \
    }
#define PA_STORE_PHASE(PH)                                                                 \
    {                                                                                      \
        if (PA_PH_IS_R(PH)) {                                                              \
            PA_UNPACK8(&sm.in.rd.qs[(tid + 0) / (HD / 8)][(tid % (HD / 8)) * 8], p0)          \
            PA_UNPACK8(&sm.in.rd.qs[(tid + 256) / (HD / 8)][(tid % (HD / 8)) * 8], p1)        \
            PA_UNPACK8(&sm.in.rd.qs[(tid + 512) / (HD / 8)][(tid % (HD / 8)) * 8], p2)        \
            PA_UNPACK8(&sm.in.rd.qs[(tid + 768) / (HD / 8)][(tid % (HD / 8)) * 8], p3)        \
            if (DPHI) {                                                                    \
                *(uint4*)&sm.in.rd.gs[(tid + 0) / (HD / 8)][(tid % (HD / 8)) * 8] = p4;    \
                *(uint4*)&sm.in.rd.gs[(tid + 256) / (HD / 8)][(tid % (HD / 8)) * 8] = p5;  \
                *(uint4*)&sm.in.rd.gs[(tid + 512) / (HD / 8)][(tid % (HD / 8)) * 8] = p6;  \
                *(uint4*)&sm.in.rd.gs[(tid + 768) / (HD / 8)][(tid % (HD / 8)) * 8] = p7;  \
            }                                                                              \
        } else {                                                                           \
            PA_UNPACK8(&sm.in.kv.xs[PA_KV_FEAT(0)][PA_KV_TOK(0)], p0)                      \
            PA_UNPACK8(&sm.in.kv.xs[PA_KV_FEAT(1)][PA_KV_TOK(1)], p1)                      \
            PA_UNPACK8(&sm.in.kv.xs[PA_KV_FEAT(2)][PA_KV_TOK(2)], p2)                      \
            PA_UNPACK8(&sm.in.kv.xs[PA_KV_FEAT(3)][PA_KV_TOK(3)], p3)                      \
            *(uint4*)&sm.in.kv.ys[PA_KV_FEAT(0)][PA_KV_TOK(0)] = p4;                       \
            *(uint4*)&sm.in.kv.ys[PA_KV_FEAT(1)][PA_KV_TOK(1)] = p5;                       \
            *(uint4*)&sm.in.kv.ys[PA_KV_FEAT(2)][PA_KV_TOK(2)] = p6;                       \
            *(uint4*)&sm.in.kv.ys[PA_KV_FEAT(3)][PA_KV_TOK(3)] = p7;                       \
        }                                                                                  \
    }
    static_assert(256 * 8 == 2048, "piece stride of the token-major rows");

    PA_LOAD_PHASE(0)
    PA_STORE_PHASE(0)
    __syncthreads();
    int ph = 0;
    for (int wc = c_lo; wc < c_hi; ++wc) {
        if (READOUT) {
            // the state entering this chunk, as the read-out's A operands (dead again once the chunk's
            // read-out phases are over)
            // read-out: [a pair][column block], k-slots = b-slots 4 g .. of blocks a, a + 1;
            // d phi: [a][column block pair], k-slots = value columns 4 g .. of column blocks vb, vb + 1
            Frag snap[NHP][DPHI ? 4 : 2][DPHI ? NVB / 2 : NVB];
            {
#pragma unroll
                for (int h = 0; h < NHP; ++h)
#pragma unroll
                    for (int i = 0; i < (DPHI ? 4 : 2); ++i)
#pragma unroll
                        for (int j = 0; j < (DPHI ? NVB / 2 : NVB); ++j)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                snap[h][i][j].v[r] = (__bf16)((DPHI ? acc[h][i][2 * j][r] : acc[h][2 * i][j][r]) * ml[h]);
                                snap[h][i][j].v[4 + r] = (__bf16)((DPHI ? acc[h][i][2 * j + 1][r] : acc[h][2 * i + 1][j][r]) * ml[h]);
                            }
            }
            // read-out: O^T[v][token] += S^T phi(q)^T, 16 tokens at a time; every OBT tokens the four waves'
            // partial results are summed in a fixed order and leave for `part`
#pragma unroll 1
            for (int gi = 0; gi < gpc; ++gi) {
            PA_LOAD_PHASE(ph + 1)
            float* dst = part + (((size_t)slab * nheads + bh) * T + PA_PH_TOK0(ph)) * HD;
#pragma unroll 1
            for (int hb = 0; hb < GRP / OBT; ++hb) {
                const int buf = hb & 1;
#pragma unroll 1
                for (int tb = 0; tb < OBT / 16; ++tb) {
                    const int tok = OBT * hb + 16 * tb + r16;
                    if (DPHI) {
                        Frag gf[NVB / 2];   // y^T: value columns 32 j + 4 g .. + 3 and 32 j + 16 + 4 g .. + 3 of this lane's token
#pragma unroll
                        for (int j = 0; j < NVB / 2; ++j) {
                            gf[j].h[0] = *(const uint2*)&sm.in.rd.gs[tok][32 * j + 4 * g];
                            gf[j].h[1] = *(const uint2*)&sm.in.rd.gs[tok][32 * j + 16 + 4 * g];
                        }
                        float* drow = &sm.ob[buf][w][16 * tb + r16][0];
                        // The four blocks a of a half-pair are four independent MFMA chains; the next half-pair's
                        // chains are issued before this one's Jacobian, which then runs in their shadow.
                        f32x4 c2[2][4];
#pragma unroll
                        for (int a = 0; a < 4; ++a) c2[0][a] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int j = 0; j < NVB / 2; ++j)
#pragma unroll
                            for (int a = 0; a < 4; ++a) c2[0][a] = mfma16(snap[0][a][j].v, gf[j].v, c2[0][a]);
#pragma unroll
                        for (int h = 0; h < NHP; ++h) {
                            const int cur = h & 1;
                            if (h + 1 < NHP) {
#pragma unroll
                                for (int a = 0; a < 4; ++a) c2[cur ^ 1][a] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int j = 0; j < NVB / 2; ++j)
#pragma unroll
                                    for (int a = 0; a < 4; ++a)
                                        c2[cur ^ 1][a] = mfma16(snap[h + 1 < NHP ? h + 1 : 0][a][j].v, gf[j].v, c2[cur ^ 1][a]);
                            }
                            const float4 qa = *(const float4*)&sm.in.rd.qs[tok][qa_col[h]];
                            const float4 qb = *(const float4*)&sm.in.rd.qs[tok][qb_col[h]];
                            const float qav[4] = {qa.x, qa.y, qa.z, qa.w};
                            float ua[4], ub[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int a = 0; a < 4; ++a) {
                                const f32x4 c = c2[cur][a];
                                ua[a] = c[0] * qb.x + c[1] * qb.y + c[2] * qb.z + c[3] * qb.w;
#pragma unroll
                                for (int r = 0; r < 4; ++r) ub[r] += c[r] * qav[a];
                            }
                            // The sums over b are spread over the four lanes g of a token.  Two swaps of 16-lane rows
                            // and one of the 32-lane halves, each followed by an add, leave the total for a = g in lane g.
                            const auto s01 = __builtin_amdgcn_permlane16_swap(__float_as_uint(ua[0]), __float_as_uint(ua[1]), false, false);
                            const auto s23 = __builtin_amdgcn_permlane16_swap(__float_as_uint(ua[2]), __float_as_uint(ua[3]), false, false);
                            const float t01 = __uint_as_float(s01[0]) + __uint_as_float(s01[1]);
                            const float t23 = __uint_as_float(s23[0]) + __uint_as_float(s23[1]);
                            const auto sf = __builtin_amdgcn_permlane32_swap(__float_as_uint(t01), __float_as_uint(t23), false, false);
                            // plain read-add-write: the buffer row belongs to this wave, an instruction's lanes hit
                            // distinct addresses, and a wave's LDS operations stay in order (LDS float atomics
                            // run at a small fraction of this rate)
                            float* pa = drow + qa_col[h] + g;
                            *pa += __uint_as_float(sf[0]) + __uint_as_float(sf[1]);
                            float4* pb = (float4*)(drow + qb_col[h]);
                            float4 cur4 = *pb;
                            cur4.x += ub[0]; cur4.y += ub[1]; cur4.z += ub[2]; cur4.w += ub[3];
                            *pb = cur4;
                        }
                        continue;
                    }
                    f32x4 o[NVB];
#pragma unroll
                    for (int vb = 0; vb < NVB; ++vb) o[vb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int h = 0; h < NHP; ++h) {
                        const float4 qa = *(const float4*)&sm.in.rd.qs[tok][qa_col[h]];
                        const float4 qb = *(const float4*)&sm.in.rd.qs[tok][qb_col[h]];
                        const float qav[4] = {qa.x, qa.y, qa.z, qa.w};
#pragma unroll
                        for (int a2 = 0; a2 < 2; ++a2) {
                            Frag bf;
                            bf.q[0] = pk_bf16(qav[2 * a2] * qb.x, qav[2 * a2] * qb.y);
                            bf.q[1] = pk_bf16(qav[2 * a2] * qb.z, qav[2 * a2] * qb.w);
                            bf.q[2] = pk_bf16(qav[2 * a2 + 1] * qb.x, qav[2 * a2 + 1] * qb.y);
                            bf.q[3] = pk_bf16(qav[2 * a2 + 1] * qb.z, qav[2 * a2 + 1] * qb.w);
#pragma unroll
                            for (int vb = 0; vb < NVB; ++vb) o[vb] = mfma16(snap[h][a2][vb].v, bf.v, o[vb]);
                        }
                    }
#pragma unroll
                    for (int vb = 0; vb < NVB; ++vb)
                        *(float4*)&sm.ob[buf][w][16 * tb + r16][16 * vb + 4 * g] = make_float4(o[vb][0], o[vb][1], o[vb][2], o[vb][3]);
                }
                __syncthreads();
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int e = tid + 256 * q;
                    const int tok = e / (HD / 4), c4 = (e % (HD / 4)) * 4;
                    const float4 a0 = *(const float4*)&sm.ob[buf][0][tok][c4], a1 = *(const float4*)&sm.ob[buf][1][tok][c4];
                    const float4 a2 = *(const float4*)&sm.ob[buf][2][tok][c4], a3 = *(const float4*)&sm.ob[buf][3][tok][c4];
                    *(float4*)(dst + (size_t)(OBT * hb + tok) * HD + c4) =
                        make_float4((a0.x + a1.x) + (a2.x + a3.x), (a0.y + a1.y) + (a2.y + a3.y), (a0.z + a1.z) + (a2.z + a3.z),
                                    (a0.w + a1.w) + (a2.w + a3.w));
                    if (DPHI) {
                        const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
                        *(float4*)&sm.ob[buf][0][tok][c4] = zero;
                        *(float4*)&sm.ob[buf][1][tok][c4] = zero;
                        *(float4*)&sm.ob[buf][2][tok][c4] = zero;
                        *(float4*)&sm.ob[buf][3][tok][c4] = zero;
                    }
                }
            }
            // every wave is past its last read of qs (the barrier above): the next phase's input may land
            if (ph + 1 < nph) PA_STORE_PHASE(ph + 1)
            __syncthreads();
            ++ph;
            }
        }
#pragma unroll 1
        for (int gi = 0; gi < gpc; ++gi) {
            PA_LOAD_PHASE(ph + 1)
            // update: S[b-slot][v] += phi(k)^T V over the group's tokens, 32 at a time.  The 4 NHP row blocks
            // of a k-step are a software pipeline: the three vector-ALU instructions that build one dword of
            // block b + 1's operand (two DPP multiplies, one conversion) follow each MFMA of block b.
#pragma unroll 1
            for (int ks = 0; ks < GRP / 32; ++ks) {
                const int t0 = 32 * ks + 8 * g;
                Frag yf[NVB];
#pragma unroll
                for (int vb = 0; vb < NVB; ++vb) yf[vb].u = *(const uint4*)&sm.in.kv.ys[16 * vb + r16][t0];
                float4 xbl[NHP], xbh[NHP];
                float xa[NHP][2];
#pragma unroll
                for (int h = 0; h < NHP; ++h) {
                    xbl[h] = *(const float4*)&sm.in.kv.xs[fb[h]][t0];
                    xbh[h] = *(const float4*)&sm.in.kv.xs[fb[h]][t0 + 4];
                    xa[h][0] = sm.in.kv.xs[fa[h]][t0 + (r16 & 7)];
                    xa[h][1] = sm.in.kv.xs[fa[h] + 2][t0 + (r16 & 7)];
                }
                Frag fr[2];
                // dword j of block (h, a): lanes 8 (a & 1) + 2 j, + 2 j + 1 of the row hold the tokens' factor
#define PA_DWORD(H_, A_, J_)                                                                                       \
    pk_bf16(row_lane_mul<8 * ((A_) & 1) + 2 * (J_)>(xa[H_][(A_) >> 1], (J_) < 2 ? ((J_) == 0 ? xbl[H_].x : xbl[H_].z) : ((J_) == 2 ? xbh[H_].x : xbh[H_].z)), \
            row_lane_mul<8 * ((A_) & 1) + 2 * (J_) + 1>(xa[H_][(A_) >> 1], (J_) < 2 ? ((J_) == 0 ? xbl[H_].y : xbl[H_].w) : ((J_) == 2 ? xbh[H_].y : xbh[H_].w)))
                fr[0].q[0] = PA_DWORD(0, 0, 0);
                fr[0].q[1] = PA_DWORD(0, 0, 1);
                fr[0].q[2] = PA_DWORD(0, 0, 2);
                fr[0].q[3] = PA_DWORD(0, 0, 3);
#pragma unroll
                for (int h = 0; h < NHP; ++h)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        constexpr int dummy = 0;
                        (void)dummy;
                        const int cur = (4 * h + a) & 1;
                        const bool last = h == NHP - 1 && a == 3;
                        const int hn = a == 3 ? h + 1 : h, an = (a + 1) & 3;
#pragma unroll
                        for (int vb = 0; vb < NVB; ++vb) {
                            __builtin_amdgcn_sched_barrier(0);
                            acc[h][a][vb] = DPHI ? mfma16(yf[vb].v, fr[cur].v, acc[h][a][vb]) : mfma16(fr[cur].v, yf[vb].v, acc[h][a][vb]);
                            if (!last && vb < 4) {
                                // (hn, an, vb) are compile-time after unrolling; the switch keeps the macro's lane indices constant
                                uint32_t dw = 0;
                                switch (4 * (4 * (hn < NHP ? hn : 0) + an) + vb) {
#define PA_CASE(L_, H_, A_, J_) case 4 * (4 * (L_) + (A_)) + (J_): dw = PA_DWORD(H_, A_, J_); break;
#define PA_CASE4(L_, H_, A_) PA_CASE(L_, H_, A_, 0) PA_CASE(L_, H_, A_, 1) PA_CASE(L_, H_, A_, 2) PA_CASE(L_, H_, A_, 3)
#define PA_CASE16(L_, H_) PA_CASE4(L_, H_, 0) PA_CASE4(L_, H_, 1) PA_CASE4(L_, H_, 2) PA_CASE4(L_, H_, 3)
                                    PA_CASE16(0, 0)
                                    PA_CASE16(1, 1)
                                    PA_CASE16(2, NHP > 2 ? 2 : 0)   // label 2 is never reached with two half-pairs
#undef PA_CASE16
#undef PA_CASE4
#undef PA_CASE
                                }
                                fr[cur ^ 1].q[vb] = dw;
                            }
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
#undef PA_DWORD
            }
            __syncthreads();
            if (ph + 1 < nph) PA_STORE_PHASE(ph + 1)
            __syncthreads();
            ++ph;
        }
    }
#undef PA_STORE_PHASE
#undef PA_UNPACK8
#undef PA_LOAD_PHASE
#undef PA_KV_TOK
#undef PA_KV_FEAT
#undef PA_KV_SRC
#undef PA_PH_TOK0
#undef PA_PH_IS_R
    if (!READOUT) {
        float* dst = tot_w + (size_t)seg * tot_seg;
#pragma unroll
        for (int h = 0; h < NHP; ++h)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) dst[(((h * 4 + a) * NVB + vb) * 16 + 4 * g + r) * 16 + r16] = acc[h][a][vb][r];
    }
}

// ---- normaliser: per-chunk Gram matrices and their running sums ---------------------------------------
// phi(q) . sum_j phi(k_j) = q^T (sum_j k_j k_j^T) q: the normaliser column of the state is kept in its d x d form.
// gram[bh][n] = sum over the tokens of chunk n of w_t x_t x_t^T (float32), from the feature-major copy Xt.
// One workgroup per (chunk, head); wave w owns the row blocks w, w + 4, ...
template <int HD>
__global__ __launch_bounds__(256) void k_gram(const bf16_t* __restrict__ Xt, const float* __restrict__ wgt,
                                              float* __restrict__ gram, int T, int cs) {
    constexpr int NB16 = HD / 16;
    const int n = blockIdx.x, bh = blockIdx.y, nchunk = T / cs;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r16 = lane & 15, g = lane >> 4;
    const bf16_t* Xh = Xt + (size_t)bh * HD * T;
    const float* wh = wgt != nullptr ? wgt + (size_t)bh * T : nullptr;
    f32x4 acc[NB16 / 4][NB16];
#pragma unroll
    for (int i = 0; i < NB16 / 4; ++i)
#pragma unroll
        for (int j = 0; j < NB16; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int t0 = n * cs; t0 < (n + 1) * cs; t0 += 32) {
        const int tk = t0 + 8 * g;    // this lane's 8 tokens
        const bf16_t* p = Xh + (size_t)(tk / TBLK) * (HD * TBLK) + (tk % TBLK);
        Frag bfr[NB16];
#pragma unroll
        for (int j = 0; j < NB16; ++j) bfr[j].u = *(const uint4*)(p + (16 * j + r16) * TBLK);
#pragma unroll
        for (int i = 0; i < NB16 / 4; ++i) {
            Frag af;
            af.u = *(const uint4*)(p + (16 * (w + 4 * i) + r16) * TBLK);
            if (wh != nullptr) {
                const float4 w0 = *(const float4*)(wh + tk), w1 = *(const float4*)(wh + tk + 4);
                const uint4 u = af.u;
                af.v[0] = (__bf16)(bf_lo(u.x) * w0.x); af.v[1] = (__bf16)(bf_hi(u.x) * w0.y);
                af.v[2] = (__bf16)(bf_lo(u.y) * w0.z); af.v[3] = (__bf16)(bf_hi(u.y) * w0.w);
                af.v[4] = (__bf16)(bf_lo(u.z) * w1.x); af.v[5] = (__bf16)(bf_hi(u.z) * w1.y);
                af.v[6] = (__bf16)(bf_lo(u.w) * w1.z); af.v[7] = (__bf16)(bf_hi(u.w) * w1.w);
            }
#pragma unroll
            for (int j = 0; j < NB16; ++j) acc[i][j] = mfma16(af.v, bfr[j].v, acc[i][j]);
        }
    }
    float* dst = gram + ((size_t)bh * nchunk + n) * HD * HD;
#pragma unroll
    for (int i = 0; i < NB16 / 4; ++i)
#pragma unroll
        for (int j = 0; j < NB16; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[(16 * (w + 4 * i) + 4 * g + r) * HD + 16 * j + r16] = acc[i][j][r];
}

// out[bh][n] = out_scale * (sum of gram[bh][m] over m < n (forward) or m > n (rev)), bf16; one thread per element
template <int HD>
__global__ __launch_bounds__(256) void k_gram_scan(const float* __restrict__ gram, bf16_t* __restrict__ out, int nchunk,
                                                   int rev, float out_scale) {
    const int e = blockIdx.x * 256 + threadIdx.x, bh = blockIdx.y;
    const float* src = gram + (size_t)bh * nchunk * HD * HD + e;
    bf16_t* dst = out + (size_t)bh * nchunk * HD * HD + e;
    float run = 0.f;
    for (int i = 0; i < nchunk; ++i) {
        const int n = rev ? nchunk - 1 - i : i;
        dst[(size_t)n * HD * HD] = f32_to_bf16(run * out_scale);
        run += src[(size_t)n * HD * HD];
    }
}

// ---- token-major -> feature-major in blocks of 64 tokens, any head size -----------------------------------
// [BH][T][HD] -> [BH][T / 64][HD][64] (bf16); each block is contiguous, so the readers' accesses stay dense.
template <int HD>
__global__ __launch_bounds__(256) void k_transpose_hd(const bf16_t* __restrict__ in, bf16_t* __restrict__ out, int T) {
    __shared__ bf16_t tile[TBLK][HD + 2];
    const int bh = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const bf16_t* src = in + ((size_t)bh * T + (size_t)blk * TBLK) * HD;
    for (int e = tid; e < TBLK * HD; e += 256) tile[e / HD][e % HD] = src[e];
    __syncthreads();
    bf16_t* dst = out + ((size_t)bh * (T / TBLK) + blk) * HD * TBLK;
    for (int e = tid; e < TBLK * HD; e += 256) dst[e] = tile[e % TBLK][e / TBLK];
}

// ---- normaliser terms per token, from the d x d states ------------------------------------------------
// With G = the matrix state of token t's chunk (gam[bh][n], bf16, symmetric) and x_t the token's row:
//     vec[bh][t][:] = cvec * (w_t) * G x_t        (w_t = wgt[bh][t], or 1)     float32, may be null
//     sca[bh][t]    = csca * x_t^T G x_t                                        float32, may be null
// One workgroup of 4 waves per 64 tokens; wave w takes 16 of them.
template <int HD>
__global__ __launch_bounds__(256) void k_gram_apply(const bf16_t* __restrict__ X, const bf16_t* __restrict__ gam,
                                                    const float* __restrict__ wgt, float* __restrict__ vec,
                                                    float* __restrict__ sca, int T, int cs, float cvec, float csca) {
    constexpr int NK = HD / 32, NB16 = HD / 16;
    const int bh = blockIdx.y, t0 = blockIdx.x * 64, nchunk = T / cs;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r16 = lane & 15, g = lane >> 4;
    const size_t row = (size_t)bh * T + t0 + 16 * w + r16;
    const bf16_t* G = gam + ((size_t)bh * nchunk + t0 / cs) * HD * HD;
    Frag xf[NK];
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) xf[ks].u = *(const uint4*)(X + row * HD + 32 * ks + 8 * g);
    const float wt = wgt != nullptr ? wgt[row] : 1.f;
    float dot = 0.f;
#pragma unroll
    for (int ab = 0; ab < NB16; ++ab) {
        f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            Frag gf;
            gf.u = *(const uint4*)(G + (size_t)(16 * ab + r16) * HD + 32 * ks + 8 * g);
            c = mfma16(gf.v, xf[ks].v, c);      // (G x^T): features 16 ab + 4 g + r of token r16
        }
        const uint2 raw = *(const uint2*)(X + row * HD + 16 * ab + 4 * g);
        dot += c[0] * bf_lo(raw.x) + c[1] * bf_hi(raw.x) + c[2] * bf_lo(raw.y) + c[3] * bf_hi(raw.y);
        if (vec != nullptr) {
            const float f = cvec * wt;
            *(float4*)(vec + row * HD + 16 * ab + 4 * g) = make_float4(f * c[0], f * c[1], f * c[2], f * c[3]);
        }
    }
    if (sca != nullptr) {
        dot += __shfl_xor(dot, 16);
        dot += __shfl_xor(dot, 32);
        if (g == 0) sca[row] = csca * dot;
    }
}

template <typename F>
bool allow_smem(F* fn, size_t bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) note_hip_error(e, "hipFuncSetAttribute(max dynamic LDS)");
    return e == hipSuccess;
}

template <int HD, int NHP, int GRP, int OBT, bool REV, int MODE>
bool launch_walk_t(const char* name, hipStream_t s, const bf16_t* Xt, const bf16_t* Yt, const bf16_t* Qr, const bf16_t* Gr,
                   float* tot, float* part, int BH, int T, int cs, int nseg, int seg_chunks, float snap_scale) {
    const size_t smem = sizeof(WalkSmem<HD, GRP, OBT, MODE>);
    auto* fn = k_res_walk<HD, NHP, GRP, OBT, REV, MODE>;
    if (!allow_smem(fn, smem)) return false;
    const int total = (MODE != 0 ? nseg : nseg - 1) * BH * ResShape<HD, NHP>::NSLAB;
    if (total <= 0) return true;
    LaunchScope ls(name, s);
    hipLaunchKernelGGL(fn, dim3(8 * ((total + 7) / 8)), dim3(256), smem, s, Xt, Yt, Qr, Gr, tot, part, T, cs, BH, nseg,
                       seg_chunks, snap_scale);
    return launch_ok();
}

}  // namespace

ResidentPlan resident_plan(int HD, int BH, int T, int cs) {
    ResidentPlan p{};
    p.nhp = HD == 64 ? 3 : 2;
    const int npair = (HD / 8) * (HD / 8 + 1) / 4;
    p.nslab = (npair + 2 * p.nhp - 1) / (2 * p.nhp);
    const int nchunk = T / cs;
    // one workgroup per compute unit: as many segments as fill the 256 of them
    int nseg = 256 / (BH * p.nslab);
    nseg = nseg < 1 ? 1 : (nseg > nchunk ? nchunk : nseg);
    p.seg_chunks = (nchunk + nseg - 1) / nseg;
    p.nseg = (nchunk + p.seg_chunks - 1) / p.seg_chunks;
    p.acc_floats = (size_t)p.nhp * 4 * (HD / 16) * 256;
    p.tot_bytes = (size_t)(p.nseg > 1 ? p.nseg - 1 : 0) * BH * p.nslab * 4 * p.acc_floats * sizeof(float);
    p.part_bytes = (size_t)p.nslab * BH * T * HD * sizeof(float);
    p.gram_bytes = (size_t)BH * nchunk * HD * HD * sizeof(float);
    return p;
}

bool launch_res_walk(const char* name, hipStream_t s, int HD, bool rev, int mode, const bf16_t* Xt, const bf16_t* Yt,
                     const bf16_t* Qr, const bf16_t* Gr, float* tot, float* part, int BH, int T, int cs, const ResidentPlan& pl,
                     float snap_scale) {
#define PA_GO(HDV, NHPV, GRPV, OBTV, R, M) \
    return launch_walk_t<HDV, NHPV, GRPV, OBTV, R, M>(name, s, Xt, Yt, Qr, Gr, tot, part, BH, T, cs, pl.nseg, pl.seg_chunks, snap_scale);
#define PA_MODES(HDV, NHPV, GRPV, OBTV)              \
    if (!rev) {                                      \
        if (mode == 0) PA_GO(HDV, NHPV, GRPV, OBTV, false, 0) \
        if (mode == 1) PA_GO(HDV, NHPV, GRPV, OBTV, false, 1) \
        if (mode == 2) PA_GO(HDV, NHPV, GRPV, OBTV, false, 2) \
    } else {                                         \
        if (mode == 0) PA_GO(HDV, NHPV, GRPV, OBTV, true, 0)  \
        if (mode == 1) PA_GO(HDV, NHPV, GRPV, OBTV, true, 1)  \
        if (mode == 2) PA_GO(HDV, NHPV, GRPV, OBTV, true, 2)  \
    }
    if (HD == 64) { PA_MODES(64, 3, 128, 32) }
    if (HD == 128) { PA_MODES(128, 2, 64, 16) }
#undef PA_MODES
#undef PA_GO
    return false;
}

bool launch_transpose_hd(hipStream_t s, int HD, const bf16_t* in, bf16_t* out, int BH, int T) {
    LaunchScope ls("res_transpose", s);
    if (HD == 64)
        hipLaunchKernelGGL(k_transpose_hd<64>, dim3(T / TBLK, BH), dim3(256), 0, s, in, out, T);
    else if (HD == 128)
        hipLaunchKernelGGL(k_transpose_hd<128>, dim3(T / TBLK, BH), dim3(256), 0, s, in, out, T);
    else
        return false;
    return launch_ok();
}

bool launch_gram_apply(hipStream_t s, int HD, const bf16_t* X, const bf16_t* gam, const float* wgt, float* vec, float* sca,
                       int BH, int T, int cs, float cvec, float csca) {
    LaunchScope ls("res_gram_apply", s);
    if (HD == 64)
        hipLaunchKernelGGL(k_gram_apply<64>, dim3(T / 64, BH), dim3(256), 0, s, X, gam, wgt, vec, sca, T, cs, cvec, csca);
    else if (HD == 128)
        hipLaunchKernelGGL(k_gram_apply<128>, dim3(T / 64, BH), dim3(256), 0, s, X, gam, wgt, vec, sca, T, cs, cvec, csca);
    else
        return false;
    return launch_ok();
}

bool launch_gram(hipStream_t s, int HD, const bf16_t* Xt, const float* wgt, float* gram, bf16_t* out, int BH, int T, int cs,
                 bool rev, float out_scale) {
    const int nchunk = T / cs;
    if (HD != 64 && HD != 128) return false;
    {
        LaunchScope ls("res_gram", s);
        if (HD == 64)
            hipLaunchKernelGGL(k_gram<64>, dim3(nchunk, BH), dim3(256), 0, s, Xt, wgt, gram, T, cs);
        else
            hipLaunchKernelGGL(k_gram<128>, dim3(nchunk, BH), dim3(256), 0, s, Xt, wgt, gram, T, cs);
        if (!launch_ok()) return false;
    }
    LaunchScope ls("res_gram_scan", s);
    if (HD == 64)
        hipLaunchKernelGGL(k_gram_scan<64>, dim3(64 * 64 / 256, BH), dim3(256), 0, s, (const float*)gram, out, nchunk,
                           rev ? 1 : 0, out_scale);
    else
        hipLaunchKernelGGL(k_gram_scan<128>, dim3(128 * 128 / 256, BH), dim3(256), 0, s, (const float*)gram, out, nchunk,
                           rev ? 1 : 0, out_scale);
    return launch_ok();
}

}  // namespace mfma
}  // namespace pa
