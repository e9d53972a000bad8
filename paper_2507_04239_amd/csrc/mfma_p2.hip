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
// grid (NTILES + 1, BH), 256 threads.  Workgroup `tile` owns the 64 x DH state tile (ti, tj);
// wave w owns its rows a in {2w, 2w+1}.  Workgroup NTILES owns Gamma = sum k k^T (same code:
// the A operand is k itself and the B operand comes from K instead of V).  The state is
// written every `cs` tokens, before the tokens of that stretch are added.  Each workgroup
// walks the sequence in stages of 64 tokens; the walk is a chain of tiny steps, so the
// operands of SCAN_PF stages are kept in flight in registers.
constexpr int SCAN_PF = 8;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory,
// i.e. waits for every outstanding global load, which would drain the register ring below.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <bool GAMMA>
__device__ __forceinline__ void scan_body(const bf16_t* __restrict__ Kt, const bf16_t* __restrict__ Vt,
                                          bf16_t* __restrict__ St, bf16_t* __restrict__ Gam, int T, int cs,
                                          bf16_t (*Vs)[DH][72]) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int tile = blockIdx.x, bh = blockIdx.y;
    const int nstate = T / cs;
    int ti = 0, tj = 0;
    if (!GAMMA) {
        for (int l = 0; l < tile; ++l) {
            if (++ti > tj) {
                ++tj;
                ti = 0;
            }
        }
    }
    const float mult = (ti == tj) ? 1.f : 2.f;
    const int fa = GAMMA ? 16 * w + r16 : 8 * ti + 2 * w + (r16 >> 3);
    const int fb = GAMMA ? fa : 8 * tj + (r16 & 7);
    constexpr int STAGE = DH * TBLK;   // elements of one 64-token block of Kt / Vt
    const bf16_t* Ka = Kt + (size_t)bh * DH * T + fa * TBLK + 8 * g;
    const bf16_t* Kb = Kt + (size_t)bh * DH * T + fb * TBLK + 8 * g;
    // B operand staging through LDS: thread -> (column, 16 tokens)
    const int vcol = tid >> 2, vpiece = tid & 3;
    const bf16_t* Bsrc = (GAMMA ? Kt : Vt) + (size_t)bh * DH * T + vcol * TBLK + 16 * vpiece;

    f32x4 acc[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) acc[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    auto write_state = [&](int n) {
        if (!GAMMA) {
            bf16_t* dst = St + ((size_t)(bh * nstate + n) * NTILES + tile) * TILE_ELEMS;
            const int a = 2 * w + (g >> 1), b0 = 4 * (g & 1);
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[cb][r] * mult);
                *(bf16x4*)(dst + ((a * DH + 16 * cb + r16) * 8 + b0)) = o;
            }
        } else {
            bf16_t* dst = Gam + (size_t)(bh * nstate + n) * DH * DH;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int r = 0; r < 4; ++r) dst[(16 * w + 4 * g + r) * DH + 16 * cb + r16] = f32_to_bf16(acc[cb][r]);
        }
    };

    // Tokens at or after T - cs never feed a state that is written, so the walk stops there.
    const int nstage = (T - cs) / 64;
    if (nstage > 0) {
        // Register ring: slot j holds the operands of stage (st0 + j).  Every load is
        // unconditional (indices are clamped instead of branching) so that the compiler can
        // count the loads in flight instead of waiting for all of them.
        // (separately named registers and macros instead of arrays and lambdas: the slot has
        // to be a compile-time name or the ring is demoted to scratch memory)
#define PA_SLOT(J) uint4 ka0_##J, ka1_##J, kb0_##J, kb1_##J, vr0_##J, vr1_##J;
        PA_SLOT(0) PA_SLOT(1) PA_SLOT(2) PA_SLOT(3) PA_SLOT(4) PA_SLOT(5) PA_SLOT(6) PA_SLOT(7)
#undef PA_SLOT
        static_assert(SCAN_PF == 8, "the ring below is written out for 8 slots");
#define PA_LOAD_STAGE(J, ST)                                                  \
    {                                                                         \
        const size_t so_ = (size_t)min((ST), nstage - 1) * STAGE;             \
        ka0_##J = *(const uint4*)(Ka + so_);                                  \
        ka1_##J = *(const uint4*)(Ka + so_ + 32);                             \
        if (!GAMMA) {                                                         \
            kb0_##J = *(const uint4*)(Kb + so_);                              \
            kb1_##J = *(const uint4*)(Kb + so_ + 32);                         \
        }                                                                     \
        vr0_##J = *(const uint4*)(Bsrc + so_);                                \
        vr1_##J = *(const uint4*)(Bsrc + so_ + 8);                            \
    }
#define PA_HALF(J, S, KA, KB)                                                                 \
    {                                                                                         \
        Frag af_;                                                                             \
        if (!GAMMA) {                                                                         \
            const uint32_t pa_[4] = {KA.x, KA.y, KA.z, KA.w};                                 \
            const uint32_t pb_[4] = {KB.x, KB.y, KB.z, KB.w};                                 \
            _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                \
                af_.v[2 * i_] = (__bf16)(bf_lo(pa_[i_]) * bf_lo(pb_[i_]));                    \
                af_.v[2 * i_ + 1] = (__bf16)(bf_hi(pa_[i_]) * bf_hi(pb_[i_]));                \
            }                                                                                 \
        } else {                                                                              \
            af_.u = KA;                                                                       \
        }                                                                                     \
        _Pragma("unroll") for (int cb_ = 0; cb_ < 4; ++cb_) {                                 \
            Frag bf_;                                                                         \
            bf_.u = *(const uint4*)&Vs[(J) & 1][16 * cb_ + r16][32 * (S) + 8 * g];            \
            acc[cb_] = mfma16(af_.v, bf_.v, acc[cb_]);                                        \
        }                                                                                     \
    }
#define PA_CONSUME(J, ST)                                                                     \
    if ((ST) < nstage) { /* uniform; no global loads inside this branch */                    \
        const int tok0_ = (ST) * 64;                                                          \
        if (tok0_ % cs == 0) write_state(tok0_ / cs);                                         \
        *(uint4*)&Vs[(J) & 1][vcol][16 * vpiece] = vr0_##J;                                   \
        *(uint4*)&Vs[(J) & 1][vcol][16 * vpiece + 8] = vr1_##J;                               \
        lds_barrier();                                                                        \
        PA_HALF(J, 0, ka0_##J, kb0_##J)                                                       \
        PA_HALF(J, 1, ka1_##J, kb1_##J)                                                       \
    }
#define PA_STEP(J) PA_CONSUME(J, st0 + J) PA_LOAD_STAGE(J, st0 + J + SCAN_PF)
        PA_LOAD_STAGE(0, 0) PA_LOAD_STAGE(1, 1) PA_LOAD_STAGE(2, 2) PA_LOAD_STAGE(3, 3)
        PA_LOAD_STAGE(4, 4) PA_LOAD_STAGE(5, 5) PA_LOAD_STAGE(6, 6) PA_LOAD_STAGE(7, 7)
        for (int st0 = 0; st0 < nstage; st0 += SCAN_PF) {
            PA_STEP(0) PA_STEP(1) PA_STEP(2) PA_STEP(3) PA_STEP(4) PA_STEP(5) PA_STEP(6) PA_STEP(7)
        }
#undef PA_STEP
#undef PA_CONSUME
#undef PA_HALF
#undef PA_LOAD_STAGE
    }
    write_state(nstate - 1);   // tok0 = T - cs
}

__global__ __launch_bounds__(256, 2) void k_mfma_scan(const bf16_t* __restrict__ Kt, const bf16_t* __restrict__ Vt,
                                                      bf16_t* __restrict__ St, bf16_t* __restrict__ Gam, int T, int cs) {
    __shared__ __attribute__((aligned(16))) bf16_t Vs[2][DH][72];
    if (blockIdx.x == NTILES)
        scan_body<true>(Kt, Vt, St, Gam, T, cs, Vs);
    else
        scan_body<false>(Kt, Vt, St, Gam, T, cs, Vs);
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
        // ---- read-out: O^T += S_n^T phi(q)^T, 72 steps of 32 expanded rows -------------------------
        // The state of this block is one linear stream (step u = 2 tile + s holds rows a = 4s + g of
        // the tile); RO_PF steps are kept in flight in registers.
        const bf16_t* Sn = St + (size_t)(bh * nstate + n) * NTILES * TILE_ELEMS + (size_t)g * DH * 8 + r16 * 8;
        constexpr int STEP_ELEMS = 4 * DH * 8;
        Frag sf[RO_PF][4];
#pragma unroll
        for (int j = 0; j < RO_PF; ++j)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) sf[j][vb].u = *(const uint4*)(Sn + (size_t)j * STEP_ELEMS + 16 * vb * 8);
        int ti = 0, tj = 0;
        float qbv[4][8];
        for (int u0 = 0; u0 < 2 * NTILES; u0 += RO_PF) {
#pragma unroll
            for (int j = 0; j < RO_PF; ++j) {
                const int u = u0 + j;
                const int s = j & 1;
                if (s == 0) {
#pragma unroll
                    for (int ib = 0; ib < 4; ++ib) {
                        const float4 lo = *(const float4*)&Qs[64 * wv + 16 * ib + r16][8 * tj];
                        const float4 hi = *(const float4*)&Qs[64 * wv + 16 * ib + r16][8 * tj + 4];
                        qbv[ib][0] = lo.x; qbv[ib][1] = lo.y; qbv[ib][2] = lo.z; qbv[ib][3] = lo.w;
                        qbv[ib][4] = hi.x; qbv[ib][5] = hi.y; qbv[ib][6] = hi.z; qbv[ib][7] = hi.w;
                    }
                }
                Frag pf[4];
#pragma unroll
                for (int ib = 0; ib < 4; ++ib) {
                    const float qa = Qs[64 * wv + 16 * ib + r16][8 * ti + 4 * s + g];
#pragma unroll
                    for (int i = 0; i < 8; ++i) pf[ib].v[i] = (__bf16)(qa * qbv[ib][i]);
                }
#pragma unroll
                for (int vb = 0; vb < 4; ++vb)
#pragma unroll
                    for (int ib = 0; ib < 4; ++ib) acc[vb][ib] = mfma16(sf[j][vb].v, pf[ib].v, acc[vb][ib]);
                {   // unconditional (clamped) so that the compiler can count the loads in flight
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

struct Layout {
    int cs, nstate;
    size_t off_kt, off_vt, off_st, off_gam, total;
};

Layout make_layout(const pa_problem& pr, bool backward) {
    Layout L;
    L.cs = pr.chunk;
    L.nstate = pr.T / L.cs;
    const size_t BH = (size_t)pr.B * pr.H;
    size_t off = 0;
    L.off_kt = off;  off = align_up(off + BH * pr.T * DH * 2, 256);
    L.off_vt = off;  off = align_up(off + BH * pr.T * DH * 2, 256);
    L.off_st = off;  off = align_up(off + BH * L.nstate * (size_t)NTILES * TILE_ELEMS * 2, 256);
    L.off_gam = off; off = align_up(off + BH * L.nstate * (size_t)DH * DH * 2, 256);
    (void)backward;
    L.total = off;
    return L;
}

}  // namespace

pa_status mfma_supported(const pa_problem& pr, bool backward) {
    if (backward) return PA_ERR_UNSUPPORTED;
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
    bf16_t* St = (bf16_t*)(c.ws + L.off_st);
    bf16_t* Gam = (bf16_t*)(c.ws + L.off_gam);
    {
        LaunchScope ls("mfma_transpose", c.stream);
        hipLaunchKernelGGL(k_transpose, dim3(pr.T / 64, BH), dim3(256), 0, c.stream, (const bf16_t*)K, Kt, pr.T);
        hipLaunchKernelGGL(k_transpose, dim3(pr.T / 64, BH), dim3(256), 0, c.stream, (const bf16_t*)V, Vt, pr.T);
    }
    if (!launch_ok()) return PA_ERR_HIP;
    {
        LaunchScope ls("mfma_state_scan", c.stream);
        hipLaunchKernelGGL(k_mfma_scan, dim3(NTILES + 1, BH), dim3(256), 0, c.stream, Kt, Vt, St, Gam, pr.T, L.cs);
    }
    if (!launch_ok()) return PA_ERR_HIP;
    {
        LaunchScope ls("mfma_fwd_chunk", c.stream);
        hipLaunchKernelGGL(k_mfma_fwd_chunk, dim3(pr.T / QBLK, BH), dim3(128), 0, c.stream, (const bf16_t*)Q,
                           (const bf16_t*)K, Vt, St, Gam, (bf16_t*)O, Z, pr.T, L.cs, pr.scale, pr.normalize);
    }
    if (!launch_ok()) return PA_ERR_HIP;
    return PA_OK;
}

pa_status mfma_bwd(const Ctx&, const void*, const void*, const void*, const void*, const float*, const void*, void*,
                   void*, void*) {
    return PA_ERR_UNSUPPORTED;
}

}  // namespace pa
