// Shared definitions of the bf16 MFMA kernel family for degree p = 2 (gfx950, wave64).
//
// Chunked form of arXiv 2507.04239 (Sec. 2 "Chunked form", App. E) with the tiled
// symmetric-power embedding of Sec. 4.1.1 at d_tile = 8:  the expanded row (ti, tj, a, b),
// ti <= tj, of phi(x) is x[8 ti + a] * x[8 tj + b]; tiles off the diagonal carry the
// multiplicity 2, which is applied once, to the state (instead of sqrt(2) on both sides).
// Expanded operands are built in registers in MFMA operand order and never stored.
//
// MFMA used: v_mfma_f32_16x16x32_bf16.  Operand layout (lane l, r16 = l % 16, g = l / 16):
//   A: row r16,   k-slots 8g..8g+7        B: column r16, k-slots 8g..8g+7
//   C: column r16, rows 4g..4g+3 (4 floats)
// Only the pairing of A and B k-slots matters, so k-slots are assigned to whatever order
// the data is already in (no shuffles between the two MFMAs of the attention form).
//
// A 64-row state tile (bf16) is stored as [a][v][b]: the 8 expanded rows b of one (a, v) are
// contiguous, which is the MFMA operand of a contraction over rows (the read-out).  The
// contraction over v (d phi in the backward pass) reads the same copy: it stages the tile in LDS
// and lets the transposing LDS read (ds_read_b64_tr_b16) gather 8 value columns per lane.
#pragma once

#include "common.hpp"

namespace pa {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int DH = 64;                         // head size (d = v)
constexpr int NTB = DH / 8;                    // 8-wide feature blocks
constexpr int NTILES = NTB * (NTB + 1) / 2;    // 36 tiles of 64 expanded rows
constexpr int TILE_ELEMS = 8 * DH * 8;         // elements of one state tile
constexpr int STATE_ELEMS = NTILES * TILE_ELEMS;
constexpr int QBLK = 128;                      // token rows per workgroup of the chunk kernels
constexpr int TBLK = 64;                       // tokens per block of the feature-major copies

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

union Frag {
    bf16x8 v;
    uint4 u;
    u32x4 q;
    uint2 h[2];
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory,
// i.e. waits for every outstanding global load, which would drain a register prefetch ring.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(size_t)((__attribute__((address_space(3))) const void*)p);
}


// Cross-lane sums without the LDS pipe: v_permlane16_swap / v_permlane32_swap exchange 16-lane rows (resp.
// 32-lane halves) between two registers.
__device__ __forceinline__ float xor16_sum(float x) {   // x + (value in lane ^ 16), in every lane
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ void halves(float x, float& lo, float& hi) {   // lane (l & 31) of each half, in every lane
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    lo = __uint_as_float(q[0]);
    hi = __uint_as_float(q[1]);
}
__device__ __forceinline__ float xor32_sum(float x) {
    float lo, hi;
    halves(x, lo, hi);
    return lo + hi;
}
// wait until at most `n` of this wave's vector-memory operations are outstanding (they retire in order)
template <int N>
__device__ __forceinline__ void vm_wait() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 0xF) | (((N >> 4) & 0x3) << 14));
}

// ---- launchers (each defined next to its kernels) ------------------------------------------
// feature-major copy in blocks of 64 tokens: [BH][T][DH] -> [BH][T/64][DH][64]
// fac (may be null): per-token factors; the copy is then of x_t * sqrt(fac_t)
// out_T (0: T): tokens per head the output buffer is laid out for
bool launch_transpose(hipStream_t s, const bf16_t* in, bf16_t* out, int BH, int T, const float* fac = nullptr, int out_T = 0);
// state scan; rev = 0: S_n from (Kt, Vt); rev = 1: R_m from (Qt, Ght) with the weights gz.
// gam receives Gamma (rev = 0) or Omega (rev = 1).
bool launch_scan(const char* name, hipStream_t s, bool rev, const bf16_t* Xt, const bf16_t* Yt, const float* wgt, bf16_t* stC,
                 bf16_t* gam, int BH, int T, int cs, float out_scale, const float* lam = nullptr);
// `bl`, `qfac` / `kfac`: per-token gating arrays (see GateBuf), all null when not gated; gated dQ / dK kernels
// also write q_i . dq_i (qdq) and k_j . dk_j (kdk) from their float32 accumulators
// part (may be null): instead of reading the chunk state stC out, the kernel adds the nslab partial
// read-outs part[slab][bh][t][:] (float32) that launch_res_walk left
bool launch_fwd_chunk(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* Vt, const bf16_t* stC,
                      const bf16_t* gam, bf16_t* O, float* Z, int BH, int T, int cs, float scale, int normalize,
                      const float* bl, const float* qfac, const float* part = nullptr, int nslab = 0);
bool launch_bwd_prep(hipStream_t s, const bf16_t* dO, const bf16_t* O, const float* Z, bf16_t* Gh, float* gz,
                     long long rows, int normalize);
bool launch_bwd_dq(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* Gh,
                   const float* gz, const bf16_t* Kt, const bf16_t* stC, const bf16_t* gam, bf16_t* dQ, int BH, int T,
                   int cs, float scale, const float* bl, const float* qfac, float* qdq);
bool launch_bwd_dkdv(hipStream_t s, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* Gh, const float* gz,
                     const bf16_t* Qt, const bf16_t* Ght, const bf16_t* rtC, const bf16_t* omg, bf16_t* dK, bf16_t* dV, int BH,
                     int T, int cs, float scale, const float* bl, const float* kfac, float* kdk);

// ---- resident-state kernels (chunk states kept in registers; see mfma_resident.hip) ----------------
struct ResidentPlan {
    int nhp, nslab;            // half-pairs per wave; workgroups (slabs of state rows) per head
    int nseg, seg_chunks;      // segments the sequence is cut into, chunks per segment
    size_t acc_floats;         // accumulator floats per wave
    size_t tot_bytes, part_bytes, gram_bytes;   // per-segment totals; per-slab partial read-outs; per-chunk Gram matrices
};
ResidentPlan resident_plan(int HD, int BH, int T, int cs);
// One pass over the sequence with the state in registers.  readout = false: every segment but the last
// adds up its own total into `tot`.  readout = true: each segment starts from the totals before it and
// writes, per slab, part[slab][bh][t][:] = (state entering t's chunk)^T phi(Qr_t) * snap_scale.
// rev: the state holds the chunks after the current one (state gradient).
// mode 2 (d phi): part[slab][bh][t][:] = J_phi(Qr_t)^T (state . Gr_t) * snap_scale, Gr the token-major rows the state's
// value columns are contracted with
bool launch_res_walk(const char* name, hipStream_t s, int HD, bool rev, int mode, const bf16_t* Xt, const bf16_t* Yt,
                     const bf16_t* Qr, const bf16_t* Gr, float* tot, float* part, int BH, int T, int cs, const ResidentPlan& pl,
                     float snap_scale);
// out[bh][n] (bf16, HD x HD) = out_scale * sum over the chunks before (rev: after) n of sum_t w_t x_t x_t^T;
// gram: float32 scratch [BH][T / cs][HD][HD]; wgt may be null (w = 1)
bool launch_gram(hipStream_t s, int HD, const bf16_t* Xt, const float* wgt, float* gram, bf16_t* out, int BH, int T, int cs,
                 bool rev, float out_scale);

// feature-major copy in blocks of 64 tokens for any head size the resident kernels take
bool launch_transpose_hd(hipStream_t s, int HD, const bf16_t* in, bf16_t* out, int BH, int T);
// normaliser terms per token from the HD x HD states gam[bh][T / cs]: vec[bh][t][:] = cvec * wgt_t * G x_t (float32),
// sca[bh][t] = csca * x_t^T G x_t; vec, sca and wgt may each be null
bool launch_gram_apply(hipStream_t s, int HD, const bf16_t* X, const bf16_t* gam, const float* wgt, float* vec, float* sca,
                       int BH, int T, int cs, float cvec, float csca);

// ---- chunked form for any degree and tile width (state kept in memory; see mfma_tiled.hip) -------------
// One tile of the tiled symmetric-power embedding: its p block indices (non-decreasing) and its multiplicity
struct TileDesc {
    unsigned char t[4];
    float mult;
};
struct TiledPlan {
    int p, dt, hd, vp;            // degree, tile width, head size, value columns of a state row (hd + 16)
    int ntile, rows_per_tile;     // tiles of the embedding, dt^p rows each
    int nunit_real, nunit;        // 64-row units that hold state, and the count the layout is padded to (a multiple of 4)
    int nentry;                   // entries of the tile table (padding entries have multiplicity 0)
    size_t state_elems;           // bf16 elements of one (head, chunk) state
};
bool tiled_shape_ok(int p, int d, int dt);
int tiled_default_dt(int p);
TiledPlan tiled_plan(int p, int d, int dt);
bool launch_tiled_table(hipStream_t s, const TiledPlan& pl, TileDesc* tab);
// Yp[row] = [Y[row] (hd values), col[row] (1 when col is null), 15 zeros], bf16
bool launch_tiled_pack(hipStream_t s, int hd, const bf16_t* Y, const float* col, bf16_t* Yp, long long rows);
// st[bh][c] = multiplicity x sum over the chunks before c (rev: after c) of phi(xscale X_t) Yp_t^T
bool launch_tiled_scan(const char* name, hipStream_t s, const TiledPlan& pl, bool rev, const bf16_t* X, const bf16_t* Yp,
                       const TileDesc* tab, bf16_t* st, int BH, int T, int cs, float xscale);
// part[bh][t][:] = (state of t's chunk)^T phi(xscale X_t), columns 0 .. hd - 1; zpart[bh][t] (may be null) = column hd
bool launch_tiled_readout(const char* name, hipStream_t s, const TiledPlan& pl, const bf16_t* X, const TileDesc* tab, const bf16_t* st,
                          float* part, float* zpart, int BH, int T, int cs, float xscale);
// part[bh][t][:] = outscale J_phi(xscale X_t)^T (state of t's chunk . Yp_t)
bool launch_tiled_dphi(const char* name, hipStream_t s, const TiledPlan& pl, const bf16_t* X, const bf16_t* Yp, const TileDesc* tab,
                       const bf16_t* st, float* part, int BH, int T, int cs, float xscale, float outscale);

// gating: xb[bh][n] = the sum over the pairs that straddle the end of chunk n, from the stored states
bool launch_gate_boundary(hipStream_t s, const bf16_t* stC, const bf16_t* rtC, const bf16_t* gam, const bf16_t* omg, float* xb,
                          int BH, int nstate);

// attention form (chunk == T): p in {2, 3, 4}, d = v in {32, 64, 128}, any T.
// Gh [BH][T][d] bf16 and gz [BH][T] float32 are scratch of the backward pass.
bool attn_shape_ok(int p, int d);
// bl (null when not gated): [BH][T] running sums of the log-gates from the start of the sequence
bool launch_attn_fwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, bf16_t* O, float* Z, int BH,
                     int T, float scale, int normalize, const float* bl = nullptr);
// The in-chunk part of the chunked form on the attention-form kernels (keys of the query's own chunk of cs
// tokens), plus what came through the state: part[slab][BH][T][d] (float32, nslab slabs) joins the numerator,
// zpart[BH][T] the denominator
bool launch_chunk_fwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, bf16_t* O, float* Z, int BH,
                      int T, int cs, float scale, int normalize, const float* part, int nslab, const float* zpart);
// ghat = dO / Z (bf16) and gz = -(ghat . O) (float32) per token, d in {32, 64, 128}
bool launch_attn_prep(hipStream_t s, int d, const bf16_t* dO, const bf16_t* O, const float* Z, bf16_t* Gh, float* gz, long long rows,
                      int normalize);
// backward of the same: the in-chunk gradients plus the per-slab parts that came through the states (float32
// [slab][BH][T][d]; the slab counts include the normaliser's slab where there is one)
bool launch_chunk_bwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* Gh,
                      const float* gz, bf16_t* dQ, bf16_t* dK, bf16_t* dV, int BH, int T, int cs, float scale, const float* part_dq,
                      int nslab_dq, const float* part_dk, int nslab_dk, const float* part_dv, int nslab_dv);
// Gated backward pass (bl non-null; T a multiple of attn_gate_block(d)): also leaves what the gradient of
// the log-gates needs: qdq [BH][T] = q_i . dq_i, kdk [BH][T] = k_j . dk_j (from float32 accumulators) and
// xb [BH][T / block] = the sum of e_ij a_ij over the pairs j <= end of block m < i.
// wsum: scratch, BH * (T / block)^2 * 4 floats.
struct AttnGate {
    const float* bl = nullptr;
    float *qdq = nullptr, *kdk = nullptr, *xb = nullptr, *wsum = nullptr;
};
int attn_gate_block(int d);
bool launch_attn_bwd(hipStream_t s, int p, int d, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* O,
                     const float* Z, const bf16_t* dO, bf16_t* Gh, float* gz, bf16_t* dQ, bf16_t* dK, bf16_t* dV, int BH, int T,
                     float scale, int normalize, const AttnGate& gate = AttnGate());

}  // namespace mfma
}  // namespace pa
