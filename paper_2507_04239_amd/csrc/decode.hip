// Single-token decode step of power attention: the recurrent form of arXiv 2507.04239, Sec. 2
// Eq. (6), one iteration per call with the state resident in device memory between calls
// (the constant-cost inference the paper argues for in App. D):
//     S <- g S + phi(k) [v, 1]^T,      y = S^T phi(scale q),      o = y[:v] / y[v].
//
// Embedding as in the generic kernel family: the monomials psi(x)_r = prod_z x[i_z] over the
// non-decreasing multi-indices of Lemma 4.2, with the integer multiplicity m_r on the state only
// (S_r = sum m_r psi(k)_r [v, 1]), read out with the bare psi(q): the product is (q.k)^p.
//
// The state is float32 and caller-owned; one buffer per problem holds
//     S     [B*H][D][v]     the value part
//     gamma [B*H][D]        the normaliser column
//     idx   [D] uchar4, mult [D] float   the multi-index table (built by decode_init)
//     part  [B*H][nblk][v+1]             partial read-outs of the step in flight
// A step reads and writes S and gamma once: it is bound by HBM bandwidth, 8 bytes per state
// element and token.
#include "common.hpp"

namespace pa {
namespace {

constexpr int DRB = 128;   // state rows per workgroup
constexpr int DMAX = 128;  // largest head size

template <int P>
__device__ __forceinline__ float monomial(const float* __restrict__ x, uchar4 ix) {
    float c = x[ix.x];
    if (P > 1) c *= x[ix.y];
    if (P > 2) c *= x[ix.z];
    if (P > 3) c *= x[ix.w];
    return c;
}

struct DecodeLayout {
    long long D;
    int nblk;
    size_t off_s, off_gam, off_idx, off_mult, off_part, total;
};

DecodeLayout make_decode_layout(const pa_problem& pr) {
    DecodeLayout L;
    L.D = generic_state_rows(pr);
    L.nblk = (int)((L.D + DRB - 1) / DRB);
    const size_t BH = (size_t)pr.B * pr.H;
    size_t off = 0;
    L.off_s = off;    off = align_up(off + BH * (size_t)L.D * pr.v * sizeof(float), 256);
    L.off_gam = off;  off = align_up(off + BH * (size_t)L.D * sizeof(float), 256);
    L.off_idx = off;  off = align_up(off + (size_t)L.D * sizeof(uchar4), 256);
    L.off_mult = off; off = align_up(off + (size_t)L.D * sizeof(float), 256);
    L.off_part = off; off = align_up(off + BH * (size_t)L.nblk * (pr.v + 1) * sizeof(float), 256);
    L.total = off;
    return L;
}

__global__ __launch_bounds__(256) void k_decode_zero(float4* __restrict__ p, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// grid (nblk, B*H): rows [DRB blk, DRB (blk + 1)) of one head's state.  A wave takes one row at
// a time (its lanes the value columns: 256-byte runs), then the block's rows of the normaliser
// column go one per thread.
template <typename T, int P>
__global__ __launch_bounds__(256) void k_decode_step(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ vin,
                                                     const float* __restrict__ log_g, float* __restrict__ S,
                                                     float* __restrict__ gam, const uchar4* __restrict__ idx,
                                                     const float* __restrict__ mult, float* __restrict__ part, long long D,
                                                     int d, int v, float scale) {
    __shared__ float qs[DMAX], ks[DMAX], vs[DMAX];
    __shared__ float red[4][DMAX + 1];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int blk = blockIdx.x, bh = blockIdx.y, nblk = gridDim.x;
    if (tid < d) {
        qs[tid] = scale * io<T>::ld(q + (size_t)bh * d + tid);
        ks[tid] = io<T>::ld(k + (size_t)bh * d + tid);
    }
    if (tid < v) vs[tid] = io<T>::ld(vin + (size_t)bh * v + tid);
    const float g = log_g != nullptr ? __expf(log_g[bh]) : 1.f;
    __syncthreads();

    const long long r_begin = (long long)blk * DRB;
    const long long r_end = r_begin + DRB < D ? r_begin + DRB : D;
    float y0 = 0.f, y1 = 0.f;
    const float v0 = lane < v ? vs[lane] : 0.f, v1 = lane + 64 < v ? vs[lane + 64] : 0.f;
    for (long long r = r_begin + w; r < r_end; r += 4) {
        const uchar4 ix = idx[r];
        const float ck = mult[r] * monomial<P>(ks, ix), cq = monomial<P>(qs, ix);
        float* row = S + ((size_t)bh * D + r) * v;
        if (lane < v) {
            const float s = g * row[lane] + ck * v0;
            row[lane] = s;
            y0 += cq * s;
        }
        if (lane + 64 < v) {
            const float s = g * row[lane + 64] + ck * v1;
            row[lane + 64] = s;
            y1 += cq * s;
        }
    }
    float zp = 0.f;
    for (long long r = r_begin + tid; r < r_end; r += 256) {
        const uchar4 ix = idx[r];
        const float ck = mult[r] * monomial<P>(ks, ix), cq = monomial<P>(qs, ix);
        const float s = g * gam[(size_t)bh * D + r] + ck;
        gam[(size_t)bh * D + r] = s;
        zp += cq * s;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) zp += __shfl_xor(zp, off);
    red[w][lane] = y0;
    red[w][lane + 64] = y1;
    if (lane == 0) red[w][DMAX] = zp;
    __syncthreads();
    if (tid <= v) {
        const int c = tid < v ? tid : DMAX;
        part[((size_t)bh * nblk + blk) * (v + 1) + tid] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
    }
}

// The same for v in {4, 8, ..., 128} (a power of two): v / 4 lanes share a row, each with four
// columns (16-byte accesses), so a wave has 256 / v rows in flight per pass and two passes
// unrolled - the row-at-a-time kernel above leaves the memory system mostly idle.
template <typename T, int P, int V>
__global__ __launch_bounds__(256) void k_decode_step_vec(const T* __restrict__ q, const T* __restrict__ k,
                                                         const T* __restrict__ vin, const float* __restrict__ log_g,
                                                         float* __restrict__ S, float* __restrict__ gam,
                                                         const uchar4* __restrict__ idx, const float* __restrict__ mult,
                                                         float* __restrict__ part, long long D, int d, float scale) {
    constexpr int LPR = V / 4, RPW = 64 / LPR, RPB = 4 * RPW;   // lanes per row, rows per wave and per block pass
    __shared__ float qs[DMAX], ks[DMAX];
    __shared__ __attribute__((aligned(16))) float vs[DMAX];
    __shared__ __attribute__((aligned(16))) float red[4][DMAX + 4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int blk = blockIdx.x, bh = blockIdx.y, nblk = gridDim.x;
    if (tid < d) {
        qs[tid] = scale * io<T>::ld(q + (size_t)bh * d + tid);
        ks[tid] = io<T>::ld(k + (size_t)bh * d + tid);
    }
    if (tid < V) vs[tid] = io<T>::ld(vin + (size_t)bh * V + tid);
    const float g = log_g != nullptr ? __expf(log_g[bh]) : 1.f;
    __syncthreads();

    const long long r_begin = (long long)blk * DRB;
    const long long r_end = r_begin + DRB < D ? r_begin + DRB : D;
    const int c4 = lane % LPR, rl = w * RPW + lane / LPR;        // column quad, row inside a block pass
    const float4 vv = *(const float4*)&vs[4 * c4];
    float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
    static_assert(DRB % (2 * RPB) == 0 || RPB > DRB / 2, "two passes per trip");
    for (long long r0 = r_begin; r0 < r_end; r0 += 2 * RPB) {
        const long long ra = r0 + rl, rb = r0 + RPB + rl;
        const bool oka = ra < r_end, okb = rb < r_end;
        float4* pa = (float4*)(S + ((size_t)bh * D + (oka ? ra : r_begin)) * V) + c4;
        float4* pb = (float4*)(S + ((size_t)bh * D + (okb ? rb : r_begin)) * V) + c4;
        const float4 sa = *pa, sb = *pb;
        const uchar4 ia = idx[oka ? ra : r_begin], ib = idx[okb ? rb : r_begin];
        const float cka = mult[oka ? ra : r_begin] * monomial<P>(ks, ia), cqa = oka ? monomial<P>(qs, ia) : 0.f;
        const float ckb = mult[okb ? rb : r_begin] * monomial<P>(ks, ib), cqb = okb ? monomial<P>(qs, ib) : 0.f;
        const float4 na = make_float4(g * sa.x + cka * vv.x, g * sa.y + cka * vv.y, g * sa.z + cka * vv.z, g * sa.w + cka * vv.w);
        const float4 nb = make_float4(g * sb.x + ckb * vv.x, g * sb.y + ckb * vv.y, g * sb.z + ckb * vv.z, g * sb.w + ckb * vv.w);
        if (oka) *pa = na;
        if (okb) *pb = nb;
        y.x += cqa * na.x + cqb * nb.x;
        y.y += cqa * na.y + cqb * nb.y;
        y.z += cqa * na.z + cqb * nb.z;
        y.w += cqa * na.w + cqb * nb.w;
    }
    float zp = 0.f;
    for (long long r = r_begin + tid; r < r_end; r += 256) {
        const uchar4 ix = idx[r];
        const float ck = mult[r] * monomial<P>(ks, ix), cq = monomial<P>(qs, ix);
        const float s = g * gam[(size_t)bh * D + r] + ck;
        gam[(size_t)bh * D + r] = s;
        zp += cq * s;
    }
    // rows of a wave: lanes LPR apart hold the same columns
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        y.x += __shfl_xor(y.x, off);
        y.y += __shfl_xor(y.y, off);
        y.z += __shfl_xor(y.z, off);
        y.w += __shfl_xor(y.w, off);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) zp += __shfl_xor(zp, off);
    if (lane < LPR) *(float4*)&red[w][4 * lane] = y;
    if (lane == 0) red[w][DMAX] = zp;
    __syncthreads();
    if (tid <= V) {
        const int c = tid < V ? tid : DMAX;
        part[((size_t)bh * nblk + blk) * (V + 1) + tid] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
    }
}

// ---- absorbing a whole prompt ------------------------------------------------------------------------
// S <- (prod of the prompt's gates) S + sum_t (prod of the gates after t) m_r psi(k_t)_r [v_t, 1], i.e. the
// state after stepping through K, V [B*H][Tlen][.] token by token, without producing outputs (those come
// from power_attn_fwd).  One thread owns a state row and every fourth column, holds them in registers
// and walks the tokens, which are staged through LDS 32 at a time; the decay is applied token by
// token (acc <- g_t acc + ...), which needs no running sums of the log-gates.
constexpr int ART = 32;   // tokens per LDS batch
// NQ: column quads per thread (thread xg of a row's four owns the quads xg, xg + 4, ...: 16-byte LDS
// reads); the normaliser column rides with thread 0 of the four.
template <typename T, int P, int NQ, bool GATED>
__global__ __launch_bounds__(256) void k_decode_absorb(const T* __restrict__ K, const T* __restrict__ V,
                                                       const float* __restrict__ log_g, float* __restrict__ S,
                                                       float* __restrict__ gam, const uchar4* __restrict__ idx,
                                                       const float* __restrict__ mult, long long D, int Tlen, int d, int v) {
    __shared__ float ks[ART][DMAX];
    __shared__ __attribute__((aligned(16))) float vs[ART][DMAX];
    __shared__ float gs[ART];
    const int tid = threadIdx.x, xg = tid & 3, bh = blockIdx.y;
    const long long row = (long long)blockIdx.x * 64 + (tid >> 2);
    const bool live = row < D;
    uchar4 ix = make_uchar4(0, 0, 0, 0);
    float m = 0.f;
    if (live) {
        ix = idx[row];
        m = mult[row];
    }
    float* srow = S + ((size_t)bh * D + (live ? row : 0)) * v;
    float* grow = gam + (size_t)bh * D + (live ? row : 0);
    const int nquad = (v + 3) / 4;
    float4 acc[NQ];
    float accz = live && xg == 0 ? *grow : 0.f;
#pragma unroll
    for (int kk = 0; kk < NQ; ++kk) {
        const int x = 4 * (xg + 4 * kk);
        acc[kk] = make_float4(live && x < v ? srow[x] : 0.f, live && x + 1 < v ? srow[x + 1] : 0.f,
                              live && x + 2 < v ? srow[x + 2] : 0.f, live && x + 3 < v ? srow[x + 3] : 0.f);
    }
    const T* Kb = K + (size_t)bh * Tlen * d;
    const T* Vb = V + (size_t)bh * Tlen * v;
    for (int t0 = 0; t0 < Tlen; t0 += ART) {
        const int nt = min(ART, Tlen - t0);
        __syncthreads();
        for (int e = tid; e < nt * d; e += 256) ks[e / d][e % d] = io<T>::ld(Kb + (size_t)t0 * d + e);
        for (int e = tid; e < nt * 4 * nquad; e += 256) {        // columns past v read as zero
            const int j = e / (4 * nquad), x = e % (4 * nquad);
            vs[j][x] = x < v ? io<T>::ld(Vb + (size_t)(t0 + j) * v + x) : 0.f;
        }
        if (GATED && tid < nt) gs[tid] = __expf(log_g[(size_t)bh * Tlen + t0 + tid]);
        __syncthreads();
#pragma unroll 4
        for (int j = 0; j < nt; ++j) {
            const float coef = m * monomial<P>(ks[j], ix);
            const float g = GATED ? gs[j] : 1.f;
            accz = GATED ? g * accz + coef : accz + coef;
#pragma unroll
            for (int kk = 0; kk < NQ; ++kk) {
                if (xg + 4 * kk < nquad) {
                    const float4 y = *(const float4*)&vs[j][4 * (xg + 4 * kk)];
                    if (GATED) {
                        acc[kk].x *= g; acc[kk].y *= g; acc[kk].z *= g; acc[kk].w *= g;
                    }
                    acc[kk].x += coef * y.x; acc[kk].y += coef * y.y; acc[kk].z += coef * y.z; acc[kk].w += coef * y.w;
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int kk = 0; kk < NQ; ++kk) {
        const int x = 4 * (xg + 4 * kk);
        if (x < v) srow[x] = acc[kk].x;
        if (x + 1 < v) srow[x + 1] = acc[kk].y;
        if (x + 2 < v) srow[x + 2] = acc[kk].z;
        if (x + 3 < v) srow[x + 3] = acc[kk].w;
    }
    if (xg == 0) *grow = accz;
}

// grid B*H: sums the blocks' partial read-outs, divides, stores
template <typename T>
__global__ __launch_bounds__(256) void k_decode_finish(const float* __restrict__ part, int nblk, T* __restrict__ o,
                                                       float* __restrict__ z, int v, int normalize) {
    __shared__ float zs;
    const int bh = blockIdx.x, tid = threadIdx.x;
    float acc = 0.f;
    if (tid <= v)
        for (int b = 0; b < nblk; ++b) acc += part[((size_t)bh * nblk + b) * (v + 1) + tid];
    if (tid == v) zs = acc;
    __syncthreads();
    const float zz = zs;
    if (tid < v) {
        const float inv = normalize ? (zz != 0.f ? 1.f / zz : 0.f) : 1.f;
        io<T>::st(o + (size_t)bh * v + tid, acc * inv);
    }
    if (tid == v && z != nullptr) z[bh] = zz;
}

pa_status decode_supported(const pa_problem& pr) {
    if (pr.p < 1 || pr.p > 4 || pr.d > DMAX || pr.v > DMAX) return PA_ERR_UNSUPPORTED;
    if ((size_t)pr.B * pr.H > 65535u) return PA_ERR_UNSUPPORTED;
    return PA_OK;
}

template <typename T, int P>
bool launch_step(const pa_problem& pr, const DecodeLayout& L, const void* q, const void* k, const void* v, const float* log_g,
                 char* st, void* o, float* z, hipStream_t s) {
    const int BH = pr.B * pr.H;
    {
        LaunchScope ls("decode_step", s);
#define PA_VEC(VV)                                                                                                          \
    if (pr.v == VV)                                                                                                         \
        hipLaunchKernelGGL((k_decode_step_vec<T, P, VV>), dim3(L.nblk, BH), dim3(256), 0, s, (const T*)q, (const T*)k,      \
                           (const T*)v, log_g, (float*)(st + L.off_s), (float*)(st + L.off_gam),                            \
                           (const uchar4*)(st + L.off_idx), (const float*)(st + L.off_mult), (float*)(st + L.off_part), L.D, \
                           pr.d, pr.scale);                                                                                 \
    else
        PA_VEC(16) PA_VEC(32) PA_VEC(64) PA_VEC(128)
#undef PA_VEC
        hipLaunchKernelGGL((k_decode_step<T, P>), dim3(L.nblk, BH), dim3(256), 0, s, (const T*)q, (const T*)k, (const T*)v, log_g,
                           (float*)(st + L.off_s), (float*)(st + L.off_gam), (const uchar4*)(st + L.off_idx),
                           (const float*)(st + L.off_mult), (float*)(st + L.off_part), L.D, pr.d, pr.v, pr.scale);
        if (!launch_ok()) return false;
    }
    LaunchScope ls("decode_finish", s);
    hipLaunchKernelGGL((k_decode_finish<T>), dim3(BH), dim3(256), 0, s, (const float*)(st + L.off_part), L.nblk, (T*)o, z, pr.v,
                       pr.normalize);
    return launch_ok();
}

template <typename T>
bool launch_step_p(const pa_problem& pr, const DecodeLayout& L, const void* q, const void* k, const void* v, const float* log_g,
                   char* st, void* o, float* z, hipStream_t s) {
    switch (pr.p) {
        case 1: return launch_step<T, 1>(pr, L, q, k, v, log_g, st, o, z, s);
        case 2: return launch_step<T, 2>(pr, L, q, k, v, log_g, st, o, z, s);
        case 3: return launch_step<T, 3>(pr, L, q, k, v, log_g, st, o, z, s);
        default: return launch_step<T, 4>(pr, L, q, k, v, log_g, st, o, z, s);
    }
}

template <typename T, int P>
bool launch_absorb_kx(const pa_problem& pr, const DecodeLayout& L, const void* K, const void* V, const float* log_g, char* st,
                      hipStream_t s) {
    const int nq = ((pr.v + 3) / 4 + 3) / 4;      // column quads per thread
    const dim3 grid((unsigned)((L.D + 63) / 64), pr.B * pr.H);
    LaunchScope ls("decode_absorb", s);
#define PA_GO(NQ, G)                                                                                                    \
    hipLaunchKernelGGL((k_decode_absorb<T, P, NQ, G>), grid, dim3(256), 0, s, (const T*)K, (const T*)V, log_g,           \
                       (float*)(st + L.off_s), (float*)(st + L.off_gam), (const uchar4*)(st + L.off_idx),                \
                       (const float*)(st + L.off_mult), L.D, pr.T, pr.d, pr.v)
    if (log_g != nullptr) {
        if (nq <= 1) PA_GO(1, true);
        else if (nq <= 2) PA_GO(2, true);
        else if (nq <= 4) PA_GO(4, true);
        else PA_GO(8, true);
    } else {
        if (nq <= 1) PA_GO(1, false);
        else if (nq <= 2) PA_GO(2, false);
        else if (nq <= 4) PA_GO(4, false);
        else PA_GO(8, false);
    }
#undef PA_GO
    return launch_ok();
}

template <typename T>
bool launch_absorb_p(const pa_problem& pr, const DecodeLayout& L, const void* K, const void* V, const float* log_g, char* st,
                     hipStream_t s) {
    switch (pr.p) {
        case 1: return launch_absorb_kx<T, 1>(pr, L, K, V, log_g, st, s);
        case 2: return launch_absorb_kx<T, 2>(pr, L, K, V, log_g, st, s);
        case 3: return launch_absorb_kx<T, 3>(pr, L, K, V, log_g, st, s);
        default: return launch_absorb_kx<T, 4>(pr, L, K, V, log_g, st, s);
    }
}

}  // namespace

size_t decode_absorb_workspace_bytes(const pa_problem& pr) {
    return decode_supported(pr) == PA_OK ? mfma_absorb_workspace_bytes(pr) : 0;
}

// With a workspace, and where the matrix-core scan applies, the prompt goes through that (the sums are then
// rounded to bf16 once, like the chunk states of the forward pass); else through the float32 kernel above.
pa_status decode_absorb(const pa_problem& pr, const void* K, const void* V, const float* log_g, void* state, void* ws,
                        size_t ws_bytes, hipStream_t s) {
    pa_status st = decode_supported(pr);
    if (st != PA_OK) return st;
    const DecodeLayout L = make_decode_layout(pr);
    if (ws != nullptr && mfma_absorb_supported(pr) && ws_bytes >= mfma_absorb_workspace_bytes(pr))
        return mfma_absorb(pr, K, V, log_g, (char*)ws, s, (float*)((char*)state + L.off_s), (float*)((char*)state + L.off_gam),
                           (int)L.D);
    const bool ok = pr.dtype == PA_DTYPE_F32 ? launch_absorb_p<float>(pr, L, K, V, log_g, (char*)state, s)
                                             : launch_absorb_p<bf16_t>(pr, L, K, V, log_g, (char*)state, s);
    return ok ? PA_OK : PA_ERR_HIP;
}

size_t decode_state_bytes(const pa_problem& pr) { return decode_supported(pr) == PA_OK ? make_decode_layout(pr).total : 0; }

pa_status decode_init(const pa_problem& pr, void* state, hipStream_t s) {
    pa_status st = decode_supported(pr);
    if (st != PA_OK) return st;
    const DecodeLayout L = make_decode_layout(pr);
    {
        // a kernel, not a memset: the call may be recorded into a graph
        LaunchScope ls("decode_zero", s);
        const size_t n4 = L.off_idx / sizeof(float4);     // S and gamma, both padded to 256 bytes
        hipLaunchKernelGGL(k_decode_zero, dim3(1024), dim3(256), 0, s, (float4*)state, n4);
        if (!launch_ok()) return PA_ERR_HIP;
    }
    char* base = (char*)state;
    return build_monomial_table(s, pr.d, pr.p, L.D, base + L.off_idx, (float*)(base + L.off_mult)) ? PA_OK : PA_ERR_HIP;
}

pa_status decode_step(const pa_problem& pr, const void* q, const void* k, const void* v, const float* log_g, void* state, void* o,
                      float* z, hipStream_t s) {
    pa_status st = decode_supported(pr);
    if (st != PA_OK) return st;
    const DecodeLayout L = make_decode_layout(pr);
    const bool ok = pr.dtype == PA_DTYPE_F32 ? launch_step_p<float>(pr, L, q, k, v, log_g, (char*)state, o, z, s)
                                             : launch_step_p<bf16_t>(pr, L, q, k, v, log_g, (char*)state, o, z, s);
    return ok ? PA_OK : PA_ERR_HIP;
}

}  // namespace pa
