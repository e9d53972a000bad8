// Generic kernel family: chunked power attention in float32 on the vector ALUs.
//
// Any degree 1 <= p <= 4 and head sizes up to 128, float32 or bf16 storage.  It is the
// float32 path of the library and the fallback for shapes the MFMA family does not
// cover.  The structure is the chunked form of arXiv 2507.04239 (Sec. 2 "Chunked form",
// App. E): a fused update-state + cumulative sum over chunks (App. E.2, E.3), and a
// per-chunk kernel doing the intra-chunk attention form (App. E.1) plus the query-state
// read-out and normalisation (App. E.4).
//
// Embedding: the monomials psi(x)_r = prod_z x[i_z] over the non-decreasing multi-indices
// r = (i_1 <= ... <= i_p) of Lemma 4.2 in lexicographic order.  Instead of the square root
// of the multiplicity on both sides, the integer multiplicity m_r = p!/prod hist! is put on
// the state only:  S = sum_j m_r psi(k_j)_r [v_j,1],  read out with the bare psi(q).  The
// product is the same (q.k)^p and no irrational constant is needed.
#include "common.hpp"

namespace pa {
namespace {

constexpr int NT = 256;    // threads per block
constexpr int TOK = 64;    // tokens per pass in the per-chunk kernels (NT / 4)
constexpr int RT = 32;     // state rows (and tokens) staged per LDS tile
constexpr int PMAX = 4;

// number of non-decreasing sequences of length m over an alphabet of a symbols: C(a+m-1, m)
__host__ __device__ inline unsigned long long ndmi_count(int a, int m) {
    if (m == 0) return 1ull;
    if (a <= 0) return 0ull;
    unsigned long long r = 1ull;
    for (int i = 1; i <= m; ++i) r = r * (unsigned long long)(a - 1 + i) / (unsigned long long)i;
    return r;
}

// Row r of the lexicographic list of non-decreasing multi-indices -> its p indices (padded
// with 0) and its multiplicity p!/prod(run lengths)!.
__global__ void k_build_table(int d, int p, long long D, uchar4* __restrict__ idx, float* __restrict__ mult) {
    long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= D) return;
    unsigned long long rem = (unsigned long long)r;
    int out[PMAX] = {0, 0, 0, 0};
    int prev = 0;
    for (int z = 0; z < p; ++z) {
        int m = p - 1 - z;
        int a = prev;
        for (; a < d - 1; ++a) {
            unsigned long long cnt = ndmi_count(d - a, m);
            if (rem < cnt) break;
            rem -= cnt;
        }
        out[z] = a;
        prev = a;
    }
    int fact[PMAX + 1] = {1, 1, 2, 6, 24};
    int mlt = fact[p];
    int run = 1;
    for (int z = 1; z <= p; ++z) {
        if (z < p && out[z] == out[z - 1]) {
            ++run;
        } else {
            mlt /= fact[run];
            run = 1;
        }
    }
    idx[r] = make_uchar4((unsigned char)out[0], (unsigned char)out[1], (unsigned char)out[2], (unsigned char)out[3]);
    mult[r] = (float)mlt;
}

template <int P>
__device__ __forceinline__ float monomial(const float* __restrict__ x, uchar4 ix) {
    float c = x[ix.x];
    if (P > 1) c *= x[ix.y];
    if (P > 2) c *= x[ix.z];
    if (P > 3) c *= x[ix.w];
    return c;
}

// product of the entries at every position except z
template <int P>
__device__ __forceinline__ float monomial_without(const float* __restrict__ x, uchar4 ix, int z) {
    float c = 1.f;
    if (z != 0) c *= x[ix.x];
    if (P > 1 && z != 1) c *= x[ix.y];
    if (P > 2 && z != 2) c *= x[ix.z];
    if (P > 3 && z != 3) c *= x[ix.w];
    return c;
}

__device__ __forceinline__ int index_at(uchar4 ix, int z) { return z == 0 ? ix.x : z == 1 ? ix.y : z == 2 ? ix.z : ix.w; }

template <int P>
__device__ __forceinline__ float ipow(float s) {
    float w = s;
#pragma unroll
    for (int i = 1; i < P; ++i) w *= s;
    return w;
}
template <int P>
__device__ __forceinline__ float ipow_m1(float s) {  // s^(P-1)
    float w = 1.f;
#pragma unroll
    for (int i = 1; i < P; ++i) w *= s;
    return w;
}

__device__ __forceinline__ float quad_sum(float x) {  // sum over the 4 adjacent lanes of a token
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    return x;
}

// ---- elementwise preparation ------------------------------------------------------------

// V' = [V, 1] widened to float32: [rows, VP]
template <typename T>
__global__ void k_prep_v(const T* __restrict__ V, float* __restrict__ Vp, long long rows, int v) {
    const int VP = v + 1;
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = rows * VP;
    if (i >= total) return;
    long long row = i / VP;
    int x = (int)(i - row * VP);
    Vp[i] = x < v ? io<T>::ld(V + row * v + x) : 1.f;
}

// ghat' = [dO / Z, -(dO . O) / Z]  (normalised) or [dO, 0]; rows with Z == 0 give zeros
template <typename T>
__global__ void k_prep_g(const T* __restrict__ dO, const T* __restrict__ O, const float* __restrict__ Z,
                         float* __restrict__ Gp, long long rows, int v, int normalize) {
    const int VP = v + 1;
    long long row = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const T* g = dO + row * v;
    float* out = Gp + row * VP;
    if (!normalize) {
        for (int x = 0; x < v; ++x) out[x] = io<T>::ld(g + x);
        out[v] = 0.f;
        return;
    }
    float z = Z[row];
    float inv = z != 0.f ? 1.f / z : 0.f;
    const T* o = O + row * v;
    float delta = 0.f;
    for (int x = 0; x < v; ++x) {
        float gx = io<T>::ld(g + x);
        delta += gx * io<T>::ld(o + x);
        out[x] = gx * inv;
    }
    out[v] = -delta * inv;
}

// ---- fused update-state + cumulative sum over chunks (App. E.2 + E.3) ---------------------
//
// St[bh][n] = sum over the chunks before n (reverse: after n) of  m_r psi(xscale * X_j)_r Yp_j^T.
// One thread owns (row r, columns x = xg, xg+4, ...) and walks the chunks in order, writing
// the running sum before it adds the chunk.  Gated (fac, lam non-null): token j enters with the
// weight fac_j and the running sum is multiplied by lam_n before chunk n is added, i.e. the
// gated update-state S <- S * gamma + phi(K)^T V and the discounted cumulative sum.
template <typename T, int P, int KX>
__global__ __launch_bounds__(NT) void k_scan(const T* __restrict__ X, const float* __restrict__ Yp,
                                             const uchar4* __restrict__ idx, const float* __restrict__ mult,
                                             float* __restrict__ St, int Tlen, int d, int VP, int chunk, long long D,
                                             float xscale, int reverse, const float* __restrict__ fac,
                                             const float* __restrict__ lam) {
    extern __shared__ float smem[];
    float* xs = smem;            // [RT][d]
    float* ys = smem + RT * d;   // [RT][VP]
    float* fs = ys + RT * VP;    // [RT]      per-token weights (gated)
    const int tid = threadIdx.x;
    const int xg = tid & 3;
    const long long row = (long long)blockIdx.x * (NT / 4) + (tid >> 2);
    const int bh = blockIdx.y;
    const int nchunk = Tlen / chunk;
    const bool live = row < D;
    uchar4 ix = make_uchar4(0, 0, 0, 0);
    float m = 0.f;
    if (live) {
        ix = idx[row];
        m = mult[row];
    }
    float acc[KX];
#pragma unroll
    for (int k = 0; k < KX; ++k) acc[k] = 0.f;
    const T* Xb = X + (size_t)bh * Tlen * d;
    const float* Yb = Yp + (size_t)bh * Tlen * VP;
    for (int ci = 0; ci < nchunk; ++ci) {
        const int n = reverse ? nchunk - 1 - ci : ci;
        if (live) {
            float* dst = St + (((size_t)bh * nchunk + n) * D + row) * VP;
#pragma unroll
            for (int k = 0; k < KX; ++k) {
                int x = xg + 4 * k;
                if (x < VP) dst[x] = acc[k];
            }
        }
        if (ci == nchunk - 1) break;  // the sum including the last chunk visited is never used
        if (lam != nullptr) {
            const float l = lam[(size_t)bh * nchunk + n];
#pragma unroll
            for (int k = 0; k < KX; ++k) acc[k] *= l;
        }
        for (int t0 = 0; t0 < chunk; t0 += RT) {
            const int nt = min(RT, chunk - t0);
            const size_t tok0 = (size_t)n * chunk + t0;
            __syncthreads();
            for (int e = tid; e < nt * d; e += NT) xs[e] = xscale * io<T>::ld(Xb + tok0 * d + e);
            for (int e = tid; e < nt * VP; e += NT) ys[e] = Yb[tok0 * VP + e];
            for (int e = tid; e < nt; e += NT) fs[e] = fac != nullptr ? fac[(size_t)bh * Tlen + tok0 + e] : 1.f;
            __syncthreads();
            for (int j = 0; j < nt; ++j) {
                float coef = m * fs[j] * monomial<P>(xs + j * d, ix);
                const float* yr = ys + j * VP;
#pragma unroll
                for (int k = 0; k < KX; ++k) {
                    int x = xg + 4 * k;
                    if (x < VP) acc[k] += coef * yr[x];
                }
            }
        }
    }
}

// ---- forward per chunk: intra-chunk attention form + query-state read-out + normalise -------
template <typename T, int P, int KX>
__global__ __launch_bounds__(NT) void k_fwd_chunk(const T* __restrict__ Q, const T* __restrict__ K,
                                                  const float* __restrict__ Vp, const uchar4* __restrict__ idx,
                                                  const float* __restrict__ St, T* __restrict__ O,
                                                  float* __restrict__ Z, int Tlen, int d, int v, int chunk,
                                                  long long D, float scale, int normalize,
                                                  const float* __restrict__ bl, const float* __restrict__ qfac) {
    extern __shared__ float smem[];
    const int VP = v + 1;
    const int dq = d + 1;
    float* qs = smem;                     // [TOK][d+1]   scale * q
    float* ks = qs + TOK * dq;            // [RT][d]
    float* ts = ks + RT * d;              // [RT][VP]     state tile or V' tile
    uchar4* ixs = (uchar4*)(ts + RT * VP);  // [RT]
    float* bls = (float*)(ixs + RT);      // [RT]         log-decay of the keys since the chunk's start (gated)
    const int tid = threadIdx.x;
    const int tok = tid >> 2, xg = tid & 3;
    const int n = blockIdx.x, bh = blockIdx.y;
    const int nchunk = Tlen / chunk;
    const size_t base_tok = (size_t)bh * Tlen + (size_t)n * chunk;
    const float* Sn = St + ((size_t)bh * nchunk + n) * D * VP;
    const int kz = v >> 2, xz = v & 3;    // where column v (the normaliser) lives

    for (int i0 = 0; i0 < chunk; i0 += TOK) {
        const int ntok = min(TOK, chunk - i0);
        const int il = i0 + tok;          // row inside the chunk
        const bool live = tok < ntok;
        __syncthreads();
        for (int e = tid; e < ntok * d; e += NT) {
            int t = e / d, a = e - t * d;
            qs[t * dq + a] = scale * io<T>::ld(Q + (base_tok + i0 + t) * d + a);
        }
        float acc[KX];
#pragma unroll
        for (int k = 0; k < KX; ++k) acc[k] = 0.f;
        const float* qrow = qs + (live ? tok : 0) * dq;

        if (n > 0) {  // query-state: phi(q) . S_n
            for (long long r0 = 0; r0 < D; r0 += RT) {
                const int nr = (int)min((long long)RT, D - r0);
                __syncthreads();
                for (int e = tid; e < nr * VP; e += NT) ts[e] = Sn[(size_t)r0 * VP + e];
                if (tid < nr) ixs[tid] = idx[r0 + tid];
                __syncthreads();
                for (int rr = 0; rr < nr; ++rr) {
                    float coef = monomial<P>(qrow, ixs[rr]);
                    const float* sr = ts + rr * VP;
#pragma unroll
                    for (int k = 0; k < KX; ++k) {
                        int x = xg + 4 * k;
                        if (x < VP) acc[k] += coef * sr[x];
                    }
                }
            }
            if (qfac != nullptr) {   // the state is seen from the chunk's start: decay up to row i
                const float f = live ? qfac[base_tok + il] : 0.f;
#pragma unroll
                for (int k = 0; k < KX; ++k) acc[k] *= f;
            }
        }
        const float bli = (bl != nullptr && live) ? bl[base_tok + il] : 0.f;
        // attention form inside the chunk, keys j <= i
        const int jmax = i0 + ntok;  // keys beyond the last row of this pass are masked for everyone
        for (int j0 = 0; j0 < jmax; j0 += RT) {
            const int nj = min(RT, chunk - j0);
            __syncthreads();
            for (int e = tid; e < nj * d; e += NT) ks[e] = io<T>::ld(K + (base_tok + j0) * d + e);
            for (int e = tid; e < nj * VP; e += NT) ts[e] = Vp[(base_tok + j0) * VP + e];
            if (bl != nullptr)
                for (int e = tid; e < nj; e += NT) bls[e] = bl[base_tok + j0 + e];
            __syncthreads();
            for (int jj = 0; jj < nj; ++jj) {
                float part = 0.f;
                for (int a = xg; a < d; a += 4) part += qrow[a] * ks[jj * d + a];
                float s = quad_sum(part);
                float w = (j0 + jj <= il) ? ipow<P>(s) : 0.f;
                if (bl != nullptr && j0 + jj <= il) w *= __expf(bli - bls[jj]);
                const float* vr = ts + jj * VP;
#pragma unroll
                for (int k = 0; k < KX; ++k) {
                    int x = xg + 4 * k;
                    if (x < VP) acc[k] += w * vr[x];
                }
            }
        }
        float zmine = 0.f;
#pragma unroll
        for (int k = 0; k < KX; ++k)
            if (k == kz) zmine = acc[k];
        const float z = __shfl(zmine, (threadIdx.x & 63 & ~3) | xz);
        if (live) {
            const size_t row = base_tok + il;
            const float inv = normalize ? (z != 0.f ? 1.f / z : 0.f) : 1.f;
#pragma unroll
            for (int k = 0; k < KX; ++k) {
                int x = xg + 4 * k;
                if (x < v) io<T>::st(O + row * v + x, acc[k] * inv);
            }
            if (Z != nullptr && xg == xz) Z[row] = z;
        }
    }
}

// ---- backward per chunk, queries: dQ -------------------------------------------------------
//   dq_i = scale * [ sum_{j<=i in chunk} t_ij k_j  +  J_psi(scale q_i)^T (S_n ghat'_i) ]
//   t_ij = p s_ij^(p-1) (ghat'_i . v'_j)
template <typename T, int P, int KX>
__global__ __launch_bounds__(NT) void k_bwd_dq(const T* __restrict__ Q, const T* __restrict__ K,
                                               const float* __restrict__ Vp, const float* __restrict__ Gp,
                                               const uchar4* __restrict__ idx, const float* __restrict__ St,
                                               T* __restrict__ dQ, int Tlen, int d, int v, int chunk, long long D,
                                               float scale, const float* __restrict__ bl,
                                               const float* __restrict__ qfac, float* __restrict__ qdq) {
    extern __shared__ float smem[];
    const int VP = v + 1;
    const int dq = d + 1;
    float* qs = smem;                 // [TOK][d+1]  scale * q
    float* dqs = qs + TOK * dq;       // [TOK][d+1]  accumulators
    float* ks = dqs + TOK * dq;       // [RT][d]
    float* ts = ks + RT * d;          // [RT][VP]
    uchar4* ixs = (uchar4*)(ts + RT * VP);
    float* bls = (float*)(ixs + RT);  // [RT]        log-decay of the keys (gated)
    const int tid = threadIdx.x;
    const int tok = tid >> 2, xg = tid & 3;
    const int n = blockIdx.x, bh = blockIdx.y;
    const int nchunk = Tlen / chunk;
    const size_t base_tok = (size_t)bh * Tlen + (size_t)n * chunk;
    const float* Sn = St + ((size_t)bh * nchunk + n) * D * VP;

    for (int i0 = 0; i0 < chunk; i0 += TOK) {
        const int ntok = min(TOK, chunk - i0);
        const int il = i0 + tok;
        const bool live = tok < ntok;
        __syncthreads();
        for (int e = tid; e < ntok * d; e += NT) {
            int t = e / d, a = e - t * d;
            qs[t * dq + a] = scale * io<T>::ld(Q + (base_tok + i0 + t) * d + a);
        }
        for (int e = tid; e < TOK * dq; e += NT) dqs[e] = 0.f;
        float gp[KX];
#pragma unroll
        for (int k = 0; k < KX; ++k) {
            int x = xg + 4 * k;
            gp[k] = (live && x < VP) ? Gp[(base_tok + il) * VP + x] : 0.f;
        }
        const float* qrow = qs + (live ? tok : 0) * dq;
        float* dqrow = dqs + tok * dq;
        const float qf = (qfac != nullptr && live) ? qfac[base_tok + il] : 1.f;
        const float bli = (bl != nullptr && live) ? bl[base_tok + il] : 0.f;

        if (n > 0) {
            for (long long r0 = 0; r0 < D; r0 += RT) {
                const int nr = (int)min((long long)RT, D - r0);
                __syncthreads();
                for (int e = tid; e < nr * VP; e += NT) ts[e] = Sn[(size_t)r0 * VP + e];
                if (tid < nr) ixs[tid] = idx[r0 + tid];
                __syncthreads();
                for (int rr = 0; rr < nr; ++rr) {
                    const float* sr = ts + rr * VP;
                    float part = 0.f;
#pragma unroll
                    for (int k = 0; k < KX; ++k) {
                        int x = xg + 4 * k;
                        if (x < VP) part += sr[x] * gp[k];
                    }
                    const float g = qf * quad_sum(part);  // d loss / d psi(q)_r
                    if (xg < P) {
                        uchar4 ix = ixs[rr];
                        atomicAdd(dqrow + index_at(ix, xg), g * monomial_without<P>(qrow, ix, xg));
                    }
                }
            }
        }
        const int jmax = i0 + ntok;
        for (int j0 = 0; j0 < jmax; j0 += RT) {
            const int nj = min(RT, chunk - j0);
            __syncthreads();
            for (int e = tid; e < nj * d; e += NT) ks[e] = io<T>::ld(K + (base_tok + j0) * d + e);
            for (int e = tid; e < nj * VP; e += NT) ts[e] = Vp[(base_tok + j0) * VP + e];
            if (bl != nullptr)
                for (int e = tid; e < nj; e += NT) bls[e] = bl[base_tok + j0 + e];
            __syncthreads();
            for (int jj = 0; jj < nj; ++jj) {
                float ps = 0.f, pe = 0.f;
                for (int a = xg; a < d; a += 4) ps += qrow[a] * ks[jj * d + a];
                const float* vr = ts + jj * VP;
#pragma unroll
                for (int k = 0; k < KX; ++k) {
                    int x = xg + 4 * k;
                    if (x < VP) pe += gp[k] * vr[x];
                }
                const float s = quad_sum(ps), e = quad_sum(pe);
                float t = (j0 + jj <= il) ? (float)P * ipow_m1<P>(s) * e : 0.f;
                if (bl != nullptr && j0 + jj <= il) t *= __expf(bli - bls[jj]);
                for (int a = xg; a < d; a += 4) dqrow[a] += t * ks[jj * d + a];
            }
        }
        __syncthreads();
        for (int e = tid; e < ntok * d; e += NT) {
            int t = e / d, a = e - t * d;
            io<T>::st(dQ + (base_tok + i0 + t) * d + a, scale * dqs[t * dq + a]);
        }
        if (qdq != nullptr) {
            // q_i . dq_i for the gate gradient, from the unrounded accumulators (qs carries the scale dq lacks)
            float part = 0.f;
            for (int a = xg; a < d; a += 4) part += qrow[a] * dqrow[a];
            part = quad_sum(part);
            if (live && xg == 0) qdq[base_tok + il] = part;
        }
    }
}

// ---- backward per chunk, keys / values: dK, dV -----------------------------------------------
//   dv'_j = sum_{i>=j in chunk} s_ij^p ghat'_i  +  (m psi(k_j)) . R_n        (first v columns kept)
//   dk_j  = sum_{i>=j in chunk} t_ij (scale q_i) +  J_psi(k_j)^T (R'_n v'_j)
// Rt holds R' = m_r * sum over later chunks of psi(scale q_i)_r ghat'_i^T.
template <typename T, int P, int KX>
__global__ __launch_bounds__(NT) void k_bwd_dkdv(const T* __restrict__ Q, const T* __restrict__ K,
                                                 const float* __restrict__ Vp, const float* __restrict__ Gp,
                                                 const uchar4* __restrict__ idx, const float* __restrict__ Rt,
                                                 T* __restrict__ dK, T* __restrict__ dV, int Tlen, int d, int v,
                                                 int chunk, long long D, float scale, const float* __restrict__ bl,
                                                 const float* __restrict__ kfac, float* __restrict__ kdk) {
    extern __shared__ float smem[];
    const int VP = v + 1;
    const int dq = d + 1;
    float* kks = smem;                // [TOK][d+1]  own keys
    float* dks = kks + TOK * dq;      // [TOK][d+1]
    float* qb = dks + TOK * dq;       // [RT][d]     scale * q of the rows i
    float* ts = qb + RT * d;          // [RT][VP]    R' tile or ghat' tile
    uchar4* ixs = (uchar4*)(ts + RT * VP);
    float* bls = (float*)(ixs + RT);  // [RT]        log-decay of the rows i (gated)
    const int tid = threadIdx.x;
    const int tok = tid >> 2, xg = tid & 3;
    const int n = blockIdx.x, bh = blockIdx.y;
    const int nchunk = Tlen / chunk;
    const size_t base_tok = (size_t)bh * Tlen + (size_t)n * chunk;
    const float* Rn = Rt + ((size_t)bh * nchunk + n) * D * VP;

    for (int j0 = 0; j0 < chunk; j0 += TOK) {
        const int ntok = min(TOK, chunk - j0);
        const int jl = j0 + tok;
        const bool live = tok < ntok;
        __syncthreads();
        for (int e = tid; e < ntok * d; e += NT) {
            int t = e / d, a = e - t * d;
            kks[t * dq + a] = io<T>::ld(K + (base_tok + j0 + t) * d + a);
        }
        for (int e = tid; e < TOK * dq; e += NT) dks[e] = 0.f;
        float vp[KX], dv[KX];
#pragma unroll
        for (int k = 0; k < KX; ++k) {
            int x = xg + 4 * k;
            vp[k] = (live && x < VP) ? Vp[(base_tok + jl) * VP + x] : 0.f;
            dv[k] = 0.f;
        }
        const float* krow = kks + (live ? tok : 0) * dq;
        float* dkrow = dks + tok * dq;
        const float kf = (kfac != nullptr && live) ? kfac[base_tok + jl] : 1.f;
        const float blj = (bl != nullptr && live) ? bl[base_tok + jl] : 0.f;

        if (n < nchunk - 1) {
            for (long long r0 = 0; r0 < D; r0 += RT) {
                const int nr = (int)min((long long)RT, D - r0);
                __syncthreads();
                for (int e = tid; e < nr * VP; e += NT) ts[e] = Rn[(size_t)r0 * VP + e];
                if (tid < nr) ixs[tid] = idx[r0 + tid];
                __syncthreads();
                for (int rr = 0; rr < nr; ++rr) {
                    const float* rrow = ts + rr * VP;
                    const uchar4 ix = ixs[rr];
                    const float coef = kf * monomial<P>(krow, ix);
                    float part = 0.f;
#pragma unroll
                    for (int k = 0; k < KX; ++k) {
                        int x = xg + 4 * k;
                        if (x < VP) {
                            float rv = rrow[x];
                            dv[k] += coef * rv;
                            part += rv * vp[k];
                        }
                    }
                    const float g = kf * quad_sum(part);  // d loss / d psi(k)_r
                    if (xg < P) atomicAdd(dkrow + index_at(ix, xg), g * monomial_without<P>(krow, ix, xg));
                }
            }
        }
        // rows i >= j inside the chunk
        for (int i0 = (j0 / RT) * RT; i0 < chunk; i0 += RT) {
            const int ni = min(RT, chunk - i0);
            __syncthreads();
            for (int e = tid; e < ni * d; e += NT) qb[e] = scale * io<T>::ld(Q + (base_tok + i0) * d + e);
            for (int e = tid; e < ni * VP; e += NT) ts[e] = Gp[(base_tok + i0) * VP + e];
            if (bl != nullptr)
                for (int e = tid; e < ni; e += NT) bls[e] = bl[base_tok + i0 + e];
            __syncthreads();
            for (int ii = 0; ii < ni; ++ii) {
                float ps = 0.f, pe = 0.f;
                for (int a = xg; a < d; a += 4) ps += krow[a] * qb[ii * d + a];
                const float* gr = ts + ii * VP;
#pragma unroll
                for (int k = 0; k < KX; ++k) {
                    int x = xg + 4 * k;
                    if (x < VP) pe += vp[k] * gr[x];
                }
                const float s = quad_sum(ps), e = quad_sum(pe);
                const bool on = (i0 + ii >= jl);
                const float gate = (bl != nullptr && on) ? __expf(bls[ii] - blj) : 1.f;
                const float sm1 = gate * ipow_m1<P>(s);
                const float t = on ? (float)P * sm1 * e : 0.f;
                const float w = on ? sm1 * s : 0.f;
                for (int a = xg; a < d; a += 4) dkrow[a] += t * qb[ii * d + a];
#pragma unroll
                for (int k = 0; k < KX; ++k) {
                    int x = xg + 4 * k;
                    if (x < VP) dv[k] += w * gr[x];
                }
            }
        }
        __syncthreads();
        for (int e = tid; e < ntok * d; e += NT) {
            int t = e / d, a = e - t * d;
            io<T>::st(dK + (base_tok + j0 + t) * d + a, dks[t * dq + a]);
        }
        if (kdk != nullptr) {
            float part = 0.f;
            for (int a = xg; a < d; a += 4) part += krow[a] * dkrow[a];
            part = quad_sum(part);
            if (live && xg == 0) kdk[base_tok + jl] = part;
        }
        if (live) {
#pragma unroll
            for (int k = 0; k < KX; ++k) {
                int x = xg + 4 * k;
                if (x < v) io<T>::st(dV + (base_tok + jl) * v + x, dv[k]);
            }
        }
    }
}

// ---- gating: the pairs that straddle a chunk boundary -------------------------------------------
// xb[bh][n] = < R_n , S_{n+1} > = sum_r St[n+1][r] . Rt[n][r] / m_r  (both hold the multiplicity
// m_r; the inner product of the expanded vectors carries it once); 0 for the last chunk.
__global__ __launch_bounds__(256) void k_gate_boundary(const float* __restrict__ St, const float* __restrict__ Rt,
                                                       const float* __restrict__ mult, float* __restrict__ xb, long long D,
                                                       int VP, int nchunk) {
    __shared__ float red[4];
    const int n = blockIdx.x, bh = blockIdx.y;
    float acc = 0.f;
    if (n < nchunk - 1) {
        const float* S = St + ((size_t)bh * nchunk + n + 1) * D * VP;
        const float* R = Rt + ((size_t)bh * nchunk + n) * D * VP;
        for (long long e = threadIdx.x; e < D * VP; e += 256) acc += S[e] * R[e] / mult[e / VP];
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) xb[(size_t)bh * nchunk + n] = red[0] + red[1] + red[2] + red[3];
}

// ---- host side -------------------------------------------------------------------------------

struct Layout {
    long long D;
    int VP, KX, nchunk;
    size_t off_idx, off_mult, off_vp, off_st, off_gp, off_rt, total;
};

long long comb_ll(int n, int k) { return (long long)ndmi_count(n - k + 1, k); }  // C(n, k)

Layout make_layout(const pa_problem& pr, bool backward) {
    Layout L;
    L.D = comb_ll(pr.d + pr.p - 1, pr.p);
    L.VP = pr.v + 1;
    int kx = (L.VP + 3) / 4;
    L.KX = kx <= 5 ? 5 : kx <= 9 ? 9 : kx <= 17 ? 17 : 33;
    L.nchunk = pr.T / pr.chunk;
    const size_t BH = (size_t)pr.B * pr.H;
    size_t off = 0;
    L.off_idx = off;  off = align_up(off + (size_t)L.D * sizeof(uchar4), 256);
    L.off_mult = off; off = align_up(off + (size_t)L.D * sizeof(float), 256);
    L.off_vp = off;   off = align_up(off + BH * pr.T * L.VP * sizeof(float), 256);
    L.off_st = off;   off = align_up(off + BH * L.nchunk * (size_t)L.D * L.VP * sizeof(float), 256);
    L.off_gp = off;
    L.off_rt = off;
    if (backward) {
        off = align_up(off + BH * pr.T * L.VP * sizeof(float), 256);
        L.off_rt = off;
        off = align_up(off + BH * L.nchunk * (size_t)L.D * L.VP * sizeof(float), 256);
    }
    L.total = off;
    return L;
}

size_t smem_scan(const pa_problem& pr) { return (size_t)(RT * pr.d + RT * (pr.v + 1) + RT) * sizeof(float); }
size_t smem_fwd(const pa_problem& pr) {
    return (size_t)(TOK * (pr.d + 1) + RT * pr.d + RT * (pr.v + 1) + RT) * sizeof(float) + RT * sizeof(uchar4);
}
size_t smem_bwd(const pa_problem& pr) {
    return (size_t)(2 * TOK * (pr.d + 1) + RT * pr.d + RT * (pr.v + 1) + RT) * sizeof(float) + RT * sizeof(uchar4);
}

// LDS beyond the default per-kernel limit has to be requested once per kernel
template <typename F>
bool allow_smem(F* fn, size_t bytes) {
    if (bytes <= 48 * 1024) return true;
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) note_hip_error(e, "hipFuncSetAttribute(max dynamic LDS)");
    return e == hipSuccess;
}

#define PA_CHECK_LAUNCH()                       \
    do {                                        \
        if (!launch_ok()) return PA_ERR_HIP;    \
    } while (0)

template <typename T, int P, int KX>
pa_status run_fwd(const Ctx& c, const Layout& L, const T* Q, const T* K, const T* V, T* O, float* Z, bool only_state) {
    const pa_problem& pr = c.prob;
    const size_t BH = (size_t)pr.B * pr.H;
    uchar4* idx = (uchar4*)(c.ws + L.off_idx);
    float* mult = (float*)(c.ws + L.off_mult);
    float* Vp = (float*)(c.ws + L.off_vp);
    float* St = (float*)(c.ws + L.off_st);
    {
        LaunchScope ls("generic_build_table", c.stream);
        hipLaunchKernelGGL(k_build_table, dim3((unsigned)((L.D + 255) / 256)), dim3(256), 0, c.stream, pr.d, pr.p, L.D, idx, mult);
    }
    PA_CHECK_LAUNCH();
    {
        long long total = (long long)BH * pr.T * L.VP;
        LaunchScope ls("generic_prep_v", c.stream);
        hipLaunchKernelGGL((k_prep_v<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c.stream, V, Vp,
                           (long long)BH * pr.T, pr.v);
    }
    PA_CHECK_LAUNCH();
    {
        LaunchScope ls("generic_state_scan", c.stream);
        hipLaunchKernelGGL((k_scan<T, P, KX>), dim3((unsigned)((L.D + NT / 4 - 1) / (NT / 4)), (unsigned)BH), dim3(NT),
                           smem_scan(pr), c.stream, K, Vp, idx, mult, St, pr.T, pr.d, L.VP, pr.chunk, L.D, 1.0f, 0,
                           (const float*)c.gate.kfac, (const float*)c.gate.lam);
    }
    PA_CHECK_LAUNCH();
    if (only_state) return PA_OK;
    if (!allow_smem(k_fwd_chunk<T, P, KX>, smem_fwd(pr))) return PA_ERR_HIP;
    {
        LaunchScope ls("generic_fwd_chunk", c.stream);
        hipLaunchKernelGGL((k_fwd_chunk<T, P, KX>), dim3(L.nchunk, (unsigned)BH), dim3(NT), smem_fwd(pr), c.stream, Q, K,
                           Vp, idx, St, O, Z, pr.T, pr.d, pr.v, pr.chunk, L.D, pr.scale, pr.normalize,
                           (const float*)c.gate.bl, (const float*)c.gate.qfac);
    }
    PA_CHECK_LAUNCH();
    return PA_OK;
}

template <typename T, int P, int KX>
pa_status run_bwd(const Ctx& c, const Layout& L, const T* Q, const T* K, const T* V, const T* O, const float* Z,
                  const T* dO, T* dQ, T* dK, T* dV) {
    const pa_problem& pr = c.prob;
    const size_t BH = (size_t)pr.B * pr.H;
    // chunk states are recomputed here (nothing but O and Z is saved by the forward pass)
    pa_status st = run_fwd<T, P, KX>(c, L, Q, K, V, (T*)nullptr, (float*)nullptr, true);
    if (st != PA_OK) return st;
    uchar4* idx = (uchar4*)(c.ws + L.off_idx);
    float* mult = (float*)(c.ws + L.off_mult);
    float* Vp = (float*)(c.ws + L.off_vp);
    float* St = (float*)(c.ws + L.off_st);
    float* Gp = (float*)(c.ws + L.off_gp);
    float* Rt = (float*)(c.ws + L.off_rt);
    {
        long long rows = (long long)BH * pr.T;
        LaunchScope ls("generic_prep_g", c.stream);
        hipLaunchKernelGGL((k_prep_g<T>), dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, c.stream, dO, O, Z, Gp, rows,
                           pr.v, pr.normalize);
    }
    PA_CHECK_LAUNCH();
    {
        LaunchScope ls("generic_state_scan_reverse", c.stream);
        hipLaunchKernelGGL((k_scan<T, P, KX>), dim3((unsigned)((L.D + NT / 4 - 1) / (NT / 4)), (unsigned)BH), dim3(NT),
                           smem_scan(pr), c.stream, Q, Gp, idx, mult, Rt, pr.T, pr.d, L.VP, pr.chunk, L.D, pr.scale, 1,
                           (const float*)c.gate.qfac, (const float*)c.gate.lam);
    }
    PA_CHECK_LAUNCH();
    if (pr.gated) {
        LaunchScope ls("generic_gate_boundary", c.stream);
        hipLaunchKernelGGL(k_gate_boundary, dim3(L.nchunk, (unsigned)BH), dim3(256), 0, c.stream, (const float*)St,
                           (const float*)Rt, (const float*)mult, c.gate.xb, L.D, L.VP, L.nchunk);
        PA_CHECK_LAUNCH();
    }
    if (!allow_smem(k_bwd_dq<T, P, KX>, smem_bwd(pr)) || !allow_smem(k_bwd_dkdv<T, P, KX>, smem_bwd(pr))) return PA_ERR_HIP;
    {
        LaunchScope ls("generic_bwd_dq", c.stream);
        hipLaunchKernelGGL((k_bwd_dq<T, P, KX>), dim3(L.nchunk, (unsigned)BH), dim3(NT), smem_bwd(pr), c.stream, Q, K, Vp,
                           Gp, idx, St, dQ, pr.T, pr.d, pr.v, pr.chunk, L.D, pr.scale, (const float*)c.gate.bl,
                           (const float*)c.gate.qfac, c.gate.db);
    }
    PA_CHECK_LAUNCH();
    {
        LaunchScope ls("generic_bwd_dkdv", c.stream);
        hipLaunchKernelGGL((k_bwd_dkdv<T, P, KX>), dim3(L.nchunk, (unsigned)BH), dim3(NT), smem_bwd(pr), c.stream, Q, K,
                           Vp, Gp, idx, Rt, dK, dV, pr.T, pr.d, pr.v, pr.chunk, L.D, pr.scale, (const float*)c.gate.bl,
                           (const float*)c.gate.kfac, c.gate.db2);
    }
    PA_CHECK_LAUNCH();
    return PA_OK;
}

// dispatch over (dtype, p, KX)
template <typename T, int P>
pa_status dispatch_kx(bool bwd, const Ctx& c, const Layout& L, const void* Q, const void* K, const void* V, const void* O,
                      const float* Zin, const void* dO, void* Oout, float* Zout, void* dQ, void* dK, void* dV) {
#define PA_GO(KXV)                                                                                               \
    return bwd ? run_bwd<T, P, KXV>(c, L, (const T*)Q, (const T*)K, (const T*)V, (const T*)O, Zin, (const T*)dO, \
                                    (T*)dQ, (T*)dK, (T*)dV)                                                      \
               : run_fwd<T, P, KXV>(c, L, (const T*)Q, (const T*)K, (const T*)V, (T*)Oout, Zout, false)
    switch (L.KX) {
        case 5: PA_GO(5);
        case 9: PA_GO(9);
        case 17: PA_GO(17);
        default: PA_GO(33);
    }
#undef PA_GO
}

template <typename T>
pa_status dispatch_p(bool bwd, const Ctx& c, const Layout& L, const void* Q, const void* K, const void* V, const void* O,
                     const float* Zin, const void* dO, void* Oout, float* Zout, void* dQ, void* dK, void* dV) {
    switch (c.prob.p) {
        case 1: return dispatch_kx<T, 1>(bwd, c, L, Q, K, V, O, Zin, dO, Oout, Zout, dQ, dK, dV);
        case 2: return dispatch_kx<T, 2>(bwd, c, L, Q, K, V, O, Zin, dO, Oout, Zout, dQ, dK, dV);
        case 3: return dispatch_kx<T, 3>(bwd, c, L, Q, K, V, O, Zin, dO, Oout, Zout, dQ, dK, dV);
        default: return dispatch_kx<T, 4>(bwd, c, L, Q, K, V, O, Zin, dO, Oout, Zout, dQ, dK, dV);
    }
}

pa_status dispatch(bool bwd, const Ctx& c, const void* Q, const void* K, const void* V, const void* O, const float* Zin,
                   const void* dO, void* Oout, float* Zout, void* dQ, void* dK, void* dV) {
    const Layout L = make_layout(c.prob, bwd);
    if (c.prob.dtype == PA_DTYPE_F32)
        return dispatch_p<float>(bwd, c, L, Q, K, V, O, Zin, dO, Oout, Zout, dQ, dK, dV);
    return dispatch_p<bf16_t>(bwd, c, L, Q, K, V, O, Zin, dO, Oout, Zout, dQ, dK, dV);
}

}  // namespace

bool build_monomial_table(hipStream_t s, int d, int p, long long D, void* idx, float* mult) {
    LaunchScope ls("build_table", s);
    hipLaunchKernelGGL(k_build_table, dim3((unsigned)((D + 255) / 256)), dim3(256), 0, s, d, p, D, (uchar4*)idx, mult);
    return launch_ok();
}

pa_status generic_supported(const pa_problem& pr) {
    if (pr.p < 1 || pr.p > PMAX) return PA_ERR_UNSUPPORTED;
    if (pr.d > 128 || pr.v > 128) return PA_ERR_UNSUPPORTED;
    if (smem_bwd(pr) > 150 * 1024) return PA_ERR_UNSUPPORTED;
    if ((size_t)pr.B * pr.H > 65535u) return PA_ERR_UNSUPPORTED;
    return PA_OK;
}

long long generic_state_rows(const pa_problem& pr) { return comb_ll(pr.d + pr.p - 1, pr.p); }

size_t generic_workspace_bytes(const pa_problem& pr, bool backward) { return make_layout(pr, backward).total; }

pa_status generic_fwd(const Ctx& c, const void* Q, const void* K, const void* V, void* O, float* Z) {
    return dispatch(false, c, Q, K, V, nullptr, nullptr, nullptr, O, Z, nullptr, nullptr, nullptr);
}

pa_status generic_bwd(const Ctx& c, const void* Q, const void* K, const void* V, const void* O, const float* Z,
                      const void* dO, void* dQ, void* dK, void* dV) {
    return dispatch(true, c, Q, K, V, O, Z, dO, nullptr, nullptr, dQ, dK, dV);
}

}  // namespace pa
