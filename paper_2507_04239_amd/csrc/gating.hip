// Gating (arXiv 2507.04239 Sec. 2 "Gating"; gated update-state of App. E.2, discounted
// cumulative sum of App. E.3): the kernels every kernel family shares.  The paper states the
// operation at chunk granularity; the per-timestep definition behind it is
//     a_ij = s_ij^p exp(b_i - b_j),   b_i = sum_{t<=i} log g_t,   j <= i.
// In the chunked form only sums of log-gates inside one chunk are ever needed (every factor is
// then a decay <= 1): see GateBuf in common.hpp.  The gradient of the log-gates follows from the
// homogeneity of the scores: dL/db_i = (q_i . dq_i - k_i . dk_i) / p, dL/dlog g_t = sum_{i>=t} dL/db_i.
#include "common.hpp"

namespace pa {
namespace {

constexpr int GT = 256;

// One workgroup per (chunk, head): inclusive running sum of the chunk's log-gates, then the factors.
__global__ __launch_bounds__(GT) void k_gate_prep(const float* __restrict__ log_g, float* __restrict__ bl,
                                                  float* __restrict__ qfac, float* __restrict__ kfac,
                                                  float* __restrict__ lam, int T, int chunk) {
    __shared__ float part[GT];
    const int n = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const size_t base = (size_t)bh * T + (size_t)n * chunk;
    const int per = (chunk + GT - 1) / GT;        // consecutive tokens per thread
    const int lo = min(tid * per, chunk), hi = min(lo + per, chunk);
    float s = 0.f;
    for (int i = lo; i < hi; ++i) s += log_g[base + i];
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < GT; off <<= 1) {      // inclusive scan of the per-thread sums
        float add = tid >= off ? part[tid - off] : 0.f;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    const float total = part[GT - 1];
    float run = tid > 0 ? part[tid - 1] : 0.f;
    for (int i = lo; i < hi; ++i) {
        run += log_g[base + i];
        bl[base + i] = run;
        qfac[base + i] = __expf(run);
        kfac[base + i] = __expf(total - run);
    }
    if (tid == 0) lam[(size_t)bh * (T / chunk) + n] = __expf(total);
}

// dlog_g[t] = sum_{i >= t} dL/db_i.  A running sum over the whole sequence would pile up the
// rounding noise of tens of thousands of terms on a result that is local (only pairs within a few
// decay lengths of t matter).  Instead: the part of the sum beyond the end of t's chunk m equals
//     X_m = sum_{j <= end_m < i} e_ij a_ij = < R_m , S_{m+1} >,
// the inner product of the two states that meet at that chunk boundary, which each kernel family
// computes from its states (xb); only the part inside the chunk is summed here.
// db holds q_i . dq_i and db2 k_i . dk_i: dL/db_i = (db[i] - db2[i]) / p.
__device__ __forceinline__ float gate_term(const float* __restrict__ db, const float* __restrict__ db2, float inv_p,
                                           size_t i) {
    return (db[i] - db2[i]) * inv_p;
}

__global__ __launch_bounds__(GT) void k_gate_finish(const float* __restrict__ db, const float* __restrict__ db2, float inv_p,
                                                    const float* __restrict__ xb, float* __restrict__ dlog_g,
                                                    int T, int chunk) {
    __shared__ float part[GT];
    const int n = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const size_t base = (size_t)bh * T + (size_t)n * chunk;
    const int per = (chunk + GT - 1) / GT;
    const int lo = min(tid * per, chunk), hi = min(lo + per, chunk);
    float s = 0.f;
    for (int i = lo; i < hi; ++i) s += gate_term(db, db2, inv_p, base + i);
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < GT; off <<= 1) {      // inclusive suffix scan of the per-thread sums
        const float add = tid + off < GT ? part[tid + off] : 0.f;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    float run = xb[(size_t)bh * (T / chunk) + n] + (tid + 1 < GT ? part[tid + 1] : 0.f);
    for (int i = hi - 1; i >= lo; --i) {
        run += gate_term(db, db2, inv_p, base + i);
        dlog_g[base + i] = run;
    }
}

}  // namespace

// entries per head of the per-chunk arrays: the boundary sums of the backward pass may be kept per
// 128 tokens when the chunk is longer (the attention form)
static size_t chunk_slots(const pa_problem& pr) {
    const size_t a = (size_t)(pr.T / pr.chunk), b = (size_t)((pr.T + 127) / 128);
    return a > b ? a : b;
}

size_t gate_workspace_bytes(const pa_problem& pr, bool backward) {
    if (!pr.gated) return 0;
    const size_t BH = (size_t)pr.B * pr.H;
    const size_t tok = align_up(BH * pr.T * sizeof(float), 256);
    return (backward ? 5 : 3) * tok + (backward ? 2 : 1) * align_up(BH * chunk_slots(pr) * sizeof(float), 256);
}

GateBuf gate_buffers(const pa_problem& pr, bool backward, char* base) {
    GateBuf g;
    if (!pr.gated) return g;
    const size_t BH = (size_t)pr.B * pr.H;
    const size_t tok = align_up(BH * pr.T * sizeof(float), 256);
    g.bl = (float*)base;
    g.qfac = (float*)(base + tok);
    g.kfac = (float*)(base + 2 * tok);
    g.lam = (float*)(base + 3 * tok);
    if (backward) {
        g.db = (float*)(base + 3 * tok + align_up(BH * chunk_slots(pr) * sizeof(float), 256));
        g.db2 = g.db + tok / sizeof(float);
        g.xb = g.db2 + tok / sizeof(float);
    }
    return g;
}

pa_status gate_prepare(const Ctx& c, const float* log_g) {
    const pa_problem& pr = c.prob;
    LaunchScope ls("gate_prep", c.stream);
    hipLaunchKernelGGL(k_gate_prep, dim3(pr.T / pr.chunk, pr.B * pr.H), dim3(GT), 0, c.stream, log_g, c.gate.bl, c.gate.qfac,
                       c.gate.kfac, c.gate.lam, pr.T, pr.chunk);
    return launch_ok() ? PA_OK : PA_ERR_HIP;
}

pa_status gate_gradient(const Ctx& c, float* dlog_g, int fin_chunk) {
    const pa_problem& pr = c.prob;
    // Under the sum normalisation q_i . dq_i is zero in exact arithmetic, yet the term stays: what the
    // device finds there is dO_i . (O_i - rounded O_i), and the k_j . dk_j of the keys after t contain
    // exactly that with the opposite sign, row by row.  Both dot products come from the kernels' float32
    // accumulators: formed from the rounded bf16 outputs they would carry 2^-9 of terms that cancel.
    // (Measured, bf16, decay 0.5 per step: relative L2 error of dlog_g 1.8e-2 without the row term, 9e-3
    // with it from rounded outputs, 3e-3 from the accumulators; no worse at weak decay.)
    LaunchScope ls("gate_finish", c.stream);
    hipLaunchKernelGGL(k_gate_finish, dim3(pr.T / fin_chunk, pr.B * pr.H), dim3(GT), 0, c.stream, (const float*)c.gate.db,
                       (const float*)c.gate.db2, 1.f / pr.p, (const float*)c.gate.xb, dlog_g, pr.T, fin_chunk);
    return launch_ok() ? PA_OK : PA_ERR_HIP;
}

}  // namespace pa
