// Shared host/device helpers of the power-attention library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "power_attn.h"

namespace pa {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; NaN is kept quiet
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct io;
template <> struct io<float> {
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float x) { *p = x; }
};
template <> struct io<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t* p, float x) { *p = f32_to_bf16(x); }
};

// ---- launch bookkeeping -------------------------------------------------------------
// Every kernel goes through launch_end(); when profiling is on, launch_begin/launch_end
// bracket it with events on the launch stream.
void profile_before(const char* name, hipStream_t s);
void profile_after(hipStream_t s);
bool profile_enabled();

struct LaunchScope {
    hipStream_t s;
    bool on;
    LaunchScope(const char* name, hipStream_t stream) : s(stream), on(profile_enabled()) {
        if (on) profile_before(name, s);
    }
    ~LaunchScope() {
        if (on) profile_after(s);
    }
};

// true if the launch just issued raised no error; a failure is remembered for
// power_attn_last_hip_error()
bool launch_ok();
void note_hip_error(hipError_t e, const char* where);

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- kernel families ------------------------------------------------------------------
// Per-token and per-chunk decay factors derived from the log-gates (all null when the problem
// is not gated).  With bl_i the sum of the log-gates from the start of token i's chunk up to i:
//   bl    [BH][T]       bl_i; a pair inside a chunk carries exp(bl_i - bl_j)
//   qfac  [BH][T]       exp(bl_i): decay of query i since the start of its chunk
//   kfac  [BH][T]       exp(bl_end - bl_j): decay of key j until the end of its chunk
//   lam   [BH][T/chunk] exp(bl_end): decay across the whole chunk
//   db    [BH][T]       backward pass: q_i . dq_i, written by the family's dQ kernel from its float32 accumulators
//   db2   [BH][T]       backward pass: k_i . dk_i, likewise
struct GateBuf {
    float *bl = nullptr, *qfac = nullptr, *kfac = nullptr, *lam = nullptr, *db = nullptr, *db2 = nullptr;
    float* xb = nullptr;    // [BH][T/chunk] backward: <R_m, S_{m+1}>, the pairs that straddle the end of chunk m (0 for the last)
};

struct Ctx {
    pa_problem prob;
    hipStream_t stream;
    char* ws;
    size_t ws_bytes;
    GateBuf gate;
};

// gating (family-independent kernels)
size_t gate_workspace_bytes(const pa_problem& pr, bool backward);
GateBuf gate_buffers(const pa_problem& pr, bool backward, char* base);
pa_status gate_prepare(const Ctx& c, const float* log_g);
// The family has already written gate.xb, q.dq into gate.db and k.dk into gate.db2.
// fin_chunk: the token granularity of gate.xb (the problem's chunk, or finer when the family says so)
pa_status gate_gradient(const Ctx& c, float* dlog_g, int fin_chunk);

// generic (vector-ALU, float32) family
size_t generic_workspace_bytes(const pa_problem& pr, bool backward);
long long generic_state_rows(const pa_problem& pr);
// Row r of the lexicographic list of non-decreasing multi-indices of Lemma 4.2 -> idx[r] (uchar4, its
// p indices padded with 0) and mult[r] (its multiplicity p! / prod(run lengths)!); device arrays of D rows
bool build_monomial_table(hipStream_t s, int d, int p, long long D, void* idx, float* mult);

// single-token decode step (state resident between calls)
size_t decode_state_bytes(const pa_problem& pr);
pa_status decode_init(const pa_problem& pr, void* state, hipStream_t s);
size_t decode_absorb_workspace_bytes(const pa_problem& pr);
pa_status decode_absorb(const pa_problem& pr, const void* K, const void* V, const float* log_g, void* state, void* ws,
                        size_t ws_bytes, hipStream_t s);
pa_status decode_step(const pa_problem& pr, const void* q, const void* k, const void* v, const float* log_g, void* state, void* o,
                      float* z, hipStream_t s);
pa_status generic_supported(const pa_problem& pr);
pa_status generic_fwd(const Ctx& c, const void* Q, const void* K, const void* V, void* O, float* Z);
pa_status generic_bwd(const Ctx& c, const void* Q, const void* K, const void* V, const void* O, const float* Z,
                      const void* dO, void* dQ, void* dK, void* dV);

// bf16 MFMA family (p = 2)
size_t mfma_workspace_bytes(const pa_problem& pr, bool backward);
long long mfma_state_rows(const pa_problem& pr);
pa_status mfma_supported(const pa_problem& pr, bool backward);
pa_status mfma_fwd(const Ctx& c, const void* Q, const void* K, const void* V, void* O, float* Z);
pa_status mfma_bwd(const Ctx& c, const void* Q, const void* K, const void* V, const void* O, const float* Z,
                   const void* dO, void* dQ, void* dK, void* dV);
// A prompt K, V [B,H,T,d] (pr.T tokens) added into a decode state (S [BH][D][v], gamd [BH][D], float32, D rows in the
// monomial basis of the decode step) by way of the state scan; bf16, p = 2, d = v = 64, T a multiple of 128
bool mfma_absorb_supported(const pa_problem& pr);
size_t mfma_absorb_workspace_bytes(const pa_problem& pr);
pa_status mfma_absorb(const pa_problem& pr, const void* K, const void* V, const float* log_g, char* ws, hipStream_t s, float* S,
                      float* gamd, int D);
// destroys the calling thread's side stream and events of the MFMA backward pass, if it has any
void mfma_release_side_stream();
// tokens per entry of GateBuf::xb as mfma_bwd leaves it (gated problems)
int mfma_gate_fin_chunk(const pa_problem& pr);

}  // namespace pa
