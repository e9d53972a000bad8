// C ABI of the power-attention library: argument validation, kernel-family selection and
// the optional per-kernel event timing.  See include/power_attn.h for the contract.
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "common.hpp"

namespace pa {
namespace {

struct Record {
    std::string name;
    hipEvent_t e0, e1;
};
// Scratch of power_attn_fwd_static: device memory that is part of the library's code object, so
// that callers who may not allocate still have a workspace.  Each GPU the library runs on holds its
// own copy of the array at its own address until the process ends.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)PA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};   // device address of `scratch` on each device, looked up once

// The array's name is a host-side stand-in here, not a device address; the address on the current
// device comes from the runtime, once per device.
pa_status static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        note_hip_error(e, "hipGetDevice (static scratch)");
        return PA_ERR_HIP;
    }
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            note_hip_error(e, "hipGetSymbolAddress(scratch)");
            return PA_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PA_OK;
}

// Per host thread: the profiling switch and its records, and the text of the last HIP error.  Calls from
// different host threads share nothing but the static scratch of power_attn_fwd_static.
thread_local bool g_profile = false;
thread_local char g_last_error[256] = "";
thread_local std::vector<Record> g_records;

// the tensor arguments are read and written with 16-byte vector accesses
bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

pa_status validate(const pa_problem* pr) {
    if (pr == nullptr) return PA_ERR_INVALID_ARG;
    if (pr->B <= 0 || pr->H <= 0 || pr->T <= 0 || pr->d <= 0 || pr->v <= 0 || pr->p <= 0 || pr->chunk < 0)
        return PA_ERR_INVALID_ARG;
    if (pr->normalize != 0 && (pr->p % 2) != 0) return PA_ERR_INVALID_ARG;  // scores must be positive to normalise
    if (pr->dtype != PA_DTYPE_F32 && pr->dtype != PA_DTYPE_BF16) return PA_ERR_INVALID_ARG;
    if (pr->impl != PA_IMPL_AUTO && pr->impl != PA_IMPL_GENERIC && pr->impl != PA_IMPL_MFMA && pr->impl != PA_IMPL_RESIDENT &&
        pr->impl != PA_IMPL_TILED)
        return PA_ERR_INVALID_ARG;
    if (pr->d_tile < 0) return PA_ERR_INVALID_ARG;
    if (!(pr->scale == pr->scale) || pr->scale == 0.f) return PA_ERR_INVALID_ARG;
    if (pr->gated != 0 && pr->gated != 1) return PA_ERR_INVALID_ARG;
    return PA_OK;
}

// chunk == 0: the library picks between the attention form (one chunk: cost ~ T per token) and the
// chunked form (cost ~ the state size per token), Sec. 2 "Chunked form".  Where the bf16 MFMA
// kernels apply the choice is measured on MI355X.  p = 2, d = 64, which has both forms on the
// matrix cores: the attention form wins up to T = 4096 (2048 with gating), and 256 is the best chunk
// beyond (128 when 256 does not divide T).  Other
// degrees and head sizes have matrix-core kernels for the attention form only, and that beats the
// chunked form on the vector ALUs at any length the latter is sensible for.  Elsewhere the two costs
// are compared by their multiply-add counts, T (4 d + 2) / 2 per token against 4 D (v + 1), with a
// factor of two against the attention form: the generic kernels' in-chunk code does about half as many
// multiply-adds per second as their state code (config 1, T = 256: 0.32 ms as one chunk, 0.14 ms chunked).
int auto_chunk(const pa_problem& pr) {
    const bool may_mfma = pr.impl == PA_IMPL_AUTO || pr.impl == PA_IMPL_MFMA || pr.impl == PA_IMPL_RESIDENT || pr.impl == PA_IMPL_TILED;
    pa_problem probe = pr;
    probe.chunk = pr.T;
    const bool attn = may_mfma && mfma_supported(probe, true) == PA_OK;
    // the chunked kernels, on the sequence rounded up to whole chunks when it is ragged (see Padding)
    probe.chunk = pr.T % 256 == 0 || pr.T % 128 != 0 ? 256 : 128;
    probe.T = (pr.T + probe.chunk - 1) / probe.chunk * probe.chunk;
    // p = 2 at the other head sizes runs chunked on the tiled kernels.  d = 128: measured at B8 H16 T32768, 110 ms a
    // step chunked against 166 ms for the attention form, whose time grows with the square of T: the two meet near
    // 23k tokens.  d = 32 (B4 H8): 0.24 against 0.15 ms at T = 2048, 0.75 against 1.20 ms at 8192, 2.2 against 6.5 ms
    // at 32768.  For the higher degrees the attention form stays ahead at every length measured (p = 3, d = 64:
    // 1.3 against 6.0 ms at T = 16384, 39 against 61 ms at 131072; p = 4, d = 32: 2.5 against 24 ms at 16384, 50
    // against 101 ms at 131072).
    const int attn_upto = pr.d == 128 ? 24575 : (pr.gated ? 2048 : 4096);
    if (may_mfma && pr.p == 2 && (pr.d == 32 || pr.d == 64 || pr.d == 128) && mfma_supported(probe, true) == PA_OK &&
        !(attn && pr.T <= attn_upto))
        return probe.chunk;
    if (attn) return pr.T;
    double D = 1.0;   // C(d + p - 1, p)
    for (int i = 1; i <= pr.p; ++i) D = D * (pr.d + pr.p - i) / i;
    if (pr.T * (4.0 * pr.d + 2.0) <= 4.0 * D * (pr.v + 1)) return pr.T;
    // chunked, generic kernels: 64 measured best on every shape tried (f32 and bf16, d = 16 .. 64, p = 2
    // and 4, forward and backward; 32 within a few per cent, 128 10 to 80 % slower)
    for (int c = 64; c >= 1; c >>= 1)
        if (pr.T % c == 0) return c;
    return 1;
}

pa_problem resolved(const pa_problem* prob) {
    pa_problem pr = *prob;
    if (pr.chunk == 0) pr.chunk = auto_chunk(pr);
    return pr;
}

// PA_IMPL_GENERIC / PA_IMPL_MFMA, or a negative status
int choose(const pa_problem& pr, bool backward, pa_status* why) {
    if (pr.impl == PA_IMPL_MFMA || pr.impl == PA_IMPL_RESIDENT || pr.impl == PA_IMPL_TILED || pr.impl == PA_IMPL_AUTO) {
        pa_status st = mfma_supported(pr, backward);
        if (st == PA_OK) return PA_IMPL_MFMA;
        if (pr.impl != PA_IMPL_AUTO || pr.d_tile > 0) {   // a tile width is a request for the kernels that have one
            *why = st;
            return -1;
        }
    }
    pa_status st = generic_supported(pr);
    if (st == PA_OK) return PA_IMPL_GENERIC;
    *why = st;
    return -1;
}

// ---- sequences that are not a multiple of the chunk -----------------------------------------------
// The chunked MFMA kernels work on whole chunks.  A ragged sequence is run as the next longer one:
// Q, K, V (dO, O, Z, log-gates) are copied into the workspace with zero rows appended - zero keys and
// values add nothing to any state or sum, zero upstream gradients and gates of one (log 0) neither -
// and the first T rows of the results are copied back.  Costs one pass over every operand.
struct Padding {
    bool on = false;
    pa_problem prob;        // the problem the kernels see (T rounded up)
    size_t tok = 0, vec = 0;   // bytes of one padded [B,H,T,d] operand and of one padded [B,H,T] float array
};

Padding padding_for(const pa_problem& pr) {
    Padding pd;
    pd.prob = pr;
    if (pr.chunk <= 0 || pr.T % pr.chunk == 0) return pd;
    pd.on = true;
    pd.prob.T = (pr.T + pr.chunk - 1) / pr.chunk * pr.chunk;
    const size_t rows = (size_t)pr.B * pr.H * pd.prob.T;
    pd.tok = align_up(rows * pr.d * (pr.dtype == PA_DTYPE_BF16 ? 2 : 4), 256);
    pd.vec = align_up(rows * sizeof(float), 256);
    return pd;
}
size_t padding_bytes(const Padding& pd, bool backward) {
    if (!pd.on) return 0;
    const size_t ntok = backward ? 8 : 4, nvec = (backward ? 1 : 1) + (pd.prob.gated ? (backward ? 2 : 1) : 0);
    return ntok * pd.tok + nvec * pd.vec;
}

// rows of `elems` elements: out [BH][T_out][elems] <- in [BH][T_in][elems], zero where t >= T_in
template <typename E>
__global__ __launch_bounds__(256) void k_copy_rows(const E* __restrict__ in, E* __restrict__ out, long long total, int T_in,
                                                   int T_out, int elems) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int e = (int)(i % elems);
    const long long r = i / elems;
    const int t = (int)(r % T_out);
    const long long bh = r / T_out;
    E zero{};
    out[i] = t < T_in ? in[(bh * T_in + t) * elems + e] : zero;
}
// bytes_per_row: 4 for the per-token float arrays, d * element size for the operands (a multiple of 16 there)
bool copy_rows(hipStream_t s, const void* in, void* out, size_t BH, int T_in, int T_out, int bytes_per_row) {
    LaunchScope ls("pad_rows", s);
    if (bytes_per_row % 16 == 0) {
        const long long total = (long long)BH * T_out * (bytes_per_row / 16);
        hipLaunchKernelGGL((k_copy_rows<uint4>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const uint4*)in,
                           (uint4*)out, total, T_in, T_out, bytes_per_row / 16);
    } else {
        const long long total = (long long)BH * T_out * (bytes_per_row / 4);
        hipLaunchKernelGGL((k_copy_rows<float>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const float*)in,
                           (float*)out, total, T_in, T_out, bytes_per_row / 4);
    }
    return launch_ok();
}

// workspace of the kernel family, rounded so that the gating buffers can follow it
size_t family_bytes(int impl, const pa_problem& pr, bool backward) {
    return align_up(impl == PA_IMPL_MFMA ? mfma_workspace_bytes(pr, backward) : generic_workspace_bytes(pr, backward), 256);
}

pa_status run_fwd(const pa_problem* prob, const void* Q, const void* K, const void* V, const float* log_g, void* O, float* Z,
                  void* workspace, size_t workspace_bytes, void* hip_stream, int gated) {
    pa_status st = validate(prob);
    if (st != PA_OK) return st;
    if (prob->gated != gated) return PA_ERR_INVALID_ARG;
    if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr || (gated && log_g == nullptr)) return PA_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(Z) || !aligned16(log_g))
        return PA_ERR_INVALID_ARG;
    const pa_problem asked = resolved(prob);
    const Padding pd = padding_for(asked);
    prob = &pd.prob;
    pa_status why = PA_ERR_UNSUPPORTED;
    int impl = choose(*prob, false, &why);
    if (impl < 0) return why;
    if (pd.on && impl != PA_IMPL_MFMA) return PA_ERR_UNSUPPORTED;     // only the MFMA kernels run padded
    const size_t fam = family_bytes(impl, *prob, false);
    const size_t inner = fam + gate_workspace_bytes(*prob, false);
    const size_t need = inner + padding_bytes(pd, false);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return PA_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return PA_ERR_WORKSPACE;
    (void)hipGetLastError();  // errors left behind by earlier, unrelated runtime calls are not ours
    hipStream_t s = (hipStream_t)hip_stream;
    void* Zout = Z;
    void* Oout = O;
    if (pd.on) {
        char* base = (char*)workspace + inner;
        const size_t BH = (size_t)asked.B * asked.H;
        const int row = asked.d * 2;
        void *Qp = base, *Kp = base + pd.tok, *Vp = base + 2 * pd.tok;
        if (!copy_rows(s, Q, Qp, BH, asked.T, prob->T, row) || !copy_rows(s, K, Kp, BH, asked.T, prob->T, row) ||
            !copy_rows(s, V, Vp, BH, asked.T, prob->T, row))
            return PA_ERR_HIP;
        Q = Qp;
        K = Kp;
        V = Vp;
        O = base + 3 * pd.tok;
        Z = (float*)(base + 4 * pd.tok);
        if (gated) {
            float* lp = (float*)(base + 4 * pd.tok + pd.vec);
            if (!copy_rows(s, log_g, lp, BH, asked.T, prob->T, 4)) return PA_ERR_HIP;
            log_g = lp;
        }
    }
    Ctx c{*prob, s, (char*)workspace, workspace_bytes, gate_buffers(*prob, false, (char*)workspace + fam)};
    if (gated) {
        st = gate_prepare(c, log_g);
        if (st != PA_OK) return st;
    }
    st = impl == PA_IMPL_MFMA ? mfma_fwd(c, Q, K, V, O, Z) : generic_fwd(c, Q, K, V, O, Z);
    if (st != PA_OK || !pd.on) return st;
    const size_t BH = (size_t)asked.B * asked.H;
    if (!copy_rows(s, O, Oout, BH, prob->T, asked.T, asked.v * 2)) return PA_ERR_HIP;
    if (Zout != nullptr && !copy_rows(s, Z, Zout, BH, prob->T, asked.T, 4)) return PA_ERR_HIP;
    return PA_OK;
}

pa_status run_bwd(const pa_problem* prob, const void* Q, const void* K, const void* V, const float* log_g, const void* O,
                  const float* Z, const void* dO, void* dQ, void* dK, void* dV, float* dlog_g, void* workspace,
                  size_t workspace_bytes, void* hip_stream, int gated) {
    pa_status st = validate(prob);
    if (st != PA_OK) return st;
    if (prob->gated != gated) return PA_ERR_INVALID_ARG;
    if (Q == nullptr || K == nullptr || V == nullptr || dO == nullptr || dQ == nullptr || dK == nullptr || dV == nullptr)
        return PA_ERR_INVALID_ARG;
    if (gated && (log_g == nullptr || dlog_g == nullptr)) return PA_ERR_INVALID_ARG;
    if (prob->normalize != 0 && (O == nullptr || Z == nullptr)) return PA_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(Z) || !aligned16(dO) || !aligned16(dQ) ||
        !aligned16(dK) || !aligned16(dV) || !aligned16(log_g) || !aligned16(dlog_g))
        return PA_ERR_INVALID_ARG;
    const pa_problem asked = resolved(prob);
    const Padding pd = padding_for(asked);
    prob = &pd.prob;
    pa_status why = PA_ERR_UNSUPPORTED;
    int impl = choose(*prob, true, &why);
    if (impl < 0) return why;
    if (pd.on && impl != PA_IMPL_MFMA) return PA_ERR_UNSUPPORTED;
    const size_t fam = family_bytes(impl, *prob, true);
    const size_t inner = fam + gate_workspace_bytes(*prob, true);
    const size_t need = inner + padding_bytes(pd, true);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return PA_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return PA_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t BH = (size_t)asked.B * asked.H;
    void *dQout = dQ, *dKout = dK, *dVout = dV;
    float* dlout = dlog_g;
    if (pd.on) {
        char* base = (char*)workspace + inner;
        const int row = asked.d * 2;
        void* buf[8];
        for (int i = 0; i < 8; ++i) buf[i] = base + i * pd.tok;
        float* Zp = (float*)(base + 8 * pd.tok);
        if (!copy_rows(s, Q, buf[0], BH, asked.T, prob->T, row) || !copy_rows(s, K, buf[1], BH, asked.T, prob->T, row) ||
            !copy_rows(s, V, buf[2], BH, asked.T, prob->T, row) || !copy_rows(s, dO, buf[3], BH, asked.T, prob->T, row))
            return PA_ERR_HIP;
        if (O != nullptr && !copy_rows(s, O, buf[4], BH, asked.T, prob->T, row)) return PA_ERR_HIP;
        if (Z != nullptr && !copy_rows(s, Z, Zp, BH, asked.T, prob->T, 4)) return PA_ERR_HIP;
        Q = buf[0];
        K = buf[1];
        V = buf[2];
        dO = buf[3];
        if (O != nullptr) O = buf[4];
        if (Z != nullptr) Z = Zp;
        dQ = buf[5];
        dK = buf[6];
        dV = buf[7];
        if (gated) {
            float* lp = (float*)(base + 8 * pd.tok + pd.vec);
            if (!copy_rows(s, log_g, lp, BH, asked.T, prob->T, 4)) return PA_ERR_HIP;
            log_g = lp;
            dlog_g = lp + pd.vec / sizeof(float);
        }
    }
    Ctx c{*prob, s, (char*)workspace, workspace_bytes, gate_buffers(*prob, true, (char*)workspace + fam)};
    if (gated) {
        // the factors are rebuilt here: the forward pass keeps its own copy only inside its workspace
        st = gate_prepare(c, log_g);
        if (st != PA_OK) return st;
    }
    st = impl == PA_IMPL_MFMA ? mfma_bwd(c, Q, K, V, O, Z, dO, dQ, dK, dV) : generic_bwd(c, Q, K, V, O, Z, dO, dQ, dK, dV);
    if (st == PA_OK && gated)
        st = gate_gradient(c, dlog_g, impl == PA_IMPL_MFMA ? mfma_gate_fin_chunk(*prob) : prob->chunk);
    if (st != PA_OK || !pd.on) return st;
    const int row = asked.d * 2;
    if (!copy_rows(s, dQ, dQout, BH, prob->T, asked.T, row) || !copy_rows(s, dK, dKout, BH, prob->T, asked.T, row) ||
        !copy_rows(s, dV, dVout, BH, prob->T, asked.T, row))
        return PA_ERR_HIP;
    if (gated && !copy_rows(s, dlog_g, dlout, BH, prob->T, asked.T, 4)) return PA_ERR_HIP;
    return PA_OK;
}

}  // namespace

bool profile_enabled() { return g_profile; }

void note_hip_error(hipError_t e, const char* where) {
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s", where, hipGetErrorString(e));
}

bool launch_ok() {
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return true;
    note_hip_error(e, "kernel launch");
    return false;
}

void profile_before(const char* name, hipStream_t s) {
    Record r;
    r.name = name;
    if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
    (void)hipEventRecord(r.e0, s);
    g_records.push_back(r);
}

void profile_after(hipStream_t s) {
    if (!g_records.empty()) (void)hipEventRecord(g_records.back().e1, s);
}

}  // namespace pa

using namespace pa;

extern "C" {

const char* power_attn_status_string(pa_status s) {
    switch (s) {
        case PA_OK: return "ok";
        case PA_ERR_INVALID_ARG: return "invalid argument";
        case PA_ERR_UNSUPPORTED: return "unsupported problem for the requested kernel family";
        case PA_ERR_WORKSPACE: return "workspace missing or too small";
        case PA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

pa_status power_attn_supported(const pa_problem* prob, int for_backward) {
    pa_status st = validate(prob);
    if (st != PA_OK) return st;
    const Padding pd = padding_for(resolved(prob));
    pa_status why = PA_ERR_UNSUPPORTED;
    const int impl = choose(pd.prob, for_backward != 0, &why);
    if (impl < 0) return why;
    return pd.on && impl != PA_IMPL_MFMA ? PA_ERR_UNSUPPORTED : PA_OK;
}

size_t power_attn_workspace_bytes(const pa_problem* prob, int for_backward) {
    if (validate(prob) != PA_OK) return 0;
    const Padding pd = padding_for(resolved(prob));
    pa_status why;
    int impl = choose(pd.prob, for_backward != 0, &why);
    if (impl < 0 || (pd.on && impl != PA_IMPL_MFMA)) return 0;
    return family_bytes(impl, pd.prob, for_backward != 0) + gate_workspace_bytes(pd.prob, for_backward != 0) +
           padding_bytes(pd, for_backward != 0);
}

long long power_attn_state_rows(const pa_problem* prob) {
    if (validate(prob) != PA_OK) return 0;
    const Padding pd = padding_for(resolved(prob));
    pa_status why;
    int impl = choose(pd.prob, false, &why);
    if (impl < 0 || (pd.on && impl != PA_IMPL_MFMA)) return 0;
    return impl == PA_IMPL_MFMA ? mfma_state_rows(pd.prob) : generic_state_rows(pd.prob);
}

// the fields a decode step reads, checked like the same fields of the other calls
static pa_status validate_decode(const pa_problem* pr) {
    if (pr == nullptr) return PA_ERR_INVALID_ARG;
    if (pr->B <= 0 || pr->H <= 0 || pr->d <= 0 || pr->v <= 0 || pr->p <= 0) return PA_ERR_INVALID_ARG;
    if (pr->normalize != 0 && (pr->p % 2) != 0) return PA_ERR_INVALID_ARG;
    if (pr->dtype != PA_DTYPE_F32 && pr->dtype != PA_DTYPE_BF16) return PA_ERR_INVALID_ARG;
    if (!(pr->scale == pr->scale) || pr->scale == 0.f) return PA_ERR_INVALID_ARG;
    if (pr->gated != 0 && pr->gated != 1) return PA_ERR_INVALID_ARG;
    return PA_OK;
}

size_t power_attn_decode_state_bytes(const pa_problem* prob) {
    return validate_decode(prob) == PA_OK ? decode_state_bytes(*prob) : 0;
}

pa_status power_attn_decode_init(const pa_problem* prob, void* state, size_t state_bytes, void* hip_stream) {
    pa_status st = validate_decode(prob);
    if (st != PA_OK) return st;
    const size_t need = decode_state_bytes(*prob);
    if (need == 0) return PA_ERR_UNSUPPORTED;
    if (state == nullptr || state_bytes < need) return PA_ERR_WORKSPACE;
    return decode_init(*prob, state, (hipStream_t)hip_stream);
}

size_t power_attn_decode_absorb_workspace_bytes(const pa_problem* prob) {
    return validate_decode(prob) == PA_OK && prob->T > 0 ? decode_absorb_workspace_bytes(*prob) : 0;
}

pa_status power_attn_decode_absorb(const pa_problem* prob, const void* K, const void* V, const float* log_g, void* state,
                                   size_t state_bytes, void* workspace, size_t workspace_bytes, void* hip_stream) {
    pa_status st = validate_decode(prob);
    if (st != PA_OK) return st;
    if (prob->T <= 0 || K == nullptr || V == nullptr) return PA_ERR_INVALID_ARG;
    if ((prob->gated != 0) != (log_g != nullptr)) return PA_ERR_INVALID_ARG;
    const size_t need = decode_state_bytes(*prob);
    if (need == 0) return PA_ERR_UNSUPPORTED;
    if (state == nullptr || state_bytes < need) return PA_ERR_WORKSPACE;
    if (!aligned16(K) || !aligned16(V) || !aligned16(state)) return PA_ERR_INVALID_ARG;
    if (workspace != nullptr && ((uintptr_t)workspace & 255u) != 0) return PA_ERR_WORKSPACE;
    return decode_absorb(*prob, K, V, log_g, state, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

pa_status power_attn_decode_step(const pa_problem* prob, const void* q, const void* k, const void* v, const float* log_g,
                                 void* state, size_t state_bytes, void* o, float* z, void* hip_stream) {
    pa_status st = validate_decode(prob);
    if (st != PA_OK) return st;
    if (q == nullptr || k == nullptr || v == nullptr || o == nullptr) return PA_ERR_INVALID_ARG;
    if ((prob->gated != 0) != (log_g != nullptr)) return PA_ERR_INVALID_ARG;
    const size_t need = decode_state_bytes(*prob);
    if (need == 0) return PA_ERR_UNSUPPORTED;
    if (state == nullptr || state_bytes < need) return PA_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(state)) return PA_ERR_INVALID_ARG;
    return decode_step(*prob, q, k, v, log_g, state, o, z, (hipStream_t)hip_stream);
}

int power_attn_resolved_chunk(const pa_problem* prob) {
    if (validate(prob) != PA_OK) return 0;
    return resolved(prob).chunk;
}

pa_status power_attn_fwd(const pa_problem* prob, const void* Q, const void* K, const void* V, void* O, float* Z,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run_fwd(prob, Q, K, V, nullptr, O, Z, workspace, workspace_bytes, hip_stream, 0);
}

size_t power_attn_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

pa_status power_attn_fwd_static(const pa_problem* prob, const void* Q, const void* K, const void* V, void* O, float* Z,
                                void* hip_stream) {
    if (power_attn_workspace_bytes(prob, 0) > STATIC_SCRATCH_BYTES) return PA_ERR_WORKSPACE;
    void* ptr = nullptr;
    pa_status st = static_scratch(&ptr);
    if (st != PA_OK) return st;
    // every kernel family fully writes what it later reads of its workspace, so what the last call
    // left in the array needs no clearing
    return run_fwd(prob, Q, K, V, nullptr, O, Z, ptr, STATIC_SCRATCH_BYTES, hip_stream, 0);
}

pa_status power_attn_bwd(const pa_problem* prob, const void* Q, const void* K, const void* V, const void* O,
                         const float* Z, const void* dO, void* dQ, void* dK, void* dV, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
    return run_bwd(prob, Q, K, V, nullptr, O, Z, dO, dQ, dK, dV, nullptr, workspace, workspace_bytes, hip_stream, 0);
}

pa_status power_attn_fwd_gated(const pa_problem* prob, const void* Q, const void* K, const void* V, const float* log_g,
                               void* O, float* Z, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run_fwd(prob, Q, K, V, log_g, O, Z, workspace, workspace_bytes, hip_stream, 1);
}

pa_status power_attn_bwd_gated(const pa_problem* prob, const void* Q, const void* K, const void* V, const float* log_g,
                               const void* O, const float* Z, const void* dO, void* dQ, void* dK, void* dV, float* dlog_g,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run_bwd(prob, Q, K, V, log_g, O, Z, dO, dQ, dK, dV, dlog_g, workspace, workspace_bytes, hip_stream, 1);
}

const char* power_attn_last_hip_error(void) { return g_last_error; }

void power_attn_release_thread(void) { mfma_release_side_stream(); }

pa_status power_attn_profile_begin(void) {
    for (auto& r : g_records) {
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    g_records.clear();
    g_profile = true;
    return PA_OK;
}

pa_status power_attn_profile_end(pa_kernel_time* out, int max_entries, int* n) {
    g_profile = false;
    if (n == nullptr || (out == nullptr && max_entries > 0)) return PA_ERR_INVALID_ARG;
    int filled = 0;
    pa_status st = PA_OK;
    for (auto& r : g_records) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) {
            st = PA_ERR_HIP;
            continue;
        }
        int k = 0;
        for (; k < filled; ++k)
            if (r.name == out[k].name) break;
        if (k == filled) {
            if (filled >= max_entries) continue;
            memset(&out[k], 0, sizeof(out[k]));
            strncpy(out[k].name, r.name.c_str(), sizeof(out[k].name) - 1);
            ++filled;
        }
        out[k].launches += 1;
        out[k].ms_total += ms;
    }
    for (auto& r : g_records) {
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    g_records.clear();
    *n = filled;
    return st;
}

}  // extern "C"
