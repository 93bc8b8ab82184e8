// C ABI of libdsla: argument checks, planning and dispatch.  Declarations and the contract
// of every entry point are in include/dsla.h.
#include <mutex>
#include <vector>

#include "dsla_internal.h"

namespace dsla {
namespace {

thread_local const char *g_last_hip_error = "";

dsla_status hip_status(hipError_t e)
{
    if (e == hipSuccess) return DSLA_OK;
    g_last_hip_error = hipGetErrorString(e);
    return DSLA_ERR_HIP;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

dsla_status check_desc(const dsla_desc *d)
{
    if (!d) return DSLA_ERR_NULL;
    if (d->B <= 0 || d->H <= 0 || d->d_k <= 0 || d->d_v <= 0) return DSLA_ERR_SHAPE;
    if (d->chunk < 0 || d->segments < 0) return DSLA_ERR_SHAPE;
    if ((d->io_dtype != DSLA_F32 && d->io_dtype != DSLA_BF16) ||
        (d->gate_dtype != DSLA_F32 && d->gate_dtype != DSLA_BF16))
        return DSLA_ERR_UNSUPPORTED;
    if (d->gate_mode != DSLA_GATE_LOG && d->gate_mode != DSLA_GATE_PREACT) return DSLA_ERR_UNSUPPORTED;
    if (d->gate_mode == DSLA_GATE_PREACT && !(d->tau > 0.f && d->tau < 3.0e38f)) return DSLA_ERR_SHAPE;
    if (static_cast<int64_t>(d->B) * d->H > 0x7fffffffLL / 8) return DSLA_ERR_SHAPE;
    if (!decode_supported(*d)) return DSLA_ERR_UNSUPPORTED;  // d_k = d_v in {64, 128}
    return DSLA_OK;
}

// ---- kernel timing --------------------------------------------------------------------------
struct Profiler {
    std::mutex mu;
    bool enabled = false;
    std::vector<hipEvent_t> ev;  // 2 per record
    std::vector<int> ids;
    int max_records = 0;
} g_prof;

}  // namespace

void profile_reserve(int kernel_id, hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_prof.enabled) return;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (static_cast<int>(g_prof.ids.size()) >= g_prof.max_records) return;
    const size_t r = g_prof.ids.size();
    *start = g_prof.ev[2 * r];
    *stop = g_prof.ev[2 * r + 1];
    g_prof.ids.push_back(kernel_id);
}

}  // namespace dsla

using namespace dsla;

extern "C" {

const char *dsla_status_string(dsla_status s)
{
    switch (s) {
    case DSLA_OK: return "ok";
    case DSLA_ERR_NULL: return "required pointer is NULL";
    case DSLA_ERR_SHAPE: return "bad size or misaligned pointer";
    case DSLA_ERR_UNSUPPORTED: return "shape, chunk or dtype combination not supported";
    case DSLA_ERR_WORKSPACE: return "workspace missing or too small";
    case DSLA_ERR_HIP: return "HIP call failed";
    }
    return "unknown status";
}

const char *dsla_last_hip_error(void) { return g_last_hip_error; }

dsla_status dsla_state_init(const dsla_desc *desc, float *S1, float *S2, void *stream)
{
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (!S1 || !S2) return DSLA_ERR_NULL;
    if (!aligned16(S1) || !aligned16(S2)) return DSLA_ERR_SHAPE;
    const size_t n = static_cast<size_t>(desc->B) * desc->H * desc->d_k * desc->d_v;
    return hip_status(launch_state_init(S1, S2, n, static_cast<hipStream_t>(stream)));
}

size_t dsla_prefill_workspace_bytes(const dsla_desc *desc, int64_t T)
{
    if (check_desc(desc) != DSLA_OK || T <= 0) return 0;
    PrefillPlan plan;
    if (!prefill_plan(*desc, T, &plan)) return 0;
    return plan.ws_total_bytes;
}

dsla_status dsla_prefill(const dsla_desc *desc, int64_t T, const void *q, const void *k, const void *v,
                         const void *g1, const void *g2, float *S1, float *S2, void *o, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (T < 0) return DSLA_ERR_SHAPE;
    if (!S1 || !S2) return DSLA_ERR_NULL;
    if (T == 0) return DSLA_OK;
    if (!q || !k || !v || !g1 || !g2 || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g1) || !aligned16(g2) || !aligned16(o) ||
        !aligned16(S1) || !aligned16(S2))
        return DSLA_ERR_SHAPE;
    if (T > (int64_t(1) << 40)) return DSLA_ERR_SHAPE;
    PrefillPlan plan;
    if (!prefill_plan(*desc, T, &plan)) return DSLA_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(desc->B) * desc->H * plan.segments > 0x7fffffffLL) return DSLA_ERR_SHAPE;
    if (plan.ws_total_bytes > 0) {
        if (!workspace || workspace_bytes < plan.ws_total_bytes) return DSLA_ERR_WORKSPACE;
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return DSLA_ERR_SHAPE;
    }
    return hip_status(launch_prefill(*desc, plan, T, nullptr, nullptr, nullptr, q, k, v, g1, g2, S1, S2, o, workspace,
                                     static_cast<hipStream_t>(stream)));
}

namespace {
// Built-in prefill workspace for callers that cannot allocate.  One copy per device, part of the loaded code
// object; its device address is looked up once per device (the name below is only a host-side handle).
constexpr size_t kStaticWorkspaceBytes = DSLA_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, or null before the first call there

hipError_t static_workspace(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

namespace {
dsla_status check_varlen(const dsla_desc *desc, int64_t total_T, int64_t max_T)
{
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (total_T < 0 || max_T < 0 || max_T > total_T || total_T > 0x7fffffffLL) return DSLA_ERR_SHAPE;
    return DSLA_OK;
}
}  // namespace

dsla_status dsla_prefill_static_ws(const dsla_desc *desc, int64_t T, const void *q, const void *k, const void *v,
                                   const void *g1, const void *g2, float *S1, float *S2, void *o, void *stream)
{
    // the size check comes first: a plan that does not fit is an argument error and touches nothing
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (T < 0) return DSLA_ERR_SHAPE;
    const size_t need = T > 0 ? dsla_prefill_workspace_bytes(desc, T) : 0;
    if (need > kStaticWorkspaceBytes) return DSLA_ERR_WORKSPACE;
    void *ws = nullptr;
    if (need > 0) {
        const hipError_t e = static_workspace(&ws);
        if (e != hipSuccess) return hip_status(e);
    }
    return dsla_prefill(desc, T, q, k, v, g1, g2, S1, S2, o, ws, need, stream);
}

size_t dsla_prefill_varlen_workspace_bytes(const dsla_desc *desc, int64_t total_T, int64_t max_T)
{
    if (check_varlen(desc, total_T, max_T) != DSLA_OK || max_T == 0) return 0;
    PrefillPlan plan;
    if (!prefill_plan_varlen(*desc, total_T, max_T, &plan)) return 0;
    return plan.ws_total_bytes;
}

dsla_status dsla_prefill_varlen(const dsla_desc *desc, int64_t total_T, int64_t max_T, const int32_t *cu_seqlens,
                                const int32_t *seq_index, const int32_t *state_slot, const void *q, const void *k, const void *v,
                                const void *g1, const void *g2, float *S1, float *S2, void *o, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    dsla_status st = check_varlen(desc, total_T, max_T);
    if (st != DSLA_OK) return st;
    if (!S1 || !S2 || !cu_seqlens) return DSLA_ERR_NULL;
    if (total_T == 0 || max_T == 0) return DSLA_OK;
    if (!q || !k || !v || !g1 || !g2 || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g1) || !aligned16(g2) || !aligned16(o) ||
        !aligned16(S1) || !aligned16(S2) || (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) ||
        (reinterpret_cast<uintptr_t>(seq_index) & 3u) || (reinterpret_cast<uintptr_t>(state_slot) & 3u))
        return DSLA_ERR_SHAPE;
    PrefillPlan plan;
    if (!prefill_plan_varlen(*desc, total_T, max_T, &plan)) return DSLA_ERR_UNSUPPORTED;
    if (plan.max_items * desc->H > 0x7fffffffLL) return DSLA_ERR_SHAPE;   // one workgroup per (segment, head)
    if (plan.ws_total_bytes > 0) {
        if (!workspace || workspace_bytes < plan.ws_total_bytes) return DSLA_ERR_WORKSPACE;
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return DSLA_ERR_SHAPE;
    }
    return hip_status(launch_prefill(*desc, plan, max_T, cu_seqlens, seq_index, state_slot, q, k, v, g1, g2, S1, S2, o,
                                     workspace, static_cast<hipStream_t>(stream)));
}

dsla_status dsla_decode(const dsla_desc *desc, const void *q, const void *k, const void *v, const void *g1,
                        const void *g2, float *S1, float *S2, void *o, void *stream)
{
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (!q || !k || !v || !g1 || !g2 || !S1 || !S2 || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g1) || !aligned16(g2) || !aligned16(o) ||
        !aligned16(S1) || !aligned16(S2))
        return DSLA_ERR_SHAPE;
    return hip_status(launch_decode(*desc, q, k, v, g1, g2, nullptr, nullptr, S1, S2, o, static_cast<hipStream_t>(stream)));
}

dsla_status dsla_decode_slots(const dsla_desc *desc, const void *q, const void *k, const void *v, const void *g1,
                              const void *g2, const int32_t *row_index, const int32_t *state_slot, float *S1,
                              float *S2, void *o, void *stream)
{
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (!q || !k || !v || !g1 || !g2 || !state_slot || !S1 || !S2 || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g1) || !aligned16(g2) || !aligned16(o) ||
        !aligned16(S1) || !aligned16(S2) || (reinterpret_cast<uintptr_t>(state_slot) & 3u) ||
        (reinterpret_cast<uintptr_t>(row_index) & 3u))
        return DSLA_ERR_SHAPE;
    return hip_status(launch_decode(*desc, q, k, v, g1, g2, row_index, state_slot, S1, S2, o,
                                    static_cast<hipStream_t>(stream)));
}

namespace {
// Argument checks shared by the calls for N states; fills the by-value pointer block.
dsla_status check_multi(const dsla_desc *desc, const dsla_multi *m, bool with_beta, MultiStatePtrs *mp, int *Hkv)
{
    dsla_status st = check_desc(desc);
    if (st != DSLA_OK) return st;
    if (!m || !m->g_alpha || !m->S || !m->weights) return DSLA_ERR_NULL;
    if (m->n_states < 1 || m->n_states > DSLA_MAX_STATES || m->H_kv < 0) return DSLA_ERR_SHAPE;
    *Hkv = m->H_kv ? m->H_kv : desc->H;
    if (*Hkv > desc->H || desc->H % *Hkv != 0) return DSLA_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(m->weights_per_head) & 3u) return DSLA_ERR_SHAPE;
    for (int n = 0; n < DSLA_MAX_STATES; ++n) {
        mp->ga[n] = mp->gb[n] = nullptr;
        mp->S[n] = nullptr;
        mp->w[n] = 0.f;
    }
    for (int n = 0; n < m->n_states; ++n) {
        if (!m->g_alpha[n] || !m->S[n]) return DSLA_ERR_NULL;
        const void *gb = m->g_beta ? m->g_beta[n] : nullptr;
        if (gb && !with_beta) return DSLA_ERR_UNSUPPORTED;
        if (!aligned16(m->g_alpha[n]) || !aligned16(m->S[n]) || !aligned16(gb)) return DSLA_ERR_SHAPE;
        for (int n2 = 0; n2 < n; ++n2)
            if (m->S[n2] == m->S[n]) return DSLA_ERR_SHAPE;   // two states in one buffer
        mp->ga[n] = m->g_alpha[n];
        mp->gb[n] = gb;
        mp->S[n] = m->S[n];
        mp->w[n] = m->weights[n];
    }
    return DSLA_OK;
}
}  // namespace

dsla_status dsla_decode_multi(const dsla_desc *desc, const dsla_multi *multi, const void *q, const void *k,
                              const void *v, void *o, void *stream)
{
    MultiStatePtrs mp;
    int Hkv = 0;
    dsla_status st = check_multi(desc, multi, true, &mp, &Hkv);
    if (st != DSLA_OK) return st;
    if (!q || !k || !v || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return DSLA_ERR_SHAPE;
    return hip_status(launch_decode_multi(*desc, mp, multi->n_states, Hkv, multi->weights_per_head, q, k, v, nullptr,
                                          nullptr, o, static_cast<hipStream_t>(stream)));
}

size_t dsla_prefill_multi_workspace_bytes(const dsla_desc *desc, const dsla_multi *multi, int64_t T)
{
    if (check_desc(desc) != DSLA_OK || !multi || multi->n_states < 1 || multi->n_states > DSLA_MAX_STATES || T <= 0)
        return 0;
    PrefillPlan plan;
    if (!prefill_plan(*desc, T, &plan)) return 0;
    // an odd state out runs beside an idle partner, whose states live behind the plan's own scratch (reserved whatever
    // the parity of the states that pair up: which of them carry a beta gate is not part of the size query's contract)
    const size_t partner = plan.state_elems * sizeof(float);
    return (plan.ws_total_bytes + 255) / 256 * 256 + partner;
}

dsla_status dsla_prefill_multi(const dsla_desc *desc, const dsla_multi *multi, int64_t T, const void *q, const void *k,
                               const void *v, void *o, void *workspace, size_t workspace_bytes, void *stream)
{
    MultiStatePtrs mp;
    int Hkv = 0;
    dsla_status st = check_multi(desc, multi, true, &mp, &Hkv);
    if (st != DSLA_OK) return st;
    if (T < 0 || T > (int64_t(1) << 40)) return DSLA_ERR_SHAPE;
    if (T == 0) return DSLA_OK;
    if (!q || !k || !v || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return DSLA_ERR_SHAPE;
    PrefillPlan plan;
    if (!prefill_plan(*desc, T, &plan)) return DSLA_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(desc->B) * desc->H * plan.segments > 0x7fffffffLL) return DSLA_ERR_SHAPE;
    const size_t need = dsla_prefill_multi_workspace_bytes(desc, multi, T);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return DSLA_ERR_WORKSPACE;
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return DSLA_ERR_SHAPE;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int N = multi->n_states;
    float *partner = reinterpret_cast<float *>(static_cast<char *>(workspace) + (plan.ws_total_bytes + 255) / 256 * 256);
    const float *wph = multi->weights_per_head;
    // states without a beta gate go through the kernels two at a time, a state with one on its own (beta mode)
    int plain[DSLA_MAX_STATES], n_plain = 0, gated[DSLA_MAX_STATES], n_gated = 0;
    for (int n = 0; n < N; ++n) (mp.gb[n] ? gated[n_gated++] : plain[n_plain++]) = n;
    int launches = 0;
    for (int at = 0; at < n_plain; at += 2) {
        const int n = plain[at];
        const bool pair = at + 1 < n_plain;
        const int n2 = pair ? plain[at + 1] : n;
        PrefillExt ext;
        ext.Hkv = Hkv;
        ext.accumulate = launches++ > 0;
        ext.beta = 0;
        ext.wa = mp.w[n];
        ext.wb = pair ? mp.w[n2] : 0.f;
        ext.wa_per_head = wph ? wph + static_cast<size_t>(n) * desc->H : nullptr;
        ext.wb_per_head = (wph && pair) ? wph + static_cast<size_t>(n2) * desc->H : nullptr;
        float *Sb = pair ? mp.S[n2] : partner;   // the idle partner follows the gates of its neighbour
        if (!pair && !desc->zero_init) {
            // the idle partner starts from zero and its blend coefficient is zero: it stays finite and adds nothing
            hipError_t e = launch_state_init(partner, partner + plan.state_elems / 2, plan.state_elems / 2, s);
            if (e != hipSuccess) return hip_status(e);
        }
        hipError_t e = launch_prefill(*desc, plan, T, nullptr, nullptr, nullptr, q, k, v, mp.ga[n], mp.ga[n2], mp.S[n], Sb, o,
                                      workspace, s, &ext);
        if (e != hipSuccess) return hip_status(e);
    }
    for (int at = 0; at < n_gated; ++at) {
        const int n = gated[at];
        PrefillExt ext;
        ext.Hkv = Hkv;
        ext.accumulate = launches++ > 0;
        ext.beta = 1;
        ext.wa = mp.w[n];
        ext.wb = 0.f;
        ext.wa_per_head = wph ? wph + static_cast<size_t>(n) * desc->H : nullptr;
        ext.wb_per_head = nullptr;
        hipError_t e = launch_prefill(*desc, plan, T, nullptr, nullptr, nullptr, q, k, v, mp.ga[n], mp.gb[n], mp.S[n], mp.S[n], o,
                                      workspace, s, &ext);
        if (e != hipSuccess) return hip_status(e);
    }
    return DSLA_OK;
}

size_t dsla_attention_entropy_workspace_bytes(int32_t B, int32_t H, int32_t d, int64_t T)
{
    EntropyPlan plan;
    if (B <= 0 || H <= 0 || T <= 0 || !entropy_plan(B, H, d, T, &plan)) return 0;
    return plan.ws_bytes;
}

dsla_status dsla_attention_entropy(int32_t B, int32_t H, int32_t d, int64_t T, int32_t io_dtype, float scale,
                                   const void *q_last, const void *k, float *entropy, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    if (B <= 0 || H <= 0 || d <= 0 || T <= 0 || T > 0x7fffffffLL) return DSLA_ERR_SHAPE;
    if (static_cast<int64_t>(B) * H > 0x7fffffffLL / 1024) return DSLA_ERR_SHAPE;
    if (io_dtype != DSLA_F32 && io_dtype != DSLA_BF16) return DSLA_ERR_UNSUPPORTED;
    EntropyPlan plan;
    if (!entropy_plan(B, H, d, T, &plan)) return DSLA_ERR_UNSUPPORTED;
    if (!q_last || !k || !entropy) return DSLA_ERR_NULL;
    if (!aligned16(q_last) || !aligned16(k) || (reinterpret_cast<uintptr_t>(entropy) & 3u)) return DSLA_ERR_SHAPE;
    if (plan.ws_bytes > 0) {
        if (!workspace || workspace_bytes < plan.ws_bytes) return DSLA_ERR_WORKSPACE;
        if (!aligned16(workspace)) return DSLA_ERR_SHAPE;
    }
    return hip_status(launch_entropy(B, H, d, T, io_dtype, plan, scale, q_last, k, entropy, workspace,
                                     static_cast<hipStream_t>(stream)));
}

size_t dsla_attention_decode_workspace_bytes(int32_t B, int32_t H, int32_t d, int64_t T)
{
    EntropyPlan plan;
    if (B <= 0 || H <= 0 || T <= 0 || !entropy_plan(B, H, d, T, &plan, 2 + d)) return 0;
    return plan.ws_bytes;
}

dsla_status dsla_attention_decode(int32_t B, int32_t H, int32_t d, int64_t T, int32_t io_dtype, float scale,
                                  const void *q, const void *k, const void *v, const int32_t *seq_lens, void *o,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (B <= 0 || H <= 0 || d <= 0 || T <= 0 || T > 0x7fffffffLL) return DSLA_ERR_SHAPE;
    if (static_cast<int64_t>(B) * H > 0x7fffffffLL / 1024) return DSLA_ERR_SHAPE;
    if (io_dtype != DSLA_F32 && io_dtype != DSLA_BF16) return DSLA_ERR_UNSUPPORTED;
    EntropyPlan plan;
    if (!entropy_plan(B, H, d, T, &plan, 2 + d)) return DSLA_ERR_UNSUPPORTED;
    if (!q || !k || !v || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || (reinterpret_cast<uintptr_t>(seq_lens) & 3u))
        return DSLA_ERR_SHAPE;
    if (plan.ws_bytes > 0) {
        if (!workspace || workspace_bytes < plan.ws_bytes) return DSLA_ERR_WORKSPACE;
        if (!aligned16(workspace)) return DSLA_ERR_SHAPE;
    }
    return hip_status(launch_attn_decode(B, H, d, T, io_dtype, plan, scale, q, k, v, seq_lens, o, workspace,
                                         static_cast<hipStream_t>(stream)));
}

dsla_status dsla_project(int64_t M, int32_t K, int32_t n_out, int32_t width, const void *x, const void *W,
                         const float *bias, void *const *outs, void *stream)
{
    if (M <= 0 || K <= 0 || n_out <= 0 || width <= 0) return DSLA_ERR_SHAPE;
    if (n_out > DSLA_MAX_PROJECTIONS || K % 32 != 0 || K > (1 << 21) || width % 128 != 0) return DSLA_ERR_UNSUPPORTED;   // 32-bit byte offsets inside a tile
    if ((M + 127) / 128 * (static_cast<int64_t>(n_out) * width / 128) > 0x7ffffff0LL) return DSLA_ERR_SHAPE;
    if (!x || !W || !outs) return DSLA_ERR_NULL;
    if (!aligned16(x) || !aligned16(W) || !aligned16(bias)) return DSLA_ERR_SHAPE;
    for (int j = 0; j < n_out; ++j) {
        if (!outs[j]) return DSLA_ERR_NULL;
        if (!aligned16(outs[j])) return DSLA_ERR_SHAPE;
    }
    return hip_status(launch_project(M, K, n_out, width, x, W, bias, outs, static_cast<hipStream_t>(stream)));
}

dsla_status dsla_attention_prefill(int32_t B, int32_t H, int32_t d, int64_t T, int32_t io_dtype, float scale,
                                   const void *q, const void *k, const void *v, void *o, void *stream)
{
    if (B <= 0 || H <= 0 || d <= 0 || T <= 0 || T > 0x7fff0000LL) return DSLA_ERR_SHAPE;   // token indices are 32-bit in the kernel
    if (io_dtype != DSLA_BF16 || (d != 64 && d != 128)) return DSLA_ERR_UNSUPPORTED;
    if (T * H * d * 2 > 0xffffffffLL) return DSLA_ERR_SHAPE;   // byte offsets inside one sequence are 32-bit (buffer loads)
    if (static_cast<int64_t>(B) * H * ((T + 127) / 128) > 0x7fffffffLL) return DSLA_ERR_SHAPE;   // one workgroup per 128 queries
    if (!q || !k || !v || !o) return DSLA_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return DSLA_ERR_SHAPE;
    return hip_status(launch_attn_prefill(B, H, d, T, scale, q, k, v, o, static_cast<hipStream_t>(stream)));
}

dsla_status dsla_profile_enable(int enable, int max_records)
{
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof.ev.clear();
    g_prof.ids.clear();
    g_prof.enabled = false;
    g_prof.max_records = 0;
    if (!enable) return DSLA_OK;
    if (max_records <= 0) return DSLA_ERR_SHAPE;
    g_prof.ev.resize(2 * static_cast<size_t>(max_records));
    for (auto &e : g_prof.ev) {
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) return hip_status(err);
    }
    g_prof.ids.reserve(max_records);
    g_prof.max_records = max_records;
    g_prof.enabled = true;
    return DSLA_OK;
}

dsla_status dsla_profile_collect(double *total_ms, int64_t *launches)
{
    if (!total_ms || !launches) return DSLA_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (int i = 0; i < DSLA_KERNEL_COUNT; ++i) {
        total_ms[i] = 0.0;
        launches[i] = 0;
    }
    const size_t n = g_prof.ids.size();
    for (size_t r = 0; r < n; ++r) {
        hipError_t err = hipEventSynchronize(g_prof.ev[2 * r + 1]);
        if (err != hipSuccess) return hip_status(err);
        float ms = 0.f;
        err = hipEventElapsedTime(&ms, g_prof.ev[2 * r], g_prof.ev[2 * r + 1]);
        if (err != hipSuccess) return hip_status(err);
        const int id = g_prof.ids[r];
        if (id >= 0 && id < DSLA_KERNEL_COUNT) {
            total_ms[id] += ms;
            launches[id] += 1;
        }
    }
    g_prof.ids.clear();
    return DSLA_OK;
}

}  // extern "C"
