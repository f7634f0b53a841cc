// Host-only entry points of libd3tom: sizes, schedule, cost model, status names.
#include <math.h>
#include <mutex>
#include <vector>
#include "common.hpp"

namespace d3tom { namespace prof {
bool g_enabled = false;
namespace {
struct Rec { int kernel; hipEvent_t e0, e1; };
std::vector<Rec> g_recs;
std::mutex g_mu;
}
void mark_begin(int kernel, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_mu);
    Rec r; r.kernel = kernel; r.e0 = nullptr; r.e1 = nullptr;
    if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
    (void)hipEventRecord(r.e0, st);
    g_recs.push_back(r);
}
void mark_end(int kernel, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (size_t i = g_recs.size(); i-- > 0;)
        if (g_recs[i].kernel == kernel) { (void)hipEventRecord(g_recs[i].e1, st); return; }
}
}}  // namespace d3tom::prof

namespace d3tom {
size_t importance_ws_bytes(int B, int max_N, int max_V, int H, int dh, int max_D);
size_t merge_ws_bytes(int B, int max_V);
}

extern "C" int d3tom_keep_count(int V, double keep_ratio) {
    if (V < 1) return 0;
    double c = ceil(keep_ratio * (double)V - 1e-9);
    if (!(c >= 1.0)) c = 1.0;
    if (c > (double)V) c = (double)V;
    return (int)c;
}

extern "C" double d3tom_schedule(int step, int T, double r_first, double r_last) {
    if (T <= 1) return r_first;
    return r_first + (r_last - r_first) * ((double)step / (double)(T - 1));
}

// Section 4.3 / Appendix B.  layer(n) = 4 n d^2 + 2 n^2 d + 3 n d m.
extern "C" double d3tom_model_flops(double alpha, int l_star, int L, int T, int V, int P, int O, int d, int m) {
    const double dd = d, mm = m, N = (double)V + P + O;
    auto attn = [&](double n) { return 4.0 * n * dd * dd + 2.0 * n * n * dd; };
    auto ffn = [&](double n) { return 3.0 * n * dd * mm; };
    const double full = (double)L * (attn(N) + ffn(N));
    if (alpha <= 0.0) return (double)T * full;
    const double Nm = N - alpha * V;
    const double merge = 2.0 * alpha * (1.0 - alpha) * (double)V * V * dd + alpha * V * dd;
    const double step = l_star * (attn(N) + ffn(N)) + attn(N) + ffn(Nm) + (double)(L - l_star - 1) * (attn(Nm) + ffn(Nm)) + merge;
    return full + (double)(T - 1) * step;      // the first step has no deciders and runs unmerged
}

extern "C" size_t d3tom_workspace_bytes(int op, int B, int max_N, int max_V, int H, int dh, int max_D) {
    if (B < 1 || max_N < 1) return 0;
    switch (op) {
        case D3TOM_OP_IMPORTANCE: return d3tom::importance_ws_bytes(B, max_N, max_V < 1 ? 1 : max_V, H, dh, max_D < 1 ? 1 : max_D);
        case D3TOM_OP_SELECT_TOPK: return 256;
        case D3TOM_OP_MERGE: return d3tom::merge_ws_bytes(B, max_V < 1 ? 1 : max_V);
        case D3TOM_OP_ATTEND: return 256;
        default: return 0;
    }
}

extern "C" int d3tom_profile_enable(int on) {
    d3tom::prof::g_enabled = (on != 0);
    return D3TOM_OK;
}

extern "C" int d3tom_profile_kernel_count(void) { return d3tom::prof::NUM_KERNELS; }

extern "C" const char* d3tom_profile_kernel_name(int kernel) {
    static const char* names[] = {"imp_stats", "imp_scores", "imp_finish", "topk_select", "merge_norms",
                                  "cos_argmax", "merge_assign", "merge_scatter", "attend", "update_deciders", "cos_reduce",
                                  "linear", "rmsnorm", "rope", "stack_meta"};
    return (kernel >= 0 && kernel < d3tom::prof::NUM_KERNELS) ? names[kernel] : "";
}

extern "C" int d3tom_profile_collect(double* ms_sum, long long* calls, int n) {
    using namespace d3tom::prof;
    if (!ms_sum || !calls || n < NUM_KERNELS) return D3TOM_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    for (int i = 0; i < n; ++i) { ms_sum[i] = 0.0; calls[i] = 0; }
    int status = D3TOM_OK;
    for (auto& r : g_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
            ms_sum[r.kernel] += ms; calls[r.kernel] += 1;
        } else status = D3TOM_ERR_DEVICE;
        (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1);
    }
    g_recs.clear();
    return status;
}

extern "C" const char* d3tom_status_string(int status) {
    switch (status) {
        case D3TOM_OK: return "ok";
        case D3TOM_ERR_INVALID_ARG: return "invalid argument";
        case D3TOM_ERR_NO_DECIDERS: return "empty decider set: merge skipped";
        case D3TOM_ERR_WORKSPACE_TOO_SMALL: return "workspace too small or misaligned";
        case D3TOM_ERR_UNSUPPORTED: return "unsupported shape or type";
        case D3TOM_ERR_DEVICE: return "HIP launch failed";
        default: return "unknown status";
    }
}
