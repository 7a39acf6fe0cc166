// Optional per-launch timing with HIP events recorded on the caller's stream.
// Not thread-safe: one profiling session at a time, driven from one host thread.
#include "bra_common.h"

#include <vector>

namespace bra {

namespace {
struct Rec { int id; hipEvent_t a, b; };
std::vector<Rec> g_recs;
int g_used = 0;
bool g_on = false;

const char *const kNames[K_COUNT] = {
    "gen_pool", "gen_region_qk", "gen_affinity_topk", "gen_gemm_qkv", "gen_attention", "gen_lce_add",
    "gen_gemm_wo", "mfma_prep", "mfma_qkv", "mfma_attention", "mfma_pool_qk", "mfma_route_rows",
    "mfma_fused_k1", "mfma_attn_small", "mfma_lce_add", "mfma_wo",
    "block_pos_ln", "block_add_ln", "block_mlp_in", "block_mlp_out", "block_mlp_fused", "gen_backward",
};
}  // namespace

ProfScope::ProfScope(hipStream_t st, int id) : st_(st), slot_(-1)
{
    if (!g_on || g_used >= (int)g_recs.size()) return;
    slot_ = g_used++;
    g_recs[slot_].id = id;
    (void)hipEventRecord(g_recs[slot_].a, st_);
}

ProfScope::~ProfScope()
{
    if (slot_ >= 0) (void)hipEventRecord(g_recs[slot_].b, st_);
}

}  // namespace bra

using namespace bra;

extern "C" {

int bra_profile_begin(int max_records)
{
    if (g_on || max_records < 1) return BRA_ERR_SHAPE;
    g_recs.resize((size_t)max_records);
    for (auto &r : g_recs) {
        if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return BRA_ERR_LAUNCH;
    }
    g_used = 0;
    g_on = true;
    return BRA_OK;
}

int bra_profile_end(int32_t *ids, float *ms, int max_records, int *n_out)
{
    if (!g_on) return BRA_ERR_SHAPE;
    if (!n_out) return BRA_ERR_NULL;
    g_on = false;
    int n = 0, rc = BRA_OK;
    for (int i = 0; i < g_used; ++i) {
        float t = 0.f;
        if (hipEventSynchronize(g_recs[i].b) != hipSuccess ||
            hipEventElapsedTime(&t, g_recs[i].a, g_recs[i].b) != hipSuccess)
            rc = BRA_ERR_LAUNCH;
        if (n < max_records && ids && ms) { ids[n] = g_recs[i].id; ms[n] = t; ++n; }
    }
    for (auto &r : g_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_recs.clear();
    g_used = 0;
    *n_out = n;
    return rc;
}

const char *bra_kernel_name(int id) { return (id >= 0 && id < K_COUNT) ? kNames[id] : "unknown"; }

}  // extern "C"
