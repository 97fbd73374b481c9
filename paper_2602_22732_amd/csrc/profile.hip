// Optional per-kernel timing with HIP events on the stream the kernels run on.
// Off by default; when switched on, every kernel launch of the library is
// bracketed by two events.  Used by the benchmark to attribute time to kernels.
#include <vector>

#include "common.h"

namespace {
struct Record { hipEvent_t start, stop; int cls; double flops, bytes; };
bool g_on = false;
std::vector<Record> g_records;       // events in flight since the last read
std::vector<Record> g_pool;          // recycled event pairs
const size_t kMaxRecords = 1 << 16;
const char *kNames[KC_COUNT] = {"gemm_bf16_mfma_256x256", "gemm_bf16_mfma_128x128", "gemm_simple", "cross_attn_flash_bf16",
                                "cross_attn_simple", "self_attn_step", "trunk_self_attn", "rmsnorm", "fuse_gate", "select_rows",
                                "select_request", "gather_rows", "broadcast_rows", "v_transpose", "gemm_bf16_ring", "masked_softmax_rows",
                                "gemm_fp8_ring", "quantize_rows", "context_attn_flash_bf16"};
}  // namespace

ProfScope::ProfScope(int cls, hipStream_t st, double flops, double bytes) : idx_(-1), st_(st) {
    if (!g_on || g_records.size() >= kMaxRecords) return;
    Record r;
    if (!g_pool.empty()) {
        r = g_pool.back();
        g_pool.pop_back();
    } else {
        if (hipEventCreate(&r.start) != hipSuccess) return;
        if (hipEventCreate(&r.stop) != hipSuccess) {
            (void)hipEventDestroy(r.start);
            return;
        }
    }
    r.cls = cls;
    r.flops = flops;
    r.bytes = bytes;
    (void)hipEventRecord(r.start, st);
    g_records.push_back(r);
    idx_ = (int)g_records.size() - 1;
}

ProfScope::~ProfScope() {
    if (idx_ >= 0) (void)hipEventRecord(g_records[idx_].stop, st_);
}

extern "C" {

int gr4ad_profile_enable(int on) {
    g_on = on != 0;
    return GR4AD_OK;
}

int gr4ad_profile_kernel_count(void) { return KC_COUNT; }

const char *gr4ad_profile_kernel_name(int cls) { return (cls >= 0 && cls < KC_COUNT) ? kNames[cls] : ""; }

int gr4ad_profile_read(double *ms, double *flops, double *bytes, int64_t *launches, int reset) {
    if (!ms || !flops || !bytes || !launches) return GR4AD_EINVAL;
    for (int i = 0; i < KC_COUNT; i++) { ms[i] = 0; flops[i] = 0; bytes[i] = 0; launches[i] = 0; }
    for (const Record &r : g_records) {
        if (hipEventSynchronize(r.stop) != hipSuccess) return GR4AD_EHIP;
        float t = 0;
        if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) return GR4AD_EHIP;
        ms[r.cls] += t;
        flops[r.cls] += r.flops;
        bytes[r.cls] += r.bytes;
        launches[r.cls] += 1;
    }
    if (reset) {
        for (const Record &r : g_records) g_pool.push_back(r);
        g_records.clear();
    }
    return GR4AD_OK;
}

}  // extern "C"
