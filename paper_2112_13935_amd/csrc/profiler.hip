// Per-launch kernel timing with HIP event pairs on the launch stream.
#include "aet_internal.h"

namespace aet {

const char *family_name(int fam) {
    static const char *names[F_COUNT] = {
        "k_begin_round", "k_gather", "k_dense_fwd", "k_dense_bwd_data", "k_dense_bwd_weight",
        "k_conv_fwd", "k_conv_bwd_data", "k_conv_bwd_weight", "k_pool_fwd", "k_pool_bwd",
        "k_softmax_ce", "server_reduce", "k_softmax_round", "k_mlp_round", "k_apply_neighbour_U",
        "k_lenet_round"};
    return (fam >= 0 && fam < F_COUNT) ? names[fam] : "";
}

static hipEvent_t take_event(Profiler *p) {
    if (!p->pool.empty()) {
        hipEvent_t e = p->pool.back();
        p->pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    hipError_t st = hipEventCreate(&e);
    if (st != hipSuccess) { p->status = st; return nullptr; }
    return e;
}

void Profiler::before(int fam, hipStream_t s) {
    (void)fam;
    cur = take_event(this);
    if (cur) { hipError_t st = hipEventRecord(cur, s); if (st != hipSuccess) status = st; }
}

void Profiler::after(int fam, hipStream_t s) {
    hipEvent_t b = take_event(this);
    if (!cur || !b) return;
    hipError_t st = hipEventRecord(b, s);
    if (st != hipSuccess) status = st;
    pending.push_back({fam, cur, b});
    cur = nullptr;
    if (pending.size() >= 16384) (void)drain(s);
}

hipError_t Profiler::drain(hipStream_t s) {
    if (status != hipSuccess) return status;
    hipError_t st = hipStreamSynchronize(s);
    if (st != hipSuccess) return st;
    for (const Pair &p : pending) {
        float ms = 0.f;
        st = hipEventElapsedTime(&ms, p.a, p.b);
        if (st != hipSuccess) return st;
        total_ms[p.fam] += (double)ms;
        launches[p.fam] += 1;
        pool.push_back(p.a);
        pool.push_back(p.b);
    }
    pending.clear();
    return hipSuccess;
}

void Profiler::clear() {
    for (const Pair &p : pending) { pool.push_back(p.a); pool.push_back(p.b); }
    pending.clear();
}

Profiler::~Profiler() {
    clear();
    if (cur) pool.push_back(cur);
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
}

}  // namespace aet
