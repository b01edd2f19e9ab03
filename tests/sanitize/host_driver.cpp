// Drives the host-only parts of the library for a build with AddressSanitizer and
// UBSan: the time-cost model, and every argument check of the C ABI that returns before
// any HIP call (fake, well aligned, never dereferenced device addresses).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "cdsgd.h"
#include "cdsgd_cost_model.h"

int main()
{
    int bad = 0;
    float *A = reinterpret_cast<float *>(0x1000);
    uint32_t *P = reinterpret_cast<uint32_t *>(0x2000);
    bad += cdsgd_quantize_pack(nullptr, A, P, 16, 0.5f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_quantize_pack(A, A, P, 0, 0.5f, nullptr) != CDSGD_ERR_SIZE;
    bad += cdsgd_quantize_pack(A, A, P, 16, -1.0f, nullptr) != CDSGD_ERR_PARAM;
    bad += cdsgd_quantize_pack(A + 1, A, P, 16, 0.5f, nullptr) != CDSGD_ERR_ALIGN;
    const uint32_t *two[2] = {P, nullptr};
    bad += cdsgd_decode_sum(two, 2, A, 16, 0.5f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_decode_sum(two, 65, A, 16, 0.5f, nullptr) != CDSGD_ERR_WORKERS;
    bad += cdsgd_update(A, A, nullptr, A, 16, 0.1f, 0.1f, 2, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_update(A, A, A, A, 16, NAN, 0.1f, 2, nullptr) != CDSGD_ERR_PARAM;
    cdsgd_tensor t = {A, A, A, A, P, A, 0};
    cdsgd_plan *plan = nullptr;
    const uint32_t *row[1] = {P};
    const uint32_t *const *rows[2] = {nullptr, row};
    bad += cdsgd_plan_create(&t, 1, rows, 2, 0, &plan) != CDSGD_ERR_SIZE;   // n == 0
    t.n = (size_t)1 << 50;                                                   // too many chunks for one launch
    bad += cdsgd_plan_create(&t, 1, rows, 2, 0, &plan) != CDSGD_ERR_SIZE;
    t.n = 100;
    bad += cdsgd_plan_create(&t, 1, rows, 2, 5, &plan) != CDSGD_ERR_WORKERS;
    bad += cdsgd_plan_create(&t, 1, nullptr, 2, 0, &plan) != CDSGD_ERR_NULL;
    bad += cdsgd_step_fused(nullptr, 0, 1, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_step_warmup(nullptr, 0, 0, 0.1f, 0.1f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_packed_words(17) != 2;
    cdsgd_trainer *tr = nullptr;
    bad += cdsgd_trainer_create(reinterpret_cast<cdsgd_plan *>(A), 2, 4, 0.5f, 0.1f, 0.1f, &tr) != CDSGD_OK;
    bad += cdsgd_trainer_iteration(tr) != 0;
    bad += cdsgd_trainer_destroy(tr) != CDSGD_OK;
    // the entry point that allocates nothing: every check that comes before its first HIP call
    {
        float *B0 = reinterpret_cast<float *>(0x100000), *B1 = reinterpret_cast<float *>(0x200000);
        float *B2 = reinterpret_cast<float *>(0x300000), *B3 = reinterpret_cast<float *>(0x400000);
        uint32_t *B4 = reinterpret_cast<uint32_t *>(0x500000), *B5 = reinterpret_cast<uint32_t *>(0x600000);
        cdsgd_tensor u = {B0, B1, B2, B3, B4, nullptr, 1000};
        const uint32_t *urow[1] = {B5};
        const uint32_t *const *urows[2] = {nullptr, urow};
        bad += cdsgd_step_fused_static(nullptr, 1, urows, 2, 0, 0, 1, 4, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_NULL;
        bad += cdsgd_step_fused_static(&u, 1, urows, 2, 0, 9, 1, 4, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_PARAM;
        bad += cdsgd_step_fused_static(&u, 1, urows, 2, 0, 0, 1, 0, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_PARAM;
        bad += cdsgd_step_fused_static(&u, 1, urows, 2, 0, 0, 0, 4, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_NULL;  // no agg_full
        bad += cdsgd_step_fused_static(&u, 1, urows, 2, 3, 0, 1, 4, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_WORKERS;
        std::vector<cdsgd_tensor> many(CDSGD_STATIC_MAX_TENSORS + 1, u);
        std::vector<const uint32_t *> manyrow(many.size(), B5);
        const uint32_t *const *manyrows[2] = {nullptr, manyrow.data()};
        bad += cdsgd_step_fused_static(many.data(), (int)many.size(), manyrows, 2, 0, 0, 1, 4, 0.5f, 0.1f, 0.1f, nullptr) !=
               CDSGD_ERR_SIZE;
        u.w_local = B0 + 4;  // overlaps w_global
        bad += cdsgd_step_fused_static(&u, 1, urows, 2, 0, 0, 1, 4, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_ALIAS;
    }
    // sparse form: sizes and argument checks
    bad += cdsgd_sparse_segments(4097) != 2 || cdsgd_sparse_words(4097) != 528;
    bad += cdsgd_sparse_encode(nullptr, 16, P, nullptr, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_sparse_encode(P, 0, P + 4096, nullptr, nullptr) != CDSGD_ERR_SIZE;
    bad += cdsgd_sparse_encode(P, 64, P, nullptr, nullptr) != CDSGD_ERR_ALIAS;
    bad += cdsgd_decode_sum_sparse(two, 2, A, 16, 0.5f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_plan_set_peer_format(nullptr, CDSGD_PEERS_SPARSE) != CDSGD_ERR_NULL;
    bad += cdsgd_plan_set_max_workgroups(nullptr, 1) != CDSGD_ERR_NULL;
    bad += cdsgd_step_fused_range(nullptr, 0, 1, 1, 4, 0.5f, 0.1f, 0.1f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_step_local_range(nullptr, 0, 1, 0.1f, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_step_global_range(nullptr, 0, 1, 1, 4, 0.5f, 0.1f, nullptr) != CDSGD_ERR_NULL;
    {
        const float *rd[3] = {A, A + 4096, A + 8192};
        float *wr[3] = {A + 12288, A + 16384, A + 12288 + 4};
        bad += cdsgd_probe_streams(rd, 18, wr, 1, 1024, A, 0, nullptr) != CDSGD_ERR_PARAM;
        bad += cdsgd_probe_streams(rd, 3, wr, 0, 1024, nullptr, 0, nullptr) != CDSGD_ERR_NULL;
        bad += cdsgd_probe_streams(rd, 3, wr, 2, 1000, nullptr, 0, nullptr) != CDSGD_ERR_SIZE;
        bad += cdsgd_probe_streams(rd, 3, wr, 3, 1024, nullptr, 8192, nullptr) != CDSGD_ERR_ALIAS;
    }
    bad += cdsgd_plan_set_thresholds(nullptr, nullptr) != CDSGD_ERR_NULL;
    bad += cdsgd_build_id() == nullptr;
    cdsgd_cost_params p = {1.0, 5.0, 1.0, 0.5, 4};
    cdsgd_cost c;
    double sum = 0;
    for (long i = 0; i < 16; ++i) {
        bad += cdsgd_cost_iteration(&p, i, &c) != 0;
        sum += c.t_cd + c.save_vs_bit + c.save_vs_loc;
    }
    bad += cdsgd_cost_period_mean(&p, &c) != 0;
    bad += std::fabs(c.t_cd - 2.375) > 1e-12;
    std::printf("host driver: %d failed checks, sum %.3f\n", bad, sum);
    return bad ? 1 : 0;
}
