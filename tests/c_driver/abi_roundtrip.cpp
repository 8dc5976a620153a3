// A caller of libadacomp written against include/adacomp.h alone: no Python, no PyTorch.  Device
// memory comes from the HIP runtime; the expected results come from the CPU oracle, which is linked
// in as the checker.  Two learners, three steps of adacomp_compress_batch with one
// adacomp_unpack_accumulate per step, a single-learner adacomp_compress, then one
// adacomp_unpack_update, then two steps of adacomp_compress_batch_lazy and an adacomp_residue_sync;
// packets, residues, the dense sum and the updated weights must equal the
// oracle's byte for byte; last, two single-learner steps through adacomp_compress_static.  Built by tests/c_driver/build.py (called from the repository's build
// entry point), run by tests/test_gpu_parity.py::test_caller_written_in_c.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "adacomp.h"
#include "adacomp_oracle.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define LIB_OK(x) do { int r_ = (x); if (r_ != ADACOMP_OK) { std::printf("libadacomp error %d (%s) at line %d\n", r_, adacomp_strerror(r_), __LINE__); return 3; } } while (0)

// a small counter-based generator: values in (-1, 1) * scale, one in 64 exactly zero
static float draw(uint64_t key, float scale)
{
    key ^= key >> 33; key *= 0xff51afd7ed558ccdull; key ^= key >> 33; key *= 0xc4ceb9fe1a85ec53ull; key ^= key >> 33;
    if ((key & 63u) == 0u) return 0.0f;
    const double u = double(key >> 11) / double(1ull << 53);
    return float((2.0 * u - 1.0) * scale);
}

int main()
{
    const uint32_t n_layers = 4, n_learners = 2, n_steps = 3;
    const adacomp_layer_t table[n_layers] = {{0, 50 * 131 + 17, 50, 0}, {6568, 500 * 77 + 123, 500, 0},
                                             {45192, 4097 * 3 + 5, 4097, 0}, {57488, 64 * 200, 64, 0}};
    adacomp_oracle_layer_t otable[n_layers];
    for (uint32_t l = 0; l < n_layers; ++l) otable[l] = adacomp_oracle_layer_t{table[l].elem_offset, table[l].n_elems, table[l].L_T, 0};
    const size_t n_total = 57488 + 64 * 200;
    const size_t bound = adacomp_packet_bound(table, n_layers);
    const size_t ws_bytes = adacomp_workspace_bytes_batch(table, n_layers, n_learners);
    if (!bound || !ws_bytes || bound != adacomp_oracle_packet_bound(otable, n_layers)) { std::printf("size queries disagree\n"); return 1; }

    void *ws = nullptr;
    float *d_grad[n_learners], *d_res[n_learners], *d_dense = nullptr, *d_w = nullptr, *d_m = nullptr;
    void *d_pk[n_learners];
    HIP_OK(hipMalloc(&ws, ws_bytes));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_dense), n_total * 4));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_w), n_total * 4));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_m), n_total * 4));
    for (uint32_t k = 0; k < n_learners; ++k) {
        HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_grad[k]), n_total * 4));
        HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_res[k]), n_total * 4));
        HIP_OK(hipMalloc(&d_pk[k], bound));
        HIP_OK(hipMemset(d_res[k], 0, n_total * 4));
    }
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    LIB_OK(adacomp_workspace_init(table, n_layers, ws, ws_bytes, stream));

    std::vector<std::vector<float>> grad(n_learners, std::vector<float>(n_total)), res(n_learners, std::vector<float>(n_total, 0.f));
    std::vector<std::vector<uint8_t>> want_pk(n_learners, std::vector<uint8_t>(bound)), got_pk(n_learners, std::vector<uint8_t>(bound));
    std::vector<float> want_dense(n_total), got(n_total);
    long long pk_bytes[n_learners];
    for (uint32_t t = 0; t < n_steps; ++t) {
        for (uint32_t k = 0; k < n_learners; ++k) {
            for (size_t i = 0; i < n_total; ++i) grad[k][i] = draw((uint64_t(t) << 40) | (uint64_t(k) << 32) | i, i % 7 == 0 ? 0.5f : 0.01f);
            HIP_OK(hipMemcpy(d_grad[k], grad[k].data(), n_total * 4, hipMemcpyHostToDevice));
            std::memset(want_pk[k].data(), 0, bound);
            pk_bytes[k] = adacomp_oracle_compress(otable, n_layers, grad[k].data(), res[k].data(), want_pk[k].data(), bound, 0, 2.0f);
            if (pk_bytes[k] <= 0) { std::printf("oracle compress failed: %lld\n", pk_bytes[k]); return 1; }
        }
        const float *grads[n_learners] = {d_grad[0], d_grad[1]};
        float *residues[n_learners] = {d_res[0], d_res[1]};
        LIB_OK(adacomp_compress_batch(table, n_layers, n_learners, grads, residues, d_pk, bound, ws, ws_bytes, stream));
        const void *packets[n_learners] = {d_pk[0], d_pk[1]};
        LIB_OK(adacomp_unpack_accumulate(table, n_layers, packets, n_learners, d_dense, ws, ws_bytes, stream));
        HIP_OK(hipStreamSynchronize(stream));
        for (uint32_t k = 0; k < n_learners; ++k) {
            HIP_OK(hipMemcpy(got_pk[k].data(), d_pk[k], size_t(pk_bytes[k]), hipMemcpyDeviceToHost));
            if (std::memcmp(got_pk[k].data(), want_pk[k].data(), size_t(pk_bytes[k])) != 0) { std::printf("step %u learner %u: packet differs\n", t, k); return 4; }
            HIP_OK(hipMemcpy(got.data(), d_res[k], n_total * 4, hipMemcpyDeviceToHost));
            if (std::memcmp(got.data(), res[k].data(), n_total * 4) != 0) { std::printf("step %u learner %u: residue differs\n", t, k); return 4; }
        }
        const void *host_pk[n_learners] = {want_pk[0].data(), want_pk[1].data()};
        if (adacomp_oracle_unpack_accumulate(otable, n_layers, host_pk, n_learners, want_dense.data()) != 0) return 1;
        HIP_OK(hipMemcpy(got.data(), d_dense, n_total * 4, hipMemcpyDeviceToHost));
        for (uint32_t l = 0; l < n_layers; ++l)
            if (std::memcmp(got.data() + table[l].elem_offset, want_dense.data() + table[l].elem_offset, table[l].n_elems * 4) != 0) {
                std::printf("step %u: dense sum of layer %u differs\n", t, l);
                return 4;
            }
    }

    // one more mini-batch of learner 0 through the single-learner entry point
    for (size_t i = 0; i < n_total; ++i) grad[0][i] = draw((uint64_t(99) << 40) | i, 0.02f);
    HIP_OK(hipMemcpy(d_grad[0], grad[0].data(), n_total * 4, hipMemcpyHostToDevice));
    std::memset(want_pk[0].data(), 0, bound);
    pk_bytes[0] = adacomp_oracle_compress(otable, n_layers, grad[0].data(), res[0].data(), want_pk[0].data(), bound, 0, 2.0f);
    LIB_OK(adacomp_compress(table, n_layers, d_grad[0], d_res[0], d_pk[0], bound, ws, ws_bytes, stream));

    // unpack + average + SGD with momentum, fused, against the oracle's three separate steps
    std::vector<float> w(n_total), m(n_total, 0.f);
    for (size_t i = 0; i < n_total; ++i) w[i] = draw((uint64_t(7) << 48) | i, 1.0f);
    HIP_OK(hipMemcpy(d_w, w.data(), n_total * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_m, 0, n_total * 4));
    adacomp_optimizer_t opt;
    std::memset(&opt, 0, sizeof opt);
    opt.kind = ADACOMP_OPT_SGD_MOMENTUM; opt.lr = 0.05f; opt.momentum = 0.9f; opt.bias1 = opt.bias2 = 1.0f;
    const void *packets[n_learners] = {d_pk[0], d_pk[1]};
    LIB_OK(adacomp_unpack_update(table, n_layers, packets, n_learners, nullptr, d_w, d_m, nullptr, &opt, ws, ws_bytes, stream));
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(got_pk[0].data(), d_pk[0], size_t(pk_bytes[0]), hipMemcpyDeviceToHost));
    if (pk_bytes[0] <= 0 || std::memcmp(got_pk[0].data(), want_pk[0].data(), size_t(pk_bytes[0])) != 0) { std::printf("single call: packet differs\n"); return 4; }
    const void *host_pk[n_learners] = {want_pk[0].data(), want_pk[1].data()};
    if (adacomp_oracle_unpack_accumulate(otable, n_layers, host_pk, n_learners, want_dense.data()) != 0) return 1;
    if (adacomp_oracle_update_sgd(otable, n_layers, want_dense.data(), n_learners, w.data(), m.data(), 0.05f, 0.9f) != 0) return 1;
    HIP_OK(hipMemcpy(got.data(), d_w, n_total * 4, hipMemcpyDeviceToHost));
    if (std::memcmp(got.data(), w.data(), n_total * 4) != 0) { std::printf("updated weights differ\n"); return 4; }
    HIP_OK(hipMemcpy(got.data(), d_m, n_total * 4, hipMemcpyDeviceToHost));
    if (std::memcmp(got.data(), m.data(), n_total * 4) != 0) { std::printf("momentum buffer differs\n"); return 4; }

    // two more mini-batches of both learners with the residue corrections deferred: packets as the
    // oracle's at every step, an eager call refused in between, residues equal after the sync
    for (uint32_t t = 0; t < 2; ++t) {
        for (uint32_t k = 0; k < n_learners; ++k) {
            for (size_t i = 0; i < n_total; ++i) grad[k][i] = draw((uint64_t(200 + t) << 40) | (uint64_t(k) << 32) | i, 0.03f);
            HIP_OK(hipMemcpy(d_grad[k], grad[k].data(), n_total * 4, hipMemcpyHostToDevice));
            std::memset(want_pk[k].data(), 0, bound);
            pk_bytes[k] = adacomp_oracle_compress(otable, n_layers, grad[k].data(), res[k].data(), want_pk[k].data(), bound, 0, 2.0f);
            if (pk_bytes[k] <= 0) return 1;
        }
        const float *grads[n_learners] = {d_grad[0], d_grad[1]};
        float *residues[n_learners] = {d_res[0], d_res[1]};
        LIB_OK(adacomp_compress_batch_lazy(table, n_layers, n_learners, grads, residues, d_pk, bound, ws, ws_bytes, stream));
        if (adacomp_compress_batch(table, n_layers, n_learners, grads, residues, d_pk, bound, ws, ws_bytes, stream) != ADACOMP_EPENDING) {
            std::printf("lazy step %u: an eager call was accepted while corrections wait\n", t);
            return 4;
        }
        HIP_OK(hipStreamSynchronize(stream));
        for (uint32_t k = 0; k < n_learners; ++k) {
            HIP_OK(hipMemcpy(got_pk[k].data(), d_pk[k], size_t(pk_bytes[k]), hipMemcpyDeviceToHost));
            if (std::memcmp(got_pk[k].data(), want_pk[k].data(), size_t(pk_bytes[k])) != 0) { std::printf("lazy step %u learner %u: packet differs\n", t, k); return 4; }
        }
    }
    LIB_OK(adacomp_residue_sync(ws, stream));
    HIP_OK(hipStreamSynchronize(stream));
    for (uint32_t k = 0; k < n_learners; ++k) {
        HIP_OK(hipMemcpy(got.data(), d_res[k], n_total * 4, hipMemcpyDeviceToHost));
        if (std::memcmp(got.data(), res[k].data(), n_total * 4) != 0) { std::printf("after the sync: residue of learner %u differs\n", k); return 4; }
    }

    // two more mini-batches of learner 1 through the entry point that takes no workspace and
    // allocates nothing (its scratch is a static array inside the library), on the same stream
    for (uint32_t t = 0; t < 2; ++t) {
        for (size_t i = 0; i < n_total; ++i) grad[1][i] = draw((uint64_t(300 + t) << 40) | i, 0.02f);
        HIP_OK(hipMemcpy(d_grad[1], grad[1].data(), n_total * 4, hipMemcpyHostToDevice));
        std::memset(want_pk[1].data(), 0, bound);
        pk_bytes[1] = adacomp_oracle_compress(otable, n_layers, grad[1].data(), res[1].data(), want_pk[1].data(), bound, 0, 2.0f);
        if (pk_bytes[1] <= 0) return 1;
        LIB_OK(adacomp_compress_static(table, n_layers, d_grad[1], d_res[1], d_pk[1], bound, stream));
        HIP_OK(hipStreamSynchronize(stream));
        HIP_OK(hipMemcpy(got_pk[1].data(), d_pk[1], size_t(pk_bytes[1]), hipMemcpyDeviceToHost));
        if (std::memcmp(got_pk[1].data(), want_pk[1].data(), size_t(pk_bytes[1])) != 0) { std::printf("static call %u: packet differs\n", t); return 4; }
        HIP_OK(hipMemcpy(got.data(), d_res[1], n_total * 4, hipMemcpyDeviceToHost));
        if (std::memcmp(got.data(), res[1].data(), n_total * 4) != 0) { std::printf("static call %u: residue differs\n", t); return 4; }
    }

    LIB_OK(adacomp_workspace_release(ws));
    std::printf("c caller ok: %u steps x %u learners, last packet %lld bytes of at most %zu\n", n_steps, n_learners, pk_bytes[0], bound);
    return 0;
}
