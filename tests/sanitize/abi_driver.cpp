// Host-only walk through the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (built and run by
// tests/test_sanitizers.py against a copy of the library whose host code is instrumented).  Every call here is one the
// library must answer before it touches a device: sizes, status texts, rejected arguments, null handles.
#include "../../include/mtp_draft.h"

#include <cstdio>
#include <cstring>

#define CHECK(cond)                                                                                                    \
    do {                                                                                                               \
        if (!(cond)) {                                                                                                 \
            std::printf("failed: %s (line %d)\n", #cond, __LINE__);                                                    \
            return 1;                                                                                                  \
        }                                                                                                              \
    } while (0)

int main() {
    mtp_config cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.d_model = 4096; cfg.n_q_heads = 32; cfg.n_kv_heads = 8; cfg.head_dim = 128; cfg.d_ffn = 11008;
    cfg.vocab_size = 151680; cfg.rms_eps = 1e-6f; cfg.rope_theta = 1e6f; cfg.max_batch = 64; cfg.kv_capacity = 32832;
    cfg.max_draft_steps = 7;
    const size_t need = mtp_workspace_bytes(&cfg);
    CHECK(need > 0 && need % 256 == 0);
    CHECK(mtp_workspace_bytes(nullptr) == 0);
    CHECK(mtp_phase_trace_bytes(&cfg) > 0);
    CHECK(mtp_train_workspace_bytes(&cfg, 512) > 0);
    CHECK(mtp_subset_workspace_bytes(cfg.vocab_size) > 0);
    CHECK(mtp_subset_static_max_vocab() >= 151680);
    mtp_config bad = cfg;
    bad.head_dim = 96;
    CHECK(mtp_workspace_bytes(&bad) == 0);
    bad = cfg;
    bad.max_batch = 0;
    CHECK(mtp_workspace_bytes(&bad) == 0);
    bad = cfg;
    bad.max_draft_steps = 0;
    CHECK(mtp_workspace_bytes(&bad) == 0);

    for (int s = 1; s >= -20; --s) CHECK(mtp_status_string(s) != nullptr);

    mtp_weights w;
    void *fake = reinterpret_cast<void *>(0x1000); // never dereferenced: every call below fails before that
    const void **slots = reinterpret_cast<const void **>(&w);
    for (size_t i = 0; i < sizeof w / sizeof(void *); ++i) slots[i] = fake;
    mtp_handle *h = nullptr;
    void *ws = reinterpret_cast<void *>(0x10000);
    CHECK(mtp_draft_init(nullptr, &cfg, &w, 0, nullptr, nullptr, ws, need) < 0);
    CHECK(mtp_draft_init(&h, nullptr, &w, 0, nullptr, nullptr, ws, need) < 0 && h == nullptr);
    CHECK(mtp_draft_init(&h, &cfg, nullptr, 0, nullptr, nullptr, ws, need) < 0 && h == nullptr);
    CHECK(mtp_draft_init(&h, &cfg, &w, 0, nullptr, nullptr, nullptr, need) < 0 && h == nullptr);
    CHECK(mtp_draft_init(&h, &cfg, &w, 0, nullptr, nullptr, ws, need - 1) < 0 && h == nullptr);
    mtp_weights w2 = w;
    w2.w_q = reinterpret_cast<void *>(0x1008); // misaligned
    CHECK(mtp_draft_init(&h, &cfg, &w2, 0, nullptr, nullptr, ws, need) < 0 && h == nullptr);
    w2 = w;
    w2.w_o = nullptr;
    CHECK(mtp_draft_init(&h, &cfg, &w2, 0, nullptr, nullptr, ws, need) < 0 && h == nullptr);
    const int32_t *lists[1] = {reinterpret_cast<const int32_t *>(0x2000)};
    int32_t sizes[1] = {0};
    CHECK(mtp_draft_init(&h, &cfg, &w, 1, lists, sizes, ws, need) < 0 && h == nullptr); // empty list
    sizes[0] = cfg.vocab_size + 1;
    CHECK(mtp_draft_init(&h, &cfg, &w, 1, lists, sizes, ws, need) < 0 && h == nullptr); // longer than the vocabulary
    CHECK(mtp_draft_init(&h, &bad, &w, 0, nullptr, nullptr, ws, need) < 0 && h == nullptr);

    int32_t out[8];
    CHECK(mtp_draft_steps(nullptr, 1, 1, -1, fake, reinterpret_cast<const int32_t *>(fake), fake, fake,
                          reinterpret_cast<const int32_t *>(fake), nullptr, out, nullptr, nullptr, nullptr) < 0);
    CHECK(mtp_accept(nullptr, 1, 1, out, out, 0, out, out, out, out, nullptr) < 0);
    CHECK(mtp_poll_error(nullptr, nullptr) < 0);
    CHECK(mtp_set_timing(nullptr, 1) < 0);
    CHECK(mtp_set_launch_mode(nullptr, 0) < 0);
    CHECK(mtp_set_phase_trace(nullptr, nullptr) < 0);
    CHECK(mtp_last_draft_ms(nullptr) < 0.f);
    CHECK(mtp_subset_build(nullptr, 16, 100, 10, ws, 1 << 20, out, out, nullptr, nullptr) < 0);
    CHECK(mtp_subset_build_static(nullptr, 16, 100, 10, out, out, nullptr, nullptr) < 0);
    CHECK(mtp_subset_build_static(reinterpret_cast<const int32_t *>(fake), 16, mtp_subset_static_max_vocab() + 1, 10, out,
                                  out, nullptr, nullptr) < 0);
    CHECK(mtp_stream_probe(nullptr, 1 << 20, out, nullptr) < 0);
    mtp_draft_destroy(nullptr);
    std::puts("host side of the C ABI under sanitizers: ok");
    return 0;
}
