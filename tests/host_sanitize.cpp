// Host-side exercise of the C ABI for a build of the library with AddressSanitizer / UndefinedBehaviorSanitizer on its
// host code (see tests/test_host_sanitizers.py).  Everything here returns before any device work: the buffer manager
// is host logic over an arena it never dereferences, and the entry points validate their arguments first.  The
// sanitizers abort the process on the first finding; reaching the last line prints "ok".
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/eet.h"

#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond);  \
            std::exit(1);                                                    \
        }                                                                    \
    } while (0)

static uint64_t rng_state = 0x2104124700000001ull;
static uint32_t rnd() {                      // xorshift64*: inputs only
    rng_state ^= rng_state >> 12;
    rng_state ^= rng_state << 25;
    rng_state ^= rng_state >> 27;
    return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}

static void buffer_manager() {
    char* const arena = reinterpret_cast<char*>(0x7F0000000000ull);          // an address, never dereferenced
    const size_t arena_bytes = (size_t)1 << 20;
    eet_bufmgr_t* m = nullptr;
    CHECK(eet_bufmgr_create(nullptr, arena_bytes, &m) != EET_OK);
    CHECK(eet_bufmgr_create(arena, arena_bytes, nullptr) != EET_OK);
    CHECK(eet_bufmgr_create(arena + 8, arena_bytes, &m) != EET_OK);          // arena alignment
    CHECK(eet_bufmgr_create(arena, arena_bytes, &m) == EET_OK && m);
    std::vector<void*> live;
    eet_bufmgr_stats st{};
    for (int it = 0; it < 30000; ++it) {
        const uint32_t r = rnd();
        if (live.empty() || (r & 3) != 0) {
            void* p = nullptr;
            const size_t bytes = (size_t)(1 + rnd() % 16) * (rnd() % 5 == 0 ? 4096 : 256) - (rnd() & 1);
            const int rc = eet_bufmgr_request(m, bytes, (int32_t)(rnd() % 4), &p);
            if (rc == EET_OK) {
                CHECK(p >= (void*)arena && p < (void*)(arena + arena_bytes) && ((uintptr_t)p & 255u) == 0);
                live.push_back(p);
            } else {
                CHECK(rc == EET_ERR_CAPACITY);                                  // the arena is full: nothing was created
                while (live.size() > 4) {
                    CHECK(eet_bufmgr_release(m, live.back()) == EET_OK);
                    live.pop_back();
                }
            }
        } else {
            const size_t i = rnd() % live.size();
            CHECK(eet_bufmgr_release(m, live[i]) == EET_OK);
            live[i] = live.back();
            live.pop_back();
        }
        if ((it & 1023) == 0) {
            CHECK(eet_bufmgr_query(m, &st) == EET_OK);
            CHECK(st.footprint_bytes <= arena_bytes && st.buffers - st.idle == (int64_t)live.size());
        }
    }
    CHECK(eet_bufmgr_release(m, arena + 12345) != EET_OK);                   // not a buffer of this manager
    CHECK(eet_bufmgr_release(m, nullptr) != EET_OK);
    if (!live.empty()) {
        CHECK(eet_bufmgr_release(m, live[0]) == EET_OK);
        CHECK(eet_bufmgr_release(m, live[0]) != EET_OK);                     // already idle
    }
    void* p = nullptr;
    CHECK(eet_bufmgr_request(m, 0, 0, &p) != EET_OK);
    CHECK(eet_bufmgr_request(m, 256, 0, nullptr) != EET_OK);
    CHECK(eet_bufmgr_request(nullptr, 256, 0, &p) != EET_OK);
    CHECK(eet_bufmgr_query(m, nullptr) != EET_OK);
    CHECK(eet_bufmgr_destroy(m) == EET_OK);
    CHECK(eet_bufmgr_destroy(nullptr) == EET_OK);
}

static void handles_and_validation() {
    void* const P = reinterpret_cast<void*>(0x200000);
    eet_layer_weights w;
    const void** wp = reinterpret_cast<const void**>(&w);
    for (int i = 0; i < 12; ++i) wp[i] = reinterpret_cast<void*>(0x10000 + 0x100 * i);
    int32_t lens[EET_MAX_BATCH + 1];
    for (int i = 0; i <= EET_MAX_BATCH; ++i) lens[i] = 1 + i % 7;
    const int32_t zero_first[2] = {0, 3};
    for (int round = 0; round < 300; ++round) {
        eet_layer_config cfg{1024, 16, 4096, (int32_t)(1 + rnd() % EET_MAX_BATCH), 64, 80, 1e-5f};
        eet_layer_t* L = nullptr;
        CHECK(eet_layer_create(&cfg, &w, reinterpret_cast<void*>(0x100000), &L) == EET_OK && L);
        CHECK(eet_decode_step(L, P, P, P, nullptr) == EET_ERR_STATE);
        CHECK(eet_prefill(L, lens, cfg.max_batch + 1, 10, P, P, P, nullptr) == EET_ERR_CAPACITY);
        CHECK(eet_prefill(L, lens, 1, 65, P, P, P, nullptr) == EET_ERR_CAPACITY);
        CHECK(eet_prefill(L, zero_first, 1, 10, P, P, P, nullptr) == EET_ERR_INVALID_ARG);   // a length of 0
        CHECK(eet_prefill_left_padded(L, nullptr, 1, 10, P, P, P, nullptr) == EET_ERR_INVALID_ARG);
        CHECK(eet_layer_encode(L, lens, 0, 10, P, P, P, nullptr) == EET_ERR_INVALID_ARG);
        CHECK(eet_restore(L, lens, cfg.max_batch + 1, nullptr) == EET_ERR_CAPACITY);
        CHECK(eet_cache_lens(L, lens, nullptr) == EET_ERR_STATE);
        CHECK(eet_last_error()[0] != 0);
        CHECK(eet_layer_destroy(L) == EET_OK);

        const int n_layers = 1 + (int)(rnd() % 6);
        std::vector<eet_layer_weights> ws((size_t)n_layers, w);
        eet_stack_t* S = nullptr;
        CHECK(eet_stack_create(&cfg, n_layers, ws.data(), reinterpret_cast<void*>(0x100000), 1, &S) == EET_OK && S);
        CHECK(eet_stack_decode_step(S, P, P, P, nullptr) == EET_ERR_STATE);
        CHECK(eet_stack_prefill(S, lens, cfg.max_batch + 1, 10, P, P, P, nullptr) == EET_ERR_CAPACITY);
        CHECK(eet_stack_prefill_left_padded(S, lens, 1, 65, P, P, P, nullptr) == EET_ERR_CAPACITY);
        CHECK(eet_stack_encode(S, nullptr, 1, 10, P, P, P, nullptr) == EET_ERR_INVALID_ARG);
        CHECK(eet_stack_restore(S, lens, 0, nullptr) == EET_ERR_INVALID_ARG);
        CHECK(eet_stack_cache_lens(S, lens, nullptr) == EET_ERR_STATE);
        eet_model_config mc{50257, 50304, 1024};
        eet_model_weights mw{P, P, P, P};
        eet_model_t* M = nullptr;
        CHECK(eet_model_create(S, &cfg, &mc, &mw, reinterpret_cast<void*>(0x100010), &M) == EET_ERR_INVALID_ARG && !M);
        mc.vocab_padded = 50257;
        CHECK(eet_model_create(S, &cfg, &mc, &mw, P, &M) == EET_ERR_UNSUPPORTED_SHAPE && !M);
        CHECK(eet_model_workspace_bytes(&cfg, &mc) == 0);
        CHECK(eet_stack_destroy(S) == EET_OK);
    }
    eet_layer_config bad{960, 10, 3072, 4, 64, 64, 1e-5f};                       // head size 96
    eet_layer_t* L = nullptr;
    CHECK(eet_layer_create(&bad, &w, reinterpret_cast<void*>(0x100000), &L) == EET_ERR_UNSUPPORTED_SHAPE && !L);
    CHECK(eet_workspace_bytes(&bad) == 0 && eet_kv_cache_bytes(nullptr) == 0);
    CHECK(eet_op_linear(P, P, P, nullptr, P, 4, 100, 64, 0, nullptr) == EET_ERR_UNSUPPORTED_SHAPE);
    CHECK(eet_op_layernorm(nullptr, P, P, P, 4, 64, 1e-5f, nullptr) == EET_ERR_INVALID_ARG);
    CHECK(eet_op_softmax_maskfree(P, lens, EET_MAX_BATCH + 1, 2, 16, 1.0f, nullptr) == EET_ERR_CAPACITY);
    CHECK(eet_op_argmax(P, 2, 100, 96, reinterpret_cast<int32_t*>(P), nullptr) == EET_ERR_INVALID_ARG);
    CHECK(eet_op_embedding(reinterpret_cast<const int32_t*>(P), lens, 2, 16, 60, 100, 16, P, P, P, nullptr) == EET_ERR_UNSUPPORTED_SHAPE);
}

int main() {
    buffer_manager();
    handles_and_validation();
    std::puts("ok");
    return 0;
}
