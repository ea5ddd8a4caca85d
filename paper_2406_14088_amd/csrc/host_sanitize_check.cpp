// Drives the host-side logic of the library -- shape validation, arena sizing, page planning, argument checks of
// every entry point that returns before it touches a device -- in a build of the host code under AddressSanitizer and
// UndefinedBehaviorSanitizer.  CPU only: nothing here launches a kernel or needs a GPU.  Built and run by the CPU test
// suite (paper_2406_14088_amd/build.py: build_host_sanitize_check).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "rl_gen.h"
#include "rl_gen_ops.h"

#define CHECK(cond)                                                                            \
    do {                                                                                       \
        if (!(cond)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); std::exit(1); } \
    } while (0)

static rl_gen_shape shape_of(int L, int d, int Hq, int Hkv, int hd, int F, int V, int B, int S, int precision) {
    rl_gen_shape s;
    std::memset(&s, 0, sizeof s);
    s.n_layers = L; s.hidden = d; s.n_heads = Hq; s.n_kv_heads = Hkv; s.head_dim = hd; s.ffn = F; s.vocab = V;
    s.rope_base = 10000.0f; s.rms_eps = 1e-5f; s.rope_style = 1; s.weight_dtype = 1; s.max_batch = B; s.max_seq = S;
    s.precision = precision;
    return s;
}

int main() {
    // sizing over benchmark shapes and every precision level, up to capacities whose byte counts need 64 bits
    const int shapes[][7] = {{2, 256, 4, 4, 64, 688, 1024},        {32, 4096, 32, 32, 128, 11008, 32000},
                             {40, 5120, 40, 40, 128, 13824, 32000}, {80, 8192, 64, 8, 128, 28672, 32000},
                             {48, 8192, 64, 8, 128, 22016, 128256}, {0, 64, 1, 1, 64, 8, 3}};
    for (const auto &c : shapes)
        for (int precision = 0; precision <= 3; ++precision)
            for (int B : {1, 128, 4096})
                for (int S : {1, 384, 4096, 1 << 20}) {
                    rl_gen_shape s = shape_of(c[0], c[1], c[2], c[3], c[4], c[5], c[6], B, S, precision);
                    CHECK(rl_gen_validate_shape(&s) == RL_GEN_OK);
                    const int level = rl_gen_precision_level(&s);
                    CHECK(level >= 1 && level <= 3 && (precision == 0 || level == precision));
                    const int bs = rl_gen_kv_block_scaled(&s);
                    const size_t row = (size_t)c[4] * 2 + (bs ? 4 : 0);
                    CHECK(rl_gen_kv_bytes(&s) == (size_t)2 * c[0] * B * c[3] * S * row);
                    CHECK(rl_gen_work_bytes(&s) > 0 && rl_gen_param_count(&s) > 0);
                    CHECK(rl_gen_packed_bytes_full(&s) >= rl_gen_packed_bytes(&s));
                    (void)rl_gen_prefers_packed_gate_up(&s);
                    for (int page : {16, 64, 4096}) CHECK(rl_gen_page_bytes(&s, page) == (size_t)2 * c[0] * c[3] * page * row);
                    for (int page : {0, 8, 24, 8192, -16}) CHECK(rl_gen_page_bytes(&s, page) == 0);
                }
    // refusals
    {
        rl_gen_shape s = shape_of(2, 256, 4, 3, 64, 688, 1024, 4, 32, 0);
        CHECK(rl_gen_validate_shape(&s) == RL_GEN_E_SHAPE && rl_gen_kv_bytes(&s) == 0 && rl_gen_work_bytes(&s) == 0);
        s = shape_of(2, 256, 4, 4, 64, 688, 1024, 4, 32, 4);
        CHECK(rl_gen_validate_shape(&s) == RL_GEN_E_SHAPE && rl_gen_precision_level(&s) < 0);
        s = shape_of(2, 256, 4, 4, 64, 688, 1024, 0, 32, 0);
        CHECK(rl_gen_validate_shape(&s) == RL_GEN_E_SHAPE);
        s = shape_of(2, 256, 4, 4, 32, 688, 1024, 4, 32, 0);
        CHECK(rl_gen_validate_shape(&s) == RL_GEN_E_SHAPE);
        CHECK(rl_gen_validate_shape(nullptr) != RL_GEN_OK && rl_gen_kv_bytes(nullptr) == 0);
    }
    // page planning: exactly-sized arrays, so a write past the table would be caught
    {
        const int32_t cap[4] = {33, 0, 16, 1};
        std::vector<int32_t> table(4 * 4, 7);
        CHECK(rl_gen_plan_pages(cap, 4, 16, 10, 4, table.data()) == 5);
        const int32_t want[16] = {0, 1, 2, -1, -1, -1, -1, -1, 3, -1, -1, -1, 4, -1, -1, -1};
        CHECK(std::memcmp(table.data(), want, sizeof want) == 0);
        const int32_t two[2] = {33, 16};
        CHECK(rl_gen_plan_pages(two, 2, 16, 3, 4, table.data()) == RL_GEN_E_CAPACITY);
        const int32_t big[1] = {65};
        CHECK(rl_gen_plan_pages(big, 1, 16, 10, 4, table.data()) == RL_GEN_E_CAPACITY);
        const int32_t neg[1] = {-1};
        CHECK(rl_gen_plan_pages(neg, 1, 16, 10, 4, table.data()) == RL_GEN_E_SHAPE);
        CHECK(rl_gen_plan_pages(nullptr, 1, 16, 1, 1, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_plan_pages(cap, 0, 16, 0, 4, table.data()) == 0);
    }
    // entry points called without a handle or without their required pointers
    {
        rl_gen_shape s = shape_of(2, 256, 4, 4, 64, 688, 1024, 4, 32, 0);
        rl_gen_t *h = nullptr;
        CHECK(rl_gen_create(&s, nullptr, nullptr, 0, nullptr, 0, &h) == RL_GEN_E_NULL && h == nullptr);
        CHECK(rl_gen_create_paged(&s, nullptr, nullptr, 0, nullptr, 0, 16, &h) == RL_GEN_E_NULL);
        CHECK(rl_gen_prefill(nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_prefill_ragged(nullptr, nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_decode_step(nullptr, nullptr, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_logprobs(nullptr, nullptr, 1, 1, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_values(nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_pack_weights(nullptr, nullptr, 0, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_set_block_table(nullptr, nullptr, nullptr, 1, 1, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_pool_pages(nullptr) == RL_GEN_E_NULL && rl_gen_packed_gate_up_layers(nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_set_eos(nullptr, 1) == RL_GEN_E_NULL && rl_gen_set_graph(nullptr, 1) == RL_GEN_E_NULL);
        CHECK(rl_gen_set_sampling(nullptr, 1.0f, nullptr) == RL_GEN_E_NULL && rl_gen_set_qkv_terms(nullptr, 1) == RL_GEN_E_NULL);
        CHECK(rl_gen_read_state(nullptr, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_compact(nullptr, nullptr, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_state(nullptr, nullptr, nullptr) == RL_GEN_E_NULL && rl_gen_reset(nullptr) == RL_GEN_E_NULL);
        CHECK(rl_gen_profile(nullptr, 1) == RL_GEN_E_NULL && rl_gen_profile_read(nullptr, nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        rl_gen_destroy(nullptr);
        CHECK(rl_gen_last_error(nullptr) != nullptr);
        for (int id = -2; id < 40; ++id) (void)rl_gen_kernel_class_name(id);
        CHECK(std::strcmp(rl_gen_kernel_class_name(4), "decode_attention") == 0);
    }
    // per-kernel entry points: NULL operands and shapes outside what the kernels serve are refused before any launch
    {
        CHECK(rl_op_argmax(nullptr, 1, 1, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_op_decode_attention(nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, 1, 4, 4, 128, 16, 1, nullptr, nullptr,
                                     nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_op_decode_attention_noalloc(nullptr, nullptr, nullptr, nullptr, 0, nullptr, 1, 4, 4, 128, 16, 1, nullptr, nullptr,
                                             nullptr, nullptr, nullptr) == RL_GEN_E_NULL);
        CHECK(rl_op_packed_weight_bytes(32, 16) == 1024 && rl_op_packed_weight_bytes(33, 17) == 4096);
        CHECK(rl_op_decode_attention_ws_floats(2, 4, 128, 1) == 0 && rl_op_decode_attention_ws_floats(2, 4, 128, 3) == 2u * 4 * 3 * 130);
    }
    std::puts("host sanitize check: ok");
    return 0;
}
