// Host-side checks of the library under AddressSanitizer and UndefinedBehaviorSanitizer: the argument
// checks, the workspace layout and the GEMM planner, none of which need a GPU.  Built and run by
// tests/test_host_sanitizers.py; exits 0 when every expectation holds (the sanitizers abort otherwise).
#include "../include/bt.h"
#include "../paper_2406_02657_amd/csrc/kernels.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static int g_checks = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    ++g_checks;                                                             \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); std::exit(1); } \
  } while (0)

static bt_config base_config() {
  bt_config c;
  std::memset(&c, 0, sizeof(c));
  c.struct_size = (int32_t)sizeof(bt_config);
  c.vocab = 1000; c.block_len = 4; c.d_model = 256; c.n_heads = 4; c.d_ff = 1024;
  c.n_block_layers = 2; c.n_token_layers = 2; c.prefix_len = 2; c.dtype = BT_BF16;
  c.max_batch = 8; c.max_blocks = 64; c.rotary_dims = 16; c.parallel_residual = 1;
  c.act_split = 2; c.use_graphs = 1; c.eos_id = -1; c.keep_logits = 1; c.ln_eps = 1e-5f;
  return c;
}

int main() {
  size_t n = 0;
  bt_config c = base_config();
  EXPECT(bt_workspace_bytes(&c, &n) == BT_OK && n > 0);
  EXPECT(bt_workspace_bytes(nullptr, &n) == BT_ERR_ARG);
  EXPECT(bt_workspace_bytes(&c, nullptr) == BT_ERR_ARG);

  // every field driven through its limits
  struct Case { int bt_config::*field; int value; int want; };
  const Case cases[] = {
      {&bt_config::struct_size, 4, BT_ERR_ARG}, {&bt_config::dtype, 2, BT_ERR_ARG}, {&bt_config::vocab, 0, BT_ERR_ARG},
      {&bt_config::block_len, 0, BT_ERR_ARG}, {&bt_config::block_len, 3, BT_ERR_ARG}, {&bt_config::n_heads, 3, BT_ERR_ARG},
      {&bt_config::n_heads, 32, BT_ERR_ARG}, {&bt_config::d_model, 8192, BT_ERR_ARG}, {&bt_config::d_ff, 1000, BT_ERR_ARG},
      {&bt_config::rotary_dims, 3, BT_ERR_ARG}, {&bt_config::rotary_dims, 128, BT_ERR_ARG}, {&bt_config::rotary_dims, 0, BT_OK},
      {&bt_config::prefix_len, 0, BT_ERR_ARG}, {&bt_config::prefix_len, -1, BT_ERR_ARG}, {&bt_config::prefix_len, 8, BT_OK},
      {&bt_config::max_batch, 0, BT_ERR_ARG}, {&bt_config::max_blocks, 0, BT_ERR_ARG}, {&bt_config::max_blocks, 1, BT_OK},
      {&bt_config::prefill_rows, -1, BT_ERR_ARG}, {&bt_config::prefill_rows, 1, BT_OK}, {&bt_config::act_split, 3, BT_ERR_ARG},
      {&bt_config::use_graphs, 2, BT_ERR_ARG}, {&bt_config::pad_id, 1000, BT_ERR_ARG}, {&bt_config::pad_id, 999, BT_OK},
      {&bt_config::eos_id, -2, BT_ERR_ARG}, {&bt_config::eos_id, 1000, BT_ERR_ARG}, {&bt_config::score_rows, -1, BT_ERR_ARG},
      {&bt_config::score_rows, 64, BT_OK}, {&bt_config::keep_logits, 2, BT_ERR_ARG}, {&bt_config::token_mix, 2, BT_ERR_ARG},
      {&bt_config::n_block_layers, -1, BT_ERR_ARG}, {&bt_config::n_block_layers, 0, BT_OK}, {&bt_config::n_token_layers, 0, BT_OK},
  };
  for (const Case& k : cases) {
    bt_config v = base_config();
    v.*(k.field) = k.value;
    EXPECT(bt_workspace_bytes(&v, &n) == k.want);
  }
  {
    bt_config v = base_config();
    v.ln_eps = -1.f;
    EXPECT(bt_workspace_bytes(&v, &n) == BT_ERR_ARG);
    v = base_config(); v.block_len = 1; v.prefix_len = 0;
    EXPECT(bt_workspace_bytes(&v, &n) == BT_OK);
    v = base_config(); v.token_mix = BT_MIX_SUM;                    // needs prefix_len == 1
    EXPECT(bt_workspace_bytes(&v, &n) == BT_ERR_ARG);
    v.prefix_len = 1;
    EXPECT(bt_workspace_bytes(&v, &n) == BT_OK);
  }

  // the workspace grows with every capacity, over the shapes of the five workloads and fp32 mode
  const int shapes[][7] = {{512, 4, 128, 4, 512, 2, 1}, {50304, 4, 768, 12, 3072, 12, 1}, {50304, 8, 1024, 16, 4096, 16, 2},
                           {50304, 4, 2048, 16, 8192, 24, 1}, {50304, 1, 2048, 16, 8192, 24, 0}};
  for (const auto& s : shapes)
    for (int dtype = 0; dtype < 2; ++dtype) {
      bt_config v = base_config();
      v.vocab = s[0]; v.block_len = s[1]; v.d_model = s[2]; v.n_heads = s[3]; v.d_ff = s[4];
      v.n_block_layers = v.n_token_layers = s[5]; v.prefix_len = s[6]; v.dtype = dtype; v.rotary_dims = s[2] / s[3] / 4;
      size_t prev = 0;
      for (int batch : {1, 7, 64, 256})
        for (int blocks : {1, 33, 1024, 4096}) {
          v.max_batch = batch; v.max_blocks = blocks;
          for (int score : {0, 512}) {
            if (score && v.prefix_len == 0) continue;
            v.score_rows = score;
            EXPECT(bt_workspace_bytes(&v, &n) == BT_OK && n % 256 == 0 && n > 0);
          }
          v.score_rows = 0;
          EXPECT(bt_workspace_bytes(&v, &n) == BT_OK);
          if (blocks == 1) { EXPECT(n > prev || batch == 1); prev = n; }
        }
    }

  // create: everything that is decided before the first HIP call
  {
    bt_model* m = reinterpret_cast<bt_model*>(0x1);
    bt_weights w;
    std::memset(&w, 0, sizeof(w));
    alignas(256) static char fake_ws[512];
    EXPECT(bt_create(nullptr, &w, fake_ws, 1 << 20, nullptr, &m) == BT_ERR_ARG);
    EXPECT(bt_create(&c, nullptr, fake_ws, 1 << 20, nullptr, &m) == BT_ERR_ARG);
    EXPECT(bt_create(&c, &w, fake_ws, 1 << 20, nullptr, nullptr) == BT_ERR_ARG);
    EXPECT(bt_create(&c, &w, nullptr, 1 << 20, nullptr, &m) == BT_ERR_ARG && m == nullptr);
    EXPECT(bt_create(&c, &w, fake_ws + 8, 1 << 20, nullptr, &m) == BT_ERR_ARG);
    EXPECT(std::strstr(bt_last_error(nullptr), "aligned") != nullptr);
    EXPECT(bt_create(&c, &w, fake_ws, 1 << 20, nullptr, &m) == BT_ERR_ARG);          // null weight pointers
    // weights that look present: the call gets as far as the workspace size
    std::vector<bt_layer_weights> layers(2);
    const void* some = fake_ws;
    for (auto& l : layers) l = bt_layer_weights{some, some, some, some, some, some, some, some, some, some, some, some};
    w = bt_weights{some, some, some, some, some, some, some, some, some, layers.data(), layers.data()};
    EXPECT(bt_create(&c, &w, fake_ws, 256, nullptr, &m) == BT_ERR_CAPACITY && m == nullptr);
    layers[1].W_up = nullptr;
    EXPECT(bt_create(&c, &w, fake_ws, (size_t)1 << 40, nullptr, &m) == BT_ERR_ARG);
    bt_config big = base_config();
    big.max_batch = 4096; big.max_blocks = 4096;
    EXPECT(bt_create_static(&big, &w, nullptr, &m) == BT_ERR_CAPACITY);
    EXPECT(std::strstr(bt_last_error(nullptr), "BT_STATIC_WORKSPACE_BYTES") != nullptr);
    // null handles
    EXPECT(bt_prefill(nullptr, nullptr, 1, 4) == BT_ERR_ARG);
    EXPECT(bt_decode_step(nullptr, 1, nullptr) == BT_ERR_ARG);
    EXPECT(bt_get_stats(nullptr, nullptr) == BT_ERR_ARG);
    bt_destroy(nullptr);
  }

  // the GEMM planner over many shapes: whatever it answers, the splits divide K into whole slices, or (uneven
  // plans: two planes, 64-element slices, 129-256 rows or partial sums with fewer rows) there are at most as many splits as slices
  {
    using namespace bt;
    const int Ms[] = {1, 5, 16, 63, 64, 65, 128, 129, 192, 193, 255, 256, 257, 1000, 16384};
    const int Ns[] = {64, 100, 768, 2304, 3072, 4160, 50304};
    const int Ks[] = {64, 128, 192, 256, 768, 1024, 3072, 8192};
    int dummy = 0;
    for (int dtype : {(int)BT_F32, (int)BT_BF16})
      for (int M : Ms)
        for (int N : Ns)
          for (int K : Ks)
            for (int hl = 0; hl < 2; ++hl)
              for (int two = 0; two < 2; ++two)
                for (int epi : {(int)EPI_F32, (int)EPI_PARTIAL}) {
                  if (hl && dtype == BT_F32) continue;
                  GemmProblem p[2];
                  std::memset(p, 0, sizeof(p));
                  for (int i = 0; i < 2; ++i) {
                    p[i].A = &dummy; p[i].W = &dummy; p[i].out = &dummy; p[i].W_frag = &dummy;
                    p[i].M = M; p[i].N = i ? 768 : N; p[i].K = i ? 3072 : K; p[i].lda = p[i].K; p[i].ldo = p[i].N; p[i].epi = epi;
                    p[i].A_lo = hl ? &dummy : nullptr;
                  }
                  GemmPlan plan;
                  std::memset(&plan, 0, sizeof(plan));
                  EXPECT(gemm_plan(dtype, p, 1 + two, &plan) == hipSuccess);
                  for (int i = 0; i <= two; ++i) {
                    EXPECT(plan.uneven == 0 || plan.uneven == 1);
                    if (plan.uneven) {
                      EXPECT(hl && plan.kind == 2 && plan.kf == 2 && plan.nt <= 2);
                      EXPECT((plan.mc == 4 && M > 128 && M <= 256) || (plan.mc == 2 && M > 64 && M <= 128 && epi == EPI_PARTIAL) ||
                             (plan.mc == 1 && M <= 64 && epi == EPI_PARTIAL));
                      EXPECT(plan.splits[i] >= 1 && p[i].K % 64 == 0 && plan.splits[i] <= p[i].K / 64);
                    } else {
                      EXPECT(plan.splits[i] >= 1 && p[i].K % plan.splits[i] == 0);
                      if (plan.kf > 0 && dtype == BT_BF16 && M <= 256) EXPECT(p[i].K % (32 * plan.kf * plan.splits[i]) == 0 || plan.kind != 2);
                    }
                    if (epi != EPI_PARTIAL) EXPECT(plan.splits[i] == 1);
                  }
                  const int tiles = gemm_row_max_tiles(p[0], plan);
                  EXPECT(tiles >= 0 && tiles <= (N + 63) / 64);
                  (void)gemm_has_lse_epilogue(plan);
                }
    GemmProblem bad;
    std::memset(&bad, 0, sizeof(bad));
    GemmPlan plan;
    EXPECT(gemm_plan(BT_BF16, &bad, 1, &plan) != hipSuccess);           // zero sizes
    EXPECT(gemm_plan(BT_BF16, &bad, 3, &plan) != hipSuccess);
    EXPECT(gemm_packed_elems(100, 64) == (size_t)112 * 64);
    for (int batch : {1, 3, 16, 64, 300})
      for (int heads : {1, 12, 16})
        for (int cap : {1, 100, 544, 4096}) {
          const int s = attn_block_decode_splits(batch, heads, cap);
          EXPECT(s >= 1 && s <= 16 && (batch * heads < 256 || s == 1) && batch * heads * s <= 512 + batch * heads);
        }
  }
  std::printf("host sanitizer driver: %d checks passed\n", g_checks);
  return 0;
}
