// Host-only driver, built with -fsanitize=address,undefined by tests/test_sanitizers.py:
// the library's planner and the oracle run side by side on small shapes.  The planner's
// segment table is applied to host buffers with explicit bounds checks and compared with
// the oracle byte for byte; the oracle's KV and merge paths run on sentinel-guarded buffers.
// Any out-of-bounds access, overflow or mismatch makes the process fail.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "../../oracle/amoeba_oracle.h"
#include "../../paper_2509_19729_amd/csrc/plan.h"

namespace amoeba { void set_error(const std::string&) {} }

static int failures = 0;
#define CHECK(c) do { if (!(c)) { std::printf("CHECK failed: %s (line %d)\n", #c, __LINE__); ++failures; } } while (0)

static std::vector<uint16_t> random_u16(size_t n, uint64_t seed) {
  std::mt19937_64 g(seed);
  std::vector<uint16_t> v(n);
  for (auto& x : v) x = uint16_t(g());
  return v;
}

// Applies the plan's segment table to host buffers with explicit bounds checks; every target
// byte must be written exactly once and the result must equal `want`.
static void apply_and_compare(const amoeba_plan_s& plan, const amoeba_model_shape& s,
                              const std::vector<std::vector<uint16_t>>& src, int k,
                              const std::vector<uint16_t>& want) {
  const size_t dst_bytes = size_t(plan.dst_layer_bytes) * s.n_layers;
  const size_t src_bytes = size_t(plan.src_layer_bytes) * s.n_layers;
  std::vector<uint8_t> got(dst_bytes, 0xEE), hits(dst_bytes, 0);
  for (const amoeba::Segment& g : plan.segments)
    for (int l = 0; l < s.n_layers; ++l)
      for (int64_t row = 0; row < g.rows; ++row) {
        const int64_t b = l * plan.dst_layer_bytes + g.dst_off + row * g.dst_pitch;
        CHECK(b >= 0 && size_t(b + g.run) <= dst_bytes);
        if (g.src_rank < 0) {
          std::memset(got.data() + b, 0, size_t(g.run));
        } else {
          const int64_t a = l * plan.src_layer_bytes + g.src_off + row * g.src_pitch;
          CHECK(g.src_rank < k && a >= 0 && size_t(a + g.run) <= src_bytes);
          std::memcpy(got.data() + b, reinterpret_cast<const uint8_t*>(src[g.src_rank].data()) + a, size_t(g.run));
        }
        for (int64_t i = 0; i < g.run; ++i) ++hits[size_t(b + i)];
      }
  for (size_t i = 0; i < dst_bytes; ++i) if (hits[i] != 1) { CHECK(hits[i] == 1); break; }
  CHECK(std::memcmp(got.data(), want.data(), dst_bytes) == 0);
}

static void weights_case(int k, int kp, bool sp, bool dp, int T, int64_t page) {
  amoeba_model_shape s;
  std::memset(&s, 0, sizeof(s));
  s.n_layers = 2; s.hidden = 24; s.n_q_heads = 8; s.n_kv_heads = 4; s.head_dim = 4; s.ffn_dim = 72;
  s.elem_bytes = 2; s.kv_block_tokens = 4; s.kv_layers = 1;
  s.w_layout_src = sp; s.w_layout_dst = dp; s.pad_max_tp = T; s.pad_page_bytes = page;
  ao_model m = {s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 2};
  ao_pad pad = {T, sp, dp, page};
  const bool padded = sp || dp;
  // sources: random dense shards, converted by the oracle if the source side is padded
  std::vector<std::vector<uint16_t>> src(k);
  std::vector<const void*> dense_ptr(k);
  std::vector<std::vector<uint16_t>> dense(k);
  for (int r = 0; r < k; ++r) { dense[r] = random_u16(size_t(ao_shard_elems(&m, k)), 7 * r + k); dense_ptr[r] = dense[r].data(); }
  for (int r = 0; r < k; ++r) {
    if (sp) {
      ao_pad up = {T, 0, 1, page};
      src[r].assign(size_t(ao_padded_shard_elems(&m, &up, k)), 0xEEEE);
      CHECK(ao_reshard_weights_padded(&m, &up, k, k, r, dense_ptr.data(), src[r].data()) == AO_OK);
    } else {
      src[r] = dense[r];
    }
  }
  std::vector<const void*> src_ptr(k);
  for (int r = 0; r < k; ++r) src_ptr[r] = src[r].data();
  for (int rp = 0; rp < kp; ++rp) {
    amoeba_plan_s plan;
    std::string err;
    CHECK(amoeba::build_plan(&plan, &s, k, kp, rp, &err));
    CHECK(size_t(plan.src_layer_bytes) * s.n_layers == src[0].size() * 2);
    std::vector<uint16_t> want(size_t(plan.dst_layer_bytes) * s.n_layers / 2, 0xEEEE);
    if (padded) CHECK(ao_reshard_weights_padded(&m, &pad, k, kp, rp, src_ptr.data(), want.data()) == AO_OK);
    else CHECK(ao_reshard_weights(&m, k, kp, rp, src_ptr.data(), want.data()) == AO_OK);
    apply_and_compare(plan, s, src, k, want);
  }
}

static void moe_case(int k, int kp, bool sp, bool dp, int64_t page) {
  amoeba_model_shape s;
  std::memset(&s, 0, sizeof(s));
  s.n_layers = 2; s.hidden = 12; s.n_q_heads = 8; s.n_kv_heads = 8; s.head_dim = 2; s.ffn_dim = 5;
  s.elem_bytes = 2; s.kv_block_tokens = 4; s.kv_layers = 1; s.n_experts = 8;
  s.w_layout_src = sp; s.w_layout_dst = dp; s.pad_page_bytes = page;
  ao_model m = {s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 2};
  ao_moe flat = {8, 0, 0, 0}, up = {8, 0, 1, page}, x = {8, sp, dp, page};
  std::vector<std::vector<uint16_t>> dense(k), src(k);
  std::vector<const void*> dense_ptr(k), src_ptr(k);
  for (int r = 0; r < k; ++r) { dense[r] = random_u16(size_t(ao_moe_shard_elems(&m, &flat, 0, k)), 11 * r + k); dense_ptr[r] = dense[r].data(); }
  for (int r = 0; r < k; ++r) {
    if (sp) {
      src[r].assign(size_t(ao_moe_shard_elems(&m, &up, 1, k)), 0xEEEE);
      CHECK(ao_reshard_weights_moe(&m, &up, k, k, r, dense_ptr.data(), src[r].data()) == AO_OK);
    } else {
      src[r] = dense[r];
    }
    src_ptr[r] = src[r].data();
  }
  for (int rp = 0; rp < kp; ++rp) {
    amoeba_plan_s plan;
    std::string err;
    CHECK(amoeba::build_plan(&plan, &s, k, kp, rp, &err));
    CHECK(size_t(plan.src_layer_bytes) * s.n_layers == src[0].size() * 2);
    std::vector<uint16_t> want(size_t(plan.dst_layer_bytes) * s.n_layers / 2, 0xEEEE);
    CHECK(want.size() == size_t(ao_moe_shard_elems(&m, &x, dp, kp)));
    CHECK(ao_reshard_weights_moe(&m, &x, k, kp, rp, src_ptr.data(), want.data()) == AO_OK);
    apply_and_compare(plan, s, src, k, want);
  }
}

static void kv_case(int k, int kp, int lay_s, int lay_d) {
  ao_kv c = {2, 8, 4, 2, 4, lay_s, lay_d, 4, 7, 20, 16};
  const int32_t lens[4] = {13, 0, 8, 22};
  int32_t table[4 * 7];
  std::fill(table, table + 28, -1);
  int next = 19;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < (lens[i] + 3) / 4; ++j) table[i * 7 + j] = next--;
  const int64_t be_s = ao_kv_block_elems(&c, k), be_d = ao_kv_block_elems(&c, kp);
  std::vector<std::vector<uint16_t>> pools(k);
  std::vector<const void*> ptr(k);
  for (int r = 0; r < k; ++r) { pools[r] = random_u16(size_t(2 * 20 * be_s), 100 + r); ptr[r] = pools[r].data(); }
  for (int rp = 0; rp < kp; ++rp) {
    const size_t n = size_t(2 * 16 * be_d), guard = 64;
    std::vector<uint16_t> dst(n + 2 * guard, 0xABCD);
    int32_t out[28];
    int64_t total = -1;
    CHECK(ao_reshard_kv(&c, k, kp, rp, ptr.data(), table, lens, dst.data() + guard, out, &total) == AO_OK);
    CHECK(total == 4 + 0 + 2 + 6);
    for (size_t i = 0; i < guard; ++i) CHECK(dst[i] == 0xABCD && dst[guard + n + i] == 0xABCD);
  }
}

static void merge_case(int m, int k) {
  ao_kv c = {2, 8, 4, 2, 4, 0, 0, 3, 6, 12, 12 * m};
  const int32_t lens[4][3] = {{13, 1, 8}, {5, 22, 3}, {16, 2, 7}, {1, 1, 9}};
  std::vector<std::vector<int32_t>> tables(m, std::vector<int32_t>(18, -1));
  for (int g = 0; g < m; ++g) { int next = (g * 5) % 12; for (int i = 0; i < 3; ++i) for (int j = 0; j < (lens[g][i] + 3) / 4; ++j) { tables[g][i * 6 + j] = next; next = (next + 1) % 12; } }
  const int64_t be = ao_kv_block_elems(&c, k);
  for (int rp = 0; rp < k * m; ++rp) {
    const int g = rp % m;
    std::vector<std::vector<uint16_t>> pools(m);
    std::vector<const void*> remote(m, nullptr);
    std::vector<const int32_t*> tp(m), lp(m);
    for (int g2 = 0; g2 < m; ++g2) { pools[g2] = random_u16(size_t(2 * 12 * be), 200 + g2); tp[g2] = tables[g2].data(); lp[g2] = lens[g2]; if (g2 != g) remote[g2] = pools[g2].data(); }
    std::vector<int32_t> out(size_t(m * 18));
    int64_t n = -1;
    CHECK(ao_merge_kv_inplace(&c, k, m, rp, pools[g].data(), remote.data(), tp.data(), lp.data(), out.data(), &n) == AO_OK);
    CHECK(n >= 0);
  }
}

static void merge_base_case(int m, int k, int lay_s, int lay_d) {
  const int32_t lens[4][3] = {{13, 1, 8}, {5, 22, 3}, {16, 2, 7}, {1, 1, 9}};
  int64_t total = 0;
  for (int g = 0; g < m; ++g) for (int i = 0; i < 3; ++i) total += (lens[g][i] + 3) / 4;
  ao_kv c = {2, 8, 4, 2, 4, lay_s, lay_d, 3, 6, 12, total + 1};
  std::vector<std::vector<int32_t>> tables(m, std::vector<int32_t>(18, -1));
  for (int g = 0; g < m; ++g) { int next = (g * 5) % 12; for (int i = 0; i < 3; ++i) for (int j = 0; j < (lens[g][i] + 3) / 4; ++j) { tables[g][i * 6 + j] = next; next = (next + 1) % 12; } }
  const int64_t be_s = ao_kv_block_elems(&c, k), be_d = ao_kv_block_elems(&c, k * m);
  for (int rp = 0; rp < k * m; ++rp) {
    std::vector<std::vector<uint16_t>> pools(m);
    std::vector<const void*> pp(m);
    std::vector<const int32_t*> tp(m), lp(m);
    for (int g2 = 0; g2 < m; ++g2) { pools[g2] = random_u16(size_t(2 * 12 * be_s), 300 + g2); pp[g2] = pools[g2].data(); tp[g2] = tables[g2].data(); lp[g2] = lens[g2]; }
    const size_t n = size_t(2 * (total + 1) * be_d), guard = 64;
    std::vector<uint16_t> fresh(n + 2 * guard, 0xABCD);
    std::vector<int32_t> out(size_t(m * 18));
    int64_t mig = -1, dfr = -1;
    CHECK(ao_merge_kv_base(&c, k, m, rp, pp.data(), tp.data(), lp.data(), fresh.data() + guard, out.data(), &mig, &dfr) == AO_OK);
    CHECK(mig + dfr == total);
    for (size_t i = 0; i < guard; ++i) CHECK(fresh[i] == 0xABCD && fresh[guard + n + i] == 0xABCD);
  }
}

int main() {
  const int tps[][2] = {{1, 1}, {1, 2}, {2, 1}, {1, 4}, {4, 1}, {2, 4}, {4, 2}, {2, 2}};
  for (auto& t : tps) {
    weights_case(t[0], t[1], false, false, 4, 64);
    weights_case(t[0], t[1], false, true, 4, 64);
    weights_case(t[0], t[1], true, true, 4, 1000);
    weights_case(t[0], t[1], true, false, 8, 128);
    moe_case(t[0], t[1], false, false, 0);
    moe_case(t[0], t[1], false, true, 64);
    moe_case(t[0], t[1], true, true, 1000);
    moe_case(t[0], t[1], true, false, 64);
    for (int ls = 0; ls < 2; ++ls) for (int ld = 0; ld < 2; ++ld) kv_case(t[0], t[1], ls, ld);
  }
  merge_case(4, 1); merge_case(2, 2); merge_case(2, 1);
  for (int ls = 0; ls < 2; ++ls) for (int ld = 0; ld < 2; ++ld) { merge_base_case(4, 1, ls, ld); merge_base_case(2, 2, ls, ld); }
  std::printf("sanitize driver: %d failure(s)\n", failures);
  return failures ? 1 : 0;
}
