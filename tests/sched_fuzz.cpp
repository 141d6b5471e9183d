// Host-only stress of the scheduler library under AddressSanitizer and UBSan: random
// arrivals, iterations and token kinds on tiny pools; after every call each instance's
// blocks must be accounted for exactly once (free + held by its requests).  Exit status 0 = clean.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../include/pascal_sched.h"

#define OK(x) do { int s_ = (x); if (s_ < 0) { std::fprintf(stderr, "status %d at line %d\n", s_, __LINE__); return 1; } } while (0)

int main(int argc, char** argv) {
  const int seeds = argc > 1 ? std::atoi(argv[1]) : 30;
  for (int seed = 0; seed < seeds; ++seed) {
    std::mt19937 rng(seed);
    auto uni = [&](int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); };
    pascal_config cfg{};
    cfg.num_instances = uni(1, 4);
    cfg.gpu_blocks = uni(6, 40);
    cfg.block_tokens = 1 << uni(0, 4);
    cfg.quantum_tokens = uni(1, 12);
    cfg.demote_tokens = uni(8, 200);
    cfg.headroom_blocks = uni(0, 3);
    cfg.max_batch = uni(0, 3);
    cfg.target_tpot_s = 0.05;
    pascal_sched* s = nullptr;
    OK(pascal_create(&cfg, &s));
    const int cap = cfg.gpu_blocks * cfg.block_tokens;
    double now = 0;
    int n_req = 0, live = 0;
    std::vector<int32_t> rids, lens, kinds, blocks, tables;
    std::vector<pascal_op> ops;
    for (int step = 0; step < 600; ++step) {
      now += 0.01 * uni(1, 9);
      if (live < 12 && uni(0, 3) == 0) {
        int32_t rid, inst;
        OK(pascal_submit(s, uni(1, cap / 3 > 1 ? cap / 3 : 1), now, &rid, &inst));
        ++n_req; ++live;
      }
      const int i = uni(0, cfg.num_instances - 1);
      int32_t n_sel, n_ops, n_blk;
      OK(pascal_plan(s, i, &n_sel, &n_ops, &n_blk));
      rids.resize(n_sel); lens.resize(n_sel); kinds.resize(n_sel);
      ops.resize(n_ops); blocks.resize(n_blk);
      OK(pascal_plan_batch(s, i, rids.data(), lens.data(), n_sel));
      OK(pascal_ops(s, i, ops.data(), n_ops, blocks.data(), n_blk));
      int maxb = 1;
      for (int k = 0; k < n_sel; ++k) maxb = std::max(maxb, (lens[k] + cfg.block_tokens - 1) / cfg.block_tokens);
      tables.assign((size_t)n_sel * maxb, 0);
      OK(pascal_plan_block_tables(s, i, tables.data(), maxb, -1));
      for (int k = 0; k < n_sel; ++k) {
        pascal_request_info info;
        OK(pascal_request(s, rids[k], &info));
        const int u = uni(0, 99);
        kinds[k] = (lens[k] + 1 >= cap || u < 3) ? PASCAL_END_OF_SEQUENCE
                   : (info.phase == PASCAL_REASONING && u < 10) ? PASCAL_END_OF_REASONING : PASCAL_TOKEN;
        live -= kinds[k] == PASCAL_END_OF_SEQUENCE;
      }
      OK(pascal_commit(s, i, now, kinds.data(), n_sel, &n_ops, &n_blk));
      ops.resize(n_ops); blocks.resize(n_blk);
      OK(pascal_ops(s, i, ops.data(), n_ops, blocks.data(), n_blk));
      // conservation: every block of every instance is free or held by exactly one request
      std::vector<std::vector<int>> seen(cfg.num_instances, std::vector<int>(cfg.gpu_blocks, 0));
      std::vector<int> held(cfg.num_instances, 0);
      std::vector<int32_t> b(cfg.gpu_blocks);
      for (int r = 0; r < n_req; ++r) {
        pascal_request_info info;
        OK(pascal_request(s, r, &info));
        const int n = pascal_request_blocks(s, r, b.data(), cfg.gpu_blocks);
        OK(n);
        int32_t vis;
        OK(pascal_request_visible_tokens(s, r, now, &vis));
        if (vis < 0 || vis > info.answering_tokens) { std::fprintf(stderr, "pacer out of range\n"); return 2; }
        for (int k = 0; k < n; ++k) {
          if (b[k] < 0 || b[k] >= cfg.gpu_blocks || seen[info.instance][b[k]]++) { std::fprintf(stderr, "block owned twice (seed %d)\n", seed); return 2; }
          ++held[info.instance];
        }
      }
      for (int j = 0; j < cfg.num_instances; ++j) {
        int32_t free_blocks;
        OK(pascal_instance_signals(s, j, now, nullptr, nullptr, nullptr, nullptr, &free_blocks));
        if (free_blocks + held[j] != cfg.gpu_blocks) { std::fprintf(stderr, "blocks leaked (seed %d step %d)\n", seed, step); return 2; }
      }
    }
    pascal_destroy(s);
  }
  std::printf("clean\n");
  return 0;
}
