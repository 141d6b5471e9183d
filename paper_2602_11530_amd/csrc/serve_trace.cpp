// serve_trace — a native driver: the scheduler library (pascal_sched.h) decides, the
// kernel library (pkv.h) executes, no Python in between.  It serves a synthetic trace
// (Poisson arrivals, fixed prompt, uniform reasoning and answering lengths: the shape of
// the paper's characterization workload, Section III-A) on several instances whose KV
// pools all live on the one GPU, and checks after every move of a request's KV cache —
// eviction, reload, migration, completion — that the blocks hold exactly the rows that
// were written for that request.  Every K/V row is a fixed function of (request, layer,
// position), so the check needs no second copy of the data.
//
// Time is simulated (an iteration costs a fixed part plus a part proportional to the
// batch's KV footprint); the GPU time of the kernels is measured and reported next to it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <random>
#include <string>
#include <vector>

#include "../../include/pascal_sched.h"
#include "../../include/pkv.h"

namespace {

constexpr int kHq = 40, kHkv = 8, kD = 128, kB = 16;
constexpr int64_t kBlockBytes = (int64_t)kHkv * kB * kD * 2;
constexpr int kRowElems = kHkv * kD;   // one token's K (or V) row over all KV heads

#define HIP_OK(x)                                                                       \
  do {                                                                                  \
    hipError_t e_ = (x);                                                                \
    if (e_ != hipSuccess) {                                                             \
      std::fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
      std::exit(2);                                                                     \
    }                                                                                   \
  } while (0)
#define PKV_OK_(x)                                                                      \
  do {                                                                                  \
    int s_ = (x);                                                                       \
    if (s_ != PKV_OK) {                                                                 \
      std::fprintf(stderr, "pkv error %d (%s) at line %d\n", s_, pkv_status_string(s_), __LINE__); \
      std::exit(3);                                                                     \
    }                                                                                   \
  } while (0)
#define SCHED_OK(x)                                                                     \
  do {                                                                                  \
    int s_ = (x);                                                                       \
    if (s_ < 0) {                                                                       \
      std::fprintf(stderr, "scheduler error %d (%s) at line %d\n", s_, pascal_status_string(s_), __LINE__); \
      std::exit(4);                                                                     \
    }                                                                                   \
  } while (0)

struct Options {
  int requests = 48, instances = 2, blocks = 160, layers = 2, prompt = 64, lo = 32, hi = 256;
  int quantum = 64, demote = 400, headroom = 1;
  double rate = 12.0, tpot = 0.05;
  uint64_t seed = 20260217;
};

// bf16 bit pattern of a small value in (-2, 2), a fixed function of its coordinates.
inline uint16_t kv_value(uint64_t seed, int pool, int rid, int layer, int pos, int elem) {
  uint64_t x = seed ^ ((uint64_t)pool << 60) ^ ((uint64_t)rid << 40) ^ ((uint64_t)layer << 32) ^
               ((uint64_t)pos << 12) ^ (uint64_t)elem;
  x ^= x >> 33; x *= 0xff51afd7ed558ccdULL; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL; x ^= x >> 33;
  const uint16_t sign = (uint16_t)((x >> 15) & 1) << 15;
  const uint16_t exp = (uint16_t)(120 + (x & 7)) << 7;      // 2^-7 .. 2^0
  const uint16_t man = (uint16_t)((x >> 8) & 0x7f);
  return sign | exp | man;
}

struct Server {
  Options o;
  pascal_sched* sched = nullptr;
  hipStream_t stream = nullptr;
  int maxb = 0;
  // device
  std::vector<uint16_t*> k_pool, v_pool;           // [instance * layers + layer]
  uint16_t *staging = nullptr, *q = nullptr, *k_new = nullptr, *v_new = nullptr, *out = nullptr;
  int32_t *tables_d = nullptr, *lens_d = nullptr, *ids_d = nullptr, *ids2_d = nullptr;
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
  int32_t* id_faults = nullptr;   // device counter of block ids the kernels refused to follow
  int max_batch = 0;
  // pinned host
  uint16_t* h_stage = nullptr;                     // upload / download area, one request image
  int32_t *h_tables = nullptr, *h_lens = nullptr, *h_ids = nullptr;
  uint16_t *h_q = nullptr, *h_new = nullptr;
  std::vector<uint16_t*> image_pool;               // recycled pinned images of offloaded requests
  std::map<int, uint16_t*> host_store;             // request -> image [layers][2][n_blocks][block]
  // accounting
  long checks = 0, iterations = 0, op_count[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  double gpu_ms = 0.0;
  hipEvent_t ev0 = nullptr, ev1 = nullptr;

  uint16_t* pool(bool v, int inst, int layer) { return (v ? v_pool : k_pool)[inst * o.layers + layer]; }
  size_t image_elems() const { return (size_t)o.layers * 2 * maxb * (kBlockBytes / 2); }

  void setup() {
    maxb = (o.prompt + 2 * o.hi + kB - 1) / kB + 1;
    max_batch = o.blocks;   // a batch cannot have more requests than the instance has blocks
    pascal_config cfg{};
    cfg.num_instances = o.instances;
    cfg.gpu_blocks = o.blocks;
    cfg.block_tokens = kB;
    cfg.quantum_tokens = o.quantum;
    cfg.demote_tokens = o.demote;
    cfg.headroom_blocks = o.headroom;
    cfg.target_tpot_s = o.tpot;
    SCHED_OK(pascal_create(&cfg, &sched));
    HIP_OK(hipStreamCreate(&stream));
    HIP_OK(hipEventCreate(&ev0));
    HIP_OK(hipEventCreate(&ev1));
    for (int i = 0; i < o.instances * o.layers; ++i) {
      uint16_t *k, *v;
      HIP_OK(hipMalloc(&k, (size_t)o.blocks * kBlockBytes));
      HIP_OK(hipMalloc(&v, (size_t)o.blocks * kBlockBytes));
      HIP_OK(hipMemset(k, 0xff, (size_t)o.blocks * kBlockBytes));   // NaN patterns: unwritten slots must never count
      HIP_OK(hipMemset(v, 0xff, (size_t)o.blocks * kBlockBytes));
      k_pool.push_back(k);
      v_pool.push_back(v);
    }
    HIP_OK(hipMalloc(&staging, (size_t)maxb * kBlockBytes));
    HIP_OK(hipMalloc(&q, (size_t)max_batch * kHq * kD * 2));
    HIP_OK(hipMalloc(&out, (size_t)max_batch * kHq * kD * 2));
    HIP_OK(hipMalloc(&k_new, (size_t)max_batch * kRowElems * 2));
    HIP_OK(hipMalloc(&v_new, (size_t)max_batch * kRowElems * 2));
    HIP_OK(hipMalloc(&tables_d, (size_t)max_batch * maxb * 4));
    HIP_OK(hipMalloc(&lens_d, (size_t)max_batch * 4));
    HIP_OK(hipMalloc(&ids_d, (size_t)maxb * 4));
    HIP_OK(hipMalloc(&ids2_d, (size_t)maxb * 4));
    pkv_attn_shape sh = shape(max_batch);
    PKV_OK_(pkv_attn_workspace_bytes(&sh, &workspace_bytes));
    HIP_OK(hipMalloc(&workspace, workspace_bytes));
    // every order the scheduler issues must name blocks inside the pools: have the library count
    // any id it refuses, and fail the run if the count is not zero at the end
    HIP_OK(hipMalloc(&id_faults, sizeof(int32_t)));
    HIP_OK(hipMemset(id_faults, 0, sizeof(int32_t)));
    PKV_OK_(pkv_set_id_fault_counter(id_faults));
    HIP_OK(hipHostMalloc((void**)&h_stage, (size_t)maxb * kBlockBytes));
    HIP_OK(hipHostMalloc((void**)&h_tables, (size_t)max_batch * maxb * 4));
    HIP_OK(hipHostMalloc((void**)&h_lens, (size_t)max_batch * 4));
    HIP_OK(hipHostMalloc((void**)&h_ids, (size_t)2 * maxb * 4));
    HIP_OK(hipHostMalloc((void**)&h_q, (size_t)max_batch * kHq * kD * 2));
    HIP_OK(hipHostMalloc((void**)&h_new, (size_t)2 * max_batch * kRowElems * 2));
  }

  pkv_attn_shape shape(int S) const {
    pkv_attn_shape sh{};
    sh.num_seqs = S;
    sh.num_q_heads = kHq;
    sh.num_kv_heads = kHkv;
    sh.head_dim = kD;
    sh.block_size = kB;
    sh.max_blocks_per_seq = maxb;
    sh.partition_size = 0;
    sh.max_context_len = 0;
    sh.num_pool_blocks = o.blocks;
    return sh;
  }

  int32_t* upload_ids(const int32_t* ids, int n, int32_t* dst_d, int slot) {
    std::memcpy(h_ids + slot * maxb, ids, (size_t)n * 4);
    HIP_OK(hipMemcpyAsync(dst_d, h_ids + slot * maxb, (size_t)n * 4, hipMemcpyHostToDevice, stream));
    return dst_d;
  }

  uint16_t* take_image() {
    if (!image_pool.empty()) { uint16_t* p = image_pool.back(); image_pool.pop_back(); return p; }
    uint16_t* p;
    HIP_OK(hipHostMalloc((void**)&p, image_elems() * 2));
    return p;
  }

  // The rows the request must hold at positions [0, tokens) of layer `layer`, as block images.
  void expected_image(bool v, int rid, int layer, int tokens, int n_blocks, uint16_t* img) const {
    for (int b = 0; b < n_blocks; ++b)
      for (int h = 0; h < kHkv; ++h)
        for (int t = 0; t < kB; ++t) {
          const int pos = b * kB + t;
          uint16_t* row = img + (((size_t)b * kHkv + h) * kB + t) * kD;
          for (int d = 0; d < kD; ++d)
            row[d] = pos < tokens ? kv_value(o.seed, v, rid, layer, pos, h * kD + d) : 0xffff;
        }
  }

  // Downloads the request's blocks and compares every valid slot with what was written for it.
  void verify(int inst, int rid, const int32_t* blocks, int n_blocks, const char* when) {
    pascal_request_info info;
    SCHED_OK(pascal_request(sched, rid, &info));
    const int tokens = info.kv_tokens;
    const int nb = (tokens + kB - 1) / kB;
    if (nb > n_blocks) { std::fprintf(stderr, "request %d: %d blocks for %d tokens\n", rid, n_blocks, tokens); std::exit(5); }
    upload_ids(blocks, nb, ids_d, 0);
    std::vector<uint16_t> want((size_t)nb * (kBlockBytes / 2));
    for (int l = 0; l < o.layers; ++l)
      for (int v = 0; v < 2; ++v) {
        PKV_OK_(kv_blocks_offload(pool(v, inst, l), ids_d, staging, h_stage, nb, kBlockBytes, o.blocks, stream));
        HIP_OK(hipStreamSynchronize(stream));
        expected_image(v, rid, l, tokens, nb, want.data());
        for (int b = 0; b < nb; ++b)
          for (int h = 0; h < kHkv; ++h) {
            const int valid = std::min(kB, tokens - b * kB);
            const size_t off = (((size_t)b * kHkv + h) * kB) * kD;
            if (std::memcmp(h_stage + off, want.data() + off, (size_t)valid * kD * 2) != 0) {
              std::fprintf(stderr, "KV of request %d differs %s (layer %d, %s, block %d, head %d)\n", rid, when, l,
                           v ? "V" : "K", b, h);
              std::exit(6);
            }
          }
      }
    ++checks;
  }

  void execute(const std::vector<pascal_op>& ops, const std::vector<int32_t>& blocks) {
    for (const pascal_op& op : ops) {
      ++op_count[op.kind];
      const int32_t* ids = blocks.data() + op.first_block;
      const int n = op.n_blocks;
      switch (op.kind) {
        case PASCAL_OP_PREFILL: {
          pascal_request_info info;
          SCHED_OK(pascal_request(sched, op.request, &info));
          upload_ids(ids, n, ids_d, 0);
          for (int l = 0; l < o.layers; ++l)
            for (int v = 0; v < 2; ++v) {
              expected_image(v, op.request, l, info.prompt_tokens, n, h_stage);
              HIP_OK(hipMemcpyAsync(staging, h_stage, (size_t)n * kBlockBytes, hipMemcpyHostToDevice, stream));
              PKV_OK_(kv_blocks_scatter(staging, pool(v, op.instance, l), ids_d, n, kBlockBytes, o.blocks, stream));
              HIP_OK(hipStreamSynchronize(stream));   // h_stage is reused
            }
          break;
        }
        case PASCAL_OP_OFFLOAD:
        case PASCAL_OP_MIGRATE_HOST: {
          verify(op.instance, op.request, ids, n, "before eviction");
          uint16_t* img = take_image();
          upload_ids(ids, n, ids_d, 0);
          for (int l = 0; l < o.layers; ++l)
            for (int v = 0; v < 2; ++v)
              PKV_OK_(kv_blocks_offload(pool(v, op.instance, l), ids_d, staging,
                                        img + ((size_t)l * 2 + v) * maxb * (kBlockBytes / 2), n, kBlockBytes,
                                        o.blocks, stream));
          HIP_OK(hipStreamSynchronize(stream));
          host_store[op.request] = img;
          poison(op.instance, ids, n);
          break;
        }
        case PASCAL_OP_RELOAD: {
          uint16_t* img = host_store.at(op.request);
          upload_ids(ids, n, ids_d, 0);
          for (int l = 0; l < o.layers; ++l)
            for (int v = 0; v < 2; ++v)
              PKV_OK_(kv_blocks_reload(img + ((size_t)l * 2 + v) * maxb * (kBlockBytes / 2), staging,
                                       pool(v, op.instance, l), ids_d, n, kBlockBytes, o.blocks, stream));
          HIP_OK(hipStreamSynchronize(stream));
          host_store.erase(op.request);
          image_pool.push_back(img);
          verify(op.instance, op.request, ids, n, "after reload");
          break;
        }
        case PASCAL_OP_MIGRATE: {
          upload_ids(ids, n, ids_d, 0);
          upload_ids(ids + n, n, ids2_d, 1);
          for (int l = 0; l < o.layers; ++l)
            for (int v = 0; v < 2; ++v)
              PKV_OK_(kv_blocks_move(pool(v, op.instance, l), ids_d, pool(v, op.other_instance, l), ids2_d, n,
                                     kBlockBytes, o.blocks, o.blocks, stream));
          HIP_OK(hipStreamSynchronize(stream));
          verify(op.other_instance, op.request, ids + n, n, "after migration");
          poison(op.instance, ids, n);
          break;
        }
        case PASCAL_OP_FREE:
          verify(op.instance, op.request, ids, n, "at completion");
          poison(op.instance, ids, n);
          break;
        default: break;   // PASCAL_OP_GROW moves no data
      }
    }
  }

  // Freed blocks are overwritten with NaN patterns: a stale table entry would poison an output row.
  void poison(int inst, const int32_t* ids, int n) {
    for (int l = 0; l < o.layers; ++l)
      for (int v = 0; v < 2; ++v)
        for (int k = 0; k < n; ++k)
          HIP_OK(hipMemsetAsync(pool(v, inst, l) + (size_t)ids[k] * (kBlockBytes / 2), 0xff, kBlockBytes, stream));
  }

  // One decode iteration of the planned batch: append the new rows, attend, check the output is finite.
  void run_batch(int inst, const std::vector<int32_t>& rids, const std::vector<int32_t>& lens) {
    const int S = (int)rids.size();
    SCHED_OK(pascal_plan_block_tables(sched, inst, h_tables, maxb, -1));
    std::memcpy(h_lens, lens.data(), (size_t)S * 4);
    HIP_OK(hipMemcpyAsync(tables_d, h_tables, (size_t)S * maxb * 4, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(lens_d, h_lens, (size_t)S * 4, hipMemcpyHostToDevice, stream));
    const pkv_attn_shape sh = shape(S);
    for (int l = 0; l < o.layers; ++l) {
      uint16_t* hk = h_new;
      uint16_t* hv = h_new + (size_t)max_batch * kRowElems;
      for (int s = 0; s < S; ++s) {
        const int pos = lens[s] - 1;   // a first-run request rewrites its last prompt row with the same values
        for (int e = 0; e < kRowElems; ++e) {
          hk[(size_t)s * kRowElems + e] = kv_value(o.seed, 0, rids[s], l, pos, e);
          hv[(size_t)s * kRowElems + e] = kv_value(o.seed, 1, rids[s], l, pos, e);
        }
        for (int e = 0; e < kHq * kD; ++e)
          h_q[(size_t)s * kHq * kD + e] = kv_value(o.seed ^ 0x9e3779b97f4a7c15ULL, 2, rids[s], l, pos, e);
      }
      HIP_OK(hipMemcpyAsync(k_new, hk, (size_t)S * kRowElems * 2, hipMemcpyHostToDevice, stream));
      HIP_OK(hipMemcpyAsync(v_new, hv, (size_t)S * kRowElems * 2, hipMemcpyHostToDevice, stream));
      HIP_OK(hipMemcpyAsync(q, h_q, (size_t)S * kHq * kD * 2, hipMemcpyHostToDevice, stream));
      HIP_OK(hipEventRecord(ev0, stream));
      PKV_OK_(kv_append(k_new, v_new, pool(false, inst, l), pool(true, inst, l), tables_d, lens_d, &sh, stream));
      PKV_OK_(paged_decode_attn(q, pool(false, inst, l), pool(true, inst, l), tables_d, lens_d,
                                1.0f / std::sqrt((float)kD), out, &sh, workspace, workspace_bytes, stream));
      HIP_OK(hipEventRecord(ev1, stream));
      HIP_OK(hipMemcpyAsync(h_q, out, (size_t)S * kHq * kD * 2, hipMemcpyDeviceToHost, stream));
      HIP_OK(hipStreamSynchronize(stream));
      float ms = 0.f;
      HIP_OK(hipEventElapsedTime(&ms, ev0, ev1));
      gpu_ms += ms;
      // |value| < 2 everywhere, so every output element is a convex combination inside (-2, 2)
      for (size_t e = 0; e < (size_t)S * kHq * kD; ++e) {
        const uint16_t bits = h_q[e];
        const int exp = (bits >> 7) & 0xff;
        if (exp == 0xff || exp > 127) {
          std::fprintf(stderr, "attention output out of range (instance %d, layer %d, element %zu: 0x%04x)\n", inst,
                       l, e, bits);
          std::exit(7);
        }
      }
    }
    ++iterations;
  }
};

double iteration_seconds(const std::vector<int32_t>& lens) {
  double tokens = 0;
  for (int32_t L : lens) tokens += L;
  return 0.02 + 4.5e-8 * tokens;
}

}  // namespace

int main(int argc, char** argv) {
  Server sv;
  Options& o = sv.o;
  for (int a = 1; a + 1 < argc; a += 2) {
    const std::string k = argv[a];
    const char* v = argv[a + 1];
    if (k == "--requests") o.requests = std::atoi(v);
    else if (k == "--instances") o.instances = std::atoi(v);
    else if (k == "--blocks") o.blocks = std::atoi(v);
    else if (k == "--layers") o.layers = std::atoi(v);
    else if (k == "--prompt") o.prompt = std::atoi(v);
    else if (k == "--lo") o.lo = std::atoi(v);
    else if (k == "--hi") o.hi = std::atoi(v);
    else if (k == "--quantum") o.quantum = std::atoi(v);
    else if (k == "--demote") o.demote = std::atoi(v);
    else if (k == "--rate") o.rate = std::atof(v);
    else if (k == "--tpot") o.tpot = std::atof(v);
    else if (k == "--seed") o.seed = std::strtoull(v, nullptr, 10);
    else { std::fprintf(stderr, "unknown option %s\n", k.c_str()); return 1; }
  }
  if (o.requests < 1 || o.instances < 1 || o.layers < 1 || o.lo < 1 || o.hi < o.lo || o.prompt < 1 ||
      (o.prompt + 2 * o.hi + kB - 1) / kB + 1 > o.blocks) {
    std::fprintf(stderr, "bad sizes (a request must fit an instance)\n");
    return 1;
  }
  sv.setup();

  // the trace
  std::mt19937_64 rng(o.seed);
  std::exponential_distribution<double> gap(o.rate);
  std::uniform_int_distribution<int> len(o.lo, o.hi);
  std::vector<double> arrival(o.requests);
  std::vector<int> n_reason(o.requests), n_answer(o.requests), made_r(o.requests, 0), made_a(o.requests, 0);
  double t = 0;
  for (int r = 0; r < o.requests; ++r) { t += gap(rng); arrival[r] = t; n_reason[r] = len(rng); n_answer[r] = len(rng); }

  std::vector<double> clock(o.instances, 0.0);
  int next = 0, done = 0;
  std::vector<pascal_op> ops;
  std::vector<int32_t> op_blocks, rids, lens, kinds;
  auto fetch_ops = [&](int inst, int n_ops, int n_blocks) {
    ops.resize(n_ops);
    op_blocks.resize(n_blocks);
    SCHED_OK(pascal_ops(sv.sched, inst, ops.data(), n_ops, op_blocks.data(), n_blocks));
  };
  while (done < o.requests) {
    const int i = (int)(std::min_element(clock.begin(), clock.end()) - clock.begin());
    while (next < o.requests && arrival[next] <= clock[i]) {
      int32_t rid, inst;
      SCHED_OK(pascal_submit(sv.sched, o.prompt, arrival[next], &rid, &inst));
      ++next;
    }
    int32_t n_sel, n_ops, n_blk;
    SCHED_OK(pascal_plan(sv.sched, i, &n_sel, &n_ops, &n_blk));
    fetch_ops(i, n_ops, n_blk);
    sv.execute(ops, op_blocks);
    rids.resize(n_sel);
    lens.resize(n_sel);
    SCHED_OK(pascal_plan_batch(sv.sched, i, rids.data(), lens.data(), n_sel));
    kinds.assign(n_sel, PASCAL_TOKEN);
    if (n_sel == 0) {
      clock[i] = std::max(clock[i] + 0.01, next < o.requests ? arrival[next] : 0.0);
    } else {
      sv.run_batch(i, rids, lens);
      clock[i] += iteration_seconds(lens);
      for (int s = 0; s < n_sel; ++s) {
        const int r = rids[s];
        if (made_r[r] < n_reason[r]) {
          if (++made_r[r] == n_reason[r]) kinds[s] = PASCAL_END_OF_REASONING;
        } else if (++made_a[r] == n_answer[r]) {
          kinds[s] = PASCAL_END_OF_SEQUENCE;
          ++done;
        }
      }
    }
    SCHED_OK(pascal_commit(sv.sched, i, clock[i], kinds.data(), n_sel, &n_ops, &n_blk));
    fetch_ops(i, n_ops, n_blk);
    sv.execute(ops, op_blocks);
  }

  double ttft = 0, worst_qoe = 1;
  int violations = 0, preemptions = 0, migrations = 0;
  for (int r = 0; r < o.requests; ++r) {
    pascal_request_info info;
    SCHED_OK(pascal_request(sv.sched, r, &info));
    if (info.state != PASCAL_FINISHED || info.kv_tokens != o.prompt + n_reason[r] + n_answer[r] - 1) {
      std::fprintf(stderr, "request %d did not finish cleanly\n", r);
      return 8;
    }
    ttft += info.ttft;
    worst_qoe = std::min(worst_qoe, info.qoe);
    violations += info.qoe < 0.95;
    preemptions += info.preemptions;
    migrations += info.migrations;
  }
  for (int i = 0; i < o.instances; ++i) {
    int32_t free_blocks = 0;
    SCHED_OK(pascal_instance_signals(sv.sched, i, 1e18, nullptr, nullptr, nullptr, nullptr, &free_blocks));
    if (free_blocks != o.blocks || !sv.host_store.empty()) { std::fprintf(stderr, "blocks or images leaked\n"); return 9; }
  }
  {
    int32_t refused = -1;
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(&refused, sv.id_faults, sizeof refused, hipMemcpyDeviceToHost));
    PKV_OK_(pkv_set_id_fault_counter(nullptr));
    if (refused != 0) { std::fprintf(stderr, "the kernels refused %d block ids\n", refused); return 10; }
  }
  std::printf("{\"requests\": %d, \"instances\": %d, \"layers\": %d, \"iterations\": %ld, \"kv_checks\": %ld, "
              "\"offloads\": %ld, \"reloads\": %ld, \"migrations\": %ld, \"migrations_via_host\": %ld, "
              "\"mean_ttft_s\": %.3f, \"qoe_violations\": %d, \"worst_qoe\": %.4f, \"preemptions\": %d, "
              "\"requests_migrated\": %d, \"gpu_ms_append_plus_attention\": %.2f, \"ok\": true}\n",
              o.requests, o.instances, o.layers, sv.iterations, sv.checks, sv.op_count[PASCAL_OP_OFFLOAD],
              sv.op_count[PASCAL_OP_RELOAD], sv.op_count[PASCAL_OP_MIGRATE], sv.op_count[PASCAL_OP_MIGRATE_HOST],
              ttft / o.requests, violations, worst_qoe, preemptions, migrations, sv.gpu_ms);
  pascal_destroy(sv.sched);
  return 0;
}
