// CPU tests of the stage runtime's host logic (paper Alg. 2's receive loop, Sec. 3.3's pipeline_limit, the
// deferred weight-gradient groups, Sec. 5.2's bucket plan and Sec. 5.3's chunks) with a simulated event layer:
// no GPU, no HIP.  Built by tests/test_host_runtime.py with -fsanitize=address,undefined and with
// -fsanitize=thread.  The model stage below does with counters what stage.cpp does with streams and events,
// and takes every decision from host_logic.h, as stage.cpp does.
#include "../../paper_2110_13005_amd/csrc/host_logic.h"

#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <string>
#include <thread>
#include <utility>
#include <vector>

using namespace axonn::host;

#define CHECK(cond)                                                                   \
  do {                                                                                \
    if (!(cond)) {                                                                    \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond);   \
      std::exit(1);                                                                   \
    }                                                                                 \
  } while (0)

namespace {

struct SlotRec { int state = SLOT_FREE; int mb_id = -1; };
struct Msg { int kind, mb_id; long ready_at; };   // ready_at: tick from which the payload "has arrived" (-1: no event)

// What stage.cpp keeps per stage, without the device.
struct ModelStage {
  int M, P, group, n_streams;
  bool ckpt;
  std::vector<SlotRec> slots;
  std::vector<Msg> inbox;
  int in_flight = 0, fwd_issued = 0, bwd_issued = 0, bwd_count = 0, fwd_rr = 0;
  long tick = 0;
  std::vector<std::pair<int, int>> log;            // (kind, mb) in dispatch order
  std::vector<std::vector<int>> wgrad_passes;      // microbatches of each weight-gradient pass
  std::vector<int> awaiting_mb;                    // microbatch of each slot in AWAIT_WGRAD, by slot
  std::vector<int> stream_of;                      // stream index per dispatched message
  bool final_pass_seen = false;
  int max_in_flight = 0;

  ModelStage(int M_, int P_, int group_, int n_streams_, bool ckpt_ = false)
      : M(M_), P(P_), group(group_), n_streams(n_streams_), ckpt(ckpt_), slots(P_), awaiting_mb(P_, -1) {}

  int post(int kind, int mb, long ready_at) {
    const auto posted = [this](size_t i) { return std::make_pair(inbox[i].kind, inbox[i].mb_id); };
    const int rc = check_post(kind, mb, inbox.size(), posted, kind == 0 ? fwd_issued : bwd_issued, M);
    if (rc == POST_OK) inbox.push_back(Msg{kind, mb, ready_at});
    return rc;
  }
  void flush(bool final_pass) {
    std::vector<int> pass;
    for (size_t i = 0; i < slots.size(); ++i)
      if (slots[i].state == SLOT_AWAIT_WGRAD) pass.push_back(awaiting_mb[i]);
    if (pass.empty()) return;
    CHECK(!final_pass_seen);
    wgrad_passes.push_back(pass);
    release_awaiting(slots);
    final_pass_seen = final_pass;
  }
  int forward(int mb) {
    int si = -1;
    int adm = admit_forward(slots, mb, in_flight, P, &si);
    if (adm == FWD_NEEDS_FLUSH) {
      flush(false);
      adm = admit_forward(slots, mb, in_flight, P, &si);
    }
    if (adm != FWD_OK) return adm;
    commit_forward(slots, si, mb, &in_flight);
    max_in_flight = std::max(max_in_flight, in_flight);
    return FWD_OK;
  }
  int backward(int mb) {
    const int si = admit_backward(slots, mb);
    if (si < 0) return -1;
    const bool last = bwd_count + 1 == M;
    ++bwd_count;
    commit_backward(slots, si, ckpt, &in_flight);
    if (ckpt) {
      wgrad_passes.push_back({mb});
    } else {
      awaiting_mb[si] = mb;
      switch (wgrad_action(last, group, count_state(slots, SLOT_AWAIT_WGRAD))) {
        case WGRAD_FLUSH_FINAL: flush(true); break;
        case WGRAD_FLUSH: flush(false); break;
        default: break;
      }
    }
    return 0;
  }
  // The receive loop.  Returns 0 when the batch is dispatched, 1 when a non-blocking call has nothing more to do,
  // -2 if nothing can ever be scheduled, -3 when a wait expired.  One tick passes per fruitless look.
  int run(bool blocking, double wait_limit_ticks, int* n_dispatched = nullptr) {
    WaitClock wait(wait_limit_ticks);
    const auto posted = [this](size_t i) { return std::make_pair(inbox[i].kind, inbox[i].mb_id); };
    const auto arrived = [this](size_t i) { return (inbox[i].ready_at < 0 || inbox[i].ready_at <= tick) ? 1 : 0; };
    while (fwd_issued < M || bwd_issued < M) {
      bool any = false;
      int err = 0;
      const int c = choose_message(inbox.size(), posted, arrived, slots, in_flight, P, &any, &err);
      CHECK(err == 0);
      if (c < 0) {
        if (!blocking) return 1;
        if (!any) return -2;
        if (wait.expired((double)tick)) return -3;
        ++tick;
        continue;
      }
      wait.dispatched();
      const Msg m = inbox[c];
      inbox.erase(inbox.begin() + c);
      stream_of.push_back(stream_index(m.kind, n_streams, &fwd_rr));
      if (m.kind == 0) { CHECK(forward(m.mb_id) == FWD_OK); ++fwd_issued; }
      else { CHECK(backward(m.mb_id) == 0); ++bwd_issued; }
      log.push_back({m.kind, m.mb_id});
      if (n_dispatched) ++*n_dispatched;
      // invariants of Sec. 3.3 / Alg. 2 after every dispatch
      CHECK(in_flight <= P);
      CHECK(count_state(slots, SLOT_LIVE) == in_flight);
    }
    return 0;
  }
  void check_batch_complete() const {
    CHECK((int)log.size() == 2 * M);
    std::vector<int> f(M, -1), b(M, -1);
    for (size_t i = 0; i < log.size(); ++i) {
      auto& v = log[i].first == 0 ? f : b;
      CHECK(v[log[i].second] < 0);            // each message exactly once
      v[log[i].second] = (int)i;
    }
    for (int i = 0; i < M; ++i) CHECK(f[i] >= 0 && b[i] > f[i]);   // backward only after its forward
    // every microbatch's weight gradients formed exactly once, none left waiting, the last pass marked final
    std::multiset<int> seen;
    for (const auto& p : wgrad_passes) for (int mb : p) seen.insert(mb);
    CHECK((int)seen.size() == M);
    for (int i = 0; i < M; ++i) CHECK(seen.count(i) == 1);
    CHECK(count_state(slots, SLOT_AWAIT_WGRAD) == 0 && in_flight == 0);
    if (!ckpt) CHECK(final_pass_seen);
  }
};

void test_pipeline_limit_and_order(unsigned seed) {
  std::mt19937 rng(seed);
  for (int rep = 0; rep < 200; ++rep) {
    const int M = 1 + rng() % 12, P = 1 + rng() % M, group = rng() % 5, ns = 1 + rng() % 4;
    const bool ckpt = rng() % 4 == 0;
    ModelStage st(M, P, group, ns, ckpt);
    // a random valid interleaving of posts (posting order != arrival order: random ready ticks)
    std::vector<std::pair<int, int>> posts;
    for (int i = 0; i < M; ++i) { posts.push_back({0, i}); posts.push_back({1, i}); }
    std::shuffle(posts.begin(), posts.end(), rng);
    for (auto& pm : posts) CHECK(st.post(pm.first, pm.second, (long)(rng() % 50) - 5) == POST_OK);
    CHECK(st.run(true, 1e9) == 0);
    st.check_batch_complete();
    CHECK(st.max_in_flight <= P);
    if (!ckpt && group > 0)
      for (size_t i = 0; i + 1 < st.wgrad_passes.size(); ++i) CHECK((int)st.wgrad_passes[i].size() <= std::max(group, 1) || P < group);
    for (size_t i = 0; i < st.log.size(); ++i) {
      if (st.log[i].first == 1 || ns == 1) CHECK(st.stream_of[i] == 0);       // backward chains on stream 0
      else CHECK(st.stream_of[i] >= 1 && st.stream_of[i] < ns);
    }
  }
}

void test_arrival_order_decides() {
  // two forwards posted; the second arrives first: it is dispatched first (Alg. 2 runs whatever has arrived)
  ModelStage st(2, 2, 0, 2);
  CHECK(st.post(0, 0, 10) == POST_OK);
  CHECK(st.post(0, 1, 0) == POST_OK);
  CHECK(st.post(1, 0, 20) == POST_OK);
  CHECK(st.post(1, 1, 12) == POST_OK);
  CHECK(st.run(true, 1e9) == 0);
  CHECK(st.log[0] == std::make_pair(0, 1) && st.log[1] == std::make_pair(0, 0));
  CHECK(st.log[2] == std::make_pair(1, 1) && st.log[3] == std::make_pair(1, 0));
  st.check_batch_complete();
}

void test_duplicates_and_surplus() {
  ModelStage st(3, 2, 0, 2);
  CHECK(st.post(0, 0, -1) == POST_OK);
  CHECK(st.post(0, 0, -1) == POST_DUPLICATE);
  CHECK(st.post(1, 0, -1) == POST_OK);                 // same microbatch, other kind: fine
  CHECK(st.post(0, 1, -1) == POST_OK);
  CHECK(st.post(0, 2, -1) == POST_OK);
  CHECK(st.post(0, 3, -1) == POST_SURPLUS);            // a fourth forward in a batch of three
  int n = 0;
  CHECK(st.run(false, 1e9, &n) == 1);                  // non-blocking: f0 f1 (limit 2) b0 f2, then nothing admissible has arrived
  CHECK(n == 4 && st.in_flight == 2);
  CHECK(st.post(0, 1, -1) == POST_SURPLUS);            // issued forwards count towards the batch
  CHECK(st.forward(1) == FWD_ALREADY_LIVE);
  CHECK(st.forward(7) == FWD_PIPELINE_FULL);
  CHECK(st.forward(-1) == FWD_NEGATIVE_ID);
  CHECK(st.backward(0) == -1);                         // already consumed
  CHECK(st.run(true, 1e9) == -2);                      // two backwards expected, none posted: cannot progress
  CHECK(st.post(1, 2, -1) == POST_OK && st.post(1, 1, -1) == POST_OK);
  CHECK(st.run(true, 1e9) == 0);
  st.check_batch_complete();
}

void test_backward_without_forward_never_runs() {
  ModelStage st(2, 1, 0, 1);
  CHECK(st.post(1, 0, -1) == POST_OK);                 // gradient for a microbatch whose forward is not even posted
  CHECK(st.run(true, 1e9) == -2);
  CHECK(st.log.empty());
  CHECK(st.post(0, 0, -1) == POST_OK);
  int n = 0;
  CHECK(st.run(false, 1e9, &n) == 1 && n == 2);
  CHECK(st.log[0] == std::make_pair(0, 0) && st.log[1] == std::make_pair(1, 0));
}

void test_wait_limit_is_per_wait() {
  // messages arrive every 40 ticks, the limit is 50: a batch of 6 takes > 200 ticks in all and still succeeds
  ModelStage st(3, 3, 0, 2);
  for (int i = 0; i < 3; ++i) { CHECK(st.post(0, i, 40 * (i + 1)) == POST_OK); CHECK(st.post(1, i, 40 * (i + 4)) == POST_OK); }
  CHECK(st.run(true, 50.0) == 0);
  CHECK(st.tick > 200);
  st.check_batch_complete();
  // one message later than the limit: the wait expires; the posted message is still there and a second run resumes
  ModelStage late(1, 1, 0, 1);
  CHECK(late.post(0, 0, 0) == POST_OK && late.post(1, 0, 500) == POST_OK);
  CHECK(late.run(true, 50.0) == -3);
  CHECK(late.inbox.size() == 1 && late.fwd_issued == 1 && late.in_flight == 1);
  CHECK(late.run(true, 1e9) == 0);
  late.check_batch_complete();
  WaitClock w(10.0);
  CHECK(!w.expired(100.0) && !w.expired(109.0) && w.expired(111.0));
  w.dispatched();
  CHECK(!w.expired(200.0));
}

void test_wgrad_groups() {
  // stored activations, 8 microbatches all in flight, groups of 3: passes of 3, 3 and 2, the last one final
  ModelStage st(8, 8, 3, 2);
  for (int i = 0; i < 8; ++i) CHECK(st.post(0, i, -1) == POST_OK);
  for (int i = 0; i < 8; ++i) CHECK(st.post(1, i, -1) == POST_OK);
  CHECK(st.run(true, 1e9) == 0);
  CHECK(st.wgrad_passes.size() == 3);
  CHECK(st.wgrad_passes[0].size() == 3 && st.wgrad_passes[1].size() == 3 && st.wgrad_passes[2].size() == 2);
  CHECK(st.wgrad_passes[2].back() == 7 || st.wgrad_passes[2].front() == 7);
  st.check_batch_complete();
  // group 0 with fewer slots than microbatches: a pass is forced whenever a forward finds no free slot
  ModelStage tight(6, 2, 0, 2);
  for (int i = 0; i < 6; ++i) { CHECK(tight.post(0, i, -1) == POST_OK); CHECK(tight.post(1, i, -1) == POST_OK); }
  CHECK(tight.run(true, 1e9) == 0);
  tight.check_batch_complete();
  CHECK(tight.wgrad_passes.size() >= 3);
  CHECK(wgrad_action(false, 0, 100) == WGRAD_NONE && wgrad_action(false, 2, 1) == WGRAD_NONE);
  CHECK(wgrad_action(false, 2, 2) == WGRAD_FLUSH && wgrad_action(true, 0, 1) == WGRAD_FLUSH_FINAL);
}

void test_bucket_plan(unsigned seed) {
  std::mt19937_64 rng(seed);
  for (int rep = 0; rep < 300; ++rep) {
    const uint64_t bucket = 8 * (1 + rng() % 64), n = 1 + rng() % (bucket * 9);
    const uint64_t nb = bucket_count(n, bucket);
    CHECK(nb == (n + bucket - 1) / bucket);
    for (int desc = 0; desc < 2; ++desc) {
      uint64_t covered = 0;
      std::vector<char> hit(nb, 0);
      for (uint64_t i = 0; i < nb; ++i) {
        const BucketPlan p = bucket_plan(n, bucket, 3, i, desc != 0);
        CHECK(p.index == (desc ? nb - 1 - i : i) && !hit[p.index]);
        hit[p.index] = 1;
        CHECK(p.offset == p.index * bucket && p.count >= 1 && p.count <= bucket && p.offset + p.count <= n);
        CHECK((p.index + 1 < nb) == (p.count == bucket) || p.count == bucket);   // only the last bucket is ragged
        if (p.index + 1 == nb) CHECK(p.offset + p.count == n);
        CHECK(p.set == (int)(i % 3));                    // three buffer sets in rotation, in processing order
        covered += p.count;
      }
      CHECK(covered == n);
    }
    // chunks of k buckets of the descending pass tile [0, n) from the top down
    const uint64_t k = 1 + rng() % 5;
    uint64_t expect_hi = n;
    for (uint64_t i = 0; i < nb; i += k) {
      uint64_t lo = 0, hi = 0;
      chunk_span(n, bucket, k, i, &lo, &hi);
      CHECK(hi == expect_hi && lo < hi && lo % bucket == 0);
      CHECK((hi - lo + bucket - 1) / bucket == std::min<uint64_t>(k, nb - i));
      expect_hi = lo;
    }
    CHECK(expect_hi == 0);
    // the gate of a chunk: the layer that holds its lowest element; every layer the chunk touches is at or
    // above it, i.e. final no later (gradients become final from the last layer down)
    const int L = 1 + (int)(rng() % 6);
    std::vector<uint64_t> begin(L);
    for (int l = 0; l < L; ++l) begin[l] = (uint64_t)l * (n / L + 1);
    for (uint64_t i = 0; i < nb; i += k) {
      uint64_t lo = 0, hi = 0;
      chunk_span(n, bucket, k, i, &lo, &hi);
      const int l = lowest_layer(begin.data(), L, lo);
      CHECK(l >= 0 && l < L && begin[l] <= lo && (l + 1 == L || begin[l + 1] > lo));
    }
  }
  // the benchmark's optimizer problem: 1.6e9 parameters in buckets of 2^26 -> 24 buckets, the last of 56 496 128
  CHECK(bucket_count(1600000000ull, 1ull << 26) == 24);
  CHECK(bucket_plan(1600000000ull, 1ull << 26, 3, 23, false).count == 56496128ull);
  CHECK(bucket_plan(1600000000ull, 1ull << 26, 3, 0, true).count == 56496128ull);
}

void test_two_stages_two_threads() {
  // handles are independent: two host threads each drive a stage of their own (no shared state in the logic)
  auto work = [](unsigned seed) { test_pipeline_limit_and_order(seed); test_bucket_plan(seed); };
  std::thread a(work, 11u), b(work, 12u);
  a.join();
  b.join();
}

}  // namespace

int main() {
  test_pipeline_limit_and_order(1);
  test_arrival_order_decides();
  test_duplicates_and_surplus();
  test_backward_without_forward_never_runs();
  test_wait_limit_is_per_wait();
  test_wgrad_groups();
  test_bucket_plan(2);
  test_two_stages_two_threads();
  std::puts("host logic: all checks passed");
  return 0;
}
