// Self-test of the host-only part of libtutti (csrc/tutti_host.cpp) for the sanitizers: random call sequences
// against exact-size heap buffers, so that an out-of-bounds access or undefined arithmetic fails even when the
// results happen to be right.  Results are checked against simple models.  Usage: host_selftest <rounds>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <vector>

#include "tutti.h"

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() {
  g_state ^= g_state << 13;
  g_state ^= g_state >> 7;
  g_state ^= g_state << 17;
  return static_cast<uint32_t>(g_state >> 11);
}

#define CHECK(c)                                                      \
  do {                                                                \
    if (!(c)) {                                                       \
      std::printf("line %d: %s\n", __LINE__, #c);                     \
      return 1;                                                       \
    }                                                                 \
  } while (0)

// get_iocb / reap against a model: slots are handed out in ring order and come back in ring order
static int ring_round() {
  const uint32_t depth = 1 + rnd() % 9;
  std::vector<uint8_t> flags(depth);
  std::vector<uint32_t> cq(16 + depth, 0xffffffffu);  // header (16 words) + depth entries, nothing beyond
  cq[0] = 0;
  cq[1] = depth;
  tutti_sq_state s;
  CHECK(tutti_sq_state_init(&s, depth, flags.data()) == TUTTI_OK);
  std::deque<uint32_t> held;       // model: slots handed out, oldest first
  std::vector<uint32_t> pending;   // handed out and not yet completed by the "device"
  std::vector<uint8_t> completed(depth, 0);
  uint32_t tail = 0, next = 0;
  for (int step = 0; step < 60; ++step) {
    const uint32_t what = rnd() % 3;
    if (what == 0) {
      const uint32_t n = 1 + rnd() % depth;
      uint32_t first = 99;
      const int rc = tutti_get_iocb(&s, n, &first);
      if (n > depth - held.size()) {
        CHECK(rc == TUTTI_EAGAIN);
      } else {
        CHECK(rc == TUTTI_OK && first == next);
        for (uint32_t k = 0; k < n; ++k) {
          held.push_back((next + k) % depth);
          pending.push_back((next + k) % depth);
        }
        next = (next + n) % depth;
      }
    } else if (what == 1 && !pending.empty()) {
      // the device completes some pending IOCBs, in any order
      const uint32_t n = 1 + rnd() % pending.size();
      for (uint32_t k = 0; k < n; ++k) {
        const uint32_t at = rnd() % pending.size();
        const uint32_t idx = pending[at];
        pending.erase(pending.begin() + at);
        cq[16 + tail % depth] = idx;
        ++tail;
        completed[idx] = 1;
      }
      cq[0] = tail;
    } else {
      uint32_t fresh = 99;
      CHECK(tutti_reap_cqe(&s, cq.data(), nullptr, &fresh) == TUTTI_OK);
      while (!held.empty() && completed[held.front()]) {
        completed[held.front()] = 0;
        held.pop_front();
      }
    }
    CHECK(tutti_sq_free_count(&s) >= depth - held.size());  // the library reaps only when asked to
  }
  CHECK(tutti_reap_cqe(&s, cq.data(), nullptr, nullptr) == TUTTI_OK);
  while (!held.empty() && completed[held.front()]) {
    completed[held.front()] = 0;
    held.pop_front();
  }
  CHECK(tutti_sq_free_count(&s) == depth - held.size());
  for (uint32_t slot = 0; slot < depth; ++slot) {
    const int r = tutti_iocb_completed(&s, slot);
    CHECK(r == 0 || r == 1);
  }
  CHECK(tutti_iocb_completed(&s, depth) == TUTTI_EINVAL);
  CHECK(tutti_wait_cqe_host(&s, cq.data(), nullptr, rnd() % depth, 3) >= 0);
  // a queue that names a slot beyond the ring changes nothing
  if (!held.empty() && pending.size() == held.size()) {
    cq[16 + tail % depth] = depth + rnd() % 3;
    cq[0] = tail + 1;
    const uint32_t before = tutti_sq_free_count(&s);
    CHECK(tutti_reap_cqe(&s, cq.data(), nullptr, nullptr) == TUTTI_EINVAL);
    CHECK(tutti_sq_free_count(&s) == before);
  }
  return 0;
}

static int slack_round() {
  const uint32_t n = rnd() % 12;
  std::vector<tutti_io_profile> rows(n);
  for (auto &r : rows) {
    r.cu_budget = rnd() % 5 * 8;
    r.n_iocbs = 1 + rnd() % 4;
    r.read_us = static_cast<float>(rnd() % 400) - 20.f;
    r.write_us = static_cast<float>(rnd() % 400) - 20.f;
  }
  const uint32_t op = (rnd() & 1) ? TUTTI_OP_READ : TUTTI_OP_WRITE;
  const double slack = rnd() % 500;
  uint32_t out = 77;
  CHECK(tutti_iocbs_for_slack(n ? rows.data() : nullptr, n, rnd() % 5 * 8, op, slack, &out) == TUTTI_OK);
  CHECK(out <= 4);
  uint32_t budget = 77;
  const int rc = tutti_budget_for_slack(n ? rows.data() : nullptr, n, 1 + rnd() % 4, op, slack, 64, &budget);
  CHECK(rc == TUTTI_OK || rc == TUTTI_EAGAIN);
  CHECK(rc == TUTTI_OK ? (budget >= 8 && budget <= 64) : budget == 0);
  return 0;
}

static int pairs_round() {
  const uint32_t n = rnd() % 24;
  std::vector<int32_t> cls(n);
  for (auto &c : cls) c = static_cast<int32_t>(rnd() % (TUTTI_PLACE_MAX_REGIONS + 1)) - 1;
  const uint32_t want = rnd() % 14;
  std::vector<uint32_t> pairs(2 * want);
  uint32_t mixed = 99;
  const uint32_t strict = rnd() & 1;
  const int rc = tutti_place_pairs(n ? cls.data() : nullptr, n, want, strict, want ? pairs.data() : nullptr, &mixed);
  CHECK(rc == TUTTI_OK || rc == TUTTI_EAGAIN || rc == TUTTI_ERANGE);
  CHECK(mixed <= want);
  const uint32_t valid = rc == TUTTI_OK ? want : mixed;
  std::vector<int> used(n, 0);
  for (uint32_t k = 0; k < 2 * valid; ++k) {
    CHECK(pairs[k] < n);
    CHECK(used[pairs[k]]++ == 0);
  }
  for (uint32_t p = 0; p < mixed; ++p)
    CHECK(cls[pairs[2 * p]] >= 0 && cls[pairs[2 * p + 1]] >= 0 && cls[pairs[2 * p]] != cls[pairs[2 * p + 1]]);
  if (rc == TUTTI_EAGAIN) CHECK(strict && mixed < want);
  if (n) {
    cls[rnd() % n] = static_cast<int32_t>(TUTTI_PLACE_MAX_REGIONS);  // a class beyond the limit is refused
    CHECK(tutti_place_pairs(cls.data(), n, want, strict, want ? pairs.data() : nullptr, nullptr) == TUTTI_EINVAL);
  }
  return 0;
}

int main(int argc, char **argv) {
  const int rounds = argc > 1 ? std::atoi(argv[1]) : 200;
  for (int r = 0; r < rounds; ++r) {
    if (ring_round() || slack_round() || pairs_round()) {
      std::printf("failed in round %d\n", r);
      return 1;
    }
  }
  std::printf("ok %d\n", rounds);
  return 0;
}
