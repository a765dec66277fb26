// Host-only part of libtutti: the application's side of the rings (get_iocb, reaping the completion queue),
// the slack-table lookups and the pairing of classified planes.  No HIP call in this file: everything here is
// O(1) or O(rows) bookkeeping on host memory the caller owns, so it runs without a GPU.
#include <stddef.h>
#include <stdint.h>

#include "tutti.h"

namespace {

// Is `slot` one of the IOCBs the application currently holds, i.e. inside the ring segment of `held` slots that
// ends just before `head`?
bool is_held(const tutti_sq_state *s, uint32_t slot) {
  const uint32_t tail = (s->head + s->depth - s->held % s->depth) % s->depth;
  const uint32_t dist = (slot + s->depth - tail) % s->depth;
  return s->held == s->depth ? true : dist < s->held;
}

bool state_ok(const tutti_sq_state *s) {
  return s && s->done && s->depth > 0 && s->head < s->depth && s->held <= s->depth;
}

}  // namespace

extern "C" {

int tutti_sq_state_init(tutti_sq_state *s, uint32_t depth, uint8_t *flags) {
  if (!s || !flags || depth == 0) return TUTTI_EINVAL;
  s->depth = depth;
  s->head = 0;
  s->held = 0;
  s->cq_seen = 0;
  s->done = flags;
  for (uint32_t i = 0; i < depth; ++i) flags[i] = 0;
  return TUTTI_OK;
}

int tutti_get_iocb(tutti_sq_state *s, uint32_t n, uint32_t *first_slot) {
  if (!state_ok(s) || !first_slot || n == 0 || n > s->depth) return TUTTI_EINVAL;
  if (n > s->depth - s->held) return TUTTI_EAGAIN;
  *first_slot = s->head;
  s->head = (s->head + n) % s->depth;
  s->held += n;
  return TUTTI_OK;
}

uint32_t tutti_sq_free_count(const tutti_sq_state *s) { return state_ok(s) ? s->depth - s->held : 0u; }

int tutti_reap_cqe(tutti_sq_state *s, const void *cq_host, tutti_iocb *sq_host, uint32_t *n_new) {
  if (!state_ok(s) || !cq_host) return TUTTI_EINVAL;
  const tutti_cq_hdr *cq = static_cast<const tutti_cq_hdr *>(cq_host);
  const uint32_t *entry = reinterpret_cast<const uint32_t *>(cq + 1);
  // whoever sees the tail also sees the entries before it: the completion kernel releases it at system scope
  const uint32_t tail = __atomic_load_n(&cq->tail, __ATOMIC_ACQUIRE);
  const uint32_t fresh = tail - s->cq_seen;  // completions are counted modulo 2^32 on both sides
  if (n_new) *n_new = 0;
  if (fresh > s->held) return TUTTI_EINVAL;  // more completions than IOCBs handed out: not this ring's queue
  // check everything first, so that a queue that is not this ring's leaves the state as it was
  for (uint32_t i = 0; i < fresh; ++i) {
    const uint32_t idx = __atomic_load_n(&entry[(s->cq_seen + i) % s->depth], __ATOMIC_RELAXED);
    if (idx >= s->depth || !is_held(s, idx) || s->done[idx]) return TUTTI_EINVAL;
    for (uint32_t k = 0; k < i; ++k)
      if (entry[(s->cq_seen + k) % s->depth] == idx) return TUTTI_EINVAL;  // the same IOCB twice in one batch
  }
  for (uint32_t i = 0; i < fresh; ++i) {
    const uint32_t idx = entry[(s->cq_seen + i) % s->depth];
    s->done[idx] = 1;
    if (sq_host) __atomic_store_n(&sq_host[idx].hdr.state, TUTTI_IOCB_FREE, __ATOMIC_RELEASE);
  }
  s->cq_seen = tail;
  // give the slots back in ring order: an IOCB that completed before an older one waits for it
  uint32_t oldest = (s->head + s->depth - s->held % s->depth) % s->depth;
  while (s->held > 0 && s->done[oldest]) {
    s->done[oldest] = 0;
    oldest = (oldest + 1) % s->depth;
    s->held -= 1;
  }
  if (n_new) *n_new = fresh;
  return TUTTI_OK;
}

int tutti_iocb_completed(const tutti_sq_state *s, uint32_t slot) {
  if (!state_ok(s) || slot >= s->depth) return TUTTI_EINVAL;
  return (!is_held(s, slot) || s->done[slot]) ? 1 : 0;
}

int tutti_wait_cqe_host(tutti_sq_state *s, const void *cq_host, tutti_iocb *sq_host, uint32_t slot,
                        uint32_t max_polls) {
  if (!state_ok(s) || slot >= s->depth) return TUTTI_EINVAL;
  for (uint32_t i = 0;; ++i) {
    const int rc = tutti_reap_cqe(s, cq_host, sq_host, nullptr);
    if (rc != TUTTI_OK) return rc;
    if (tutti_iocb_completed(s, slot) == 1) return 1;
    if (i >= max_polls) return 0;
  }
}

// ---- slack table

int tutti_iocbs_for_slack(const tutti_io_profile *rows, uint32_t n_rows, uint32_t cu_budget, uint32_t opcode,
                          double slack_us, uint32_t *n_iocbs) {
  if ((n_rows > 0 && !rows) || !n_iocbs || (opcode != TUTTI_OP_READ && opcode != TUTTI_OP_WRITE)) return TUTTI_EINVAL;
  uint32_t best = 0;
  for (uint32_t i = 0; i < n_rows; ++i) {
    if (rows[i].cu_budget != cu_budget) continue;
    const double us = opcode == TUTTI_OP_READ ? rows[i].read_us : rows[i].write_us;
    if (us > 0.0 && us <= slack_us && rows[i].n_iocbs > best) best = rows[i].n_iocbs;
  }
  *n_iocbs = best;
  return TUTTI_OK;
}

int tutti_budget_for_slack(const tutti_io_profile *rows, uint32_t n_rows, uint32_t n_iocbs, uint32_t opcode,
                           double slack_us, uint32_t max_budget, uint32_t *cu_budget) {
  if ((n_rows > 0 && !rows) || !cu_budget || n_iocbs == 0 || (opcode != TUTTI_OP_READ && opcode != TUTTI_OP_WRITE))
    return TUTTI_EINVAL;
  // for every budget, the profiled row with the fewest IOCBs that still covers n_iocbs stands for the launch
  // (a launch is never faster than a smaller one at the same budget); the smallest budget that fits wins
  bool found = false;
  uint32_t best_budget = 0;
  for (uint32_t i = 0; i < n_rows; ++i) {
    const uint32_t b = rows[i].cu_budget;
    if (b == 0 || b > max_budget || rows[i].n_iocbs < n_iocbs) continue;
    bool tighter = false;  // another row of the same budget covers n_iocbs with fewer IOCBs
    for (uint32_t k = 0; k < n_rows; ++k)
      if (k != i && rows[k].cu_budget == b && rows[k].n_iocbs >= n_iocbs &&
          (rows[k].n_iocbs < rows[i].n_iocbs || (rows[k].n_iocbs == rows[i].n_iocbs && k < i)))
        tighter = true;
    if (tighter) continue;
    const double us = opcode == TUTTI_OP_READ ? rows[i].read_us : rows[i].write_us;
    if (us > 0.0 && us <= slack_us && (!found || b < best_budget)) {
      found = true;
      best_budget = b;
    }
  }
  *cu_budget = found ? best_budget : 0u;
  return found ? TUTTI_OK : TUTTI_EAGAIN;
}

// ---- pool placement: pairing the classified planes

int tutti_place_pairs(const int32_t *classes, uint32_t n, uint32_t n_pairs, uint32_t strict, uint32_t *pairs,
                      uint32_t *n_mixed) {
  if (n_mixed) *n_mixed = 0;
  if ((n > 0 && !classes) || (n_pairs > 0 && !pairs)) return TUTTI_EINVAL;
  uint32_t left[TUTTI_PLACE_MAX_REGIONS] = {};  // planes of the class not yet used
  uint32_t next[TUTTI_PLACE_MAX_REGIONS] = {};  // every plane of the class below this index is used
  for (uint32_t i = 0; i < n; ++i) {
    if (classes[i] < -1 || classes[i] >= static_cast<int32_t>(TUTTI_PLACE_MAX_REGIONS)) return TUTTI_EINVAL;
    if (classes[i] >= 0) ++left[classes[i]];
  }
  auto take = [&](uint32_t c) {
    uint32_t i = next[c];
    while (classes[i] != static_cast<int32_t>(c)) ++i;  // left[c] > 0: there is one
    next[c] = i + 1;
    --left[c];
    return i;
  };
  uint32_t made = 0;
  while (made < n_pairs) {
    // the two classes with the most planes left (ties: the lower class first)
    int a = -1, b = -1;
    for (uint32_t c = 0; c < TUTTI_PLACE_MAX_REGIONS; ++c) {
      if (left[c] == 0) continue;
      if (a < 0 || left[c] > left[a]) {
        b = a;
        a = static_cast<int>(c);
      } else if (b < 0 || left[c] > left[b]) {
        b = static_cast<int>(c);
      }
    }
    if (b < 0) break;
    pairs[2 * made] = take(static_cast<uint32_t>(a));
    pairs[2 * made + 1] = take(static_cast<uint32_t>(b));
    ++made;
  }
  if (n_mixed) *n_mixed = made;
  if (made == n_pairs) return TUTTI_OK;
  if (strict) return TUTTI_EAGAIN;
  // what is left over, lowest indices first: planes of one class, and those no round reached
  uint32_t spare = 0;
  for (uint32_t i = 0; i < n; ++i)
    if (classes[i] < 0 || i >= next[classes[i]]) ++spare;
  if (spare / 2 < n_pairs - made) return TUTTI_ERANGE;
  uint32_t slot = 2 * made;
  for (uint32_t i = 0; i < n && slot < 2 * n_pairs; ++i)
    if (classes[i] < 0 || i >= next[classes[i]]) pairs[slot++] = i;
  return TUTTI_OK;
}

}  // extern "C"
