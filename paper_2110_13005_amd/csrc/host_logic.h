// Host-side decisions of the stage runtime, free of any HIP call: which posted message Alg. 2's receive loop
// takes next, the bookkeeping of the activation stash slots (Sec. 3.3: at most pipeline_limit microbatches in
// flight), when the deferred weight gradients of a group of microbatches are formed, how long the loop waits
// for a message, and the bucket plan of the offloaded optimizer (Sec. 5.2) with the chunks of the step that
// overlaps the backward tail (Sec. 5.3).  stage.cpp calls these with its HIP streams and events around them; the
// CPU tests compile this header alone (with the address, undefined-behaviour and thread sanitizers) and drive it
// with simulated events.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <cstddef>

namespace axonn {
namespace host {

// ------------------------------------------------------------------------------ stash slots
// A slot is FREE, LIVE (forward issued, backward not yet: it counts as in flight) or AWAIT_WGRAD (backward chain
// issued, the slot's tensors are still operands of a weight-gradient contraction that has not been issued).
// `Slots` is any container of records with the members `state` and `mb_id`.
enum SlotState { SLOT_FREE = 0, SLOT_LIVE = 1, SLOT_AWAIT_WGRAD = 2 };

template <class Slots>
int find_live(const Slots& slots, int mb_id) {
  int i = 0;
  for (const auto& s : slots) {
    if (s.state == SLOT_LIVE && s.mb_id == mb_id) return i;
    ++i;
  }
  return -1;
}
template <class Slots>
int find_free(const Slots& slots) {
  int i = 0;
  for (const auto& s : slots) {
    if (s.state == SLOT_FREE) return i;
    ++i;
  }
  return -1;
}
template <class Slots>
int count_state(const Slots& slots, int state) {
  int n = 0;
  for (const auto& s : slots) n += (s.state == state);
  return n;
}

// Forward(msg) for microbatch mb_id: may it start, and where?
enum ForwardAdmission {
  FWD_OK = 0,            // *slot is free
  FWD_NEEDS_FLUSH = 1,   // admissible, but every slot not in flight awaits its weight gradients: form them first
  FWD_NEGATIVE_ID = -1, FWD_ALREADY_LIVE = -2, FWD_PIPELINE_FULL = -3, FWD_NO_SLOT = -4
};
template <class Slots>
int admit_forward(const Slots& slots, int mb_id, int in_flight, int pipeline_limit, int* slot) {
  *slot = -1;
  if (mb_id < 0) return FWD_NEGATIVE_ID;
  if (find_live(slots, mb_id) >= 0) return FWD_ALREADY_LIVE;
  if (in_flight >= pipeline_limit) return FWD_PIPELINE_FULL;
  *slot = find_free(slots);
  if (*slot >= 0) return FWD_OK;
  return count_state(slots, SLOT_AWAIT_WGRAD) > 0 ? FWD_NEEDS_FLUSH : FWD_NO_SLOT;
}
template <class Slots>
void commit_forward(Slots& slots, int slot, int mb_id, int* in_flight) {
  slots[slot].state = SLOT_LIVE;
  slots[slot].mb_id = mb_id;
  ++*in_flight;
}
// Backward(msg): the slot of the microbatch's forward, or -1 if none is in flight.
template <class Slots>
int admit_backward(const Slots& slots, int mb_id) { return mb_id >= 0 ? find_live(slots, mb_id) : -1; }
// The backward chain of `slot` is issued: the microbatch leaves the pipeline; the slot waits for its weight
// gradients unless they were issued with the chain (activation checkpointing).
template <class Slots>
void commit_backward(Slots& slots, int slot, bool wgrad_issued_with_chain, int* in_flight) {
  slots[slot].mb_id = -1;
  slots[slot].state = wgrad_issued_with_chain ? SLOT_FREE : SLOT_AWAIT_WGRAD;
  --*in_flight;
}
// A weight-gradient pass over all waiting slots is issued (or a new batch drops them).
template <class Slots>
int release_awaiting(Slots& slots) {
  int n = 0;
  for (auto& s : slots)
    if (s.state == SLOT_AWAIT_WGRAD) { s.state = SLOT_FREE; ++n; }
  return n;
}

// What follows the backward chain of a microbatch with stored activations: the batch's last microbatch closes
// every open group (and that pass finishes the gradients layer by layer); otherwise a group closes once
// `group` microbatches wait (group == 0: only when a slot is needed or the batch ends).
enum WgradAction { WGRAD_NONE = 0, WGRAD_FLUSH = 1, WGRAD_FLUSH_FINAL = 2 };
inline int wgrad_action(bool last_of_batch, int group, int n_awaiting) {
  if (last_of_batch) return WGRAD_FLUSH_FINAL;
  return (group > 0 && n_awaiting >= group) ? WGRAD_FLUSH : WGRAD_NONE;
}

// ------------------------------------------------------------------------------ messages
// A message is admissible if its work may start now: a forward needs a pipeline place and must not be in
// flight already; a backward needs its forward.
template <class Slots>
bool admissible(int kind, int mb_id, const Slots& slots, int in_flight, int pipeline_limit) {
  return kind == 0 ? (in_flight < pipeline_limit && find_live(slots, mb_id) < 0) : (find_live(slots, mb_id) >= 0);
}

// The receive loop's choice: the first posted message (in posting order) that is admissible and has arrived.
// msg(i) -> (kind, mb_id) of posted message i; arrived(i) -> 1 arrived, 0 not yet, < 0 an error of the event
// layer (returned in *error, the choice is then -1).  *any_admissible tells a loop that found nothing whether
// waiting can help.
template <class Slots, class Msg, class Arrived>
int choose_message(size_t n_posted, Msg&& msg, Arrived&& arrived, const Slots& slots, int in_flight,
                   int pipeline_limit, bool* any_admissible, int* error) {
  *any_admissible = false;
  *error = 0;
  for (size_t i = 0; i < n_posted; ++i) {
    const auto km = msg(i);
    if (!admissible(km.first, km.second, slots, in_flight, pipeline_limit)) continue;
    *any_admissible = true;
    const int a = arrived(i);
    if (a < 0) { *error = a; return -1; }
    if (a == 0) continue;
    return (int)i;
  }
  return -1;
}

// post(): a message is refused if one of the same kind for the same microbatch is already posted, or if the
// batch has no room for another of its kind (issued + posted would exceed n_microbatches).
enum PostCheck { POST_OK = 0, POST_DUPLICATE = -1, POST_SURPLUS = -2 };
template <class Msg>
int check_post(int kind, int mb_id, size_t n_posted, Msg&& msg, int issued_of_kind, int n_microbatches) {
  int same = 0;
  for (size_t i = 0; i < n_posted; ++i) {
    const auto km = msg(i);
    if (km.first != kind) continue;
    ++same;
    if (km.second == mb_id) return POST_DUPLICATE;
  }
  return issued_of_kind + same >= n_microbatches ? POST_SURPLUS : POST_OK;
}

// Library stream of a message's work: backward chains keep to stream 0 (they share accumulators and the
// workspace), forwards go round robin over the others.
inline int stream_index(int kind, int n_streams, int* fwd_rr) {
  if (kind == 1 || n_streams == 1) return 0;
  return 1 + ((*fwd_rr)++ % (n_streams - 1));
}

// How long the blocking loop waits for the next message: the limit applies to each wait, from the moment the
// loop first found nothing to dispatch until a message is dispatched again.
struct WaitClock {
  double limit_s;
  double since = -1.0;          // < 0: not waiting
  explicit WaitClock(double limit) : limit_s(limit) {}
  void dispatched() { since = -1.0; }
  bool expired(double now) {    // call when nothing could be dispatched
    if (since < 0) since = now;
    return now - since > limit_s;
  }
};

// ------------------------------------------------------------------------------ optimizer buckets
inline uint64_t bucket_count(uint64_t n, uint64_t bucket) { return bucket ? (n + bucket - 1) / bucket : 0; }

// The i-th bucket a pass processes (ascending offsets, or descending for the pass that follows the backward
// tail from the last layer down): its index, element range and the device buffer set it uses.
struct BucketPlan { uint64_t index, offset, count; int set; };
inline BucketPlan bucket_plan(uint64_t n, uint64_t bucket, int n_sets, uint64_t i, bool descending) {
  const uint64_t nb = bucket_count(n, bucket);
  BucketPlan p;
  p.index = descending ? nb - 1 - i : i;
  p.offset = p.index * bucket;
  p.count = std::min<uint64_t>(bucket, n - p.offset);
  p.set = (int)(i % (uint64_t)n_sets);
  return p;
}
// Descending pass in chunks of k buckets: the element range [lo, hi) of the chunk that starts at processing
// index i (i a multiple of k).  The chunk's updates may start when every gradient in [lo, hi) is final.
inline void chunk_span(uint64_t n, uint64_t bucket, uint64_t k, uint64_t i, uint64_t* lo, uint64_t* hi) {
  const uint64_t nb = bucket_count(n, bucket);
  const BucketPlan first = bucket_plan(n, bucket, 1, i, true);
  const uint64_t n_in_chunk = std::min<uint64_t>(k, nb - i);
  *lo = (first.index + 1 - n_in_chunk) * bucket;
  *hi = first.offset + first.count;
}
// Gradients become final from the last layer down, so a range is final once the layer that holds its lowest
// element is: the largest l with layer_begin[l] <= lo (layer_begin ascending, layer_begin[0] == 0).
inline int lowest_layer(const uint64_t* layer_begin, int n_layers, uint64_t lo) {
  int l = 0;
  while (l + 1 < n_layers && layer_begin[l + 1] <= lo) ++l;
  return l;
}

}  // namespace host
}  // namespace axonn
