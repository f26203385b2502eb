// Block manager of the paged KV pool: a stack of free block ids, a state byte and a holder count
// per block (the samples of one prompt name the prompt's blocks in their tables: a block goes
// back on the stack when its last holder frees it).
#include "heddle_internal.h"

namespace heddle {

BlockManager::BlockManager(int32_t n_blocks)
    : state_(static_cast<size_t>(n_blocks), kFree), holders_(static_cast<size_t>(n_blocks), 0) {
  stack_.reserve(static_cast<size_t>(n_blocks));
  // a fresh pool hands out 0, 1, 2, ...: block 0 must be on top
  for (int32_t id = n_blocks - 1; id >= 0; --id) stack_.push_back(id);
}

int BlockManager::alloc(int32_t n, int32_t* out) {
  if (n < 0 || (n > 0 && out == nullptr)) return HEDDLE_E_INVAL;
  if (static_cast<size_t>(n) > stack_.size()) return HEDDLE_E_NOMEM;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t id = stack_.back();
    stack_.pop_back();
    state_[static_cast<size_t>(id)] = kHeld;
    holders_[static_cast<size_t>(id)] = 1;
    out[i] = id;
  }
  return HEDDLE_OK;
}

bool BlockManager::valid_held_list(int32_t n, const int32_t* ids) {
  const int64_t cap = static_cast<int64_t>(state_.size());
  // mark as we go: a second sighting of an id finds it marked
  int32_t checked = 0;
  bool ok = true;
  for (; checked < n; ++checked) {
    const int64_t id = ids[checked];
    if (id < 0 || id >= cap || state_[static_cast<size_t>(id)] != kHeld) {
      ok = false;
      break;
    }
    state_[static_cast<size_t>(id)] = kMarked;
  }
  for (int32_t i = 0; i < checked; ++i) state_[static_cast<size_t>(ids[i])] = kHeld;
  return ok;
}

int BlockManager::retain(int32_t n, const int32_t* ids) {
  if (n < 0 || (n > 0 && ids == nullptr)) return HEDDLE_E_INVAL;
  if (!valid_held_list(n, ids)) return HEDDLE_E_INVAL;
  for (int32_t i = 0; i < n; ++i) ++holders_[static_cast<size_t>(ids[i])];
  return HEDDLE_OK;
}

int BlockManager::release(int32_t n, const int32_t* ids) {
  if (n < 0 || (n > 0 && ids == nullptr)) return HEDDLE_E_INVAL;
  if (!valid_held_list(n, ids)) return HEDDLE_E_INVAL;
  // commit, in the order given: a block whose last holder this was goes back on the stack
  for (int32_t i = 0; i < n; ++i) {
    const size_t id = static_cast<size_t>(ids[i]);
    if (--holders_[id] == 0) {
      state_[id] = kFree;
      stack_.push_back(ids[i]);
    }
  }
  return HEDDLE_OK;
}

}  // namespace heddle
