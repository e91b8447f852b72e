// Host-side bookkeeping of the instant request pool (paper Sec. 2.2.2): which
// slot holds which request, who is advanced by the next step, how many frames
// each request has produced and how many have been handed out.  No device
// code and no HIP calls in here.
#pragma once
#include <cstdint>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

namespace tts {

enum class SlotState : int { Free = 0, Active = 1, Finished = 2 };

struct SlotInfo {
    int64_t id = -1;
    int L = 0;
    int n_steps = 0;
    int t = 0;        // frames produced (host mirror; an upper bound while a stop threshold may fire)
    int drained = 0;  // frames already handed out
    int parity = 0;   // which half of the double-buffered activations holds this request's newest state
    bool lost = false; // ended by the device before its time: a step could not be completed for it
    SlotState state = SlotState::Free;
};

class PoolBook {
public:
    PoolBook(int max_pool, int max_enc_len, int max_steps, int chunk_frames)
        : max_pool_(max_pool), max_enc_len_(max_enc_len), max_steps_(max_steps),
          chunk_(chunk_frames), slots_(max_pool) {
        for (int s = 0; s < max_pool; ++s) free_.insert(s);
        active_.reserve(max_pool);
    }

    // 0 ok, -1 invalid argument, -2 full
    int add(int L, int n_steps, int64_t* out_id, int* out_slot) {
        if (L < 1 || L > max_enc_len_ || n_steps < 1 || n_steps > max_steps_) return -1;
        if (free_.empty()) return -2;
        // lowest free slot first: keeps the occupied slots packed into few 16-slot tiles
        int s = *free_.begin();
        free_.erase(free_.begin());
        SlotInfo& si = slots_[s];
        si = SlotInfo();
        si.id = next_id_++;
        si.L = L;
        si.n_steps = n_steps;
        si.state = SlotState::Active;
        by_id_[si.id] = s;
        active_.push_back(s);
        dirty_ = true;
        if (out_id) *out_id = si.id;
        if (out_slot) *out_slot = s;
        return 0;
    }

    int find(int64_t id) const {
        auto it = by_id_.find(id);
        return it == by_id_.end() ? -1 : it->second;
    }

    // Advance every active request by one frame.  Requests that reach their cap
    // leave the active list (they keep their slot until retired).  Returns the
    // number of requests advanced.  `new_parity` is the activation buffer half
    // their newest state now lives in.
    int step(int new_parity, std::vector<int>* advanced = nullptr) {
        int n = (int)active_.size();
        if (advanced) advanced->assign(active_.begin(), active_.end());
        size_t keep = 0;
        for (size_t i = 0; i < active_.size(); ++i) {
            SlotInfo& si = slots_[active_[i]];
            si.t += 1;
            si.parity = new_parity;
            if (si.t >= si.n_steps) {
                si.state = SlotState::Finished;
                dirty_ = true;
            } else {
                active_[keep++] = active_[i];
            }
        }
        active_.resize(keep);
        return n;
    }

    // A request found finished early by the device (stop threshold) after `t` frames.
    void finish_early(int slot, int t) {
        SlotInfo& si = slots_[slot];
        if (si.state == SlotState::Free) return;
        si.t = t;
        if (si.state == SlotState::Active) {
            si.state = SlotState::Finished;
            remove_active(slot);
        }
    }

    // A request the device froze after `t` frames (a step's kernels could not complete it): it ends there.
    void lose(int slot, int t) {
        SlotInfo& si = slots_[slot];
        if (si.state == SlotState::Free) return;
        if (t < si.t) si.t = t;
        if (si.drained > si.t) si.drained = si.t;
        si.lost = true;
        if (si.state == SlotState::Active) remove_active(slot);
        si.state = SlotState::Finished;
    }

    // What the next drain hands out: frames [first, first+count).  count = 0 if
    // the chunk is not full yet and the request is still running.
    void drain_plan(int slot, int* first, int* count, int* finished_after) const {
        const SlotInfo& si = slots_[slot];
        int avail = si.t - si.drained;
        bool fin = si.state == SlotState::Finished;
        int n = 0;
        if (avail >= chunk_) n = chunk_;
        else if (fin) n = avail;
        *first = si.drained;
        *count = n;
        *finished_after = (fin && si.drained + n == si.t) ? 1 : 0;
    }
    void drain_commit(int slot, int count) { slots_[slot].drained += count; }

    int retire(int64_t id) {
        int s = find(id);
        if (s < 0) return -3;
        if (slots_[s].state == SlotState::Active) remove_active(s);
        slots_[s].state = SlotState::Free;
        by_id_.erase(id);
        free_.insert(s);
        return 0;
    }

    // Slots the step kernels must cover: one past the highest running request's.
    int span() const {
        int sp = 0;
        for (int sl : active_) sp = sl + 1 > sp ? sl + 1 : sp;
        return sp;
    }

    // Span classes (what launch shapes are keyed by): whole tiles of 16 slots, powers of two within the first.
    static int span_class(int n) {
        if (n > 16) return (n + 15) / 16 * 16;
        int b = 1;
        while (b < n) b <<= 1;
        return b;
    }

    // When requests have left, the running ones may sit far apart.  If they would fit a smaller span class (but not
    // below `min_span`, under which a smaller launch saves nothing) and enough slots under it are free, the running
    // requests above move into those free slots, lowest first: (from, to) pairs, in the order to carry them out.
    // Finished requests that have not been retired keep their slots and may make this impossible: then no moves.
    std::vector<std::pair<int, int>> plan_moves(int min_span) const {
        std::vector<std::pair<int, int>> moves;
        if (active_.empty()) return moves;
        int target = span_class((int)active_.size());
        if (target < min_span) target = min_span;
        if (span_class(span()) <= target) return moves;
        std::vector<int> high;
        for (int sl : active_)
            if (sl >= target) high.push_back(sl);
        auto hole = free_.begin();
        for (int from : high) {
            if (hole == free_.end() || *hole >= target) return {};
            moves.emplace_back(from, *hole++);
        }
        return moves;
    }

    // A running request changes slots (`to` must be free); its id, counters and place in the order of the running
    // requests go along.
    void move(int from, int to) {
        SlotInfo& a = slots_[from];
        slots_[to] = a;
        by_id_[a.id] = to;
        a = SlotInfo();
        for (size_t i = 0; i < active_.size(); ++i)
            if (active_[i] == from) active_[i] = to;
        free_.erase(to);
        free_.insert(from);
        dirty_ = true;
    }

    const std::vector<int>& active() const { return active_; }
    const SlotInfo& slot(int s) const { return slots_[s]; }
    SlotInfo& slot(int s) { return slots_[s]; }
    int size() const { return max_pool_ - (int)free_.size(); }
    bool dirty() const { return dirty_; }
    void clear_dirty() { dirty_ = false; }
    int max_pool() const { return max_pool_; }
    int chunk() const { return chunk_; }

private:
    void remove_active(int slot) {
        for (size_t i = 0; i < active_.size(); ++i)
            if (active_[i] == slot) {
                active_.erase(active_.begin() + i);
                break;
            }
        dirty_ = true;
    }

    int max_pool_, max_enc_len_, max_steps_, chunk_;
    std::vector<SlotInfo> slots_;
    std::set<int> free_;
    std::vector<int> active_;
    std::unordered_map<int64_t, int> by_id_;
    int64_t next_id_ = 1;
    bool dirty_ = true;
};

}  // namespace tts
