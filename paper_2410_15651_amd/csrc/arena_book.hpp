// Host-side integer bookkeeping of the KV arena: free list, page table,
// sequence lengths and the allocator counters the paper defines (Section 2.2:
// reserved vs allocated memory).  No device code and no HIP calls in here, so
// the same object serves arenas with and without a GPU behind them.
#pragma once

#include <algorithm>
#include <cstdint>
#include <deque>
#include <vector>

namespace rlhf {

struct NewPage {
    int32_t table_index;  // seq * max_pages_per_seq + logical page
    int32_t page;
};

struct AppendPlan {
    // one entry per appended sequence, in call order
    struct Seq {
        int32_t token_offset;  // first row of this sequence in the packed k_new / v_new
        int32_t seq;
        int32_t start_len;
        int32_t n_new;
    };
    std::vector<Seq> seqs;
    std::vector<NewPage> new_pages;
    int64_t total_tokens = 0;
    int32_t peak_before = 0;  // peak_pages_in_use before the call, for undo_append
};

// What free_seq took away, for undo_free_seq.
struct FreePlan {
    int32_t seq = -1;
    int32_t len = 0;
    std::vector<int32_t> pages;  // in logical order
};

class ArenaBook {
public:
    enum Result { kOk = 0, kInvalid = -1, kOom = -2 };

    ArenaBook(int32_t max_seqs, int32_t n_pages, int32_t max_pages_per_seq, int32_t page_tokens,
              uint64_t page_bytes_kv, uint64_t token_bytes_kv, const int32_t *initial_free_order)
        : max_seqs_(max_seqs), n_pages_(n_pages), mpps_(max_pages_per_seq), page_tokens_(page_tokens),
          page_bytes_kv_(page_bytes_kv), token_bytes_kv_(token_bytes_kv), initial_(n_pages),
          table_((size_t)max_seqs * max_pages_per_seq), lens_(max_seqs)
    {
        for (int32_t i = 0; i < n_pages; ++i)
            initial_[i] = initial_free_order ? initial_free_order[i] : i;
        reset();
    }

    // True when `order` is a permutation of 0 .. n-1.
    static bool is_permutation(const int32_t *order, int32_t n)
    {
        std::vector<char> seen(n, 0);
        for (int32_t i = 0; i < n; ++i) {
            if (order[i] < 0 || order[i] >= n || seen[order[i]])
                return false;
            seen[order[i]] = 1;
        }
        return true;
    }

    void reset()
    {
        free_.assign(initial_.begin(), initial_.end());
        std::fill(table_.begin(), table_.end(), -1);
        std::fill(lens_.begin(), lens_.end(), 0);
        live_tokens_ = 0;
        live_seqs_ = 0;
        peak_in_use_ = 0;
    }

    // Validates the whole call first; on failure nothing has changed.
    Result append(const int32_t *seq_ids, const int32_t *n_new, int32_t n_seqs, AppendPlan *plan)
    {
        if (n_seqs < 0 || (n_seqs > 0 && (!seq_ids || !n_new)))
            return kInvalid;
        std::vector<char> seen(max_seqs_, 0);
        int64_t need = 0;
        for (int32_t i = 0; i < n_seqs; ++i) {
            const int32_t s = seq_ids[i], n = n_new[i];
            if (s < 0 || s >= max_seqs_ || n < 0 || seen[s])
                return kInvalid;
            seen[s] = 1;
            const int64_t after = pages_for((int64_t)lens_[s] + n);
            if (after > mpps_)
                return kInvalid;
            need += after - pages_for(lens_[s]);
        }
        if (need > (int64_t)free_.size())
            return kOom;

        plan->seqs.clear();
        plan->new_pages.clear();
        plan->total_tokens = 0;
        plan->peak_before = peak_in_use_;
        for (int32_t i = 0; i < n_seqs; ++i) {
            const int32_t s = seq_ids[i], n = n_new[i];
            const int32_t start = lens_[s];
            const int32_t have = (int32_t)pages_for(start);
            const int32_t want = (int32_t)pages_for((int64_t)start + n);
            for (int32_t lp = have; lp < want; ++lp) {
                const int32_t page = free_.front();
                free_.pop_front();
                table_[(size_t)s * mpps_ + lp] = page;
                plan->new_pages.push_back({s * mpps_ + lp, page});
            }
            plan->seqs.push_back({(int32_t)plan->total_tokens, s, start, n});
            plan->total_tokens += n;
            if (start == 0 && n > 0)
                ++live_seqs_;
            lens_[s] = start + n;
            live_tokens_ += n;
        }
        peak_in_use_ = std::max(peak_in_use_, pages_in_use());
        return kOk;
    }

    // Takes back an append that has just succeeded (nothing else happened in
    // between): every list and counter is as it was before the call.
    void undo_append(const AppendPlan &plan)
    {
        for (auto it = plan.seqs.rbegin(); it != plan.seqs.rend(); ++it) {
            lens_[it->seq] = it->start_len;
            live_tokens_ -= it->n_new;
            if (it->start_len == 0 && it->n_new > 0)
                --live_seqs_;
        }
        for (auto it = plan.new_pages.rbegin(); it != plan.new_pages.rend(); ++it) {
            table_[it->table_index] = -1;
            free_.push_front(it->page);
        }
        peak_in_use_ = plan.peak_before;
    }

    Result free_seq(int32_t s, FreePlan *plan = nullptr)
    {
        if (s < 0 || s >= max_seqs_)
            return kInvalid;
        const int32_t have = (int32_t)pages_for(lens_[s]);
        if (plan) {
            plan->seq = s;
            plan->len = lens_[s];
            plan->pages.assign(table_.begin() + (size_t)s * mpps_, table_.begin() + (size_t)s * mpps_ + have);
        }
        for (int32_t lp = 0; lp < have; ++lp) {
            free_.push_back(table_[(size_t)s * mpps_ + lp]);
            table_[(size_t)s * mpps_ + lp] = -1;
        }
        if (lens_[s] > 0)
            --live_seqs_;
        live_tokens_ -= lens_[s];
        lens_[s] = 0;
        return kOk;
    }

    // Takes back a free_seq that has just succeeded.
    void undo_free_seq(const FreePlan &plan)
    {
        for (size_t lp = 0; lp < plan.pages.size(); ++lp) {
            free_.pop_back();
            table_[(size_t)plan.seq * mpps_ + lp] = plan.pages[lp];
        }
        lens_[plan.seq] = plan.len;
        live_tokens_ += plan.len;
        if (plan.len > 0)
            ++live_seqs_;
    }

    int32_t max_seqs() const { return max_seqs_; }
    int32_t max_pages_per_seq() const { return mpps_; }
    int32_t n_pages() const { return n_pages_; }
    int32_t pages_free() const { return (int32_t)free_.size(); }
    int32_t pages_in_use() const { return n_pages_ - (int32_t)free_.size(); }
    int32_t peak_pages_in_use() const { return peak_in_use_; }
    int32_t live_seqs() const { return live_seqs_; }
    uint64_t reserved_bytes() const { return (uint64_t)n_pages_ * page_bytes_kv_; }
    uint64_t allocated_bytes() const { return (uint64_t)pages_in_use() * page_bytes_kv_; }
    uint64_t live_token_bytes() const { return (uint64_t)live_tokens_ * token_bytes_kv_; }
    const int32_t *table() const { return table_.data(); }
    const int32_t *lens() const { return lens_.data(); }
    int32_t len(int32_t s) const { return lens_[s]; }

    // Contiguous copy of the free list, head first (rebuilt on request).
    const int32_t *free_list_snapshot()
    {
        snapshot_.assign(free_.begin(), free_.end());
        return snapshot_.data();
    }

private:
    int64_t pages_for(int64_t tokens) const { return (tokens + page_tokens_ - 1) / page_tokens_; }

    int32_t max_seqs_, n_pages_, mpps_, page_tokens_;
    uint64_t page_bytes_kv_;   // bytes of one page, K and V parts together
    uint64_t token_bytes_kv_;  // bytes of one token, K and V rows together
    std::vector<int32_t> initial_;
    std::deque<int32_t> free_;
    std::vector<int32_t> table_;
    std::vector<int32_t> lens_;
    std::vector<int32_t> snapshot_;
    int64_t live_tokens_ = 0;
    int32_t live_seqs_ = 0;
    int32_t peak_in_use_ = 0;
};

}  // namespace rlhf
