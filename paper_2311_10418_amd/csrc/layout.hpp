// Internal representation of a micro-batch layout (host side).
#pragma once
#include <cstdint>
#include <vector>
#include <atomic>

struct ds_layout {
    int32_t n_seq = 0, n_mb = 0;
    int32_t total_rows = 0, total_rows_tgt = 0;
    int64_t total_tokens = 0, total_tokens_tgt = 0;
    int64_t objective = 0, t_max = 0;
    bool has_tgt = false;
    uint64_t uid = 0;                       // distinguishes layouts for the stage's table cache
    std::vector<int32_t> perm, mb_start, mb_count, mb_lpad, mb_ltgt, mb_row, mb_nrows, mb_row_tgt, mb_nrows_tgt;
    std::vector<int32_t> seq_row, seq_len, seq_row_tgt, seq_len_tgt;
    std::vector<int64_t> mb_cost;           // t(M_m) under the cost model the layout was built with (may be empty)
};

uint64_t ds_next_layout_uid();
