// Host-side planning and validation for the resume prefill (integer work only).
#pragma once
#include <cstdint>
#include <vector>

#include "gdn_resume.h"

namespace gdn {

struct ChunkPlan {
    std::vector<int32_t> chunk_tok0;    // first packed token of the chunk
    std::vector<int32_t> chunk_len;     // 1..GDN_CHUNK valid tokens
    std::vector<int32_t> chunk_emit;    // flat emission index stored after the chunk, or -1
    std::vector<int32_t> req_chunk_cu;  // n_req + 1
    int32_t max_chunks_per_req = 0;
};

// Validates cu_seqlens / start_pos / emit lists (Sec. 3: positions are 1-based, a state at
// position c is the state after token c) and cuts every request at its emit positions and
// then into chunks.  Returns GDN_OK or the error code.
int32_t plan_chunks(int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos,
                    const int32_t* emit_cu, const int32_t* emit_pos, ChunkPlan* out);

// Slot checks of one prefill call: ranges and distinct destinations (overlaps between source and
// destination slots are checked by address where the pools are known).
int32_t check_slots(int32_t n_req, const int32_t* src_slot, int32_t src_n_slots,
                    const int32_t* emit_cu, const int32_t* emit_slot, int32_t dst_n_slots);

// Requests ordered by decreasing chunk count (longest chains are launched first).
std::vector<int32_t> longest_first(const ChunkPlan& plan, int32_t n_req);

int32_t check_shape(const gdn_shape* s);

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

}  // namespace gdn
