// Argument block of the token-routed kernels (dispatch, combine), shared by their translation units.
#pragma once
#include "msx_device.hpp"

namespace msx {

struct MoeArgs {
    const void* tokens[kMaxRanks];
    const int* topk[kMaxRanks];
    void* recv[kMaxRanks];
    int* recv_src[kMaxRanks];
    int* recv_counts;       // [n dst][n src]
    unsigned short* slots;  // plan scratch: [n src][T][8] slot of the token in destination d, 0xFFFF = not sent
    unsigned* base;         // plan scratch: [n src][8] first row of source s inside destination d
    int T, K, n, per_rank;  // per_rank = experts per rank
    int n_experts;
    unsigned per_rank_magic; // ceil(2^32 / per_rank) when n_experts < 65536 and per_rank > 1 (e / per_rank is then the
                             // high word of e * magic), else 0: divide
    unsigned row_vecs;      // 16-byte vectors per row
    unsigned cap;           // rows per destination buffer
    int chans;
    int has_src;
};

}  // namespace msx
