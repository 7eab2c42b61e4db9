// Builds the group / offset / tile tables from tensor sizes and a plan.  Pure host code.
//
// Grouping follows the communication handler of Algorithm 2: gradients arrive L-1, L-2, ..., 0 and
// a buffer is sent (closed) when the arriving layer is a normal layer.  The offsets follow
// Sec. 5.3: a group's buffer is exactly as long as the sum of its members, so members are laid
// end to end in arrival order.
#include <algorithm>
#include <cstdint>
#include <limits>

#include "mgwfbp.h"
#include "tables.h"

int mgwfbp_build_tables(const uint64_t* n_elems, int32_t L, const uint8_t* merged, HostTables& out) {
    if (L < 0) return MGWFBP_EINVAL;
    if (L > 0 && (n_elems == nullptr || merged == nullptr)) return MGWFBP_EINVAL;
    if (L > 0 && merged[0] != 0) return MGWFBP_EINVAL;
    const uint64_t TILE = MGWFBP_TILE_ELEMS;
    const uint64_t limit = std::numeric_limits<uint64_t>::max() / 8;   // byte offsets must not wrap
    uint64_t total = 0;
    for (int32_t i = 0; i < L; ++i) {
        if (merged[i] > 1) return MGWFBP_EINVAL;
        if (n_elems[i] > limit - total) return MGWFBP_EINVAL;
        total += n_elems[i];
    }
    try {
        out = HostTables();
        out.L = L;
        out.tensor_off.assign(static_cast<size_t>(L), 0);
        out.tensor_group.assign(static_cast<size_t>(L), 0);
        out.tensor_n.assign(n_elems, n_elems + L);
        out.group_tile.push_back(0);
        uint64_t next_tile = 0;                        // first free tile of the arena
        int32_t i = L - 1;
        while (i >= 0) {
            // one group: i is its first-arriving member; extend down while the member is merged
            const int32_t k = out.G++;
            const uint64_t base = next_tile * TILE;
            const size_t seg_begin = out.seg_layer.size();
            uint64_t fill = 0;
            for (;;) {
                out.tensor_group[static_cast<size_t>(i)] = k;
                out.tensor_off[static_cast<size_t>(i)] = fill;
                if (n_elems[i] > 0) {
                    out.seg_off.push_back(base + fill);
                    out.seg_n.push_back(static_cast<uint32_t>(std::min<uint64_t>(n_elems[i], 0xffffffffull)));
                    out.seg_layer.push_back(i);
                    fill += n_elems[i];
                }
                const bool closes = merged[i] == 0;
                --i;
                if (closes) break;
            }
            out.group_base.push_back(base);
            out.group_elems.push_back(fill);

            // tile headers of this group
            const uint64_t ntile = (fill + TILE - 1) / TILE;
            if (next_tile + ntile > static_cast<uint64_t>(std::numeric_limits<int32_t>::max())) return MGWFBP_EINVAL;
            if (out.seg_layer.size() > static_cast<size_t>(std::numeric_limits<int32_t>::max())) return MGWFBP_EINVAL;
            const size_t seg_end = out.seg_layer.size();
            size_t s = seg_begin;                      // first segment not entirely before the tile
            for (uint64_t t = 0; t < ntile; ++t) {
                const uint64_t lo = t * TILE;          // tile range inside the group slice
                const uint64_t valid = std::min<uint64_t>(TILE, fill - lo);
                const uint64_t hi = lo + valid;
                auto seg_lo = [&](size_t q) { return out.seg_off[q] - base; };
                auto seg_hi = [&](size_t q) { return (q + 1 < seg_end ? out.seg_off[q + 1] - base : fill); };
                while (seg_hi(s) <= lo) ++s;
                size_t e = s;
                while (e + 1 < seg_end && seg_lo(e + 1) < hi) ++e;
                TileHdr h;
                h.first_start = static_cast<int64_t>(seg_lo(s)) - static_cast<int64_t>(lo);
                h.first_end = static_cast<int32_t>(std::min<uint64_t>(seg_hi(s), hi) - lo);
                h.seg0 = static_cast<int32_t>(s);
                h.nseg = static_cast<int32_t>(e - s + 1);
                h.valid = static_cast<int32_t>(valid);
                h.layer0 = out.seg_layer[s];
                h.flags = 0;
                out.tiles.push_back(h);
            }
            next_tile += ntile;
            out.group_tile.push_back(static_cast<int32_t>(next_tile));
        }
        out.arena_elems = next_tile * TILE;
        out.seg_off.push_back(out.arena_elems);
    } catch (const std::bad_alloc&) {
        return MGWFBP_ENOMEM;
    }
    return MGWFBP_OK;
}
