// Host-side compiler from a per-head plan to per-(batch, head, query tile) work records.
//
// Sec. 4.5 of the paper names the per-thread-block determination of the arrow pattern as
// the overhead that shows when little work remains.  Here the pattern is resolved once per
// distinct plan on the host, in integers: each record lists the key tiles a query tile has
// to visit (text tiles, then the tiles its rows' bands touch) and which of them are free of
// any masked pair, so the kernel never loads a fully masked tile and applies the element
// mask (Sec. 3.1: text quadrants whole, image-image band |i-j| <= w) only on edge tiles.
#include <stdint.h>

#include <algorithm>
#include <new>
#include <vector>

#include "difa.h"
#include "difa_schedule.h"

namespace {

// Token order: the image tokens are [img0, img1), the text tokens the rest ([0, n_text) when the text
// comes first, [n_img, n_tokens) when the image does).  Key tiles are numbered in a rotated order that
// starts at the first tile holding a text key: position u is tile (u + rot) % n_kv_tiles.  With the
// text in front rot is 0; with the image in front the text tiles still come first in that order, so a
// record keeps the same two-range form.
struct Geometry {
    int n_text, n_tokens, bm, bn;
    int img0, img1;
    int rot, n_kv_tiles;
    int tile_at(int u) const { const int t = u + rot; return t >= n_kv_tiles ? t - n_kv_tiles : t; }
};

// Is there a pair (row in [i0,i1), key in [j0, j0+bn)) that must be masked out?
// w < 0 means a full head.  Keys >= n_tokens count as masked.
bool tile_needs_mask(const Geometry& g, int w, int i0, int i1, int j0) {
    const int j1 = j0 + g.bn;
    if (j1 > g.n_tokens) return true;
    if (w < 0) return false;
    const int qi0 = std::max(i0, g.img0), qi1 = std::min(i1, g.img1) - 1;  // image rows [qi0, qi1]
    const int kj0 = std::max(j0, g.img0), kj1 = std::min(j1, g.img1) - 1;  // image keys [kj0, kj1]
    if (qi0 > qi1 || kj0 > kj1) return false;
    return (kj1 - qi0 > w) || (qi1 - kj0 > w);
}

// Mask-free tiles of a range [begin, end) of positions in the rotated order: for the first range the
// mask-free prefix, for the second the longest run of consecutive mask-free tiles.  Treating a mask-free tile as masked
// is always safe, so any sub-run is a valid answer.
void mask_free_run(const Geometry& g, int w, int i0, int i1, int begin, int end, bool prefix_only,
                   int* run_begin, int* run_end) {
    int best_b = begin, best_e = begin;
    int t = begin;
    while (t < end) {
        if (tile_needs_mask(g, w, i0, i1, g.tile_at(t) * g.bn)) {
            if (prefix_only) break;
            ++t;
            continue;
        }
        int e = t;
        while (e < end && !tile_needs_mask(g, w, i0, i1, g.tile_at(e) * g.bn)) ++e;
        if (e - t > best_e - best_b) { best_b = t; best_e = e; }
        if (prefix_only) break;
        t = e;
    }
    *run_begin = best_b;
    *run_end = best_e;
}

}  // namespace

extern "C" int32_t difa_tile_shape(int32_t head_dim, int32_t dtype, int32_t* bm, int32_t* bn) {
    if ((head_dim != 64 && head_dim != 128) || (dtype != DIFA_DTYPE_BF16 && dtype != DIFA_DTYPE_F32))
        return 1;
    if (bm) *bm = 256;
    if (bn) *bn = 64;
    return 0;
}

namespace {
difa_status_t worklist_build(int32_t batch, int32_t heads, const int32_t* head_plan,
                             const int32_t* window, int32_t n_text, int32_t n_img,
                             int32_t bm, int32_t bn, int32_t n_xcd, uint32_t flags,
                             difa_work_item_t* items,
                             int32_t capacity, int32_t* n_items_out,
                             int32_t* copy_heads, int32_t* n_copy_out) {
    if (!head_plan || !n_items_out || batch < 1 || heads < 1 || n_text < 0 || n_img < 0 ||
        bm < 1 || bn < 1 || n_xcd < 1 || n_xcd > 64 || capacity < 0 || (capacity > 0 && !items) ||
        (flags & ~(uint32_t)(DIFA_FLAG_BLOCK_BAND | DIFA_FLAG_IMAGE_FIRST)) != 0)
        return DIFA_ERR_INVALID_ARG;
    const int64_t n64 = (int64_t)n_text + (int64_t)n_img;
    if (n64 < 1 || n64 > (int64_t)1 << 30) return DIFA_ERR_INVALID_ARG;
    for (int h = 0; h < heads; ++h) {
        const int mode = head_plan[h];
        if (mode != DIFA_HEAD_FULL && mode != DIFA_HEAD_ARROW && mode != DIFA_HEAD_CACHE && mode != DIFA_HEAD_ARROW_RESIDUAL)
            return DIFA_ERR_INVALID_ARG;
        if ((mode == DIFA_HEAD_ARROW || mode == DIFA_HEAD_ARROW_RESIDUAL) && (!window || window[h] < 0)) return DIFA_ERR_INVALID_ARG;
    }
    const bool image_first = (flags & DIFA_FLAG_IMAGE_FIRST) != 0 && n_text > 0 && n_img > 0;
    const int n_kv_tiles = (int)((n64 + bn - 1) / bn);
    Geometry g{n_text, (int)n64, bm, bn, 0, 0, 0, n_kv_tiles};
    if (image_first) { g.img0 = 0; g.img1 = n_img; g.rot = n_img / bn; }
    else if (flags & DIFA_FLAG_IMAGE_FIRST) { g.img0 = 0; g.img1 = n_img; }      // one kind of token only
    else { g.img0 = n_text; g.img1 = g.n_tokens; }
    const int n_q_tiles = (g.n_tokens + bm - 1) / bm;
    // tiles that hold at least one text key: the first ones of the rotated order
    const int text_tiles = image_first ? n_kv_tiles - g.rot : (n_text + bn - 1) / bn;

    // Records are first collected head by head (query tiles in ascending order).
    struct HeadSpan { size_t first, count; int64_t cost; };
    std::vector<difa_work_item_t> recs;
    std::vector<HeadSpan> spans;
    int n_copy = 0;
    for (int b = 0; b < batch; ++b) {
        for (int h = 0; h < heads; ++h) {
            const int mode = head_plan[h];
            if (mode == DIFA_HEAD_CACHE) {
                if (b == 0) {
                    if (copy_heads) copy_heads[n_copy] = h;
                    ++n_copy;
                }
                continue;
            }
            // A band that covers the whole image is full attention.
            const bool full = (mode == DIFA_HEAD_FULL) || (window[h] >= n_img - 1);
            const int w = full ? -1 : window[h];
            HeadSpan span{recs.size(), 0, 0};
            for (int qt = 0; qt < n_q_tiles; ++qt) {
                const int i0 = qt * bm, i1 = std::min(i0 + bm, g.n_tokens);
                difa_work_item_t r{};
                r.bh = b * heads + h;
                r.q_tile = qt;
                r.window = w;
                r.flags = mode == DIFA_HEAD_ARROW_RESIDUAL ? DIFA_ITEM_ADD_RESIDUAL : 0;   // arrow attention, then + r
                if (full && !image_first) {
                    r.kv0_end = n_kv_tiles;
                    r.kv1_begin = r.kv1_end = n_kv_tiles;
                } else if (full || i0 < g.img0 || i1 > g.img1) {
                    // every key: a full head, or a tile that holds text queries (they see every key).
                    // (Two ranges when the order is rotated, so that the sequence tail, the one tile a
                    // full head masks, ends the first range and the image tiles are mask-free as a run.)
                    r.kv0_end = text_tiles;
                    r.kv1_begin = text_tiles;
                    r.kv1_end = n_kv_tiles;
                } else {
                    r.kv0_end = text_tiles;
                    // image keys [lo, hi] that some row of the tile sees, as tiles; the tiles that also hold
                    // text keys are in the first range already
                    const int lo = std::max(g.img0, i0 - w);
                    const int hi = std::min(g.img1 - 1, (i1 - 1) + w);
                    if (image_first) {
                        const int t_lo = lo / bn, t_hi = std::min(hi / bn, g.rot - 1);
                        r.kv1_begin = text_tiles + t_lo;
                        r.kv1_end = std::max(r.kv1_begin, text_tiles + t_hi + 1);
                    } else {
                        r.kv1_begin = std::max(text_tiles, lo / bn);
                        r.kv1_end = std::max(r.kv1_begin, hi / bn + 1);
                    }
                }
                // Block-granular band (Sec. 3.3, Fig. 4): every visited block is dense, so the record is
                // masked like a full head's: on the sequence tail only.
                const int wm = (flags & DIFA_FLAG_BLOCK_BAND) ? -1 : w;
                r.window = wm;
                int b0, e0;
                mask_free_run(g, wm, i0, i1, 0, r.kv0_end, true, &b0, &e0);
                r.nm0_end = e0;
                mask_free_run(g, wm, i0, i1, r.kv1_begin, r.kv1_end, false, &r.nm1_begin, &r.nm1_end);
                r.n_tiles = r.kv0_end + (r.kv1_end - r.kv1_begin);
                recs.push_back(r);
                span.cost += r.n_tiles;
            }
            span.count = recs.size() - span.first;
            spans.push_back(span);
        }
    }
    if (n_xcd == 1) {
        // Heaviest records first: the hardware hands workgroups out in index order, so the long
        // full-attention tiles start early and the short band tiles fill the tail.
        std::stable_sort(recs.begin(), recs.end(), [](const difa_work_item_t& a, const difa_work_item_t& b) {
            return a.n_tiles > b.n_tiles;
        });
    } else if (!recs.empty()) {
        // Workgroup p runs on accelerator die p % n_xcd, and every die has its own L2.  If the query
        // tiles of one head are spread over all dies, each die streams that head's K and V from
        // memory: n_xcd times the traffic.  So the records are laid out as n_xcd queues, queue x at
        // positions x, x + n_xcd, ...: heads in order of decreasing cost, the whole sequence cut into
        // n_xcd runs of equal cost, so that a head lives on one die (two where a cut falls inside it),
        // its query tiles run side by side and share the K/V tiles in that die's L2, and every die
        // gets the same amount of work.  Short queues are padded with records whose q_tile is -1.
        std::stable_sort(spans.begin(), spans.end(), [](const HeadSpan& a, const HeadSpan& b) { return a.cost > b.cost; });
        int64_t total = 0;
        for (const HeadSpan& sp : spans) total += sp.cost;
        std::vector<std::vector<difa_work_item_t>> queue((size_t)n_xcd);
        int64_t cum = 0;
        for (const HeadSpan& sp : spans)
            for (size_t k = 0; k < sp.count; ++k) {
                const difa_work_item_t& r = recs[sp.first + k];
                int64_t x = total > 0 ? ((2 * cum + r.n_tiles) * n_xcd) / (2 * total) : 0;
                x = std::min<int64_t>(std::max<int64_t>(x, 0), n_xcd - 1);
                queue[(size_t)x].push_back(r);
                cum += r.n_tiles;
            }
        // Inside a queue: longest records first (a query tile that holds text rows visits every key
        // tile and would otherwise start late and finish last), in classes of 16 key tiles so that
        // records of one head, which differ by a tile or two, stay next to each other.
        for (auto& q : queue)
            std::stable_sort(q.begin(), q.end(), [](const difa_work_item_t& a, const difa_work_item_t& b) {
                return a.n_tiles / 16 > b.n_tiles / 16;
            });
        size_t longest = 0;
        for (const auto& q : queue) longest = std::max(longest, q.size());
        difa_work_item_t pad{};
        pad.q_tile = -1;
        pad.window = -1;
        std::vector<difa_work_item_t> laid(longest * (size_t)n_xcd, pad);
        for (int x = 0; x < n_xcd; ++x)
            for (size_t k = 0; k < queue[(size_t)x].size(); ++k) laid[k * (size_t)n_xcd + (size_t)x] = queue[(size_t)x][k];
        while (!laid.empty() && laid.back().q_tile < 0) laid.pop_back();
        recs.swap(laid);
    }
    *n_items_out = (int32_t)recs.size();
    if (n_copy_out) *n_copy_out = n_copy;
    if ((int64_t)recs.size() > capacity) return capacity == 0 && !items ? DIFA_OK : DIFA_ERR_ALLOC;
    std::copy(recs.begin(), recs.end(), items);
    return DIFA_OK;
}
}  // namespace

extern "C" difa_status_t difa_worklist_build(int32_t batch, int32_t heads, const int32_t* head_plan,
                                             const int32_t* window, int32_t n_text, int32_t n_img,
                                             int32_t bm, int32_t bn, int32_t n_xcd, uint32_t flags,
                                             difa_work_item_t* items,
                                             int32_t capacity, int32_t* n_items_out,
                                             int32_t* copy_heads, int32_t* n_copy_out) {
    try {
        return worklist_build(batch, heads, head_plan, window, n_text, n_img, bm, bn, n_xcd, flags, items, capacity,
                              n_items_out, copy_heads, n_copy_out);
    } catch (const std::bad_alloc&) {
        return DIFA_ERR_ALLOC;
    }
}

// ------------------------------------------------------------------------------------------
// Records -> per-workgroup segment lists for the persistent attention kernel.
//
// The hardware dispatcher would hand whole records to compute units as they free up; with records
// of a few hundred key tiles each, the last round leaves most of the chip idle (1584 equal records on
// 256 compute units: 6.19 rounds cost 7).  Here the distribution is computed on the host instead:
// whole records are dealt out, costliest first, to the least loaded workgroup of their die (which keeps
// the workgroups of a die on neighbouring query tiles of one head, marching through its K/V together),
// and the records that no longer fit under a target load are cut along their key-tile positions into
// pieces that fill the workgroups up to it.  The target is found by a few dry runs (a cut costs a
// good part of a short record, so how much load there is depends on how much is cut); for layers of few,
// long records, filling the workgroups one after the other, or not cutting at all, is tried as well, and
// the plan with the earliest predicted finish is kept.
// ------------------------------------------------------------------------------------------
namespace {

// Cost model of a segment, in eighths of a plain key-tile iteration.  Fitted on MI355X from clock counters
// around the kernel's phases, regressed per workgroup on what the schedule had given it (head_dim 128 and
// 64, the 1K and 2K layers): a plain iteration takes about 3000 clocks (2300 at head_dim 64), one on a tile
// that needs the element mask 0.8-1.0 iterations more; starting and finishing a whole record costs 4-5
// iterations; a piece of a cut record 7-12 (its partial result goes to scratch and a ticket is drawn, both
// round trips to memory), and the piece that arrives last pays 3-9 more per other piece it folds in.  Who
// arrives last is not known here, so every piece is charged its share.
constexpr int kUnit = 8;                  // cost units per key-tile iteration
constexpr int kMaskedExtra = 7;           // extra units of an iteration on a masked tile
constexpr int kWholeOverhead = 36;        // starting and finishing a whole record
constexpr int kPieceOverhead = 72;        // ... a piece of a cut record, without the fold
constexpr int kFoldPerSlot = 40;          // folding one other piece's partial result in
constexpr int kPieceExpected = kPieceOverhead + kFoldPerSlot / 2;   // what a piece is charged while cutting
constexpr int kMinPiece = 12;             // shortest piece (in key tiles) worth cutting off a record

// Masked tiles among positions [p0, p1) of a record's visiting order.
int masked_between(const difa_work_item_t& r, int p0, int p1) {
    int n = 0;
    const int e0 = std::min(p1, r.kv0_end);
    if (p0 < e0) n += std::max(0, e0 - std::max(p0, std::min(r.nm0_end, r.kv0_end)));
    const int b1 = std::max(p0, r.kv0_end);
    if (b1 < p1) {
        const int a = r.kv1_begin + (b1 - r.kv0_end), b = r.kv1_begin + (p1 - r.kv0_end);
        const int free = std::max(0, std::min(b, r.nm1_end) - std::max(a, r.nm1_begin));
        n += (b - a) - free;
    }
    return n;
}

int64_t tiles_cost(const difa_work_item_t& r, int p0, int p1) {
    return (int64_t)kUnit * (p1 - p0) + (int64_t)kMaskedExtra * masked_between(r, p0, p1);
}
int64_t whole_cost(const difa_work_item_t& r) { return tiles_cost(r, 0, r.n_tiles) + kWholeOverhead; }

difa_segment_t whole_segment(const difa_work_item_t& r) {
    difa_segment_t s{};
    s.bh = r.bh; s.q_tile = r.q_tile;
    s.kv0_end = r.kv0_end; s.nm0_end = r.nm0_end;
    s.kv1_begin = r.kv1_begin; s.kv1_end = r.kv1_end;
    s.nm1_begin = r.nm1_begin; s.nm1_end = r.nm1_end;
    s.window = r.window;
    s.flags = r.flags;
    s.pos_begin = 0; s.pos_end = r.n_tiles;
    s.part_slot = -1;
    s.merge_idx = -1;
    s.n_parts = 1;
    s.first_slot = -1;
    return s;
}

// One die's share of the schedule.  A dry run fills in the loads and counts only.
struct DiePlan {
    std::vector<std::vector<difa_segment_t>> lists;   // a segment list per workgroup, slots numbered from 0
    std::vector<difa_merge_item_t> merges;
    std::vector<int64_t> load;
    int n_slots = 0;
    int most_parts = 1;
    int64_t makespan = 0, total = 0;
};

struct Piece { int wg, pos_begin, pos_end; };

void finish_record(DiePlan& plan, const difa_work_item_t& r, const std::vector<Piece>& pieces, bool dry) {
    const int n = (int)pieces.size();
    plan.most_parts = std::max(plan.most_parts, n);
    if (n > 1) {
        // the pieces were charged kPieceExpected each; put the fold at what this record's piece count makes it
        const int64_t fold = (int64_t)kFoldPerSlot * (n - 1) / n - kFoldPerSlot / 2;
        for (const Piece& pc : pieces) plan.load[(size_t)pc.wg] += fold;
    }
    if (dry) {
        if (n > 1) plan.n_slots += n;
        return;
    }
    const int first_slot = plan.n_slots;
    for (const Piece& pc : pieces) {
        difa_segment_t s = whole_segment(r);
        s.pos_begin = pc.pos_begin;
        s.pos_end = pc.pos_end;
        if (n > 1) {
            s.first_slot = first_slot;
            s.part_slot = plan.n_slots++;
            s.merge_idx = (int32_t)plan.merges.size();
            s.n_parts = n;
        }
        plan.lists[(size_t)pc.wg].push_back(s);
    }
    if (n > 1) plan.merges.push_back(difa_merge_item_t{r.bh, r.q_tile, first_slot, n});
}

void close_plan(DiePlan& plan) {
    plan.makespan = *std::max_element(plan.load.begin(), plan.load.end());
    plan.total = 0;
    for (int64_t l : plan.load) plan.total += l;
}

// Records in order of decreasing cost.  A record goes whole to the least loaded workgroup (so neighbouring
// query tiles of a head run side by side and share its K/V tiles in the die's L2) as long as that leaves the
// workgroup room for another half of it; otherwise it is poured: laid into the room of the workgroup that is
// being filled, cut where that room ends, the rest into the room of the workgroup that is then the least
// loaded, and so on.  Rooms are therefore of the order of a record when long records are cut (two or three
// pieces each, so the workgroup that folds them together at the end reads one or two slots, not ten), and
// short records, which are not worth cutting, fill the gaps that remain.
DiePlan deal_and_pour(const std::vector<difa_work_item_t>& q, const std::vector<int64_t>& cost, int per_die,
                      int64_t target, int slot_budget, bool dry) {
    DiePlan plan;
    if (!dry) plan.lists.resize((size_t)per_die);
    plan.load.assign((size_t)per_die, 0);
    std::vector<int64_t>& load = plan.load;
    auto least = [&]() { return (int)(std::min_element(load.begin(), load.end()) - load.begin()); };
    std::vector<Piece> pieces;
    std::vector<size_t> n_whole((size_t)per_die, 0);
    std::vector<char> poured((size_t)per_die, 0);
    int cur = -1;
    auto room_of = [&](int w) { return (target - load[(size_t)w] - kPieceExpected) / kUnit; };   // in key tiles
    for (size_t i = 0; i < q.size(); ++i) {
        const difa_work_item_t& r = q[i];
        const int64_t c = cost[i];
        const int lw = least();
        if (load[(size_t)lw] + c + c / 2 <= target) {
            load[(size_t)lw] += c;
            if (!dry) plan.lists[(size_t)lw].push_back(whole_segment(r));
            if (!poured[(size_t)lw]) ++n_whole[(size_t)lw];
            continue;
        }
        pieces.clear();
        int pos = 0;
        while (pos < r.n_tiles) {
            if (cur < 0 || room_of(cur) < kMinPiece) cur = least();
            const int w = cur;
            const int remaining = r.n_tiles - pos;
            const int64_t room = room_of(w);
            int take = remaining;
            const bool may_cut = plan.n_slots + (int)pieces.size() + 2 <= slot_budget;
            if (pos == 0 && load[(size_t)w] + c <= target) {
                // the whole record fits
            } else if (may_cut && room >= kMinPiece && room < remaining) {
                take = (int)room;
                if (remaining - take < kMinPiece) take = remaining - kMinPiece >= kMinPiece ? remaining - kMinPiece : remaining;
            } else if (may_cut && room < kMinPiece && remaining >= 4 * kMinPiece) {
                // no room anywhere (the target was too low): spread what is left over the least loaded
                // workgroups in pieces of two to four times the shortest one, rather than on one of them
                const int n = (remaining + 3 * kMinPiece - 1) / (3 * kMinPiece);
                take = (remaining + n - 1) / n;
            }
            pieces.push_back(Piece{w, pos, pos + take});
            load[(size_t)w] += tiles_cost(r, pos, pos + take) + (take == r.n_tiles ? kWholeOverhead : kPieceExpected);
            poured[(size_t)w] = 1;
            pos += take;
        }
        finish_record(plan, r, pieces, dry);
    }
    // A poured room holds the tail of one record and the head of the next one, neighbouring query tiles of
    // one head as a rule.  Run in the order of their first key position (the shorter one first among equals),
    // the workgroups of the die walk through that head's K/V within a fraction of a record of each other and
    // share the tiles in the die's L2, as they do on whole records; the pieces of a record may finish in any
    // order, since the last one to arrive folds them.
    if (!dry)
        for (int w = 0; w < per_die; ++w) {
            auto& l = plan.lists[(size_t)w];
            std::stable_sort(l.begin() + (std::ptrdiff_t)n_whole[(size_t)w], l.end(),
                             [](const difa_segment_t& a, const difa_segment_t& b) {
                                 return a.pos_begin != b.pos_begin ? a.pos_begin < b.pos_begin
                                                                   : a.pos_end - a.pos_begin < b.pos_end - b.pos_begin;
                             });
        }
    close_plan(plan);
    return plan;
}

// The records laid end to end and handed out in runs of the target cost: workgroup 0 is filled, then
// workgroup 1, ...; a record that crosses a boundary is cut there.
DiePlan fill_in_order(const std::vector<difa_work_item_t>& q, const std::vector<int64_t>& cost, int per_die,
                      int64_t target, int slot_budget, bool dry) {
    DiePlan plan;
    if (!dry) plan.lists.resize((size_t)per_die);
    plan.load.assign((size_t)per_die, 0);
    std::vector<int64_t>& load = plan.load;
    std::vector<Piece> pieces;
    int w = 0;
    for (size_t i = 0; i < q.size(); ++i) {
        const difa_work_item_t& r = q[i];
        pieces.clear();
        int pos = 0;
        if (w < per_die - 1 && load[(size_t)w] > 0 && load[(size_t)w] + cost[i] > target &&
            (target - load[(size_t)w] - kPieceExpected) / kUnit < kMinPiece)
            ++w;                                                      // no room worth a piece: the next workgroup goes on
        while (pos < r.n_tiles) {
            const int remaining = r.n_tiles - pos;
            const int64_t ovh = pos == 0 ? kWholeOverhead : kPieceExpected;
            int take = remaining;
            if (w < per_die - 1 && load[(size_t)w] + tiles_cost(r, pos, r.n_tiles) + ovh > target) {
                const int64_t room = (target - load[(size_t)w] - kPieceExpected) / kUnit;   // in key tiles
                const bool may_cut = plan.n_slots + (int)pieces.size() + 2 <= slot_budget;
                if (may_cut && room >= kMinPiece && remaining - room >= kMinPiece) take = (int)room;
                else if (may_cut && room >= kMinPiece && remaining - kMinPiece >= kMinPiece) take = remaining - kMinPiece;
                else if (load[(size_t)w] > 0 && pos == 0) { ++w; continue; }   // rather start it on the next workgroup
            }                                                         // else: overfill
            pieces.push_back(Piece{w, pos, pos + take});
            load[(size_t)w] += tiles_cost(r, pos, pos + take) + (take == r.n_tiles ? kWholeOverhead : kPieceExpected);
            pos += take;
            if (pos < r.n_tiles && w < per_die - 1) ++w;              // cut: the rest starts the next workgroup
        }
        finish_record(plan, r, pieces, dry);
    }
    close_plan(plan);
    return plan;
}

// The smallest target a method gets along with: too low a target leaves work over that lands on one
// workgroup, too high a one leaves the last workgroups idle.  A few dry runs, each aiming just above the mean
// load of the one before (the mean moves little: only the number of pieces changes it).
template <class Run>
int64_t settle_target(int64_t first, int per_die, Run run) {
    int64_t target = first, best_target = first, best_span = -1;
    for (int round = 0; round < 3; ++round) {
        const DiePlan p = run(target, true);
        if (best_span < 0 || p.makespan < best_span) { best_span = p.makespan; best_target = target; }
        const int64_t mean = (p.total + per_die - 1) / per_die;
        int64_t next;
        if (p.makespan > target + target / 128) next = target + std::max<int64_t>(kUnit, (p.makespan - target) / 8);   // work was left over
        else next = mean + kUnit;                                    // it all went in: aim just above the mean load
        if (next == target || (p.makespan <= target + target / 128 && next > target)) break;
        target = next;
    }
    return best_target;
}

// Whole records only, each to the least loaded workgroup: the plan to beat when records are few and a cut
// costs a good part of a record.
DiePlan deal_whole(const std::vector<difa_work_item_t>& q, const std::vector<int64_t>& cost, int per_die, bool dry) {
    DiePlan plan;
    if (!dry) plan.lists.resize((size_t)per_die);
    plan.load.assign((size_t)per_die, 0);
    for (size_t i = 0; i < q.size(); ++i) {
        const int w = (int)(std::min_element(plan.load.begin(), plan.load.end()) - plan.load.begin());
        plan.load[(size_t)w] += cost[i];
        if (!dry) plan.lists[(size_t)w].push_back(whole_segment(q[i]));
    }
    close_plan(plan);
    return plan;
}

difa_status_t schedule_build(const difa_work_item_t* items, int32_t n_items, int32_t n_wg,
                             int32_t n_xcd, const double* die_speed, int64_t* die_span, difa_segment_t* segs,
                             int32_t seg_capacity, int32_t* wg_begin, int32_t* n_segs_out, difa_merge_item_t* merges,
                             int32_t merge_capacity, int32_t* n_merges_out, int32_t* n_slots_out) {
    if (n_items < 0 || (n_items > 0 && !items) || n_wg < 1 || n_xcd < 1 || n_wg % n_xcd != 0 || !wg_begin ||
        !n_segs_out || !n_merges_out || !n_slots_out || seg_capacity < 0 || merge_capacity < 0 ||
        (seg_capacity > 0 && !segs) || (merge_capacity > 0 && !merges))
        return DIFA_ERR_INVALID_ARG;
    std::vector<difa_work_item_t> recs;
    for (int32_t i = 0; i < n_items; ++i) {
        if (items[i].q_tile < 0) continue;
        if (items[i].n_tiles < 1) return DIFA_ERR_INVALID_ARG;
        recs.push_back(items[i]);
    }
    std::stable_sort(recs.begin(), recs.end(), [](const difa_work_item_t& a, const difa_work_item_t& b) {
        return a.bh != b.bh ? a.bh < b.bh : a.q_tile < b.q_tile;
    });
    // heads in order of decreasing cost, the whole sequence cut into n_xcd runs whose costs are in
    // proportion to the dies' speeds (equal when none are given)
    struct HeadSpan { size_t first, count; int64_t cost; };
    std::vector<HeadSpan> spans;
    for (size_t i = 0; i < recs.size();) {
        size_t j = i;
        int64_t cost = 0;
        while (j < recs.size() && recs[j].bh == recs[i].bh) { cost += whole_cost(recs[j]); ++j; }
        spans.push_back({i, j - i, cost});
        i = j;
    }
    std::stable_sort(spans.begin(), spans.end(), [](const HeadSpan& a, const HeadSpan& b) { return a.cost > b.cost; });
    int64_t total = 0;
    for (const HeadSpan& sp : spans) total += sp.cost;
    const int per_die = n_wg / n_xcd;
    const int slot_capacity = 2 * n_wg;
    std::vector<double> speed((size_t)n_xcd, 1.0);         // relative speeds of the dies (their clocks differ under load)
    if (die_speed)
        for (int x = 0; x < n_xcd; ++x) speed[(size_t)x] = die_speed[x] > 0.5 && die_speed[x] < 2.0 ? die_speed[x] : 1.0;
    std::vector<double> share(speed);                      // the part of the work each die is given, up to a common factor
    std::vector<DiePlan> plans((size_t)n_xcd), first_plans;
    double first_t_max = 0.0;
    std::vector<int64_t> cost;
    // Two rounds at most: the first hands out the work in proportion to the dies' speeds; where the plans that
    // come out of it would finish more than three hundredths apart (a die whose records had to be cut carries the
    // overhead of the cuts), the shares are corrected by that and the plans made again, and kept if they are better.
    for (int round = 0; round < 2; ++round) {
        std::vector<double> upto((size_t)n_xcd + 1, 0.0);  // cumulative share of the work that dies 0 .. x-1 take
        {
            double sum = 0.0;
            for (int x = 0; x < n_xcd; ++x) sum += share[(size_t)x];
            for (int x = 0; x < n_xcd; ++x) upto[(size_t)x + 1] = upto[(size_t)x] + share[(size_t)x] / sum;
            upto[(size_t)n_xcd] = 2.0;
        }
        std::vector<std::vector<difa_work_item_t>> die((size_t)n_xcd);
        int64_t cum = 0;
        int x_at = 0;
        for (const HeadSpan& sp : spans)
            for (size_t k = 0; k < sp.count; ++k) {
                const difa_work_item_t& r = recs[sp.first + k];
                const int64_t c = whole_cost(r);
                const double mid = total > 0 ? (double)(2 * cum + c) / (double)(2 * total) : 0.0;
                while (x_at < n_xcd - 1 && mid >= upto[(size_t)x_at + 1]) ++x_at;
                die[(size_t)x_at].push_back(r);
                cum += c;
            }
        int slots_so_far = 0;
        for (int x = 0; x < n_xcd; ++x) {
            std::vector<difa_work_item_t>& q = die[(size_t)x];
            // costliest records first (a query tile that holds text rows visits every key tile); the interior
            // query tiles of a head cost the same and stay neighbours
            {
                std::vector<std::pair<int64_t, int>> key(q.size());
                for (size_t i = 0; i < q.size(); ++i) key[i] = {-whole_cost(q[i]), (int)i};
                std::sort(key.begin(), key.end());                   // (ties keep their order: the index decides)
                std::vector<difa_work_item_t> sorted(q.size());
                cost.resize(q.size());
                for (size_t i = 0; i < q.size(); ++i) { sorted[i] = q[(size_t)key[i].second]; cost[i] = -key[i].first; }
                q.swap(sorted);
            }
            int64_t die_cost = 0;
            for (size_t i = 0; i < q.size(); ++i) die_cost += cost[i];
            const int budget = slot_capacity - slots_so_far - 2 * per_die * (n_xcd - 1 - x);   // this die's share of the slots
            // every workgroup is expected to take one piece
            const int64_t first = (die_cost + (int64_t)per_die * kPieceExpected + per_die - 1) / per_die;
            auto deal = [&](int64_t t, bool dry) { return deal_and_pour(q, cost, per_die, t, budget, dry); };
            auto fill = [&](int64_t t, bool dry) { return fill_in_order(q, cost, per_die, t, budget, dry); };
            DiePlan dealt = deal(settle_target(first, per_die, deal), false);
            // When the records are few and long compared with a workgroup's share (small layers), dealing whole
            // records and cutting the rest leaves the workgroups uneven; filling them one after the other may
            // then be the better plan, or not cutting at all.
            const int64_t even = die_cost / per_die;
            if (dealt.makespan * 20 > even * 21) {
                DiePlan filled = fill(settle_target(first, per_die, fill), false);
                if (filled.makespan < dealt.makespan) dealt = std::move(filled);
                const DiePlan whole = deal_whole(q, cost, per_die, true);
                if (whole.makespan * 50 <= dealt.makespan * 51) dealt = deal_whole(q, cost, per_die, false);
            }
            slots_so_far += dealt.n_slots;
            plans[(size_t)x] = std::move(dealt);
        }
        // predicted finishing times, in cost units of a die of speed 1
        double t_min = 0.0, t_max = 0.0, t_sum = 0.0;
        for (int x = 0; x < n_xcd; ++x) {
            const double t = (double)plans[(size_t)x].makespan / speed[(size_t)x];
            t_min = x == 0 ? t : std::min(t_min, t);
            t_max = std::max(t_max, t);
            t_sum += t;
        }
        if (round == 1) {
            if (t_max >= first_t_max) plans.swap(first_plans);       // the correction did not help: keep the first plans
            break;
        }
        if (t_sum <= 0.0 || t_min <= 0.0 || (t_max - t_min) * n_xcd <= 0.03 * t_sum) break;
        for (int x = 0; x < n_xcd; ++x)
            share[(size_t)x] *= (t_sum / n_xcd) / ((double)plans[(size_t)x].makespan / speed[(size_t)x]);
        first_t_max = t_max;
        first_plans = plans;
    }
    std::vector<std::vector<difa_segment_t>> lists((size_t)n_wg);
    std::vector<difa_merge_item_t> merge_list;
    int n_slots = 0;
    for (int x = 0; x < n_xcd; ++x) {
        const DiePlan& dealt = plans[(size_t)x];
        if (die_span) die_span[x] = dealt.makespan;
        for (int w = 0; w < per_die; ++w)
            for (difa_segment_t sg : dealt.lists[(size_t)w]) {
                if (sg.part_slot >= 0) { sg.part_slot += n_slots; sg.first_slot += n_slots; sg.merge_idx += (int32_t)merge_list.size(); }
                lists[(size_t)(w * n_xcd + x)].push_back(sg);
            }
        for (difa_merge_item_t m : dealt.merges) {
            m.first_slot += n_slots;
            merge_list.push_back(m);
        }
        n_slots += dealt.n_slots;
    }
    int64_t n_segs = 0;
    for (const auto& l : lists) n_segs += (int64_t)l.size();
    *n_segs_out = (int32_t)n_segs;
    *n_merges_out = (int32_t)merge_list.size();
    *n_slots_out = n_slots;
    if (n_segs > seg_capacity || (int64_t)merge_list.size() > merge_capacity) return DIFA_ERR_ALLOC;
    int32_t at = 0;
    for (int w = 0; w < n_wg; ++w) {
        wg_begin[w] = at;
        for (const difa_segment_t& s : lists[(size_t)w]) segs[at++] = s;
    }
    wg_begin[n_wg] = at;
    std::copy(merge_list.begin(), merge_list.end(), merges);
    return DIFA_OK;
}
}  // namespace

extern "C" difa_status_t difa_schedule_build(const difa_work_item_t* items, int32_t n_items, int32_t n_wg,
                                             int32_t n_xcd, difa_segment_t* segs, int32_t seg_capacity,
                                             int32_t* wg_begin, int32_t* n_segs_out, difa_merge_item_t* merges,
                                             int32_t merge_capacity, int32_t* n_merges_out, int32_t* n_slots_out) {
    try {
        return schedule_build(items, n_items, n_wg, n_xcd, nullptr, nullptr, segs, seg_capacity, wg_begin, n_segs_out,
                              merges, merge_capacity, n_merges_out, n_slots_out);
    } catch (const std::bad_alloc&) {
        return DIFA_ERR_ALLOC;
    }
}

// The same for the library's own calls: with the dies' relative speeds as measured on earlier launches (NULL:
// all alike), and returning each die's predicted finishing time in the scheduler's cost units.
difa_status_t difa::schedule_for_dies(const difa_work_item_t* items, int32_t n_items, int32_t n_wg, int32_t n_xcd,
                                      const double* die_speed, int64_t* die_span, difa_segment_t* segs,
                                      int32_t seg_capacity, int32_t* wg_begin, int32_t* n_segs_out,
                                      difa_merge_item_t* merges, int32_t merge_capacity, int32_t* n_merges_out,
                                      int32_t* n_slots_out) {
    try {
        return schedule_build(items, n_items, n_wg, n_xcd, die_speed, die_span, segs, seg_capacity, wg_begin, n_segs_out,
                              merges, merge_capacity, n_merges_out, n_slots_out);
    } catch (const std::bad_alloc&) {
        return DIFA_ERR_ALLOC;
    }
}
