// Host side of the C ABI: plan construction, validation, queries.
// No HIP call is made from this file (destroying a plan that still holds profiling
// events releases them through rsdgc_profile_end).
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>

#include "rsdgc_internal.h"

namespace rsdgc {

// Eq. 11: k = ceil((G / p^2) * rho), evaluated in double in that order,
// clamped to [0, G].
int64_t keep_count(int64_t G, int p, double rho) {
    const double per_window = static_cast<double>(G) / static_cast<double>(int64_t(p) * int64_t(p));
    const double kf = std::ceil(per_window * rho);
    if (!(kf > 0.0)) return 0;
    if (kf > static_cast<double>(G)) return G;
    return static_cast<int64_t>(kf);
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int build_tables(rsdgc_plan_s *plan) {
    const int L = plan->n_layers;
    plan->layers.assign(L, LayerDev{});
    plan->groups.clear();
    plan->tile_dir.clear();
    plan->chunk_dir.clear();
    plan->all_tile_dir.clear();
    plan->large_dir.clear();
    plan->samples.clear();
    plan->cand_groups.clear();
    plan->map_chunks.clear();
    plan->map_tiles.clear();
    plan->any_large = false;
    plan->big_map_layers = false;

    int64_t elem_off = 0, out_off = 0, centre_off = 0;
    uint32_t chunk_begin = 0, tile_begin_all = 0, group_begin = 0, cgroup_begin = 0;
    uint64_t list_off = 0, slot_off = 0;
    for (int l = 0; l < L; ++l) {
        LayerDev &d = plan->layers[l];
        int64_t R = plan->shapes[l].rows, C = plan->shapes[l].cols;
        const int64_t G = R * C;
        const int p = plan->p[l];
        // A single column is handled as a single row: the same elements at the same flat indices with
        // the same neighbours (Eq. 7's distance on one axis only), and rows are what the tiles stream.
        // (Not for a block grid, whose wire format depends on the orientation of the p x p blocks.)
        if (C == 1 && !plan->blocks && plan->k_override.empty()) std::swap(R, C);
        const int64_t k = plan->k_override.empty() ? keep_count(G, p, plan->ratio[l]) : plan->k_override[l];
        int64_t cap = k * p * p;
        if (cap > G && !plan->blocks) cap = G;   // (a kept block always sends p*p values, padding included)
        d.elem_off = elem_off;
        d.out_off = out_off;
        d.centre_off = centre_off;
        d.R = static_cast<uint32_t>(R);
        d.C = static_cast<uint32_t>(C);
        d.G = static_cast<uint32_t>(G);
        d.k = static_cast<uint32_t>(k);
        d.p = static_cast<uint32_t>(p);
        d.tiles_x = static_cast<uint32_t>((C + kTileCols - 1) / kTileCols);
        d.n_tiles = d.tiles_x * static_cast<uint32_t>((R + kTileRows - 1) / kTileRows);
        if (plan->blocks) {   // tiles of the block-score kernel instead: 8 x block_tile_cols(p) blocks
            const int64_t BR = (R + p - 1) / p, BC = (C + p - 1) / p;
            d.tiles_x = static_cast<uint32_t>((BC + block_tile_cols(p) - 1) / block_tile_cols(p));
            d.n_tiles = d.tiles_x * static_cast<uint32_t>((BR + kBlockTileRows - 1) / kBlockTileRows);
        }
        d.chunk_begin = chunk_begin;
        d.n_chunks = static_cast<uint32_t>((G + kChunk - 1) / kChunk);
        d.cap = static_cast<uint32_t>(cap);
        d.tile_begin_all = tile_begin_all;
        d.group_begin = group_begin;
        d.cgroup_begin = cgroup_begin;
        d.pad_ = 0;
        d.n_groups = (d.n_tiles + kSlotGroup - 1) / kSlotGroup;
        d.list_off = list_off;
        // a block grid is ranked on its full score map whatever its size: its threshold bucket may hold
        // a large part of a large layer, so the list takes all of it (else 1/32, see kListDiv)
        d.list_cap = plan->k_override.empty()
                         ? static_cast<uint32_t>(std::min<int64_t>(G, std::max<int64_t>(kListMin, G / kListDiv)))
                         : static_cast<uint32_t>(G);
        // workgroups append through kListShards counters so that few atomics meet on one address
        // (each takes the shard of its id modulo kListShards: an even split unless nearly the whole
        // layer lies in the bucket, in which case the ranking streams the score map instead)
        d.list_shards = kListShards;
        list_off += d.list_cap;

        // Candidate path: only the centres whose score reaches a bound are recorded, per tile, and
        // ranked.  The bound aims at up to two times k_l centres (a predicted bound at fewer).  A layer
        // is eligible when 8 k_l / tiles -- four times that aim, for tiles that hold more than their
        // share -- fits a tile's slot of kSlotCapMax entries.  A tile that still overflows sends the
        // layer to the full map for that call.  Small layers are eligible too: once their bounds are
        // predicted, no layer of a typical plan needs the separate score-map pass any more.  (Their
        // thresholds move more from call to call, so their bounds sit lower; a tile of a narrow
        // layer has fewer elements than a slot has entries and cannot overflow at all.)
        uint32_t n_sampled = 0;
        const uint32_t sshift = sample_shift(d.n_tiles);
        for (uint32_t t = 0; t < d.n_tiles; ++t) n_sampled += tile_is_sampled(t, sshift) ? 1u : 0u;
        d.n_sampled = n_sampled;
        const double frac = d.n_tiles ? double(n_sampled) / double(d.n_tiles) : 0.0;
        const double want = 2.0 * double(k) * frac;
        const double per_tile = d.n_tiles ? 8.0 * double(k) / double(d.n_tiles) : 0.0;
        d.large = (plan->allow_candidates && k > 0 && per_tile <= double(kSlotCapMax)) ? 1u : 0u;
        // (a tile of a narrow or flat layer holds fewer elements than kSlotCapMax: its slots are that short.
        // The size follows from the shape alone, so the layout does not move with the ratios.)
        const int64_t tile_elems = std::min<int64_t>(R, kTileRows) * std::min<int64_t>(C, kTileCols);
        d.slot_cap = static_cast<uint32_t>(std::min<int64_t>(kSlotCapMax, (tile_elems + 1) & ~int64_t(1)));
        d.slot_off = slot_off;
        slot_off += static_cast<uint64_t>(d.n_tiles) * d.slot_cap;
        d.hint_target = d.large ? static_cast<uint32_t>(std::ceil(want + 4.0 * std::sqrt(want) + 8.0)) : 0u;
        plan->any_large = plan->any_large || d.large;
        plan->big_map_layers = plan->big_map_layers || (!d.large && k > 0 && G >= kBigMapLayer);

        plan->chunk_dir.push_back(DirEntry{chunk_begin, static_cast<uint32_t>(l)});
        plan->all_tile_dir.push_back(DirEntry{tile_begin_all, static_cast<uint32_t>(l)});
        chunk_begin += d.n_chunks;
        tile_begin_all += d.n_tiles;
        group_begin += d.n_groups;
        cgroup_begin += (d.n_chunks + kChunkGroup - 1) / kChunkGroup;
        elem_off += (G + kLayerAlign - 1) / kLayerAlign * kLayerAlign;
        out_off += cap;
        centre_off += k;
    }
    plan->chunk_dir.push_back(DirEntry{chunk_begin, static_cast<uint32_t>(L)});
    plan->all_tile_dir.push_back(DirEntry{tile_begin_all, static_cast<uint32_t>(L)});
    plan->n_chunks = chunk_begin;
    plan->n_chunk_groups = 0;
    plan->n_count_groups = 0;
    for (const LayerDev &d : plan->layers) {
        plan->n_chunk_groups += (d.n_chunks + kChunkGroup - 1) / kChunkGroup;
        plan->n_count_groups += (d.n_chunks + kCountChunks - 1) / kCountChunks;
    }
    plan->n_tiles_all = tile_begin_all;
    plan->slot_entries = slot_off;
    plan->n_slot_groups = group_begin;
    plan->total_elems = elem_off;
    plan->out_capacity = out_off;
    plan->centre_capacity = centre_off;

    // static work lists of the passes after the NSI kernels: which slot groups can hold
    // candidates, which chunks / tiles belong to layers that are ranked on the full map
    for (int l = 0; l < L; ++l) {
        const LayerDev &d = plan->layers[l];
        if (d.large) {
            for (uint32_t g = 0; g < d.n_groups; ++g) {
                const uint32_t t0 = g * kSlotGroup;
                plan->cand_groups.push_back(GroupEntry{static_cast<uint32_t>(l), d.tile_begin_all + t0,
                                                       std::min<uint32_t>(kSlotGroup, d.n_tiles - t0), 0u});
            }
        } else if (d.k > 0) {
            for (uint32_t c = 0; c < d.n_chunks; ++c) {
                const uint32_t start = c * kChunk;
                plan->map_chunks.push_back(ChunkEntry{static_cast<uint32_t>(l), start,
                                                      std::min<uint32_t>(kChunk, d.G - start), 0u,
                                                      static_cast<uint64_t>(d.elem_off) + start});
            }
            for (uint32_t t = 0; t < d.n_tiles; ++t)
                plan->map_tiles.push_back(SampleEntry{static_cast<uint32_t>(l), t});
        }
    }

    // one launch of each NSI pass per distinct neighbourhood side
    for (int p = 1; p <= RSDGC_MAX_P; p += 2) {
        PGroup g;
        g.p = p;
        g.dir_begin = static_cast<uint32_t>(plan->tile_dir.size());
        g.large_dir_begin = static_cast<uint32_t>(plan->large_dir.size());
        g.sample_begin = static_cast<uint32_t>(plan->samples.size());
        for (int l = 0; l < L; ++l) {
            if (plan->p[l] != p) continue;
            LayerDev &d = plan->layers[l];
            d.tile_begin = g.n_tiles;
            plan->tile_dir.push_back(DirEntry{g.n_tiles, static_cast<uint32_t>(l)});
            g.n_tiles += d.n_tiles;
            ++g.dir_count;
            if (d.large) {
                plan->large_dir.push_back(DirEntry{g.n_large_tiles, static_cast<uint32_t>(l)});
                g.n_large_tiles += d.n_tiles;
                ++g.large_dir_count;
            }
        }
        // tile list of the first NSI pass: every tile of the layers that select something and are not
        // on the candidate path, then the sampled tiles of those that are (wanted only while bounds
        // are still sampled)
        for (int part = 0; part < 2; ++part) {
            for (int l = 0; l < L; ++l) {
                if (plan->p[l] != p) continue;
                const LayerDev &d = plan->layers[l];
                if ((d.large != 0u) != (part == 1)) continue;
                for (uint32_t t = 0; t < d.n_tiles; ++t)
                    if (d.large ? tile_is_sampled(t, sample_shift(d.n_tiles)) : d.k > 0)
                        plan->samples.push_back(SampleEntry{static_cast<uint32_t>(l), t});
            }
            if (part == 0) g.n_map_samples = static_cast<uint32_t>(plan->samples.size()) - g.sample_begin;
        }
        if (g.dir_count == 0) continue;
        g.n_samples = static_cast<uint32_t>(plan->samples.size()) - g.sample_begin;
        plan->tile_dir.push_back(DirEntry{g.n_tiles, static_cast<uint32_t>(L)});  // sentinel
        plan->large_dir.push_back(DirEntry{g.n_large_tiles, static_cast<uint32_t>(L)});
        plan->groups.push_back(g);
    }

    // workspace layout
    WsLayout &w = plan->ws;
    const size_t A = 256;
    const size_t words = static_cast<size_t>(plan->total_elems / 32);
    // sized for the worst case so that new ratios never change the workspace size
    const size_t max_samples = plan->n_tiles_all;
    size_t off = 0;
    w.layers = off;       off = align_up(off + sizeof(LayerDev) * L, A);
    w.tile_dir = off;     off = align_up(off + sizeof(DirEntry) * (L + (RSDGC_MAX_P + 1) / 2), A);
    w.chunk_dir = off;    off = align_up(off + sizeof(DirEntry) * (L + 1), A);
    w.large_dir = off;    off = align_up(off + sizeof(DirEntry) * (L + (RSDGC_MAX_P + 1) / 2), A);
    w.all_tile_dir = off; off = align_up(off + sizeof(DirEntry) * (L + 1), A);
    w.samples = off;      off = align_up(off + sizeof(SampleEntry) * (max_samples + 1), A);
    w.chunk_layer = off;  off = align_up(off + sizeof(uint32_t) * plan->n_chunks, A);
    w.chunk_info = off;   off = align_up(off + sizeof(ChunkInfo) * plan->n_chunks, A);
    w.cand_groups = off;  off = align_up(off + sizeof(GroupEntry) * plan->n_slot_groups, A);
    w.map_chunks = off;   off = align_up(off + sizeof(ChunkEntry) * plan->n_chunks, A);
    w.map_tiles = off;    off = align_up(off + sizeof(SampleEntry) * (size_t(plan->n_tiles_all) + 1), A);
    w.count_groups = off; off = align_up(off + sizeof(CountGroup) * plan->n_count_groups, A);
    w.pred = off;         off = align_up(off + sizeof(PredState) * L, A);
    w.table_bytes = off;
    w.state = off;        off = align_up(off + sizeof(SelState) * L, A);   // written in full each call
    w.flags = off;        off = align_up(off + sizeof(uint32_t) * 64, A);
    w.zero_begin = off;
    w.hist = off;         off = align_up(off + sizeof(uint32_t) * kHistBins * L, A);
    w.hist_s = off;       off = align_up(off + sizeof(uint32_t) * kHistBins * L, A);
    w.hist1 = off;        off = align_up(off + sizeof(uint32_t) * kLevel1Bins * L, A);
    w.chunk_cnt = off;    off = align_up(off + sizeof(uint32_t) * plan->n_chunks, A);
    w.chunk_ccnt = off;   off = align_up(off + sizeof(uint32_t) * plan->n_chunks, A);
    w.group_cnt = off;    off = align_up(off + sizeof(uint32_t) * kGroupCntStride * plan->n_chunk_groups, A);
    w.group_ccnt = off;   off = align_up(off + sizeof(uint32_t) * kGroupCntStride * plan->n_chunk_groups, A);
    w.list_cnt = off;     off = align_up(off + sizeof(uint32_t) * kListShards * kListCntStride * size_t(L), A);
    w.list2_cnt = off;    off = align_up(off + sizeof(uint32_t) * L, A);
    w.feed = off;         off = align_up(off + sizeof(uint32_t) * 16 * 8 * 32, A);
    w.mask = off;         off = align_up(off + sizeof(uint32_t) * words, A);
    w.cmask = off;        off = align_up(off + sizeof(uint32_t) * words, A);
    w.zero_end = off;
    w.slot_cnt = off;     off = align_up(off + sizeof(uint32_t) * plan->n_tiles_all, A);
    // (the plan of a block grid never takes the candidate path and has no tile slots)
    w.slot_ent = off;     off = align_up(off + (plan->k_override.empty() ? sizeof(uint64_t) * size_t(plan->slot_entries) : 0), A);
    w.list_ent = off;     off = align_up(off + sizeof(uint64_t) * static_cast<size_t>(list_off), A);
    w.list2_ent = off;    off = align_up(off + sizeof(uint64_t) * 2048 * size_t(L), A);
    // the score map covers every layer: which layers are ranked on it depends on the keep ratios
    // (set_ratios must not change the workspace size), and any large layer may fall back to it in
    // any call, several of them in the same one
    w.nsi = off;          off = align_up(off + sizeof(float) * static_cast<size_t>(plan->total_elems), A);
    w.dyn = off;          off = align_up(off + 256 + sizeof(uint64_t) * kHistBins + sizeof(uint32_t) * 2 * size_t(L), A);
    w.apply_ranges = off; off = align_up(off + sizeof(uint32_t) * 2 * RSDGC_MAX_MSGS * static_cast<size_t>(plan->n_chunks), A);
    w.total = off;

    plan->table.assign(w.table_bytes, 0);
    std::memcpy(plan->table.data() + w.layers, plan->layers.data(), sizeof(LayerDev) * L);
    std::memcpy(plan->table.data() + w.tile_dir, plan->tile_dir.data(),
                sizeof(DirEntry) * plan->tile_dir.size());
    std::memcpy(plan->table.data() + w.chunk_dir, plan->chunk_dir.data(),
                sizeof(DirEntry) * plan->chunk_dir.size());
    std::memcpy(plan->table.data() + w.all_tile_dir, plan->all_tile_dir.data(),
                sizeof(DirEntry) * plan->all_tile_dir.size());
    if (!plan->large_dir.empty())
        std::memcpy(plan->table.data() + w.large_dir, plan->large_dir.data(),
                    sizeof(DirEntry) * plan->large_dir.size());
    if (!plan->samples.empty())
        std::memcpy(plan->table.data() + w.samples, plan->samples.data(),
                    sizeof(SampleEntry) * plan->samples.size());
    {
        uint32_t *cl = reinterpret_cast<uint32_t *>(plan->table.data() + w.chunk_layer);
        ChunkInfo *ci = reinterpret_cast<ChunkInfo *>(plan->table.data() + w.chunk_info);
        CountGroup *cg = reinterpret_cast<CountGroup *>(plan->table.data() + w.count_groups);
        static_assert(kChunkGroup % kCountChunks == 0, "a count item lies inside one chunk group");
        uint32_t first_group = 0, n_cg = 0;
        for (int l = 0; l < L; ++l) {
            const LayerDev &d = plan->layers[l];
            for (uint32_t c = 0; c < d.n_chunks; c += kCountChunks) {
                const uint32_t n = std::min<uint32_t>(kCountChunks, d.n_chunks - c);
                const uint64_t first_elem = static_cast<uint64_t>(c) * kChunk;
                const uint64_t end_elem = std::min<uint64_t>(first_elem + static_cast<uint64_t>(n) * kChunk, d.G);
                cg[n_cg++] =
                    CountGroup{(static_cast<uint64_t>(d.elem_off) + first_elem) >> 5, d.chunk_begin + c, n,
                               static_cast<uint32_t>((end_elem - first_elem + 31) / 32),
                               first_group + c / kChunkGroup};
            }
            for (uint32_t c = 0; c < d.n_chunks; ++c) {
                cl[d.chunk_begin + c] = static_cast<uint32_t>(l);
                const uint32_t start = c * kChunk;
                ci[d.chunk_begin + c] = ChunkInfo{static_cast<uint64_t>(d.elem_off) + start,
                                                  static_cast<uint64_t>(d.out_off), static_cast<uint32_t>(l),
                                                  start, std::min<uint32_t>(kChunk, d.G - start), d.cap,
                                                  first_group + c / kChunkGroup,
                                                  d.chunk_begin + c / kChunkGroup * kChunkGroup, first_group,
                                                  c + 1 == d.n_chunks ? 1u : 0u,
                                                  plan->n_chunks <= kInlineCountChunks ? uint32_t(kGroupCntStride) : 1u, 0u};
            }
            first_group += (d.n_chunks + kChunkGroup - 1) / kChunkGroup;
        }
    }
    if (!plan->cand_groups.empty())
        std::memcpy(plan->table.data() + w.cand_groups, plan->cand_groups.data(),
                    sizeof(GroupEntry) * plan->cand_groups.size());
    if (!plan->map_chunks.empty())
        std::memcpy(plan->table.data() + w.map_chunks, plan->map_chunks.data(),
                    sizeof(ChunkEntry) * plan->map_chunks.size());
    if (!plan->map_tiles.empty())
        std::memcpy(plan->table.data() + w.map_tiles, plan->map_tiles.data(),
                    sizeof(SampleEntry) * plan->map_tiles.size());
    ++plan->version;

    if (plan->blocks) {       // the block grids as a plan of their own: p = 1, the same k_l, full-map ranking
        if (!plan->inner) plan->inner = new rsdgc_plan_s;
        rsdgc_plan_s *in = plan->inner;
        in->n_layers = L;
        in->alpha = plan->alpha;
        in->shapes.resize(L);
        in->p.assign(L, 1);
        in->ratio.assign(L, 0.0);
        in->k_override.resize(L);
        in->allow_candidates = false;
        for (int l = 0; l < L; ++l) {
            const int64_t p = plan->p[l];
            in->shapes[l].rows = (plan->shapes[l].rows + p - 1) / p;
            in->shapes[l].cols = (plan->shapes[l].cols + p - 1) / p;
            in->k_override[l] = plan->layers[l].k;     // Eq. 11; never more than the number of blocks
        }
        build_tables(in);
    }
    return RSDGC_OK;
}

static bool ratio_ok(double r) { return r >= 0.0 && r <= 1.0; }  // false for NaN

}  // namespace rsdgc

using namespace rsdgc;

extern "C" {

static int make_plan(const rsdgc_shape_t *shapes, int32_t n_layers, int32_t p,
                     const int32_t *p_per_layer, double alpha, const double *keep_ratio,
                     bool blocks, rsdgc_plan_t **out_plan) {
    if (!shapes || !keep_ratio || !out_plan || n_layers < 1 || n_layers > 65536) return RSDGC_EINVAL;
    *out_plan = nullptr;
    if (!(alpha >= 0.0 && alpha <= 1.0)) return RSDGC_EINVAL;
    int64_t total = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int pl = p_per_layer ? p_per_layer[l] : p;
        if (pl < 1 || pl > RSDGC_MAX_P || pl % 2 == 0) return RSDGC_EINVAL;
        const int64_t R = shapes[l].rows, C = shapes[l].cols;
        if (R < 1 || C < 1 || R > 0x7fffffffLL || C > 0x7fffffffLL) return RSDGC_EINVAL;
        if (R > 0xffffffffLL / C) return RSDGC_EINVAL;            // G_l must fit uint32
        if (!ratio_ok(keep_ratio[l])) return RSDGC_EINVAL;
        total += R * C + kLayerAlign;
        if (total > (int64_t(1) << 34)) return RSDGC_EINVAL;         // 64 GiB per float32 arena
        // a kept block always sends p*p values: the layer's value segment, k_l * p^2 floats, is
        // counted in 32 bits like every other per-layer quantity
        if (blocks && keep_count(R * C, pl, keep_ratio[l]) * pl * pl > 0xffffffffLL) return RSDGC_EINVAL;
    }
    if ((total + kChunk - 1) / kChunk + n_layers > 0x7fffffffLL) return RSDGC_EINVAL;
    rsdgc_plan_s *plan = new (std::nothrow) rsdgc_plan_s;
    if (!plan) return RSDGC_ENOMEM;
    static std::atomic<uint64_t> next_serial{1};
    plan->serial = next_serial.fetch_add(1);
    try {
        plan->n_layers = n_layers;
        plan->alpha = alpha;
        plan->shapes.assign(shapes, shapes + n_layers);
        plan->p.resize(n_layers);
        for (int l = 0; l < n_layers; ++l) plan->p[l] = p_per_layer ? p_per_layer[l] : p;
        plan->ratio.assign(keep_ratio, keep_ratio + n_layers);
        plan->blocks = blocks;
        build_tables(plan);
    } catch (const std::bad_alloc &) {
        delete plan;
        return RSDGC_ENOMEM;
    }
    *out_plan = plan;
    return RSDGC_OK;
}

int rsdgc_plan(const rsdgc_shape_t *shapes, int32_t n_layers, int32_t p,
               const int32_t *p_per_layer, double alpha, const double *keep_ratio,
               rsdgc_plan_t **out_plan) {
    return make_plan(shapes, n_layers, p, p_per_layer, alpha, keep_ratio, false, out_plan);
}

int rsdgc_plan_blocks(const rsdgc_shape_t *shapes, int32_t n_layers, int32_t p,
                      const int32_t *p_per_layer, double alpha, const double *keep_ratio,
                      rsdgc_plan_t **out_plan) {
    return make_plan(shapes, n_layers, p, p_per_layer, alpha, keep_ratio, true, out_plan);
}

int rsdgc_plan_set_ratios(rsdgc_plan_t *plan, const double *keep_ratio) {
    if (!plan || !keep_ratio) return RSDGC_EINVAL;
    for (int l = 0; l < plan->n_layers; ++l) {
        if (!ratio_ok(keep_ratio[l])) return RSDGC_EINVAL;
        const int64_t G = plan->shapes[l].rows * plan->shapes[l].cols, pl = plan->p[l];
        if (plan->blocks && keep_count(G, static_cast<int>(pl), keep_ratio[l]) * pl * pl > 0xffffffffLL) return RSDGC_EINVAL;
    }
    try {
        plan->ratio.assign(keep_ratio, keep_ratio + plan->n_layers);
        build_tables(plan);
    } catch (const std::bad_alloc &) {
        return RSDGC_ENOMEM;
    }
    return RSDGC_OK;
}

int rsdgc_plan_set_path(rsdgc_plan_t *plan, int32_t path) {
    if (!plan || (path != RSDGC_PATH_AUTO && path != RSDGC_PATH_FULL_MAP)) return RSDGC_EINVAL;
    try {
        plan->allow_candidates = (path == RSDGC_PATH_AUTO);
        build_tables(plan);
    } catch (const std::bad_alloc &) {
        return RSDGC_ENOMEM;
    }
    return RSDGC_OK;
}

int rsdgc_plan_set_work_feed(rsdgc_plan_t *plan, int32_t mode) {
    if (!plan || mode < RSDGC_FEED_AUTO || mode > RSDGC_FEED_ON) return RSDGC_EINVAL;
    plan->work_feed = mode;
    if (plan->inner) plan->inner->work_feed = mode;
    return RSDGC_OK;
}

int rsdgc_plan_forget_workspace(rsdgc_plan_t *plan) {
    if (!plan) return RSDGC_EINVAL;
    plan->uploaded_ws = nullptr;       // the next call uploads the tables again
    if (plan->inner) plan->inner->uploaded_ws = nullptr;
    return RSDGC_OK;
}

void rsdgc_plan_destroy(rsdgc_plan_t *plan) {
    if (plan) {
        int32_t n = 0;
        double ms[RSDGC_N_STAGES];
        if (!plan->prof_events.empty()) rsdgc_profile_end(plan, ms, &n);   // releases the events
        delete plan;
    }
}

int32_t rsdgc_n_layers(const rsdgc_plan_t *plan) { return plan ? plan->n_layers : -1; }
int64_t rsdgc_total_elems(const rsdgc_plan_t *plan) { return plan ? plan->total_elems : -1; }

static bool layer_ok(const rsdgc_plan_t *plan, int32_t l) {
    return plan && l >= 0 && l < plan->n_layers;
}
int64_t rsdgc_layer_offset(const rsdgc_plan_t *plan, int32_t l) {
    return layer_ok(plan, l) ? plan->layers[l].elem_off : -1;
}
int64_t rsdgc_layer_elems(const rsdgc_plan_t *plan, int32_t l) {
    return layer_ok(plan, l) ? int64_t(plan->layers[l].G) : -1;
}
int64_t rsdgc_layer_k(const rsdgc_plan_t *plan, int32_t l) {
    return layer_ok(plan, l) ? int64_t(plan->layers[l].k) : -1;
}
int64_t rsdgc_out_offset(const rsdgc_plan_t *plan, int32_t l) {
    return layer_ok(plan, l) ? plan->layers[l].out_off : -1;
}
int64_t rsdgc_out_capacity(const rsdgc_plan_t *plan) { return plan ? plan->out_capacity : -1; }
int64_t rsdgc_centre_offset(const rsdgc_plan_t *plan, int32_t l) {
    return layer_ok(plan, l) ? plan->layers[l].centre_off : -1;
}
int64_t rsdgc_centre_capacity(const rsdgc_plan_t *plan) {
    return plan ? plan->centre_capacity : -1;
}
size_t rsdgc_workspace_bytes(const rsdgc_plan_t *plan) {
    if (!plan) return 0;
    // a block plan: its own tables, then the workspace of the plan that ranks the block grids
    // (both multiples of 256)
    if (plan->blocks) return plan->ws.table_bytes + plan->inner->ws.total;
    return plan->ws.total;
}

const char *rsdgc_strerror(int code) {
    switch (code) {
        case RSDGC_OK: return "ok";
        case RSDGC_EINVAL: return "invalid argument";
        case RSDGC_ENOMEM: return "host allocation failed";
        case RSDGC_EHIP: return "HIP call failed";
        case RSDGC_ETOOBIG: return "the plan's workspace exceeds the library's built-in one";
        default: return "unknown error code";
    }
}

}  // extern "C"
