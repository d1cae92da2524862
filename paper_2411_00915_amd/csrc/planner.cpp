// Host-side batch planner: segment table -> token/adapter maps, stable grouping
// by adapter, and the tile lists of the shrink and expand launches.
//
// Stands where ATMM consults its shape-keyed table for the tile configuration of
// the input at hand (paper section 4.3.1, adaptive tiling; section 4.3.2, the
// table built by profiling).  No HIP calls in this file: everything here runs,
// and is tested, without a GPU.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <queue>
#include <utility>
#include <vector>

#include "plan_internal.h"

namespace {
std::mutex g_tuning_mutex;                       // guards the process defaults and the shape table
lora_tuning g_lora_tuning = {
    /*shrink_waves*/ 8,
    /*shrink_tb2_min_rows*/ 64,
    /*shrink_max_jb*/ 4,
    /*expand_wave_bytes*/ 16384,
    /*expand_tb2_min_rows*/ 64,
    /*expand_tb4_min_rows*/ 1 << 30,
    /*tiled_min_tokens*/ 1,
    /*shrink_small_waves*/ 16,
    /*shrink_small_jb*/ 1,
    /*shrink_target_wgs*/ 768,
    /*fused_wait_us*/ 2001,
    /*fused_delay*/ 3,
    /*expand_wave_bytes_big*/ 131072,
    /*shrink_tb4_min_rows*/ 64,
    /*shrink_stream_min_tokens*/ 1024,
    /*shrink_stream_wgs*/ 512,
    /*expand_stream_stages*/ 16,
};

// The shape table the library ships with: written by the offline search (autotune.py) on MI355X.
const lora_tuning_entry kShippedTable[] = {
#include "tuning_table.inc"
};
constexpr int32_t kShippedCount = (int32_t)(sizeof(kShippedTable) / sizeof(kShippedTable[0]));
std::vector<lora_tuning_entry> g_table(kShippedTable, kShippedTable + kShippedCount);

int32_t rank_class(int32_t r)
{
    int32_t c = 8;
    while (c < r) c *= 2;
    return c;
}

void overlay(lora_tuning* t, const int32_t* values, int32_t count)
{
    int32_t* dst = reinterpret_cast<int32_t*>(t);
    for (int32_t i = 0; i < count && i < LORA_TUNING_COUNT; ++i)
        if (values[i] > 0) dst[i] = values[i];
}

// The tunables of one plan: defaults, then the table entry of the batch's shape class, then the descriptor's own.
void snapshot_tuning(lora_plan* p, const lora_batch_desc* d, int32_t active_tokens, int32_t max_rank, int32_t max_group)
{
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    p->tuning = g_lora_tuning;
    p->tuning_source = 0;
    // group class: 0 every adapter group below 64 tokens (decode-shaped); 2 groups of 512 tokens or more on average
    // (few long requests, e.g. image-sized prefill); 1 everything between
    const int32_t n_groups = (int32_t)p->group_adapter.size();
    const int32_t rc = rank_class(max_rank),
                  gc = max_group < 64 ? 0 : ((int64_t)active_tokens >= 512ll * std::max(n_groups, 1) ? 2 : 1);
    const lora_tuning_entry* best = nullptr;
    for (const lora_tuning_entry& e : g_table) {
        if (e.k != p->K || e.n != p->N || e.max_rank != rc || e.group_class != gc) continue;
        if (!best) { best = &e; continue; }
        const bool e_covers = e.tokens >= active_tokens, b_covers = best->tokens >= active_tokens;
        if (e_covers != b_covers ? e_covers : (e_covers ? e.tokens < best->tokens : e.tokens > best->tokens)) best = &e;
    }
    if (best && active_tokens > 0) {                             // (a row of zeros: the class keeps the defaults)
        bool any = false;
        for (int32_t i = 0; i < LORA_TUNING_COUNT; ++i) any = any || best->values[i] > 0;
        overlay(&p->tuning, best->values, LORA_TUNING_COUNT);
        if (any) p->tuning_source = 1;
    }
    if (d->tuning && d->tuning_count > 0) {
        bool any = false;
        for (int32_t i = 0; i < d->tuning_count && i < LORA_TUNING_COUNT; ++i) any = any || d->tuning[i] > 0;
        overlay(&p->tuning, d->tuning, d->tuning_count);
        if (any) p->tuning_source += 2;
    }
}
}  // namespace

extern "C" void lora_tuning_set(const int32_t* values, int32_t count)
{
    if (!values) return;
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    overlay(&g_lora_tuning, values, count);
}

extern "C" void lora_tuning_get(int32_t* values, int32_t count)
{
    if (!values) return;
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    const int32_t* src = reinterpret_cast<const int32_t*>(&g_lora_tuning);
    for (int32_t i = 0; i < count && i < LORA_TUNING_COUNT; ++i) values[i] = src[i];
}

extern "C" lora_status lora_tuning_table_set(const lora_tuning_entry* entries, int32_t count)
{
    if (count < 0 || (count > 0 && !entries)) return LORA_ERR_INVALID_ARG;
    for (int32_t i = 0; i < count; ++i)
        if (entries[i].tokens < 0 || entries[i].k < 1 || entries[i].n < 1 || entries[i].max_rank != rank_class(entries[i].max_rank) ||
            entries[i].max_rank > LORA_MAX_RANK || entries[i].group_class < 0 || entries[i].group_class > 2)
            return LORA_ERR_INVALID_ARG;
    try {
        std::vector<lora_tuning_entry> next = count ? std::vector<lora_tuning_entry>(entries, entries + count)
                                                    : std::vector<lora_tuning_entry>(kShippedTable, kShippedTable + kShippedCount);
        std::lock_guard<std::mutex> lock(g_tuning_mutex);
        g_table.swap(next);
    } catch (const std::bad_alloc&) {
        return LORA_ERR_NOMEM;
    }
    return LORA_OK;
}

extern "C" int32_t lora_tuning_table_get(lora_tuning_entry* entries, int32_t capacity)
{
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    if (entries)
        for (int32_t i = 0; i < capacity && i < (int32_t)g_table.size(); ++i) entries[i] = g_table[i];
    return (int32_t)g_table.size();
}

static bool validate(const lora_batch_desc* d)
{
    if (d->num_tokens < 0 || d->num_segments < 0 || d->num_adapters < 0) return false;
    if (d->k < 1 || d->n < 1) return false;
    if (d->dtype != LORA_F32 && d->dtype != LORA_BF16) return false;
    if (d->variant < LORA_VARIANT_AUTO || d->variant > LORA_VARIANT_TILED) return false;
    if (d->tuning_count < 0 || (d->tuning_count > 0 && !d->tuning)) return false;
    if (d->merged_adapter_plus1 < 0 || d->merged_adapter_plus1 > d->num_adapters) return false;
    if (!d->seg_indptr) return false;                       // even S = 0 has the single entry [0]
    if (d->num_segments > 0 && !d->seg_adapter) return false;
    if (d->num_adapters > 0 && (!d->adapter_rank || !d->adapter_scale)) return false;
    if (d->seg_indptr[0] != 0) return false;
    for (int32_t s = 0; s < d->num_segments; ++s) {
        if (d->seg_indptr[s + 1] < d->seg_indptr[s]) return false;
        const int32_t a = d->seg_adapter[s];
        if (a < -1 || a >= d->num_adapters) return false;
    }
    if (d->seg_indptr[d->num_segments] != d->num_tokens) return false;
    for (int32_t a = 0; a < d->num_adapters; ++a) {
        if (d->adapter_rank[a] < 0 || d->adapter_rank[a] > LORA_MAX_RANK) return false;
        if (!std::isfinite(d->adapter_scale[a])) return false;
    }
    return true;
}

static int32_t round_up(int32_t v, int32_t m) { return (v + m - 1) / m * m; }

// Tile lists of the tiled (MFMA) family.  A shrink tile is 16*TB tokens of one
// adapter times 16*JB of its rank indices over the whole K range (the
// workgroup's wavefronts split K).  An expand tile is 16*TB tokens times a range
// of output features that the workgroup's four wavefronts split evenly.
// shrink_only: tiles for the shrink alone (ranks the expand kernels cannot take), for the kernels that tile the rank
// axis in blocks of 16 rows -- no streaming, no single launch.
static void build_tiles(lora_plan* p, bool shrink_only = false)
{
    const lora_tuning& tu = p->tuning;
    p->shrink_max_blocks = 1;
    p->shrink_small = true;
    p->expand_small = true;
    const int G = (int)p->group_adapter.size();
    // Prefill-sized batches (ranks up to 128) take the streaming shrink; its tiles hold 128 tokens, or 64
    // when 128 would leave the launch with few workgroups even after the K split.
    // Smaller batches take it too when they cannot run as the single decode launch (a group too long or a rank
    // too high for the small tiles) and have a group of at least 64 tokens or 128 tokens in all: measured, the
    // streaming kernels then need 18-33 us where the 32- and 64-token tiles of the other family need 24-52.
    int32_t max_rank = 0, max_group = 0;
    bool small_tiles_only = true;
    for (int g = 0; g < G; ++g) {
        const int32_t r = p->rank[p->group_adapter[g]], m = p->group_offset[g + 1] - p->group_offset[g];
        max_rank = std::max(max_rank, r);
        max_group = std::max(max_group, m);
        if (m >= tu.shrink_tb2_min_rows || m >= tu.shrink_tb4_min_rows || m >= tu.expand_tb2_min_rows ||
            m >= tu.expand_tb4_min_rows || r > 64)
            small_tiles_only = false;
    }
    const int64_t active = (int64_t)p->perm.size();
    p->shrink_stream = max_rank <= 128 && p->K >= 1024 &&
                       (active >= tu.shrink_stream_min_tokens ||
                        (tu.shrink_stream_min_tokens < (1 << 30) && !small_tiles_only && (max_group >= 64 || active >= 128)));
    if (shrink_only) p->shrink_stream = false;
    p->expand_stream = p->shrink_stream && p->N >= 64;
    p->expand_stream_ks = 1;
    p->expand_stream_lds = 0;
    int32_t stream_tokens = 128;
    if (p->shrink_stream) {
        int64_t n128 = 0;
        for (int g = 0; g < G; ++g) n128 += (p->group_offset[g + 1] - p->group_offset[g] + 127) / 128;
        if (n128 * 4 < tu.shrink_stream_wgs) stream_tokens = 64;
    }
    // streaming expand: feature range per workgroup, in stages; halved while the launch would have
    // fewer than two workgroups per CU (but at least 4 stages: the start-up of a tile has to pay off)
    int32_t expand_stages = std::max(1, tu.expand_stream_stages);
    // (its token tiles: 128 tokens -- every token tile of an adapter fetches Bt_a again, and the launch has feature
    // ranges to make workgroups of -- unless that leaves fewer than two rounds of tiles)
    int32_t expand_tokens = 128;
    if (p->expand_stream) {
        auto token_tiles = [&](int32_t per) {
            int64_t n = 0;
            for (int g = 0; g < G; ++g) n += (p->group_offset[g + 1] - p->group_offset[g] + per - 1) / per;
            return n;
        };
        if (token_tiles(128) * ((p->N + expand_stages * 64 - 1) / (expand_stages * 64)) < 512) expand_tokens = stream_tokens;
        const int64_t n_tt = token_tiles(expand_tokens);
        while (expand_stages > 4 && n_tt * ((p->N + expand_stages * 64 - 1) / (expand_stages * 64)) < 512) expand_stages /= 2;
    }
    for (int g = 0; g < G; ++g) {
        const int32_t a = p->group_adapter[g];
        const int32_t r = p->rank[a];
        const int32_t lo = p->group_offset[g], hi = p->group_offset[g + 1];
        const int32_t m = hi - lo;

        // ---- shrink, prefill-sized batches: streaming tiles of up to 128 (or 64) tokens over all rank rows
        if (p->shrink_stream) {
            const int jblocks = (r + 15) / 16;
            const int jbk = jblocks <= 1 ? 1 : (jblocks <= 2 ? 2 : (jblocks <= 4 ? 4 : 8));
            for (int32_t row = lo; row < hi; row += stream_tokens) {
                lora_tile t{};
                t.adapter = a; t.row0 = row; t.nrows = std::min<int32_t>(stream_tokens, hi - row);
                t.c0 = 0; t.cn = r;
                const int nblk = (t.nrows + 15) / 16;
                t.shape = lora_shape_code(nblk > 4 ? 8 : (nblk > 2 ? 4 : 2), jbk) | ((g & 0xffff) << 16);
                t.reserved0 = r;
                std::memcpy(&t.reserved1, &p->scale[a], sizeof(float));
                p->shrink_max_blocks = std::max(p->shrink_max_blocks, jbk);
                p->shrink_small = false;
                p->shrink_tiles.push_back(t);
            }
        } else
        // ---- shrink: groups with many tokens take 32- or 64-token tiles over up to 64
        // rank rows (x is the big stream, and At is re-read once per tile); groups with few tokens
        // take 16-token tiles over 16 (or 32) rank rows so that the launch has
        // many workgroups (A is the big stream, each byte is read once anyway)
        {
            const int jblocks = (r + 15) / 16;
            const bool large = m >= tu.shrink_tb2_min_rows;
            const int tb = m >= tu.shrink_tb4_min_rows ? 4 : (large ? 2 : 1);
            const int jb = std::min(jblocks, large ? std::max(1, std::min(tu.shrink_max_jb, 4))
                                                   : std::max(1, std::min(tu.shrink_small_jb, 2)));
            for (int32_t row = lo; row < hi; row += 16 * tb) {
                const int32_t nrows = std::min<int32_t>(16 * tb, hi - row);
                for (int32_t j0 = 0; j0 < r; j0 += 16 * jb) {
                    lora_tile t{};
                    t.adapter = a; t.row0 = row; t.nrows = nrows;
                    t.c0 = j0; t.cn = std::min<int32_t>(16 * jb, r - j0);
                    const int tbk = nrows > 32 ? 4 : (nrows > 16 ? 2 : 1), jbk = (t.cn + 15) / 16;
                    t.shape = lora_shape_code(tbk, jbk) | ((g & 0xffff) << 16);   // bits 16..31: adapter group
                    t.reserved0 = r;
                    std::memcpy(&t.reserved1, &p->scale[a], sizeof(float));   // s_a travels with the tile
                    p->shrink_max_blocks = std::max(p->shrink_max_blocks, tbk * jbk);
                    if (tbk != 1 || jbk > 2) p->shrink_small = false;
                    p->shrink_tiles.push_back(t);
                }
            }
        }
        // ---- expand, prefill-sized batches: streaming tiles, the same token ranges as the streaming shrink;
        // with fewer than 8 token blocks the wavefronts also spread over FW 64-feature chunks per stage
        // (as far as the slab of Bt rows, 64 FW x 32 KS ranks, stays within 32 KB)
        if (shrink_only) {
            p->expand_small = false;
        } else if (p->expand_stream) {
            const int ks = r <= 32 ? 1 : (r <= 64 ? 2 : 4);
            const int fw_max = 8 / ks;
            for (int32_t row = lo; row < hi; row += expand_tokens) {
                const int32_t nrows = std::min<int32_t>(expand_tokens, hi - row);
                const int nblk = (nrows + 15) / 16;
                const int nb = nblk > 4 ? 8 : (nblk > 2 ? 4 : (nblk > 1 ? 2 : 1));
                const int fw = std::min(8 / nb, fw_max);
                const int32_t n_tile = expand_stages * 64 * fw;
                for (int32_t n0 = 0; n0 < p->N; n0 += n_tile) {
                    lora_tile t{};
                    t.adapter = a; t.row0 = row; t.nrows = nrows;
                    t.c0 = n0; t.cn = std::min<int32_t>(n_tile, p->N - n0);
                    t.shape = lora_shape_code(nb, fw);
                    t.reserved0 = r;
                    t.reserved1 = g;
                    p->expand_small = false;
                    p->expand_stream_ks = std::max(p->expand_stream_ks, ks);
                    p->expand_stream_lds = std::max(p->expand_stream_lds, fw * ks * 4 * 2048 + 8 * 16 * 68 * 4);
                    p->expand_tiles.push_back(t);
                }
            }
        } else
        // ---- expand ----
        {
            int tb = 1;
            if (m >= tu.expand_tb4_min_rows && r <= 64) tb = 4;
            else if (m >= tu.expand_tb2_min_rows) tb = 2;
            // output features per wavefront: a multiple of 64, sized so that the
            // wavefront streams about expand_wave_bytes of Bt and y
            const int64_t per_n = 2 * (int64_t)r + 4 * 16 * (int64_t)tb;
            // (long ranges for big groups and big batches: the wavefront loops with the next chunk in flight;
            // short ranges for decode-sized batches, where the launch is one round of memory latency)
            const int64_t wave_bytes = (tb > 1 || p->perm.size() >= 1024) ? tu.expand_wave_bytes_big : tu.expand_wave_bytes;
            int32_t nw = (int32_t)std::max<int64_t>(64, (wave_bytes / per_n) / 64 * 64);
            const int32_t n_tile = 4 * nw;
            for (int32_t row = lo; row < hi; row += 16 * tb) {
                const int32_t nrows = std::min<int32_t>(16 * tb, hi - row);
                for (int32_t n0 = 0; n0 < p->N; n0 += n_tile) {
                    lora_tile t{};
                    t.adapter = a; t.row0 = row; t.nrows = nrows;
                    t.c0 = n0; t.cn = std::min<int32_t>(n_tile, p->N - n0);
                    const int tbk = (nrows + 15) / 16;
                    t.shape = lora_shape_code(tbk == 3 ? 4 : tbk, 0);
                    t.reserved0 = r;
                    t.reserved1 = g;                                             // adapter group
                    if (tbk != 1 || r > 64) p->expand_small = false;
                    p->expand_tiles.push_back(t);
                }
            }
        }
    }
    // wavefronts per shrink workgroup: they split K in steps of 32; the LDS
    // reduction buffer (1 KB per wavefront and 16x16 block) stays within 64 KB
    const int steps = (p->K + 31) / 32;
    // Small build: a workgroup's bandwidth is bounded (one CU), so a launch with
    // fewer workgroups than CUs leaves HBM idle.  Split K over P workgroups per
    // tile (P in 1, 2, 4); each part writes its own slice of v and every consumer
    // of v adds the parts in order, so there are no atomics and no zeroing.
    p->v_parts = 1;
    {
        int P = 1;
        // (the streaming shrink has 8 wavefronts per workgroup and long tiles: half as many workgroups do)
        const int64_t target = p->shrink_stream ? std::max(1, tu.shrink_stream_wgs / 2) : tu.shrink_target_wgs;
        while (P < 4 && (int64_t)p->shrink_tiles.size() * P < target && steps / (2 * P) >= 8) P *= 2;
        p->v_parts = P;
    }
    {
        std::vector<lora_tile> split;
        split.reserve(p->shrink_tiles.size() * p->v_parts);
        for (const lora_tile& t : p->shrink_tiles)
            for (int q = 0; q < p->v_parts; ++q) {
                lora_tile u = t;
                u.shape |= (q << 8) | (p->v_parts << 12);
                split.push_back(u);
            }
        p->shrink_tiles.swap(split);
    }
    if (p->shrink_stream)
        p->shrink_waves = 8;
    else if (p->shrink_small)
        p->shrink_waves = std::max(1, std::min({tu.shrink_small_waves / p->v_parts, 16, steps / p->v_parts}));
    else
        p->shrink_waves = std::max(1, std::min({tu.shrink_waves, 8, 64 / p->shrink_max_blocks, steps / p->v_parts}));
    // Single-launch decode kernel: an expand tile carries (bits 8..31 of its shape)
    // the numbers of shrink tiles
    // (bits 8..19 of its shape) and of expand tiles (bits 20..31) of its adapter group.
    p->fused_ok = p->shrink_small && p->expand_small && G <= 4096;
    p->fused_wait_us = tu.fused_wait_us - 1;
    p->fused_delay = std::max(0, std::min(tu.fused_delay - 1, 64));
    // The single launch holds 5 workgroups per compute unit at a time (1280 on the 256 units of an MI355X).  A few
    // workgroups beyond that start only when earlier ones end, microseconds into a launch that lasts little longer,
    // and then end it late.  While the launch is over that number by less than a tenth, the expand tiles of the
    // adapter groups with the least bytes per tile (lowest rank first, then fewest tokens) are joined in pairs
    // along the features -- they are the cheapest to double.
    constexpr size_t kResidentWorkgroups = 1280;
    if (p->fused_ok && p->shrink_tiles.size() + p->expand_tiles.size() > kResidentWorkgroups &&
        (p->shrink_tiles.size() + p->expand_tiles.size()) * 10 <= kResidentWorkgroups * 11) {
        std::vector<int> groups((size_t)G);
        for (int g = 0; g < G; ++g) groups[(size_t)g] = g;
        std::stable_sort(groups.begin(), groups.end(), [&](int a, int b) {
            const int32_t ra = p->rank[p->group_adapter[a]], rb = p->rank[p->group_adapter[b]];
            if (ra != rb) return ra < rb;
            return p->group_offset[a + 1] - p->group_offset[a] < p->group_offset[b + 1] - p->group_offset[b];
        });
        std::vector<char> join((size_t)G, 0);
        size_t total = p->shrink_tiles.size() + p->expand_tiles.size();
        std::vector<size_t> tiles_of((size_t)G, 0);
        for (const lora_tile& t : p->expand_tiles) tiles_of[(size_t)t.reserved1] += 1;
        for (int g : groups) {
            if (total <= kResidentWorkgroups) break;
            join[(size_t)g] = 1;
            total -= tiles_of[(size_t)g] / 2;
        }
        std::vector<lora_tile> joined;
        joined.reserve(p->expand_tiles.size());
        for (size_t i = 0; i < p->expand_tiles.size(); ++i) {
            lora_tile t = p->expand_tiles[i];
            if (join[(size_t)t.reserved1] && i + 1 < p->expand_tiles.size()) {
                const lora_tile& n = p->expand_tiles[i + 1];
                if (n.reserved1 == t.reserved1 && n.row0 == t.row0 && n.c0 == t.c0 + t.cn) {
                    t.cn += n.cn;
                    ++i;
                }
            }
            joined.push_back(t);
        }
        p->expand_tiles.swap(joined);
    }
    if (p->fused_ok) {
        std::vector<int32_t> need((size_t)G, 0), ncons((size_t)G, 0);
        for (const lora_tile& t : p->shrink_tiles) need[(size_t)((uint32_t)t.shape >> 16)] += 1;
        for (const lora_tile& t : p->expand_tiles) ncons[(size_t)t.reserved1] += 1;
        for (int g = 0; g < G; ++g)
            if (need[g] > 4095 || ncons[g] > 4095) p->fused_ok = false;
        if (p->fused_ok)
            for (lora_tile& t : p->expand_tiles)
                t.shape |= (need[(size_t)t.reserved1] << 8) | (int32_t)((uint32_t)ncons[(size_t)t.reserved1] << 20);
    }
    // Heaviest tiles first so the tail of the launch is made of light ones;
    // stable, so equal descriptors give identical lists.
    auto weight = [&](const lora_tile& t) { return (int64_t)((t.nrows + 15) / 16) * t.cn; };
    std::stable_sort(p->shrink_tiles.begin(), p->shrink_tiles.end(),
                     [&](const lora_tile& x, const lora_tile& y) { return weight(x) > weight(y); });
    // (the streaming expand's tiles differ in size by up to 8x: the same for them)
    if (p->expand_stream) {
        std::stable_sort(p->expand_tiles.begin(), p->expand_tiles.end(),
                         [&](const lora_tile& x, const lora_tile& y) { return weight(x) > weight(y); });
        // Workgroups start in index order, one per compute unit at a time.  With equal tiles a launch of 3.3
        // rounds of them takes 4: so towards the end of the list the tiles shrink (guided self-scheduling): a
        // tile heavier than its share of what is left -- the remaining work over the number of compute units --
        // is cut along the features into 2 or 4, as long as a piece keeps at least 4 stages (the start-up of a
        // tile has to pay off).
        constexpr int64_t kComputeUnits = 256;
        int64_t remaining = 0;
        for (const lora_tile& t : p->expand_tiles) remaining += weight(t);
        std::vector<lora_tile> cut;
        cut.reserve(p->expand_tiles.size() + 4 * (size_t)kComputeUnits);
        for (const lora_tile& t : p->expand_tiles) {
            const int64_t w = weight(t);
            const int32_t stage = 64 * lora_shape_jb(t.shape);           // features per stage (64 FW)
            const int32_t stages = (t.cn + stage - 1) / stage;
            int32_t pieces = 1;
            while (pieces < 4 && w / pieces > std::max<int64_t>(remaining / kComputeUnits, 1) && stages / (pieces * 2) >= 4)
                pieces *= 2;
            const int32_t per = (stages + pieces - 1) / pieces * stage;
            for (int32_t c = 0; c < t.cn; c += per) {
                lora_tile q = t;
                q.c0 = t.c0 + c;
                q.cn = std::min(per, t.cn - c);
                cut.push_back(q);
            }
            remaining -= w;
        }
        // Taken only if it pays: finish time of both lists when every compute unit takes the next tile as soon as
        // it is free, a tile costing its weight plus a start-up of about two stages.
        auto finish = [&](const std::vector<lora_tile>& tiles) {
            std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> free_at;
            for (int64_t c = 0; c < kComputeUnits; ++c) free_at.push(0);
            int64_t last = 0;
            for (const lora_tile& t : tiles) {
                const int64_t at = free_at.top() + weight(t) + (int64_t)((t.nrows + 15) / 16) * 2 * 64 * lora_shape_jb(t.shape);
                free_at.pop();
                free_at.push(at);
                last = std::max(last, at);
            }
            return last;
        };
        if (finish(cut) * 100 < finish(p->expand_tiles) * 97) p->expand_tiles.swap(cut);
    }
    // Single-launch decode kernel: the 16 tokens of every tile, in tile order and padded with the tile's
    // first token, so that a workgroup can fetch them by its index alone, at the same time as its
    // tile descriptor instead of after it
    p->shrink_rows.clear();
    p->expand_rows.clear();
    if (p->fused_ok) {
        auto rows_of = [&](const std::vector<lora_tile>& tiles, std::vector<int32_t>& rows) {
            rows.resize(tiles.size() * 16);
            for (size_t i = 0; i < tiles.size(); ++i)
                for (int m = 0; m < 16; ++m)
                    rows[i * 16 + m] = p->perm[(size_t)tiles[i].row0 + (m < tiles[i].nrows ? m : 0)];
        };
        rows_of(p->shrink_tiles, p->shrink_rows);
        rows_of(p->expand_tiles, p->expand_rows);
    }
}

// Tables of the fused GEMM: it walks the tokens in adapter-sorted order, so a tile of rows holds few
// adapters, and folds each adapter's delta in (v_hi, v_lo against Bt_a; the register-staged kernels as extra
// k-stages from the lists below, the ring kernel per wavefront from the row keys).  The full
// blocks of 256 sorted rows are then put heaviest first (most adapter stages): workgroups start in
// index order, so the long tiles run early and the short ones fill the tail of the launch.
// Mixture mode: the removal of the merged adapter concerns every token of `unmerge`'s single adapter group; a tile
// that holds such a token gets the merged adapter's stages once more, marked, after its own.  Tokens without adapter
// that need the removal sort before the merged adapter's tokens, so that tiles of the latter keep no stage at all.
static void build_gemm_tables(lora_plan* p)
{
    const lora_plan* u = p->unmerge;
    p->row_key.resize((size_t)p->T);
    for (int32_t t = 0; t < p->T; ++t) {
        const int32_t a = p->token_adapter[t];
        p->row_key[t] = (a < 0 ? LORA_UNMERGE_BIT - 1 : a) | (u && u->token_adapter[t] >= 0 ? LORA_UNMERGE_BIT : 0);
    }
    std::vector<int32_t> sorted = p->perm;
    sorted.reserve((size_t)p->T);
    for (int pass = 0; pass < 2; ++pass)
        for (int32_t t = 0; t < p->T; ++t)
            if (p->token_adapter[t] < 0 && ((p->row_key[t] & LORA_UNMERGE_BIT) != 0) == (pass == 0)) sorted.push_back(t);

    // adapter stages of the rows [p0, p1) of `rows`: one per `cols` columns of [v_hi | v_lo] (2 r columns) and
    // adapter; the rows of one adapter are adjacent
    auto stages_of = [&](const std::vector<int32_t>& rows, int32_t p0, int32_t p1, int32_t cols, std::vector<int32_t>* lst) {
        int32_t n = 0, last = -1;
        bool removal = false;
        for (int32_t q = p0; q < p1; ++q) {
            removal = removal || (p->row_key[rows[q]] & LORA_UNMERGE_BIT);
            const int32_t a = p->token_adapter[rows[q]];
            if (a < 0 || a == last) continue;
            last = a;
            for (int32_t jb = 0; jb * cols < 2 * p->rank[a]; ++jb, ++n)
                if (lst) lst->push_back(a | (jb << 24));
        }
        if (removal)
            for (int32_t jb = 0; jb * cols < 2 * p->rank[p->merged]; ++jb, ++n)
                if (lst) lst->push_back(p->merged | LORA_UNMERGE_BIT | (jb << 24));
        return n;
    };

    const int32_t full = p->T / 256;
    std::vector<int32_t> weight((size_t)full), blocks((size_t)full);
    for (int32_t b = 0; b < full; ++b) {
        weight[b] = stages_of(sorted, b * 256, b * 256 + 256, 64, nullptr);
        blocks[b] = b;
    }
    std::stable_sort(blocks.begin(), blocks.end(), [&](int32_t x, int32_t y) { return weight[x] > weight[y]; });
    p->order.resize((size_t)p->T);
    for (int32_t b = 0; b < full; ++b)
        std::copy(sorted.begin() + (size_t)blocks[b] * 256, sorted.begin() + (size_t)blocks[b] * 256 + 256,
                  p->order.begin() + (size_t)b * 256);
    std::copy(sorted.begin() + (size_t)full * 256, sorted.end(), p->order.begin() + (size_t)full * 256);

    for (int h = 0; h < 2; ++h) {
        const int32_t rows = h == 0 ? 128 : 256, cols = 64;
        std::vector<int32_t>& ptr = h == 0 ? p->extra_ptr128 : p->extra_ptr256;
        std::vector<int32_t>& lst = h == 0 ? p->extra128 : p->extra256;
        const int32_t tiles = (p->T + rows - 1) / rows;
        ptr.assign(1, 0);
        lst.clear();
        for (int32_t tile = 0; tile < tiles; ++tile) {
            stages_of(p->order, tile * rows, std::min(tile * rows + rows, p->T), cols, &lst);
            ptr.push_back((int32_t)lst.size());
        }
    }
}

// One plan over the descriptor's segments as they stand; `unmerge` (may be null) is the removal's plan of a batch
// in mixture mode, which the new plan takes over.
static lora_status create_plain(const lora_batch_desc* d, int32_t merged, lora_plan* unmerge, lora_plan** out)
{
    lora_plan* p = new (std::nothrow) lora_plan();
    if (!p) {
        lora_plan_destroy(unmerge);
        return LORA_ERR_NOMEM;
    }
    p->merged = unmerge ? merged : -1;
    p->unmerge = unmerge;
    try {
        p->T = d->num_tokens; p->S = d->num_segments; p->n_a = d->num_adapters;
        p->K = d->k; p->N = d->n; p->dtype = d->dtype; p->variant_req = d->variant;
        p->rank.assign(d->adapter_rank, d->adapter_rank + p->n_a);
        p->scale.assign(d->adapter_scale, d->adapter_scale + p->n_a);

        // adapter of every token; adapters of rank 0 count as "none"
        p->token_adapter.assign((size_t)p->T, -1);
        std::vector<int32_t> count((size_t)p->n_a + 1, 0);
        for (int32_t s = 0; s < p->S; ++s) {
            int32_t a = d->seg_adapter[s];
            if (a >= 0 && p->rank[a] == 0) a = -1;
            for (int32_t t = d->seg_indptr[s]; t < d->seg_indptr[s + 1]; ++t) p->token_adapter[t] = a;
            if (a >= 0) count[a] += d->seg_indptr[s + 1] - d->seg_indptr[s];
        }
        // counting sort by adapter id = stable grouping
        std::vector<int32_t> start((size_t)p->n_a + 1, 0);
        int32_t max_rank = 0;
        bool ranks_mult8 = true;
        p->group_offset.push_back(0);
        for (int32_t a = 0; a < p->n_a; ++a) {
            start[a + 1] = start[a] + count[a];
            if (count[a] > 0) {
                p->group_adapter.push_back(a);
                p->group_offset.push_back(start[a + 1]);
                max_rank = std::max(max_rank, p->rank[a]);
                if (p->rank[a] % 8) ranks_mult8 = false;
            }
        }
        p->perm.resize((size_t)start[p->n_a]);
        std::vector<int32_t> cursor(start.begin(), start.end() - 1);
        for (int32_t t = 0; t < p->T; ++t) {
            const int32_t a = p->token_adapter[t];
            if (a >= 0) p->perm[cursor[a]++] = t;
        }
        int32_t table_max = 0;
        for (int32_t a = 0; a < p->n_a; ++a) table_max = std::max(table_max, p->rank[a]);
        p->R = std::max(8, round_up(table_max, 8));

        int32_t max_group = 0;
        for (size_t g = 0; g + 1 < p->group_offset.size(); ++g)
            max_group = std::max(max_group, p->group_offset[g + 1] - p->group_offset[g]);
        snapshot_tuning(p, d, (int32_t)p->perm.size(), max_rank, max_group);

        // the tiled kernels take bf16, 16-byte rows (K and ranks multiples of 8), ranks <= 128
        p->tiled_layout_ok = (p->dtype == LORA_BF16) && (p->K % 8 == 0) && ranks_mult8 && max_rank <= 128;
        const int32_t n_active = (int32_t)p->perm.size();
        if (p->variant_req == LORA_VARIANT_GENERAL || !p->tiled_layout_ok)
            p->family = LORA_VARIANT_GENERAL;
        else if (p->variant_req == LORA_VARIANT_TILED)
            p->family = LORA_VARIANT_TILED;
        else
            p->family = (n_active >= p->tuning.tiled_min_tokens) ? LORA_VARIANT_TILED : LORA_VARIANT_GENERAL;
        if (p->family == LORA_VARIANT_TILED) build_tiles(p);
        // Ranks that only the expand kernels cannot take (not multiples of 8: rows of Bt_a would not be 16-byte
        // aligned; above 128): the shrink still runs on the MFMA kernels, which tile the rank axis in blocks of 16
        // rows of At_a and mask what they store.  That is also the path of task heads, whose widths are arbitrary.
        p->shrink_tiled_only = false;
        if (p->family == LORA_VARIANT_GENERAL && !p->tiled_layout_ok && p->variant_req != LORA_VARIANT_GENERAL &&
            p->dtype == LORA_BF16 && p->K % 8 == 0 && max_rank <= LORA_MAX_RANK &&
            (p->variant_req == LORA_VARIANT_TILED || n_active >= p->tuning.tiled_min_tokens)) {
            build_tiles(p, true);
            p->shrink_tiled_only = !p->shrink_tiles.empty();
        }
        // (in mixture mode the removal's v must have the layout the GEMM's stages read, too)
        if (p->tiled_layout_ok && p->n_a < LORA_UNMERGE_BIT && (!unmerge || unmerge->tiled_layout_ok)) build_gemm_tables(p);
    } catch (const std::bad_alloc&) {
        lora_plan_destroy(p);
        return LORA_ERR_NOMEM;
    }
    *out = p;
    return LORA_OK;
}

extern "C" lora_status lora_plan_create(const lora_batch_desc* d, lora_plan** out)
{
    if (!d || !out) return LORA_ERR_INVALID_ARG;
    *out = nullptr;
    if (!validate(d)) return LORA_ERR_INVALID_ARG;
    const int32_t m = d->merged_adapter_plus1 - 1;
    if (m < 0 || d->adapter_rank[m] == 0) return create_plain(d, -1, nullptr, out);

    // Mixture mode (section 4.4.1) as two batches over the same tokens: the removal of the merged adapter
    // (every segment that is not m's uses m, scale negated) and the tokens' own branches (m's segments use none).
    lora_plan* removal = nullptr;
    try {
        std::vector<int32_t> seg((size_t)d->num_segments);
        std::vector<float> scale(d->adapter_scale, d->adapter_scale + d->num_adapters);
        scale[m] = -scale[m];
        for (int32_t s = 0; s < d->num_segments; ++s) seg[s] = d->seg_adapter[s] == m ? -1 : m;
        lora_batch_desc dr = *d;
        dr.seg_adapter = seg.data();
        dr.adapter_scale = scale.data();
        dr.merged_adapter_plus1 = 0;
        lora_status st = create_plain(&dr, -1, nullptr, &removal);
        if (st != LORA_OK) return st;
        for (int32_t s = 0; s < d->num_segments; ++s) seg[s] = d->seg_adapter[s] == m ? -1 : d->seg_adapter[s];
        lora_batch_desc own = *d;
        own.seg_adapter = seg.data();
        own.merged_adapter_plus1 = 0;
        return create_plain(&own, m, removal, out);
    } catch (const std::bad_alloc&) {
        lora_plan_destroy(removal);
        return LORA_ERR_NOMEM;
    }
}

void (*lora_plan_device_release)(lora_plan*) = nullptr;

extern "C" void lora_plan_destroy(lora_plan* p)
{
    if (!p) return;
    if (p->d_buf && lora_plan_device_release) lora_plan_device_release(p);
    lora_plan_destroy(p->unmerge);
    delete p;
}

extern "C" lora_status lora_plan_query(const lora_plan* p, int32_t* v_row_stride, size_t* v_bytes,
                                       size_t* fused_workspace_bytes)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    size_t vb = lora_own_v_bytes(p);
    size_t split = ((size_t)p->T * 2 * p->R * 2 + 255) / 256 * 256;
    if (p->unmerge) {
        vb = lora_unmerge_v_offset(p) + lora_own_v_bytes(p->unmerge);
        split += ((size_t)p->T * 2 * p->unmerge->R * 2 + 255) / 256 * 256;
    }
    if (v_row_stride) *v_row_stride = p->R;
    if (v_bytes) *v_bytes = vb;
    // workspace of the fused call: v (all parts; in mixture mode the removal's share behind it), then the bf16
    // split [T][2][R] of each
    if (fused_workspace_bytes) *fused_workspace_bytes = (vb + 255) / 256 * 256 + split;
    return LORA_OK;
}

extern "C" lora_status lora_plan_export(const lora_plan* p, lora_plan_view* v)
{
    if (!p || !v) return LORA_ERR_INVALID_ARG;
    v->num_tokens = p->T;
    v->num_active = (int32_t)p->perm.size();
    v->num_groups = (int32_t)p->group_adapter.size();
    v->v_row_stride = p->R;
    v->kernel_family = p->family;
    v->shrink_kernel_family = (p->family == LORA_VARIANT_TILED || p->shrink_tiled_only) ? LORA_VARIANT_TILED : LORA_VARIANT_GENERAL;
    v->shrink_waves = p->shrink_waves;
    v->v_parts = p->v_parts;
    v->tuning_source = p->tuning_source;
    std::memcpy(v->tuning, &p->tuning, sizeof(p->tuning));
    v->token_adapter = p->token_adapter.data();
    v->perm = p->perm.data();
    v->group_adapter = p->group_adapter.data();
    v->group_offset = p->group_offset.data();
    v->shrink_tiles = p->shrink_tiles.data();
    v->num_shrink_tiles = (int32_t)p->shrink_tiles.size();
    v->expand_tiles = p->expand_tiles.data();
    v->num_expand_tiles = (int32_t)p->expand_tiles.size();
    const bool gemm_tables = !p->extra_ptr256.empty() && (int32_t)p->order.size() == p->T;
    v->num_gemm_rows = gemm_tables ? p->T : 0;
    v->num_gemm_tiles = gemm_tables ? (int32_t)p->extra_ptr256.size() - 1 : 0;
    v->gemm_order = gemm_tables ? p->order.data() : nullptr;
    v->gemm_stage_offset = gemm_tables ? p->extra_ptr256.data() : nullptr;
    v->gemm_stage = gemm_tables ? p->extra256.data() : nullptr;
    const lora_plan* u = p->unmerge;
    v->merged_adapter = p->merged;
    v->num_unmerge = u ? (int32_t)u->perm.size() : 0;
    v->unmerge_v_row_stride = u ? u->R : 0;
    v->unmerge_v_parts = u ? u->v_parts : 0;
    v->unmerge_v_offset = u ? lora_unmerge_v_offset(p) : 0;
    v->unmerge_perm = u ? u->perm.data() : nullptr;
    v->unmerge_shrink_tiles = u ? u->shrink_tiles.data() : nullptr;
    v->num_unmerge_shrink_tiles = u ? (int32_t)u->shrink_tiles.size() : 0;
    v->unmerge_expand_tiles = u ? u->expand_tiles.data() : nullptr;
    v->num_unmerge_expand_tiles = u ? (int32_t)u->expand_tiles.size() : 0;
    return LORA_OK;
}

extern "C" const char* lora_status_str(lora_status s)
{
    switch (s) {
        case LORA_OK: return "ok";
        case LORA_ERR_INVALID_ARG: return "invalid argument";
        case LORA_ERR_UNSUPPORTED: return "unsupported";
        case LORA_ERR_NOMEM: return "out of memory";
        case LORA_ERR_WORKSPACE: return "workspace too small or misaligned";
        case LORA_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}
