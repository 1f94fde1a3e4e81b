// Host side of mf_load_blocks: cut the rating matrix into a grid of blocks (Section 3.1 of the
// paper: blocks that share neither a row strip nor a column strip are independent), order the
// ratings block by block, and derive the per-wavefront work lists of the two epoch modes.
//
// Method: strip lookup tables -> block id per rating -> stable parallel counting sort by block
// -> per-block sort by (row, column, original position) -> gather into packed arrays.
#include "mf_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <thread>

#include "../../include/mf_sgd.h"

namespace mf {
namespace {

int host_threads()
{
    int t = (int)std::thread::hardware_concurrency();
    if (const char* e = std::getenv("MF_HOST_THREADS")) t = std::atoi(e);
    return std::max(1, std::min(t, 16));
}

// Run fn(thread_index, begin, end) over [0, total) split into contiguous ranges.
template <class F>
void parallel_ranges(int64_t total, int threads, F fn)
{
    if (total < (1 << 16)) threads = 1;
    std::vector<std::thread> pool;
    for (int i = 0; i < threads; ++i) {
        int64_t b = total * i / threads, e = total * (i + 1) / threads;
        pool.emplace_back([=] { fn(i, b, e); });
    }
    for (auto& th : pool) th.join();
}

// Run fn(item) for item in [0, total), items handed out dynamically.
template <class F>
void parallel_items(int64_t total, int threads, F fn)
{
    std::atomic<int64_t> next{0};
    std::vector<std::thread> pool;
    for (int i = 0; i < threads; ++i)
        pool.emplace_back([&] {
            for (;;) {
                int64_t it = next.fetch_add(1);
                if (it >= total) break;
                fn(it);
            }
        });
    for (auto& th : pool) th.join();
}

}  // namespace

// `width_weight` = false: every id weighs its number of ratings.  true: its number of ratings
// times the axis length plus the number of ratings in total, i.e. its share of the ratings plus
// its share of the axis, so that a strip is bounded in ratings and in width.
void bounds_from_degrees(const int32_t* degree, int64_t nnz, int64_t size, int32_t g, bool width_weight,
                         std::vector<int32_t>& b)
{
    b.assign((size_t)g + 1, 0);
    b[g] = (int32_t)size;
    const int64_t unit = nnz > 0 ? nnz : 1;
    const __int128 total = width_weight ? (__int128)nnz * size + (__int128)size * unit : (__int128)nnz;
    int64_t before = 0;   // ratings with id < x
    int32_t a = 1;
    for (int64_t x = 0; x < size && a < g; ++x) {
        // strip boundary a sits at the first id whose exclusive weight prefix reaches ceil(a*total/g)
        const __int128 prefix = width_weight ? (__int128)before * size + (__int128)x * unit : (__int128)before;
        while (a < g && prefix >= ((__int128)a * total + g - 1) / g) b[a++] = (int32_t)x;
        before += degree[x];
    }
    while (a < g) b[a++] = (int32_t)size;
}

void equal_width_bounds(int64_t size, int32_t g, std::vector<int32_t>& b)
{
    b.resize((size_t)g + 1);
    for (int32_t a = 0; a <= g; ++a) b[a] = (int32_t)(((int64_t)a * size + g - 1) / g);
}

namespace {

void balanced_bounds(const int32_t* idx, int64_t nnz, int64_t size, int32_t g, int threads,
                     bool width_weight, std::vector<int32_t>& b)
{
    // degree histogram with one private histogram per thread
    std::vector<std::vector<int32_t>> priv((size_t)threads);
    parallel_ranges(nnz, threads, [&](int i, int64_t s, int64_t e) {
        priv[i].assign((size_t)size, 0);
        for (int64_t t = s; t < e; ++t) priv[i][idx[t]] += 1;
    });
    std::vector<int32_t> degree((size_t)size, 0);
    for (auto& h : priv)
        if (!h.empty())
            for (int64_t x = 0; x < size; ++x) degree[x] += h[x];
    bounds_from_degrees(degree.data(), nnz, size, g, width_weight, b);
}

}  // namespace

void strip_table(const std::vector<int32_t>& bounds, int64_t size, std::vector<int32_t>& table)
{
    table.resize((size_t)size);
    int32_t g = (int32_t)bounds.size() - 1;
    for (int32_t a = 0; a < g; ++a)
        for (int64_t x = bounds[a]; x < bounds[a + 1]; ++x) table[x] = a;
}

namespace {

struct KeyPos {
    uint64_t key;   // row << 32 | column
    int64_t t;      // original position
};

}  // namespace

int build_partition(const int32_t* rows, const int32_t* cols, const float* vals, int64_t nnz,
                    int64_t m, int64_t n, int32_t gr, int32_t gc, int32_t split, uint64_t row_seed, Partition& out,
                    std::vector<int32_t>& pu, std::vector<int32_t>& pv, std::vector<float>& pr,
                    std::string& err)
{
    const int threads = host_threads();
    std::atomic<int> bad{0};
    parallel_ranges(nnz, threads, [&](int, int64_t s, int64_t e) {
        for (int64_t t = s; t < e; ++t)
            if (rows[t] < 0 || rows[t] >= m || cols[t] < 0 || cols[t] >= n) { bad = 1; return; }
    });
    if (bad) { err = "a row or column index lies outside the matrix"; return MF_ERANGE; }

    out.nnz = nnz;
    out.gr = gr;
    out.gc = gc;
    if (split == MF_SPLIT_EQUAL_WIDTH) {
        equal_width_bounds(m, gr, out.row_bounds);
        equal_width_bounds(n, gc, out.col_bounds);
    } else {
        const bool width_weight = split == MF_SPLIT_NNZ_WIDTH_BALANCED;
        balanced_bounds(rows, nnz, m, gr, threads, width_weight, out.row_bounds);
        balanced_bounds(cols, nnz, n, gc, threads, width_weight, out.col_bounds);
    }
    std::vector<int32_t> row_strip, col_strip;
    strip_table(out.row_bounds, m, row_strip);
    strip_table(out.col_bounds, n, col_strip);

    const int64_t nblocks = (int64_t)gr * gc;
    // stable counting sort by block id: thread i owns a contiguous range of original positions
    int ct = threads;
    while (ct > 1 && nblocks * ct > ((int64_t)1 << 27)) ct /= 2;
    if (nnz < (1 << 16)) ct = 1;
    std::vector<int32_t> blk((size_t)nnz);
    std::vector<std::vector<int64_t>> hist((size_t)ct);
    auto range_of = [&](int i, int64_t& s, int64_t& e) { s = nnz * i / ct; e = nnz * (i + 1) / ct; };
    {
        std::vector<std::thread> pool;
        for (int i = 0; i < ct; ++i)
            pool.emplace_back([&, i] {
                int64_t s, e;
                range_of(i, s, e);
                hist[i].assign((size_t)nblocks, 0);
                for (int64_t t = s; t < e; ++t) {
                    int32_t a = row_strip[rows[t]], b = col_strip[cols[t]];
                    int32_t st = b - a;
                    if (st < 0) st += gc;
                    int32_t L = st * gr + a;
                    blk[t] = L;
                    hist[i][L] += 1;
                }
            });
        for (auto& th : pool) th.join();
    }
    out.block_ptr.assign((size_t)nblocks + 1, 0);
    {
        int64_t run = 0;
        for (int64_t L = 0; L < nblocks; ++L) {
            out.block_ptr[L] = run;
            for (int i = 0; i < ct; ++i) {
                int64_t c = hist[i][L];
                hist[i][L] = run;      // becomes thread i's write cursor for block L
                run += c;
            }
        }
        out.block_ptr[nblocks] = run;
    }
    out.perm.resize((size_t)nnz);
    {
        std::vector<std::thread> pool;
        for (int i = 0; i < ct; ++i)
            pool.emplace_back([&, i] {
                int64_t s, e;
                range_of(i, s, e);
                for (int64_t t = s; t < e; ++t) out.perm[hist[i][blk[t]]++] = t;
            });
        for (auto& th : pool) th.join();
    }
    hist.clear();
    blk.clear();
    blk.shrink_to_fit();

    // inside every block: ascending (row, column, original position), the rows in their seeded
    // order if one is asked for
    parallel_items(nblocks, threads, [&](int64_t L) {
        int64_t b = out.block_ptr[L], e = out.block_ptr[L + 1];
        if (e - b < 2) return;
        const int32_t a = (int32_t)(L % gr);
        const int32_t first = out.row_bounds[a], width = out.row_bounds[a + 1] - first;
        const uint32_t shift = row_seed ? row_order_shift(row_seed, a, width) : 0;
        std::vector<KeyPos> tmp((size_t)(e - b));
        for (int64_t i = b; i < e; ++i) {
            int64_t t = out.perm[i];
            const uint32_t place = row_seed ? row_order_rank((uint32_t)(rows[t] - first), shift, (uint32_t)width)
                                            : (uint32_t)rows[t];
            tmp[i - b] = {((uint64_t)place << 32) | (uint32_t)cols[t], t};
        }
        std::sort(tmp.begin(), tmp.end(), [](const KeyPos& x, const KeyPos& y) {
            return x.key != y.key ? x.key < y.key : x.t < y.t;
        });
        for (int64_t i = b; i < e; ++i) out.perm[i] = tmp[i - b].t;
    });

    pu.resize((size_t)nnz);
    pv.resize((size_t)nnz);
    pr.resize((size_t)nnz);
    parallel_ranges(nnz, threads, [&](int, int64_t s, int64_t e) {
        for (int64_t i = s; i < e; ++i) {
            int64_t t = out.perm[i];
            pu[i] = rows[t];
            pv[i] = cols[t];
            pr[i] = vals[t];
        }
    });
    return MF_OK;
}

void row_starts_from_rows(const int32_t* pu, int64_t nnz, RowStarts& out)
{
    out.bits.assign((size_t)((nnz + 63) / 64), 0);
    parallel_ranges((nnz + 63) / 64, host_threads(), [&](int, int64_t s, int64_t e) {
        for (int64_t w = s; w < e; ++w) {
            uint64_t word = 0;
            const int64_t last = std::min<int64_t>(nnz, (w + 1) * 64);
            for (int64_t i = w * 64; i < last; ++i)
                if (i == 0 || pu[i] != pu[i - 1]) word |= 1ull << (i & 63);
            out.bits[(size_t)w] = word;
        }
    });
}

// Entries of one stratum are laid out for a launch of kWavesPerGroup wavefronts per workgroup:
// entry e of the stratum is taken by workgroup e / kWavesPerGroup, wavefront e % kWavesPerGroup.
// With XCD affinity workgroup w serves die (w mod kXcds) and block row a is bound to die
// a mod kXcds, so every row of P and every row of Qt touched during one launch is touched from
// one die only (each die has a private L2).  Lists shorter than the longest one are padded with
// empty entries.
static void lay_out_stratum(const std::vector<std::vector<std::pair<int64_t, int32_t>>>& per_die,
                            bool xcd_affinity, Schedule& out)
{
    if (!xcd_affinity) {
        int64_t count = 0;
        for (auto& l : per_die)
            for (auto& c : l) {
                out.begin.push_back(c.first);
                out.len.push_back(c.second);
                ++count;
            }
        while (count % kWavesPerGroup) {
            out.begin.push_back(0);
            out.len.push_back(0);
            ++count;
        }
        return;
    }
    size_t longest = 0;
    for (auto& l : per_die) longest = std::max(longest, l.size());
    size_t groups_per_die = (longest + kWavesPerGroup - 1) / kWavesPerGroup;
    for (size_t g = 0; g < groups_per_die; ++g)
        for (int die = 0; die < kXcds; ++die)
            for (int w = 0; w < kWavesPerGroup; ++w) {
                size_t i = g * kWavesPerGroup + w;
                if (i < per_die[die].size()) {
                    out.begin.push_back(per_die[die][i].first);
                    out.len.push_back(per_die[die][i].second);
                } else {
                    out.begin.push_back(0);
                    out.len.push_back(0);
                }
            }
}

void build_det_schedule(const Partition& part, bool xcd_affinity, Schedule& out)
{
    out.begin.clear();
    out.len.clear();
    out.stratum_entry.assign((size_t)part.gc + 1, 0);
    std::vector<std::vector<std::pair<int64_t, int32_t>>> per_die((size_t)kXcds);
    for (int32_t s = 0; s < part.gc; ++s) {
        for (auto& l : per_die) l.clear();
        for (int32_t a = 0; a < part.gr; ++a) {
            int64_t L = (int64_t)s * part.gr + a;
            int64_t b = part.block_ptr[L], e = part.block_ptr[L + 1];
            if (e > b) per_die[a % kXcds].push_back({b, (int32_t)(e - b)});
        }
        lay_out_stratum(per_die, xcd_affinity, out);
        out.stratum_entry[(size_t)s + 1] = (int64_t)out.begin.size();
    }
}

// Cut the packed range [pos, end) of one block into chunks of whole matrix rows of about `chunk`
// ratings; a row longer than 2*chunk is cut into pieces of `chunk`, each flagged (sign bit of
// the length) as sharing its row of P with other entries.  emit(begin, length_with_flag).
template <class Emit>
static void chunk_block(const RowStarts& rs, int64_t pos, int64_t end, int32_t chunk, Emit emit_raw)
{
    const int32_t long_row = 2 * chunk;
    auto emit = [&](int64_t b, int64_t e, bool shares_row) {
        if (e <= b) return;
        int32_t len = (int32_t)(e - b);
        if (shares_row) len |= (int32_t)0x80000000;
        emit_raw(b, len);
    };
    int64_t cur = pos;   // start of the chunk being filled with whole rows
    while (pos < end) {
        int64_t row_end = pos + 1;
        while (row_end < end && !rs.starts(row_end)) ++row_end;
        if (row_end - pos > long_row) {
            emit(cur, pos, false);
            for (int64_t b = pos; b < row_end; b += chunk) emit(b, std::min<int64_t>(b + chunk, row_end), true);
            cur = row_end;
        } else if (pos > cur && (row_end - cur) > chunk) {
            emit(cur, pos, false);
            cur = pos;
        }
        pos = row_end;
    }
    emit(cur, end, false);
}

// Cut [pos, end) into at most `pieces` chunks of nearly equal size whose boundaries are moved
// forward to the next row boundary; if that would move a boundary by more than two target
// lengths (a very long row), the cut stays inside the row and the chunks on both sides of it
// are flagged as sharing a row of P.
template <class Emit>
static void chunk_block_even(const RowStarts& rs, int64_t pos, int64_t end, int32_t pieces, Emit emit_raw)
{
    const int64_t size = end - pos;
    if (size <= 0) return;
    const int64_t target = std::max<int64_t>(8, (size + pieces - 1) / pieces);
    int64_t cur = pos;
    bool starts_inside_row = false;
    while (cur < end) {
        int64_t cut = std::min(end, cur + target);
        bool ends_inside_row = false;
        if (cut < end) {
            int64_t b = cut;
            while (b < end && !rs.starts(b)) ++b;
            if (b - cut > 2 * target) ends_inside_row = true;   // keep the cut inside the long row
            else cut = b;
        }
        int32_t len = (int32_t)(cut - cur);
        if (starts_inside_row || ends_inside_row) len |= (int32_t)0x80000000;
        emit_raw(cur, len);
        starts_inside_row = ends_inside_row;
        cur = cut;
    }
}

// Cut [pos, end) greedily into chunks of at most `cap` ratings.  A chunk ends at a row boundary
// unless the row that straddles its cap is long (more than cap/2 ratings in this block) or began
// the chunk already: then the cut stays inside the row, and the chunks on both sides of it are
// flagged as sharing a row of P.  A short straddling row goes whole to the next chunk, so every
// chunk but the last is more than half full.  The workgroup is as slow as its longest chunk: the
// caller looks for the smallest cap whose division fits its wavefronts and its slots for cut rows.
template <class Emit>
static void chunk_block_capped(const RowStarts& rs, int64_t pos, int64_t end, int64_t cap, Emit emit_raw)
{
    int64_t cur = pos;
    bool starts_inside_row = false;
    while (cur < end) {
        int64_t cut = std::min(end, cur + cap);
        bool ends_inside_row = false;
        if (cut < end && !rs.starts(cut)) {
            int64_t row_begin = cut, row_end = cut;
            while (row_begin > cur && !rs.starts(row_begin)) --row_begin;
            while (row_end < end && !rs.starts(row_end)) ++row_end;
            if (row_begin > cur && 2 * (row_end - row_begin) <= cap) cut = row_begin;
            else ends_inside_row = true;
        }
        int32_t len = (int32_t)(cut - cur);
        if (starts_inside_row || ends_inside_row) len |= (int32_t)0x80000000;
        emit_raw(cur, len);
        starts_inside_row = ends_inside_row;
        cur = cut;
    }
}

void build_hogwild_schedule(const Partition& part, const RowStarts& rs, int32_t chunk,
                            int32_t waves, bool xcd_affinity, Schedule& out)
{
    // chunk == 0: at most `waves` chunks per block, which bounds the number of wavefronts that
    // change one column of Qt at the same time (each adds a change computed from a value the
    // others may have changed meanwhile: with hundreds of them the sum overshoots)
    out.begin.clear();
    out.len.clear();
    out.stratum_entry.assign((size_t)part.gc + 1, 0);
    std::vector<std::vector<std::pair<int64_t, int32_t>>> per_die((size_t)kXcds);
    int64_t spread = 0;
    for (int32_t s = 0; s < part.gc; ++s) {
        for (auto& l : per_die) l.clear();
        for (int32_t a = 0; a < part.gr; ++a) {
            int64_t L = (int64_t)s * part.gr + a;
            auto push = [&](int64_t b, int32_t len) {
                int die = xcd_affinity ? a % kXcds : (int)(spread++ % kXcds);
                per_die[die].push_back({b, len});
            };
            if (chunk > 0) chunk_block(rs, part.block_ptr[L], part.block_ptr[L + 1], chunk, push);
            else chunk_block_even(rs, part.block_ptr[L], part.block_ptr[L + 1], waves, push);
        }
        lay_out_stratum(per_die, xcd_affinity, out);
        out.stratum_entry[(size_t)s + 1] = (int64_t)out.begin.size();
    }
}

void build_lds_schedule(const Partition& part, const RowStarts& rs, int32_t chunk,
                        int32_t waves, int32_t hot_slots, LdsSchedule& out)
{
    // chunk == 0: cut every block into about one chunk per wavefront of its workgroup
    out.begin.clear();
    out.len.clear();
    out.blocks.clear();
    out.hot_pos.clear();
    out.max_hot = 0;
    out.stratum_block.assign((size_t)part.gc + 1, 0);
    out.max_cols = 0;
    for (int32_t b = 0; b < part.gc; ++b)
        out.max_cols = std::max(out.max_cols, part.col_bounds[b + 1] - part.col_bounds[b]);
    out.ring.assign((size_t)part.gr * part.gc, LdsBlock{0, 0, 0, 0, 0, 0, 0});
    hot_slots = std::min(hot_slots, kMaxHotRows);
    for (int32_t s = 0; s < part.gc; ++s) {
        for (int32_t a = 0; a < part.gr; ++a) {
            int64_t L = (int64_t)s * part.gr + a;
            if (part.block_ptr[L + 1] == part.block_ptr[L]) continue;
            int32_t b = (a + s) % part.gc;
            LdsBlock blk;
            blk.first_entry = (int64_t)out.begin.size();
            blk.col0 = part.col_bounds[b];
            blk.ncols = part.col_bounds[b + 1] - part.col_bounds[b];
            blk.hot = 0;
            blk.id = (int32_t)L;
            blk.reserved = 0;
            auto push = [&](int64_t pos, int32_t len) {
                out.begin.push_back(pos);
                out.len.push_back(len);
            };
            // The rows of this block that an entry boundary cuts (each is named by the position of
            // one of its ratings) are kept in LDS while the block runs.  A boundary lies inside a
            // row when the entry after it does not begin a row; it continues the row of the
            // boundary before it when that one lay inside a row too and no row begins between the
            // two.  A block may have at most `waves` entries and cut at most hot_slots rows: the
            // division starts from chunks of size/waves ratings and is repeated with longer chunks
            // (an eighth longer each time; a given chunk length is doubled) until both hold --
            // at the latest with a single chunk, which cuts none.
            const int64_t hot_first = (int64_t)out.hot_pos.size();
            int32_t n_hot = 0;
            int32_t try_chunk = chunk;
            const int64_t size = part.block_ptr[L + 1] - part.block_ptr[L];
            int64_t cap = std::max<int64_t>(8, (size + waves - 1) / waves);
            for (;;) {
                out.begin.resize((size_t)blk.first_entry);
                out.len.resize((size_t)blk.first_entry);
                out.hot_pos.resize((size_t)hot_first);
                if (try_chunk > 0) chunk_block(rs, part.block_ptr[L], part.block_ptr[L + 1], try_chunk, push);
                else chunk_block_capped(rs, part.block_ptr[L], part.block_ptr[L + 1], cap, push);
                n_hot = 0;
                bool previous_cut_inside_row = false;
                for (int64_t e = blk.first_entry + 1; e < (int64_t)out.begin.size(); ++e) {
                    const int64_t at = out.begin[(size_t)e];
                    const bool inside_row = !rs.starts(at);
                    bool same_row = false;
                    if (inside_row && previous_cut_inside_row) {
                        same_row = true;
                        for (int64_t i = out.begin[(size_t)e - 1] + 1; i < at && same_row; ++i) same_row = !rs.starts(i);
                    }
                    if (inside_row && !same_row) {
                        n_hot += 1;
                        if (n_hot <= hot_slots) out.hot_pos.push_back(at);
                    }
                    previous_cut_inside_row = inside_row;
                }
                const bool indexable = hot_first + n_hot < ((int64_t)1 << 27);   // what `hot` can index
                const int64_t entries = (int64_t)out.begin.size() - blk.first_entry;
                const bool fits = n_hot <= hot_slots && indexable && (try_chunk > 0 || entries <= waves);
                if (fits || entries <= 1) break;
                if (try_chunk > 0) try_chunk = try_chunk > (1 << 29) ? (1 << 30) : 2 * try_chunk;
                else cap += std::max<int64_t>(1, cap / 8);
            }
            blk.n_entries = (int32_t)((int64_t)out.begin.size() - blk.first_entry);
            blk.hot = (int32_t)((hot_first << 4) | n_hot);
            out.max_hot = std::max(out.max_hot, n_hot);
            out.blocks.push_back(blk);
            out.ring[(size_t)L] = blk;
        }
        out.stratum_block[(size_t)s + 1] = (int64_t)out.blocks.size();
    }
}

int32_t widest_strip(const Partition& part)
{
    int32_t widest = 0;
    for (int32_t b = 0; b < part.gc; ++b) widest = std::max(widest, part.col_bounds[b + 1] - part.col_bounds[b]);
    return widest;
}

int64_t lds_hot_bound(int64_t nnz, int32_t gr, int32_t gc)
{
    // at most kMaxHotRows per block, and a cut row has a rating on either side of the cut
    return std::min<int64_t>((int64_t)kMaxHotRows * gr * gc, nnz / 2 + 1);
}

int64_t det_entries_bound(int32_t gr, int32_t gc)
{
    // per stratum: kXcds lists of at most ceil(gr/kXcds) entries, padded to whole workgroups
    int64_t per_die = (gr + kXcds - 1) / kXcds;
    int64_t groups = (per_die + kWavesPerGroup - 1) / kWavesPerGroup;
    return (int64_t)gc * groups * kXcds * kWavesPerGroup;
}

int64_t hogwild_entries_bound(int64_t nnz, int32_t gr, int32_t gc, int32_t chunk, int32_t waves)
{
    if (chunk == 0) {
        int64_t chunks = std::min<int64_t>(nnz / 8 + 1, (int64_t)waves * gr * gc) + (int64_t)gr * gc;
        return chunks * kXcds + (int64_t)gc * kXcds * kWavesPerGroup;
    }
    // Two consecutive chunks of whole rows of a block hold more than `chunk` ratings together
    // (at most 2c/chunk + 1 of them for c ratings); a row longer than 2*chunk gives
    // ceil(len/chunk) pieces and may close one short chunk before it (together at most
    // 2*len/chunk).  Padding can multiply one die's list by kXcds in the worst case.
    int64_t chunks = 4 * (nnz / chunk + 1) + 2 * (int64_t)gr * gc;
    return chunks * kXcds + (int64_t)gc * kXcds * kWavesPerGroup;
}

void build_det_lds_schedule(const Partition& part, LdsSchedule& out)
{
    out.begin.clear();
    out.len.clear();
    out.blocks.clear();
    out.stratum_block.assign((size_t)part.gc + 1, 0);
    out.max_cols = 0;
    for (int32_t b = 0; b < part.gc; ++b)
        out.max_cols = std::max(out.max_cols, part.col_bounds[b + 1] - part.col_bounds[b]);
    out.ring.assign((size_t)part.gr * part.gc, LdsBlock{0, 0, 0, 0, 0, 0, 0});
    for (int32_t s = 0; s < part.gc; ++s) {
        for (int32_t a = 0; a < part.gr; ++a) {
            int64_t L = (int64_t)s * part.gr + a;
            int64_t size = part.block_ptr[L + 1] - part.block_ptr[L];
            if (size == 0) continue;
            int32_t b = (a + s) % part.gc;
            LdsBlock blk;
            blk.first_entry = (int64_t)out.begin.size();
            blk.n_entries = 1;
            blk.col0 = part.col_bounds[b];
            blk.ncols = part.col_bounds[b + 1] - part.col_bounds[b];
            blk.hot = 0;
            blk.id = (int32_t)L;
            blk.reserved = 0;
            out.begin.push_back(part.block_ptr[L]);
            out.len.push_back((int32_t)size);
            out.blocks.push_back(blk);
            out.ring[(size_t)L] = blk;
        }
        out.stratum_block[(size_t)s + 1] = (int64_t)out.blocks.size();
    }
}

int64_t lds_entries_bound(int64_t nnz, int32_t gr, int32_t gc, int32_t chunk, int32_t waves)
{
    // as above, without padding; with chunk == 0 a block is cut into at most `waves` chunks
    if (chunk > 0) return 4 * (nnz / chunk + 1) + 2 * (int64_t)gr * gc;
    // (chunks but the last of a block are more than half full, and a full one has at least 8 ratings)
    return std::min<int64_t>(nnz / 4 + 1, (int64_t)waves * gr * gc) + (int64_t)gr * gc;
}

}  // namespace mf
