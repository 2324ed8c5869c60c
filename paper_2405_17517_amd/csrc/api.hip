// C ABI of the library: argument checks, per-segment thresholds (Eq. 6 feeds
// these through the caller), the cached device segment table, and the launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <list>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/wash.h"
#include "../../include/wash_bench.h"
#include "gaplog.hpp"
#include "kernels.hpp"

namespace {

thread_local char g_detail[256] = "";

__attribute__((format(printf, 2, 3))) int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(g_detail, sizeof(g_detail), fmt, ap);
    va_end(ap);
    return status;
}

int fail_hip(const char *what, hipError_t e)
{
    std::snprintf(g_detail, sizeof(g_detail), "%s: %s", what, hipGetErrorString(e));
    return WASH_EHIP;
}

// round(p * 2^32) as an integer in [0, 2^32]
uint64_t threshold_of(double p)
{
    const double t = std::floor(p * 4294967296.0 + 0.5);
    if (t <= 0.0) return 0;
    if (t >= 4294967296.0) return 4294967296ull;
    return static_cast<uint64_t>(t);
}

// ---- cached device tables: one per (device, P, tile size, active segment list) -------------

struct TableKey {
    int device;
    uint64_t P;
    uint32_t tile_coords;
    int gap;                    // 1: segment params are gap-stream scales, 0: stream-v1 thresholds
    std::vector<wash::DevSegment> segs;
    bool operator==(const TableKey &o) const
    {
        return device == o.device && P == o.P && tile_coords == o.tile_coords && gap == o.gap && segs.size() == o.segs.size() &&
               (segs.empty() || std::memcmp(segs.data(), o.segs.data(), segs.size() * sizeof(wash::DevSegment)) == 0);
    }
};

struct Table {
    TableKey key;
    void *dev = nullptr;            // [uint32 x kCountSlots: active tiles per ticket word][DevSegment x nsegs][uint32 x num_tiles]
    uint64_t num_tiles = 0;
    uint32_t active_words = 0;      // ticket words that at least one active tile reports to
    bool pinned = false;            // recorded into a captured graph: kept until wash_shutdown
};

std::mutex g_mutex;
std::list<Table> g_tables;          // most recently used first
constexpr size_t kMaxTables = 16;
int64_t g_tile_coords_option = 0;   // 0 = choose by P
int64_t g_gap_blocks_option = 0;    // 0 = choose by P
int64_t g_average_chunks = 0;       // 1024-coordinate chunks per block of wash_average; 0 = choose by P
int64_t g_dense_option = 0;         // wash_shuffle's dense path: 0 = by probability, 1 = never, 2 = whenever it fits
int64_t g_shuffle_blocks_per_cu = 0; // cap on resident blocks per compute unit of the sparse shuffle kernel; 0 = none
int64_t g_stream_min_bytes = 256ll << 20;  // papa_ema on populations at least this large uses non-temporal accesses

// Coordinates scanned by one wavefront of wash_shuffle.  `moved_per_coord` is the expected number
// of values moved per coordinate of the row: (selected fraction) * N * (number of buffers).
uint32_t choose_tile_coords(uint64_t P, double moved_per_coord)
{
    if (g_tile_coords_option != 0) return static_cast<uint32_t>(g_tile_coords_option);
    // Above about 0.05 values per coordinate the scattered accesses take longer than the mask scan
    // (measured crossover, N = 20: p between 1e-3 and 3e-3).  Then many short-lived wavefronts with
    // one batch each do best: the batches of a long tile run one after the other, each waiting
    // for the stores of the one before (measured, N = 20, P = 87 M, tiles of 512 against 4096:
    // p = 0.003: 221 / 219 us, 0.01: 715 / 757, 0.03: 1741 / 1977, 0.1: 3201 / 3410; tiles of
    // 256 lose at p = 0.003: 321 us).
    if (moved_per_coord >= 0.05) return 512;
    // The scan dominates: long tiles amortise a wavefront's start-up and its one short batch
    // (p = 1e-3: 85 us at 4096, 163 us at 512), but keep enough tiles to give each of the 1024
    // SIMDs several wavefronts.
    uint32_t t = 4096;
    while (t > 256 && (P + t - 1) / t < 8192) t >>= 1;
    return t;
}

// Builds (or finds) the device table for this call; on success *out points at the cached entry.
int get_table(int device, uint64_t P, uint32_t tile_coords, bool gap, std::vector<wash::DevSegment> &&active,
              Table **out)
{
    TableKey key{device, P, tile_coords, gap ? 1 : 0, std::move(active)};
    for (auto it = g_tables.begin(); it != g_tables.end(); ++it) {
        if (it->key == key) {
            g_tables.splice(g_tables.begin(), g_tables, it);
            *out = &g_tables.front();
            return WASH_OK;
        }
    }
    const uint64_t num_tiles = (P + tile_coords - 1) / tile_coords;
    const size_t nsegs = key.segs.size();
    const size_t seg_bytes = nsegs * sizeof(wash::DevSegment);
    const size_t bytes = wash::kExpectedBytes + seg_bytes + num_tiles * sizeof(uint32_t);
    std::vector<unsigned char> host;
    try {
        host.resize(bytes);
    } catch (const std::bad_alloc &) {
        return fail(WASH_ENOMEM, "segment table of %zu bytes", bytes);
    }
    std::memset(host.data(), 0, wash::kExpectedBytes);
    std::memcpy(host.data() + wash::kExpectedBytes, key.segs.data(), seg_bytes);
    uint32_t *expected = reinterpret_cast<uint32_t *>(host.data());
    uint32_t *tile_first = reinterpret_cast<uint32_t *>(host.data() + wash::kExpectedBytes + seg_bytes);
    size_t s = 0;
    for (uint64_t t = 0; t < num_tiles; ++t) {
        const uint64_t begin = t * tile_coords;
        const uint64_t end = (begin + tile_coords < P) ? begin + tile_coords : P;
        while (s < nsegs && key.segs[s].end <= begin) ++s;
        const bool active = s < nsegs && key.segs[s].begin < end;
        tile_first[t] = active ? static_cast<uint32_t>(s) : wash::kNoSegment;
        if (active) ++expected[t % wash::kCountSlots];      // the tile's wavefront reports to this ticket word
    }
    uint32_t active_words = 0;
    for (uint32_t w = 0; w < wash::kCountSlots; ++w) active_words += expected[w] != 0 ? 1u : 0u;
    if (g_tables.size() >= kMaxTables) {
        // drop the least recently used table that no captured graph refers to (if every table is
        // pinned the cache grows); hipFree waits for the device, so no launched kernel still reads it
        for (auto it = g_tables.end(); it != g_tables.begin();) {
            --it;
            if (it->pinned) continue;
            (void)hipSetDevice(it->key.device);
            (void)hipFree(it->dev);
            (void)hipSetDevice(device);
            g_tables.erase(it);
            break;
        }
    }
    void *dev = nullptr;
    hipError_t e = hipMalloc(&dev, bytes);
    if (e != hipSuccess) return fail_hip("hipMalloc(segment table)", e);
    e = hipMemcpy(dev, host.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dev);
        return fail_hip("hipMemcpy(segment table)", e);
    }
    g_tables.emplace_front();
    g_tables.front().key = std::move(key);
    g_tables.front().dev = dev;
    g_tables.front().num_tiles = num_tiles;
    g_tables.front().active_words = active_words;
    *out = &g_tables.front();
    return WASH_OK;
}

// ---- workspaces: device memory a call needs beyond its arguments -----------------------------------------------
// [ticket words of the shuffle kernels][partial sums of wash_consensus_sqdist], one per (device, stream), so that
// calls on different streams never share any; calls on one stream are ordered.  A stream under capture gets a
// workspace of its own per capture (the recorded kernels keep using it at every replay).  Nothing may be allocated
// while a stream captures, so every allocation also sets a few spare workspaces aside for later captures.
// Workspaces live until wash_shutdown.
struct Workspace {
    int device;
    bool assigned;                  // false: spare
    bool capture;                   // key is a capture id, not a stream
    unsigned long long key;
    void *dev;
};
std::vector<Workspace> g_workspaces;
constexpr size_t kWorkspaceBytes = wash::kTicketBytes + wash::kSqdistScratchBytes;
constexpr int kSpareWorkspaces = 3;
constexpr size_t kMaxWorkspaces = 256;

int new_workspace(int device, Workspace **out)
{
    void *dev = nullptr;
    hipError_t e = hipMalloc(&dev, kWorkspaceBytes);
    if (e != hipSuccess) return fail_hip("hipMalloc(workspace)", e);
    e = hipMemset(dev, 0, wash::kTicketBytes);                  // ticket words are zero between calls
    if (e != hipSuccess) {
        (void)hipFree(dev);
        return fail_hip("hipMemset(workspace)", e);
    }
    try {
        g_workspaces.push_back(Workspace{device, false, false, 0, dev});
    } catch (const std::bad_alloc &) {
        (void)hipFree(dev);
        return fail(WASH_ENOMEM, "workspace list");
    }
    *out = &g_workspaces.back();
    return WASH_OK;
}

// The workspace of `stream` on `device` (g_mutex held).  need = false: the call itself uses none, but, like every
// call outside a capture, it makes sure that spares exist for captures to come.
int get_workspace(int device, hipStream_t stream, bool need, void **out)
{
    *out = nullptr;
    bool capturing = false;
    unsigned long long key = reinterpret_cast<uintptr_t>(stream);
    if (stream != nullptr) {
        hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
        unsigned long long id = 0;
        if (hipStreamGetCaptureInfo(stream, &status, &id) != hipSuccess) {
            (void)hipGetLastError();
        } else if (status == hipStreamCaptureStatusActive) {
            capturing = true;
            key = id;
        }
    }
    void *mine = nullptr;
    size_t spare_index = g_workspaces.size();
    int spares = 0;
    for (size_t k = 0; k < g_workspaces.size(); ++k) {
        Workspace &w = g_workspaces[k];
        if (w.device != device) continue;
        if (w.assigned && w.capture == capturing && w.key == key) mine = w.dev;
        if (!w.assigned) {
            spare_index = k;
            ++spares;
        }
    }
    if (need && mine == nullptr) {
        if (spare_index == g_workspaces.size()) {
            if (capturing)
                return fail(WASH_EHIP, "no workspace is set aside for this capture (device memory cannot be allocated while "
                                       "a stream captures): make one call of the library on this device outside the capture first");
            if (g_workspaces.size() >= kMaxWorkspaces) {
                // Every workspace is taken (a long-lived process that keeps making streams).  Once the device is
                // idle no launched kernel uses any of them and their ticket words are zero again, so those of
                // ordinary streams go back to the pool; the ones recorded into graphs stay with their graphs.
                const hipError_t e = hipDeviceSynchronize();
                if (e != hipSuccess) return fail_hip("hipDeviceSynchronize(workspace pool)", e);
                for (size_t k = 0; k < g_workspaces.size(); ++k) {
                    Workspace &w = g_workspaces[k];
                    if (w.device != device || !w.assigned || w.capture) continue;
                    w.assigned = false;
                    spare_index = k;
                    ++spares;
                }
                if (spare_index == g_workspaces.size())
                    return fail(WASH_ENOMEM, "all %zu workspaces belong to captured graphs or other devices", kMaxWorkspaces);
            } else {
                Workspace *fresh = nullptr;
                if (int rc = new_workspace(device, &fresh)) return rc;
                spare_index = g_workspaces.size() - 1;
                ++spares;
            }
        }
        Workspace &w = g_workspaces[spare_index];
        w.assigned = true;
        w.capture = capturing;
        w.key = key;
        mine = w.dev;
        --spares;
    }
    if (!capturing) {
        // keep a few spares for captures to come (failing to is not an error of this call)
        for (; spares < kSpareWorkspaces && g_workspaces.size() < kMaxWorkspaces; ++spares) {
            Workspace *extra = nullptr;
            if (new_workspace(device, &extra) != WASH_OK) {
                g_detail[0] = 0;
                break;
            }
        }
    }
    *out = mine;
    return WASH_OK;
}

bool ranges_overlap(const void *a, uint64_t abytes, const void *b, uint64_t bbytes)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + bbytes && y < x + abytes;
}

int check_population(const void *params, uint32_t N, uint64_t P)
{
    if (params == nullptr) return fail(WASH_EINVAL, "params is NULL");
    if (N == 0 || N > WASH_MAX_N) return fail(WASH_EINVAL, "N must be in 1..32, got %u", N);
    if (P == 0) return fail(WASH_EINVAL, "P must be >= 1");
    if (P > (1ull << 40)) return fail(WASH_EINVAL, "P larger than 2^40 is not supported");
    return WASH_OK;
}

}  // namespace

extern "C" {

// bufs[0] is the parameter population, bufs[1 .. nbufs-1] the optimizer states that travel with it
// step_dev != nullptr: the kernel reads the step from device memory (and `advance` asks for *step_dev += 1 afterwards)
static int shuffle_common(bool gap, float *const *bufs, uint32_t nbufs, uint32_t N, uint64_t P,
                          const wash_segment *segs, uint32_t nsegs, uint64_t seed, uint64_t step,
                          uint64_t *selected_count, void *stream, uint64_t *step_dev = nullptr, bool advance = false)
{
    g_detail[0] = 0;
    static_assert(WASH_MAX_STATES == wash::kMaxBufs, "header and kernel disagree on the number of buffers");
    if (bufs == nullptr) return fail(WASH_EINVAL, "buffers is NULL");
    if (nbufs == 0 || nbufs > WASH_MAX_STATES)
        return fail(WASH_EINVAL, "number of buffers must be in 1..%d, got %u", WASH_MAX_STATES, nbufs);
    if (int rc = check_population(bufs[0], N, P)) return rc;
    if (step >= (1ull << 32)) return fail(WASH_EINVAL, "step must be < 2^32");
    if (nsegs > 0 && segs == nullptr) return fail(WASH_EINVAL, "segs is NULL");
    const uint64_t pop_bytes = static_cast<uint64_t>(N) * P * sizeof(float);
    for (uint32_t b = 1; b < nbufs; ++b) {
        if (bufs[b] == nullptr) return fail(WASH_EINVAL, "buffer %u is NULL", b);
        for (uint32_t c = 0; c < b; ++c)
            if (ranges_overlap(bufs[c], pop_bytes, bufs[b], pop_bytes))
                return fail(WASH_EINVAL, "buffers %u and %u overlap (0 = params, 1 = momentum)", c, b);
    }
    if (step_dev != nullptr) {
        for (uint32_t b = 0; b < nbufs; ++b)
            if (ranges_overlap(bufs[b], pop_bytes, step_dev, sizeof(uint64_t)))
                return fail(WASH_EINVAL, "step_dev lies inside buffer %u", b);
        if (step_dev == selected_count) return fail(WASH_EINVAL, "step_dev and selected_count are the same word");
    }

    std::vector<wash::DevSegment> active;
    try {
        active.reserve(nsegs);
    } catch (const std::bad_alloc &) {
        return fail(WASH_ENOMEM, "segment list");
    }
    uint64_t prev_end = 0;
    for (uint32_t s = 0; s < nsegs; ++s) {
        const wash_segment &sg = segs[s];
        if (!(sg.p >= 0.0 && sg.p <= 1.0))
            return fail(WASH_EINVAL, "segment %u: probability outside [0,1]", s);
        if (sg.offset > P || sg.length > P - sg.offset)
            return fail(WASH_EINVAL, "segment %u: outside [0,P)", s);
        if (sg.offset < prev_end)
            return fail(WASH_EINVAL, "segment %u: unsorted or overlapping", s);
        prev_end = sg.offset + sg.length;
        if (sg.length == 0) continue;
        if (gap) {
            // touching neighbours with the same p are one segment of the stream; the param slot holds p until
            // the merge is done (p = 0 segments take part in the merge and are dropped afterwards)
            uint64_t pbits;
            const double pval = (sg.p == 0.0) ? 0.0 : sg.p;   // -0.0 and 0.0 are the same probability
            std::memcpy(&pbits, &pval, sizeof(pbits));
            wash::DevSegment d{sg.offset, sg.offset + sg.length, pbits};
            if (!active.empty() && active.back().end == d.begin && active.back().param == d.param)
                active.back().end = d.end;
            else
                active.push_back(d);
            continue;
        }
        const uint64_t T = threshold_of(sg.p);
        if (T == 0) continue;                       // never selected: not scanned at all
        wash::DevSegment d{sg.offset, sg.offset + sg.length, T - 1u};
        // neighbours with the same threshold behave as one segment
        if (!active.empty() && active.back().end == d.begin && active.back().param == d.param)
            active.back().end = d.end;
        else
            active.push_back(d);
    }
    double p_max = 0.0;
    if (gap) {
        size_t kept = 0;
        for (const wash::DevSegment &d : active) {
            double pval;
            std::memcpy(&pval, &d.param, sizeof(pval));
            if (wash::gap_never_selects(pval)) continue;
            if (pval > p_max) p_max = pval;
            const double scale = wash::gap_scale(pval);
            wash::DevSegment out = d;
            std::memcpy(&out.param, &scale, sizeof(scale));
            active[kept++] = out;
        }
        active.resize(kept);
    }
    if (active.empty()) {
        if (step_dev != nullptr && advance) {
            const hipError_t e0 = wash::launch_step_advance(reinterpret_cast<unsigned long long *>(step_dev),
                                                            static_cast<hipStream_t>(stream));
            if (e0 != hipSuccess) return fail_hip("step advance launch", e0);
        }
        return WASH_OK;
    }

    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return fail_hip("hipGetDevice", e);

    std::lock_guard<std::mutex> lock(g_mutex);
    const hipStream_t hstream = static_cast<hipStream_t>(stream);
    bool capturing = false;
    if (stream != nullptr) {
        hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(hstream, &capture) != hipSuccess)
            (void)hipGetLastError();
        else
            capturing = capture == hipStreamCaptureStatusActive;
    }
    // the selected count and the step advance are carried by ticket words in the workspace of this stream
    void *workspace = nullptr;
    if (int rc = get_workspace(device, hstream, selected_count != nullptr || (step_dev != nullptr && advance), &workspace))
        return rc;
    // Finds or builds the device table of `list` and fills the kernel arguments that go with it.
    auto prepare = [&](std::vector<wash::DevSegment> &&list, uint32_t tile_coords, wash::ShuffleArgs *a) -> int {
        Table *table = nullptr;
        if (int rc = get_table(device, P, tile_coords, gap, std::move(list), &table)) return rc;
        // a launch recorded into a graph keeps using this table at every replay: never evict it
        if (capturing) table->pinned = true;
        *a = wash::ShuffleArgs{};
        for (uint32_t b = 0; b < nbufs; ++b) a->bufs[b] = reinterpret_cast<uint32_t *>(bufs[b]);
        a->nbufs = nbufs;
        a->N = N;
        a->P = P;
        unsigned char *base = static_cast<unsigned char *>(table->dev);
        a->segs = reinterpret_cast<const wash::DevSegment *>(base + wash::kExpectedBytes);
        a->nsegs = static_cast<uint32_t>(table->key.segs.size());
        a->tile_first = reinterpret_cast<const uint32_t *>(base + wash::kExpectedBytes +
                                                           table->key.segs.size() * sizeof(wash::DevSegment));
        a->num_tiles = table->num_tiles;
        a->tile_coords = tile_coords;
        a->blocks_per_cu = static_cast<uint32_t>(g_shuffle_blocks_per_cu);
        a->stream_stores = pop_bytes * nbufs >= (4ull << 30) ? 1u : 0u;
        a->key_lo = static_cast<uint32_t>(seed);
        a->key_hi = static_cast<uint32_t>(seed >> 32);
        a->step = static_cast<uint32_t>(step);
        a->step_ptr = reinterpret_cast<const unsigned long long *>(step_dev);
        a->step_advance = (step_dev != nullptr && advance) ? reinterpret_cast<unsigned long long *>(step_dev) : nullptr;
        a->selected_count = reinterpret_cast<unsigned long long *>(selected_count);
        a->tickets = static_cast<unsigned long long *>(workspace);            // nullptr: no count, no step advance
        a->expected = reinterpret_cast<const uint32_t *>(base);
        a->active_words = table->active_words;
        return WASH_OK;
    };

    if (gap) {
        wash::ShuffleArgs a;
        if (int rc = prepare(std::move(active), wash::kGapPiece, &a)) return rc;
        // Blocks walked by one wavefront.  The kernel is bound by the scattered read-modify-write rate as soon
        // as a few coordinates per block are selected, and that rate grows with the number of batches in
        // flight, i.e. with the number of wavefronts: aim at about 16 finds per wavefront (measured best from
        // p = 1e-3 to 1e-1), and never leave the 1024 SIMDs short of wavefronts when p is tiny.
        uint32_t bpw = 64;
        while (bpw > 1 && static_cast<double>(bpw) * wash::kGapPiece * p_max > 16.0) bpw >>= 1;
        while (bpw > 1 && a.num_tiles / bpw < 2048) bpw >>= 1;
        if (g_gap_blocks_option != 0) bpw = static_cast<uint32_t>(g_gap_blocks_option);
        a.blocks_per_wave = bpw;
        a.nwaves = (a.num_tiles + bpw - 1) / bpw;          // every wavefront of the grid reports
        a.expected = nullptr;
        a.active_words = static_cast<uint32_t>(a.nwaves < wash::kCountSlots ? a.nwaves : wash::kCountSlots);
        e = wash::launch_shuffle_gap(a, hstream);
        if (e != hipSuccess) return fail_hip("shuffle launch", e);
        return WASH_OK;
    }

    // Default stream.  Streaming a 256-coordinate strip of all rows through LDS (the dense kernel) costs the
    // same whatever p is; the sparse kernel's scattered accesses grow with p until every half line is touched.
    // Measured crossover at p = 0.08 (N = 20, P = 87 M: dense 2.92 ms; sparse 2.38 ms at p = 0.05, 2.79 at 0.07,
    // 3.20 at 0.1, 3.57 from 0.25 on.  N = 10, P = 26 M, two buffers: dense 0.82-0.86 ms; sparse 0.68 at 0.05,
    // 0.91 at 0.1, 1.03 at 1).  The whole strips inside segments at least that dense go to the dense kernel, the
    // rest of the list (sparser segments, and the ragged ends of dense ones) to the sparse kernel; the stream is
    // addressed by the coordinate, so the split changes no bit.
    const bool dense_fits = N >= 2 && wash::shuffle_dense_lds_bytes(N, nbufs) <= 65536;
    const bool dense_allowed = dense_fits && g_tile_coords_option == 0 && g_dense_option != 1;
    const uint64_t dense_threshold = g_dense_option == 2 ? 1 : threshold_of(0.08);
    std::vector<wash::DevSegment> dense_list, sparse_list;
    double expected_sparse = 0.0;
    try {
        for (const wash::DevSegment &d : active) {
            uint64_t b = d.begin, t = d.end;
            if (dense_allowed && d.param + 1 >= dense_threshold) {
                b = (d.begin + 255u) / 256u * 256u;
                t = d.end == P ? P : d.end / 256u * 256u;
            }
            if (!dense_allowed || d.param + 1 < dense_threshold || b >= t) {
                sparse_list.push_back(d);
                continue;
            }
            if (d.begin < b) sparse_list.push_back(wash::DevSegment{d.begin, b, d.param});
            dense_list.push_back(wash::DevSegment{b, t, d.param});
            if (t < d.end) sparse_list.push_back(wash::DevSegment{t, d.end, d.param});
        }
    } catch (const std::bad_alloc &) {
        return fail(WASH_ENOMEM, "segment list");
    }
    for (const wash::DevSegment &d : sparse_list)
        expected_sparse += static_cast<double>(d.param + 1) / 4294967296.0 * static_cast<double>(d.end - d.begin);
    const bool have_dense = !dense_list.empty(), have_sparse = !sparse_list.empty();
    wash::ShuffleArgs ad, as;
    if (have_dense)
        if (int rc = prepare(std::move(dense_list), 256u, &ad)) return rc;
    if (have_sparse)
        if (int rc = prepare(std::move(sparse_list),
                             choose_tile_coords(P, expected_sparse / static_cast<double>(P) * N * nbufs), &as))
            return rc;
    if (have_dense) {
        if (have_sparse) ad.step_advance = nullptr;           // the step advances after the last kernel of the call
        ad.dense_nontemporal = pop_bytes * nbufs >= (4ull << 30) ? 1u : 0u;
        e = wash::launch_shuffle_dense(ad, hstream);
        if (e != hipSuccess) return fail_hip("shuffle launch", e);
    }
    if (have_sparse) e = wash::launch_shuffle(as, hstream);
    if (e != hipSuccess) return fail_hip("shuffle launch", e);
    return WASH_OK;
}

int wash_shuffle(float *params, float *momentum, uint32_t N, uint64_t P, const wash_segment *segs,
                 uint32_t nsegs, uint64_t seed, uint64_t step, uint64_t *selected_count, void *stream)
{
    float *const bufs[2] = {params, momentum};
    return shuffle_common(false, bufs, momentum ? 2u : 1u, N, P, segs, nsegs, seed, step, selected_count, stream);
}

int wash_shuffle_gap(float *params, float *momentum, uint32_t N, uint64_t P, const wash_segment *segs,
                     uint32_t nsegs, uint64_t seed, uint64_t step, uint64_t *selected_count, void *stream)
{
    float *const bufs[2] = {params, momentum};
    return shuffle_common(true, bufs, momentum ? 2u : 1u, N, P, segs, nsegs, seed, step, selected_count, stream);
}

int wash_shuffle_states(float *const *buffers, uint32_t nbuffers, uint32_t N, uint64_t P, const wash_segment *segs,
                        uint32_t nsegs, uint64_t seed, uint64_t step, int gap_stream, uint64_t *selected_count,
                        void *stream)
{
    if (gap_stream != 0 && gap_stream != 1) {
        g_detail[0] = 0;
        return fail(WASH_EINVAL, "gap_stream must be 0 or 1, got %d", gap_stream);
    }
    return shuffle_common(gap_stream == 1, buffers, nbuffers, N, P, segs, nsegs, seed, step, selected_count, stream);
}


int wash_shuffle_device_step(float *const *buffers, uint32_t nbuffers, uint32_t N, uint64_t P,
                             const wash_segment *segs, uint32_t nsegs, uint64_t seed, uint64_t *step_dev, int advance,
                             int gap_stream, uint64_t *selected_count, void *stream)
{
    g_detail[0] = 0;
    if (gap_stream != 0 && gap_stream != 1) return fail(WASH_EINVAL, "gap_stream must be 0 or 1, got %d", gap_stream);
    if (advance != 0 && advance != 1) return fail(WASH_EINVAL, "advance must be 0 or 1, got %d", advance);
    if (step_dev == nullptr) return fail(WASH_EINVAL, "step_dev is NULL");
    return shuffle_common(gap_stream == 1, buffers, nbuffers, N, P, segs, nsegs, seed, 0, selected_count, stream,
                          step_dev, advance == 1);
}

int wash_average(const float *params, float *out, uint32_t N, uint64_t P, void *stream)
{
    g_detail[0] = 0;
    if (int rc = check_population(params, N, P)) return rc;
    if (out == nullptr) return fail(WASH_EINVAL, "out is NULL");
    if (ranges_overlap(params, static_cast<uint64_t>(N) * P * sizeof(float), out, P * sizeof(float)))
        return fail(WASH_EINVAL, "out overlaps params");
    const int chunks = static_cast<int>(g_average_chunks);     // 0: the launcher chooses kernel and shape
    const bool streaming = static_cast<int64_t>(N * P * sizeof(float)) >= g_stream_min_bytes;
    const hipError_t e = wash::launch_average(params, out, N, P, chunks, streaming, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("wash_average launch", e);
    return WASH_OK;
}

int papa_ema(float *params, uint32_t N, uint64_t P, float alpha, void *stream)
{
    g_detail[0] = 0;
    if (int rc = check_population(params, N, P)) return rc;
    if (!std::isfinite(alpha)) return fail(WASH_EINVAL, "alpha is not finite");
    const bool nt = static_cast<int64_t>(N * P * sizeof(float)) >= g_stream_min_bytes;
    const hipError_t e = wash::launch_ema(params, N, P, alpha, nt, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("papa_ema launch", e);
    return WASH_OK;
}

int wash_consensus_sqdist(const float *params, uint32_t N, uint64_t P, uint64_t g_begin, uint64_t g_end,
                          double *out, void *stream)
{
    g_detail[0] = 0;
    if (int rc = check_population(params, N, P)) return rc;
    if (out == nullptr) return fail(WASH_EINVAL, "out is NULL");
    if (g_begin > g_end || g_end > P) return fail(WASH_EINVAL, "slice outside [0,P]");
    if (ranges_overlap(params, static_cast<uint64_t>(N) * P * sizeof(float), out, N * sizeof(double)))
        return fail(WASH_EINVAL, "out overlaps params");
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return fail_hip("hipGetDevice", e);
    std::lock_guard<std::mutex> lock(g_mutex);
    void *workspace = nullptr;
    if (int rc = get_workspace(device, static_cast<hipStream_t>(stream), true, &workspace)) return rc;
    double *partial = reinterpret_cast<double *>(static_cast<unsigned char *>(workspace) + wash::kTicketBytes);
    e = wash::launch_sqdist(params, N, P, g_begin, g_end, partial, out, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("wash_consensus_sqdist launch", e);
    return WASH_OK;
}

int wash_consensus_sqdist_noalloc(const float *params, uint32_t N, uint64_t P, uint64_t g_begin, uint64_t g_end,
                                  double *out, void *stream)
{
    g_detail[0] = 0;
    if (int rc = check_population(params, N, P)) return rc;      // N <= 32 and P <= 2^40 are what the fixed scratch covers
    if (out == nullptr) return fail(WASH_EINVAL, "out is NULL");
    if (g_begin > g_end || g_end > P) return fail(WASH_EINVAL, "slice outside [0,P]");
    if (ranges_overlap(params, static_cast<uint64_t>(N) * P * sizeof(float), out, N * sizeof(double)))
        return fail(WASH_EINVAL, "out overlaps params");
    static_assert(static_cast<size_t>(wash::kSqdistMaxBlocks) * WASH_MAX_N * sizeof(double) <= wash::kSqdistScratchBytes,
                  "the fixed scratch must hold the partial sums of the largest launch");
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return fail_hip("hipGetDevice", e);
    double *partial = nullptr;
    e = wash::static_sqdist_scratch(device, &partial);
    if (e != hipSuccess) return fail_hip("hipGetSymbolAddress(scratch)", e);
    e = wash::launch_sqdist(params, N, P, g_begin, g_end, partial, out, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("wash_consensus_sqdist_noalloc launch", e);
    return WASH_OK;
}

int wash_weighted_average(const float *params, const double *weights, float *out, uint32_t N, uint64_t P,
                          void *stream)
{
    g_detail[0] = 0;
    if (int rc = check_population(params, N, P)) return rc;
    if (out == nullptr) return fail(WASH_EINVAL, "out is NULL");
    if (weights == nullptr) return fail(WASH_EINVAL, "weights is NULL");
    if (ranges_overlap(params, static_cast<uint64_t>(N) * P * sizeof(float), out, P * sizeof(float)))
        return fail(WASH_EINVAL, "out overlaps params");
    wash::Weights w{};
    for (uint32_t n = 0; n < N; ++n) {
        if (!std::isfinite(weights[n])) return fail(WASH_EINVAL, "weight %u is not finite", n);
        w.w[n] = weights[n];
    }
    const hipError_t e = wash::launch_weighted_average(params, out, N, P, w, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("wash_weighted_average launch", e);
    return WASH_OK;
}

int wash_copy_f32(const float *src, float *dst, uint64_t n, void *stream)
{
    g_detail[0] = 0;
    if (src == nullptr || dst == nullptr) return fail(WASH_EINVAL, "src or dst is NULL");
    if (n == 0 || n > (1ull << 40)) return fail(WASH_EINVAL, "n must be in 1..2^40");
    if (ranges_overlap(src, n * sizeof(float), dst, n * sizeof(float))) return fail(WASH_EINVAL, "dst overlaps src");
    const hipError_t e = wash::launch_copy(src, dst, n, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("wash_copy_f32 launch", e);
    return WASH_OK;
}

int wash_probe_scattered(float *buf, uint64_t lines, int mode, uint32_t rounds, uint32_t blocks, void *stream)
{
    g_detail[0] = 0;
    if (buf == nullptr) return fail(WASH_EINVAL, "buf is NULL");
    if (lines < 2 || (lines & (lines - 1)) != 0 || lines > (1ull << 32))
        return fail(WASH_EINVAL, "lines must be a power of two in [2, 2^32]");
    if (mode < 0 || mode > 3) return fail(WASH_EINVAL, "mode must be 0, 1, 2 or 3");
    if (mode == 3 && reinterpret_cast<uintptr_t>(buf) % 16 != 0) return fail(WASH_EINVAL, "mode 3 needs a 16-byte aligned buf");
    if (rounds == 0 || blocks == 0 || blocks > (1u << 20)) return fail(WASH_EINVAL, "rounds >= 1, 1 <= blocks <= 2^20");
    // the last word of the buffer takes the (never written) sink of the load-only mode
    uint32_t *words = reinterpret_cast<uint32_t *>(buf);
    const hipError_t e = wash::launch_scatter_probe(words, lines, mode, rounds, blocks, words + lines * 32u - 1u,
                                                    static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip("wash_probe_scattered launch", e);
    return WASH_OK;
}

int wash_layer_probs(double p, uint32_t L, int schedule, double *out)
{
    g_detail[0] = 0;
    if (!(p >= 0.0 && p <= 1.0)) return fail(WASH_EINVAL, "p outside [0,1]");
    if (L == 0) return fail(WASH_EINVAL, "L must be >= 1");
    if (out == nullptr) return fail(WASH_EINVAL, "out is NULL");
    if (schedule < 0 || schedule > 2) return fail(WASH_EINVAL, "unknown schedule %d", schedule);
    for (uint32_t l = 0; l < L; ++l) {
        // depth fraction l/(L-1); a single layer keeps the base probability
        const double depth = (L > 1) ? static_cast<double>(l) / static_cast<double>(L - 1) : 0.0;
        switch (schedule) {
        case 0: out[l] = p * (1.0 - depth); break;
        case 1: out[l] = p; break;
        default: out[l] = (L > 1) ? p * depth : p; break;
        }
    }
    return WASH_OK;
}

const char *wash_strerror(int status)
{
    switch (status) {
    case WASH_OK: return "success";
    case WASH_EINVAL: return "invalid argument";
    case WASH_EHIP: return "HIP call failed";
    case WASH_ENOMEM: return "out of host memory";
    default: return "unknown status";
    }
}

const char *wash_last_error_detail(void) { return g_detail; }

int wash_set_option(int option, int64_t value)
{
    g_detail[0] = 0;
    if (option == WASH_OPT_TILE_COORDS) {
        if (value != 0 && (value < 256 || value > 65536 || value % 256 != 0))
            return fail(WASH_EINVAL, "tile coordinates must be 0 or a multiple of 256 in [256, 65536]");
        std::lock_guard<std::mutex> lock(g_mutex);
        g_tile_coords_option = value;
        return WASH_OK;
    }
    if (option == WASH_OPT_GAP_BLOCKS) {
        if (value != 0 && (value < 1 || value > 64 || (value & (value - 1)) != 0))
            return fail(WASH_EINVAL, "gap blocks per wavefront must be 0 or a power of two in [1, 64]");
        std::lock_guard<std::mutex> lock(g_mutex);
        g_gap_blocks_option = value;
        return WASH_OK;
    }
    if (option == WASH_OPT_AVERAGE_CHUNKS) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
            return fail(WASH_EINVAL, "average chunks per block must be 0 (choose by P), 1, 2, 4 or 8");
        std::lock_guard<std::mutex> lock(g_mutex);
        g_average_chunks = value;
        return WASH_OK;
    }
    if (option == WASH_OPT_DENSE) {
        if (value < 0 || value > 2) return fail(WASH_EINVAL, "dense path option must be 0 (automatic), 1 (never) or 2 (always)");
        std::lock_guard<std::mutex> lock(g_mutex);
        g_dense_option = value;
        return WASH_OK;
    }
    if (option == WASH_OPT_SHUFFLE_BLOCKS_PER_CU) {
        if (value < 0 || value > 20) return fail(WASH_EINVAL, "blocks per compute unit must be 0 (no cap) or 1 .. 20");
        std::lock_guard<std::mutex> lock(g_mutex);
        g_shuffle_blocks_per_cu = value;
        return WASH_OK;
    }
    if (option == WASH_OPT_STREAM_MIN_BYTES) {
        if (value < 0) return fail(WASH_EINVAL, "byte threshold must be >= 0");
        std::lock_guard<std::mutex> lock(g_mutex);
        g_stream_min_bytes = value;
        return WASH_OK;
    }
    return fail(WASH_EINVAL, "unknown option %d", option);
}

int wash_shutdown(void)
{
    g_detail[0] = 0;
    std::lock_guard<std::mutex> lock(g_mutex);
    int rc = WASH_OK;
    int current = 0;
    const bool have_current = hipGetDevice(&current) == hipSuccess;
    for (Table &t : g_tables) {
        if (hipSetDevice(t.key.device) != hipSuccess || hipFree(t.dev) != hipSuccess) rc = WASH_EHIP;
    }
    g_tables.clear();
    for (Workspace &w : g_workspaces) {
        if (hipSetDevice(w.device) != hipSuccess || hipFree(w.dev) != hipSuccess) rc = WASH_EHIP;
    }
    g_workspaces.clear();
    if (have_current) (void)hipSetDevice(current);
    return rc;
}

}  // extern "C"
