// Host side of the C ABI declared in include/flora.h: argument validation,
// work-table construction for the grouped launches, the cached device copies
// of descriptor tables and seeds, and the launch sequences that make up each
// entry point.  No arithmetic of the method happens here; it all runs in the
// gfx950 kernels.
#include "../../include/flora.h"
#include "../../include/flora_debug.h"
#include "flora_gen.hip.h"
#include "flora_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <unordered_map>
#include <vector>

namespace flora {

namespace {

thread_local int g_last_hip_error = 0;
std::mutex g_lock;

#define FLORA_HIP(call)                                  \
    do {                                                 \
        const hipError_t e__ = (call);                   \
        if (e__ != hipSuccess) {                         \
            g_last_hip_error = (int)e__;                 \
            (void)hipGetLastError();                     \
            return FLORA_ERR_DEVICE;                     \
        }                                                \
    } while (0)

enum Kind : int {
    kKindCompress = 0,
    kKindDecompress = 1,   // also SGD update: needs only the decompress table
    kKindTransfer = 2,
    kKindFactored = 3,     // the Adafactor rules: statistic partials, per-workgroup sums, scalars
    kKindSumsq = 4         // sum of W^2 from scratch
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool rank_f32(int r) { return r == 8 || r == 16 || r == 32; }
bool rank_bf16(int r) { return r == 64 || r == 128 || r == 256; }

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------ plans
// One uploaded copy of a descriptor table: the caller's pointers (and, for the transfer, seeds)
// with the plan's workspace pointers and tiling filled in.
struct Image {
    std::vector<MatDev> img;     // what the device copy holds
    uint64_t hash = 0;
    MatDev* d_mats = nullptr;    // device copy (inside one of the plan's slabs)
    char* h_stage = nullptr;     // pinned staging of the same size
    hipEvent_t ev = nullptr;     // recorded after the upload
    bool ev_pending = false;
    uint64_t tick = 0;
};

// Everything that depends only on the shapes of a request (and the stream it runs on): work
// tables, launch shape, workspace.  Requests that differ in pointers share all of it and own
// only a descriptor image; an image that has been uploaded before is found by its hash and
// costs nothing, a new one costs one small asynchronous copy.  Calls that come with new
// pointers every time (one matrix per call, gradients freshly allocated) therefore neither
// allocate nor synchronise once the plan exists.
struct Plan {
    int device = -1;
    hipStream_t stream = nullptr;
    int kind = -1;
    int count = 0;
    int r = 0;
    int variant = 0;          // compress: 0 fp32 grads, 1 bf16 grads on the fp32 path, 2 bf16 path,
                              // 3 bf16 path with fp32 grads (rounded in registers); + 4 when the
                              // input is mapped (squared) on the way in
    uint64_t shape_hash = 0;
    std::vector<MatDev> host_mats;      // shapes and tiling fields (pointers unset)
    std::vector<WorkItem> items;        // main work table
    std::vector<WorkItem> items2;       // transfer: state <- state T table
    int mt = 1;                         // bf16 compress: rows per workgroup = 128 * mt
    int vec = 0;                        // decompress: the 16-byte-per-lane bf16 kernel (256-column workgroups)
    int kc = 0;                         // fp32 compress: columns per part (0: whole rows)
    size_t ws_floats = 0;               // compress: floats of partial products (shared-column mode)
    size_t ws_counters = 0;             // ... and arrival counters
    void* d_tables = nullptr;           // items + items2 (uploaded once)
    const WorkItem* d_items = nullptr;
    const WorkItem* d_items2 = nullptr;
    void* h_tables = nullptr;           // pinned source of that upload
    void* d_work = nullptr;             // T / statistic partials / partial products
    size_t work_cap = 0;
    size_t mats_bytes = 0;              // size of one descriptor image
    int image_cap = 16;
    int images_per_slab = 1;
    std::vector<void*> dev_slabs, pin_slabs;
    std::vector<Image> images;
    std::unordered_multimap<uint64_t, int> index;   // image hash -> slot
    const MatDev* cur_mats = nullptr;   // the image of the current call
    uint64_t tick = 0;
    // device side: a plan exists on the host first (tables and sizes) and is then placed, either in
    // memory the library allocates or in the caller's workspace
    bool placed = false;
    bool in_arena = false;
    size_t off2 = 0;                    // offset of items2 within the tables
    size_t tbytes = 0;                  // bytes of the tables
    size_t wbytes = 0;                  // bytes of the work area
    bool pending = false;               // needed by the call being prepared (caller's workspace)
    // factored rule through Gram matrices: items2 = [Gram sums over m | over n | quadratic forms over the
    // rows of S | over the rows of A]
    bool gram = false;
    int n_gm = 0, n_gn = 0, n_qr = 0, n_qc = 0;
};

// Caller-owned workspace (flora_set_workspace).  While one is set every device buffer of a plan
// -- tables, work area, descriptor images -- is carved from it with a bump allocator, uploads
// come from pageable host memory (the copy call returns once the source has been staged) and
// the library calls no hipMalloc / hipHostMalloc.  When the plans a call needs do not fit
// beside those already placed, all placed plans are dropped and the workspace is refilled: the
// caller keeps the calls that use it ordered (one stream, or events), so kernels of earlier calls
// have consumed their tables before the refill's copies land.
struct Arena {
    char* base = nullptr;
    size_t size = 0;
    size_t used = 0;
};
Arena g_ws;
constexpr int kArenaImages = 8;         // descriptor images per plan in the caller's workspace

// Launch-shape knobs, settable through flora_set_tuning (0 = let the library choose).
struct Tuning {
    int compress_f32_kgroups = 0;   // column groups per workgroup in the fp32 compress kernel: 1, 2 or 4
    int compress_bf16_mt = 0;       // bf16 compress: rows per workgroup / 128: 1, 2 or 4; wide kernel: 8, 16, 32
    int compress_f32_mt = 0;        // fp32 compress: rows per workgroup / 64: 1 or 2
    int compress_splitk_cols = 0;   // wide bf16 compress: columns per part when a row block's columns are shared
    int decompress_rows = 0;        // decompress / update: rows per workgroup, a multiple of 32
    int decompress_vec = -1;        // bf16 decompress: -1 choose, 0 scalar kernel, 1 vector kernel when aligned
    int update_wpolicy = 0;         // update passes: 0 choose; 1 + (bit 0 stream reads of W, bit 1 stream writes)
    int factored_gram = 0;          // factored rule at ranks >= 64: 0 choose; 1 reduction passes over the n x m
                                    // product; 2 quadratic forms in r x r Gram matrices
    int gram_chunk = 0;             // long-index entries per workgroup of the Gram sums (0: kGramChunk)
};
Tuning g_tune;

constexpr int kMaxPlans = 1024;
std::vector<Plan*> g_plans;
uint64_t g_tick = 0;

void free_plan(Plan* p)
{
    for (Image& im : p->images) {
        if (im.ev_pending) (void)hipEventSynchronize(im.ev);
        if (im.ev) (void)hipEventDestroy(im.ev);
    }
    if (!p->in_arena) {
        // hipFree waits for the device, so kernels still reading these buffers have finished
        if (p->d_tables) (void)hipFree(p->d_tables);
        if (p->d_work) (void)hipFree(p->d_work);
        for (void* d : p->dev_slabs) (void)hipFree(d);
        for (void* h : p->pin_slabs) (void)hipHostFree(h);
        if (p->h_tables) (void)hipHostFree(p->h_tables);
    }
    delete p;
}

// Bytes of the caller's workspace a plan occupies once placed there.
size_t arena_need(const Plan& p)
{
    return round_up(p.tbytes, 256) + round_up(p.wbytes, 256) + (size_t)kArenaImages * p.mats_bytes;
}

// Work tables -----------------------------------------------------------------
void build_compress_f32_items(Plan& p)
{
    std::vector<int> order(p.count);
    for (int i = 0; i < p.count; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return p.host_mats[a].m > p.host_mats[b].m; });
    p.mt = g_tune.compress_f32_mt ? g_tune.compress_f32_mt : 1;
    const int rows_per_wg = 64 * p.mt;
    const int rp = (p.r + 15) / 16 * 16;
    // A workgroup streams through one compute unit's load path, which carries about an eighth
    // of a percent of the chip's bandwidth: in a launch of a few thousand row blocks the
    // long ones would finish last and alone.  Their columns are then shared between
    // workgroups of about 512 columns (partial products combined by the last one to finish;
    // nparts * rows * r * 8 bytes of extra traffic per block, little at these ranks).
    long long kc = g_tune.compress_splitk_cols;
    if (kc == 0) {
        long long blocks = 0;
        for (int l = 0; l < p.count; ++l) blocks += (p.host_mats[l].n + rows_per_wg - 1) / rows_per_wg;
        if (blocks < 8192) kc = 512;
    }
    p.kc = (int)kc;
    p.ws_floats = 0;
    p.ws_counters = 0;
    for (int l : order) {
        const long long n = p.host_mats[l].n, m = p.host_mats[l].m;
        int parts = kc > 0 ? (int)((m + kc - 1) / kc) : 1;
        const long long pcols = ((m + parts - 1) / parts + 63) / 64 * 64;
        parts = (int)((m + pcols - 1) / pcols);
        int rb = 0;
        for (long long r0 = 0; r0 < n; r0 += rows_per_wg, ++rb) {
            const long long poff = (long long)p.ws_floats;
            const int cidx = (int)p.ws_counters;
            if (parts > 1) {
                p.ws_floats += (size_t)parts * rows_per_wg * rp;
                p.ws_counters += 1;
            }
            for (int part = 0; part < parts; ++part) {
                WorkItem w{};
                w.mat = l; w.row0 = (int)r0;
                w.rows = (int)std::min<long long>(rows_per_wg, n - r0);
                w.rblock = rb;
                w.col0 = (int)(part * pcols);
                w.col1 = (int)std::min<long long>(m, (part + 1) * pcols);
                w.part = part; w.nparts = parts; w.poff = poff; w.cidx = cidx;
                p.items.push_back(w);
            }
        }
    }
}

void build_compress_bf16_items(Plan& p)
{
    // The wide kernel (512, 256 or 128 rows per workgroup, rank slices of 128) regenerates A least
    // often; it needs 16-byte aligned rows of G.  A launch should give the chip at least one
    // and a half workgroups per compute unit: if whole row blocks do not, the columns of a row
    // block are shared between up to a few workgroups (partial products, combined by the last
    // one to finish), then the row blocks are halved.  Sharing costs nparts * rows * r * 8
    // bytes of extra traffic per block, so parts stay at 768 columns or more.
    // Unaligned sets take the narrow kernel with the largest rows-per-workgroup (128 * mt)
    // that still gives the chip two workgroups per compute unit.
    bool aligned = (p.variant & 3) == 2;      // fp32 gradients take the narrow kernel
    for (int l = 0; l < p.count; ++l)   // 16-byte aligned rows, 32-bit byte offsets within 64 rows
        aligned = aligned && (p.host_mats[l].m % 8) == 0 && p.host_mats[l].m <= (1LL << 23);
    const int wide_slice = (p.r == 64) ? 64 : 128;
    auto wide_wgs = [&](int rows, long long kc) {
        long long wgs = 0;
        for (int l = 0; l < p.count; ++l) {
            const long long parts = kc > 0 ? (p.host_mats[l].m + kc - 1) / kc : 1;
            wgs += (p.host_mats[l].n + rows - 1) / rows * (p.r / wide_slice) * parts;
        }
        return wgs;
    };
    int mt = 4;
    long long kc = 0;       // columns per part (0: whole rows)
    if (g_tune.compress_bf16_mt && (aligned || g_tune.compress_bf16_mt <= 4)) {
        mt = g_tune.compress_bf16_mt;
        kc = g_tune.compress_splitk_cols;
    } else if (aligned) {
        const int rows_opt[2] = {512, 256};
        const long long kc_opt[3] = {0, 1536, 768};
        mt = 16; kc = 768;
        bool found = false;
        // An option also has to be balanced: a workgroup sweeps its columns 64 at a time, and when
        // the longest sweep is more than one and a half times a compute unit's even share of all
        // tiles, that workgroup finishes long after the rest (24 matrices of T5-3B shapes with whole
        // rows: 384 workgroups, the 16384-column ones 256 tiles long against an even share of 48,
        // 574 us; in parts of 1536 columns 210 us).
        auto balanced = [&](int rows, long long kc) {
            long long total = 0, longest = 0;
            for (int l = 0; l < p.count; ++l) {
                const long long m = p.host_mats[l].m;
                const long long tiles = (m + 63) / 64;
                total += (p.host_mats[l].n + rows - 1) / rows * (p.r / wide_slice) * tiles;
                longest = std::max(longest, kc > 0 ? std::min(tiles, (kc + 63) / 64) : tiles);
            }
            return 2 * longest <= 3 * std::max<long long>(1, total / 256);
        };
        for (int ri = 0; ri < 2 && !found; ++ri)
            for (int ki = 0; ki < 3 && !found; ++ki)
                if (wide_wgs(rows_opt[ri], kc_opt[ki]) >= 384 && (kc_opt[ki] > 0 || balanced(rows_opt[ri], 0))) {
                    mt = rows_opt[ri] == 512 ? 8 : 16;
                    kc = kc_opt[ki];
                    found = true;
                }
        // Launches over one or two matrices cannot fill the chip either way; what counts then is
        // how long the longest workgroup runs.  Fewer than about 130 workgroups of 256 rows: rows
        // are taken 128 at a time, and below about 150 of those the columns in parts of 384
        // (single matrices of GPT-2 XL and T5-3B shapes: 23-47 -> 21-37 us at r = 256, 21-38 ->
        // 14-26 us at r = 64; taller or wider ones lose with smaller pieces and keep 256 x 768).
        if (!found && wide_wgs(256, 768) < 130) {
            mt = 32;
            kc = wide_wgs(128, 768) < 150 ? 384 : 768;
        }
        if (g_tune.compress_splitk_cols) kc = g_tune.compress_splitk_cols;
    } else for (; mt > 1; mt >>= 1) {
        long long wgs = 0;
        for (int l = 0; l < p.count; ++l)
            wgs += (p.host_mats[l].n + 128 * mt - 1) / (128 * mt) * (p.r / kCompressBf16Slice);
        if (wgs >= 512) break;
    }
    if (mt >= 8 && !aligned) mt = 4;
    const bool wide = mt >= 8;
    if (!wide) kc = 0;
    p.mt = mt;
    const int rows_per_wg = (mt == 8) ? 512 : (mt == 16) ? 256 : (mt == 32) ? 128 : 128 * mt;
    const int slice_w = wide ? wide_slice : kCompressBf16Slice;
    const int S = p.r / slice_w;
    struct Block { int mat, row0, rows, rblock; long long m; };
    std::vector<Block> blocks;
    for (int l = 0; l < p.count; ++l) {
        const long long n = p.host_mats[l].n;
        const long long nb = (n + rows_per_wg - 1) / rows_per_wg;
        long long per = (n + nb - 1) / nb;
        per = (per + 31) / 32 * 32;
        int rb = 0;
        for (long long r0 = 0; r0 < n; r0 += per, ++rb)
            blocks.push_back(Block{l, (int)r0, (int)std::min<long long>(per, n - r0), rb, p.host_mats[l].m});
    }
    std::stable_sort(blocks.begin(), blocks.end(), [](const Block& a, const Block& b) { return a.m > b.m; });
    // Workgroup ids go round-robin over the 8 XCDs.  Give the S rank slices of one
    // row block ids that are equal modulo 8, close together, so that they run on
    // one XCD at about the same time and share its L2 copy of G.
    p.ws_floats = 0;
    p.ws_counters = 0;
    for (size_t base = 0; base < blocks.size(); base += 8) {
        const size_t nb = std::min<size_t>(8, blocks.size() - base);
        // parts of the blocks of this group of 8 (equal column shares, whole 64-column tiles)
        int maxparts = 1;
        int parts[8];
        long long pcols[8];
        for (size_t x = 0; x < nb; ++x) {
            const long long m = blocks[base + x].m;
            parts[x] = kc > 0 ? (int)((m + kc - 1) / kc) : 1;
            pcols[x] = ((m + parts[x] - 1) / parts[x] + 63) / 64 * 64;
            parts[x] = (int)((m + pcols[x] - 1) / pcols[x]);
            maxparts = std::max(maxparts, parts[x]);
        }
        for (int s = 0; s < S; ++s) {
            long long poff[8];
            int cidx[8];
            for (size_t x = 0; x < nb; ++x) {
                poff[x] = (long long)p.ws_floats;
                cidx[x] = (int)p.ws_counters;
                if (parts[x] > 1) {
                    p.ws_floats += (size_t)parts[x] * rows_per_wg * slice_w;
                    p.ws_counters += 1;
                }
            }
            for (int part = 0; part < maxparts; ++part)
                for (size_t x = 0; x < nb; ++x) {
                    if (part >= parts[x]) continue;
                    const Block& b = blocks[base + x];
                    WorkItem w{};
                    w.mat = b.mat; w.row0 = b.row0; w.rows = b.rows; w.slice = s; w.rblock = b.rblock;
                    w.col0 = (int)(part * pcols[x]);
                    w.col1 = (int)std::min<long long>(b.m, (part + 1) * pcols[x]);
                    w.part = part; w.nparts = parts[x]; w.poff = poff[x]; w.cidx = cidx[x];
                    p.items.push_back(w);
                }
        }
    }
}

// Rows per decompress workgroup (an upper limit; each matrix splits its rows evenly below it).
// A workgroup regenerates its slice of A once and reuses it for every row it owns, so the
// generator's work is n m r / rows: 1024 rows make it a few percent of the kernel.  More
// would only make workgroups long and unequal (the last ones to start then run alone);
// fewer are chosen when the launch would otherwise not fill the chip: at ranks up to 64, where
// the pass is bound by the weights' traffic, until there are 2048 workgroups (but not below
// 256 rows); at r = 256, where regenerating A is a large part of a workgroup's time, 140 are
// enough, and at r = 128 about 1000 (launches over the matrices of one to eight transformer
// blocks of GPT-2 XL and T5-3B shapes, r = 256: update 84-453 -> 63-407 us).  A launch over one
// or two matrices cannot fill the chip whatever the rows; there the fewest workgroups per
// compute unit in a row finish first, and rows go down (to 32 at least) until there are about
// 140 workgroups (single matrices of those shapes: update 27-31 -> 18-27 us at r = 256, 17-20 ->
// 10-17 us at r = 64).
int choose_decompress_rows(const std::vector<MatDev>& mats, int cols, int r)
{
    if (g_tune.decompress_rows) return g_tune.decompress_rows;
    auto wgs = [&](int rows) {
        long long w = 0;
        for (const MatDev& M : mats) w += ((M.n + rows - 1) / rows) * ((M.m + cols - 1) / cols);
        return w;
    };
    const long long enough = r >= 256 ? 140 : (r >= 128 ? 1000 : 2048);
    int rows = 1024;
    for (; rows > kDecompressRows; rows /= 2)
        if (wgs(rows) >= enough) break;
    for (; rows > 32 && wgs(rows) < 140; rows /= 2) {}
    return rows;
}

void build_decompress_items(Plan& p)
{
    // the 16-byte-per-lane kernel needs rows of W that start on 16-byte boundaries and 32-bit
    // lane offsets (32 m * 4 bytes below 2^31)
    int vec = rank_bf16(p.r) && (g_tune.decompress_vec != 0);
    for (const MatDev& M : p.host_mats) vec = vec && (M.m % 4) == 0 && M.m <= (1LL << 23);
    p.vec = vec;
    const int cols = vec ? kDecompressColsVec : kDecompressCols;
    // (the vector kernel addresses a workgroup's state rows with 32-bit byte offsets)
    const int rows_per_wg = std::min(choose_decompress_rows(p.host_mats, cols, p.r), vec ? (1 << 20) : 0x7fffffe0);
    struct Group { int mat, rb, row0, rows, nchunks; };
    std::vector<Group> groups;
    for (int l = 0; l < p.count; ++l) {
        MatDev& M = p.host_mats[l];
        M.nrowblocks = (int)((M.n + rows_per_wg - 1) / rows_per_wg);
        M.ncolchunks = (int)((M.m + cols - 1) / cols);
        // equal row blocks, a multiple of 32 rows each
        long long per = (M.n + M.nrowblocks - 1) / M.nrowblocks;
        per = (per + 31) / 32 * 32;
        M.nrowblocks = (int)((M.n + per - 1) / per);
        M.item0 = 0;
        M.nitems = M.nrowblocks * M.ncolchunks;
        for (int rb = 0; rb < M.nrowblocks; ++rb)
            groups.push_back(Group{l, rb, (int)(rb * per), (int)std::min<long long>(per, M.n - rb * per), M.ncolchunks});
    }
    // Every workgroup of a row block reads that block of the state.  Workgroup ids go
    // round-robin over the 8 XCDs, each with its own L2: if the column chunks of one row
    // block simply followed each other, every XCD would fetch every state block from HBM
    // (8 times the state's size; at r = 256 that was a third of the kernel's traffic).  So
    // row blocks are taken eight at a time (with equal chunk counts) and their chunks
    // interleaved: all chunks of one row block get ids equal modulo 8, close together, and
    // find the block in their XCD's L2 after the first.  Row blocks that do not fill a
    // bundle of eight come last.
    std::stable_sort(groups.begin(), groups.end(), [](const Group& a, const Group& b) { return a.nchunks > b.nchunks; });
    auto emit = [&](const Group* g, size_t ng) {
        for (int cc = 0; cc < g[0].nchunks; ++cc)
            for (size_t x = 0; x < ng; ++x) {
                if (cc >= g[x].nchunks) continue;
                WorkItem w{};
                w.mat = g[x].mat; w.row0 = g[x].row0; w.rows = g[x].rows;
                w.col0 = cc * cols; w.slice = cc; w.rblock = g[x].rb;
                w.part = g[x].rb * g[x].nchunks + cc;
                p.items.push_back(w);
            }
    };
    std::vector<Group> rest;
    for (size_t i = 0; i < groups.size();) {
        size_t j = i;
        while (j < groups.size() && groups[j].nchunks == groups[i].nchunks) ++j;
        size_t k = i;
        for (; k + 8 <= j; k += 8) emit(&groups[k], 8);
        for (; k < j; ++k) rest.push_back(groups[k]);
        i = j;
    }
    for (size_t k = 0; k < rest.size(); k += 8) emit(&rest[k], std::min<size_t>(8, rest.size() - k));
}

void build_apply_T_items(Plan& p)
{
    const int rows = p.r >= 64 ? kApplyTRowsBig : kApplyTRows;
    for (int l = 0; l < p.count; ++l) {
        const long long n = p.host_mats[l].n;
        for (long long r0 = 0; r0 < n; r0 += rows) {
            WorkItem w{};
            w.mat = l; w.row0 = (int)r0; w.rows = (int)std::min<long long>(rows, n - r0);
            p.items2.push_back(w);
        }
    }
}

// T = A_old^T A_new at ranks 64 and above: (matrix, chunk of 1024 columns, slab of up to 128 rows
// of T); ncolchunks of the matrix = its number of chunks (the partials the combine pass adds).
void build_transfer_T_items(Plan& p)
{
    if (p.r < 64) return;
    const int slabs = p.r / std::min(p.r, 128);
    for (int l = 0; l < p.count; ++l) {
        const long long m = p.host_mats[l].m;
        const int chunks = (int)((m + kTransferChunk - 1) / kTransferChunk);
        p.host_mats[l].ncolchunks = chunks;
        for (int c = 0; c < chunks; ++c)
            for (int s = 0; s < slabs; ++s) {
                WorkItem w{};
                w.mat = l; w.slice = s; w.part = c;
                w.col0 = (int)((long long)c * kTransferChunk);
                w.col1 = (int)std::min<long long>(m, (long long)(c + 1) * kTransferChunk);
                p.items.push_back(w);
            }
    }
}

// The factored rule's reduction passes as quadratic forms in Gram matrices (flora_gram.hip): chosen
// when that is clearly less arithmetic than two passes over the n x m product, 6 (m + n) r^2 against
// 4 n m r flops per matrix (with a margin: kernels with r x r outputs and split sums run the
// matrix cores less efficiently than the long sweeps of the decompression).
bool choose_gram(const Plan& p)
{
    if (!rank_bf16(p.r)) return false;
    if (g_tune.factored_gram) return g_tune.factored_gram == 2;
    double pass = 0.0, gram = 0.0;
    for (const MatDev& M : p.host_mats) {
        pass += 4.0 * (double)M.n * (double)M.m * p.r;
        gram += 6.0 * ((double)M.n + (double)M.m) * p.r * p.r;
    }
    return 1.5 * gram < pass;
}

void build_gram_items(Plan& p)
{
    const long long gchunk = g_tune.gram_chunk ? g_tune.gram_chunk : kGramChunk;
    auto chunks_of = [&](long long len) { return (int)((len + gchunk - 1) / gchunk); };
    auto emit_chunks = [&](int l, long long len, int chunks) {
        const long long per = ((len + chunks - 1) / chunks + 63) / 64 * 64;
        for (int c = 0; c < chunks; ++c) {
            WorkItem w{};
            w.mat = l; w.part = c;
            w.col0 = (int)std::min<long long>(len, (long long)c * per);
            w.col1 = (int)std::min<long long>(len, (long long)(c + 1) * per);
            p.items2.push_back(w);
        }
    };
    auto emit_blocks = [&](int l, long long len) {
        const long long nb = (len + kQuadformRows - 1) / kQuadformRows;
        const long long per = ((len + nb - 1) / nb + 31) / 32 * 32;
        int b = 0;
        for (long long r0 = 0; r0 < len; r0 += per, ++b) {
            WorkItem w{};
            w.mat = l; w.part = b; w.row0 = (int)r0; w.rows = (int)std::min<long long>(per, len - r0);
            p.items2.push_back(w);
        }
        return b;
    };
    for (int l = 0; l < p.count; ++l) {
        MatDev& M = p.host_mats[(size_t)l];
        M.gchunks_m = chunks_of(M.m);
        M.gchunks_n = chunks_of(M.n);
    }
    // longest first within each table
    std::vector<int> by_m(p.count), by_n(p.count);
    for (int i = 0; i < p.count; ++i) by_m[i] = by_n[i] = i;
    std::stable_sort(by_m.begin(), by_m.end(), [&](int a, int b) { return p.host_mats[a].m > p.host_mats[b].m; });
    std::stable_sort(by_n.begin(), by_n.end(), [&](int a, int b) { return p.host_mats[a].n > p.host_mats[b].n; });
    size_t before = p.items2.size();
    for (int l : by_m) emit_chunks(l, p.host_mats[(size_t)l].m, p.host_mats[(size_t)l].gchunks_m);
    p.n_gm = (int)(p.items2.size() - before); before = p.items2.size();
    for (int l : by_n) emit_chunks(l, p.host_mats[(size_t)l].n, p.host_mats[(size_t)l].gchunks_n);
    p.n_gn = (int)(p.items2.size() - before); before = p.items2.size();
    for (int l : by_n) p.host_mats[(size_t)l].item0 = emit_blocks(l, p.host_mats[(size_t)l].n);
    p.n_qr = (int)(p.items2.size() - before); before = p.items2.size();
    for (int l : by_m) (void)emit_blocks(l, p.host_mats[(size_t)l].m);
    p.n_qc = (int)(p.items2.size() - before);
}

size_t workspace_bytes_for(const std::vector<MatDev>& mats, int kind, int r, bool gram = false)
{
    size_t b = 0;
    for (const MatDev& M : mats) {
        if (kind == kKindFactored && gram) {
            b += 3 * round_up((size_t)r * r * 2, 256);
            b += round_up((size_t)(2 * M.gchunks_m + M.gchunks_n) * r * r * 4, 256);
        }
        if (kind == kKindTransfer) {
            b += round_up((size_t)r * r * 4, 256);
            if (r >= 64) b += round_up((size_t)M.ncolchunks * r * r * 4, 256);
        }
        if (kind == kKindFactored) {
            b += round_up((size_t)M.ncolchunks * M.n * 4, 256);
            b += round_up((size_t)M.nrowblocks * M.m * 4, 256);
            b += round_up((size_t)M.nitems * 4, 256);
            b += 256;
        }
        if (kind == kKindSumsq) b += (size_t)kSumsqBlocks * 4;
    }
    return b;
}

uint64_t hash_bytes(const void* data, size_t bytes, uint64_t h)
{
    const unsigned char* c = static_cast<const unsigned char*>(data);
    size_t i = 0;
    for (; i + 8 <= bytes; i += 8) {
        uint64_t w;
        std::memcpy(&w, c + i, 8);
        h = (h ^ w) * 0x9E3779B97F4A7C15ull;
        h ^= h >> 29;
    }
    for (; i < bytes; ++i) h = (h ^ c[i]) * 0x100000001B3ull;
    return h;
}

uint64_t hash_shapes(const std::vector<MatDev>& mats)
{
    uint64_t h = 0x243F6A8885A308D3ull;
    for (const MatDev& M : mats) {
        const long long nm[2] = {M.n, M.m};
        h = hash_bytes(nm, sizeof(nm), h);
    }
    return h;
}

bool same_shapes(const Plan& p, const std::vector<MatDev>& mats)
{
    for (size_t l = 0; l < mats.size(); ++l)
        if (p.host_mats[l].n != mats[l].n || p.host_mats[l].m != mats[l].m) return false;
    return true;
}

// Host part of a plan: work tables, launch shape and the sizes of its device buffers.  Pure host
// work, nothing is allocated on or sent to the device.
void build_host_plan(Plan* p, const std::vector<MatDev>& mats)
{
    const int kind = p->kind, r = p->r, count = p->count;
    p->host_mats = mats;
    for (MatDev& M : p->host_mats) {      // shapes only
        const long long n = M.n, m = M.m;
        M = MatDev{};
        M.n = n; M.m = m;
    }
    if (kind == kKindCompress) {
        if ((p->variant & 3) >= 2) build_compress_bf16_items(*p);
        else build_compress_f32_items(*p);
    } else if (kind == kKindTransfer) {
        build_transfer_T_items(*p);
        build_apply_T_items(*p);
    } else if (kind != kKindSumsq) {
        build_decompress_items(*p);
        if (kind == kKindFactored && (p->variant & 3) == 2) {     // the factored rule (not the unfactored one)
            p->gram = choose_gram(*p);
            if (p->gram) build_gram_items(*p);
        }
    }
    p->off2 = round_up(sizeof(WorkItem) * p->items.size(), 256);
    p->tbytes = p->off2 + round_up(sizeof(WorkItem) * p->items2.size(), 256);
    p->wbytes = workspace_bytes_for(p->host_mats, kind, r, p->gram);
    if (kind == kKindCompress) p->wbytes = round_up(p->ws_floats * 4, 256) + p->ws_counters * 4;
    p->mats_bytes = round_up(sizeof(MatDev) * (size_t)count, 256);
    // descriptor images kept per plan: many for calls on a few matrices (a training loop that
    // steps one layer per call cycles through hundreds of pointer sets), a few for large sets
    p->image_cap = count <= 4 ? 512 : (count <= 32 ? 64 : 16);
    p->images_per_slab = (int)std::max<size_t>(1, std::min<size_t>(64, (64 * 1024) / p->mats_bytes));
}

// Device part: tables uploaded, work area ready.  In library-allocated memory, or (in_arena) at
// the next free bytes of the caller's workspace, whose capacity the caller of this function
// has already checked.
int place_plan(Plan* p, hipStream_t stream)
{
    const size_t off2 = p->off2, tbytes = p->tbytes, wbytes = p->wbytes;
    if (p->in_arena) {
        p->image_cap = kArenaImages;
        p->images_per_slab = kArenaImages;
    }
    auto arena_take = [&](size_t bytes) {
        char* q = g_ws.base + g_ws.used;
        g_ws.used += round_up(bytes, 256);
        return static_cast<void*>(q);
    };
    if (tbytes > 0) {
        if (p->in_arena) {
            p->d_tables = arena_take(tbytes);
            // pageable source: the copy call returns once the source has been staged
            static thread_local std::vector<char> stage;
            stage.assign(tbytes, 0);
            if (!p->items.empty()) std::memcpy(stage.data(), p->items.data(), sizeof(WorkItem) * p->items.size());
            if (!p->items2.empty()) std::memcpy(stage.data() + off2, p->items2.data(), sizeof(WorkItem) * p->items2.size());
            FLORA_HIP(hipMemcpyAsync(p->d_tables, stage.data(), tbytes, hipMemcpyHostToDevice, stream));
        } else {
            FLORA_HIP(hipMalloc(&p->d_tables, tbytes));
            FLORA_HIP(hipHostMalloc(&p->h_tables, tbytes, hipHostMallocDefault));
            char* hp = static_cast<char*>(p->h_tables);
            if (!p->items.empty()) std::memcpy(hp, p->items.data(), sizeof(WorkItem) * p->items.size());
            if (!p->items2.empty()) std::memcpy(hp + off2, p->items2.data(), sizeof(WorkItem) * p->items2.size());
            // (the plan is only ever used on this stream, so everything after this copy sees it)
            FLORA_HIP(hipMemcpyAsync(p->d_tables, p->h_tables, tbytes, hipMemcpyHostToDevice, stream));
        }
        p->d_items = static_cast<const WorkItem*>(p->d_tables);
        p->d_items2 = reinterpret_cast<const WorkItem*>(static_cast<char*>(p->d_tables) + off2);
    }
    if (wbytes > 0) {
        if (p->in_arena) p->d_work = arena_take(wbytes);
        else FLORA_HIP(hipMalloc(&p->d_work, wbytes));
        p->work_cap = wbytes;
        // arrival counters start at zero (the kernel leaves them at zero again)
        if (p->kind == kKindCompress && p->ws_counters > 0)
            FLORA_HIP(hipMemsetAsync(static_cast<char*>(p->d_work) + round_up(p->ws_floats * 4, 256), 0,
                                     p->ws_counters * 4, stream));
    }
    if (p->in_arena) p->dev_slabs.push_back(arena_take((size_t)kArenaImages * p->mats_bytes));
    p->placed = true;
    return FLORA_OK;
}

// Plans the call being prepared needs (caller's workspace only).
std::vector<Plan*> g_pending;

void drop_plan_at(size_t i)
{
    free_plan(g_plans[i]);
    g_plans.erase(g_plans.begin() + (long)i);
}

// Finds or creates the plan for (kind, variant, r, shapes, stream) and the device copy of this
// request's descriptor table; p->cur_mats points at it on return.  With `dry` set (first pass of
// a call that uses the caller's workspace) the plan is only found or built on the host and noted
// as needed: nothing is allocated, uploaded or launched.
int get_plan(int kind, int variant, int r, const std::vector<MatDev>& mats, hipStream_t stream, Plan** out,
             bool dry = false)
{
    int device = 0;
    if (dry) {
        // the dry pass is host work only: on a machine without a device the capacity check of
        // arena_commit is still reached (and reports a workspace that is too small)
        if (hipGetDevice(&device) != hipSuccess) { (void)hipGetLastError(); device = -1; }
    } else {
        FLORA_HIP(hipGetDevice(&device));
    }
    const int count = (int)mats.size();
    const uint64_t sh = hash_shapes(mats);
    const bool arena = g_ws.base != nullptr;

    Plan* p = nullptr;
    for (Plan* q : g_plans)
        if (q->shape_hash == sh && q->device == device && q->stream == stream && q->kind == kind &&
            q->variant == variant && q->r == r && q->count == count && same_shapes(*q, mats)) {
            p = q;
            break;
        }
    if (!p) {
        if ((int)g_plans.size() >= kMaxPlans) {
            size_t lru = g_plans.size();
            for (size_t i = 0; i < g_plans.size(); ++i)
                if (!g_plans[i]->pending && (lru == g_plans.size() || g_plans[i]->tick < g_plans[lru]->tick)) lru = i;
            if (lru == g_plans.size()) return FLORA_ERR_INVALID;     // one call needing more than kMaxPlans plans
            // (a plan dropped from the caller's workspace leaves its bytes unused until the next refill)
            drop_plan_at(lru);
        }
        p = new Plan();
        p->device = device; p->stream = stream; p->kind = kind; p->variant = variant; p->count = count; p->r = r;
        p->shape_hash = sh;
        p->in_arena = arena;
        build_host_plan(p, mats);
        if (!arena) {
            const int st = place_plan(p, stream);
            if (st != FLORA_OK) {
                free_plan(p);
                return st;
            }
        }
        g_plans.push_back(p);
    }
    p->tick = ++g_tick;
    if (dry) {
        if (!p->pending) {
            p->pending = true;
            g_pending.push_back(p);
        }
        *out = p;
        return FLORA_OK;
    }
    if (!p->placed) return FLORA_ERR_INVALID;      // (cannot happen: arena_commit places what the dry pass noted)

    // this request's image: the caller's pointers, the plan's tiling and workspace
    static thread_local std::vector<MatDev> img;
    img = mats;
    {
        char* w = static_cast<char*>(p->d_work);
        for (int l = 0; l < count; ++l) {
            MatDev& M = img[(size_t)l];
            const MatDev& t = p->host_mats[(size_t)l];
            M.ncolchunks = t.ncolchunks; M.nrowblocks = t.nrowblocks; M.item0 = t.item0; M.nitems = t.nitems;
            M.gchunks_m = t.gchunks_m; M.gchunks_n = t.gchunks_n;
            if (kind == kKindFactored && p->gram) {
                M.gramP = reinterpret_cast<uint16_t*>(w); w += round_up((size_t)r * r * 2, 256);
                M.gramQ = reinterpret_cast<uint16_t*>(w); w += 2 * round_up((size_t)r * r * 2, 256);   // Q, then P'
                M.grampart = reinterpret_cast<float*>(w);
                w += round_up((size_t)(2 * M.gchunks_m + M.gchunks_n) * r * r * 4, 256);
            }
            if (kind == kKindTransfer) {
                M.T = reinterpret_cast<float*>(w); w += round_up((size_t)r * r * 4, 256);
                if (r >= 64) { M.rowpart = reinterpret_cast<float*>(w); w += round_up((size_t)M.ncolchunks * r * r * 4, 256); }
            }
            if (kind == kKindFactored) {
                M.rowpart = reinterpret_cast<float*>(w); w += round_up((size_t)M.ncolchunks * M.n * 4, 256);
                M.colpart = reinterpret_cast<float*>(w); w += round_up((size_t)M.nrowblocks * M.m * 4, 256);
                M.itempart = reinterpret_cast<float*>(w); w += round_up((size_t)M.nitems * 4, 256);
                M.scal = reinterpret_cast<float*>(w); w += 256;
            }
        }
    }
    const size_t ibytes = sizeof(MatDev) * (size_t)count;
    const uint64_t h = hash_bytes(img.data(), ibytes, 0x13198A2E03707344ull);
    auto range = p->index.equal_range(h);
    for (auto it = range.first; it != range.second; ++it) {
        Image& im = p->images[(size_t)it->second];
        if (std::memcmp(im.img.data(), img.data(), ibytes) == 0) {
            im.tick = g_tick;
            p->cur_mats = im.d_mats;
            *out = p;
            return FLORA_OK;
        }
    }

    int slot = -1;
    if ((int)p->images.size() < p->image_cap) {
        slot = (int)p->images.size();
        const int slab = slot / p->images_per_slab, within = slot % p->images_per_slab;
        if (slab >= (int)p->dev_slabs.size()) {
            // (never in the caller's workspace: its one slab of kArenaImages images was placed with the plan)
            void* d = nullptr;
            void* hp = nullptr;
            FLORA_HIP(hipMalloc(&d, p->mats_bytes * (size_t)p->images_per_slab));
            p->dev_slabs.push_back(d);
            FLORA_HIP(hipHostMalloc(&hp, p->mats_bytes * (size_t)p->images_per_slab, hipHostMallocDefault));
            p->pin_slabs.push_back(hp);
        }
        Image im;
        im.d_mats = reinterpret_cast<MatDev*>(static_cast<char*>(p->dev_slabs[(size_t)slab]) + p->mats_bytes * (size_t)within);
        if (!p->in_arena) {
            im.h_stage = static_cast<char*>(p->pin_slabs[(size_t)slab]) + p->mats_bytes * (size_t)within;
            FLORA_HIP(hipEventCreateWithFlags(&im.ev, hipEventDisableTiming));
        }
        p->images.push_back(std::move(im));
    } else {
        // every slot is taken: the least recently used image gives way.  Kernels that read its
        // device copy were enqueued on this stream before the copy below; its staging buffer may
        // still be the source of its previous upload.
        slot = 0;
        for (size_t i = 1; i < p->images.size(); ++i)
            if (p->images[i].tick < p->images[(size_t)slot].tick) slot = (int)i;
        Image& old = p->images[(size_t)slot];
        auto rg = p->index.equal_range(old.hash);
        for (auto it = rg.first; it != rg.second; ++it)
            if (it->second == slot) {
                p->index.erase(it);
                break;
            }
        if (old.ev_pending) { FLORA_HIP(hipEventSynchronize(old.ev)); old.ev_pending = false; }
    }
    Image& im = p->images[(size_t)slot];
    im.img = img;
    im.hash = h;
    im.tick = g_tick;
    if (p->in_arena) {
        // pageable source: the copy call returns once the source has been staged
        FLORA_HIP(hipMemcpyAsync(im.d_mats, im.img.data(), ibytes, hipMemcpyHostToDevice, stream));
    } else {
        std::memcpy(im.h_stage, img.data(), ibytes);
        FLORA_HIP(hipMemcpyAsync(im.d_mats, im.h_stage, ibytes, hipMemcpyHostToDevice, stream));
        FLORA_HIP(hipEventRecord(im.ev, stream));
        im.ev_pending = true;
    }
    p->index.emplace(h, slot);
    p->cur_mats = im.d_mats;
    *out = p;
    return FLORA_OK;
}

// Second half of preparing a call that uses the caller's workspace: the plans the dry pass noted
// are placed.  If those not yet placed do not fit in what is left, every placed plan is dropped
// and the workspace refilled from its start with this call's plans; if these alone exceed the
// workspace the call fails with FLORA_ERR_INVALID and nothing has been enqueued.
int arena_commit(hipStream_t stream)
{
    auto clear_pending = [&]() {
        for (Plan* p : g_pending) p->pending = false;
        g_pending.clear();
    };
    size_t need_new = 0, need_all = 0;
    for (Plan* p : g_pending) {
        need_all += arena_need(*p);
        if (!p->placed) need_new += arena_need(*p);
    }
    if (need_new > g_ws.size - g_ws.used) {
        if (need_all > g_ws.size) {
            // also forget the host halves built for this call: they could never be placed
            for (size_t i = g_plans.size(); i-- > 0;)
                if (g_plans[i]->pending && !g_plans[i]->placed) drop_plan_at(i);
            g_pending.clear();
            for (Plan* p : g_plans) p->pending = false;
            return FLORA_ERR_INVALID;
        }
        for (size_t i = g_plans.size(); i-- > 0;) {
            Plan* p = g_plans[i];
            if (!p->in_arena) continue;
            if (p->pending) {           // stays, but loses its place: tables and images are uploaded again
                p->placed = false;
                p->d_tables = nullptr; p->d_work = nullptr; p->d_items = nullptr; p->d_items2 = nullptr;
                p->dev_slabs.clear(); p->images.clear(); p->index.clear(); p->cur_mats = nullptr;
            } else {
                drop_plan_at(i);
            }
        }
        g_ws.used = 0;
    }
    for (Plan* p : g_pending)
        if (!p->placed) {
            const int st = place_plan(p, stream);
            if (st != FLORA_OK) {
                clear_pending();
                return st;
            }
        }
    clear_pending();
    return FLORA_OK;
}

void drop_all_plans()
{
    for (Plan* p : g_plans) free_plan(p);
    g_plans.clear();
    g_pending.clear();
}

void abort_pending()
{
    for (size_t i = g_plans.size(); i-- > 0;)
        if (g_plans[i]->pending && !g_plans[i]->placed) drop_plan_at(i);
    for (Plan* p : g_plans) p->pending = false;
    g_pending.clear();
}

// Runs the chunks of one call.  With a caller-owned workspace the chunks are first walked dry (plans
// found or built on the host and noted), then the workspace's capacity is checked and the plans
// placed, and only then is anything launched.
template <typename Body>
int run_call(hipStream_t s, Body&& body)
{
    if (g_ws.base) {
        int st = body(true);
        if (st != FLORA_OK) {
            abort_pending();
            return st;
        }
        st = arena_commit(s);
        if (st != FLORA_OK) return st;
    }
    return body(false);
}

// ------------------------------------------------------------- validation
int check_common(const flora_matrix_t* mats, int count, int r)
{
    if (count < 0) return FLORA_ERR_INVALID;
    if (count > 0 && !mats) return FLORA_ERR_INVALID;
    if (r <= 0) return FLORA_ERR_INVALID;
    if (!rank_f32(r) && !rank_bf16(r)) return FLORA_ERR_UNSUPPORTED;
    for (int l = 0; l < count; ++l) {
        if (mats[l].n < 1 || mats[l].m < 1) return FLORA_ERR_INVALID;
        if (mats[l].n > 0x7fffffffLL - 1024 || mats[l].m > (1LL << 24)) return FLORA_ERR_INVALID;
        if (!mats[l].state || !aligned16(mats[l].state)) return FLORA_ERR_INVALID;
    }
    return FLORA_OK;
}

bool dtype_ok(int d) { return d == FLORA_F32 || d == FLORA_BF16; }

}  // namespace

}  // namespace flora

using namespace flora;

// Seeds travel as kernel arguments (SeedArgs) for compress / decompress / update, so the
// cached descriptor tables hold only pointers and shapes and a resample uploads nothing.
// The transfer kernels read both seeds from their (rarely used) table instead.
static void fill_seed(MatDev& M, const flora_matrix_t& f)
{
    M.seed_lo = (uint32_t)(f.seed & 0xffffffffu);
    M.seed_hi = (uint32_t)(f.seed >> 32);
    M.seedn_lo = (uint32_t)(f.seed_next & 0xffffffffu);
    M.seedn_hi = (uint32_t)(f.seed_next >> 32);
}

static void fill_seed_args(SeedArgs& sa, const flora_matrix_t* mats, int count, bool use_next)
{
    for (int l = 0; l < count; ++l) {
        const uint64_t sd = use_next ? mats[l].seed_next : mats[l].seed;
        sa.s[l] = make_uint2((uint32_t)(sd & 0xffffffffu), (uint32_t)(sd >> 32));
    }
}

// ---- one chunk (count <= kMaxSeedArgs) of each entry point; arguments already validated ----
static int compress_chunk(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype, int map,
                          float a, float b, bool use_next, hipStream_t s, bool dry)
{
    std::vector<MatDev> md((size_t)count);
    for (int l = 0; l < count; ++l) {
        MatDev M{};
        M.grad = mats[l].grad; M.state = mats[l].state; M.n = mats[l].n; M.m = mats[l].m;
        md[(size_t)l] = M;
    }
    SeedArgs sa;
    fill_seed_args(sa, mats, count, use_next);
    const int variant = rank_bf16(r) ? (grad_dtype == FLORA_BF16 ? 2 : 3) : (grad_dtype == FLORA_BF16 ? 1 : 0);
    Plan* p = nullptr;
    int st = get_plan(kKindCompress, variant + 4 * map, r, md, s, &p, dry);
    if (st != FLORA_OK || dry) return st;
    const MatDev* dm = p->cur_mats;
    const WorkItem* di = p->d_items;
    if (variant >= 2) {
        float* partials = static_cast<float*>(p->d_work);
        uint32_t* counters = p->d_work ? reinterpret_cast<uint32_t*>(static_cast<char*>(p->d_work) +
                                                                   round_up(p->ws_floats * 4, 256))
                                       : nullptr;
        FLORA_HIP(launch_compress_bf16_mt(dm, di, (int)p->items.size(), sa, r, p->mt, variant == 3, map, a, b,
                                          partials, counters, s));
    }
    else {
        // column groups per workgroup: two for whole rows; one when the pieces are 512 columns
        const int kg = g_tune.compress_f32_kgroups ? g_tune.compress_f32_kgroups : (p->kc > 0 ? 1 : 2);
        float* partials = static_cast<float*>(p->d_work);
        uint32_t* counters = p->d_work ? reinterpret_cast<uint32_t*>(static_cast<char*>(p->d_work) +
                                                                   round_up(p->ws_floats * 4, 256))
                                       : nullptr;
        FLORA_HIP(launch_compress_f32(dm, di, (int)p->items.size(), sa, r, variant == 1, map, a, b, kg, p->mt,
                                      partials, counters, s));
    }
    return FLORA_OK;
}

static int run_decompress(Plan* p, const SeedArgs& sa, int r, int mode, int out_bf16, DecompressParams dp,
                          hipStream_t s)
{
    const MatDev* dm = p->cur_mats;
    const WorkItem* di = p->d_items;
    if (rank_bf16(r)) FLORA_HIP(launch_decompress_bf16(dm, di, (int)p->items.size(), sa, r, mode, out_bf16, p->vec, dp, s));
    else FLORA_HIP(launch_decompress_f32(dm, di, (int)p->items.size(), sa, r, mode, out_bf16, dp, s));
    return FLORA_OK;
}

static int decompress_chunk(const flora_matrix_t* mats, int count, int r, float alpha, void* const* out,
                            flora_dtype_t out_dtype, hipStream_t s, bool dry)
{
    std::vector<MatDev> md((size_t)count);
    for (int l = 0; l < count; ++l) {
        MatDev M{};
        M.state = mats[l].state; M.out = out[l]; M.n = mats[l].n; M.m = mats[l].m;
        md[(size_t)l] = M;
    }
    SeedArgs sa;
    fill_seed_args(sa, mats, count, false);
    Plan* p = nullptr;
    int st = get_plan(kKindDecompress, out_dtype == FLORA_BF16 ? 1 : 0, r, md, s, &p, dry);
    if (st != FLORA_OK || dry) return st;
    DecompressParams dp{alpha, 0.f, 0.f, 0.f, 0};
    return run_decompress(p, sa, r, kModeOut, out_dtype == FLORA_BF16, dp, s);
}

// dst == nullptr: state <- state T in place; else dst[l] <- ca * dst[l] + cb * (state T)
static int transfer_chunk(const flora_matrix_t* mats, int count, int r, float* const* dst, float ca, float cb,
                          hipStream_t s, bool dry)
{
    std::vector<MatDev> md((size_t)count);
    for (int l = 0; l < count; ++l) {
        MatDev M{};
        M.state = mats[l].state; M.n = mats[l].n; M.m = mats[l].m;
        if (dst) M.out = dst[l];
        fill_seed(M, mats[l]);
        md[(size_t)l] = M;
    }
    Plan* p = nullptr;
    int st = get_plan(kKindTransfer, dst ? 1 : 0, r, md, s, &p, dry);
    if (st != FLORA_OK || dry) return st;
    const MatDev* dm = p->cur_mats;
    const WorkItem* di2 = p->d_items2;
    FLORA_HIP(launch_transfer_T(dm, p->d_items, (int)p->items.size(), count, r, s));
    FLORA_HIP(launch_apply_T(dm, di2, (int)p->items2.size(), r, ca, cb, s));
    return FLORA_OK;
}

// Cache policy for the n x m arrays an update call reads and writes once per step (weights,
// elementwise second moment), from their total size over the whole call.  The chip's last-level
// cache is 256 MB.  A set well inside it is found there again by the next step and is accessed
// plainly.  One that does not fit is written with the non-temporal hint (its dirty lines would
// otherwise be written back under the next launches' reads); while it is less than about one
// and a half times the cache, and the compress launches stream their gradients past the cache
// (one rank slice: every rank but 256), part of it is still found there at the next step, so the
// reads stay plain.  Anything larger is read with the hint as well: nothing of it survives.
// Whole steps, same box (plain / streamed writes / both): GPT-2 base, r = 64, 324 MiB: 0.193 /
// 0.171 / 0.190 ms; GPT-2 XL shapes: r = 64, 234 MiB 0.145 / 0.144 / 0.152, 469 MiB 0.308 / 0.300 /
// 0.292, 1875 MiB 1.124 / 1.119 / 1.072; r = 256, 117 MiB 0.148 / 0.150 / 0.154, 234 MiB 0.272 /
// 0.272 / 0.264, 5.6 GiB 3.70 / 3.69 / 3.58.
static int choose_wpolicy(const flora_matrix_t* mats, int count, int r, const flora_update_t* u, int wbf16)
{
    if (g_tune.update_wpolicy) return g_tune.update_wpolicy - 1;
    // bf16 weights: a wave's piece of a row is half a 128-byte line, and the two halves meet in the
    // caches only with plain accesses (GPT-2 XL, 2.8 GiB of bf16 weights: update 1.90 ms plain, 1.91
    // with streamed writes, 2.04 with both)
    if (wbf16) return 0;
    double bytes = 0.0;
    const double per = (wbf16 ? 2.0 : 4.0) + (u->rule == FLORA_RULE_UNFACTORED ? 4.0 : 0.0);
    for (int l = 0; l < count; ++l) bytes += per * (double)mats[l].n * (double)mats[l].m;
    // a caller that spreads one optimizer step over several calls says how large the whole set is
    const double mib = std::max(bytes / (1024.0 * 1024.0), (double)u->step_weight_mib);
    if (mib <= 192.0) return 0;
    if (mib <= 400.0 && r != 256) return 2;
    return 3;
}

static int update_chunk(const flora_matrix_t* mats, int count, int r, int wbf16, const flora_update_t* u,
                        int wpolicy, bool use_next, hipStream_t s, bool dry)
{
    const bool factored = u->rule == FLORA_RULE_FACTORED, unfactored = u->rule == FLORA_RULE_UNFACTORED;
    const bool scaled = (factored || unfactored) && u->scale_parameter != 0;
    std::vector<MatDev> md((size_t)count);
    bool any_sumsq = false;
    for (int l = 0; l < count; ++l) {
        MatDev M{};
        M.weight = mats[l].weight; M.state = mats[l].state;
        M.n = mats[l].n; M.m = mats[l].m;
        if (factored) { M.row_stat = mats[l].row_stat; M.col_stat = mats[l].col_stat; }
        if (unfactored) M.vfull = mats[l].second_moment;
        if (factored || unfactored) M.wsumsq = mats[l].weight_sumsq;
        any_sumsq = any_sumsq || M.wsumsq != nullptr;
        md[(size_t)l] = M;
    }
    SeedArgs sa;
    fill_seed_args(sa, mats, count, use_next);
    Plan* p = nullptr;
    const int kind = (factored || unfactored) ? kKindFactored : kKindDecompress;
    int st = get_plan(kind, (unfactored ? 3 : 2) + (wbf16 ? 4 : 0), r, md, s, &p, dry);
    if (st != FLORA_OK || dry) return st;
    const MatDev* dm = p->cur_mats;
    if (u->rule == FLORA_RULE_SGD) {
        DecompressParams dp{u->alpha, u->lr * u->alpha, 0.f, 0.f, wpolicy};
        st = run_decompress(p, sa, r, kModeSgd, wbf16, dp, s);
        if (st != FLORA_OK) return st;
    } else {
        DecompressParams dp{u->alpha, u->lr, u->beta2, u->eps1, wpolicy};
        const int gram = (factored && p->gram) ? 1 : 0;
        if (gram) {
            // row and column sums of Gt^2 as quadratic forms in A^T A and S^T S, then the clipping
            // sum as one in A^T diag(1 / K) A: no pass over the n x m product before the update
            const WorkItem* gm = p->d_items2;
            const WorkItem* gn = gm + p->n_gm;
            const WorkItem* qr = gn + p->n_gn;
            const WorkItem* qc = qr + p->n_qr;
            // K first (S^T S, then the column sums from regenerated rows of A), because the one further
            // regeneration of A then yields both A^T A and A^T diag(1 / K) A
            const bool clip = u->clip_d > 0.f;
            FLORA_HIP(launch_gram(dm, gn, p->n_gn, count, sa, r, 2, s));
            FLORA_HIP(launch_quadform(dm, qc, p->n_qc, sa, r, 1, u->alpha, u->beta2, u->eps1, s));
            FLORA_HIP(launch_gram(dm, gm, p->n_gm, count, sa, r, clip ? 3 : 0, s));
            FLORA_HIP(launch_quadform(dm, qr, p->n_qr, sa, r, 0, u->alpha, u->beta2, u->eps1, s));
            if (clip) FLORA_HIP(launch_quadform(dm, qr, p->n_qr, sa, r, 2, u->alpha, u->beta2, u->eps1, s));
        } else if (factored) {
            st = run_decompress(p, sa, r, kModeStats, 0, dp, s);
            if (st != FLORA_OK) return st;
            FLORA_HIP(launch_stats_finalize(dm, count, u->beta2, u->eps1, 0, s));
            if (u->clip_d > 0.f) {
                st = run_decompress(p, sa, r, kModeRms, 0, dp, s);
                if (st != FLORA_OK) return st;
            }
        } else {
            st = run_decompress(p, sa, r, kModeFull1, 0, dp, s);
            if (st != FLORA_OK) return st;
        }
        // clip factor from the partial sums of U^2; parameter scale from the caller's sum of W^2
        FLORA_HIP(launch_rms_finalize(dm, count, u->clip_d, scaled ? 1 : 0, u->eps2, gram, s));
        st = run_decompress(p, sa, r, factored ? kModeFactored : kModeFull2, wbf16, dp, s);
        if (st != FLORA_OK) return st;
        // the update pass left per-workgroup sums of the new W^2
        if (any_sumsq) FLORA_HIP(launch_wsumsq_finalize(dm, count, s));
    }
    if (u->zero_state_after) FLORA_HIP(launch_zero_state(dm, count, r, s));
    return FLORA_OK;
}

static int sumsq_chunk(const flora_matrix_t* mats, int count, int wbf16, hipStream_t s, bool dry)
{
    std::vector<MatDev> md((size_t)count);
    for (int l = 0; l < count; ++l) {
        MatDev M{};
        M.weight = mats[l].weight; M.wsumsq = mats[l].weight_sumsq;
        M.n = mats[l].n; M.m = mats[l].m;
        md[(size_t)l] = M;
    }
    Plan* p = nullptr;
    int st = get_plan(kKindSumsq, wbf16, 0, md, s, &p, dry);
    if (st != FLORA_OK || dry) return st;
    FLORA_HIP(launch_weight_sumsq(p->cur_mats, count, wbf16, static_cast<float*>(p->d_work), s));
    return FLORA_OK;
}

// ---- validation of whole calls ----
static int check_grads(const flora_matrix_t* mats, int count, flora_dtype_t grad_dtype)
{
    if (!dtype_ok((int)grad_dtype)) return FLORA_ERR_INVALID;
    for (int l = 0; l < count; ++l)
        if (!mats[l].grad || !aligned16(mats[l].grad) || mats[l].grad == (const void*)mats[l].state)
            return FLORA_ERR_INVALID;
    return FLORA_OK;
}

static int check_update(const flora_matrix_t* mats, int count, int r, flora_dtype_t weight_dtype,
                        const flora_update_t* u)
{
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    if (!u) return FLORA_ERR_INVALID;
    if (!dtype_ok((int)weight_dtype)) return FLORA_ERR_INVALID;
    if (u->rule != FLORA_RULE_SGD && u->rule != FLORA_RULE_FACTORED && u->rule != FLORA_RULE_UNFACTORED)
        return FLORA_ERR_INVALID;
    const bool ada = u->rule != FLORA_RULE_SGD;
    if (ada && (!(u->beta2 >= 0.f && u->beta2 <= 1.f) || !(u->clip_d >= 0.f) || !(u->eps1 >= 0.f)))
        return FLORA_ERR_INVALID;
    if (ada && u->scale_parameter && !(u->eps2 >= 0.f)) return FLORA_ERR_INVALID;
    if (!(u->step_weight_mib >= 0.f) || !std::isfinite(u->step_weight_mib)) return FLORA_ERR_INVALID;
    for (int l = 0; l < count; ++l) {
        if (!mats[l].weight || !aligned16(mats[l].weight) || mats[l].weight == (void*)mats[l].state)
            return FLORA_ERR_INVALID;
        if (u->rule == FLORA_RULE_FACTORED &&
            (!mats[l].row_stat || !mats[l].col_stat || !aligned16(mats[l].row_stat) || !aligned16(mats[l].col_stat)))
            return FLORA_ERR_INVALID;
        if (u->rule == FLORA_RULE_UNFACTORED &&
            (!mats[l].second_moment || !aligned16(mats[l].second_moment) ||
             (void*)mats[l].second_moment == mats[l].weight || mats[l].second_moment == mats[l].state))
            return FLORA_ERR_INVALID;
        if (ada && u->scale_parameter && !mats[l].weight_sumsq) return FLORA_ERR_INVALID;
        if (ada && mats[l].weight_sumsq && (reinterpret_cast<uintptr_t>(mats[l].weight_sumsq) & 3u))
            return FLORA_ERR_INVALID;
    }
    return FLORA_OK;
}

#define FLORA_FOR_CHUNKS(count, c0, cn) \
    for (int c0 = 0, cn = 0; c0 < (count) && ((cn = std::min((count) - c0, kMaxSeedArgs)), true); c0 += cn)

extern "C" {

int flora_compress(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype,
                   float a, float b, void* hip_stream)
{
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    st = check_grads(mats, count, grad_dtype);
    if (st != FLORA_OK) return st;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = compress_chunk(mats + c0, cn, r, grad_dtype, 0, a, b, false, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_compress_mapped(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype,
                          flora_input_map_t map, float a, float b, void* hip_stream)
{
    if ((int)map != FLORA_INPUT_IDENTITY && (int)map != FLORA_INPUT_SQUARE) return FLORA_ERR_INVALID;
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    st = check_grads(mats, count, grad_dtype);
    if (st != FLORA_OK) return st;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = compress_chunk(mats + c0, cn, r, grad_dtype, (int)map, a, b, false, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_decompress(const flora_matrix_t* mats, int count, int r, float alpha, void* const* out,
                     flora_dtype_t out_dtype, void* hip_stream)
{
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    if (!dtype_ok((int)out_dtype)) return FLORA_ERR_INVALID;
    if (count > 0 && !out) return FLORA_ERR_INVALID;
    for (int l = 0; l < count; ++l)
        if (!out[l] || !aligned16(out[l]) || out[l] == (void*)mats[l].state) return FLORA_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = decompress_chunk(mats + c0, cn, r, alpha, out + c0, out_dtype, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_momentum_transfer(const flora_matrix_t* mats, int count, int r, void* hip_stream)
{
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = transfer_chunk(mats + c0, cn, r, nullptr, 0.f, 1.f, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_transfer_accumulate(const flora_matrix_t* mats, int count, int r, float a, float b,
                              float* const* dst, void* hip_stream)
{
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    if (count > 0 && !dst) return FLORA_ERR_INVALID;
    for (int l = 0; l < count; ++l)
        if (!dst[l] || !aligned16(dst[l]) || dst[l] == mats[l].state) return FLORA_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = transfer_chunk(mats + c0, cn, r, dst + c0, a, b, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_apply_update(const flora_matrix_t* mats, int count, int r, flora_dtype_t weight_dtype,
                       const flora_update_t* u, void* hip_stream)
{
    int st = check_update(mats, count, r, weight_dtype, u);
    if (st != FLORA_OK) return st;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int wpolicy = choose_wpolicy(mats, count, r, u, weight_dtype == FLORA_BF16);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = update_chunk(mats + c0, cn, r, weight_dtype == FLORA_BF16, u, wpolicy, false, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_fused_step(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype,
                     flora_dtype_t weight_dtype, float a, float b, int do_transfer,
                     const flora_update_t* u, void* hip_stream)
{
    int st = check_update(mats, count, r, weight_dtype, u);
    if (st != FLORA_OK) return st;
    st = check_grads(mats, count, grad_dtype);
    if (st != FLORA_OK) return st;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool next = do_transfer != 0;
    const int wpolicy = choose_wpolicy(mats, count, r, u, weight_dtype == FLORA_BF16);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            int st2 = FLORA_OK;
            if (next) {
                st2 = transfer_chunk(mats + c0, cn, r, nullptr, 0.f, 1.f, s, dry);
                if (st2 != FLORA_OK) return st2;
            }
            st2 = compress_chunk(mats + c0, cn, r, grad_dtype, 0, a, b, next, s, dry);
            if (st2 != FLORA_OK) return st2;
            st2 = update_chunk(mats + c0, cn, r, weight_dtype == FLORA_BF16, u, wpolicy, next, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

int flora_weight_sumsq(const flora_matrix_t* mats, int count, flora_dtype_t weight_dtype, void* hip_stream)
{
    if (count < 0 || (count > 0 && !mats) || !dtype_ok((int)weight_dtype)) return FLORA_ERR_INVALID;
    for (int l = 0; l < count; ++l) {
        if (mats[l].n < 1 || mats[l].m < 1) return FLORA_ERR_INVALID;
        if (mats[l].n > 0x7fffffffLL - 1024 || mats[l].m > (1LL << 24)) return FLORA_ERR_INVALID;
        if (!mats[l].weight || !aligned16(mats[l].weight)) return FLORA_ERR_INVALID;
        if (!mats[l].weight_sumsq || (reinterpret_cast<uintptr_t>(mats[l].weight_sumsq) & 3u))
            return FLORA_ERR_INVALID;
    }
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return run_call(s, [&](bool dry) {
        FLORA_FOR_CHUNKS(count, c0, cn) {
            const int st2 = sumsq_chunk(mats + c0, cn, weight_dtype == FLORA_BF16, s, dry);
            if (st2 != FLORA_OK) return st2;
        }
        return (int)FLORA_OK;
    });
}

void flora_adafactor_schedule(uint64_t t, float* rho, float* beta2)
{
    const double tt = t < 1 ? 1.0 : (double)t;
    if (rho) *rho = (float)std::min(1e-2, 1.0 / std::sqrt(tt));
    if (beta2) *beta2 = (float)(1.0 - std::pow(tt, -0.8));
}

int flora_debug_generate(uint64_t seed, int64_t m, int r, float* A_out, uint32_t* raw_out, void* hip_stream)
{
    if (m < 0 || r <= 0 || (r % 4) != 0 || r > 1024) return FLORA_ERR_INVALID;
    if ((A_out && !aligned16(A_out)) || (raw_out && !aligned16(raw_out))) return FLORA_ERR_INVALID;
    if (m == 0 || (!A_out && !raw_out)) return FLORA_OK;
    FLORA_HIP(launch_debug_generate(seed, (long long)m, r, A_out, raw_out, static_cast<hipStream_t>(hip_stream)));
    return FLORA_OK;
}

int64_t flora_debug_work_items(int kind, const flora_matrix_t* mats, int count, int r,
                               flora_dtype_t grad_dtype, int64_t* out, int64_t cap, int64_t* info)
{
    if (count < 0 || (count > 0 && !mats) || kind < 0 || kind > 4) return FLORA_ERR_INVALID;
    if (!rank_f32(r) && !rank_bf16(r)) return FLORA_ERR_UNSUPPORTED;
    for (int l = 0; l < count; ++l)
        if (mats[l].n < 1 || mats[l].m < 1 || mats[l].n > 0x7fffffffLL - 1024 || mats[l].m > (1LL << 24))
            return FLORA_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_lock);
    Plan p;
    p.count = count; p.r = r;
    p.host_mats.resize((size_t)count);
    for (int l = 0; l < count; ++l) { p.host_mats[(size_t)l].n = mats[l].n; p.host_mats[(size_t)l].m = mats[l].m; }
    if (kind == 0 || kind == 4) {
        p.kind = kKindCompress;
        p.variant = rank_bf16(r) ? (grad_dtype == FLORA_BF16 ? 2 : 3) : (grad_dtype == FLORA_BF16 ? 1 : 0);
        if (kind == 4) p.variant += 4;
        if ((p.variant & 3) >= 2) build_compress_bf16_items(p);
        else build_compress_f32_items(p);
    } else {
        p.kind = kind == 1 ? kKindDecompress : kKindTransfer;
        if (kind == 1) build_decompress_items(p);
        else if (kind == 2) build_apply_T_items(p);
        else build_transfer_T_items(p);
    }
    const std::vector<WorkItem>& items = (kind == 2) ? p.items2 : p.items;
    if (info) {
        info[0] = p.mt; info[1] = p.vec; info[2] = p.kc;
        info[3] = (int64_t)p.ws_floats; info[4] = (int64_t)p.ws_counters;
    }
    if (out)
        for (size_t i = 0; i < items.size() && (int64_t)i < cap; ++i) {
            const WorkItem& w = items[i];
            int64_t* o = out + 12 * i;
            o[0] = w.mat; o[1] = w.row0; o[2] = w.rows; o[3] = w.col0; o[4] = w.slice; o[5] = w.rblock;
            o[6] = w.col1; o[7] = w.part; o[8] = w.nparts; o[9] = w.cidx; o[10] = w.poff; o[11] = 0;
        }
    return (int64_t)items.size();
}

int flora_debug_copy(const void* src, void* dst, size_t bytes, void* hip_stream)
{
    if (!src || !dst || !aligned16(src) || !aligned16(dst) || (bytes % 16) != 0) return FLORA_ERR_INVALID;
    FLORA_HIP(launch_debug_copy(src, dst, (long long)bytes, static_cast<hipStream_t>(hip_stream)));
    return FLORA_OK;
}

int flora_debug_read(const void* src, size_t bytes, int pattern, size_t row_bytes, int chunk_bytes, void* sink,
                     void* hip_stream)
{
    if (!src || !sink || !aligned16(src) || (bytes % 16) != 0 || (pattern != 0 && pattern != 1)) return FLORA_ERR_INVALID;
    if (pattern == 1 && (row_bytes == 0 || chunk_bytes <= 0 || (chunk_bytes % 256) != 0 || (row_bytes % (size_t)chunk_bytes) != 0 ||
                         (bytes % row_bytes) != 0))
        return FLORA_ERR_INVALID;
    FLORA_HIP(launch_debug_read(src, (long long)bytes, pattern, (long long)row_bytes, chunk_bytes,
                                static_cast<uint32_t*>(sink), static_cast<hipStream_t>(hip_stream)));
    return FLORA_OK;
}

int flora_debug_compute_loop(int kind, int iters, void* sink, double* work_out, void* hip_stream)
{
    if (kind < 0 || kind > 3 || iters < 1 || !sink || !work_out) return FLORA_ERR_INVALID;
    FLORA_HIP(launch_debug_compute_loop(kind, iters, static_cast<float*>(sink), work_out, static_cast<hipStream_t>(hip_stream)));
    return FLORA_OK;
}

uint64_t flora_derive_seed(uint64_t global_seed, uint64_t matrix_id, uint64_t epoch)
{
    const Words4 x = philox4x32_10((uint32_t)matrix_id, (uint32_t)(epoch & 0xffffffffu), (uint32_t)(epoch >> 32),
                                   kDomainSeed, (uint32_t)(global_seed & 0xffffffffu),
                                   (uint32_t)(global_seed >> 32));
    return (uint64_t)x.w[0] | ((uint64_t)x.w[1] << 32);
}

void flora_derive_seeds(uint64_t global_seed, uint64_t first_matrix_id, int count, uint64_t epoch,
                        uint64_t* seeds_out)
{
    if (!seeds_out) return;
    for (int i = 0; i < count; ++i) seeds_out[i] = flora_derive_seed(global_seed, first_matrix_id + (uint64_t)i, epoch);
}

// Bytes of a caller-owned workspace one plan of this kind would occupy (host work only).
static size_t plan_need(int kind, int variant, int r, const flora_matrix_t* mats, int count)
{
    Plan p;
    p.kind = kind; p.variant = variant; p.r = r; p.count = count;
    std::vector<MatDev> md((size_t)count);
    for (int l = 0; l < count; ++l) { md[(size_t)l].n = mats[l].n; md[(size_t)l].m = mats[l].m; }
    build_host_plan(&p, md);
    return arena_need(p);
}

size_t flora_workspace_bytes(const flora_matrix_t* mats, int count, int r)
{
    if (!mats || count <= 0 || r <= 0) return 0;
    if (!rank_f32(r) && !rank_bf16(r)) return 0;
    for (int l = 0; l < count; ++l)
        if (mats[l].n < 1 || mats[l].m < 1 || mats[l].n > 0x7fffffffLL - 1024 || mats[l].m > (1LL << 24)) return 0;
    std::lock_guard<std::mutex> guard(g_lock);      // reads the tuning knobs
    // The most demanding call is flora_fused_step with a transfer and an Adafactor rule: its
    // transfer, compress and update plans are resident together, for every chunk of the call.
    size_t step = 0, sumsq = 0;
    FLORA_FOR_CHUNKS(count, c0, cn) {
        size_t comp = 0;
        if (rank_bf16(r)) comp = std::max(plan_need(kKindCompress, 2, r, mats + c0, cn), plan_need(kKindCompress, 3, r, mats + c0, cn));
        else comp = plan_need(kKindCompress, 0, r, mats + c0, cn);
        step += comp + plan_need(kKindFactored, 2, r, mats + c0, cn) + plan_need(kKindTransfer, 0, r, mats + c0, cn);
        sumsq += plan_need(kKindSumsq, 0, 0, mats + c0, cn);
    }
    return std::max(step, sumsq);
}

int flora_set_workspace(void* dev_ptr, size_t bytes)
{
    if ((dev_ptr == nullptr) != (bytes == 0)) return FLORA_ERR_INVALID;
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255u)) return FLORA_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_lock);
    // plans placed in the old workspace, or in memory of the library's own, are dropped: from here on
    // every plan lives where this call says
    drop_all_plans();
    g_ws = Arena{};
    g_ws.base = static_cast<char*>(dev_ptr);
    g_ws.size = bytes / 256 * 256;
    return FLORA_OK;
}

int64_t flora_debug_plan_bytes(int plan_kind, const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype)
{
    if (count <= 0 || !mats || plan_kind < 0 || plan_kind > 4 || count > kMaxSeedArgs) return FLORA_ERR_INVALID;
    if (plan_kind != 4 && !rank_f32(r) && !rank_bf16(r)) return FLORA_ERR_UNSUPPORTED;
    for (int l = 0; l < count; ++l)
        if (mats[l].n < 1 || mats[l].m < 1 || mats[l].n > 0x7fffffffLL - 1024 || mats[l].m > (1LL << 24))
            return FLORA_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_lock);
    switch (plan_kind) {
    case 0: return (int64_t)plan_need(kKindCompress, rank_bf16(r) ? (grad_dtype == FLORA_BF16 ? 2 : 3) : 0, r, mats, count);
    case 1: return (int64_t)plan_need(kKindDecompress, 0, r, mats, count);
    case 2: return (int64_t)plan_need(kKindTransfer, 0, r, mats, count);
    case 3: return (int64_t)plan_need(kKindFactored, 2, r, mats, count);
    default: return (int64_t)plan_need(kKindSumsq, 0, 0, mats, count);
    }
}

int flora_set_tuning(const char* name, int value)
{
    if (!name) return FLORA_ERR_INVALID;
    std::lock_guard<std::mutex> guard(g_lock);
    const bool pow2_124 = value == 0 || value == 1 || value == 2 || value == 4;
    if (std::strcmp(name, "compress_f32_kgroups") == 0) {
        if (!pow2_124) return FLORA_ERR_INVALID;
        g_tune.compress_f32_kgroups = value;
    } else if (std::strcmp(name, "compress_f32_mt") == 0) {
        if (value != 0 && value != 1 && value != 2) return FLORA_ERR_INVALID;
        g_tune.compress_f32_mt = value;
    } else if (std::strcmp(name, "compress_splitk_cols") == 0) {
        if (value < 0 || (value % 64) != 0) return FLORA_ERR_INVALID;
        g_tune.compress_splitk_cols = value;
    } else if (std::strcmp(name, "compress_bf16_mt") == 0) {
        if (!pow2_124 && value != 8 && value != 16 && value != 32) return FLORA_ERR_INVALID;
        g_tune.compress_bf16_mt = value;
    } else if (std::strcmp(name, "decompress_vec") == 0) {
        if (value < 0 || value > 2) return FLORA_ERR_INVALID;
        g_tune.decompress_vec = value == 0 ? -1 : value - 1;     // 0 default, 1 scalar, 2 vector
    } else if (std::strcmp(name, "update_wpolicy") == 0) {
        if (value < 0 || value > 4) return FLORA_ERR_INVALID;
        g_tune.update_wpolicy = value;
    } else if (std::strcmp(name, "gram_chunk") == 0) {
        if (value < 0 || (value % 64) != 0) return FLORA_ERR_INVALID;
        g_tune.gram_chunk = value;
    } else if (std::strcmp(name, "factored_gram") == 0) {
        if (value < 0 || value > 2) return FLORA_ERR_INVALID;
        g_tune.factored_gram = value;
    } else if (std::strcmp(name, "decompress_rows") == 0) {
        if (value < 0 || (value % 32) != 0) return FLORA_ERR_INVALID;
        g_tune.decompress_rows = value;
    } else {
        return FLORA_ERR_INVALID;
    }
    // cached work tables were built for the old shapes
    drop_all_plans();
    g_ws.used = 0;
    return FLORA_OK;
}

int flora_last_device_error(void) { return g_last_hip_error; }

const char* flora_status_string(int status)
{
    switch (status) {
    case FLORA_OK: return "ok";
    case FLORA_ERR_INVALID: return "invalid argument";
    case FLORA_ERR_UNSUPPORTED: return "unsupported rank or dtype";
    case FLORA_ERR_DEVICE: return "HIP call failed";
    case FLORA_ERR_TOO_LARGE: return "request exceeds the entry point's fixed scratch buffer";
    default: return "unknown status";
    }
}

void flora_shutdown(void)
{
    std::lock_guard<std::mutex> guard(g_lock);
    drop_all_plans();
    g_ws = Arena{};
}

int flora_version(void) { return 400; }

}  // extern "C"

// ---------------------------------------------------------------------------------------------
// flora_momentum_transfer_static: the momentum transfer for callers that cannot allocate.  The
// device memory the transfer needs beyond M itself (descriptor table, work tables, the r x r
// matrices T and their per-chunk partials) lives in this fixed array instead of in allocated
// memory.  Every GPU the library runs on holds its own copy of the array, at its own address,
// until the process ends.
static __device__ __align__(256) unsigned char scratch[FLORA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxScratchDevices = 64;
unsigned char* g_scratch_ptr[kMaxScratchDevices] = {};   // device address of `scratch`, per device
Plan g_static_plan;                                      // host tables of the current call (capacity is reused)
std::vector<char> g_static_stage;                        // image + tables, source of the one upload
}  // namespace

extern "C" int flora_momentum_transfer_static(const flora_matrix_t* mats, int count, int r, void* hip_stream)
{
    int st = check_common(mats, count, r);
    if (st != FLORA_OK) return st;
    if (count == 0) return FLORA_OK;
    if (count > kMaxSeedArgs) return FLORA_ERR_TOO_LARGE;
    std::lock_guard<std::mutex> guard(g_lock);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    // host tables and sizes (no device work yet)
    Plan& p = g_static_plan;
    p.kind = kKindTransfer; p.variant = 0; p.r = r; p.count = count;
    p.items.clear(); p.items2.clear();
    static std::vector<MatDev> md;
    md.assign((size_t)count, MatDev{});
    for (int l = 0; l < count; ++l) {
        MatDev& M = md[(size_t)l];
        M.state = mats[l].state; M.n = mats[l].n; M.m = mats[l].m;
        fill_seed(M, mats[l]);
    }
    build_host_plan(&p, md);
    const size_t need = p.mats_bytes + round_up(p.tbytes, 256) + round_up(p.wbytes, 256);
    if (need > (size_t)FLORA_STATIC_SCRATCH_BYTES) return FLORA_ERR_TOO_LARGE;

    // this device's copy of the array
    int device = 0;
    FLORA_HIP(hipGetDevice(&device));
    if (device < 0 || device >= kMaxScratchDevices) return FLORA_ERR_UNSUPPORTED;
    if (!g_scratch_ptr[device]) {
        void* sp = nullptr;
        FLORA_HIP(hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)));
        g_scratch_ptr[device] = static_cast<unsigned char*>(sp);
    }
    unsigned char* base = g_scratch_ptr[device];
    unsigned char* d_tab = base + p.mats_bytes;
    unsigned char* w = d_tab + round_up(p.tbytes, 256);
    for (int l = 0; l < count; ++l) {
        MatDev& M = md[(size_t)l];
        M.ncolchunks = p.host_mats[(size_t)l].ncolchunks;
        M.T = reinterpret_cast<float*>(w); w += round_up((size_t)r * r * 4, 256);
        if (r >= 64) { M.rowpart = reinterpret_cast<float*>(w); w += round_up((size_t)M.ncolchunks * r * r * 4, 256); }
    }
    // descriptor image and both work tables in one copy from pageable memory (the call returns
    // once the source has been staged, so the buffer can be reused by the next call)
    const size_t up = p.mats_bytes + p.tbytes;
    g_static_stage.assign(up, 0);
    std::memcpy(g_static_stage.data(), md.data(), sizeof(MatDev) * (size_t)count);
    if (!p.items.empty()) std::memcpy(g_static_stage.data() + p.mats_bytes, p.items.data(), sizeof(WorkItem) * p.items.size());
    if (!p.items2.empty())
        std::memcpy(g_static_stage.data() + p.mats_bytes + p.off2, p.items2.data(), sizeof(WorkItem) * p.items2.size());
    FLORA_HIP(hipMemcpyAsync(base, g_static_stage.data(), up, hipMemcpyHostToDevice, s));
    const MatDev* dm = reinterpret_cast<const MatDev*>(base);
    const WorkItem* di = reinterpret_cast<const WorkItem*>(d_tab);
    const WorkItem* di2 = reinterpret_cast<const WorkItem*>(d_tab + p.off2);
    // T and its partials are written in full before they are read: nothing of the previous call's
    // contents is used and nothing needs clearing
    FLORA_HIP(launch_transfer_T(dm, di, (int)p.items.size(), count, r, s));
    FLORA_HIP(launch_apply_T(dm, di2, (int)p.items2.size(), r, 0.f, 1.f, s));
    return FLORA_OK;
}
