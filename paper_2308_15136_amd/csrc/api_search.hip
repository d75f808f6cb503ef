// C ABI: search entry points.  Host-side validation, automatic parameters and launch
// geometry; every step of the search itself runs in the kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstdint>
#include <mutex>

#include "../../include/cagra_hip.h"
#include "device_util.h"
#include "search_params.h"

namespace cagra {

struct DeviceInfo {
    int cus = 0;
    size_t lds_per_cu = 0;
};

// Compute-unit count and LDS size of the current device, asked once per device.
const DeviceInfo &device_info()
{
    static DeviceInfo info[64];
    static std::once_flag once[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    std::call_once(once[dev], [dev]() {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            info[dev].cus = prop.multiProcessorCount;
            info[dev].lds_per_cu = prop.maxSharedMemoryPerMultiProcessor;
        }
        if (info[dev].cus <= 0) info[dev].cus = 256;
        if (info[dev].lds_per_cu < 65536) info[dev].lds_per_cu = 65536;
    });
    return info[dev];
}

static int auto_max_iterations(int itopk, int width) { return 2 * ((itopk + width - 1) / width) + 32; }

// Smallest team whose lanes cover a row in at most four 16-byte loads each (Sec. IV-B.1).
static int auto_team(int chunks)
{
    for (int team = 4; team <= 32; team *= 2)
        if ((chunks + team - 1) / team <= 4) return team;
    return 32;
}

// elements of the dataset's storage type in one 16-byte piece (0 for an unknown type)
static int elems_per_piece(int dataset_type)
{
    return dataset_type == CAGRA_F32 ? 4 : dataset_type == CAGRA_F16 ? 8 : dataset_type == CAGRA_U8 ? 16 : 0;
}

#ifndef CAGRA_SHORT_MAX_ROW_BYTES
#define CAGRA_SHORT_MAX_ROW_BYTES 384
#endif
#ifndef CAGRA_AUTO_SET_TABLE
#define CAGRA_AUTO_SET_TABLE 2560
#endif
constexpr int kAutoSetTableEntries = CAGRA_AUTO_SET_TABLE;

struct SinglePlan {
    int mr, cr, table_words, table_policy, reset_interval, team_log2, max_iterations;
    bool wide;   // more than 256 candidates per pass: taken in chunks of 256
    bool short_rows;   // fp32 rows of at most 384 bytes, up to 64 or 129 to 256 candidates per pass: the kernel variants with one more wavefront per SIMD
    int waves;   // wavefronts per query: 1, or a team of 2 or 4 sharing the visited table
    size_t smem;
    int off_query, off_newid, off_newdist, off_parents;
    int off_team, off_pub, pub_cap;   // wave teams only
};

constexpr int kMaxCandidates = 2048;   // search_width * degree, single mode
constexpr int kMaxWidth = 64;          // parents per pass (their ids sit in a 64-entry LDS array)

static int plan_single(int degree, int dim, int64_t B, int itopk, int width, const cagra_search_opts &o, SinglePlan &pl)
{
    const int pieces = dim / elems_per_piece(o.dataset_type);   // 16-byte pieces per dataset row
    if (itopk > 512) return CAGRA_ERR_BAD_TOPK;
    const int n_cand = width * degree;
    if (n_cand > kMaxCandidates || width > kMaxWidth) return CAGRA_ERR_BAD_TOPK;
    int mr = (itopk + 63) / 64;
    pl.mr = mr <= 1 ? 1 : mr <= 2 ? 2 : mr <= 4 ? 4 : 8;
    pl.cr = n_cand <= 64 ? 1 : n_cand <= 128 ? 2 : 4;
    pl.wide = n_cand > 256;
    pl.short_rows = false;   // decided below, once the table management is known

    int team = o.team_size == 0 ? auto_team(pieces) : o.team_size;
    if (team != 4 && team != 8 && team != 16 && team != 32) return CAGRA_ERR_BAD_OPTION;
    pl.team_log2 = team == 4 ? 2 : team == 8 ? 3 : team == 16 ? 4 : 5;

    if (o.max_iterations < 0) return CAGRA_ERR_BAD_OPTION;
    pl.max_iterations = o.max_iterations == 0 ? auto_max_iterations(itopk, width) : o.max_iterations;

    // Visited table in LDS (Sec. IV-B.3), in one of two managements.
    //  - replacement (default): sets of four ids, a new id replaces the oldest of its set.  Any size
    //    works; automatic size 2560 or 4096 entries (10 or 16 KB plus a byte of cursor per set), see below:
    //    smaller tables forget more, larger ones cost wavefronts per CU.
    //  - periodic reset (the paper's; chosen by table_policy 1, or when hash_bits or reset_interval
    //    are given): open addressing.  Between two resets the table receives at most
    //    itopk + interval * n_cand ids; probing in LDS is cheap, so it may fill up to 7/8.
    if (o.table_policy < 0 || o.table_policy > 2) return CAGRA_ERR_BAD_OPTION;
    if (o.workgroups_per_cu < 0 || o.workgroups_per_cu > 16) return CAGRA_ERR_BAD_OPTION;
    if (o.hash_bits < 0 || o.reset_interval < 0 || o.table_entries < 0) return CAGRA_ERR_BAD_OPTION;
    const bool reset = o.table_policy == 1 || (o.table_policy == 0 && (o.hash_bits != 0 || o.reset_interval != 0));
    if (!reset && (o.hash_bits != 0 || o.reset_interval != 0)) return CAGRA_ERR_BAD_OPTION;
    pl.short_rows = (n_cand <= 64 || (n_cand > 128 && !pl.wide)) && !reset && o.dataset_type == CAGRA_F32 && dim * 4 <= CAGRA_SHORT_MAX_ROW_BYTES && pl.mr <= 2;
    int words;
    if (o.table_entries != 0) {
        if (o.hash_bits != 0 || o.table_entries < 256 || o.table_entries > 8192 || (o.table_entries & 63))
            return CAGRA_ERR_BAD_OPTION;
        words = o.table_entries;
    } else if (o.hash_bits != 0) {
        if (o.hash_bits < 8 || o.hash_bits > 13) return CAGRA_ERR_BAD_OPTION;
        words = 1 << o.hash_bits;
    } else if (reset) {
        const int want = ((itopk + 8 * n_cand) * 8 / 7 + 63) & ~63;
        words = std::min(8192, std::max(4096, want));
    } else {
        // Up to 128 candidates per pass the kernels need few enough registers for three wavefronts per SIMD, so the
        // table is what decides how many fit: 2560 entries leave room for twelve per CU (measured on the 1M x 96
        // workload with 128 candidates per pass: 0.92 ms against 0.98 ms with 3584 entries and nine wavefronts, 0.3 %
        // more distances; on the 1M x 128 workload with 64 candidates per pass the two are level).  Beyond that the
        // candidate buffers and the rows in flight bind the kernel to eight wavefronts per CU, and 4096 entries are
        // the measured optimum (smaller tables forget more, larger ones cost wavefronts).
        words = n_cand <= 128 ? kAutoSetTableEntries : kAutoSetTableEntries + 1536;
        // Rows of the narrow storage types are short: the memory system is not what limits their search, a third
        // wavefront per SIMD is (0.90 against 1.05 ms with byte rows at the benchmark's timed point), and with lists of
        // at most 128 entries the kernels leave registers for it.  2304 entries make the LDS fit twelve per CU.
        if (o.dataset_type != CAGRA_F32 && pl.mr <= 2 && n_cand > 128) words = 2304;
        // With at most 64 candidates per pass their kernels are built for four wavefronts per SIMD (fp16 rows with lists
        // up to 64 entries, byte rows up to 128); 2048 entries let sixteen workgroups share a CU's LDS.
        if (o.dataset_type != CAGRA_F32 && n_cand <= 64 && pl.mr <= (o.dataset_type == CAGRA_F16 ? 1 : 2)) words = 2048;
        // Short fp32 rows: the kernel variants with one more wavefront per SIMD; twelve workgroups per CU with 129 to 256
        // candidates per pass, sixteen with at most 64.
        if (pl.short_rows) words = n_cand <= 64 ? 2048 : 2304;
        // a long query (many dimensions) must not push the workgroup over an eighth of the CU's LDS: the
        // eighth wavefront is worth more than the last 512 table entries
        const size_t rest = (size_t)4 * ((dim + 3) & ~3) + (size_t)8 * 64 * pl.cr + 256;
        while (words > kAutoSetTableEntries + 1024 && (size_t)4 * words + words / 4 + 16 + rest > (size_t)160 * 1024 / 8) words -= 512;
        // (also beyond 256 candidates: measured with 320 to 2048 per pass, larger tables lose more to the
        // wavefronts they displace than they save in distances computed twice)
    }
    pl.table_words = words;
    pl.table_policy = reset ? 1 : 2;
    pl.reset_interval = 0;
    if (reset) {
        // Between two resets the table receives the list (itopk ids) and `interval` passes of candidates; before
        // the first reset, which follows pass `interval`, it receives the seeds and `interval` passes.
        const int capacity = words / 8 * 7;
        int interval = o.reset_interval;
        if (interval == 0) interval = std::min((capacity - itopk) / n_cand, capacity / n_cand - 1);
        if (interval < 1 || itopk + (int64_t)interval * n_cand > capacity ||
            ((int64_t)interval + 1) * n_cand > capacity)
            return CAGRA_ERR_HASH_CAPACITY;
        pl.reset_interval = interval;
    }

    // wavefronts per query (waves_per_query): 0 automatic
    if (o.waves_per_query != 0 && o.waves_per_query != 1 && o.waves_per_query != 2 && o.waves_per_query != 4)
        return CAGRA_ERR_BAD_OPTION;
    if (o.waves_per_query != 0) {
        pl.waves = o.waves_per_query;
        if (pl.waves > 1 && (reset || degree < 2)) return CAGRA_ERR_BAD_OPTION;   // teams share a replacement table
    } else {
        // Automatic: a batch that cannot fill the device with one wavefront per query gets a team per query, which
        // makes every query finish sooner (measured on the 1M x 128 and 1M x 96 workloads: 4 wavefronts are 35 % faster
        // up to two queries per compute unit, 2 wavefronts 15 % up to four); a full device is served best by one
        // wavefront per query.  Below 128 candidates per pass there is too little to share out.
        const int64_t cus = device_info().cus;
        pl.waves = (reset || degree < 2 || n_cand < 128) ? 1 : B <= 2 * cus ? 4 : B <= 4 * cus ? 2 : 1;
    }
    pl.off_team = pl.off_pub = pl.pub_cap = 0;

    size_t off = (size_t)4 * words;
    if (!reset) off += (size_t)(words / 4 + 15) & ~(size_t)15;   // one cursor byte per set of four
    if (pl.waves > 1) {
        // every wavefront of a team stages up to 256 candidates and publishes at most min(256, list) of them
        pl.off_team = (int)off;       off += 64;
        pl.off_query = (int)off;      off += (size_t)4 * ((dim + 3) & ~3);
        pl.off_newid = (int)off;      off += (size_t)4 * 256 * pl.waves;
        pl.off_newdist = (int)off;    off += (size_t)4 * 256 * pl.waves;
        pl.off_parents = (int)off;    off += (size_t)4 * 64;
        pl.pub_cap = std::min(256, 64 * pl.mr);
        pl.off_pub = (int)off;        off += (size_t)8 * 2 * pl.waves * pl.pub_cap;
    } else {
        pl.off_query = (int)off;      off += (size_t)4 * ((dim + 3) & ~3);
        pl.off_newid = (int)off;      off += (size_t)4 * 64 * pl.cr;
        pl.off_newdist = (int)off;    off += (size_t)4 * 64 * pl.cr;
        pl.off_parents = (int)off;    off += (size_t)4 * 64;
    }
    pl.smem = off;
    if (pl.smem > 64 * 1024) return CAGRA_ERR_BAD_SHAPE;  // dim too large for the LDS query copy
    return CAGRA_OK;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Persistent single-wavefront workgroups per compute unit: what the LDS allows (at most 16), or fewer on request.
static int single_per_cu(const cagra_search_opts &o, const SinglePlan &pl, const DeviceInfo &di)
{
    int per_cu = (int)std::min<size_t>(16 / pl.waves, di.lds_per_cu / align256(pl.smem));
    if (o.workgroups_per_cu > 0) per_cu = std::min(per_cu, (int)o.workgroups_per_cu);
    return std::max(per_cu, 1);
}

#ifndef CAGRA_MULTI_TABLE_FACTOR
#define CAGRA_MULTI_TABLE_FACTOR 4
#endif

struct MultiPlan {
    int mr, cr, workers, itopk_local, hash_bits, team_log2, max_iterations;
    // workspace: [256 bytes kept free for the single mode's query counter | done | which | tables | lists | notes]
    size_t smem, table_bytes, list_bytes, done_bytes, note_bytes;
    size_t off_done, off_which, off_tables, off_lists, off_notes, total_bytes;
    int off_query, off_newid, off_newdist, off_parents;
};

// Several workgroups per query (Sec. IV-C.2).  Every worker expands one parent per pass and
// keeps a list of max(k, 32, ceil(itopk / workers)) entries; the shared table is sized for
// at least four times the ids the workers can ever offer (Sec. IV-B.3 asks for twice; the sparser
// table saves second probes, each a round trip to device memory, and a call of one query is
// bound by such round trips).
static int plan_multi(int degree, int dim, int64_t B, int k, int itopk, int width,
                      const cagra_search_opts &o, MultiPlan &pl)
{
    const int pieces = dim / elems_per_piece(o.dataset_type);
    if (o.wg_per_query < 0 || o.wg_per_query > 1024) return CAGRA_ERR_BAD_OPTION;
    if (o.wg_per_query != 0) {
        pl.workers = o.wg_per_query;
    } else {
        // Automatic: at least search_width workers, enough of them that a worker's list stays within one register
        // per lane (64 entries), and for batches below the number of compute units as many as fill the device
        // once (at most 32: beyond that the final merge and the shared table cost more than the workers gain).
        const int64_t fill = std::min<int64_t>(device_info().cus / std::max<int64_t>(B, 1), 32);
        pl.workers = (int)std::min<int64_t>(1024, std::max<int64_t>(std::max(width, (itopk + 63) / 64), fill));
    }
    if (pl.workers > 1024 || B * pl.workers > 0x7FFFFFFFll) return CAGRA_ERR_BAD_OPTION;
    int local = (itopk + pl.workers - 1) / pl.workers;
    local = std::max(local, std::max(k, 32));
    if (local > 512) return CAGRA_ERR_BAD_TOPK;
    if (degree > 256) return CAGRA_ERR_BAD_DEGREE;
    pl.itopk_local = local;
    int mr = (local + 63) / 64;
    pl.mr = mr <= 1 ? 1 : mr <= 2 ? 2 : mr <= 4 ? 4 : 8;
    pl.cr = degree <= 64 ? 1 : degree <= 128 ? 2 : 4;
    int team = o.team_size == 0 ? auto_team(pieces) : o.team_size;
    if (team != 4 && team != 8 && team != 16 && team != 32) return CAGRA_ERR_BAD_OPTION;
    pl.team_log2 = team == 4 ? 2 : team == 8 ? 3 : team == 16 ? 4 : 5;
    if (o.max_iterations < 0) return CAGRA_ERR_BAD_OPTION;
    pl.max_iterations = o.max_iterations == 0 ? auto_max_iterations(local, 1) : o.max_iterations;
    const int64_t offered = (int64_t)pl.workers * degree * ((int64_t)pl.max_iterations + 1);
    int bits = 10;
    while (bits < 27 && ((int64_t)1 << bits) < CAGRA_MULTI_TABLE_FACTOR * offered) ++bits;
    if (bits > 26) return CAGRA_ERR_HASH_CAPACITY;
    pl.hash_bits = bits;
    pl.table_bytes = align256(((size_t)2 * B << bits) * 4);   // two tables per query, used in turn
    pl.list_bytes = align256((size_t)B * pl.workers * 64 * pl.mr * 8);
    pl.done_bytes = align256((size_t)B * 4);
    pl.note_bytes = align256((size_t)B * pl.workers * 8 * 4);
    pl.off_done = 256;
    pl.off_which = pl.off_done + pl.done_bytes;
    pl.off_tables = pl.off_which + pl.done_bytes;
    pl.off_lists = pl.off_tables + pl.table_bytes;
    pl.off_notes = pl.off_lists + pl.list_bytes;
    pl.total_bytes = pl.off_notes + pl.note_bytes;
    size_t off = 0;
    pl.off_query = (int)off;      off += (size_t)4 * ((dim + 3) & ~3);
    pl.off_newid = (int)off;      off += (size_t)4 * 64 * pl.cr;
    pl.off_newdist = (int)off;    off += (size_t)4 * 64 * pl.cr;
    pl.off_parents = (int)off;    off += (size_t)4 * 64;
    pl.smem = off;
    if (pl.smem > 64 * 1024) return CAGRA_ERR_BAD_SHAPE;
    return CAGRA_OK;
}

static int resolve_mode(const cagra_search_opts &o, int64_t B, int itopk)
{
    if (o.mode == 1 || o.mode == 2) return o.mode;
    return (B < device_info().cus || itopk > 512) ? 2 : 1;
}

// ---- scratch for callers that cannot allocate (cagra_search_static) ----------------------------
// One array per GPU, held until the process ends.  In host code the array's name only stands for the
// symbol; its device address is asked once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[CAGRA_STATIC_SCRATCH_BYTES];

static void *static_scratch()
{
    static void *ptr[64] = {};
    static std::once_flag once[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::call_once(once[dev], [dev]() {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) == hipSuccess) ptr[dev] = p;
    });
    return ptr[dev];
}

// Layout (batch size, table size) of the last multi-mode search on this device's static array; a search with the
// same layout finds its tables and tickets clean.  Remembers the new layout.
static bool static_layout_is(int64_t B, int hash_bits)
{
    static int64_t last_b[64];
    static int last_bits[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    const bool same = last_b[dev] == B && last_bits[dev] == hash_bits;
    last_b[dev] = B;
    last_bits[dev] = hash_bits;
    return same;
}

}  // namespace cagra

using namespace cagra;

// Validation, plan and launch of one search.  workspace == kStaticScratch: the scratch memory is this
// device's static array (cagra_search_static), looked up only after every argument check has passed.
static void *const kStaticScratch = reinterpret_cast<void *>(~(uintptr_t)0);

static int search_impl(const uint32_t *graph, int64_t N, int32_t degree, const void *dataset, int32_t dim,
                       int64_t ld, cagra_metric metric, const float *queries, int64_t B, int64_t ld_queries,
                       int32_t k, int32_t itopk, int32_t search_width, const cagra_search_opts &o,
                       uint32_t *ids_out, float *dists_out, void *workspace, size_t workspace_bytes,
                       void *hip_stream, bool init_only = false)
{
    if (!init_only && (!graph || !dataset)) return CAGRA_ERR_NULL_POINTER;
    if (!init_only && B > 0 && (!queries || !ids_out || !dists_out)) return CAGRA_ERR_NULL_POINTER;
    const int epp = elems_per_piece(o.dataset_type);
    if (epp == 0) return CAGRA_ERR_BAD_OPTION;
    if (N < 1 || N > 0x7FFFFFFFll || dim < 1 || dim > 0x7FFFFFFF - 16 || B < 0 || B > 0x7FFFFFFFll || ld_queries < dim)
        return CAGRA_ERR_BAD_SHAPE;
    // The kernels read rows in 16-byte pieces: a row is `dim` rounded up to whole pieces, and the caller vouches that
    // the elements beyond `dim` are zero (they then add nothing to either distance); the query is padded in LDS.
    const int32_t dim_query = dim;
    dim = (dim + epp - 1) / epp * epp;
    if (ld < dim || (ld % epp)) return CAGRA_ERR_BAD_SHAPE;
    if (!init_only && ((uintptr_t)dataset & 15) != 0) return CAGRA_ERR_BAD_SHAPE;
    if (metric != CAGRA_L2 && metric != CAGRA_IP) return CAGRA_ERR_BAD_OPTION;
    if (degree < 1 || degree > 256) return CAGRA_ERR_BAD_DEGREE;
    if (k < 1 || itopk < 1 || k > itopk || search_width < 1) return CAGRA_ERR_BAD_TOPK;
    if (o.mode < 0 || o.mode > 2) return CAGRA_ERR_BAD_OPTION;
    if (B == 0) return CAGRA_OK;
    const int mode = resolve_mode(o, B, itopk);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    SearchParams P = {};
    P.graph = graph; P.dataset = dataset; P.queries = queries;
    P.ids_out = ids_out; P.dists_out = dists_out; P.stats = o.stats;
    P.N = N; P.B = B; P.ld = ld; P.ld_queries = ld_queries; P.seed = o.seed;
    P.degree = degree; P.dim = dim; P.dim_query = dim_query; P.metric = (int)metric; P.k = k;

    if (mode == 2) {
        MultiPlan pl;
        int rc = plan_multi(degree, dim, B, k, itopk, search_width, o, pl);
        if (rc != CAGRA_OK) return rc;
        if (o.workspace_clean != 0 && o.workspace_clean != 1) return CAGRA_ERR_BAD_OPTION;
        bool clean = o.workspace_clean == 1;
        if (workspace == kStaticScratch) {
            if (pl.total_bytes > (size_t)CAGRA_STATIC_SCRATCH_BYTES) return CAGRA_ERR_WORKSPACE;
            if (!(workspace = static_scratch())) return CAGRA_ERR_LAUNCH;
            workspace_bytes = CAGRA_STATIC_SCRATCH_BYTES;
            // The library's own array: it is clean if the last multi-mode search on it had this layout (every search
            // leaves its tables and tickets clean; single-mode searches only touch the first 256 bytes).
            clean = static_layout_is(B, pl.hash_bits);
        }
        if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < pl.total_bytes)
            return CAGRA_ERR_WORKSPACE;
        unsigned char *w = static_cast<unsigned char *>(workspace);
        P.done = reinterpret_cast<uint32_t *>(w + pl.off_done);
        P.which = reinterpret_cast<uint32_t *>(w + pl.off_which);
        P.tables = reinterpret_cast<uint32_t *>(w + pl.off_tables);
        P.lists = reinterpret_cast<uint64_t *>(w + pl.off_lists);
        P.notes = reinterpret_cast<uint32_t *>(w + pl.off_notes);
        P.workspace_clean = clean ? 1 : 0;
        P.itopk = pl.itopk_local; P.search_width = 1; P.workers = pl.workers;
        P.max_iterations = pl.max_iterations; P.reset_interval = 0;
        P.hash_bits = pl.hash_bits; P.team_log2 = pl.team_log2;
        P.off_query = pl.off_query; P.off_newid = pl.off_newid;
        P.off_newdist = pl.off_newdist; P.off_parents = pl.off_parents;
        if (init_only) {
            launch_multi_init(P, stream);
            return hipGetLastError() == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
        }
        hipError_t e = o.dataset_type == CAGRA_F32   ? launch_search_multi_f32(P, pl.mr, pl.cr, pl.smem, stream)
                       : o.dataset_type == CAGRA_F16 ? launch_search_multi_f16(P, pl.mr, pl.cr, pl.smem, stream)
                                                     : launch_search_multi_u8(P, pl.mr, pl.cr, pl.smem, stream);
        return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
    }

    SinglePlan pl;
    int rc = plan_single(degree, dim, B, itopk, search_width, o, pl);
    if (rc != CAGRA_OK) return rc;
    if (init_only) return CAGRA_OK;   // the single mode resets its query counter itself
    if (workspace == kStaticScratch) {
        if (!(workspace = static_scratch())) return CAGRA_ERR_LAUNCH;
        workspace_bytes = CAGRA_STATIC_SCRATCH_BYTES;
    }
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < 256) return CAGRA_ERR_WORKSPACE;
    P.counter = static_cast<uint32_t *>(workspace);
    P.itopk = itopk; P.search_width = search_width; P.workers = 1;
    P.max_iterations = pl.max_iterations; P.reset_interval = pl.reset_interval;
    P.table_words = pl.table_words; P.team_log2 = pl.team_log2;
    P.off_query = pl.off_query; P.off_newid = pl.off_newid;
    P.off_newdist = pl.off_newdist; P.off_parents = pl.off_parents;
    P.off_team = pl.off_team; P.off_pub = pl.off_pub; P.pub_cap = pl.pub_cap;
    P.short_rows = pl.short_rows ? 1 : 0;

    const DeviceInfo &di = device_info();
    // persistent grid: as many workgroups as fit (LDS-bound, at most 16 wavefronts per CU)
    int grid = (int)std::min<int64_t>(B, (int64_t)single_per_cu(o, pl, di) * di.cus);
    hipError_t e;
    if (pl.waves > 1)
        e = o.dataset_type == CAGRA_F32   ? launch_search_team_f32(P, pl.mr, pl.waves, grid, di.cus, pl.smem, stream)
            : o.dataset_type == CAGRA_F16 ? launch_search_team_f16(P, pl.mr, pl.waves, grid, di.cus, pl.smem, stream)
                                          : launch_search_team_u8(P, pl.mr, pl.waves, grid, di.cus, pl.smem, stream);
    else if (pl.wide)
        e = o.dataset_type == CAGRA_F32   ? launch_search_wide_f32(P, pl.mr, grid, pl.smem, stream)
            : o.dataset_type == CAGRA_F16 ? launch_search_wide_f16(P, pl.mr, grid, pl.smem, stream)
                                          : launch_search_wide_u8(P, pl.mr, grid, pl.smem, stream);
    else
        e = o.dataset_type == CAGRA_F32   ? launch_search_single_f32(P, pl.mr, pl.cr, grid, pl.smem, stream)
            : o.dataset_type == CAGRA_F16 ? launch_search_single_f16(P, pl.mr, pl.cr, grid, pl.smem, stream)
                                          : launch_search_single_u8(P, pl.mr, pl.cr, grid, pl.smem, stream);
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

extern "C" {

const char *cagra_strerror(int code)
{
    switch (code) {
        case CAGRA_OK: return "success";
        case CAGRA_ERR_NULL_POINTER: return "a required pointer is NULL";
        case CAGRA_ERR_BAD_SHAPE: return "N, dim, ld or B out of range, or rows not 16-byte aligned";
        case CAGRA_ERR_BAD_DEGREE: return "degree / init_degree not usable";
        case CAGRA_ERR_BAD_TOPK: return "k, itopk or search_width out of range";
        case CAGRA_ERR_BAD_OPTION: return "unsupported value in cagra_search_opts";
        case CAGRA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case CAGRA_ERR_HASH_CAPACITY: return "visited table too small for what it receives between two resets";
        case CAGRA_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown cagra status";
}

uint32_t cagra_seed_id(uint64_t seed, uint64_t query, uint64_t slot, uint64_t N)
{
    return seed_slot_id(seed_query_hash(seed, query), slot, N);
}

int cagra_search_auto_mode(int64_t B, int32_t itopk)
{
    cagra_search_opts o = {};
    return resolve_mode(o, B, itopk);
}

size_t cagra_search_workspace_bytes(int64_t N, int32_t degree, int64_t B, int32_t k, int32_t itopk,
                                    int32_t search_width, const cagra_search_opts *opts)
{
    (void)N;
    cagra_search_opts o = {};
    if (opts) o = *opts;
    if (B < 1 || degree < 1 || k < 1 || itopk < 1 || search_width < 1) return 256;
    if (elems_per_piece(o.dataset_type) == 0) return 256;
    if (resolve_mode(o, B, itopk) == 1) return 256;  // the persistent-scheduling counter
    MultiPlan pl;
    if (plan_multi(degree, 16, B, k, itopk, search_width, o, pl) != CAGRA_OK) return 256;
    return pl.total_bytes;
}

int cagra_search_describe(int32_t degree, int32_t dim, int64_t B, int32_t k, int32_t itopk,
                          int32_t search_width, const cagra_search_opts *opts, cagra_search_plan *plan)
{
    cagra_search_opts o = {};
    if (opts) o = *opts;
    if (!plan) return CAGRA_ERR_NULL_POINTER;
    if (elems_per_piece(o.dataset_type) == 0) return CAGRA_ERR_BAD_OPTION;
    if (dim < 1 || dim > 0x7FFFFFFF - 16 || B < 0) return CAGRA_ERR_BAD_SHAPE;
    dim = (dim + elems_per_piece(o.dataset_type) - 1) / elems_per_piece(o.dataset_type) * elems_per_piece(o.dataset_type);
    if (degree < 1 || degree > 256) return CAGRA_ERR_BAD_DEGREE;
    if (k < 1 || itopk < 1 || k > itopk || search_width < 1) return CAGRA_ERR_BAD_TOPK;
    if (o.mode < 0 || o.mode > 2) return CAGRA_ERR_BAD_OPTION;
    cagra_search_plan out = {};
    out.mode = resolve_mode(o, B, itopk);
    const DeviceInfo &di = device_info();
    if (out.mode == 2) {
        MultiPlan pl;
        int rc = plan_multi(degree, dim, std::max<int64_t>(B, 1), k, itopk, search_width, o, pl);
        if (rc != CAGRA_OK) return rc;
        out.team_size = 1 << pl.team_log2; out.table_entries = 1 << pl.hash_bits; out.reset_interval = 0;
        out.table_policy = 0;
        out.max_iterations = pl.max_iterations; out.wg_per_query = pl.workers; out.itopk_local = pl.itopk_local;
        out.lds_bytes = (int32_t)pl.smem; out.workgroups = (int32_t)(B * pl.workers); out.waves_per_query = 1;
        out.ws_tickets_offset = (int64_t)pl.off_done; out.ws_which_offset = (int64_t)pl.off_which;
        out.ws_tables_offset = (int64_t)pl.off_tables;
    } else {
        SinglePlan pl;
        int rc = plan_single(degree, dim, B, itopk, search_width, o, pl);
        if (rc != CAGRA_OK) return rc;
        out.team_size = 1 << pl.team_log2; out.table_entries = pl.table_words; out.reset_interval = pl.reset_interval;
        out.table_policy = pl.table_policy;
        out.max_iterations = pl.max_iterations; out.wg_per_query = 1; out.itopk_local = itopk;
        out.lds_bytes = (int32_t)pl.smem; out.waves_per_query = pl.waves;
        out.workgroups = (int32_t)std::min<int64_t>(B, (int64_t)single_per_cu(o, pl, di) * di.cus);
    }
    *plan = out;
    return CAGRA_OK;
}

int cagra_search(const uint32_t *graph, int64_t N, int32_t degree, const void *dataset, int32_t dim,
                 int64_t ld, cagra_metric metric, const float *queries, int64_t B, int64_t ld_queries,
                 int32_t k, int32_t itopk, int32_t search_width, const cagra_search_opts *opts,
                 uint32_t *ids_out, float *dists_out, void *workspace, size_t workspace_bytes,
                 void *hip_stream)
{
    cagra_search_opts o = {};
    if (opts) o = *opts;
    if (workspace == kStaticScratch) return CAGRA_ERR_WORKSPACE;
    return search_impl(graph, N, degree, dataset, dim, ld, metric, queries, B, ld_queries, k, itopk, search_width,
                       o, ids_out, dists_out, workspace, workspace_bytes, hip_stream);
}

int cagra_search_workspace_init(int64_t N, int32_t degree, int32_t dim, int64_t B, int32_t k, int32_t itopk,
                                int32_t search_width, const cagra_search_opts *opts, void *workspace,
                                size_t workspace_bytes, void *hip_stream)
{
    cagra_search_opts o = {};
    if (opts) o = *opts;
    if (workspace == kStaticScratch) return CAGRA_ERR_WORKSPACE;
    if (B == 0) return CAGRA_OK;
    o.workspace_clean = 0;
    const int epp = elems_per_piece(o.dataset_type);
    if (epp == 0) return CAGRA_ERR_BAD_OPTION;
    const int64_t ld = dim < 1 ? 0 : ((int64_t)dim + epp - 1) / epp * epp;
    return search_impl(nullptr, N, degree, nullptr, dim, ld, CAGRA_L2, nullptr, B, dim, k, itopk, search_width, o, nullptr,
                       nullptr, workspace, workspace_bytes, hip_stream, true);
}

int cagra_search_static(const uint32_t *graph, int64_t N, int32_t degree, const void *dataset, int32_t dim,
                        int64_t ld, cagra_metric metric, const float *queries, int64_t B, int64_t ld_queries,
                        int32_t k, int32_t itopk, int32_t search_width, const cagra_search_opts *opts,
                        uint32_t *ids_out, float *dists_out, void *hip_stream)
{
    cagra_search_opts o = {};
    if (opts) o = *opts;
    return search_impl(graph, N, degree, dataset, dim, ld, metric, queries, B, ld_queries, k, itopk, search_width,
                       o, ids_out, dists_out, kStaticScratch, 0, hip_stream);
}

int cagra_convert_dataset(const float *src, int64_t N, int32_t dim, int64_t ld_src, cagra_dtype dst_type,
                          void *dst, int64_t ld_dst, void *hip_stream)
{
    if (!src || !dst) return CAGRA_ERR_NULL_POINTER;
    if (dst_type != CAGRA_F32 && dst_type != CAGRA_F16 && dst_type != CAGRA_U8) return CAGRA_ERR_BAD_OPTION;
    if (N < 0 || N > 0x7FFFFFFFll || dim < 1 || ld_src < dim || ld_dst < dim) return CAGRA_ERR_BAD_SHAPE;
    if (N == 0) return CAGRA_OK;
    hipError_t e = launch_convert(src, N, dim, ld_src, (int)dst_type, dst, ld_dst, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

}  // extern "C"
