// libterngrad.so: C ABI of the TernGrad hot path (see include/terngrad.h).
// Host side: argument checks, the plan (offset tables + reduction workspace),
// launch geometry.  Every step of the path runs in the HIP kernels included below.
#include "../../include/terngrad.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "tg_float.hpp"
#include "tg_stats.hpp"
#include "tg_ternarize.hpp"
#include "tg_unpack.hpp"

static_assert(TG_MAX_WORKERS == tg::kMaxWorkers, "header and kernels disagree on the worker limit");

// Workspace of tg_clip_stats_static: the per-segment partial sums, in device memory that exists from
// the moment the library is loaded (every GPU the library runs on holds its own copy until the process
// ends).  In host code this name is only a handle for hipGetSymbolAddress, never an address.
#define TG_STATIC_SCRATCH_BYTES_IMPL (16 * 1024 * 1024)
static __device__ __align__(256) unsigned char scratch[TG_STATIC_SCRATCH_BYTES_IMPL];
static_assert(TG_STATIC_SCRATCH_BYTES_IMPL == TG_STATIC_SCRATCH_BYTES, "header and library disagree on the scratch size");

namespace {

thread_local int g_last_hip_error = 0;

bool hip_ok(hipError_t e) {
    if (e == hipSuccess) return true;
    g_last_hip_error = (int)e;
    (void)hipGetLastError();
    return false;
}

constexpr int64_t kTilePad = 8;

struct Tables {
    int64_t n = 0, n_tiles = 0, chunk = 0;
    std::vector<uint32_t> tile_info;  // [n_tiles + kTilePad]
    std::vector<int32_t> seg_layer;
    std::vector<int64_t> seg_begin, seg_end, seg_pivot;
    std::vector<int64_t> layer_seg;   // [L+1]
    std::vector<tg::StatUnit> units;  // workgroups of the statistics pass (looping shape)
    std::vector<tg::StatChunk> chunks;  // one-shot shape: a record per chunk ...
    std::vector<tg::StatSeg> segs;      // ... and per segment
    bool wide = false;
};

tg_status check_offsets(int64_t n_layers, const int64_t* off) {
    // limits keep every launch below 2^32 threads per grid dimension
    if (n_layers < 1 || n_layers > TG_MAX_LAYERS || off == nullptr) return TG_ERR_INVALID_ARG;
    if (off[0] != 0) return TG_ERR_INVALID_ARG;
    for (int64_t l = 0; l < n_layers; ++l)
        if (off[l + 1] < off[l]) return TG_ERR_INVALID_ARG;
    if (off[n_layers] < 1 || off[n_layers] > TG_MAX_ELEMENTS) return TG_ERR_INVALID_ARG;
    return TG_OK;
}

void build_tables(int64_t L, const int64_t* off, int max_workers, Tables& T) {
    const int64_t n = off[L];
    const int64_t tile = tg::kWaveTile;
    T.n = n;
    T.n_tiles = (n + tile - 1) / tile;
    // One entry per wave tile: the layer of its first element, flagged when no other layer begins
    // inside the tile (elements past n belong to nobody).  The kernels read their entry before they
    // know whether the tile lies past the end, so a few padding entries follow (the code buffers are
    // padded to 16 bytes and the base-3 kernel works in groups of five tiles).
    T.tile_info.resize((size_t)(T.n_tiles + kTilePad));
    int64_t l = 0;
    for (int64_t t = 0; t < T.n_tiles; ++t) {
        const int64_t e = t * tile;
        while (e >= off[l + 1]) ++l;          // e < n = off[L]: stops at the layer that holds e
        const int64_t last = e + tile < n ? e + tile : n;
        T.tile_info[(size_t)t] = (uint32_t)l | (off[l + 1] >= last ? tg::kTileWhole : 0u);
    }
    for (int64_t t = T.n_tiles; t < T.n_tiles + kTilePad; ++t)
        T.tile_info[(size_t)t] = (uint32_t)(L - 1) | tg::kTileWhole;

    // segments = chunks cut at the layer boundaries; returns the number of chunks that hold more than
    // one segment or are ragged
    auto cut = [&](int64_t chunk) {
        T.seg_layer.clear(), T.seg_begin.clear(), T.seg_end.clear(), T.seg_pivot.clear();
        T.layer_seg.assign((size_t)L + 1, 0);
        const int64_t n_chunks = (n + chunk - 1) / chunk;
        int64_t lay = 0, mixed = 0;
        int64_t next_layer_mark = 0;              // layers < this already have layer_seg set
        for (int64_t c = 0; c < n_chunks; ++c) {
            const int64_t cb = c * chunk;
            const int64_t ce = (cb + chunk < n) ? cb + chunk : n;
            int64_t pos = cb, in_chunk = 0;
            while (pos < ce) {
                while (pos >= off[lay + 1]) ++lay;
                const int64_t end = off[lay + 1] < ce ? off[lay + 1] : ce;
                while (next_layer_mark <= lay) T.layer_seg[(size_t)next_layer_mark++] = (int64_t)T.seg_layer.size();
                T.seg_layer.push_back((int32_t)lay);
                T.seg_begin.push_back(pos);
                T.seg_end.push_back(end);
                T.seg_pivot.push_back(off[lay]);
                pos = end;
                ++in_chunk;
            }
            if (in_chunk > 1 || ce - cb < chunk) ++mixed;
        }
        while (next_layer_mark <= L) T.layer_seg[(size_t)next_layer_mark++] = (int64_t)T.seg_layer.size();
        return mixed;
    };
    const int64_t total = n * (int64_t)max_workers;
    if (total >= tg::kStatWideFrom) {
        T.chunk = tg::kStatWideChunk;
        const int64_t mixed = cut(T.chunk);
        T.wide = tg::stat_wide(total, (n + T.chunk - 1) / T.chunk, mixed);
    }
    if (!T.wide) {
        T.chunk = tg::stat_chunk(total);
        cut(T.chunk);
    }
    if (T.wide) {
        // one-shot shape: the segments of chunk c are consecutive, beginning with the first one that
        // starts at or after c * chunk (every chunk below n holds at least one element)
        const int64_t n_chunks = (n + T.chunk - 1) / T.chunk;
        const int64_t n_segs = (int64_t)T.seg_layer.size();
        T.segs.resize((size_t)n_segs);
        T.chunks.resize((size_t)n_chunks);
        for (int64_t i = 0; i < n_segs; ++i) {
            T.segs[(size_t)i] = tg::StatSeg{T.seg_begin[(size_t)i], T.seg_end[(size_t)i], T.seg_pivot[(size_t)i], 0};
            const int64_t c = T.seg_begin[(size_t)i] / T.chunk;
            tg::StatChunk& r = T.chunks[(size_t)c];
            if (r.nseg == 0) {
                r.seg0 = i;
                r.pivot = T.seg_pivot[(size_t)i];
            }
            ++r.nseg;
        }
        return;
    }
    // workgroups: one large segment each, or up to four consecutive small ones (a wave each)
    const int64_t n_segs = (int64_t)T.seg_layer.size();
    for (int64_t i = 0; i < n_segs;) {
        auto small = [&](int64_t k) { return T.seg_end[(size_t)k] - T.seg_begin[(size_t)k] <= tg::kSmallSeg; };
        tg::StatUnit u{};
        int32_t cnt = 1, kind = 0;
        if (small(i)) {
            while (cnt < tg::kBlock / tg::kWave && i + cnt < n_segs && small(i + cnt)) ++cnt;
            kind = cnt;
        }
        for (int32_t j = 0; j < tg::kBlock / tg::kWave; ++j) {
            // slot j is read by wave j: its own small segment, or the one large segment of the unit;
            // unused slots keep an empty range and a valid pivot index
            const int64_t k = kind == 0 ? i : (j < cnt ? i + j : -1);
            u.slot[j].seg_kind = (k < 0 ? 0 : 8 * k) + kind;
            if (k < 0) continue;
            u.slot[j].begin = T.seg_begin[(size_t)k];
            u.slot[j].end = T.seg_end[(size_t)k];
            u.slot[j].pivot = T.seg_pivot[(size_t)k];
        }
        T.units.push_back(u);
        i += cnt;
    }
}

// The address of `scratch` on the current device (each device has its own copy at its own address),
// resolved once per device and kept.  Allocates nothing.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

bool scratch_address(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return false;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || ptr == nullptr) return false;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return true;
}

template <class T>
bool upload(T** dst, const std::vector<T>& src) {
    const size_t bytes = (src.empty() ? 1 : src.size()) * sizeof(T);
    if (!hip_ok(hipMalloc((void**)dst, bytes))) return false;
    if (!src.empty() && !hip_ok(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice))) return false;
    return true;
}

bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

struct tg_plan {
    int64_t n_layers = 0, n = 0, packed_bytes = 0, n_tiles = 0, n_segs = 0, n_units = 0;
    int max_workers = 0;
    bool stat_wide = false;         // statistics pass in its one-shot shape (jobs of max_workers * n elements)
    int update_mode = 0;            // kernel of the fused update: 0 by size, 1 cooperative, 2 quarter tiles
    int device = -1;                // the device that was current at tg_plan_create
    void* d_scratch = nullptr;      // that device's copy of the static scratch array
    int64_t* d_off = nullptr;
    uint32_t* d_tile_info = nullptr;
    tg::StatUnit* d_units = nullptr;
    tg::StatChunk* d_chunks = nullptr;
    tg::StatSeg* d_segs = nullptr;
    int64_t n_chunks = 0;
    uint8_t* d_layer_float = nullptr;                       // [L] when some layer is kept in floating point
    bool any_float = false;                                 // some layer is flagged (it may be empty)
    std::vector<std::pair<int64_t, int64_t>> float_runs;    // their element ranges, maximal and in order
    std::vector<int64_t> off_host;                          // [L+1]
    int64_t* d_layer_seg = nullptr;
    double* d_psum = nullptr;
    double* d_psq = nullptr;
    float* d_pmax = nullptr;
};

static int64_t sum_bytes(const tg_plan* p, int bits) { return ((p->n * bits + 7) / 8 + 15) / 16 * 16; }

// store policy of the decoders' float4 sinks (non-temporal: measured best at every size)
constexpr int kSinkPolicy = tg::ST_NT;

template <int SRC, int DST, int BITS = 0>
static tg_status launch_unpack(const tg::UnpackArgs& a, void* stream) {
    const int64_t blocks = (a.n_wave_tiles + tg::kTilesPerBlock - 1) / tg::kTilesPerBlock;
    hipLaunchKernelGGL((tg::unpack_average_kernel<kSinkPolicy, SRC, DST, BITS>), dim3((unsigned)blocks), dim3(tg::kBlock), 0,
                       (hipStream_t)stream, a);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

// The sinks that read and write the weights.  From 2^28 elements on (1 GiB of weights) a wave per
// quarter tile (see unpack_quarter_kernel): +7 % for the update and +6 % with momentum on 4 * 10^8 and
// 10^9 elements.  Smaller jobs live partly in the 256 MB memory-side cache, where the workgroup-
// cooperative kernel is the faster one (10^8 elements, 8 workers: update 0.141 against 0.168 ms).
constexpr int64_t kQuarterFromElements = (int64_t)1 << 28;

template <int DST>
static tg_status launch_update(tg::UnpackArgs& a, int mode, void* stream) {
    const bool quarter = mode == 2 || (mode == 0 && a.n >= kQuarterFromElements);
    if (!quarter) return launch_unpack<tg::SRC_CODES, DST>(a, stream);
    const int64_t blocks = a.n_wave_tiles;                 // four quarter tiles = four waves per workgroup
    hipLaunchKernelGGL((tg::unpack_quarter_kernel<kSinkPolicy, DST>), dim3((unsigned)blocks), dim3(tg::kBlock), 0,
                       (hipStream_t)stream, a);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

// plain fp32 mean of the slice [first, first + n) of every gradient buffer into avg (which points AT the slice)
static tg_status average_float_launch(int n_workers, int64_t n, const float* const* grads, int64_t first,
                                      float* avg, void* stream) {
    tg::FloatAvgArgs a{};
    // a float layer is usually a slice of a flat buffer: every pointer must be a float address and all
    // must sit at the same position inside a 16-byte line, so that one shift aligns them together
    if (!aligned(avg, 4)) return TG_ERR_ALIGNMENT;
    const uintptr_t phase = ((uintptr_t)avg >> 2) & 3;
    for (int w = 0; w < n_workers; ++w) {
        if (grads[w] == nullptr) return TG_ERR_INVALID_ARG;
        const float* g = grads[w] + first;
        if (!aligned(g, 4) || (((uintptr_t)g >> 2) & 3) != phase) return TG_ERR_ALIGNMENT;
        a.grads[w] = g;
    }
    a.avg = avg;
    a.n = n;
    a.n_workers = n_workers;
    a.head = (int32_t)((4 - phase) & 3);
    const int64_t body = n > a.head ? n - a.head : 0;
    const int64_t threads = (body + 3) / 4;
    int64_t blocks = (threads + tg::kBlock - 1) / tg::kBlock;
    if (blocks < 1) blocks = 1;
    if (blocks > 0x7FFFFFFF) return TG_ERR_INVALID_ARG;
    if (n * (int64_t)sizeof(float) > tg::kCodeStreamNtFrom)
        hipLaunchKernelGGL(tg::average_float_kernel<true>, dim3((unsigned)blocks), dim3(tg::kBlock), 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL(tg::average_float_kernel<false>, dim3((unsigned)blocks), dim3(tg::kBlock), 0, (hipStream_t)stream, a);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

static tg_status fill_unpack(const tg_plan* p, int n_workers, const uint8_t* const* codes, tg::UnpackArgs& a) {
    a.off = p->d_off;
    a.tile_info = p->d_tile_info;
    a.n = p->n;
    a.n_wave_tiles = (p->n + tg::kWaveTile - 1) / tg::kWaveTile;
    a.packed_bytes = p->packed_bytes;
    a.n_layers = (int32_t)p->n_layers;
    a.n_workers = n_workers;
    if (codes != nullptr)
        for (int w = 0; w < n_workers; ++w) {
            if (codes[w] == nullptr) return TG_ERR_INVALID_ARG;
            if (!aligned(codes[w], 4)) return TG_ERR_ALIGNMENT;
            a.codes[w] = codes[w];
        }
    return TG_OK;
}

// a two's-complement field of `bits` bits holds -N .. N when N < 2^(bits-1); 8 bits serve every N <= 64
static bool bits_valid(int bits) { return bits >= 2 && bits <= 8; }
static bool bits_hold(int bits, int n_workers) {
    return bits_valid(bits) && (bits == 8 || n_workers <= (1 << (bits - 1)) - 1);
}

extern "C" {

const char* tg_strerror(int status) {
    switch (status) {
        case TG_OK: return "ok";
        case TG_ERR_INVALID_ARG: return "invalid argument";
        case TG_ERR_ALIGNMENT: return "device pointer not aligned as required";
        case TG_ERR_TOO_MANY_WORKERS: return "too many workers for this plan";
        case TG_ERR_HIP: return "a HIP call failed (see tg_last_hip_error)";
        case TG_ERR_ALLOC: return "allocation failed";
        case TG_ERR_TOO_LARGE: return "job too large for the static scratch buffer";
        default: return "unknown status";
    }
}

int tg_last_hip_error(void) { return g_last_hip_error; }

tg_status tg_describe_tables(int64_t n_layers, const int64_t* offsets, int max_workers,
                             int64_t* tile_elems, int64_t* n_tiles, int32_t* tile_layer, uint8_t* tile_whole, int64_t tile_cap,
                             int64_t* chunk_elems, int64_t* n_segments, int64_t* seg, int64_t seg_cap) {
    const tg_status st = check_offsets(n_layers, offsets);
    if (st != TG_OK) return st;
    if (max_workers < 1 || max_workers > TG_MAX_WORKERS) return TG_ERR_INVALID_ARG;
    Tables T;
    try {
        build_tables(n_layers, offsets, max_workers, T);
    } catch (const std::bad_alloc&) {
        return TG_ERR_ALLOC;
    }
    if (tile_elems) *tile_elems = tg::kWaveTile;
    if (chunk_elems) *chunk_elems = T.chunk;
    if (n_tiles) *n_tiles = T.n_tiles;
    if (n_segments) *n_segments = (int64_t)T.seg_layer.size();
    if (tile_cap >= T.n_tiles)
        for (int64_t t = 0; t < T.n_tiles; ++t) {
            if (tile_layer) tile_layer[t] = (int32_t)(T.tile_info[(size_t)t] & ~tg::kTileWhole);
            if (tile_whole) tile_whole[t] = (T.tile_info[(size_t)t] & tg::kTileWhole) ? 1 : 0;
        }
    if (seg && seg_cap >= (int64_t)T.seg_layer.size())
        for (size_t i = 0; i < T.seg_layer.size(); ++i) {
            seg[3 * i] = T.seg_layer[i];
            seg[3 * i + 1] = T.seg_begin[i];
            seg[3 * i + 2] = T.seg_end[i];
        }
    return TG_OK;
}

tg_status tg_plan_create(int64_t n_layers, const int64_t* offsets, int max_workers, tg_plan** out) {
    if (out == nullptr) return TG_ERR_INVALID_ARG;
    *out = nullptr;
    const tg_status st = check_offsets(n_layers, offsets);
    if (st != TG_OK) return st;
    if (max_workers < 1) return TG_ERR_INVALID_ARG;
    if (max_workers > TG_MAX_WORKERS) return TG_ERR_TOO_MANY_WORKERS;

    Tables T;
    std::vector<int64_t> off;
    tg_plan* p = nullptr;
    try {
        build_tables(n_layers, offsets, max_workers, T);
        off.assign(offsets, offsets + n_layers + 1);
        p = new tg_plan();
        p->off_host = off;
    } catch (const std::bad_alloc&) {
        delete p;
        return TG_ERR_ALLOC;
    }
    // set-up work of tg_clip_stats_static, done here so that the call itself touches no runtime state
    if (!hip_ok(hipGetDevice(&p->device)) || !scratch_address(p->device, &p->d_scratch)) {
        delete p;
        return TG_ERR_HIP;
    }
    p->n_layers = n_layers;
    p->n = T.n;
    p->packed_bytes = (((T.n + 3) / 4) + 15) / 16 * 16;
    p->n_tiles = T.n_tiles;
    p->n_segs = (int64_t)T.seg_layer.size();
    p->n_units = (int64_t)T.units.size();
    p->max_workers = max_workers;
    p->stat_wide = T.wide;
    p->n_chunks = (int64_t)T.chunks.size();

    const size_t np = (size_t)p->n_segs * (size_t)max_workers;
    bool ok = upload(&p->d_off, off) && upload(&p->d_tile_info, T.tile_info) &&
              upload(&p->d_units, T.units) && upload(&p->d_chunks, T.chunks) && upload(&p->d_segs, T.segs) &&
              upload(&p->d_layer_seg, T.layer_seg) &&
              hip_ok(hipMalloc((void**)&p->d_psum, np * sizeof(double))) &&
              hip_ok(hipMalloc((void**)&p->d_psq, np * sizeof(double))) &&
              hip_ok(hipMalloc((void**)&p->d_pmax, np * sizeof(float)));
    if (!ok) {
        const bool oom = g_last_hip_error == (int)hipErrorOutOfMemory;
        tg_plan_destroy(p);
        return oom ? TG_ERR_ALLOC : TG_ERR_HIP;
    }
    *out = p;
    return TG_OK;
}

tg_status tg_plan_destroy(tg_plan* p) {
    if (p == nullptr) return TG_OK;
    void* bufs[] = {p->d_off, p->d_tile_info, p->d_units, p->d_chunks, p->d_segs, p->d_layer_seg, p->d_psum, p->d_psq, p->d_pmax,
                    p->d_layer_float};
    bool ok = true;
    for (void* b : bufs)
        if (b != nullptr) ok = hip_ok(hipFree(b)) && ok;
    delete p;
    return ok ? TG_OK : TG_ERR_HIP;
}

tg_status tg_plan_set_update_kernel(tg_plan* p, int mode) {
    if (p == nullptr || mode < 0 || mode > 2) return TG_ERR_INVALID_ARG;
    p->update_mode = mode;
    return TG_OK;
}

tg_status tg_plan_set_layer_modes(tg_plan* p, const uint8_t* layer_float) {
    if (p == nullptr) return TG_ERR_INVALID_ARG;
    std::vector<std::pair<int64_t, int64_t>> runs;
    std::vector<uint8_t> flags;
    bool any = false;
    try {
        flags.assign((size_t)p->n_layers, 0);
        if (layer_float != nullptr)
            for (int64_t l = 0; l < p->n_layers; ++l) {
                if (layer_float[l] > 1) return TG_ERR_INVALID_ARG;
                flags[(size_t)l] = layer_float[l];
                any = any || layer_float[l] != 0;
                const int64_t b = p->off_host[(size_t)l], e = p->off_host[(size_t)l + 1];
                if (layer_float[l] == 0 || b == e) continue;
                if (!runs.empty() && runs.back().second == b) runs.back().second = e;
                else runs.emplace_back(b, e);
            }
    } catch (const std::bad_alloc&) {
        return TG_ERR_ALLOC;
    }
    if (any || p->d_layer_float != nullptr) {
        // the device copy is written with a blocking copy: calls already queued on a stream must have
        // finished reading the old flags (the caller's duty, as for any change of a plan in use)
        if (p->d_layer_float == nullptr && !hip_ok(hipMalloc((void**)&p->d_layer_float, (size_t)p->n_layers)))
            return TG_ERR_ALLOC;
        if (!hip_ok(hipMemcpy(p->d_layer_float, flags.data(), (size_t)p->n_layers, hipMemcpyHostToDevice))) return TG_ERR_HIP;
    }
    p->float_runs.swap(runs);
    p->any_float = any;
    return TG_OK;
}

int64_t tg_num_elements(const tg_plan* p) { return p ? p->n : -1; }
int64_t tg_num_layers(const tg_plan* p) { return p ? p->n_layers : -1; }
int64_t tg_packed_bytes(const tg_plan* p) { return p ? p->packed_bytes : -1; }

static tg_status check_workers(const tg_plan* p, int n_workers) {
    if (p == nullptr || n_workers < 1) return TG_ERR_INVALID_ARG;
    if (n_workers > p->max_workers || n_workers > TG_MAX_WORKERS) return TG_ERR_TOO_MANY_WORKERS;
    return TG_OK;
}

// the two launches of the statistics pass, with the partial sums in the given workspace
static tg_status clip_stats_launch(tg_plan* p, int n_workers, const float* const* grads, float c,
                                   float* tau, float* s_local, double* psum, double* psq, float* pmax,
                                   void* stream) {
    if (grads == nullptr || tau == nullptr || s_local == nullptr || std::isnan(c)) return TG_ERR_INVALID_ARG;
    const float* checked[TG_MAX_WORKERS];
    for (int w = 0; w < n_workers; ++w) {
        if (grads[w] == nullptr) return TG_ERR_INVALID_ARG;
        if (!aligned(grads[w], 16)) return TG_ERR_ALIGNMENT;
        checked[w] = grads[w];
    }
    if (!aligned(tau, 4) || !aligned(s_local, 4)) return TG_ERR_ALIGNMENT;
    hipStream_t s = (hipStream_t)stream;
    if (p->stat_wide) {
        tg::StatsWideArgs a{};
        for (int w = 0; w < n_workers; ++w) a.grads[w] = checked[w];
        a.chunks = p->d_chunks;
        a.segs = p->d_segs;
        a.psum = psum;
        a.psq = psq;
        a.pmax = pmax;
        a.n_segs = p->n_segs;
        a.n_chunks = p->n_chunks;
        a.n = p->n;
        const int64_t per = (int64_t)tg::kXcds * tg::kStatXcdRun;
        const int64_t blocks = (p->n_chunks + per - 1) / per * per;
        hipLaunchKernelGGL(tg::clip_stats_wide_kernel, dim3((unsigned)blocks, (unsigned)n_workers),
                           dim3(tg::kStatWideBlock), 0, s, a);
    } else {
        tg::StatsArgs a{};
        for (int w = 0; w < n_workers; ++w) a.grads[w] = checked[w];
        a.units = p->d_units;
        a.psum = psum;
        a.psq = psq;
        a.pmax = pmax;
        a.n_segs = p->n_segs;
        hipLaunchKernelGGL(tg::clip_stats_partial_kernel,
                           dim3((unsigned)p->n_units, (unsigned)n_workers), dim3(tg::kBlock), 0, s, a);
    }
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;

    tg::StatsFinalArgs f{};
    f.off = p->d_off;
    f.layer_seg = p->d_layer_seg;
    f.psum = psum;
    f.psq = psq;
    f.pmax = pmax;
    f.tau = tau;
    f.s_local = s_local;
    f.n_segs = p->n_segs;
    f.n_layers = (int32_t)p->n_layers;
    f.c = c;
    f.noclip = (!(c > 0.0f) || std::isinf(c)) ? 1 : 0;
    f.layer_float = p->any_float ? p->d_layer_float : nullptr;
    if (p->n_layers < tg::kFinalPerThreadFrom) {
        hipLaunchKernelGGL(tg::clip_stats_final_kernel, dim3((unsigned)p->n_layers, (unsigned)n_workers),
                           dim3(tg::kFinalBlock), 0, s, f);
    } else {
        const int64_t fblocks = (p->n_layers + tg::kBlock - 1) / tg::kBlock;
        hipLaunchKernelGGL(tg::clip_stats_final_per_thread_kernel, dim3((unsigned)fblocks, (unsigned)n_workers),
                           dim3(tg::kBlock), 0, s, f);
    }
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

tg_status tg_clip_stats(tg_plan* p, int n_workers, const float* const* grads, float c,
                        float* tau, float* s_local, void* stream) {
    const tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    return clip_stats_launch(p, n_workers, grads, c, tau, s_local, p->d_psum, p->d_psq, p->d_pmax, stream);
}

int64_t tg_static_scratch_needed(const tg_plan* p, int n_workers) {
    if (p == nullptr || n_workers < 1 || n_workers > TG_MAX_WORKERS) return -1;
    // [W][n_segs] doubles twice, then [W][n_segs] floats: every part starts on an 8-byte boundary
    return p->n_segs * (int64_t)n_workers * (int64_t)(2 * sizeof(double) + sizeof(float));
}

tg_status tg_clip_stats_static(tg_plan* p, int n_workers, const float* const* grads, float c,
                               float* tau, float* s_local, void* stream) {
    if (p == nullptr || n_workers < 1) return TG_ERR_INVALID_ARG;
    if (n_workers > TG_MAX_WORKERS) return TG_ERR_TOO_MANY_WORKERS;     // the plan's own workspace is not used
    if (tg_static_scratch_needed(p, n_workers) > TG_STATIC_SCRATCH_BYTES) return TG_ERR_TOO_LARGE;
    if (p->d_scratch == nullptr) return TG_ERR_HIP;
    const size_t np = (size_t)p->n_segs * (size_t)n_workers;
    double* psum = reinterpret_cast<double*>(p->d_scratch);
    double* psq = psum + np;
    float* pmax = reinterpret_cast<float*>(psq + np);
    // every partial that the second kernel reads is written by the first one in this call: nothing in
    // the array has to start at zero
    return clip_stats_launch(p, n_workers, grads, c, tau, s_local, psum, psq, pmax, stream);
}

tg_status tg_share_scalers(tg_plan* p, int n_workers, const float* s_local, float* s_shared, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (s_local == nullptr || s_shared == nullptr) return TG_ERR_INVALID_ARG;
    if (!aligned(s_local, 4) || !aligned(s_shared, 4)) return TG_ERR_ALIGNMENT;
    const int L = (int)p->n_layers;
    hipLaunchKernelGGL(tg::share_scalers_kernel, dim3((unsigned)((L + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, s_local, s_shared, n_workers, L);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

static int64_t base3_bytes(const tg_plan* p) { return ((p->n + 4) / 5 + 15) / 16 * 16; }

static tg_status ternarize_launch(tg_plan* p, int n_workers, uint32_t worker_base,
                                  const float* const* grads, const float* tau, const float* s_shared,
                                  uint64_t seed, uint32_t step, const uint32_t* step_dev,
                                  uint8_t* const* codes, void* stream, bool base3 = false) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (grads == nullptr || codes == nullptr || tau == nullptr || s_shared == nullptr) return TG_ERR_INVALID_ARG;
    tg::TernArgs a{};
    for (int w = 0; w < n_workers; ++w) {
        if (grads[w] == nullptr || codes[w] == nullptr) return TG_ERR_INVALID_ARG;
        if (!aligned(grads[w], 16) || !aligned(codes[w], 4)) return TG_ERR_ALIGNMENT;
        a.grads[w] = grads[w];
        a.codes[w] = codes[w];
    }
    if (!aligned(tau, 4) || !aligned(s_shared, 4)) return TG_ERR_ALIGNMENT;
    a.tau = tau;
    a.s_shared = s_shared;
    a.off = p->d_off;
    a.tile_info = p->d_tile_info;
    a.n = p->n;
    a.packed_bytes = p->packed_bytes;
    a.n_wave_tiles = (p->packed_bytes * 4 + tg::kWaveTile - 1) / tg::kWaveTile;
    a.n_layers = (int32_t)p->n_layers;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.step = step;
    a.step_dev = step_dev;
    a.worker_base = worker_base;
    if (base3) {
        a.packed_bytes = base3_bytes(p);
        const int64_t b3 = (a.packed_bytes + 1023) / 1024;
        const dim3 g3((unsigned)b3, (unsigned)n_workers), t3(tg::kBase3Block);
        if (a.packed_bytes * n_workers > tg::kCodeStreamNtFrom)
            hipLaunchKernelGGL(tg::ternarize_pack_base3_kernel<true>, g3, t3, 0, (hipStream_t)stream, a);
        else
            hipLaunchKernelGGL(tg::ternarize_pack_base3_kernel<false>, g3, t3, 0, (hipStream_t)stream, a);
        if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
        return TG_OK;
    }
    // a wave per half tile: four half tiles per workgroup
    int64_t blocks = (2 * a.n_wave_tiles + tg::kBlock / tg::kWave - 1) / (tg::kBlock / tg::kWave);
    // whole groups of 8 XCDs x kEncoderXcdRun workgroups (the kernel skips what lies past the last tile)
    constexpr int64_t group = (int64_t)tg::kXcds * tg::kEncoderXcdRun;
    blocks = (blocks + group - 1) / group * group;
    // cache policy of the code stream by the size of the job (see store_through)
    const dim3 grid((unsigned)blocks, (unsigned)n_workers), block(tg::kBlock);
    if (a.packed_bytes * n_workers > tg::kCodeStreamNtFrom)
        hipLaunchKernelGGL(tg::ternarize_pack_kernel<true>, grid, block, 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL(tg::ternarize_pack_kernel<false>, grid, block, 0, (hipStream_t)stream, a);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

tg_status tg_ternarize_pack(tg_plan* p, int n_workers, uint32_t worker_base,
                            const float* const* grads, const float* tau, const float* s_shared,
                            uint64_t seed, uint32_t step, uint8_t* const* codes, void* stream) {
    return ternarize_launch(p, n_workers, worker_base, grads, tau, s_shared, seed, step, nullptr, codes, stream);
}

tg_status tg_ternarize_pack_devstep(tg_plan* p, int n_workers, uint32_t worker_base,
                                    const float* const* grads, const float* tau, const float* s_shared,
                                    uint64_t seed, const uint32_t* step_dev, uint8_t* const* codes, void* stream) {
    if (step_dev == nullptr) return TG_ERR_INVALID_ARG;
    if (!aligned(step_dev, 4)) return TG_ERR_ALIGNMENT;
    return ternarize_launch(p, n_workers, worker_base, grads, tau, s_shared, seed, 0u, step_dev, codes, stream);
}

int64_t tg_packed_bytes_base3(const tg_plan* p) { return p ? base3_bytes(p) : -1; }

tg_status tg_ternarize_pack_base3(tg_plan* p, int n_workers, uint32_t worker_base,
                                  const float* const* grads, const float* tau, const float* s_shared,
                                  uint64_t seed, uint32_t step, uint8_t* const* codes3, void* stream) {
    return ternarize_launch(p, n_workers, worker_base, grads, tau, s_shared, seed, step, nullptr, codes3, stream, true);
}

tg_status tg_unpack_average_base3(tg_plan* p, int n_workers, const uint8_t* const* codes3,
                                  const float* s_shared, float* avg, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (codes3 == nullptr || s_shared == nullptr || avg == nullptr) return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    if ((st = fill_unpack(p, n_workers, codes3, a)) != TG_OK) return st;
    if (!aligned(s_shared, 4) || !aligned(avg, 16)) return TG_ERR_ALIGNMENT;
    a.s_shared = s_shared;
    a.avg = avg;
    a.packed_bytes = base3_bytes(p);
    const int64_t blocks = (p->n + tg::kBase3Elems - 1) / tg::kBase3Elems;
    hipLaunchKernelGGL((tg::unpack_average_base3_kernel<kSinkPolicy, tg::DST_AVG>), dim3((unsigned)blocks),
                       dim3(tg::kBase3Block), 0, (hipStream_t)stream, a);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

tg_status tg_step_advance(uint32_t* step_dev, uint32_t by, void* stream) {
    if (step_dev == nullptr) return TG_ERR_INVALID_ARG;
    if (!aligned(step_dev, 4)) return TG_ERR_ALIGNMENT;
    hipLaunchKernelGGL(tg::step_advance_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, step_dev, by);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

tg_status tg_unpack_average(tg_plan* p, int n_workers, const uint8_t* const* codes,
                            const float* s_shared, float* avg, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (codes == nullptr || s_shared == nullptr || avg == nullptr) return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    if ((st = fill_unpack(p, n_workers, codes, a)) != TG_OK) return st;
    if (!aligned(s_shared, 4) || !aligned(avg, 16)) return TG_ERR_ALIGNMENT;
    a.s_shared = s_shared;
    a.avg = avg;
    return launch_unpack<tg::SRC_CODES, tg::DST_AVG>(a, stream);
}

tg_status tg_unpack_average_scalers(tg_plan* p, int n_workers, const uint8_t* const* codes,
                                    const float* s_workers, float* avg, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (codes == nullptr || s_workers == nullptr || avg == nullptr) return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    if ((st = fill_unpack(p, n_workers, codes, a)) != TG_OK) return st;
    if (!aligned(s_workers, 4) || !aligned(avg, 16)) return TG_ERR_ALIGNMENT;
    a.s_workers = s_workers;
    a.avg = avg;
    const int64_t blocks = (a.n_wave_tiles + tg::kTilesPerBlock - 1) / tg::kTilesPerBlock;
    hipLaunchKernelGGL((tg::unpack_average_scalers_kernel<kSinkPolicy>), dim3((unsigned)blocks), dim3(tg::kBlock), 0,
                       (hipStream_t)stream, a);
    if (!hip_ok(hipGetLastError())) return TG_ERR_HIP;
    return TG_OK;
}

tg_status tg_unpack_update(tg_plan* p, int n_workers, const uint8_t* const* codes,
                           const float* s_shared, float eta, float* weights, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (codes == nullptr || s_shared == nullptr || weights == nullptr || std::isnan(eta) || std::isinf(eta))
        return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    if ((st = fill_unpack(p, n_workers, codes, a)) != TG_OK) return st;
    if (!aligned(s_shared, 4) || !aligned(weights, 16)) return TG_ERR_ALIGNMENT;
    a.s_shared = s_shared;
    a.avg = weights;
    a.eta = eta;
    return launch_update<tg::DST_UPDATE>(a, p->update_mode, stream);
}

tg_status tg_unpack_update_momentum(tg_plan* p, int n_workers, const uint8_t* const* codes,
                                    const float* s_shared, float eta, float mu, float* velocity,
                                    float* weights, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (codes == nullptr || s_shared == nullptr || weights == nullptr || velocity == nullptr ||
        !std::isfinite(eta) || !std::isfinite(mu) || velocity == weights)
        return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    if ((st = fill_unpack(p, n_workers, codes, a)) != TG_OK) return st;
    if (!aligned(s_shared, 4) || !aligned(weights, 16) || !aligned(velocity, 16)) return TG_ERR_ALIGNMENT;
    a.s_shared = s_shared;
    a.avg = weights;
    a.velocity = velocity;
    a.eta = eta;
    a.mu = mu;
    return launch_update<tg::DST_MOMENTUM>(a, p->update_mode, stream);
}

int tg_sum_bits(int n_workers) {
    if (n_workers < 1 || n_workers > TG_MAX_WORKERS) return -1;
    int bits = 2;
    while ((1 << bits) < 2 * n_workers + 1) ++bits;
    return bits;
}

int64_t tg_sum_bytes(const tg_plan* p, int bits) {
    if (p == nullptr || !bits_valid(bits)) return -1;
    return sum_bytes(p, bits);
}

tg_status tg_unpack_sum_pack(tg_plan* p, int n_workers, const uint8_t* const* codes, int bits,
                             uint8_t* ksum, void* stream) {
    tg_status st = check_workers(p, n_workers);
    if (st != TG_OK) return st;
    if (codes == nullptr || ksum == nullptr || !bits_hold(bits, n_workers))
        return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    if ((st = fill_unpack(p, n_workers, codes, a)) != TG_OK) return st;
    if (!aligned(ksum, 16)) return TG_ERR_ALIGNMENT;
    a.ksum_out = ksum;
    a.ksum_bytes = sum_bytes(p, bits);
    // the tiles must cover the pad fields too
    a.n_wave_tiles = (a.ksum_bytes * 8 / bits + tg::kWaveTile - 1) / tg::kWaveTile;
    switch (bits) {
        case 4: return launch_unpack<tg::SRC_CODES, tg::DST_K4>(a, stream);
        case 8: return launch_unpack<tg::SRC_CODES, tg::DST_K8>(a, stream);
        case 2: return launch_unpack<tg::SRC_CODES, tg::DST_KB, 2>(a, stream);
        case 3: return launch_unpack<tg::SRC_CODES, tg::DST_KB, 3>(a, stream);
        case 5: return launch_unpack<tg::SRC_CODES, tg::DST_KB, 5>(a, stream);
        case 6: return launch_unpack<tg::SRC_CODES, tg::DST_KB, 6>(a, stream);
        default: return launch_unpack<tg::SRC_CODES, tg::DST_KB, 7>(a, stream);
    }
}

tg_status tg_decode_sum(tg_plan* p, int n_workers, const uint8_t* ksum, int bits,
                        const float* s_shared, float* avg, void* stream) {
    if (p == nullptr || n_workers < 1) return TG_ERR_INVALID_ARG;
    if (n_workers > TG_MAX_WORKERS) return TG_ERR_TOO_MANY_WORKERS;
    if (ksum == nullptr || s_shared == nullptr || avg == nullptr || !bits_hold(bits, n_workers))
        return TG_ERR_INVALID_ARG;
    tg::UnpackArgs a{};
    tg_status st = fill_unpack(p, n_workers, nullptr, a);
    if (st != TG_OK) return st;
    if (!aligned(ksum, 16) || !aligned(s_shared, 4) || !aligned(avg, 16)) return TG_ERR_ALIGNMENT;
    a.ksum_in = ksum;
    a.ksum_bytes = sum_bytes(p, bits);
    a.s_shared = s_shared;
    a.avg = avg;
    switch (bits) {
        case 4: return launch_unpack<tg::SRC_K4, tg::DST_AVG>(a, stream);
        case 8: return launch_unpack<tg::SRC_K8, tg::DST_AVG>(a, stream);
        case 2: return launch_unpack<tg::SRC_KB, tg::DST_AVG, 2>(a, stream);
        case 3: return launch_unpack<tg::SRC_KB, tg::DST_AVG, 3>(a, stream);
        case 5: return launch_unpack<tg::SRC_KB, tg::DST_AVG, 5>(a, stream);
        case 6: return launch_unpack<tg::SRC_KB, tg::DST_AVG, 6>(a, stream);
        default: return launch_unpack<tg::SRC_KB, tg::DST_AVG, 7>(a, stream);
    }
}

tg_status tg_average_float(int n_workers, int64_t n, const float* const* grads, float* avg, void* stream) {
    if (n_workers < 1 || n < 1 || grads == nullptr || avg == nullptr) return TG_ERR_INVALID_ARG;
    if (n_workers > TG_MAX_WORKERS) return TG_ERR_TOO_MANY_WORKERS;
    return average_float_launch(n_workers, n, grads, 0, avg, stream);
}

tg_status tg_unpack_average_mixed(tg_plan* p, int n_workers, const uint8_t* const* codes, const float* const* grads,
                                  const float* s_shared, float* avg, void* stream) {
    if (p != nullptr && !p->float_runs.empty() && grads == nullptr) return TG_ERR_INVALID_ARG;
    if (p != nullptr && !p->float_runs.empty())
        for (int w = 0; w < n_workers && w < TG_MAX_WORKERS; ++w)
            if (grads[w] == nullptr) return TG_ERR_INVALID_ARG;
    tg_status st = tg_unpack_average(p, n_workers, codes, s_shared, avg, stream);
    if (st != TG_OK) return st;
    // the layers kept in floating point (they came out as zeros above): the plain mean of the gradients
    for (const auto& r : p->float_runs)
        if ((st = average_float_launch(n_workers, r.second - r.first, grads, r.first, avg + r.first, stream)) != TG_OK) return st;
    return TG_OK;
}

}  // extern "C"
