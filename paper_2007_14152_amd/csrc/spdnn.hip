// Host side of the spdnn C-ABI (see include/spdnn.h): argument checks, arena
// carving, weight set-up, and the per-layer launch loop.  Every arithmetic step
// of the inference runs in the kernels of spdnn_kernels.h.
#include "../../include/spdnn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "spdnn_kernels.h"
#include "spdnn_cut.h"

// Work memory of spdnn_infer_static, the entry point for callers that cannot allocate: a fixed array in
// every GPU's memory instead of a caller-made work arena.  In host code this name is only a stand-in for
// the symbol; the device address comes from hipGetSymbolAddress (see static_scratch()).
constexpr size_t kStaticScratchBytes = SPDNN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int static_scratch(void** out);  // defined below

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(SPDNN_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),    \
                        __FILE__, __LINE__);                                                  \
    } while (0)

constexpr size_t kAlign = 256;
inline size_t up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

constexpr int kLag = 2;  // the host runs at most this many layers ahead of the GPU
// Set-up of device-resident layers runs on this many streams, a layer per stream in turn: its kernels
// are single-wave, latency-bound searches that fill a fraction of the chip, so several layers overlap.
constexpr int kSetupStreams = 8;

enum LayerMode { kSingle = 0, kStaged = 1, kWide = 2, kPair = 3, kWidePair = 4, kRow2 = 5 };
struct LayerDesc {
    spdnn::LayerWeights w;
    spdnn::WideWeights ww;
    spdnn::Row2Weights r2;
    uint16_t* r2_codes = nullptr;  // arena room for the two-row-tile format (NULL: none)
    int32_t* r2_map = nullptr;
    int* r2_ngroups = nullptr;
    // kRow2: one weight for the whole layer, N a multiple of 4096, every 4096-neuron unit's window within 16384
    // columns but wider than one LDS stage: four neurons per lane, two rows per tile (fused_row2_kernel);
    // kSingle: every window fits one LDS stage; kStaged: 2 stages (or fallback); kWide: 3+ stages;
    // kPair: one stage, one weight for the whole layer, two output neurons per lane; kWidePair: the same for 3-8 stages
    int mode;
    int lds_cols;  // columns the LDS tile must hold for this layer
    float wuni;    // kPair, kWidePair: the layer's weight
    bool pair4;    // kWidePair: 3 or 4 stages -> slot lists resident in registers
    bool multi;    // one of several launches of a layer with more than 32 connections per neuron: each computes the
                   // outputs of a slice of the neurons, several lanes per neuron (spdnn::VirtInfo)
    spdnn::VirtInfo virt;
    int virt_lanes = 1;  // multi: lanes of the layer's longest neuron (the layer's passes)
    int virt_blocks = 0;  // multi: workgroups of this launch that have neurons
    bool relabel = false;  // kPair under new names for neurons and columns (spdnn::PairRelabel)
    spdnn::PairRelabel rn{};
};

}  // namespace

struct spdnn_model {
    int32_t N = 0, L = 0, nblk = 0, G = 1;
    hipStream_t stream = nullptr;
    int num_cu = 256;
    const float* bias_dev = nullptr;
    std::vector<LayerDesc> layers;     // one per pass (launch); a layer is one pass unless some neuron has more than 32 connections
    std::vector<int32_t> first_pass;   // L+1 entries: layer l is passes first_pass[l] .. first_pass[l+1]-1
    int* host_counts = nullptr;  // pinned, L+1 entries: rows active on entry to layer l
    // all layers in one launch (fused_chain_kernel): possible if every layer is a single-stage layer of one output block
    const spdnn::LayerWeights* chain_layers = nullptr;  // device copy of the layers' descriptors (NULL: not possible)
    int* chain_rows = nullptr;                          // device, L + 1 counters
    int chain_lds_cols = 0;
    // out-of-core weights: pass p's block lives in host memory and is copied into device slot p & 1
    const char* ooc_host = nullptr;
    char* ooc_slot[2] = {nullptr, nullptr};
    size_t ooc_block = 0;
    hipStream_t ooc_stream = nullptr;
    hipEvent_t ooc_ready[2] = {nullptr, nullptr};  // the copy into the slot has landed
    hipEvent_t ooc_freed[2] = {nullptr, nullptr};  // the kernels that read the slot are done
    // inputs in host memory (spdnn_infer_host): copy stream and "batch has landed" events, made on first use
    hipStream_t in_stream = nullptr;
    hipEvent_t in_ready[2] = {nullptr, nullptr};
    // profiling
    int profiling = 0;
    std::vector<hipEvent_t> t0, t1;
    int32_t prof_layers = 0;
    std::vector<float> prof_ms;
    std::vector<int32_t> prof_rows;
};

namespace {

bool valid_n(int32_t N) { return N >= 32 && N <= 65536 && (N % 4) == 0; }

size_t layer_bytes(int32_t nblk) {
    const size_t e = (size_t)nblk * spdnn::kNnz * spdnn::kBlk;
    return up((size_t)nblk * sizeof(int2)) + up(e * sizeof(uint16_t)) + up(e * sizeof(float)) +
           up((size_t)nblk * spdnn::kBlk * sizeof(uint32_t)) +
           // several lanes per neuron: slots, steps per wave, neurons per workgroup, slots per neuron
           up((size_t)nblk * spdnn::kBlk * sizeof(uint16_t)) + up((size_t)nblk * 16) + up((size_t)nblk * sizeof(int2)) +
           up((size_t)nblk * spdnn::kBlk * sizeof(uint32_t));
}
int stages_of(int32_t window) { return (window + spdnn::kCap - 1) / spdnn::kCap; }
// extra bytes per layer for the wide format with up to `nstage` stages (0 if not needed)
// Steps per neuron the wide format needs at most, for a layer of 2 .. nstage stages (an
// arena sized for nstage stages also holds layers with fewer, which may use more steps per stage).
size_t wide_steps_max(int nstage) {
    size_t m = 0;
    for (int n = 2; n <= nstage; ++n) m = std::max(m, (size_t)n * spdnn::wide_steps(n));
    return m;
}
bool wide_has_slots(int nstage) { return nstage <= 8; }  // the compact 16-bit form exists for 2..8 stages
// the two-row-tile format (fused_row2_kernel): step codes, gathered-footprint list, groups per unit
size_t row2_bytes(int32_t nblk) {
    if (nblk % 4) return 0;
    const size_t nunit = nblk / 4;
    return up((size_t)nblk * spdnn::kBlk * spdnn::kNnz * sizeof(uint16_t)) +
           up(nunit * (spdnn::kRow2Cols / 4) * sizeof(int32_t)) + up(nunit * sizeof(int));
}
size_t wide_bytes(int32_t nblk, int nstage) {
    if (nstage < 2) return 0;
    const size_t e = (size_t)nblk * wide_steps_max(nstage) * spdnn::kBlk;
    const size_t sp = (size_t)nblk * spdnn::kSpill * spdnn::kBlk;
    return up(e * sizeof(uint2)) + up((size_t)nblk * nstage * 16) + up(sp * sizeof(uint16_t)) +
           up(sp * sizeof(float)) + up((size_t)nblk * 16) +
           (wide_has_slots(nstage) ? up(e * sizeof(uint16_t)) + up(sp * sizeof(uint16_t))
                                   : 0) +  // compact slots and spills
           row2_bytes(nblk);
}
size_t staging_bytes(int32_t N, int32_t L) {
    const int32_t nblk = (N + spdnn::kBlk - 1) / spdnn::kBlk;
    const size_t lanes = (size_t)nblk * spdnn::kBlk;  // rows of the staging arrays: the lanes of a launch
    return up(lanes * spdnn::kNnz * sizeof(int32_t)) + up(lanes * spdnn::kNnz * sizeof(float)) + up(lanes) +
           kSetupStreams * up((size_t)nblk * spdnn::kCap * sizeof(uint16_t)) +  // column -> LDS slot tables of the layers being set up
           up(sizeof(int) * (size_t)nblk) +                     // general layers: smallest column of every block
           up(sizeof(int) * (size_t)(5 * L + 1));  // error flag; per layer: wide failure, widest window, weights differ, pair info[2]
}
size_t block_bytes(int32_t N, int nstage_cap) {  // one pass's re-laid weights
    const int32_t nblk = (N + spdnn::kBlk - 1) / spdnn::kBlk;
    return layer_bytes(nblk) + wide_bytes(nblk, nstage_cap);
}
size_t chain_bytes(int32_t L) {  // all layers in one launch: the layers' descriptors and the rows-per-layer counters
    return up((size_t)L * sizeof(spdnn::LayerWeights)) + up(((size_t)L + 1) * sizeof(int));
}
size_t arena_bytes_for(int32_t N, int32_t L, int nstage_cap) {
    return up((size_t)N * sizeof(float)) + (size_t)L * block_bytes(N, nstage_cap) + staging_bytes(N, L) + chain_bytes(L);
}
// out-of-core: the device holds the bias, two blocks and the staging area; the host holds all blocks
size_t ooc_device_bytes_for(int32_t N, int32_t L, int nstage_cap) {
    return up((size_t)N * sizeof(float)) + 2 * block_bytes(N, nstage_cap) + staging_bytes(N, L) + chain_bytes(L);
}

struct WorkView {
    float* Y[2];
    int* cat[2];        // layer l writes and reads cat[l & 1]: slots, in layer l-1's buffer, of the rows active on entry
    int* gid[2];        // gid[l & 1]: their original row numbers (derived from gid[(l + 1) & 1], layer l-1's)
    uint8_t* flags[3];  // one byte per row; layer l raises flags[l % 3], reads flags[(l + 2) % 3] (layer l-1's) and
                        // clears flags[(l + 1) % 3] for layer l+1
    int* count[2];      // count[l & 1]: rows active on entry to layer l, written by layer l's kernel
};
size_t carve_work(int32_t N, int32_t batch, char* base, WorkView* v) {
    size_t o = 0;
    const size_t yb = up((size_t)batch * N * sizeof(float));
    const size_t lb = up(((size_t)batch + 4) * sizeof(int));  // lists are read 4 entries at a time
    for (int i = 0; i < 2; ++i) {
        if (v) v->Y[i] = reinterpret_cast<float*>(base + o);
        o += yb;
    }
    for (int i = 0; i < 2; ++i) {
        if (v) v->cat[i] = reinterpret_cast<int*>(base + o);
        o += lb;
    }
    for (int i = 0; i < 2; ++i) {
        if (v) v->gid[i] = reinterpret_cast<int*>(base + o);
        o += lb;
    }
    const size_t fb = up((size_t)batch + 16);  // flags are read 16 bytes at a time
    for (int i = 0; i < 3; ++i) {
        if (v) v->flags[i] = reinterpret_cast<uint8_t*>(base + o);
        o += fb;
    }
    for (int i = 0; i < 2; ++i) {
        if (v) v->count[i] = reinterpret_cast<int*>(base + o);
        o += kAlign;
    }
    return o;
}

constexpr int kVirtLds = 2 * spdnn::kBlk * 16;  // two sets of slots for the lanes' sums (spdnn::VirtInfo)
template <bool MULTI, bool VIRT>
hipError_t allow_big_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_layer_kernel<MULTI, VIRT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)spdnn::tile_pair_bytes(spdnn::kCap) + (VIRT ? kVirtLds : 0));
}


// The fused kernels and set-up kernels use more dynamic LDS than the default limit allows.
int allow_large_lds() {
    constexpr size_t wide_lds = spdnn::kOrderThreads * sizeof(spdnn::WideScratch);
    const int tile_lds = (int)spdnn::tile_pair_bytes(spdnn::kCap);
    HIP_TRY((allow_big_lds<false, false>()));
    HIP_TRY((allow_big_lds<true, false>()));
    HIP_TRY((allow_big_lds<false, true>()));
    HIP_TRY((allow_big_lds<true, true>()));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::wide_pack_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::balance_kernel<1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(spdnn::BalanceScratch<1>)));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::balance_kernel<2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(spdnn::BalanceScratch<2>)));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_pair_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_pair_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_wide_pair_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds + spdnn::kPadLds));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_wide_pair4_kernel<4, 16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds + spdnn::kPair4LdsExtra));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_wide_pair4_kernel<2, 32>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds + spdnn::kPair4LdsExtra));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_row2_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, spdnn::kRow2LdsBytes));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_wide_kernel<16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_wide_kernel<8>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, tile_lds));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&spdnn::fused_chain_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)spdnn::tile_pair_bytes(spdnn::kBlk)));
    return SPDNN_OK;
}

// Longest neuron of every layer of a general model -> passes of 32 connections; with idx also the
// widest column window of any 1024-neuron block (of any aligned pair of blocks when N is a multiple
// of 2048, as spdnn_scan_windows counts).  scratch: device, 8*L + 8*ceil(N/1024) bytes.
int scan_csr(int32_t N, int32_t L, const int32_t* const* ptr, void* scratch_dev, size_t scratch_bytes,
             hipStream_t stream, std::vector<int32_t>* passes_of, const int32_t* const* idx = nullptr,
             int32_t* widest_window = nullptr) {
    const int32_t nblk = (N + spdnn::kBlk - 1) / spdnn::kBlk;
    const size_t need = sizeof(int) * 2 * (size_t)L + sizeof(int2) * (size_t)nblk;
    if (scratch_bytes < need) return fail(SPDNN_ESIZE, "scratch has %zu bytes, %zu needed", scratch_bytes, need);
    if (reinterpret_cast<uintptr_t>(scratch_dev) % 8) return fail(SPDNN_EINVAL, "scratch must be 8-byte aligned");
    int* out = static_cast<int*>(scratch_dev);
    int2* win = reinterpret_cast<int2*>(out + 2 * (size_t)L);
    HIP_TRY(hipMemsetAsync(out, 0, sizeof(int) * 2 * (size_t)L, stream));
    for (int32_t l = 0; l < L; ++l) {
        if (!ptr[l]) return fail(SPDNN_EINVAL, "ptr[%d] is NULL", l);
        spdnn::csr_scan_kernel<<<(N + 255) / 256, 256, 0, stream>>>(ptr[l], N, out + 2 * l);
    }
    HIP_TRY(hipGetLastError());
    std::vector<int> h(2 * (size_t)L);
    HIP_TRY(hipMemcpyAsync(h.data(), out, sizeof(int) * h.size(), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    passes_of->assign((size_t)L, 1);
    for (int32_t l = 0; l < L; ++l) {
        if (h[2 * l + 1]) return fail(SPDNN_EINVAL, "ptr[%d] is negative somewhere or decreases", l);
        // parts of 32 connections per neuron, rounded up to a power of two (lanes per neuron)
        const int parts = std::max(1, (h[2 * l] + spdnn::kNnz - 1) / spdnn::kNnz);
        int p2 = 1;
        while (p2 < parts) p2 *= 2;
        if (p2 > spdnn::kBlk / 4)
            return fail(SPDNN_EINVAL, "layer %d has a neuron of %d connections; at most %d are supported", l, h[2 * l],
                        spdnn::kNnz * spdnn::kBlk / 4);
        (*passes_of)[l] = p2;
    }
    if (idx && widest_window) {  // after the ptr arrays are known to be sound
        std::vector<int2> hw(nblk);
        int widest = 4;
        for (int32_t l = 0; l < L; ++l) {
            if (!idx[l]) return fail(SPDNN_EINVAL, "idx[%d] is NULL", l);
            spdnn::csr_block_window_kernel<<<nblk, spdnn::kBlk, 0, stream>>>(ptr[l], idx[l], N, win);
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipMemcpyAsync(hw.data(), win, sizeof(int2) * nblk, hipMemcpyDeviceToHost, stream));
            HIP_TRY(hipStreamSynchronize(stream));
            for (int32_t b = 0; b < nblk; ++b) {
                const int lo = hw[b].x & ~3;  // windows start at a multiple of 4 columns
                widest = std::max(widest, (hw[b].x + hw[b].y - lo + 3) & ~3);
            }
            if (N % (2 * spdnn::kBlk) == 0)
                for (int32_t b = 0; b + 1 < nblk; b += 2) {
                    if (!hw[b].y || !hw[b + 1].y) continue;
                    const int lo = std::min(hw[b].x, hw[b + 1].x) & ~3;
                    const int hi = std::max(hw[b].x + hw[b].y, hw[b + 1].x + hw[b + 1].y);
                    widest = std::max(widest, (hi - lo + 3) & ~3);
                }
        }
        *widest_window = widest;
    }
    return SPDNN_OK;
}

// Set-up shared by spdnn_create (ptr == NULL: every layer is [N][32]) and spdnn_create_csr
// (device arrays; layer l is cut into passes_of[l] passes of 32 connections per neuron).
int create_impl(spdnn_t* out, int32_t N, int32_t L, const std::vector<int32_t>& passes_of, const int32_t* const* ptr,
                const int32_t* const* idx, const float* const* val, const float* bias, int32_t where,
                void* weights_arena, size_t weights_arena_bytes, hipStream_t stream, void* host_arena = nullptr,
                size_t host_arena_bytes = 0) {
    const bool ooc = host_arena != nullptr;
    int32_t P = 0;  // passes = layers as the kernels see them
    std::vector<int32_t> layer_of, round_of, first_pass((size_t)L + 1, 0);
    for (int32_t l = 0; l < L; ++l) {
        first_pass[l] = P;
        for (int32_t r = 0; r < passes_of[l]; ++r) {
            layer_of.push_back(l);
            round_of.push_back(r);
        }
        P += passes_of[l];
    }
    first_pass[L] = P;
    // The arena decides how many stages the wide format may use (0 = none: layers with
    // wide windows then run the staged kernel, which is slower but needs no extra room).
    auto fits = [&](int cap) {
        return ooc ? ooc_device_bytes_for(N, P, cap) <= weights_arena_bytes &&
                         (size_t)P * block_bytes(N, cap) <= host_arena_bytes
                   : arena_bytes_for(N, P, cap) <= weights_arena_bytes;
    };
    int nstage_cap = stages_of(N);
    while (nstage_cap > 1 && !fits(nstage_cap)) --nstage_cap;
    if (nstage_cap < 2) nstage_cap = 0;
    if (!fits(nstage_cap)) {
        if (ooc)
            return fail(SPDNN_ESIZE, "out-of-core arenas have %zu (device) and %zu (host) bytes, at least %zu and %zu needed",
                        weights_arena_bytes, host_arena_bytes, ooc_device_bytes_for(N, P, 0),
                        (size_t)P * block_bytes(N, 0));
        return fail(SPDNN_ESIZE, "weights arena has %zu bytes, at least %zu needed", weights_arena_bytes,
                    arena_bytes_for(N, P, 0));
    }

    const int32_t nblk = (N + spdnn::kBlk - 1) / spdnn::kBlk;

    // bias: must be <= 0 everywhere, otherwise a dropped (all-zero) row would not stay zero
    std::vector<float> hb(N);
    if (where == SPDNN_HOST) {
        std::memcpy(hb.data(), bias, sizeof(float) * N);
    } else {
        // on the model's stream: the caller may have produced the bias there
        HIP_TRY(hipMemcpyAsync(hb.data(), bias, sizeof(float) * N, hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
    }
    for (int32_t j = 0; j < N; ++j)
        if (!(hb[j] <= 0.0f) || !std::isfinite(hb[j]))
            return fail(SPDNN_EBIAS, "bias[%d] = %g: every bias must be finite and <= 0", j, (double)hb[j]);

    spdnn_model* m = new (std::nothrow) spdnn_model;
    if (!m) return fail(SPDNN_EHIP, "out of host memory");
    struct Guard {
        spdnn_model* m;
        ~Guard() {
            if (m) spdnn_destroy(m);
        }
    } guard{m};

    m->N = N;
    m->L = L;
    m->first_pass = first_pass;
    m->nblk = nblk;
    m->G = (nblk % 4 == 0) ? 4 : (nblk % 3 == 0) ? 3 : (nblk % 2 == 0) ? 2 : 1;
    m->stream = stream;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    m->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    if (allow_large_lds() != SPDNN_OK) return SPDNN_EHIP;
    {  // set-up is also where this device's copy of the static scratch array is looked up
        void* unused = nullptr;
        if (static_scratch(&unused) != SPDNN_OK) return SPDNN_EHIP;
    }
    constexpr size_t wide_lds = spdnn::kOrderThreads * sizeof(spdnn::WideScratch);
    HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&m->host_counts), sizeof(int) * (size_t)(L + 2),  // [L + 1]: see infer_impl
                          hipHostMallocDefault));

    // carve the arena: bias | P x (win, rel, val) | staging (raw idx, raw val, error flag)
    char* base = static_cast<char*>(weights_arena);
    size_t o = 0;
    float* bias_dev = reinterpret_cast<float*>(base + o);
    o += up((size_t)N * sizeof(float));
    HIP_TRY(hipMemcpyAsync(bias_dev, hb.data(), sizeof(float) * N, hipMemcpyHostToDevice, stream));
    m->bias_dev = bias_dev;
    const size_t e = (size_t)nblk * spdnn::kNnz * spdnn::kBlk;
    std::vector<int2*> win_dev(P);
    m->layers.resize(P);
    const size_t blk_bytes = block_bytes(N, nstage_cap);
    if (ooc) {  // two device slots; pass p is built in slot p & 1 and runs from there
        m->ooc_host = static_cast<const char*>(host_arena);
        m->ooc_block = blk_bytes;
        m->ooc_slot[0] = base + o;
        m->ooc_slot[1] = base + o + blk_bytes;
        HIP_TRY(hipStreamCreateWithFlags(&m->ooc_stream, hipStreamNonBlocking));
        for (int i = 0; i < 2; ++i) {
            HIP_TRY(hipEventCreateWithFlags(&m->ooc_ready[i], hipEventDisableTiming));
            HIP_TRY(hipEventCreateWithFlags(&m->ooc_freed[i], hipEventDisableTiming));
        }
    }
    const size_t blocks_at = o;
    for (int32_t l = 0; l < P; ++l) {
        o = blocks_at + (size_t)(ooc ? (l & 1) : l) * blk_bytes;
        int2* win = reinterpret_cast<int2*>(base + o);
        o += up((size_t)nblk * sizeof(int2));
        uint16_t* rel = reinterpret_cast<uint16_t*>(base + o);
        o += up(e * sizeof(uint16_t));
        float* wv = reinterpret_cast<float*>(base + o);
        o += up(e * sizeof(float));
        uint32_t* qsel = reinterpret_cast<uint32_t*>(base + o);
        o += up((size_t)nblk * spdnn::kBlk * sizeof(uint32_t));
        m->layers[l].virt.slot = reinterpret_cast<const uint16_t*>(base + o);
        o += up((size_t)nblk * spdnn::kBlk * sizeof(uint16_t));
        m->layers[l].virt.nb8 = reinterpret_cast<const uint8_t*>(base + o);
        o += up((size_t)nblk * 16);
        m->layers[l].virt.range = reinterpret_cast<const int2*>(base + o);
        o += up((size_t)nblk * sizeof(int2));
        m->layers[l].virt.fin = reinterpret_cast<const uint32_t*>(base + o);
        o += up((size_t)nblk * spdnn::kBlk * sizeof(uint32_t));
        m->layers[l].w = spdnn::LayerWeights{rel, wv, win, qsel};
        win_dev[l] = win;
        spdnn::WideWeights ww{};
        ww.win = win;
        if (nstage_cap >= 2) {  // room for the wide format; the layer's own stage count strides the arrays
            const size_t we = (size_t)nblk * wide_steps_max(nstage_cap) * spdnn::kBlk;
            const size_t sp = (size_t)nblk * spdnn::kSpill * spdnn::kBlk;
            ww.pk = reinterpret_cast<uint2*>(base + o);
            o += up(we * sizeof(uint2));
            ww.nb8 = reinterpret_cast<uint8_t*>(base + o);
            o += up((size_t)nblk * nstage_cap * 16);
            ww.spill_col = reinterpret_cast<uint16_t*>(base + o);
            o += up(sp * sizeof(uint16_t));
            ww.spill_val = reinterpret_cast<float*>(base + o);
            o += up(sp * sizeof(float));
            ww.spill_n = reinterpret_cast<uint8_t*>(base + o);
            o += up((size_t)nblk * 16);
            if (wide_has_slots(nstage_cap)) {
                ww.ps = reinterpret_cast<uint4*>(base + o);
                o += up(we * sizeof(uint16_t));
                ww.sp16 = reinterpret_cast<uint16_t*>(base + o);
                o += up(sp * sizeof(uint16_t));
            }
            if (nblk % 4 == 0) {
                const size_t nunit = nblk / 4;
                m->layers[l].r2_codes = reinterpret_cast<uint16_t*>(base + o);
                o += up((size_t)nblk * spdnn::kBlk * spdnn::kNnz * sizeof(uint16_t));
                m->layers[l].r2_map = reinterpret_cast<int32_t*>(base + o);
                o += up(nunit * (spdnn::kRow2Cols / 4) * sizeof(int32_t));
                m->layers[l].r2_ngroups = reinterpret_cast<int*>(base + o);
                o += up(nunit * sizeof(int));
            }
        }
        m->layers[l].ww = ww;
    }
    o = blocks_at + (size_t)(ooc ? 2 : P) * blk_bytes;
    const size_t lanes = (size_t)nblk * spdnn::kBlk;
    int32_t* st_idx = reinterpret_cast<int32_t*>(base + o);
    o += up(lanes * spdnn::kNnz * sizeof(int32_t));
    float* st_val = reinterpret_cast<float*>(base + o);
    o += up(lanes * spdnn::kNnz * sizeof(float));
    uint8_t* st_len = reinterpret_cast<uint8_t*>(base + o);  // several lanes per neuron: connections of every lane
    o += up(lanes);
    uint16_t* slot_tabs = reinterpret_cast<uint16_t*>(base + o);  // one table per set-up stream
    const size_t slot_tab_elems = up((size_t)nblk * spdnn::kCap * sizeof(uint16_t)) / sizeof(uint16_t);
    o += kSetupStreams * up((size_t)nblk * spdnn::kCap * sizeof(uint16_t));
    int* blockmin = reinterpret_cast<int*>(base + o);
    o += up(sizeof(int) * (size_t)nblk);
    // [0] bad column seen; [1 + p] pass p could not use the wide format; [1 + P + p] pass p's widest window;
    // [1 + 2P + p] pass p has more than one weight value; [1 + 3P + 2p] {two neurons per lane possible, weight bits}
    int* err_dev = reinterpret_cast<int*>(base + o);
    HIP_TRY(hipMemsetAsync(err_dev, 0, sizeof(int) * (size_t)(5 * P + 1), stream));
    o += up(sizeof(int) * (size_t)(5 * P + 1));
    spdnn::LayerWeights* chain_layers_dev = reinterpret_cast<spdnn::LayerWeights*>(base + o);
    o += up((size_t)P * sizeof(spdnn::LayerWeights));
    int* chain_rows_dev = reinterpret_cast<int*>(base + o);

    // Layers that are already on the device and need no staging are set up on several streams in turn.
    struct SetupStreams {
        hipStream_t s[kSetupStreams] = {};
        hipEvent_t start = nullptr;
        int n = 1;
        ~SetupStreams() {
            for (int i = 1; i < n; ++i)
                if (s[i]) (void)hipStreamDestroy(s[i]);
            if (start) (void)hipEventDestroy(start);
        }
    } ss;
    ss.s[0] = stream;
    if (!ptr && where == SPDNN_DEVICE && !ooc && P > 1) {
        HIP_TRY(hipEventCreateWithFlags(&ss.start, hipEventDisableTiming));
        HIP_TRY(hipEventRecord(ss.start, stream));  // bias and cleared flags are in place
        for (int i = 1; i < kSetupStreams; ++i) {
            HIP_TRY(hipStreamCreateWithFlags(&ss.s[i], hipStreamNonBlocking));
            ss.n = i + 1;
            HIP_TRY(hipStreamWaitEvent(ss.s[i], ss.start, 0));
        }
    }

    const size_t raw = (size_t)N * spdnn::kNnz;
    std::vector<int2> hw((size_t)P * nblk);
    std::vector<int2> virt_ranges;  // several lanes per neuron: {first neuron, neurons} of the current layer's workgroups
    for (int32_t l = 0; l < P; ++l) {  // l = pass; it belongs to layer ll
        hipStream_t stream = ss.s[l % ss.n];  // everything of this pass goes to one stream
        uint16_t* slot_tab = slot_tabs + (size_t)(l % ss.n) * slot_tab_elems;
        const int32_t ll = layer_of[l];
        const int32_t* di = idx[ll];
        const float* dv = val[ll];
        LayerDesc& d = m->layers[l];
        d.multi = passes_of[ll] > 1;
        int nrows = -1;                 // rows of di / dv if not N
        const uint8_t* lens = nullptr;  // connections per row if not 32
        if (ptr && d.multi) {
            // More than 32 connections somewhere: a neuron takes as many lanes as it has parts of 32 connections, and
            // a workgroup as many neighbouring neurons (in fours) as fill its 1024 lanes -- fewer where the next
            // four would widen its column window beyond one LDS stage.  The layer's workgroups
            // are cut into launches of nblk; launch r is pass r.  Their lanes are set up like the neurons of a
            // fixed-32 layer.
            if (round_of[l] == 0) {
                std::vector<int32_t> hp((size_t)N + 1);
                std::vector<int2> qw((size_t)N / 4);  // columns of every four neurons (the staging area as scratch)
                int2* qw_dev = reinterpret_cast<int2*>(st_idx);
                spdnn::csr_quartet_window_kernel<<<(N / 4 + 255) / 256, 256, 0, stream>>>(ptr[ll], idx[ll], N, qw_dev);
                HIP_TRY(hipGetLastError());
                HIP_TRY(hipMemcpyAsync(hp.data(), ptr[ll], sizeof(int32_t) * hp.size(), hipMemcpyDeviceToHost, stream));
                HIP_TRY(hipMemcpyAsync(qw.data(), qw_dev, sizeof(int2) * qw.size(), hipMemcpyDeviceToHost, stream));
                HIP_TRY(hipStreamSynchronize(stream));
                // how the layer's neurons are cut into workgroups: spdnn_cut.h (host code, tested without a GPU)
                const std::vector<spdnn::NeuronRange> cut =
                    spdnn::cut_workgroups(hp.data(), reinterpret_cast<const int*>(qw.data()), N, passes_of[ll], nblk, m->G,
                                          spdnn::kBlk, spdnn::kNnz, spdnn::kCap);
                virt_ranges.clear();
                for (const spdnn::NeuronRange& r : cut) virt_ranges.push_back(make_int2(r.first, r.count));
            }
            std::vector<int2> mine((size_t)nblk, make_int2(N, 0));
            for (int32_t b = 0; b < nblk; ++b) {
                const size_t vb = (size_t)round_of[l] * nblk + b;
                if (vb < virt_ranges.size()) {
                    mine[b] = virt_ranges[vb];
                    d.virt_blocks = b + 1;
                }
            }
            HIP_TRY(hipMemcpyAsync(const_cast<int2*>(d.virt.range), mine.data(), sizeof(int2) * (size_t)nblk, hipMemcpyHostToDevice, stream));
            HIP_TRY(hipStreamSynchronize(stream));  // `mine` goes out of scope
            d.virt_lanes = passes_of[ll];
            spdnn::csr_virtual_kernel<<<nblk, spdnn::kBlk, 0, stream>>>(ptr[ll], idx[ll], val[ll], N, d.virt.range, st_idx, st_val,
                                                                        st_len, const_cast<uint16_t*>(d.virt.slot),
                                                                        const_cast<uint32_t*>(d.virt.fin));
            HIP_TRY(hipGetLastError());
            di = st_idx;
            dv = st_val;
            nrows = nblk * spdnn::kBlk;
            lens = st_len;
        } else if (ptr) {  // general layer of at most 32 connections per neuron, padded with zero weights
            const int r = round_of[l];
            spdnn::csr_block_min_kernel<<<nblk, spdnn::kBlk, 0, stream>>>(ptr[ll], idx[ll], N, r, blockmin);
            spdnn::csr_round_kernel<<<(unsigned)((raw + 255) / 256), 256, 0, stream>>>(ptr[ll], idx[ll], val[ll], N, r,
                                                                                     blockmin, st_idx, st_val);
            HIP_TRY(hipGetLastError());
            di = st_idx;
            dv = st_val;
        } else if (where == SPDNN_HOST) {
            HIP_TRY(hipMemcpyAsync(st_idx, idx[ll], raw * sizeof(int32_t), hipMemcpyHostToDevice, stream));
            HIP_TRY(hipMemcpyAsync(st_val, val[ll], raw * sizeof(float), hipMemcpyHostToDevice, stream));
            di = st_idx;
            dv = st_val;
        }
        int* widest_dev = err_dev + 1 + P + l;
        int* pair_dev = err_dev + 1 + 3 * P + 2 * l;
        spdnn::block_window_kernel<<<nblk, spdnn::kBlk, 0, stream>>>(di, N, win_dev[l], err_dev, widest_dev, dv,
                                                                       err_dev + 1 + 2 * P + l, nrows);
        // a layer of several passes runs the one-neuron-per-lane kernels, whose epilogue knows about passes
        if (!d.multi)
            spdnn::pair_merge_kernel<<<1, 64, 0, stream>>>(win_dev[l], nblk, N, dv, err_dev + 1 + 2 * P + l, widest_dev,
                                                           pair_dev);
        HIP_TRY(hipGetLastError());
        // the windows decide the layer's kernel and its set-up; they are small, so read them back now
        int pair_info[2] = {0, 0};
        // Layers that may run on two-row tiles: how many groups of four columns a 4096-neuron unit touches, for
        // every segment length of unit_neuron, asked for now so that it comes back with the windows (the list
        // area serves as the kernel's output).
        constexpr int kCand = spdnn::kSegLog2Max - spdnn::kSegLog2Min + 1;
        const bool r2_room = !d.multi && N % spdnn::kUnit4 == 0 && d.r2_codes != nullptr &&
                             (size_t)(nblk / 4) * (N / 4) <= slot_tab_elems;
        std::vector<int> ngr;
        if (r2_room) {
            ngr.resize((size_t)(nblk / 4) * kCand);
            spdnn::row2_footprint_kernel<<<dim3(nblk / 4, kCand), spdnn::kBlk, 0, stream>>>(di, N, reinterpret_cast<int*>(d.r2_map));
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipMemcpyAsync(ngr.data(), d.r2_map, sizeof(int) * ngr.size(), hipMemcpyDeviceToHost, stream));
        }
        HIP_TRY(hipMemcpyAsync(&hw[(size_t)l * nblk], win_dev[l], sizeof(int2) * nblk, hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipMemcpyAsync(pair_info, pair_dev, sizeof(pair_info), hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        // One weight, but the windows are too wide for two neurons per lane.  If units of 2048 neurons in segments
        // (unit_neuron) read columns that do not overlap, at most 2048 each -- the strided patterns that RadiX-Net
        // layers are (Section II-A) -- neurons and columns get new names under which every unit has a contiguous
        // window, and the layer is set up again as an ordinary one for the two-neurons-per-lane kernel.
        if (pair_info[0] == 2 && r2_room && d.ww.pk != nullptr && N % spdnn::kPairUnit == 0) {
            const int32_t nunit2 = N / spdnn::kPairUnit;
            constexpr int kCand2 = spdnn::kSegLog2Max - 1 - 5 + 1;  // segments of 2048 down to 32 neurons
            std::vector<int> ngr2((size_t)nunit2 * kCand2);
            int* cnt_dev = reinterpret_cast<int*>(d.r2_map);
            spdnn::row2_footprint_kernel<<<dim3(nunit2, kCand2), spdnn::kBlk, 0, stream>>>(di, N, cnt_dev, spdnn::kPairUnit);
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipMemcpyAsync(ngr2.data(), cnt_dev, sizeof(int) * ngr2.size(), hipMemcpyDeviceToHost, stream));
            HIP_TRY(hipStreamSynchronize(stream));
            int best_a = -1, best = spdnn::kPairUnit / 4 + 1;
            for (int y = 0; y < kCand2; ++y) {
                const int most = *std::max_element(ngr2.begin() + (size_t)y * nunit2, ngr2.begin() + (size_t)(y + 1) * nunit2);
                if (most < best) {
                    best = most;
                    best_a = spdnn::kSegLog2Max - 1 - y;
                }
            }
            if (best_a >= 0) {  // every unit within 2048 columns: do they overlap?
                const int stride2 = nunit2 << best_a;
                int* owner = reinterpret_cast<int*>(slot_tab);  // this stream's table as scratch: N/4 owners, N/4 new names, a flag
                int* newname = owner + N / 4;
                int* conflict = newname + N / 4;
                HIP_TRY(hipMemsetAsync(owner, 0xff, sizeof(int) * (size_t)(N / 4), stream));
                HIP_TRY(hipMemsetAsync(conflict, 0, sizeof(int), stream));
                spdnn::relabel_owner_kernel<<<nunit2, spdnn::kBlk, 0, stream>>>(di, N, best_a, stride2, owner, conflict);
                spdnn::relabel_rank_kernel<<<nunit2, spdnn::kBlk, 0, stream>>>(owner, N, newname, d.r2_map, conflict);
                HIP_TRY(hipGetLastError());
                int clash = 1;
                HIP_TRY(hipMemcpyAsync(&clash, conflict, sizeof(int), hipMemcpyDeviceToHost, stream));
                HIP_TRY(hipStreamSynchronize(stream));
                if (!clash) {
                    // the layer under its new names is written where its wide format would go (it will not have one):
                    // room for 32 steps of 8 bytes per neuron, of which 4 bytes per connection are needed
                    int32_t* renamed = reinterpret_cast<int32_t*>(const_cast<uint2*>(d.ww.pk));
                    spdnn::relabel_apply_kernel<<<(unsigned)((raw + 255) / 256), 256, 0, stream>>>(di, N, best_a, stride2, newname, renamed);
                    HIP_TRY(hipGetLastError());
                    di = renamed;
                    d.relabel = true;
                    d.rn = spdnn::PairRelabel{d.r2_map, best_a, stride2};
                    // the windows, and whether pairs of blocks fit one stage, under the new names
                    HIP_TRY(hipMemsetAsync(widest_dev, 0, sizeof(int), stream));
                    spdnn::block_window_kernel<<<nblk, spdnn::kBlk, 0, stream>>>(di, N, win_dev[l], err_dev, widest_dev, dv,
                                                                                   err_dev + 1 + 2 * P + l, nrows);
                    spdnn::pair_merge_kernel<<<1, 64, 0, stream>>>(win_dev[l], nblk, N, dv, err_dev + 1 + 2 * P + l, widest_dev,
                                                                   pair_dev);
                    HIP_TRY(hipGetLastError());
                    HIP_TRY(hipMemcpyAsync(&hw[(size_t)l * nblk], win_dev[l], sizeof(int2) * nblk, hipMemcpyDeviceToHost, stream));
                    HIP_TRY(hipMemcpyAsync(pair_info, pair_dev, sizeof(pair_info), hipMemcpyDeviceToHost, stream));
                    HIP_TRY(hipStreamSynchronize(stream));
                    if (pair_info[0] != 1) return fail(SPDNN_EHIP, "layer %d: relabelled units do not fit one stage", ll);
                }
            }
        }
        const int pair = pair_info[0] == 1;        // two neurons per lane, single stage
        const bool wide_pair = pair_info[0] == 2;  // ... if the layer also fits the wide format
        // one weight, every block wider than one stage, and every 4096-neuron unit within 16384 columns:
        // four neurons per lane on two-row tiles; needs nothing of the other formats
        const bool row2_ok = wide_pair && !d.multi && N % spdnn::kUnit4 == 0 && d.r2_codes != nullptr;
        bool row2 = row2_ok;
        for (int32_t u = 0; row2 && u < nblk / 4; ++u) {
            int x = 0, y = 0;  // the unit's window: the union of its blocks' cyclic windows
            for (int i = 0; i < 4; ++i)
                spdnn::win_union(x, y, hw[(size_t)l * nblk + 4 * u + i].x, hw[(size_t)l * nblk + 4 * u + i].y, N, x, y);
            row2 = y <= spdnn::kRow2Cols;
        }
        // Windows too wide for the tile, or much wider than the unit itself: the gathered footprint (Section
        // III-A-2's preload list at 4-column granularity) may fit it -- every unit's connections within 4096
        // groups of four columns -- and units of interleaved segments (unit_neuron) may need far fewer columns
        // than units of 4096 neighbours: in a strided pattern the neurons j, j + stride, j + 2 stride, ... read
        // the same columns.  Every segment length from 4096 down to 64 is tried and the one whose largest unit
        // needs the fewest groups wins (the longer segment on a tie).
        // The rank table is set-up scratch: this stream's column -> slot table, which such a layer does not use.
        const int32_t* gather_map = nullptr;
        const uint16_t* gather_rank = nullptr;
        int seg_log2 = spdnn::kSegLog2Max, seg_stride = N;
        int widest_unit = 0;  // columns of the widest unit's window, units of 4096 neighbours
        for (int32_t u = 0; row2_ok && u < nblk / 4; ++u) {
            int x = 0, y = 0;
            for (int i = 0; i < 4; ++i)
                spdnn::win_union(x, y, hw[(size_t)l * nblk + 4 * u + i].x, hw[(size_t)l * nblk + 4 * u + i].y, N, x, y);
            widest_unit = std::max(widest_unit, y);
        }
        if (row2_ok && r2_room && widest_unit > spdnn::kUnit4) {
            const int32_t nunit = nblk / 4;
            int best_a = -1, best = spdnn::kRow2Cols / 4 + 1;
            for (int y = 0; y < kCand; ++y) {
                const int most = *std::max_element(ngr.begin() + (size_t)y * nunit, ngr.begin() + (size_t)(y + 1) * nunit);
                if (most < best) {
                    best = most;
                    best_a = spdnn::kSegLog2Max - y;
                }
            }
            // worth it if the window does not fit the tile at all, or if the tile shrinks to half the window or less
            const bool take = best_a >= 0 && (!row2 || 4 * best <= widest_unit / 2);
            if (take) {
                spdnn::row2_gather_kernel<<<nunit, spdnn::kBlk, 0, stream>>>(di, N, best_a, (N / spdnn::kUnit4) << best_a, d.r2_map,
                                                                           slot_tab, d.r2_ngroups);
                HIP_TRY(hipGetLastError());
                row2 = true;
                seg_log2 = best_a;
                seg_stride = (N / spdnn::kUnit4) << best_a;
                gather_map = d.r2_map;
                gather_rank = slot_tab;
            }
        }
        if (row2) {
            // the windows read back above are the blocks' own; pair_merge_kernel has widened them on the device to
            // common windows of block pairs, whose unions per unit are the same
            d.r2 = spdnn::Row2Weights{reinterpret_cast<const uint4*>(d.r2_codes), win_dev[l], gather_map, seg_log2, seg_stride};
            const int groups = N / spdnn::kGroup32;
            spdnn::row2_pack_kernel<<<groups, spdnn::kRow2PackThreads, 0, stream>>>(di, N, win_dev[l], gather_rank, seg_log2,
                                                                                    seg_stride, d.r2_codes);
            HIP_TRY(hipGetLastError());
            d.mode = kRow2;
            d.lds_cols = spdnn::kRow2Cols;
            std::memcpy(&d.wuni, &pair_info[1], sizeof(float));
            if (ooc)
                HIP_TRY(hipMemcpyAsync(static_cast<char*>(host_arena) + (size_t)l * blk_bytes, m->ooc_slot[l & 1], blk_bytes,
                                       hipMemcpyDeviceToHost, stream));
            if (where == SPDNN_HOST) HIP_TRY(hipStreamSynchronize(stream));  // staging is reused
            continue;
        }
        if (pair)
            spdnn::balance_kernel<2><<<nblk / 2, spdnn::kBalanceThreads, sizeof(spdnn::BalanceScratch<2>), stream>>>(
                di, N, win_dev[l], widest_dev, slot_tab, const_cast<uint32_t*>(d.w.qsel));
        else
            spdnn::balance_kernel<1><<<nblk, spdnn::kBalanceThreads, sizeof(spdnn::BalanceScratch<1>), stream>>>(
                di, N, win_dev[l], widest_dev, slot_tab, const_cast<uint32_t*>(d.w.qsel), nrows);
        spdnn::order_pack_kernel<<<nblk * spdnn::kOrderThreads, spdnn::kOrderPackThreads, 0, stream>>>(
            di, dv, N, win_dev[l], widest_dev, slot_tab, pair, const_cast<uint16_t*>(d.w.rel),
            const_cast<float*>(d.w.val), nrows, lens, lens ? const_cast<uint8_t*>(d.virt.nb8) : nullptr);
        HIP_TRY(hipGetLastError());
        int widest = 4;
        for (int32_t b = 0; b < nblk; ++b) widest = std::max(widest, hw[(size_t)l * nblk + b].y);
        const int nst = stages_of(widest);
        d.lds_cols = std::min(widest, spdnn::kCap);
        d.mode = pair ? kPair : nst <= 1 ? kSingle : kStaged;
        std::memcpy(&d.wuni, &pair_info[1], sizeof(float));
        // the wide format: 3 and more stages, or 2 stages when the layer can run two neurons per lane
        if (!d.multi && (nst >= 3 || (nst == 2 && wide_pair && d.ww.ps)) && nst <= nstage_cap) {
            d.ww.nstage = nst;
            spdnn::wide_pack_kernel<<<nblk, spdnn::kOrderThreads, wide_lds, stream>>>(
                di, dv, N, win_dev[l], nst, const_cast<uint2*>(d.ww.pk), const_cast<uint8_t*>(d.ww.nb8), const_cast<uint16_t*>(d.ww.spill_col),
                const_cast<float*>(d.ww.spill_val), const_cast<uint8_t*>(d.ww.spill_n), err_dev + 1 + l);
            HIP_TRY(hipGetLastError());
            d.mode = kWide;
            if (wide_pair && spdnn::wide_steps(nst) >= 16 && d.ww.ps) {
                const int S = spdnn::wide_steps(nst);
                const size_t n_out = (size_t)nblk * nst * (S / 8) * spdnn::kBlk;
                spdnn::wide_slots_kernel<<<(unsigned)((n_out + 255) / 256), 256, 0, stream>>>(
                    d.ww.pk, const_cast<uint4*>(d.ww.ps), n_out, S);
                const size_t n_sp = (size_t)nblk * spdnn::kSpill * spdnn::kBlk;
                spdnn::wide_spill16_kernel<<<(unsigned)((n_sp + 255) / 256), 256, 0, stream>>>(
                    d.ww.spill_col, d.ww.spill_val, const_cast<uint16_t*>(d.ww.sp16), n_sp);
                HIP_TRY(hipGetLastError());
                d.mode = kWidePair;
                d.pair4 = nst <= 4;
            }
        }
        if (ooc)  // the finished block goes to the host; its slot is rebuilt two passes later, after this copy
            HIP_TRY(hipMemcpyAsync(static_cast<char*>(host_arena) + (size_t)l * blk_bytes, m->ooc_slot[l & 1], blk_bytes,
                                   hipMemcpyDeviceToHost, stream));
        if (where == SPDNN_HOST) HIP_TRY(hipStreamSynchronize(stream));  // staging is reused
    }
    for (int i = 1; i < ss.n; ++i) HIP_TRY(hipStreamSynchronize(ss.s[i]));
    // error flag and the layers whose patterns did not fit the wide format
    std::vector<int> herr((size_t)P + 1, 0);
    HIP_TRY(hipMemcpyAsync(herr.data(), err_dev, sizeof(int) * (size_t)(P + 1), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    if (herr[0]) return fail(SPDNN_EINVAL, "a column index is outside [0, N)");
    for (int32_t l = 0; l < P; ++l)
        if ((m->layers[l].mode == kWide || m->layers[l].mode == kWidePair) && herr[1 + l]) m->layers[l].mode = kStaged;
    // One output block and nothing but single-stage layers of one launch each: the whole network can run in one
    // launch (fused_chain_kernel), which takes the layers' descriptors from device memory.
    bool chain = nblk == 1 && !ooc && P == L;
    for (int32_t l = 0; chain && l < P; ++l) chain = m->layers[l].mode == kSingle && !m->layers[l].multi;
    if (chain) {
        std::vector<spdnn::LayerWeights> lw((size_t)L);
        for (int32_t l = 0; l < L; ++l) {
            lw[l] = m->layers[l].w;
            m->chain_lds_cols = std::max(m->chain_lds_cols, m->layers[l].lds_cols);
        }
        HIP_TRY(hipMemcpyAsync(chain_layers_dev, lw.data(), sizeof(spdnn::LayerWeights) * (size_t)L, hipMemcpyHostToDevice, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        m->chain_layers = chain_layers_dev;
        m->chain_rows = chain_rows_dev;
    }
    guard.m = nullptr;
    *out = m;
    return SPDNN_OK;
}


// No entry point lets an exception out (a failed host allocation in a std::vector, for example).
template <typename F>
int guarded(F f) {
    try {
        return f();
    } catch (const std::bad_alloc&) {
        return fail(SPDNN_EHIP, "out of host memory");
    } catch (...) {
        return fail(SPDNN_EHIP, "unexpected exception");
    }
}

// Argument checks shared by the inference entry points; batch == 0 is answered here (n_active = 0).
int check_infer_args(spdnn_t h, const float* Y0_dev, int32_t batch, int32_t* n_active_host,
                     const int32_t* active_rows_dev, const float* Y_final_dev) {
    if (!h) return fail(SPDNN_EINVAL, "handle is NULL");
    if (!n_active_host) return fail(SPDNN_EINVAL, "n_active_host is NULL");
    if (batch < 0) return fail(SPDNN_EINVAL, "batch < 0");
    h->prof_layers = 0;
    if (batch == 0) {
        *n_active_host = 0;
        return SPDNN_OK;
    }
    if (!Y0_dev || !active_rows_dev) return fail(SPDNN_EINVAL, "null argument");
    if (reinterpret_cast<uintptr_t>(Y0_dev) % 16) return fail(SPDNN_EINVAL, "Y0 must be 16-byte aligned");
    if (Y_final_dev && reinterpret_cast<uintptr_t>(Y_final_dev) % 16) return fail(SPDNN_EINVAL, "Y_final must be 16-byte aligned");
    return SPDNN_OK;
}

// Address of the current device's copy of the static scratch array.  The array's name is only a
// host-side stand-in; every GPU holds its own copy at its own address, looked up once per device
// (at spdnn_create, else on the first spdnn_infer_static on that device) and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch(void** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SPDNN_EINVAL, "device %d: only devices 0..%d are supported", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || reinterpret_cast<uintptr_t>(p) % kAlign) return fail(SPDNN_EHIP, "static scratch array has no usable device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SPDNN_OK;
}

// All layers in one launch (fused_chain_kernel)?  Yes if the model allows it and a workgroup's share of the rows is
// small enough; *q = the launch's row chunks.
bool one_launch_shape(spdnn_t h, int32_t batch, int32_t* q) {
    const int32_t groups = (batch + spdnn::kRows - 1) / spdnn::kRows;
    const int32_t chunks = std::max(1, std::min(h->num_cu, groups));
    if (q) *q = chunks;
    return batch > 0 && h->chain_layers != nullptr && (groups + chunks - 1) / chunks * spdnn::kRows <= spdnn::kChainRows;
}

// All L layers on `batch` rows whose first row has the original number row_offset; wv = the carved
// work memory.  Returns with the model's stream drained, also when a HIP call fails half way.
int infer_impl(spdnn_t h, const float* Y0_dev, int32_t batch, const WorkView& wv, int32_t row_offset,
               int32_t* n_active_host, int32_t* active_rows_dev, float* Y_final_dev) {
    const int32_t N = h->N, L = h->L;
    hipStream_t s = h->stream;
    // Kernels may be queued when a later HIP call fails: nothing of this call is left running on return.
    struct DrainModel {
        hipStream_t s;
        bool armed = true;
        ~DrainModel() {
            if (armed) (void)hipStreamSynchronize(s);
        }
    } drain_model{s};

    for (int32_t l = 1; l <= L; ++l) h->host_counts[l] = -1;  // "not reported yet"
    h->host_counts[0] = batch;
    int32_t chain_q = 1;
    const bool chain = one_launch_shape(h, batch, &chain_q);
    // "layer -1": every row of the batch is flagged alive, under its own number
    spdnn::init_lists_kernel<<<(batch + 255) / 256, 256, 0, s>>>(wv.gid[1], wv.flags[2], wv.flags[0], wv.count[1], batch,
                                                                 row_offset, chain ? h->chain_rows : nullptr, chain ? L + 1 : 0);
    int32_t bound = batch;  // upper bound of the rows active at the layer being launched
    int32_t run = 0;        // layers launched
    int32_t rot = 0;        // how often the lists have rotated (= run, unless all layers ran in one launch)
    int32_t final_buf = 0;  // work buffer that holds the last layer's output
    std::vector<int> chain_rows_host;
    // All layers in one launch, if the model allows it and a workgroup's share of the rows fits its lists.
    if (chain) {
        if (h->profiling) HIP_TRY(hipEventRecord(h->t0[0], s));
        spdnn::RowLists rl;  // as "layer 0" of the lists' rotation
        rl.flags_prev = wv.flags[2];
        rl.count_prev = wv.count[1];
        rl.gid_prev = wv.gid[1];
        rl.cat = wv.cat[0];
        rl.gid = wv.gid[0];
        rl.count = wv.count[0];
        rl.host_count = h->host_counts;
        rl.flags_clear = wv.flags[1];
        const spdnn::ChainArgs ca{h->chain_layers, L, h->chain_rows};
        const size_t lds = spdnn::tile_pair_bytes((h->chain_lds_cols + 255) / 256 * 256);
        spdnn::fused_chain_kernel<<<(chain_q + 7) / 8 * 8, spdnn::kBlk, lds, s>>>(Y0_dev, wv.Y[0], wv.Y[1], wv.flags[0], rl, ca,
                                                                                  h->bias_dev, N, chain_q);
        HIP_TRY(hipGetLastError());
        if (h->profiling) HIP_TRY(hipEventRecord(h->t1[0], s));
        chain_rows_host.resize((size_t)L + 1);
        HIP_TRY(hipMemcpyAsync(chain_rows_host.data(), h->chain_rows, sizeof(int) * ((size_t)L + 1), hipMemcpyDeviceToHost, s));
        rot = 1;
        final_buf = (L - 1) & 1;
    }
    // Out-of-core weights (Section III-B-1): pass p runs from device slot p & 1.  The copy stream fills
    // the two slots, and refills a slot with pass p + 2 as soon as the kernels of pass p are done with
    // it, so the transfer of the next layer runs under the current layer's kernel.
    const int32_t P = (int32_t)h->layers.size();
    auto ooc_fetch = [&](int32_t p) -> hipError_t {
        hipError_t e = hipMemcpyAsync(h->ooc_slot[p & 1], h->ooc_host + (size_t)p * h->ooc_block, h->ooc_block,
                                      hipMemcpyHostToDevice, h->ooc_stream);
        return e != hipSuccess ? e : hipEventRecord(h->ooc_ready[p & 1], h->ooc_stream);
    };
    // whatever happens below, the copy stream is idle again when the call returns
    struct Drain {
        hipStream_t cs;
        ~Drain() {
            if (cs) (void)hipStreamSynchronize(cs);
        }
    } drain{h->ooc_stream};
    if (h->ooc_host)
        for (int32_t p = 0; p < std::min(P, 2); ++p) HIP_TRY(ooc_fetch(p));
    for (int32_t l = 0; l < L && !chain; ++l) {
        const float* Yin = (l == 0) ? Y0_dev : wv.Y[(l - 1) & 1];
        float* Yout = wv.Y[l & 1];
        if (h->profiling) HIP_TRY(hipEventRecord(h->t0[l], s));
        // one launch per pass: a layer is a single pass unless some neuron has more than 32 connections
        for (int32_t p = h->first_pass[l]; p < h->first_pass[l + 1]; ++p) {
            const LayerDesc& d = h->layers[p];
            if (d.multi && d.virt_blocks == 0 && p != h->first_pass[l]) continue;  // no workgroup of the layer is left for this launch
            if (h->ooc_host) HIP_TRY(hipStreamWaitEvent(s, h->ooc_ready[p & 1], 0));
            // The layer's first kernel compacts the list of active rows on its way in (the flags layer l-1
            // raised -> slots and row numbers); later passes of the same layer find the lists in place.
            spdnn::RowLists rl;
            rl.flags_prev = p == h->first_pass[l] ? wv.flags[(l + 2) % 3] : nullptr;
            rl.count_prev = wv.count[(l + 1) & 1];
            rl.gid_prev = wv.gid[(l + 1) & 1];
            rl.cat = wv.cat[l & 1];
            rl.gid = wv.gid[l & 1];
            rl.count = wv.count[l & 1];
            rl.host_count = h->host_counts + l;
            rl.flags_clear = wv.flags[(l + 1) % 3];
            // launch shape: one workgroup per CU; the rows are cut into Q chunks per output block
            const int32_t rows_per_group = d.mode == kRow2 ? spdnn::kRows2 : spdnn::kRows;
            const int32_t ngroups = (bound + rows_per_group - 1) / rows_per_group;
            // kPair: the workgroups' column blocks are pairs of output blocks
            const bool two = d.mode == kPair || d.mode == kWidePair;
            const int32_t ncb = d.mode == kRow2 ? h->nblk / 4 : two ? h->nblk / 2 : h->nblk;
            // Workgroups that read the same rows go to one XCD (32 CUs, one L2).  In a wide layer every
            // column block reads whole rows: as many of them as possible share an XCD, so that a row is
            // fetched from memory once, not once per XCD.
            int32_t G = d.mode == kPair ? ((ncb % 2 == 0) ? 2 : 1) : h->G;
            if (d.multi)  // fewer neurons per workgroup: up to P times as many workgroups read the same window
                for (int32_t g : {32, 16, 8, 4, 3, 2, 1})
                    if (g <= h->G * d.virt_lanes && ncb % g == 0) {
                        G = g;
                        break;
                    }
            if (d.mode == kWide || d.mode == kWidePair || d.mode == kRow2)
                for (int32_t g : {32, 16, 8, 4, 3, 2, 1})
                    if (ncb % g == 0) {
                        G = g;
                        break;
                    }
            int32_t Q = std::max(1, h->num_cu / ncb);
            // several lanes per neuron: the launches of a layer have different numbers of workgroups with neurons,
            // rarely a divisor of the CUs; four times as many workgroups as CUs, taken up as CUs fall free
            if (d.multi) Q = (4 * h->num_cu + std::max(1, d.virt_blocks) - 1) / std::max(1, d.virt_blocks);
            Q = std::max(1, std::min(Q, ngroups));
            const int32_t units = (ncb / G) * Q;
            const int32_t grid = (units + 7) / 8 * 8 * G;
            const size_t lds = spdnn::tile_pair_bytes((d.lds_cols + 255) / 256 * 256);  // whole waves of 256 columns
            if (d.mode == kRow2)
                spdnn::fused_row2_kernel<<<grid, spdnn::kBlk, spdnn::kRow2LdsBytes, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.r2, h->bias_dev, N, ncb, G, Q, d.wuni);
            else if (d.multi) {  // several lanes per neuron: the lanes' sums meet in LDS behind the tile pair
                spdnn::VirtInfo vi = d.virt;
                vi.part_off = (uint32_t)lds;
                if (d.mode == kStaged)
                    spdnn::fused_layer_kernel<true, true><<<grid, spdnn::kBlk, lds + kVirtLds, s>>>(
                        Yin, Yout, wv.flags[l % 3], rl, d.w, h->bias_dev, N, h->nblk, G, Q, vi);
                else
                    spdnn::fused_layer_kernel<false, true><<<grid, spdnn::kBlk, lds + kVirtLds, s>>>(
                        Yin, Yout, wv.flags[l % 3], rl, d.w, h->bias_dev, N, h->nblk, G, Q, vi);
            }
            else if (d.mode == kPair && d.relabel)
                spdnn::fused_pair_kernel<true><<<grid, spdnn::kBlk, lds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.w, h->bias_dev, N, ncb, G, Q, d.wuni, d.rn);
            else if (d.mode == kPair)
                spdnn::fused_pair_kernel<false><<<grid, spdnn::kBlk, lds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.w, h->bias_dev, N, ncb, G, Q, d.wuni);
            else if (d.mode == kWidePair && d.pair4 && d.ww.nstage == 2)  // + the all-zero entries and the spill table
                spdnn::fused_wide_pair4_kernel<2, 32><<<grid, spdnn::kBlk, lds + spdnn::kPair4LdsExtra, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.ww, h->bias_dev, N, ncb, G, Q, d.wuni);
            else if (d.mode == kWidePair && d.pair4)
                spdnn::fused_wide_pair4_kernel<4, 16><<<grid, spdnn::kBlk, lds + spdnn::kPair4LdsExtra, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.ww, h->bias_dev, N, ncb, G, Q, d.wuni);
            else if (d.mode == kWidePair)
                spdnn::fused_wide_pair_kernel<<<grid, spdnn::kBlk, lds + spdnn::kPadLds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.ww, h->bias_dev, N, ncb, G, Q, d.wuni);
            else if (d.mode == kWide && d.ww.nstage > 8)
                spdnn::fused_wide_kernel<8><<<grid, spdnn::kBlk, lds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.ww, h->bias_dev, N, ncb, G, Q);
            else if (d.mode == kWide)
                spdnn::fused_wide_kernel<16><<<grid, spdnn::kBlk, lds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.ww, h->bias_dev, N, ncb, G, Q);
            else if (d.mode == kStaged)
                spdnn::fused_layer_kernel<true><<<grid, spdnn::kBlk, lds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.w, h->bias_dev, N, h->nblk, G, Q);
            else
                spdnn::fused_layer_kernel<false><<<grid, spdnn::kBlk, lds, s>>>(
                    Yin, Yout, wv.flags[l % 3], rl, d.w, h->bias_dev, N, h->nblk, G, Q);
            if (h->ooc_host) {  // the slot is free once this kernel is done: refill it with pass p + 2
                HIP_TRY(hipEventRecord(h->ooc_freed[p & 1], s));
                if (p + 2 < P) {
                    HIP_TRY(hipStreamWaitEvent(h->ooc_stream, h->ooc_freed[p & 1], 0));
                    HIP_TRY(ooc_fetch(p + 2));
                }
            }
        }
        if (h->profiling) HIP_TRY(hipEventRecord(h->t1[l], s));
        HIP_TRY(hipGetLastError());
        run = l + 1;
        // Feedback with bounded lag: the number of rows active on entry to layer l+2-kLag bounds all later
        // ones.  That layer's kernel stores it to pinned host memory as it starts, which is polled here
        // (so at most kLag-1 kernels are queued behind the running one); the stream is asked now and then
        // whether it has run dry, only so that a failed launch ends the wait.  Nothing else is put between two
        // layers' kernels: an event recorded after every layer made the gap between them longer.
        if (l + 2 >= kLag) {
            const int32_t lr = l + 2 - kLag;
            volatile int* slot = h->host_counts + lr;
            int32_t c = *slot;
            for (uint32_t spin = 1; c < 0; ++spin) {
                if ((spin & 1023u) == 0) {
                    const hipError_t q = hipStreamQuery(s);
                    if (q == hipSuccess) {  // everything launched is done: the count has been stored
                        c = *slot;
                        if (c < 0) return fail(SPDNN_EHIP, "layer %d finished without reporting its active rows", lr);
                        break;
                    }
                    if (q != hipErrorNotReady) HIP_TRY(q);
                }
                c = *slot;
            }
            std::atomic_thread_fence(std::memory_order_acquire);
            bound = c;
            if (bound == 0) break;
        }
    }
    if (!chain) {
        rot = run;
        final_buf = (run - 1) & 1;
    }
    // the rows that survive the last layer launched: the same compaction, as a kernel of its own.  Its count goes
    // to host_counts[run] (rows on entry to the layer that would come next); after a one-launch run the entries
    // 1 .. L are the launch's own counts, and the survivors' count goes to the spare entry L + 1.
    const int32_t final_slot = chain ? L + 1 : run;
    h->host_counts[L + 1] = -1;
    spdnn::compact_kernel<<<spdnn::kCompactWGs, 1024, 0, s>>>(wv.flags[(rot + 2) % 3], wv.flags[(rot + 1) % 3],
                                                              wv.count[(rot + 1) & 1], wv.count[rot & 1], wv.gid[(rot + 1) & 1],
                                                              wv.gid[rot & 1], wv.cat[rot & 1], h->host_counts + final_slot);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));
    const int32_t n = h->host_counts[final_slot];
    if (n < 0) return fail(SPDNN_EHIP, "layer %d finished without reporting its active rows", run - 1);
    if (chain) {  // rows on entry to every layer, from the launch's counters; "launched" = up to the first layer without rows
        run = L;
        for (int32_t l = 1; l <= L; ++l) {
            h->host_counts[l] = chain_rows_host[(size_t)l];
            if (chain_rows_host[(size_t)l] == 0 && run == L && l < L) run = l + 1;
        }
    }
    *n_active_host = n;
    if (n > 0) {
        const int* cat_f = wv.cat[rot & 1];
        const int* gid_f = wv.gid[rot & 1];
        HIP_TRY(hipMemcpyAsync(active_rows_dev, gid_f, sizeof(int) * (size_t)n, hipMemcpyDeviceToDevice, s));
        if (Y_final_dev) {
            const int n4 = N / 4;
            const size_t total = (size_t)n * n4;
            const int g = (int)std::min<size_t>((total + 255) / 256, 65536);
            spdnn::gather_rows_kernel<<<g, 256, 0, s>>>(reinterpret_cast<const float4*>(wv.Y[final_buf]), cat_f, n, n4,
                                                       reinterpret_cast<float4*>(Y_final_dev));
            HIP_TRY(hipGetLastError());
        }
        HIP_TRY(hipStreamSynchronize(s));
    }
    drain_model.armed = false;
    if (h->profiling) {
        h->prof_layers = run;
        h->prof_ms.assign(run, 0.0f);
        h->prof_rows.assign(run, 0);
        float chain_ms = 0.0f;
        double chain_rows_sum = 0.0;
        if (chain) {  // one launch: its time is shared out among the layers by the rows they had
            HIP_TRY(hipEventElapsedTime(&chain_ms, h->t0[0], h->t1[0]));
            for (int32_t l = 0; l < run; ++l) chain_rows_sum += (double)h->host_counts[l];
        }
        for (int32_t l = 0; l < run; ++l) {
            h->prof_rows[l] = h->host_counts[l];
            if (chain)
                h->prof_ms[l] = chain_rows_sum > 0 ? (float)(chain_ms * (double)h->host_counts[l] / chain_rows_sum) : 0.0f;
            else
                HIP_TRY(hipEventElapsedTime(&h->prof_ms[l], h->t0[l], h->t1[l]));
        }
    }
    return SPDNN_OK;
}

}  // namespace

extern "C" {

const char* spdnn_last_error(void) { return g_err.c_str(); }

int spdnn_weights_bytes(int32_t N, int32_t L, size_t* bytes) {
    if (!bytes) return fail(SPDNN_EINVAL, "bytes is NULL");
    if (!valid_n(N) || L < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1");
    *bytes = arena_bytes_for(N, L, stages_of(N));
    return SPDNN_OK;
}

int spdnn_weights_bytes_for_window(int32_t N, int32_t L, int32_t widest_window, size_t* bytes) {
    if (!bytes) return fail(SPDNN_EINVAL, "bytes is NULL");
    if (!valid_n(N) || L < 1 || widest_window < 1)
        return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1, widest_window >= 1");
    *bytes = arena_bytes_for(N, L, stages_of(std::min(widest_window, N)));
    return SPDNN_OK;
}

int spdnn_scan_windows(int32_t N, int32_t L, const int32_t* const* idx, int32_t where, void* scratch_dev,
                       size_t scratch_bytes, void* hip_stream, int32_t* widest_window) {
    return guarded([&]() -> int {
        if (!widest_window) return fail(SPDNN_EINVAL, "widest_window is NULL");
        if (!valid_n(N) || L < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1");
        if (!idx || !scratch_dev) return fail(SPDNN_EINVAL, "null argument");
        if (where != SPDNN_HOST && where != SPDNN_DEVICE) return fail(SPDNN_EINVAL, "where must be SPDNN_HOST or SPDNN_DEVICE");
        const int32_t nblk = (N + spdnn::kBlk - 1) / spdnn::kBlk;
        const size_t raw = up((size_t)N * spdnn::kNnz * sizeof(int32_t));
        const size_t need = raw + up((size_t)nblk * sizeof(int2)) + up(sizeof(int));
        if (scratch_bytes < need) return fail(SPDNN_ESIZE, "scan scratch has %zu bytes, %zu needed", scratch_bytes, need);
        if (reinterpret_cast<uintptr_t>(scratch_dev) % kAlign) return fail(SPDNN_EINVAL, "scratch must be 256-byte aligned");
        hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
        char* base = static_cast<char*>(scratch_dev);
        int32_t* st_idx = reinterpret_cast<int32_t*>(base);
        int2* win = reinterpret_cast<int2*>(base + raw);
        int* err = reinterpret_cast<int*>(base + raw + up((size_t)nblk * sizeof(int2)));
        HIP_TRY(hipMemsetAsync(err, 0, 2 * sizeof(int), stream));  // error flag, widest window (unused here)
        std::vector<int2> hw(nblk);
        int widest = 4;
        for (int32_t l = 0; l < L; ++l) {
            if (!idx[l]) return fail(SPDNN_EINVAL, "idx[%d] is NULL", l);
            const int32_t* di = idx[l];
            if (where == SPDNN_HOST) {
                HIP_TRY(hipMemcpyAsync(st_idx, idx[l], (size_t)N * spdnn::kNnz * sizeof(int32_t), hipMemcpyHostToDevice, stream));
                di = st_idx;
            }
            spdnn::block_window_kernel<<<nblk, spdnn::kBlk, 0, stream>>>(di, N, win, err, err + 1);
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipMemcpyAsync(hw.data(), win, sizeof(int2) * nblk, hipMemcpyDeviceToHost, stream));
            HIP_TRY(hipStreamSynchronize(stream));
            for (int32_t b = 0; b < nblk; ++b) widest = std::max(widest, hw[b].y);
            // layers that run two neurons per lane give blocks 2u and 2u+1 their common window
            if (N % (2 * spdnn::kBlk) == 0)
                for (int32_t b = 0; b + 1 < nblk; b += 2) {
                    int x, y;  // windows are cyclic
                    spdnn::win_union(hw[b].x, hw[b].y, hw[b + 1].x, hw[b + 1].y, N, x, y);
                    widest = std::max(widest, y);
                }
        }
        int herr = 0;
        HIP_TRY(hipMemcpy(&herr, err, sizeof(int), hipMemcpyDeviceToHost));
        if (herr) return fail(SPDNN_EINVAL, "a column index is outside [0, N)");
        *widest_window = widest;
        return SPDNN_OK;
    });
}

int spdnn_work_bytes(int32_t N, int32_t max_batch, size_t* bytes) {
    if (!bytes) return fail(SPDNN_EINVAL, "bytes is NULL");
    if (!valid_n(N) || max_batch < 0) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, batch >= 0");
    *bytes = carve_work(N, max_batch, nullptr, nullptr);
    return SPDNN_OK;
}

int spdnn_create(spdnn_t* out, int32_t N, int32_t L, const int32_t* const* idx, const float* const* val,
                 const float* bias, int32_t where, void* weights_arena, size_t weights_arena_bytes,
                 void* hip_stream) {
    return guarded([&]() -> int {
        if (!out) return fail(SPDNN_EINVAL, "out is NULL");
        *out = nullptr;
        if (!valid_n(N) || L < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1");
        if (!idx || !val || !bias || !weights_arena) return fail(SPDNN_EINVAL, "null argument");
        if (where != SPDNN_HOST && where != SPDNN_DEVICE) return fail(SPDNN_EINVAL, "where must be SPDNN_HOST or SPDNN_DEVICE");
        if (reinterpret_cast<uintptr_t>(weights_arena) % kAlign) return fail(SPDNN_EINVAL, "weights_arena must be 256-byte aligned");
        for (int32_t l = 0; l < L; ++l)
            if (!idx[l] || !val[l]) return fail(SPDNN_EINVAL, "idx[%d] or val[%d] is NULL", l, l);
        return create_impl(out, N, L, std::vector<int32_t>((size_t)L, 1), nullptr, idx, val, bias, where, weights_arena,
                           weights_arena_bytes, reinterpret_cast<hipStream_t>(hip_stream));
    });
}

int spdnn_ooc_bytes(int32_t N, int32_t L, int32_t widest_window, size_t* device_bytes, size_t* host_bytes) {
    if (!device_bytes || !host_bytes) return fail(SPDNN_EINVAL, "null argument");
    if (!valid_n(N) || L < 1 || widest_window < 1)
        return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1, widest_window >= 1");
    const int cap = stages_of(std::min(widest_window, N));
    *device_bytes = ooc_device_bytes_for(N, L, cap);
    *host_bytes = (size_t)L * block_bytes(N, cap);
    return SPDNN_OK;
}

int spdnn_create_ooc(spdnn_t* out, int32_t N, int32_t L, const int32_t* const* idx, const float* const* val,
                     const float* bias, int32_t where, void* device_arena, size_t device_arena_bytes,
                     void* host_arena, size_t host_arena_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        if (!out) return fail(SPDNN_EINVAL, "out is NULL");
        *out = nullptr;
        if (!valid_n(N) || L < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1");
        if (!idx || !val || !bias || !device_arena || !host_arena) return fail(SPDNN_EINVAL, "null argument");
        if (where != SPDNN_HOST && where != SPDNN_DEVICE) return fail(SPDNN_EINVAL, "where must be SPDNN_HOST or SPDNN_DEVICE");
        if (reinterpret_cast<uintptr_t>(device_arena) % kAlign || reinterpret_cast<uintptr_t>(host_arena) % 16)
            return fail(SPDNN_EINVAL, "device_arena must be 256-byte aligned, host_arena 16-byte aligned");
        for (int32_t l = 0; l < L; ++l)
            if (!idx[l] || !val[l]) return fail(SPDNN_EINVAL, "idx[%d] or val[%d] is NULL", l, l);
        return create_impl(out, N, L, std::vector<int32_t>((size_t)L, 1), nullptr, idx, val, bias, where, device_arena,
                           device_arena_bytes, reinterpret_cast<hipStream_t>(hip_stream), host_arena, host_arena_bytes);
    });
}

int spdnn_csr_passes(int32_t N, int32_t L, const int32_t* const* ptr, const int32_t* const* idx, void* scratch_dev,
                     size_t scratch_bytes, void* hip_stream, int32_t* passes, int32_t* total, int32_t* widest_window) {
    return guarded([&]() -> int {
        if (!valid_n(N) || L < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1");
        if (!ptr || !scratch_dev || !total) return fail(SPDNN_EINVAL, "null argument");
        if (widest_window && !idx) return fail(SPDNN_EINVAL, "widest_window needs idx");
        std::vector<int32_t> po;
        const int rc = scan_csr(N, L, ptr, scratch_dev, scratch_bytes, reinterpret_cast<hipStream_t>(hip_stream), &po, idx,
                                widest_window);
        if (rc != SPDNN_OK) return rc;
        int64_t sum = 0;
        for (int32_t l = 0; l < L; ++l) {
            if (passes) passes[l] = po[l];
            sum += po[l];
        }
        if (sum > INT32_MAX) return fail(SPDNN_EINVAL, "too many passes");
        *total = (int32_t)sum;
        return SPDNN_OK;
    });
}

int spdnn_create_csr(spdnn_t* out, int32_t N, int32_t L, const int32_t* const* ptr, const int32_t* const* idx,
                     const float* const* val, const float* bias, void* weights_arena, size_t weights_arena_bytes,
                     void* hip_stream) {
    return guarded([&]() -> int {
        if (!out) return fail(SPDNN_EINVAL, "out is NULL");
        *out = nullptr;
        if (!valid_n(N) || L < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, L >= 1");
        if (!ptr || !idx || !val || !bias || !weights_arena) return fail(SPDNN_EINVAL, "null argument");
        if (reinterpret_cast<uintptr_t>(weights_arena) % kAlign) return fail(SPDNN_EINVAL, "weights_arena must be 256-byte aligned");
        for (int32_t l = 0; l < L; ++l)
            if (!ptr[l] || !idx[l] || !val[l]) return fail(SPDNN_EINVAL, "ptr[%d], idx[%d] or val[%d] is NULL", l, l, l);
        // the arena's head serves as scratch for the scan; nothing else is in it yet
        hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
        std::vector<int32_t> passes_of;
        const int rc = scan_csr(N, L, ptr, weights_arena, weights_arena_bytes, stream, &passes_of);
        if (rc != SPDNN_OK) return rc;
        return create_impl(out, N, L, passes_of, ptr, idx, val, bias, SPDNN_DEVICE, weights_arena, weights_arena_bytes, stream);
    });
}

int spdnn_destroy(spdnn_t h) {
    return guarded([&]() -> int {
        if (!h) return SPDNN_OK;
        if (h->host_counts) (void)hipHostFree(h->host_counts);
        for (int i = 0; i < 2; ++i) {
            if (h->ooc_ready[i]) (void)hipEventDestroy(h->ooc_ready[i]);
            if (h->ooc_freed[i]) (void)hipEventDestroy(h->ooc_freed[i]);
        }
        if (h->ooc_stream) (void)hipStreamDestroy(h->ooc_stream);
        for (int i = 0; i < 2; ++i)
            if (h->in_ready[i]) (void)hipEventDestroy(h->in_ready[i]);
        if (h->in_stream) (void)hipStreamDestroy(h->in_stream);
        for (hipEvent_t e : h->t0) (void)hipEventDestroy(e);
        for (hipEvent_t e : h->t1) (void)hipEventDestroy(e);
        delete h;
        return SPDNN_OK;
    });
}

int spdnn_set_profiling(spdnn_t h, int32_t on) {
    return guarded([&]() -> int {
        if (!h) return fail(SPDNN_EINVAL, "handle is NULL");
        if (on && h->t0.empty()) {
            h->t0.resize(h->L, nullptr);
            h->t1.resize(h->L, nullptr);
            for (int32_t l = 0; l < h->L; ++l) {
                HIP_TRY(hipEventCreate(&h->t0[l]));
                HIP_TRY(hipEventCreate(&h->t1[l]));
            }
        }
        h->profiling = on ? 1 : 0;
        return SPDNN_OK;
    });
}

int spdnn_layer_kernel(spdnn_t h, int32_t l, int32_t* kind) {
    if (!h || !kind) return fail(SPDNN_EINVAL, "null argument");
    if (l < 0 || l >= h->L) return fail(SPDNN_EINVAL, "layer %d outside [0, %d)", l, h->L);
    static_assert(kSingle == SPDNN_KERNEL_SINGLE && kStaged == SPDNN_KERNEL_STAGED && kWide == SPDNN_KERNEL_WIDE &&
                      kPair == SPDNN_KERNEL_PAIR && kWidePair == SPDNN_KERNEL_WIDE_PAIR,
                  "layer modes are the header's kernel kinds");
    const LayerDesc& d = h->layers[h->first_pass[l]];
    *kind = (d.mode == kWidePair && d.pair4) ? SPDNN_KERNEL_WIDE_PAIR4 : d.mode == kRow2 ? SPDNN_KERNEL_ROW2 : d.mode;
    return SPDNN_OK;
}

int spdnn_one_launch(spdnn_t h, int32_t batch, int32_t* yes) {
    if (!h || !yes) return fail(SPDNN_EINVAL, "null argument");
    if (batch < 0) return fail(SPDNN_EINVAL, "batch < 0");
    *yes = one_launch_shape(h, batch, nullptr) ? 1 : 0;
    return SPDNN_OK;
}

int spdnn_layer_passes(spdnn_t h, int32_t l, int32_t* passes) {
    if (!h || !passes) return fail(SPDNN_EINVAL, "null argument");
    if (l < 0 || l >= h->L) return fail(SPDNN_EINVAL, "layer %d outside [0, %d)", l, h->L);
    *passes = h->first_pass[l + 1] - h->first_pass[l];
    return SPDNN_OK;
}

int spdnn_get_profile(spdnn_t h, int32_t cap, int32_t* layers_run, int32_t* rows_in, float* fused_ms) {
    return guarded([&]() -> int {
        if (!h || !layers_run) return fail(SPDNN_EINVAL, "null argument");
        *layers_run = h->prof_layers;
        const int32_t n = std::min<int32_t>(cap, h->prof_layers);
        for (int32_t l = 0; l < n; ++l) {
            if (rows_in) rows_in[l] = h->prof_rows[l];
            if (fused_ms) fused_ms[l] = l < (int32_t)h->prof_ms.size() ? h->prof_ms[l] : 0.0f;
        }
        return SPDNN_OK;
    });
}

int spdnn_infer(spdnn_t h, const float* Y0_dev, int32_t batch, void* work_arena, size_t work_arena_bytes,
                int32_t* n_active_host, int32_t* active_rows_dev, float* Y_final_dev) {
    return guarded([&]() -> int {
        const int rc = check_infer_args(h, Y0_dev, batch, n_active_host, active_rows_dev, Y_final_dev);
        if (rc != SPDNN_OK || batch == 0) return rc;
        if (!work_arena) return fail(SPDNN_EINVAL, "null argument");
        if (reinterpret_cast<uintptr_t>(work_arena) % kAlign) return fail(SPDNN_EINVAL, "work_arena must be 256-byte aligned");
        const size_t need = carve_work(h->N, batch, nullptr, nullptr);
        if (work_arena_bytes < need) return fail(SPDNN_ESIZE, "work arena has %zu bytes, %zu needed", work_arena_bytes, need);
        WorkView wv;
        carve_work(h->N, batch, static_cast<char*>(work_arena), &wv);
        return infer_impl(h, Y0_dev, batch, wv, 0, n_active_host, active_rows_dev, Y_final_dev);
    });
}

int spdnn_infer_static(spdnn_t h, const float* Y0_dev, int32_t batch, int32_t* n_active_host,
                       int32_t* active_rows_dev, float* Y_final_dev) {
    return guarded([&]() -> int {
        const int rc = check_infer_args(h, Y0_dev, batch, n_active_host, active_rows_dev, Y_final_dev);
        if (rc != SPDNN_OK || batch == 0) return rc;
        const size_t need = carve_work(h->N, batch, nullptr, nullptr);
        if (need > kStaticScratchBytes)
            return fail(SPDNN_ESIZE,
                        "batch %d x N %d needs %zu bytes of scratch, the static scratch array holds %zu: use spdnn_infer "
                        "with a work arena",
                        batch, h->N, need, kStaticScratchBytes);
        void* ptr = nullptr;
        const int rs = static_scratch(&ptr);  // this device's copy of the array (looked up at spdnn_create)
        if (rs != SPDNN_OK) return rs;
        WorkView wv;
        carve_work(h->N, batch, static_cast<char*>(ptr), &wv);
        return infer_impl(h, Y0_dev, batch, wv, 0, n_active_host, active_rows_dev, Y_final_dev);
    });
}

int spdnn_host_work_bytes(int32_t N, int32_t rows_per_batch, size_t* bytes) {
    if (!bytes) return fail(SPDNN_EINVAL, "bytes is NULL");
    if (!valid_n(N) || rows_per_batch < 1) return fail(SPDNN_EINVAL, "need 32 <= N <= 65536, N %% 4 == 0, rows_per_batch >= 1");
    *bytes = 2 * up((size_t)rows_per_batch * N * sizeof(float)) + carve_work(N, rows_per_batch, nullptr, nullptr);
    return SPDNN_OK;
}

int spdnn_infer_host(spdnn_t h, const float* Y0_host, int32_t batch, int32_t rows_per_batch, void* work_arena,
                     size_t work_arena_bytes, int32_t* n_active_host, int32_t* active_rows_dev, float* Y_final_dev) {
    return guarded([&]() -> int {
        if (!h) return fail(SPDNN_EINVAL, "handle is NULL");
        if (!n_active_host) return fail(SPDNN_EINVAL, "n_active_host is NULL");
        if (batch < 0 || rows_per_batch < 1) return fail(SPDNN_EINVAL, "need batch >= 0 and rows_per_batch >= 1");
        h->prof_layers = 0;
        *n_active_host = 0;
        if (batch == 0) return SPDNN_OK;
        if (!Y0_host || !work_arena || !active_rows_dev) return fail(SPDNN_EINVAL, "null argument");
        if (Y_final_dev && reinterpret_cast<uintptr_t>(Y_final_dev) % 16) return fail(SPDNN_EINVAL, "Y_final must be 16-byte aligned");
        if (reinterpret_cast<uintptr_t>(work_arena) % kAlign) return fail(SPDNN_EINVAL, "work_arena must be 256-byte aligned");
        const int32_t N = h->N;
        const int32_t step = std::min(rows_per_batch, batch);
        const size_t in_bytes = up((size_t)step * N * sizeof(float));
        const size_t need = 2 * in_bytes + carve_work(N, step, nullptr, nullptr);
        if (work_arena_bytes < need) return fail(SPDNN_ESIZE, "work arena has %zu bytes, %zu needed", work_arena_bytes, need);
        char* base = static_cast<char*>(work_arena);
        float* in[2] = {reinterpret_cast<float*>(base), reinterpret_cast<float*>(base + in_bytes)};
        WorkView wv;
        carve_work(N, step, base + 2 * in_bytes, &wv);
        if (!h->in_stream) {  // made on first use: a second stream of default priority, and one event per input buffer
            HIP_TRY(hipStreamCreateWithFlags(&h->in_stream, hipStreamNonBlocking));
            for (int i = 0; i < 2; ++i) HIP_TRY(hipEventCreateWithFlags(&h->in_ready[i], hipEventDisableTiming));
        }
        // whatever happens below, the copy stream is idle again when the call returns
        struct Drain {
            hipStream_t cs;
            ~Drain() { (void)hipStreamSynchronize(cs); }
        } drain{h->in_stream};
        const int32_t nb = (batch + step - 1) / step;
        auto rows_of = [&](int32_t k) { return std::min(step, batch - k * step); };
        auto fetch = [&](int32_t k) -> hipError_t {  // batch k -> input buffer k & 1, on the copy stream
            hipError_t e = hipMemcpyAsync(in[k & 1], Y0_host + (size_t)k * step * N, sizeof(float) * (size_t)rows_of(k) * N,
                                          hipMemcpyHostToDevice, h->in_stream);
            return e != hipSuccess ? e : hipEventRecord(h->in_ready[k & 1], h->in_stream);
        };
        HIP_TRY(fetch(0));
        int32_t total = 0;
        for (int32_t k = 0; k < nb; ++k) {
            HIP_TRY(hipStreamWaitEvent(h->stream, h->in_ready[k & 1], 0));
            // the other buffer was last read by batch k-1, whose inference has drained the model's stream:
            // its refill runs under the kernels of batch k
            if (k + 1 < nb) HIP_TRY(fetch(k + 1));
            int32_t n = 0;
            const int rc = infer_impl(h, in[k & 1], rows_of(k), wv, k * step, &n, active_rows_dev + total,
                                      Y_final_dev ? Y_final_dev + (size_t)total * N : nullptr);
            if (rc != SPDNN_OK) return rc;
            total += n;
        }
        *n_active_host = total;
        return SPDNN_OK;
    });
}

}  // extern "C"
