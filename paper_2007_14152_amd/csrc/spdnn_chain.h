// a1 + a2 + a3 for networks whose layers have at most 1024 neurons: all layers in one launch.
//
// With one output block per layer a workgroup computes every neuron of the rows it is given, so
// the next layer's input for those rows is its own output: nothing crosses workgroups between two
// layers, and the host loop of Listing 1 (kernel, pruning, buffer swap) can run inside the
// workgroup.  A workgroup takes its share of the rows that are active on entry (derive_work, as
// every fused kernel) and walks them through ALL layers: layer l reads its rows from one work
// buffer (layer 0: from the list's slots in the input) and writes them to the other at the slot
// "first row of my share + local number"; the rows of its share that still have a positive output
// are kept as a list of local numbers in LDS, rebuilt after every layer (the pruning of Listing 1,
// per workgroup), and rows that have died are simply not visited again.  A workgroup whose rows
// have all died is done.  After the last layer the survivors' flags are raised as after any
// layer, and the ordinary compaction turns them into the result.
//
// What it saves is everything between two layers of a small network: a 1024-neuron layer on 1000
// rows is a 12-microsecond kernel followed by a gap of about 10 microseconds before the next
// dependent kernel starts.  What it costs: the rows stay with the workgroup they started in, so
// the workgroups' loads drift apart as rows die (no rebalancing), and every workgroup fetches every
// layer's connections (192 KB, from L2 after the first).
//
// Per layer the tile pipeline is that of fused_layer_kernel<false>: single-stage windows, balanced
// tile layout, a neuron's 32 connections in registers.
#pragma once

namespace spdnn {

// Most rows a workgroup may own.  Measured on a 120-layer network of 1024 neurons with rows alive in every layer,
// one launch against one launch per layer: 1000 rows 0.93 against 2.67 ms, 8000 rows 2.16 against 3.36, 30 000 rows
// (118 per workgroup) 5.28 against 5.73, 60 000 rows (236 per workgroup) 9.42 against 8.59: with many rows per
// workgroup the gaps between kernels matter less than the rebalancing the launches give.
constexpr int kChainRows = 128;

struct ChainArgs {
    const LayerWeights* layers;  // [L], device memory: every layer single-stage, one output block
    int L;
    int* layer_rows;             // [L + 1], zero on entry: [l] += rows of this workgroup alive on entry to layer l >= 1
};

// finish_rows for four rows that are not neighbours in the output buffer: row r goes to slot rows[r].
__device__ __forceinline__ unsigned finish_rows_at(float (&a)[kRows], float bj, float* Yout, int N, int j, bool jok,
                                                   int4 rows, int nlive, int lane) {
    float y0 = fminf(fmaxf(a[0] + bj, 0.0f), kClip);
    float y1 = fminf(fmaxf(a[1] + bj, 0.0f), kClip);
    float y2 = fminf(fmaxf(a[2] + bj, 0.0f), kClip);
    float y3 = fminf(fmaxf(a[3] + bj, 0.0f), kClip);
    a[0] = a[1] = a[2] = a[3] = 0.0f;
    const unsigned pos = (__builtin_amdgcn_ballot_w64(y0 > 0.0f) != 0ull ? 1u : 0u) |
                         (__builtin_amdgcn_ballot_w64(y1 > 0.0f) != 0ull ? 2u : 0u) |
                         (__builtin_amdgcn_ballot_w64(y2 > 0.0f) != 0ull ? 4u : 0u) |
                         (__builtin_amdgcn_ballot_w64(y3 > 0.0f) != 0ull ? 8u : 0u);
    transpose_quartet(y0, y1, y2, y3);
    const int r = lane & 3;
    const int row = r == 0 ? rows.x : r == 1 ? rows.y : r == 2 ? rows.z : rows.w;
    if (jok && r < nlive) *reinterpret_cast<float4*>(Yout + (size_t)row * N + (j & ~3)) = make_float4(y0, y1, y2, y3);
    return pos;
}

__global__ __launch_bounds__(kBlk) void fused_chain_kernel(
    const float* __restrict__ Y0, float* Ya, float* Yb,  // layer l writes (l odd ? Yb : Ya) and reads the other one (layer 0: Y0)
    uint8_t* __restrict__ flags, RowLists rl, ChainArgs ca, const float* __restrict__ bias, int N, int Q) {
    extern __shared__ float4 lds4[];
    __shared__ int red_mem[17], scan_mem[17];
    __shared__ uint16_t loc[kChainRows];  // local numbers of my rows that are alive, ascending
    __shared__ uint8_t alive[kChainRows];  // raised by the layer that is running
    __shared__ int in_slot[kChainRows];    // slot of my row i in Y0's buffer (the list of active rows on entry)
    __shared__ int wave_cnt[17];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    WorkItem wi;
    if (!derive_work(rl, 1, 1, Q, wi, kRows, red_mem, scan_mem)) return;
    const int r0 = wi.g0 * kRows;                          // my rows are r0 .. r0 + nrows - 1 of the list on entry,
    const int nrows = min(wi.A, wi.g1 * kRows) - r0;       // and those are their slots in both work buffers
    for (int i = tid; i < nrows; i += kBlk) {
        loc[i] = (uint16_t)i;
        alive[i] = 0;
        in_slot[i] = wi.identity ? r0 + i : rl.cat[r0 + i];
    }
    int nloc = nrows;
    __syncthreads();

    const int j = tid;
    const bool jok = j < N;
    const float bj = jok ? bias[j] : 0.0f;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;
    const uint32_t st_addr = lds_base + tile_offset(store_group(4 * tid) << 4);
    const int wave_col = (tid & ~63) * 4;
    {
        const int pw = __builtin_amdgcn_readfirstlane(3 - ((threadIdx.x >> 8) & 3));
        if (pw == 1) __builtin_amdgcn_s_setprio(1);
        else if (pw == 2) __builtin_amdgcn_s_setprio(2);
        else if (pw == 3) __builtin_amdgcn_s_setprio(3);
    }

    for (int l = 0; l < ca.L; ++l) {
        const LayerWeights w = ca.layers[l];
        const float* Yin = l == 0 ? Y0 : ((l & 1) ? Ya : Yb);
        float* Yout = (l & 1) ? Yb : Ya;
        const int2 win = w.win[0];
        const int c_lo = win.x, ncols = win.y;
        const uint32_t qp = w.qsel[tid];
        const size_t coff = (size_t)win_col(c_lo, min(4 * tid, ncols - 4), N);  // my four staged columns (windows are cyclic)
        const bool staging = wave_col < ncols;

        const int T = (nloc + kRows - 1) / kRows;
        f32x4 st[kRows];
        int4 in4 = make_int4(0, 0, 0, 0);  // slots (in Yin) of the rows of the tile to load next
        // rows of tile t: the alive rows number 4t .. 4t+3 of my share (the last tile repeats its last row)
        auto local_row = [&](int t, int r) -> int {
            return __builtin_amdgcn_readfirstlane((int)loc[min(kRows * t + r, nloc - 1)]);
        };
        auto fetch_rows = [&](int t) {
            const int a = local_row(t, 0), b = local_row(t, 1), c = local_row(t, 2), d = local_row(t, 3);
            if (l == 0)
                in4 = make_int4(__builtin_amdgcn_readfirstlane(in_slot[a]), __builtin_amdgcn_readfirstlane(in_slot[b]),
                                __builtin_amdgcn_readfirstlane(in_slot[c]), __builtin_amdgcn_readfirstlane(in_slot[d]));
            else
                in4 = make_int4(r0 + a, r0 + b, r0 + c, r0 + d);
        };
        auto load_tile = [&]() {
            if (!staging) return;
            st[0] = *reinterpret_cast<const f32x4*>(Yin + (size_t)in4.x * N + coff);
            st[1] = *reinterpret_cast<const f32x4*>(Yin + (size_t)in4.y * N + coff);
            st[2] = *reinterpret_cast<const f32x4*>(Yin + (size_t)in4.z * N + coff);
            st[3] = *reinterpret_cast<const f32x4*>(Yin + (size_t)in4.w * N + coff);
        };
        auto store_tile = [&](int P) {
            if (staging) stage_store(st, st_addr + P * kBufSkew, qp);
        };
        // the first tile's loads go out ahead of the layer's connections, so that both are in flight together
        fetch_rows(0);
        load_tile();
        // my neuron's connections: LDS byte address (buffer 0) of the column, and the weight
        uint32_t off[kNnz];
        float wv[kNnz];
        {
            // (the lane number is made opaque per layer: the 64 load addresses it leads to would otherwise be worked
            // out once, ahead of the layer loop, and kept -- spilled -- for all layers)
            int tl = tid;
            asm volatile("" : "+v"(tl));
            const uint16_t* prel = w.rel + tl;
            const float* pval = w.val + tl;
#pragma unroll
            for (int k = 0; k < kNnz; ++k) {
                off[k] = lds_base + tile_offset((uint32_t)prel[k * kBlk] & (kCap - 1));
                wv[k] = pval[k * kBlk];
            }
        }

        float acc[kRows] = {0.f, 0.f, 0.f, 0.f};
        auto compute = [&](auto Ptag, auto Ktag) {
            constexpr int P = decltype(Ptag)::value;
            constexpr int kbeg = decltype(Ktag)::value;
#pragma unroll
            for (int kk = 0; kk < 16; kk += 8) {
                uint32_t o[8];
                float v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    o[i] = off[kbeg + kk + i];
                    v[i] = wv[kbeg + kk + i];
                }
                fma_block8<P>(acc, o, v);
            }
        };
        auto step = [&](int t, auto Ptag) {
            constexpr int P = decltype(Ptag)::value;
            compute(Ptag, std::integral_constant<int, 0>{});
            if (t + 1 < T) store_tile(P ^ 1);
            if (t + 2 < T) {
                fetch_rows(t + 2);
                load_tile();
            }
            compute(Ptag, std::integral_constant<int, 16>{});
            const int nlive = min(kRows, nloc - kRows * t);
            const int a = local_row(t, 0), b = local_row(t, 1), c = local_row(t, 2), d = local_row(t, 3);
            const unsigned pos = finish_rows_at(acc, bj, Yout, N, j, jok, make_int4(r0 + a, r0 + b, r0 + c, r0 + d), nlive, lane);
            if (lane < nlive && ((pos >> lane) & 1u)) alive[loc[kRows * t + lane]] = 1;  // lane r speaks for row r of the tile
            __syncthreads();
        };
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        store_tile(0);
        if (T > 1) {
            fetch_rows(1);
            load_tile();
        }
        __syncthreads();
        int t = 0;
        for (; t + 1 < T; t += 2) {
            step(t, P0{});
            step(t + 1, P1{});
        }
        if (t < T) step(t, P0{});

        // Listing 1's pruning, inside my share: the rows with a positive output, in ascending order.
        // (Every wave has passed the last step's barrier: alive[] is complete, loc[] no longer read.)
        int base = 0;
        for (int c0 = 0; c0 < nrows; c0 += kBlk) {
            const int i = c0 + tid;
            const bool keep = i < nrows && alive[i] != 0;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(keep);
            if (lane == 0) wave_cnt[wave] = __popcll(m);
            __syncthreads();
            if (tid == 0) {
                int run = 0;
                for (int k = 0; k < 16; ++k) {
                    const int v = wave_cnt[k];
                    wave_cnt[k] = run;
                    run += v;
                }
                wave_cnt[16] = run;
            }
            __syncthreads();
            if (keep) loc[base + wave_cnt[wave] + __popcll(m & ((1ull << lane) - 1ull))] = (uint16_t)i;
            if (i < nrows) alive[i] = 0;
            base += wave_cnt[16];
            __syncthreads();
        }
        nloc = base;
        if (tid == 0 && nloc > 0) atomicAdd(&ca.layer_rows[l + 1], nloc);
        if (nloc == 0) return;  // the same in every lane of the workgroup
    }
    // survivors of the last layer: their flags, as after any layer
    for (int k = tid; k < nloc; k += kBlk) flags[r0 + loc[k]] = 1;
}

}  // namespace spdnn
