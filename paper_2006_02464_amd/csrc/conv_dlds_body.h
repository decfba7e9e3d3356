// Implicit-GEMM convolution on gfx950 MFMA whose K slices travel global -> LDS directly: the
// per-tile body, shared by the per-layer kernels (kernels_conv_dlds.hip) and the resident
// multi-layer kernel (kernels_resident.hip).
//
// Same GEMM view, weight layout, LDS swizzle, MFMA roles and epilogue as the register-staged
// kernel (kernels_conv.hip), for Cin % 64 == 0 (K slices of 64, or of 128 when Cin % 128 == 0
// and the tile says so).  What differs is the pipeline:
// a K slice is fetched by buffer loads that write LDS themselves (buffer_load_dwordx4 ... lds),
// so no registers hold data in flight, no wave spends issue slots on LDS writes, and the LDS
// is a ring of NS stages: while the MFMAs consume slice kt out of stage kt % NS, the loads of
// slices kt+1 .. kt+NS-1 are in flight into the other stages.  One barrier per slice.
//
// Such a load writes the 64 lanes' 16-byte pieces to 1 KiB of consecutive LDS bytes starting
// at the address in M0, i.e. (for 128-byte rows) lane l lands in row l/8 at chunk position l%8
// (row l/16, position l%16 for 256-byte rows).
// The XOR swizzle that the MFMA operand reads need is therefore applied on the global side:
// the lane that owns LDS position (row, pc) fetches the row's logical chunk pc ^ key(row).
// Padded taps and rows beyond M or Cout use an out-of-range offset, for which the load writes
// zeros.  The compiler does not see these loads (inline asm), so the kernel counts them itself:
// every slice is exactly LOADS instructions per thread, they complete in order, and before
// slice kt is read each thread waits until at most (slices still in flight behind kt) * LOADS
// of its loads are outstanding, then the barrier makes every thread's part visible.
#pragma once
#include <algorithm>
#include <type_traits>

#include "conv_common.h"

namespace cw {

// One 16-byte-per-lane buffer load straight into LDS at byte address lds_addr (+ 16*lane).
static __device__ __forceinline__ void load_to_lds(u32x4 desc, unsigned voff, unsigned soff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(desc), "s"(soff)
                 : "memory", "m0");
}

// Waits until at most N of this thread's loads are outstanding, then the workgroup barrier.
template <int N>
static __device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" : : "n"(N) : "memory");
}

// The same, also waiting for this thread's own LDS accesses (reads returned, writes done).
template <int N>
static __device__ __forceinline__ void wait_lds_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(N) : "memory");
}

// Raw buffer descriptor (stride 0) as four scalars, for use as an asm operand.
static __device__ __forceinline__ u32x4 make_desc(const void *p, unsigned bytes) {
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    return u32x4{(unsigned)v, (unsigned)(v >> 32) & 0xffffu, bytes, 0x00020000u};
}

extern __shared__ __attribute__((aligned(16))) unsigned char cw_dyn_lds[];

// LDS bytes of the fused second layer (see the end of the kernel): the first layer's tile, two
// buffers of {a chunk of W2, the matching residual tile}, and one chunk of a third layer's weights.
// The layers' biases sit behind whichever is larger, this or the ring, from the start of the kernel.
constexpr int fused_chunk(int bn, int kg) { return kg > 1 ? 128 : (bn == 128 ? 64 : bn); }   // second-layer channels per chunk
constexpr unsigned fused_lds_bytes(int bm, int bn, int kg) {
    const int p = bm * bn * 2, w2 = fused_chunk(bn, kg) * bn * 2, r = bm * fused_chunk(bn, kg) * 2;
    // with a projection (64-channel form only): 2 x {W2, Wd chunk} + the x2 tile (as large as p)
    const int w3 = bn * fused_chunk(bn, kg) * 2;   // third layer: Cout3 = bn output rows x a chunk of its K
    const int plain = 2 * (w2 + r) + w3, proj = bn == 64 ? 4 * w2 + p + w3 : 0;
    return (unsigned)(p + (plain > proj ? plain : proj));
}
constexpr int kFusedMaxCout2 = 1024;

// KG > 1: KG groups of WARPS_M x WARPS_N waves share the tile; group g takes the 16-k steps
// g, g+KG, ... of every slice and the groups' accumulators are added through LDS at the end.  For
// small tiles with a long K this shortens the per-slice MFMA chain of a wave (and puts several
// waves on each SIMD) without the global exchange of split-K; with split-K on top (tiny M*N, very
// long K) the first group carries the workgroup's sum into that exchange and the others end.
// The body takes the launch's arguments and this workgroup's place bid among the nb workgroups of
// the convolution (a launch may hold two convolutions, see conv_dlds_pair_kernel).
// RAW: bid is the tile index itself (the caller has chosen which tile this workgroup computes).
template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, int BK, int NS, int MODE, bool SPLITK, bool FUSED = false, int KG = 1, bool RAW = false>
static __device__ __forceinline__ void conv_dlds_body(const ConvArgs &a, const int bid, const int nb_packed) {
    // nb_packed: the convolution's tile count with its tile numbering in the top bits (conv_pack_nb)
    const int nb = conv_nb_tiles(nb_packed), panel = conv_nb_panel(nb_packed);
    static_assert(BK == 64 || BK == 128, "K slices of 64 or 128");
    static_assert(KG == 1 || ((BK / 16) % KG == 0 && (!FUSED || KG == 2)), "K groups: whole steps per group");
    static_assert(!FUSED || (!SPLITK && MODE != MODE_STEM && (BN == 64 || BN == 128)), "fused form: whole first layer in one tile");
    constexpr int NT = 64 * WARPS_M * WARPS_N * KG;
    constexpr int WM = BM / WARPS_M, WN = BN / WARPS_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CPR = BK / 8;  // 16-byte chunks per LDS row
    constexpr int X_CHUNKS = BM * CPR, W_CHUNKS = BN * CPR;
    static_assert(X_CHUNKS % NT == 0 && W_CHUNKS % NT == 0, "tile/threads mismatch");
    static_assert(MODE != MODE_STEM || BK == 64, "stem mode: one K slice = two filter rows of 8 taps x 4 channels");
    static_assert(NS >= 2 && NS <= 4, "ring of 2..4 stages");
    constexpr int X_PER = X_CHUNKS / NT, W_PER = W_CHUNKS / NT;
    constexpr int LOADS = X_PER + W_PER;               // load instructions per thread per slice
    constexpr int STAGE = (BM + BN) * BK;              // elements per LDS stage
    constexpr unsigned STAGE_BYTES = STAGE * 2u;
    static_assert((NS - 2) * LOADS < 64, "too many loads in flight for vmcnt");
    typedef typename Mfma<T>::v8 v8;

    T *lds = reinterpret_cast<T *>(cw_dyn_lds);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)cw_dyn_lds;

    const int tid = threadIdx.x;
    // Fused form: both layers' biases are requested now, with ordinary loads, and go to LDS at the
    // end of the set-up arithmetic below, which covers their latency; no counted load is in
    // flight yet at that point (visible to every wave after the first barrier).
    constexpr unsigned BIAS_OFF = FUSED ? (NS * STAGE_BYTES > fused_lds_bytes(BM, BN, KG) ? NS * STAGE_BYTES : fused_lds_bytes(BM, BN, KG)) : 0u;
    constexpr int B2_PER = FUSED ? (kFusedMaxCout2 + NT - 1) / NT : 1;
    float bias1_v = 0.f, bias2_v[B2_PER], bias3_v = 0.f;
    if constexpr (FUSED) {
        if (tid < BN) bias1_v = a.bias[tid];
        if (tid < BN && a.w3) bias3_v = a.bias3[tid];
#pragma unroll
        for (int j = 0; j < B2_PER; ++j) {
            const int n = tid + j * NT;
            bias2_v[j] = n < a.Cout2 ? a.bias2[n] + (a.wd ? a.biasd[n] : 0.f) : 0.f;
        }
    }
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / (WARPS_M * WARPS_N);        // K group of this wave
    const int wq = wave - kg * (WARPS_M * WARPS_N);   // its place in the WARPS_M x WARPS_N layout
    const int wm0 = (wq / WARPS_N) * WM;
    const int wn0 = (wq % WARPS_N) * WN;
    const int lrow = lane & 31;
    const int lhalf = lane >> 5;

    const int tile_id = RAW ? bid : xcd_tile_id(bid, nb);
    const int tiles_n = a.Cout / BN + (a.Cout % BN != 0);
    int tile_m, tile_n;
    if (RAW || FUSED || panel == 0) {   // uniform
        tile_m = tile_id / tiles_n;
        tile_n = tile_id - tile_m * tiles_n;
    } else {
        // panel after panel of tiles_n >> panel channel tiles, row by row inside a panel
        const int pw = tiles_n >> panel;
        const int per = ((a.M + BM - 1) / BM) * pw;
        const int p = tile_id / per, r = tile_id - p * per;
        tile_m = r / pw;
        tile_n = p * pw + (r - tile_m * pw);
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int ktiles = a.K / BK;
    const int kt0 = SPLITK ? blockIdx.y * a.ktiles_per_split : 0;
    const int kt1 = SPLITK ? min(ktiles, kt0 + a.ktiles_per_split) : ktiles;  // no split: the whole K
    const int nsteps = kt1 - kt0;
    int kt = kt0;  // the slice being computed

    // The activation buffer is described from D bytes before its start, D = the offset of the
    // top-left tap relative to a filter's centre pixel, so that  centre offset (per thread, in a
    // VGPR) + tap/channel offset (uniform, in an SGPR)  is never negative.
    // x may be the first Cin channels of a wider tensor: ldx elements from one pixel to the next.
    const unsigned ldx = (unsigned)conv_ldx(a);
    const int pad_h = conv_pad_h(a), pad_w = conv_pad_w(a);
    const unsigned x_bytes = (((unsigned)a.B * a.H * a.W - 1u) * ldx + (unsigned)a.Cin) * 2u;
    const unsigned x_shift = MODE != MODE_CONV ? 0u : (unsigned)(pad_h * a.W + pad_w) * ldx * 2u;
    const u32x4 dx = make_desc(static_cast<const char *>(a.x) - x_shift, x_bytes + x_shift);
    const u32x4 dw = make_desc(a.w, (unsigned)a.Cout * a.K * 2u);

    // This thread's pieces of a slice.  Piece j is LDS position cid = tid + j*NT of the operand's
    // [rows][CPR chunks] stage: row cid/CPR, chunk position cid%CPR, holding logical chunk
    // (cid%CPR) ^ key(row).  Per piece, fixed for the whole K walk: the byte offset of that chunk
    // at the filter's centre pixel, and which taps fall inside the image (bit r*kw+s; for the
    // 1x1 stride-1 case bit 0 = the pixel exists).
    unsigned x_voff[X_PER], x_mask[X_PER];
    if constexpr (MODE == MODE_GEMM) {
#pragma unroll
        for (int j = 0; j < X_PER; ++j) {
            const int cid = tid + j * NT;
            const int row = cid / CPR;
            const int c = (cid % CPR) ^ swz_key<BK>(row);
            const unsigned m = m0 + row;
            x_voff[j] = m * ldx * 2u + c * 16u;
            x_mask[j] = m < (unsigned)a.M ? 1u : 0u;
        }
    } else {
        // The pixel arithmetic (two divisions and the tap mask) is done once per tile row, by
        // thread `row`, and handed to the threads that load the row's chunks through LDS: a
        // thread has up to 8 pieces in as many rows, and with one wave per SIMD the arithmetic
        // of each would cost about as much as a K slice.
        static_assert(NT >= BM, "one thread per tile row");
        __shared__ u32x2 s_row[BM];
        if (tid < BM) {
            const unsigned m = m0 + tid;
            unsigned mask = 0, voff = 0;
            if (m < (unsigned)a.M) {
                const unsigned t = fast_div(m, a.wo_div);
                const unsigned q = m - t * a.Wo;
                const unsigned n = fast_div(t, a.ho_div);
                const unsigned p = t - n * a.Ho;
                if (MODE == MODE_STEM) {
                    // Input = 4-channel pixels (8 bytes) of an image already padded by the cast; no masks.
                    voff = ((n * a.H + p * a.stride) * a.W + q * a.stride) * 8u;
                    mask = 1u;
                } else {
                    const int ihc = p * a.stride, iwc = q * a.stride;
                    voff = (unsigned)((n * a.H + ihc) * a.W + iwc) * ldx * 2u;
                    const int r_lo = max(0, pad_h - ihc), r_hi = min(a.kh, a.H + pad_h - ihc);
                    const int s_lo = max(0, pad_w - iwc), s_hi = min(a.kw, a.W + pad_w - iwc);
                    // in-range columns s_lo..s_hi-1 replicated into every in-range filter row r_lo..r_hi-1:
                    // a multiplication by the rows' unit bits (no carries: cols < 2^kw)
                    unsigned row_units = 0;  // bit r*kw for every filter row r
                    for (int r = 0; r < a.kh; ++r) row_units |= 1u << (r * a.kw);
                    const unsigned cols = ((1u << s_hi) - 1u) & ~((1u << s_lo) - 1u);
                    const unsigned rows = row_units & (unsigned)((1ull << (r_hi * a.kw)) - 1ull) & ~((1u << (r_lo * a.kw)) - 1u);
                    mask = cols * rows;
                }
            }
            s_row[tid] = u32x2{voff, mask};
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < X_PER; ++j) {
            const int cid = tid + j * NT;
            const int row = cid / CPR;
            const int c = (cid % CPR) ^ swz_key<BK>(row);
            const u32x2 ri = s_row[row];
            // Stem: a K slice is filter rows 2kt, 2kt+1; of its 8 chunks, chunk c is row c/4, taps
            // 2(c%4), 2(c%4)+1: 16 contiguous, 16-byte aligned bytes (even stride, even W).
            x_voff[j] = ri.x + (MODE == MODE_STEM ? (unsigned)(c >> 2) * a.W * 8u + (c & 3) * 16u : c * 16u);
            x_mask[j] = ri.y;
        }
    }
    unsigned w_off[W_PER];
#pragma unroll
    for (int j = 0; j < W_PER; ++j) {
        const int cid = tid + j * NT;
        const int row = cid / CPR;
        const int c = (cid % CPR) ^ swz_key<BK>(row);
        const int n = n0 + row;
        w_off[j] = n < a.Cout ? ((unsigned)n * a.K + c * 8) * 2u : kOob;
    }
    if constexpr (FUSED) {
        float *sb = reinterpret_cast<float *>(cw_dyn_lds + BIAS_OFF);
        if (tid < BN) sb[tid] = bias1_v;
#pragma unroll
        for (int j = 0; j < B2_PER; ++j) {
            const int n = tid + j * NT;
            if (n < a.Cout2) sb[BN + n] = bias2_v[j];
        }
        if (tid < BN && a.w3) sb[BN + a.Cout2 + tid] = bias3_v;
    }

    // (r, s, c0) of the next K slice to load: k0 = kt*BK = (r*kw + s)*Cin + c0.
    int fr = 0, fs = 0, fc0 = 0;
    if (!SPLITK) {
        // one workgroup walks the whole K: it starts at (0, 0, 0), no divisions needed
    } else if (MODE == MODE_GEMM) {
        fc0 = kt0 * BK;
    } else if (MODE == MODE_CONV) {
        const int k0 = kt0 * BK;
        const int rs = k0 / a.Cin;
        fc0 = k0 - rs * a.Cin;
        fr = rs / a.kw;
        fs = rs - fr * a.kw;
    }

    // The loads of the next slice to fetch, in pieces: piece idx < X_PER is an activation load,
    // the others are weight loads.  begin() fixes the slice's uniform operands, piece() issues
    // one load, end() advances (r, s, c0).
    unsigned is_soff = 0, is_tbit = 0, is_dst = 0, is_kb = 0;
    auto issue_begin = [&](int kt, int stage) {
        is_soff = MODE == MODE_GEMM   ? (unsigned)fc0 * 2u
                  : MODE == MODE_STEM ? (unsigned)kt * (2u * a.W * 8u)
                                      : ((unsigned)(fr * a.W + fs) * ldx + (unsigned)fc0) * 2u;
        is_tbit = MODE == MODE_CONV ? (1u << (fr * a.kw + fs)) : 1u;
        is_dst = lds_base + (unsigned)stage * STAGE_BYTES + (unsigned)wave * 1024u;
        is_kb = (unsigned)kt * (BK * 2u);
    };
    auto issue_piece = [&](int idx) {  // idx is a compile-time constant after unrolling
        if (idx < X_PER)
            load_to_lds(dx, (x_mask[idx] & is_tbit) ? x_voff[idx] : kOob, is_soff, is_dst + idx * (NT * 16));
        else
            load_to_lds(dw, w_off[idx - X_PER], is_kb, is_dst + BM * BK * 2 + (idx - X_PER) * (NT * 16));
    };
    auto issue_end = [&]() {
        fc0 += BK;
        if (MODE == MODE_CONV && fc0 == a.Cin) {
            fc0 = 0;
            if (++fs == a.kw) { fs = 0; ++fr; }
        }
    };
    auto issue = [&](int kt, int stage) {
        issue_begin(kt, stage);
#pragma unroll
        for (int idx = 0; idx < LOADS; ++idx) issue_piece(idx);
        issue_end();
    };

    f32x16 acc[TM][TN];  // [pixel tile][channel tile]; MFMA rows = channels, columns = pixels
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // MFMAs of one K slice.  Operand fragments are fetched from LDS DEPTH-1 16-k steps ahead of
    // the MFMAs that use them.  A wave tile of 64x64 has 4 MFMAs per step, enough to cover the
    // LDS latency with one step of lookahead; the smaller wave tiles have 1 or 2, less than that
    // latency, and look 3 steps ahead.
    // with_loads: the loads of the slice announced by issue_begin() are issued a few at a time
    // behind each 16-k step's MFMAs.  A load instruction occupies the CU's address path for 16
    // clocks per wave; issued in one burst ahead of the MFMAs, the four waves' bursts would hold
    // every wave back for about as long as the MFMAs themselves take.
    auto compute = [&](int stage, auto with_loads) {
        const T *sX = lds + stage * STAGE;
        const T *sW = sX + BM * BK;
        constexpr int KK = BK / 16 / KG;                               // 16-k steps of this wave per slice
        constexpr int DEPTH0 = TM * TN >= 4 ? 2 : 4;
        constexpr int DEPTH = DEPTH0 < KK ? DEPTH0 : (KK > 1 ? KK : 2);  // fragment sets held
        v8 fx[DEPTH][TM], fw[DEPTH][TN];
        auto fetch = [&](int t, v8(&qx)[TM], v8(&qw)[TN]) {
            const int kk = KG == 1 ? t : kg + t * KG;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                qx[i] = *reinterpret_cast<const v8 *>(sX + swz<BK>(wm0 + i * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                qw[j] = *reinterpret_cast<const v8 *>(sW + swz<BK>(wn0 + j * 32 + lrow, kk * 2 + lhalf));
        };
#pragma unroll
        for (int t = 0; t < DEPTH - 1 && t < KK; ++t) fetch(t, fx[t], fw[t]);
#pragma unroll
        for (int t = 0; t < KK; ++t) {
            if (t + DEPTH - 1 < KK) fetch(t + DEPTH - 1, fx[(t + DEPTH - 1) % DEPTH], fw[(t + DEPTH - 1) % DEPTH]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::mma(fw[t % DEPTH][j], fx[t % DEPTH][i], acc[i][j]);
            if (decltype(with_loads)::value) {
#pragma unroll
                for (int idx = t * LOADS / KK; idx < (t + 1) * LOADS / KK; ++idx) issue_piece(idx);
            }
        }
    };

    const EpiPos pos{m0, n0, wm0, wn0, lrow, lhalf};
    EpiOperands<TM, TN> eo;

    // Prologue: the first min(NS-1, nsteps) slices into stages 0, 1, ...
    const int ahead = min(NS - 1, nsteps);
#pragma unroll
    for (int u = 0; u < NS - 1; ++u)
        if (u < ahead) issue(kt0 + u, u);  // uniform

    // Steady state: slice kt sits in stage `cur`; behind it NS-2 more slices are in flight.  After
    // the barrier every wave has finished the MFMAs of slice kt-1, so its stage (the one before
    // `cur` in the ring) takes the loads of slice kt+NS-1, which then fly during NS-1 slices of
    // MFMAs.
    int cur = 0;
    for (; kt + (NS - 1) < kt1; ++kt) {
        wait_loads_and_barrier<(NS - 2) * LOADS>();
        issue_begin(kt + NS - 1, cur == 0 ? NS - 1 : cur - 1);
        compute(cur, std::true_type{});
        issue_end();
        cur = cur + 1 == NS ? 0 : cur + 1;
    }
    // Tail: the last `ahead` slices, nothing left to load; with r slices still behind the one
    // about to be read, r*LOADS loads may stay outstanding.  Without split-K the operands of the
    // epilogue are requested before the last slice's MFMAs (measured: requesting them at the very
    // start instead delays the first slice by as much as it saves at the end).
    auto tail = [&](auto behind) {
        constexpr int u = decltype(behind)::value;  // slices still in flight behind this one
        if (u < kt1 - kt) {                         // uniform
            wait_loads_and_barrier<u * LOADS>();
            if (!SPLITK && !FUSED && u == 0 && kg == 0) epilogue_load<TM, TN>(eo, a, pos);
            compute(cur, std::false_type{});
            cur = cur + 1 == NS ? 0 : cur + 1;
            ++kt;
        }
    };
    if constexpr (NS >= 4) tail(std::integral_constant<int, 2>{});
    if constexpr (NS >= 3) tail(std::integral_constant<int, 1>{});
    tail(std::integral_constant<int, 0>{});

    if (!SPLITK && !FUSED && nsteps <= 0 && kg == 0) epilogue_load<TM, TN>(eo, a, pos);
    if constexpr (KG > 1 && !FUSED) {
        // Groups 1.. hand their accumulators to group 0 through LDS (the ring is free once every
        // wave has passed the barrier); group 0 adds them in group order and goes on alone.
        static_assert((KG - 1) * BM * BN * 4 <= NS * (int)STAGE_BYTES, "K-group exchange does not fit the ring");
        float *xch = reinterpret_cast<float *>(cw_dyn_lds);
        wait_lds_loads_and_barrier<0>();
        if (kg > 0) {
            float *dst = xch + ((kg - 1) * (WARPS_M * WARPS_N) + wq) * (TM * TN * 16 * 64) + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) dst[((i * TN + j) * 16 + e) * 64] = acc[i][j][e];
        }
        wait_lds_loads_and_barrier<0>();
        if (kg > 0) return;
#pragma unroll
        for (int g = 1; g < KG; ++g) {
            const float *src = xch + ((g - 1) * (WARPS_M * WARPS_N) + wq) * (TM * TN * 16 * 64) + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] += src[((i * TN + j) * 16 + e) * 64];
        }
    }

    if constexpr (FUSED) {
        // ---- second layer: y[m][:] = act2(res[m][:] + bias2 + W2 * p[m][:]),  p = act(acc + bias) ----
        // BN == Cout: the tile holds every channel of its BM pixels, so the 1x1 convolution that
        // consumes them needs nothing from other workgroups.  p goes to LDS in operand layout
        // (rows of BN elements, swizzled) and stays; the second layer's Cout2 channels are walked
        // in chunks of BN2 (= BN, or 64 when BN is 128 so that two workgroups still share a CU's
        // LDS) with the same waves and accumulators.  Per chunk, W2[chunk] (BN2 x BN) and the
        // residual tile (BM x BN2) are fetched straight into LDS, double buffered: chunk
        // c+1 is requested before the MFMAs of chunk c.  Loads and stores complete in issue order,
        // so when chunk c is awaited only the stores of chunk c-1 may still be outstanding.
        // With two wave groups (which split K in the first layer) the chunk is 128 channels wide and
        // the groups take its two halves.
        constexpr int BN2 = fused_chunk(BN, KG);                   // second-layer channels per chunk
        constexpr int CP2 = BN / 8, CR2 = BN2 / 8;                 // 16-byte chunks per row: p and W2 / residual
        constexpr int W2_PER = BN2 * CP2 / NT, R_PER = BM * CR2 / NT, X2_PER = BM * CP2 / NT;
        static_assert(BN2 * CP2 % NT == 0 && BM * CR2 % NT == 0 && BM * CP2 % NT == 0, "tile/threads mismatch");
        constexpr int TN2 = BN2 / (WARPS_N * KG) / 32;             // channel tiles per wave in the second layer
        static_assert(TN2 >= 1 && TN2 <= TN, "second-layer wave tile");
        const int wn2 = (kg * WARPS_N + wq % WARPS_N) * (BN2 / (WARPS_N * KG));
        constexpr int ST = TM * TN2 * 2;                           // stores per thread per chunk
        constexpr unsigned P_BYTES = BM * BN * 2u, W2_BYTES = BN2 * BN * 2u, R_BYTES = BM * BN2 * 2u;
        constexpr unsigned BUF_BYTES = W2_BYTES + R_BYTES;
        static_assert(BIAS_OFF + (BN + kFusedMaxCout2 + BN) * 4 <= 160 * 1024, "second layer does not fit the LDS");
        T *sP = lds;
        const float *sBias1 = reinterpret_cast<const float *>(cw_dyn_lds + BIAS_OFF);
        const float *sBias = sBias1 + BN;
        const int chunks = a.Cout2 / BN2;
        const u32x4 dw2 = make_desc(a.w2, (unsigned)a.Cout2 * BN * 2u);
        const u32x4 dres = make_desc(a.res, (unsigned)a.M * a.Cout2 * 2u);
        unsigned w2_voff[W2_PER], r_voff[R_PER];
#pragma unroll
        for (int j = 0; j < W2_PER; ++j) {
            const int cid = tid + j * NT, row = cid / CP2, c = (cid % CP2) ^ swz_key<BN>(row);
            w2_voff[j] = (unsigned)(row * BN + c * 8) * 2u;
        }
#pragma unroll
        for (int j = 0; j < R_PER; ++j) {
            const int cid = tid + j * NT, row = cid / CR2, c = (cid % CR2) ^ swz_key<BN2>(row);
            const unsigned m = m0 + row;
            r_voff[j] = m < (unsigned)a.M ? (m * (unsigned)a.Cout2 + c * 8) * 2u : kOob;
        }
        // With a projection shortcut (a.wd): no residual tile is read.  The x2 tile (BM x BN) is
        // fetched once with chunk 0 and stays; per chunk Wd[chunk] (BN x BN) comes with W2[chunk],
        // and the chunk's sum runs over both products (K = 2*BN).
        const bool proj = BN == 64 && a.wd != nullptr;  // uniform
        const u32x4 dwd = make_desc(proj ? a.wd : a.w2, (unsigned)a.Cout2 * BN * 2u);
        const u32x4 dx2 = make_desc(proj ? a.x2 : a.res, (unsigned)a.M * BN * 2u);
        unsigned x2_voff[X2_PER];
#pragma unroll
        for (int j = 0; j < X2_PER; ++j) {
            const int cid = tid + j * NT, row = cid / CP2, c = (cid % CP2) ^ swz_key<BN>(row);
            const unsigned m = m0 + row;
            x2_voff[j] = m < (unsigned)a.M ? (m * (unsigned)BN + c * 8) * 2u : kOob;
        }
        constexpr unsigned XB_OFF = P_BYTES + 4 * W2_BYTES;   // x2 tile, projection form only
        // Third layer (a.w3; Cout3 = BN): y3 = act3(bias3 + W3 * y).
        // Its K is the second layer's Cout2, walked in the same chunks: once a chunk of y is final
        // (rounded to the storage type, as it is stored), the threads write it back over the residual
        // tile they have just read, element for element, which is then the chunk's activation operand;
        // W3[:, chunk] comes into a buffer of its own while the chunk's second-layer MFMAs run.  The
        // waves keep the first layer's channel split; acc3 lives across the chunks.
        constexpr bool THIRD_OK = BN / (WARPS_N * KG) >= 32;   // every wave gets whole 32-channel tiles of the third layer
        const bool third = THIRD_OK && a.w3 != nullptr;        // uniform
        constexpr int W3_PER = BN * CR2 / NT;
        static_assert(BN * CR2 % NT == 0, "tile/threads mismatch");
        // behind the chunk buffers and, in the 64-channel form (which may carry a projection), the x2 tile
        constexpr unsigned W3_OFF = (BN == 64 && XB_OFF + P_BYTES > P_BYTES + 2 * BUF_BYTES) ? XB_OFF + P_BYTES : P_BYTES + 2 * BUF_BYTES;
        static_assert(W3_OFF + BN * BN2 * 2u <= fused_lds_bytes(BM, BN, KG), "third layer's weights do not fit the LDS plan");
        constexpr int TN3 = THIRD_OK ? BN / (WARPS_N * KG) / 32 : 1;
        static_assert(TN3 <= TN, "third-layer wave tile");
        const int wn3 = (kg * WARPS_N + wq % WARPS_N) * (BN / (WARPS_N * KG));
        const u32x4 dw3 = make_desc(third ? a.w3 : a.w2, (unsigned)BN * a.Cout2 * 2u);
        unsigned w3_voff[W3_PER];
#pragma unroll
        for (int j = 0; j < W3_PER; ++j) {
            const int cid = tid + j * NT, row = cid / CR2, c = (cid % CR2) ^ swz_key<BN2>(row);
            w3_voff[j] = (unsigned)(row * a.Cout2 + c * 8) * 2u;
        }
        auto issue_w3 = [&](int c) {
            const unsigned dst = lds_base + W3_OFF + (unsigned)wave * 1024u;
#pragma unroll
            for (int j = 0; j < W3_PER; ++j) load_to_lds(dw3, w3_voff[j], (unsigned)c * (BN2 * 2u), dst + j * (NT * 16));
        };
        f32x16 acc3[TM][TN3];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN3; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc3[i][j][e] = 0.f;
        // Third layer together with the projection: there is no residual tile to write the chunk of y over,
        // so it goes to the room of the second {W2, Wd} buffer, and the chunks' weights come through
        // the first buffer alone, requested as soon as every wave has finished the chunk's products.
        const bool single = third && proj;
        auto buf_off = [&](int c) { return P_BYTES + (single ? 0u : (unsigned)(c & 1)) * (proj ? 2 * W2_BYTES : BUF_BYTES); };
        auto issue_chunk = [&](int c) {
            const unsigned dst = lds_base + buf_off(c) + (unsigned)wave * 1024u;
#pragma unroll
            for (int j = 0; j < W2_PER; ++j) load_to_lds(dw2, w2_voff[j], (unsigned)c * W2_BYTES, dst + j * (NT * 16));
            if (proj) {
#pragma unroll
                for (int j = 0; j < W2_PER; ++j) load_to_lds(dwd, w2_voff[j], (unsigned)c * W2_BYTES, dst + W2_BYTES + j * (NT * 16));
                if (c == 0) {
#pragma unroll
                    for (int j = 0; j < X2_PER; ++j) load_to_lds(dx2, x2_voff[j], 0u, lds_base + XB_OFF + (unsigned)wave * 1024u + j * (NT * 16));
                }
            } else {
#pragma unroll
                for (int j = 0; j < R_PER; ++j) load_to_lds(dres, r_voff[j], (unsigned)c * (BN2 * 2u), dst + W2_BYTES + j * (NT * 16));
            }
        };

        // every wave is done with the ring (the last slice's barrier came before its MFMAs)
        wait_loads_and_barrier<0>();
        issue_chunk(0);
        if constexpr (KG > 1) {
            // The second group hands its accumulators to the first through the room of chunk
            // buffer 1, which chunk 1 claims only after the barrier that ends the additions;
            // chunk 0's loads stay in flight meanwhile.
            static_assert((KG - 1) * BM * BN * 4 <= (int)(2 * W2_BYTES < BUF_BYTES ? 2 * W2_BYTES : BUF_BYTES), "K-group exchange does not fit a chunk buffer");
            float *xch = reinterpret_cast<float *>(cw_dyn_lds + buf_off(1)) + wq * (TM * TN * 16 * 64) + lane;
            if (kg > 0) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) xch[((i * TN + j) * 16 + e) * 64] = acc[i][j][e];
            }
            wait_lds_loads_and_barrier<2 * W2_PER + (R_PER > X2_PER ? R_PER : X2_PER)>();
            if (kg == 0) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[i][j][e] += xch[((i * TN + j) * 16 + e) * 64];
            }
        }
        // first layer's epilogue into LDS: + bias, activation, one rounding to the storage type
        if (kg == 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int n = wn0 + j * 32 + q * 16 + lhalf * 8;
                    T out[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float v = acc[i][j][8 * q + e] + sBias1[n + e];
                        out[e] = (T)(a.relu ? fmaxf(v, 0.f) : v);   // the fused form is planned for ReLU / no activation only
                    }
                    *reinterpret_cast<u32x4 *>(sP + swz<BN>(wm0 + i * 32 + lrow, n >> 3)) = *reinterpret_cast<const u32x4 *>(out);
                }
        }
        const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (unsigned)a.M * a.Cout2 * 2u);
        for (int c = 0; c < chunks; ++c) {
            // chunk c has landed (mine: vmcnt; everyone's: barrier); p and the bias are visible;
            // every wave has finished reading the buffer that chunk c+1 is about to overwrite
            if (c == 0) wait_lds_loads_and_barrier<0>(); else wait_lds_loads_and_barrier<ST>();
            if (third) issue_w3(c);   // ahead of the next chunk's loads: it is awaited first
            if (!single && c + 1 < chunks) issue_chunk(c + 1);
            const T *sW2 = reinterpret_cast<const T *>(cw_dyn_lds + buf_off(c));
            T *sR = reinterpret_cast<T *>(cw_dyn_lds + buf_off(c)) + BN2 * BN;  // residual tile, or Wd[chunk] in projection form
            T *sQ = proj ? reinterpret_cast<T *>(cw_dyn_lds + P_BYTES + 2 * W2_BYTES) : sR;   // the chunk of y as the third layer's operand
            const T *sXb = reinterpret_cast<const T *>(cw_dyn_lds + XB_OFF);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
            auto product = [&](const T *sA, const T *sB) {
#pragma unroll
                for (int kk = 0; kk < BN / 16; ++kk) {
                    v8 px[TM], pw[TN2];
#pragma unroll
                    for (int i = 0; i < TM; ++i) px[i] = *reinterpret_cast<const v8 *>(sA + swz<BN>(wm0 + i * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
                    for (int j = 0; j < TN2; ++j) pw[j] = *reinterpret_cast<const v8 *>(sB + swz<BN>(wn2 + j * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN2; ++j) acc[i][j] = Mfma<T>::mma(pw[j], px[i], acc[i][j]);
                }
            };
            product(sP, sW2);
            if (proj) product(sXb, sR);
            if (single) {
                // every wave is done with the one weight buffer (only LDS reads are awaited: older than
                // the third layer's weights there are at most the last chunk's stores)
                wait_lds_loads_and_barrier<ST + W3_PER>();
                if (c + 1 < chunks) issue_chunk(c + 1);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const unsigned m = m0 + wm0 + i * 32 + lrow;
#pragma unroll
                for (int j = 0; j < TN2; ++j)
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int nl = wn2 + j * 32 + q * 16 + lhalf * 8;   // channel inside the chunk
                        u32x4 rraw = *reinterpret_cast<const u32x4 *>(sR + swz<BN2>(wm0 + i * 32 + lrow, nl >> 3));
                        if (proj) rraw = u32x4{0u, 0u, 0u, 0u};   // the shortcut is already in the sum
                        const T *r = reinterpret_cast<const T *>(&rraw);
                        const float *b = sBias + c * BN2 + nl;
                        T out[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float v = acc[i][j][8 * q + e] + b[e] + (float)r[e];
                            out[e] = (T)(a.relu2 ? fmaxf(v, 0.f) : v);
                        }
                        const unsigned o = m < (unsigned)a.M ? (m * (unsigned)a.Cout2 + (unsigned)(c * BN2 + nl)) * 2u : kOob;
                        __builtin_amdgcn_raw_buffer_store_b128(*reinterpret_cast<const u32x4 *>(out), ry, o, 0, 0);
                        if (third) *reinterpret_cast<u32x4 *>(sQ + swz<BN2>(wm0 + i * 32 + lrow, nl >> 3)) = *reinterpret_cast<const u32x4 *>(out);
                    }
            }
            if (third) {
                // The chunk of y is in LDS (everyone's: barrier) and W3[:, chunk] has landed: younger than
                // it are only the next chunk's loads and this chunk's stores.
                if (c + 1 >= chunks) wait_lds_loads_and_barrier<ST>();
                else if (proj) wait_lds_loads_and_barrier<2 * W2_PER + ST>();
                else wait_lds_loads_and_barrier<W2_PER + R_PER + ST>();
                const T *sW3 = reinterpret_cast<const T *>(cw_dyn_lds + W3_OFF);
#pragma unroll
                for (int kk = 0; kk < BN2 / 16; ++kk) {
                    v8 px[TM], pw[TN3];
#pragma unroll
                    for (int i = 0; i < TM; ++i) px[i] = *reinterpret_cast<const v8 *>(sQ + swz<BN2>(wm0 + i * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
                    for (int j = 0; j < TN3; ++j) pw[j] = *reinterpret_cast<const v8 *>(sW3 + swz<BN2>(wn3 + j * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN3; ++j) acc3[i][j] = Mfma<T>::mma(pw[j], px[i], acc3[i][j]);
                }
            }
        }
        if (third) {
            const float *sBias3 = sBias + a.Cout2;
            const __amdgpu_buffer_rsrc_t ry3 = make_rsrc(a.y3, (unsigned)a.M * BN * 2u);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const unsigned m = m0 + wm0 + i * 32 + lrow;
#pragma unroll
                for (int j = 0; j < TN3; ++j)
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int n = wn3 + j * 32 + q * 16 + lhalf * 8;
                        T out[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float v = acc3[i][j][8 * q + e] + sBias3[n + e];
                            out[e] = (T)(a.relu3 ? fmaxf(v, 0.f) : v);
                        }
                        const unsigned o = m < (unsigned)a.M ? (m * (unsigned)BN + (unsigned)n) * 2u : kOob;
                        __builtin_amdgcn_raw_buffer_store_b128(*reinterpret_cast<const u32x4 *>(out), ry3, o, 0, 0);
                    }
            }
        }
        return;
    }
    if (SPLITK) {
        if (!splitk_exchange<TM, TN>(acc, a, pos, tile_id)) return;
        epilogue_load<TM, TN>(eo, a, pos);
    }
    epilogue_store<T, TM, TN>(acc, eo, a, pos);
}

// LDS stages per tile: 4 where that still lets two workgroups share a CU's 160 KiB, else 3.
template <int BM, int BN, int BK>
struct RingDepth {
    static constexpr int stage = (BM + BN) * BK * 2;
    static constexpr int value = stage * 4 <= 80 * 1024 ? 4 : (stage * 3 <= 160 * 1024 ? 3 : 2);
};

}  // namespace cw
