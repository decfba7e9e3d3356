// A run of convolution layers as ONE launch of resident workgroups.
//
// Per-layer launches pay, for every layer, a dispatch, a cache write-back and invalidate, the
// ramp-up of 200-400 workgroups and their tail: 3.5-4.5 us around K loops of 1.5-6 us in the later
// stages of a ResNet at batch 16.  Here 256 workgroups (one per CU) are launched once and walk the
// layers themselves.  The batch is cut into 8 partitions of B/8 images; partition p belongs to the 32
// workgroups that run on XCD p: a workgroup reads the XCC_ID register to learn where it is (the
// hardware deals workgroups out to the XCDs in turn, 32 to each, but where the turn starts depends on
// the launches before).
// Everything a partition produces is consumed by the same XCD, so producer and consumer
// meet in that XCD's L2 and no cache maintenance is needed between layers:
//   * a tensor written inside the run has its own workspace region, written once per launch and
//     read only after it is complete, so no cache can hold a stale copy of it;
//   * a tile's stores are complete (vmcnt(0) in every thread, then the workgroup barrier) before
//     its completion flag is stored with device scope; consumers poll the flags of the layers they
//     read (all tiles of the partition) with device-scope loads, then start their own loads.
// Tile t of a layer is computed by workgroup t % 32 of the partition (static, in order), so the
// plan stays a pure function of (model, batch).  Every wait is bounded: after spin_limit polls the
// workgroup raises the error word (host-visible) and leaves, and every other wait sees the word and
// leaves too; EXEC then reports an error instead of hanging.
// Flags hold epoch numbers: "done" means equal to *epoch + 1, and a one-thread launch behind the
// run increments *epoch, so flags never need clearing.
//
// Measured on an MI355X (ResNet-50, 224x224, batch 16, the 52 convolutions after the max pool): 846 us
// as one resident launch against 445 us as per-layer launches (fused and paired).  Without any
// waiting the resident form still takes 723 us: a workgroup owns its CU alone (the kernel holds
// every tile shape, 256 + 91 registers per lane and up to 144 KiB of LDS) and runs its tiles one
// after the other, so nothing overlaps a tile's set-up, first loads and store drain, which is most
// of a tile in the short-K layers of stages 1-2 (6-7 tiles per workgroup and layer); the flags cost
// another 2.4 us per layer, more than the 1.7 us dispatch they replace.  The per-layer plan therefore
// stays the default and this form is an option (cw_set_resident) with its own parity tests.
#include "conv_dlds_body.h"

namespace cw {

template <typename T, int BM, int BN, int BK, int KG>
static __device__ __forceinline__ void res_tile(const ConvArgs &a, bool gemm, int tile, int tiles) {
    constexpr int WM = BM >= 64 ? 2 : 1, WN = BN >= 64 ? 2 : 1;
    constexpr int NS = RingDepth<BM, BN, BK>::value;
    if (gemm) conv_dlds_body<T, BM, BN, WM, WN, BK, NS, MODE_GEMM, false, false, KG, true>(a, tile, tiles);
    else conv_dlds_body<T, BM, BN, WM, WN, BK, NS, MODE_CONV, false, false, KG, true>(a, tile, tiles);
}

template <typename T>
__global__ __launch_bounds__(256) void resident_kernel(const ResLayer *__restrict__ layers, int n_layers, char *workspace, unsigned *flags,
                                                       int flags_per_part, unsigned *epoch, unsigned *error, unsigned spin_limit) {
    __shared__ int s_go;
    const int tid = threadIdx.x;
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    const int part = __builtin_amdgcn_readfirstlane((int)(xcc & (unsigned)(kResPartitions - 1)));
    // This workgroup's place among its partition's 32: the hardware deals consecutive workgroups out
    // to the 8 XCDs in turn (where the turn starts depends on earlier launches), so the 8 workgroups
    // blockIdx.x = 8g .. 8g+7 land on 8 different XCDs and g is unique within each.  If the hardware
    // ever dealt otherwise, some tiles would have no owner: their consumers' waits time out and the
    // launch reports an error.
    const int wg = blockIdx.x >> 3;
    const unsigned want = __hip_atomic_load(epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
    unsigned *myflags = flags + (size_t)part * flags_per_part;
    for (int L = 0; L < n_layers; ++L) {
        const ResLayer &ly = layers[L];
        const int tiles = ly.tiles;
        if (wg >= tiles) continue;   // uniform
        // ---- wait until every tile of the layers this one reads (same partition) is complete
        if (tid < 64) {
            int ok = 1;
            for (int k = 0; k < 2 && ok; ++k) {
                const int d = ly.dep[k];
                if (d < 0) continue;
                const unsigned *f = myflags + __builtin_amdgcn_readfirstlane(layers[d].flag_base);
                const int n = __builtin_amdgcn_readfirstlane(layers[d].tiles);
                unsigned spins = 0;
                for (;;) {
                    bool all = true;
                    for (int base = 0; base < n; base += 64) {
                        const int i = base + tid;
                        const unsigned v = i < n ? __hip_atomic_load(f + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : want;
                        all = all && v == want;
                    }
                    if (__ballot(!all) == 0ull) break;
                    // giving up: after spin_limit polls, or (looked at now and then) when another workgroup has;
                    // the abort word is device memory beside the epoch, the host-visible word is only written
                    if (++spins > spin_limit || ((spins & 255u) == 0u && __hip_atomic_load(epoch + 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == want)) { ok = 0; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            if (tid == 0) {
                if (!ok) {
                    __hip_atomic_store(epoch + 32, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // this launch is abandoned
                    __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
                s_go = ok;
            }
        }
        __syncthreads();
        const int go = __builtin_amdgcn_readfirstlane(s_go);
        __syncthreads();
        if (!go) return;   // uniform
        // ---- this workgroup's tiles of the layer
        ConvArgs a = ly.a;
        a.x = workspace + reinterpret_cast<size_t>(ly.a.x) + (long long)part * ly.ps_x;
        a.y = workspace + reinterpret_cast<size_t>(ly.a.y) + (long long)part * ly.ps_y;
        a.res = ly.a.res ? workspace + (reinterpret_cast<size_t>(ly.a.res) - 1) + (long long)part * ly.ps_res : nullptr;
        const bool gemm = a.kh == 1 && a.kw == 1 && a.stride == 1 && a.pad == 0;
        for (int t = wg; t < tiles; t += kResGroupsPerPartition) {
            switch (ly.variant) {
                case RV_128x128: res_tile<T, 128, 128, 64, 1>(a, gemm, t, tiles); break;
                case RV_128x64: res_tile<T, 128, 64, 64, 1>(a, gemm, t, tiles); break;
                case RV_64x64: res_tile<T, 64, 64, 64, 1>(a, gemm, t, tiles); break;
                case RV_128x64k128: res_tile<T, 128, 64, 128, 1>(a, gemm, t, tiles); break;
                case RV_64x64k128: res_tile<T, 64, 64, 128, 1>(a, gemm, t, tiles); break;
                case RV_32x32k128g4: res_tile<T, 32, 32, 128, 4>(a, gemm, t, tiles); break;
                default: res_tile<T, 32, 32, 64, 4>(a, gemm, t, tiles); break;
            }
            // the tile's stores are complete in every thread, then the flag goes up
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (tid == 0) __hip_atomic_store(myflags + ly.flag_base + t, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ void resident_bump_kernel(unsigned *epoch) { *epoch = *epoch + 1u; }

static constexpr int kResidentLds = 3 * (128 + 64) * 128 * 2;   // the largest ring among the variants (128x64, K slices of 128)

bool resident_layer_ok(const ResLayer &l, size_t ws_bytes) {
    const ConvArgs &a = l.a;
    if (l.variant < 0 || l.variant >= N_RES_VARIANTS) return false;
    const ResVariantDim d = res_variant_dim(l.variant);
    if (a.Cin <= 0 || a.Cin % d.bk != 0 || a.K != a.kh * a.kw * a.Cin || a.kwp != a.kw || a.khp != a.kh || a.kh * a.kw > 32) return false;
    if (a.M <= 0 || a.Cout <= 0 || a.Cout % 32 != 0 || a.split_k != 1 || a.ktiles_per_split != a.K / d.bk || a.partial || a.nz > 1) return false;
    if (a.relu < 0 || a.relu > 2 || a.B < 1 || a.stride < 1 || !a.w || !a.bias) return false;
    const int ldx = conv_ldx(a), ldy = conv_ldy(a);
    if (ldx < a.Cin || ldy < a.Cout || ldx >= kMaxChannels || ldy >= kMaxChannels) return false;
    if (a.M != a.B * a.Ho * a.Wo) return false;
    if (a.Ho != (a.H + 2 * conv_pad_h(a) - a.kh) / a.stride + 1 || a.Wo != (a.W + 2 * conv_pad_w(a) - a.kw) / a.stride + 1) return false;
    if (l.tiles != ((a.M + d.bm - 1) / d.bm) * ((a.Cout + d.bn - 1) / d.bn) || l.tiles < 1) return false;
    const long long x_bytes = (long long)a.B * a.H * a.W * ldx * 2, y_bytes = (long long)a.M * ldy * 2, r_bytes = (long long)a.M * a.Cout * 2;
    if (x_bytes + (long long)(conv_pad_h(a) * a.W + conv_pad_w(a)) * ldx * 2 >= (1ll << 31) || y_bytes >= (1ll << 31) || (long long)a.Cout * a.K * 2 >= (1ll << 31)) return false;
    // every partition's tensors inside the workspace (offsets are stored as pointers; res carries +1 so that 0 means none)
    const size_t xo = reinterpret_cast<size_t>(a.x), yo = reinterpret_cast<size_t>(a.y);
    if (xo + (kResPartitions - 1) * (size_t)l.ps_x + (size_t)x_bytes > ws_bytes) return false;
    if (yo + (kResPartitions - 1) * (size_t)l.ps_y + (size_t)y_bytes > ws_bytes) return false;
    if (a.res) {
        const size_t ro = reinterpret_cast<size_t>(a.res) - 1;
        if (ro + (kResPartitions - 1) * (size_t)l.ps_res + (size_t)r_bytes > ws_bytes) return false;
    }
    if (xo % 16 != 0 || yo % 16 != 0 || l.ps_x % 16 != 0 || l.ps_y % 16 != 0 || l.ps_res % 16 != 0) return false;
    if (l.flag_base < 0 || l.dep[0] < -1 || l.dep[1] < -1) return false;
    return true;
}

hipError_t launch_resident(DType dt, const ResidentArgs &a, hipStream_t s) {
    if (!a.layers || a.n_layers < 1 || !a.workspace || !a.flags || !a.epoch || !a.error || a.flags_per_part < 1) return hipErrorInvalidValue;
    if ((size_t)kResPartitions * a.flags_per_part * 4 > kResidentBytes - kResidentFlagsOff) return hipErrorInvalidValue;
    auto kf = resident_kernel<f16>;
    auto kb = resident_kernel<bf16>;
    static hipError_t attr_f = hipFuncSetAttribute(reinterpret_cast<const void *>(kf), hipFuncAttributeMaxDynamicSharedMemorySize, kResidentLds);
    static hipError_t attr_b = hipFuncSetAttribute(reinterpret_cast<const void *>(kb), hipFuncAttributeMaxDynamicSharedMemorySize, kResidentLds);
    if (attr_f != hipSuccess) return attr_f;
    if (attr_b != hipSuccess) return attr_b;
    const dim3 grid(kResPartitions * kResGroupsPerPartition);
    if (dt == DT_F16) kf<<<grid, 256, kResidentLds, s>>>(a.layers, a.n_layers, a.workspace, a.flags, a.flags_per_part, a.epoch, a.error, a.spin_limit);
    else kb<<<grid, 256, kResidentLds, s>>>(a.layers, a.n_layers, a.workspace, a.flags, a.flags_per_part, a.epoch, a.error, a.spin_limit);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    resident_bump_kernel<<<1, 1, 0, s>>>(a.epoch);
    return hipGetLastError();
}

}  // namespace cw
