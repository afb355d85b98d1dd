// Resident-grid ("streaming") variant of the 3x3 convolution in the paper's channel-slowest flattening, for grids
// of several workgroup tiles per compute unit (Sec. 3.3 Eq. 6, the same contraction as ss_conv_kernel.h).
//
// What differs from the one-tile-per-workgroup kernel:
//   * One workgroup per compute unit walks over its pixel tiles.  The reduction chunks of consecutive tiles form one
//     sequence: while the multiplying waves work on the last chunk of a tile (and write that tile out), the producer
//     waves are already building the first chunks of the next tile in LDS, and the weight fragments of its first
//     steps are already on their way.  The prologue (first loads, first LDS fill) and the store drain of a tile are
//     paid once per workgroup instead of once per tile.
//   * Tile 128*TM output channels x 32*TN pixels with all four multiplying waves along the output channels: no
//     weight fragment is fetched twice inside a workgroup, and with TN = 4 every fetched weight fragment is used for
//     128 pixels, which halves the bytes per matrix instruction through the vector-memory path (the busiest unit of
//     the 64-pixel tiles) at the same LDS traffic per instruction.
//   * Activation fragments and weight fragments travel in register rings whose slots are compile-time registers
//     (the chunk body is fully unrolled); the workgroup barrier that publishes the next chunk sits one step before
//     the end of the current one, so the first fragments of the next chunk are read while the last step multiplies.
//   * The output tile leaves through a small LDS slab private to each wave (32 pixels x 32 channels), so that no
//     workgroup barrier is needed between a tile's last matrix instruction and the next tile's first.
// Staging (tap transpose with v_perm_b32, XOR-swizzled unpadded LDS rows), operand layouts and the arithmetic are
// those of ss_conv_kernel.h; the bias is placed in the accumulators before the first step instead of being added
// after the last (same sum, other order of the fp32 additions).
#ifndef SS_CONV_STREAM_H_
#define SS_CONV_STREAM_H_
#include "ss_conv_kernel.h"

namespace ss {

#ifndef SS_STREAM_PACE
#define SS_STREAM_PACE 0      // s_sleep argument (units of 64 clocks) between a producer thread's load / LDS-write pairs; 0 = none
#endif

// Workgroup barrier that orders LDS traffic only: the waves' outstanding global loads (weight ring, staging loads)
// and stores (output tile) stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int TN>
struct StreamShape {
    static constexpr int TAPS = 9, KSTEPS = 9, BK = 288, ROW = 288;      // a chunk = 32 channels x 9 taps, unpadded swizzled rows
    static constexpr int BN = 32 * TN;
    static constexpr int SLAB_ROW = 32 + 4;                               // 16-bit units per pixel row of a wave's output slab
    static constexpr size_t stage_bytes = (size_t)2 * BN * ROW * 2;
    static constexpr size_t slab_bytes = (size_t)4 * 32 * SLAB_ROW * 2;
};
template <int TM, int TN>
constexpr size_t stream_smem_bytes()
{
    return StreamShape<TN>::stage_bytes + StreamShape<TN>::slab_bytes + (size_t)(128 * TM) * 4;
}

template <int DT, bool SPARSE, int TM, int TN>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv3x3_stream_kernel(ConvParams p, int tiles_n, int slots_n)
{
    using SH = StreamShape<TN>;
    constexpr int BM = 128 * TM, BN = SH::BN, ROW = SH::ROW, TAPS = 9, KSTEPS = 9;
    constexpr int FR = KSTEPS * TN;                  // activation fragments per chunk
    constexpr int RB = 6, D = 4;                     // activation-fragment ring: slots, prefetch distance (fragments)
    constexpr int AF = KSTEPS * TM;                  // weight fragments per chunk
    constexpr int RA = SPARSE ? (TM == 2 ? 9 : 3) : (TM == 2 ? 6 : 3);     // weight-fragment ring slots
    static_assert(FR % RB == 0 && AF % RA == 0 && D < RB && D < FR, "rings must nest with the chunk");
    static_assert(TM == 1 || TM == 2, "one or two row tiles per wave");
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *const Bs0 = smem, *const Bs1 = smem + BN * ROW;
    uint16_t *slab_all = smem + 2 * BN * ROW;
    float *bias_s = reinterpret_cast<float *>(slab_all + 4 * 32 * SH::SLAB_ROW);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= 4;
    // Workgroups are handed to the 8 XCDs round-robin; renumber them so that an XCD (own L2) owns a contiguous run
    // of pixel tiles in every round.
    const int nb = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int lid = xcd * (nb >> 3) + min(xcd, nb & 7) + slot;
    const int tile_m = lid % p.tiles_m;              // the same row tile for every tile of this workgroup
    const int nslot = lid / p.tiles_m;               // first pixel tile; the next ones follow at a stride of slots_n
    const int ntl = nslot < tiles_n ? (tiles_n - nslot + slots_n - 1) / slots_n : 0;
    const int nchunks = p.Ks / KSTEPS;               // (cin % 32 == 0: the reduction is a whole number of chunks)
    const int total = ntl * nchunks;                 // chunks this workgroup multiplies, over all its tiles
    const int m0 = tile_m * BM;
    const int HoWo = p.Ho * p.Wo;

    if (total == 0) return;                          // (uniform)

    if (producer) {
        // ------------------------------------------------------------------ producer waves
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, (int)p.x_bytes, kRsrcFlags);
        constexpr int ITEMS = BN / 64;               // pixel rows per thread (256 threads x 4 units of 8 channels = 64 rows per pass)
        const int stid = tid - 256;
        const int unit = stid & 3, pr0 = stid >> 2;
        unsigned tapoff[ITEMS][TAPS];
        // Byte offsets of the nine taps of this thread's pixels in tile number `it` of the workgroup (out of range
        // for padding, pixels past the end, and tiles past the last one: such loads return zeros).
        auto setup_tile = [&](int it) {
            const int n0 = (nslot + it * slots_n) * BN;
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
                const int pg = n0 + pr0 + i * 64;
                const bool live = it < ntl && pg < p.P;
                const int n = fast_div(live ? pg : 0, p.howo_mul, p.howo_sh);
                const int rem = (live ? pg : 0) - n * HoWo;
                const int ho = fast_div(rem, p.wo_mul, p.wo_sh);
                const int wo = rem - ho * p.Wo;
                const int ih0 = ho * p.sh - p.ph, iw0 = wo * p.sw - p.pw;
                const unsigned pixbyte = (unsigned)(((n * p.H + ih0) * p.W + iw0) * p.Cin * 2);
#pragma unroll
                for (int tap = 0; tap < TAPS; tap++) {
                    const int r = tap / 3, t = tap % 3;
                    const bool ok = live && (unsigned)(ih0 + r) < (unsigned)p.H && (unsigned)(iw0 + t) < (unsigned)p.W;
                    tapoff[i][tap] = ok ? pixbyte + (unsigned)(((r * p.W + t) * p.Cin + unit * 8) * 2) : kOutOfRange;
                }
            }
        };
        u32x4 st[2][ITEMS][TAPS];
        int gen_it = 0, gen_c = 0;                   // the chunk the next load belongs to
        setup_tile(0);
        auto advance = [&]() {                       // (the addresses of the loads just issued are spent: overwrite them)
            if (++gen_c == nchunks) {
                gen_c = 0;
                setup_tile(++gen_it);
            }
        };
        auto load_one = [&](int set, int i, int tap) {      // set, i, tap: compile time at every call site
            st[set][i][tap] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)tapoff[i][tap], gen_c * 64, 0);
        };
        // One transposed 16-byte vector: [tap][8 channels] -> [channel][tap], output element h = c*9 + tap, two per dword.
        auto store_one = [&](uint16_t *buf, int set, int i, int v) {
            const int pr = pr0 + i * 64;
            u32x4 *rowp = reinterpret_cast<u32x4 *>(buf + pr * ROW);
            const int vec0 = unit * TAPS, swz = (pr >> 2) & 3;
            uint32_t o[4];
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int d = 4 * v + q;
                const int ha = 2 * d, hb = 2 * d + 1;
                const int ca = ha / TAPS, ta = ha % TAPS, cb = hb / TAPS, tb = hb % TAPS;
                const uint32_t sa = st[set][i][ta][ca >> 1], sb = st[set][i][tb][cb >> 1];
                const uint32_t sel = (uint32_t)(2 * (ca & 1)) | ((uint32_t)(2 * (ca & 1) + 1) << 8) |
                                     ((uint32_t)(4 + 2 * (cb & 1)) << 16) | ((uint32_t)(5 + 2 * (cb & 1)) << 24);
                o[q] = __builtin_amdgcn_perm(sb, sa, sel);
            }
            const u32x4 w = {o[0], o[1], o[2], o[3]};
            rowp[(vec0 + v) ^ swz] = w;
        };
        auto load = [&](int set) {
#pragma unroll
            for (int i = 0; i < ITEMS; i++)
#pragma unroll
                for (int tap = 0; tap < TAPS; tap++) load_one(set, i, tap);
            advance();
        };
        auto store = [&](uint16_t *buf, int set) {
#pragma unroll
            for (int i = 0; i < ITEMS; i++)
#pragma unroll
                for (int v = 0; v < TAPS; v++) store_one(buf, set, i, v);
        };
        // Steady state: the loads of one chunk and the LDS writes of the previous one, interleaved, so that neither the
        // vector-memory path nor the LDS write port sees a burst of 18 requests per thread in front of the multiplying
        // waves' weight loads and fragment reads.  (Pacing the pairs with s_sleep was measured too: no gain at 64
        // clocks per pair, a loss from 128 on.)
        auto load_store = [&](int lset, uint16_t *buf, int sset) {
#pragma unroll
            for (int i = 0; i < ITEMS; i++)
#pragma unroll
                for (int v = 0; v < TAPS; v++) {
                    load_one(lset, i, v);
                    store_one(buf, sset, i, v);
                    if (SS_STREAM_PACE > 0) __builtin_amdgcn_s_sleep(SS_STREAM_PACE);
                    __builtin_amdgcn_sched_barrier(0);
                }
            advance();
        };
        // Chunk k is written to buffer k % 2 and published by barrier number k; the loads of chunk k + 1 are issued
        // before chunk k is written (loads past the last chunk address nothing and return zeros).
        load(0);
        load(1);
        store(Bs0, 0);
        lds_barrier();                                // barrier 0: chunk 0
        for (int k = 1; k < total; k += 2) {
            // loads of chunk k + 1 (set 0 held chunk k - 1, which is in LDS); chunk k goes to buffer 1, which held
            // chunk k - 2, whose last read precedes barrier k - 1
            load_store(0, Bs1, 1);
            lds_barrier();                            // barrier k
            if (k + 1 >= total) break;
            load_store(1, Bs0, 0);                    // loads of chunk k + 2, LDS writes of chunk k + 1
            lds_barrier();                            // barrier k + 1
        }
        lds_barrier();                                // answers the multiplying waves' barrier inside the last chunk
        return;
    }

    // ------------------------------------------------------------------ multiplying waves
    // (they set the pace -- the producers wait for them at every chunk's barrier -- so they get the issue slots first)
    __builtin_amdgcn_s_setprio(3);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a_vals), 0, (int)p.a_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.a_meta), 0, (int)p.meta_bytes, kRsrcFlags);
    // A weight tile is lane-linear: the lane's share sits at lane * 16 (values) / lane * 4 (index words) from the tile's
    // start, and the tile's start (row tile, step) is wave-uniform and travels in the scalar offset of the load.
    const unsigned a_lane = (unsigned)lane * 16u, m_lane = (unsigned)lane * 4u;
    int a_tile[TM], m_tile[TM];
#pragma unroll
    for (int tm = 0; tm < TM; tm++) {
        const int mt = min((m0 >> 5) + wave * TM + tm, p.Mt - 1);      // rows past the last are clamped; they are never stored
        a_tile[tm] = mt * p.Ks * (SPARSE ? 1024 : 2048);
        m_tile[tm] = mt * p.Kp * 256;
    }
    struct AFrag {
        u32x4 v[SPARSE ? 1 : 2];
        uint32_t idx;
    };
    AFrag a[RA];
    // Weight fragment number j of the chunk whose first step is ks0 (steps wrap to the next tile's first ones: every
    // tile of this workgroup has the same weights).
    auto load_a = [&](AFrag &f, int ks0, int j) {
        int ks = ks0 + j / TM;
        if (ks >= p.Ks) ks -= p.Ks;
        const int tm = j % TM;
        if constexpr (SPARSE) {
            f.v[0] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_lane, a_tile[tm] + ks * 1024, 0);
            f.idx = __builtin_amdgcn_raw_buffer_load_b32(rm, (int)m_lane, m_tile[tm] + (ks >> 1) * 256, 0);
        } else {
            f.v[0] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_lane, a_tile[tm] + ks * 2048, 0);
            f.v[1] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_lane, a_tile[tm] + ks * 2048 + 1024, 0);
        }
    };
    // This lane's two 16-byte vectors of a fragment inside the step's aligned group of four, swizzled as the rows are.
    const int frag_key = (lane >> 2) & 3;
    const int frag_lo = ((2 * (lane >> 5)) ^ frag_key) * 8, frag_hi = ((2 * (lane >> 5) + 1) ^ frag_key) * 8;
    const int brow = (lane & 31) * ROW;
    B32 b[RB];
    auto load_b = [&](B32 &f, const uint16_t *buf, int fr) {      // fragment fr = step * TN + pixel subtile
        const uint16_t *src = buf + (fr % TN) * 32 * ROW + brow + (fr / TN) * 32;
        f.lo = *reinterpret_cast<const u32x4 *>(src + frag_lo);
        f.hi = *reinterpret_cast<const u32x4 *>(src + frag_hi);
    };
    Acc<DT> acc[TM][TN];
    auto init_acc = [&]() {                           // the bias goes in first: rows 8q + 4(lane / 32) + e of each row tile
#pragma unroll
        for (int tm = 0; tm < TM; tm++)
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const float4 bq = *reinterpret_cast<const float4 *>(bias_s + (wave * TM + tm) * 32 + 8 * q + 4 * (lane >> 5));
#pragma unroll
                for (int tn = 0; tn < TN; tn++) {
                    acc[tm][tn][4 * q + 0] = bq.x; acc[tm][tn][4 * q + 1] = bq.y;
                    acc[tm][tn][4 * q + 2] = bq.z; acc[tm][tn][4 * q + 3] = bq.w;
                }
            }
    };
    uint16_t *slab = slab_all + wave * 32 * SH::SLAB_ROW;
    const float relu_floor = p.act == SS_ACT_RELU ? 0.f : -__builtin_inff();
    constexpr int ODT = DT;
    // Output: raw buffer stores whose range check does the pixel tail (a pixel past the last lies past the buffer's
    // end); rows past the last output channel get an out-of-range offset.
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.P * (unsigned)p.Cout * 2u), kRsrcFlags);
    // The eight 32 x 32 pieces of the tile cross the wave's slab one after the other.  A wave's LDS operations execute
    // in order, so piece t + 1 may be written as soon as the reads of piece t have been *issued*: the conversion and
    // the writes of the next piece sit between a piece's reads and the stores that wait for them, and cover the slab's
    // read latency (the largest part of a piece's time otherwise).  (Keeping two pieces' runs in flight would cover
    // all of it, but the sixteen registers are not there: the weight and activation rings of the next tile are live.)
    auto write_tile = [&](int n0, auto actf) {
        unsigned yoff[TM][2];                         // byte offset of this lane's 16-byte run for pixel subtile 0
#pragma unroll
        for (int tm = 0; tm < TM; tm++)
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const int px = (lane >> 2) + 16 * j, o = m0 + (wave * TM + tm) * 32 + (lane & 3) * 8;
                yoff[tm][j] = o < p.Cout ? (unsigned)((n0 + px) * p.Cout + o) * 2u : kOutOfRange;
            }
        auto put = [&](int t) {                       // piece t = tm * TN + tn into the slab
            const int tm = t / TN, tn = t % TN;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; e++) r[e] = actf(acc[tm][tn][4 * q + e]);
                *reinterpret_cast<uint2 *>(slab + (lane & 31) * SH::SLAB_ROW + 8 * q + 4 * (lane >> 5)) =
                    make_uint2(cvt_pack2<ODT>(r[0], r[1]), cvt_pack2<ODT>(r[2], r[3]));
            }
        };
        auto get = [&](u32x4 (&w)[2]) {               // this lane's two 16-byte runs of the piece in the slab
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const int px = (lane >> 2) + 16 * j, run = lane & 3;
                const uint2 lo = *reinterpret_cast<const uint2 *>(slab + px * SH::SLAB_ROW + run * 8);
                const uint2 hi = *reinterpret_cast<const uint2 *>(slab + px * SH::SLAB_ROW + run * 8 + 4);
                w[j] = u32x4{lo.x, lo.y, hi.x, hi.y};
            }
        };
        auto send = [&](int t, const u32x4 (&w)[2]) {
            const int tm = t / TN, tn = t % TN;
#pragma unroll
            for (int j = 0; j < 2; j++) __builtin_amdgcn_raw_buffer_store_b128(w[j], ry, (int)yoff[tm][j], tn * 32 * p.Cout * 2, 0);
        };
        put(0);
#pragma unroll
        for (int t = 0; t < TM * TN; t++) {
            u32x4 w[2];
            get(w);
            if (t + 1 < TM * TN) put(t + 1);
            send(t, w);
        }
    };

    // prologue: the first weight fragments, the tile's bias values (parked in LDS by these waves; barrier 0 makes them
    // visible), then the first activation fragments of chunk 0
#pragma unroll
    for (int j = 0; j < RA - TM; j++) {
        load_a(a[j], 0, j);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int i = tid; i < BM; i += 256) bias_s[i] = (p.bias != nullptr && m0 + i < p.Cout) ? p.bias[m0 + i] : 0.f;
    lds_barrier();                                    // barrier 0: chunk 0 is in LDS
    init_acc();
#pragma unroll
    for (int f = 0; f < D; f++) load_b(b[f], Bs0, f);

    int g = 0;                                        // chunk counter over all tiles
    for (int it = 0; it < ntl; it++) {
        for (int c = 0; c < nchunks; c++, g++) {
            const uint16_t *cur = (g & 1) ? Bs1 : Bs0, *nxt = (g & 1) ? Bs0 : Bs1;
            const int ks0 = c * KSTEPS;
            const int par = (ks0 & 1) * 16;           // index half of the chunk's even steps
#pragma unroll
            for (int s = 0; s < KSTEPS; s++) {
#pragma unroll
                for (int tn = 0; tn < TN; tn++) {
                    const int f = s * TN + tn;
                    // barrier g + 1: the next chunk is in LDS; this one's reads are all done.  After the very last chunk
                    // the barrier and the reads that follow it are idle (the producers answer it once more, the
                    // fragments are never used): a branch here would make every wait in the loop body conservative.
                    if (f == FR - D) lds_barrier();
                    if (f + D < FR) load_b(b[(f + D) % RB], cur, f + D);
                    else load_b(b[(f + D) % RB], nxt, f + D - FR);
                    if (tn < TM) {                    // this step's share of the weight prefetch: fragments s*TM + RA - TM + tn
                        const int j = s * TM + RA - TM + tn;
                        load_a(a[j % RA], ks0, j);
                    }
#pragma unroll
                    for (int tm = 0; tm < TM; tm++) {
                        const AFrag &af = a[(s * TM + tm) % RA];
                        if constexpr (SPARSE) {
                            const uint32_t idx = af.idx >> ((s & 1) ? 16 - par : par);
                            acc[tm][tn] = mma_sparse<DT>(af.v[0], b[f % RB], acc[tm][tn], idx);
                        } else {
                            acc[tm][tn] = mma_dense<DT>(af.v[0], b[f % RB].lo, acc[tm][tn]);
                            acc[tm][tn] = mma_dense<DT>(af.v[1], b[f % RB].hi, acc[tm][tn]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        const int n0 = (nslot + it * slots_n) * BN;
        if (p.act == SS_ACT_GELU) write_tile(n0, [](float v) { return gelu_erfc(v); });
        else write_tile(n0, [&](float v) { return floor_at(v, relu_floor); });     // ReLU, or the identity with a floor of -inf (a NaN passes)
        init_acc();
    }
}

// Launches the streaming kernel on a grid of at most `max_blocks` workgroups (one per compute unit).
template <int DT, bool SPARSE, int TM, int TN>
static int launch_stream(const ConvParams &p0, int max_blocks, hipStream_t s)
{
    constexpr int BM = 128 * TM, BN = 32 * TN;
    constexpr size_t smem = stream_smem_bytes<TM, TN>();
    static_assert(smem <= 160 * 1024, "LDS tile too large");
    ConvParams p = p0;
    p.tiles_m = (p.Cout + BM - 1) / BM;
    const long long tiles_n = ((long long)p.P + BN - 1) / BN;
    if (tiles_n <= 0 || tiles_n > 0x7FFFFFFFll || p.tiles_m > 0xFFFF) return SS_ERR_UNSUPPORTED;
    long long slots_n = max_blocks / p.tiles_m;      // pixel tiles in flight per round (every row tile of a pixel tile runs in the same round)
    if (slots_n < 1) slots_n = 1;
    if (slots_n > tiles_n) slots_n = tiles_n;
    const long long blocks = slots_n * p.tiles_m;
    auto kern = conv3x3_stream_kernel<DT, SPARSE, TM, TN>;
    static std::atomic<unsigned long long> done_mask{0};      // dynamic-LDS limit raised, per device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SS_ERR_HIP;
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev >= 64 || !(done_mask.load(std::memory_order_acquire) & bit)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return SS_ERR_HIP;
        if (dev < 64) done_mask.fetch_or(bit, std::memory_order_release);
    }
    kern<<<dim3((unsigned)blocks), dim3(512), smem, s>>>(p, (int)tiles_n, (int)slots_n);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

// Can the streaming kernel take this problem?  3x3 kernel in the channel-slowest flattening, 16-bit operands, whole
// chunks (cin % 32 == 0), 16-byte output runs (cout % 8 == 0), no residual, output below 2 GiB (32-bit store offsets,
// with room for the offsets of a last tile's pixels past the end to stay below the out-of-range mark).
static inline bool stream_eligible(const ss_weight_desc *desc, const ConvParams &p)
{
    return !is_byte_type(desc->dtype) && desc->korder == SS_K_CRS && desc->kh == 3 && desc->kw == 3 && desc->cin % 32 == 0 &&
           desc->cout % 8 == 0 && p.residual == nullptr && (long long)p.P * p.Cout * 2 < (1ll << 31) - (1ll << 27);
}

}  // namespace ss

#endif
