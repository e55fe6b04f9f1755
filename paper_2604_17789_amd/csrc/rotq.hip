// Rotate + MXFP4-quantise kernel (the online X -> Q(X . R^) of the paper's Eq. 5 / Remark 2,
// with Q from Eq. 2), hand-written for gfx950.
//
// Mapping.  One wavefront owns two adjacent 32-channel blocks and walks down 32-token tiles.
// The 32x32 rotation of a tile runs on the matrix cores as  Y^T = R^T . X^T  with
// v_mfma_f32_32x32x16_bf16: the A operand is R^T (M = output channel), the B operand is the
// token tile (N = token), so the 32 rotated channels of one token land in just two lanes
// (l and l^32), which makes the group amax one cross-lane step.
// fp32 accuracy on bf16 matrix cores: X is bf16 already; each fp32 entry of R is split
// exactly into three bf16 pieces (8 + 8 + 8 significant bits), so every product is exact in
// fp32 and only the fp32 accumulation order differs from a plain fp32 dot product.
// The quantiser uses the hardware E2M1 convert (v_cvt_scalef32_pk_fp4_f32), which rounds to
// nearest even, saturates at 6, keeps the sign of zero and divides by the power of two held
// in the exponent field of its scale operand (field 0 meaning 2^-127).
#include "duqpp_internal.h"
#include "rotq_device.h"

namespace duqpp {

constexpr int kRotqWaves = 8;              // wavefronts per workgroup
constexpr int kRotqWGPerCU = 1;            // workgroups resident per CU (bounded by LDS)
constexpr int kBlocksPerWave = 2;
constexpr int kBlocksPerWG = kRotqWaves * kBlocksPerWave;
// cache policy of the activation loads (aux operand of the LDS-DMA builtin, bit 1 = non-temporal): every byte of x
// is read once, so it should not displace the codes being written, which the GEMM reads next (measured: 6-10 %
// less time per launch at the prefill shapes)
constexpr int kStreamedLoad = 2;

__device__ __forceinline__ void logical_workgroup(int& logical) {
    // Workgroups are dealt round-robin to the 8 XCDs; renumber so that each XCD gets a
    // contiguous range of logical workgroups.
    int id = blockIdx.x, n = gridDim.x;
    int per = n / kNumXCD, rem = n % kNumXCD;
    int xcd = id % kNumXCD, slot = id / kNumXCD;
    logical = xcd * per + (xcd < rem ? xcd : rem) + slot;
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

// LDS reads issued as asm: the compiler cannot tell which LDS-DMA transfer a read depends on
// and would otherwise wait for ALL outstanding ones (vmcnt(0)) before every LDS read, which
// would drain the prefetched tiles.  The waits that matter are placed by hand below.
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const void*)p);
}
__device__ __forceinline__ void lds_read4_b128(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                               u32x4& r0, u32x4& r1, u32x4& r2, u32x4& r3) {
    asm volatile(
        "ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
        : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
        : "memory");
}
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t a) {
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(r) : "v"(a) : "memory");
    return r;
}
// LDS writes of the output staging go the same way (the compiler would drain the DMA queue
// before any LDS write it cannot prove disjoint from the DMA targets).
__device__ __forceinline__ void lds_write_b64(uint32_t a, uint2 v) {
    asm volatile("ds_write_b64 %0, %1" ::"v"(a), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_b8(uint32_t a, uint32_t v) {
    asm volatile("ds_write_b8 %0, %1" ::"v"(a), "v"(v) : "memory");
}
// all LDS accesses of this wave have completed, then workgroup barrier
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// s_waitcnt takes an immediate: wait until at most the largest constant <= n (n <= MAX) operations are
// outstanding.  n is uniform over the wave.
template <int MAX>
__device__ __forceinline__ void wait_vmcnt_at_most(int n) {
    if constexpr (MAX == 0) {
        wait_vmcnt<0>();
    } else {
        if (n >= MAX) wait_vmcnt<MAX>();
        else wait_vmcnt_at_most<MAX - 1>(n);
    }
}

// Workgroup tile: 32 tokens x (WAVES * 2) blocks.  Per token row that is WAVES*128 bytes of
// bf16 in, WAVES*32 bytes of codes out and WAVES*2 scale bytes out.
//
// Data movement is shaped for whole cache lines.  Activations arrive by LDS-DMA
// (global_load_lds_dwordx4: 64 lanes x 16 B land lane-linear in LDS) with one wave instruction
// covering a contiguous WAVES*128-byte piece of 8/WAVES rows; the MFMA B operands are then read
// from LDS (lane = token, which would be a whole-wave bank conflict at a row stride of WAVES*128
// bytes, so the 16-byte chunks of row r are stored XOR-swizzled by r & 15 -- applied on the
// global side of the DMA, as the LDS side is fixed lane-linear).  Codes and scales go back
// through LDS so that one store instruction writes full rows of the workgroup tile.
// STAGES activation tiles rotate through LDS; STAGES-1 of them are in flight while one is used.
template <int WAVES, int STAGES>
struct RotqTile {
    static constexpr int kRowBytes = WAVES * 128;
    static constexpr int kChunks = kRowBytes / 16;          // 16-byte chunks per row (= lanes per row)
    static constexpr int kRowsPerInstr = 64 / kChunks;      // WAVES = 8: 1, WAVES = 4: 2
    static constexpr int kStageBytes = 32 * kRowBytes;
    static constexpr int kCodeRowBytes = WAVES * 32;
    static constexpr int kCodeChunks = kCodeRowBytes / 16;  // = WAVES * 2
    static constexpr int kScaleRowBytes = WAVES * 2;
    static constexpr int kInBytes = STAGES * kStageBytes;
    static constexpr int kCodesOff = kInBytes;
    static constexpr int kScalesOff = kCodesOff + 32 * kCodeRowBytes;
    static constexpr int kLdsBytes = kScalesOff + 32 * 16;  // scale rows padded to 16 bytes
    static_assert(kChunks >= 16 && kChunks <= 64, "2 <= WAVES <= 8");
};

template <int WAVES, int STAGES>
__device__ __forceinline__ void issue_tile_loads(const RotqParams& p, uint8_t* lds, int stage, int tile, int chunk0,
                                                 int wave, int lane) {
    using TL = RotqTile<WAVES, STAGES>;
    const int nchunk16 = p.G * 4;                            // 16-byte chunks in a full row of X
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = wave * 4 + i;                          // instruction index within the tile
        const int r = q * TL::kRowsPerInstr + lane / TL::kChunks;   // token row within the tile
        const int pos = lane % TL::kChunks;                  // chunk position in LDS
        int gch = chunk0 + (pos ^ (r & 15));                 // chunk of the row that belongs there
        if (gch >= nchunk16) gch = chunk0;                   // ragged last column chunk: any valid address
        int row = tile * 32 + r;
        if (row >= p.rows) row = p.rows - 1;                 // ragged last tile
        const uint16_t* g = p.x + (int64_t)row * p.ldx + (int64_t)gch * 8;
        __builtin_amdgcn_global_load_lds((global_void_ptr)g, (lds_void_ptr)(lds + stage * TL::kStageBytes + q * 1024),
                                         16, 0, kStreamedLoad);
    }
}

// TILED selects the output placement: row-major through LDS staging, or the tiled operand
// layout, where a wave's 32 tokens x 16 code bytes of one block are 512 contiguous bytes and
// go out straight from registers.
template <int WAVES, int STAGES, bool TILED>
__global__ __launch_bounds__(WAVES * 64) void rotq_kernel(RotqParams p) {
    using TL = RotqTile<WAVES, STAGES>;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    int logical;
    logical_workgroup(logical);
    const int chunk = logical % p.nchunks;                   // neighbours on an XCD: neighbouring columns, same rows
    const int tg = logical / p.nchunks;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const uint32_t lds_base = lds_offset(lds);

    // every wave stays to the end (barriers, cooperative loads and stores); waves past the last
    // block compute on a clamped block and their outputs are masked
    const int jb = chunk * WAVES * 2;                        // first block of the workgroup
    int j0 = jb + wave * 2, j1 = j0 + 1;
    if (j0 >= p.G) j0 = p.G - 1;
    if (j1 >= p.G) j1 = p.G - 1;

    const int tile0 = tg * p.tiles_per_wg;
    int tile1 = tile0 + p.tiles_per_wg;
    if (tile1 > p.ntiles) tile1 = p.ntiles;
    const int chunk0 = jb * 4;                               // first 16-byte chunk of X rows for this workgroup

    constexpr int P = STAGES - 1;                            // tiles in flight
    RotOperand op0, op1;
    load_rot_operand(p.R + (int64_t)j0 * p.r_stride, c, h, op0);
    load_rot_operand(p.R + (int64_t)j1 * p.r_stride, c, h, op1);
#pragma unroll
    for (int d = 0; d < P; ++d)
        if (tile0 + d < tile1) issue_tile_loads<WAVES, STAGES>(p, lds, d, tile0 + d, chunk0, wave, lane);

    int stage = 0;
    for (int tile = tile0; tile < tile1; ++tile) {
        // Wait for this tile only: LDS-DMA loads complete in issue order and every wave issues
        // exactly 4 per tile, so "at most 4 * (tiles issued after this one)" outstanding means this
        // tile has landed (stores issued in between only make the wait stricter).
        const int ahead = tile1 - 1 - tile;                  // tiles after this one
        if (P >= 3 && ahead >= 2) wait_vmcnt<8>();
        else if (P >= 2 && ahead >= 1) wait_vmcnt<4>();
        else wait_vmcnt<0>();
        static_assert(P <= 3, "extend the wait ladder for deeper pipelines");
        __builtin_amdgcn_s_barrier();                        // all waves' pieces of this tile are in LDS,
                                                             // and every wave is done with the previous tile
        // refill the stage the previous tile occupied, P tiles ahead
        if (ahead >= P) {
            int pre_stage = stage + P;
            if (pre_stage >= STAGES) pre_stage -= STAGES;
            issue_tile_loads<WAVES, STAGES>(p, lds, pre_stage, tile + P, chunk0, wave, lane);
        }

        const uint32_t in = lds_base + stage * TL::kStageBytes + c * TL::kRowBytes;
        u32x4 x0[2], x1[2];
        const int cw = wave * 8 + h;                         // chunk of (block 0, k-step 0) for this lane
        lds_read4_b128(in + (((cw) ^ (c & 15)) << 4), in + (((cw + 2) ^ (c & 15)) << 4),
                       in + (((cw + 4) ^ (c & 15)) << 4), in + (((cw + 6) ^ (c & 15)) << 4),
                       x0[0], x0[1], x1[0], x1[1]);

        f32x16 acc0 = rotate_tile(op0, x0);
        f32x16 acc1 = rotate_tile(op1, x1);
        uint2 o0, o1;
        uint32_t byte0 = quantize_group(acc0, o0);
        uint32_t byte1 = quantize_group(acc1, o1);

        if constexpr (TILED) {
            // rows past the end and groups past K are padding of the tiled layout: code 0, scale 127
            const int jt0 = jb + wave * 2, jt1 = jt0 + 1;
            const int rt = tile;
            const bool row_ok = tile * 32 + c < p.rows;
            if (!row_ok || jt0 >= p.G) { o0 = make_uint2(0, 0); byte0 = 127; }
            if (!row_ok || jt1 >= p.G) { o1 = make_uint2(0, 0); byte1 = 127; }
            if (jt0 < p.GP) {                                // GP is even, so jt1 < GP as well
                uint8_t* ct = p.codes + (((int64_t)rt * p.GP + jt0) * 32 + c) * 16 + 8 * h;
                *(uint2*)ct = o0;
                *(uint2*)(ct + 512) = o1;
                if (h == 0) {
                    uint8_t* st = p.scales + ((((int64_t)rt * (p.GP / 8) + jt0 / 8) * 2 + (jt0 % 8) / 4) * 32 + c) * 4 + (jt0 % 4);
                    *(uint16_t*)st = (uint16_t)(byte0 | (byte1 << 8));
                }
            }
        } else {
            // stage the outputs: codes [token][WAVES*2 chunks of 16 B], chunk index swizzled by the token
            const uint32_t oc = lds_base + TL::kCodesOff + c * TL::kCodeRowBytes + 8 * h;
            lds_write_b64(oc + (((wave * 2) ^ (c & 15) & (TL::kCodeChunks - 1)) << 4), o0);
            lds_write_b64(oc + (((wave * 2 + 1) ^ (c & 15) & (TL::kCodeChunks - 1)) << 4), o1);
            lds_write_b8(lds_base + TL::kScalesOff + c * 16 + wave * 2 + h, h ? byte1 : byte0);
        }
        if (p.ydbg) {
            const int row = tile * 32 + c;
            if (row < p.rows) {
                float* yr = p.ydbg + (int64_t)row * p.G * 32 + 4 * h;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (jb + wave * 2 < p.G)
                        *(float4*)(yr + 32 * j0 + 8 * q) = make_float4(acc0[4 * q], acc0[4 * q + 1], acc0[4 * q + 2], acc0[4 * q + 3]);
                    if (jb + wave * 2 + 1 < p.G)
                        *(float4*)(yr + 32 * j1 + 8 * q) = make_float4(acc1[4 * q], acc1[4 * q + 1], acc1[4 * q + 2], acc1[4 * q + 3]);
                }
            }
        }
        if constexpr (!TILED) {
            lds_barrier();                                       // outputs of all waves are staged

            // codes: thread i stores 16 bytes; one wave instruction covers 64 / (WAVES*2) full rows
            {
                const int r = threadIdx.x / TL::kCodeChunks;     // 0..31
                const int ch = threadIdx.x % TL::kCodeChunks;
                const int row = tile * 32 + r;
                if (row < p.rows && jb + ch < p.G) {
                    u32x4 v = lds_read_b128(lds_base + TL::kCodesOff + r * TL::kCodeRowBytes + ((ch ^ (r & 15) & (TL::kCodeChunks - 1)) << 4));
                    *(u32x4*)(p.codes + ((int64_t)row * p.G + jb + ch) * 16) = v;
                }
            }
            // scales: one row of the tile per lane of wave 0
            if (threadIdx.x < 32) {
                const int row = tile * 32 + threadIdx.x;
                if (row < p.rows) {
                    const uint32_t sr = lds_base + TL::kScalesOff + threadIdx.x * 16;
                    uint8_t* dst = p.scales + (int64_t)row * p.G + jb;
                    u32x4 v = lds_read_b128(sr);
                    if (jb + TL::kScaleRowBytes <= p.G && (((uintptr_t)dst) & (TL::kScaleRowBytes - 1)) == 0) {
                        if (TL::kScaleRowBytes == 16) *(u32x4*)dst = v;
                        else if (TL::kScaleRowBytes == 8) *(uint2*)dst = make_uint2(v[0], v[1]);
                        else *(uint32_t*)dst = v[0];
                    } else {
#pragma unroll
                        for (int b = 0; b < TL::kScaleRowBytes; ++b)
                            if (jb + b < p.G) dst[b] = (uint8_t)(v[b / 4] >> (8 * (b % 4)));
                    }
                }
            }
        }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
    }
}


// ---- Tiled-output kernel: every wavefront runs a pipeline of its own ---------------------------
// With the tiled operand layout a wave's output for one block is 512 contiguous bytes, so nothing has
// to be exchanged between waves.  Each wave therefore owns two adjacent blocks (one 128-byte line per
// token row) of a run of 32-token tiles, moves its own 4 KiB tiles by LDS-DMA into a private ring of
// LDS stages and never meets a workgroup barrier: eight such pipelines per CU drift apart, and one
// wave's matrix-core and convert work fills another's memory waits.
// A tile is 32 rows x 8 chunks of 16 bytes; chunk q of row r is kept at position q ^ (r & 7) (applied
// on the global side of the transfer), which makes the per-token reads conflict-free.
// The output stores are asm statements so that their number per tile is fixed (kWaveStores): the waits
// count outstanding vector-memory operations, which complete in issue order.
constexpr int kWaveTileBytes = 4096;
constexpr int kWaveStores = 3;             // two code stores and one scale store per tile

__device__ __forceinline__ void store_b64(void* ptr, uint2 v) {
    asm volatile("global_store_dwordx2 %0, %1, off" ::"v"(ptr), "v"(v) : "memory");
}
__device__ __forceinline__ void store_b16(void* ptr, uint32_t v) {
    asm volatile("global_store_short %0, %1, off" ::"v"(ptr), "v"(v) : "memory");
}

__device__ __forceinline__ void issue_wave_tile(const RotqParams& p, uint32_t lds_stage, int tile, int pair, int lane) {
    const int pos = lane & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 8 * i + (lane >> 3);                   // token row within the tile
        int gch = pair * 8 + (pos ^ (r & 7));                // 16-byte chunk of the row that belongs at `pos`
        if (gch >= p.G * 4) gch = 0;                         // padding groups: any valid address, output is masked
        int row = tile * 32 + r;
        if (row >= p.rows) row = p.rows - 1;                 // ragged last tile
        const uint16_t* g = p.x + (int64_t)row * p.ldx + (int64_t)gch * 8;
        __builtin_amdgcn_global_load_lds((global_void_ptr)g,
                                         (lds_void_ptr)(uintptr_t)(lds_stage + i * 1024), 16, 0, kStreamedLoad);
    }
}

template <int STAGES, bool PACKED>
__global__ __launch_bounds__(512) void rotq_wave_kernel(RotqParams p) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    int logical;
    logical_workgroup(logical);
    // Which workgroups share an XCD (the renumbering keeps consecutive logical ones together):
    //  - by_columns: an XCD owns a few column chunks for all token runs, so each rotation block is fetched into one
    //    L2 only, and (token tiles being dealt to the runs in turn, below) its workgroups read neighbouring rows of
    //    those columns at any moment;
    //  - otherwise consecutive workgroups take consecutive chunks of the same token rows: together they read whole
    //    rows and every XCD fetches every rotation block.  Kept for rows shorter than 4 KiB, where it measures a few
    //    per cent faster; from 4 KiB on owning columns wins or ties at every shape tried (up to 19 %, most with few
    //    hundred tokens).
    const int chunk = p.by_columns ? logical / p.ngroups : logical % p.nchunks;
    const int tg = p.by_columns ? logical % p.ngroups : logical / p.nchunks;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 31, h = lane >> 5;
    const int pair = chunk * p.waves + wave;
    if (pair * 2 >= p.GP) return;                            // no barrier anywhere: a spare wave just leaves
    const int jt0 = pair * 2, jt1 = jt0 + 1;                 // < GP (GP is even)
    const int j0 = jt0 < p.G ? jt0 : p.G - 1, j1 = jt1 < p.G ? jt1 : p.G - 1;

    // Token tiles are dealt to the ngroups runs in turn: run tg takes tiles tg, tg + ngroups, ...  At any moment the
    // runs of a column chunk are then at neighbouring token tiles, i.e. the chip reads a band of adjacent rows rather
    // than ngroups bands far apart (measured against contiguous runs: 16.1 -> 15.8 us at 2048 x 14336, 58.9 -> 57.5 us
    // at 4096 x 28672, 17.3 -> 17.1 us at 8192 x 4096).
    const int nmine = (p.ntiles - tg + p.ngroups - 1) / p.ngroups;
    const int ts = p.ngroups;
    const uint32_t ring = lds_offset(lds) + wave * (STAGES * kWaveTileBytes);

    // A stage is refilled as soon as its tile has been read into registers, so the ring holds exactly
    // the tiles in flight.
    constexpr int P = STAGES;
    // Order of the first requests.  Packed blocks are asked for ahead of the first tiles: nothing is computed before
    // both have arrived, the CU's return path delivers in request order, and with R in front the 12 KiB of a wave's
    // blocks are not queued behind every other wave's two tiles (measured against the opposite order, launch to launch:
    // 16.2 -> 15.95 us at 2048 x 14336, 17.8 -> 17.4 us at 8192 x 4096, no difference at 4096 x 28672).  The fp32 blocks
    // are asked for behind the tiles: their split into pieces is arithmetic that then overlaps the tiles' arrival.
    RotOperand op0, op1;
    if constexpr (PACKED) {
        const uint8_t* rp = (const uint8_t*)p.R;
        load_rot_operand_packed(rp + (int64_t)j0 * p.r_stride, lane, op0);
        load_rot_operand_packed(rp + (int64_t)j1 * p.r_stride, lane, op1);
        __builtin_amdgcn_sched_barrier(0);                   // or the scheduler moves these loads behind the transfers below
    }
    // Every stage gets a transfer here, with no branch: a run with fewer tiles than stages transfers its last tile
    // again (in bounds, never read; the waits below count it).  With branches in this stretch the compiler moves the
    // loads above into the block in front of the loop, i.e. behind the transfers.
#pragma unroll
    for (int d = 0; d < P; ++d)
        issue_wave_tile(p, ring + d * kWaveTileBytes, tg + (d < nmine ? d : nmine - 1) * ts, pair, lane);
    if constexpr (!PACKED) {
        load_rot_operand(p.R + (int64_t)j0 * p.r_stride, c, h, op0);
        load_rot_operand(p.R + (int64_t)j1 * p.r_stride, c, h, op1);
    }

    int stage = 0;
    for (int it = 0; it < nmine; ++it) {
        const int tile = tg + it * ts;
        // This tile's four transfers have landed once at most the transfers issued after them (up to P - 1
        // tiles) are outstanding: transfers complete in issue order.  Stores complete in no fixed order
        // relative to them, so they are not counted; one that is still outstanding only makes the wait stricter.
        const int ahead = nmine - 1 - it;
        wait_vmcnt_at_most<4 * (P - 1)>(4 * (ahead < P - 1 ? ahead : P - 1));
        const uint32_t in = ring + stage * kWaveTileBytes + c * 128;
        u32x4 x0[2], x1[2];
        lds_read4_b128(in + ((h ^ (c & 7)) << 4), in + (((2 + h) ^ (c & 7)) << 4),
                       in + (((4 + h) ^ (c & 7)) << 4), in + (((6 + h) ^ (c & 7)) << 4),
                       x0[0], x0[1], x1[0], x1[1]);
        // this stage is free again (the reads above have returned): refill it P tiles ahead
        if (ahead >= P) issue_wave_tile(p, ring + stage * kWaveTileBytes, tile + P * ts, pair, lane);

        f32x16 acc0 = rotate_tile(op0, x0);
        f32x16 acc1 = rotate_tile(op1, x1);
        uint2 o0, o1;
        uint32_t byte0 = quantize_group(acc0, o0);
        uint32_t byte1 = quantize_group(acc1, o1);

        // rows past the end and groups past K are padding of the tiled layout: code 0, scale 127
        const bool row_ok = tile * 32 + c < p.rows;
        if (!row_ok || jt0 >= p.G) { o0 = make_uint2(0, 0); byte0 = 127; }
        if (!row_ok || jt1 >= p.G) { o1 = make_uint2(0, 0); byte1 = 127; }
        uint8_t* ct = p.codes + (((int64_t)tile * p.GP + jt0) * 32 + c) * 16 + 8 * h;
        store_b64(ct, o0);
        store_b64(ct + 512, o1);
        // both half-waves hold the same two scale bytes and write them to the same place
        uint8_t* st = p.scales + ((((int64_t)tile * (p.GP / 8) + jt0 / 8) * 2 + (jt0 % 8) / 4) * 32 + c) * 4 + (jt0 % 4);
        store_b16(st, byte0 | (byte1 << 8));
        stage = stage + 1 == STAGES ? 0 : stage + 1;
    }
}

constexpr int kRotqStages = 4;             // 3 tiles in flight, one in use

constexpr int kWaveStages = 2;             // per-wave ring of the tiled-output kernel: 2 tiles of 4 KiB in flight, or
constexpr int kWaveStagesDeep = 3;         // 3 where a workgroup has only four waves to keep the CU's requests going

void plan_rotq(RotqParams& p) {
    p.ntiles = (p.rows + 31) / 32;
    p.stages = kWaveStages;
    bool one_per_cu = true;                                 // one workgroup resident per CU, or 8 / waves of them
    if (p.tiled) {
        // wave-private pipelines: a workgroup is `waves` independent waves on adjacent block pairs.
        // Fewer waves per workgroup when the problem is too small to give every CU a full one.
        const int npairs = p.GP / 2;
        p.waves = 8;
        while (p.waves > 1 && (int64_t)((npairs + p.waves - 1) / p.waves) * p.ntiles < kNumCU) p.waves /= 2;
        one_per_cu = p.waves >= 5;
        if (p.waves == 8 && (p.G & (p.G - 1)) == 0) {
            // Enough work for every CU, and a row length that is a power of two (K = 4096, 8192, ...).  With
            // eight-wave workgroups such rows are cut into 1 KiB chunks that sit at the same offset in every row, and
            // the time then depends on where the buffers happen to lie (8192 x 4096 on two boxes: 17.3 and 20.4 us;
            // 4096 x 8192: 17.6 and 20.7 us); four waves per workgroup, one workgroup per CU, each wave with twice
            // the tiles and a ring one deeper, run at the better of those figures on both (17.5, 17.5; 17.6, 17.4)
            // and fetch R half as often.  The deeper ring pays from 8 tiles per wave on; with fewer, two stages are
            // 3 % faster.  Other row lengths (14336, 28672: seven times a power of two) keep the search below, which
            // measures as fast there or faster.
            p.waves = 4;
            one_per_cu = true;
            const int nch = npairs / 4;
            int groups = kNumCU / nch;
            groups = groups < 1 ? 1 : (groups > p.ntiles ? p.ntiles : groups);
            if ((p.ntiles + groups - 1) / groups >= 8) p.stages = kWaveStagesDeep;
        } else if (p.waves == 8) {
            // Enough work for every CU: 5 to 8 waves per workgroup, whichever leaves the busiest CU the fewest
            // (wave, tile) units in the one resident round; more waves when equal.  K = 14336 has 224 block pairs:
            // 8 waves give 28 column chunks x 8 token runs = 224 workgroups on 256 CUs, 7 waves 32 x 8 = 256.
            int64_t best = -1;
            for (int w = 8; w >= 5; --w) {
                const int nch = (npairs + w - 1) / w;
                int groups = kNumCU / nch;
                groups = groups < 1 ? 1 : (groups > p.ntiles ? p.ntiles : groups);
                const int per = (p.ntiles + groups - 1) / groups;
                const int64_t wgs = (int64_t)nch * ((p.ntiles + per - 1) / per);
                const int64_t cost = (int64_t)w * per * ((wgs + kNumCU - 1) / kNumCU);
                if (best < 0 || cost < best) { best = cost; p.waves = w; }
            }
        }
        p.nchunks = (npairs + p.waves - 1) / p.waves;
        p.by_columns = p.G >= 64;                           // rows of 4 KiB or more (K >= 2048)
    } else {
        p.waves = kRotqWaves;
        p.nchunks = (p.G + kBlocksPerWG - 1) / kBlocksPerWG;
    }
    // One resident round: each wave keeps its R blocks in registers and walks as many token
    // tiles as the problem allows, so the fetch and split of R is amortised.
    const int64_t slots = (int64_t)kNumCU * kRotqWGPerCU * (one_per_cu ? 1 : kRotqWaves / p.waves);
    int groups = (int)(slots / p.nchunks);
    if (groups < 1) groups = 1;
    if (groups > p.ntiles) groups = p.ntiles;
    p.tiles_per_wg = (p.ntiles + groups - 1) / groups;
    // the fewest runs that keep the longest run as short: 64 tiles over 9 runs are 8 tiles for the longest anyway,
    // and 8 runs of 8 fetch and split R once less per block pair
    p.ngroups = (p.ntiles + p.tiles_per_wg - 1) / p.tiles_per_wg;
}

hipError_t setup_rotq() {
    static PerDeviceOnce once;
    return once.run([] {
        using TL = RotqTile<kRotqWaves, kRotqStages>;
        constexpr int kWaveLdsMax = 8 * kWaveStages * kWaveTileBytes;
        hipError_t e = allow_dynamic_lds((const void*)rotq_kernel<kRotqWaves, kRotqStages, false>, TL::kLdsBytes);
        if (e != hipSuccess) return e;
        e = allow_dynamic_lds((const void*)rotq_wave_kernel<kWaveStages, false>, kWaveLdsMax);
        if (e != hipSuccess) return e;
        e = allow_dynamic_lds((const void*)rotq_wave_kernel<kWaveStages, true>, kWaveLdsMax);
        if (e != hipSuccess) return e;
        constexpr int kDeepLdsMax = 8 * kWaveStagesDeep * kWaveTileBytes;
        e = allow_dynamic_lds((const void*)rotq_wave_kernel<kWaveStagesDeep, false>, kDeepLdsMax);
        if (e != hipSuccess) return e;
        return allow_dynamic_lds((const void*)rotq_wave_kernel<kWaveStagesDeep, true>, kDeepLdsMax);
    });
}

hipError_t launch_rotq(const RotqParams& p, hipStream_t stream) {
    using TL = RotqTile<kRotqWaves, kRotqStages>;
    hipError_t e = setup_rotq();
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((int64_t)p.nchunks * p.ngroups));
    if (p.tiled) {
        if (p.waves < 1 || p.waves > 8) return hipErrorInvalidValue;
        if (p.stages != kWaveStages && p.stages != kWaveStagesDeep) return hipErrorInvalidValue;
        const size_t lds = (size_t)p.waves * p.stages * kWaveTileBytes;
        const dim3 block(p.waves * 64);
        if (p.stages == kWaveStagesDeep)
            return p.r_packed ? launch(rotq_wave_kernel<kWaveStagesDeep, true>, grid, block, lds, stream, p)
                              : launch(rotq_wave_kernel<kWaveStagesDeep, false>, grid, block, lds, stream, p);
        return p.r_packed ? launch(rotq_wave_kernel<kWaveStages, true>, grid, block, lds, stream, p)
                          : launch(rotq_wave_kernel<kWaveStages, false>, grid, block, lds, stream, p);
    }
    if (p.r_packed) return hipErrorInvalidValue;             // the packed blocks feed the tiled-output kernel only
    return launch(rotq_kernel<kRotqWaves, kRotqStages, false>, grid, dim3(kRotqWaves * 64), TL::kLdsBytes, stream, p);
}

// Offline: the rotation blocks in the packed form load_rot_operand_packed reads.  One wave per block; the pieces are
// made by the very code the unpacked kernels run at their start, so both forms rotate with the same bits.
__global__ __launch_bounds__(64) void pack_rotation_kernel(PackRotationParams p) {
    const int lane = threadIdx.x, c = lane & 31, h = lane >> 5;
    RotOperand op;
    load_rot_operand(p.R + (int64_t)blockIdx.x * 1024, c, h, op);
    u32x4* q = (u32x4*)(p.packed + (int64_t)blockIdx.x * kPackedBlockBytes) + lane;
    q[0 * 64] = __builtin_bit_cast(u32x4, op.lo[0]);
    q[1 * 64] = __builtin_bit_cast(u32x4, op.lo[1]);
    q[2 * 64] = __builtin_bit_cast(u32x4, op.mid[0]);
    q[3 * 64] = __builtin_bit_cast(u32x4, op.mid[1]);
    q[4 * 64] = __builtin_bit_cast(u32x4, op.hi[0]);
    q[5 * 64] = __builtin_bit_cast(u32x4, op.hi[1]);
}

hipError_t launch_pack_rotation(const PackRotationParams& p, hipStream_t stream) {
    return launch(pack_rotation_kernel, dim3((unsigned)p.n_blocks), dim3(64), 0, stream, p);
}

// Test-only: the same quantize_group on fp32 values read from memory in the accumulator layout.
__global__ __launch_bounds__(64) void quant_dbg_kernel(QuantDbgParams p) {
    const int lane = threadIdx.x, c = lane & 31, h = lane >> 5;
    const int j = blockIdx.x;
    const int row = blockIdx.y * 32 + c;
    const int rl = row < p.rows ? row : p.rows - 1;
    const float* yr = p.y + (int64_t)rl * p.ldy + 32 * j + 4 * h;
    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float4 v = *(const float4*)(yr + 8 * q);
        acc[4 * q] = v.x; acc[4 * q + 1] = v.y; acc[4 * q + 2] = v.z; acc[4 * q + 3] = v.w;
    }
    uint2 o;
    uint32_t byte = quantize_group(acc, o);
    if (row < p.rows) {
        *(uint2*)(p.codes + (int64_t)row * p.G * 16 + 16 * j + 8 * h) = o;
        if (h == 0) p.scales[(int64_t)row * p.G + j] = (uint8_t)byte;
    }
}

hipError_t launch_quant_dbg(const QuantDbgParams& p, hipStream_t stream) {
    dim3 grid((unsigned)p.G, (unsigned)((p.rows + 31) / 32)), block(64);
    return launch(quant_dbg_kernel, grid, block, 0, stream, p);
}

}  // namespace duqpp
