// Recompute GEMM for gfx950 (Eq. 7 with fused bias):
//     C[M, N] = A[M, K] . W[N, K]^T + bias[N]        float16 in / float32 accumulate / float16 out
// A = X[0:l] flattened to [l*batch, hidden], W = [Wk^T ; Wv^T] ([2h, h], K contiguous), C = rows
// [0, l) of the device KV buffer (row stride ldc = 2h), so the result needs no copy or merge pass.
//
// Design (MI355X):
//  * One workgroup owns a BM x BN tile of C (256 x 256 by default, 8 waves as 4 x 2) and walks K in
//    stages of 32.  A stage is (BM + BN) rows of 64 bytes in LDS; NSTAGE = 4 stages form a ring.
//  * Stages are filled by direct global->LDS DMA (global_load_lds_dwordx4): no staging registers, no
//    ds_write.  A wave-load covers 16 rows x 64 B; the 16-byte chunks of a row are XOR-swizzled by
//    (row/4)%4 on the global-address side so that the ds_read_b128 of 16 consecutive rows touches 16
//    different bank groups (measured: SQ_LDS_BANK_CONFLICT = 0).
//  * The loop is software-pipelined by hand: the workgroup barrier sits between two MFMA groups, each
//    group covers the LDS latency of the next operand fragments and the issue of the refill DMA, and
//    the wait before the barrier is a counted vmcnt (the NSTAGE-2 younger stages stay in flight).
//  * v_mfma_f32_32x32x16_f16 is issued "transposed" (W rows feed the instruction's row operand, X
//    rows its column operand) so a lane owns 4 consecutive output columns per accumulator quad.
//  * Epilogue: bias + conversion in registers, C tile staged through LDS, global stores of whole
//    512-byte row pieces (the direct 8-byte stores of the first version cost ~15 % of the kernel).
//  * Workgroup ids are remapped so that the workgroups an XCD runs concurrently (ids equal mod 8)
//    form a compact block of tiles sharing A/W panels in that XCD's L2.  Across XCDs there are two
//    mappings: each XCD takes a contiguous share of the tile rows (W is re-read by all XCDs and lives in
//    the memory-side cache; best while W is small), or each XCD takes a band of tile columns and all
//    walk the tile rows together (the A panels in flight are shared by the eight XCDs; best for large W).
//  * Tail rows in M / N are clamped on load (they re-read the last valid row) and skipped on store.
//  * Rotary models (HD = head width 64 or 128): the cache holds K after the rotary embedding, so the
//    recomputed K columns are rotated in the epilogue with the position of their row
//    (pos0 + row / batch), in float32 and in registers: a wave tile is 128 columns wide, so a
//    column and its partner at distance HD/2 sit in the same lane, two or one accumulator tiles
//    apart.  cos/sin come from a float2 table [position][HD/2] (L1/L2 hits: a tile spans few positions).
#include "kvpr_internal.h"
#include <type_traits>

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

constexpr int BK = 32;          // halfs per stage
constexpr int ROW_BYTES = 64;   // one LDS row of a stage

// rotary epilogue: table[pos * HD/2 + i] = (cos, sin)(pos * theta_i); columns [0, cols) of C are rotated
struct RopeArgs {
    const float2* table;
    int cols, batch, pos0;
    int xcd_split_n;     // tile -> workgroup mapping (not a rotary parameter; rides in the same argument block)
};

template <int VM, int LGKM0>
__device__ __forceinline__ void wait_counts() {
    // vmcnt(VM) [bits 3:0 and 15:14], expcnt untouched (7), lgkmcnt(0) if LGKM0 else untouched (15)
    __builtin_amdgcn_s_waitcnt((VM & 15) | ((VM >> 4) << 14) | 0x0070 | (LGKM0 ? 0 : 0x0F00));
}

template <int BM, int BN, int WM, int WN, int NSTAGE, int GROUP_M, int HD>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bias_f16(
    const _Float16* __restrict__ A, const _Float16* __restrict__ W, const _Float16* __restrict__ bias,
    _Float16* __restrict__ C, int64_t M, int N, int K, int64_t ldc, int tiles_m, int tiles_n, int tiles_per_xcd,
    RopeArgs rope) {
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int BLOCKS = (BM + BN) / 16;
    constexpr int LOADS = BLOCKS / NW;
    static_assert(BLOCKS % NW == 0, "tile/waves mismatch");
    static_assert(NSTAGE >= 3 && NSTAGE <= 4, "ring depth");
    constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    constexpr int NMFMA = TM * TN, NFRAG = TM + TN;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int pid = blockIdx.x;
    int tile_m, tile_n;
    if (rope.xcd_split_n) {
        // every XCD owns a band of tile columns and all XCDs walk the tile rows together: the A panels in use are
        // shared by the eight XCDs (one HBM fetch, then memory-side cache hits) and W can stay in that cache
        const int xcd = pid & 7, i = pid >> 3;
        const int n_lo = xcd * tiles_n / 8, width = (xcd + 1) * tiles_n / 8 - n_lo;
        if (i >= width * tiles_m) return;
        const int group_sz = GROUP_M * width;
        const int group = i / group_sz;
        const int first_m = group * GROUP_M;
        const int gm = min(tiles_m - first_m, GROUP_M);
        const int in_group = i - group * group_sz;
        tile_m = first_m + in_group % gm;
        tile_n = n_lo + in_group / gm;
    } else {
        const int logical = (pid & 7) * tiles_per_xcd + (pid >> 3);
        if (logical >= tiles_m * tiles_n) return;
        const int group_sz = GROUP_M * tiles_n;
        const int group = logical / group_sz;
        const int first_m = group * GROUP_M;
        const int gm = min(tiles_m - first_m, GROUP_M);
        const int in_group = logical - group * group_sz;
        tile_m = first_m + in_group % gm;
        tile_n = in_group / gm;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // wave-load i of this wave fills stage rows [16*blk, 16*blk+16) (A rows first, then W rows); lane L
    // lands at row 16*blk + L/4, physical chunk L%4, and therefore fetches logical chunk (L%4)^((row/4)%4)
    const _Float16* src[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int blk = wave + i * NW;
        const int row = blk * 16 + (lane >> 2);
        const int pc = lane & 3;
        if (blk * 16 < BM) {
            int64_t gr = m0 + row;
            if (gr > M - 1) gr = M - 1;
            src[i] = A + gr * K + ((pc ^ ((row >> 2) & 3)) << 3);
        } else {
            const int wr = row - BM;
            int gr = n0 + wr;
            if (gr > N - 1) gr = N - 1;
            src[i] = W + (int64_t)gr * K + ((pc ^ ((wr >> 2) & 3)) << 3);
        }
    }
    auto issue_loads = [&](int kt) {
        unsigned char* base = lds + (kt % NSTAGE) * STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src[i] + kt * BK), (lds_ptr_t)(base + i * NW * 1024), 16, 0, 0);
    };

    const int frow = lane & 31, fhalf = lane >> 5;
    int a_off[TM][2], w_off[TN][2];
#pragma unroll
    for (int t = 0; t < TM; ++t) {
        const int r = wm * WTM + t * 32 + frow;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) a_off[t][kk] = r * ROW_BYTES + (((kk * 2 + fhalf) ^ ((r >> 2) & 3)) << 4);
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int r = wn * WTN + t * 32 + frow;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) w_off[t][kk] = BM * ROW_BYTES + r * ROW_BYTES + (((kk * 2 + fhalf) ^ ((r >> 2) & 3)) << 4);
    }

    floatx16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    half8 af0[TM], wf0[TN], af1[TM], wf1[TN];
    auto load_frags = [&](int kt, int kk, half8* af, half8* wf) {
        const unsigned char* st = lds + (kt % NSTAGE) * STAGE_BYTES;
#pragma unroll
        for (int t = 0; t < TM; ++t) af[t] = *reinterpret_cast<const half8*>(st + a_off[t][kk]);
#pragma unroll
        for (int t = 0; t < TN; ++t) wf[t] = *reinterpret_cast<const half8*>(st + w_off[t][kk]);
    };
    auto mfma_group = [&](const half8* af, const half8* wf) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[i], af[j], acc[i][j], 0, 0, 0);
    };
    const int KT = K / BK;
#pragma unroll
    for (int d = 0; d < NSTAGE; ++d)
        if (d < KT) issue_loads(d);
    if (KT >= NSTAGE) wait_counts<(NSTAGE - 1) * LOADS, 0>();
    else wait_counts<0, 0>();
    __builtin_amdgcn_s_barrier();
    load_frags(0, 0, af0, wf0);

    // one ring step: consumes stage kt, leaves the fragments of k-step 0 of stage kt+1 in (af0, wf0)
    auto step = [&](int kt, auto refill) {
        // phase A: fetch the fragments of k-step 1 of this stage while the MFMAs of k-step 0 run
        load_frags(kt, 1, af1, wf1);
        mfma_group(af0, wf0);
#pragma unroll
        for (int x = 0; x < NFRAG; ++x) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
        __builtin_amdgcn_sched_barrier(0);
        // this wave's reads of stage kt are complete (lgkmcnt 0) and stage kt+1 has landed: in the
        // steady state the NSTAGE-2 stages issued after it may still be in flight
        if (decltype(refill)::value) wait_counts<(NSTAGE - 2) * LOADS, 1>();
        else wait_counts<0, 1>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // phase B: refill the slot just freed, fetch k-step 0 of the next stage, run k-step 1 of this one
        if (decltype(refill)::value) issue_loads(kt + NSTAGE);
        load_frags(kt + 1, 0, af0, wf0);
        mfma_group(af1, wf1);
#pragma unroll
        for (int x = 0; x < NFRAG; ++x) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    int kt = 0;
    for (; kt < KT - NSTAGE; ++kt) step(kt, std::true_type{});
    for (; kt < KT - 1; ++kt) step(kt, std::false_type{});
    load_frags(kt, 1, af1, wf1);
    mfma_group(af0, wf0);
    mfma_group(af1, wf1);

    // ---- epilogue: bias + float16 conversion in registers, then through LDS so that every global
    //      store instruction writes whole 512-byte pieces of C rows (accumulator register r of tile
    //      (i, j) holds n = 32*i + 8*(r/4) + 4*(lane/32) + r%4, m = 32*j + lane%32 of the wave tile).
    //      Rows are padded by 16 bytes: the 8-byte writes of 32 consecutive rows then spread over all banks.
    constexpr int CROW = BN * 2 + 16;
    __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): this wave's operand reads are done
    __builtin_amdgcn_s_barrier();                  // ... and everybody else's: the stages can be overwritten
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = wn * WTN + i * 32 + 8 * g + 4 * fhalf;
            if (bias && n0 + nl < N) {
                const half4 b4 = *reinterpret_cast<const half4*>(bias + n0 + nl);
#pragma unroll
                for (int j = 0; j < TM; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][j][g * 4 + e] += (float)b4[e];
            }
        }
    }
    if constexpr (HD > 0) {
        constexpr int IH = HD / 64;                // accumulator tiles between a column and its partner HD/2 columns on
        static_assert(WTN % HD == 0 && TN % (2 * IH) == 0, "a wave tile must hold whole heads");
        if (n0 + wn * WTN < rope.cols) {           // wave-uniform: this wave's 128 columns are K columns
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                int64_t m = m0 + wm * WTM + j * 32 + frow;
                if (m > M - 1) m = M - 1;
                const float2* trow = rope.table + (int64_t)(rope.pos0 + (int)(m / rope.batch)) * (HD / 2);
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    if ((i / IH) % 2 != 0) continue;   // second half of a head: handled with its partner
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int f = (i % IH) * 32 + 8 * g + 4 * fhalf;
                        const float4 cs0 = *reinterpret_cast<const float4*>(trow + f);
                        const float4 cs1 = *reinterpret_cast<const float4*>(trow + f + 2);
                        const float cv[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, sv[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float x1 = acc[i][j][g * 4 + e], x2 = acc[i + IH][j][g * 4 + e];
                            acc[i][j][g * 4 + e] = x1 * cv[e] - x2 * sv[e];
                            acc[i + IH][j][g * 4 + e] = x2 * cv[e] + x1 * sv[e];
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = wn * WTN + i * 32 + 8 * g + 4 * fhalf;
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int ml = wm * WTM + j * 32 + frow;
                half4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (_Float16)acc[i][j][g * 4 + e];
                *reinterpret_cast<half4*>(lds + ml * CROW + nl * 2) = o;
            }
        }
    }
    __syncthreads();
    constexpr int CHUNKS_PER_ROW = BN / 8;         // 16-byte pieces
    constexpr int NT = NW * 64;
#pragma unroll 4
    for (int q = tid; q < BM * CHUNKS_PER_ROW; q += NT) {
        const int ml = q / CHUNKS_PER_ROW, cc = q % CHUNKS_PER_ROW;
        const int64_t m = m0 + ml;
        const int n = n0 + cc * 8;
        if (m < M && n < N)
            __builtin_nontemporal_store(*reinterpret_cast<const half8*>(lds + ml * CROW + cc * 16),
                                        reinterpret_cast<half8*>(C + m * ldc + n));   // C is not re-read here: keep it out of L2
    }
}

int g_gemm_xcd_split_n = -1;   // -1 = default choice

template <int BM, int BN, int WM, int WN, int NSTAGE, int GROUP_M, int HD = 0>
int launch_tile(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                hipStream_t st, RopeArgs rope = RopeArgs{nullptr, 0, 1, 0, 0}) {
    auto kern = gemm_bias_f16<BM, BN, WM, WN, NSTAGE, GROUP_M, HD>;
    constexpr int stage_bytes = NSTAGE * (BM + BN) * ROW_BYTES, c_bytes = BM * (BN * 2 + 16);
    constexpr int lds_bytes = stage_bytes > c_bytes ? stage_bytes : c_bytes;
    static bool configured = false;   // per process and instantiation (one device is used)
    if (!configured) {
        KVPR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     lds_bytes));
        configured = true;
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
    const int64_t total = (int64_t)tiles_m * tiles_n;
    // Which mapping: measured on MI355X, giving every XCD a band of W wins once W no longer sits comfortably in the
    // memory-side cache next to the A panels in flight (N = 14336, K = 7168, 196 MiB: +12 %), and loses 1-2 % when W
    // is small (64 MiB at K = 4096); equal at 100 MiB.
    const bool big_w = (int64_t)N * K * 2 > ((int64_t)128 << 20);
    rope.xcd_split_n = g_gemm_xcd_split_n >= 0 ? g_gemm_xcd_split_n : (big_w ? 1 : 0);
    if (tiles_n < 8) rope.xcd_split_n = 0;
    const int max_width = (tiles_n + 7) / 8;
    const int tiles_per_xcd = rope.xcd_split_n ? max_width * tiles_m : (int)((total + 7) / 8);
    const unsigned grid = (unsigned)(tiles_per_xcd * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds_bytes, st, (const _Float16*)a, (const _Float16*)w,
                       (const _Float16*)bias, (_Float16*)c, M, N, K, ldc, tiles_m, tiles_n, tiles_per_xcd, rope);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

int g_gemm_variant = 0;

}  // namespace

int launch_gemm(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                hipStream_t st) {
    if (M == 0) return KVPR_OK;
    switch (g_gemm_variant) {   // variants other than 0 exist for tests and tuning sweeps
        case 1: return launch_tile<256, 256, 2, 2, 4, 8>(a, w, bias, c, M, N, K, ldc, st);
        case 2: return launch_tile<256, 128, 2, 2, 3, 8>(a, w, bias, c, M, N, K, ldc, st);
        case 3: return launch_tile<128, 128, 2, 2, 4, 8>(a, w, bias, c, M, N, K, ldc, st);
        default: return launch_tile<256, 256, 4, 2, 4, 8>(a, w, bias, c, M, N, K, ldc, st);
    }
}

// Eq. 7 for a rotary model: as launch_gemm, with columns [0, rope_cols) (the K half) rotated by the position
// pos0 + row / batch of their row.  table: float2 [positions][head_dim/2] on the device.
int launch_gemm_rope(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                     const void* table, int rope_cols, int head_dim, int batch, int pos0, hipStream_t st) {
    if (M == 0) return KVPR_OK;
    const RopeArgs r{(const float2*)table, rope_cols, batch, pos0, 0};
    if (head_dim == 64) return launch_tile<256, 256, 4, 2, 4, 8, 64>(a, w, bias, c, M, N, K, ldc, st, r);
    return launch_tile<256, 256, 4, 2, 4, 8, 128>(a, w, bias, c, M, N, K, ldc, st, r);
}

}  // namespace kvpr

extern "C" int kvpr_debug_set_gemm_variant(int v) {
    kvpr::g_gemm_variant = v;
    return KVPR_OK;
}

extern "C" int kvpr_debug_set_gemm_mapping(int xcd_split_n) {
    kvpr::g_gemm_xcd_split_n = xcd_split_n;
    return KVPR_OK;
}
