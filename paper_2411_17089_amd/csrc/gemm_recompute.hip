// Recompute GEMM for gfx950 (Eq. 7 with fused bias):
//     C[M, N] = A[M, K] . W[N, K]^T + bias[N]        float16 in / float32 accumulate / float16 out
// A = X[0:l] flattened to [l*batch, hidden], W = [Wk^T ; Wv^T] ([2h, h], K contiguous), C = rows
// [0, l) of the device KV buffer (row stride ldc = 2h), so the result needs no copy or merge pass.
//
// Design (MI355X):
//  * One workgroup owns a BM x BN tile of C (256 x 256 by default, 8 waves as 4 x 2) and walks K in
//    stages of 64: one whole 128-byte line of every operand row.  A stage is two blocks in LDS (the A
//    rows and the W rows, 32 KiB each); five blocks form a ring that fills the 160 KiB of LDS.
//  * Blocks are filled by direct global->LDS DMA (global_load_lds_dwordx4): no staging registers, no
//    ds_write.  An instruction covers 8 rows x 128 B.  What limits this kernel is that path: measured
//    alone it delivers 40 B/clk/CU with 64-byte row pieces, 50 with 128-byte ones and 56 with 256-byte
//    ones, against the 32 B/clk/CU that a 256 x 256 tile consumes at the full MFMA rate; with the DMA
//    taken out of the loop the same schedule runs 25 % faster.  Whole lines per row is what moved it.
//  * The 16-byte chunks of a row are XOR-swizzled by (row/2)%8 on the global-address side so that the
//    ds_read_b128 of 16 consecutive rows touches 16 different bank groups.
//  * The loop is software-pipelined by hand: per stage four groups of MFMAs, each covering the LDS
//    latency of the next operand fragments; one workgroup barrier per stage, placed before the last
//    group; the wait in front of it is a counted vmcnt (the youngest block stays in flight).
//  * v_mfma_f32_32x32x16_f16 is issued "transposed" (W rows feed the instruction's row operand, X
//    rows its column operand) so a lane owns 4 consecutive output columns per accumulator quad.
//  * Epilogue: bias + conversion in registers, C tile staged through LDS, global stores of whole
//    512-byte row pieces.  Stores straight from registers (8-byte pieces, or 16-byte pieces after a
//    v_permlane32_swap) cost 10-15 % of the kernel: 32 rows x 32 bytes per instruction is a poor write.
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
#include <mutex>
#include <type_traits>

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

constexpr int BK = 64;           // halfs per stage: one 128-byte line per row
constexpr int ROW_BYTES = 128;   // one LDS row of a block
constexpr int NBLK = 5;          // ring of half-stage blocks (A rows or W rows of one stage)

// rotary epilogue: table[pos * HD/2 + i] = (cos, sin)(pos * theta_i); columns [0, cols) of C are rotated
struct RopeArgs {
    const float2* table;
    int cols, batch, pos0;
};

template <int VM, int LGKM0>
__device__ __forceinline__ void wait_counts() {
    // vmcnt(VM) [bits 3:0 and 15:14], expcnt untouched (7), lgkmcnt(0) if LGKM0 else untouched (15)
    __builtin_amdgcn_s_waitcnt((VM & 15) | ((VM >> 4) << 14) | 0x0070 | (LGKM0 ? 0 : 0x0F00));
}

template <int BM, int BN, int WM, int WN, int GROUP_M, int HD>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bias_f16(
    const _Float16* __restrict__ A, const _Float16* __restrict__ W, const _Float16* __restrict__ bias,
    _Float16* __restrict__ C, int64_t M, int N, int K, int64_t ldc, int tiles_m, int tiles_n, int tiles_per_xcd,
    int xcd_split_n, RopeArgs rope) {
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int LA = BM / 8 / NW, LW = BN / 8 / NW;     // DMA instructions per wave per block (8 rows x 128 B each)
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile/waves mismatch");
    constexpr int BLK_BYTES = (BM > BN ? BM : BN) * ROW_BYTES;
    constexpr int NMFMA = TM * TN, NFRAG = TM + TN;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int pid = blockIdx.x;
    int tile_m, tile_n;
    if (xcd_split_n) {
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

    // DMA: instruction i of this wave fills block rows [8*(wave + NW*i), +8); lane L lands at row 8*blk + L/8,
    // physical 16-byte chunk L%8, and therefore fetches logical chunk (L%8) ^ ((row/2)%8): with 128-byte rows the
    // ds_read_b128 of 16 consecutive rows then touches 16 different bank groups.
    const _Float16* srca[LA];
    const _Float16* srcw[LW];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = (wave + NW * i) * 8 + (lane >> 3);
        int64_t gr = m0 + row;
        if (gr > M - 1) gr = M - 1;
        srca[i] = A + gr * K + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int row = (wave + NW * i) * 8 + (lane >> 3);
        int gr = n0 + row;
        if (gr > N - 1) gr = N - 1;
        srcw[i] = W + (int64_t)gr * K + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
    }
    auto issue_a = [&](int kt, int slot) {
        unsigned char* base = lds + slot * BLK_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(srca[i] + kt * BK), (lds_ptr_t)(base + i * NW * 1024), 16, 0, 0);
    };
    auto issue_w = [&](int kt, int slot) {
        unsigned char* base = lds + slot * BLK_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LW; ++i)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(srcw[i] + kt * BK), (lds_ptr_t)(base + i * NW * 1024), 16, 0, 0);
    };
    auto inc = [](int s, int d) { s += d; return s >= NBLK ? s - NBLK : s; };

    // fragment addresses: row r of a block, k-step kk (16 halfs = two 16-byte chunks, lane half picks one).  The
    // swizzle term (r/2)%8 depends only on lane%32 because every wave / tile offset is a multiple of 32 rows.
    const int frow = lane & 31, fhalf = lane >> 5;
    int koff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = frow * ROW_BYTES + (((kk * 2 + fhalf) ^ ((frow >> 1) & 7)) << 4);

    floatx16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    half8 af0[TM], wf0[TN], af1[TM], wf1[TN];
    auto load_frags = [&](int sa, int sw, int kk, half8* af, half8* wf) {
        const unsigned char* pa = lds + sa * BLK_BYTES + wm * WTM * ROW_BYTES + koff[kk];
        const unsigned char* pw = lds + sw * BLK_BYTES + wn * WTN * ROW_BYTES + koff[kk];
#pragma unroll
        for (int t = 0; t < TM; ++t) af[t] = *reinterpret_cast<const half8*>(pa + t * 32 * ROW_BYTES);
#pragma unroll
        for (int t = 0; t < TN; ++t) wf[t] = *reinterpret_cast<const half8*>(pw + t * 32 * ROW_BYTES);
    };
    auto mfma_group = [&](const half8* af, const half8* wf) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[i], af[j], acc[i][j], 0, 0, 0);
    };
    auto interleave = [&](auto id) {
        constexpr int ID = decltype(id)::value;
#pragma unroll
        for (int x = 0; x < NFRAG; ++x) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, ID);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, ID);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, ID);
        __builtin_amdgcn_sched_barrier(0);
    };
    // Ring protocol.  Block 2*kt holds the A rows of stage kt, block 2*kt+1 its W rows; block j lives in slot j % 5.
    // Stage kt issues block 2*kt+4 (A of stage kt+2) in its first k-step and block 2*kt+5 (W of stage kt+2) after its
    // barrier, into the slots that stage kt-1's W rows and stage kt's A rows have left.
    const int KT = K / BK;
    issue_a(0, 0);
    issue_w(0, 1);
    if (KT > 1) {
        issue_a(1, 2);
        issue_w(1, 3);
        wait_counts<LA + LW, 0>();
    } else {
        wait_counts<0, 0>();
    }
    __builtin_amdgcn_s_barrier();
    load_frags(0, 1, 0, af0, wf0);

    // consumes the stage whose A rows sit in slot sa (W rows in sa + 1); on return (af0, wf0) hold k-step 0 of the next
    auto stage = [&](int kt, int sa, auto more) {
        constexpr bool MORE = decltype(more)::value;   // stage kt + 2 exists
        const int sw = inc(sa, 1), sa2 = inc(sa, 2), sw2 = inc(sa, 3), sfree = inc(sa, 4);
        if (MORE) issue_a(kt + 2, sfree);
        load_frags(sa, sw, 1, af1, wf1);
        mfma_group(af0, wf0);
        interleave(std::integral_constant<int, 0>{});
        load_frags(sa, sw, 2, af0, wf0);
        mfma_group(af1, wf1);
        interleave(std::integral_constant<int, 1>{});
        load_frags(sa, sw, 3, af1, wf1);
        mfma_group(af0, wf0);
        interleave(std::integral_constant<int, 2>{});
        // this wave's reads of the stage are complete and its share of the next stage has landed
        if (MORE) wait_counts<LA, 1>();
        else wait_counts<0, 1>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (MORE) issue_w(kt + 2, sa);
        load_frags(sa2, sw2, 0, af0, wf0);
        mfma_group(af1, wf1);
        interleave(std::integral_constant<int, 3>{});
    };
    int kt = 0, sa = 0;
    for (; kt + 2 < KT; ++kt) {
        stage(kt, sa, std::true_type{});
        sa = inc(sa, 2);
    }
    if (kt + 1 < KT) {
        stage(kt, sa, std::false_type{});
        sa = inc(sa, 2);
        ++kt;
    }
    {   // last stage: nothing follows
        const int sw = inc(sa, 1);
        load_frags(sa, sw, 1, af1, wf1);
        mfma_group(af0, wf0);
        load_frags(sa, sw, 2, af0, wf0);
        mfma_group(af1, wf1);
        load_frags(sa, sw, 3, af1, wf1);
        mfma_group(af0, wf0);
        mfma_group(af1, wf1);
    }

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

int g_gemm_xcd_split_n = -1;   // -1 = default choice (debug hook; process-wide, set it only while no launch is in progress)

// Which mapping of workgroups to tiles: measured on MI355X at M = 24576-26624, giving every XCD a band of W wins once
// W no longer sits comfortably in the memory-side cache next to the A panels in flight (+3.7 % at N = 10240, K = 5120,
// 100 MiB; more at N = 14336, K = 7168, 196 MiB), and loses 1-2 % when W is small (64 MiB at K = 4096).
bool band_mapping(int N, int K) {
    if ((N + 255) / 256 < 8) return false;
    if (g_gemm_xcd_split_n >= 0) return g_gemm_xcd_split_n != 0;
    return (int64_t)N * K * 2 > ((int64_t)80 << 20);
}

template <int BM, int BN, int WM, int WN, int GROUP_M, int HD = 0>
int launch_tile(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                hipStream_t st, RopeArgs rope = RopeArgs{nullptr, 0, 1, 0}) {
    auto kern = gemm_bias_f16<BM, BN, WM, WN, GROUP_M, HD>;
    constexpr int ring_bytes = NBLK * (BM > BN ? BM : BN) * ROW_BYTES, c_bytes = BM * (BN * 2 + 16);
    constexpr int lds_bytes = ring_bytes > c_bytes ? ring_bytes : c_bytes;
    // once per process and instantiation; call_once makes concurrent first launches from several threads safe
    static std::once_flag configured;
    static hipError_t configure_status = hipSuccess;
    std::call_once(configured, [&] {
        configure_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    KVPR_HIP(configure_status);
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
    const int64_t total = (int64_t)tiles_m * tiles_n;
    const int xcd_split_n = band_mapping(N, K) ? 1 : 0;
    const int max_width = (tiles_n + 7) / 8;
    const int tiles_per_xcd = xcd_split_n ? max_width * tiles_m : (int)((total + 7) / 8);
    const unsigned grid = (unsigned)(tiles_per_xcd * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds_bytes, st, (const _Float16*)a, (const _Float16*)w,
                       (const _Float16*)bias, (_Float16*)c, M, N, K, ldc, tiles_m, tiles_n, tiles_per_xcd, xcd_split_n, rope);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

int g_gemm_variant = 0;

}  // namespace

int launch_gemm(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                hipStream_t st) {
    if (M == 0) return KVPR_OK;
    switch (g_gemm_variant) {   // variants other than 0 exist for tests and tuning sweeps
        case 1: return launch_tile<256, 256, 2, 4, 8>(a, w, bias, c, M, N, K, ldc, st);
        case 2: return launch_tile<256, 128, 2, 2, 8>(a, w, bias, c, M, N, K, ldc, st);
        case 3: return launch_tile<128, 128, 2, 2, 8>(a, w, bias, c, M, N, K, ldc, st);
        default:
            // raster groups of 4 tile rows inside an XCD's band of W (7 tile columns at N = 14336: a 4 x 7 block is
            // what 32 compute units cover), 8 with the row mapping: 1.5 % at M = 24576, N = 14336, K = 7168
            return band_mapping(N, K) ? launch_tile<256, 256, 4, 2, 4>(a, w, bias, c, M, N, K, ldc, st)
                                      : launch_tile<256, 256, 4, 2, 8>(a, w, bias, c, M, N, K, ldc, st);
    }
}

// Eq. 7 for a rotary model: as launch_gemm, with columns [0, rope_cols) (the K half) rotated by the position
// pos0 + row / batch of their row.  table: float2 [positions][head_dim/2] on the device.
int launch_gemm_rope(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                     const void* table, int rope_cols, int head_dim, int batch, int pos0, hipStream_t st) {
    if (M == 0) return KVPR_OK;
    const RopeArgs r{(const float2*)table, rope_cols, batch, pos0};
    if (head_dim == 64) return launch_tile<256, 256, 4, 2, 8, 64>(a, w, bias, c, M, N, K, ldc, st, r);
    return band_mapping(N, K) ? launch_tile<256, 256, 4, 2, 4, 128>(a, w, bias, c, M, N, K, ldc, st, r)
                              : launch_tile<256, 256, 4, 2, 8, 128>(a, w, bias, c, M, N, K, ldc, st, r);
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
