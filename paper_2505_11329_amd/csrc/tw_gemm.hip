// bf16 GEMM for gfx950 on the matrix cores: the stand-in for the projection of
// the "other" token split that runs next to the fused kernel (TokenWeave, arXiv
// 2505.11329, Fig. 7b and Section 4.1.2; the paper uses a vendor GEMM there).
// C[M x N] = A[M x K] * B(k, n), fp32 accumulation, one rounding to bf16.
//
// Design
//   - Workgroup tile 256 (M) x 128 (N), K step 64, 512 threads = 8 wave64 laid
//     out 4 x 2, each wave owning a 64 x 64 sub-tile as 4 x 4 blocks of
//     v_mfma_f32_16x16x32_bf16 (64 accumulator registers per lane). The part
//     runs this kernel at its power limit, and per flop the 16 x 16 x 32 shape
//     moves half the accumulator registers of the 32 x 32 x 16 one: loops of
//     nothing but MFMAs on N(0, 0.02^2) operands sustain 1.99 PFLOP/s with the
//     former and 1.75 with the latter on this device.
//   - Operand tiles go from global memory straight into LDS (gfx950's 16-byte
//     buffer_load ... lds): no register staging and no ds_write. Three LDS
//     stages of 32 + 16 KiB, so a load has two full K steps to land; one
//     workgroup per compute unit.
//   - LDS rows are 128 bytes (64 bf16 of K); two rows make a 256-byte line over
//     all 64 banks and the 16-byte pieces are xor-swizzled with the line number,
//     which makes the MFMA operand reads free of bank conflicts without padding
//     (measured: 178 B/clk/CU against 128 for a swizzle that assumes 32 banks,
//     32 unswizzled; with K steps of 32 a row is a quarter of a line and the
//     swizzle is a different one, see lds_piece). An LDS-direct load writes 64
//     consecutive 16-byte slots per wave instruction, so the swizzle is applied
//     on the global side: the lane that fills slot s of line l fetches piece
//     (s & 7) ^ (l & 7) of row 2l + (s >> 3).
//   - The compiler cannot tell which LDS stage an asynchronous load targets and
//     would wait for ALL outstanding loads before any LDS read it can see;
//     operand fragments are therefore read with inline ds_read and the waits
//     (vmcnt for landed stages, lgkmcnt for fragments) are placed by hand.
//     Dynamic LDS is the kernel's only LDS object, so its byte offsets are LDS
//     addresses.
//   - The K loop is software-pipelined by hand, instruction by instruction:
//     between the MFMAs of one K sub-step (k = 32) a wave issues the LDS reads
//     of the next sub-step's fragments (during the first half, so that they
//     have the second half to arrive) and its share of the global loads of
//     K step kt + 2; the "next stage has landed" check (vmcnt + workgroup
//     barrier) sits before the last MFMA group of a K step, when every wave
//     still has matrix work queued.
//   - Large products launched on their own take 256 x 256 tiles instead: four
//     waves of 128 x 128 (256 accumulator registers per lane), K steps of 64 whose
//     operand areas rotate through a ring of five 32 KiB LDS slots, one operand's
//     loads per sub-step (see the K loop). With one wave per SIMD every
//     instruction between two MFMAs counts: a wave issues one instruction in
//     four clocks and an MFMA lasts sixteen.
//   - Each MFMA gets the B fragment as its first operand and the A fragment as
//     its second, so the 16x16 result block is held transposed: a lane owns one
//     row m of C and the block's four accumulator registers are four consecutive
//     columns n: one 8-byte bf16 quad. The quads of a wave's sub-tile are collected
//     in LDS and leave as 16-byte stores that cover whole rows of it.
//   - Ragged edges need no branches: operands are fetched through range-checked
//     buffer descriptors sized to the rows that exist (rows past M or N read as
//     zeros), K pieces past K are redirected out of range, and stores past the
//     edge are dropped the same way.
//   - Persistent grid of at most `budget` workgroups walking the tile list.
//     Workgroups are dealt to the 8 XCDs round-robin by the hardware, so
//     workgroup w takes tile (w mod 8) * ceil(T/8) + w / 8 of a list ordered in
//     compact blocks: the tiles an XCD works on share rows of A and columns of
//     B in that XCD's L2.
//   - B stored [K x N] (B_KN): the B tile lands as 64 k-rows of 256 bytes and the
//     MFMA operand (8 consecutive k of one column n) is gathered with the
//     transposing LDS read ds_read_b64_tr_b16.
#include <atomic>
#include <type_traits>
#include <utility>

#include "tw_device.h"
#include "tw_internal.h"

namespace tw {

static constexpr int BM = kGemmTileM;
static constexpr int kXcds = 8;
// what the tracing variant counts per wave, in shader clocks (tw_measure.h lists them in this order)
enum { kPhaseSub0, kPhaseLanded, kPhaseBarrier, kPhaseSub1, kPhaseFill, kPhaseStores, kPhaseTiles, kPhaseTotal };
static constexpr int kGemmPhases = TW_GEMM_PHASES;
static_assert(kPhaseTotal + 1 == kGemmPhases, "phase list");

// A tile configuration: WM x WN blocks of 16 x 16 per wave, 32 / WM waves laid
// out (16 / WM) x 2, hence a 256 x (32 * WN) workgroup tile; K steps of BK_;
// STAGES LDS stages. The library builds <4, 4, 3, 64>: eight waves of 64 x 64,
// tile 256 x 128, 3 x 48 KiB of LDS; for products with few tiles <4, 2, 3, 64>:
// eight waves of 64 x 32, tile 256 x 64, 3 x 40 KiB; and for large products
// <8, 8, 2, 64>: four waves of 128 x 128, tile 256 x 256, two K steps of 64 in a
// ring of five 32 KiB slots (STAGES = 2 stands for that ring, see the K loop).
static constexpr int kBlk = 16;    // rows and columns of one MFMA result block
static constexpr int kSubK = 32;   // K depth of one MFMA
template <int WM, int WN, int STAGES, int BK_>
struct TileCfg {
    static constexpr int kWaves = 2 * BM / (kBlk * WM);
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kBN = 2 * kBlk * WN;
    static constexpr int kStageABytes = BM * BK_ * 2;
    static constexpr int kStageBBytes = kBN * BK_ * 2;
    static constexpr int kStageBytes = kStageABytes + kStageBBytes;
    // Two stages of 2 x 32 KiB leave a fifth 32 KiB slot of the compute unit's LDS
    // free: the operand areas then rotate through five slots.
    static constexpr bool kRing = STAGES == 2;
    static constexpr int kRingSlots = 5;
    static constexpr int kLdsBytes = kRing ? kRingSlots * kStageABytes : STAGES * kStageBytes;
    static_assert(!kRing || kStageABytes == kStageBBytes, "ring slots hold either operand");
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct GemmParams {
    const char *A;
    const char *B;
    char *C;
    long long M, N, K;
    int tiles_m, tiles_n;
    int group_m;        // tile rows per block of the tile ordering
    int tiles_per_xcd;  // ceil(tiles / 8)
    unsigned long long *phase_cycles;  // tracing variant only: kGemmPhases counters per wave
};

// Byte offset inside a stage's A (or B) area of the 16-byte piece c of row r,
// rows of BK_ bf16, with the piece index xor-swizzled so that an MFMA operand
// fetch (lane l reads piece l / 16 of row l % 16) is free of bank conflicts. A
// ds_read_b128 is served in four passes of sixteen lanes over the 64 banks, and
// the passes are not runs of consecutive lanes (probed with reads that collide
// on purpose): lanes 0-3, 12-15, 20-23, 24-27 form one pass, lanes 4-11, 16-19,
// 28-31 the next, and the upper half of the wave likewise. One pass therefore
// fetches piece c of rows 0-3 and 12-15 together with piece c ^ 1 of rows 4-11.
//   BK_ = 64: two rows per 256-byte line, piece ^ (line & 7);
//   BK_ = 32: four rows per line, piece ^ ((r >> 1) & 3): of the four rows that
//   share a quarter of a line (r, r+4, r+8, r+12) two are read at piece c and two
//   at c ^ 1, and the swizzle sends the four to different pieces (a swizzle by
//   the line number, which would do for passes of consecutive lanes, leaves
//   every read two-way conflicted: 8.0 clocks against 5.7).
// Either way the sixteen lanes that write one line in the global->LDS copy
// touch every bank once.
template <int BK_>
__device__ __forceinline__ uint32_t lds_piece(int r, int c)
{
    if constexpr (BK_ == 64) {
        const int line = r / 2;
        return line * 256 + (((r % 2) * 8 + (c ^ (line & 7))) << 4);
    } else {
        return r * 64 + ((c ^ ((r >> 1) & 3)) << 4);
    }
}

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef __attribute__((address_space(3))) char *lds_char_ptr_t;

template <int OFF>
__device__ __forceinline__ bf16x8 lds_read16(uint32_t addr)
{
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
// gfx950's transposing LDS read. Within each group of 16 lanes, lane 4a+b
// receives, for j = 0..3, the b-th 16-bit element of the 8-byte chunk that lane
// a + 4j points at (lane mapping established with a probe kernel). With lane
// a + 4j pointing at row k0+j, columns 4a..4a+3 of a [k][n] tile, lane d = 4a+b
// ends up with column d of rows k0..k0+3: four consecutive k of one n, which is
// what an MFMA operand register pair holds.
template <int OFF>
__device__ __forceinline__ u32x2 lds_read_tr8(uint32_t addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}

// Operand fragments of one K sub-step (one MFMA deep, k = 32) for a wave that
// owns WM x WN blocks of 16 x 16: per block row of A and block column of B eight
// consecutive k per lane (lane l: row or column l % 16, k group l / 16). With B
// stored [K x N] (WN = 4 only) a B fragment arrives as two register pairs (k 0..3
// and k 4..7 of the lane's group).
template <bool B_KN, int WM, int WN>
struct Frags {
    bf16x8 a[WM];
    bf16x8 b[B_KN ? 1 : WN];
    u32x2 blo[B_KN ? WN : 1], bhi[B_KN ? WN : 1];
    // LDS reads that fill one set of fragments = registers (or register pairs)
    // a wait has to name: WM of A, and WN of B or, stored [K x N], 2 WN halves
    static constexpr int kReads = WM + (B_KN ? 2 * WN : WN);
};
// Wait until at most N of this wave's LDS reads are outstanding. The fragments
// are passed through so that no use of them can be moved above the wait. Each
// operand list comes with its length, which wait_lgkm checks against the number
// of reads that fill the fragments: a tile shape whose reads and waits disagree
// does not compile.
#define TW_FRAG_A4(f) "+v"((f).a[0]), "+v"((f).a[1]), "+v"((f).a[2]), "+v"((f).a[3])
#define TW_FRAG_A4_LEN 4
#define TW_FRAG_A8(f) TW_FRAG_A4(f), "+v"((f).a[4]), "+v"((f).a[5]), "+v"((f).a[6]), "+v"((f).a[7])
#define TW_FRAG_A8_LEN 8
#define TW_FRAG_B2(f) "+v"((f).b[0]), "+v"((f).b[1])
#define TW_FRAG_B2_LEN 2
#define TW_FRAG_B4(f) TW_FRAG_B2(f), "+v"((f).b[2]), "+v"((f).b[3])
#define TW_FRAG_B4_LEN 4
#define TW_FRAG_B8(f) TW_FRAG_B4(f), "+v"((f).b[4]), "+v"((f).b[5]), "+v"((f).b[6]), "+v"((f).b[7])
#define TW_FRAG_B8_LEN 8
#define TW_FRAG_B_KN4(f)                                                                            \
    "+v"((f).blo[0]), "+v"((f).bhi[0]), "+v"((f).blo[1]), "+v"((f).bhi[1]), "+v"((f).blo[2]),       \
        "+v"((f).bhi[2]), "+v"((f).blo[3]), "+v"((f).bhi[3])
#define TW_FRAG_B_KN4_LEN 8
#define TW_WAIT_LGKM(N, f, A_LIST, B_LIST)                                                               \
    do {                                                                                                  \
        static_assert(A_LIST##_LEN + B_LIST##_LEN == std::remove_reference_t<decltype(f)>::kReads,        \
                      "the wait must name every register an LDS fragment read writes");                   \
        asm volatile("s_waitcnt lgkmcnt(%[cnt])" : A_LIST(f), B_LIST(f) : [cnt] "n"(N) : "memory");       \
    } while (0)

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), unrolled
template <int... I, typename Fn>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, Fn &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename Fn>
__device__ __forceinline__ void static_for(Fn &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <int N, bool B_KN, int WM, int WN>
__device__ __forceinline__ void wait_lgkm(Frags<B_KN, WM, WN> &f)
{
    static_assert(WM == 4 || WM == 8, "fragment operand lists below");
    static_assert(B_KN ? (WM == 4 && WN == 4) : (WN == 2 || WN == 4 || WN == 8), "fragment operand lists below");
    if constexpr (B_KN) TW_WAIT_LGKM(N, f, TW_FRAG_A4, TW_FRAG_B_KN4);
    if constexpr (!B_KN && WM == 4 && WN == 2) TW_WAIT_LGKM(N, f, TW_FRAG_A4, TW_FRAG_B2);
    if constexpr (!B_KN && WM == 4 && WN == 4) TW_WAIT_LGKM(N, f, TW_FRAG_A4, TW_FRAG_B4);
    if constexpr (!B_KN && WM == 4 && WN == 8) TW_WAIT_LGKM(N, f, TW_FRAG_A4, TW_FRAG_B8);
    if constexpr (!B_KN && WM == 8 && WN == 4) TW_WAIT_LGKM(N, f, TW_FRAG_A8, TW_FRAG_B4);
    if constexpr (!B_KN && WM == 8 && WN == 8) TW_WAIT_LGKM(N, f, TW_FRAG_A8, TW_FRAG_B8);
}

// TRACE (256 x 256 tiles only): every wave also adds up the shader clocks it
// spends in each phase of the K loop and of a tile, and writes the sums out at
// its end (tw_gemm_bf16_traced). Reading the clock costs a scalar memory read and
// a wait for it each time, so the traced kernel is a few percent slower than the
// plain one and its figures are for comparing phases, not for the total.
template <bool B_KN, int WM, int WN, int STAGES, int BK, bool TRACE = false>
__global__ __launch_bounds__(64 * (2 * BM / (kBlk * WM))) void gemm_bf16_kernel(const GemmParams prm)
{
    // The body is for the device pass only: the host pass needs the launch stub,
    // and silently drops it when it cannot make sense of the target-specific
    // builtins and inline assembly below.
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ __attribute__((aligned(16))) char lds[];
    using Cfg = TileCfg<WM, WN, STAGES, BK>;
    constexpr int NW = Cfg::kWaves;
    constexpr int BN = Cfg::kBN;
    constexpr int kStageABytes = Cfg::kStageABytes;
    constexpr int kStageBytes = Cfg::kStageBytes;
    constexpr int kStages = STAGES;
    constexpr int kSubs = BK / kSubK;                        // K sub-steps (one MFMA deep) per K step
    constexpr bool kRing = Cfg::kRing;
    constexpr int kBlockBytes = kBlk * BK * 2;               // LDS distance between 16-row blocks
    constexpr int A_LOADS = kStageABytes / 1024 / NW;        // wave instructions (1 KiB each) per wave that
    constexpr int B_LOADS = Cfg::kStageBBytes / 1024 / NW;   // fill a stage's A area, and its B area
    constexpr int kLoads = A_LOADS + B_LOADS;                // loads of one K step per lane
    static_assert(BK == 64 || BK == 32, "LDS layouts below");
    static_assert(STAGES >= 2 && (STAGES - 1) * kLoads < 64 && 2 * kLoads < 64, "vmcnt field");
    static_assert(!B_KN || (WN == 4 && BK == 64), "[K x N] operands: 256 x 128 x 64 tiles only");
    static_assert(Cfg::kLdsBytes <= 160 * 1024, "LDS of one compute unit");
    static_assert(!kRing || (kSubs == 2 && !B_KN), "the ring schedule below");
    static_assert(!TRACE || kRing, "phases are counted in the ring schedule");
    // shader clock, with nothing of this wave's outstanding on the LDS/scalar counter afterwards
    auto now = [&]() {
        const unsigned long long t = __builtin_readcyclecounter();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        return t;
    };
    unsigned long long phase[kGemmPhases] = {};
    unsigned long long t_prev = 0, t_kernel = 0;
    if constexpr (TRACE) t_kernel = now();

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps LDS targets in scalar registers
    const int wave_m = wave >> 1;
    const int wave_n = wave & 1;
    const int l15 = lane & 15;   // the lane's row (A) or column (B) inside a block
    const int lgrp = lane >> 4;  // its group of eight k inside the MFMA's 32

    const long long row_bytes = prm.K * 2;      // of A, and of B when it is stored [N x K]
    const long long bkn_row_bytes = prm.N * 2;  // of B when it is stored [K x N]
    // An offset that is out of range whatever scalar offset (< 2^31) is added to it,
    // without wrapping: a tile's descriptor covers at most 256 rows of 2^23 bytes.
    constexpr uint32_t kPastK = 0x80000000u;
    // (at least one: with K = 0 it loads nothing but zeros)
    const int k_tiles = prm.K > 0 ? static_cast<int>((prm.K + BK - 1) / BK) : 1;
    const int total_tiles = prm.tiles_m * prm.tiles_n;

    // global -> LDS duty: wave instruction i of this wave fills slots
    // [(i * NW + wave) * 64, +64); this lane's slot inside a line and the row and
    // piece that belong there (the same for every instruction up to a row offset)
    const int line_in_instr = lane >> 4;            // 0..3
    const int slot = lane & 15;
    constexpr int kRowsPerLine = 128 / BK, kPieces = BK / 8;
    // line = (i * NW + wave) * 4 + line_in_instr, of which the swizzle uses the low bits
    // (BK = 32: a row is a quarter of a line, and the swizzle uses bits 1-2 of the row number)
    const int line_low = BK == 64 ? (((wave * 4) | line_in_instr) & 7) : (((line_in_instr * 4 + slot / 4) >> 1) & 3);
    const int piece = (slot % kPieces) ^ line_low;
    const int row_lo = kRowsPerLine * (wave * 4 + line_in_instr) + slot / kPieces;  // + 4 * kRowsPerLine * NW * i
    constexpr int kRowsPerInstr = 4 * kRowsPerLine * NW;  // rows all waves' instruction i cover
    // B stored [K x N]: its LDS area holds 64 k-rows of 256 bytes (128 n); a wave
    // instruction fills four rows; row r keeps 16-byte piece s at slot
    // s ^ ((r & 3) << 1) ^ ((r & 8) ? 8 : 0), so that the eight rows the first (and
    // the second) half of a wave's transposing read touches fall into different
    // banks: four rows per 16-lane group, two groups eight rows apart.
    const int bkn_row_lo = wave * 4 + line_in_instr;                  // + 4 * NW * i
    static_assert(!B_KN || NW == 8, "bit 3 of a row number below");
    const int bkn_piece = slot ^ (line_in_instr << 1) ^ (((wave >> 1) & 1) << 3);

    // fragment read addresses inside a stage's A area and inside its B area for
    // the wave's first 16-row block; block i lies 16 rows = kBlockBytes further
    // (the swizzle repeats within that), which goes into the read's offset field
    uint32_t fa_addr[kSubs], fb_addr[kSubs], fbkn_addr[B_KN ? WN : 1];
#pragma unroll
    for (int kk = 0; kk < kSubs; ++kk) {
        fa_addr[kk] = lds_piece<BK>(wave_m * (kBlk * WM) + l15, kk * 4 + lgrp);
        fb_addr[kk] = lds_piece<BK>(wave_n * (kBlk * WN) + l15, kk * 4 + lgrp);
    }
    if constexpr (B_KN) {
        // the 16-lane group lgrp gathers k group lgrp: its lane s = a + 4 j points at
        // row 8 lgrp + j, columns 4a..4a+3 of the 16-wide block (the second read of
        // a fragment, rows + 4, and the sub-step, rows + 32, are immediates: neither
        // changes the row bits the swizzle looks at)
        const int a4 = l15 & 3, j = l15 >> 2;
        const int row = lgrp * 8 + j;
#pragma unroll
        for (int i = 0; i < WN; ++i) {
            const int col = wave_n * (kBlk * WN) + i * kBlk + 4 * a4;
            const int piece_slot = (col >> 3) ^ (j << 1) ^ ((lgrp & 1) << 3);
            fbkn_addr[i] = row * 256 + (piece_slot << 4) + (col & 7) * 2;
        }
    } else {
        fbkn_addr[0] = 0;
    }

    using F = Frags<B_KN, WM, WN>;
    constexpr int kFragReads = F::kReads;  // LDS reads of one sub-step: what read_one issues and wait_lgkm names

    for (int w = blockIdx.x; w < prm.tiles_per_xcd * kXcds; w += gridDim.x) {
        const int slot_w = w / kXcds;
        const int lin = (w % kXcds) * prm.tiles_per_xcd + slot_w;
        if (lin >= total_tiles) continue;
        const int per_group = prm.group_m * prm.tiles_n;
        const int grp = lin / per_group;
        const int first_tm = grp * prm.group_m;
        const int gsz = min(prm.group_m, prm.tiles_m - first_tm);
        const int in_grp = lin - grp * per_group;
        const int tm = first_tm + in_grp % gsz;
        const int tn = in_grp / gsz;

        unsigned long long t_tile = 0;
        if constexpr (TRACE) t_tile = now();
        const long long m0 = static_cast<long long>(tm) * BM;
        const long long n0 = static_cast<long long>(tn) * BN;
        const int rows_a = static_cast<int>(min(static_cast<long long>(BM), prm.M - m0));
        const int rows_b = static_cast<int>(min(static_cast<long long>(BN), prm.N - n0));
        const __amdgpu_buffer_rsrc_t ra = make_rsrc(prm.A + m0 * row_bytes, static_cast<uint32_t>(rows_a * row_bytes));
        const __amdgpu_buffer_rsrc_t rb = make_rsrc(prm.B + n0 * row_bytes, static_cast<uint32_t>(rows_b * row_bytes));

        f32x4 acc[WN][WM];
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int j = 0; j < WM; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // Zeroed by an instruction the compiler takes for an ordinary definition,
                    // not by a constant: a constant is set afresh on the path that skips the K
                    // loop (no K steps), in registers of its own choosing, and with all 256
                    // accumulator registers of the large tile taken, bringing the two paths
                    // together before the stores costs a spilled accumulator, whose reload
                    // then waits for every store issued before it.
                    float z;
                    if constexpr (WM * WN == 64) asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(z));
                    else asm volatile("v_mov_b32 %0, 0" : "=v"(z));
                    acc[i][j][e] = z;
                }

        // A_LOADS + B_LOADS asynchronous 16-byte loads per lane fill one stage with
        // a K step; load `idx` of them is issued by fetch_one
        // A load's byte offset into its tile of A (or B) is the lane's share (its row
        // and piece within the rows one wave instruction covers, plus the K step: a
        // vector register, the same for every load of the K step) plus the
        // instruction's first row: a scalar offset that never changes, which the range
        // check of the descriptor takes into account as well. With one wave per SIMD
        // every instruction between two MFMAs counts (a wave issues one instruction in
        // four clocks, an MFMA lasts sixteen): a load comes to two, the LDS target in
        // M0 and the load itself.
        const uint32_t lane_off = static_cast<uint32_t>(row_lo * row_bytes) + piece * 16;
        const uint32_t instr_rows_bytes = static_cast<uint32_t>(kRowsPerInstr * row_bytes);
        struct FetchCtx {
            uint32_t voff;     // lane_off + the K step's bytes, or kPastK if the lane's piece lies past K
            lds_char_ptr_t sa; // the stage's A area in LDS
            lds_char_ptr_t sb; // and its B area
            long long bk_off;  // [K x N] only: byte offset of row k0 of B, and how many
            uint32_t bk_len;   // bytes of B the rows k0 .. k0+63 that exist take
        };
        // (area_a, area_b: byte offsets of the LDS areas that take the K step)
        auto fetch_ctx = [&](int kt, uint32_t area_a, uint32_t area_b) {
            FetchCtx c;
            const int k = kt * BK + piece * 8;  // K < 2^23, K steps run two past it at most
            c.voff = k < static_cast<int>(prm.K) ? lane_off + static_cast<uint32_t>(kt) * (BK * 2) : kPastK;
            c.sa = (lds_char_ptr_t)(lds + area_a);
            c.sb = (lds_char_ptr_t)(lds + area_b);
            const long long k0 = static_cast<long long>(kt) * BK;
            const long long k_left = prm.K - k0;
            const int rows_k = static_cast<int>(k_left < 0 ? 0 : (k_left > BK ? BK : k_left));
            c.bk_off = (k_left > 0 ? k0 : 0) * bkn_row_bytes;
            c.bk_len = static_cast<uint32_t>(rows_k * bkn_row_bytes);
            return c;
        };
        // (not a generic lambda: idx is a constant at every call site and folds
        // after inlining)
        auto fetch_one = [&](const FetchCtx &c, const int idx) {
            if (idx < A_LOADS) {
                const int i = idx;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_ptr_t)(c.sa + (i * NW + wave) * 1024), 16, c.voff,
                                                         instr_rows_bytes * i, 0, 0);
            } else if constexpr (!B_KN) {
                const int i = idx - A_LOADS;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_ptr_t)(c.sb + (i * NW + wave) * 1024), 16, c.voff,
                                                         instr_rows_bytes * i, 0, 0);
            } else {
                // rows k0 .. k0+63 of B through a descriptor of their own: rows past K
                // fall outside it, columns past N are redirected out of range
                const int i = idx - A_LOADS;
                const __amdgpu_buffer_rsrc_t rbk = make_rsrc(prm.B + c.bk_off, c.bk_len);
                const long long n = n0 + bkn_piece * 8;
                const uint32_t off = static_cast<uint32_t>((bkn_row_lo + 4 * NW * i) * bkn_row_bytes + n * 2);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rbk, (lds_ptr_t)(c.sb + (i * NW + wave) * 1024), 16,
                    n < prm.N ? off : kOutOfRange, 0, 0, 0);
            }
        };
        auto stage_ctx = [&](int kt, int stage) {
            return fetch_ctx(kt, static_cast<uint32_t>(stage * kStageBytes),
                             static_cast<uint32_t>(stage * kStageBytes + kStageABytes));
        };
        auto fetch = [&](int kt, int stage) {
            const FetchCtx c = stage_ctx(kt, stage);
            static_for<kLoads>([&](auto i) { fetch_one(c, decltype(i)::value); });
        };
        // LDS read `j` of the kFragReads that make up the fragments of sub-step kk
        auto read_one = [&](F &f, uint32_t base_a, uint32_t base_b, auto kk_tag, auto j_tag) {
            constexpr int kk = decltype(kk_tag)::value;
            constexpr int j = decltype(j_tag)::value;
            if constexpr (j < WM) {
                f.a[j] = lds_read16<kBlockBytes * j>(base_a + fa_addr[kk]);
            } else if constexpr (!B_KN) {
                f.b[j - WM] = lds_read16<kBlockBytes * (j - WM)>(base_b + fb_addr[kk]);
            } else {
                constexpr int i = (j - WM) >> 1;
                constexpr int kRowBytes = 256, kOff = kk * kSubK * kRowBytes;
                if constexpr (((j - WM) & 1) == 0) f.blo[i] = lds_read_tr8<kOff>(base_b + fbkn_addr[i]);
                else f.bhi[i] = lds_read_tr8<kOff + 4 * kRowBytes>(base_b + fbkn_addr[i]);
            }
        };
        auto load_frags = [&](F &f, uint32_t base_a, uint32_t base_b, auto kk_tag) {
            static_for<kFragReads>([&](auto j) { read_one(f, base_a, base_b, kk_tag, j); });
        };
        // One K sub-step: the WN * WM MFMAs on `cur`, and between them the LDS
        // reads of the next sub-step's fragments into `nxt` and n_loads of the
        // global loads of a later K step (loads first_load ... of `fc`), spread
        // evenly over the first load_slots MFMAs: the memory pipes are fed while
        // the matrix core works and nothing is issued in a burst.
        auto sub_step = [&](F &cur, F &nxt, uint32_t nxt_a, uint32_t nxt_b, auto kk_next, const FetchCtx &fc,
                            auto first_load, auto n_loads, auto load_slots, auto &&late) {
            constexpr int kFirst = decltype(first_load)::value;
            constexpr int kHere = decltype(n_loads)::value;
            constexpr int kLoadSlots = decltype(load_slots)::value;
            constexpr int kSlots = WN * WM;
            static_for<kSlots>([&](auto m_tag) {
                constexpr int m = decltype(m_tag)::value;
                constexpr int nb = m / WM, mb = m % WM;
                bf16x8 bfrag;
                if constexpr (B_KN) {
                    const u32x4 t = {cur.blo[nb].x, cur.blo[nb].y, cur.bhi[nb].x, cur.bhi[nb].y};
                    bfrag = __builtin_bit_cast(bf16x8, t);
                } else {
                    bfrag = cur.b[nb];
                }
                acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfrag, cur.a[mb], acc[nb][mb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                // What follows MFMA m: the fragment reads go out during the first
                // half of the sub-step (they are waited for at its end and need the
                // second half to arrive), the global loads over their share of it.
                constexpr int kReadSlots = kSlots / 2;
                static_for<kFragReads>([&](auto t_tag) {
                    constexpr int t = decltype(t_tag)::value;
                    if constexpr (t * kReadSlots / kFragReads == m) read_one(nxt, nxt_a, nxt_b, kk_next, t_tag);
                });
                static_for<(kHere > 0 ? kHere : 1)>([&](auto t_tag) {
                    constexpr int t = decltype(t_tag)::value;
                    // (one wave per SIMD: a load never shares its MFMA with a fragment read)
                    if constexpr (t < kHere && t * kLoadSlots / (kHere > 0 ? kHere : 1) + (kRing ? 1 : 0) == m)
                        fetch_one(fc, kFirst + t);
                });
                if constexpr (m == kSlots * 3 / 4) late();  // bookkeeping for the next K step, out of everybody's way
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        using K0 = std::integral_constant<int, 0>;
        using AllSlots = std::integral_constant<int, WN * WM>;
        using HalfSlots = std::integral_constant<int, WN * WM / 2>;
        auto stage_a = [&](int st) { return static_cast<uint32_t>(st * kStageBytes); };
        auto stage_b = [&](int st) { return static_cast<uint32_t>(st * kStageBytes + kStageABytes); };

        // All waves are done with the previous tile's LDS reads before it is refilled.
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        // At most n of this wave's global loads outstanding, then a workgroup
        // barrier that extends "landed" to the loads of the other waves.
        auto wait_vm = [&](auto n_tag) {
            constexpr int n = decltype(n_tag)::value;
            __builtin_amdgcn_s_waitcnt(((n >> 4) << 14) | 0x0F70 | (n & 15));  // vmcnt(n)
            __builtin_amdgcn_s_barrier();
        };
        // K step kt + 1 has landed once at most the loads of the kStages - 2 later
        // K steps are outstanding (loads past the end are issued too, out of range,
        // so the count is the same in every trip).
        auto wait_landed = [&]() { wait_vm(std::integral_constant<int, (kStages - 2) * kLoads>{}); };

        F f0, f1;
        int stage = 0;
        if constexpr (kRing) {
            // Five slots of 32 KiB, each one operand's share of a K step. K step j keeps A
            // in slot 2j mod 5 and B in the slot after it; while step j is worked on, step
            // j + 1 sits in the next two slots (landed, or landing) and one slot is free:
            // it takes A of step j + 2 during the first sub-step. The barrier before the
            // second sub-step tells that every wave has fetched its last fragments of step
            // j; the slot that held its A then takes B of step j + 2. So one operand's loads
            // go out per sub-step, none in a burst (16 KiB-per-wave bursts after the barrier
            // of a two-stage rotation stalled the issuing waves for ~400 clocks a step).
            constexpr int kSlotBytes = kStageABytes;
            auto slot_off = [&](int sl) { return static_cast<uint32_t>(sl * kSlotBytes); };
            static_for<2>([&](auto st) {
                constexpr int j = decltype(st)::value;
                const FetchCtx c = fetch_ctx(j, slot_off(2 * j), slot_off(2 * j + 1));
                static_for<kLoads>([&](auto i) { fetch_one(c, decltype(i)::value); });
            });
            wait_vm(std::integral_constant<int, kLoads>{});  // K step 0 has landed
            load_frags(f0, slot_off(0), slot_off(1), K0{});
            if constexpr (TRACE) {
                t_prev = now();
                phase[kPhaseFill] += t_prev - t_tile;
            }
            // byte offsets of the slots of this K step's A and B, of the next step's, and of the free one
            uint32_t o_a = slot_off(0), o_b = slot_off(1), o_na = slot_off(2), o_nb = slot_off(3), o_free = slot_off(4);
            FetchCtx fc = fetch_ctx(2, o_free, o_a);
            auto nothing = [] {};
            for (int kt = 0; kt < k_tiles; ++kt) {
                wait_lgkm<0>(f0);
                if constexpr (TRACE) {
                    const unsigned long long t = now();
                    phase[kPhaseSub1] += t - t_prev;  // (of the previous K step; the first one's share is nil)
                    t_prev = t;
                }
                sub_step(f0, f1, o_a, o_b, std::integral_constant<int, 1>{}, fc, std::integral_constant<int, 0>{},
                         std::integral_constant<int, A_LOADS>{}, HalfSlots{}, nothing);
                wait_lgkm<0>(f1);
                // K step kt + 1 has landed when only the A loads just issued are outstanding;
                // after the barrier nobody reads this step's slots any more
                if constexpr (TRACE) {
                    const unsigned long long t0 = now();
                    phase[kPhaseSub0] += t0 - t_prev;
                    __builtin_amdgcn_s_waitcnt(((A_LOADS >> 4) << 14) | 0x0F70 | (A_LOADS & 15));
                    const unsigned long long t1 = now();
                    phase[kPhaseLanded] += t1 - t0;
                    __builtin_amdgcn_s_barrier();
                    t_prev = now();
                    phase[kPhaseBarrier] += t_prev - t1;
                } else {
                    wait_vm(std::integral_constant<int, A_LOADS>{});
                }
                sub_step(f1, f0, o_na, o_nb, K0{}, fc, std::integral_constant<int, A_LOADS>{},
                         std::integral_constant<int, B_LOADS>{}, HalfSlots{}, [&] {
                             // late in the sub-step, when its reads and loads are out: the slots
                             // move on by two, and the next step's loads get their offsets
                             const uint32_t t_a = o_a, t_b = o_b;
                             o_a = o_na;
                             o_b = o_nb;
                             o_na = o_free;
                             o_nb = t_a;
                             o_free = t_b;
                             fc = fetch_ctx(kt + 3, o_free, o_a);
                         });
            }
        } else if constexpr (kSubs > 1) {
            // The loads of K step kt + kStages - 1 go, during all but the last sub-step,
            // into the stage that was read during the previous trip.
            static_for<kStages - 1>([&](auto st) { fetch(decltype(st)::value, decltype(st)::value); });
            wait_landed();
            load_frags(f0, stage_a(0), stage_b(0), K0{});
            for (int kt = 0; kt < k_tiles; ++kt) {
                const int next_stage = stage + 1 >= kStages ? 0 : stage + 1;
                // the stage that was read during the previous trip is free
                const int fetch_stage = stage == 0 ? kStages - 1 : stage - 1;
                const FetchCtx fc = stage_ctx(kt + kStages - 1, fetch_stage);

                // sub-steps alternate between the two fragment sets; the global loads go
                // out during all but the last one
                static_for<kSubs>([&](auto sub_tag) {
                    constexpr int sub = decltype(sub_tag)::value;
                    F &cur = (sub & 1) ? f1 : f0;
                    F &nxt = (sub & 1) ? f0 : f1;
                    wait_lgkm<0>(cur);
                    if constexpr (sub < kSubs - 1) {
                        constexpr int first = sub * kLoads / (kSubs - 1);
                        constexpr int count = (sub + 1) * kLoads / (kSubs - 1) - first;
                        sub_step(cur, nxt, stage_a(stage), stage_b(stage), std::integral_constant<int, sub + 1>{}, fc,
                                 std::integral_constant<int, first>{}, std::integral_constant<int, count>{}, AllSlots{}, [] {});
                    } else {
                        // the last fragments of this stage have arrived: this wave is done
                        // reading it. Has K step kt + 1 landed (for every wave)? After the
                        // barrier every wave is also done reading this stage, so the loads
                        // the next trip issues may overwrite the stage before it.
                        wait_landed();
                        sub_step(cur, nxt, stage_a(next_stage), stage_b(next_stage), K0{}, fc,
                                 std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, AllSlots{}, [] {});
                    }
                });
                stage = next_stage;
            }
        } else {
            // A K step is one MFMA deep: its whole stage is in a fragment set once
            // that set has arrived, so after the barrier below the stage of the
            // CURRENT step is free and takes the loads of K step kt + kStages. Two
            // steps per trip, one per fragment set (a step past an odd end works on
            // zeros: loads past K are out of range and land as zeros).
            static_for<kStages>([&](auto st) { fetch(decltype(st)::value, decltype(st)::value); });
            wait_vm(std::integral_constant<int, (kStages - 1) * kLoads>{});  // K step 0 has landed
            load_frags(f0, stage_a(0), stage_b(0), K0{});
            for (int kt = 0; kt < k_tiles; kt += 2) {
                static_for<2>([&](auto h_tag) {
                    constexpr int h = decltype(h_tag)::value;
                    F &cur = h ? f1 : f0;
                    F &nxt = h ? f0 : f1;
                    const int next_stage = stage + 1 >= kStages ? 0 : stage + 1;
                    const FetchCtx fc = stage_ctx(kt + h + kStages, stage);
                    wait_lgkm<0>(cur);
                    wait_landed();  // K step kt + h + 1 is in LDS, and nobody reads this step's stage any more
                    sub_step(cur, nxt, stage_a(next_stage), stage_b(next_stage), K0{}, fc,
                             std::integral_constant<int, 0>{}, std::integral_constant<int, kLoads>{}, AllSlots{}, [] {});
                    stage = next_stage;
                });
            }
        }
        // The last trip has read the fragments of a K step past the end: they are
        // never used, but the reads are still in flight, and the compiler, which
        // takes an inline ds_read for complete, is free to reuse their destination
        // registers for the store addresses below. Wait for them while both
        // fragment sets are still live.
        wait_lgkm<0>(f0);
        wait_lgkm<0>(f1);
        unsigned long long t_stores = 0;
        if constexpr (TRACE) {
            t_stores = now();
            phase[kPhaseSub1] += t_stores - t_prev;
            phase[kPhaseTiles] += 1;
        }
        // the prefetches past the end are still in flight and target LDS
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

        // Stores. The view of C covers the tile's rows: rows past M are dropped by the range
        // check, which counts the scalar offset (the rows of the store instruction) too.
        const long long c_row_bytes = prm.N * 2;
        const __amdgpu_buffer_rsrc_t rc = make_rsrc(prm.C + m0 * c_row_bytes, static_cast<uint32_t>(rows_a * c_row_bytes));
        // The tile goes out through LDS (idle at this point; the next tile refills it):
        // each wave writes its bf16 results into a region of its own, rows padded by 32
        // bytes, and reads them back as 16-byte pieces, so that a store instruction
        // covers whole rows of the wave's sub-tile (whole 128-byte lines where it is 64
        // columns wide or more) instead of sixteen rows of 32 bytes, with half as many
        // store instructions. And no global store is in flight while the accumulators
        // are read: with all 256 accumulator registers of the 256 x 256 tile taken the
        // register allocator spills one, and a reload in the middle of the stores would
        // wait for all of them.
        constexpr int kRowPitch = kBlk * WN * 2 + 32;
        constexpr int kRegion = kBlk * WM * kRowPitch;
        constexpr int kPieces = kBlk * WN * 2 / 16;          // 16-byte pieces per row of the sub-tile
        constexpr int kRowsPerStore = 64 / kPieces;          // rows one store instruction covers
        static_assert(NW * kRegion <= Cfg::kLdsBytes && 64 % kPieces == 0 && (kBlk * WM) % kRowsPerStore == 0,
                      "the waves' staging regions");
        __builtin_amdgcn_s_barrier();  // every wave has fetched its last fragments: LDS is free
        const uint32_t region = static_cast<uint32_t>(wave * kRegion);
        const uint32_t w_addr = region + l15 * kRowPitch + lgrp * 8;
#pragma unroll
        for (int mb = 0; mb < WM; ++mb) {
#pragma unroll
            for (int nb = 0; nb < WN; ++nb) {
                u32x2 v;
                v.x = pack_bf16x2(acc[nb][mb][0], acc[nb][mb][1]);
                v.y = pack_bf16x2(acc[nb][mb][2], acc[nb][mb][3]);
                *reinterpret_cast<__attribute__((address_space(3))) u32x2 *>(
                    static_cast<uintptr_t>(w_addr + mb * kBlk * kRowPitch + nb * kBlk * 2)) = v;
            }
            __builtin_amdgcn_sched_barrier(0);  // one block row's accumulators at a time
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the region is this wave's own, no barrier
        // piece lane % kPieces of row lane / kPieces + kRowsPerStore * i
        const int piece_c = lane % kPieces, row_c = lane / kPieces;
        const int n = static_cast<int>(n0) + wave_n * (kBlk * WN) + piece_c * 8;  // N < 2^23
        const uint32_t g_off = n < static_cast<int>(prm.N)
                                   ? static_cast<uint32_t>((wave_m * (kBlk * WM) + row_c) * c_row_bytes) + n * 2
                                   : kPastK;
        const uint32_t r_addr = region + row_c * kRowPitch + piece_c * 16;
        const uint32_t store_rows_bytes = static_cast<uint32_t>(kRowsPerStore * c_row_bytes);
#pragma unroll
        for (int i = 0; i < kBlk * WM / kRowsPerStore; ++i) {
            const u32x4 v = *reinterpret_cast<__attribute__((address_space(3))) u32x4 *>(
                static_cast<uintptr_t>(r_addr + i * kRowsPerStore * kRowPitch));
            __builtin_amdgcn_raw_buffer_store_b128(v, rc, g_off, store_rows_bytes * i, 0);
        }
        if constexpr (TRACE) phase[kPhaseStores] += now() - t_stores;
    }
    if constexpr (TRACE) {
        phase[kPhaseTotal] = now() - t_kernel;
        if (lane == 0) {
            unsigned long long *dst = prm.phase_cycles + (static_cast<size_t>(blockIdx.x) * NW + wave) * kGemmPhases;
            for (int i = 0; i < kGemmPhases; ++i) dst[i] = phase[i];
        }
    }
#else
    (void)prm;
#endif
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

tw_status validate_gemm(const tw_gemm_args &g)
{
    if (g.M < 0 || g.N < 0 || g.K < 0) return TW_ERR_SHAPE;
    if (g.b_layout != TW_B_NK && g.b_layout != TW_B_KN) return TW_ERR_SHAPE;
    if (g.M == 0 || g.N == 0) return TW_OK;
    if (!g.C) return TW_ERR_NULL;
    if (g.K > 0 && (!g.A || !g.B)) return TW_ERR_NULL;
    if (g.K % 8 != 0 || g.N % 8 != 0) return TW_ERR_UNSUPPORTED;
    // a tile's rows are addressed with 32-bit byte offsets
    if (g.K > (int64_t(1) << 22) || g.N > (int64_t(1) << 22) || g.M > (int64_t(1) << 40)) return TW_ERR_UNSUPPORTED;
    if (!aligned16(g.A) || !aligned16(g.B) || !aligned16(g.C)) return TW_ERR_ALIGN;
    const uint64_t a_bytes = uint64_t(g.M) * uint64_t(g.K) * 2, b_bytes = uint64_t(g.N) * uint64_t(g.K) * 2;
    const uint64_t c_bytes = uint64_t(g.M) * uint64_t(g.N) * 2;
    if (ranges_overlap(g.C, c_bytes, g.A, a_bytes) || ranges_overlap(g.C, c_bytes, g.B, b_bytes))
        return TW_ERR_ALIAS;
    return TW_OK;
}

template <bool B_KN, int WM, int WN, int STAGES, int BK, bool TRACE = false>
static tw_status launch_cfg(const tw_gemm_args &g, int budget, hipStream_t stream,
                            unsigned long long *phase_cycles = nullptr, int64_t phase_len = 0)
{
    using Cfg = TileCfg<WM, WN, STAGES, BK>;
    constexpr int BN = Cfg::kBN;
    GemmParams prm;
    prm.A = static_cast<const char *>(g.A);
    prm.B = static_cast<const char *>(g.B);
    prm.C = static_cast<char *>(g.C);
    prm.M = g.M;
    prm.N = g.N;
    prm.K = g.K;
    prm.phase_cycles = phase_cycles;
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    if (tiles_m * tiles_n > (int64_t(1) << 30)) return TW_ERR_UNSUPPORTED;
    prm.tiles_m = static_cast<int>(tiles_m);
    prm.tiles_n = static_cast<int>(tiles_n);
    const int64_t total = tiles_m * tiles_n;
    prm.tiles_per_xcd = static_cast<int>((total + kXcds - 1) / kXcds);
    // Block shape of the tile ordering: the tiles an XCD works on at one time (one per
    // compute unit it contributes to the launch) should touch as few distinct rows of A
    // and columns of B as possible, i.e. form a block as square as the tile shape lets
    // them: what they fetch at one K step they fetch once into that XCD's L2. (Sizing the
    // block by the XCD's whole share of the tile list instead made the blocks twice as
    // tall as wide for large products: 6 % slower on a 16K-token layer boundary.)
    const int64_t at_once = (int64_t(budget) + kXcds - 1) / kXcds;
    int best_gm = 1;
    int64_t best_cost = INT64_MAX;
    for (int gm = 1; gm <= 8; gm *= 2) {
        if (gm > tiles_m && gm != 1) break;
        const int64_t gn = (at_once + gm - 1) / gm;
        const int64_t cost = int64_t(gm) * BM + gn * BN;
        if (cost < best_cost) {
            best_cost = cost;
            best_gm = gm;
        }
    }
    prm.group_m = best_gm;

    const int64_t slots = int64_t(prm.tiles_per_xcd) * kXcds;
    const unsigned grid = static_cast<unsigned>(slots < budget ? slots : budget);

    if (TRACE && phase_len < int64_t(grid) * Cfg::kWaves * kGemmPhases) return TW_ERR_SHAPE;
    static std::atomic<int> allowed[kMaxDevices];
    TW_TRY(allow_dynamic_lds(reinterpret_cast<const void *>(gemm_bf16_kernel<B_KN, WM, WN, STAGES, BK, TRACE>),
                             Cfg::kLdsBytes, allowed));
    TW_HIP(launch_kernel(gemm_bf16_kernel<B_KN, WM, WN, STAGES, BK, TRACE>, dim3(grid), dim3(Cfg::kThreads),
                         Cfg::kLdsBytes, stream, prm));
    return TW_OK;
}

// Share of the launch's compute-unit slots that hold a tile when `tiles` tiles
// are dealt to `budget` compute units in whole waves.
static double wave_fill(int64_t tiles, int budget)
{
    const int64_t waves = (tiles + budget - 1) / budget;
    return double(tiles) / double(waves * budget);
}

tw_status launch_gemm(const tw_gemm_args &g, hipStream_t stream, bool beside_other_kernels)
{
    if (g.M == 0 || g.N == 0) return TW_OK;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const int budget = resolve_budget(g.cu_budget, cus);
    // The default: eight waves of 64 x 64, tile 256 x 128 x 64, three LDS stages.
    // The part runs this kernel at its power limit (1.2-1.9 GHz on N(0, 0.02^2)
    // operands against 2.4 GHz idle), so what a tile shape is worth is decided by
    // the energy it spends per flop, not by its share of busy matrix-core cycles.
    if (g.b_layout == TW_B_KN) return launch_cfg<true, 4, 4, 3, 64>(g, budget, stream);
    const int64_t tiles_m = (g.M + BM - 1) / BM;
    const int64_t wide_tiles = tiles_m * ((g.N + kGemmTileN - 1) / kGemmTileN);
    if (!beside_other_kernels) {
        // A product whose 256 x 128 tiles fill at most half of the compute units it may
        // use is cut into 256 x 64 tiles instead (eight waves of 64 x 32, 3 x 40 KiB of
        // LDS): twice the workgroups, each with half the work. A tile of that shape
        // fetches 5/3 of the operand bytes per flop and takes ~0.77 of the wide tile's
        // time, so it only pays while it brings idle compute units in: 14-23 % faster
        // on 40 ... 128 wide tiles, 25-40 % slower once the wide tiles already fill
        // more than half.
        if (2 * wide_tiles <= budget) return launch_cfg<false, 4, 2, 3, 64>(g, budget, stream);
        // A large product takes 256 x 256 tiles: four waves of 128 x 128 (all 512
        // registers of a lane: 256 accumulators and two fragment sets), K steps of
        // 64 over two LDS stages of 64 KiB. Two thirds of the operand bytes fetched
        // per flop and half the LDS reads. (K steps of 32 over four stages of 32 KiB
        // fit the same LDS and give the loads twice as long to land, but fetch every
        // 128-byte line of A and B in two halves a K step apart, by which time the
        // line has left the L1: twice the L2 requests, and 27 % more cycles.)
        const int64_t big_tiles = tiles_m * ((g.N + 255) / 256);
        if (wave_fill(big_tiles, budget) >= wave_fill(wide_tiles, budget) - 0.05)
            return launch_cfg<false, 8, 8, 2, 64>(g, budget, stream);
    }
    // Next to other kernels (tw_overlap_launch, the split schedules of
    // tw_weave_layer) the 256 x 128 tiles are kept: the compute units are not idle
    // there, the narrow tiles' extra operand traffic competes for the same L1
    // request slots (a woven layer measured level to 3 % slower with them), and
    // the 256 x 256 tiles leave no registers for a co-resident workgroup.
    return launch_cfg<false, 4, 4, 3, 64>(g, budget, stream);
}

}  // namespace tw

using namespace tw;

extern "C" tw_status tw_gemm_bf16_traced(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                                         unsigned long long *phase_cycles, int64_t phase_len, void *stream)
{
    const tw_gemm_args g = {A, B, C, M, N, K, TW_B_NK, 0};
    TW_TRY(validate_gemm(g));
    if (!phase_cycles) return TW_ERR_NULL;
    if (g.M == 0 || g.N == 0) return TW_ERR_UNSUPPORTED;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    // only a product that takes the 256 x 256 tiles on the whole device is traced
    const int64_t tiles_m = (g.M + BM - 1) / BM;
    const int64_t wide_tiles = tiles_m * ((g.N + kGemmTileN - 1) / kGemmTileN), big_tiles = tiles_m * ((g.N + 255) / 256);
    if (2 * wide_tiles <= cus || wave_fill(big_tiles, cus) < wave_fill(wide_tiles, cus) - 0.05) return TW_ERR_UNSUPPORTED;
    return launch_cfg<false, 8, 8, 2, 64, true>(g, cus, static_cast<hipStream_t>(stream), phase_cycles, phase_len);
}

extern "C" tw_status tw_gemm_bf16(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                                  int b_layout, int cu_budget, void *stream)
{
    const tw_gemm_args g = {A, B, C, M, N, K, b_layout, cu_budget};
    TW_TRY(validate_gemm(g));
    return launch_gemm(g, static_cast<hipStream_t>(stream));
}
