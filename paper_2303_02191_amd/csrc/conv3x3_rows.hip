// 3x3 stride-1 pattern-sparse convolution for large layers: the pipelined kernel on the sparse
// matrix instruction (operand layouts, fragment format and the corner / edge / centre split of the
// taps: see conv3x3_sparse.hip and sparse_frag.h).
//
// Shape of the work.  A workgroup (4 waves) owns 128 output channels x a strip of 16 output columns x
// 4*TN output rows; wave v owns the TN rows [v*TN, v*TN + TN) of the strip, all 128 channels.  The 16
// columns of a matrix instruction are 16 CONSECUTIVE positions of one output row.  That makes the B
// operands (activations) of the nine taps overlapping windows of the same LDS rows: with
//     R[i][kw] = the 16-byte read (8 channels) of input row i of the wave at column shift kw,
// output row j takes tap (kh, kw) from R[j + kh][kw].  A wave reads the 3 * (TN + 2) vectors R once per
// stage and every one serves up to three output rows and three taps, instead of nine reads per output
// row: the LDS read traffic of the activations drops by half (TN = 5: 21 reads instead of 45), and each
// read is 1024 contiguous bytes, free of bank conflicts at any row pitch.
//
// K runs over stages of 32 input channels, double-buffered in LDS: the stage's weight fragments (one
// contiguous chunk of the packed blob) and its activation tile with halo are copied global -> LDS
// without passing through registers while the previous stage is multiplied.  A stage is 5 phases
// (centre, corner step 0/1, edge step 0/1) x 4 pairs of channel tiles = 20 units of 2*TN matrix
// instructions.  The centre phase multiplies R[j+1][1] as it is; the sparse phases need, per lane,
// 4 channels x the 4 taps of a group, i.e. 4x4 (tap x channel) transposes of four R vectors, done with
// byte permutes behind the matrix instructions of earlier units.
//
// Workgroups are persistent, one per compute unit.  Rows of a strip are cut into tall tiles (TN = 5:
// 20 rows) and short ones (TN = 4: 16 rows); the host picks the cut per strip so that every workgroup's
// share of tiles takes about the same time (see plan_rows below): a workgroup runs its tall tiles, then
// its short ones.
#include <algorithm>
#include <map>
#include <mutex>
#include <tuple>
#include <type_traits>

#include "common.h"
#include "dtypes.h"
#include "epilogue.h"
#include "mma.h"
#include "rows_plan.h"
#include "sparse_frag.h"

namespace rtoss {

namespace {

// Which unit of a stage reads and permutes what (TN = rows per wave).
//   prologue (issued inside the previous stage's last unit): R[1..TN][1], R[0..3][0], R[0..3][2]
//   unit u <= TN-3: R[u+4][0], R[u+4][2];   unit TN-2: R[0][1], R[TN+1][1]
//   corner job j (taps 0,2,6,8 of output row j: R[j][0], R[j][2], R[j+2][0], R[j+2][2]) is permuted in unit
//   max(0, j-1), the unit after its last read; edge job j (taps 1,3,5,7: R[j][1], R[j+1][0], R[j+1][2],
//   R[j+2][1]) in unit TN-1+j.  Corner operands are complete before unit 4, edge operands before unit 12.
template <int TN> struct RowSchedule {
    static_assert(TN >= 3 && TN <= 5, "corner jobs must be permuted within the centre phase");
    static constexpr int jobs = 2 * TN;  // job q < TN: corner taps of row q; job TN + j: edge taps of row j
    static constexpr int perm_unit(int q) { return q < TN ? (q < 2 ? 0 : q - 1) : TN - 1 + (q - TN); }
    static constexpr int perm_count(int u)
    {
        int n = 0;
        for (int q = 0; q < jobs; ++q) n += perm_unit(q) == u;
        return n;
    }
    static constexpr int perm_first(int u)
    {
        for (int q = 0; q < jobs; ++q)
            if (perm_unit(q) == u) return q;
        return 0;
    }
    // row whose shifted columns 0 and 2 are read in unit u (-1: none)
    static constexpr int side_row(int u) { return u <= TN - 3 ? u + 4 : -1; }
    static constexpr bool reads_outer_mid(int u) { return u == TN - 2; }
};

// (input row, column shift) of tap slot f of a job
template <int TN> struct JobTap {
    static constexpr int row(int q, int f)
    {
        return q < TN ? q + (f >> 1) * 2                               // corners: rows j, j, j+2, j+2
                      : (q - TN) + (f == 0 ? 0 : f == 3 ? 2 : 1);      // edges: rows j, j+1, j+1, j+2
    }
    static constexpr int shift(int q, int f)
    {
        return q < TN ? (f & 1) * 2                                    // corners: columns 0, 2, 0, 2
                      : (f == 1 ? 0 : f == 2 ? 2 : 1);                 // edges: columns 1, 0, 2, 1
    }
};

// FUSED: scale / bias / SiLU / residual in the epilogue.  The plain instantiation (ReLU or nothing) keeps
// its branch-free epilogue; the fused one pays for generality with a few uniform branches per tile.
template <typename T, typename TO, bool FUSED>
__global__ __launch_bounds__(256, 1) void conv3x3_rows_kernel(const T* __restrict__ x, TO* __restrict__ y,
                                                              const char* __restrict__ wfrag,
                                                              const char* __restrict__ zeros, int H, int W, int Ci,
                                                              int Co, int m_tiles_total, RowPlan plan, Epilogue ep)
{
    constexpr int TM = kRowsTM;
    constexpr int A_BYTES = TM * kTileBytes;
    constexpr int A_WAVE_COPIES = A_BYTES / 1024;  // 64 lanes x 16 B per copy instruction
    constexpr int A_PER_WAVE = A_WAVE_COPIES / 4;
    static_assert(A_WAVE_COPIES % 4 == 0, "every wave issues the same number of weight copies");
    constexpr int X_CHUNKS = (4 * kTall + 2) * kLW * 4;  // 16-byte chunks of the tall tile's activation tile
    constexpr int X_WAVE_COPIES = (X_CHUNKS + 63) / 64;
    constexpr int X_PER_WAVE = (X_WAVE_COPIES + 3) / 4;
    constexpr int X_AREA = X_PER_WAVE * 4 * 1024;  // what the copy instructions cover
    constexpr int REGION = A_BYTES + X_AREA;       // one pipeline buffer: [weights][activations]
    constexpr int COPY_SLOTS = A_PER_WAVE + X_PER_WAVE;
    static_assert(COPY_SLOTS <= 20, "two copies per unit in the first ten units of a stage");
    extern __shared__ __attribute__((aligned(16))) char smem[];  // two regions

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int stages = Ci / 32;
    const int Ho = H, Wo = W;  // stride 1, padding 1
    const int64_t a_stage_stride = (int64_t)m_tiles_total * kTileBytes;

    // ---- this workgroup's entries: tall tiles first, then short ones.  Within an XCD the tall list is
    // dealt to the slots in ascending order and the short list in descending order, so that the slots
    // that get one tall tile fewer are the first to get a short one. ----
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const int tall_end = min((xcd + 1) * plan.tall_per_xcd, plan.tall_total);
    const int short_end = min((xcd + 1) * plan.short_per_xcd, plan.short_total);
    int tall_next = xcd * plan.tall_per_xcd + slot;
    int short_next = xcd * plan.short_per_xcd + (slots - 1 - slot);
    if (tall_next >= tall_end && short_next >= short_end) return;

    // ---- copy state: the tile whose stages are being fetched (runs ahead of the tile being multiplied
    // by one stage at tile boundaries).  Every lane copies 16 bytes in every copy instruction, so the copy
    // code has no branches: a lane whose LDS slot is zero padding of the tile reads from a block of zeros
    // that the packer appended to the weight fragments (2*Ci + 16 bytes, so that the per-stage advance of
    // 64 bytes stays inside it). ----
    int c_mt0 = 0;
    const char* x_ptr[X_PER_WAVE];  // per lane and copy slot: source address for stage 0
    // A lane's source of activation copy slot k for tile t, worked out in four parts (position in the tile;
    // image coordinates and chunk number; address; zero padding).  The first tile does them in one go; after
    // that the last stage of a tile spreads the parts of the next tile's sources over its matrix instructions
    // (as one block in front of a stage they cost ~1.3 k cycles with nothing to overlap them).  The empty asm
    // statements pin each part's results where it is written: they are ordered with the matrix instructions.
    int sp_a = 0, sp_b = 0, sp_off = 0;
    const char* sp_addr = nullptr;
    auto source_part = [&](auto K, auto P, const TileCoord& t, int in_rows) {
        constexpr int k = decltype(K)::value, part = decltype(P)::value;
        if constexpr (part == 0) {
            int l = lane;
            asm volatile("" : "+v"(l));  // recomputed here rather than kept in registers through the K loop
            const int pos = (k * 4 + wave) * 16 + (l >> 2);
            sp_a = pos / kLW;
            sp_b = pos - sp_a * kLW;
            asm volatile("" : "+v"(sp_a), "+v"(sp_b));
        } else if constexpr (part == 1) {
            sp_a += t.oh0 - 1;  // input row and column
            sp_b += t.ow0 - 1;
            // offset in 16-byte chunks: fits 31 bits (checked by the launcher)
            sp_off = ((t.n_img * H + sp_a) * W + sp_b) * (Ci >> 3) + (lane & 3);
            asm volatile("" : "+v"(sp_a), "+v"(sp_b), "+v"(sp_off));
        } else if constexpr (part == 2) {
            sp_addr = (const char*)x + (int64_t)sp_off * 16;
            asm volatile("" : "+v"(sp_addr));
        } else {
            const int row_end = min(H, t.oh0 - 1 + in_rows);  // rows of the tile, and of the image
            const bool inside = (unsigned)sp_a < (unsigned)row_end && (unsigned)sp_b < (unsigned)W;
            x_ptr[k] = inside ? sp_addr : zeros;
            asm volatile("" : "+v"(x_ptr[k]));
        }
    };
    auto setup_tile_sources = [&](const TileCoord& t, int in_rows) {
        c_mt0 = t.mt0;
        static_for<X_PER_WAVE>([&](auto K) {
            static_for<4>([&](auto P) { source_part(K, P, t, in_rows); });
        });
    };
    // One copy instruction (64 lanes x 16 bytes) of stage `stage` of the copy state's tile into region
    // `par`: slots 0 .. A_PER_WAVE-1 move weight fragments, the rest move activations.
    auto issue_copy_slot = [&](int cslot, int stage, int par) {
        char* region = smem + par * REGION;
        if (cslot < A_PER_WAVE) {
            const int kk = cslot * 4 + wave;
            const char* asrc = wfrag + (int64_t)c_mt0 * kTileBytes + lane * 16 + stage * a_stage_stride;
            copy16_to_lds(asrc + kk * 1024, region + kk * 1024);
        } else {
            const int k = cslot - A_PER_WAVE;
            const int kk = k * 4 + wave;
            // (the last copy instructions reach past the activation tile into the slack of X_AREA)
            copy16_to_lds(x_ptr[k] + stage * 64, region + A_BYTES + kk * 1024);
        }
    };

    const int nn = lane & 15, qq = lane >> 4;

    f32x4 acc[TM][kTall];
    // Operand registers that cross stage boundaries: what a stage needs before its first matrix
    // instruction is read from inside the previous stage's last unit.
    u32x4 R[kTall + 2][3];
    u32x4 a_nxt[2];
    int gpar = 0;  // region that holds the stage about to be multiplied

    // byte offset in the activation tile of a lane's column (shift 0) of its wave's first input row, for a
    // tile of tn rows per wave
    auto lane_x_offset = [&](int tn) { return ((wave * tn) * kLW + nn) * kPosBytes + qq * 16; };
    // The reads a stage needs before its first matrix instruction: centre-tap operands of its rows, weight
    // fragments of unit 0, side columns of rows 0..3 (corner jobs 0 and 1).  xoff: lane_x_offset of the tile
    // the stage belongs to.  (Rows are read for a tall tile; a short tile has one fewer, and the extra row is
    // inside its activation tile too.)
    auto load_stage_prologue = [&](int par, int xoff) {
        const char* A = smem + par * REGION + lane * 16;
        const char* X = smem + par * REGION + A_BYTES + xoff;
#pragma unroll
        for (int j = 1; j <= kTall; ++j) R[j][1] = *(const u32x4*)(X + (j * kLW + 1) * kPosBytes);
        a_nxt[0] = *(const u32x4*)(A + 4 * kFragBytes);
        a_nxt[1] = *(const u32x4*)(A + kTileBytes + 4 * kFragBytes);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            R[i][0] = *(const u32x4*)(X + (i * kLW + 0) * kPosBytes);
            R[i][2] = *(const u32x4*)(X + (i * kLW + 2) * kPosBytes);
        }
    };

    // ---- one tile of TN rows per wave ----
    auto run_tile = [&](auto tn_tag, const TileCoord& cur, bool has_next, const TileCoord& nxt, bool nxt_tall) {
        constexpr int TN = decltype(tn_tag)::value;
        using Sched = RowSchedule<TN>;
        using Tap = JobTap<TN>;
        constexpr int UNIT = 2 * TN;  // matrix instructions per unit
        const int xrd = lane_x_offset(TN);
        const int nxt_in_rows = nxt_tall ? 4 * kTall + 2 : 4 * kShort + 2;
        auto read_R = [&](const char* X, int i, int kw) {
            R[i][kw] = *(const u32x4*)(X + xrd + (i * kLW + kw) * kPosBytes);
        };

        // The first reads of the tile's first stage.  (Its data landed, and the workgroup met, inside the previous
        // tile's last stage.  That stage also issued reads for "its next stage", but nothing except the stage loop
        // may lie between such reads and their use: across the epilogue the register allocator would park the
        // values and bring them back right in front of the first matrix instructions -- too late for them, see
        // mma.h.  So a tile starts with reads of its own.)
        load_stage_prologue(gpar, xrd);

        auto run_stage = [&](auto first_tag, auto last_tag, int stage) {
            constexpr bool FIRST = decltype(first_tag)::value, LAST = decltype(last_tag)::value;
            // the stage copied while this one is multiplied: the tile's next stage, or the next tile's first
            // (in the very last stage of the last tile there is nothing left to fetch; `nxt` is the same
            // tile then and its stage 0 is fetched again into the free region, which keeps this code free of
            // branches).  The last stage works out the next tile's activation sources as it goes: slot k in
            // unit k, before the unit (>= 5) that issues the slot's copy.
            const int copy_stage = LAST ? 0 : stage + 1;
            if constexpr (LAST) c_mt0 = nxt.mt0;
            const char* A = smem + gpar * REGION + lane * 16;
            const char* AI = smem + gpar * REGION + 5 * kFragBytes + lane * 4;
            const char* X = smem + gpar * REGION + A_BYTES;

            // output o (0..15) of a job: dword o%8 of step o/8; element 4*c + f of a step's B operand =
            // channel c (of this lane's 4 in that step), tap slot f
            auto transposed = [&](auto Q, int o) -> uint32_t {
                constexpr int q = decltype(Q)::value;
                const int d = o & 7, comp = (o >> 3) * 2 + (d >> 2);
                const uint32_t sel = (d & 2) ? 0x07060302u : 0x05040100u;
                return (d & 1) ? __builtin_amdgcn_perm(R[Tap::row(q, 3)][Tap::shift(q, 3)][comp],
                                                       R[Tap::row(q, 2)][Tap::shift(q, 2)][comp], sel)
                               : __builtin_amdgcn_perm(R[Tap::row(q, 1)][Tap::shift(q, 1)][comp],
                                                       R[Tap::row(q, 0)][Tap::shift(q, 0)][comp], sel);
            };
            u32x8 bfc[2][TN], bfe[2][TN];  // B operands of the sparse phases
            u32x4 a_cur[2] = {a_nxt[0], a_nxt[1]};
            int i_cur[2] = {0, 0}, i_nxt[2] = {0, 0};
            static_for<20>([&](auto U) {
                constexpr int u = decltype(U)::value;
                constexpr int phase = u / 4, m0 = (u % 4) * 2;
                constexpr int perm_first = Sched::perm_first(u), perm_count = Sched::perm_count(u);
                static_for<UNIT>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    constexpr int mi = i / TN, j = i % TN, m = m0 + mi;
                    if constexpr (phase == 0) {
                        if constexpr (FIRST) Mat<T>::dense_first(a_cur[mi], R[j + 1][1], acc[m][j]);
                        else Mat<T>::dense(a_cur[mi], R[j + 1][1], acc[m][j]);
                    }
                    if constexpr (phase == 1) Mat<T>::template sparse<0>(a_cur[mi], bfc[0][j], acc[m][j], i_cur[mi]);
                    if constexpr (phase == 2) Mat<T>::template sparse<1>(a_cur[mi], bfc[1][j], acc[m][j], i_cur[mi]);
                    if constexpr (phase == 3) Mat<T>::template sparse<0>(a_cur[mi], bfe[0][j], acc[m][j], i_cur[mi]);
                    if constexpr (phase == 4) Mat<T>::template sparse<1>(a_cur[mi], bfe[1][j], acc[m][j], i_cur[mi]);
                    if constexpr (LAST && u < X_PER_WAVE) {
                        constexpr int part = i == 1 ? 0 : i == 3 ? 1 : i == 4 ? 2 : i == 5 ? 3 : -1;
                        if constexpr (part >= 0)
                            source_part(std::integral_constant<int, u>{}, std::integral_constant<int, part>{}, nxt, nxt_in_rows);
                    }
                    if constexpr (i == 2 && 2 * u < COPY_SLOTS) issue_copy_slot(2 * u, copy_stage, gpar ^ 1);
                    if constexpr (i == 2 + TN && 2 * u + 1 < COPY_SLOTS) issue_copy_slot(2 * u + 1, copy_stage, gpar ^ 1);
                    if constexpr (i == 0) {  // issue the next unit's LDS reads behind the first matrix instruction
                        if constexpr (u + 1 < 20) {
                            constexpr int np = (u + 1) / 4, nm0 = ((u + 1) % 4) * 2;
                            constexpr int nstep = np == 0 ? 4 : np - 1;
#pragma unroll
                            for (int t = 0; t < 2; ++t) {
                                a_nxt[t] = *(const u32x4*)(A + (nm0 + t) * kTileBytes + nstep * kFragBytes);
                                if constexpr (np > 0) i_nxt[t] = *(const int*)(AI + (nm0 + t) * kTileBytes + ((np - 1) >> 1) * 256);
                            }
                        }
                        if constexpr (Sched::side_row(u) >= 0) {
                            read_R(X, Sched::side_row(u), 0);
                            read_R(X, Sched::side_row(u), 2);
                        }
                        if constexpr (Sched::reads_outer_mid(u)) {
                            read_R(X, 0, 1);
                            read_R(X, TN + 1, 1);
                        }
                        if constexpr (u == 19) {
                            // Stage hand-over without a bubble: all copies of the next stage were issued in
                            // this stage's first ten units and this unit's operands were read in unit 18; the
                            // wave waits for its copies and its reads, meets the others at a bare barrier (the
                            // next stage's data is now complete and nobody reads this stage's region any more)
                            // and issues the next stage's first reads, which complete under the rest of this unit.
                            asm volatile("" ::: "memory");
                            __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): copies landed, reads of this region done
                            __builtin_amdgcn_s_barrier();
                            asm volatile("" ::: "memory");
                            load_stage_prologue(gpar ^ 1, xrd);
                        }
                    }
                    // this instruction's share of the unit's 16 * perm_count permutes
                    constexpr int o_begin = i * 16 * perm_count / UNIT, o_end = (i + 1) * 16 * perm_count / UNIT;
                    static_for<o_end - o_begin>([&](auto O) {
                        constexpr int o = o_begin + decltype(O)::value;
                        constexpr int q = perm_first + o / 16, oo = o % 16;
                        const uint32_t v = transposed(std::integral_constant<int, q>{}, oo);
                        if constexpr (q < TN) bfc[oo >> 3][q][oo & 7] = v;
                        else bfe[oo >> 3][q - TN][oo & 7] = v;
                    });
                    __builtin_amdgcn_sched_barrier(0);
                });
                if constexpr (u + 1 < 20) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        a_cur[t] = a_nxt[t];
                        i_cur[t] = i_nxt[t];
                    }
                }
            });
            gpar = __builtin_amdgcn_readfirstlane(gpar ^ 1);  // (kept scalar: it feeds the LDS address of every copy)
        };
        run_stage(std::true_type{}, std::false_type{}, 0);  // (the launcher admits Ci >= 96: three stages or more)
        for (int stage = 1; stage + 1 < stages; ++stage) run_stage(std::false_type{}, std::false_type{}, stage);
        run_stage(std::false_type{}, std::true_type{}, stages - 1);

        // the last matrix instructions must have written their accumulators before anything reads them
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        // ---- epilogue ----
        // Per lane and group of 4 channel tiles the accumulators hold 16 consecutive output channels of one
        // position (tile_row_channel): column nn of row j of the wave.  16-bit outputs without a fused output
        // stage are stored directly: 32 contiguous bytes per lane.  Otherwise each wave transposes its
        // 16*TN positions x 16*TM channels through its own slice of the region that was multiplied last
        // (free now; the other region is receiving the next tile's first stage) and writes whole
        // channel rows, 16 bytes per lane; fp32 output goes in two halves of the channel tiles.
        {
            constexpr int EB = (int)sizeof(TO);
            constexpr int HALVES = EB == 4 ? 2 : 1;
            constexpr int TMH = TM / HALVES;
            static_assert(TM % HALVES == 0 && TMH % 4 == 0, "each half is whole groups of 4 channel tiles (tile_row_channel)");
            constexpr int ROW = TMH * 16 * EB + (EB == 2 ? 8 : 16);  // padded row pitch: spreads the banks
            // output rows staged together: as many as fit when the four waves share one region
            constexpr int JG = (REGION / (4 * 16 * ROW)) < TN ? (REGION / (4 * 16 * ROW)) : TN;
            static_assert(JG >= 1, "epilogue staging must fit in one region");
            char* stage_out = smem + (gpar ^ 1) * REGION + wave * (16 * JG * ROW);
            // lane-derived addresses of the epilogue are recomputed per tile (opaque copy of the lane id)
            // instead of staying live in registers through the K loop
            int lane_e = lane;
            asm volatile("" : "+v"(lane_e));
            const int nn_e = lane_e & 15, qq_e = lane_e >> 4;
            const int row_first = cur.oh0 + wave * TN;  // first output row of the wave
            // 64-bit address of the tile's first output element once; everything else is 32-bit
            const int64_t pos_tile = ((int64_t)cur.n_img * Ho + cur.oh0) * Wo + cur.ow0;  // position number
            TO* const y_tile = y + pos_tile * ep.ldy;
            const float relu_floor = ep.act == 1 ? 0.f : -__builtin_inff();
            if constexpr (kDirectEpilogue && EB == 2 && !FUSED) {
                const bool col_inside = cur.ow0 + nn_e < Wo;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const bool inside = col_inside && row_first + j < Ho;
                    TO* yp = y_tile + ((wave * TN + j) * Wo + nn_e) * ep.ldy + 16 * cur.mt0 + 16 * qq_e;
#pragma unroll
                    for (int mg = 0; mg < TM; mg += 4) {
                        uint32_t o[8];
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            float r[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) asm("v_max_f32 %0, %1, %2" : "=v"(r[e]) : "v"(acc[mg + m][j][e]), "v"(relu_floor));
                            o[2 * m] = pack2_from_f32<TO>(r[0], r[1]);
                            o[2 * m + 1] = pack2_from_f32<TO>(r[2], r[3]);
                        }
                        if (inside && 16 * (cur.mt0 + mg) + 16 * qq_e < Co) {
                            *(u32x4*)(yp + 16 * mg) = u32x4{o[0], o[1], o[2], o[3]};
                            *(u32x4*)(yp + 16 * mg + 8) = u32x4{o[4], o[5], o[6], o[7]};
                        }
                    }
                }
            } else {
#pragma unroll
                for (int h = 0; h < HALVES; ++h) {
#pragma unroll
                    for (int j0 = 0; j0 < TN; j0 += JG) {
                        const int jn = j0 + JG <= TN ? JG : TN - j0;  // rows in this group
#pragma unroll
                        for (int jj = 0; jj < jn; ++jj) {
                            const int j = j0 + jj;
                            f32x4 vals[TMH];
#pragma unroll
                            for (int mm = 0; mm < TMH; ++mm) vals[mm] = acc[h * TMH + mm][j];
                            if constexpr (FUSED) {
                                // this lane's position in row j and its 4 consecutive channels of every channel tile
                                const int dr_f = wave * TN + j;
                                const bool inside_f = cur.oh0 + dr_f < Ho && cur.ow0 + nn_e < Wo;
                                const int64_t pos_f = pos_tile + dr_f * Wo + nn_e;
#pragma unroll
                                for (int mm = 0; mm < TMH; ++mm) {
                                    const int co4 = 16 * (cur.mt0 + h * TMH) + tile_quarter_offset(mm, qq_e);
                                    if (inside_f && co4 < Co) {
                                        float vv[4] = {vals[mm].x, vals[mm].y, vals[mm].z, vals[mm].w};
                                        epi_scale_bias_act<4>(vv, ep, co4);
                                        epi_residual<TO, 4>(vv, ep, pos_f, co4);
                                        vals[mm] = f32x4{vv[0], vv[1], vv[2], vv[3]};
                                    }
                                }
                            } else {
                                // fused ReLU without a branch: max with 0, or with -inf when ReLU is off (one v_max_f32
                                // per value, written as asm so that no NaN-quieting pass is put in front of it)
#pragma unroll
                                for (int mm = 0; mm < TMH; ++mm)
#pragma unroll
                                    for (int e = 0; e < 4; ++e) {
                                        float r;
                                        asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(vals[mm][e]), "v"(relu_floor));
                                        vals[mm][e] = r;
                                    }
                            }
#pragma unroll
                            for (int mm = 0; mm < TMH; ++mm) {
                                char* dst = stage_out + (jj * 16 + nn_e) * ROW + tile_quarter_offset(mm, qq_e) * EB;
                                if constexpr (EB == 4) {
                                    *(f32x4*)dst = vals[mm];
                                } else {
                                    uint2 o;
                                    o.x = pack2_from_f32<TO>(vals[mm].x, vals[mm].y);
                                    o.y = pack2_from_f32<TO>(vals[mm].z, vals[mm].w);
                                    *(uint2*)dst = o;
                                }
                            }
                        }
                        // read back: a row of 16*TMH channels is CH 16-byte chunks; 64 lanes cover 64/CH positions
                        // per pass.  (A wave's LDS accesses execute in order, so the next group's writes to this
                        // slice cannot pass these reads.)
                        constexpr int CH = TMH * 16 * EB / 16;
                        static_assert(64 % CH == 0, "row chunks must tile the wave");
                        constexpr int POS_PER_PASS = 64 / CH;
                        const int passes = (16 * jn) / POS_PER_PASS;
                        const int co_first = 16 * (cur.mt0 + h * TMH);
                        const int sub = lane_e / CH, chunk = lane_e % CH;  // position within the pass, chunk within the row
                        const int co = co_first + chunk * (16 / EB);
#pragma unroll
                        for (int ps = 0; ps < passes; ++ps) {
                            const int p = ps * POS_PER_PASS + sub;
                            const int dr = wave * TN + j0 + (p >> 4), dc = p & 15;
                            const u32x4 v = *(const u32x4*)(stage_out + p * ROW + chunk * 16);
                            if (cur.oh0 + dr < Ho && cur.ow0 + dc < Wo && co < Co)  // Co is a multiple of 16: a chunk is all in or all out
                                *(u32x4*)(y_tile + (dr * Wo + dc) * ep.ldy + co) = v;
                        }
                    }
                }
            }
        }
        // staging slices are read (LDS only): the region may be overwritten by the next copies.  A bare
        // barrier, because __syncthreads() carries a fence that would wait here for this tile's output
        // stores to drain; they drain behind the next tile's first stage instead.  (The direct epilogue
        // does not touch LDS: nothing to wait for.)
        if constexpr (!(kDirectEpilogue && sizeof(TO) == 2 && !FUSED)) {
            if (has_next) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) only
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
        }
    };

    // ---- walk the entries ----
    bool cur_tall = tall_next < tall_end;
    TileCoord cur = decode_entry(plan, cur_tall, cur_tall ? tall_next : short_next);
    if (cur_tall) tall_next += slots;
    else short_next += slots;
    // (the weight copies need only the tile's channel block: they are under way while the lanes work out
    // their activation sources, ~3 k cycles of address arithmetic)
    c_mt0 = cur.mt0;
#pragma unroll
    for (int s = 0; s < A_PER_WAVE; ++s) issue_copy_slot(s, 0, 0);
    setup_tile_sources(cur, cur_tall ? 4 * kTall + 2 : 4 * kShort + 2);
#pragma unroll
    for (int s = A_PER_WAVE; s < COPY_SLOTS; ++s) issue_copy_slot(s, 0, 0);
    bool first_tile = true;
    for (;;) {
        const bool nxt_tall = tall_next < tall_end;
        const bool has_next = nxt_tall || short_next < short_end;
        TileCoord nxt = cur;
        if (has_next) {
            nxt = decode_entry(plan, nxt_tall, nxt_tall ? tall_next : short_next);
            if (nxt_tall) tall_next += slots;
            else short_next += slots;
        }
        if (first_tile) {
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's copies have landed in LDS
            __syncthreads();                     // ... and everybody's
            first_tile = false;
        }
        if (cur_tall) run_tile(std::integral_constant<int, kTall>{}, cur, has_next, nxt, nxt_tall);
        else run_tile(std::integral_constant<int, kShort>{}, cur, has_next, nxt, nxt_tall);
        if (!has_next) break;
        cur = nxt;
        cur_tall = nxt_tall;
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------------------------
// Host: cutting the rows into tiles.
// ---------------------------------------------------------------------------------------------------------
// Relative cost of one tile of TN rows per wave over `stages` stages: a stage costs a fixed part (weight
// operand reads, hand-over) plus a part per row; the epilogue and the prologue of a tile scale with its
// rows.  (Fitted to per-workgroup time stamps of both tile classes on a 256 -> 256 channel layer.)
namespace {

inline double tile_cost(int tn, int stages) { return stages * (tn + 0.7) + 1.5 * tn; }

struct PlanKey {
    int N, H, W, co_blocks, stages, slots;
    bool operator<(const PlanKey& o) const
    {
        return std::tie(N, H, W, co_blocks, stages, slots) < std::tie(o.N, o.H, o.W, o.co_blocks, o.stages, o.slots);
    }
};

// The busiest workgroup's cost under a plan, by the kernel's own dealing rule.
double plan_makespan(const RowPlan& p, int slots, int stages)
{
    const double c5 = tile_cost(kTall, stages), c4 = tile_cost(kShort, stages);
    double worst = 0;
    for (int xcd = 0; xcd < 8; ++xcd) {
        const int nt = std::max(0, std::min((xcd + 1) * p.tall_per_xcd, p.tall_total) - xcd * p.tall_per_xcd);
        const int ns = std::max(0, std::min((xcd + 1) * p.short_per_xcd, p.short_total) - xcd * p.short_per_xcd);
        for (int s = 0; s < slots; ++s) {
            const int mine_t = nt > s ? (nt - s + slots - 1) / slots : 0;
            const int rs = slots - 1 - s;
            const int mine_s = ns > rs ? (ns - rs + slots - 1) / slots : 0;
            worst = std::max(worst, mine_t * c5 + mine_s * c4);
        }
    }
    return worst;
}

RowPlan make_plan(int N, int H, int W, int co_blocks, int sa, int a5, int a4, int b5, int b4)
{
    RowPlan p;
    p.col_strips = (W + 15) / 16;
    p.co_blocks = co_blocks;
    p.strips = N * p.col_strips;
    p.sa = sa;
    p.a5 = a5;
    p.a4 = a4;
    p.b5 = b5;
    p.b4 = b4;
    p.tall_total = (sa * a5 + (p.strips - sa) * b5) * co_blocks;
    p.short_total = (sa * a4 + (p.strips - sa) * b4) * co_blocks;
    p.tall_per_xcd = (p.tall_total + 7) / 8;
    p.short_per_xcd = (p.short_total + 7) / 8;
    return p;
}

}  // namespace

// Searches the cuts (n5 tall + n4 short tiles covering H rows with no tile to spare) for the two strip
// classes and the number of strips of the first class; results are remembered per launch shape.
RowPlan plan_rows(int N, int H, int W, int co_blocks, int stages, int slots)
{
    static std::mutex mu;
    static std::map<PlanKey, RowPlan> cache;
    const PlanKey key{N, H, W, co_blocks, stages, slots};
    {
        std::lock_guard<std::mutex> lock(mu);
        auto it = cache.find(key);
        if (it != cache.end()) return it->second;
    }
    struct Cut {
        int n5, n4;
    };
    std::vector<Cut> cuts;
    for (int n5 = 0; n5 * 4 * kTall < H + 4 * kTall; ++n5) {
        const int rest = H - n5 * 4 * kTall;
        cuts.push_back(Cut{n5, rest > 0 ? (rest + 4 * kShort - 1) / (4 * kShort) : 0});
        if (rest <= 0) break;
    }
    const int strips = N * ((W + 15) / 16);
    RowPlan best = make_plan(N, H, W, co_blocks, 0, 0, 0, cuts.back().n5, cuts.back().n4);
    double best_cost = plan_makespan(best, slots, stages);
    for (const Cut& a : cuts)
        for (const Cut& b : cuts) {
            if (&a > &b) continue;
            // candidate numbers of first-class strips: all of them when the list is short, else a coarse scan
            const int step = std::max(1, strips / 64);
            for (int sa = (&a == &b ? strips : 0); sa <= strips; sa += step) {
                const RowPlan p = make_plan(N, H, W, co_blocks, sa, a.n5, a.n4, b.n5, b.n4);
                const double c = plan_makespan(p, slots, stages);
                if (c < best_cost) {
                    best_cost = c;
                    best = p;
                }
            }
        }
    std::lock_guard<std::mutex> lock(mu);
    if (cache.size() > 4096) cache.clear();
    cache[key] = best;
    return best;
}

RowPlan plan_rows_for_device(int N, int H, int W, int co_blocks, int stages, int cus, int* slots_out)
{
    // one workgroup per compute unit (a workgroup owns nearly all of a unit's LDS)
    const int full = std::max(8, cus) / 8;
    RowPlan plan = plan_rows(N, H, W, co_blocks, stages, full);
    // (fewer entries than workgroups: launch only as many slots per XCD as the longer list needs)
    const int slots = std::max(1, std::min(full, std::max(plan.tall_per_xcd, plan.short_per_xcd)));
    if (slots != full) plan = plan_rows(N, H, W, co_blocks, stages, slots);
    *slots_out = slots;
    return plan;
}

namespace {

template <typename T, typename TO, bool FUSED>
rtoss_status launch_rows(const rtoss_wdesc& d, const ConvParams& c, const char* wfrag, const void* x, void* y, hipStream_t s)
{
    constexpr int x_copies_per_wave = ((((4 * kTall + 2) * kLW * 4 + 63) / 64) + 3) / 4;
    const size_t smem = 2 * ((size_t)kRowsTM * kTileBytes + (size_t)x_copies_per_wave * 4096);
    auto kern = conv3x3_rows_kernel<T, TO, FUSED>;
    static LaunchOnce lds_once;  // per instantiation
    if (rtoss_status st = ensure_dynamic_lds((const void*)kern, smem, lds_once, "conv3x3 shared memory attribute")) return st;
    DeviceInfo dev;
    if (rtoss_status st = current_device(&dev)) return st;
    const int co_blocks = ((d.Co + 15) / 16 + kRowsTM - 1) / kRowsTM;
    if (c.stride != 1 || d.Ci % 32 || d.Ci < 96) return fail(RTOSS_ESHAPE, "conv: the pipelined kernel needs stride 1 and three or more stages of 32 input channels");
    if ((int64_t)c.N * c.H * c.W * d.Ci / 8 > 0x7fffffff) return fail(RTOSS_ESHAPE, "conv: input too large for 32-bit chunk offsets");
    if ((int64_t)c.N * ((c.W + 15) / 16) * ((c.H + 15) / 16 + 1) * co_blocks > 0x3fffffff) return fail(RTOSS_ESHAPE, "conv: too many tiles");
    int slots = 0;
    const RowPlan plan = plan_rows_for_device(c.N, c.H, c.W, co_blocks, d.Ci / 32, dev.cus, &slots);
    dim3 grid((unsigned)(slots * 8)), block(256);
    kern<<<grid, block, smem, s>>>((const T*)x, (TO*)y, wfrag, wfrag + fragment_bytes(d), c.H, c.W, d.Ci, d.Co,
                                   padded_m_tiles(d.Co), plan, c.ep);
    return check_hip(hipGetLastError(), "conv3x3 rows launch");
}

}  // namespace

bool rows3x3_needs_fused_stage(const ConvParams& c) { return c.ep.scale || c.ep.bias || c.ep.residual || c.ep.act > 1; }

rtoss_status launch_conv3x3_rows(const rtoss_wdesc& d, const ConvParams& c, const void* section, const void* x, void* y,
                                 hipStream_t s)
{
    const char* wf = (const char*)section;
    const bool f32out = c.out_dt == RTOSS_F32;
    const bool fused = rows3x3_needs_fused_stage(c);
#define RTOSS_ROWS(T, TO) (fused ? launch_rows<T, TO, true>(d, c, wf, x, y, s) : launch_rows<T, TO, false>(d, c, wf, x, y, s))
    if (d.dt == RTOSS_F16) return f32out ? RTOSS_ROWS(f16_t, float) : RTOSS_ROWS(f16_t, f16_t);
    return f32out ? RTOSS_ROWS(bf16_t, float) : RTOSS_ROWS(bf16_t, bf16_t);
#undef RTOSS_ROWS
}

}  // namespace rtoss
