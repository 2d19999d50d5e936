// Per-layer kernel for large bf16 / int8 layers: persistent, pipelined "stream" variant.  Included by
// ogc_kernels.hip after the epilogue has been defined.
//
// Same tile mathematics as ogc_layer_kernel, but
//   * the operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: no staging
//     registers, no ds_write) through a ring of three stages, so two k-steps of loads are in flight per
//     workgroup.  Packed weights and KB16 activations are already in lane order: every wave-level load
//     moves one contiguous KiB on both sides;
//   * a workgroup is persistent: it walks a list of tiles and treats (tile, k-step) as one long stream, so
//     the loads of the next tile's first k-steps are already in flight while the current tile's epilogue
//     runs, and no pipeline ramp is paid per tile;
//   * two workgroups share a CU (256 VGPRs each): one workgroup's epilogue and barrier waits overlap the
//     other's MFMA main loop;
//   * the main loop is hand scheduled in inline assembly on a fixed register map, software pipelined by half
//     a k-step, one block per k-step: LDS operand reads for the next half-step go out ahead of the 8 MFMAs
//     on the current operands, the workgroup barrier sits between two MFMAs so the matrix pipe keeps working
//     while the waves synchronise, and the direct loads of a later ring stage (with their address updates)
//     are issued between the remaining MFMAs.  (A load instruction occupies the wave until the
//     texture-address unit accepts it, and that unit serves the whole CU at about one KiB per 19 clocks:
//     issued back to back the loads would stall the wave for as long as its MFMAs take.  And the compiler's
//     own wait insertion cannot tell ring slots apart: it would wait for every outstanding direct load
//     before any LDS read.)  Nothing but scalar bookkeeping runs between two blocks.
//
//   workgroup tile: 128 channels x 256 batch rows, 4 waves as 2 x 2, wave tile 64 x 128 (2 x 4 MFMA blocks),
//                   64-byte k-steps; stage layout [4 weight chunks of 2 KiB][8 activation chunks of 2 KiB]
//   register map  : v0..v79   compiler (addresses, epilogue) -- amdgpu_num_vgpr keeps it below v80 (on this
//                             unified register file the attribute counts in pairs, hence 40); the kernel
//                             contains no calls (they would bring the callee's register conventions in)
//                   v80..v103 operand set F0: W0 W1 X0 X1 X2 X3 (4 registers each)
//                   v104..v127 operand set F1
//                   v128..v255 accumulators, block b = 2*... i*4+j at v[128+16b .. 143+16b]
// X_PLAIN reads the caller's row-major x (16-byte aligned rows, no K padding; rows past M are clamped to
// the last row and never stored); u8 inputs are flipped to s8 after the LDS read.
// Loads land in order: waiting until at most 6*(newer stages) remain guarantees the oldest stage is
// complete.  An epilogue's stores share that counter and complete in issue order with the loads.
#ifndef OGC_LAYER_STREAM_H
#define OGC_LAYER_STREAM_H

OGC_DEV uint32_t lds_addr_of(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// Two shapes share the code below:
//   shape 0: 4 waves (2 x 2), workgroup tile 128 channels x 256 rows, 3-stage ring of 24 KiB, two workgroups
//            per CU (one's epilogue overlaps the other's main loop); 48 bytes loaded per CU clock at MFMA peak
//   shape 1: 8 waves (4 x 2), workgroup tile 256 x 256, 4-stage ring of 32 KiB, one workgroup per CU; 32 bytes
//            per CU clock at MFMA peak -- the global->LDS path delivers about 53, so this is the shape for
//            layers with enough tiles to fill the chip
// In both, a wave owns 64 channels x 128 rows (2 x 4 MFMA blocks) and 256 VGPRs.
//   shape 2: 8 waves as 2 x 2 x 2: two k groups of four waves, each group on every second k-step of the same
//            128 x 128 tile (k-slicing inside the workgroup, Section III), a wave owning 64 x 64 (2 x 2 blocks).  For
//            layers with few outputs against a long reduction axis: 128 x 128 is what a CU's share of such a layer
//            comes to, and cutting K between workgroups instead costs a pass over fp32 partials in memory.  A stage
//            holds two k-steps (32 KiB); at the end of a tile the second group's accumulators cross LDS to the first
template <int SHAPE> struct StreamCfg {
    enum {
        KG = SHAPE == 2 ? 2 : 1,  // k groups: k-steps of a stage, each taken by its own group of waves
        TN = 2, TM = SHAPE == 2 ? 2 : 4, WAVES_N = SHAPE == 1 ? 4 : 2, WAVES_M = 2, WAVES = WAVES_N * WAVES_M * KG, NT = WAVES * 64,
        NST = SHAPE ? 4 : 3, BN = WAVES_N * TN * 32, BM = WAVES_M * TM * 32,
        W_OPS = KG * BN / 16, X_OPS = KG * BM / 16, OPS = W_OPS + X_OPS, OPW = OPS / WAVES,
        STAGE = KG * (BN + BM) * 64, RING = STAGE * NST, PARAMS = 2 * BN * 4,
        // the eight-wave shape (one workgroup per CU) has room for 2 KiB per wave through which the last layer's
        // result chunks are regrouped into whole row segments
        ROWS64 = SHAPE == 1 ? WAVES * 2048 : 0,
        KRED = SHAPE == 2 ? 4 * 4096 : 0,  // one accumulator block of each wave of the second k group
        LDS = RING + 2 * PARAMS + ROWS64 + KRED,
        COMPILER_VGPRS = 80, NUM_VGPR_ATTR = COMPILER_VGPRS / 2
    };
    static_assert(OPW == (SHAPE ? 4 : 6) && OPS % WAVES == 0, "loads per wave and stage");
};

// ---- assembly building blocks ----------------------------------------------------------------------------
// operand registers of set F (base 80 or 104): W0 = v[F:F+3], W1 = v[F+4:F+7], Xj = v[F+8+4j : F+11+4j]
#define OGC_W(F, i) "v[" #F "+4*" #i ":" #F "+3+4*" #i "]"
#define OGC_X(F, j) "v[" #F "+8+4*" #j ":" #F "+11+4*" #j "]"
#define OGC_ACC(b) "v[128+16*" #b ":143+16*" #b "]"
// reads the operand set F from LDS at the addresses in the registers WA / XA
#define OGC_READ_W(F, WA)                                           \
    "ds_read_b128 " OGC_W(F, 0) ", " WA "\n\t"                       \
    "ds_read_b128 " OGC_W(F, 1) ", " WA " offset:2048\n\t"
#define OGC_READ_X(F, XA)                                           \
    "ds_read_b128 " OGC_X(F, 0) ", " XA "\n\t"                       \
    "ds_read_b128 " OGC_X(F, 1) ", " XA " offset:2048\n\t"           \
    "ds_read_b128 " OGC_X(F, 2) ", " XA " offset:4096\n\t"           \
    "ds_read_b128 " OGC_X(F, 3) ", " XA " offset:6144\n\t"
#define OGC_READ(F, WA, XA) OGC_READ_W(F, WA) OGC_READ_X(F, XA)
// u8 -> s8 on the four registers of activation operand j of set F; %[flip] = 0x80808080
#define OGC_FLIP4(F, j)                                          \
    "v_xor_b32 v[" #F "+8+4*" #j "], %[flip], v[" #F "+8+4*" #j "]\n\t"   \
    "v_xor_b32 v[" #F "+9+4*" #j "], %[flip], v[" #F "+9+4*" #j "]\n\t"   \
    "v_xor_b32 v[" #F "+10+4*" #j "], %[flip], v[" #F "+10+4*" #j "]\n\t" \
    "v_xor_b32 v[" #F "+11+4*" #j "], %[flip], v[" #F "+11+4*" #j "]\n\t" \
    "s_nop 1\n\t"
#define OGC_NOFLIP4(F, j)
#define OGC_FLIP(F) OGC_FLIP4(F, 0) OGC_FLIP4(F, 1) OGC_FLIP4(F, 2) OGC_FLIP4(F, 3)
#define OGC_MFMA(OP, F, b, i, j) OP " " OGC_ACC(b) ", " OGC_W(F, i) ", " OGC_X(F, j) ", " OGC_ACC(b) "\n\t"
#define OGC_MFMA_Z(OP, F, b, i, j) OP " " OGC_ACC(b) ", " OGC_W(F, i) ", " OGC_X(F, j) ", 0\n\t"
// one direct load of 1 KiB into LDS at m0 = %[m0b] + off, then the cursor of that load moves on by INC
#define OGC_DMA(i, off, INC)                                                                   \
    "s_add_u32 m0, %[m0b], " #off "\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[g" #i "], off\n\t"  \
    "v_lshl_add_u64 %[g" #i "], %[g" #i "], 0, %[" INC "]\n\t"
#define OGC_NODMA(i, off, INC)

// One k-step of the main loop as a single block.  On entry operand set F0 (v80..) holds the first 32 bytes of
// this step's operands; SOC / SON are the LDS byte offsets of this step's second half and of the next
// step's first half.
//   reads F1 | 8 MFMAs on F0 | wait F1 | 2 MFMAs on F1 | wait for the next stage's loads, barrier |
//   reads F0 of the next step | 6 MFMAs on F1 with this wave's direct loads between them | wait F0
// The two MFMAs ahead of the barrier keep the matrix pipe fed while the workgroup synchronises.
//   MZ: MFMA macro of the first half (accumulate or start from zero); FL: flip macro (X_PLAIN u8 input);
//   SYNC: text of the wait + barrier; RD: reads of the next step or nothing; D: load macro; LW/LX: which
//   loads of a wave fetch weights (ops 0,1) and activations (the rest); OFS: LDS stride between a wave's loads
#define OGC_STEP_HEAD                                   \
    "v_add_u32 %[t0], %[soc], %[wrd]\n\t"               \
    "v_add_u32 %[t1], %[sox], %[xrdh]\n\t"              \
    "v_add_u32 %[t2], %[son], %[wrd]\n\t"               \
    "v_add_u32 %[t3], %[son], %[xrd]\n\t"
#define OGC_STEP_FIRST(OP, MZ, FL)                                                                        \
    OGC_READ_W(104, "%[t0]") OGC_READ_X(104, "%[t1]")                                                                     \
    FL(80, 0) MZ(OP, 80, 0, 0, 0) FL(80, 1) MZ(OP, 80, 1, 0, 1) FL(80, 2) MZ(OP, 80, 2, 0, 2) FL(80, 3)   \
        MZ(OP, 80, 3, 0, 3) MZ(OP, 80, 4, 1, 0) MZ(OP, 80, 5, 1, 1) MZ(OP, 80, 6, 1, 2) MZ(OP, 80, 7, 1, 3) \
            "s_waitcnt lgkmcnt(0)\n\t" FL(104, 0) OGC_MFMA(OP, 104, 0, 0, 0) FL(104, 1) OGC_MFMA(OP, 104, 1, 0, 1)
#define OGC_STEP_SYNC(VMN) "s_waitcnt vmcnt(" #VMN ")\n\ts_barrier\n\t" OGC_READ(80, "%[t2]", "%[t3]")
#define OGC_STEP_NOSYNC
#define OGC_STEP_REST6(OP, FL, D, O1, O2, O3, O4, O5)                                                     \
    FL(104, 2) OGC_MFMA(OP, 104, 2, 0, 2) D(0, 0, "incw") FL(104, 3) OGC_MFMA(OP, 104, 3, 0, 3)           \
        D(1, O1, "incw") OGC_MFMA(OP, 104, 4, 1, 0) D(2, O2, "incx") OGC_MFMA(OP, 104, 5, 1, 1)           \
            D(3, O3, "incx") OGC_MFMA(OP, 104, 6, 1, 2) D(4, O4, "incx") OGC_MFMA(OP, 104, 7, 1, 3)       \
                D(5, O5, "incx") "s_waitcnt lgkmcnt(0)"
#define OGC_STEP_REST4(OP, FL, D, O1, O2, O3)                                                             \
    FL(104, 2) OGC_MFMA(OP, 104, 2, 0, 2) D(0, 0, "incw") FL(104, 3) OGC_MFMA(OP, 104, 3, 0, 3)           \
        D(1, O1, "incw") OGC_MFMA(OP, 104, 4, 1, 0) D(2, O2, "incx") OGC_MFMA(OP, 104, 5, 1, 1)           \
            D(3, O3, "incx") OGC_MFMA(OP, 104, 6, 1, 2) OGC_MFMA(OP, 104, 7, 1, 3) "s_waitcnt lgkmcnt(0)"

// ---- the 64 x 64 wave tile of shape 2: operands W0 W1 X0 X1, blocks 0, 1 (W0 x X0, X1) and 4, 5 (W1 x X0, X1) ----
#define OGC_READ2_X(F, XA)                                          \
    "ds_read_b128 " OGC_X(F, 0) ", " XA "\n\t"                       \
    "ds_read_b128 " OGC_X(F, 1) ", " XA " offset:2048\n\t"
#define OGC_READ2(F, WA, XA) OGC_READ_W(F, WA) OGC_READ2_X(F, XA)
#define OGC_READ2_HI(F, WA, XH)                                     \
    "ds_read_b128 " OGC_W(F, 0) ", " WA " offset:1024\n\t"           \
    "ds_read_b128 " OGC_W(F, 1) ", " WA " offset:3072\n\t"           \
    OGC_READ2_X(F, XH)
// single step: reads F1 | 4 MFMAs on F0 | wait F1 | 1 MFMA on F1 | wait for the next stage's loads, barrier |
// reads F0 of the next step | 3 MFMAs on F1 with the direct loads between and after them | wait F0
#define OGC_STEP2_FIRST(OP, MZ, FL)                                                                       \
    OGC_READ_W(104, "%[t0]") OGC_READ2_X(104, "%[t1]")                                                    \
    FL(80, 0) MZ(OP, 80, 0, 0, 0) FL(80, 1) MZ(OP, 80, 1, 0, 1) MZ(OP, 80, 4, 1, 0) MZ(OP, 80, 5, 1, 1)   \
    "s_waitcnt lgkmcnt(0)\n\t" FL(104, 0) OGC_MFMA(OP, 104, 0, 0, 0)
#define OGC_STEP2_SYNC(VMN) "s_waitcnt vmcnt(" #VMN ")\n\ts_barrier\n\t" OGC_READ2(80, "%[t2]", "%[t3]")
#define OGC_STEP2_REST(OP, FL, D)                                                                         \
    FL(104, 1) OGC_MFMA(OP, 104, 1, 0, 1) D(0, 0, "incw") D(1, 8192, "incw") OGC_MFMA(OP, 104, 4, 1, 0)   \
    D(2, 16384, "incx") D(3, 24576, "incx") OGC_MFMA(OP, 104, 5, 1, 1) "s_waitcnt lgkmcnt(0)"
#define OGC_RUN2(OP, FL, DA, DB, SLOT)                                                                    \
    ".Lks%=:\n\t"                                                                                         \
    "s_add_u32 %[son], %[sst], %[stg]\n\t"                                                                \
    "s_cmp_lg_u32 %[son], %[ring]\n\t"                                                                    \
    "s_cselect_b32 %[son], %[son], 0\n\t"                                                                 \
    OGC_READ2_HI(104, "%[tw]", "%[txh]")                                                                  \
    "s_waitcnt lgkmcnt(4)\n\t"                                                                            \
    FL(80, 0) OGC_MFMA(OP, 80, 0, 0, 0)                                                                   \
    "v_add_u32 %[tw], %[son], %[wrd]\n\t"                                                                 \
    "v_add_u32 %[tx], %[son], %[xrd]\n\t"                                                                 \
    "v_add_u32 %[txh], %[son], %[xrdh]\n\t"                                                               \
    FL(80, 1) OGC_MFMA(OP, 80, 1, 0, 1)                                                                   \
    "s_add_u32 %[kph], %[kph], 1\n\t"                                                                     \
    "s_cmp_eq_u32 %[kph], %[ktt]\n\t"                                                                     \
    "s_cselect_b64 %[incw], %[incww], %[incwn]\n\t"                                                       \
    "s_cselect_b64 %[incx], %[incxw], %[incxn]\n\t"                                                       \
    "s_cselect_b32 %[kph], 0, %[kph]\n\t"                                                                 \
    "s_add_u32 %[m0b], %[m0w], %[" SLOT "]\n\t"                                                           \
    DA(0, 0, "incw") DA(1, 8192, "incw") OGC_MFMA(OP, 80, 4, 1, 0)                                        \
    DA(2, 16384, "incx") DA(3, 24576, "incx") OGC_MFMA(OP, 80, 5, 1, 1)                                   \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                            \
    FL(104, 0) OGC_MFMA(OP, 104, 0, 0, 0)                                                                 \
    "s_waitcnt vmcnt(8)\n\ts_barrier\n\t"                                                                 \
    FL(104, 1) OGC_MFMA(OP, 104, 1, 0, 1)                                                                 \
    OGC_READ2(80, "%[tw]", "%[tx]")                                                                       \
    DB(0, 0, "incw") DB(1, 8192, "incw") OGC_MFMA(OP, 104, 4, 1, 0)                                       \
    DB(2, 16384, "incx") DB(3, 24576, "incx") OGC_MFMA(OP, 104, 5, 1, 1)                                  \
    "s_mov_b32 %[sprev], %[sst]\n\t"                                                                      \
    "s_mov_b32 %[sst], %[son]\n\t"                                                                        \
    "s_sub_u32 %[n], %[n], 1\n\t"                                                                         \
    "s_cmp_lg_u32 %[n], 0\n\t"                                                                            \
    "s_cbranch_scc1 .Lks%=\n\t"                                                                           \
    "s_waitcnt lgkmcnt(0)"

// Step modes: 0 = loads of the stage NST steps ahead are issued and VM newer loads may stay in flight at the
// barrier (after an epilogue too: its stores were issued after the loads this wait is for, and loads and stores
// complete in issue order, so they only make the wait longer than needed); 2 = no loads left to issue, everything
// awaited; 3 = last step of the stream: no barrier, no reads
template <int DT, int OPW, int VM, int MODE, bool ZERO, bool FLIP, int TMV = 4>
OGC_DEV void k_step(uint32_t w_rd, uint32_t x_rd, uint32_t x_rd_hi, uint32_t soc, uint32_t son, uint64_t (&g)[6], uint64_t incw,
                    uint64_t incx, uint32_t m0b) {
    const uint32_t sox = soc - 1024;  // the stage itself: the second half's activation chunks are addressed from x_rd_hi
    static_assert((OPW == 6 && VM == 6) || (OPW == 4 && (VM == 8 || VM == 4)), "loads allowed in flight at the barrier");
    const uint32_t flip = 0x80808080u;
    uint32_t t0, t1, t2, t3;
#define OGC_STEP_OUT [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3)
#define OGC_STEP_IN [wrd] "v"(w_rd), [xrd] "v"(x_rd), [xrdh] "v"(x_rd_hi), [soc] "s"(soc), [sox] "s"(sox), [son] "s"(son), [flip] "s"(flip)
#define OGC_STEP_G6 [g0] "+v"(g[0]), [g1] "+v"(g[1]), [g2] "+v"(g[2]), [g3] "+v"(g[3]), [g4] "+v"(g[4]), [g5] "+v"(g[5])
#define OGC_STEP_G4 [g0] "+v"(g[0]), [g1] "+v"(g[1]), [g2] "+v"(g[2]), [g3] "+v"(g[3])
#define OGC_STEP_DMA_IN [incw] "s"(incw), [incx] "s"(incx), [m0b] "s"(m0b)
#define OGC_STEP(OP, MZ, FL)                                                                                        \
    if constexpr (TMV == 2 && MODE == 0 && VM == 8)                                                                 \
        asm volatile(OGC_STEP_HEAD OGC_STEP2_FIRST(OP, MZ, FL) OGC_STEP2_SYNC(8) OGC_STEP2_REST(OP, FL, OGC_DMA)    \
                     : OGC_STEP_OUT, OGC_STEP_G4 : OGC_STEP_IN, OGC_STEP_DMA_IN : "memory");                        \
    else if constexpr (TMV == 2 && MODE == 0)                                                                       \
        asm volatile(OGC_STEP_HEAD OGC_STEP2_FIRST(OP, MZ, FL) OGC_STEP2_SYNC(4) OGC_STEP2_REST(OP, FL, OGC_DMA)    \
                     : OGC_STEP_OUT, OGC_STEP_G4 : OGC_STEP_IN, OGC_STEP_DMA_IN : "memory");                        \
    else if constexpr (TMV == 2 && MODE == 2)                                                                       \
        asm volatile(OGC_STEP_HEAD OGC_STEP2_FIRST(OP, MZ, FL) OGC_STEP2_SYNC(0) OGC_STEP2_REST(OP, FL, OGC_NODMA)  \
                     : OGC_STEP_OUT : OGC_STEP_IN : "memory");                                                      \
    else if constexpr (TMV == 2)                                                                                    \
        asm volatile(OGC_STEP_HEAD OGC_STEP2_FIRST(OP, MZ, FL) OGC_STEP2_REST(OP, FL, OGC_NODMA)                    \
                     : OGC_STEP_OUT : OGC_STEP_IN : "memory");                                                      \
    else if constexpr (MODE == 0 && OPW == 6)                                                                            \
        asm volatile(OGC_STEP_HEAD OGC_STEP_FIRST(OP, MZ, FL) OGC_STEP_SYNC(6)                                      \
                         OGC_STEP_REST6(OP, FL, OGC_DMA, 4096, 8192, 12288, 16384, 20480)                           \
                     : OGC_STEP_OUT, OGC_STEP_G6 : OGC_STEP_IN, OGC_STEP_DMA_IN : "memory");                        \
    else if constexpr (MODE == 0 && OPW == 4 && VM == 8)                                                            \
        asm volatile(OGC_STEP_HEAD OGC_STEP_FIRST(OP, MZ, FL) OGC_STEP_SYNC(8)                                      \
                         OGC_STEP_REST4(OP, FL, OGC_DMA, 8192, 16384, 24576)                                        \
                     : OGC_STEP_OUT, OGC_STEP_G4 : OGC_STEP_IN, OGC_STEP_DMA_IN : "memory");                        \
    else if constexpr (MODE == 0 && OPW == 4 && VM == 4)                                                            \
        asm volatile(OGC_STEP_HEAD OGC_STEP_FIRST(OP, MZ, FL) OGC_STEP_SYNC(4)                                      \
                         OGC_STEP_REST4(OP, FL, OGC_DMA, 8192, 16384, 24576)                                        \
                     : OGC_STEP_OUT, OGC_STEP_G4 : OGC_STEP_IN, OGC_STEP_DMA_IN : "memory");                        \
    else if constexpr (MODE == 2)                                                                                   \
        asm volatile(OGC_STEP_HEAD OGC_STEP_FIRST(OP, MZ, FL) OGC_STEP_SYNC(0)                                      \
                         OGC_STEP_REST4(OP, FL, OGC_NODMA, 0, 0, 0)                                                 \
                     : OGC_STEP_OUT : OGC_STEP_IN : "memory");                                                      \
    else                                                                                                            \
        asm volatile(OGC_STEP_HEAD OGC_STEP_FIRST(OP, MZ, FL) OGC_STEP_NOSYNC                                       \
                         OGC_STEP_REST4(OP, FL, OGC_NODMA, 0, 0, 0)                                                 \
                     : OGC_STEP_OUT : OGC_STEP_IN : "memory");
#define OGC_STEP_ZF(OP)                                        \
    if constexpr (ZERO && FLIP) {                              \
        OGC_STEP(OP, OGC_MFMA_Z, OGC_FLIP4)                    \
    } else if constexpr (ZERO && !FLIP) {                      \
        OGC_STEP(OP, OGC_MFMA_Z, OGC_NOFLIP4)                  \
    } else if constexpr (!ZERO && FLIP) {                      \
        OGC_STEP(OP, OGC_MFMA, OGC_FLIP4)                      \
    } else {                                                   \
        OGC_STEP(OP, OGC_MFMA, OGC_NOFLIP4)                    \
    }
    if constexpr (DT == OGC_I8) {
        OGC_STEP_ZF("v_mfma_i32_32x32x32_i8")
    } else {
        static_assert(DT == OGC_BF16, "this step covers int8 and bf16 (E4M3 has k_step8)");
        OGC_STEP_ZF("v_mfma_f32_32x32x16_bf16")
    }
#undef OGC_STEP_ZF
#undef OGC_STEP
}

// A run of n ordinary k-steps (accumulating, loads to issue in every one, no tile change of the prefetch
// cursor) as one block with its loop control inside, so that between two MFMAs of a wave there are never more
// than a handful of other instructions: with two waves per SIMD running in lockstep (they meet at the barrier
// every step) any stretch without MFMAs is a stretch where the matrix pipe idles.
//   tw / tx : LDS read addresses of the current stage (first half; the second half is 1 KiB further)
//   sst     : byte offset of the current stage in the ring; sprev: of the previous one
//   kph     : physical k-step the prefetch cursor points at (the walk over k is rotated and wraps at KT)
// LATE waves issue their loads among the first-half MFMAs (for the stage freed by the previous step's
// barrier), the others after the barrier: the two waves of a SIMD then never wait for the texture-address
// unit at the same time, and only half the workgroup's loads queue up there at once.
#define OGC_READ_HI(F, WA, XH)                                      \
    "ds_read_b128 " OGC_W(F, 0) ", " WA " offset:1024\n\t"           \
    "ds_read_b128 " OGC_W(F, 1) ", " WA " offset:3072\n\t"           \
    "ds_read_b128 " OGC_X(F, 0) ", " XH "\n\t"                       \
    "ds_read_b128 " OGC_X(F, 1) ", " XH " offset:2048\n\t"           \
    "ds_read_b128 " OGC_X(F, 2) ", " XH " offset:4096\n\t"           \
    "ds_read_b128 " OGC_X(F, 3) ", " XH " offset:6144\n\t"
#define OGC_RUN(OP, FL, DA, DB, SLOT, VMN, O1, O2, O3, O4, O5, D45)                                             \
    ".Lks%=:\n\t"                                                                                                \
    "s_add_u32 %[son], %[sst], %[stg]\n\t"                                                                       \
    "s_cmp_lg_u32 %[son], %[ring]\n\t"                                                                           \
    "s_cselect_b32 %[son], %[son], 0\n\t"                                                                        \
    OGC_READ_HI(104, "%[tw]", "%[txh]")                                                                          \
    "s_waitcnt lgkmcnt(6)\n\t"                                                                                   \
    FL(80, 0) OGC_MFMA(OP, 80, 0, 0, 0)                                                                          \
    "v_add_u32 %[tw], %[son], %[wrd]\n\t"                                                                        \
    "v_add_u32 %[tx], %[son], %[xrd]\n\t"                                                                        \
    "v_add_u32 %[txh], %[son], %[xrdh]\n\t"                                                                      \
    FL(80, 1) OGC_MFMA(OP, 80, 1, 0, 1)                                                                          \
    "s_add_u32 %[kph], %[kph], 1\n\t"                                                                            \
    "s_cmp_eq_u32 %[kph], %[ktt]\n\t"                                                                            \
    "s_cselect_b64 %[incw], %[incww], %[incwn]\n\t"                                                              \
    "s_cselect_b64 %[incx], %[incxw], %[incxn]\n\t"                                                              \
    "s_cselect_b32 %[kph], 0, %[kph]\n\t"                                                                        \
    "s_add_u32 %[m0b], %[m0w], %[" SLOT "]\n\t"                                                                  \
    FL(80, 2) OGC_MFMA(OP, 80, 2, 0, 2) DA(0, 0, "incw") FL(80, 3) OGC_MFMA(OP, 80, 3, 0, 3) DA(1, O1, "incw")   \
    OGC_MFMA(OP, 80, 4, 1, 0) DA(2, O2, "incx") OGC_MFMA(OP, 80, 5, 1, 1) DA(3, O3, "incx")                      \
    OGC_MFMA(OP, 80, 6, 1, 2) OGC_MFMA(OP, 80, 7, 1, 3)                                                          \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                   \
    FL(104, 0) OGC_MFMA(OP, 104, 0, 0, 0) FL(104, 1) OGC_MFMA(OP, 104, 1, 0, 1)                                  \
    "s_waitcnt vmcnt(" #VMN ")\n\ts_barrier\n\t"                                                                 \
    FL(104, 2) OGC_MFMA(OP, 104, 2, 0, 2)                                                                        \
    OGC_READ(80, "%[tw]", "%[tx]")                                                                               \
    DB(0, 0, "incw") FL(104, 3) OGC_MFMA(OP, 104, 3, 0, 3)                                                       \
    DB(1, O1, "incw") OGC_MFMA(OP, 104, 4, 1, 0) DB(2, O2, "incx") OGC_MFMA(OP, 104, 5, 1, 1) DB(3, O3, "incx")  \
    OGC_MFMA(OP, 104, 6, 1, 2) D45(4, O4, "incx") OGC_MFMA(OP, 104, 7, 1, 3) D45(5, O5, "incx")                  \
    "s_mov_b32 %[sprev], %[sst]\n\t"                                                                             \
    "s_mov_b32 %[sst], %[son]\n\t"                                                                               \
    "s_sub_u32 %[n], %[n], 1\n\t"                                                                                \
    "s_cmp_lg_u32 %[n], 0\n\t"                                                                                   \
    "s_cbranch_scc1 .Lks%=\n\t"                                                                                  \
    "s_waitcnt lgkmcnt(0)"

template <int DT, int SHAPE, bool LATE, bool FLIP>
OGC_DEV void k_steps_run(uint32_t w_rd, uint32_t x_rd, uint32_t x_rd_hi, uint64_t (&g)[6], uint32_t& sst, uint32_t& sprev, uint32_t& kph, uint32_t n,
                         uint32_t kt_total, uint32_t m0w, uint64_t incwn, uint64_t incww, uint64_t incxn, uint64_t incxw) {
    typedef StreamCfg<SHAPE> C;
    static_assert(!(LATE && SHAPE == 0), "only the eight-wave shapes split their waves into an early and a late group");
    const uint32_t flip = 0x80808080u;
    sst = __builtin_amdgcn_readfirstlane(sst);
    sprev = __builtin_amdgcn_readfirstlane(sprev);
    kph = __builtin_amdgcn_readfirstlane(kph);
    n = __builtin_amdgcn_readfirstlane(n);
    kt_total = __builtin_amdgcn_readfirstlane(kt_total);
    m0w = __builtin_amdgcn_readfirstlane(m0w);
    uint32_t tw = sst + w_rd, tx = sst + x_rd, txh = sst + x_rd_hi, son, m0b;
    uint64_t incw, incx;
#define OGC_RUN_OUT [son] "=&s"(son), [m0b] "=&s"(m0b), [incw] "=&s"(incw), [incx] "=&s"(incx), [tw] "+v"(tw), [tx] "+v"(tx), [txh] "+v"(txh), \
                    [sst] "+s"(sst), [sprev] "+s"(sprev), [kph] "+s"(kph), [n] "+s"(n)
#define OGC_RUN_IN [wrd] "v"(w_rd), [xrd] "v"(x_rd), [xrdh] "v"(x_rd_hi), [ktt] "s"(kt_total), [m0w] "s"(m0w), [incwn] "s"(incwn), [incww] "s"(incww), \
                   [incxn] "s"(incxn), [incxw] "s"(incxw), [flip] "s"(flip), [stg] "n"(C::STAGE), [ring] "n"(C::RING)
#define OGC_RUN_SHAPES(OP, FL)                                                                                              \
    if constexpr (SHAPE == 2 && !LATE)                                                                                      \
        asm volatile(OGC_RUN2(OP, FL, OGC_NODMA, OGC_DMA, "sst") : OGC_RUN_OUT, OGC_STEP_G4 : OGC_RUN_IN : "memory", "scc"); \
    else if constexpr (SHAPE == 2)                                                                                          \
        asm volatile(OGC_RUN2(OP, FL, OGC_DMA, OGC_NODMA, "sprev") : OGC_RUN_OUT, OGC_STEP_G4 : OGC_RUN_IN : "memory", "scc"); \
    else if constexpr (SHAPE == 0)                                                                                               \
        asm volatile(OGC_RUN(OP, FL, OGC_NODMA, OGC_DMA, "sst", 6, 4096, 8192, 12288, 16384, 20480, OGC_DMA)                \
                     : OGC_RUN_OUT, OGC_STEP_G6 : OGC_RUN_IN : "memory", "scc");                                            \
    else if constexpr (!LATE)                                                                                               \
        asm volatile(OGC_RUN(OP, FL, OGC_NODMA, OGC_DMA, "sst", 8, 8192, 16384, 24576, 0, 0, OGC_NODMA)                     \
                     : OGC_RUN_OUT, OGC_STEP_G4 : OGC_RUN_IN : "memory", "scc");                                            \
    else                                                                                                                    \
        asm volatile(OGC_RUN(OP, FL, OGC_DMA, OGC_NODMA, "sprev", 8, 8192, 16384, 24576, 0, 0, OGC_NODMA)                   \
                     : OGC_RUN_OUT, OGC_STEP_G4 : OGC_RUN_IN : "memory", "scc");
#define OGC_RUN_FL(OP)                          \
    if constexpr (FLIP) {                       \
        OGC_RUN_SHAPES(OP, OGC_FLIP4)           \
    } else {                                    \
        OGC_RUN_SHAPES(OP, OGC_NOFLIP4)         \
    }
    if constexpr (DT == OGC_I8) {
        OGC_RUN_FL("v_mfma_i32_32x32x32_i8")
    } else {
        OGC_RUN_FL("v_mfma_f32_32x32x16_bf16")
    }
#undef OGC_RUN_FL
#undef OGC_RUN_SHAPES
}

// ---- 8-bit floats (E4M3), eight-wave shape only ------------------------------------------------------------
// The full-rate fp8 matrix instruction contracts 64 bytes of K at once and takes each operand as EIGHT consecutive
// registers: the lane's 16 bytes of the first half k-step followed by its 16 bytes of the second half.  Register map
// of the operands (accumulators as above): W0 = v[80:87], W1 = v[88:95], X0..X3 = v[96:103] .. v[120:127]; a k-step is
// eight instructions, W0 x X0..X3 then W1 x X0..X3, 64 clocks each.  There is one operand set, so the reads of the next
// step go out as this step's instructions retire their operands (an instruction reads its A / B registers when it
// issues; LDS data comes back a hundred clocks later): the barrier sits after the fourth instruction, then
//   W1xX0 | read W0' | W1xX1 | read X0' | W1xX2 | read X1' | W1xX3 | read X2', X3', W1'
// and the next step's instructions wait for exactly the reads they need (LDS reads return in order): 8, 6, 4, 2
// outstanding before W0'xX0'..X3', none before W1'xX0'.
#define OGC8_W(i) "v[80+8*" #i ":87+8*" #i "]"
#define OGC8_X(j) "v[96+8*" #j ":103+8*" #j "]"
#define OGC8_MFMA(b, i, j) "v_mfma_f32_32x32x64_f8f6f4 " OGC_ACC(b) ", " OGC8_W(i) ", " OGC8_X(j) ", " OGC_ACC(b) "\n\t"
#define OGC8_MFMA_Z(b, i, j) "v_mfma_f32_32x32x64_f8f6f4 " OGC_ACC(b) ", " OGC8_W(i) ", " OGC8_X(j) ", 0\n\t"
// both halves of weight operand i (WA: LDS address of the stage's weights for this wave) / activation operand j
// (XA / XH: addresses of the first / second half)
#define OGC8_READ_W(i, WA)                                                                          \
    "ds_read_b128 v[80+8*" #i ":83+8*" #i "], " WA " offset:2048*" #i "\n\t"                         \
    "ds_read_b128 v[84+8*" #i ":87+8*" #i "], " WA " offset:1024+2048*" #i "\n\t"
#define OGC8_READ_X(j, XA, XH)                                                                      \
    "ds_read_b128 v[96+8*" #j ":99+8*" #j "], " XA " offset:2048*" #j "\n\t"                         \
    "ds_read_b128 v[100+8*" #j ":103+8*" #j "], " XH " offset:2048*" #j "\n\t"
#define OGC8_FIRST(MZ)                                                                              \
    "s_waitcnt lgkmcnt(8)\n\t" MZ(0, 0, 0) "s_waitcnt lgkmcnt(6)\n\t" MZ(1, 0, 1)                   \
    "s_waitcnt lgkmcnt(4)\n\t" MZ(2, 0, 2) "s_waitcnt lgkmcnt(2)\n\t" MZ(3, 0, 3)
// second half with the reads of the next step (TW / TX / TXH: its addresses) and the direct loads D between
#define OGC8_SECOND(MZ, D, TW, TX, TXH)                                                             \
    "s_waitcnt lgkmcnt(0)\n\t" MZ(4, 1, 0) OGC8_READ_W(0, TW) D(0, 0, "incw")                        \
    MZ(5, 1, 1) OGC8_READ_X(0, TX, TXH) D(1, 8192, "incw")                                          \
    MZ(6, 1, 2) OGC8_READ_X(1, TX, TXH) D(2, 16384, "incx")                                         \
    MZ(7, 1, 3) OGC8_READ_X(2, TX, TXH) D(3, 24576, "incx") OGC8_READ_X(3, TX, TXH) OGC8_READ_W(1, TW)
#define OGC8_SECOND_NOREAD(MZ) "s_waitcnt lgkmcnt(0)\n\t" MZ(4, 1, 0) MZ(5, 1, 1) MZ(6, 1, 2) MZ(7, 1, 3)

// One k-step.  MODE / VM / ZERO as for k_step; son: ring offset of the next step's stage.
template <int VM, int MODE, bool ZERO>
OGC_DEV void k_step8(uint32_t w_rd, uint32_t x_rd, uint32_t x_rd_hi, uint32_t son, uint64_t (&g)[6], uint64_t incw, uint64_t incx,
                     uint32_t m0b) {
    static_assert(VM == 8 || VM == 4, "loads allowed in flight at the barrier");
    uint32_t tw, tx, txh;
#define OGC8_HEAD "v_add_u32 %[tw], %[son], %[wrd]\n\tv_add_u32 %[tx], %[son], %[xrd]\n\tv_add_u32 %[txh], %[son], %[xrdh]\n\t"
#define OGC8_OUT [tw] "=&v"(tw), [tx] "=&v"(tx), [txh] "=&v"(txh)
#define OGC8_IN [wrd] "v"(w_rd), [xrd] "v"(x_rd), [xrdh] "v"(x_rd_hi), [son] "s"(son)
#define OGC8_STEP(MZ)                                                                                                   \
    if constexpr (MODE == 0 && VM == 8)                                                                                 \
        asm volatile(OGC8_HEAD OGC8_FIRST(MZ) "s_waitcnt vmcnt(8)\n\ts_barrier\n\t"                                    \
                         OGC8_SECOND(MZ, OGC_DMA, "%[tw]", "%[tx]", "%[txh]") "s_waitcnt lgkmcnt(0)"                    \
                     : OGC8_OUT, OGC_STEP_G4 : OGC8_IN, OGC_STEP_DMA_IN : "memory");                                    \
    else if constexpr (MODE == 0)                                                                                       \
        asm volatile(OGC8_HEAD OGC8_FIRST(MZ) "s_waitcnt vmcnt(4)\n\ts_barrier\n\t"                                    \
                         OGC8_SECOND(MZ, OGC_DMA, "%[tw]", "%[tx]", "%[txh]") "s_waitcnt lgkmcnt(0)"                    \
                     : OGC8_OUT, OGC_STEP_G4 : OGC8_IN, OGC_STEP_DMA_IN : "memory");                                    \
    else if constexpr (MODE == 2)                                                                                       \
        asm volatile(OGC8_HEAD OGC8_FIRST(MZ) "s_waitcnt vmcnt(0)\n\ts_barrier\n\t"                                    \
                         OGC8_SECOND(MZ, OGC_NODMA, "%[tw]", "%[tx]", "%[txh]") "s_waitcnt lgkmcnt(0)"                  \
                     : OGC8_OUT : OGC8_IN : "memory");                                                                  \
    else                                                                                                                \
        asm volatile(OGC8_FIRST(MZ) OGC8_SECOND_NOREAD(MZ) ::: "memory");
    if constexpr (ZERO) {
        OGC8_STEP(OGC8_MFMA_Z)
    } else {
        OGC8_STEP(OGC8_MFMA)
    }
#undef OGC8_STEP
}

// A run of n ordinary k-steps with the loop control inside (see k_steps_run): LATE waves issue their direct loads
// among the first four instructions, into the stage freed by the previous step's barrier, the others after the barrier.
#define OGC8_RUN(DA, DB, SLOT, VMN)                                                                      \
    ".Lks8%=:\n\t"                                                                                       \
    "s_add_u32 %[son], %[sst], %[stg]\n\t"                                                               \
    "s_cmp_lg_u32 %[son], %[ring]\n\t"                                                                   \
    "s_cselect_b32 %[son], %[son], 0\n\t"                                                                \
    "s_waitcnt lgkmcnt(8)\n\t" OGC8_MFMA(0, 0, 0)                                                        \
    "v_add_u32 %[tw], %[son], %[wrd]\n\t"                                                                \
    "v_add_u32 %[tx], %[son], %[xrd]\n\t"                                                                \
    "v_add_u32 %[txh], %[son], %[xrdh]\n\t"                                                              \
    "s_add_u32 %[kph], %[kph], 1\n\t"                                                                    \
    "s_cmp_eq_u32 %[kph], %[ktt]\n\t"                                                                    \
    "s_cselect_b64 %[incw], %[incww], %[incwn]\n\t"                                                      \
    "s_cselect_b64 %[incx], %[incxw], %[incxn]\n\t"                                                      \
    "s_cselect_b32 %[kph], 0, %[kph]\n\t"                                                                \
    "s_add_u32 %[m0b], %[m0w], %[" SLOT "]\n\t"                                                          \
    "s_waitcnt lgkmcnt(6)\n\t" OGC8_MFMA(1, 0, 1) DA(0, 0, "incw") DA(1, 8192, "incw")                   \
    "s_waitcnt lgkmcnt(4)\n\t" OGC8_MFMA(2, 0, 2) DA(2, 16384, "incx")                                   \
    "s_waitcnt lgkmcnt(2)\n\t" OGC8_MFMA(3, 0, 3) DA(3, 24576, "incx")                                   \
    "s_waitcnt vmcnt(" #VMN ")\n\ts_barrier\n\t"                                                        \
    OGC8_SECOND(OGC8_MFMA, DB, "%[tw]", "%[tx]", "%[txh]")                                               \
    "s_mov_b32 %[sprev], %[sst]\n\t"                                                                     \
    "s_mov_b32 %[sst], %[son]\n\t"                                                                       \
    "s_sub_u32 %[n], %[n], 1\n\t"                                                                        \
    "s_cmp_lg_u32 %[n], 0\n\t"                                                                           \
    "s_cbranch_scc1 .Lks8%=\n\t"                                                                         \
    "s_waitcnt lgkmcnt(0)"

template <bool LATE>
OGC_DEV void k_steps_run8(uint32_t w_rd, uint32_t x_rd, uint32_t x_rd_hi, uint64_t (&g)[6], uint32_t& sst, uint32_t& sprev, uint32_t& kph,
                          uint32_t n, uint32_t kt_total, uint32_t m0w, uint64_t incwn, uint64_t incww, uint64_t incxn, uint64_t incxw) {
    typedef StreamCfg<1> C;
    sst = __builtin_amdgcn_readfirstlane(sst);
    sprev = __builtin_amdgcn_readfirstlane(sprev);
    kph = __builtin_amdgcn_readfirstlane(kph);
    n = __builtin_amdgcn_readfirstlane(n);
    kt_total = __builtin_amdgcn_readfirstlane(kt_total);
    m0w = __builtin_amdgcn_readfirstlane(m0w);
    uint32_t tw = 0, tx = 0, txh = 0, son, m0b;
    uint64_t incw, incx;
#define OGC8_RUN_OUT [son] "=&s"(son), [m0b] "=&s"(m0b), [incw] "=&s"(incw), [incx] "=&s"(incx), [tw] "+v"(tw), [tx] "+v"(tx), [txh] "+v"(txh), \
                     [sst] "+s"(sst), [sprev] "+s"(sprev), [kph] "+s"(kph), [n] "+s"(n)
#define OGC8_RUN_IN [wrd] "v"(w_rd), [xrd] "v"(x_rd), [xrdh] "v"(x_rd_hi), [ktt] "s"(kt_total), [m0w] "s"(m0w), [incwn] "s"(incwn), [incww] "s"(incww), \
                    [incxn] "s"(incxn), [incxw] "s"(incxw), [stg] "n"(C::STAGE), [ring] "n"(C::RING)
    if constexpr (!LATE)
        asm volatile(OGC8_RUN(OGC_NODMA, OGC_DMA, "sst", 8) : OGC8_RUN_OUT, OGC_STEP_G4 : OGC8_RUN_IN : "memory", "scc");
    else
        asm volatile(OGC8_RUN(OGC_DMA, OGC_NODMA, "sprev", 8) : OGC8_RUN_OUT, OGC_STEP_G4 : OGC8_RUN_IN : "memory", "scc");
}

// block b of the accumulators to LDS as four 16-byte pieces per lane, 1 KiB apart (ra: the lane's LDS address)
#define OGC_LDS_PUT_ACC(b)                                                                            \
    asm volatile("ds_write_b128 %0, v[128+16*" #b ":131+16*" #b "]\n\t"                                \
                 "ds_write_b128 %0, v[132+16*" #b ":135+16*" #b "] offset:1024\n\t"                    \
                 "ds_write_b128 %0, v[136+16*" #b ":139+16*" #b "] offset:2048\n\t"                    \
                 "ds_write_b128 %0, v[140+16*" #b ":143+16*" #b "] offset:3072" ::"v"(ra) : "memory")

// Hands accumulator block B (v[128+16B ..]) to the compiler where it is: the empty statement declares the
// sixteen registers as its output, and the epilogue then reads them as source operands (no copies; the
// compiler cannot allocate, hence cannot write, registers above its cap).  The block's last MFMA may still be
// in flight: the caller has waited for it (see the s_nop before the epilogue).  Every use feeds a store, and
// the stores are ordered before the next k-step block, which overwrites the accumulators.
template <int DT, int B> OGC_DEV typename AccT<DT>::type take_acc_block() {
    v16i r;
    if constexpr (B == 0) asm volatile("" : "={v[128:143]}"(r));
    if constexpr (B == 1) asm volatile("" : "={v[144:159]}"(r));
    if constexpr (B == 2) asm volatile("" : "={v[160:175]}"(r));
    if constexpr (B == 3) asm volatile("" : "={v[176:191]}"(r));
    if constexpr (B == 4) asm volatile("" : "={v[192:207]}"(r));
    if constexpr (B == 5) asm volatile("" : "={v[208:223]}"(r));
    if constexpr (B == 6) asm volatile("" : "={v[224:239]}"(r));
    if constexpr (B == 7) asm volatile("" : "={v[240:255]}"(r));
    if constexpr (DT == OGC_I8) return r;
    else return __builtin_bit_cast(v16f, r);
}

// Grid: 8 * slots workgroups (slots <= tiles_per_xcd).  Workgroup wg belongs to XCD wg%8 and is slot wg/8 of
// it; XCD x owns the contiguous tile range [x*tiles_per_xcd, (x+1)*tiles_per_xcd) and its slots walk that
// range with stride `slots`, so the workgroups of one XCD always work on neighbouring tiles (the n-tiles of
// one batch tile share its activations through that XCD's L2).
// EPI: 1 / 3 / 4 = requantizing epilogue with ReLU / no activation / GELU only (int8 or E4M3), 0 = every other combination, 2 = split-K: `tiles_n` counts
// (channel tile, k range) pairs, a workgroup accumulates one k range of its tile and stores the raw accumulators
template <int DT, int SHAPE, int X_PLAIN, int OUT_PLAIN, int EPI>
__global__ void __launch_bounds__(StreamCfg<SHAPE>::NT, 2) __attribute__((amdgpu_num_vgpr(40)))
ogc_layer_dma_kernel(const OgcLayerArgs a, int tiles_n, int tiles_total, int tiles_per_xcd, int slots) {
    typedef StreamCfg<SHAPE> C;
    static_assert(C::NUM_VGPR_ATTR == 40, "keep the attribute above in step with the register map");
    constexpr int OPW = C::OPW, NST = C::NST, VM = (NST - 2) * OPW;
    constexpr int TN = C::TN, TM = C::TM;
    constexpr bool FLIP = X_PLAIN && DT == OGC_I8;
    static_assert(DT != OGC_F8 || (SHAPE == 1 && EPI != 2), "E4M3 runs the eight-wave shape and is not split along K");
    static_assert(EPI <= 2 || (DT != OGC_BF16 && SHAPE != 2), "the single-activation requantizing epilogues: quantized dtypes, not the k-sliced shape");
    extern __shared__ __align__(1024) uint8_t smem[];
    // v80..v255 are used by the assembly below only; naming the last one makes the kernel own all 256.
    asm volatile("; operand sets and accumulators live in v80..v255" ::: "v255");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int KG = C::KG;
    static_assert(!(KG == 2 && EPI == 2), "the shape that slices K inside the workgroup is not split between workgroups");
    const int wn = wave % C::WAVES_N, wm = (wave / C::WAVES_N) % C::WAVES_M, kg = wave / (C::WAVES_N * C::WAVES_M);
    const int LS = EPI == 2 ? a.ksplit_log2 : 0;  // log2 of the number of k ranges
    const int KT = ((a.KC >> 2) >> LS) / KG;      // steps of one tile (of one k range of it); a step is KG k-steps of 64 bytes
    const int xcd = blockIdx.x & 7;
    int t_end = (xcd + 1) * tiles_per_xcd;
    t_end = t_end < tiles_total ? t_end : tiles_total;
    const int first_tile = xcd * tiles_per_xcd + (blockIdx.x >> 3);
    if (first_tile >= t_end) return;
    if (a.clocks && tid == 0) {  // diagnostic runs: when this workgroup started, on both clocks
        a.clocks[blockIdx.x * 4] = wall_clock64();
        a.clocks[blockIdx.x * 4 + 1] = clock64();
    }
    // (integer divisions run on the vector ALU: readfirstlane tells the compiler the results are wave-uniform)
    const int my_tiles = __builtin_amdgcn_readfirstlane((t_end - first_tile + slots - 1) / slots);
    const int total_steps = my_tiles * KT;
    // tile coordinates advance by `slots` tiles at a time: (n, m) += (dn, dm) with a carry, no division
    const int dm = __builtin_amdgcn_readfirstlane(slots / tiles_n), dn = slots - dm * tiles_n;
    auto next_tile = [&](int& n, int& m) {
        n += dn;
        m += dm;
        if (n >= tiles_n) {
            n -= tiles_n;
            ++m;
        }
    };

    // ---- prefetch cursor ------------------------------------------------------------------------------
    // A stage is OPS loads of 1 KiB (two 512-byte slabs of one 32-row chunk); load i of wave w is op
    // o = i*WAVES + w, so loads 0 and 1 of every wave fetch weights and the others activations.  g[i] is the
    // global address of this wave's load i for the k-step the cursor points at; the step block advances it.
    // The k-steps of a tile are walked in rotated order, starting at rot = min(n_tile, n_tile*KT/tiles_n): the
    // workgroups that share a batch tile (its n-tiles, resident together on one XCD) then touch neighbouring
    // k-slices of the activations at any moment, so each slice is missed in L2 by one of them and hit by the others
    // a step later, instead of all of them waiting on the same miss.  One step apart and no more: spread over the
    // whole reduction axis (as first built) the n-tiles of a long-K layer each pulled their own copy of every
    // slice through the fabric, the first having long left the 4 MiB L2 when the next arrived (K = 4096, eight
    // n-tiles: 41 against 49 us).  Accumulation order within a tile is free (integer sums are exact; float sums
    // stay within the stated tolerance).
    static_assert(C::W_OPS == 2 * C::WAVES, "loads 0,1 of a wave are weights, the rest activations");
    uint64_t g[6] = {0, 0, 0, 0, 0, 0};
    const long long x_step = (X_PLAIN ? 64 : 2048) * KG, w_step = 2048 * KG;  // bytes a step advances along K
    int pf_m = __builtin_amdgcn_readfirstlane(first_tile / tiles_n), pf_n = first_tile - pf_m * tiles_n;
    int pf_left = my_tiles, pf_kt = 0, pf_kphys = 0;
    auto setup_src = [&]() {  // addresses of the cursor tile's first (rotated) k-step
        pf_kphys = __builtin_amdgcn_readfirstlane((int)((uint32_t)(pf_n * KT) / (uint32_t)tiles_n));
        pf_kphys = pf_kphys < pf_n ? pf_kphys : pf_n;  // one step apart at most (see above)
        pf_kt = 0;
        const int n_base = (pf_n >> LS) * C::BN, m_base = pf_m * C::BM;
        const int k_first = (pf_n & ((1 << LS) - 1)) * KT + pf_kphys;  // physical k-step in the whole reduction axis
#pragma unroll
        for (int i = 0; i < OPW; ++i) {
            long long src_kofs = 0;
            // (with two k groups the ops of a stage are [W group 0][W group 1][X group 0][X group 1]: the second group's
            // pieces are those of the next k-step)
            const int oo = i * C::WAVES + wave;
            const int og = KG == 2 ? ((oo % (C::W_OPS)) >= C::W_OPS / 2 ? 1 : 0) : 0;     // k group of this op (W and X have the same count)
            const int o = KG == 2 ? (oo < C::W_OPS ? oo - og * (C::W_OPS / 2) : oo - og * (C::X_OPS / 2) - C::W_OPS / 2) : oo;
            const uint8_t* src;
            if (i < 2) {
                src = a.w + ((size_t)((n_base >> 5) + (o >> 1)) * a.KC + (o & 1) * 2) * 512 + lane * 16 + (long long)k_first * w_step + og * 2048;
            } else {
                const int ox = o - C::W_OPS / KG;
                if (og) src_kofs = X_PLAIN ? 64 : 2048;
                if constexpr (X_PLAIN) {
                    const int qrow = lane >> 2;  // 16 rows per load, four lanes per row
                    int row = m_base + ox * 16 + qrow;
                    row = row < a.M ? row : a.M - 1;
                    src = a.x + (long long)row * a.ldx_bytes + ((((lane & 3) + (qrow >> 2)) & 3) << 4);
                } else {
                    src = a.x + ((size_t)((m_base >> 5) + (ox >> 1)) * a.KC + (ox & 1) * 2) * 512 + lane * 16;
                }
                src += (long long)k_first * x_step + src_kofs;
            }
            g[i] = (uint64_t)(uintptr_t)src;
        }
    };
    // The address increments that take the cursor from its current k-step to the next one of the same tile
    // (the rotated walk wraps from the last physical k-step back to the first).
    uint64_t incw = (uint64_t)w_step, incx = (uint64_t)x_step;
    const uint64_t incw_wrap = (uint64_t)(-(long long)(KT - 1) * w_step), incx_wrap = (uint64_t)(-(long long)(KT - 1) * x_step);
    auto set_increments = [&]() {  // for the transition out of the cursor's current k-step
        const bool wrap = pf_kphys + 1 == KT;
        incw = wrap ? incw_wrap : (uint64_t)w_step;
        incx = wrap ? incx_wrap : (uint64_t)x_step;
        pf_kphys = wrap ? 0 : pf_kphys + 1;
    };
    // after the loads of `n` more k-steps have been issued: a finished tile moves the cursor to the next one
    auto cursor_advanced = [&](int n) {
        pf_kt += n;
        if (pf_kt == KT) {
            --pf_left;
            next_tile(pf_n, pf_m);
            if (pf_left > 0) setup_src();
            else pf_kt = 0;
        }
    };
    const uint32_t lds0 = lds_addr_of(smem);
    const uint32_t m0_wave = lds0 + wave * 1024;  // + stage*STAGE + i*WAVES*1024: where this wave's load i lands
    const uint32_t w_rd = lds0 + kg * (C::BN * 64) + (wn * TN) * 2048 + lane * 16;
    // Activation chunks of a stage.  From a blocked tensor: [32-row block][4 chunks of a k-step][32 rows][16 bytes], the
    // operand order, the second half of a k-step 1 KiB after the first.  From the caller's plain rows (X_PLAIN): a load
    // instruction fetches the 64 bytes of a k-step for 16 rows, four lanes per row, so that each group of four lanes
    // reads one contiguous segment (32 rows x 32 bytes per instruction, as the operand order would need, costs the
    // texture-address unit four cache lines per lane group and made the first layer that much slower).  They land
    // [32-row block][32 rows][4 slots of 16 bytes]; row r keeps chunk c in slot (c - r/4) mod 4, which makes the 128-bit
    // reads of 16 consecutive rows conflict-free; the second half of a k-step is the slot two further, i.e. address ^ 32.
    uint32_t x_rd, x_rd_hi;
    if constexpr (X_PLAIN) {
        const int r = lane & 31;
        x_rd = lds0 + KG * C::BN * 64 + kg * (C::BM * 64) + (wm * TM) * 2048 + r * 64 + ((((lane >> 5) - (r >> 2)) & 3) << 4);
        x_rd_hi = x_rd ^ 32;
    } else {
        x_rd = lds0 + KG * C::BN * 64 + kg * (C::BM * 64) + (wm * TM) * 2048 + lane * 16;
        x_rd_hi = x_rd + 1024;
    }

    // Schedule (the ring slot of step q is q % NST):
    //   prologue: loads of the first steps in flight; wait for step 0; barrier; read F0(step 0)
    //   step q  : its barrier B_q comes after every wave has finished ALL its LDS reads of steps <= q and has
    //             seen its own loads of step q+1 land, so after B_q stage q+1 is complete and slot q % NST is
    //             free.  An "early" wave issues the loads of step q+NST right after B_q; a "late" wave (the
    //             second wave of each SIMD in the eight-wave shape) issues them during the first half of step
    //             q+1, so it runs one stage behind: its prologue issues NST-1 stages
    //   last step of a tile: epilogue from registers (the next tile's loads keep flying)
    // Per-channel parameters of a tile's 128/256 channels are staged in LDS (two buffers, alternating per tile)
    // as soon as the previous tile's epilogue is done: the epilogue then reads them with LDS loads, which do
    // not queue behind the direct loads in flight the way global loads would.  Layout: scale | bias.  (The plan
    // selects this kernel only for int8 layers whose input zero point is 128: no compensation term.)
    typedef __attribute__((address_space(3))) uint8_t lds_u8;
    lds_u8* const params_lds = (lds_u8*)smem + C::RING;
    // The parameters go from global memory straight into LDS as well (one dword per lane and load): no staging
    // register, hence no compiler-inserted wait for everything outstanding in the middle of the stream.  They are
    // issued ahead of a tile's epilogue stores and are older than every load that a later step waits for, so the
    // ordinary in-order waits of the steps cover them.
    auto stage_params = [&](int n_tile, int buf) {
        if (EPI != 2 && wave < C::BN / 64) {
            const int n = n_tile * C::BN + tid;
            const uint64_t sp = (uint64_t)(uintptr_t)(a.scale + n), bp = (uint64_t)(uintptr_t)(a.bias + n);
            const uint32_t m0s = __builtin_amdgcn_readfirstlane(lds0 + C::RING + buf * C::PARAMS + wave * 256);
            asm volatile("s_mov_b32 m0, %[ms]\n\ts_nop 0\n\tglobal_load_lds_dword %[sp], off\n\t"
                         "s_add_u32 m0, %[ms], %[bo]\n\ts_nop 0\n\tglobal_load_lds_dword %[bp], off\n\ts_nop 0"
                         :: [sp] "v"(sp), [bp] "v"(bp), [ms] "s"(m0s), [bo] "n"(C::BN * 4) : "memory", "scc");
        }
    };
    const bool late = SHAPE != 0 && wave >= 4;  // (shape 2: the second k group; the two groups pair up on the SIMDs)
    int cur_n = pf_n, cur_m = pf_m, tiles_left = my_tiles;
    int pbuf = 0;
    stage_params(cur_n >> LS, 0);
    setup_src();
    int fetched = 0;  // k-steps whose loads this wave has issued
    {
        const int want = late ? NST - 1 : NST;
#pragma unroll
        for (int st = 0; st < NST; ++st) {
            if (st < want && fetched < total_steps) {
                set_increments();
                const uint32_t m0b = __builtin_amdgcn_readfirstlane(m0_wave + st * C::STAGE);
                if constexpr (OPW == 6)
                    asm volatile(OGC_DMA(0, 0, "incw") OGC_DMA(1, 4096, "incw") OGC_DMA(2, 8192, "incx") OGC_DMA(3, 12288, "incx")
                                     OGC_DMA(4, 16384, "incx") OGC_DMA(5, 20480, "incx") "s_nop 0"
                                 : OGC_STEP_G6 : OGC_STEP_DMA_IN : "memory", "scc");
                else
                    asm volatile(OGC_DMA(0, 0, "incw") OGC_DMA(1, 8192, "incw") OGC_DMA(2, 16384, "incx") OGC_DMA(3, 24576, "incx")
                                     "s_nop 0"
                                 : OGC_STEP_G4 : OGC_STEP_DMA_IN : "memory", "scc");
                ++fetched;
                cursor_advanced(1);
            }
        }
        // step 0 has landed when at most fetched-1 newer stages remain in flight
        if (fetched >= 4) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(3 * OPW) : "memory");
        else if (fetched == 3) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * OPW) : "memory");
        else if (fetched == 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(OPW) : "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
    if constexpr (DT == OGC_F8)
        asm volatile(OGC8_READ_W(0, "%[wa]") OGC8_READ_X(0, "%[xa]", "%[xh]") OGC8_READ_X(1, "%[xa]", "%[xh]") OGC8_READ_X(2, "%[xa]", "%[xh]")
                         OGC8_READ_X(3, "%[xa]", "%[xh]") OGC8_READ_W(1, "%[wa]") "s_waitcnt lgkmcnt(0)"
                     ::[wa] "v"(w_rd), [xa] "v"(x_rd), [xh] "v"(x_rd_hi) : "memory");
    else if constexpr (TM == 2) asm volatile(OGC_READ2(80, "%[wa]", "%[xa]") "s_waitcnt lgkmcnt(0)" ::[wa] "v"(w_rd), [xa] "v"(x_rd) : "memory");
    else asm volatile(OGC_READ(80, "%[wa]", "%[xa]") "s_waitcnt lgkmcnt(0)" ::[wa] "v"(w_rd), [xa] "v"(x_rd) : "memory");
    uint32_t sst = 0, sprev = (NST - 1) * C::STAGE;  // ring offsets of the current and the previous step's stage
    int kt = 0, q = 0;
    while (q < total_steps) {
        const bool can_fetch = fetched < total_steps;
        if (kt > 0 && can_fetch) {
            // a run of ordinary steps: up to the end of this tile, of the cursor's tile, or of the stream
            int n = KT - kt;
            n = n < KT - pf_kt ? n : KT - pf_kt;
            n = n < total_steps - fetched ? n : total_steps - fetched;
            uint32_t kph = (uint32_t)pf_kphys;
            if constexpr (DT == OGC_F8) {
                if (late) k_steps_run8<true>(w_rd, x_rd, x_rd_hi, g, sst, sprev, kph, n, KT, m0_wave, (uint64_t)w_step, incw_wrap, (uint64_t)x_step, incx_wrap);
                else k_steps_run8<false>(w_rd, x_rd, x_rd_hi, g, sst, sprev, kph, n, KT, m0_wave, (uint64_t)w_step, incw_wrap, (uint64_t)x_step, incx_wrap);
            } else if (late) k_steps_run<DT, SHAPE, SHAPE != 0, FLIP>(w_rd, x_rd, x_rd_hi, g, sst, sprev, kph, n, KT, m0_wave, (uint64_t)w_step, incw_wrap, (uint64_t)x_step, incx_wrap);
            else k_steps_run<DT, SHAPE, false, FLIP>(w_rd, x_rd, x_rd_hi, g, sst, sprev, kph, n, KT, m0_wave, (uint64_t)w_step, incw_wrap, (uint64_t)x_step, incx_wrap);
            pf_kphys = (int)kph;
            kt += n;
            q += n;
            fetched += n;
            cursor_advanced(n);
        } else {
            const uint32_t snext = sst + C::STAGE == C::RING ? 0 : sst + C::STAGE;
            const uint32_t soc = sst + 1024, son = snext;
            const bool zero = kt == 0;
            if constexpr (DT == OGC_F8) {
                if (can_fetch) {
                    set_increments();
                    const uint32_t m0b = __builtin_amdgcn_readfirstlane(m0_wave + (late ? sprev : sst));
                    if (late) {
                        if (zero) k_step8<4, 0, true>(w_rd, x_rd, x_rd_hi, son, g, incw, incx, m0b);
                        else k_step8<4, 0, false>(w_rd, x_rd, x_rd_hi, son, g, incw, incx, m0b);
                    } else {
                        if (zero) k_step8<8, 0, true>(w_rd, x_rd, x_rd_hi, son, g, incw, incx, m0b);
                        else k_step8<8, 0, false>(w_rd, x_rd, x_rd_hi, son, g, incw, incx, m0b);
                    }
                    ++fetched;
                    cursor_advanced(1);
                } else if (q + 1 < total_steps) {
                    if (zero) k_step8<8, 2, true>(w_rd, x_rd, x_rd_hi, son, g, 0, 0, 0);
                    else k_step8<8, 2, false>(w_rd, x_rd, x_rd_hi, son, g, 0, 0, 0);
                } else {
                    if (zero) k_step8<8, 3, true>(w_rd, x_rd, x_rd_hi, son, g, 0, 0, 0);
                    else k_step8<8, 3, false>(w_rd, x_rd, x_rd_hi, son, g, 0, 0, 0);
                }
            } else
            if (can_fetch) {
                set_increments();
                const uint32_t m0b = __builtin_amdgcn_readfirstlane(m0_wave + (late ? sprev : sst));
                // a late wave has one stage fewer in flight at this point (its loads follow the barrier here)
                if (late) {
                    if (zero) k_step<DT, OPW, SHAPE != 0 ? 4 : VM, 0, true, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, incw, incx, m0b);
                    else k_step<DT, OPW, SHAPE != 0 ? 4 : VM, 0, false, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, incw, incx, m0b);
                } else {
                    if (zero) k_step<DT, OPW, VM, 0, true, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, incw, incx, m0b);
                    else k_step<DT, OPW, VM, 0, false, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, incw, incx, m0b);
                }
                ++fetched;
                cursor_advanced(1);
            } else if (q + 1 < total_steps) {
                if (zero) k_step<DT, OPW, VM, 2, true, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, 0, 0, 0);
                else k_step<DT, OPW, VM, 2, false, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, 0, 0, 0);
            } else {
                if (zero) k_step<DT, OPW, VM, 3, true, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, 0, 0, 0);
                else k_step<DT, OPW, VM, 3, false, FLIP, TM>(w_rd, x_rd, x_rd_hi, soc, son, g, 0, 0, 0);
            }
            sprev = sst;
            sst = snext;
            ++kt;
            ++q;
        }
        if (kt == KT) {
            kt = 0;
            // the accumulators are read by ordinary vector instructions next: let the last MFMA drain first
            asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
            const int n_base = (cur_n >> LS) * C::BN + wn * TN * 32, m_base = cur_m * C::BM + wm * TM * 32;
            BlockParams prm;
            auto read_params = [&](int i) {  // the lane's parameters for weight block i of this wave
                const lds_u8* pb = params_lds + pbuf * C::PARAMS;
                const int nl = (wn * TN + i) * 32 + 4 * (lane >> 5);
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    prm.s[gq] = *(const __attribute__((address_space(3))) v4f*)(pb + (nl + 8 * gq) * 4);
                    prm.b[gq] = *(const __attribute__((address_space(3))) v4f*)(pb + (C::BN + nl + 8 * gq) * 4);
                    prm.c[gq] = (v4i){0, 0, 0, 0};
                }
            };
            auto block = [&](auto tag) {
                constexpr int B = decltype(tag)::value;
                const int n0 = n_base + (B / 4) * 32, m0 = m_base + (B % 4) * 32;
                if constexpr (EPI == 2) {
                    const int range = cur_n & ((1 << LS) - 1);
                    uint8_t* dst = a.partial + ((((size_t)range * a.pmb + (m0 >> 5)) * a.pnb + (n0 >> 5)) * 4) * 1024 + lane * 16;
                    const auto acc = take_acc_block<DT, B>();
                    v16i ai;
                    if constexpr (DT == OGC_I8) ai = acc;
                    else ai = __builtin_bit_cast(v16i, acc);
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq)
                        store16_through(dst + qq * 1024, (v4i){ai[4 * qq], ai[4 * qq + 1], ai[4 * qq + 2], ai[4 * qq + 3]});
                } else if constexpr (OUT_PLAIN) {
                    if (n0 < a.N && m0 < a.M)
                        epilogue_block<DT, 1, false, EPI>(take_acc_block<DT, B>(), a, prm, n0, m0, lane, (uint8_t*)nullptr);
                } else {
                    if ((n0 >> 5) < a.NB_out)
                        epilogue_block<DT, 0, false, EPI>(take_acc_block<DT, B>(), a, prm, n0, m0, lane,
                                                     GlobalY{a.y + (size_t)(m0 >> 5) * a.KC_out * 512});
                }
            };
            // The next tile's parameters go to the other buffer (waves still in this epilogue keep reading this one),
            // ahead of this epilogue's stores: loads and stores complete in the order they were issued, so every wait
            // of the next tile's steps that covers a later ring load covers them, and the steps' barriers order them
            // before the next epilogue's reads.  The waits of those steps count ring loads only: the stores issued
            // here in between make them wait for more than they need, never for less.
            int next_n = cur_n, next_m = cur_m;
            next_tile(next_n, next_m);
            if (tiles_left > 1 && KT >= 4) stage_params(next_n >> LS, pbuf ^ 1);
            bool done = false;
            if constexpr ((EPI == 1 || EPI == 3 || EPI == 4) && OUT_PLAIN && C::ROWS64 > 0) {
                if (a.y_vec_ok && (a.N & 63) == 0) {
                    // whole 64-byte row segments: the two channel blocks of the same rows one after the other
                    lds_u8* const scratch = (lds_u8*)smem + C::RING + 2 * C::PARAMS + wave * 2048;
                    auto pair = [&](auto tag) {
                        constexpr int J = decltype(tag)::value;
                        const int m0 = m_base + J * 32;
                        if (m0 < a.M) {  // (n_base < N: N is a multiple of 64 and the tile starts inside it, or the wave has no work)
                            read_params(0);
                            const v4i c0 = requant_block_epi<DT, EPI>(take_acc_block<DT, J>(), a, prm);
                            read_params(1);
                            const v4i c1 = requant_block_epi<DT, EPI>(take_acc_block<DT, 4 + J>(), a, prm);
                            store_plain_rows64(c0, c1, a, n_base, m0, lane, scratch);
                        }
                    };
                    if (n_base < a.N) {
                        pair(std::integral_constant<int, 0>());
                        pair(std::integral_constant<int, 1>());
                        pair(std::integral_constant<int, 2>());
                        pair(std::integral_constant<int, 3>());
                    }
                    done = true;
                }
            }
            if constexpr (KG == 2) {
                // The two k groups hold two halves of every sum.  Block by block, the second group's sixteen registers
                // cross LDS (4 KiB per wave pair, next to the ring: the next tile's loads keep landing in the ring
                // meanwhile), the first group adds them to its own and runs the epilogue: group 0 + group 1, a fixed order.
                lds_u8* const red = (lds_u8*)smem + C::RING + 2 * C::PARAMS + (wave & 3) * 4096 + lane * 16;
                auto round = [&](auto tag) {
                    constexpr int B = decltype(tag)::value;
                    if (kg == 1) {
                        const uint32_t ra = (uint32_t)(uintptr_t)red;
                        if constexpr (B == 0) OGC_LDS_PUT_ACC(0);
                        if constexpr (B == 1) OGC_LDS_PUT_ACC(1);
                        if constexpr (B == 4) OGC_LDS_PUT_ACC(4);
                        if constexpr (B == 5) OGC_LDS_PUT_ACC(5);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                    if (kg == 0) {
                        typedef __attribute__((address_space(3))) v4i lds_v4i;
                        v4i o[4];
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq) o[qq] = *(const lds_v4i*)(red + qq * 1024);
                        const auto mine = take_acc_block<DT, B>();
                        typename AccT<DT>::type sum;
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq) {
                            const v4f of = __builtin_bit_cast(v4f, o[qq]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if constexpr (DT == OGC_I8) sum[4 * qq + e] = mine[4 * qq + e] + o[qq][e];
                                else sum[4 * qq + e] = mine[4 * qq + e] + of[e];
                            }
                        }
                        const int n0 = n_base + (B / 4) * 32, m0 = m_base + (B % 4) * 32;
                        if constexpr (OUT_PLAIN) {
                            if (n0 < a.N && m0 < a.M) epilogue_block<DT, 1, false, EPI>(sum, a, prm, n0, m0, lane, (uint8_t*)nullptr);
                        } else {
                            if ((n0 >> 5) < a.NB_out)
                                epilogue_block<DT, 0, false, EPI>(sum, a, prm, n0, m0, lane, GlobalY{a.y + (size_t)(m0 >> 5) * a.KC_out * 512});
                        }
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // the scratch is written again next round
                };
                if (kg == 0) read_params(0);
                round(std::integral_constant<int, 0>());
                round(std::integral_constant<int, 1>());
                if (kg == 0) read_params(1);
                round(std::integral_constant<int, 4>());
                round(std::integral_constant<int, 5>());
                done = true;
            }
            if (!done) {
                if constexpr (EPI != 2) read_params(0);
                block(std::integral_constant<int, 0>());
                block(std::integral_constant<int, 1>());
                block(std::integral_constant<int, 2>());
                block(std::integral_constant<int, 3>());
                if constexpr (EPI != 2) read_params(1);
                block(std::integral_constant<int, 4>());
                block(std::integral_constant<int, 5>());
                block(std::integral_constant<int, 6>());
                block(std::integral_constant<int, 7>());
            }
            cur_n = next_n, cur_m = next_m;
            if (--tiles_left > 0 && KT < 4) {
                // too few steps for the steps' own waits to cover the parameter loads before the next epilogue
                stage_params(cur_n >> LS, pbuf ^ 1);
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            }
            pbuf ^= 1;
        }
    }
    if (a.clocks && tid == 0) {  // ... and when its first wave had issued its last instruction
        a.clocks[blockIdx.x * 4 + 2] = wall_clock64();
        a.clocks[blockIdx.x * 4 + 3] = clock64();
    }
}

#endif
